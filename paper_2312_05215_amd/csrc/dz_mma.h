// Device-side building blocks shared by the streaming (decode) and the tiled (prefill) kernels:
// MFMA / sparse-MFMA wrappers, in-register dequantisation of packed delta codes, buffer-load
// helpers and the two software-pipeline stages (base step, delta tile).  Internal to libdz.
#pragma once
#include "dz_internal.h"
#include <limits.h>

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

// Halfs of padding per LDS row of x.  A fragment read (lane 16q + r: row r, 16 bytes at 16 q) is free of
// bank conflicts when the row stride is 32 bytes more than a multiple of 256: measured on gfx950, 4.0
// cycles per ds_read_b128 and CU against 7.2 with 16 bytes of padding and 28 with none.
constexpr int LDS_PAD = 16;

__device__ inline unsigned lanes_below(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load (vmcnt(0)), which would drain the weight prefetch at each barrier.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }

template <int ABID>
__device__ __forceinline__ f4 smfmac(h8 a, h16 b, f4 c, int idx)
{
    return __builtin_amdgcn_smfmac_f32_16x16x64_f16(a, b, c, idx, 0, ABID);
}

// Eight b-bit codes of one step -> eight fp16 values (code - zero) * scale.
// w: for 4-bit the step's dword; for 2-bit the dword shifted so the step's codes sit at bits
// 0..7 and 16..23.  The pair at bit position p of both halves becomes 1024 + code * 2^p after
// or-ing into fp16 1024.0 (exponent 25, ulp 1), and fma(v, 2^-p, -(2^(10-p) + zero)) is the
// exact integer code - zero.
// (w & mask) | magic in one VALU instruction.  The compiler emits an and and an or here because
// the instruction cannot carry two literals: the mask travels in an SGPR, 0x64006400 in a VGPR.
__device__ __forceinline__ h2 mask_or_magic(uint32_t w, uint32_t mask, uint32_t magic)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(magic));
    return as_h2(r);
}

template <int BITS>
__device__ __forceinline__ h8 dequant_step(uint32_t w, h2 s2, h2 z2)
{
    const uint32_t magic = 0x64006400u;
    h2 v0, v1, v2, v3;
    if (BITS == 4) {
        const uint32_t w1 = w >> 8;
        h2 r0 = mask_or_magic(w, 0x000F000Fu, magic);
        h2 r1 = mask_or_magic(w, 0x00F000F0u, magic);
        h2 r2 = mask_or_magic(w1, 0x000F000Fu, magic);
        h2 r3 = mask_or_magic(w1, 0x00F000F0u, magic);
        const h2 c0 = (h2){(_Float16)-1024.f, (_Float16)-1024.f} - z2;
        const h2 c1 = (h2){(_Float16)-64.f, (_Float16)-64.f} - z2;
        const h2 i16 = (h2){(_Float16)0.0625f, (_Float16)0.0625f};
        v0 = (r0 + c0) * s2;
        v1 = __builtin_elementwise_fma(r1, i16, c1) * s2;
        v2 = (r2 + c0) * s2;
        v3 = __builtin_elementwise_fma(r3, i16, c1) * s2;
    } else {
        h2 r0 = mask_or_magic(w, 0x00030003u, magic);
        h2 r1 = mask_or_magic(w, 0x000C000Cu, magic);
        h2 r2 = mask_or_magic(w, 0x00300030u, magic);
        h2 r3 = mask_or_magic(w, 0x00C000C0u, magic);
        const h2 c0 = (h2){(_Float16)-1024.f, (_Float16)-1024.f} - z2;
        const h2 c1 = (h2){(_Float16)-256.f, (_Float16)-256.f} - z2;
        const h2 c2 = (h2){(_Float16)-64.f, (_Float16)-64.f} - z2;
        const h2 c3 = (h2){(_Float16)-16.f, (_Float16)-16.f} - z2;
        const h2 i4 = (h2){(_Float16)0.25f, (_Float16)0.25f};
        const h2 i16 = (h2){(_Float16)0.0625f, (_Float16)0.0625f};
        const h2 i64 = (h2){(_Float16)0.015625f, (_Float16)0.015625f};
        v0 = (r0 + c0) * s2;
        v1 = __builtin_elementwise_fma(r1, i4, c1) * s2;
        v2 = __builtin_elementwise_fma(r2, i16, c2) * s2;
        v3 = __builtin_elementwise_fma(r3, i64, c3) * s2;
    }
    return (h8){v0.x, v0.y, v1.x, v1.y, v2.x, v2.y, v3.x, v3.y};
}

struct Geo {
    int lane, row, q;       // lane = 16q + row
    int KT;
    int LDW;                // LDS row stride in halfs
};

// B operand of one step for one column block: lane 16b + c reads the LDS row of its request
// column (boff = that row's offset in halfs), k = 8b..8b+7 (slots 0-7) and 32+8b..32+8b+7
// (slots 8-15) of the step.
__device__ __forceinline__ h16 load_b(const _Float16 *xs, int boff, const Geo &g, int kofs)
{
    const _Float16 *p = xs + boff + kofs + 8 * g.q;
    h8 lo = *(const h8 *)p;
    h8 hi = *(const h8 *)(p + 32);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
}

__device__ __forceinline__ h8 as_h8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(h8, (u4){a, b, c, d});
}

struct LaneOffs {
    uint32_t w;         // row * K * 2 + q * 16      (W fragment of a base step)
    uint32_t c;         // lane * 16                 (packed codes)
    uint32_t i;         // lane * 8                  (packed positions, 4-bit layout)
    uint32_t s;         // row * GPT * 4             (scale/zero pairs)
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// Inside one LDS round (a slice of k whose x rows sit in LDS) a wave first streams its rows of W
// (base phase), then the packed tiles of every delta that has requests (delta phase).  Both phases
// are software pipelines over fixed-size loads held in named register buffers:
//   base step  : 2 x 16 bytes of W per lane and row tile  -> two dense MFMAs per column block
//   delta task : one packed tile (16 rows x 256 k)         -> four sparse MFMAs per column block
// Loads go through buffer instructions: a wave-uniform resource (base pointer + size in bytes,
// bounds-checked by the hardware), a wave-uniform byte offset in an SGPR and a per-lane byte
// offset that never changes.  No branch surrounds a streaming load, so the hardware load counter
// the compiler waits on is exact and the prefetched loads really stay in flight.
//
// QO selects the quantisation-only format (no 2:4 pruning, a code for every column).  A dense group
// of four is the sum of two 2:4 patterns with fixed positions -- columns {0, 1} and columns {2, 3}
// -- so a quantisation-only tile is stored as two such halves and multiplied by the same sparse
// MFMAs with constant position words: the kernels differ only in what a tile's loads fetch and in
// running the four steps twice.
template <int BITS, int GROUP, bool QO = false>
struct Fmt {
    static constexpr int GPT = 256 / GROUP;                         // quantisation groups per tile row
    static constexpr int NH = QO ? 2 : 1;                           // 2:4 halves per tile
    static constexpr int SC0 = QO ? ((BITS == 4) ? 8 : 4) : ((BITS == 4) ? 6 : 4);   // first scale dword in a stage
    static constexpr int SD = SC0 + GPT;                            // dwords per lane and row tile
    static constexpr uint32_t TILE_BYTES = (QO && BITS == 4) ? 2048u : 1024u;   // plane C bytes per tile
};

// The codes of step s of half h of a lane's stage registers (shifted as dequant_step wants them)
// and the dword that carries the step's positions.
template <int BITS, bool QO>
__device__ __forceinline__ uint32_t step_codes(const uint32_t *st, int s, int h, uint32_t &idxw)
{
    if constexpr (QO) {
        idxw = h ? 0xEEEEEEEEu : 0x44444444u;       // every group keeps columns (2, 3) / (0, 1)
        if (BITS == 4) return st[4 * h + s];
        return st[2 * h + (s >> 1)] >> (8 * (s & 1));
    } else {
        if (BITS == 4) { idxw = st[4 + (s >> 1)]; return st[s]; }
        idxw = st[2 + (s >> 1)];
        return st[s >> 1] >> (8 * (s & 1));
    }
}

// The loads of one packed tile for one row tile into its stage registers.
template <int BITS, int GROUP, bool QO>
__device__ __forceinline__ void tile_loads(__amdgpu_buffer_rsrc_t rs, uint32_t tile, const LaneOffs &lo, uint32_t off_idx,
                                           uint32_t off_scale, uint32_t (&st)[Fmt<BITS, GROUP, QO>::SD])
{
    typedef Fmt<BITS, GROUP, QO> F;
    const uint32_t sc = off_scale + tile * (16u * F::GPT * 4u);
    const u32x4 x0 = __builtin_amdgcn_raw_buffer_load_b128(rs, lo.c, tile * F::TILE_BYTES, 0);
    st[0] = x0.x; st[1] = x0.y; st[2] = x0.z; st[3] = x0.w;
    if constexpr (QO && BITS == 4) {
        const u32x4 x1 = __builtin_amdgcn_raw_buffer_load_b128(rs, lo.c, tile * F::TILE_BYTES + 1024u, 0);
        st[4] = x1.x; st[5] = x1.y; st[6] = x1.z; st[7] = x1.w;
    }
    if constexpr (!QO && BITS == 4) {
        const u32x2 x1 = __builtin_amdgcn_raw_buffer_load_b64(rs, lo.i, off_idx + tile * 512u, 0);
        st[4] = x1.x; st[5] = x1.y;
    }
    if constexpr (F::GPT == 2) {
        const u32x2 x2 = __builtin_amdgcn_raw_buffer_load_b64(rs, lo.s, sc, 0);
        st[F::SC0] = x2.x; st[F::SC0 + 1] = x2.y;
    } else {
        const u32x4 x2 = __builtin_amdgcn_raw_buffer_load_b128(rs, lo.s, sc, 0);
        st[F::SC0] = x2.x; st[F::SC0 + 1] = x2.y; st[F::SC0 + 2] = x2.z; st[F::SC0 + 3] = x2.w;
    }
}


// ------------------------------------------------------------------------------------ base phase
// One step = 64 k of W for R row tiles.  step index s counts from the start of the round.
template <int R>
__device__ __forceinline__ void base_issue(__amdgpu_buffer_rsrc_t rw, const uint32_t (&wbase)[R], uint32_t voff, int s,
                                           u32x4 (&buf)[R][2])
{
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t o = wbase[r] + (uint32_t)s * 128u;
        buf[r][0] = __builtin_amdgcn_raw_buffer_load_b128(rw, voff, o, 0);
        buf[r][1] = __builtin_amdgcn_raw_buffer_load_b128(rw, voff, o + 64u, 0);
    }
}

template <int R, int J, int JA = J>
__device__ __forceinline__ void base_compute(const u32x4 (&buf)[R][2], const _Float16 *xs, const Geo &g,
                                             const int (&brow)[J], int kofs, f4 (&acc)[R][JA])
{
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const h16 b = load_b(xs, brow[j], g, kofs);
        const h8 b0 = __builtin_shufflevector(b, b, 0, 1, 2, 3, 4, 5, 6, 7);
        const h8 b1 = __builtin_shufflevector(b, b, 8, 9, 10, 11, 12, 13, 14, 15);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, buf[r][0]), b0, acc[r][j], 0, 0, 0);
            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, buf[r][1]), b1, acc[r][j], 0, 0, 0);
        }
    }
}

// ----------------------------------------------------------------------------------- delta phase
struct Cursor {
    int kt;         // k tile
    int seg;        // segment number
};

template <int BITS, int GROUP, bool QO, int R>
__device__ __forceinline__ void delta_issue(const Cursor &c, bool valid, const Geo &g, const int (&rtc)[R], const LaneOffs &lo,
                                            const unsigned long long *s_dptr, const int *s_seg_delta,
                                            uint32_t off_idx, uint32_t off_scale, uint32_t blob_bytes,
                                            uint32_t (&st)[R][Fmt<BITS, GROUP, QO>::SD])
{
    // With no delta task in this round the loads are still issued (so the load count never
    // depends on a branch) but against an empty resource: the hardware returns zeros and touches
    // no memory.
    const unsigned long long bp = s_dptr[valid ? s_seg_delta[c.seg] : 0];
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)bp);
    const uint32_t h = __builtin_amdgcn_readfirstlane((uint32_t)(bp >> 32));
    const __amdgpu_buffer_rsrc_t rs = make_rsrc((const void *)(((unsigned long long)h << 32) | l), valid ? blob_bytes : 0u);
#pragma unroll
    for (int r = 0; r < R; ++r)
        tile_loads<BITS, GROUP, QO>(rs, (uint32_t)rtc[r] * (uint32_t)g.KT + (uint32_t)c.kt, lo, off_idx, off_scale, st[r]);
}

__device__ __forceinline__ void advance(Cursor &c, int kr0, int kr1)
{
    if (++c.kt == kr1) { c.kt = kr0; ++c.seg; }
}

// k-tile-major order: the segments lo .. hi - 1 of a k tile, then the next k tile
__device__ __forceinline__ void advance_seg(Cursor &c, int lo, int hi)
{
    if (++c.seg >= hi) { c.seg = lo; ++c.kt; }
}

__device__ __forceinline__ void store_row4(_Float16 *p, f4 v, int accumulate)
{
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    if (accumulate) {
        h4 o = *(const h4 *)p;
        v.x += (float)o.x; v.y += (float)o.y; v.z += (float)o.z; v.w += (float)o.w;
    }
    h4 r = {(_Float16)v.x, (_Float16)v.y, (_Float16)v.z, (_Float16)v.w};
    *(h4 *)p = r;
}




}  // namespace

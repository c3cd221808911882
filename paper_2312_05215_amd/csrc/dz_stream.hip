// The streaming kernel: base GEMM + SBMM for a small batch of request rows (decode), one launch.
//
//   out[t] = f16( x[t] . W^T + x[t] . Delta_{Idx[t]}^T )      (paper Section 5.1 Eq. (2); Section 5.2)
//
// Decode is bound by the bytes of W and of the packed deltas that must cross HBM once per call
// (Section 5.1: "decoding latency is proportional to the GPU memory consumption of the model
// weights"), so the kernel is organised around streaming those bytes exactly once with 16-byte
// loads per lane, and keeping everything else (x, dequantisation, 2:4 expansion, the merge of base
// and delta results) on chip:
//
//   * a workgroup (4 waves) owns a block of 4*R row tiles (16 rows each) and one slice of k;
//     its slice of x -- rows already in delta-sorted order -- sits in LDS and is the B operand
//     of every MFMA; request rows are the MFMA N dimension, 16 per column block;
//   * base: W fragments go from global memory straight into the A operand of
//     V_MFMA_F32_16X16X32_F16 (lane 16q+r holds W[r][8q..8q+7], one 16-byte load);
//   * deltas: for each delta that has requests in the batch (segments of the sorted order; deltas
//     nobody asked for are never touched) the packed tile is loaded, codes are turned into fp16
//     pairs with a mask-or into the mantissa of 1024.0 and one packed fma, scaled, and fed with
//     the stored 2-bit positions to V_SMFMAC_F32_16X16X64_F16, the 2:4 sparse MFMA -- the sparse
//     expansion costs no instruction.  A segment only multiplies the column blocks it overlaps;
//     columns of a shared block that belong to a neighbouring segment are masked when the
//     segment's accumulator is merged;
//   * split-k partial sums meet in fp32: every workgroup stores its partial tile, the last one to
//     arrive for a row block (an arrival counter) adds them in fixed order and rounds to fp16
//     once.  With one slice the result is rounded and stored directly.
//
// The paper's kernel launches per-delta child kernels from a parent kernel; HIP has no device-side
// launch, so "one launch for all deltas" is a loop over the batch's segment list inside each
// workgroup.  Larger T is served as chunks of 64 sorted rows (grid dimension), which re-reads the
// weights from cache per chunk.
#include "dz_internal.h"
#include <limits.h>

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int LDS_PAD = 8;          // halfs of padding per LDS row (keeps 16-byte reads off one bank set)

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
template <int BITS>
__device__ __forceinline__ h8 dequant_step(uint32_t w, h2 s2, h2 z2)
{
    const uint32_t magic = 0x64006400u;
    h2 v0, v1, v2, v3;
    if (BITS == 4) {
        const uint32_t w1 = w >> 8;
        h2 r0 = as_h2((w & 0x000F000Fu) | magic);
        h2 r1 = as_h2((w & 0x00F000F0u) | magic);
        h2 r2 = as_h2((w1 & 0x000F000Fu) | magic);
        h2 r3 = as_h2((w1 & 0x00F000F0u) | magic);
        const h2 c0 = (h2){(_Float16)-1024.f, (_Float16)-1024.f} - z2;
        const h2 c1 = (h2){(_Float16)-64.f, (_Float16)-64.f} - z2;
        const h2 i16 = (h2){(_Float16)0.0625f, (_Float16)0.0625f};
        v0 = (r0 + c0) * s2;
        v1 = __builtin_elementwise_fma(r1, i16, c1) * s2;
        v2 = (r2 + c0) * s2;
        v3 = __builtin_elementwise_fma(r3, i16, c1) * s2;
    } else {
        h2 r0 = as_h2((w & 0x00030003u) | magic);
        h2 r1 = as_h2((w & 0x000C000Cu) | magic);
        h2 r2 = as_h2((w & 0x00300030u) | magic);
        h2 r3 = as_h2((w & 0x00C000C0u) | magic);
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

// Inside one LDS round (a slice of k whose x rows sit in LDS) a wave first streams its rows of W
// (base phase), then the packed tiles of every delta that has requests (delta phase).  Both phases
// are software pipelines over fixed-size loads held in named register buffers:
//   base step  : 2 x 16 bytes of W per lane and row tile  -> two dense MFMAs per column block
//   delta task : one packed tile (16 rows x 256 k)         -> four sparse MFMAs per column block
// Loads go through buffer instructions: a wave-uniform resource (base pointer + size in bytes,
// bounds-checked by the hardware), a wave-uniform byte offset in an SGPR and a per-lane byte
// offset that never changes.  No branch surrounds a streaming load, so the hardware load counter
// the compiler waits on is exact and the prefetched loads really stay in flight.
template <int BITS, int GROUP>
struct Fmt {
    static constexpr int GPT = 256 / GROUP;                         // quantisation groups per tile row
    static constexpr int SC0 = (BITS == 4) ? 6 : 4;                 // first scale dword in a stage
    static constexpr int SD = SC0 + GPT;                            // dwords per lane and row tile
};

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

template <int R, int J>
__device__ __forceinline__ void base_compute(const u32x4 (&buf)[R][2], const _Float16 *xs, const Geo &g,
                                             const int (&brow)[J], int kofs, f4 (&acc)[R][J])
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

template <int BITS, int GROUP, int R>
__device__ __forceinline__ void delta_issue(const Cursor &c, bool valid, const Geo &g, const int (&rtc)[R], const LaneOffs &lo,
                                            const unsigned long long *s_dptr, const int *s_seg_delta,
                                            uint32_t off_idx, uint32_t off_scale, uint32_t blob_bytes,
                                            uint32_t (&st)[R][Fmt<BITS, GROUP>::SD])
{
    typedef Fmt<BITS, GROUP> F;
    // With no delta task in this round the loads are still issued (so the load count never
    // depends on a branch) but against an empty resource: the hardware returns zeros and touches
    // no memory.
    const unsigned long long bp = s_dptr[valid ? s_seg_delta[c.seg] : 0];
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)bp);
    const uint32_t h = __builtin_amdgcn_readfirstlane((uint32_t)(bp >> 32));
    const __amdgpu_buffer_rsrc_t rs = make_rsrc((const void *)(((unsigned long long)h << 32) | l), valid ? blob_bytes : 0u);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t tile = (uint32_t)rtc[r] * (uint32_t)g.KT + (uint32_t)c.kt;
        const uint32_t sc = off_scale + tile * (16u * F::GPT * 4u);
        const u32x4 x0 = __builtin_amdgcn_raw_buffer_load_b128(rs, lo.c, tile * 1024u, 0);
        st[r][0] = x0.x; st[r][1] = x0.y; st[r][2] = x0.z; st[r][3] = x0.w;
        if constexpr (BITS == 4) {
            const u32x2 x1 = __builtin_amdgcn_raw_buffer_load_b64(rs, lo.i, off_idx + tile * 512u, 0);
            st[r][4] = x1.x; st[r][5] = x1.y;
        }
        if constexpr (F::GPT == 2) {
            const u32x2 x2 = __builtin_amdgcn_raw_buffer_load_b64(rs, lo.s, sc, 0);
            st[r][F::SC0] = x2.x; st[r][F::SC0 + 1] = x2.y;
        } else {
            const u32x4 x2 = __builtin_amdgcn_raw_buffer_load_b128(rs, lo.s, sc, 0);
            st[r][F::SC0] = x2.x; st[r][F::SC0 + 1] = x2.y; st[r][F::SC0 + 2] = x2.z; st[r][F::SC0 + 3] = x2.w;
        }
    }
}

// The four steps of one packed tile against column blocks j0 .. j0 + C - 1.
template <int BITS, int GROUP, int R, int J, int C>
__device__ __forceinline__ void delta_steps(const uint32_t (&st)[R][Fmt<BITS, GROUP>::SD], const _Float16 *xs,
                                            const Geo &g, int kofs, const int (&boff)[C], f4 (&tmp)[R][J])
{
    typedef Fmt<BITS, GROUP> F;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        h8 av[R];
        uint32_t idxw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const h2 sz2 = as_h2(st[r][F::SC0 + s * F::GPT / 4]);
            const h2 s2 = (h2){sz2.x, sz2.x};
            const h2 z2 = (h2){sz2.y, sz2.y};
            uint32_t w;
            if (BITS == 4) { w = st[r][s]; idxw[r] = st[r][4 + (s >> 1)]; }
            else { w = st[r][s >> 1] >> (8 * (s & 1)); idxw[r] = st[r][2 + (s >> 1)]; }
            av[r] = dequant_step<BITS>(w, s2, z2);
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const h16 b = load_b(xs, boff[c], g, kofs + s * 64);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (s & 1) tmp[r][c] = smfmac<1>(av[r], b, tmp[r][c], (int)idxw[r]);
                else tmp[r][c] = smfmac<0>(av[r], b, tmp[r][c], (int)idxw[r]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);      // keep one step's operands live at a time
    }
}

template <int BITS, int GROUP, int R, int J>
__device__ __forceinline__ void delta_compute(const Cursor &c, int kr0, int kr1,
                                              const uint32_t (&st)[R][Fmt<BITS, GROUP>::SD], const _Float16 *xs,
                                              const Geo &g, const int *s_seg_begin, const int *s_boff,
                                              f4 (&acc)[R][J], f4 (&tmp)[R][J])
{
    const int sb = __builtin_amdgcn_readfirstlane(s_seg_begin[c.seg]);
    const int se = __builtin_amdgcn_readfirstlane(s_seg_begin[c.seg + 1]);
    const int j0 = sb >> 4;
    const int C = ((se - 1) >> 4) - j0 + 1;
    if (c.kt == kr0) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < J; ++j) tmp[r][j] = (f4){0.f, 0.f, 0.f, 0.f};
    }
    const int kofs = (c.kt - kr0) * 256;
    // LDS rows of this lane's request column in each overlapped block
    int boff[J];
#pragma unroll
    for (int cc = 0; cc < J; ++cc) boff[cc] = s_boff[min(16 * (j0 + cc), 48) + g.row];
    if (C == 1) {
        const int b1[1] = {boff[0]};
        delta_steps<BITS, GROUP, R, J, 1>(st, xs, g, kofs, b1, tmp);
    }
    if constexpr (J >= 2) {
        if (C == 2) {
            const int b2[2] = {boff[0], boff[1]};
            delta_steps<BITS, GROUP, R, J, 2>(st, xs, g, kofs, b2, tmp);
        }
    }
    if constexpr (J >= 3) {
        if (C == 3) {
            const int b3[3] = {boff[0], boff[1], boff[2]};
            delta_steps<BITS, GROUP, R, J, 3>(st, xs, g, kofs, b3, tmp);
        }
    }
    if constexpr (J >= 4) {
        if (C == 4) {
            const int b4[4] = {boff[0], boff[1], boff[2], boff[3]};
            delta_steps<BITS, GROUP, R, J, 4>(st, xs, g, kofs, b4, tmp);
        }
    }
    if (c.kt == kr1 - 1) {
        // merge: only the columns (sorted positions) that belong to this segment
#pragma unroll
        for (int cc = 0; cc < J; ++cc) {
            const int pos = 16 * (j0 + cc) + g.row;
            const bool in = cc < C && pos >= sb && pos < se;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                f4 t = tmp[r][cc];
                if (!in) t = (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < J; ++j)
                    if (j == j0 + cc) acc[r][j] += t;
            }
        }
    }
}

__device__ __forceinline__ void advance(Cursor &c, int kr0, int kr1)
{
    if (++c.kt == kr1) { c.kt = kr0; ++c.seg; }
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



template <int BITS, int GROUP, int WAVES, int R, int J, bool HAS_BASE, bool HAS_DELTA>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu((WAVES * R <= 8 && J <= 2) ? 4 : 2)))
void stream_kernel(DzStreamArgs a, DzDeltaPtrs dp, int NRB, int round_tiles,
                                                            size_t off_idx, size_t off_scale, size_t blob_total)
{
    typedef Fmt<BITS, GROUP> F;
    constexpr int SD = F::SD;
    constexpr int THREADS = WAVES * 64;
    constexpr int ZROW = 16 * J;            // an all-zero LDS row for column slots without a request
    extern __shared__ __attribute__((aligned(16))) _Float16 xs[];     // [16J + 1][LDW]
    __shared__ int s_tok[64];               // request row of each sorted position (-1: none)
    __shared__ int s_key[64];               // delta of each sorted position
    __shared__ int s_raw[64];
    __shared__ int s_rank[64];
    __shared__ int s_boff[64];              // LDS offset (halfs) of the x row of each sorted position
    __shared__ unsigned long long s_dptr[DZ_MAX_DELTAS];   // packed-delta pointers (copied from the arguments)
    __shared__ int s_seg_delta[64];
    __shared__ int s_seg_begin[65];
    __shared__ int s_nseg;
    __shared__ int s_last;

    const int tid = threadIdx.x;
#ifdef DZ_PROF
#define DZ_T(i) do { if (tid == 0) a.prof[(size_t)blockIdx.x * 8 + (i)] = (long long)wall_clock64(); } while (0)
#else
#define DZ_T(i) do { } while (0)
#endif
    DZ_T(0);
    Geo g;
    g.lane = tid & 63; g.row = g.lane & 15; g.q = g.lane >> 4;
    g.KT = a.K >> 8;
    g.LDW = round_tiles * 256 + LDS_PAD;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    LaneOffs lo;
    lo.w = (uint32_t)g.row * (uint32_t)a.K * 2u + (uint32_t)g.q * 16u;
    lo.c = (uint32_t)g.lane * 16u;
    lo.i = (uint32_t)g.lane * 8u;
    lo.s = (uint32_t)g.row * (uint32_t)(F::GPT * 4);

    // Work decomposition: the (row block, k tile) grid of this call, flattened row block by row
    // block, is cut into G equal contiguous ranges, one per workgroup (G = a.S, a multiple of the
    // CU count whenever the call is large enough), so every CU streams the same number of bytes
    // whatever the shape.  A range may end inside a row block and continue in the next one: each
    // piece is a *segment* with its own partial result.
    const int G = a.S;
    const int chunk = blockIdx.x / G;
    const int wg = blockIdx.x - chunk * G;
    const long long P = (long long)NRB * g.KT;
    const int p_begin = (int)((long long)wg * P / G);
    const int p_end = (int)((long long)(wg + 1) * P / G);
    const int p0 = chunk * 64;
    const int cnt = min(64, a.T - p0);
    const int RT = a.N >> 4;

    // Request order (paper Section 5.2: requests of one delta are grouped).  Batches of up to 64
    // rows are ranked by every workgroup itself from the raw index vector (rank = rows with a
    // smaller delta + earlier rows of the same delta) -- no extra launch and no dependent load;
    // x then sits in LDS in request order and a lane finds the row of its column through s_boff.
    // Larger batches read the sorted order a segment pass left in the workspace and stage x rows
    // already sorted.
    const bool sort_here = HAS_DELTA && a.ids != nullptr;
    if (HAS_DELTA && tid < max(a.D, 1)) s_dptr[tid] = tid < a.D ? (unsigned long long)dp.p[tid] : (unsigned long long)a.x;   // before any long-latency load
    int my_id = -1;
    if (sort_here && tid < cnt) my_id = a.ids[tid];                 // earliest possible load
    if (!sort_here) {
        if (tid < 64) {
            int tok = -1, key = INT_MAX;
            if (tid < cnt) {
                tok = a.perm ? a.perm[p0 + tid] : p0 + tid;
                if (HAS_DELTA && a.key) key = a.key[p0 + tid];
            }
            s_tok[tid] = tok;
            s_key[tid] = key;
            s_boff[tid] = tid * g.LDW;
        }
        lds_barrier();
    }

    const _Float16 *x = (const _Float16 *)a.x;
    const uint32_t w_bytes = (uint32_t)a.N * (uint32_t)a.K * 2u;
    const uint32_t blob_bytes = (uint32_t)blob_total;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.W ? a.W : a.x, HAS_BASE ? w_bytes : 0u);
    _Float16 *out = (_Float16 *)a.out;
    constexpr int AGENT = 0x10;                  // cache-policy bit sc1
    const int Tp = ((a.T + 63) >> 6) << 6;
    const uint32_t slice_bytes = (uint32_t)Tp * (uint32_t)a.N * 4u;
    const __amdgpu_buffer_rsrc_t prs = make_rsrc(a.partial, slice_bytes * (uint32_t)a.max_slots);
    bool tables_ready = !sort_here;
    bool first_round = true;
    int nseg = 0;
    int brow[J];
#pragma unroll
    for (int j = 0; j < J; ++j) brow[j] = 0;

  for (int p = p_begin; p < p_end;) {
    const int rb = p / g.KT;
    const int kt0 = p - rb * g.KT;
    const int kt1 = min(g.KT, kt0 + (p_end - p));
    p += kt1 - kt0;
    int rtc[R];
    bool rvalid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int rt = rb * (WAVES * R) + wave * R + r;
        rvalid[r] = rt < RT;
        rtc[r] = rvalid[r] ? rt : RT - 1;
    }
    f4 acc[R][J], tmp[R][J];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < J; ++j) {
            acc[r][j] = (f4){0.f, 0.f, 0.f, 0.f};
            tmp[r][j] = (f4){0.f, 0.f, 0.f, 0.f};
        }
    for (int kr0 = kt0; kr0 < kt1; kr0 += round_tiles) {
        const int kr1 = min(kt1, kr0 + round_tiles);
        const int ntr = kr1 - kr0;
        const int nsteps = 4 * ntr;              // base steps of this round
        int nd = nseg * ntr;                     // delta tasks of this round (set after the sort in round one)
        Cursor ci, cc;
        ci.kt = kr0; ci.seg = 0;
        cc = ci;
        // named stage buffers (so each stays in registers), rotated by hand.  Issue cursors stop at
        // the last task / step and re-issue it (a few redundant cache hits at the end of a round)
        // so that issuing needs no branch.
        uint32_t st0[R][SD], st1[R][SD], st2[R][SD];
        u32x4 bw0[R][2], bw1[R][2], bw2[R][2], bw3[R][2];
        uint32_t wbase[R];
#pragma unroll
        for (int r = 0; r < R; ++r) wbase[r] = ((uint32_t)rtc[r] * 16u * (uint32_t)a.K + (uint32_t)kr0 * 256u) * 2u;
        int ti = 0, tc = 0;
#define DZ_ISSUE(buf)                                                                                              \
    do {                                                                                                           \
        delta_issue<BITS, GROUP, R>(ci, nd > 0, g, rtc, lo, s_dptr, s_seg_delta, (uint32_t)off_idx, (uint32_t)off_scale, blob_bytes, \
                                    buf);                                                                          \
        if (++ti < nd) advance(ci, kr0, kr1);                                                                      \
    } while (0)
#define DZ_STEP(cur, nxt)                                                                                          \
    do {                                                                                                           \
        DZ_ISSUE(nxt);                                                                                             \
        if (tc < nd) {                                                                                             \
            delta_compute<BITS, GROUP, R, J>(cc, kr0, kr1, cur, xs, g, s_seg_begin, s_boff, acc, tmp);             \
            advance(cc, kr0, kr1);                                                                                 \
        }                                                                                                          \
        ++tc;                                                                                                      \
    } while (0)
#define DZ_BSTEP(s, cur, nxt)                                                                                      \
    do {                                                                                                           \
        base_issue<R>(rw, wbase, lo.w, min((s) + 3, nsteps - 1), nxt);                                             \
        base_compute<R, J>(cur, xs, g, brow, (s) * 64, acc);                                                       \
    } while (0)
        if (!first_round) lds_barrier();       // previous LDS readers are done
        // ---- x[:, k-slice of this round] -> LDS (rows past cnt zero).  Order of issue: x first
        // (loads return in order and x is needed first), then the first weight loads, which then
        // fly while the batch is being sorted and x is written to LDS.
        const int cpr = ntr * 32;                // 16-byte pieces per row
        const int npieces = 16 * J * cpr;
        const uint32_t rcp = (65536u + (uint32_t)ntr - 1u) / (uint32_t)ntr;
        constexpr int XB = 2;                    // x pieces per thread and batch
        uint4 xv[XB];
        int xdst[XB];
#define DZ_XLOAD(i0)                                                                                               \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < XB; ++u) {                                                          \
            const int i = (i0) + u * THREADS;                                                                      \
            const int rr = (int)((((uint32_t)i >> 5) * rcp) >> 16);                                                \
            const int cc2 = i - rr * cpr;                                                                          \
            int tok = -1;                                                                                          \
            if (i < npieces) tok = sort_here ? (rr < cnt ? rr : -1) : s_tok[rr];                                   \
            xdst[u] = (i < npieces) ? rr * g.LDW + cc2 * 8 : -1;                                                   \
            xv[u] = (uint4){0u, 0u, 0u, 0u};                                                                       \
            if (tok >= 0) xv[u] = *(const uint4 *)(x + (size_t)tok * a.K + (size_t)kr0 * 256 + cc2 * 8);          \
        }                                                                                                          \
    } while (0)
#define DZ_XSTORE()                                                                                                \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < XB; ++u)                                                            \
            if (xdst[u] >= 0) *(uint4 *)(xs + xdst[u]) = xv[u];                                                    \
    } while (0)
        // all batches but the last go to LDS right away (nothing else is in flight yet); the last
        // batch stays in registers while the weight prefetch is issued behind it
        int xb0 = 0;
        for (; xb0 + THREADS * XB < npieces; xb0 += THREADS * XB) {
            DZ_XLOAD(xb0 + tid);
            DZ_XSTORE();
        }
        DZ_XLOAD(xb0 + tid);
        if constexpr (HAS_BASE) {
            base_issue<R>(rw, wbase, lo.w, 0, bw0);
            base_issue<R>(rw, wbase, lo.w, min(1, nsteps - 1), bw1);
            base_issue<R>(rw, wbase, lo.w, min(2, nsteps - 1), bw2);
        }
        if (!tables_ready) {
            // ---- rank the batch (all threads; four short barriers)
            if (tid < 64) {
                int key = INT_MAX;
                if (tid < cnt) {
                    const bool valid = my_id >= 0 && my_id < a.D;
                    key = valid ? my_id : a.D;
                    if (!valid && my_id != -1 && blockIdx.x == 0) atomicOr(a.err_flag, 1);
                }
                s_raw[tid] = key;
                s_rank[tid] = 0;
            }
            lds_barrier();
            {
                constexpr int PER = 64 / WAVES;     // each wave compares against its share of the rows
                const int t = tid & 63, part = tid >> 6;
                const int kme = s_raw[t];
                int c = 0;
#pragma unroll
                for (int jj = 0; jj < PER; ++jj) {
                    const int j = part * PER + jj;
                    const int kj = s_raw[j];
                    c += (kj < kme || (kj == kme && j < t)) ? 1 : 0;
                }
                atomicAdd(&s_rank[t], c);
            }
            lds_barrier();
            if (tid < 64) {
                const int r = s_rank[tid];
                s_tok[r] = tid < cnt ? tid : -1;
                s_key[r] = s_raw[tid];
                s_boff[r] = (tid < cnt ? tid : ZROW) * g.LDW;
            }
            lds_barrier();
        }
        if (first_round) {
            if (HAS_DELTA && tid < 64) {
                const int key = s_key[tid];
                const int prev = tid ? s_key[tid - 1] : -1;
                const bool valid = key >= 0 && key < a.D;
                const bool start = valid && (tid == 0 || prev != key);
                const unsigned long long sm = __ballot(start);
                const unsigned long long vm = __ballot(valid);
                if (start) {
                    const int i = (int)lanes_below(sm);
                    s_seg_delta[i] = key;
                    s_seg_begin[i] = tid;
                }
                if (tid == 0) {
                    const int ns = __builtin_popcountll(sm);
                    s_nseg = ns;
                    s_seg_begin[ns] = __builtin_popcountll(vm);     // rows that name a delta are a prefix
                }
            }
            if (tid < g.LDW / 8) *(uint4 *)(xs + ZROW * g.LDW + tid * 8) = (uint4){0u, 0u, 0u, 0u};
            lds_barrier();
            tables_ready = true;
            nseg = HAS_DELTA ? s_nseg : 0;
            nd = nseg * ntr;
#pragma unroll
            for (int j = 0; j < J; ++j) brow[j] = s_boff[16 * j + g.row];
            DZ_T(1);
        }
        if constexpr (HAS_DELTA) {
            DZ_ISSUE(st0);
            DZ_ISSUE(st1);
        }
        DZ_XSTORE();
        lds_barrier();
        first_round = false;
        DZ_T(2);
        if constexpr (HAS_BASE) {
            for (int s = 0; s < nsteps; s += 4) {
                DZ_BSTEP(s, bw0, bw3);
                DZ_BSTEP(s + 1, bw1, bw0);
                DZ_BSTEP(s + 2, bw2, bw1);
                DZ_BSTEP(s + 3, bw3, bw2);
            }
        }
        if constexpr (HAS_DELTA) {
            while (tc < nd) {
                DZ_STEP(st0, st2);
                DZ_STEP(st1, st0);
                DZ_STEP(st2, st1);
            }
        }
#undef DZ_ISSUE
#undef DZ_STEP
#undef DZ_BSTEP
#undef DZ_XLOAD
#undef DZ_XSTORE
    }

    DZ_T(3);
    // ---- results of this segment: lane 16q + c holds rows 4q..4q+3 of the row tile for request
    // column c.  Which workgroups contribute to row block rb follows from the range formula:
    // the owner of flat position f is ceil((f + 1) * G / P) - 1.
    const int w_first = (int)((((long long)rb * g.KT + 1) * G + P - 1) / P) - 1;
    const int w_last = (int)((((long long)(rb + 1) * g.KT) * G + P - 1) / P) - 1;
    const int ncontrib = w_last - w_first + 1;
    if (ncontrib == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!rvalid[r]) continue;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int tok = s_tok[16 * j + g.row];
                if (tok >= 0) store_row4(out + (size_t)tok * a.N + rtc[r] * 16 + 4 * g.q, acc[r][j], a.accumulate);
            }
        }
        continue;
    }

    // ---- several workgroups share the row block: partial tiles meet in fp32.  Partials are
    // written and later read with agent-scope (sc1) accesses, which are coherent across the chip's
    // L2s without flushing them; each wave waits for its stores to complete before the barrier,
    // then one thread bumps the arrival counter of the row block.  The last workgroup to arrive
    // adds the slots in fixed order (so the result does not depend on arrival order) and rounds
    // once.
    const int slot = wg - w_first;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (!rvalid[r]) continue;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int pr = 16 * j + g.row;
            if (pr < cnt) {
                const uint32_t off = ((uint32_t)(p0 + pr) * (uint32_t)a.N + (uint32_t)rtc[r] * 16u + 4u * g.q) * 4u;
                const u32x4 v = __builtin_bit_cast(u32x4, acc[r][j]);
                __builtin_amdgcn_raw_buffer_store_b128(v, prs, off, (uint32_t)slot * slice_bytes, AGENT);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);               // this wave's stores have completed
    __syncthreads();
    DZ_T(4);
    if (tid == 0) {
        int32_t *ctr = a.counters + chunk * NRB + rb;
        const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = (old == ncontrib - 1);
        if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        s_last = last;
    }
    __syncthreads();
    DZ_T(5);
    if (s_last) {
        constexpr int width = WAVES * R * 16;        // rows of N per row block
        constexpr int nq = width / 4;
        for (int i = tid; i < cnt * nq; i += THREADS) {
            const int pr = i / nq, c4 = i - pr * nq;
            const int n = rb * width + c4 * 4;
            if (n >= a.N) continue;
            const uint32_t off = ((uint32_t)(p0 + pr) * (uint32_t)a.N + (uint32_t)n) * 4u;
            f4 sum = (f4){0.f, 0.f, 0.f, 0.f};
            for (int s0 = 0; s0 < ncontrib; s0 += 8) {
                f4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int sl = min(s0 + u, ncontrib - 1);
                    v[u] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(prs, off, (uint32_t)sl * slice_bytes, AGENT));
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (s0 + u < ncontrib) sum += v[u];
            }
            const int tok = s_tok[pr];
            store_row4(out + (size_t)tok * a.N + n, sum, a.accumulate);
        }
    }
#ifdef DZ_PROF
    __builtin_amdgcn_s_waitcnt(0);
    DZ_T(6);
#endif
  }   // segments
}

template <int BITS, int GROUP, int WAVES, int R, int J, bool HB, bool HD>
hipError_t launch_one(const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int round_tiles, int grid,
                      size_t lds, const DzLayout &L, hipStream_t st)
{
    auto k = stream_kernel<BITS, GROUP, WAVES, R, J, HB, HD>;
    static bool attr_set = false;       // per instantiation; the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(WAVES * 64), lds, st, a, dp, NRB, round_tiles, L.off_idx, L.off_scale, L.total);
    return hipGetLastError();
}

template <int BITS, int GROUP, int WAVES, int R, bool HB, bool HD>
hipError_t launch_j(int J, const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int rt, int grid, size_t lds,
                    const DzLayout &L, hipStream_t st)
{
    switch (J) {
    case 1: return launch_one<BITS, GROUP, WAVES, R, 1, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    case 2: return launch_one<BITS, GROUP, WAVES, R, 2, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    case 3: return launch_one<BITS, GROUP, WAVES, R, 3, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    default: return launch_one<BITS, GROUP, WAVES, R, 4, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    }
}

template <int WAVES, int R, bool HB, bool HD>
hipError_t launch_fmt(int bits, int group, int J, const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int rt,
                      int grid, size_t lds, const DzLayout &L, hipStream_t st)
{
    if (!HD) return launch_j<4, 128, WAVES, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    if (bits == 4 && group == 128) return launch_j<4, 128, WAVES, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    if (bits == 4) return launch_j<4, 64, WAVES, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    if (group == 128) return launch_j<2, 128, WAVES, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    return launch_j<2, 64, WAVES, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
}

template <int WAVES, int R>
hipError_t launch_kind(const DzStreamArgs &a, int J, const DzDeltaPtrs &dp, int NRB, int rt, int grid, size_t lds,
                       const DzLayout &L, hipStream_t st)
{
    if (a.has_base && a.has_delta) return launch_fmt<WAVES, R, true, true>(a.bits, a.group, J, a, dp, NRB, rt, grid, lds, L, st);
    if (a.has_base) return launch_fmt<WAVES, R, true, false>(a.bits, a.group, J, a, dp, NRB, rt, grid, lds, L, st);
    return launch_fmt<WAVES, R, false, true>(a.bits, a.group, J, a, dp, NRB, rt, grid, lds, L, st);
}

}  // namespace

// Host side: choose the decomposition, make sure the workspace is large enough, launch.
int dz_ensure_partial(dz_ctx *ctx, size_t bytes, hipStream_t st);
int dz_ensure_counters(dz_ctx *ctx, int n, hipStream_t st);

int dz_launch_stream(dz_ctx *ctx, const DzStreamArgs &args, const DzDeltaPtrs &dp, hipStream_t st)
{
    DzStreamArgs a = args;
    const int RT = a.N / 16, KT = a.K / 256;
    const int nchunks = (a.T + 63) / 64;
    const int J = (a.T >= 64) ? 4 : (a.T + 15) / 16;
    // workgroup shape: few request columns -> 8 waves x 1 row tile (most waves in flight); three or
    // four column blocks -> 4 waves x 2 row tiles (each B fragment read from LDS feeds two MFMAs,
    // which the 2-bit format needs to stay under the LDS bandwidth)
    int WAVES = ctx->wg_waves, R = ctx->wg_rtiles;
    if (WAVES <= 0 || R <= 0) { WAVES = (J <= 2) ? 8 : 4; R = (J <= 2) ? 1 : 2; }
    const int NRB = (RT + WAVES * R - 1) / (WAVES * R);
    const long long units0 = (long long)nchunks * NRB;
    // number of workgroups per chunk: the target (a multiple of the CU count) unless the call has
    // fewer (row block, k tile) positions than that
    const long long P = (long long)NRB * KT;
    long long G = ctx->force_splits > 0 ? (long long)ctx->force_splits * NRB : ctx->target_wgs;
    if (G > P) G = P;
    if (G < 1) G = 1;
    // most workgroups that can share one row block = partial slots needed
    int max_slots = 1;
    for (int rb = 0; rb < NRB; ++rb) {
        const long long wf = (((long long)rb * KT + 1) * G + P - 1) / P - 1;
        const long long wl = (((long long)(rb + 1) * KT) * G + P - 1) / P - 1;
        if (wl - wf + 1 > max_slots) max_slots = (int)(wl - wf + 1);
    }
    const size_t Tp = (size_t)nchunks * 64;
    if ((size_t)max_slots * Tp * a.N * 4 >= ((size_t)1 << 32)) return DZ_ERR_SHAPE;    // 32-bit byte offsets
    // one batch of x loads per thread must cover a round (see XB in the kernel)
    const int round_cap = (J <= 2 ? 4 : 2);
    int round_tiles = (ctx->round_tiles > 0 && ctx->round_tiles < round_cap) ? ctx->round_tiles : round_cap;
    const int max_slice = (int)((P + G - 1) / G) < KT ? (int)((P + G - 1) / G) : KT;
    if (round_tiles > max_slice) round_tiles = max_slice;
    const size_t lds = (size_t)(16 * J + 1) * (round_tiles * 256 + LDS_PAD) * sizeof(_Float16);
    a.S = (int)G;
    a.max_slots = max_slots;
    if (max_slots > 1) {
        int rc = dz_ensure_partial(ctx, (size_t)max_slots * Tp * a.N * 4, st);
        if (rc) return rc;
        rc = dz_ensure_counters(ctx, (int)units0, st);
        if (rc) return rc;
    }
    a.partial = ctx->partial;
    a.counters = ctx->counters;
    const long long grid = (long long)nchunks * G;
    if (grid > 0x7fffffffLL) return DZ_ERR_SHAPE;
    if ((unsigned long long)a.N * a.K * 2ull >= (1ull << 32)) return DZ_ERR_SHAPE;     // 32-bit byte offsets
    DzLayout L = dz_make_layout(a.N, a.K, a.has_delta ? a.bits : 4, a.has_delta ? a.group : 128);
    hipError_t e;
    if (WAVES == 8 && R == 1) e = launch_kind<8, 1>(a, J, dp, NRB, round_tiles, (int)grid, lds, L, st);
    else if (WAVES == 8 && R == 2) e = launch_kind<8, 2>(a, J, dp, NRB, round_tiles, (int)grid, lds, L, st);
    else e = launch_kind<4, 2>(a, J, dp, NRB, round_tiles, (int)grid, lds, L, st);
    return dz_set_hip_error(ctx, e);
}

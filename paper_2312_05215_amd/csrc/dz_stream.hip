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

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int LDS_PAD = 8;          // halfs of padding per LDS row (keeps 16-byte reads off one bank set)

__device__ inline unsigned lanes_below(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
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

// B operand of one step for column block j: lane 16b + c reads request row 16j + c,
// k = 8b..8b+7 (slots 0-7) and 32+8b..32+8b+7 (slots 8-15) of the step.
__device__ __forceinline__ h16 load_b(const _Float16 *xs, const Geo &g, int j, int kofs)
{
    const _Float16 *p = xs + (16 * j + g.row) * g.LDW + kofs + 8 * g.q;
    h8 lo = *(const h8 *)p;
    h8 hi = *(const h8 *)(p + 32);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
}

template <int R, int J>
__device__ __forceinline__ void base_pass(const _Float16 *__restrict__ W, int K, const int (&rtc)[R], int kr0,
                                          int kr1, const _Float16 *xs, const Geo &g, f4 (&acc)[R][J])
{
    for (int kt = kr0; kt < kr1; ++kt) {
        h8 aw[R][4][2];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const _Float16 *wp = W + (size_t)(rtc[r] * 16 + g.row) * K + (size_t)kt * 256 + 8 * g.q;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                aw[r][st][0] = *(const h8 *)(wp + st * 64);
                aw[r][st][1] = *(const h8 *)(wp + st * 64 + 32);
            }
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
#pragma unroll
            for (int j = 0; j < J; ++j) {
                h16 b = load_b(xs, g, j, (kt - kr0) * 256 + st * 64);
                h8 b0 = __builtin_shufflevector(b, b, 0, 1, 2, 3, 4, 5, 6, 7);
                h8 b1 = __builtin_shufflevector(b, b, 8, 9, 10, 11, 12, 13, 14, 15);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aw[r][st][0], b0, acc[r][j], 0, 0, 0);
                    acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aw[r][st][1], b1, acc[r][j], 0, 0, 0);
                }
            }
        }
    }
}

// One delta's contribution for the sorted positions [sb, se) of this chunk, which overlap column
// blocks j0 .. j0 + C - 1.
template <int BITS, int GROUP, int R, int J, int C>
__device__ __forceinline__ void delta_pass(const uint8_t *__restrict__ blob, size_t off_idx, size_t off_scale,
                                           const int (&rtc)[R], int kr0, int kr1, const _Float16 *xs,
                                           const Geo &g, int j0, int sb, int se, f4 (&acc)[R][J])
{
    constexpr int GPT = 256 / GROUP;            // quantisation groups per tile row (2 or 4)
    f4 tmp[R][C];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int c = 0; c < C; ++c) tmp[r][c] = (f4){0.f, 0.f, 0.f, 0.f};

    for (int kt = kr0; kt < kr1; ++kt) {
        uint32_t cw[R][4];      // 4-bit: dword per step; 2-bit: [0],[1] hold two steps each
        uint32_t iw[R][2];
        uint32_t sz[R][GPT];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const size_t tile = (size_t)rtc[r] * g.KT + kt;
            const uint4 v = *(const uint4 *)(blob + tile * 1024 + (size_t)g.lane * 16);
            if (BITS == 4) {
                cw[r][0] = v.x; cw[r][1] = v.y; cw[r][2] = v.z; cw[r][3] = v.w;
                const uint2 iv = *(const uint2 *)(blob + off_idx + tile * 512 + (size_t)g.lane * 8);
                iw[r][0] = iv.x; iw[r][1] = iv.y;
            } else {
                cw[r][0] = v.x; cw[r][1] = v.y; cw[r][2] = 0; cw[r][3] = 0;
                iw[r][0] = v.z; iw[r][1] = v.w;
            }
            const uint8_t *sp = blob + off_scale + tile * (16 * GPT * 4) + (size_t)g.row * (GPT * 4);
            if (GPT == 2) {
                const uint2 s = *(const uint2 *)sp;
                sz[r][0] = s.x; sz[r][1] = s.y;
            } else {
                const uint4 s = *(const uint4 *)sp;
                sz[r][0] = s.x; sz[r][1] = s.y; sz[r][GPT - 2] = s.z; sz[r][GPT - 1] = s.w;
            }
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            h16 b[C];
#pragma unroll
            for (int c = 0; c < C; ++c) b[c] = load_b(xs, g, j0 + c, (kt - kr0) * 256 + st * 64);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t szw = sz[r][st * GPT / 4];
                const h2 sz2 = as_h2(szw);
                const h2 s2 = (h2){sz2.x, sz2.x};
                const h2 z2 = (h2){sz2.y, sz2.y};
                uint32_t w;
                if (BITS == 4) w = cw[r][st];
                else w = cw[r][st >> 1] >> (8 * (st & 1));
                const h8 a = dequant_step<BITS>(w, s2, z2);
                const int idxw = (int)iw[r][st >> 1];
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    if (st & 1) tmp[r][c] = smfmac<1>(a, b[c], tmp[r][c], idxw);
                    else tmp[r][c] = smfmac<0>(a, b[c], tmp[r][c], idxw);
                }
            }
        }
    }
    // merge: only the columns (sorted positions) that belong to this segment
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int pos = 16 * (j0 + c) + g.row;
        const bool in = pos >= sb && pos < se;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f4 t = tmp[r][c];
            if (!in) t = (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < J; ++j)
                if (j == j0 + c) acc[r][j] += t;
        }
    }
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

template <int BITS, int GROUP, int R, int J, bool HAS_BASE, bool HAS_DELTA>
__global__ __launch_bounds__(THREADS) void stream_kernel(DzStreamArgs a, DzDeltaPtrs dp, int NRB, int round_tiles,
                                                         size_t off_idx, size_t off_scale)
{
    extern __shared__ __attribute__((aligned(16))) _Float16 xs[];     // [16J][LDW]
    __shared__ int s_tok[64];
    __shared__ int s_seg_delta[64];
    __shared__ int s_seg_begin[65];
    __shared__ int s_nseg;
    __shared__ int s_last;

    const int tid = threadIdx.x;
    Geo g;
    g.lane = tid & 63; g.row = g.lane & 15; g.q = g.lane >> 4;
    g.KT = a.K >> 8;
    g.LDW = round_tiles * 256 + LDS_PAD;
    const int wave = tid >> 6;

    int unit = blockIdx.x;
    const int ks = unit % a.S; unit /= a.S;
    const int rb = unit % NRB;
    const int chunk = unit / NRB;
    const int kt0 = (int)((long long)ks * g.KT / a.S);
    const int kt1 = (int)((long long)(ks + 1) * g.KT / a.S);
    const int p0 = chunk * 64;
    const int cnt = min(64, a.T - p0);
    const int RT = a.N >> 4;

    // ---- this chunk's rows and delta segments (sorted order comes from the segment pass)
    if (tid < 64) {
        int tok = -1, key = INT_MAX;
        if (tid < cnt) {
            tok = a.perm ? a.perm[p0 + tid] : p0 + tid;
            if (HAS_DELTA && a.key) key = a.key[p0 + tid];
        }
        s_tok[tid] = tok;
        if (HAS_DELTA) {
            const bool valid = key >= 0 && key < a.D;
            const int prev = __shfl_up(key, 1, 64);
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
                s_seg_begin[ns] = __builtin_popcountll(vm);     // valid rows are a prefix of the chunk
            }
        }
    }

    int rtc[R];
    bool rvalid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int rt = rb * (WAVES * R) + wave * R + r;
        rvalid[r] = rt < RT;
        rtc[r] = rvalid[r] ? rt : RT - 1;
    }

    f4 acc[R][J];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < J; ++j) acc[r][j] = (f4){0.f, 0.f, 0.f, 0.f};

    const _Float16 *x = (const _Float16 *)a.x;
    for (int kr0 = kt0; kr0 < kt1; kr0 += round_tiles) {
        const int kr1 = min(kt1, kr0 + round_tiles);
        __syncthreads();                         // s_tok visible; previous round's readers done
        // ---- x[:, k-slice of this round] -> LDS, rows in sorted order, rows past cnt zero
        const int cpr = (kr1 - kr0) * 32;        // 16-byte pieces per row
        for (int i = tid; i < 16 * J * cpr; i += THREADS) {
            const int rr = i / cpr, cc = i - rr * cpr;
            const int tok = s_tok[rr];
            uint4 v = {0u, 0u, 0u, 0u};
            if (tok >= 0) v = *(const uint4 *)(x + (size_t)tok * a.K + (size_t)kr0 * 256 + cc * 8);
            *(uint4 *)(xs + rr * g.LDW + cc * 8) = v;
        }
        __syncthreads();

        if (HAS_BASE) base_pass<R, J>((const _Float16 *)a.W, a.K, rtc, kr0, kr1, xs, g, acc);

        if (HAS_DELTA) {
            const int nseg = s_nseg;
            for (int si = 0; si < nseg; ++si) {
                const int m = __builtin_amdgcn_readfirstlane(s_seg_delta[si]);
                const int sb = __builtin_amdgcn_readfirstlane(s_seg_begin[si]);
                const int se = __builtin_amdgcn_readfirstlane(s_seg_begin[si + 1]);
                const int j0 = sb >> 4;
                const int C = ((se - 1) >> 4) - j0 + 1;
                const uint8_t *blob = (const uint8_t *)dp.p[m];
                if (C == 1)
                    delta_pass<BITS, GROUP, R, J, 1>(blob, off_idx, off_scale, rtc, kr0, kr1, xs, g, j0, sb, se, acc);
                else if (J >= 2 && C == 2)
                    delta_pass<BITS, GROUP, R, J, (J >= 2 ? 2 : 1)>(blob, off_idx, off_scale, rtc, kr0, kr1, xs, g, j0, sb, se, acc);
                else if (J >= 3 && C == 3)
                    delta_pass<BITS, GROUP, R, J, (J >= 3 ? 3 : 1)>(blob, off_idx, off_scale, rtc, kr0, kr1, xs, g, j0, sb, se, acc);
                else if (J >= 4 && C == 4)
                    delta_pass<BITS, GROUP, R, J, (J >= 4 ? 4 : 1)>(blob, off_idx, off_scale, rtc, kr0, kr1, xs, g, j0, sb, se, acc);
            }
        }
    }

    // ---- results: lane 16q + c holds rows 4q..4q+3 of the row tile for request column c
    _Float16 *out = (_Float16 *)a.out;
    if (a.S == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!rvalid[r]) continue;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int tok = s_tok[16 * j + g.row];
                if (tok >= 0) store_row4(out + (size_t)tok * a.N + rtc[r] * 16 + 4 * g.q, acc[r][j], a.accumulate);
            }
        }
        return;
    }

    const int Tp = ((a.T + 63) >> 6) << 6;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (!rvalid[r]) continue;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int pr = 16 * j + g.row;
            if (pr < cnt)
                *(f4 *)(a.partial + ((size_t)ks * Tp + p0 + pr) * a.N + rtc[r] * 16 + 4 * g.q) = acc[r][j];
        }
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        int32_t *ctr = a.counters + chunk * NRB + rb;
        const int old = atomicAdd(ctr, 1);
        const int last = (old == a.S - 1);
        if (last) *ctr = 0;                      // ready for the next launch
        s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    const int width = WAVES * R * 16;            // rows of N per row block
    const int nq = width / 4;
    for (int i = tid; i < cnt * nq; i += THREADS) {
        const int pr = i / nq, c4 = i - pr * nq;
        const int n = rb * width + c4 * 4;
        if (n >= a.N) continue;
        f4 sum = (f4){0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < a.S; ++s)
            sum += *(const f4 *)(a.partial + ((size_t)s * Tp + p0 + pr) * a.N + n);
        const int tok = s_tok[pr];
        store_row4(out + (size_t)tok * a.N + n, sum, a.accumulate);
    }
}

template <int BITS, int GROUP, int R, int J, bool HB, bool HD>
hipError_t launch_one(const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int round_tiles, int grid,
                      size_t lds, const DzLayout &L, hipStream_t st)
{
    auto k = stream_kernel<BITS, GROUP, R, J, HB, HD>;
    static bool attr_set = false;       // per instantiation; the attribute is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 2048);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(k, dim3(grid), dim3(THREADS), lds, st, a, dp, NRB, round_tiles, L.off_idx, L.off_scale);
    return hipGetLastError();
}

template <int BITS, int GROUP, int R, bool HB, bool HD>
hipError_t launch_j(int J, const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int rt, int grid, size_t lds,
                    const DzLayout &L, hipStream_t st)
{
    switch (J) {
    case 1: return launch_one<BITS, GROUP, R, 1, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    case 2: return launch_one<BITS, GROUP, R, 2, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    case 3: return launch_one<BITS, GROUP, R, 3, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    default: return launch_one<BITS, GROUP, R, 4, HB, HD>(a, dp, NRB, rt, grid, lds, L, st);
    }
}

template <int R, bool HB, bool HD>
hipError_t launch_fmt(int bits, int group, int J, const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int rt,
                      int grid, size_t lds, const DzLayout &L, hipStream_t st)
{
    if (!HD) return launch_j<4, 128, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    if (bits == 4 && group == 128) return launch_j<4, 128, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    if (bits == 4) return launch_j<4, 64, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    if (group == 128) return launch_j<2, 128, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
    return launch_j<2, 64, R, HB, HD>(J, a, dp, NRB, rt, grid, lds, L, st);
}

}  // namespace

// Host side: choose the decomposition, make sure the workspace is large enough, launch.
int dz_ensure_partial(dz_ctx *ctx, size_t bytes, hipStream_t st);
int dz_ensure_counters(dz_ctx *ctx, int n, hipStream_t st);

int dz_launch_stream(dz_ctx *ctx, const DzStreamArgs &args, const DzDeltaPtrs &dp, hipStream_t st)
{
    DzStreamArgs a = args;
    constexpr int R = 2;
    const int RT = a.N / 16, KT = a.K / 256;
    const int nchunks = (a.T + 63) / 64;
    const int J = (a.T >= 64) ? 4 : (a.T + 15) / 16;
    const int NRB = (RT + WAVES * R - 1) / (WAVES * R);
    const long long units0 = (long long)nchunks * NRB;
    int S = ctx->force_splits > 0 ? ctx->force_splits : (int)((ctx->target_wgs + units0 - 1) / units0);
    if (S > KT) S = KT;
    if (S < 1) S = 1;
    const size_t Tp = (size_t)nchunks * 64;
    // keep the partial-sum workspace modest
    while (S > 1 && (size_t)S * Tp * a.N * 4 > ((size_t)256 << 20)) --S;
    int round_tiles = 2;
    const int max_slice = (KT + S - 1) / S;
    if (round_tiles > max_slice) round_tiles = max_slice;
    const size_t lds = (size_t)16 * J * (round_tiles * 256 + LDS_PAD) * sizeof(_Float16);
    a.S = S;
    if (S > 1) {
        int rc = dz_ensure_partial(ctx, (size_t)S * Tp * a.N * 4, st);
        if (rc) return rc;
        rc = dz_ensure_counters(ctx, (int)units0, st);
        if (rc) return rc;
    }
    a.partial = ctx->partial;
    a.counters = ctx->counters;
    const long long grid = units0 * S;
    if (grid > 0x7fffffffLL) return DZ_ERR_SHAPE;
    DzLayout L = dz_make_layout(a.N, a.K, a.has_delta ? a.bits : 4, a.has_delta ? a.group : 128);
    hipError_t e;
    if (a.has_base && a.has_delta)
        e = launch_fmt<R, true, true>(a.bits, a.group, J, a, dp, NRB, round_tiles, (int)grid, lds, L, st);
    else if (a.has_base)
        e = launch_fmt<R, true, false>(a.bits, a.group, J, a, dp, NRB, round_tiles, (int)grid, lds, L, st);
    else
        e = launch_fmt<R, false, true>(a.bits, a.group, J, a, dp, NRB, round_tiles, (int)grid, lds, L, st);
    return dz_set_hip_error(ctx, e);
}

// The tiled kernel for large batches (prefill): base GEMM + SBMM + merge, MFMA-bound.
//
//   out[t] = f16( x[t] . W^T + x[t] . Delta_{Idx[t]}^T )      (paper Section 5.1 Eq. (2); Section 5.2)
//
// With hundreds of request rows per delta the path is a dense contraction (the paper: prompt
// processing "is usually compute-bound", Section 2.1), so the kernel is organised around MFMA
// reuse instead of around HBM bytes:
//   * a workgroup (8 waves) owns an output tile of 256 rows of N x 128 request rows (in
//     delta-sorted order, from the segment pass) and the whole k range -- no split k;
//   * a wave owns 2 row tiles x 8 column blocks = 16 accumulator tiles (64 registers); W and
//     packed-delta fragments go from global memory straight into MFMA A operands (each wave owns
//     its rows, so A needs no sharing), the 128 x 256 slice of x of the current k tile sits in LDS
//     (double buffered, the next slice is fetched while the current one is multiplied) and every
//     B fragment read from LDS feeds 2 (dense: 4) MFMAs;
//   * deltas: contiguous segments of the sorted order; a segment multiplies only the column blocks
//     it overlaps, and in a block shared with a neighbour the foreign columns of B are zeroed, so
//     the sparse MFMAs accumulate into the same registers as the base product;
//   * workgroups are numbered so that the 16 request tiles of one row block run on the same XCD
//     at the same time and share its L2 copy of the W rows.
#include "dz_mma.h"

namespace {

constexpr int PJ = 8;               // column blocks (16 request rows) per workgroup
constexpr int PCH = 16 * PJ;        // request rows per workgroup tile
constexpr int PLDW = 256 + LDS_PAD; // LDS row stride in halfs (one k tile)

template <int BITS, int GROUP, int PR>
__device__ __forceinline__ void delta_steps_direct(const uint32_t (&st)[PR][Fmt<BITS, GROUP>::SD], const _Float16 *xs,
                                                   const Geo &g, const int (&brow)[PJ], int sb, int se,
                                                   f4 (&acc)[PR][PJ])
{
    typedef Fmt<BITS, GROUP> F;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        h8 av[PR];
        uint32_t idxw[PR];
#pragma unroll
        for (int r = 0; r < PR; ++r) {
            const h2 sz2 = as_h2(st[r][F::SC0 + s * F::GPT / 4]);
            const h2 s2 = (h2){sz2.x, sz2.x};
            const h2 z2 = (h2){sz2.y, sz2.y};
            uint32_t w;
            if (BITS == 4) { w = st[r][s]; idxw[r] = st[r][4 + (s >> 1)]; }
            else { w = st[r][s >> 1] >> (8 * (s & 1)); idxw[r] = st[r][2 + (s >> 1)]; }
            av[r] = dequant_step<BITS>(w, s2, z2);
        }
#pragma unroll
        for (int j = 0; j < PJ; ++j) {
            const int lo = 16 * j, hi = lo + 16;
            if (hi <= sb || lo >= se) continue;                 // block outside the segment (uniform)
            h16 b = load_b(xs, brow[j], g, s * 64);
            if (lo < sb || hi > se) {                           // block shared with a neighbour segment
                const int pos = lo + g.row;
                if (!(pos >= sb && pos < se)) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) b[e] = (_Float16)0.f;
                }
            }
#pragma unroll
            for (int r = 0; r < PR; ++r) {
                if (s & 1) acc[r][j] = smfmac<1>(av[r], b, acc[r][j], (int)idxw[r]);
                else acc[r][j] = smfmac<0>(av[r], b, acc[r][j], (int)idxw[r]);
            }
        }
    }
}

template <int BITS, int GROUP, int PW, int PR, bool HAS_BASE, bool HAS_DELTA>
__global__ __launch_bounds__(PW * 64) void prefill_kernel(DzStreamArgs a, DzDeltaPtrs dp, int NRB, int nchunks,
                                                          size_t off_idx, size_t off_scale, size_t blob_total)
{
    typedef Fmt<BITS, GROUP> F;
    constexpr int SD = F::SD;
    constexpr int THREADS = PW * 64;
    extern __shared__ __attribute__((aligned(16))) _Float16 xs_all[];     // 2 x [PCH][PLDW]
    __shared__ int s_tok[PCH];
    __shared__ int s_key[PCH];
    __shared__ unsigned long long s_dptr[DZ_MAX_DELTAS];
    __shared__ int s_seg_delta[PCH];
    __shared__ int s_seg_begin[PCH + 1];
    __shared__ int s_cnt[4];                // starts and valid rows of the first wave, number of segments

    const int tid = threadIdx.x;
    Geo g;
    g.lane = tid & 63; g.row = g.lane & 15; g.q = g.lane >> 4;
    g.KT = a.K >> 8;
    g.LDW = PLDW;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    LaneOffs lo;
    lo.w = (uint32_t)g.row * (uint32_t)a.K * 2u + (uint32_t)g.q * 16u;
    lo.c = (uint32_t)g.lane * 16u;
    lo.i = (uint32_t)g.lane * 8u;
    lo.s = (uint32_t)g.row * (uint32_t)(F::GPT * 4);

    // workgroup b runs on XCD b % 8: give each XCD a contiguous run of tiles, request tiles fastest
    const int total = NRB * nchunks;
    const int per_xcd = (total + 7) / 8;
    const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
    if (logical >= total) return;
    const int rb = logical / nchunks;
    const int chunk = logical - rb * nchunks;
    const int p0 = chunk * PCH;
    const int cnt = min(PCH, a.T - p0);
    const int RT = a.N >> 4;

    if (HAS_DELTA && tid < max(a.D, 1)) s_dptr[tid] = tid < a.D ? (unsigned long long)dp.p[tid] : (unsigned long long)a.x;
    if (tid < PCH) {
        int tok = -1, key = INT_MAX;
        if (tid < cnt) {
            tok = a.perm ? a.perm[p0 + tid] : p0 + tid;
            if (HAS_DELTA && a.key) key = a.key[p0 + tid];
        }
        s_tok[tid] = tok;
        s_key[tid] = key;
    }
    __syncthreads();
    // segments of this tile: starts found with one ballot per wave, numbered across the two waves
    bool start = false, valid = false;
    int key = INT_MAX;
    if (HAS_DELTA && tid < PCH) {
        key = s_key[tid];
        const int prev = tid ? s_key[tid - 1] : -1;
        valid = key >= 0 && key < a.D;
        start = valid && (tid == 0 || prev != key);
    }
    const unsigned long long sm = __ballot(start);
    const unsigned long long vm = __ballot(valid);
    if (tid == 0) { s_cnt[0] = __builtin_popcountll(sm); s_cnt[1] = __builtin_popcountll(vm); }
    __syncthreads();
    if (HAS_DELTA && tid < PCH) {
        const int base = (tid >= 64) ? s_cnt[0] : 0;
        if (start) {
            const int i = base + (int)lanes_below(sm);
            s_seg_delta[i] = key;
            s_seg_begin[i] = tid;
        }
        if (tid == 64) {
            const int ns = s_cnt[0] + __builtin_popcountll(sm);
            s_cnt[2] = ns;
            s_seg_begin[ns] = s_cnt[1] + __builtin_popcountll(vm);      // rows that name a delta are a prefix
        }
    }
    __syncthreads();
    const int nseg = HAS_DELTA ? s_cnt[2] : 0;

    int rtc[PR];
    bool rvalid[PR];
    uint32_t wrow[PR];
#pragma unroll
    for (int r = 0; r < PR; ++r) {
        const int rt = rb * (PW * PR) + wave * PR + r;
        rvalid[r] = rt < RT;
        rtc[r] = rvalid[r] ? rt : RT - 1;
        wrow[r] = (uint32_t)rtc[r] * 16u * (uint32_t)a.K * 2u;
    }
    int brow[PJ];
#pragma unroll
    for (int j = 0; j < PJ; ++j) brow[j] = (16 * j + g.row) * PLDW;

    f4 acc[PR][PJ];
#pragma unroll
    for (int r = 0; r < PR; ++r)
#pragma unroll
        for (int j = 0; j < PJ; ++j) acc[r][j] = (f4){0.f, 0.f, 0.f, 0.f};

    const _Float16 *x = (const _Float16 *)a.x;
    const uint32_t w_bytes = (uint32_t)a.N * (uint32_t)a.K * 2u;
    const uint32_t blob_bytes = (uint32_t)blob_total;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.W ? a.W : a.x, HAS_BASE ? w_bytes : 0u);

    // ---- x slice of one k tile -> LDS buffer: 128 rows x 32 pieces of 16 bytes, 16 per thread,
    // moved in four batches of four so that a batch can ride along with one MFMA step
    constexpr int XB = 4096 / THREADS / 4;  // pieces per thread and batch
    uint4 xv[XB];
    int xdst[XB];
#define PF_XLOAD(kt, batch)                                                                                        \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < XB; ++u) {                                                          \
            const int i = ((batch) * XB + u) * THREADS + tid;                                                       \
            const int rr = i >> 5, cc2 = i & 31;                                                                   \
            const int tok = s_tok[rr];                                                                             \
            xdst[u] = rr * PLDW + cc2 * 8;                                                                         \
            xv[u] = (uint4){0u, 0u, 0u, 0u};                                                                       \
            if (tok >= 0 && (kt) < g.KT) xv[u] = *(const uint4 *)(x + (size_t)tok * a.K + (size_t)(kt) * 256 + cc2 * 8); \
        }                                                                                                          \
    } while (0)
#define PF_XSTORE(buf)                                                                                             \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < XB; ++u) *(uint4 *)((buf) + xdst[u]) = xv[u];                       \
    } while (0)

    _Float16 *xcur = xs_all, *xnxt = xs_all + PCH * PLDW;
#pragma unroll 1
    for (int b = 0; b < 4; ++b) {
        PF_XLOAD(0, b);
        PF_XSTORE(xcur);
    }

    u32x4 bwA[PR][2], bwB[PR][2], bwC[PR][2], bwD[PR][2];
    uint32_t st0[PR][SD], st1[PR][SD];
    Cursor ci;                       // next delta tile to fetch: (segment, k tile)
    ci.kt = 0; ci.seg = 0;
    const int ndelta = nseg * g.KT;  // delta tiles this workgroup multiplies
    int ti = 0;
    // W prefetch distance: three steps when the registers allow it (no deltas), else one
    constexpr int DIST = HAS_DELTA ? 1 : 3;
    if constexpr (HAS_BASE) {
        base_issue<PR>(rw, wrow, lo.w, 0, bwA);
        if constexpr (DIST == 3) {
            base_issue<PR>(rw, wrow, lo.w, 1, bwB);
            base_issue<PR>(rw, wrow, lo.w, 2, bwC);
        }
    }
#define PF_DISSUE(buf)                                                                                             \
    do {                                                                                                           \
        delta_issue<BITS, GROUP, PR>(ci, ti < ndelta, g, rtc, lo, s_dptr, s_seg_delta, (uint32_t)off_idx,          \
                                     (uint32_t)off_scale, blob_bytes, buf);                                        \
        ++ti;                                                                                                      \
        if (++ci.seg >= nseg) { ci.seg = 0; ++ci.kt; }                                                             \
    } while (0)
    if constexpr (HAS_DELTA) PF_DISSUE(st0);
    __syncthreads();

    const int last_step = 4 * g.KT - 1;
    int parity = 0;
    for (int kt = 0; kt < g.KT; ++kt) {
        // ---- base: four steps of 64 k; each step also moves a quarter of the next x slice
#define PF_BSTEP(st_, cur, nxt)                                                                                    \
    do {                                                                                                           \
        PF_XLOAD(kt + 1, st_);                                                                                     \
        if constexpr (HAS_BASE) {                                                                                  \
            base_issue<PR>(rw, wrow, lo.w, min(kt * 4 + (st_) + DIST, last_step), nxt);                               \
            base_compute<PR, PJ>(cur, xcur, g, brow, (st_) * 64, acc);                                            \
        }                                                                                                          \
        PF_XSTORE(xnxt);                                                                                           \
    } while (0)
        if constexpr (DIST == 3) {
            PF_BSTEP(0, bwA, bwD);
            PF_BSTEP(1, bwB, bwA);
            PF_BSTEP(2, bwC, bwB);
            PF_BSTEP(3, bwD, bwC);
        } else {
            PF_BSTEP(0, bwA, bwB);
            PF_BSTEP(1, bwB, bwA);
            PF_BSTEP(2, bwA, bwB);
            PF_BSTEP(3, bwB, bwA);
        }
#undef PF_BSTEP
        // ---- deltas of this k tile, one packed tile per segment, the next one in flight.  The two
        // stage buffers swap roles whenever a k tile has an odd number of segments.
        if constexpr (HAS_DELTA) {
#define PF_DELTA(A, B)                                                                                             \
    do {                                                                                                           \
        for (int sg = 0; sg < nseg; sg += 2) {                                                                     \
            {                                                                                                      \
                PF_DISSUE(B);                                                                                      \
                const int sb = __builtin_amdgcn_readfirstlane(s_seg_begin[sg]);                                    \
                const int se = __builtin_amdgcn_readfirstlane(s_seg_begin[sg + 1]);                                \
                delta_steps_direct<BITS, GROUP, PR>(A, xcur, g, brow, sb, se, acc);                                    \
            }                                                                                                      \
            if (sg + 1 < nseg) {                                                                                   \
                PF_DISSUE(A);                                                                                      \
                const int sb = __builtin_amdgcn_readfirstlane(s_seg_begin[sg + 1]);                                \
                const int se = __builtin_amdgcn_readfirstlane(s_seg_begin[sg + 2]);                                \
                delta_steps_direct<BITS, GROUP, PR>(B, xcur, g, brow, sb, se, acc);                                    \
            }                                                                                                      \
        }                                                                                                          \
    } while (0)
            if (parity == 0) PF_DELTA(st0, st1);
            else PF_DELTA(st1, st0);
            parity ^= (nseg & 1);
#undef PF_DELTA
        }
        lds_barrier();                           // next slice complete, current slice no longer read
        _Float16 *t = xcur; xcur = xnxt; xnxt = t;
    }
#undef PF_XLOAD
#undef PF_XSTORE
#undef PF_DISSUE

    // ---- results: lane 16q + c holds rows 4q..4q+3 of each row tile for request column c
    _Float16 *out = (_Float16 *)a.out;
#pragma unroll
    for (int r = 0; r < PR; ++r) {
        if (!rvalid[r]) continue;
#pragma unroll
        for (int j = 0; j < PJ; ++j) {
            const int tok = s_tok[16 * j + g.row];
            if (tok >= 0) store_row4(out + (size_t)tok * a.N + rtc[r] * 16 + 4 * g.q, acc[r][j], a.accumulate);
        }
    }
}

template <int BITS, int GROUP, int PW, int PR, bool HB, bool HD>
hipError_t launch_pf(const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int nchunks, const DzLayout &L, hipStream_t st)
{
    auto k = prefill_kernel<BITS, GROUP, PW, PR, HB, HD>;
    const size_t lds = (size_t)2 * PCH * PLDW * sizeof(_Float16);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int total = NRB * nchunks;
    const int grid = ((total + 7) / 8) * 8;
    hipLaunchKernelGGL(k, dim3(grid), dim3(PW * 64), lds, st, a, dp, NRB, nchunks, L.off_idx, L.off_scale, L.total);
    return hipGetLastError();
}

template <int PW, int PR, bool HB, bool HD>
hipError_t launch_pf_fmt(const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int nchunks, const DzLayout &L, hipStream_t st)
{
    if (!HD || (a.bits == 4 && a.group == 128)) return launch_pf<4, 128, PW, PR, HB, HD>(a, dp, NRB, nchunks, L, st);
    if (a.bits == 4) return launch_pf<4, 64, PW, PR, HB, HD>(a, dp, NRB, nchunks, L, st);
    if (a.group == 128) return launch_pf<2, 128, PW, PR, HB, HD>(a, dp, NRB, nchunks, L, st);
    return launch_pf<2, 64, PW, PR, HB, HD>(a, dp, NRB, nchunks, L, st);
}

template <int PW, int PR>
hipError_t launch_pf_kind(const DzStreamArgs &a, const DzDeltaPtrs &dp, int nchunks, const DzLayout &L, hipStream_t st)
{
    const int NRB = (a.N / 16 + PW * PR - 1) / (PW * PR);
    if (a.has_base && a.has_delta) return launch_pf_fmt<PW, PR, true, true>(a, dp, NRB, nchunks, L, st);
    if (a.has_base) return launch_pf_fmt<PW, PR, true, false>(a, dp, NRB, nchunks, L, st);
    return launch_pf_fmt<PW, PR, false, true>(a, dp, NRB, nchunks, L, st);
}

}  // namespace

int dz_launch_prefill(dz_ctx *ctx, const DzStreamArgs &args, const DzDeltaPtrs &dp, hipStream_t st)
{
    DzStreamArgs a = args;
    const int nchunks = (a.T + PCH - 1) / PCH;
    if ((unsigned long long)a.N * a.K * 2ull >= (1ull << 32)) return DZ_ERR_SHAPE;     // 32-bit byte offsets
    DzLayout L = dz_make_layout(a.N, a.K, a.has_delta ? a.bits : 4, a.has_delta ? a.group : 128);
    hipError_t e;
    // 8 waves x 2 row tiles measured faster than 4 x 4 (two waves per SIMD hide each other's waits)
    if (ctx->wg_waves == 4) e = launch_pf_kind<4, 4>(a, dp, nchunks, L, st);
    else e = launch_pf_kind<8, 2>(a, dp, nchunks, L, st);
    return dz_set_hip_error(ctx, e);
}

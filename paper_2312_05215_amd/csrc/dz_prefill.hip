// The tiled kernel for large batches (prefill): base GEMM + SBMM + merge, MFMA-bound.
//
//   out[t] = f16( x[t] . W^T + x[t] . Delta_{Idx[t]}^T )      (paper Section 5.1 Eq. (2); Section 5.2)
//
// With hundreds of request rows per delta the path is a dense contraction (prompt processing is
// the compute-bound phase of serving, Section 2.1), so the kernel is organised around MFMA reuse
// instead of around HBM bytes:
//   * a workgroup (8 waves) owns an output tile of 256 rows of N x 128 request rows (in
//     delta-sorted order, from the segment pass) and the whole k range; the tiles of the last,
//     partly filled round of one-tile-per-CU are cut into slices of k that meet in fp32;
//   * a wave owns 2 row tiles x 8 column blocks = 16 accumulator tiles (64 registers); W and
//     packed-delta fragments go from global memory straight into MFMA A operands (each wave owns
//     its rows, so A needs no sharing), the 128 x 256 slice of x of the current k tile sits in LDS
//     (double buffered; the next slice is fetched in four batches that ride along with the four
//     base steps, each batch loaded one step before it is stored) and every B fragment read from
//     LDS feeds 4 dense or 2 sparse MFMAs;
//   * the order of loads and MFMAs is written out and pinned with scheduling fences: W one step
//     ahead (three without deltas), B fragments two column blocks ahead, the next packed tile
//     one delta ahead; a fused launch multiplies its delta tiles between the base steps of the
//     k tile, so the loads of the next steps are in flight during the delta work;
//   * deltas: contiguous segments of the sorted order; a segment multiplies only the column blocks
//     it overlaps, and in a block shared with a neighbour the lanes of foreign request rows read a
//     zero row of LDS, so the sparse MFMAs accumulate into the same registers as the base product;
//   * a tile whose request rows all name one delta runs a shorter loop: each step dequantises its
//     quarter of the packed tile and issues the sparse MFMAs of a column block right behind the
//     dense ones, on the B fragment those already hold;
//   * workgroups are numbered so that the request tiles of one row block run on the same XCD
//     at the same time and share its L2 copy of the W rows.
// Measured on the 13B shapes the kernel is bound by the rate at which L2 feeds the CUs (the tile
// moves 192 KB per 256 k), not by the MFMA pipes.
#include "dz_mma.h"


namespace {

constexpr int PLDW = 256 + LDS_PAD; // LDS row stride in halfs (one k tile)
constexpr int PFB = 2;              // column blocks by which the B fragment reads run ahead of their MFMAs
                                    // (3 measured the same, 4 spills)

// One base step (64 k) for R row tiles x J column blocks.  B fragments are read from LDS two
// column blocks ahead of the MFMAs that use them: bq holds the fragments of blocks j and j + 1 on
// entry and, when NEXT is set, those of blocks 0 and 1 of the following step on exit.
template <int R, int J, bool NEXT>
__device__ __forceinline__ void base_step(const u32x4 (&buf)[R][2], const _Float16 *xs, const Geo &g,
                                          const int (&brow)[J], int kofs, f4 (&acc)[R][J], h16 (&bq)[PFB])
{
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const h16 b = bq[j % PFB];
        if (j + PFB < J) bq[j % PFB] = load_b(xs, brow[j + PFB], g, kofs);
        else if (NEXT) bq[j % PFB] = load_b(xs, brow[j + PFB - J], g, kofs + 64);
        const h8 b0 = __builtin_shufflevector(b, b, 0, 1, 2, 3, 4, 5, 6, 7);
        const h8 b1 = __builtin_shufflevector(b, b, 8, 9, 10, 11, 12, 13, 14, 15);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, buf[r][0]), b0, acc[r][j], 0, 0, 0);
            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, buf[r][1]), b1, acc[r][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);      // keep the reads two blocks ahead of their MFMAs
    }
}

// One step of a tile whose request rows all belong to one delta: the B fragment a column block
// reads for the base product also feeds the sparse MFMA of the delta (av: the step's dequantised
// kept values, idxw: their positions, ODD: which half of idxw the step uses).
template <int R, int J, bool NEXT, int ODD, int NH>
__device__ __forceinline__ void fused_step(const u32x4 (&buf)[R][2], const h8 (&av)[NH][R], const uint32_t (&idxw)[NH][R],
                                           const _Float16 *xs, const Geo &g, const int (&brow)[J], int kofs,
                                           f4 (&acc)[R][J], h16 (&bq)[PFB])
{
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const h16 b = bq[j % PFB];
        if (j + PFB < J) bq[j % PFB] = load_b(xs, brow[j + PFB], g, kofs);
        else if (NEXT) bq[j % PFB] = load_b(xs, brow[j + PFB - J], g, kofs + 64);
        const h8 b0 = __builtin_shufflevector(b, b, 0, 1, 2, 3, 4, 5, 6, 7);
        const h8 b1 = __builtin_shufflevector(b, b, 8, 9, 10, 11, 12, 13, 14, 15);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, buf[r][0]), b0, acc[r][j], 0, 0, 0);
            acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, buf[r][1]), b1, acc[r][j], 0, 0, 0);
        }
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r][j] = smfmac<ODD>(av[h][r], b, acc[r][j], (int)idxw[h][r]);
        __builtin_amdgcn_sched_barrier(0);      // keep the reads two blocks ahead of their MFMAs
    }
}

// Dequantised kept values and positions of step s (half h) of a packed tile held in stage registers.
template <int BITS, int GROUP, bool QO, int R>
__device__ __forceinline__ void step_dequant(const uint32_t (&st)[R][Fmt<BITS, GROUP, QO>::SD], int s, int h, h8 (&av)[R],
                                             uint32_t (&idxw)[R])
{
    typedef Fmt<BITS, GROUP, QO> F;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const h2 sz2 = as_h2(st[r][F::SC0 + s * F::GPT / 4]);
        const h2 s2 = (h2){sz2.x, sz2.x};
        const h2 z2 = (h2){sz2.y, sz2.y};
        const uint32_t w = step_codes<BITS, QO>(st[r], s, h, idxw[r]);
        av[r] = dequant_step<BITS>(w, s2, z2);
    }
}

// Packed tile (16 rows x 256 k; half h of it) of R row tiles -> MFMA A operands of the four steps.
template <int BITS, int GROUP, bool QO, int R>
__device__ __forceinline__ void delta_dequant(const uint32_t (&st)[R][Fmt<BITS, GROUP, QO>::SD], int h, h8 (&av)[4][R],
                                              uint32_t (&idxw)[2][R])
{
    typedef Fmt<BITS, GROUP, QO> F;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const h2 sz2 = as_h2(st[r][F::SC0 + s * F::GPT / 4]);
            const h2 s2 = (h2){sz2.x, sz2.x};
            const h2 z2 = (h2){sz2.y, sz2.y};
            const uint32_t w = step_codes<BITS, QO>(st[r], s, h, idxw[s >> 1][r]);
            av[s][r] = dequant_step<BITS>(w, s2, z2);
        }
    }
}

// One delta's k tile against the column blocks its segment [sb, se) of the sorted request order
// overlaps.  A lane whose request row lies outside the segment reads the zero row instead, which
// removes that column from the product, so the sparse MFMAs can accumulate straight into the
// registers of the base product.  Blocks outside the segment are skipped by a wave-uniform branch;
// the four B fragments of a block are reloaded in place for the next overlapped block as soon as
// the MFMAs of the current one have taken them.
template <int R, int J>
__device__ __forceinline__ void delta_mm(const h8 (&av)[4][R], const uint32_t (&idxw)[2][R], const _Float16 *xs,
                                         int ldw, int zoff, const Geo &g, int sb, int se, f4 (&acc)[R][J])
{
    const int j0 = sb >> 4, j1 = (se - 1) >> 4;
    h16 b[4];
    {
        const int pos = 16 * j0 + g.row;
        const int bo = (pos >= sb && pos < se) ? pos * ldw : zoff;
#pragma unroll
        for (int s = 0; s < 4; ++s) b[s] = load_b(xs, bo, g, s * 64);
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
        if (j < j0 || j > j1) continue;                      // wave-uniform
        const int pos = 16 * min(j + 1, j1) + g.row;         // the last block re-reads itself (unused)
        const int bn = (pos >= sb && pos < se) ? pos * ldw : zoff;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (s & 1) acc[r][j] = smfmac<1>(av[s][r], b[s], acc[r][j], (int)idxw[s >> 1][r]);
                else acc[r][j] = smfmac<0>(av[s][r], b[s], acc[r][j], (int)idxw[s >> 1][r]);
            }
            b[s] = load_b(xs, bn, g, s * 64);
            __builtin_amdgcn_sched_barrier(0);  // reload right behind the MFMAs that took the fragment
        }
    }
}

template <int BITS, int GROUP, bool QO, int PW, int PR, int PJ, bool HAS_BASE, bool HAS_DELTA>
__global__ __launch_bounds__(PW * 64) void prefill_kernel(DzStreamArgs a, DzDeltaPtrs dp, int NRB, int nchunks,
                                                          size_t off_idx, size_t off_scale, size_t blob_total)
{
    typedef Fmt<BITS, GROUP, QO> F;
    constexpr int SD = F::SD;
    constexpr int THREADS = PW * 64;
    constexpr int PCH = 16 * PJ;            // request rows per workgroup tile
    extern __shared__ __attribute__((aligned(16))) _Float16 xs_all[];     // 2 x [PCH][PLDW], then one zero row
    __shared__ int s_tok[PCH];
    __shared__ int s_key[PCH];
    __shared__ unsigned long long s_dptr[DZ_MAX_DELTAS];
    __shared__ int s_seg_delta[PCH];
    __shared__ int s_seg_begin[PCH + 1];
    __shared__ int s_cnt[4];                // segment starts / rows with a delta seen by waves 0 and 1
    __shared__ int s_nseg;
    __shared__ int s_last;                  // this workgroup is the last k slice of its tile to arrive

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

    // Workgroup b runs on XCD b % 8, and workgroups start in the order of b.  Each XCD first gets a
    // contiguous run of I0 whole tiles (request tiles fastest, so the tiles of a row block share the
    // XCD's L2 copy of the W rows) -- together the full rounds of one tile per CU -- and then its
    // share of the remaining tiles cut into S slices of k each, so that the last, partly filled
    // round is short; the slices of a tile are neighbours and meet in fp32 at the end.
    const int I0 = a.max_slots, tiles = NRB * nchunks;
    const int Tt = (tiles - 8 * I0 + 7) / 8;            // sliced tiles per XCD
    const int xcd = (int)(blockIdx.x % 8), bi = (int)(blockIdx.x / 8);
    int tile, ks = 0, S = 1;
    if (bi < I0) {
        tile = xcd * I0 + bi;
        if (tile >= tiles) return;
    } else {
        S = a.S;
        const int tt = (bi - I0) / S;
        ks = (bi - I0) - tt * S;
        tile = 8 * I0 + xcd * Tt + tt;
        if (tt >= Tt || tile >= tiles) return;
    }
    const int slot0 = (tile - 8 * I0) * S;              // first partial-sum slot of a sliced tile
    const int rb = tile / nchunks;
    const int chunk = tile - rb * nchunks;
    const int kb = (int)((uint32_t)ks * (uint32_t)g.KT / (uint32_t)S);      // k tiles [kb, ke)
    const int ke = (int)((uint32_t)(ks + 1) * (uint32_t)g.KT / (uint32_t)S);
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
    if ((tid & 63) == 0 && tid < 128) { s_cnt[wave] = __builtin_popcountll(sm); s_cnt[2 + wave] = __builtin_popcountll(vm); }
    __syncthreads();
    if (HAS_DELTA && tid < PCH) {
        const int base = (tid >= 64) ? s_cnt[0] : 0;
        if (start) {
            const int i = base + (int)lanes_below(sm);
            s_seg_delta[i] = key;
            s_seg_begin[i] = tid;
        }
        if (tid == 0) {
            const int ns = s_cnt[0] + (PCH > 64 ? s_cnt[1] : 0);
            s_nseg = ns;
            s_seg_begin[ns] = s_cnt[2] + (PCH > 64 ? s_cnt[3] : 0);      // rows that name a delta are a prefix
        }
    }
    __syncthreads();
    const int nseg = HAS_DELTA ? s_nseg : 0;

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

    const uint32_t w_bytes = (uint32_t)a.N * (uint32_t)a.K * 2u;
    const uint32_t blob_bytes = (uint32_t)blob_total;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.W ? a.W : a.x, HAS_BASE ? w_bytes : 0u);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (uint32_t)a.T * (uint32_t)a.K * 2u);

    // ---- x slice of one k tile -> LDS buffer: PCH rows x 32 pieces of 16 bytes, moved in four
    // batches so that a batch can ride along with one MFMA step.  Piece p of a thread is row
    // p * THREADS / 32 + tid / 32, bytes 16 * (tid % 32) of the slice; rows past the end of the
    // batch get an offset beyond the resource, which the hardware answers with zeros.
    constexpr int XB = PCH * 32 / THREADS / 4;   // pieces per thread and batch
    uint32_t xoff[4 * XB];
#pragma unroll
    for (int p = 0; p < 4 * XB; ++p) {
        const int tok = s_tok[p * (THREADS / 32) + (tid >> 5)];
        xoff[p] = tok >= 0 ? (uint32_t)tok * (uint32_t)a.K * 2u + (uint32_t)(tid & 31) * 16u : 0x80000000u;
    }
    const int xdst0 = (tid >> 5) * PLDW + (tid & 31) * 8;
    u32x4 xvA[XB], xvB[XB];                      // two batches in flight: loaded a step before they are stored
#define PF_XLOAD(xv, kt, batch)                                                                                    \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < XB; ++u)                                                            \
            xv[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff[(batch) * XB + u], (uint32_t)(kt) * 512u, 0);  \
    } while (0)
#define PF_XSTORE(xv, buf, batch)                                                                                  \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < XB; ++u)                                                            \
            *(u32x4 *)((buf) + xdst0 + ((batch) * XB + u) * (THREADS / 32) * PLDW) = xv[u];                        \
    } while (0)

    _Float16 *xcur = xs_all, *xnxt = xs_all + PCH * PLDW;
    const int zoff = 2 * PCH * PLDW;         // the zero row, relative to either buffer's start: see below
    if (tid < PLDW / 8) *(u32x4 *)(xs_all + zoff + tid * 8) = (u32x4){0u, 0u, 0u, 0u};
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        PF_XLOAD(xvA, kb, b);
        PF_XSTORE(xvA, xcur, b);
    }
    PF_XLOAD(xvA, min(kb + 1, ke - 1), 0);

    u32x4 bwA[PR][2], bwB[PR][2], bwC[PR][2], bwD[PR][2];
    uint32_t st0[PR][SD];
    Cursor ci;                       // next delta tile to fetch: (segment, k tile)
    ci.kt = kb; ci.seg = 0;
    const int ndelta = nseg * (ke - kb);  // delta tiles this workgroup multiplies
    int ti = 0;
    // Fused launches multiply the delta tiles between the base steps of their k tile -- segment sg
    // after step sg % 4 -- so that the W and x loads each step sends out keep flowing during the
    // delta work; the W ring is then two buffers deep (one step ahead), which leaves the registers
    // for it.  Base-only launches prefetch W three steps ahead.
    constexpr bool ILV = HAS_BASE && HAS_DELTA;
    constexpr int DIST = ILV ? 1 : 3;          // W prefetch distance in steps
    if constexpr (HAS_BASE) {
        base_issue<PR>(rw, wrow, lo.w, 4 * kb, bwA);
        if constexpr (DIST == 3) {
            base_issue<PR>(rw, wrow, lo.w, 4 * kb + 1, bwB);
            base_issue<PR>(rw, wrow, lo.w, 4 * kb + 2, bwC);
        }
    }
    int cs = 0;                      // interleaved order: the step the fetch cursor is at
#define PF_DISSUE(buf)                                                                                             \
    do {                                                                                                           \
        delta_issue<BITS, GROUP, QO, PR>(ci, ti < ndelta, g, rtc, lo, s_dptr, s_seg_delta, (uint32_t)off_idx,          \
                                     (uint32_t)off_scale, blob_bytes, buf);                                        \
        ++ti;                                                                                                      \
        if constexpr (ILV) {                                                                                       \
            ci.seg += 4;                                                                                           \
            while (nseg > 0 && ci.seg >= nseg) {                                                                   \
                if (++cs == 4) { cs = 0; ++ci.kt; }                                                                \
                ci.seg = cs;                                                                                       \
            }                                                                                                      \
        } else {                                                                                                   \
            if (++ci.seg >= nseg) { ci.seg = 0; ++ci.kt; }                                                         \
        }                                                                                                          \
    } while (0)
    if constexpr (HAS_DELTA) PF_DISSUE(st0);
    __syncthreads();

    const int last_step = 4 * ke - 1;
    // A tile whose request rows all name the same delta (long prompts: most tiles) runs the delta
    // product inside the base steps: one read of a B fragment from LDS feeds both.
    bool whole = false;
    if constexpr (ILV) whole = nseg == 1 && s_seg_begin[0] == 0 && s_seg_begin[1] >= cnt;
    whole = __builtin_amdgcn_readfirstlane(whole);
    if constexpr (ILV) {
        if (whole) {
            for (int kt = kb; kt < ke; ++kt) {
                const int ktn = min(kt + 1, ke - 1), ktnn = min(kt + 2, ke - 1);
                h16 bq[PFB];
#pragma unroll
                for (int u = 0; u < PFB; ++u) bq[u] = load_b(xcur, brow[u], g, 0);
#define PF_FSTEP(st_, cur, nxt, xcurv, xnxtv)                                                                      \
    do {                                                                                                           \
        PF_XLOAD(xnxtv, (st_) < 3 ? ktn : ktnn, ((st_) + 1) & 3);                                                  \
        base_issue<PR>(rw, wrow, lo.w, min(kt * 4 + (st_) + DIST, last_step), nxt);                                \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        h8 av[F::NH][PR];                                                                                          \
        uint32_t idxw[F::NH][PR];                                                                                  \
        _Pragma("unroll") for (int h = 0; h < F::NH; ++h) step_dequant<BITS, GROUP, QO, PR>(st0, st_, h, av[h], idxw[h]); \
        if ((st_) == 3) {       /* the stage registers are free: request the next k tile's packed tile */          \
            __builtin_amdgcn_sched_barrier(0);                                                                     \
            PF_DISSUE(st0);                                                                                        \
        }                                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        fused_step<PR, PJ, ((st_) < 3), ((st_) & 1), F::NH>(cur, av, idxw, xcur, g, brow, (st_) * 64, acc, bq);    \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        PF_XSTORE(xcurv, xnxt, st_);                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
    } while (0)
                PF_FSTEP(0, bwA, bwB, xvA, xvB);
                PF_FSTEP(1, bwB, bwA, xvB, xvA);
                PF_FSTEP(2, bwA, bwB, xvA, xvB);
                PF_FSTEP(3, bwB, bwA, xvB, xvA);
#undef PF_FSTEP
                lds_barrier();
                _Float16 *t = xcur; xcur = xnxt; xnxt = t;
            }
        }
    }
    for (int kt = kb; kt < (whole ? kb : ke); ++kt) {
        // x slices fetched past the last k tile repeat it and land in the idle buffer
        const int ktn = min(kt + 1, ke - 1), ktnn = min(kt + 2, ke - 1);
        // ---- base: four steps of 64 k; each step also moves a quarter of the next x slice
        h16 bq[PFB];
        if constexpr (HAS_BASE) {
#pragma unroll
            for (int u = 0; u < PFB; ++u) bq[u] = load_b(xcur, brow[u], g, 0);
        }
        // one delta's packed tile: expand it into MFMA operands, request the next tile into the
        // freed stage buffer, multiply
#define PF_DSEG(buf, sg_)                                                                                          \
    do {                                                                                                           \
        const int sb = __builtin_amdgcn_readfirstlane(s_seg_begin[sg_]);                                           \
        const int se = __builtin_amdgcn_readfirstlane(s_seg_begin[(sg_) + 1]);                                     \
        _Pragma("unroll") for (int h = 0; h < F::NH; ++h) {                                                       \
            h8 av[4][PR];                                                                                          \
            uint32_t idxw[2][PR];                                                                                  \
            delta_dequant<BITS, GROUP, QO, PR>(buf, h, av, idxw);                                                  \
            __builtin_amdgcn_sched_barrier(0);                                                                     \
            if (h == F::NH - 1) PF_DISSUE(buf);     /* the stage registers are free for the next tile */           \
            __builtin_amdgcn_sched_barrier(0);                                                                     \
            delta_mm<PR, PJ>(av, idxw, xcur, PLDW, (int)(xs_all + zoff - xcur), g, sb, se, acc);                   \
        }                                                                                                          \
    } while (0)
#define PF_BSTEP(st_, cur, nxt, xcurv, xnxtv)                                                                      \
    do {                                                                                                           \
        PF_XLOAD(xnxtv, (st_) < 3 ? ktn : ktnn, ((st_) + 1) & 3);                                                  \
        if constexpr (HAS_BASE) {                                                                                  \
            base_issue<PR>(rw, wrow, lo.w, min(kt * 4 + (st_) + DIST, last_step), nxt);                            \
            __builtin_amdgcn_sched_barrier(0);      /* the loads go out before the step's MFMAs */                 \
            base_step<PR, PJ, ((st_) < 3)>(cur, xcur, g, brow, (st_) * 64, acc, bq);                              \
        }                                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        PF_XSTORE(xcurv, xnxt, st_);                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        if constexpr (ILV) {                                                                                       \
            for (int sg = (st_); sg < nseg; sg += 4) PF_DSEG(st0, sg);                                             \
        }                                                                                                          \
    } while (0)
        if constexpr (DIST == 3) {
            PF_BSTEP(0, bwA, bwD, xvA, xvB);
            PF_BSTEP(1, bwB, bwA, xvB, xvA);
            PF_BSTEP(2, bwC, bwB, xvA, xvB);
            PF_BSTEP(3, bwD, bwC, xvB, xvA);
        } else {
            PF_BSTEP(0, bwA, bwB, xvA, xvB);
            PF_BSTEP(1, bwB, bwA, xvB, xvA);
            PF_BSTEP(2, bwA, bwB, xvA, xvB);
            PF_BSTEP(3, bwB, bwA, xvB, xvA);
        }
#undef PF_BSTEP
        // ---- deltas of this k tile, one packed tile per segment
        if constexpr (HAS_DELTA) {
            if constexpr (!ILV) {
                for (int sg = 0; sg < nseg; ++sg) PF_DSEG(st0, sg);
            }
        }
#undef PF_DSEG
        lds_barrier();                           // next slice complete, current slice no longer read
        _Float16 *t = xcur; xcur = xnxt; xnxt = t;
    }
#undef PF_XLOAD
#undef PF_XSTORE
#undef PF_DISSUE

    // ---- k slices of one tile meet in fp32: every slice stores its accumulators (agent-scope
    // stores, register by register so that a store instruction writes 8 KB in a row), waits for
    // them, and bumps the tile's arrival counter; the last one adds the slices in slice order --
    // its own from registers -- so the sum does not depend on who arrives last.
    if (S > 1) {
        constexpr int AGENT = 0x10;
        const uint32_t tile_bytes = (uint32_t)(PR * PJ) * THREADS * 16u;
        const __amdgpu_buffer_rsrc_t prs = make_rsrc(a.partial, (uint32_t)(8 * Tt * S) * tile_bytes);
        const uint32_t lane_off = (uint32_t)tid * 16u;
#pragma unroll
        for (int r = 0; r < PR; ++r)
#pragma unroll
            for (int j = 0; j < PJ; ++j)
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[r][j]), prs,
                                                       lane_off + (uint32_t)(r * PJ + j) * THREADS * 16u,
                                                       (uint32_t)(slot0 + ks) * tile_bytes, AGENT);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid == 0) {
            int32_t *ctr = a.counters + (tile - 8 * I0);
            const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = (old == S - 1);
            if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
            s_last = last;
        }
        __syncthreads();
        if (!s_last) return;
#pragma unroll
        for (int r = 0; r < PR; ++r)
#pragma unroll
            for (int j = 0; j < PJ; ++j) {
                f4 sum = (f4){0.f, 0.f, 0.f, 0.f};
                for (int sl = 0; sl < S; ++sl) {
                    f4 v = acc[r][j];
                    if (sl != ks)
                        v = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(
                                                       prs, lane_off + (uint32_t)(r * PJ + j) * THREADS * 16u,
                                                       (uint32_t)(slot0 + sl) * tile_bytes, AGENT));
                    sum += v;
                }
                acc[r][j] = sum;
            }
    }
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

template <int BITS, int GROUP, bool QO, int PW, int PR, int PJ, bool HB, bool HD>
hipError_t launch_pf(const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int nchunks, const DzLayout &L, hipStream_t st)
{
    auto k = prefill_kernel<BITS, GROUP, QO, PW, PR, PJ, HB, HD>;
    const size_t lds = (size_t)(2 * 16 * PJ + 1) * PLDW * sizeof(_Float16);
    static unsigned long long lds_allowed = 0;      // per instantiation
    const hipError_t e = dz_allow_lds((const void *)k, (int)lds, lds_allowed);
    if (e != hipSuccess) return e;
    const int tail = NRB * nchunks - 8 * a.max_slots;
    const int grid = 8 * (a.max_slots + ((tail + 7) / 8) * a.S);
    hipLaunchKernelGGL(k, dim3(grid), dim3(PW * 64), lds, st, a, dp, NRB, nchunks, L.off_idx, L.off_scale, L.total);
    return hipGetLastError();
}

template <bool QO, int PW, int PR, int PJ, bool HB, bool HD>
hipError_t launch_pf_fmt(const DzStreamArgs &a, const DzDeltaPtrs &dp, int NRB, int nchunks, const DzLayout &L, hipStream_t st)
{
    if (!HD) return launch_pf<4, 128, false, PW, PR, PJ, HB, HD>(a, dp, NRB, nchunks, L, st);
    if (a.bits == 4 && a.group == 128) return launch_pf<4, 128, QO, PW, PR, PJ, HB, HD>(a, dp, NRB, nchunks, L, st);
    if (a.bits == 4) return launch_pf<4, 64, QO, PW, PR, PJ, HB, HD>(a, dp, NRB, nchunks, L, st);
    if (a.group == 128) return launch_pf<2, 128, QO, PW, PR, PJ, HB, HD>(a, dp, NRB, nchunks, L, st);
    return launch_pf<2, 64, QO, PW, PR, PJ, HB, HD>(a, dp, NRB, nchunks, L, st);
}

template <int PW, int PR, int PJ>
hipError_t launch_pf_kind(dz_ctx *ctx, const DzStreamArgs &args, const DzDeltaPtrs &dp, const DzLayout &L, hipStream_t st,
                          int *rc)
{
    DzStreamArgs a = args;
    const int nchunks = (a.T + 16 * PJ - 1) / (16 * PJ);
    const int NRB = (a.N / 16 + PW * PR - 1) / (PW * PR);
    // One workgroup per CU: `tiles` tiles take ceil(tiles / CUs) rounds, the last one partly
    // filled.  The tiles of the full rounds run whole; those of the last round are cut into up to
    // four slices of k, as many as still fit the CUs at once (320 tiles on 256 CUs: 256 whole,
    // then 64 x 4 quarter tiles), and only they pay for the fp32 meeting.
    const int tiles = NRB * nchunks;
    int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    cus -= cus % 8;
    a.S = 1;
    a.max_slots = (tiles + 7) / 8;          // whole tiles per XCD: all of them
    if (ctx->force_splits > 0) {
        a.S = ctx->force_splits;
        a.max_slots = 0;
    } else if (cus >= 8 && tiles % cus != 0) {
        const int whole = (tiles / cus) * cus, tail = tiles - whole;
        int S = cus / tail;
        if (S > 4) S = 4;
        if (S > 1) { a.S = S; a.max_slots = whole / 8; }
    }
    if (a.S > a.K / 256) a.S = a.K / 256;
    const size_t tile_bytes = (size_t)PR * PJ * PW * 64 * 16;
    const int sliced = 8 * ((tiles - 8 * a.max_slots + 7) / 8);
    if (a.S > 1 && (size_t)sliced * a.S * tile_bytes >= ((size_t)1 << 32)) a.S = 1;     // 32-bit byte offsets
    if (a.S <= 1) { a.S = 1; a.max_slots = (tiles + 7) / 8; }
    if (a.S > 1) {
        *rc = dz_ensure_partial(ctx, (size_t)sliced * a.S * tile_bytes, st);
        if (*rc == DZ_OK) *rc = dz_ensure_counters(ctx, sliced, st);
        if (*rc != DZ_OK) return hipSuccess;
    }
    a.partial = ctx->partial;
    a.counters = ctx->counters;
    if (a.has_delta && a.quant_only) {
        if (a.has_base) return launch_pf_fmt<true, PW, PR, PJ, true, true>(a, dp, NRB, nchunks, L, st);
        return launch_pf_fmt<true, PW, PR, PJ, false, true>(a, dp, NRB, nchunks, L, st);
    }
    if (a.has_base && a.has_delta) return launch_pf_fmt<false, PW, PR, PJ, true, true>(a, dp, NRB, nchunks, L, st);
    if (a.has_base) return launch_pf_fmt<false, PW, PR, PJ, true, false>(a, dp, NRB, nchunks, L, st);
    return launch_pf_fmt<false, PW, PR, PJ, false, true>(a, dp, NRB, nchunks, L, st);
}

}  // namespace

int dz_launch_prefill(dz_ctx *ctx, const DzStreamArgs &args, const DzDeltaPtrs &dp, hipStream_t st)
{
    DzStreamArgs a = args;
    if ((unsigned long long)a.N * a.K * 2ull >= (1ull << 32)) return DZ_ERR_SHAPE;     // 32-bit byte offsets
    if ((unsigned long long)a.T * a.K * 2ull >= (1ull << 31)) return DZ_ERR_SHAPE;     // x offsets, bit 31 = no row
    // The base product alone goes to the 256 x 256 tile kernel when that leaves enough tiles to keep
    // enough CUs busy (measured: faster from about 0.3 tiles per CU on, slower below); DZ_TILE=2 sends
    // every such call there, DZ_TILE=0 none.
    if (ctx->tile_kernel && dz_tile_fits(a)) {
        const long long wide_tiles = (long long)((a.N + 255) / 256) * ((a.T + 255) / 256);
        const int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
        if (ctx->tile_kernel > 1 || wide_tiles * 10 >= (long long)cus * 3) return dz_launch_tile(ctx, a, st);
    }
    DzLayout L = (a.has_delta && a.quant_only) ? dz_make_qlayout(a.N, a.K, a.bits, a.group)
                                               : dz_make_layout(a.N, a.K, a.has_delta ? a.bits : 4, a.has_delta ? a.group : 128);
    hipError_t e;
    int rc = DZ_OK;
    // 8 waves x 2 row tiles measured faster than 4 x 4 (two waves per SIMD hide each other's waits)
    e = launch_pf_kind<8, 2, 8>(ctx, a, dp, L, st, &rc);
    if (rc != DZ_OK) return rc;
    return dz_set_hip_error(ctx, e);
}

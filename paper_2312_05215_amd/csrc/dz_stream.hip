// The streaming kernel: base GEMM + SBMM for a small batch of request rows (decode), one launch.
//
//   out[t] = f16( x[t] . W^T + x[t] . Delta_{Idx[t]}^T )      (paper Section 5.1 Eq. (2); Section 5.2)
//
// Decode is bound by the bytes of W and of the packed deltas that must cross HBM once per call
// (Section 5.1: decode latency follows the memory footprint of the weights), so the kernel is
// organised around streaming those bytes exactly once with 16-byte loads per lane, and keeping
// everything else (x, dequantisation, 2:4 expansion, the merge of base and delta results) on chip:
//
//   * a workgroup of 8 waves owns, one after the other, the pieces of a contiguous range of the
//     (row block, k tile) grid; a wave owns one row tile (16 rows) of the row block at hand.  The
//     workgroup's slice of x sits in LDS (two buffers filled by buffer loads with an LDS destination)
//     and is the B operand of every MFMA; request rows are the MFMA N dimension, 16 per column block,
//     in delta-sorted order;
//   * base: W fragments go from global memory straight into the A operand of
//     V_MFMA_F32_16X16X32_F16 (lane 16q+r holds W[r][8q..8q+7], one 16-byte load);
//   * deltas: for each delta that has requests in the batch (segments of the sorted order; deltas
//     nobody asked for are never touched) the packed tile is loaded, codes are turned into fp16
//     pairs with a mask-or into the mantissa of 1024.0 and one packed fma, scaled, and fed with
//     the stored 2-bit positions to V_SMFMAC_F32_16X16X64_F16, the 2:4 sparse MFMA -- the sparse
//     expansion costs no instruction.  The product covers a window of two column blocks whose B
//     fragments stay in registers for all segments of a k tile; a per-lane select keeps it only for
//     the request columns of the segment;
//   * split-k partial sums meet in fp32: every workgroup stores its partial tile, the last one to
//     arrive for a row block (an arrival counter) adds them in fixed order and rounds to fp16
//     once.  With one slice the result is rounded and stored directly;
//   * several projections that read the same x (q,k,v or gate,up of a transformer layer) can share
//     one launch: their row blocks are numbered one projection after the other and each piece of
//     work looks up its projection's W, packed deltas and output.
//
// The paper's kernel launches per-delta child kernels from a parent kernel; HIP has no device-side
// launch, so "one launch for all deltas" is a loop over the batch's segment list inside each
// workgroup.  Batches of more than 64 rows normally go to the tiled kernel; when they are sent
// here they run as chunks of 64 sorted rows (a grid dimension).
#include "dz_mma.h"

namespace {

// ---- delta phase of the streaming kernel -------------------------------------------------------
// A task = one packed tile (16 rows x 256 k per row tile) of one delta segment.  The delta phase works
// on *windows* of two column blocks (32 sorted request positions).  The B fragments of one k tile for
// the window's column blocks and all four steps are held in registers (64 per wave) for as long as
// that k tile's segments are multiplied: every segment's sparse MFMAs read them from there, so the
// delta phase reads x from LDS once per k tile and window instead of once per segment.  A batch of
// more than 32 rows has two windows; the sorted order makes the segments that overlap a window a
// contiguous run of the segment list, so each window streams only its own segments' packed tiles (a
// segment that straddles position 32 is streamed by both).
//
// The tasks of a k tile are the *entries* of the batch: window 0's segments, then window 1's.  What a
// task needs to know about its entry sits in registers, entry e in lane e, and is fetched with a lane
// read: no LDS round trip and no cursor arithmetic stands between a task and its loads.
struct EntryTable {
    uint32_t plo, phi;      // packed-delta blob of the entry's delta (for the current projection)
    int rel;                // first sorted position of the segment, counted from the window's first position
    int lenf;               // rows of the segment | window << 8 | (first entry of its window) << 9
};
constexpr int WIN = 2;              // column blocks per window
constexpr int ENTRY_WINDOW = 0x100, ENTRY_FIRST = 0x200;

template <int JW>
__device__ __forceinline__ void load_window_frags(const _Float16 *xs, const int (&wrow)[WIN], const Geo &g, int kofs,
                                                  h16 (&bf)[4][WIN])
{
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < JW; ++j) bf[s][j] = load_b(xs, wrow[j], g, kofs + s * 64);
}

template <int BITS, int GROUP, bool QO, int R>
__device__ __forceinline__ void stream_delta_issue(int e, int kt, bool valid, const Geo &g, const int (&rtc)[R],
                                                   const LaneOffs &lo, const EntryTable &tab, uint32_t off_idx,
                                                   uint32_t off_scale, uint32_t blob_bytes,
                                                   uint32_t (&st)[R][Fmt<BITS, GROUP, QO>::SD])
{
    // With no task left the loads are still issued (so the load count never depends on a branch)
    // but against an empty resource: the hardware returns zeros and touches no memory.
    const uint32_t l = (uint32_t)__builtin_amdgcn_readlane((int)tab.plo, e);
    const uint32_t h = (uint32_t)__builtin_amdgcn_readlane((int)tab.phi, e);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc((const void *)(((unsigned long long)h << 32) | l), valid ? blob_bytes : 0u);
#pragma unroll
    for (int r = 0; r < R; ++r)
        tile_loads<BITS, GROUP, QO>(rs, (uint32_t)rtc[r] * (uint32_t)g.KT + (uint32_t)kt, lo, off_idx, off_scale, st[r]);
}

// The four steps of one packed tile (stage registers st) of a segment of `len` sorted positions that
// begins at position `rel` of the current window, whose accumulators are acc[.][0 .. JW-1].  The sparse
// MFMAs multiply all request columns of the window (the fragments in registers are not masked) into a
// copy of the accumulators; lanes whose request column lies in the segment then keep the copy, the
// others keep what they had: one select per accumulator register and task instead of a masked read of
// x per step.
template <int BITS, int GROUP, bool QO, int R, int JA, int JW>
__device__ __forceinline__ void stream_delta_task(const uint32_t (&st)[R][Fmt<BITS, GROUP, QO>::SD], int rel, int len,
                                                  const h16 (&bf)[4][WIN], const Geo &g, f4 (&acc)[R][JA])
{
    typedef Fmt<BITS, GROUP, QO> F;
    f4 tmp[R][JW];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < JW; ++j) tmp[r][j] = acc[r][j];
#pragma unroll
    for (int h = 0; h < F::NH; ++h)
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        h8 av[R];
        uint32_t idxw[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const h2 sz2 = as_h2(st[r][F::SC0 + s * F::GPT / 4]);
            const h2 s2 = (h2){sz2.x, sz2.x};
            const h2 z2 = (h2){sz2.y, sz2.y};
            const uint32_t w = step_codes<BITS, QO>(st[r], s, h, idxw[r]);
            av[r] = dequant_step<BITS>(w, s2, z2);
        }
#pragma unroll
        for (int j = 0; j < JW; ++j) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (s & 1) tmp[r][j] = smfmac<1>(av[r], bf[s][j], tmp[r][j], (int)idxw[r]);
                else tmp[r][j] = smfmac<0>(av[r], bf[s][j], tmp[r][j], (int)idxw[r]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < JW; ++j) {
        const bool in = (unsigned)(16 * j + g.row - rel) < (unsigned)len;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            acc[r][j].x = in ? tmp[r][j].x : acc[r][j].x;
            acc[r][j].y = in ? tmp[r][j].y : acc[r][j].y;
            acc[r][j].z = in ? tmp[r][j].z : acc[r][j].z;
            acc[r][j].w = in ? tmp[r][j].w : acc[r][j].w;
        }
    }
}

// The accumulators of the window the delta phase works on are always the first two column blocks'
// registers: entering the other window exchanges the two halves (and leaving it exchanges them back).
template <int R, int JA>
__device__ __forceinline__ void swap_windows(f4 (&acc)[R][JA])
{
    static_assert(JA == 2 * WIN, "two windows");
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < WIN; ++j) {
            const f4 t = acc[r][j];
            acc[r][j] = acc[r][WIN + j];
            acc[r][WIN + j] = t;
        }
}

// An LDS round holds the x rows of RT2 k tiles (8 for one column block, 4 for two, 2 for three or four:
// 66 KB either way), twice: while a round is multiplied, the x slice of the next one lands in the other
// buffer, written there by buffer loads with an LDS destination (no staging registers; one load
// instruction moves the 1 KB that two k tiles of one request row occupy).  DSTG: packed-tile stage
// buffers of the delta phase (3: two tiles in flight while one computes).
template <int J> struct RoundOf { static constexpr int TILES = (J == 1) ? 8 : (J == 2) ? 4 : 2; };
constexpr int DSTG = 3;
typedef __attribute__((address_space(3))) void lds_void;

template <int BITS, int GROUP, bool QO, int WAVES, int R, int J, bool HAS_BASE, bool HAS_DELTA>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
void stream_kernel(DzStreamArgs a, DzGroup gp, DzGroupPtrs dp, int NRB, int round_tiles)
{
    typedef Fmt<BITS, GROUP, QO> F;
    constexpr int SD = F::SD;
    constexpr int THREADS = WAVES * 64;
    constexpr int RT2 = RoundOf<J>::TILES;  // k tiles of x per LDS buffer
    constexpr int LDW = RT2 * 256 + LDS_PAD;
    constexpr int ZROW = 16 * J;            // an all-zero LDS row for column slots without a request
    constexpr int BUFH = (16 * J + 1) * LDW;        // halfs per x buffer: the request rows, then the zero row
    constexpr int XNI = 16 * J * (RT2 / 2) / WAVES; // LDS-destination loads per wave and round
    static_assert((16 * J * (RT2 / 2)) % WAVES == 0 && R == 1, "round geometry");
    constexpr int BDIST = 3;                // steps by which the W loads of the base phase run ahead
    extern __shared__ __attribute__((aligned(16))) _Float16 xs[];     // 2 x [16J + 1][LDW]
    __shared__ int s_tok[64];               // request row of each sorted position (-1: none)
    __shared__ int s_key[64];               // delta of each sorted position
    __shared__ int s_raw[64];
    __shared__ int s_rank[64];
    __shared__ int s_boff[64];              // LDS offset (halfs) of the x row of each sorted position
    __shared__ unsigned long long s_dptr[DZ_GROUP_PTRS];   // packed-delta pointers of every projection (copied from the arguments)
    __shared__ int s_seg_delta[64];
    __shared__ int s_seg_begin[65];
    __shared__ int s_nseg;
    __shared__ int s_last;

    const int tid = threadIdx.x;
    Geo g;
    g.lane = tid & 63; g.row = g.lane & 15; g.q = g.lane >> 4;
    g.KT = a.K >> 8;
    g.LDW = LDW;
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
    // (32-bit arithmetic: the host keeps (P + 1) * (G + 1) below 2^31; a 64-bit division is some 150
    // scalar instructions, and four of them stood between a workgroup and its first load)
    const uint32_t P = (uint32_t)NRB * (uint32_t)g.KT;
    const int p_begin = (int)((uint32_t)wg * P / (uint32_t)G);
    const int p_end = (int)((uint32_t)(wg + 1) * P / (uint32_t)G);
    const int p0 = chunk * 64;
    const int cnt = min(64, a.T - p0);

    // W ring of the base phase: named buffers (so each stays in registers), rotated by hand.  Inside a
    // piece the pipeline runs on across the rounds: when a round ends, the first three steps of the
    // next one are already in flight.  The very first weight loads of the workgroup go out here, before
    // anything else is set up: they take longest to arrive (first touch of this launch's weights) and
    // the rest of the start-up -- tables, the x slice, the ranking of the batch -- runs under them.
    u32x4 bw0[R][2], bw1[R][2], bw2[R][2], bw3[R][2];
    bool w_ahead = false;
    // row block and k tile the range starts at; the pieces that follow begin at k tile 0 of the next row block
    int rb_next = (int)((uint32_t)p_begin / (uint32_t)g.KT);
    int kt_next = p_begin - rb_next * g.KT;
    if (HAS_BASE && p_begin < p_end) {
        const int rb = rb_next;
        const int kt0 = kt_next;
        const int steps = 4 * min(g.KT - kt0, p_end - p_begin);
        int pj = 0;
        while (pj + 1 < gp.P && rb >= gp.rb_start[pj + 1]) ++pj;
        const int Np = gp.N[pj];
        const __amdgpu_buffer_rsrc_t rw = make_rsrc(gp.W[pj], (uint32_t)Np * (uint32_t)a.K * 2u);
        uint32_t wbase[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int rt = min((rb - gp.rb_start[pj]) * (WAVES * R) + wave * R + r, (Np >> 4) - 1);
            wbase[r] = ((uint32_t)rt * 16u * (uint32_t)a.K + (uint32_t)kt0 * 256u) * 2u;
        }
        base_issue<R>(rw, wbase, lo.w, 0, bw0);
        base_issue<R>(rw, wbase, lo.w, min(1, steps - 1), bw1);
        base_issue<R>(rw, wbase, lo.w, min(2, steps - 1), bw2);
        w_ahead = true;
    }

    // Request order (paper Section 5.2: requests of one delta are grouped).  Batches of up to 64
    // rows are ranked by every workgroup itself from the raw index vector (rank = rows with a
    // smaller delta + earlier rows of the same delta) -- no extra launch and no dependent load;
    // x then sits in LDS in request order and a lane finds the row of its column through s_boff.
    // Larger batches read the sorted order a segment pass left in the workspace and stage x rows
    // already sorted.
    const bool sort_here = HAS_DELTA && a.ids != nullptr;
    // this thread's entry of the packed-delta pointer table: requested now, written to LDS behind the
    // sort (a write here would have to wait for every load requested so far, the weights included)
    static_assert(DZ_GROUP_PTRS <= THREADS, "one pointer per thread");
    unsigned long long my_dptr = (unsigned long long)a.x;
    if (HAS_DELTA && tid < gp.P * a.D) my_dptr = (unsigned long long)dp.p[tid];
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
            s_boff[tid] = tid * LDW;
        }
        lds_barrier();
    }
    // the zero rows of both buffers (no load ever writes them)
    if (tid < LDW / 8) {
        *(uint4 *)(xs + ZROW * LDW + tid * 8) = (uint4){0u, 0u, 0u, 0u};
        *(uint4 *)(xs + BUFH + ZROW * LDW + tid * 8) = (uint4){0u, 0u, 0u, 0u};
    }

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (uint32_t)a.T * (uint32_t)a.K * 2u);
    constexpr int AGENT = 0x10;                  // cache-policy bit sc1
    const int Tp = ((a.T + 63) >> 6) << 6;
    const uint32_t slice_bytes = (uint32_t)Tp * (uint32_t)a.N * 4u;
    const __amdgpu_buffer_rsrc_t prs = make_rsrc(a.partial, slice_bytes * (uint32_t)a.max_slots);
    // ---- x[:, RT2 k tiles from kr on] -> LDS buffer bufi.  Unit u of the workgroup is request row
    // u / (RT2 / 2), bytes 1024 * (u % (RT2 / 2)) .. + 1023 of that row's slice: one load instruction, lane l
    // moving 16 bytes to LDS byte 16 l of the unit.  A row without a request, and the columns past the
    // end of a row, get an offset beyond the resource: the hardware touches no memory for them (what
    // lands in LDS there is never read: such columns belong to no k tile, such rows to no column slot).
    // The per-lane offsets of a wave's units never change (the rows are fixed once the request order is
    // known), so they are worked out once: a load then costs a handful of scalar instructions.
    uint32_t xvo[XNI];
#pragma unroll
    for (int i = 0; i < XNI; ++i) {
        const int row = (wave * XNI + i) / (RT2 / 2);
        const int tok = sort_here ? (row < cnt ? row : -1) : s_tok[row];
        xvo[i] = tok >= 0 ? (uint32_t)tok * (uint32_t)a.K * 2u + (uint32_t)g.lane * 16u : 0xFFFFFFF0u;
    }
    const bool upper_half = g.lane >= 32;        // lanes that move the second k tile of a unit
#define DZ_XDMA(bufi, kr)                                                                                          \
    do {                                                                                                           \
        _Pragma("unroll") for (int i = 0; i < XNI; ++i) {                                                         \
            const int u = wave * XNI + i;                                                                          \
            const int row = u / (RT2 / 2), piece = u % (RT2 / 2);                                                  \
            const int k0 = (kr) + 2 * piece;        /* the unit's k tiles are k0 and k0 + 1 */                     \
            const bool past = k0 >= g.KT || (upper_half && k0 + 1 >= g.KT);                                        \
            const uint32_t vo = past ? 0xFFFFFFF0u : xvo[i];                                                       \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void *)(xs + (bufi) * BUFH + row * LDW + piece * 512), 16, vo, \
                                                     (uint32_t)k0 * 512u, 0, 0);                                   \
        }                                                                                                          \
    } while (0)
    const int rtiles = (round_tiles > 0 && round_tiles < RT2) ? round_tiles : RT2;      // k tiles a round multiplies
    int xbuf = 0;                                // the buffer that holds the current round's x
    if (p_begin < p_end) DZ_XDMA(0, kt_next);
    bool tables_ready = !sort_here;
    bool first_round = true;
    int nseg = 0;
    // segments of the sorted order that overlap window 0 (positions 0 .. 31) and window 1 (32 .. 63)
    constexpr int NW = (J + WIN - 1) / WIN;
    int wlo1 = 0, ns0 = 0, ne = 0;               // window 1's first segment; entries of window 0, of both windows
    int brow[J];
#pragma unroll
    for (int j = 0; j < J; ++j) brow[j] = 0;

  for (int p = p_begin; p < p_end;) {
    const int rb = rb_next;
    const int kt0 = kt_next;
    const int kt1 = min(g.KT, kt0 + (p_end - p));
    p += kt1 - kt0;
    ++rb_next; kt_next = 0;                      // a piece that is not the last ends with its row block
    // the projection this row block belongs to (a call may carry several projections that share
    // x: their row blocks are numbered one projection after the other)
    int pj = 0;
    while (pj + 1 < gp.P && rb >= gp.rb_start[pj + 1]) ++pj;
    const int rbl = rb - gp.rb_start[pj];
    const int Np = gp.N[pj];
    const int RT = Np >> 4;
    const int n_off = gp.n_off[pj];
    const uint32_t off_idx = gp.off_idx[pj], off_scale = gp.off_scale[pj], blob_bytes = gp.blob_total[pj];
    const __amdgpu_buffer_rsrc_t rw =
        make_rsrc(HAS_BASE ? gp.W[pj] : a.x, HAS_BASE ? (uint32_t)Np * (uint32_t)a.K * 2u : 0u);
    _Float16 *out = (_Float16 *)gp.out[pj];
    const unsigned long long *sd = s_dptr + pj * a.D;
    int rtc[R];
    bool rvalid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int rt = rbl * (WAVES * R) + wave * R + r;
        rvalid[r] = rt < RT;
        rtc[r] = rvalid[r] ? rt : RT - 1;
    }
    // with two windows there are always four column blocks of accumulators (J = 3: the fourth is window 1's
    // unused second block, whose request positions lie in no segment)
    constexpr int JA = (NW > 1) ? 2 * WIN : J;
    constexpr int JW = (J < WIN) ? J : WIN;      // column blocks a delta task multiplies
    f4 acc[R][JA];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < JA; ++j) acc[r][j] = (f4){0.f, 0.f, 0.f, 0.f};
    for (int kr0 = kt0; kr0 < kt1; kr0 += rtiles) {
        const int kr1 = min(kt1, kr0 + rtiles);
        const int ntr = kr1 - kr0;
        const int nsteps = 4 * ntr;              // base steps of this round
        const int seg_last = 4 * (kt1 - kr0) - 1;    // last base step of the segment, counted from this round's start
        const _Float16 *xc = xs + xbuf * BUFH;   // this round's x
        // ---- the next round's x starts its way into the other buffer (everybody left that buffer at
        // the barrier that ended the previous round)
        {
            const int nk = kr1 < kt1 ? kr1 : 0;     // the next piece starts a row block
            if (kr1 < kt1 || p < p_end) DZ_XDMA(xbuf ^ 1, nk);
        }
        // Delta tasks of this round, in issue order: k tile by k tile, all entries per k tile (window 0's
        // segments, then window 1's).  Set after the sort in round one.
        int nd = ne * ntr;
        int ie = 0, ikt = kr0;                   // issue cursor: entry and k tile of the next task to request
        // named stage buffers, rotated by hand; entry and k tile (counted from the round's first) of the task
        // a buffer holds travel with it in scalars of their own
        uint32_t st0[R][SD], st1[R][SD], st2[R][SD];
        int de0 = 0, dk0 = 0, de1 = 0, dk1 = 0, de2 = 0, dk2 = 0;
        uint32_t wbase[R];
#pragma unroll
        for (int r = 0; r < R; ++r) wbase[r] = ((uint32_t)rtc[r] * 16u * (uint32_t)a.K + (uint32_t)kr0 * 256u) * 2u;
        int ti = 0, tc = 0;
        int wcur = 0;                            // the window whose accumulators are in front
        // the issue cursor walks the same order two tasks ahead of the multiplying one; past the end the
        // loads are issued against an empty resource
#define DZ_ISSUE(buf, de, dk)                                                                                      \
    do {                                                                                                           \
        stream_delta_issue<BITS, GROUP, QO, R>(ie, ikt, ti < nd, g, rtc, lo, tab, off_idx, off_scale, blob_bytes, buf); \
        de = ie; dk = ikt - kr0;                                                                                   \
        ++ti;                                                                                                      \
        const int wrap_ = (ie + 1 >= ne) ? 1 : 0;                                                                  \
        ie = wrap_ ? 0 : ie + 1;                                                                                   \
        ikt += wrap_;                                                                                              \
    } while (0)
        // (the empty asm statement keeps the exchange behind a real branch: as selects it would cost more
        // than the exchange itself at every start of a window)
#define DZ_STEP(cur, de, dk, nxt, den, dkn)                                                                        \
    do {                                                                                                           \
        DZ_ISSUE(nxt, den, dkn);                                                                                   \
        if (tc < nd) {                                                                                             \
            const int lenf = __builtin_amdgcn_readlane(tab.lenf, de);                                              \
            const int rel = __builtin_amdgcn_readlane(tab.rel, de);                                                \
            if (lenf & ENTRY_FIRST) {               /* new (window, k tile): its B fragments */                    \
                if constexpr (NW > 1) {                                                                            \
                    const int w_ = (lenf & ENTRY_WINDOW) ? 1 : 0;                                                  \
                    if (w_ != wcur) { asm volatile("; window switch"); swap_windows<R, JA>(acc); wcur = w_; }      \
                    const int wrow[WIN] = {w_ ? brow[WIN] : brow[0], w_ ? brow_last : brow[1]};                    \
                    load_window_frags<JW>(xc, wrow, g, (dk) * 256, bf);                                            \
                } else {                                                                                           \
                    const int wrow[WIN] = {brow[0], brow[JW - 1]};                                                 \
                    load_window_frags<JW>(xc, wrow, g, (dk) * 256, bf);                                            \
                }                                                                                                  \
            }                                                                                                      \
            stream_delta_task<BITS, GROUP, QO, R, JA, JW>(cur, rel, lenf & 0xff, bf, g, acc);                      \
        }                                                                                                          \
        ++tc;                                                                                                      \
    } while (0)
#define DZ_BSTEP(s, cur, nxt)                                                                                      \
    do {                                                                                                           \
        base_issue<R>(rw, wbase, lo.w, min((s) + BDIST, seg_last), nxt);                                           \
        base_compute<R, J, JA>(cur, xc, g, brow, (s) * 64, acc);                                                       \
    } while (0)
        if constexpr (HAS_BASE) {
            if (!w_ahead) {                      // first round of a segment: the weight loads start here and
                base_issue<R>(rw, wbase, lo.w, 0, bw0);             // fly while the batch is being sorted
                base_issue<R>(rw, wbase, lo.w, min(1, seg_last), bw1);
                base_issue<R>(rw, wbase, lo.w, min(2, seg_last), bw2);
            }
        }
        if (!tables_ready) {
            // ---- rank the batch (all threads; three short barriers)
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
                s_boff[r] = (tid < cnt ? tid : ZROW) * LDW;
            }
            lds_barrier();
        }
        if (first_round) {
            if (HAS_DELTA && tid < max(gp.P * a.D, 1)) s_dptr[tid] = my_dptr;
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
            // this wave's pieces of the first x slice have landed (and so have its first weight loads,
            // which the base phase needs at once anyway); after the barrier everybody's have
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            lds_barrier();
            tables_ready = true;
            nseg = HAS_DELTA ? s_nseg : 0;
            if constexpr (HAS_DELTA) {
                // the segments are in position order: those that begin below 32 come first (window 0's),
                // those that end above 32 come last (window 1's); one that does both is an entry of both
                const bool mine = g.lane < nseg;
                const int sbl = mine ? s_seg_begin[g.lane] : 0, sel = mine ? s_seg_begin[g.lane + 1] : 0;
                const unsigned long long m0 = __ballot(mine && sbl < 16 * WIN);
                const unsigned long long m1 = __ballot(mine && sel > 16 * WIN);
                ns0 = __builtin_popcountll(m0);
                ne = ns0;
                if (NW > 1 && m1) { wlo1 = (int)__builtin_ctzll(m1); ne += __builtin_popcountll(m1); }
            }
            nd = ne * ntr;
#pragma unroll
            for (int j = 0; j < J; ++j) brow[j] = s_boff[16 * j + g.row];
            first_round = false;
        }
        EntryTable tab = {0u, 0u, 0, 0};
        if constexpr (HAS_DELTA) {
            if (g.lane < ne) {                      // entry table: entry e in lane e
                const int w = g.lane >= ns0 ? 1 : 0;
                const int sg = w ? wlo1 + (g.lane - ns0) : g.lane;
                const unsigned long long bp = sd[s_seg_delta[sg]];
                const int sb = s_seg_begin[sg], se = s_seg_begin[sg + 1];
                tab.plo = (uint32_t)bp; tab.phi = (uint32_t)(bp >> 32);
                tab.rel = sb - 16 * WIN * w;
                tab.lenf = (se - sb) | (w ? ENTRY_WINDOW : 0) | ((g.lane == 0 || g.lane == ns0) ? ENTRY_FIRST : 0);
            }
            DZ_ISSUE(st0, de0, dk0);
            DZ_ISSUE(st1, de1, dk1);
        }
        if constexpr (HAS_BASE) {
            for (int s = 0; s < nsteps; s += 4) {
                DZ_BSTEP(s, bw0, bw3);
                DZ_BSTEP(s + 1, bw1, bw0);
                DZ_BSTEP(s + 2, bw2, bw1);
                DZ_BSTEP(s + 3, bw3, bw2);
            }
            w_ahead = true;                      // bw0 .. bw2 now hold (or await) steps 0 .. 2 of the next round
        }
        if constexpr (HAS_DELTA) {
            static_assert(DSTG == 3, "the rotation below is written for three stage buffers");
            h16 bf[4][WIN];
            // window 1's second column block does not exist with three column blocks: its lanes read zeros
            const int brow_last = (J > WIN + 1) ? brow[J - 1] : ZROW * LDW;
            while (tc < nd) {
                DZ_STEP(st0, de0, dk0, st2, de2, dk2);
                DZ_STEP(st1, de1, dk1, st0, de0, dk0);
                DZ_STEP(st2, de2, dk2, st1, de1, dk1);
            }
            if constexpr (NW > 1) {
                if (wcur) swap_windows<R, JA>(acc);      // the base phase and the epilogue want window 0 in front
            }
        }
#undef DZ_ISSUE
#undef DZ_STEP
#undef DZ_BSTEP
        // ---- end of the round: everybody is done with this round's x, and the next round's is complete.
        // A wave's pieces of it were requested before every weight load of this round; loads return
        // in order, so a wave that has consumed one of those has its pieces in LDS.  A launch without
        // a base product may have consumed nothing: it waits for whatever it still has in flight.
        if constexpr (!HAS_BASE) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        xbuf ^= 1;
    }
    w_ahead = false;                             // the next piece starts its own weight loads

    // ---- results of this segment: lane 16q + c holds rows 4q..4q+3 of the row tile for request
    // column c.  Which workgroups contribute to row block rb follows from the range formula:
    // the owner of flat position f is ceil((f + 1) * G / P) - 1.
    const int w_first = (int)((((uint32_t)rb * (uint32_t)g.KT + 1u) * (uint32_t)G + P - 1u) / P) - 1;
    const int w_last = (int)((((uint32_t)(rb + 1) * (uint32_t)g.KT) * (uint32_t)G + P - 1u) / P) - 1;
    const int ncontrib = w_last - w_first + 1;
    if (ncontrib == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!rvalid[r]) continue;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int tok = s_tok[16 * j + g.row];
                if (tok >= 0) store_row4(out + (size_t)tok * Np + rtc[r] * 16 + 4 * g.q, acc[r][j], a.accumulate);
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
                const uint32_t off = ((uint32_t)(p0 + pr) * (uint32_t)a.N + (uint32_t)(n_off + rtc[r] * 16) + 4u * g.q) * 4u;
                const u32x4 v = __builtin_bit_cast(u32x4, acc[r][j]);
                __builtin_amdgcn_raw_buffer_store_b128(v, prs, off, (uint32_t)slot * slice_bytes, AGENT);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0);               // this wave's stores have completed
    __syncthreads();
    if (tid == 0) {
        int32_t *ctr = a.counters + chunk * NRB + rb;
        const int old = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = (old == ncontrib - 1);
        if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
        s_last = last;
    }
    __syncthreads();
    if (s_last) {
        constexpr int width = WAVES * R * 16;        // rows of N per row block
        constexpr int nq = width / 4;
        for (int i = tid; i < cnt * nq; i += THREADS) {
            const int pr = i / nq, c4 = i - pr * nq;
            const int n = rbl * width + c4 * 4;
            if (n >= Np) continue;
            const uint32_t off = ((uint32_t)(p0 + pr) * (uint32_t)a.N + (uint32_t)(n_off + n)) * 4u;
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
            store_row4(out + (size_t)tok * Np + n, sum, a.accumulate);
        }
    }
  }   // segments
#undef DZ_XDMA
}

template <int BITS, int GROUP, bool QO, int WAVES, int R, int J, bool HB, bool HD>
hipError_t launch_one(const DzStreamArgs &a, const DzGroup &gp, const DzGroupPtrs &dp, int NRB, int round_tiles, int grid,
                      size_t lds, hipStream_t st)
{
    auto k = stream_kernel<BITS, GROUP, QO, WAVES, R, J, HB, HD>;
    static unsigned long long lds_allowed = 0;      // per instantiation
    const hipError_t e = dz_allow_lds((const void *)k, 160 * 1024 - 8192, lds_allowed);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, dim3(grid), dim3(WAVES * 64), lds, st, a, gp, dp, NRB, round_tiles);
    return hipGetLastError();
}

template <int BITS, int GROUP, bool QO, int WAVES, int R, bool HB, bool HD>
hipError_t launch_j(int J, const DzStreamArgs &a, const DzGroup &gp, const DzGroupPtrs &dp, int NRB, int rt, int grid,
                    size_t lds, hipStream_t st)
{
    switch (J) {
    case 1: return launch_one<BITS, GROUP, QO, WAVES, R, 1, HB, HD>(a, gp, dp, NRB, rt, grid, lds, st);
    case 2: return launch_one<BITS, GROUP, QO, WAVES, R, 2, HB, HD>(a, gp, dp, NRB, rt, grid, lds, st);
    case 3: return launch_one<BITS, GROUP, QO, WAVES, R, 3, HB, HD>(a, gp, dp, NRB, rt, grid, lds, st);
    default: return launch_one<BITS, GROUP, QO, WAVES, R, 4, HB, HD>(a, gp, dp, NRB, rt, grid, lds, st);
    }
}

template <bool QO, int WAVES, int R, bool HB, bool HD>
hipError_t launch_fmt(int bits, int group, int J, const DzStreamArgs &a, const DzGroup &gp, const DzGroupPtrs &dp, int NRB,
                      int rt, int grid, size_t lds, hipStream_t st)
{
    if (!HD) return launch_j<4, 128, false, WAVES, R, HB, HD>(J, a, gp, dp, NRB, rt, grid, lds, st);
    if (bits == 4 && group == 128) return launch_j<4, 128, QO, WAVES, R, HB, HD>(J, a, gp, dp, NRB, rt, grid, lds, st);
    if (bits == 4) return launch_j<4, 64, QO, WAVES, R, HB, HD>(J, a, gp, dp, NRB, rt, grid, lds, st);
    if (group == 128) return launch_j<2, 128, QO, WAVES, R, HB, HD>(J, a, gp, dp, NRB, rt, grid, lds, st);
    return launch_j<2, 64, QO, WAVES, R, HB, HD>(J, a, gp, dp, NRB, rt, grid, lds, st);
}

template <int WAVES, int R>
hipError_t launch_kind(const DzStreamArgs &a, int J, const DzGroup &gp, const DzGroupPtrs &dp, int NRB, int rt, int grid,
                       size_t lds, hipStream_t st)
{
    if (a.has_delta && a.quant_only) {
        if (a.has_base) return launch_fmt<true, WAVES, R, true, true>(a.bits, a.group, J, a, gp, dp, NRB, rt, grid, lds, st);
        return launch_fmt<true, WAVES, R, false, true>(a.bits, a.group, J, a, gp, dp, NRB, rt, grid, lds, st);
    }
    if (a.has_base && a.has_delta) return launch_fmt<false, WAVES, R, true, true>(a.bits, a.group, J, a, gp, dp, NRB, rt, grid, lds, st);
    if (a.has_base) return launch_fmt<false, WAVES, R, true, false>(a.bits, a.group, J, a, gp, dp, NRB, rt, grid, lds, st);
    return launch_fmt<false, WAVES, R, false, true>(a.bits, a.group, J, a, gp, dp, NRB, rt, grid, lds, st);
}

}  // namespace

// Host side: choose the decomposition, make sure the workspace is large enough, launch.

int dz_launch_stream(dz_ctx *ctx, const DzStreamArgs &args, const DzGroup &group, const DzGroupPtrs &dp, hipStream_t st)
{
    DzStreamArgs a = args;
    DzGroup gp = group;
    const int KT = a.K / 256;
    const int nchunks = (a.T + 63) / 64;
    const int J = (a.T >= 64) ? 4 : (a.T + 15) / 16;
    // workgroup shape: 8 waves x 1 row tile (the B fragments of a k tile fill 32 J registers of every
    // wave during the delta phase, which leaves room for one row tile's accumulators and stage buffers)
    constexpr int WAVES = 8, R = 1;
    // row blocks of the projections, one projection after the other; a row block never spans two
    int NRB = 0, n_total = 0;
    for (int p = 0; p < gp.P; ++p) {
        if ((unsigned long long)gp.N[p] * a.K * 2ull >= (1ull << 32)) return DZ_ERR_SHAPE;     // 32-bit byte offsets
        const DzLayout L = (a.has_delta && a.quant_only) ? dz_make_qlayout(gp.N[p], a.K, a.bits, a.group)
                                                         : dz_make_layout(gp.N[p], a.K, a.has_delta ? a.bits : 4, a.has_delta ? a.group : 128);
        gp.off_idx[p] = (uint32_t)L.off_idx; gp.off_scale[p] = (uint32_t)L.off_scale; gp.blob_total[p] = (uint32_t)L.total;
        gp.rb_start[p] = NRB;
        gp.n_off[p] = n_total;
        NRB += (gp.N[p] / 16 + WAVES * R - 1) / (WAVES * R);
        n_total += gp.N[p];
    }
    for (int p = gp.P; p <= DZ_MAX_GROUP; ++p) gp.rb_start[p] = NRB;
    a.N = n_total;                       // row length of the partial-sum tiles
    const long long units0 = (long long)nchunks * NRB;
    // number of workgroups per chunk: the target (a multiple of the CU count) unless the call has
    // fewer (row block, k tile) positions than that
    const long long P = (long long)NRB * KT;
    // Eight waves per CU (two per SIMD) stream fastest: one workgroup of 8 waves or two of 4 per CU;
    // twice as many waves measured 7-10 % slower on every decode shape
    const int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    const long long auto_wgs = (long long)cus * 8 / WAVES;
    long long G = ctx->force_splits > 0 ? (long long)ctx->force_splits * NRB : (ctx->target_wgs > 0 ? ctx->target_wgs : auto_wgs);
    if (G > P) G = P;
    if ((P + 1) * (G + 1) >= (1ll << 31)) G = (1ll << 31) / (P + 1) - 2;      // the kernel divides in 32 bits
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
    if ((unsigned long long)a.T * a.K * 2ull >= 0xFFFFFFF0ull) return DZ_ERR_SHAPE;
    // k tiles per round: what one of the two x buffers in LDS holds (RoundOf in the kernel), or fewer on request
    const int round_cap = (J == 1) ? 8 : (J == 2) ? 4 : 2;
    const int round_tiles = (ctx->round_tiles > 0 && ctx->round_tiles < round_cap) ? ctx->round_tiles : round_cap;
    const size_t lds = (size_t)2 * (16 * J + 1) * (round_cap * 256 + LDS_PAD) * sizeof(_Float16);
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
    hipError_t e;
    e = launch_kind<WAVES, R>(a, J, gp, dp, NRB, round_tiles, (int)grid, lds, st);
    return dz_set_hip_error(ctx, e);
}

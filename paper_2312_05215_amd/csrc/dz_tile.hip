// The wide tiled kernel for the base product of large batches (prefill):
//
//   out[t] = f16( x[t] . W^T )      (the batched base GEMM of paper Section 5.1 Eq. (2))
//
// What bounds a tiled kernel on this chip is the operand bytes a CU has to bring in per flop (a CU
// keeps only so many cache lines in flight, and they arrive with HBM latency), so the tile is as
// large as the registers allow and both operands travel the cheapest way:
//   * a workgroup (8 waves, 4 x 2) owns 256 rows of N x 256 request rows and walks k in steps of
//     64; a wave owns 4 row tiles x 8 column blocks = 32 accumulator tiles (128 registers), the
//     squarest wave tile, which needs the fewest fragment bytes from LDS per MFMA;
//   * the W and x slices of a step go from global memory straight into LDS (buffer loads with an
//     LDS destination: no staging registers, no LDS store instructions), double buffered, one
//     barrier per step.  Such a load writes the 64 lanes' 16-byte pieces side by side, so LDS rows
//     are unpadded 128-byte runs; to keep fragment reads off one bank set, slot s of row r holds
//     piece s ^ ((r >> 1) & 7) of the row -- the swizzle is applied to the global address a lane
//     fetches, and again by the lanes that read fragments.  A wave's load covers 8 rows x 128
//     bytes: whole cache lines.  A and B fragments of the MFMAs are read from LDS, B two column
//     blocks ahead of the MFMAs that use it;
//   * the tiles of the last, partly filled round of one-tile-per-CU are cut into k slices that
//     meet in fp32, as in the narrower tiled kernel.
// Fused and delta-only calls stay with the narrower kernel: with 128 registers of accumulators the
// packed-delta operands of a wave no longer fit beside them.
#include "dz_mma.h"


namespace {

constexpr int TLD = 64;             // LDS row stride in halfs of a 64-k slice (no padding: see the swizzle)
constexpr int TWR = 4, TWC = 2;     // waves along the rows of N and along the request rows
constexpr int TW = TWR * TWC;       // 8 waves
constexpr int TRT = 4;              // row tiles per wave
constexpr int TJ = 8;               // column blocks per wave
constexpr int TROWS = TWR * TRT * 16;   // 256 rows of N per tile
constexpr int TCH = TWC * TJ * 16;      // 256 request rows per tile
constexpr int TTHREADS = TW * 64;

__global__ __launch_bounds__(TTHREADS) void tile_kernel(DzStreamArgs a, int NRB, int nchunks)
{
    extern __shared__ __attribute__((aligned(16))) _Float16 lds[];     // W: 2 x [256][TLD]; x: 2 x [256][TLD]
    _Float16 *const ws = lds;
    _Float16 *const xs = lds + 2 * TROWS * TLD;
    __shared__ int s_last;

    const int tid = threadIdx.x;
    Geo g;
    g.lane = tid & 63; g.row = g.lane & 15; g.q = g.lane >> 4;
    g.KT = a.K >> 8;
    g.LDW = TLD;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave % TWR, wc = wave / TWR;     // this wave's block of rows and of request rows

    // tile of this workgroup: as in the narrower tiled kernel (whole tiles first, XCD by XCD, then
    // the tiles of the last round cut into S slices of k)
    const int I0 = a.max_slots, tiles = NRB * nchunks;
    const int Tt = (tiles - 8 * I0 + 7) / 8;
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
    const int slot0 = (tile - 8 * I0) * S;
    const int rb = tile / nchunks;
    const int chunk = tile - rb * nchunks;
    const int kb = (int)((uint32_t)ks * (uint32_t)g.KT / (uint32_t)S);      // k tiles [kb, ke)
    const int ke = (int)((uint32_t)(ks + 1) * (uint32_t)g.KT / (uint32_t)S);
    const int p0 = chunk * TCH;
    const int RT = a.N >> 4;

    int rtc[TRT];
    bool rvalid[TRT];
#pragma unroll
    for (int r = 0; r < TRT; ++r) {
        const int rt = rb * (TWR * TRT) + wr * TRT + r;
        rvalid[r] = rt < RT;
        rtc[r] = rvalid[r] ? rt : RT - 1;
    }
    f4 acc[TRT][TJ];
#pragma unroll
    for (int r = 0; r < TRT; ++r)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[r][j] = (f4){0.f, 0.f, 0.f, 0.f};

    // ---- the W and x slices: piece u of a thread is row u * 64 + tid / 8 of the slice, LDS slot
    // tid % 8 of that row, which holds global piece (tid % 8) ^ ((row >> 1) & 7).  A wave's 64
    // lanes cover 8 consecutive rows = 1 KB of LDS in lane order, as the LDS-destination load
    // writes it.  Rows that do not exist get an offset beyond the resource (the hardware reads
    // zeros; whatever lands in LDS for them only reaches output rows that are never stored).
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.W, (uint32_t)a.N * (uint32_t)a.K * 2u);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (uint32_t)a.T * (uint32_t)a.K * 2u);
    uint32_t woff[4], xoff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int r = u * 64 + (tid >> 3);
        const uint32_t c = (uint32_t)((tid & 7) ^ ((r >> 1) & 7)) * 16u;
        const int n = rb * TROWS + r, t = p0 + r;
        woff[u] = n < a.N ? (uint32_t)n * (uint32_t)a.K * 2u + c : 0x80000000u;
        xoff[u] = t < a.T ? (uint32_t)t * (uint32_t)a.K * 2u + c : 0x80000000u;
    }
    typedef __attribute__((address_space(3))) void lds_void;
#define TK_LOAD(buf, step)                                                                                         \
    do {                                                                                                           \
        _Pragma("unroll") for (int u = 0; u < 4; ++u) {                                                           \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void *)(ws + (buf) * TROWS * TLD + (u * 64 + wave * 8) * TLD), \
                                                     16, woff[u], (uint32_t)(step) * 128u, 0, 0);                  \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void *)(xs + (buf) * TCH * TLD + (u * 64 + wave * 8) * TLD),   \
                                                     16, xoff[u], (uint32_t)(step) * 128u, 0, 0);                  \
        }                                                                                                          \
    } while (0)

    const int s_first = 4 * kb, s_final = 4 * ke - 1;
    TK_LOAD(0, s_first);

    const int sw = (g.row >> 1) & 7;                 // swizzle of this lane's fragment rows (row & 15 decides it)
    const int f0 = (g.q ^ sw) * 8, f1 = ((g.q + 4) ^ sw) * 8;      // slots of k 8q.. and 32 + 8q.. (halfs)
    const int aoff = (wr * TRT * 16 + g.row) * TLD;
    const int boff = (wc * TJ * 16 + g.row) * TLD;
    // One step: wait for the slice, request the next one into the other buffer, multiply.  A
    // workgroup walks a multiple of four steps, so the loop is unrolled by two and the buffer of a
    // step is known at compile time (all LDS addresses become immediates).
#define TK_STEP(BUF, step)                                                                                         \
    do {                                                                                                           \
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  /* this wave's pieces of slice `step` are in LDS */      \
        lds_barrier();                       /* everybody's are, and slice step - 1 is no longer read */           \
        TK_LOAD((BUF) ^ 1, min((step) + 1, s_final));                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        const _Float16 *wb = ws + (BUF) * TROWS * TLD;                                                             \
        const _Float16 *xb = xs + (BUF) * TCH * TLD;                                                               \
        h8 af[TRT][2];                                                                                             \
        _Pragma("unroll") for (int r = 0; r < TRT; ++r) {                                                         \
            af[r][0] = *(const h8 *)(wb + aoff + r * 16 * TLD + f0);                                               \
            af[r][1] = *(const h8 *)(wb + aoff + r * 16 * TLD + f1);                                               \
        }                                                                                                          \
        h8 bq[2][2];                                                                                               \
        bq[0][0] = *(const h8 *)(xb + boff + f0);                                                                  \
        bq[0][1] = *(const h8 *)(xb + boff + f1);                                                                  \
        bq[1][0] = *(const h8 *)(xb + boff + 16 * TLD + f0);                                                       \
        bq[1][1] = *(const h8 *)(xb + boff + 16 * TLD + f1);                                                       \
        _Pragma("unroll") for (int j = 0; j < TJ; ++j) {                                                          \
            const h8 b0 = bq[j & 1][0], b1 = bq[j & 1][1];                                                         \
            if (j + 2 < TJ) {                                                                                      \
                bq[j & 1][0] = *(const h8 *)(xb + boff + (j + 2) * 16 * TLD + f0);                                 \
                bq[j & 1][1] = *(const h8 *)(xb + boff + (j + 2) * 16 * TLD + f1);                                 \
            }                                                                                                      \
            _Pragma("unroll") for (int r = 0; r < TRT; ++r) {                                                     \
                acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[r][0], b0, acc[r][j], 0, 0, 0);              \
                acc[r][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[r][1], b1, acc[r][j], 0, 0, 0);              \
            }                                                                                                      \
            __builtin_amdgcn_sched_barrier(0);   /* keep the reads two blocks ahead of their MFMAs */               \
        }                                                                                                          \
    } while (0)
    for (int step = s_first; step <= s_final; step += 2) {
        TK_STEP(0, step);
        TK_STEP(1, step + 1);
    }
#undef TK_STEP
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // the last, redundant request has landed too
#undef TK_LOAD

    // ---- k slices of one tile meet in fp32 (as in the narrower tiled kernel): every slice stores
    // its accumulators with agent-scope stores, waits for them and bumps the tile's arrival
    // counter; the last one adds the slices in slice order, its own from registers.
    if (S > 1) {
        constexpr int AGENT = 0x10;
        const uint32_t tile_bytes = (uint32_t)(TRT * TJ) * TTHREADS * 16u;
        const __amdgpu_buffer_rsrc_t prs = make_rsrc(a.partial, (uint32_t)(8 * Tt * S) * tile_bytes);
        const uint32_t lane_off = (uint32_t)tid * 16u;
#pragma unroll
        for (int r = 0; r < TRT; ++r)
#pragma unroll
            for (int j = 0; j < TJ; ++j)
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[r][j]), prs,
                                                       lane_off + (uint32_t)(r * TJ + j) * TTHREADS * 16u,
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
        for (int r = 0; r < TRT; ++r)
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                f4 sum = (f4){0.f, 0.f, 0.f, 0.f};
                for (int sl2 = 0; sl2 < S; ++sl2) {
                    f4 v = acc[r][j];
                    if (sl2 != ks)
                        v = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(
                                                       prs, lane_off + (uint32_t)(r * TJ + j) * TTHREADS * 16u,
                                                       (uint32_t)(slot0 + sl2) * tile_bytes, AGENT));
                    sum += v;
                }
                acc[r][j] = sum;
            }
    }
    // ---- results: lane 16q + c holds rows 4q..4q+3 of each row tile for request column c
    _Float16 *out = (_Float16 *)a.out;
#pragma unroll
    for (int r = 0; r < TRT; ++r) {
        if (!rvalid[r]) continue;
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int tok = p0 + (wc * TJ + j) * 16 + g.row;
            if (tok < a.T) store_row4(out + (size_t)tok * a.N + rtc[r] * 16 + 4 * g.q, acc[r][j], a.accumulate);
        }
    }
}

hipError_t launch_tile(const DzStreamArgs &a, int NRB, int nchunks, hipStream_t st)
{
    const size_t lds = (size_t)(2 * TROWS + 2 * TCH) * TLD * sizeof(_Float16);
    static unsigned long long lds_allowed = 0;
    const hipError_t e = dz_allow_lds((const void *)tile_kernel, (int)lds, lds_allowed);
    if (e != hipSuccess) return e;
    const int tail = NRB * nchunks - 8 * a.max_slots;
    const int grid = 8 * (a.max_slots + ((tail + 7) / 8) * a.S);
    hipLaunchKernelGGL(tile_kernel, dim3(grid), dim3(TTHREADS), lds, st, a, NRB, nchunks);
    return hipGetLastError();
}

}  // namespace

// Does the wide kernel take this call?  Base product only, requests in their own order, and every
// real byte offset below 2^31 (its missing-row trick uses the upper half of the offset range).
bool dz_tile_fits(const DzStreamArgs &a)
{
    if (!a.has_base || a.has_delta || a.perm != nullptr) return false;
    return (unsigned long long)a.N * a.K * 2ull < (1ull << 31) && (unsigned long long)a.T * a.K * 2ull < (1ull << 31);
}

int dz_launch_tile(dz_ctx *ctx, const DzStreamArgs &args, hipStream_t st)
{
    DzStreamArgs a = args;
    if (!dz_tile_fits(a)) return DZ_ERR_SHAPE;
    const int nchunks = (a.T + TCH - 1) / TCH;
    const int NRB = (a.N + TROWS - 1) / TROWS;
    // one workgroup per CU: the tiles of the full rounds run whole, those of the last, partly
    // filled round are cut into up to four slices of k, as many as still fit the CUs at once
    const int tiles = NRB * nchunks;
    int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    cus -= cus % 8;
    a.S = 1;
    a.max_slots = (tiles + 7) / 8;
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
    const size_t tile_bytes = (size_t)TRT * TJ * TTHREADS * 16;
    const int sliced = 8 * ((tiles - 8 * a.max_slots + 7) / 8);
    if (a.S > 1 && (size_t)sliced * a.S * tile_bytes >= ((size_t)1 << 32)) a.S = 1;     // 32-bit byte offsets
    if (a.S <= 1) { a.S = 1; a.max_slots = (tiles + 7) / 8; }
    if (a.S > 1) {
        int rc = dz_ensure_partial(ctx, (size_t)sliced * a.S * tile_bytes, st);
        if (rc == DZ_OK) rc = dz_ensure_counters(ctx, sliced, st);
        if (rc != DZ_OK) return rc;
    }
    a.partial = ctx->partial;
    a.counters = ctx->counters;
    return dz_set_hip_error(ctx, launch_tile(a, NRB, nchunks, st));
}

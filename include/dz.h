/*
 * libdz -- the per-linear-layer hot path of delta serving on one AMD MI355X (gfx950).
 *
 * Many fine-tuned variants of one base model are served together.  Each variant is the base weight
 * plus a compressed delta; for one linear layer and a batch of T request rows (tokens) the layer
 * output is
 *
 *     out[t] = x[t] . W_base^T  +  x[t] . Delta_{Idx[t]}^T                  (Section 5.1, Eq. (2))
 *
 * i.e. one fp16 GEMM over the whole batch plus a selective batched matmul (SBMM, Section 5.2) in
 * which every row is multiplied by the delta its own request names.  A delta is 2:4 sparse along
 * the input dimension and stored as low-bit codes on a group-wise grid (Section 4.1, steps 2-3);
 * it is never expanded in device memory: the kernels dequantise and de-sparsify on the fly.
 *
 * Conventions
 *   W, Delta : [N][K] row-major, N = output features, K = input features (torch nn.Linear layout)
 *   x        : [T][K] fp16 row-major;  out : [T][N] fp16 row-major
 *   fp16 buffers are passed as const void* / void*; every pointer marked DEVICE must be device
 *   memory of the context's GPU, 16-byte aligned unless stated otherwise.
 *   Canonical (unpacked) delta tables, the library's input format for dz_pack_delta:
 *     codes u8 [N][K/2]  b-bit code of each kept value, two per group of four consecutive k
 *     idx   u8 [N][K/2]  position 0..3 of each kept value in its group of four; the two positions
 *                        of a group are distinct and ascending
 *     scale f16[N][K/G]  grid step of the G dense columns one quantisation group spans
 *     zero  f16[N][K/G]  integer zero-point (0 .. 2^b-1) of that grid, stored as fp16
 *   The value stored for kept entry j of group g in row n is
 *     (codes[n][2g+j] - zero[n][4g/G]) * scale[n][4g/G]   at column 4g + idx[n][2g+j].
 *
 * Shapes the kernels accept: bits in {2,4}; group in {64,128}; N % 16 == 0; K % 256 == 0;
 * 0 <= D <= DZ_MAX_DELTAS; T >= 0 (T == 0 is a no-op).  (The format itself only needs K % group == 0
 * and group % 4 == 0; the kernels stream whole tiles of 16 rows x 256 columns, and every layer shape
 * of the Llama family is a multiple of that.)
 *
 * Ownership and synchronisation: the caller owns every buffer it passes.  The library owns only
 * the workspace inside dz_ctx (segment tables, split-K partial sums, an error flag), which may grow
 * on a call that needs more than any earlier call (that growth allocates -- it does not wait for the
 * stream; the buffer it replaces stays allocated until dz_destroy, so launches still in flight keep it
 * and a HIP graph recorded before the growth can still be replayed).
 * A stream that is being captured into a HIP graph can be passed once an eager call with the same
 * shapes has sized the workspace: the calls then record only kernels.  A call that would have to
 * grow the workspace during a capture returns DZ_ERR_HIP and records nothing.
 * Otherwise all compute entry points only enqueue work on `stream` (a hipStream_t passed as
 * void*, NULL = the default stream) and return; nothing is synchronised except in dz_check and
 * dz_destroy.  One dz_ctx serves one stream at a time.  x and out must not overlap.
 *
 * Errors: every function returns DZ_OK (0) or a negative code; nothing throws, exits or prints.
 */
#ifndef DZ_H
#define DZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DZ_OK          0
#define DZ_ERR_ARG    (-1)  /* null pointer, negative count, D > DZ_MAX_DELTAS                      */
#define DZ_ERR_SHAPE  (-2)  /* N, K, group outside the accepted shapes listed above                  */
#define DZ_ERR_BITS   (-3)  /* bits not 2 or 4                                                       */
#define DZ_ERR_ALIGN  (-4)  /* a device pointer is not 16-byte aligned                               */
#define DZ_ERR_HIP    (-5)  /* the HIP runtime reported a failure (its text: dz_strerror on this thread) */
#define DZ_ERR_INDEX  (-6)  /* dz_check: some earlier call saw a request index outside [-1, D)       */
#define DZ_ERR_LIMIT  (-7)  /* the call needs more workspace than the entry point or context may use */

#define DZ_MAX_DELTAS 128   /* deltas resident for one call                                          */
#define DZ_MAX_GROUP  4     /* projections in one dz_linear_group call                               */
#define DZ_STATIC_PARTIAL_BYTES ((size_t)32 << 20)   /* split-k room of dz_linear_static                   */

typedef struct dz_ctx dz_ctx;

/* Text for a return code: static, except for DZ_ERR_HIP, where it carries the HIP runtime's own text of
 * the calling thread's last failure (a thread-local buffer, valid until that thread's next failure). */
const char *dz_strerror(int rc);
/* Text of the last HIP failure seen through this context ("" if none).  Valid until the next call. */
const char *dz_last_hip_error(const dz_ctx *ctx);

/* Create / destroy a context on GPU `device`.  dz_destroy synchronises the device. */
int dz_create(dz_ctx **ctx, int device);
int dz_destroy(dz_ctx *ctx);

/*
 * Per-context options.  The defaults are what the kernels were tuned with; the options exist so that
 * a test or a sweep can force a particular route through the kernels.  value >= 0; an unknown key or
 * a value the key does not take returns DZ_ERR_ARG and changes nothing.
 */
#define DZ_OPT_SPLIT_K               1  /* k slices per row block (streaming kernel) / per tile (tiled kernels); 0 = chosen per call */
#define DZ_OPT_WORKGROUPS            2  /* workgroups per launch of the streaming kernel; 0 = eight waves per compute unit            */
#define DZ_OPT_ROUND_TILES           3  /* k tiles of x a workgroup of the streaming kernel stages at once; 0 = as many as fit        */
#define DZ_OPT_LARGE_BATCH_STREAMING 4  /* 1 = batches of more than 64 rows also go through the streaming kernel, 64 rows at a time  */
#define DZ_OPT_WIDE_TILE             5  /* dz_base_gemm on large batches: 0 = never the 256 x 256 tile kernel, 1 = when it has enough
                                           tiles (default), 2 = always                                                                */
#define DZ_OPT_REUSE_SEGMENTS        6  /* 1 = the caller promises that a token_to_delta vector passed again at the same address
                                           with the same T and D is unchanged: consecutive large-batch calls of one layer then share
                                           one sort.  Setting the option (to either value) forgets the remembered order.             */
int dz_set_option(dz_ctx *ctx, int key, int value);

/*
 * Size in bytes of one packed delta: the kept values' codes, their 2-bit positions (Section 4.1:
 * step 2 keeps the non-zero values with a 2-bit position each, step 3 puts 32/b codes in a 32-bit
 * word) and one fp16 (scale, zero) pair per row and group:
 *     N*K*(2*bits + 4)/32  +  4*N*K/group.
 * Returns 0 for shapes the library does not accept.
 */
size_t dz_packed_bytes(int N, int K, int bits, int group);

/*
 * Lay one delta's canonical tables out in the order the kernels stream them (the packing step that
 * ends Algorithm 1).  All pointers DEVICE; codes/idx need no alignment beyond 1, scale/zero 2 bytes;
 * packed_out is caller-allocated, dz_packed_bytes() long, 16-byte aligned.  The packed layout is
 * private to the library but position independent: the bytes may be saved, copied and reloaded.
 * Table contents are not validated; codes are masked to `bits`, positions to 2 bits.
 */
int dz_pack_delta(dz_ctx *ctx, const uint8_t *codes, const uint8_t *idx, const void *scale_f16,
                  const void *zero_f16, int N, int K, int bits, int group, void *packed_out,
                  void *stream);

/*
 * The data-free compressor: a dense fp16 delta [N][K] (DEVICE, 8-byte aligned) -> the canonical tables
 * dz_pack_delta takes (all DEVICE, caller-allocated).  Section 4.1 step 2 prunes the delta to the 2:4
 * pattern and step 3 quantises the kept values; Algorithm 1 chooses mask and codes with calibration
 * data, this call applies the rule that needs none: per group of four keep the two entries of largest
 * magnitude (ties: the lower position), then per row and `group` dense columns an asymmetric uniform grid
 * that contains zero, rounded to nearest (half to even) in fp32:
 *   s = f16((hi - lo) / (2^bits - 1)) with lo = min(0, min v), hi = max(0, max v) over the group's kept
 *   values (s = 1, z = 0 if that is zero), z = clamp(rint((0 - lo) / s)) (never a negative zero), code = clamp(rint(v / s) + z).
 */
int dz_compress_delta(dz_ctx *ctx, const void *delta_f16, int N, int K, int bits, int group,
                      uint8_t *codes, uint8_t *idx, void *scale_f16, void *zero_f16, void *stream);

/*
 * Inverse of dz_pack_delta, for checking: any output may be NULL.  codes/idx/scale/zero reproduce
 * the canonical tables bit for bit; dense_f32 [N][K] is the matrix the delta stands for, computed
 * in fp32 (exact, see the value formula above).  All pointers DEVICE.
 */
int dz_unpack_delta(dz_ctx *ctx, const void *packed, int N, int K, int bits, int group,
                    uint8_t *codes, uint8_t *idx, void *scale_f16, void *zero_f16,
                    float *dense_f32, void *stream);

/*
 * Request reordering (Section 5.2, first optimisation: requests of the same delta are grouped
 * together).  Stable counting sort of token_to_delta (DEVICE int32 [T]) over D deltas:
 *   counts [D]   requests per delta
 *   offsets[D+1] exclusive prefix sum; offsets[D] = number of requests that name a delta
 *   perm   [T]   request indices, delta by delta, each delta's requests in original order;
 *                requests with an index outside [0, D) follow at the end in original order
 * Outputs DEVICE int32, 4-byte aligned, any may be NULL.  An index outside [-1, D) also raises
 * the sticky error that dz_check reports.  D <= 8192 here.
 */
int dz_segment(dz_ctx *ctx, const int32_t *token_to_delta, int T, int D, int32_t *counts,
               int32_t *offsets, int32_t *perm, void *stream);

/* out[t] = f16( x[t] . W^T ), fp32 accumulation: the batched base product of Eq. (2). */
int dz_base_gemm(dz_ctx *ctx, const void *x_f16, const void *W_f16, void *out_f16, int T, int N,
                 int K, void *stream);

/*
 * SBMM (Section 5.2): for every request t with m = token_to_delta[t] in [0, D),
 *   y[t] = x[t] . Delta_m^T  (fp32 accumulation over the kept entries),
 * all deltas of the batch in one launch; requests with m == -1 (or out of range) get y[t] = 0.
 *   accumulate == 0 : out[t] = f16(y[t]);   accumulate != 0 : out[t] = f16(float(out[t]) + y[t]).
 * packed_deltas is a HOST array of D DEVICE pointers (read before the call returns), each a
 * dz_pack_delta result for the same N, K, bits, group.  Deltas no request names are not read.
 */
int dz_sbmm(dz_ctx *ctx, const void *x_f16, const void *const *packed_deltas, int D,
            const int32_t *token_to_delta, void *out_f16, int T, int N, int K, int bits, int group,
            int accumulate, void *stream);

/*
 * Fused linear layer (Section 5.1: base and delta results are merged after each linear layer):
 *   out[t] = f16( x[t] . W^T + x[t] . Delta_{token_to_delta[t]}^T ),
 * both terms accumulated in fp32 and rounded to fp16 once.  Arguments as in dz_sbmm.
 */
int dz_linear(dz_ctx *ctx, const void *x_f16, const void *W_f16, const void *const *packed_deltas,
              int D, const int32_t *token_to_delta, void *out_f16, int T, int N, int K, int bits,
              int group, void *stream);

/*
 * Low-rank adapters in place of deltas (Section 3.2: adapters are registered and served next to deltas;
 * Section 6.4).  For every request t with m = token_to_adapter[t] in [0, D)
 *   y[t] = B_m . (A_m . x[t]),   A_m f16 [rank][K],  B_m f16 [N][rank],  fp32 accumulation,
 * requests with m == -1 (or out of range, which dz_check reports) get y[t] = 0;
 *   accumulate == 0 : out[t] = f16(y[t]);   accumulate != 0 : out[t] = f16(float(out[t]) + y[t]),
 * so a base product or a dz_linear result can be completed in place.  A and B are HOST arrays of D
 * DEVICE pointers (16-byte aligned, read before the call returns).  rank in {8, 16, ..., 64};
 * K % 8 == 0; N % 4 == 0; out 8-byte aligned.  The batch is walked in adapter-sorted order.
 */
int dz_lora_sbmm(dz_ctx *ctx, const void *x_f16, const void *const *A_f16, const void *const *B_f16, int D,
                 int rank, const int32_t *token_to_adapter, void *out_f16, int T, int N, int K,
                 int accumulate, void *stream);

/*
 * Two variants of the compressed product, kept for the comparison the paper's compressed-matmul
 * microbenchmark makes (Section 4.1: 2:4 sparsity on top of quantisation against quantisation alone
 * at inputs of 1 .. 4096 rows) and for serving a single variant from a merged weight.
 *
 * Quantisation-only deltas (Section 4.1 step 3 without step 2): every column has a b-bit code,
 *   value[n][k] = (codes[n][k] - zero[n][k / group]) * scale[n][k / group],
 * codes u8 [N][K], scale / zero f16 [N][K / group] (all DEVICE).  dz_qpacked_bytes =
 * N*K*bits/8 + 4*N*K/group.  dz_qpack_delta / dz_qunpack_delta are bit-exact inverses
 * (dense_f32 [N][K], any output may be NULL); dz_qsbmm and dz_qlinear are dz_sbmm and dz_linear over
 * blobs of this format (same arguments, shapes, index semantics and rounding).
 */
size_t dz_qpacked_bytes(int N, int K, int bits, int group);
int dz_qpack_delta(dz_ctx *ctx, const uint8_t *codes, const void *scale_f16, const void *zero_f16, int N, int K,
                   int bits, int group, void *packed_out, void *stream);
int dz_qunpack_delta(dz_ctx *ctx, const void *packed, int N, int K, int bits, int group, uint8_t *codes,
                     void *scale_f16, void *zero_f16, float *dense_f32, void *stream);
int dz_qsbmm(dz_ctx *ctx, const void *x_f16, const void *const *qpacked_deltas, int D,
             const int32_t *token_to_delta, void *out_f16, int T, int N, int K, int bits, int group,
             int accumulate, void *stream);
int dz_qlinear(dz_ctx *ctx, const void *x_f16, const void *W_f16, const void *const *qpacked_deltas, int D,
               const int32_t *token_to_delta, void *out_f16, int T, int N, int K, int bits, int group,
               void *stream);

/*
 * Merged weight of one variant (Section 5.1 Eq. (2) read right to left: W_base + delta is the variant's
 * weight): merged[n][k] = f16(float(W[n][k]) + delta[n][k]) for a blob of dz_pack_delta, delta being its
 * dequantised value (zero at the pruned columns).  W, packed, merged: DEVICE, 16-byte aligned;
 * merged f16 [N][K], may not alias W.  dz_base_gemm on the result serves requests that all name this
 * variant with one dense product; the extra rounding of W + delta to fp16 is part of that trade.
 */
int dz_merge_delta(dz_ctx *ctx, const void *W_f16, const void *packed, int N, int K, int bits, int group,
                   void *merged_f16, void *stream);

/*
 * Several linear layers that read the same x for the same requests -- the q, k, v projections of a
 * transformer layer, or gate and up -- in one call:
 *   out[p][t] = f16( x[t] . W[p]^T + x[t] . Delta[p][token_to_delta[t]]^T ),   p = 0 .. P-1,
 * each exactly what dz_linear computes for projection p alone.  The base and delta products of a
 * layer are independent per output feature (Section 5.1, Eq. (2)), so stacking projections along
 * the output dimension changes no result; for decode-sized batches (T <= 64) all P projections go
 * through one kernel launch, which saves the fixed cost of P - 1 launches (Section 5.2 argues the
 * same way for batching all deltas of a layer into one launch).
 *   W, out          HOST arrays of P DEVICE pointers; N a HOST array of P output sizes
 *   packed_deltas   HOST array of P * D DEVICE pointers, projection-major: [p * D + m] is delta m
 *                   packed for projection p (shape N[p] x K)
 * All projections share K, bits, group and D.  1 <= P <= DZ_MAX_GROUP and P * D <= 3 * DZ_MAX_DELTAS.
 */
int dz_linear_group(dz_ctx *ctx, const void *x_f16, int P, const void *const *W_f16,
                    const void *const *packed_deltas, int D, const int32_t *token_to_delta,
                    void *const *out_f16, const int *N, int T, int K, int bits, int group, void *stream);

/*
 * dz_linear for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It takes no context; the workspace the kernels need (split-k
 * partial sums, arrival counters, the error word) is a static device array of the library, fixed at
 * DZ_STATIC_PARTIAL_BYTES + 64.25 KiB per GPU, which every GPU the library runs on holds until the
 * process ends.  The call allocates nothing, frees nothing and synchronises nothing.
 * Arguments as dz_linear, with `device` in place of the context.  Limits: T <= 64, and the split-k
 * partial sums of the call (a multiple of 64 * N * 4 bytes, chosen from N and K) must fit the array;
 * beyond either the call returns DZ_ERR_LIMIT and enqueues no compute.  All calls on one GPU share that
 * GPU's array: two calls whose kernels may overlap on one GPU (different streams, different
 * threads) race and must be serialised by the caller.  A request index outside [-1, D) is served
 * with the base model only and reported by the next dz_check on any context of that GPU.
 */
int dz_linear_static(int device, const void *x_f16, const void *W_f16, const void *const *packed_deltas,
                     int D, const int32_t *token_to_delta, void *out_f16, int T, int N, int K, int bits,
                     int group, void *stream);

/* Synchronise `stream`; return DZ_ERR_INDEX if any call since the last dz_check met a request
 * index outside [-1, D) (that request was served with the base model only), else DZ_OK. */
int dz_check(dz_ctx *ctx, void *stream);

/*
 * Measured ceilings of the device, for pricing the kernels (a benchmark prints them beside the
 * nominal peaks).  Both only enqueue one kernel on `stream`; the caller times it with events.
 *   dz_probe_read  reads `bytes` (a multiple of 16) of DEVICE memory at buf once, 16 bytes per lane and
 *                  load, and does nothing else: bytes / time is the read rate HBM sustains.
 *   dz_probe_mfma  issues iters x 32 dense fp16 matrix instructions per wave on register operands,
 *                  sixteen waves per compute unit; *flops_out (HOST, may be NULL) receives the floating
 *                  point operations the launch performs: flops / time is the matrix rate with every
 *                  memory cost removed.
 */
int dz_probe_read(dz_ctx *ctx, const void *buf, size_t bytes, void *stream);
int dz_probe_mfma(dz_ctx *ctx, int iters, double *flops_out, void *stream);

/*
 * Resident-delta cache: the step before the hot path.  The engine keeps the base model on the GPU
 * and brings compressed deltas in on demand (Section 5.1), a fixed, pre-set number of them per
 * batch at most, moving deltas between GPU memory, host memory and disk as needed (Section 5.4,
 * paragraph "Scalability").  The paper names no replacement rule; this cache evicts the least
 * recently used delta.
 *
 * A cache owns `slots` device buffers of slot_bytes each (16-byte aligned, allocated at creation,
 * freed by dz_cache_destroy, which synchronises the device).  dz_cache_acquire makes the packed
 * deltas named by keys[0..n) resident and returns their device addresses:
 *   - a key already resident is a hit: nothing is copied;
 *   - otherwise a slot is taken -- an empty one first (lowest index), else the least recently
 *     handed-out slot among those neither handed out by this call nor by the previous one -- and
 *     host_blobs[i] (HOST memory, `bytes` <= slot_bytes long, pinned if the copy is to overlap with
 *     compute; it must stay valid until the copy has run) is copied into it asynchronously on
 *     copy_stream.
 * Nothing is synchronised and the compute stream is not touched by dz_cache_acquire: ordering is by
 * events, through the ticket the call returns.
 *   dz_cache_wait(cache, ticket, compute_stream)     compute_stream waits for the copies of that
 *       acquire; call it right before enqueuing the compute that reads the returned addresses.
 *   dz_cache_release(cache, ticket, compute_stream)  call it right after enqueuing that compute: the
 *       work enqueued on compute_stream so far was the last reader of that acquire's slots.  A later
 *       copy that evicts one of them waits for exactly that point and for nothing else.
 * So a caller acquires the deltas of batch i+1 before it enqueues the compute of batch i (the slots
 * of the previous acquire are never evicted), and the copies of batch i+1 run while batch i computes:
 *     t1 = acquire(batch 1)
 *     for i = 1, 2, ...:  t(i+1) = acquire(batch i+1);  wait(t(i));  compute(batch i);  release(t(i))
 * A ticket that is never released stays remembered and its slots have no "last reader" event:
 * evicting one of them drains the whole device first (safe, but it serialises).
 * device_blobs_out[n] receives the addresses; slot_out[n] (slot index), hit_out[n] (1 = was
 * resident) and ticket_out may be NULL.  Keys may repeat within a call (the repeats are hits).  A
 * call with n == 0 does nothing (ticket 0; it does not count as "the previous call" afterwards).
 * Errors: DZ_ERR_ARG for null / negative arguments, bytes > slot_bytes, an unknown ticket, or more
 * keys to bring in than there are slots outside this and the previous call's (nothing is changed
 * then); DZ_ERR_HIP for runtime failures (keys handled before the failure stay resident, the others
 * keep their old state, addresses from the failing key on come back NULL).
 * dz_cache_create with device < 0 makes a cache without device memory that takes the same
 * decisions and copies nothing (addresses come back NULL, wait and release do nothing): for
 * planning and for tests.
 */
typedef struct dz_cache dz_cache;
int dz_cache_create(dz_cache **cache, int device, int slots, size_t slot_bytes);
int dz_cache_destroy(dz_cache *cache);
int dz_cache_acquire(dz_cache *cache, int n, const int64_t *keys, const void *const *host_blobs,
                     size_t bytes, const void **device_blobs_out, int32_t *slot_out,
                     int32_t *hit_out, void *copy_stream, int64_t *ticket_out);
int dz_cache_wait(dz_cache *cache, int64_t ticket, void *compute_stream);
int dz_cache_release(dz_cache *cache, int64_t ticket, void *compute_stream);
/* Totals since creation; any pointer may be NULL. */
int dz_cache_stats(const dz_cache *cache, int64_t *hits, int64_t *misses, int64_t *evictions);

#ifdef __cplusplus
}
#endif
#endif /* DZ_H */

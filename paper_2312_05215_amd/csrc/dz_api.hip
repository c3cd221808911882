// C ABI of libdz (include/dz.h): argument checks, the context's workspace, and dispatch to the
// kernels.  No compute happens here.
#include "dz_internal.h"
#include <stdio.h>
#include <cstdlib>
#include <cstring>
#include <new>

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int N, int K, int bits, int group, bool need_fmt)
{
    if (N <= 0 || K <= 0) return DZ_ERR_SHAPE;
    if (N % 16 != 0 || K % 256 != 0) return DZ_ERR_SHAPE;
    if (need_fmt) {
        if (bits != 2 && bits != 4) return DZ_ERR_BITS;
        if (group != 64 && group != 128) return DZ_ERR_SHAPE;
    }
    return DZ_OK;
}

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

}  // namespace

// text of the last HIP failure seen by the calling thread, for dz_strerror(DZ_ERR_HIP)
static thread_local char t_hip_err[288] = "HIP runtime failure";

int dz_set_hip_error(dz_ctx *ctx, hipError_t e)
{
    if (e == hipSuccess) return DZ_OK;
    snprintf(t_hip_err, sizeof(t_hip_err), "HIP runtime failure: %s", hipGetErrorString(e));
    if (ctx) {
        strncpy(ctx->hip_err, hipGetErrorString(e), sizeof(ctx->hip_err) - 1);
        ctx->hip_err[sizeof(ctx->hip_err) - 1] = 0;
    }
    return DZ_ERR_HIP;
}

__global__ void dz_clear_words_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// The workspace grows by allocating, which a stream that is being recorded into a graph does not
// allow.  Such a call fails here, before it touches the stream, so the capture itself stays valid.
// Nothing waits for the stream: launches that are still running keep the buffer they were given
// (a replaced buffer is retired, not freed).
static int quiesce_for_growth(dz_ctx *ctx, hipStream_t st)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    hipError_t e = hipStreamIsCapturing(st, &cs);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    if (cs != hipStreamCaptureStatusNone) return dz_set_hip_error(ctx, hipErrorStreamCaptureUnsupported);
    return DZ_OK;
}

// A buffer that a growth replaces is kept until dz_destroy: the kernel nodes of a HIP graph recorded
// earlier still hold its address, and a replay must find it allocated.
static int retire(dz_ctx *ctx, void *p)
{
    if (!p) return DZ_OK;
    if (ctx->n_retired >= (int)(sizeof(ctx->retired) / sizeof(ctx->retired[0]))) return DZ_ERR_LIMIT;
    ctx->retired[ctx->n_retired++] = p;
    return DZ_OK;
}

int dz_ensure_partial(dz_ctx *ctx, size_t bytes, hipStream_t st)
{
    if (bytes <= ctx->partial_bytes) return DZ_OK;
    if (ctx->static_ws) return DZ_ERR_LIMIT;
    if (int rc = quiesce_for_growth(ctx, st)) return rc;
    if (int rc = retire(ctx, ctx->partial)) return rc;
    ctx->partial = nullptr;
    ctx->partial_bytes = 0;
    size_t want = bytes + bytes / 4;
    hipError_t e = hipMalloc((void **)&ctx->partial, want);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    ctx->partial_bytes = want;
    return DZ_OK;
}

int dz_ensure_counters(dz_ctx *ctx, int n, hipStream_t st)
{
    if (n <= ctx->counters_cap) return DZ_OK;
    if (ctx->static_ws) return DZ_ERR_LIMIT;
    if (int rc = quiesce_for_growth(ctx, st)) return rc;
    if (int rc = retire(ctx, ctx->counters)) return rc;
    ctx->counters = nullptr;
    ctx->counters_cap = 0;
    int want = n * 2;
    hipError_t e = hipMalloc((void **)&ctx->counters, (size_t)want * 4);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    // cleared on the caller's stream, ahead of the launch that asked for them
    hipLaunchKernelGGL(dz_clear_words_kernel, dim3((unsigned)((want + 255) / 256)), dim3(256), 0, st, ctx->counters, want);
    e = hipGetLastError();
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    ctx->counters_cap = want;
    return DZ_OK;
}

int dz_ensure_lora(dz_ctx *ctx, size_t bytes, hipStream_t st)
{
    if (bytes <= ctx->lora_u_bytes) return DZ_OK;
    if (ctx->static_ws) return DZ_ERR_LIMIT;
    if (int rc = quiesce_for_growth(ctx, st)) return rc;
    if (int rc = retire(ctx, ctx->lora_u)) return rc;
    ctx->lora_u = nullptr;
    ctx->lora_u_bytes = 0;
    size_t want = bytes + bytes / 4;
    hipError_t e = hipMalloc((void **)&ctx->lora_u, want);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    ctx->lora_u_bytes = want;
    return DZ_OK;
}

static int ensure_seg(dz_ctx *ctx, int T, hipStream_t st)
{
    if (T <= ctx->seg_cap) return DZ_OK;
    if (ctx->static_ws) return DZ_ERR_LIMIT;
    if (int rc = quiesce_for_growth(ctx, st)) return rc;
    if (int rc = retire(ctx, ctx->seg_perm)) return rc;
    if (int rc = retire(ctx, ctx->seg_key)) return rc;
    ctx->seg_perm = ctx->seg_key = nullptr;
    ctx->seg_cap = 0;
    ctx->seg_ids = nullptr;
    int want = T * 2;
    hipError_t e = hipMalloc((void **)&ctx->seg_perm, (size_t)want * 4);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    e = hipMalloc((void **)&ctx->seg_key, (size_t)want * 4);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    ctx->seg_cap = want;
    return DZ_OK;
}

// The entry point that allocates nothing keeps a sticky error word of its own per GPU; dz_check
// reports it too when that translation unit is part of the library.
extern "C" int32_t *dz_static_err_word(int device) __attribute__((weak));

extern "C" {

const char *dz_strerror(int rc)
{
    switch (rc) {
    case DZ_OK: return "ok";
    case DZ_ERR_ARG: return "invalid argument (null pointer, negative count, or too many deltas)";
    case DZ_ERR_SHAPE: return "unsupported shape (need N % 16 == 0, K % 256 == 0, group 64 or 128)";
    case DZ_ERR_BITS: return "bits must be 2 or 4";
    case DZ_ERR_ALIGN: return "device pointer is not 16-byte aligned";
    case DZ_ERR_HIP: return t_hip_err;          // carries the runtime's own text for this thread's last failure
    case DZ_ERR_INDEX: return "a request index was outside [-1, D)";
    case DZ_ERR_LIMIT: return "the call needs more workspace than this entry point or context may use";
    default: return "unknown error";
    }
}

const char *dz_last_hip_error(const dz_ctx *ctx) { return ctx ? ctx->hip_err : ""; }

int dz_create(dz_ctx **out, int device)
{
    if (!out) return DZ_ERR_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return DZ_ERR_ARG;
    dz_ctx *ctx = new (std::nothrow) dz_ctx();
    if (!ctx) return DZ_ERR_ARG;
    ctx->device = device;
    DeviceGuard guard(device);
    hipError_t e = guard.ok ? hipSuccess : hipErrorInvalidDevice;
    if (e == hipSuccess) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess) ctx->num_cus = n;
    }
    if (e == hipSuccess && dz_static_err_word) (void)dz_static_err_word(device);   // set-up of the static workspace on this GPU
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->err_flag, 4);
    if (e == hipSuccess) e = hipMemset(ctx->err_flag, 0, 4);
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->seg_counts, (size_t)(DZ_SEG_MAX_D + 1) * 4);
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->seg_offsets, (size_t)(DZ_SEG_MAX_D + 2) * 4);
    if (e == hipSuccess) {
        ctx->seg_cap = 4096;
        e = hipMalloc((void **)&ctx->seg_perm, (size_t)ctx->seg_cap * 4);
        if (e == hipSuccess) e = hipMalloc((void **)&ctx->seg_key, (size_t)ctx->seg_cap * 4);
    }
    if (e == hipSuccess) {
        ctx->counters_cap = 8192;
        e = hipMalloc((void **)&ctx->counters, (size_t)ctx->counters_cap * 4);
        if (e == hipSuccess) e = hipMemset(ctx->counters, 0, (size_t)ctx->counters_cap * 4);
    }
    if (e == hipSuccess) {
        ctx->partial_bytes = (size_t)32 << 20;
        e = hipMalloc((void **)&ctx->partial, ctx->partial_bytes);
    }
    if (e != hipSuccess) {
        (void)dz_set_hip_error(nullptr, e);     // the context goes away: keep the text for dz_strerror
        dz_destroy(ctx);
        return DZ_ERR_HIP;
    }
    *out = ctx;
    return DZ_OK;
}

int dz_destroy(dz_ctx *ctx)
{
    if (!ctx) return DZ_ERR_ARG;
    {
        DeviceGuard guard(ctx->device);
        (void)hipDeviceSynchronize();
        if (ctx->err_flag) (void)hipFree(ctx->err_flag);
        if (ctx->seg_counts) (void)hipFree(ctx->seg_counts);
        if (ctx->seg_offsets) (void)hipFree(ctx->seg_offsets);
        if (ctx->seg_perm) (void)hipFree(ctx->seg_perm);
        if (ctx->seg_key) (void)hipFree(ctx->seg_key);
        if (ctx->counters) (void)hipFree(ctx->counters);
        if (ctx->partial) (void)hipFree(ctx->partial);
        if (ctx->lora_u) (void)hipFree(ctx->lora_u);
        for (int i = 0; i < ctx->n_retired; ++i) (void)hipFree(ctx->retired[i]);
    }
    delete ctx;
    return DZ_OK;
}

size_t dz_packed_bytes(int N, int K, int bits, int group)
{
    if (check_shape(N, K, bits, group, true) != DZ_OK) return 0;
    return (size_t)N * K * (2 * bits + 4) / 32 + (size_t)4 * N * K / group;
}

int dz_pack_delta(dz_ctx *ctx, const uint8_t *codes, const uint8_t *idx, const void *scale, const void *zero,
                  int N, int K, int bits, int group, void *packed, void *stream)
{
    if (!ctx || !codes || !idx || !scale || !zero || !packed) return DZ_ERR_ARG;
    int rc = check_shape(N, K, bits, group, true);
    if (rc) return rc;
    if (!aligned16(packed) || (reinterpret_cast<uintptr_t>(scale) & 1) || (reinterpret_cast<uintptr_t>(zero) & 1))
        return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    return dz_launch_pack(ctx, codes, idx, scale, zero, N, K, bits, group, packed, (hipStream_t)stream);
}

int dz_unpack_delta(dz_ctx *ctx, const void *packed, int N, int K, int bits, int group, uint8_t *codes,
                    uint8_t *idx, void *scale, void *zero, float *dense, void *stream)
{
    if (!ctx || !packed) return DZ_ERR_ARG;
    int rc = check_shape(N, K, bits, group, true);
    if (rc) return rc;
    if (!aligned16(packed) || (reinterpret_cast<uintptr_t>(scale) & 1) || (reinterpret_cast<uintptr_t>(zero) & 1) ||
        (reinterpret_cast<uintptr_t>(dense) & 3))
        return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    return dz_launch_unpack(ctx, packed, N, K, bits, group, codes, idx, scale, zero, dense, (hipStream_t)stream);
}

int dz_segment(dz_ctx *ctx, const int32_t *ids, int T, int D, int32_t *counts, int32_t *offsets, int32_t *perm,
               void *stream)
{
    if (!ctx || T < 0 || D < 0 || D > DZ_SEG_MAX_D || (T > 0 && !ids)) return DZ_ERR_ARG;
    if ((reinterpret_cast<uintptr_t>(ids) | reinterpret_cast<uintptr_t>(counts) | reinterpret_cast<uintptr_t>(offsets) |
         reinterpret_cast<uintptr_t>(perm)) & 3)
        return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    // T == 0 still has to produce counts = 0 and offsets = 0: the kernel handles an empty loop
    return dz_launch_segment(ctx, ids, T, D, counts, offsets, perm, nullptr, (hipStream_t)stream);
}

// P projections that share x and the request indices.  Small batches: one launch of the streaming
// kernel for all of them.  Large batches: the tiled kernel, one projection after the other.
static int run_group(dz_ctx *ctx, const void *x, int P, const void *const *W, const void *const *deltas, int D,
                     const int32_t *ids, void *const *out, const int *N, int T, int K, int bits, int group,
                     int accumulate, bool has_base, bool has_delta, hipStream_t st, bool quant_only = false)
{
    if (!ctx || T < 0 || D < 0 || D > DZ_MAX_DELTAS || P < 1 || P > DZ_MAX_GROUP || !N || !out) return DZ_ERR_ARG;
    if (has_base && !W) return DZ_ERR_ARG;
    if (has_delta && P * D > DZ_GROUP_PTRS) return DZ_ERR_ARG;
    for (int p = 0; p < P; ++p) {
        int rc = check_shape(N[p], K, bits, group, has_delta);
        if (rc) return rc;
    }
    if (T == 0) return DZ_OK;
    if (!x || (has_delta && D > 0 && (!deltas || !ids))) return DZ_ERR_ARG;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(ids) & 3)) return DZ_ERR_ALIGN;
    for (int p = 0; p < P; ++p) {
        if (!out[p] || (has_base && !W[p])) return DZ_ERR_ARG;
        if (!aligned16(out[p]) || (has_base && !aligned16(W[p]))) return DZ_ERR_ALIGN;
    }
    if (has_delta)
        for (int m = 0; m < P * D; ++m) {
            if (!deltas[m]) return DZ_ERR_ARG;
            if (!aligned16(deltas[m])) return DZ_ERR_ALIGN;
        }
    DeviceGuard guard(ctx->device);
    DzStreamArgs a;
    memset(&a, 0, sizeof(a));
    a.x = x;
    a.T = T; a.K = K; a.D = D; a.bits = bits; a.group = group;
    a.accumulate = accumulate;
    a.has_base = has_base;
    // an SBMM with no deltas still runs (every request gets a zero delta term)
    a.has_delta = has_delta && (D > 0 || !has_base);
    a.quant_only = quant_only ? 1 : 0;
    a.err_flag = ctx->err_flag;
    const bool tiled = T > 64 && !ctx->no_prefill;      // large batches: MFMA-bound tiled kernel
    if (has_delta && D > 0 && T <= 64) {
        a.ids = ids;                    // small batches are sorted inside the streaming kernel
    } else if (has_delta && D > 0) {
        int rc = ensure_seg(ctx, T, st);
        if (rc) return rc;
        // With DZ_OPT_REUSE_SEGMENTS the caller promises that an index vector at the same address with
        // the same T and D still holds the same values: the projections of one layer then share one sort.
        const bool same = ctx->reuse_segments && ctx->seg_ids == ids && ctx->seg_T == T && ctx->seg_D == D;
        if (!same) {
            rc = dz_launch_segment(ctx, ids, T, D, nullptr, nullptr, ctx->seg_perm, ctx->seg_key, st);
            if (rc) return rc;
            ctx->seg_ids = ids; ctx->seg_T = T; ctx->seg_D = D;
        }
        a.perm = ctx->seg_perm;
        a.key = ctx->seg_key;
    }
    if (!tiled) {                       // small batches: HBM-bound streaming kernel, all projections in one launch
        DzGroup gp;
        DzGroupPtrs dp;
        memset(&gp, 0, sizeof(gp));
        memset(&dp, 0, sizeof(dp));
        gp.P = P;
        for (int p = 0; p < P; ++p) {
            gp.N[p] = N[p];
            gp.W[p] = has_base ? W[p] : nullptr;
            gp.out[p] = out[p];
        }
        if (has_delta)
            for (int m = 0; m < P * D; ++m) dp.p[m] = deltas[m];
        return dz_launch_stream(ctx, a, gp, dp, st);
    }
    for (int p = 0; p < P; ++p) {
        DzDeltaPtrs dp;
        memset(&dp, 0, sizeof(dp));
        if (has_delta)
            for (int m = 0; m < D; ++m) dp.p[m] = deltas[p * D + m];
        a.W = has_base ? W[p] : nullptr;
        a.out = out[p];
        a.N = N[p];
        int rc = dz_launch_prefill(ctx, a, dp, st);
        if (rc) return rc;
    }
    return DZ_OK;
}

int dz_run_linear(dz_ctx *ctx, const void *x, const void *W, const void *const *deltas, int D,
                      const int32_t *ids, void *out, int T, int N, int K, int bits, int group, int accumulate,
                      bool has_base, bool has_delta, hipStream_t st)
{
    return run_group(ctx, x, 1, &W, deltas, D, ids, &out, &N, T, K, bits, group, accumulate, has_base, has_delta, st);
}

int dz_base_gemm(dz_ctx *ctx, const void *x, const void *W, void *out, int T, int N, int K, void *stream)
{
    return dz_run_linear(ctx, x, W, nullptr, 0, nullptr, out, T, N, K, 4, 128, 0, true, false, (hipStream_t)stream);
}

int dz_sbmm(dz_ctx *ctx, const void *x, const void *const *deltas, int D, const int32_t *ids, void *out, int T,
            int N, int K, int bits, int group, int accumulate, void *stream)
{
    return dz_run_linear(ctx, x, nullptr, deltas, D, ids, out, T, N, K, bits, group, accumulate ? 1 : 0, false, true,
                      (hipStream_t)stream);
}

int dz_linear(dz_ctx *ctx, const void *x, const void *W, const void *const *deltas, int D, const int32_t *ids,
              void *out, int T, int N, int K, int bits, int group, void *stream)
{
    return dz_run_linear(ctx, x, W, deltas, D, ids, out, T, N, K, bits, group, 0, true, true, (hipStream_t)stream);
}

int dz_linear_group(dz_ctx *ctx, const void *x, int P, const void *const *W, const void *const *deltas, int D,
                    const int32_t *ids, void *const *out, const int *N, int T, int K, int bits, int group,
                    void *stream)
{
    return run_group(ctx, x, P, W, deltas, D, ids, out, N, T, K, bits, group, 0, true, true, (hipStream_t)stream);
}

size_t dz_qpacked_bytes(int N, int K, int bits, int group)
{
    if (check_shape(N, K, bits, group, true) != DZ_OK) return 0;
    return (size_t)N * K * bits / 8 + (size_t)4 * N * K / group;
}

int dz_qpack_delta(dz_ctx *ctx, const uint8_t *codes, const void *scale, const void *zero, int N, int K, int bits,
                   int group, void *packed, void *stream)
{
    if (!ctx || !codes || !scale || !zero || !packed) return DZ_ERR_ARG;
    int rc = check_shape(N, K, bits, group, true);
    if (rc) return rc;
    if (!aligned16(packed) || (reinterpret_cast<uintptr_t>(scale) & 1) || (reinterpret_cast<uintptr_t>(zero) & 1))
        return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    return dz_launch_qpack(ctx, codes, scale, zero, N, K, bits, group, packed, (hipStream_t)stream);
}

int dz_qunpack_delta(dz_ctx *ctx, const void *packed, int N, int K, int bits, int group, uint8_t *codes, void *scale,
                     void *zero, float *dense, void *stream)
{
    if (!ctx || !packed) return DZ_ERR_ARG;
    int rc = check_shape(N, K, bits, group, true);
    if (rc) return rc;
    if (!aligned16(packed) || (reinterpret_cast<uintptr_t>(scale) & 1) || (reinterpret_cast<uintptr_t>(zero) & 1) ||
        (reinterpret_cast<uintptr_t>(dense) & 3))
        return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    return dz_launch_qunpack(ctx, packed, N, K, bits, group, codes, scale, zero, dense, (hipStream_t)stream);
}

int dz_qsbmm(dz_ctx *ctx, const void *x, const void *const *deltas, int D, const int32_t *ids, void *out, int T, int N,
             int K, int bits, int group, int accumulate, void *stream)
{
    return run_group(ctx, x, 1, nullptr, deltas, D, ids, &out, &N, T, K, bits, group, accumulate ? 1 : 0, false, true,
                     (hipStream_t)stream, true);
}

int dz_qlinear(dz_ctx *ctx, const void *x, const void *W, const void *const *deltas, int D, const int32_t *ids, void *out,
               int T, int N, int K, int bits, int group, void *stream)
{
    return run_group(ctx, x, 1, &W, deltas, D, ids, &out, &N, T, K, bits, group, 0, true, true, (hipStream_t)stream, true);
}

int dz_merge_delta(dz_ctx *ctx, const void *W, const void *packed, int N, int K, int bits, int group, void *merged,
                   void *stream)
{
    if (!ctx || !W || !packed || !merged) return DZ_ERR_ARG;
    int rc = check_shape(N, K, bits, group, true);
    if (rc) return rc;
    if (!aligned16(W) || !aligned16(packed) || !aligned16(merged)) return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    return dz_launch_merge(ctx, W, packed, N, K, bits, group, merged, (hipStream_t)stream);
}

int dz_compress_delta(dz_ctx *ctx, const void *delta, int N, int K, int bits, int group, uint8_t *codes, uint8_t *idx,
                      void *scale, void *zero, void *stream)
{
    if (!ctx || !delta || !codes || !idx || !scale || !zero) return DZ_ERR_ARG;
    int rc = check_shape(N, K, bits, group, true);
    if (rc) return rc;
    if ((reinterpret_cast<uintptr_t>(delta) & 7) || (reinterpret_cast<uintptr_t>(scale) & 1) || (reinterpret_cast<uintptr_t>(zero) & 1))
        return DZ_ERR_ALIGN;
    DeviceGuard guard(ctx->device);
    return dz_launch_compress(ctx, delta, N, K, bits, group, codes, idx, scale, zero, (hipStream_t)stream);
}

int dz_lora_sbmm(dz_ctx *ctx, const void *x, const void *const *A, const void *const *B, int D, int rank,
                 const int32_t *ids, void *out, int T, int N, int K, int accumulate, void *stream)
{
    if (!ctx || T < 0 || D < 0 || D > DZ_MAX_DELTAS) return DZ_ERR_ARG;
    if (N <= 0 || K <= 0 || N % 4 != 0 || K % 8 != 0 || rank < 8 || rank > 64 || rank % 8 != 0) return DZ_ERR_SHAPE;
    if (T == 0) return DZ_OK;
    if (!x || !out || !ids || (D > 0 && (!A || !B))) return DZ_ERR_ARG;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(out) & 7) || (reinterpret_cast<uintptr_t>(ids) & 3)) return DZ_ERR_ALIGN;
    for (int m = 0; m < D; ++m) {
        if (!A[m] || !B[m]) return DZ_ERR_ARG;
        if (!aligned16(A[m]) || !aligned16(B[m])) return DZ_ERR_ALIGN;
    }
    DeviceGuard guard(ctx->device);
    hipStream_t st = (hipStream_t)stream;
    int rc = ensure_seg(ctx, T, st);
    if (rc) return rc;
    rc = dz_ensure_lora(ctx, (size_t)T * rank * sizeof(float), st);
    if (rc) return rc;
    // the adapter-sorted order of the batch (Section 5.2: requests of one model are grouped)
    rc = dz_launch_segment(ctx, ids, T, D, nullptr, nullptr, ctx->seg_perm, ctx->seg_key, st);
    if (rc) return rc;
    ctx->seg_ids = nullptr;         // the remembered order of DZ_OPT_REUSE_SEGMENTS is gone
    return dz_launch_lora(ctx, x, A, B, D, rank, ids, ctx->seg_perm, ctx->lora_u, out, T, N, K, accumulate ? 1 : 0, st);
}

int dz_check(dz_ctx *ctx, void *stream)
{
    if (!ctx) return DZ_ERR_ARG;
    DeviceGuard guard(ctx->device);
    hipStream_t st = (hipStream_t)stream;
    // the context's own error word, and the one dz_linear_static keeps in the static workspace of this GPU
    int32_t *words[2] = {ctx->err_flag, nullptr};
    if (dz_static_err_word) words[1] = dz_static_err_word(ctx->device);
    int32_t flag[2] = {0, 0};
    hipError_t e = hipSuccess;
    for (int i = 0; i < 2 && e == hipSuccess; ++i)
        if (words[i]) e = hipMemcpyAsync(&flag[i], words[i], 4, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    if (flag[0] | flag[1]) {
        for (int i = 0; i < 2 && e == hipSuccess; ++i)
            if (words[i] && flag[i]) {
                hipLaunchKernelGGL(dz_clear_words_kernel, dim3(1), dim3(64), 0, st, words[i], 1);
                e = hipGetLastError();
            }
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return dz_set_hip_error(ctx, e);
        return DZ_ERR_INDEX;
    }
    return DZ_OK;
}

int dz_set_option(dz_ctx *ctx, int key, int value)
{
    if (!ctx || value < 0) return DZ_ERR_ARG;
    switch (key) {
    case DZ_OPT_SPLIT_K: ctx->force_splits = value; return DZ_OK;
    case DZ_OPT_WORKGROUPS: ctx->target_wgs = value; return DZ_OK;
    case DZ_OPT_ROUND_TILES: ctx->round_tiles = value; return DZ_OK;
    case DZ_OPT_LARGE_BATCH_STREAMING: ctx->no_prefill = value ? 1 : 0; return DZ_OK;
    case DZ_OPT_WIDE_TILE:
        if (value > 2) return DZ_ERR_ARG;
        ctx->tile_kernel = value;
        return DZ_OK;
    case DZ_OPT_REUSE_SEGMENTS:
        ctx->reuse_segments = value ? 1 : 0;
        ctx->seg_ids = nullptr;
        return DZ_OK;
    default: return DZ_ERR_ARG;
    }
}

}  // extern "C"

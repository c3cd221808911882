// Two probe kernels that measure what the device itself sustains, so that a benchmark can print the
// measured ceilings beside the nominal peaks it prices the kernels against:
//   dz_probe_read  streams a buffer once with 16-byte loads per lane (nothing else): the HBM read
//                  rate a kernel of this library could reach at best;
//   dz_probe_mfma  issues dense fp16 MFMAs (V_MFMA_F32_16X16X32_F16) back to back on register
//                  operands: the matrix rate with every memory cost removed.
// Neither touches the serving path; both only enqueue work (the caller times them with events).
#include "dz_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_THREADS = 512;

// Every workgroup walks its own contiguous share of the buffer, eight 16-byte loads per lane in
// flight.  The xor of everything read is stored only if it equals a value it cannot have by
// accident, which keeps the loads alive without writing anything.
__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                                    unsigned int *__restrict__ sink)
{
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per_wg;
    const size_t b1 = b0 + per_wg < n16 ? b0 + per_wg : n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = b0 + threadIdx.x;
    for (; i + 7 * PROBE_THREADS < b1; i += 8 * PROBE_THREADS) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * PROBE_THREADS);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    for (; i < b1; i += PROBE_THREADS) acc ^= __builtin_nontemporal_load(src + i);
    const unsigned int x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u && sink) *sink = x;
}

// 32 MFMAs per iteration on eight independent accumulators: no dependent pair is closer than
// eight instructions, so the matrix pipe never waits for a result.
__global__ __launch_bounds__(PROBE_THREADS) void probe_mfma_kernel(int iters, float *__restrict__ sink)
{
    h8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.001f * (float)((threadIdx.x + i) & 7));
        b[i] = (_Float16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
    }
    f4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (f4){0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i].x + acc[i].y + acc[i].z + acc[i].w;
    if (s == -1.0f && sink) *sink = s;
}

}  // namespace

extern "C" {

int dz_probe_read(dz_ctx *ctx, const void *buf, size_t bytes, void *stream)
{
    if (!ctx || !buf || bytes < 16) return DZ_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(buf) & 15u) return DZ_ERR_ALIGN;
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess || (prev != ctx->device && hipSetDevice(ctx->device) != hipSuccess)) return DZ_ERR_HIP;
    const int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    hipLaunchKernelGGL(probe_read_kernel, dim3(cus * 8), dim3(PROBE_THREADS), 0, (hipStream_t)stream, (const u32x4 *)buf,
                       bytes / 16, (unsigned int *)ctx->seg_counts);
    const int rc = dz_set_hip_error(ctx, hipGetLastError());
    if (prev != ctx->device) (void)hipSetDevice(prev);
    return rc;
}

int dz_probe_mfma(dz_ctx *ctx, int iters, double *flops_out, void *stream)
{
    if (!ctx || iters <= 0) return DZ_ERR_ARG;
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess || (prev != ctx->device && hipSetDevice(ctx->device) != hipSuccess)) return DZ_ERR_HIP;
    const int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    const int grid = cus * 2;                           // sixteen waves per compute unit
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(PROBE_THREADS), 0, (hipStream_t)stream, iters, (float *)ctx->seg_counts);
    const int rc = dz_set_hip_error(ctx, hipGetLastError());
    if (flops_out) *flops_out = (double)grid * (PROBE_THREADS / 64) * (double)iters * 32.0 * (2.0 * 16 * 16 * 32);
    if (prev != ctx->device) (void)hipSetDevice(prev);
    return rc;
}

}  // extern "C"

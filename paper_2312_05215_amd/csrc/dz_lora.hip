// Low-rank adapters served like compressed deltas (paper Section 3.2: adapters are registered next to
// deltas and served by the same engine; Section 6.4).  For request t with adapter m = Idx[t]
//
//     y[t] = B_m . (A_m . x[t]),        A_m [rank][K],  B_m [N][rank],  fp16
//
// the selective batched product of Section 5.2 with a low-rank matrix in place of a delta.  Adapters
// are a few hundred KB per layer, so neither kernel is shaped by bandwidth or by the matrix cores; the
// batch is walked in the delta-sorted order the segment pass produces, so that neighbouring waves read
// the same adapter.
//   shrink: u[t] = A_m . x[t]  (fp32 [T][rank]) -- one wave per (request, 8 ranks), lanes stride over k
//           with 16-byte loads and packed dot products, then a lane reduction;
//   expand: y[t] = B_m . u[t]  -- one thread per (request, 4 outputs), fp32, one rounding at the store.
#include "dz_internal.h"

namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

struct LoraPtrs { const void *p[DZ_MAX_DELTAS]; };

__device__ __forceinline__ float dot8(h8 a, h8 b, float acc)
{
    acc = __builtin_amdgcn_fdot2((h2){a[0], a[1]}, (h2){b[0], b[1]}, acc, false);
    acc = __builtin_amdgcn_fdot2((h2){a[2], a[3]}, (h2){b[2], b[3]}, acc, false);
    acc = __builtin_amdgcn_fdot2((h2){a[4], a[5]}, (h2){b[4], b[5]}, acc, false);
    acc = __builtin_amdgcn_fdot2((h2){a[6], a[7]}, (h2){b[6], b[7]}, acc, false);
    return acc;
}

// grid: (T, rank / 8); block: one wave
__global__ __launch_bounds__(64) void lora_shrink_kernel(const _Float16 *__restrict__ x, LoraPtrs A, int D, int rank,
                                                          const int32_t *__restrict__ ids, const int32_t *__restrict__ perm,
                                                          float *__restrict__ u, int T, int K)
{
    const int t = perm[blockIdx.x];             // requests in adapter-sorted order
    const int m = ids[t];
    if (m < 0 || m >= D) return;                // no adapter: the expand pass writes the zero
    const int r0 = blockIdx.y * 8;
    const _Float16 *a = (const _Float16 *)A.p[m] + (size_t)r0 * K;
    const _Float16 *xr = x + (size_t)t * K;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int k = threadIdx.x * 8; k < K; k += 64 * 8) {
        const h8 xv = *(const h8 *)(xr + k);
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = dot8(*(const h8 *)(a + (size_t)r * K + k), xv, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc[r] += __shfl_xor(acc[r], d, 64);
    }
    if (threadIdx.x == 0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) u[(size_t)t * rank + r0 + r] = acc[r];
    }
}

// grid: (ceil(N / 1024), T); block: 256 threads, 4 outputs each
__global__ __launch_bounds__(256) void lora_expand_kernel(const float *__restrict__ u, LoraPtrs B, int D, int rank,
                                                           const int32_t *__restrict__ ids, _Float16 *__restrict__ out, int T, int N,
                                                           int accumulate, int32_t *__restrict__ err_flag)
{
    const int t = blockIdx.y;
    const int n0 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (n0 >= N) return;
    const int m = ids[t];
    const bool valid = m >= 0 && m < D;
    if (!valid && m != -1 && blockIdx.x == 0 && threadIdx.x == 0) atomicOr(err_flag, 1);
    float y[4] = {0.f, 0.f, 0.f, 0.f};
    if (valid) {
        const _Float16 *b = (const _Float16 *)B.p[m] + (size_t)n0 * rank;
        const float *ut = u + (size_t)t * rank;
        for (int r = 0; r < rank; r += 8) {
            float uv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) uv[i] = ut[r + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const h8 bv = *(const h8 *)(b + (size_t)j * rank + r);
#pragma unroll
                for (int i = 0; i < 8; ++i) y[j] = fmaf((float)bv[i], uv[i], y[j]);
            }
        }
    }
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    _Float16 *o = out + (size_t)t * N + n0;
    if (accumulate) {
        const h4 prev = *(const h4 *)o;
        y[0] += (float)prev.x; y[1] += (float)prev.y; y[2] += (float)prev.z; y[3] += (float)prev.w;
    }
    *(h4 *)o = (h4){(_Float16)y[0], (_Float16)y[1], (_Float16)y[2], (_Float16)y[3]};
}

}  // namespace

int dz_launch_lora(dz_ctx *ctx, const void *x, const void *const *A, const void *const *B, int D, int rank, const int32_t *ids,
                   const int32_t *perm, float *u, void *out, int T, int N, int K, int accumulate, hipStream_t st)
{
    LoraPtrs pa, pb;
    for (int m = 0; m < DZ_MAX_DELTAS; ++m) { pa.p[m] = m < D ? A[m] : nullptr; pb.p[m] = m < D ? B[m] : nullptr; }
    hipLaunchKernelGGL(lora_shrink_kernel, dim3(T, rank / 8), dim3(64), 0, st, (const _Float16 *)x, pa, D, rank, ids, perm, u, T, K);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return dz_set_hip_error(ctx, e);
    hipLaunchKernelGGL(lora_expand_kernel, dim3((N + 1023) / 1024, T), dim3(256), 0, st, (const float *)u, pb, D, rank, ids,
                       (_Float16 *)out, T, N, accumulate, ctx->err_flag);
    return dz_set_hip_error(ctx, hipGetLastError());
}

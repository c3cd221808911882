// Request reordering on the device (paper Section 5.2: requests of one delta are grouped together
// before the delta product).  A stable counting sort of the request->delta index vector, done by
// one workgroup: LDS histogram, prefix sum, then a wave-level stable scatter in which each chunk
// of 64 requests ranks itself with ballot / mbcnt (lanes naming the same delta are found with a
// ballot, a lane's rank among them is the population count of the lower lanes in that mask).
#include "dz_internal.h"

namespace {

constexpr int SEG_THREADS = 256;

__device__ inline unsigned lanes_below(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// key = delta index, or D for "no delta" (index -1 or out of range).
__global__ __launch_bounds__(SEG_THREADS) void segment_kernel(const int32_t *__restrict__ ids, int T, int D,
                                                              int32_t *__restrict__ counts,
                                                              int32_t *__restrict__ offsets,
                                                              int32_t *__restrict__ perm,
                                                              int32_t *__restrict__ key_out,
                                                              int32_t *__restrict__ err_flag)
{
    extern __shared__ int32_t cursor[];          // [D + 1] histogram, then running write cursors
    const int tid = threadIdx.x;
    for (int i = tid; i <= D; i += SEG_THREADS) cursor[i] = 0;
    __syncthreads();
    bool bad = false;
    for (int t = tid; t < T; t += SEG_THREADS) {
        int id = ids[t];
        bool valid = id >= 0 && id < D;
        bad |= !valid && id != -1;
        atomicAdd(&cursor[valid ? id : D], 1);
    }
    if (bad) atomicOr(err_flag, 1);
    __syncthreads();
    if (counts)
        for (int i = tid; i < D; i += SEG_THREADS) counts[i] = cursor[i];
    __syncthreads();
    // exclusive prefix sum over D + 1 bins by wave 0: 64 bins per round, carried total in `base`
    if (tid < 64) {
        int base = 0;
        for (int i0 = 0; i0 <= D; i0 += 64) {
            int i = i0 + tid;
            int c = (i <= D) ? cursor[i] : 0;
            int incl = c;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                int up = __shfl_up(incl, d, 64);
                if (tid >= d) incl += up;
            }
            int excl = base + incl - c;
            if (i <= D) {
                cursor[i] = excl;
                if (offsets) offsets[i] = excl;
            }
            base += __shfl(incl, 63, 64);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        // stable scatter, 64 requests at a time, in request order
        volatile int32_t *cur = cursor;
        for (int t0 = 0; t0 < T; t0 += 64) {
            int t = t0 + tid;
            bool active = t < T;
            int id = active ? ids[t] : 0;
            int key = (id >= 0 && id < D) ? id : D;
            unsigned long long todo = __ballot(active);
            while (todo) {
                int leader = __builtin_ctzll(todo);
                int k0 = __shfl(key, leader, 64);
                unsigned long long same = __ballot(active && key == k0);
                int start = cur[k0];
                __builtin_amdgcn_wave_barrier();
                if (active && key == k0) {
                    int pos = start + (int)lanes_below(same);
                    if (perm) perm[pos] = t;
                    if (key_out) key_out[pos] = key;
                }
                if (tid == leader) cur[k0] = start + __builtin_popcountll(same);
                __builtin_amdgcn_wave_barrier();
                todo &= ~same;
            }
        }
    }
}

}  // namespace

int dz_launch_segment(dz_ctx *ctx, const int32_t *ids, int T, int D, int32_t *counts, int32_t *offsets,
                      int32_t *perm, int32_t *key, hipStream_t st)
{
    size_t lds = (size_t)(D + 1) * sizeof(int32_t);
    hipLaunchKernelGGL(segment_kernel, dim3(1), dim3(SEG_THREADS), lds, st, ids, T, D, counts, offsets, perm, key,
                       ctx->err_flag);
    return dz_set_hip_error(ctx, hipGetLastError());
}

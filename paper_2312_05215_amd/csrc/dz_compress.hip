// The data-free delta compressor on the GPU: a dense fp16 delta -> canonical compressed tables.
//
// Paper Section 4.1: step 2 prunes the delta to the 2:4 pattern (two of every four consecutive
// entries are kept, each with a 2-bit position), step 3 stores the kept values as b-bit codes.  The
// paper's Algorithm 1 picks mask and codes with calibration data; this kernel applies the data-free
// rule instead: keep the two entries of largest magnitude (ties: the lower position), and quantise the
// kept values of each row and group of `group` dense columns on an asymmetric uniform grid that
// contains zero, rounding to nearest (half to even), all in fp32:
//     lo = min(0, min v), hi = max(0, max v), s = f16((hi - lo) / (2^b - 1))  (s = 1, z = 0 if that is 0)
//     z = clamp(rint((0 - lo) / s), 0, 2^b - 1),  q = clamp(rint(v / s) + z, 0, 2^b - 1)
// Its output feeds dz_pack_delta.  One wave handles 256 dense columns of one row: lane l owns the
// group of four l, picks its two entries, and the lanes of a quantisation group (group / 4 of them)
// find the group's range with lane exchanges.  Memory-bound and off the per-token path.
#include "dz_internal.h"

namespace {

__global__ __launch_bounds__(256) void compress_kernel(const _Float16 *__restrict__ delta, int N, int K, int bits, int group,
                                                        uint8_t *__restrict__ codes, uint8_t *__restrict__ idx,
                                                        _Float16 *__restrict__ scale, _Float16 *__restrict__ zero)
{
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int KT = K >> 8;
    if (wave >= (long long)N * KT) return;
    const int n = (int)(wave / KT), kt = (int)(wave - (long long)n * KT);
    const int g4 = kt * 64 + lane;                  // group of four along k
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    const h4 raw = *(const h4 *)(delta + (size_t)n * K + 4 * (size_t)g4);
    const float v[4] = {(float)raw.x, (float)raw.y, (float)raw.z, (float)raw.w};
    // rank by (magnitude descending, position ascending): entry i is kept if it beats at least two others
    int first = -1, second = -1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int wins = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j != i) wins += (fabsf(v[i]) > fabsf(v[j]) || (fabsf(v[i]) == fabsf(v[j]) && i < j)) ? 1 : 0;
        if (wins >= 2) {
            if (first < 0) first = i; else second = i;
        }
    }
    const float k0 = v[first], k1 = v[second];
    // range of the quantisation group: group / 4 consecutive lanes
    float lo = fminf(0.f, fminf(k0, k1)), hi = fmaxf(0.f, fmaxf(k0, k1));
    for (int d = group / 8; d >= 1; d >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, d, 64));
        hi = fmaxf(hi, __shfl_xor(hi, d, 64));
    }
    const float qmax = (float)((1 << bits) - 1);
    _Float16 s16 = (_Float16)((hi - lo) / qmax);
    const bool dead = (float)s16 == 0.f;
    if (dead) s16 = (_Float16)1.f;
    const float s = (float)s16;
    float z = fminf(fmaxf(rintf((0.f - lo) / s), 0.f), qmax);
    if (dead) z = 0.f;
    const float q0 = fminf(fmaxf(rintf(k0 / s) + z, 0.f), qmax);
    const float q1 = fminf(fmaxf(rintf(k1 / s) + z, 0.f), qmax);
    const size_t e = (size_t)n * (K / 2) + 2 * (size_t)g4;
    codes[e] = (uint8_t)q0; codes[e + 1] = (uint8_t)q1;
    idx[e] = (uint8_t)first; idx[e + 1] = (uint8_t)second;
    if ((lane & (group / 4 - 1)) == 0) {
        const size_t gq = (size_t)n * (K / group) + (size_t)(4 * g4) / group;
        scale[gq] = s16;
        zero[gq] = (_Float16)z;
    }
}

}  // namespace

int dz_launch_compress(dz_ctx *ctx, const void *delta, int N, int K, int bits, int group, uint8_t *codes, uint8_t *idx,
                       void *scale, void *zero, hipStream_t st)
{
    const long long waves = (long long)N * (K / 256);
    const long long blocks = (waves + 3) / 4;
    if (blocks > 0x7fffffffLL) return DZ_ERR_SHAPE;
    hipLaunchKernelGGL(compress_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const _Float16 *)delta, N, K, bits, group,
                       codes, idx, (_Float16 *)scale, (_Float16 *)zero);
    return dz_set_hip_error(ctx, hipGetLastError());
}

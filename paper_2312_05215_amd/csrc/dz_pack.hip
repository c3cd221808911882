// dz_pack_delta / dz_unpack_delta kernels: canonical tables <-> streaming layout (dz_layout.h).
// Off the per-token path (run once per delta, the packing step that ends Algorithm 1), so these are plain
// gather kernels: one thread per packed dword (pack) or per group of four (unpack).
#include "dz_internal.h"

namespace {

// One thread builds one dword of plane C (and, for it, the matching position bits).
// 4-bit: dword (tile, lane, step) holds 8 codes; position dword (tile, lane, h) holds 2 steps.
// 2-bit: dword (tile, lane, c) c<2 holds 16 codes of steps 2c, 2c+1; dwords 2,3 hold positions.
__global__ void pack_codes_kernel(DzLayout L, const uint8_t *__restrict__ codes, uint32_t *__restrict__ out)
{
    const size_t tiles = (size_t)L.RT * L.KT;
    const size_t total = tiles * 64 * (L.bits == 4 ? 4 : 2);
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int per_lane = (L.bits == 4) ? 4 : 2;
    int d = (int)(i % per_lane);
    int lane = (int)((i / per_lane) % 64);
    size_t tile = i / ((size_t)per_lane * 64);
    int rt = (int)(tile / L.KT), kt = (int)(tile % L.KT);
    int n = rt * 16 + (lane & 15), q = lane >> 4;
    const uint8_t *row = codes + (size_t)n * (L.K / 2);
    uint32_t w = 0;
    const uint32_t mask = (1u << L.bits) - 1u;
    const int nsteps = (L.bits == 4) ? 1 : 2;
    for (int ss = 0; ss < nsteps; ++ss) {
        int step = (L.bits == 4) ? d : 2 * d + ss;
        int k = kt * 256 + step * 64 + q * 16;          // first dense column of this lane's step
        for (int e = 0; e < 8; ++e) {
            uint32_t c = row[k / 2 + e] & mask;
            int j = e >> 1, h = e & 1;
            int sh = (L.bits == 4) ? 16 * h + 4 * j : 16 * h + 8 * ss + 2 * j;
            w |= c << sh;
        }
    }
    out[(tile * 1024 + (size_t)lane * 16) / 4 + d] = w;
}

__global__ void pack_idx_kernel(DzLayout L, const uint8_t *__restrict__ idx, uint32_t *__restrict__ out)
{
    const size_t tiles = (size_t)L.RT * L.KT;
    const size_t total = tiles * 64 * 2;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int h = (int)(i % 2);
    int lane = (int)((i / 2) % 64);
    size_t tile = i / 128;
    int rt = (int)(tile / L.KT), kt = (int)(tile % L.KT);
    int n = rt * 16 + (lane & 15), q = lane >> 4;
    const uint8_t *row = idx + (size_t)n * (L.K / 2);
    uint32_t w = 0;
    for (int ss = 0; ss < 2; ++ss) {
        int step = 2 * h + ss;
        int k = kt * 256 + step * 64 + q * 16;
        for (int e = 0; e < 8; ++e) w |= (uint32_t)(row[k / 2 + e] & 3u) << (16 * ss + 2 * e);
    }
    size_t dw = (L.bits == 4) ? (L.off_idx + tile * 512 + (size_t)lane * 8) / 4 + h
                              : (tile * 1024 + (size_t)lane * 16) / 4 + 2 + h;
    out[dw] = w;
}

__global__ void pack_scale_kernel(DzLayout L, const uint16_t *__restrict__ scale,
                                  const uint16_t *__restrict__ zero, uint32_t *__restrict__ out)
{
    const int ng = L.K / L.group;
    size_t total = (size_t)L.N * ng;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int n = (int)(i / ng), gq = (int)(i % ng);
    out[dz_scale_dword(L, n, gq)] = (uint32_t)scale[i] | ((uint32_t)zero[i] << 16);
}

__device__ inline float half_bits_to_float(uint16_t h)
{
    _Float16 v;
    __builtin_memcpy(&v, &h, 2);
    return (float)v;
}

// One thread per (row, group of four): writes the two codes, two positions and, if asked, the
// four dense fp32 values  (code - zero) * scale  (an exact product in fp32).
__global__ void unpack_kernel(DzLayout L, const uint32_t *__restrict__ blob, uint8_t *__restrict__ codes,
                              uint8_t *__restrict__ idx, float *__restrict__ dense)
{
    const int g4n = L.K / 4;
    size_t total = (size_t)L.N * g4n;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int n = (int)(i / g4n), g4 = (int)(i % g4n);
    const uint32_t mask = (1u << L.bits) - 1u;
    uint32_t c[2], p[2];
    for (int j = 0; j < 2; ++j) {
        DzSlot s = dz_slot_of(L, n, 2 * g4 + j);
        c[j] = (blob[dz_code_dword(L, s)] >> dz_code_shift(L, s)) & mask;
        p[j] = (blob[dz_idx_dword(L, s)] >> dz_idx_shift(s)) & 3u;
    }
    size_t e = (size_t)n * (L.K / 2) + 2 * (size_t)g4;
    if (codes) { codes[e] = (uint8_t)c[0]; codes[e + 1] = (uint8_t)c[1]; }
    if (idx) { idx[e] = (uint8_t)p[0]; idx[e + 1] = (uint8_t)p[1]; }
    if (dense) {
        uint32_t sz = blob[dz_scale_dword(L, n, (4 * g4) / L.group)];
        float s = half_bits_to_float((uint16_t)(sz & 0xffff));
        float z = half_bits_to_float((uint16_t)(sz >> 16));
        float a = ((float)c[0] - z) * s, b = ((float)c[1] - z) * s;
        float *o = dense + (size_t)n * L.K + 4 * (size_t)g4;
#pragma unroll
        for (uint32_t pos = 0; pos < 4; ++pos) o[pos] = (p[1] == pos) ? b : (p[0] == pos) ? a : 0.f;
    }
}

__global__ void unpack_scale_kernel(DzLayout L, const uint32_t *__restrict__ blob,
                                    uint16_t *__restrict__ scale, uint16_t *__restrict__ zero)
{
    const int ng = L.K / L.group;
    size_t total = (size_t)L.N * ng;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int n = (int)(i / ng), gq = (int)(i % ng);
    uint32_t sz = blob[dz_scale_dword(L, n, gq)];
    if (scale) scale[i] = (uint16_t)(sz & 0xffff);
    if (zero) zero[i] = (uint16_t)(sz >> 16);
}

// ---- quantisation-only format: one thread per dword of codes (pack) or per column (unpack)
__global__ void qpack_codes_kernel(DzLayout L, const uint8_t *__restrict__ codes, uint32_t *__restrict__ out)
{
    const int per_dword = 32 / L.bits;                  // 8 or 16 codes
    const size_t total = (size_t)L.N * L.K / per_dword;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    // dword i of plane C: find (tile, half, lane, dword-in-lane), then gather its codes
    const size_t tile_dwords = (L.bits == 4) ? 512 : 256;
    const size_t tile = i / tile_dwords;
    const int r = (int)(i % tile_dwords);
    int h, lane, d;
    if (L.bits == 4) { h = r / 256; lane = (r % 256) / 4; d = r % 4; }
    else { lane = r / 4; d = r % 4; h = d >> 1; }
    const int rt = (int)(tile / L.KT), kt = (int)(tile % L.KT);
    const int n = rt * 16 + (lane & 15), q = lane >> 4;
    const uint8_t *row = codes + (size_t)n * L.K;
    const uint32_t mask = (1u << L.bits) - 1u;
    uint32_t w = 0;
    const int nsteps = (L.bits == 4) ? 1 : 2;
    for (int ss = 0; ss < nsteps; ++ss) {
        const int step = (L.bits == 4) ? d : 2 * (d & 1) + ss;
        const int k0 = kt * 256 + step * 64 + q * 16;   // first column of this lane's step
        for (int j = 0; j < 4; ++j)
            for (int hh = 0; hh < 2; ++hh) {
                const uint32_t c = row[k0 + 4 * j + 2 * h + hh] & mask;
                w |= c << ((L.bits == 4) ? 16 * hh + 4 * j : 16 * hh + 8 * ss + 2 * j);
            }
    }
    out[i] = w;
}

__global__ void qunpack_kernel(DzLayout L, const uint32_t *__restrict__ blob, uint8_t *__restrict__ codes,
                               float *__restrict__ dense)
{
    const size_t total = (size_t)L.N * L.K;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int n = (int)(i / L.K), k = (int)(i % L.K);
    const uint32_t c = (blob[dz_qcode_dword(L, n, k)] >> dz_qcode_shift(L, k)) & ((1u << L.bits) - 1u);
    if (codes) codes[i] = (uint8_t)c;
    if (dense) {
        const uint32_t sz = blob[dz_scale_dword(L, n, k / L.group)];
        dense[i] = ((float)c - half_bits_to_float((uint16_t)(sz >> 16))) * half_bits_to_float((uint16_t)(sz & 0xffff));
    }
}

// merged[n][k] = f16( float(W[n][k]) + (code - zero) * scale at the kept columns ): one thread per
// group of four columns of a 2:4 blob
__global__ void merge_kernel(DzLayout L, const _Float16 *__restrict__ W, const uint32_t *__restrict__ blob,
                             _Float16 *__restrict__ merged)
{
    const int g4n = L.K / 4;
    size_t total = (size_t)L.N * g4n;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int n = (int)(i / g4n), g4 = (int)(i % g4n);
    const uint32_t mask = (1u << L.bits) - 1u;
    const uint32_t sz = blob[dz_scale_dword(L, n, (4 * g4) / L.group)];
    const float s = half_bits_to_float((uint16_t)(sz & 0xffff)), z = half_bits_to_float((uint16_t)(sz >> 16));
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    const h4 w = *(const h4 *)(W + (size_t)n * L.K + 4 * (size_t)g4);
    float v[4] = {(float)w.x, (float)w.y, (float)w.z, (float)w.w};
    for (int j = 0; j < 2; ++j) {
        const DzSlot sl = dz_slot_of(L, n, 2 * g4 + j);
        const uint32_t c = (blob[dz_code_dword(L, sl)] >> dz_code_shift(L, sl)) & mask;
        const uint32_t p = (blob[dz_idx_dword(L, sl)] >> dz_idx_shift(sl)) & 3u;
        const float d = ((float)c - z) * s;
#pragma unroll
        for (uint32_t pos = 0; pos < 4; ++pos) v[pos] += (p == pos) ? d : 0.f;
    }
    *(h4 *)(merged + (size_t)n * L.K + 4 * (size_t)g4) = (h4){(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
}

inline unsigned blocks_for(size_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

}  // namespace

int dz_launch_pack(dz_ctx *ctx, const uint8_t *codes, const uint8_t *idx, const void *scale,
                   const void *zero, int N, int K, int bits, int group, void *packed, hipStream_t st)
{
    DzLayout L = dz_make_layout(N, K, bits, group);
    const int bs = 256;
    size_t tiles = (size_t)L.RT * L.KT;
    hipLaunchKernelGGL(pack_codes_kernel, dim3(blocks_for(tiles * 64 * (bits == 4 ? 4 : 2), bs)), dim3(bs), 0,
                       st, L, codes, (uint32_t *)packed);
    hipLaunchKernelGGL(pack_idx_kernel, dim3(blocks_for(tiles * 128, bs)), dim3(bs), 0, st, L, idx,
                       (uint32_t *)packed);
    hipLaunchKernelGGL(pack_scale_kernel, dim3(blocks_for((size_t)N * (K / group), bs)), dim3(bs), 0, st, L,
                       (const uint16_t *)scale, (const uint16_t *)zero, (uint32_t *)packed);
    return dz_set_hip_error(ctx, hipGetLastError());
}

int dz_launch_unpack(dz_ctx *ctx, const void *packed, int N, int K, int bits, int group, uint8_t *codes,
                     uint8_t *idx, void *scale, void *zero, float *dense, hipStream_t st)
{
    DzLayout L = dz_make_layout(N, K, bits, group);
    const int bs = 256;
    if (codes || idx || dense)
        hipLaunchKernelGGL(unpack_kernel, dim3(blocks_for((size_t)N * (K / 4), bs)), dim3(bs), 0, st, L,
                           (const uint32_t *)packed, codes, idx, dense);
    if (scale || zero)
        hipLaunchKernelGGL(unpack_scale_kernel, dim3(blocks_for((size_t)N * (K / group), bs)), dim3(bs), 0, st,
                           L, (const uint32_t *)packed, (uint16_t *)scale, (uint16_t *)zero);
    return dz_set_hip_error(ctx, hipGetLastError());
}

int dz_launch_qpack(dz_ctx *ctx, const uint8_t *codes, const void *scale, const void *zero, int N, int K, int bits,
                    int group, void *packed, hipStream_t st)
{
    DzLayout L = dz_make_qlayout(N, K, bits, group);
    const int bs = 256;
    hipLaunchKernelGGL(qpack_codes_kernel, dim3(blocks_for((size_t)N * K * bits / 32, bs)), dim3(bs), 0, st, L, codes,
                       (uint32_t *)packed);
    hipLaunchKernelGGL(pack_scale_kernel, dim3(blocks_for((size_t)N * (K / group), bs)), dim3(bs), 0, st, L,
                       (const uint16_t *)scale, (const uint16_t *)zero, (uint32_t *)packed);
    return dz_set_hip_error(ctx, hipGetLastError());
}

int dz_launch_qunpack(dz_ctx *ctx, const void *packed, int N, int K, int bits, int group, uint8_t *codes, void *scale,
                      void *zero, float *dense, hipStream_t st)
{
    DzLayout L = dz_make_qlayout(N, K, bits, group);
    const int bs = 256;
    if (codes || dense)
        hipLaunchKernelGGL(qunpack_kernel, dim3(blocks_for((size_t)N * K, bs)), dim3(bs), 0, st, L, (const uint32_t *)packed,
                           codes, dense);
    if (scale || zero)
        hipLaunchKernelGGL(unpack_scale_kernel, dim3(blocks_for((size_t)N * (K / group), bs)), dim3(bs), 0, st, L,
                           (const uint32_t *)packed, (uint16_t *)scale, (uint16_t *)zero);
    return dz_set_hip_error(ctx, hipGetLastError());
}

int dz_launch_merge(dz_ctx *ctx, const void *W, const void *packed, int N, int K, int bits, int group, void *merged,
                    hipStream_t st)
{
    DzLayout L = dz_make_layout(N, K, bits, group);
    hipLaunchKernelGGL(merge_kernel, dim3(blocks_for((size_t)N * (K / 4), 256)), dim3(256), 0, st, L, (const _Float16 *)W,
                       (const uint32_t *)packed, (_Float16 *)merged);
    return dz_set_hip_error(ctx, hipGetLastError());
}

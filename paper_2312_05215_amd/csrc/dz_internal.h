// Internal declarations shared by the translation units of libdz.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dz.h"
#include "dz_layout.h"

struct dz_ctx {
    int device = 0;
    // workspace (device memory owned by the context)
    int32_t *seg_perm = nullptr;    // [seg_cap] request indices in delta-sorted order
    int32_t *seg_key = nullptr;     // [seg_cap] delta index of each sorted position (D = none)
    int32_t *seg_counts = nullptr;  // [DZ_SEG_MAX_D + 1]
    int32_t *seg_offsets = nullptr; // [DZ_SEG_MAX_D + 2]
    int seg_cap = 0;
    float *partial = nullptr;       // split-K partial sums
    size_t partial_bytes = 0;
    int32_t *counters = nullptr;    // arrival counters, one per (chunk, row block); all zero between calls
    int counters_cap = 0;
    int32_t *err_flag = nullptr;    // sticky device-side error word
    float *lora_u = nullptr;        // low-rank SBMM: x . A^T of every request, fp32 [T][rank]
    size_t lora_u_bytes = 0;
    // Buffers a growth replaced.  A HIP graph recorded earlier may still hold their addresses in its
    // kernel nodes, so they stay allocated until dz_destroy.
    void *retired[64] = {};
    int n_retired = 0;
    bool static_ws = false;         // the workspace is the library's static device array: it never grows
    char hip_err[256] = {};
    // options (dz_set_option)
    int force_splits = 0;           // DZ_OPT_SPLIT_K
    int target_wgs = 0;             // DZ_OPT_WORKGROUPS
    int round_tiles = 0;            // DZ_OPT_ROUND_TILES
    int no_prefill = 0;             // DZ_OPT_LARGE_BATCH_STREAMING
    int num_cus = 0;                // compute units of the device
    int tile_kernel = 1;            // DZ_OPT_WIDE_TILE
    int reuse_segments = 0;         // DZ_OPT_REUSE_SEGMENTS
    // the request order the last segment pass left in seg_perm / seg_key
    const int32_t *seg_ids = nullptr;
    int seg_T = -1, seg_D = -1;
};

#define DZ_SEG_MAX_D 8192

struct DzDeltaPtrs { const void *p[DZ_MAX_DELTAS]; };

// Several projections that share x and the request indices (q,k,v or gate,up of one transformer
// layer) can go through the streaming kernel in one launch.  Filled in part by the caller (P, N, W,
// out) and in part by the launcher.
#define DZ_GROUP_PTRS (3 * DZ_MAX_DELTAS)       /* projections x deltas of one launch */
struct DzGroupPtrs { const void *p[DZ_GROUP_PTRS]; };   // packed deltas, projection-major: p[proj * D + delta]
struct DzGroup {
    int P;                              // projections (1 .. DZ_MAX_GROUP)
    int rb_start[DZ_MAX_GROUP + 1];     // first row block of each projection in the concatenated numbering
    int N[DZ_MAX_GROUP];                // output features of each projection
    int n_off[DZ_MAX_GROUP];            // first column of each projection in the partial-sum tiles
    const void *W[DZ_MAX_GROUP];        // [N[p]][K] fp16
    void *out[DZ_MAX_GROUP];            // [T][N[p]] fp16
    uint32_t off_idx[DZ_MAX_GROUP], off_scale[DZ_MAX_GROUP], blob_total[DZ_MAX_GROUP];   // packed layout of each projection
};

// One launch of the streaming kernel (decode-shaped; large T is processed as chunks of 64 rows).
struct DzStreamArgs {
    const void *x;              // [T][K] fp16
    const void *W;              // [N][K] fp16 or null
    void *out;                  // [T][N] fp16
    const int32_t *perm;        // sorted request order or null (identity)
    const int32_t *key;         // delta of each sorted position or null (no deltas)
    const int32_t *ids;         // raw request->delta indices: the kernel sorts them itself (T <= 64)
    int32_t *err_flag;
    float *partial;
    int32_t *counters;
    int T, N, K, D, bits, group;   // streaming kernel: N = sum over the projections of the launch
    int accumulate;
    int S;                      // streaming kernel: workgroups per chunk of 64 request rows; tiled kernel: k slices per tile
    int max_slots;              // most workgroups sharing one row block (partial-sum slots)
    int has_base, has_delta;
    int quant_only;             // the packed deltas are in the quantisation-only format (no 2:4 pruning)
};

int dz_set_hip_error(dz_ctx *ctx, hipError_t e);
// one projection through the same dispatch as the public entry points (which are thin wrappers of it)
extern "C" int dz_run_linear(dz_ctx *ctx, const void *x, const void *W, const void *const *deltas, int D,
                             const int32_t *ids, void *out, int T, int N, int K, int bits, int group, int accumulate,
                             bool has_base, bool has_delta, hipStream_t st);
int dz_ensure_partial(dz_ctx *ctx, size_t bytes, hipStream_t st);
int dz_ensure_counters(dz_ctx *ctx, int n, hipStream_t st);
int dz_ensure_lora(dz_ctx *ctx, size_t bytes, hipStream_t st);

// A kernel may use more than 64 KB of dynamic LDS only after an attribute has been set for it, once
// per device.  `done` (one static word per kernel instantiation) remembers the devices it has been
// set on; two threads racing here at worst set it twice, which is harmless.
inline hipError_t dz_allow_lds(const void *kernel, int bytes, unsigned long long &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done |= bit;
    return e;
}
int dz_launch_pack(dz_ctx *, const uint8_t *, const uint8_t *, const void *, const void *, int, int,
                   int, int, void *, hipStream_t);
int dz_launch_unpack(dz_ctx *, const void *, int, int, int, int, uint8_t *, uint8_t *, void *, void *,
                     float *, hipStream_t);
int dz_launch_segment(dz_ctx *, const int32_t *ids, int T, int D, int32_t *counts, int32_t *offsets,
                      int32_t *perm, int32_t *key, hipStream_t);
int dz_launch_stream(dz_ctx *, const DzStreamArgs &, const DzGroup &, const DzGroupPtrs &, hipStream_t);
int dz_launch_prefill(dz_ctx *, const DzStreamArgs &, const DzDeltaPtrs &, hipStream_t);
int dz_launch_tile(dz_ctx *, const DzStreamArgs &, hipStream_t);
bool dz_tile_fits(const DzStreamArgs &);
int dz_launch_qpack(dz_ctx *, const uint8_t *codes, const void *scale, const void *zero, int N, int K, int bits, int group,
                    void *packed, hipStream_t);
int dz_launch_qunpack(dz_ctx *, const void *packed, int N, int K, int bits, int group, uint8_t *codes, void *scale,
                      void *zero, float *dense, hipStream_t);
int dz_launch_merge(dz_ctx *, const void *W, const void *packed, int N, int K, int bits, int group, void *merged, hipStream_t);
int dz_launch_compress(dz_ctx *, const void *delta, int N, int K, int bits, int group, uint8_t *codes, uint8_t *idx,
                       void *scale, void *zero, hipStream_t);
int dz_launch_lora(dz_ctx *, const void *x, const void *const *A, const void *const *B, int D, int rank, const int32_t *ids,
                   const int32_t *perm, float *u, void *out, int T, int N, int K, int accumulate, hipStream_t);

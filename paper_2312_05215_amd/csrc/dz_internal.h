// Internal declarations shared by the translation units of libdz.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dz.h"
#include "dz_layout.h"

struct dz_ctx {
    int device;
    // workspace (device memory owned by the context)
    int32_t *seg_perm;      // [seg_cap] request indices in delta-sorted order
    int32_t *seg_key;       // [seg_cap] delta index of each sorted position (D = none)
    int32_t *seg_counts;    // [DZ_SEG_MAX_D + 1]
    int32_t *seg_offsets;   // [DZ_SEG_MAX_D + 2]
    int seg_cap;
    float *partial;         // split-K partial sums
    size_t partial_bytes;
    int32_t *counters;      // arrival counters, one per (chunk, row block); all zero between calls
    int counters_cap;
    int32_t *err_flag;      // sticky device-side error word
    char hip_err[256];
    // tuning knobs (environment overrides, read once)
    int force_splits;       // DZ_SPLITS
    int target_wgs;         // DZ_TARGET_WGS
    int round_tiles;        // DZ_ROUND_TILES
    int no_prefill;         // DZ_NO_PREFILL: serve large batches with the streaming kernel (chunks of 64 rows)
    int wg_waves, wg_rtiles; // DZ_WAVES, DZ_RTILES: workgroup shape of the streaming kernel
#ifdef DZ_PROF
    long long *prof;
#endif
};

#define DZ_SEG_MAX_D 8192

struct DzDeltaPtrs { const void *p[DZ_MAX_DELTAS]; };

// One launch of the streaming kernel (decode-shaped; large T is processed as chunks of 64 rows).
struct DzStreamArgs {
    const void *x;              // [T][K] fp16
    const void *W;              // [N][K] fp16 or null
    void *out;                  // [T][N] fp16
    const int32_t *perm;        // sorted request order or null (identity)
    const int32_t *key;         // delta of each sorted position or null (no deltas)
    const int32_t *ids;         // raw request->delta indices: the kernel sorts them itself (T <= 64)
    int32_t *err_flag;
#ifdef DZ_PROF
    long long *prof;            // 8 timestamps per workgroup (development builds only)
#endif
    float *partial;
    int32_t *counters;
    int T, N, K, D, bits, group;
    int accumulate;
    int S;                      // workgroups per chunk of 64 request rows
    int max_slots;              // most workgroups sharing one row block (partial-sum slots)
    int has_base, has_delta;
};

int dz_set_hip_error(dz_ctx *ctx, hipError_t e);
int dz_launch_pack(dz_ctx *, const uint8_t *, const uint8_t *, const void *, const void *, int, int,
                   int, int, void *, hipStream_t);
int dz_launch_unpack(dz_ctx *, const void *, int, int, int, int, uint8_t *, uint8_t *, void *, void *,
                     float *, hipStream_t);
int dz_launch_segment(dz_ctx *, const int32_t *ids, int T, int D, int32_t *counts, int32_t *offsets,
                      int32_t *perm, int32_t *key, hipStream_t);
int dz_launch_stream(dz_ctx *, const DzStreamArgs &, const DzDeltaPtrs &, hipStream_t);
int dz_launch_prefill(dz_ctx *, const DzStreamArgs &, const DzDeltaPtrs &, hipStream_t);

// dz_linear_static: the fused linear layer for callers that cannot allocate (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  Same kernels as dz_linear; the
// workspace they need -- split-k partial sums, arrival counters, the sticky error word -- is a
// file-scope device array instead of memory the context allocates.
//
// The array's name is only a host-side handle.  Its address on a GPU comes from
// hipGetSymbolAddress with that GPU current, looked up once per device (at dz_create, else at the
// first call) and kept; every use below goes through that pointer.  Each GPU holds its own copy of
// the array, from the moment the code object is loaded there until the process ends.
#include "dz_internal.h"

namespace {

// Layout: [0, 256) the sticky error word; then DZ_STATIC_COUNTERS arrival counters; then
// DZ_STATIC_PARTIAL_BYTES of split-k partial sums.
constexpr size_t DZ_STATIC_COUNTERS = 16384;
constexpr size_t DZ_STATIC_COUNTER_OFF = 256;
constexpr size_t DZ_STATIC_PARTIAL_OFF = DZ_STATIC_COUNTER_OFF + DZ_STATIC_COUNTERS * 4;
constexpr size_t DZ_STATIC_BYTES = DZ_STATIC_PARTIAL_OFF + DZ_STATIC_PARTIAL_BYTES;

}  // namespace

static __device__ __align__(256) unsigned char scratch[DZ_STATIC_BYTES];

namespace {

constexpr int DZ_MAX_DEVICES = 64;
unsigned char *g_scratch_ptr[DZ_MAX_DEVICES];   // device address of `scratch` on each GPU, null until looked up
int g_scratch_cus[DZ_MAX_DEVICES];

// `device` must be current.  Not an allocation: the array already exists on the device.
hipError_t scratch_lookup(int device)
{
    if (device < 0 || device >= DZ_MAX_DEVICES) return hipErrorInvalidDevice;
    if (g_scratch_ptr[device]) return hipSuccess;
    void *ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device);
    if (e != hipSuccess) return e;
    g_scratch_cus[device] = n;
    g_scratch_ptr[device] = (unsigned char *)ptr;
    return hipSuccess;
}

struct CurrentDevice {
    int prev = -1;
    bool ok = false;
    explicit CurrentDevice(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    }
    ~CurrentDevice() { if (prev >= 0) (void)hipSetDevice(prev); }
};

__global__ void static_clear_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace

extern "C" {

// Address of the static workspace's error word on `device` (looks the array up if that has not
// happened yet); null if the lookup fails.  dz_create calls this as part of the library's set-up,
// dz_check to report what dz_linear_static flagged.
int32_t *dz_static_err_word(int device)
{
    CurrentDevice cur(device);
    if (!cur.ok || scratch_lookup(device) != hipSuccess) return nullptr;
    return (int32_t *)g_scratch_ptr[device];
}

int dz_linear_static(int device, const void *x, const void *W, const void *const *deltas, int D, const int32_t *ids,
                     void *out, int T, int N, int K, int bits, int group, void *stream)
{
    if (device < 0 || device >= DZ_MAX_DEVICES) return DZ_ERR_ARG;
    if (T > 64) return DZ_ERR_LIMIT;            // larger batches need the sorted-order workspace too
    CurrentDevice cur(device);
    if (!cur.ok) return DZ_ERR_HIP;
    if (scratch_lookup(device) != hipSuccess) return DZ_ERR_HIP;
    unsigned char *base = g_scratch_ptr[device];
    dz_ctx ctx;                                     // a view of the static workspace; owns nothing
    ctx.device = device;
    ctx.static_ws = true;
    ctx.num_cus = g_scratch_cus[device];
    ctx.err_flag = (int32_t *)base;
    ctx.counters = (int32_t *)(base + DZ_STATIC_COUNTER_OFF);
    ctx.counters_cap = (int)DZ_STATIC_COUNTERS;
    ctx.partial = (float *)(base + DZ_STATIC_PARTIAL_OFF);
    ctx.partial_bytes = DZ_STATIC_PARTIAL_BYTES;
    hipStream_t st = (hipStream_t)stream;
    // The array keeps what the last call left in it.  The arrival counters must start at zero: every
    // launch leaves them at zero again, but a launch that was torn down half way would not have, so
    // they are cleared here -- with a kernel, which a stream under capture records like any other.
    if (T > 0) {
        hipLaunchKernelGGL(static_clear_kernel, dim3((unsigned)(DZ_STATIC_COUNTERS / 256)), dim3(256), 0, st, ctx.counters,
                           (int)DZ_STATIC_COUNTERS);
        if (hipGetLastError() != hipSuccess) return DZ_ERR_HIP;
    }
    return dz_run_linear(&ctx, x, W, deltas, D, ids, out, T, N, K, bits, group, 0, true, true, st);
}

}  // extern "C"

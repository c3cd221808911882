// Resident-delta cache: a fixed pool of device buffers for packed deltas, filled from host memory
// on demand with asynchronous copies, least recently used delta evicted first (the engine keeps the
// base model on the GPU and swaps compressed deltas in as requests need them: paper Section 5.1 and
// Section 5.4, paragraph "Scalability").  Host code only; see include/dz.h for the contract.
#include "dz_internal.h"
#include <new>
#include <unordered_map>
#include <unordered_set>
#include <vector>

struct dz_cache {
    int device = -1;                    // < 0: decisions only, no device memory
    int slots = 0;
    size_t slot_bytes = 0;
    char *pool = nullptr;               // slots * slot_bytes of device memory
    std::vector<int64_t> key;           // delta held by each slot
    std::vector<char> used;
    std::vector<uint64_t> tick;         // when the slot was last handed out
    std::vector<long long> call_no;     // number (ticket) of the acquire call that last handed it out
    std::vector<hipEvent_t> ready;      // the last copy into the slot has finished
    std::vector<hipEvent_t> done;       // the last compute that read the slot has finished (dz_cache_release)
    std::vector<long long> done_for;    // ticket done[s] was recorded for (-1: never)
    std::unordered_map<int64_t, int> where;
    std::unordered_map<long long, std::vector<int>> ticket_slots;   // slots each unreleased ticket handed out
    uint64_t clock = 0;
    long long call = 0;
    int64_t hits = 0, misses = 0, evictions = 0;
};

namespace {

struct CacheDeviceGuard {
    int prev = -1;
    bool active = false, ok = true;
    explicit CacheDeviceGuard(int device)
    {
        if (device < 0) return;
        active = true;
        ok = hipGetDevice(&prev) == hipSuccess && hipSetDevice(device) == hipSuccess;
    }
    ~CacheDeviceGuard()
    {
        if (active && prev >= 0) (void)hipSetDevice(prev);
    }
};

}  // namespace

extern "C" {

int dz_cache_create(dz_cache **out, int device, int slots, size_t slot_bytes)
{
    if (!out || slots <= 0 || slot_bytes == 0) return DZ_ERR_ARG;
    *out = nullptr;
    dz_cache *c = new (std::nothrow) dz_cache();
    if (!c) return DZ_ERR_ARG;
    c->device = device < 0 ? -1 : device;
    c->slots = slots;
    c->slot_bytes = (slot_bytes + 255) & ~(size_t)255;      // keeps every slot 256-byte aligned
    c->key.assign(slots, 0);
    c->used.assign(slots, 0);
    c->tick.assign(slots, 0);
    c->call_no.assign(slots, -2);
    c->done_for.assign(slots, -1);
    if (c->device >= 0) {
        CacheDeviceGuard guard(c->device);
        hipError_t e = guard.ok ? hipSuccess : hipErrorInvalidDevice;
        if (e == hipSuccess) e = hipMalloc((void **)&c->pool, (size_t)slots * c->slot_bytes);
        c->ready.assign(slots, nullptr);
        c->done.assign(slots, nullptr);
        for (int s = 0; s < slots && e == hipSuccess; ++s) e = hipEventCreateWithFlags(&c->ready[s], hipEventDisableTiming);
        for (int s = 0; s < slots && e == hipSuccess; ++s) e = hipEventCreateWithFlags(&c->done[s], hipEventDisableTiming);
        if (e != hipSuccess) {
            dz_cache_destroy(c);
            return DZ_ERR_HIP;
        }
    }
    *out = c;
    return DZ_OK;
}

int dz_cache_destroy(dz_cache *c)
{
    if (!c) return DZ_ERR_ARG;
    if (c->device >= 0) {
        CacheDeviceGuard guard(c->device);
        (void)hipDeviceSynchronize();
        for (hipEvent_t ev : c->ready)
            if (ev) (void)hipEventDestroy(ev);
        for (hipEvent_t ev : c->done)
            if (ev) (void)hipEventDestroy(ev);
        if (c->pool) (void)hipFree(c->pool);
    }
    delete c;
    return DZ_OK;
}

int dz_cache_acquire(dz_cache *c, int n, const int64_t *keys, const void *const *host_blobs, size_t bytes,
                     const void **device_blobs_out, int32_t *slot_out, int32_t *hit_out, void *copy_stream,
                     int64_t *ticket_out)
{
    if (!c || n < 0) return DZ_ERR_ARG;
    if (ticket_out) *ticket_out = 0;
    if (n == 0) return DZ_OK;
    const bool dry = c->device < 0;
    if (!keys || !device_blobs_out || bytes > c->slot_bytes || (!dry && !host_blobs)) return DZ_ERR_ARG;

    // Can every missing key get a slot?  Slots of this call's resident keys and of the previous
    // call are not available.  Checked before anything changes.
    std::unordered_set<int64_t> wanted(keys, keys + n);
    int missing = 0;
    for (int64_t k : wanted)
        if (!c->where.count(k)) ++missing;
    if (!dry)
        for (int i = 0; i < n; ++i)
            if (!c->where.count(keys[i]) && !host_blobs[i]) return DZ_ERR_ARG;
    const long long prev_call = c->call;
    int available = 0;
    for (int s = 0; s < c->slots; ++s) {
        if (!c->used[s]) ++available;
        else if (c->call_no[s] != prev_call && !wanted.count(c->key[s])) ++available;
    }
    if (missing > available) return DZ_ERR_ARG;

    const long long this_call = ++c->call;
    CacheDeviceGuard guard(c->device);
    if (!guard.ok) { --c->call; return DZ_ERR_HIP; }
    hipStream_t cs = (hipStream_t)copy_stream;
    // A failure half way leaves a consistent table: a slot's mapping changes only after its copy has
    // been enqueued, so a slot whose copy never started still holds, and is still listed under, its old
    // delta.
    int orphan = -1;        // slot whose copy was enqueued but whose ready event could not be recorded
    std::vector<int> handed;
    bool synced = false;
    int rc = DZ_OK;
    int i = 0;
    for (; i < n; ++i) {
        const int64_t k = keys[i];
        int s;
        auto it = c->where.find(k);
        const bool hit = it != c->where.end();
        if (hit) {
            s = it->second;
        } else {
            s = -1;
            for (int t = 0; t < c->slots && s < 0; ++t)
                if (!c->used[t]) s = t;
            bool evict = false;
            if (s < 0) {
                for (int t = 0; t < c->slots; ++t) {
                    if (c->call_no[t] == prev_call || c->call_no[t] == this_call || wanted.count(c->key[t])) continue;
                    if (s < 0 || c->tick[t] < c->tick[s]) s = t;
                }
                if (s < 0) { rc = DZ_ERR_ARG; break; }  // cannot happen after the check above
                evict = true;
            }
            if (!dry) {
                hipError_t e = hipSuccess;
                if (evict) {
                    // The delta being evicted may still be read by compute that is enqueued or running:
                    // the copy waits for the event recorded after its last reader (dz_cache_release).
                    // A slot whose last acquire was never released has no such event; then the whole
                    // device is drained once, which is always safe.
                    if (c->done_for[s] == c->call_no[s]) e = hipStreamWaitEvent(cs, c->done[s], 0);
                    else if (!synced) { e = hipDeviceSynchronize(); synced = true; }
                }
                if (e == hipSuccess)
                    e = hipMemcpyAsync(c->pool + (size_t)s * c->slot_bytes, host_blobs[i], bytes, hipMemcpyHostToDevice, cs);
                if (e != hipSuccess) { rc = DZ_ERR_HIP; break; }      // nothing was enqueued for slot s: it keeps its old delta
                if (evict) c->where.erase(c->key[s]);
                c->used[s] = 1; c->key[s] = k; c->where[k] = s;
                e = hipEventRecord(c->ready[s], cs);
                if (e != hipSuccess) { rc = DZ_ERR_HIP; orphan = s; break; }
            } else {
                if (evict) c->where.erase(c->key[s]);
                c->used[s] = 1; c->key[s] = k; c->where[k] = s;
            }
            if (evict) ++c->evictions;
        }
        if (hit) ++c->hits; else ++c->misses;
        c->tick[s] = ++c->clock;
        c->call_no[s] = this_call;
        handed.push_back(s);
        device_blobs_out[i] = dry ? nullptr : (const void *)(c->pool + (size_t)s * c->slot_bytes);
        if (slot_out) slot_out[i] = s;
        if (hit_out) hit_out[i] = hit ? 1 : 0;
    }
    if (rc != DZ_OK) {
        // a slot whose copy was enqueued but whose ready event could not be recorded cannot be
        // handed out safely: forget its mapping (the next request for that delta copies it again)
        if (orphan >= 0) {
            c->where.erase(c->key[orphan]);
            c->used[orphan] = 0;
            c->call_no[orphan] = -2;
        }
        for (int j = i; j < n; ++j) device_blobs_out[j] = nullptr;
    }
    if (!dry) c->ticket_slots[this_call] = handed;
    if (ticket_out) *ticket_out = this_call;
    return rc;
}

int dz_cache_wait(dz_cache *c, int64_t ticket, void *compute_stream)
{
    if (!c) return DZ_ERR_ARG;
    if (c->device < 0 || ticket == 0) return DZ_OK;
    auto it = c->ticket_slots.find(ticket);
    if (it == c->ticket_slots.end()) return DZ_ERR_ARG;
    CacheDeviceGuard guard(c->device);
    if (!guard.ok) return DZ_ERR_HIP;
    // ready[s] is the latest copy into slot s, so this also covers a hit on a delta whose copy an
    // earlier acquire started; a wait on an event that has already happened costs nothing
    for (int s : it->second)
        if (hipStreamWaitEvent((hipStream_t)compute_stream, c->ready[s], 0) != hipSuccess) return DZ_ERR_HIP;
    return DZ_OK;
}

int dz_cache_release(dz_cache *c, int64_t ticket, void *compute_stream)
{
    if (!c) return DZ_ERR_ARG;
    if (c->device < 0 || ticket == 0) return DZ_OK;
    auto it = c->ticket_slots.find(ticket);
    if (it == c->ticket_slots.end()) return DZ_ERR_ARG;
    CacheDeviceGuard guard(c->device);
    if (!guard.ok) return DZ_ERR_HIP;
    int rc = DZ_OK;
    for (int s : it->second) {
        if (c->call_no[s] != ticket) continue;          // a later acquire handed the slot out again: its release covers it
        if (hipEventRecord(c->done[s], (hipStream_t)compute_stream) != hipSuccess) { rc = DZ_ERR_HIP; break; }
        c->done_for[s] = ticket;
    }
    c->ticket_slots.erase(it);
    return rc;
}

int dz_cache_stats(const dz_cache *c, int64_t *hits, int64_t *misses, int64_t *evictions)
{
    if (!c) return DZ_ERR_ARG;
    if (hits) *hits = c->hits;
    if (misses) *misses = c->misses;
    if (evictions) *evictions = c->evictions;
    return DZ_OK;
}

}  // extern "C"

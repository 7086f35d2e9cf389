// C ABI of the library: plan objects, argument checks, per-call pointer tables
// and kernel launches.  Host code; the kernels live in the .hip files beside it.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "kt_internal.h"

// ---- error reporting -------------------------------------------------------

static thread_local char g_err[512] = "";

void kt_set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

extern "C" const char *kt_last_error(void) { return g_err; }
extern "C" const char *kt_version(void) { return "kt 0.1 (gfx950)"; }

extern "C" const char *kt_status_string(kt_status s)
{
    switch (s) {
    case KT_OK: return "KT_OK";
    case KT_EINVAL: return "KT_EINVAL";
    case KT_EALIGN: return "KT_EALIGN";
    case KT_ENOMEM: return "KT_ENOMEM";
    case KT_EHIP: return "KT_EHIP";
    case KT_EUNSUPPORTED: return "KT_EUNSUPPORTED";
    }
    return "KT_?";
}

static kt_status hip_fail(const char *what, hipError_t e)
{
    kt_set_error("%s: %s", what, hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? KT_ENOMEM : KT_EHIP;
}

// True while `s` is recording into a HIP graph.  Under capture the library only
// enqueues kernels: it uploads nothing, allocates nothing and records no events.
static bool capturing(hipStream_t s)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(s, &st) == hipSuccess && st == hipStreamCaptureStatusActive;
}

// No exception may cross the C boundary.
#define KT_GUARD_BEGIN try {
#define KT_GUARD_END(who)                                              \
    }                                                                  \
    catch (const std::bad_alloc &) {                                   \
        kt_set_error("%s: out of host memory", who);                   \
        return KT_ENOMEM;                                              \
    }                                                                  \
    catch (...) {                                                      \
        kt_set_error("%s: unexpected internal error", who);            \
        return KT_EINVAL;                                              \
    }

// ---- store window ------------------------------------------------------------

// The period in nanoseconds: KT_WINDOW_NS, or what the environment variable KT_STORE_WINDOW_NS
// says (read once; 0 switches the windows off, e.g. when other work shares the GPU).
static long window_ns()
{
    static const long ns = [] {
        const char *e = getenv("KT_STORE_WINDOW_NS");
        if (!e || !*e) return (long)KT_WINDOW_NS;
        char *end = nullptr;
        const long v = strtol(e, &end, 10);
        return (end && *end == 0 && v >= 0 && v <= 1000000) ? v : (long)KT_WINDOW_NS;
    }();
    return ns;
}

KtWindow kt_store_window(int K, int64_t ntiles, int64_t min_tiles)
{
    KtWindow off{0, 0};
    const long ns = window_ns();
    if (ns <= 0 || K < 4 || ntiles < min_tiles) return off;
    // rate of the device-wide constant clock in kHz, looked up once per device
    static std::atomic<int> rate_khz[64];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return off;
    int r = rate_khz[dev].load(std::memory_order_relaxed);
    if (r == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeWallClockRate, dev) != hipSuccess || v <= 0) v = -1;
        rate_khz[dev].store(v, std::memory_order_relaxed);
        r = v;
    }
    if (r <= 0) { (void)hipGetLastError(); return off; }
    const uint64_t period = (uint64_t)r * (uint64_t)ns / 1000000;     // ticks
    const uint64_t width = period * KT_WINDOW_OPEN_PCT / 100;
    if (period < 64 || period > (1u << 30) || width < 1) return off;
    return KtWindow{(uint32_t)period, (uint32_t)width};
}

// ---- plan object -----------------------------------------------------------

// A per-call table of device pointers (tensor/bucket or peer/out pointers)
// lives in a small ring of device buffers.  A call whose pointers equal a
// resident table reuses it, so a steady training loop uploads nothing.
struct PtrSlot {
    void *dev = nullptr;          // device copy
    uint64_t *pinned = nullptr;   // pinned host staging of the same size
    size_t cap = 0;               // capacity in entries
    size_t n = 0;                 // entries in use
    hipEvent_t uploaded = nullptr;
    hipStream_t upload_stream = nullptr;
    hipStream_t use_stream = nullptr;   // stream of the last launch that read the table
    uint64_t last_seq = 0;              // plan-wide sequence number of that launch
    bool multi_stream = false;
    bool valid = false;
    bool in_graph = false;              // read by a launch recorded under stream capture: never reused
    uint64_t stamp = 0;
};

static void release_slot(PtrSlot &s)
{
    if (s.dev) (void)hipFree(s.dev);
    if (s.pinned) (void)hipHostFree(s.pinned);
    if (s.uploaded) (void)hipEventDestroy(s.uploaded);
    s = PtrSlot();
}

// Before a table is overwritten, the launches that read it must have finished.
// Recording an event after every launch would put a marker between all kernels;
// instead every KT_TICK_EVERY-th launch records a "tick" event carrying the
// launch sequence number, and a table may be overwritten once a tick that is
// not older than its last use has completed (streams run in order).
struct Tick {
    hipEvent_t ev = nullptr;
    hipStream_t stream = nullptr;
    uint64_t seq = 0;
    bool valid = false;
};

static const int KT_SLOTS = 8;
static const int KT_TICKS = 16;
static const uint64_t KT_TICK_EVERY = 4;
static const int KT_WSTAGE = 4;

struct kt_plan {
    KtHostPlan hp;
    std::mutex mu;
    int device = -1;
    void *dev_blob = nullptr;
    KtDeviceTables tb{};
    uint64_t serial = 0;   // identifies the plan for the lifetime of the process
    PtrSlot slots[KT_SLOTS];
    // Tables read by launches recorded into HIP graphs: moved out of the ring
    // (so that eager calls keep all KT_SLOTS tables) and kept until the plan
    // is destroyed, because a graph may be replayed at any time.
    std::vector<PtrSlot *> graph_tables;
    // device-resident weights (kt_plan_set_weights): one array of KT_MAX_PEERS floats on the
    // device, a small ring of pinned staging copies so that successive updates do not wait
    float *dev_w = nullptr;
    int dev_w_K = 0;
    // device-resident optimizer scalars (kt_plan_set_sgd): {scale, lr, momentum, weight decay},
    // uploaded through the same staging ring
    float *dev_sgd = nullptr;
    float *w_stage = nullptr;                 // KT_WSTAGE * KT_MAX_PEERS floats, pinned
    hipEvent_t w_done[4] = {nullptr, nullptr, nullptr, nullptr};
    int w_head = 0;
    Tick ticks[KT_TICKS];
    int tick_head = 0;
    uint64_t seq = 0;      // launches issued through this plan
    uint64_t clock = 0;
};

extern "C" kt_status kt_plan_create(const int64_t *numel, int T, kt_dtype dt, int64_t cap_bytes, int align_bytes,
                                    kt_plan **out)
{
    if (!out) { kt_set_error("kt_plan_create: NULL out"); return KT_EINVAL; }
    kt_plan *p = new (std::nothrow) kt_plan;
    if (!p) { kt_set_error("kt_plan_create: out of host memory"); return KT_ENOMEM; }
    const char *msg = "";
    kt_status st;
    try {
        st = kt_build_host_plan(numel, T, dt, cap_bytes, align_bytes, p->hp, &msg);
    } catch (const std::bad_alloc &) {
        st = KT_ENOMEM; msg = "out of host memory";
    }
    if (st != KT_OK) {
        kt_set_error("kt_plan_create: %s", msg);
        delete p;
        return st;
    }
    static std::atomic<uint64_t> next_serial{1};
    p->serial = next_serial.fetch_add(1);
    *out = p;
    return KT_OK;
}

const KtHostPlan &kt_plan_host(const kt_plan *p) { return p->hp; }
uint64_t kt_plan_serial(const kt_plan *p) { return p->serial; }

extern "C" kt_status kt_plan_destroy(kt_plan *p)
{
    if (!p) return KT_OK;
    kt_status st = KT_OK;
    if (p->device >= 0) {
        int cur = -1;
        (void)hipGetDevice(&cur);
        if (cur != p->device) (void)hipSetDevice(p->device);
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) st = hip_fail("kt_plan_destroy: hipDeviceSynchronize", e);
        for (PtrSlot &s : p->slots) release_slot(s);
        for (PtrSlot *g : p->graph_tables) { release_slot(*g); delete g; }
        for (Tick &t : p->ticks)
            if (t.ev) (void)hipEventDestroy(t.ev);
        if (p->dev_w) (void)hipFree(p->dev_w);
        if (p->dev_sgd) (void)hipFree(p->dev_sgd);
        if (p->w_stage) (void)hipHostFree(p->w_stage);
        for (hipEvent_t ev : p->w_done)
            if (ev) (void)hipEventDestroy(ev);
        if (p->dev_blob) (void)hipFree(p->dev_blob);
        if (cur != p->device && cur >= 0) (void)hipSetDevice(cur);
    }
    delete p;
    return st;
}

extern "C" int kt_plan_num_buckets(const kt_plan *p) { return p ? (int)p->hp.b_elems.size() : -1; }
extern "C" int kt_plan_num_tensors(const kt_plan *p) { return p ? (int)p->hp.t_numel.size() : -1; }

extern "C" kt_status kt_plan_bucket_info(const kt_plan *p, int b, int64_t *n_elems, int *first_tensor, int *n_tensors)
{
    if (!p || b < 0 || b >= (int)p->hp.b_elems.size()) { kt_set_error("kt_plan_bucket_info: bad plan or bucket"); return KT_EINVAL; }
    if (n_elems) *n_elems = p->hp.b_elems[b];
    if (first_tensor) *first_tensor = p->hp.b_first[b];
    if (n_tensors) *n_tensors = p->hp.b_count[b];
    return KT_OK;
}

extern "C" kt_status kt_plan_tensor_info(const kt_plan *p, int t, int *bucket, int64_t *elem_offset)
{
    if (!p || t < 0 || t >= (int)p->hp.t_numel.size()) { kt_set_error("kt_plan_tensor_info: bad plan or tensor"); return KT_EINVAL; }
    if (bucket) *bucket = p->hp.t_bucket[t];
    if (elem_offset) *elem_offset = p->hp.t_off[t];
    return KT_OK;
}

extern "C" int64_t kt_plan_num_tiles(const kt_plan *p) { return p ? (int64_t)p->hp.tiles.size() : -1; }

extern "C" kt_status kt_plan_tile_info(const kt_plan *p, int64_t i, int *bucket, int64_t *tile_in_bucket,
                                       int *first_tensor, int *n_tensors)
{
    if (!p || i < 0 || i >= (int64_t)p->hp.tiles.size()) { kt_set_error("kt_plan_tile_info: bad plan or tile"); return KT_EINVAL; }
    const KtTile &tl = p->hp.tiles[(size_t)i];
    if (bucket) *bucket = tl.bucket;
    if (tile_in_bucket) *tile_in_bucket = tl.tile_in_bucket;
    if (first_tensor) *first_tensor = tl.t0;
    if (n_tensors) *n_tensors = tl.nt;
    return KT_OK;
}

// Upload the plan tables on the first device call.  Caller holds p->mu.
static kt_status ensure_device(kt_plan *p, hipStream_t stream)
{
    if (p->device < 0 && capturing(stream)) {
        kt_set_error("the first device call on a plan uploads its tables and cannot be recorded into a graph; "
                     "make one call outside stream capture first");
        return KT_EUNSUPPORTED;
    }
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return hip_fail("hipGetDevice", e);
    if (p->device >= 0) {
        if (cur != p->device) { kt_set_error("plan is bound to device %d, current device is %d", p->device, cur); return KT_EINVAL; }
        return KT_OK;
    }
    const KtHostPlan &hp = p->hp;
    const size_t T = hp.t_numel.size(), nb = hp.b_elems.size(), nt = hp.tiles.size();
    auto pad = [](size_t x) { return (x + 255) / 256 * 256; };
    const size_t o_tiles = 0;
    const size_t o_off = o_tiles + pad(nt * sizeof(KtTile));
    const size_t o_numel = o_off + pad(T * 8);
    const size_t o_belems = o_numel + pad(T * 8);
    const size_t total = o_belems + pad(nb * 8) + 256;
    std::vector<char> host(total, 0);
    if (nt) memcpy(host.data() + o_tiles, hp.tiles.data(), nt * sizeof(KtTile));
    if (T) memcpy(host.data() + o_off, hp.t_off.data(), T * 8);
    if (T) memcpy(host.data() + o_numel, hp.t_numel.data(), T * 8);
    if (nb) memcpy(host.data() + o_belems, hp.b_elems.data(), nb * 8);
    void *blob = nullptr;
    e = hipMalloc(&blob, total);
    if (e != hipSuccess) return hip_fail("hipMalloc(plan tables)", e);
    e = hipMemcpy(blob, host.data(), total, hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(blob); return hip_fail("hipMemcpy(plan tables)", e); }
    char *d = static_cast<char *>(blob);
    p->dev_blob = blob;
    p->tb.tiles = reinterpret_cast<const KtTile *>(d + o_tiles);
    p->tb.t_off = reinterpret_cast<const int64_t *>(d + o_off);
    p->tb.t_numel = reinterpret_cast<const int64_t *>(d + o_numel);
    p->tb.b_elems = reinterpret_cast<const int64_t *>(d + o_belems);
    p->device = cur;
    return KT_OK;
}

// Wait until every launch that read table `v` has finished.  Caller holds p->mu.
static hipError_t wait_retired(kt_plan *p, const PtrSlot *v)
{
    hipError_t e;
    if (v->last_seq == 0) {
        e = hipEventSynchronize(v->uploaded);
    } else if (v->multi_stream) {
        return hipDeviceSynchronize();
    } else {
        const Tick *best = nullptr;
        for (const Tick &t : p->ticks)
            if (t.valid && t.stream == v->use_stream && t.seq >= v->last_seq && (!best || t.seq < best->seq))
                best = &t;
        e = best ? hipEventSynchronize(best->ev) : hipStreamSynchronize(v->use_stream);
    }
    if (e != hipSuccess) {
        // e.g. the caller destroyed the stream of that launch: the targeted wait is
        // impossible, waiting for the whole device is always sufficient
        (void)hipGetLastError();
        e = hipDeviceSynchronize();
    }
    return e;
}

// Make `vals[0..n)` resident on the device for a launch on `stream`.
// Caller holds p->mu.  On success *slot_out is the slot to mark after launch.
static kt_status stage_pointers(kt_plan *p, const uint64_t *vals, size_t n, hipStream_t stream, PtrSlot **slot_out)
{
    hipError_t e;
    const bool cap = capturing(stream);
    for (PtrSlot *g : p->graph_tables) {
        if (g->n == n && memcmp(g->pinned, vals, n * 8) == 0) {
            // its upload was waited for when it was moved here
            *slot_out = g;
            return KT_OK;
        }
    }
    PtrSlot *hit = nullptr, *victim = nullptr;
    for (PtrSlot &s : p->slots) {
        if (s.valid && s.n == n && memcmp(s.pinned, vals, n * 8) == 0) { hit = &s; break; }
    }
    if (hit) {
        if (cap) {
            // A graph keeps using this table for as long as it is replayed: take
            // it out of the ring, whose slot becomes free for eager calls again.
            e = hipEventSynchronize(hit->uploaded);
            if (e != hipSuccess) return hip_fail("hipEventSynchronize", e);
            PtrSlot *g = new PtrSlot(*hit);
            g->in_graph = true;
            p->graph_tables.push_back(g);
            *hit = PtrSlot();
            *slot_out = g;
            return KT_OK;
        }
        if (hit->upload_stream != stream) {
            e = hipStreamWaitEvent(stream, hit->uploaded, 0);
            if (e != hipSuccess) return hip_fail("hipStreamWaitEvent", e);
        }
        hit->stamp = ++p->clock;
        *slot_out = hit;
        return KT_OK;
    }
    if (cap) {
        kt_set_error("these pointers have no resident table yet and an upload cannot be recorded into a graph; "
                     "make the same call once outside stream capture first");
        return KT_EUNSUPPORTED;
    }
    for (PtrSlot &s : p->slots) {
        if (!s.valid) { victim = &s; break; }
        if (!victim || s.stamp < victim->stamp) victim = &s;
    }
    if (victim->valid) {
        // the upload and the launches that read this table must have finished
        e = wait_retired(p, victim);
        if (e != hipSuccess) return hip_fail("waiting for a pointer table to retire", e);
    }
    victim->valid = false;
    if (victim->cap < n) {
        if (victim->dev) (void)hipFree(victim->dev);
        if (victim->pinned) (void)hipHostFree(victim->pinned);
        victim->dev = nullptr; victim->pinned = nullptr; victim->cap = 0;
        const size_t entries = n < 64 ? 64 : n;
        e = hipMalloc(&victim->dev, entries * 8);
        if (e != hipSuccess) return hip_fail("hipMalloc(pointer table)", e);
        e = hipHostMalloc(reinterpret_cast<void **>(&victim->pinned), entries * 8, hipHostMallocDefault);
        if (e != hipSuccess) { (void)hipFree(victim->dev); victim->dev = nullptr; return hip_fail("hipHostMalloc(pointer table)", e); }
        victim->cap = entries;
    }
    if (!victim->uploaded) {
        e = hipEventCreateWithFlags(&victim->uploaded, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail("hipEventCreate", e);
    }
    memcpy(victim->pinned, vals, n * 8);
    e = hipMemcpyAsync(victim->dev, victim->pinned, n * 8, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return hip_fail("hipMemcpyAsync(pointer table)", e);
    e = hipEventRecord(victim->uploaded, stream);
    if (e != hipSuccess) return hip_fail("hipEventRecord", e);
    victim->n = n;
    victim->upload_stream = stream;
    victim->use_stream = stream;
    victim->last_seq = 0;
    victim->multi_stream = false;
    victim->valid = true;
    victim->stamp = ++p->clock;
    *slot_out = victim;
    return KT_OK;
}

// Bookkeeping after a launch that read `s` on `stream`.  Caller holds p->mu.
static kt_status mark_used(kt_plan *p, PtrSlot *s, hipStream_t stream)
{
    if (s->in_graph) return KT_OK;   // the table stays resident until the plan is destroyed
    if (s->last_seq > 0 && s->use_stream != stream) s->multi_stream = true;
    s->use_stream = stream;
    s->last_seq = ++p->seq;
    if (p->seq % KT_TICK_EVERY == 0) {
        Tick &t = p->ticks[p->tick_head];
        p->tick_head = (p->tick_head + 1) % KT_TICKS;
        if (!t.ev) {
            hipError_t e = hipEventCreateWithFlags(&t.ev, hipEventDisableTiming);
            if (e != hipSuccess) return hip_fail("hipEventCreate", e);
        }
        t.valid = false;
        hipError_t e = hipEventRecord(t.ev, stream);
        if (e != hipSuccess) return hip_fail("hipEventRecord", e);
        t.stream = stream;
        t.seq = p->seq;
        t.valid = true;
    }
    return KT_OK;
}

// Per-thread scratch for the pointer table of the current call: no heap
// allocation once it has grown to the size a caller needs.
static std::vector<uint64_t> &call_table(size_t n)
{
    static thread_local std::vector<uint64_t> tbl;
    tbl.resize(n);
    return tbl;
}

// Resolve the bucket selector into a bucket range and a tile range.
static kt_status select(const kt_plan *p, int bucket, const char *who, int *b0, int *b1, int64_t *tile0, int64_t *ntiles)
{
    const int nb = (int)p->hp.b_elems.size();
    if (bucket == KT_ALL_BUCKETS) { *b0 = 0; *b1 = nb; }
    else if (bucket >= 0 && bucket < nb) { *b0 = bucket; *b1 = bucket + 1; }
    else { kt_set_error("%s: bucket %d outside [0,%d)", who, bucket, nb); return KT_EINVAL; }
    *tile0 = p->hp.b_tile0[*b0];
    *ntiles = p->hp.b_tile0[*b1] - *tile0;
    return KT_OK;
}

// The weights of a launch: the caller's K values by value, or (weights == NULL) the plan's
// device-resident ones.  Host-only check.
static kt_status resolve_weights(const kt_plan *p, const float *weights, int K, const char *who, KtWeights *w)
{
    memset(w, 0, sizeof *w);
    if (weights) {
        for (int k = 0; k < K; ++k) w->w[k] = weights[k];
        return KT_OK;
    }
    if (!p->dev_w) { kt_set_error("%s: NULL weights and no weights set with kt_plan_set_weights", who); return KT_EINVAL; }
    if (p->dev_w_K != K) { kt_set_error("%s: K=%d but the plan's resident weights are for K=%d", who, K, p->dev_w_K); return KT_EINVAL; }
    w->dev = p->dev_w;
    return KT_OK;
}

// Shared by pack and unpack: validate, build [tensor ptrs | bucket ptrs], stage.
static kt_status prepare_tensor_call(kt_plan *p, int bucket, const void *const *tensor_ptrs,
                                     const void *const *bucket_bufs, const char *who, hipStream_t stream,
                                     int64_t *tile0, int64_t *ntiles, bool *vector_ok, PtrSlot **slot)
{
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    int b0, b1;
    kt_status st = select(p, bucket, who, &b0, &b1, tile0, ntiles);
    if (st != KT_OK) return st;
    const KtHostPlan &hp = p->hp;
    const size_t T = hp.t_numel.size(), nb = hp.b_elems.size();
    if (*ntiles == 0) return KT_OK;
    if (!tensor_ptrs || !bucket_bufs) { kt_set_error("%s: NULL pointer array", who); return KT_EINVAL; }
    const uintptr_t emask = (uintptr_t)hp.elem_size - 1;
    // The whole arrays go into the table (so that per-bucket calls made with
    // the same arrays share one resident table); only the selected buckets'
    // entries are validated and dereferenced.
    std::vector<uint64_t> &vals = call_table(T + nb);
    for (size_t t = 0; t < T; ++t) vals[t] = reinterpret_cast<uintptr_t>(tensor_ptrs[t]);
    for (size_t b = 0; b < nb; ++b) vals[T + b] = reinterpret_cast<uintptr_t>(bucket_bufs[b]);
    bool vec = hp.align_bytes % KT_VEC_BYTES == 0;
    for (int b = b0; b < b1; ++b) {
        const uintptr_t bp = reinterpret_cast<uintptr_t>(bucket_bufs[b]);
        if (hp.b_elems[b] > 0 && !bp) { kt_set_error("%s: NULL buffer for bucket %d", who, b); return KT_EINVAL; }
        if (bp & emask) { kt_set_error("%s: bucket %d buffer not aligned to the element size", who, b); return KT_EALIGN; }
        if (bp & (KT_VEC_BYTES - 1)) vec = false;
        for (int t = hp.b_first[b]; t < hp.b_first[b] + hp.b_count[b]; ++t) {
            const uintptr_t tp = reinterpret_cast<uintptr_t>(tensor_ptrs[t]);
            if (hp.t_numel[t] > 0 && !tp) { kt_set_error("%s: NULL pointer for tensor %d", who, t); return KT_EINVAL; }
            if (tp & emask) { kt_set_error("%s: tensor %d not aligned to the element size", who, t); return KT_EALIGN; }
            // a tensor and its bucket must not overlap
            const uintptr_t tn = (uintptr_t)hp.t_numel[t] * hp.elem_size, bn = (uintptr_t)hp.b_elems[b] * hp.elem_size;
            if (tn && tp < bp + bn && bp < tp + tn) { kt_set_error("%s: tensor %d overlaps bucket %d", who, t, b); return KT_EINVAL; }
        }
    }
    *vector_ok = vec;
    st = ensure_device(p, stream);
    if (st != KT_OK) return st;
    return stage_pointers(p, vals.data(), vals.size(), stream, slot);
}

extern "C" kt_status kt_bucket_pack(kt_plan *p, int bucket, const void *const *tensor_ptrs, void *const *bucket_bufs,
                                    void *stream)
{
    KT_GUARD_BEGIN
    if (!p) { kt_set_error("kt_bucket_pack: NULL plan"); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t tile0 = 0, ntiles = 0;
    bool vec = false;
    PtrSlot *slot = nullptr;
    kt_status st = prepare_tensor_call(p, bucket, tensor_ptrs, bucket_bufs, "kt_bucket_pack", s, &tile0, &ntiles, &vec, &slot);
    if (st != KT_OK || ntiles == 0) return st;
    const size_t T = p->hp.t_numel.size();
    const void *const *d_t = static_cast<const void *const *>(slot->dev);
    void *const *d_b = reinterpret_cast<void *const *>(static_cast<uint64_t *>(slot->dev) + T);
    int e = kt_launch_pack(p->tb, p->hp.dt, tile0, ntiles, d_t, d_b, vec, stream);
    if (e != 0) return hip_fail("kt_bucket_pack: launch", (hipError_t)e);
    return mark_used(p, slot, s);
    KT_GUARD_END("kt_bucket_pack")
}

extern "C" kt_status kt_bucket_unpack_scale(kt_plan *p, int bucket, const void *const *bucket_bufs, float scale,
                                            void *const *tensor_ptrs, void *stream)
{
    KT_GUARD_BEGIN
    if (!p) { kt_set_error("kt_bucket_unpack_scale: NULL plan"); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t tile0 = 0, ntiles = 0;
    bool vec = false;
    PtrSlot *slot = nullptr;
    kt_status st = prepare_tensor_call(p, bucket, tensor_ptrs, bucket_bufs, "kt_bucket_unpack_scale", s, &tile0, &ntiles, &vec, &slot);
    if (st != KT_OK || ntiles == 0) return st;
    const size_t T = p->hp.t_numel.size();
    void *const *d_t = static_cast<void *const *>(slot->dev);
    const void *const *d_b = reinterpret_cast<const void *const *>(static_cast<uint64_t *>(slot->dev) + T);
    int e = kt_launch_unpack(p->tb, p->hp.dt, tile0, ntiles, d_b, scale, d_t, vec, stream);
    if (e != 0) return hip_fail("kt_bucket_unpack_scale: launch", (hipError_t)e);
    return mark_used(p, slot, s);
    KT_GUARD_END("kt_bucket_unpack_scale")
}

extern "C" kt_status kt_weighted_reduce(kt_plan *p, int bucket, const void *const *peer_bufs, int K,
                                        const float *weights, void *const *out_bufs, void *stream)
{
    KT_GUARD_BEGIN
    const char *who = "kt_weighted_reduce";
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    if (K < 1 || K > KT_MAX_PEERS) { kt_set_error("%s: K=%d outside [1,%d]", who, K, KT_MAX_PEERS); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    KtWeights w;
    kt_status st = resolve_weights(p, weights, K, who, &w);
    if (st != KT_OK) return st;
    int b0, b1;
    int64_t tile0, ntiles;
    st = select(p, bucket, who, &b0, &b1, &tile0, &ntiles);
    if (st != KT_OK || ntiles == 0) return st;
    if (!peer_bufs || !out_bufs) { kt_set_error("%s: NULL pointer array", who); return KT_EINVAL; }
    const KtHostPlan &hp = p->hp;
    const size_t nb = hp.b_elems.size();
    const uintptr_t emask = (uintptr_t)hp.elem_size - 1;
    std::vector<uint64_t> &vals = call_table(nb * K + nb);
    for (size_t i = 0; i < nb * K; ++i) vals[i] = reinterpret_cast<uintptr_t>(peer_bufs[i]);
    for (size_t b = 0; b < nb; ++b) vals[nb * K + b] = reinterpret_cast<uintptr_t>(out_bufs[b]);
    bool vec = true;
    for (int b = b0; b < b1; ++b) {
        const uintptr_t bytes = (uintptr_t)hp.b_elems[b] * hp.elem_size;
        const uintptr_t op = reinterpret_cast<uintptr_t>(out_bufs[b]);
        if (bytes && !op) { kt_set_error("%s: NULL output for bucket %d", who, b); return KT_EINVAL; }
        if (op & emask) { kt_set_error("%s: output %d not aligned to the element size", who, b); return KT_EALIGN; }
        if (op & (KT_VEC_BYTES - 1)) vec = false;
        for (int k = 0; k < K; ++k) {
            const uintptr_t pp = reinterpret_cast<uintptr_t>(peer_bufs[(size_t)b * K + k]);
            if (bytes && !pp) { kt_set_error("%s: NULL peer %d of bucket %d", who, k, b); return KT_EINVAL; }
            if (pp & emask) { kt_set_error("%s: peer %d of bucket %d not aligned to the element size", who, k, b); return KT_EALIGN; }
            if (pp & (KT_VEC_BYTES - 1)) vec = false;
            // the output may be exactly one of the inputs (in place), never a partial overlap
            if (bytes && pp != op && pp < op + bytes && op < pp + bytes) {
                kt_set_error("%s: output of bucket %d partially overlaps peer %d", who, b, k);
                return KT_EINVAL;
            }
        }
    }
    st = ensure_device(p, s);
    if (st != KT_OK) return st;
    PtrSlot *slot = nullptr;
    st = stage_pointers(p, vals.data(), vals.size(), s, &slot);
    if (st != KT_OK) return st;
    const void *const *d_p = static_cast<const void *const *>(slot->dev);
    void *const *d_o = reinterpret_cast<void *const *>(static_cast<uint64_t *>(slot->dev) + nb * K);
    int e = kt_launch_reduce(p->tb, hp.dt, tile0, ntiles, d_p, K, w, d_o, vec, stream);
    if (e != 0) return hip_fail("kt_weighted_reduce: launch", (hipError_t)e);
    return mark_used(p, slot, s);
    KT_GUARD_END("kt_weighted_reduce")
}

// Copies n (<= KT_MAX_PEERS) floats into a small device array of the plan (allocated on first
// use, KT_MAX_PEERS floats, the rest zero) in stream order, through a ring of pinned staging
// copies so that successive updates do not wait for each other.  Not under stream capture.
static kt_status push_resident(kt_plan *p, float **dev, const float *src, int n, hipStream_t s)
{
    kt_status st = ensure_device(p, s);
    if (st != KT_OK) return st;
    hipError_t e;
    if (!p->w_stage) {
        void *h = nullptr;
        e = hipHostMalloc(&h, KT_WSTAGE * KT_MAX_PEERS * sizeof(float), hipHostMallocDefault);
        if (e != hipSuccess) return hip_fail("hipHostMalloc(resident scalars)", e);
        p->w_stage = static_cast<float *>(h);
    }
    if (!*dev) {
        void *d = nullptr;
        e = hipMalloc(&d, KT_MAX_PEERS * sizeof(float));
        if (e != hipSuccess) return hip_fail("hipMalloc(resident scalars)", e);
        *dev = static_cast<float *>(d);
    }
    const int i = p->w_head;
    p->w_head = (i + 1) % KT_WSTAGE;
    if (!p->w_done[i]) {
        e = hipEventCreateWithFlags(&p->w_done[i], hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail("hipEventCreate", e);
    } else {
        e = hipEventSynchronize(p->w_done[i]);        // the upload that last used this staging copy
        if (e != hipSuccess) return hip_fail("hipEventSynchronize", e);
    }
    float *stage = p->w_stage + (size_t)i * KT_MAX_PEERS;
    memset(stage, 0, KT_MAX_PEERS * sizeof(float));
    memcpy(stage, src, (size_t)n * sizeof(float));
    e = hipMemcpyAsync(*dev, stage, KT_MAX_PEERS * sizeof(float), hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return hip_fail("hipMemcpyAsync(resident scalars)", e);
    e = hipEventRecord(p->w_done[i], s);
    if (e != hipSuccess) return hip_fail("hipEventRecord", e);
    return KT_OK;
}

extern "C" kt_status kt_plan_set_weights(kt_plan *p, const float *weights, int K, void *stream)
{
    KT_GUARD_BEGIN
    const char *who = "kt_plan_set_weights";
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    if (!weights) { kt_set_error("%s: NULL weights", who); return KT_EINVAL; }
    if (K < 1 || K > KT_MAX_PEERS) { kt_set_error("%s: K=%d outside [1,%d]", who, K, KT_MAX_PEERS); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (capturing(s)) {
        kt_set_error("%s: the upload cannot be recorded into a graph; call it outside stream capture, on the stream "
                     "that replays the graph", who);
        return KT_EUNSUPPORTED;
    }
    kt_status st = push_resident(p, &p->dev_w, weights, K, s);
    if (st != KT_OK) return st;
    p->dev_w_K = K;
    return KT_OK;
    KT_GUARD_END("kt_plan_set_weights")
}

extern "C" kt_status kt_plan_set_sgd(kt_plan *p, float scale, float lr, float momentum, float weight_decay,
                                     void *stream)
{
    KT_GUARD_BEGIN
    const char *who = "kt_plan_set_sgd";
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (capturing(s)) {
        kt_set_error("%s: the upload cannot be recorded into a graph; call it outside stream capture, on the stream "
                     "that replays the graph", who);
        return KT_EUNSUPPORTED;
    }
    const float v[4] = {scale, lr, momentum, weight_decay};
    return push_resident(p, &p->dev_sgd, v, 4, s);
    KT_GUARD_END("kt_plan_set_sgd")
}

kt_status kt_fused_prepare(const kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                           const void *const *peer_bufs, int K, const float *weights,
                           void *const *out_tensor_ptrs, const char *who, std::vector<uint64_t> &vals,
                           KtWeights *w, int64_t *tile0, int64_t *ntiles, bool *vector_ok)
{
    *ntiles = 0;
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    if (K < 1 || K > KT_MAX_PEERS) { kt_set_error("%s: K=%d outside [1,%d]", who, K, KT_MAX_PEERS); return KT_EINVAL; }
    kt_status st = resolve_weights(p, weights, K, who, w);
    if (st != KT_OK) return st;
    int b0, b1;
    st = select(p, bucket, who, &b0, &b1, tile0, ntiles);
    if (st != KT_OK || *ntiles == 0) return st;
    if (!local_tensor_ptrs || !out_tensor_ptrs || (K > 1 && !peer_bufs)) { kt_set_error("%s: NULL pointer array", who); return KT_EINVAL; }
    const KtHostPlan &hp = p->hp;
    const size_t T = hp.t_numel.size(), nb = hp.b_elems.size(), KP = (size_t)(K - 1);
    const uintptr_t emask = (uintptr_t)hp.elem_size - 1;
    // table layout: [local tensors T | output tensors T | peers nb*(K-1)]
    vals.resize(2 * T + nb * KP);
    for (size_t t = 0; t < T; ++t) {
        vals[t] = reinterpret_cast<uintptr_t>(local_tensor_ptrs[t]);
        vals[T + t] = reinterpret_cast<uintptr_t>(out_tensor_ptrs[t]);
    }
    for (size_t i = 0; i < nb * KP; ++i) vals[2 * T + i] = reinterpret_cast<uintptr_t>(peer_bufs[i]);
    bool vec = hp.align_bytes % KT_VEC_BYTES == 0;
    for (int b = b0; b < b1; ++b) {
        const uintptr_t bbytes = (uintptr_t)hp.b_elems[b] * hp.elem_size;
        for (size_t k = 0; k < KP; ++k) {
            const uintptr_t pp = vals[2 * T + (size_t)b * KP + k];
            if (bbytes && !pp) { kt_set_error("%s: NULL peer %zu of bucket %d", who, k + 1, b); return KT_EINVAL; }
            if (pp & emask) { kt_set_error("%s: peer %zu of bucket %d not aligned to the element size", who, k + 1, b); return KT_EALIGN; }
            if (pp & (KT_VEC_BYTES - 1)) vec = false;
        }
        for (int t = hp.b_first[b]; t < hp.b_first[b] + hp.b_count[b]; ++t) {
            const uintptr_t lp = vals[t], op = vals[T + t];
            const uintptr_t tn = (uintptr_t)hp.t_numel[t] * hp.elem_size;
            if (tn && (!lp || !op)) { kt_set_error("%s: NULL pointer for tensor %d", who, t); return KT_EINVAL; }
            if ((lp | op) & emask) { kt_set_error("%s: tensor %d not aligned to the element size", who, t); return KT_EALIGN; }
            // the output may be the local gradient itself (in place), never a partial overlap
            if (tn && lp != op && lp < op + tn && op < lp + tn) { kt_set_error("%s: output %d partially overlaps its input", who, t); return KT_EINVAL; }
            for (size_t k = 0; k < KP; ++k) {
                const uintptr_t pp = vals[2 * T + (size_t)b * KP + k];
                if (tn && op < pp + bbytes && pp < op + tn) { kt_set_error("%s: output %d overlaps peer %zu of bucket %d", who, t, k + 1, b); return KT_EINVAL; }
            }
        }
    }
    *vector_ok = vec;
    return KT_OK;
}

extern "C" kt_status kt_fused_step(kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                                   const void *const *peer_bufs, int K, const float *weights, float scale,
                                   void *const *out_tensor_ptrs, void *stream)
{
    KT_GUARD_BEGIN
    const char *who = "kt_fused_step";
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t tile0 = 0, ntiles = 0;
    bool vec = false;
    KtWeights w;
    std::vector<uint64_t> &vals = call_table(0);
    kt_status st = kt_fused_prepare(p, bucket, local_tensor_ptrs, peer_bufs, K, weights, out_tensor_ptrs, who, vals, &w,
                                    &tile0, &ntiles, &vec);
    if (st != KT_OK || ntiles == 0) return st;
    const size_t T = p->hp.t_numel.size();
    st = ensure_device(p, s);
    if (st != KT_OK) return st;
    PtrSlot *slot = nullptr;
    st = stage_pointers(p, vals.data(), vals.size(), s, &slot);
    if (st != KT_OK) return st;
    const uint64_t *d = static_cast<const uint64_t *>(slot->dev);
    int e = kt_launch_fused(p->tb, p->hp.dt, tile0, ntiles, reinterpret_cast<const void *const *>(d),
                            reinterpret_cast<const void *const *>(d + 2 * T), K, w, scale,
                            reinterpret_cast<void *const *>(const_cast<uint64_t *>(d + T)), vec, stream);
    if (e != 0) return hip_fail("kt_fused_step: launch", (hipError_t)e);
    return mark_used(p, slot, s);
    KT_GUARD_END("kt_fused_step")
}

// kt_bucket_unpack_sgd and its mixed-precision form (model_ptrs != NULL).
static kt_status unpack_sgd_impl(kt_plan *p, int bucket, const void *const *bucket_bufs, float scale,
                                 void *const *param_ptrs, void *const *momentum_ptrs, void *const *model_ptrs,
                                 bool master, float lr, float momentum, float weight_decay, int first_step,
                                 void *stream, const char *who, bool resident = false)
{
    KT_GUARD_BEGIN
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int b0, b1;
    int64_t tile0, ntiles;
    kt_status st = select(p, bucket, who, &b0, &b1, &tile0, &ntiles);
    if (st != KT_OK || ntiles == 0) return st;
    if (!bucket_bufs || !param_ptrs || !momentum_ptrs || (master && !model_ptrs)) { kt_set_error("%s: NULL pointer array", who); return KT_EINVAL; }
    if (resident && !p->dev_sgd) { kt_set_error("%s: no optimizer scalars set with kt_plan_set_sgd", who); return KT_EINVAL; }
    if (first_step && capturing(s)) {
        kt_set_error("%s: first_step is frozen into a recorded kernel and would reset the momentum on every replay; "
                     "make the first step outside stream capture", who);
        return KT_EUNSUPPORTED;
    }
    const KtHostPlan &hp = p->hp;
    const size_t T = hp.t_numel.size(), nb = hp.b_elems.size();
    const size_t M = master ? T : 0;
    // table layout: [parameters T | momentum T | model parameters T (mixed precision only) | buckets nb]
    std::vector<uint64_t> &vals = call_table(2 * T + M + nb);
    for (size_t t = 0; t < T; ++t) {
        vals[t] = reinterpret_cast<uintptr_t>(param_ptrs[t]);
        vals[T + t] = reinterpret_cast<uintptr_t>(momentum_ptrs[t]);
        if (master) vals[2 * T + t] = reinterpret_cast<uintptr_t>(model_ptrs[t]);
    }
    for (size_t b = 0; b < nb; ++b) vals[2 * T + M + b] = reinterpret_cast<uintptr_t>(bucket_bufs[b]);
    bool vec = hp.align_bytes % KT_VEC_BYTES == 0;
    for (int b = b0; b < b1; ++b) {
        const uintptr_t bp = vals[2 * T + M + b], bn = (uintptr_t)hp.b_elems[b] * hp.elem_size;
        if (bn && !bp) { kt_set_error("%s: NULL buffer for bucket %d", who, b); return KT_EINVAL; }
        if (bp & ((uintptr_t)hp.elem_size - 1)) { kt_set_error("%s: bucket %d buffer not aligned to the element size", who, b); return KT_EALIGN; }
        if (bp & (KT_VEC_BYTES - 1)) vec = false;
        for (int t = hp.b_first[b]; t < hp.b_first[b] + hp.b_count[b]; ++t) {
            const uintptr_t pp = vals[t], vp = vals[T + t], tn = (uintptr_t)hp.t_numel[t] * 4;
            if (tn && (!pp || !vp)) { kt_set_error("%s: NULL parameter or momentum pointer for tensor %d", who, t); return KT_EINVAL; }
            if ((pp | vp) & 3u) { kt_set_error("%s: tensor %d parameters/momentum not 4-byte aligned", who, t); return KT_EALIGN; }
            if (tn && ((pp < vp + tn && vp < pp + tn) || (pp < bp + bn && bp < pp + tn) || (vp < bp + bn && bp < vp + tn))) {
                kt_set_error("%s: parameters, momentum and bucket of tensor %d overlap", who, t);
                return KT_EINVAL;
            }
            if (master) {
                const uintptr_t mp = vals[2 * T + t], mn = (uintptr_t)hp.t_numel[t] * 2;
                if (mn && !mp) { kt_set_error("%s: NULL model-parameter pointer for tensor %d", who, t); return KT_EINVAL; }
                if (mp & 1u) { kt_set_error("%s: tensor %d model parameters not 2-byte aligned", who, t); return KT_EALIGN; }
                if (mn && ((mp < pp + tn && pp < mp + mn) || (mp < vp + tn && vp < mp + mn) || (mp < bp + bn && bp < mp + mn))) {
                    kt_set_error("%s: model parameters of tensor %d overlap its parameters, momentum or bucket", who, t);
                    return KT_EINVAL;
                }
            }
        }
    }
    st = ensure_device(p, s);
    if (st != KT_OK) return st;
    PtrSlot *slot = nullptr;
    st = stage_pointers(p, vals.data(), vals.size(), s, &slot);
    if (st != KT_OK) return st;
    uint64_t *d = static_cast<uint64_t *>(slot->dev);
    KtSgd a{scale, lr, momentum, weight_decay, first_step ? 1 : 0, resident ? p->dev_sgd : nullptr};
    int e = kt_launch_unpack_sgd(p->tb, hp.dt, tile0, ntiles, reinterpret_cast<const void *const *>(d + 2 * T + M),
                                 reinterpret_cast<void *const *>(d), reinterpret_cast<void *const *>(d + T),
                                 master ? reinterpret_cast<void *const *>(d + 2 * T) : nullptr, a, vec, stream);
    if (e != 0) { kt_set_error("%s: launch: %s", who, hipGetErrorString((hipError_t)e)); return KT_EHIP; }
    return mark_used(p, slot, s);
    KT_GUARD_END(who)
}

extern "C" kt_status kt_bucket_unpack_sgd(kt_plan *p, int bucket, const void *const *bucket_bufs, float scale,
                                          void *const *param_ptrs, void *const *momentum_ptrs, float lr,
                                          float momentum, float weight_decay, int first_step, void *stream)
{
    return unpack_sgd_impl(p, bucket, bucket_bufs, scale, param_ptrs, momentum_ptrs, nullptr, false, lr, momentum,
                           weight_decay, first_step, stream, "kt_bucket_unpack_sgd");
}

extern "C" kt_status kt_bucket_unpack_sgd_master(kt_plan *p, int bucket, const void *const *bucket_bufs, float scale,
                                                 void *const *master_ptrs, void *const *momentum_ptrs,
                                                 void *const *model_ptrs, float lr, float momentum,
                                                 float weight_decay, int first_step, void *stream)
{
    return unpack_sgd_impl(p, bucket, bucket_bufs, scale, master_ptrs, momentum_ptrs, model_ptrs, true, lr, momentum,
                           weight_decay, first_step, stream, "kt_bucket_unpack_sgd_master");
}

extern "C" kt_status kt_bucket_unpack_sgd_resident(kt_plan *p, int bucket, const void *const *bucket_bufs,
                                                   void *const *param_ptrs, void *const *momentum_ptrs,
                                                   void *const *model_ptrs, int first_step, void *stream)
{
    return unpack_sgd_impl(p, bucket, bucket_bufs, 0.0f, param_ptrs, momentum_ptrs, model_ptrs, model_ptrs != nullptr,
                           0.0f, 0.0f, 0.0f, first_step, stream, "kt_bucket_unpack_sgd_resident", true);
}

// kt_fused_step_sgd and its form with device-resident weights and optimizer scalars.
static kt_status fused_sgd_impl(kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                                const void *const *peer_bufs, int K, const float *weights, float scale,
                                void *const *param_ptrs, void *const *momentum_ptrs, void *const *model_ptrs,
                                float lr, float momentum, float weight_decay, int first_step, void *stream,
                                const char *who, bool resident)
{
    KT_GUARD_BEGIN
    if (!p) { kt_set_error("%s: NULL plan", who); return KT_EINVAL; }
    std::lock_guard<std::mutex> lock(p->mu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (K < 1 || K > KT_MAX_PEERS) { kt_set_error("%s: K=%d outside [1,%d]", who, K, KT_MAX_PEERS); return KT_EINVAL; }
    KtWeights w;
    kt_status st = resolve_weights(p, weights, K, who, &w);
    if (st != KT_OK) return st;
    int b0, b1;
    int64_t tile0, ntiles;
    st = select(p, bucket, who, &b0, &b1, &tile0, &ntiles);
    if (st != KT_OK || ntiles == 0) return st;
    if (!local_tensor_ptrs || !param_ptrs || !momentum_ptrs || (K > 1 && !peer_bufs)) { kt_set_error("%s: NULL pointer array", who); return KT_EINVAL; }
    if (resident && !p->dev_sgd) { kt_set_error("%s: no optimizer scalars set with kt_plan_set_sgd", who); return KT_EINVAL; }
    if (first_step && capturing(s)) {
        kt_set_error("%s: first_step is frozen into a recorded kernel and would reset the momentum on every replay; "
                     "make the first step outside stream capture", who);
        return KT_EUNSUPPORTED;
    }
    const KtHostPlan &hp = p->hp;
    const bool master = model_ptrs != nullptr;
    const size_t T = hp.t_numel.size(), nb = hp.b_elems.size(), KP = (size_t)(K - 1), M = master ? T : 0;
    const uintptr_t emask = (uintptr_t)hp.elem_size - 1;
    // table layout: [local gradients T | parameters T | momentum T | model parameters T (optional) | peers nb*(K-1)]
    std::vector<uint64_t> &vals = call_table(3 * T + M + nb * KP);
    for (size_t t = 0; t < T; ++t) {
        vals[t] = reinterpret_cast<uintptr_t>(local_tensor_ptrs[t]);
        vals[T + t] = reinterpret_cast<uintptr_t>(param_ptrs[t]);
        vals[2 * T + t] = reinterpret_cast<uintptr_t>(momentum_ptrs[t]);
        if (master) vals[3 * T + t] = reinterpret_cast<uintptr_t>(model_ptrs[t]);
    }
    const size_t P0 = 3 * T + M;
    for (size_t i = 0; i < nb * KP; ++i) vals[P0 + i] = reinterpret_cast<uintptr_t>(peer_bufs[i]);
    auto overlap = [](uintptr_t a, uintptr_t an, uintptr_t b, uintptr_t bn) { return an && bn && a < b + bn && b < a + an; };
    bool vec = hp.align_bytes % KT_VEC_BYTES == 0;
    for (int b = b0; b < b1; ++b) {
        const uintptr_t bbytes = (uintptr_t)hp.b_elems[b] * hp.elem_size;
        for (size_t k = 0; k < KP; ++k) {
            const uintptr_t pp = vals[P0 + (size_t)b * KP + k];
            if (bbytes && !pp) { kt_set_error("%s: NULL peer %zu of bucket %d", who, k + 1, b); return KT_EINVAL; }
            if (pp & emask) { kt_set_error("%s: peer %zu of bucket %d not aligned to the element size", who, k + 1, b); return KT_EALIGN; }
            if (pp & (KT_VEC_BYTES - 1)) vec = false;
        }
        for (int t = hp.b_first[b]; t < hp.b_first[b] + hp.b_count[b]; ++t) {
            const uintptr_t lp = vals[t], pa = vals[T + t], va = vals[2 * T + t], ma = master ? vals[3 * T + t] : 0;
            const uintptr_t ln = (uintptr_t)hp.t_numel[t] * hp.elem_size, fn = (uintptr_t)hp.t_numel[t] * 4,
                            mn = master ? (uintptr_t)hp.t_numel[t] * 2 : 0;
            if (ln && (!lp || !pa || !va || (master && !ma))) { kt_set_error("%s: NULL pointer for tensor %d", who, t); return KT_EINVAL; }
            if (lp & emask) { kt_set_error("%s: tensor %d gradient not aligned to the element size", who, t); return KT_EALIGN; }
            if ((pa | va) & 3u) { kt_set_error("%s: tensor %d parameters/momentum not 4-byte aligned", who, t); return KT_EALIGN; }
            if (ma & 1u) { kt_set_error("%s: tensor %d model parameters not 2-byte aligned", who, t); return KT_EALIGN; }
            if (overlap(pa, fn, va, fn) || overlap(pa, fn, lp, ln) || overlap(va, fn, lp, ln) || overlap(ma, mn, lp, ln) ||
                overlap(ma, mn, pa, fn) || overlap(ma, mn, va, fn)) {
                kt_set_error("%s: gradient, parameters, momentum and model parameters of tensor %d overlap", who, t);
                return KT_EINVAL;
            }
            for (size_t k = 0; k < KP; ++k) {
                const uintptr_t pp = vals[P0 + (size_t)b * KP + k];
                if (overlap(pa, fn, pp, bbytes) || overlap(va, fn, pp, bbytes) || overlap(ma, mn, pp, bbytes)) {
                    kt_set_error("%s: parameters, momentum or model parameters of tensor %d overlap peer %zu of bucket %d", who, t, k + 1, b);
                    return KT_EINVAL;
                }
            }
        }
    }
    st = ensure_device(p, s);
    if (st != KT_OK) return st;
    PtrSlot *slot = nullptr;
    st = stage_pointers(p, vals.data(), vals.size(), s, &slot);
    if (st != KT_OK) return st;
    uint64_t *d = static_cast<uint64_t *>(slot->dev);
    KtSgd a{scale, lr, momentum, weight_decay, first_step ? 1 : 0, resident ? p->dev_sgd : nullptr};
    int e = kt_launch_fused_sgd(p->tb, hp.dt, tile0, ntiles, reinterpret_cast<const void *const *>(d),
                                reinterpret_cast<const void *const *>(d + P0), K, w,
                                reinterpret_cast<void *const *>(d + T), reinterpret_cast<void *const *>(d + 2 * T),
                                master ? reinterpret_cast<void *const *>(d + 3 * T) : nullptr, a, vec, stream);
    if (e != 0) { kt_set_error("%s: launch: %s", who, hipGetErrorString((hipError_t)e)); return KT_EHIP; }
    return mark_used(p, slot, s);
    KT_GUARD_END(who)
}

extern "C" kt_status kt_fused_step_sgd(kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                                       const void *const *peer_bufs, int K, const float *weights, float scale,
                                       void *const *param_ptrs, void *const *momentum_ptrs, void *const *model_ptrs,
                                       float lr, float momentum, float weight_decay, int first_step, void *stream)
{
    return fused_sgd_impl(p, bucket, local_tensor_ptrs, peer_bufs, K, weights, scale, param_ptrs, momentum_ptrs,
                          model_ptrs, lr, momentum, weight_decay, first_step, stream, "kt_fused_step_sgd", false);
}

extern "C" kt_status kt_fused_step_sgd_resident(kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                                                const void *const *peer_bufs, int K, void *const *param_ptrs,
                                                void *const *momentum_ptrs, void *const *model_ptrs, int first_step,
                                                void *stream)
{
    return fused_sgd_impl(p, bucket, local_tensor_ptrs, peer_bufs, K, nullptr, 0.0f, param_ptrs, momentum_ptrs,
                          model_ptrs, 0.0f, 0.0f, 0.0f, first_step, stream, "kt_fused_step_sgd_resident", true);
}

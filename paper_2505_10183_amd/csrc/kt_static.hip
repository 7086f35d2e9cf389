// The entry point that allocates nothing: kt_fused_step_noalloc.
//
// kt_fused_step keeps two things in device memory that it allocates itself: the
// plan's tables (tile table, tensor offsets and sizes, bucket lengths) and the
// per-call pointer table.  Here both live in one file-scope device array of fixed
// size, `scratch`, that every GPU the library runs on holds until the process
// ends.  The kernels are the ones kt_fused_step launches; they receive addresses
// inside the array exactly as they receive the allocated tables there.
//
// In host code the array's name is only a stand-in for the device symbol: its
// device address is obtained once per device with hipGetSymbolAddress and every
// use below (kernel arguments, copies) goes through that address.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "kt_internal.h"

#define KT_STATIC_BYTES (4u << 20)        // size of the device array
#define KT_STATIC_MAX_PTRS 65536          // entries of the per-call pointer table
#define KT_STATIC_MAX_DEVICES 16

static __device__ __align__(256) unsigned char scratch[KT_STATIC_BYTES];

namespace {

struct DevState {
    unsigned char *ptr = nullptr;   // device address of `scratch` on this device
    uint64_t plan_serial = 0;       // plan whose tables the array holds (0 = none)
    size_t nptr = 0;                // entries of the pointer table it holds
    bool ptrs_valid = false;
    uint64_t mirror[KT_STATIC_MAX_PTRS];   // host copy of that pointer table (and the source of its upload)
};

DevState g_dev[KT_STATIC_MAX_DEVICES];
std::mutex g_mu;

kt_status fail(const char *what, hipError_t e)
{
    kt_set_error("kt_fused_step_noalloc: %s: %s", what, hipGetErrorString(e));
    return KT_EHIP;
}

size_t pad256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

extern "C" kt_status kt_fused_step_noalloc(kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                                           const void *const *peer_bufs, int K, const float *weights, float scale,
                                           void *const *out_tensor_ptrs, void *stream)
{
    const char *who = "kt_fused_step_noalloc";
    // per-thread, grows once to the size a caller needs (host memory only)
    static thread_local std::vector<uint64_t> vals;
    try {
        int64_t tile0 = 0, ntiles = 0;
        bool vec = false;
        KtWeights w;
        kt_status st = kt_fused_prepare(p, bucket, local_tensor_ptrs, peer_bufs, K, weights, out_tensor_ptrs, who, vals,
                                        &w, &tile0, &ntiles, &vec);
        if (st != KT_OK || ntiles == 0) return st;

        // layout inside the array: [tiles | tensor offsets | tensor sizes | bucket lengths | pointer table]
        const KtHostPlan &hp = kt_plan_host(p);
        const size_t T = hp.t_numel.size(), nb = hp.b_elems.size(), nt = hp.tiles.size(), np = vals.size();
        const size_t o_tiles = 0;
        const size_t o_off = o_tiles + pad256(nt * sizeof(KtTile));
        const size_t o_numel = o_off + pad256(T * 8);
        const size_t o_belems = o_numel + pad256(T * 8);
        const size_t o_ptrs = o_belems + pad256(nb * 8);
        const size_t total = o_ptrs + np * 8;
        if (np > KT_STATIC_MAX_PTRS || total > KT_STATIC_BYTES) {
            kt_set_error("%s: the plan needs %zu bytes of tables and %zu pointers; this entry point holds at most "
                         "%u bytes and %d pointers (use kt_fused_step)", who, total, np, (unsigned)KT_STATIC_BYTES,
                         KT_STATIC_MAX_PTRS);
            return KT_EUNSUPPORTED;
        }

        int dev = -1;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return fail("hipGetDevice", e);
        if (dev < 0 || dev >= KT_STATIC_MAX_DEVICES) {
            kt_set_error("%s: device %d outside [0,%d)", who, dev, KT_STATIC_MAX_DEVICES);
            return KT_EUNSUPPORTED;
        }
        std::lock_guard<std::mutex> lock(g_mu);
        DevState &d = g_dev[dev];
        if (!d.ptr) {
            // once per device, with that device current: every GPU has its own copy of the array
            void *sym = nullptr;
            e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !sym) return fail("hipGetSymbolAddress(scratch)", e);
            d.ptr = static_cast<unsigned char *>(sym);
        }
        unsigned char *base = d.ptr;
        hipStream_t s = static_cast<hipStream_t>(stream);

        const bool need_plan = d.plan_serial != kt_plan_serial(p);
        const bool need_ptrs = need_plan || !d.ptrs_valid || d.nptr != np || memcmp(d.mirror, vals.data(), np * 8) != 0;
        if (need_plan || need_ptrs) {
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(s, &cs) == hipSuccess && cs == hipStreamCaptureStatusActive) {
                kt_set_error("%s: the tables of this call are not in the device array yet and an upload cannot be "
                             "recorded into a graph; make the same call once outside stream capture first", who);
                return KT_EUNSUPPORTED;
            }
            // The uploads are ordered on `s` behind earlier launches that read the array.
            // Whatever fails below, the array no longer holds what the state says.
            d.plan_serial = 0;
            d.ptrs_valid = false;
            if (need_plan) {
                if (nt) { e = hipMemcpyAsync(base + o_tiles, hp.tiles.data(), nt * sizeof(KtTile), hipMemcpyHostToDevice, s); if (e != hipSuccess) return fail("upload of the tile table", e); }
                if (T) { e = hipMemcpyAsync(base + o_off, hp.t_off.data(), T * 8, hipMemcpyHostToDevice, s); if (e != hipSuccess) return fail("upload of the tensor offsets", e); }
                if (T) { e = hipMemcpyAsync(base + o_numel, hp.t_numel.data(), T * 8, hipMemcpyHostToDevice, s); if (e != hipSuccess) return fail("upload of the tensor sizes", e); }
                if (nb) { e = hipMemcpyAsync(base + o_belems, hp.b_elems.data(), nb * 8, hipMemcpyHostToDevice, s); if (e != hipSuccess) return fail("upload of the bucket lengths", e); }
            }
            memcpy(d.mirror, vals.data(), np * 8);
            if (np) { e = hipMemcpyAsync(base + o_ptrs, d.mirror, np * 8, hipMemcpyHostToDevice, s); if (e != hipSuccess) return fail("upload of the pointer table", e); }
            // the sources are ordinary host memory (the plan's tables, the mirror): they may
            // change or go away once this call returns, so the copies must have left them
            e = hipStreamSynchronize(s);
            if (e != hipSuccess) return fail("hipStreamSynchronize", e);
            d.plan_serial = kt_plan_serial(p);
            d.nptr = np;
            d.ptrs_valid = true;
        }

        KtDeviceTables tb;
        tb.tiles = reinterpret_cast<const KtTile *>(base + o_tiles);
        tb.t_off = reinterpret_cast<const int64_t *>(base + o_off);
        tb.t_numel = reinterpret_cast<const int64_t *>(base + o_numel);
        tb.b_elems = reinterpret_cast<const int64_t *>(base + o_belems);
        const uint64_t *dp = reinterpret_cast<const uint64_t *>(base + o_ptrs);
        int le = kt_launch_fused(tb, hp.dt, tile0, ntiles, reinterpret_cast<const void *const *>(dp),
                                 reinterpret_cast<const void *const *>(dp + 2 * T), K, w, scale,
                                 reinterpret_cast<void *const *>(const_cast<uint64_t *>(dp + T)), vec, stream);
        if (le != 0) return fail("launch", (hipError_t)le);
        return KT_OK;
    } catch (const std::bad_alloc &) {
        kt_set_error("%s: out of host memory", who);
        return KT_ENOMEM;
    } catch (...) {
        kt_set_error("%s: unexpected internal error", who);
        return KT_EINVAL;
    }
}

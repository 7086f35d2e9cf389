// Internal structures shared by the host plan code, the C ABI and the kernels.
#ifndef KT_INTERNAL_H
#define KT_INTERNAL_H

#include <stdint.h>
#include <vector>

#include "kt.h"

// A tile is a fixed-size slice of one bucket; one workgroup processes one tile.
#ifndef KT_TILE_BYTES
#define KT_TILE_BYTES 16384
#endif
#define KT_VEC_BYTES 16
#define KT_TILE_VECS (KT_TILE_BYTES / KT_VEC_BYTES)
#define KT_BLOCK 256
// Mixed tiles holding at most this many tensors stage their slice of the
// tensor table in LDS; larger ones search the table in global memory.
#ifndef KT_LDS_TENSORS
#define KT_LDS_TENSORS 512
#endif

// Per-tile record (device table).  `nt == 0` marks a solid tile: tensor `t0`
// covers every element of the tile and the tile is a whole number of 16-byte
// vectors.  Otherwise tensors t0 .. t0+nt-1 are the ones that may own
// elements of the tile (the rest is padding).
struct KtTile {
    int32_t bucket;
    uint32_t tile_in_bucket;
    int32_t t0;
    int32_t nt;
};

struct KtHostPlan {
    kt_dtype dt;
    int elem_size;
    int64_t cap_bytes;
    int align_bytes;
    int64_t tile_elems;
    // per tensor
    std::vector<int64_t> t_numel, t_off;
    std::vector<int32_t> t_bucket;
    // per bucket
    std::vector<int64_t> b_elems;
    std::vector<int32_t> b_first, b_count;
    std::vector<int64_t> b_tile0;      // first tile of each bucket, nb+1 entries
    std::vector<KtTile> tiles;
};

// Builds the layout and the tile table.  Returns KT_OK or an error with `msg` set.
kt_status kt_build_host_plan(const int64_t *numel, int T, kt_dtype dt,
                             int64_t cap_bytes, int align_bytes,
                             KtHostPlan &hp, const char **msg);

// Device-side view of the plan tables plus the per-call pointer tables.
struct KtDeviceTables {
    const KtTile *tiles;
    const int64_t *t_off;
    const int64_t *t_numel;
    const int64_t *b_elems;
};

// Launchers (defined next to their kernels in the .hip files).  `tile0`/`ntiles` select a contiguous tile range.
// All return a hipError_t cast to int.
int kt_launch_pack(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0,
                   int64_t ntiles, const void *const *d_tensor_ptrs,
                   void *const *d_bucket_ptrs, bool vector_ok, void *stream);
int kt_launch_unpack(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0,
                     int64_t ntiles, const void *const *d_bucket_ptrs,
                     float scale, void *const *d_tensor_ptrs, bool vector_ok,
                     void *stream);
// Store window of the read-dominated kernels (reduce, fused pass) on large launches: every wave
// holds its finished results back until the device-wide constant-rate clock, masked to a period
// of about 10 us, is inside the first `width` ticks, so that the whole chip alternates between
// reading and writing instead of sprinkling one written line among eight read ones.  Measured on
// 8 peers: 72-73 % -> 77-78 % of 8 TB/s, flat for periods of 9-18 us, and a steep loss once the
// period exceeds the time the resident workgroups need for their loads (about 14-19 us), which
// is why it is used only where that time is known to be longer (K >= 4, many tiles).
// width == 0: no window.
struct KtWindow {
    uint32_t period;  // clock ticks
    uint32_t width;   // ticks at the start of each period in which stores are issued
};
// The window for a launch of `ntiles` tiles with K peers on the current device (host); none
// below `min_tiles` tiles: a launch of a few generations of workgroups only pays for the waits
// of its first and last one.
KtWindow kt_store_window(int K, int64_t ntiles, int64_t min_tiles);
// KT_WINDOW_NS: period in nanoseconds (0 switches the window off); KT_WINDOW_OPEN_PCT: the share
// of the period in which stores are issued.
#ifndef KT_WINDOW_NS
#define KT_WINDOW_NS 12000
#endif
#ifndef KT_WINDOW_OPEN_PCT
#define KT_WINDOW_OPEN_PCT 10
#endif
// Smallest launches that use the window.  The fused pass is a step of its own and gains from
// 16 Ki tiles (256 MiB per copy) on; the reduce inside the chained step (between pack and
// unpack) measured 2 % slower with the window at 21 Ki tiles and 5 % faster at 160 Ki.
#ifndef KT_WINDOW_MIN_TILES_FUSED
#define KT_WINDOW_MIN_TILES_FUSED 16384
#endif
#ifndef KT_WINDOW_MIN_TILES_REDUCE
#define KT_WINDOW_MIN_TILES_REDUCE 65536
#endif

// The K weights of a launch travel in the kernel-argument block (`w`), unless
// `dev` is set: then the kernels read them from that device array when they
// run (kt_plan_set_weights), so that a recorded graph follows later updates.
struct KtWeights {
    float w[KT_MAX_PEERS];
    const float *dev;
};
int kt_launch_reduce(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0,
                     int64_t ntiles, const void *const *d_peer_ptrs, int K,
                     const KtWeights &w, void *const *d_out_ptrs,
                     bool vector_ok, void *stream);
int kt_launch_fused(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0,
                    int64_t ntiles, const void *const *d_local_ptrs,
                    const void *const *d_peer_ptrs, int K, const KtWeights &w,
                    float scale, void *const *d_out_ptrs, bool vector_ok,
                    void *stream);

struct KtSgd {
    float scale, lr, mu, wd;
    int first;
    const float *dev;   // non-NULL: {scale, lr, mu, wd} are read from these 4 device floats when the kernel runs
};
int kt_launch_unpack_sgd(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0,
                         int64_t ntiles, const void *const *d_bucket_ptrs,
                         void *const *d_param_ptrs, void *const *d_mom_ptrs,
                         void *const *d_model_ptrs /* NULL: no bf16 model copy */,
                         const KtSgd &a, bool vector_ok, void *stream);

// The single pass from K gradient copies to updated parameters (kt_fused_sgd.hip).
int kt_launch_fused_sgd(const KtDeviceTables &tb, kt_dtype dt, int64_t tile0,
                        int64_t ntiles, const void *const *d_local_ptrs,
                        const void *const *d_peer_ptrs, int K, const KtWeights &w,
                        void *const *d_param_ptrs, void *const *d_mom_ptrs,
                        void *const *d_model_ptrs /* NULL: no bf16 model copy */,
                        const KtSgd &a, bool vector_ok, void *stream);

// ---- shared between the C ABI (kt_api.cpp) and the entry point that
// allocates nothing (kt_static.hip) ------------------------------------------

void kt_set_error(const char *fmt, ...);

// The immutable host tables of a plan and a number that identifies the plan
// for the lifetime of the process (never reused).
const KtHostPlan &kt_plan_host(const kt_plan *p);
uint64_t kt_plan_serial(const kt_plan *p);

// Argument checks of the fused single pass and its pointer table
// [local tensors T | output tensors T | peers nb*(K-1)] written to `vals`
// (2T + nb*(K-1) entries).  *ntiles == 0 on return means nothing to do.
kt_status kt_fused_prepare(const kt_plan *p, int bucket, const void *const *local_tensor_ptrs,
                           const void *const *peer_bufs, int K, const float *weights,
                           void *const *out_tensor_ptrs, const char *who, std::vector<uint64_t> &vals,
                           KtWeights *w, int64_t *tile0, int64_t *ntiles, bool *vector_ok);

#endif

// Measuring aid of bench.py, not part of the library: a read-only stream with
// the access pattern of the K-way reduce (16 KiB tiles, 256 lanes, four 16-byte
// non-temporal loads per lane and buffer, all in flight together) that stores
// nothing.  The rate it reaches is what the device sustains for pure reads; the
// reduce adds one written vector per K read ones.  Built into
// libkt_bench_probe.so beside bench.py; nothing in the library links to it.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define PROBE_TILE_VECS 1024
#define PROBE_BLOCK 256

namespace {

struct ProbeBufs {
    const void *p[8];
};

template <int K>
__global__ __launch_bounds__(PROBE_BLOCK) void bench_probe_read_kernel(ProbeBufs b, void *sink)
{
    constexpr int VPT = PROBE_TILE_VECS / PROBE_BLOCK;
    const int64_t base = (int64_t)blockIdx.x * PROBE_TILE_VECS + threadIdx.x;
    u32x4 r[VPT][K];
#pragma unroll
    for (int u = 0; u < VPT; ++u)
#pragma unroll
        for (int k = 0; k < K; ++k)
            r[u][k] = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4 *)b.p[k] + base + u * PROBE_BLOCK);
    u32x4 acc = {0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < VPT; ++u)
#pragma unroll
        for (int k = 0; k < K; ++k) acc ^= r[u][k];
    // keeps the loads alive; the pattern does not occur in data worth probing with
    if (acc[0] == 0x6B745F70u && acc[1] == 0x726F6265u && acc[2] == 0x5F726561u && acc[3] == 0x645F5F21u)
        *(u32x4 *)sink = acc;
}

}  // namespace

// Streams the first bytes_each bytes, rounded down to a multiple of 16 KiB, of
// each of K (1..8) device buffers (16-byte aligned); `sink` is 16 writable,
// 16-byte aligned device bytes, written only if the XOR of everything a lane
// read equals one fixed 128-bit pattern.  Returns the bytes streamed per buffer,
// or -1 for bad arguments, -2 if the launch failed.
extern "C" int64_t bench_probe_read(const void *const *bufs, int K, int64_t bytes_each, void *sink, void *stream)
{
    if (!bufs || !sink || K < 1 || K > 8 || bytes_each < 0 || ((uintptr_t)sink & 15u)) return -1;
    ProbeBufs b;
    for (int k = 0; k < 8; ++k) {
        b.p[k] = k < K ? bufs[k] : nullptr;
        if (k < K && (!bufs[k] || ((uintptr_t)bufs[k] & 15u))) return -1;
    }
    const int64_t ntiles = bytes_each / (PROBE_TILE_VECS * 16);
    if (ntiles >= ((int64_t)1 << 24)) return -1;
    if (ntiles == 0) return 0;
    dim3 grid((unsigned)ntiles), block(PROBE_BLOCK);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    switch (K) {
#define PROBE_CASE(KK) \
    case KK: bench_probe_read_kernel<KK><<<grid, block, 0, s>>>(b, sink); break;
        PROBE_CASE(1) PROBE_CASE(2) PROBE_CASE(3) PROBE_CASE(4) PROBE_CASE(5) PROBE_CASE(6) PROBE_CASE(7) PROBE_CASE(8)
#undef PROBE_CASE
    }
    return hipGetLastError() == hipSuccess ? ntiles * PROBE_TILE_VECS * 16 : -2;
}

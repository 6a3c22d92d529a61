// Benchmark-only helpers, built into their own shared object (not part of the library and
// not declared in its ABI header):
//   * arithmetic-free streams with the byte mix of the two bandwidth-bound steps, so that a
//     benchmark can put what the machine reaches for that mix of reads and writes beside
//     what the real kernels reach;
//   * HIP timing events created without the system-scope fence, recorded on a given stream.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBlock = 256;

// DEPTH consecutive 256-item pieces per workgroup: a lane issues its DEPTH loads first, then
// its DEPTH stores, every instruction coalesced and linear over the wave.  DEPTH 1 is the
// plain one-item-per-thread stream; DEPTH 4 is the fastest form found for both mixes.
// mode 0: 4 bytes in, 16 bytes out per item (the dequant-gather's mix);
// mode 1: 16 bytes in, 4 bytes out (the quantize-append's mix); mode 2: 16 in, 16 out.
template <int MODE, int DEPTH>
__global__ void __launch_bounds__(kBlock) stream_probe_kernel(const char* __restrict__ src,
                                                             char* __restrict__ dst, const int64_t items) {
    const int64_t base = (int64_t)blockIdx.x * (kBlock * DEPTH) + threadIdx.x;
    if constexpr (MODE == 0) {
        uint32_t v[DEPTH];
#pragma unroll
        for (int j = 0; j < DEPTH; ++j)
            v[j] = base + j * kBlock < items ? reinterpret_cast<const uint32_t*>(src)[base + j * kBlock] : 0u;
#pragma unroll
        for (int j = 0; j < DEPTH; ++j)
            if (base + j * kBlock < items) {
                const u32x4 o = {v[j], v[j] + 1u, v[j] ^ 7u, v[j] * 3u};
                __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(dst) + base + j * kBlock);
            }
    } else {
        u32x4 v[DEPTH];
#pragma unroll
        for (int j = 0; j < DEPTH; ++j)
            v[j] = base + j * kBlock < items ? reinterpret_cast<const u32x4*>(src)[base + j * kBlock] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < DEPTH; ++j)
            if (base + j * kBlock < items) {
                if constexpr (MODE == 1)
                    reinterpret_cast<uint32_t*>(dst)[base + j * kBlock] = v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
                else
                    __builtin_nontemporal_store(v[j], reinterpret_cast<u32x4*>(dst) + base + j * kBlock);
            }
    }
}

template <int MODE>
hipError_t launch_probe(int depth, const char* sp, char* dp, int64_t items, hipStream_t s) {
    const int64_t per = (int64_t)kBlock * depth;
    const int64_t blocks = (items + per - 1) / per;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(kBlock);
    switch (depth) {
        case 1: stream_probe_kernel<MODE, 1><<<grid, block, 0, s>>>(sp, dp, items); break;
        case 2: stream_probe_kernel<MODE, 2><<<grid, block, 0, s>>>(sp, dp, items); break;
        case 4: stream_probe_kernel<MODE, 4><<<grid, block, 0, s>>>(sp, dp, items); break;
        case 8: stream_probe_kernel<MODE, 8><<<grid, block, 0, s>>>(sp, dp, items); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

// Streams `items` units from src to dst (device pointers, 16-byte aligned, items * bytes per
// item large), `depth` (1, 2, 4 or 8) pieces per workgroup.  Returns a hipError_t value
// (0 = success); bad arguments give hipErrorInvalidValue.
int bench_stream_probe(int32_t mode, int32_t depth, const void* src, void* dst, int64_t items,
                       void* hip_stream) {
    if (mode < 0 || mode > 2 || items < 0) return (int)hipErrorInvalidValue;
    if (items == 0) return 0;
    if (!src || !dst || ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const char* sp = static_cast<const char*>(src);
    char* dp = static_cast<char*>(dst);
    (void)hipGetLastError();
    switch (mode) {
        case 0: return (int)launch_probe<0>(depth, sp, dp, items, s);
        case 1: return (int)launch_probe<1>(depth, sp, dp, items, s);
        default: return (int)launch_probe<2>(depth, sp, dp, items, s);
    }
}

// A timing event for the benchmark's per-kernel figures.  Created with
// hipEventDisableSystemFence: recording it does not make the stream perform a system-scope
// release (a write-back of the caches towards the host) between the two kernels it separates.
// Nothing in the benchmark reads the kernels' results on the host between two events, and
// the plain event's fence is most of what an event costs the stream after a kernel that
// wrote hundreds of megabytes (about 8 us against 3 to 4 us per event).
void* bench_event_create(void) {
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
    return e;
}
int bench_event_record(void* ev, void* hip_stream) {
    return (int)hipEventRecord(static_cast<hipEvent_t>(ev), static_cast<hipStream_t>(hip_stream));
}
// Milliseconds between two recorded, completed events; negative on error.
float bench_event_elapsed_ms(void* a, void* b) {
    float ms = -1.0f;
    if (hipEventElapsedTime(&ms, static_cast<hipEvent_t>(a), static_cast<hipEvent_t>(b)) != hipSuccess) return -1.0f;
    return ms;
}
void bench_event_destroy(void* ev) { (void)hipEventDestroy(static_cast<hipEvent_t>(ev)); }

}  // extern "C"
#pragma GCC visibility pop

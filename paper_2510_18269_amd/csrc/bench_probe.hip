// Benchmark-only helpers, built into their own shared object (not part of the library and
// not declared in its ABI header):
//   * arithmetic-free streams with the byte mix of the two bandwidth-bound steps, so that a
//     benchmark can put what the machine reaches for that mix of reads and writes beside
//     what the real kernels reach;
//   * HIP events created with chosen flags, recorded on a given stream.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBlock = 256;

// One item per thread, every access coalesced and linear.
// mode 0: 4 bytes in, 16 bytes out (the dequant-gather's mix);
// mode 1: 16 bytes in, 4 bytes out (the quantize-append's mix); mode 2: 16 in, 16 out.
template <int MODE>
__global__ void __launch_bounds__(kBlock) stream_probe_kernel(const char* __restrict__ src,
                                                             char* __restrict__ dst, const int64_t items) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= items) return;
    if constexpr (MODE == 0) {
        const uint32_t v = reinterpret_cast<const uint32_t*>(src)[i];
        const u32x4 o = {v, v + 1u, v ^ 7u, v * 3u};
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(dst) + i);
    } else if constexpr (MODE == 1) {
        const u32x4 v = reinterpret_cast<const u32x4*>(src)[i];
        reinterpret_cast<uint32_t*>(dst)[i] = v[0] ^ v[1] ^ v[2] ^ v[3];
    } else {
        const u32x4 v = reinterpret_cast<const u32x4*>(src)[i];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst) + i);
    }
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

// Streams `items` units from src to dst (device pointers, 16-byte aligned, items * bytes per
// item large).  Returns a hipError_t value (0 = success); bad arguments give hipErrorInvalidValue.
int bench_stream_probe(int32_t mode, const void* src, void* dst, int64_t items, void* hip_stream) {
    if (mode < 0 || mode > 2 || items < 0) return (int)hipErrorInvalidValue;
    if (items == 0) return 0;
    if (!src || !dst || ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return (int)hipErrorInvalidValue;
    const int64_t blocks = (items + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffffLL) return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const char* sp = static_cast<const char*>(src);
    char* dp = static_cast<char*>(dst);
    (void)hipGetLastError();
    switch (mode) {
        case 0: stream_probe_kernel<0><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(sp, dp, items); break;
        case 1: stream_probe_kernel<1><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(sp, dp, items); break;
        default: stream_probe_kernel<2><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(sp, dp, items); break;
    }
    return (int)hipGetLastError();
}

// A timing event.  light != 0: created with hipEventDisableSystemFence, i.e. recording it
// does not make the stream perform a system-scope release (cache write-back) between the
// kernels it separates, which is most of what an event costs the stream.
void* bench_event_create(int32_t light) {
    hipEvent_t e = nullptr;
    const unsigned flags = light ? hipEventDisableSystemFence : hipEventDefault;
    if (hipEventCreateWithFlags(&e, flags) != hipSuccess) return nullptr;
    return e;
}
int bench_event_record(void* ev, void* hip_stream) {
    return (int)hipEventRecord(static_cast<hipEvent_t>(ev), static_cast<hipStream_t>(hip_stream));
}
int bench_event_synchronize(void* ev) { return (int)hipEventSynchronize(static_cast<hipEvent_t>(ev)); }
// Milliseconds between two recorded, completed events; negative on error.
float bench_event_elapsed_ms(void* a, void* b) {
    float ms = -1.0f;
    if (hipEventElapsedTime(&ms, static_cast<hipEvent_t>(a), static_cast<hipEvent_t>(b)) != hipSuccess) return -1.0f;
    return ms;
}
void bench_event_destroy(void* ev) { (void)hipEventDestroy(static_cast<hipEvent_t>(ev)); }

}  // extern "C"
#pragma GCC visibility pop

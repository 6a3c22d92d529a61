// Measurement aid (not part of the method): arithmetic-free streams with the byte mix of the
// two bandwidth-bound steps, one item per thread, every access coalesced and linear.  A
// benchmark runs them beside the real kernels to state what the machine reaches for that
// mix of reads and writes.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

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

hipError_t launch_stream_probe(int mode, const void* src, void* dst, int64_t items, hipStream_t s) {
    if (items == 0) return hipSuccess;
    const int64_t blocks = (items + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const char* sp = static_cast<const char*>(src);
    char* dp = static_cast<char*>(dst);
    switch (mode) {
        case 0: stream_probe_kernel<0><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(sp, dp, items); break;
        case 1: stream_probe_kernel<1><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(sp, dp, items); break;
        case 2: stream_probe_kernel<2><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(sp, dp, items); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace oqm

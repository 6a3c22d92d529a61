// Exhaustive check, on the GPU, that the short division sequences used by the quantize
// kernel (div15_exact, div3_exact, rcp_exact in oqm_device.h) reproduce correctly rounded IEEE float32
// division for every input the quantizer can produce:
//   s   = range / 15 and range / 3   for all 2^31 - 2^23 non-negative finite floats `range`
//                      (compared after the "below FLT_MIN -> 0" rule the kernel applies)
//   inv = 1 / s        for every normal s in [FLT_MIN, 2^126] (beyond that, reachable only
//                      with 2-bit codes, the kernels use the full division)
// The reference is the compiler's own IEEE division (no fast-math).  Prints the mismatch
// counts and exits non-zero if any is not 0.  All accesses are to three small counters.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "oqm_device.h"

__global__ void check_all(unsigned long long* bad) {
    const uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;  // [0, 2^31)
    if (u >= 0x7f800000u) return;                              // finite, non-negative
    const float a = __uint_as_float(u);
    const float ref = a / 15.0f;
    const float fast = oqm::div15_exact(a);
    const float sref = ref >= 1.17549435e-38f ? ref : 0.0f;
    const float sfast = fast >= 1.17549435e-38f ? fast : 0.0f;
    if (__float_as_uint(sref) != __float_as_uint(sfast)) atomicAdd(&bad[0], 1ull);
    const float ref3 = a / 3.0f;
    const float fast3 = oqm::div3_exact(a);
    const float sref3 = ref3 >= 1.17549435e-38f ? ref3 : 0.0f;
    const float sfast3 = fast3 >= 1.17549435e-38f ? fast3 : 0.0f;
    if (__float_as_uint(sref3) != __float_as_uint(sfast3)) atomicAdd(&bad[2], 1ull);
    if (u >= 0x00800000u && a <= 0x1p126f) {  // every normal s with a normal quotient
        const float rr = 1.0f / a, rf = oqm::rcp_exact(a);
        if (__float_as_uint(rr) != __float_as_uint(rf)) atomicAdd(&bad[1], 1ull);
    }
}

int main() {
    unsigned long long* bad = nullptr;
    if (hipMalloc(&bad, 32) != hipSuccess || hipMemset(bad, 0, 32) != hipSuccess) {
        std::printf("selfcheck_division: no GPU memory\n");
        return 2;
    }
    check_all<<<(1u << 31) / 256, 256>>>(bad);
    unsigned long long h[3] = {~0ull, ~0ull, ~0ull};
    if (hipMemcpy(h, bad, 24, hipMemcpyDeviceToHost) != hipSuccess) {
        std::printf("selfcheck_division: kernel failed: %s\n", hipGetErrorString(hipGetLastError()));
        return 2;
    }
    std::printf("div15_exact mismatches: %llu\nrcp_exact mismatches: %llu\ndiv3_exact mismatches: %llu\n", h[0], h[1],
                h[2]);
    hipFree(bad);
    return (h[0] == 0 && h[1] == 0 && h[2] == 0) ? 0 : 1;
}

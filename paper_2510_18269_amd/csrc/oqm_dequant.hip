// Reconstruction of the selected frame-groups into the bounded active KV buffer
// (paper Sec. 3.4, Eq. 11 and Eq. 13; supplement "Cache reconstruction for decoding").
//
// One workgroup of 256 threads owns one (layer, rank, K|V, head) tile: it reads
// the group index from device memory (the index array never visits the host),
// streams the tile's packed nibbles and (scale, zero) pairs, and writes G x d
// outputs to token rows [rank*G, (rank+1)*G) of the layer's active buffer.  A
// lane turns one 32-bit word of codes (8 channels) into one 128-bit store, so
// each store instruction of a wave writes 1 KB of contiguous bf16.  HBM-bound:
// 0.5 + 8/gs bytes read and 2 bytes written per element.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

constexpr int kUnroll = 4;

template <typename OUT, int LPG>
__global__ void __launch_bounds__(kBlock) dequant_gather_kernel(const DequantArgs a) {
    constexpr int EB = elem_bytes<OUT>::value;
    const int H = a.n_kv_heads, d = a.head_dim, G = a.group_tokens;

    // blockIdx -> (layer li, rank r, kv, head h), head fastest
    int b = blockIdx.x;
    const int h = b % H;
    b /= H;
    const int kv = b & 1;
    b >>= 1;
    const int r = b % a.k_eff;
    const int li = b / a.k_eff;

    const int t = a.idx[(int64_t)li * a.k + r];
    if ((unsigned)t >= (unsigned)a.n_groups) return;  // not a stored group: leave the rows alone

    const int lpr = d >> 3;
    const int rpp = kBlock / lpr;
    const int tid = threadIdx.x;
    const int row0 = tid / lpr;
    const int slot = tid - row0 * lpr;
    if (row0 >= rpp) return;
    const int ng = lpr / LPG;
    const int g = slot / LPG;

    const int64_t tile = (((int64_t)(a.layer0 + li) * 2 + kv) * a.capacity_groups + t) * H + h;
    const uint32_t* codes_t =
        reinterpret_cast<const uint32_t*>(a.codes + tile * ((int64_t)G * d / 2));
    const float* scale_t = a.scale + tile * ((int64_t)G * ng);
    const float* zero_t = a.zero + tile * ((int64_t)G * ng);
    char* out = static_cast<char*>(kv ? a.v_out : a.k_out) +
                ((((int64_t)li * H + h) * a.k + r) * G) * (int64_t)d * EB;

    for (int r0 = row0; r0 < G; r0 += kUnroll * rpp) {
        uint32_t w[kUnroll];
        float s[kUnroll], m[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int row = r0 + u * rpp;
            if (row < G) {
                w[u] = __builtin_nontemporal_load(codes_t + (int64_t)row * lpr + slot);
                s[u] = scale_t[(int64_t)row * ng + g];
                m[u] = zero_t[(int64_t)row * ng + g];
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int row = r0 + u * rpp;
            if (row < G) {
                float x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float c = (float)((w[u] >> (4 * i)) & 15u);
                    x[i] = __fadd_rn(__fmul_rn(c, s[u]), m[u]);  // Eq. 11, multiply then add
                }
                store8(out + ((int64_t)row * d + slot * 8) * EB, OUT{}, x);
            }
        }
    }
}

template <typename OUT, int LPG>
hipError_t launch_t(const DequantArgs& a, hipStream_t s) {
    const int64_t blocks = (int64_t)a.n_layers * a.k_eff * 2 * a.n_kv_heads;
    if (blocks == 0) return hipSuccess;
    dequant_gather_kernel<OUT, LPG><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(a);
    return hipGetLastError();
}

template <typename OUT>
hipError_t launch_lpg(const DequantArgs& a, hipStream_t s) {
    switch (a.qgroup) {
        case 8: return launch_t<OUT, 1>(a, s);
        case 16: return launch_t<OUT, 2>(a, s);
        case 32: return launch_t<OUT, 4>(a, s);
        case 64: return launch_t<OUT, 8>(a, s);
        case 128: return launch_t<OUT, 16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_dequant_gather(const DequantArgs& a, int out_dtype, hipStream_t s) {
    switch (out_dtype) {
        case TOM_F32: return launch_lpg<In_f32>(a, s);
        case TOM_BF16: return launch_lpg<In_bf16>(a, s);
        case TOM_F16: return launch_lpg<In_f16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace oqm

// Reconstruction of the selected frame-groups into the bounded active KV buffer
// (paper Sec. 3.4, Eq. 11 and Eq. 13; supplement "Cache reconstruction for decoding").
//
// One workgroup of 256 threads owns one (layer, rank, K|V, head) tile: it reads
// the group index from device memory (the index array never visits the host),
// streams the tile's packed nibbles and (scale, zero) pairs, and writes G x d
// outputs to token rows [rank*G, (rank+1)*G) of the layer's active buffer.  A
// lane turns one 32-bit word of codes (8 channels) into one 128-bit store, so
// each store instruction of a wave writes 1 KB of contiguous bf16.  HBM-bound:
// 0.5 + 8/gs bytes read and 2 bytes written per element; the loads of the next
// rows are issued before the current rows are converted and stored.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

constexpr int kUnroll = 4;

struct Row {
    uint32_t w;  // 8 packed codes
    float s, m;  // scale and zero point of their quant-group
};

template <typename OUT>
__global__ void __launch_bounds__(kBlock) dequant_gather_kernel(const DequantArgs a, const int lpg) {
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
    const int ng = lpr / lpg;

    const int64_t tile = (((int64_t)(a.layer0 + li) * 2 + kv) * a.capacity_groups + t) * H + h;
    const char* codes_t = reinterpret_cast<const char*>(a.codes + tile * ((int64_t)G * d / 2));
    const char* scale_t = reinterpret_cast<const char*>(a.scale + tile * ((int64_t)G * ng));
    const char* zero_t = reinterpret_cast<const char*>(a.zero + tile * ((int64_t)G * ng));
    char* out = static_cast<char*>(kv ? a.v_out : a.k_out) +
                ((((int64_t)li * H + h) * a.k + r) * G) * (int64_t)d * EB;
    // offsets inside one tile fit 32 bits (G * d * 4 < 2^31 is checked on the host)
    const uint32_t code_lane = ((uint32_t)row0 * lpr + slot) * 4u;
    const uint32_t meta_lane = ((uint32_t)row0 * ng + slot / lpg) * 4u;
    const uint32_t out_lane = ((uint32_t)row0 * d + slot * 8u) * EB;

    Row cur[kUnroll], nxt[kUnroll];
    auto fetch = [&](Row (&dst)[kUnroll], int r0) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rb = r0 + u * rpp;
            dst[u].w = 0u;
            dst[u].s = 0.0f;
            dst[u].m = 0.0f;
            if (rb + row0 < G) {
                dst[u].w = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t*>(codes_t + (code_lane + (uint32_t)rb * lpr * 4u)));
                const uint32_t mo = meta_lane + (uint32_t)rb * ng * 4u;
                dst[u].s = __builtin_nontemporal_load(reinterpret_cast<const float*>(scale_t + mo));
                dst[u].m = __builtin_nontemporal_load(reinterpret_cast<const float*>(zero_t + mo));
            }
        }
    };
    fetch(cur, 0);
    for (int r0 = 0; r0 < G; r0 += kUnroll * rpp) {
        fetch(nxt, r0 + kUnroll * rpp);  // rows past the tile are not loaded
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rb = r0 + u * rpp;
            if (rb + row0 < G) {
                float x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float c = (float)((cur[u].w >> (4 * i)) & 15u);
                    x[i] = __fadd_rn(__fmul_rn(c, cur[u].s), cur[u].m);  // Eq. 11, multiply then add
                }
                store8(out + (out_lane + (uint32_t)rb * d * EB), OUT{}, x);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) cur[u] = nxt[u];
    }
}

template <typename OUT>
hipError_t launch_t(const DequantArgs& a, hipStream_t s) {
    const int64_t blocks = (int64_t)a.n_layers * a.k_eff * 2 * a.n_kv_heads;
    if (blocks == 0) return hipSuccess;
    dequant_gather_kernel<OUT><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(a, a.qgroup / 8);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_dequant_gather(const DequantArgs& a, int out_dtype, hipStream_t s) {
    switch (out_dtype) {
        case TOM_F32: return launch_t<In_f32>(a, s);
        case TOM_BF16: return launch_t<In_bf16>(a, s);
        case TOM_F16: return launch_t<In_f16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace oqm

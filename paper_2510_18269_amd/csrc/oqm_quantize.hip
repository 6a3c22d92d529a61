// Store step of Online Quantized Memory on gfx950: 4-bit quantization of one
// frame-group tile per workgroup (paper Sec. 3.4, Eq. 8 and Eq. 9), nibble
// packing, and the summary key (mean of the un-quantized keys over the G
// tokens of the group) in the same pass over K.
//
// Work decomposition.  One workgroup of 256 threads owns one
// (frame, layer, K|V, head) tile of G x d elements.  A lane owns 8 consecutive
// channels of one token row: one 128-bit load in, one 32-bit word of packed
// nibbles out, so every load and store instruction of a wave covers one
// contiguous span (1 KB in, 256 B out).  A quant-group of gs channels lives in
// gs/8 adjacent lanes; its min and max are all-reduced with DPP lane swaps, no
// LDS.  The kernel is HBM-bound: per element it reads 2 B (bf16) and writes
// 0.5 B of codes + 8/gs B of scale/zero.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

constexpr int kUnroll = 4;  // independent 128-bit loads in flight per lane

template <typename IN, int LPG, bool SEPARATE_SUMMARY>
__global__ void __launch_bounds__(kBlock) quantize_append_kernel(const QuantArgs a) {
    constexpr int EB = elem_bytes<IN>::value;
    const int H = a.n_kv_heads, d = a.head_dim, G = a.group_tokens;

    // blockIdx -> (frame f, layer li, kv, head h), head fastest
    int b = blockIdx.x;
    const int h = b % H;
    b /= H;
    const int kv = b & 1;
    b >>= 1;
    const int li = b % a.n_layers;
    const int f = b / a.n_layers;
    const int l = a.layer0 + li;
    const int64_t t = (int64_t)a.first_group + f;

    const int lpr = d >> 3;         // lanes per token row
    const int rpp = kBlock / lpr;   // token rows per pass of the workgroup
    const int tid = threadIdx.x;
    const int row0 = tid / lpr;
    const int slot = tid - row0 * lpr;
    const bool active = row0 < rpp;
    const int ng = lpr / LPG;       // quant-groups per token row

    const int64_t in_off = f * a.stride_frame + li * a.stride_layer + h * a.stride_head;
    const char* src = static_cast<const char*>(kv ? a.v : a.k) + in_off * EB;
    const int64_t tile = (((int64_t)l * 2 + kv) * a.capacity_groups + t) * H + h;
    uint32_t* codes_t = reinterpret_cast<uint32_t*>(a.codes + tile * ((int64_t)G * d / 2));
    float* scale_t = a.scale + tile * ((int64_t)G * ng);
    float* zero_t = a.zero + tile * ((int64_t)G * ng);

    const bool do_sum = (kv == 0);
    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0;

    for (int r0 = 0; r0 < G; r0 += kUnroll * rpp) {
        float x[kUnroll][8];
        bool ok[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int row = r0 + u * rpp + row0;
            ok[u] = active && row < G;
            if (ok[u]) {
                load8(src + ((int64_t)row * a.stride_token + slot * 8) * EB, IN{}, x[u]);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) x[u][i] = 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int row = r0 + u * rpp + row0;
            // Eq. 9: m = min, s = (max - min) / 15 over the quant-group.  Every lane takes
            // part in the lane swaps (idle lanes carry zeros) so the DPP reads are defined.
            float mn = x[u][0], mx = x[u][0];
#pragma unroll
            for (int i = 1; i < 8; ++i) {
                mn = fminf(mn, x[u][i]);
                mx = fmaxf(mx, x[u][i]);
            }
            group_minmax<LPG>(mn, mx);
            mn = mn + 0.0f;  // never store -0 as a zero point
            float s = (mx - mn) / 15.0f;
            float inv;
            if (s >= 1.17549435e-38f) {
                inv = 1.0f / s;
            } else {  // flat or sub-normal range: all codes 0
                s = 0.0f;
                inv = 0.0f;
            }
            uint32_t packed = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float q = rintf((x[u][i] - mn) * inv);  // ties to even
                uint32_t c = (uint32_t)q;                     // saturating: negative -> 0
                c = c < 15u ? c : 15u;
                packed |= c << (4 * i);                       // even channel = low nibble
            }
            if (ok[u]) {
                __builtin_nontemporal_store(packed, codes_t + (int64_t)row * lpr + slot);
                if ((slot & (LPG - 1)) == 0) {
                    const int g = slot / LPG;
                    __builtin_nontemporal_store(s, scale_t + (int64_t)row * ng + g);
                    __builtin_nontemporal_store(mn, zero_t + (int64_t)row * ng + g);
                }
            }
            if (!SEPARATE_SUMMARY && do_sum) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] += (double)x[u][i];  // idle lanes add 0
            }
        }
    }

    if (!do_sum) return;  // uniform per workgroup

    if (SEPARATE_SUMMARY) {
        // The keys to average come from another tensor (e.g. taken before the rotary
        // embedding): one more pass, over that tensor only.
        const char* ssrc = static_cast<const char*>(a.ksum) + in_off * EB;
        for (int row = row0; active && row < G; row += rpp) {
            float x[8];
            load8(ssrc + ((int64_t)row * a.stride_token + slot * 8) * EB, IN{}, x);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += (double)x[i];
        }
    }

    // Summary key: column sums over the rpp row slots of the workgroup, in float64.
    __shared__ double red[kBlock * 8];
    if (active) {
#pragma unroll
        for (int i = 0; i < 8; ++i) red[row0 * d + slot * 8 + i] = acc[i];
    }
    __syncthreads();
    float* key = a.keys + (((int64_t)l * a.capacity_groups + t) * H + h) * d;
    for (int c = tid; c < d; c += kBlock) {
        double sum = 0.0;
        for (int r = 0; r < rpp; ++r) sum += red[r * d + c];
        key[c] = (float)(sum / (double)G);
    }
}

template <typename IN, int LPG>
hipError_t launch_t(const QuantArgs& a, hipStream_t s) {
    const int64_t blocks = (int64_t)a.n_frames * a.n_layers * 2 * a.n_kv_heads;
    if (blocks == 0) return hipSuccess;
    if (a.ksum != a.k)
        quantize_append_kernel<IN, LPG, true><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(a);
    else
        quantize_append_kernel<IN, LPG, false><<<dim3((unsigned)blocks), dim3(kBlock), 0, s>>>(a);
    return hipGetLastError();
}

template <typename IN>
hipError_t launch_lpg(const QuantArgs& a, hipStream_t s) {
    switch (a.qgroup) {
        case 8: return launch_t<IN, 1>(a, s);
        case 16: return launch_t<IN, 2>(a, s);
        case 32: return launch_t<IN, 4>(a, s);
        case 64: return launch_t<IN, 8>(a, s);
        case 128: return launch_t<IN, 16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_quantize_append(const QuantArgs& a, int in_dtype, hipStream_t s) {
    switch (in_dtype) {
        case TOM_F32: return launch_lpg<In_f32>(a, s);
        case TOM_BF16: return launch_lpg<In_bf16>(a, s);
        case TOM_F16: return launch_lpg<In_f16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace oqm

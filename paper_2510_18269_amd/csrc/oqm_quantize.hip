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
// 0.5 B of codes + 8/gs B of scale/zero, so the instruction count per element
// is kept low (about 7 vector instructions) and the next rows are already in
// flight while the current ones are quantized.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

constexpr int kUnroll = 4;  // token rows per lane and loop trip; twice that many loads in flight

// Packs the 4-bit codes of 8 values t[i] in [0, 15] (already divided by the step).
// Adding 2^23 rounds t to the nearest integer, ties to even, and leaves that integer in
// the low mantissa bits: bits(t + 2^23) = 0x4B000000 | code.
__device__ __forceinline__ uint32_t pack8(const float (&t)[8]) {
    uint32_t m[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) m[i] = __float_as_uint(__fadd_rn(t[i], 8388608.0f));
    // byte 0 of (m[2j+1] << 4 | m[2j]) is the packed byte j; bits 8..23 of it are zero
    const uint32_t b01 = (m[1] << 4) | m[0];
    const uint32_t b23 = (m[3] << 4) | m[2];
    const uint32_t b45 = (m[5] << 4) | m[4];
    const uint32_t b67 = (m[7] << 4) | m[6];
    const uint32_t lo = (b23 << 8) | b01;  // bytes 0, 1 valid
    const uint32_t hi = (b67 << 8) | b45;
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);  // {lo.b0, lo.b1, hi.b0, hi.b1}
}

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

    // Tile bases are uniform per workgroup; per-lane offsets inside a tile fit 32 bits
    // (checked on the host), which keeps the address arithmetic per row to one add.
    const int64_t in_off = f * a.stride_frame + li * a.stride_layer + h * a.stride_head;
    const char* src = static_cast<const char*>(kv ? a.v : a.k) + in_off * EB;
    const int64_t tile = (((int64_t)l * 2 + kv) * a.capacity_groups + t) * H + h;
    char* codes_t = reinterpret_cast<char*>(a.codes + tile * ((int64_t)G * d / 2));
    char* scale_t = reinterpret_cast<char*>(a.scale + tile * ((int64_t)G * ng));
    char* zero_t = reinterpret_cast<char*>(a.zero + tile * ((int64_t)G * ng));
    const uint32_t in_row_bytes = (uint32_t)a.stride_token * EB;
    const uint32_t in_lane = (uint32_t)row0 * in_row_bytes + (uint32_t)slot * 8u * EB;
    const uint32_t code_lane = ((uint32_t)row0 * lpr + slot) * 4u;
    const uint32_t meta_lane = ((uint32_t)row0 * ng + slot / LPG) * 4u;
    const bool meta_writer = (slot & (LPG - 1)) == 0;

    const bool do_sum = (kv == 0);
    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0;

    Raw8<IN> cur[kUnroll], nxt[kUnroll];
    auto fetch = [&](Raw8<IN> (&dst)[kUnroll], int r0) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int row = r0 + u * rpp + row0;
            if (active && row < G)
                load_raw(src + (in_lane + (uint32_t)(r0 + u * rpp) * in_row_bytes), dst[u]);
            else
                zero_raw(dst[u]);
        }
    };
    fetch(cur, 0);

    for (int r0 = 0; r0 < G; r0 += kUnroll * rpp) {
        fetch(nxt, r0 + kUnroll * rpp);  // rows past the tile are not loaded (zeros)
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rbase = r0 + u * rpp;
            const bool ok = active && rbase + row0 < G;
            float x[8];
            widen(cur[u], x);
            // Eq. 9: m = min, s = (max - min) / 15 over the quant-group.  Every lane takes
            // part in the lane swaps (idle lanes carry zeros) so the DPP reads are defined.
            float mn = x[0], mx = x[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) {
                mn = fminf(mn, x[i]);
                mx = fmaxf(mx, x[i]);
            }
            group_minmax<LPG>(mn, mx);
            mn = mn + 0.0f;  // never store -0 as a zero point
            float s = div15_exact(__fsub_rn(mx, mn));
            float inv;
            if (s >= 1.17549435e-38f) {
                inv = rcp_exact(s);
            } else {  // flat or sub-normal range: all codes 0
                s = 0.0f;
                inv = 0.0f;
            }
            float tq[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) tq[i] = __fmul_rn(__fsub_rn(x[i], mn), inv);  // in [0, 15]
            const uint32_t packed = pack8(tq);  // even channel = low nibble
            if (ok) {
                __builtin_nontemporal_store(
                    packed, reinterpret_cast<uint32_t*>(codes_t + (code_lane + (uint32_t)rbase * lpr * 4u)));
                if (meta_writer) {
                    const uint32_t mo = meta_lane + (uint32_t)rbase * ng * 4u;
                    __builtin_nontemporal_store(s, reinterpret_cast<float*>(scale_t + mo));
                    __builtin_nontemporal_store(mn, reinterpret_cast<float*>(zero_t + mo));
                }
            }
            if (!SEPARATE_SUMMARY && do_sum) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] += (double)x[i];  // idle lanes add 0
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) cur[u] = nxt[u];
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

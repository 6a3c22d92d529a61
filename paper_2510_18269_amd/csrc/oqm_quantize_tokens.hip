// Store step with the quantization axis of the paper's Eq. 9: one (scale, zero) pair per
// head and channel, taken over the G tokens of the frame-group (Sec. 3.4, Eq. 8 and Eq. 9),
// plus nibble packing and the summary key, for one head tile per workgroup.
//
// Same decomposition as the head_dim-axis kernel (grid (head, 2*layer + K|V, frame), lane =
// 8 channels of one token row), but the min/max run down the token rows: each lane keeps
// 8 running minima and maxima over its rows, the 256/(d/8) row slots of the workgroup are
// combined through LDS, one thread per channel derives scale, reciprocal and zero point,
// and a second sweep quantizes and packs.  When a lane's share of the tile fits a few
// registers (HOLD rows: up to 13 x 16 B) the rows stay in registers between the sweeps;
// otherwise the second sweep reads the tile again (from the caches: it was read a moment ago).  HBM traffic per element: 2 B read + 0.5 B written + 8/G B of
// (scale, zero) pairs.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

constexpr int kUnroll = 2;

template <typename IN, bool SEPARATE_SUMMARY, int HOLD, int BITS, bool MB>
__global__ void __launch_bounds__(kBlock) quantize_append_tokens_kernel(const QuantArgs a) {
    constexpr int EB = elem_bytes<IN>::value;
    constexpr uint32_t CW = BITS;  // bytes of packed codes per lane and row (8 channels)
    const int H = a.n_kv_heads, d = a.head_dim, G = a.group_tokens;
    const int h = blockIdx.x;
    const int kv = blockIdx.y & 1;
    const int li = blockIdx.y >> 1;
    const int f = blockIdx.z;
    const int l = a.layer0 + li;
    const int64_t t = (int64_t)a.first_group + f;

    const int lpr = d >> 3;
    const int rpp = kBlock / lpr;
    const int tid = threadIdx.x;
    const int row0 = tid / lpr;
    const int slot = tid - row0 * lpr;
    const bool active = row0 < rpp;

    const int64_t in_off = f * a.stride_frame + li * a.stride_layer + h * a.stride_head;
    const char* src = static_cast<const char*>(kv ? a.v : a.k) + in_off * EB;
    const int64_t tile = (((int64_t)l * 2 + kv) * a.capacity_groups + t) * H + h;
    char* codes_t = reinterpret_cast<char*>(a.codes + tile * ((int64_t)G * d * BITS / 8));
    typedef typename MetaPair<MB>::type meta_pair;  // two float32, or two bfloat16 in one word
    meta_pair* meta_t = reinterpret_cast<meta_pair*>(a.meta) + tile * (int64_t)d;  // [d] (scale, zero)
    const uint32_t in_row_bytes = (uint32_t)a.stride_token * EB;
    const uint32_t in_lane = (uint32_t)row0 * in_row_bytes + (uint32_t)slot * 8u * EB;
    const uint32_t code_lane = ((uint32_t)row0 * lpr + slot) * CW;

    __shared__ double shared_buf[kBlock * 8];        // 16 KB: (min, max) per row slot, then key sums
    extern __shared__ f32x2 fin[];                    // [d] (zero point, 1/scale) per channel
    f32x2* mm = reinterpret_cast<f32x2*>(shared_buf);

    const bool do_sum = (kv == 0);
    double acc[8];
    float mn[8], mx[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        acc[i] = 0.0;
        mn[i] = __builtin_inff();
        mx[i] = -__builtin_inff();
    }

    // ---- sweep 1: per-channel min / max (and the key sums) down the token rows
    const int step = kUnroll * rpp;
    constexpr int kHeld = HOLD > 0 ? HOLD : 1;
    Raw8<IN> held[kHeld];
    auto reduce_row = [&](const Raw8<IN>& raw) {
        float x[8];
        widen(raw, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            mn[i] = fminf(mn[i], x[i]);
            mx[i] = fmaxf(mx[i], x[i]);
        }
        if (!SEPARATE_SUMMARY && do_sum) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += (double)x[i];
        }
    };
    if (HOLD > 0) {
#pragma unroll
        for (int u = 0; u < kHeld; ++u) {
            zero_raw(held[u]);
            if (active && u * rpp + row0 < G) load_raw(src + (in_lane + (uint32_t)(u * rpp) * in_row_bytes), held[u]);
        }
#pragma unroll
        for (int u = 0; u < kHeld; ++u)
            if (active && u * rpp + row0 < G) reduce_row(held[u]);
    } else {
        for (int r0 = 0; active && r0 + row0 < G; r0 += step) {
            Raw8<IN> raw[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (r0 + u * rpp + row0 < G)
                    load_raw(src + (in_lane + (uint32_t)(r0 + u * rpp) * in_row_bytes), raw[u]);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                if (r0 + u * rpp + row0 < G) reduce_row(raw[u]);
        }
    }
    if (active) {
#pragma unroll
        for (int i = 0; i < 8; ++i) mm[row0 * d + i * lpr + slot] = f32x2{mn[i], mx[i]};  // position, not channel
    }
    __syncthreads();
    // ---- one thread per channel: Eq. 9 over the whole token axis.  The LDS arrays are indexed
    // by position q = i * lpr + slot (channel slot * 8 + i), so that the lanes of a wave touch
    // consecutive words instead of words 64 bytes apart (16-way bank conflicts otherwise).
    for (int q = tid; q < d; q += kBlock) {
        float cmn = mm[q][0], cmx = mm[q][1];
        for (int r = 1; r < rpp; ++r) {
            cmn = fminf(cmn, mm[r * d + q][0]);
            cmx = fmaxf(cmx, mm[r * d + q][1]);
        }
        cmn = cmn + 0.0f;  // never store -0 as a zero point
        float s = div_levels_exact<BITS>(__fsub_rn(cmx, cmn));
        if (!(s >= 1.17549435e-38f)) s = 0.0f;
        meta_pair stored;
        if constexpr (MB) stored = round_pair_bf16(s, cmn);  // the codes follow the rounded pair
        else stored = f32x2{s, cmn};
        const float inv = s >= 1.17549435e-38f ? rcp_scale<BITS>(s) : 0.0f;
        const int c = (q % lpr) * 8 + q / lpr;
        meta_t[c] = stored;
        fin[q] = f32x2{cmn, inv};
    }
    __syncthreads();

    // ---- sweep 2: quantize and pack
    if (active) {
        float zm[8], zi[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const f32x2 v = fin[i * lpr + slot];
            zm[i] = v[0];
            zi[i] = v[1];
        }
        auto quantize_row = [&](const Raw8<IN>& raw, int rb) {
            float x[8], tq[8];
            widen(raw, x);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                tq[i] = __builtin_fmaf(__fsub_rn(x[i], zm[i]), zi[i], 8388608.0f);
                if constexpr (MB) tq[i] = clamp_code<BITS>(tq[i]);  // m may lie above the minimum
            }
            store_codes8<BITS>(codes_t + (code_lane + (uint32_t)rb * lpr * CW), tq);
        };
        if (HOLD > 0) {
#pragma unroll
            for (int u = 0; u < kHeld; ++u)
                if (u * rpp + row0 < G) quantize_row(held[u], u * rpp);
        } else {
            for (int r0 = 0; r0 + row0 < G; r0 += step) {
                Raw8<IN> raw[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
                    if (r0 + u * rpp + row0 < G)
                        load_raw(src + (in_lane + (uint32_t)(r0 + u * rpp) * in_row_bytes), raw[u]);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
                    if (r0 + u * rpp + row0 < G) quantize_row(raw[u], r0 + u * rpp);
            }
        }
    }
    if (!do_sum) return;  // uniform per workgroup

    if (SEPARATE_SUMMARY) {
        const char* ssrc = static_cast<const char*>(a.ksum) + in_off * EB;
        for (int row = row0; active && row < G; row += rpp) {
            float x[8];
            load8(ssrc + ((int64_t)row * a.stride_token + slot * 8) * EB, IN{}, x);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] += (double)x[i];
        }
    }
    __syncthreads();  // the (min, max) use of shared_buf is over
    if (active) {
#pragma unroll
        for (int i = 0; i < 8; ++i) shared_buf[row0 * d + i * lpr + slot] = acc[i];
    }
    __syncthreads();
    float* key = a.keys + (((int64_t)l * a.capacity_groups + t) * H + h) * d;
    for (int q = tid; q < d; q += kBlock) {
        double sum = 0.0;
        for (int r = 0; r < rpp; ++r) sum += shared_buf[r * d + q];
        key[(q % lpr) * 8 + q / lpr] = (float)(sum / (double)G);
    }
}

template <typename IN, int HOLD, int BITS, bool MB>
hipError_t launch_m(const QuantArgs& a, hipStream_t s) {
    const dim3 grid(a.n_kv_heads, 2 * a.n_layers, a.n_frames);
    const size_t lds = (size_t)a.head_dim * sizeof(f32x2);
    if (a.ksum != a.k)
        quantize_append_tokens_kernel<IN, true, HOLD, BITS, MB><<<grid, dim3(kBlock), lds, s>>>(a);
    else
        quantize_append_tokens_kernel<IN, false, HOLD, BITS, MB><<<grid, dim3(kBlock), lds, s>>>(a);
    return hipGetLastError();
}

template <typename IN, int HOLD>
hipError_t launch_h(const QuantArgs& a, hipStream_t s) {
    if (a.meta_bf16) return a.bits == 2 ? launch_m<IN, HOLD, 2, true>(a, s) : launch_m<IN, HOLD, 4, true>(a, s);
    return a.bits == 2 ? launch_m<IN, HOLD, 2, false>(a, s) : launch_m<IN, HOLD, 4, false>(a, s);
}

template <typename IN>
hipError_t launch_t(const QuantArgs& a, hipStream_t s) {
    if (a.n_frames == 0 || a.n_layers == 0) return hipSuccess;
    const int rpp = kBlock / (a.head_dim / 8);
    const int trips = (a.group_tokens + rpp - 1) / rpp;  // rows per lane
    if (trips <= 4) return launch_h<IN, 4>(a, s);
    if (trips <= 8) return launch_h<IN, 8>(a, s);
    if constexpr (sizeof(Raw8<IN>) <= 16) {  // 13 float32 rows would not fit the register budget
        if (trips <= 13) return launch_h<IN, 13>(a, s);
    }
    return launch_h<IN, 0>(a, s);
}

}  // namespace

hipError_t launch_quantize_append_tokens(const QuantArgs& a, int in_dtype, hipStream_t s) {
    switch (in_dtype) {
        case TOM_F32: return launch_t<In_f32>(a, s);
        case TOM_BF16: return launch_t<In_bf16>(a, s);
        case TOM_F16: return launch_t<In_f16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace oqm

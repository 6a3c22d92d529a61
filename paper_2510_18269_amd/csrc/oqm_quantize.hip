// Store step of Online Quantized Memory on gfx950: 4-bit (or 2-bit) quantization
// of the frame-group tiles of K and V (paper Sec. 3.4, Eq. 8 and Eq. 9), code
// packing, and the summary key (mean of the un-quantized keys over the G tokens
// of the group) in the same pass over K.
//
// Work decomposition.  A lane owns 8 consecutive channels of one token row: one
// 128-bit load in, one 32-bit word of packed nibbles out, so every load and
// store instruction of a wave covers one contiguous span (1 KB in, 256 B out).
// A quant-group of gs channels lives in gs/8 adjacent lanes; its min and max are
// all-reduced with DPP lane swaps; the first lane of the group stores its
// (scale, zero) pair (8 bytes).
//
// A K tile (one (frame, layer, head) block of G x d keys) is walked by ONE
// workgroup of 256 threads, a few token rows per trip, because the summary key
// needs the column sums over all G rows and a reduction across workgroups costs
// more than it saves (measured: float64 atomics or written-through partials plus an
// arrival counter add 10 to 40 % to the kernel).  A V tile has no such coupling:
// it is cut into equal chunks of at most one trip (7 x 28 rows at 196 x 128) and
// every chunk is a workgroup of its own (two rows per lane in flight; one row per
// lane is 40 % slower, three to five rows 5 % slower).  The 1-D grid holds all V chunks first, in the order the
// tiles lie in memory, then all K tiles.  Measured on MI355X at 28 layers x 32
// frames x 196 x 128 (474 MB per launch): whole tiles for K and V 100 us; V chunks
// then K tiles 93 us; K tiles then V chunks 94 us; chunks and tiles interleaved in
// blocks of 16 to 896 tiles 96 to 99 us (two address streams at once are slower
// than one after the other); a role pattern with period 8 in the workgroup id
// (e.g. one K tile after every 7 V chunks) puts all K tiles on one of the eight
// XCDs, which take workgroups round-robin: 204 us.  Chunked workgroups stream
// faster because the workgroups in flight then cover one dense, moving address
// window instead of thousands of tiles at once; the same kernel with every tile
// chunked and no summary key takes 86 us, an arithmetic-free linear stream of the
// same byte mix 80 us.
//
// The kernel moves 2.64 B per element (bf16 in, gs 64).  At HBM speed that leaves
// room for only about a dozen instructions per element on the plain fp32 vector
// pipe (64 lanes per CU and clock), so the arithmetic is arranged to need few:
//   widen 1, min/max 1, subtract 1, fused scale-and-round 1, pack 1, plus two
//   float64 instructions per element of K for the summary key,
// and the register footprint is kept small: measured, more resident waves help
// this kernel more than deeper software prefetch does.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

// Two forms of the kernel.
// Streaming (more than kShallowTiles tiles): 256 threads, two token rows per lane and trip.  The
// small register footprint keeps eight workgroups on a compute unit, and V tiles are cut into
// one-trip chunks (see above).
// Shallow (a launch of at most three tiles per compute unit, e.g. one frame of a live stream:
// 224 tiles at 28 layers x 4 heads): such a launch is bound by the dependent memory round trips
// and the serial arithmetic of the one workgroup that owns a tile, not by bandwidth, so a tile
// gets 1024 threads with four rows per lane in flight (the whole 196 x 128 tile in one trip).
// Measured kernel time, shallow against streaming form: 224 tiles 6.4 / 9.8 us (7.7 us with 256
// threads and 13 rows per lane), 448 tiles 9.6 / 11.3 us, 672 tiles 13.6 / 15.2 us, 896 tiles
// 17.1 / 17.5 us, 1344 tiles 23.6 / 21.6 us.
constexpr int kUnrollStream = 2;
constexpr int kUnrollShallow = 4;
constexpr int kShallowThreads = 1024;
constexpr int64_t kShallowTiles = 768;  // three per compute unit

// a.v_chunks: workgroups per V tile, a.v_rows_per_chunk token rows each (at most one trip of
// kUnroll * rows-per-pass rows); 1 = whole tile.
template <typename IN, int LPG, bool SEPARATE_SUMMARY, int BITS, bool MB, int kUnroll, int NT>
__global__ void __launch_bounds__(NT) quantize_append_kernel(const QuantArgs a) {
    constexpr int EB = elem_bytes<IN>::value;
    constexpr uint32_t CW = BITS;  // bytes of packed codes per lane and row (8 channels)
    const int H = a.n_kv_heads, d = a.head_dim, G = a.group_tokens;

    const int lpr = a.lanes_per_row;  // d / 8
    const int rpp = a.rows_per_pass;  // token rows per pass of the workgroup: 256 / lpr
    const int step = kUnroll * rpp;   // token rows per trip
    const int v_chunks = a.v_chunks;

    // Workgroup id -> role.  [0, items * v_chunks): chunk (id % v_chunks) of the V tile of item
    // id / v_chunks; after those: the K tile of item id - items * v_chunks.  Items run over
    // (frame, layer, head), head fastest, which is the order of a contiguous input tensor.
    const int items = a.n_frames * a.n_layers * H;
    int item = blockIdx.x, kv = 1, row_begin = 0, row_end = G;
    if (item >= items * v_chunks) {
        kv = 0;
        item -= items * v_chunks;
    } else if (v_chunks > 1) {
        const int tile_item = div_by(item, v_chunks, a.inv_v_chunks);
        row_begin = (item - tile_item * v_chunks) * a.v_rows_per_chunk;
        row_end = min(G, row_begin + a.v_rows_per_chunk);
        item = tile_item;
    }
    const int fl = div_by(item, H, a.inv_heads);
    const int h = item - fl * H;
    const int f = div_by(fl, a.n_layers, a.inv_layers);
    const int li = fl - f * a.n_layers;
    const int l = a.layer0 + li;
    const int64_t t = (int64_t)a.first_group + f;

    const int tid = threadIdx.x;
    const int row0 = div_by(tid, lpr, a.inv_lanes_per_row);
    const int slot = tid - row0 * lpr;
    const bool active = row0 < rpp;
    const int ng = lpr / LPG;       // quant-groups per token row
    const int wave_row0 = __builtin_amdgcn_readfirstlane(row0);  // lowest row of this wave

    // Tile bases are uniform per workgroup; per-lane offsets inside a tile fit 32 bits
    // (checked on the host), which keeps the address arithmetic per row to one add.
    const int64_t in_off = f * a.stride_frame + li * a.stride_layer + h * a.stride_head;
    const char* src = static_cast<const char*>(kv ? a.v : a.k) + in_off * EB;
    const int64_t tile = (((int64_t)l * 2 + kv) * a.capacity_groups + t) * H + h;
    char* codes_t = reinterpret_cast<char*>(a.codes + tile * ((int64_t)G * d * BITS / 8));
    typedef typename MetaPair<MB>::type meta_pair;  // two float32, or two bfloat16 in one word
    meta_pair* meta_t = reinterpret_cast<meta_pair*>(a.meta) + tile * ((int64_t)G * ng);
    const uint32_t in_row_bytes = (uint32_t)a.stride_token * EB;
    const uint32_t in_lane = (uint32_t)row0 * in_row_bytes + (uint32_t)slot * 8u * EB;
    const uint32_t code_lane = ((uint32_t)row0 * lpr + slot) * CW;
    const int meta_lane = row0 * ng + slot / LPG;
    const bool meta_writer = (slot & (LPG - 1)) == 0;

    __shared__ double shared_buf[NT * 8];  // 16 KB at 256 threads, key reduction

    const bool do_sum = (kv == 0);
    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0;

    auto fetch = [&](Raw8<IN> (&dst)[kUnroll], int r0) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rb = r0 + u * rpp;
            if (active && rb + row0 < row_end)
                load_raw(src + (in_lane + (uint32_t)rb * in_row_bytes), dst[u]);
        }
    };
    auto process = [&](const Raw8<IN> (&buf)[kUnroll], int r0) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rb = r0 + u * rpp;
            if (rb + wave_row0 >= row_end) break;  // nothing left for this wave (uniform)
            const bool ok = active && rb + row0 < row_end;
            float x[8];
            widen(buf[u], x);  // lanes past the tile compute on stale rows; their results are dropped
            // Eq. 9: m = min, s = (max - min) / 15 over the quant-group.  All lanes of a
            // quant-group share one row, so a live lane only ever swaps with live lanes.
            float mn = x[0], mx = x[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) {
                mn = fminf(mn, x[i]);
                mx = fmaxf(mx, x[i]);
            }
            group_minmax<LPG>(mn, mx);
            mn = mn + 0.0f;  // never store -0 as a zero point
            float s = div_levels_exact<BITS>(__fsub_rn(mx, mn));
            if (!(s >= 1.17549435e-38f)) s = 0.0f;  // flat or sub-normal range: all codes 0
            meta_pair stored;
            if constexpr (MB) stored = round_pair_bf16(s, mn);  // the codes follow the rounded pair
            const float inv = s >= 1.17549435e-38f ? rcp_scale<BITS>(s) : 0.0f;
            if constexpr (!MB) stored = f32x2{s, mn};
            float tq[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                tq[i] = __builtin_fmaf(__fsub_rn(x[i], mn), inv, 8388608.0f);
                if constexpr (MB) tq[i] = clamp_code<BITS>(tq[i]);  // m may lie above the minimum
            }
            if (ok) {
                store_codes8<BITS>(codes_t + (code_lane + (uint32_t)rb * lpr * CW), tq);
                if (meta_writer) meta_t[meta_lane + rb * ng] = stored;
                if (!SEPARATE_SUMMARY && do_sum) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[i] += (double)x[i];
                }
            }
        }
    };

    Raw8<IN> buf[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) zero_raw(buf[u]);  // defined contents for rows never loaded
    for (int r0 = row_begin; r0 < row_end; r0 += step) {
        if (r0 + wave_row0 >= row_end) break;  // nothing left for this wave (uniform)
        fetch(buf, r0);
        process(buf, r0);
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
    if (active) {
#pragma unroll
        for (int i = 0; i < 8; ++i) shared_buf[row0 * d + i * lpr + slot] = acc[i];
    }
    __syncthreads();
    float* key = a.keys + (((int64_t)l * a.capacity_groups + t) * H + h) * d;
    // position q = i * lpr + slot holds channel slot * 8 + i: the lanes of a wave write
    // consecutive doubles (channel order would put them 64 bytes apart: 16-way bank conflicts)
    for (int q = tid; q < d; q += NT) {
        double sum = 0.0;
        for (int r = 0; r < rpp; ++r) sum += shared_buf[r * d + q];
        key[(q % lpr) * 8 + q / lpr] = (float)(sum / (double)G);
    }
}

template <typename IN, int LPG, int BITS, bool MB>
hipError_t launch_b(const QuantArgs& args, hipStream_t s) {
    QuantArgs a = args;
    const int64_t items = (int64_t)a.n_kv_heads * a.n_layers * a.n_frames;
    const bool shallow = 2 * items <= kShallowTiles && a.ksum == a.k;
    // V tiles: one workgroup per trip of the streaming form; whole tiles in the shallow form
    const int rows_per_trip = kUnrollStream * (kBlock / (a.head_dim / 8));
    const int v_chunks = shallow ? 1 : (a.group_tokens + rows_per_trip - 1) / rows_per_trip;
    const int64_t blocks = items * (v_chunks + 1);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;  // the API layer has refused this already
    a.v_chunks = v_chunks;
    a.v_rows_per_chunk = (a.group_tokens + v_chunks - 1) / v_chunks;  // equal chunks, each within one trip
    a.lanes_per_row = (uint32_t)a.head_dim / 8u;
    const int threads = shallow ? kShallowThreads : kBlock;
    a.rows_per_pass = (uint32_t)threads / a.lanes_per_row;
    a.inv_lanes_per_row = reciprocal_u32(a.lanes_per_row);
    a.inv_heads = reciprocal_u32((uint32_t)a.n_kv_heads);
    a.inv_layers = reciprocal_u32((uint32_t)a.n_layers);
    a.inv_v_chunks = reciprocal_u32((uint32_t)v_chunks);
    const dim3 grid((unsigned)blocks);
    if (a.ksum != a.k)
        quantize_append_kernel<IN, LPG, true, BITS, MB, kUnrollStream, kBlock><<<grid, dim3(kBlock), 0, s>>>(a);
    else if (shallow)
        quantize_append_kernel<IN, LPG, false, BITS, MB, kUnrollShallow, kShallowThreads>
            <<<grid, dim3(kShallowThreads), 0, s>>>(a);
    else
        quantize_append_kernel<IN, LPG, false, BITS, MB, kUnrollStream, kBlock><<<grid, dim3(kBlock), 0, s>>>(a);
    return hipGetLastError();
}

template <typename IN, int LPG>
hipError_t launch_t(const QuantArgs& a, hipStream_t s) {
    if (a.n_frames == 0 || a.n_layers == 0) return hipSuccess;
    if (a.meta_bf16) return a.bits == 2 ? launch_b<IN, LPG, 2, true>(a, s) : launch_b<IN, LPG, 4, true>(a, s);
    return a.bits == 2 ? launch_b<IN, LPG, 2, false>(a, s) : launch_b<IN, LPG, 4, false>(a, s);
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
    if (a.qaxis == TOM_QAXIS_TOKENS) return launch_quantize_append_tokens(a, in_dtype, s);
    switch (in_dtype) {
        case TOM_F32: return launch_lpg<In_f32>(a, s);
        case TOM_BF16: return launch_lpg<In_bf16>(a, s);
        case TOM_F16: return launch_lpg<In_f16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace oqm

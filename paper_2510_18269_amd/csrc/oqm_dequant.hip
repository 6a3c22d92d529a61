// Reconstruction of the selected frame-groups into the bounded active KV buffer
// (paper Sec. 3.4, Eq. 11 and Eq. 13; supplement "Cache reconstruction for decoding").
//
// Grid (rank * chunks + chunk, 2*head + K|V, layer): a workgroup of 256 threads owns
// up to three row passes (48 token rows at head_dim 128) of one head tile of one
// selected group; consecutive workgroups write consecutive row blocks of the active
// buffer.  It reads the group index from device memory (the index array never visits
// the host), streams its rows' packed nibbles and (scale, zero) pairs, and writes them
// to token rows [rank*G, (rank+1)*G) of the layer's active buffer.  A lane turns one
// 32-bit word of codes (8 channels) into one 128-bit non-temporal store, so each store
// instruction of a wave writes 1 KB of contiguous bf16.  HBM-bound: 0.5 + 8/gs bytes
// read and 2 bytes written per element.
//
// Rows per workgroup, measured at 28 layers x 64 groups x 196 x 128 (944 MB, random
// groups): whole tile (13 passes, all loads first) 171 us; 7 / 6 chunks 178 / 176 us;
// 5 chunks of 40 rows 167 us; 3 chunks of 66 rows 168 us; 2 chunks 173 us; chunks of one
// pass 216 us.  Chunks of unequal size whose count divides 8 are slow (3 x 64 + 4 rows:
// 193 us): workgroup ids go round-robin over the eight XCDs, so all the short chunks land
// on the same two.  With contiguous groups instead of random ones the same kernel takes
// 152 us: what is left to a dense stream is the DRAM row locality of 12.5 KB pieces.
#include <type_traits>

#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

// kUnroll: rows per lane whose loads are issued before any is converted (the host cuts the tile
// into chunks that one trip covers).
template <typename OUT, int kUnroll, bool TOKEN_AXIS, int BITS, bool MB>
__global__ void __launch_bounds__(kBlock) dequant_gather_kernel(const DequantArgs a, const int lpg) {
    constexpr int EB = elem_bytes<OUT>::value;
    constexpr uint32_t CW = BITS;          // bytes of packed codes per lane and row (8 channels)
    constexpr uint32_t CMASK = (1u << BITS) - 1u;
    const int H = a.n_kv_heads, d = a.head_dim, G = a.group_tokens;
    const int r = a.chunks > 1 ? (int)div_by(blockIdx.x, a.chunks, a.inv_chunks) : (int)blockIdx.x;
    const int row_begin = ((int)blockIdx.x - r * a.chunks) * a.rows_per_chunk;
    const int row_end = min(G, row_begin + a.rows_per_chunk);
    const int kv = blockIdx.y & 1;
    const int h = blockIdx.y >> 1;
    const int li = blockIdx.z;

    const int t = a.idx[(int64_t)li * a.k + r];
    if ((unsigned)t >= (unsigned)a.n_groups) return;  // not a stored group: leave the rows alone

    const int lpr = d >> 3;
    const int rpp = kBlock / lpr;
    const int tid = threadIdx.x;
    const int row0 = tid / lpr;
    const int slot = tid - row0 * lpr;
    if (row0 >= rpp) return;
    const int ng = TOKEN_AXIS ? 0 : lpr / lpg;

    const int64_t tile = (((int64_t)(a.layer0 + li) * 2 + kv) * a.capacity_groups + t) * H + h;
    const char* codes_t = reinterpret_cast<const char*>(a.codes + tile * ((int64_t)G * d * BITS / 8));
    // token axis (Eq. 9): one pair per channel, d pairs per tile; else G * d/gs pairs
    typedef typename MetaPair<MB>::type meta_pair;  // two float32, or two bfloat16 in one word
    const meta_pair* meta_t =
        reinterpret_cast<const meta_pair*>(a.meta) + tile * (TOKEN_AXIS ? (int64_t)d : (int64_t)G * ng);
    f32x2 ch[8];  // token axis: the pairs of this lane's 8 channels, loaded once
    if (TOKEN_AXIS) {
#pragma unroll
        for (int i = 0; i < 8; ++i) ch[i] = widen_pair(meta_t[slot * 8 + i]);
    }
    const int64_t head_rows = (int64_t)a.prefix_rows + (int64_t)a.k * G;  // rows per head buffer
    char* out = static_cast<char*>(kv ? a.v_out : a.k_out) +
                (((int64_t)li * H + h) * head_rows + a.prefix_rows + (int64_t)r * G) * (int64_t)d * EB;
    // offsets inside one tile fit 32 bits (G * d * 4 < 2^31 is checked on the host)
    const uint32_t code_lane = ((uint32_t)row0 * lpr + slot) * CW;
    const int meta_lane = TOKEN_AXIS ? 0 : row0 * ng + slot / lpg;
    const uint32_t out_lane = ((uint32_t)row0 * d + slot * 8u) * EB;

    for (int r0 = row_begin; r0 + row0 < row_end; r0 += kUnroll * rpp) {
        uint32_t w[kUnroll];
        meta_pair sm[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rb = r0 + u * rpp;
            w[u] = 0u;
            sm[u] = meta_pair{};
            if (rb + row0 < row_end) {
                w[u] = load_codes8<BITS>(codes_t + (code_lane + (uint32_t)rb * lpr * CW));
                if (!TOKEN_AXIS) sm[u] = meta_t[meta_lane + rb * ng];
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int rb = r0 + u * rpp;
            if (rb + row0 < row_end) {
                float x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float c = (float)((w[u] >> (BITS * i)) & CMASK);
                    const f32x2 p = TOKEN_AXIS ? ch[i] : widen_pair(sm[u]);
                    x[i] = __builtin_fmaf(c, p[0], p[1]);  // Eq. 11, rounded once to float32
                }
                store8(out + (out_lane + (uint32_t)rb * d * EB), OUT{}, x);
            }
        }
    }
}

// System-token prefix (the part of the paper's dual-structure memory that stays in 16 bits):
// rows [0, prefix_rows) of every head's active buffer are copied from
// sys [n_layers][H_k][prefix_rows][d].  grid (chunks, H_k * n_layers, 2), 16 bytes per lane.
__global__ void __launch_bounds__(kBlock) prefix_copy_kernel(const DequantArgs a, const char* sys_k,
                                                             const char* sys_v, const int64_t head_bytes,
                                                             const int64_t prefix_bytes) {
    const int64_t off = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 16;
    if (off >= prefix_bytes) return;
    const char* src = (blockIdx.z ? sys_v : sys_k) + (int64_t)blockIdx.y * prefix_bytes + off;
    char* dst = static_cast<char*>(blockIdx.z ? a.v_out : a.k_out) + (int64_t)blockIdx.y * head_bytes + off;
    *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(src);
}

template <typename OUT>
hipError_t launch_t(const DequantArgs& args, hipStream_t s) {
    if (args.n_layers == 0 || args.k_eff == 0) return hipSuccess;
    DequantArgs a = args;
    const int rpp = kBlock / (a.head_dim / 8);
    const int passes = (a.group_tokens + rpp - 1) / rpp;  // row passes per tile
    // up to four passes: one workgroup per tile; more: equal chunks of at most three passes
    a.chunks = passes <= 4 ? 1 : (passes + 2) / 3;
    a.rows_per_chunk = (a.group_tokens + a.chunks - 1) / a.chunks;
    a.inv_chunks = reciprocal_u32((uint32_t)a.chunks);
    if ((int64_t)a.k_eff * a.chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(a.k_eff * a.chunks), 2 * a.n_kv_heads, a.n_layers), block(kBlock);
    const int lpg = a.qgroup / 8;  // unused for the token axis
    const bool tok = a.qaxis == TOM_QAXIS_TOKENS;
    auto go = [&](auto unroll, auto bits, auto mb) {
        constexpr int U = decltype(unroll)::value, B = decltype(bits)::value;
        constexpr bool M = decltype(mb)::value;
        if (tok) dequant_gather_kernel<OUT, U, true, B, M><<<grid, block, 0, s>>>(a, 1);
        else dequant_gather_kernel<OUT, U, false, B, M><<<grid, block, 0, s>>>(a, lpg);
    };
    auto with_meta = [&](auto unroll, auto bits) {
        if (a.meta_bf16) go(unroll, bits, std::true_type{});
        else go(unroll, bits, std::false_type{});
    };
    auto with_bits = [&](auto unroll) {
        if (a.bits == 2) with_meta(unroll, std::integral_constant<int, 2>{});
        else with_meta(unroll, std::integral_constant<int, 4>{});
    };
    if (passes <= 4) with_bits(std::integral_constant<int, 4>{});
    else with_bits(std::integral_constant<int, 3>{});
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_copy(const DequantArgs& a, const void* sys_k, const void* sys_v, int out_dtype,
                              hipStream_t s) {
    const int64_t eb = out_dtype == TOM_F32 ? 4 : 2;
    const int64_t prefix_bytes = (int64_t)a.prefix_rows * a.head_dim * eb;  // multiple of 16: d % 8 == 0
    const int64_t head_bytes = ((int64_t)a.prefix_rows + (int64_t)a.k * a.group_tokens) * a.head_dim * eb;
    if (prefix_bytes == 0 || a.n_layers == 0) return hipSuccess;
    const int64_t chunks = (prefix_bytes / 16 + kBlock - 1) / kBlock;
    if (chunks > 0x7fffffffLL || (int64_t)a.n_kv_heads * a.n_layers > 65535) return hipErrorInvalidValue;
    prefix_copy_kernel<<<dim3((unsigned)chunks, a.n_kv_heads * a.n_layers, 2), dim3(kBlock), 0, s>>>(
        a, static_cast<const char*>(sys_k), static_cast<const char*>(sys_v), head_bytes, prefix_bytes);
    return hipGetLastError();
}

hipError_t launch_dequant_gather(const DequantArgs& a, int out_dtype, hipStream_t s) {
    if (a.k_eff == 0) return hipSuccess;
    switch (out_dtype) {
        case TOM_F32: return launch_t<In_f32>(a, s);
        case TOM_BF16: return launch_t<In_bf16>(a, s);
        case TOM_F16: return launch_t<In_f16>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace oqm

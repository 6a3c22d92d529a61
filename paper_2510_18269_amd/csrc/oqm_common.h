// Internal declarations shared by the host dispatch and the gfx950 kernels.
// Not part of the ABI (that is include/tom_oqm.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

// The library is built with hidden visibility: only the functions of the ABI header are
// exported from the shared object.
#pragma GCC visibility push(default)
#include "tom_oqm.h"
#pragma GCC visibility pop

struct tom_oqm {
    tom_oqm_config_t cfg;
    uint8_t* codes = nullptr;
    void* meta = nullptr;   // (scale, zero) pairs: float32 x 2, or bfloat16 x 2 (cfg.meta_dtype)
    float* keys = nullptr;
    int32_t n_groups = 0;
    bool bound = false;
};

namespace oqm {

// Sets the thread-local error string returned by tom_last_error().
tom_status_t fail(tom_status_t st, const char* fmt, ...);

constexpr int kBlock = 256;  // threads per workgroup of the streaming kernels (4 waves)

// ---- element offsets of the storage arrays -------------------------------
struct Layout {
    int64_t tile_code_bytes;  // G * d * bits / 8
    int64_t tile_meta;        // (scale, zero) pairs per head tile (2 floats each)
    int64_t tile_elems;       // G * d
};

inline Layout layout_of(const tom_oqm_config_t& c) {
    Layout l;
    l.tile_elems = (int64_t)c.group_tokens * c.head_dim;
    l.tile_code_bytes = l.tile_elems * c.bits / 8;
    l.tile_meta = c.qaxis == TOM_QAXIS_HEAD_DIM ? (int64_t)c.group_tokens * (c.head_dim / c.qgroup)
                                                : (int64_t)c.head_dim;
    return l;
}

// ---- kernel argument blocks (plain data, passed by value) -----------------
struct QuantArgs {
    const void* k;
    const void* v;
    const void* ksum;  // source of the summary key (== k unless the caller gave another)
    int64_t stride_frame, stride_layer, stride_head, stride_token;  // elements
    uint8_t* codes;
    void* meta;   // [..][G][d/gs][2]: (scale, zero) pairs, float32 or bfloat16
    float* keys;
    int32_t n_kv_heads, head_dim, group_tokens, qgroup, capacity_groups;
    int32_t layer0, n_layers, n_frames, first_group;
    int32_t qaxis;
    int32_t bits;  // 4 or 2
    int32_t meta_bf16;  // (scale, zero) stored as bfloat16 pairs
    // Filled in by the head_dim-axis launcher: its grid decomposition and the reciprocals
    // (floor(2^32 / d)) that let the kernel divide by these run-time constants in three
    // instructions instead of a full integer division per workgroup and lane.
    int32_t v_chunks;  // workgroups per V tile
    int32_t v_rows_per_chunk;  // token rows each of them takes
    uint32_t lanes_per_row, rows_per_pass;
    uint32_t inv_lanes_per_row, inv_heads, inv_layers, inv_v_chunks;
};

// floor(2^32 / d) for d >= 1 (saturated for d == 1): the constant of oqm::div_by in the device header.
inline uint32_t reciprocal_u32(uint32_t d) { return d <= 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / d); }

struct DequantArgs {
    const uint8_t* codes;
    const void* meta;
    const int32_t* idx;  // [n_layers][k]
    void* k_out;
    void* v_out;
    int32_t n_kv_heads, head_dim, group_tokens, qgroup, capacity_groups;
    int32_t layer0, n_layers, k, k_eff, n_groups;
    int32_t qaxis;
    int32_t bits;         // 4 or 2
    int32_t meta_bf16;    // (scale, zero) stored as bfloat16 pairs
    int32_t prefix_rows;  // rows of each head's active buffer that precede the gathered groups
    // Filled in by the launcher: workgroups per tile, the token rows each takes, and the
    // reciprocal floor(2^32 / chunks) for oqm::div_by.
    int32_t chunks, rows_per_chunk;
    uint32_t inv_chunks;
};

struct ScoreArgs {
    const float* keys;  // [L][T_cap][H_k*d]
    const void* q;      // [n_layers][H_q][T_q][d]
    float* scores;      // [n_layers][score_stride]
    float* token_scores;
    double* ws_qbar;    // [n_layers][H_k*d]
    double* ws_qnorm2;  // [n_layers][H_k] partial squared norms of q-bar
    double* ws_qtok;    // [n_layers][T_q][H_k*d] (TOKEN_GEMM only)
    int64_t score_stride;
    int32_t n_kv_heads, n_q_heads, head_dim, capacity_groups;
    int32_t layer0, n_layers, t_q, n_groups, sim, q_dtype;
    // Filled in by the launcher of the per-token contraction: its unit decomposition.
    int32_t gemm_units, gemm_units_per_xcd, gemm_tiles_per_layer;
    uint32_t inv_gemm_tiles_per_layer;
};

// ---- launchers (each validates nothing: the API layer has done that) ------
hipError_t launch_quantize_append(const QuantArgs& a, int in_dtype, hipStream_t s);
hipError_t launch_quantize_append_tokens(const QuantArgs& a, int in_dtype, hipStream_t s);
hipError_t launch_dequant_gather(const DequantArgs& a, int out_dtype, hipStream_t s);
hipError_t launch_prefix_copy(const DequantArgs& a, const void* sys_k, const void* sys_v, int out_dtype,
                              hipStream_t s);
hipError_t launch_query_fold(const ScoreArgs& a, bool want_tokens, hipStream_t s);
hipError_t launch_score_mean_query(const ScoreArgs& a, hipStream_t s);
hipError_t launch_score_token_gemm(const ScoreArgs& a, hipStream_t s);
hipError_t launch_topk(const float* scores, int64_t stride, int n_rows, int n_groups, int k,
                       int k_eff, int order, int32_t* idx, hipStream_t s);

constexpr int kTopkMaxSortedK = 4096;

}  // namespace oqm

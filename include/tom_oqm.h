/*
 * tom_oqm.h — C ABI of the MI355X (gfx950) Online Quantized Memory library.
 *
 * The library implements the storage / retrieval hot path of StreamingTOM's
 * Online Quantized Memory (paper Sec. 3.4 and the supplement's "Text-Video
 * Retrieval" paragraphs):
 *
 *   store        Q_4(X_t) = (uint4 codes, scale s_t, zero m_t, summary key)   Eq. 8, Eq. 9
 *   score        sim(q, summary key_i) over all stored frame-groups           Eq. 12
 *   select       TopK of the scores, indices kept in temporal order           Eq. 12, supplement
 *   reconstruct  depack(codes) * s + m for the selected groups only           Eq. 11, Eq. 13
 *
 * Vocabulary
 *   frame-group  the G tokens kept for one frame: the unit that is stored,
 *                scored and retrieved (the paper's "group").  Index t.
 *   quant-group  the elements that share one (scale, zero) pair.
 *   L, H_k, H_q, d   layers, KV heads, query heads, head_dim.
 *
 * Conventions
 *   - Every pointer named "device" is a HIP device pointer; everything else is
 *     host memory.  The library never allocates or frees device memory: the
 *     caller owns all buffers (storage, inputs, outputs, workspace) and must
 *     keep them alive until the work queued on the stream has finished.
 *   - Every call that takes a `hip_stream` only enqueues kernels on that
 *     hipStream_t (NULL = the default stream) and returns without
 *     synchronising.  Calls on one stream execute in order.
 *   - Arguments are validated on the host before anything is launched; a call
 *     that returns an error has queued nothing and changed no state.  Errors
 *     are returned as codes, never thrown.  tom_last_error() gives a
 *     thread-local description of the most recent failure.
 *   - Non-finite inputs give unspecified values (never out-of-bounds access).
 *
 * Device memory layout (all contiguous, row-major, element offsets):
 *   codes  [L][2 (0 = K, 1 = V)][T_cap][H_k][G][d * bits / 8]   uint8
 *          4-bit: channel 2j in the low nibble of byte j, channel 2j+1 in the high nibble
 *          2-bit: channel 4j + u in bits [2u, 2u + 2) of byte j
 *   meta   (scale, zero) pairs, scale first; float32 each, or with cfg.meta_dtype = TOM_BF16
 *          bfloat16 each (one 32-bit word per pair, scale in the low half)
 *          qaxis HEAD_DIM: [L][2][T_cap][H_k][G][d / gs][2]      float32
 *          qaxis TOKENS  : [L][2][T_cap][H_k][d][2]              float32
 *   keys   [L][T_cap][H_k][d]                                    float32 (summary keys)
 * One (layer, K|V, frame-group, head) tile is contiguous in every array, so a
 * tile is appended with full-width stores and retrieved with full-width loads.
 */
#ifndef TOM_OQM_H
#define TOM_OQM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tom_oqm tom_oqm_t; /* opaque; lives in host memory */

typedef enum {
    TOM_OK = 0,
    TOM_ERR_INVALID_ARG = 1, /* bad pointer, shape, range or enum value             */
    TOM_ERR_CAPACITY = 2,    /* append would exceed capacity_groups (no eviction)   */
    TOM_ERR_UNSUPPORTED = 3, /* valid request the kernels do not cover              */
    TOM_ERR_NOT_BOUND = 4,   /* tom_oqm_bind has not been called                    */
    TOM_ERR_HIP = 5          /* a HIP runtime call (launch) failed                  */
} tom_status_t;

typedef enum { TOM_F32 = 0, TOM_BF16 = 1, TOM_F16 = 2 } tom_dtype_t;

typedef enum {
    TOM_QAXIS_HEAD_DIM = 0, /* one (scale, zero) per token and gs consecutive channels  */
    TOM_QAXIS_TOKENS = 1    /* one (scale, zero) per channel over the G tokens (Eq. 9)   */
} tom_qaxis_t;

typedef enum { TOM_SIM_DOT = 0, TOM_SIM_COSINE = 1 } tom_sim_t;

typedef enum {
    TOM_ORDER_INDEX_ASC = 0, /* temporal order (the paper's "sorted order") */
    TOM_ORDER_SCORE_DESC = 1 /* best first; equal scores by lower index     */
} tom_order_t;

typedef enum {
    TOM_SCORE_AUTO = 0,  /* TOKEN_GEMM if per-token scores are requested, else MEAN_QUERY      */
    TOM_SCORE_MEAN_QUERY = 1, /* average the query tokens first, then one dot per group         */
    TOM_SCORE_TOKEN_GEMM = 2  /* dense [T_q x H_k*d] x [H_k*d x T] contraction on the matrix
                                 cores, then the mean over query tokens                        */
} tom_score_path_t;

typedef struct {
    int32_t n_layers;        /* L                                                        */
    int32_t n_kv_heads;      /* H_k; H_k * d <= 8192 (the score kernels stage the folded
                                query of a layer, H_k * d float64, in 64 KB of LDS)      */
    int32_t n_q_heads;       /* H_q, a multiple of H_k (GQA blocks of consecutive heads) */
    int32_t head_dim;        /* d, a multiple of 8, at most 2048                         */
    int32_t group_tokens;    /* G >= 1, tokens per frame-group; (G + 1024) * d * 4 must
                                stay below 2 GiB (offsets inside one head tile are 32-bit) */
    int32_t qgroup;          /* gs in {8, 16, 32, 64, 128}, divides d (HEAD_DIM axis);
                                ignored on the TOKENS axis                               */
    int32_t qaxis;           /* tom_qaxis_t                                              */
    int32_t bits;            /* 4 (paper default) or 2 (the paper's bit-width ablation)  */
    int32_t capacity_groups; /* T_cap: frame-groups the bound storage can hold           */
    int32_t in_dtype;        /* tom_dtype_t of K/V handed to quantize_append             */
    int32_t out_dtype;       /* tom_dtype_t of the active KV buffer                      */
    int32_t sim;             /* tom_sim_t                                                */
    int32_t meta_dtype;      /* TOM_F32, or TOM_BF16: (scale, zero) kept as bfloat16 pairs */
} tom_oqm_config_t;

typedef struct {
    size_t codes; /* bytes of each storage array for this configuration */
    size_t meta;
    size_t keys;
} tom_oqm_sizes_t;

/* ---- handle management (host only, no GPU work) ------------------------- */

/* Byte sizes of the three storage arrays the caller must allocate (layout
 * above).  INVALID_ARG / UNSUPPORTED if the configuration is not usable. */
tom_status_t tom_oqm_query_sizes(const tom_oqm_config_t* cfg, tom_oqm_sizes_t* sizes);

/* Creates a handle (a small host struct: configuration, bound pointers, the
 * number of stored frame-groups).  *out is NULL on failure. */
tom_status_t tom_oqm_create(const tom_oqm_config_t* cfg, tom_oqm_t** out);

/* Binds caller-owned device arrays of at least the sizes reported by
 * tom_oqm_query_sizes.  The contents are not touched: binding arrays that
 * already hold a stream, then tom_oqm_set_num_groups, restores a checkpoint. */
tom_status_t tom_oqm_bind(tom_oqm_t* h, void* codes_device, void* meta_device,
                          void* keys_device);

/* Forget all stored groups (the memory itself is not cleared). */
tom_status_t tom_oqm_reset(tom_oqm_t* h);
/* Number of committed frame-groups T (host counter); -1 if h is NULL. */
int32_t tom_oqm_num_groups(const tom_oqm_t* h);
/* Sets the counter, 0 <= n <= capacity_groups (checkpoint restore). */
tom_status_t tom_oqm_set_num_groups(tom_oqm_t* h, int32_t n);
void tom_oqm_destroy(tom_oqm_t* h);
const char* tom_last_error(void);

/* Supplement, "Question-guided single-pass retrieval": K = min(ceil(B / G), T)
 * with B the token budget, G tokens per frame-group, T stored frame-groups. */
int32_t tom_oqm_k_from_budget(int64_t budget_tokens, int32_t group_tokens, int32_t stored_groups);

/* ---- the hot path -------------------------------------------------------- */

/*
 * Store step (Sec. 3.4, Eq. 8 and Eq. 9; summary key: Sec. 3.4 and the
 * supplement's "Layer-wise vision memory").
 *
 * Quantizes n_frames frame-groups of layers [layer0, layer0 + n_layers) and
 * writes them to group slots T .. T + n_frames - 1, T = tom_oqm_num_groups(h).
 * Per quant-group (gs consecutive channels of one token, or with qaxis TOKENS
 * all G tokens of one channel): m = min, s = (max - min) / n in float32 with
 * n = 2^bits - 1 steps (15; 3 for 2-bit codes);
 * code = clamp(round_half_even(d * inv), 0, n) with d = float32(x - m),
 * inv = float32(1 / s) computed once per quant-group, and the product d * inv
 * not rounded before the rounding to an integer; s below FLT_MIN (e.g.
 * max == min) is stored as 0 with all codes 0; m is stored as +0 rather than
 * -0.  K and V use the same quantizer.
 * With meta_dtype TOM_BF16 (a storage variant; halves the metadata) s and m are rounded
 * to bfloat16, nearest even, right after the "below FLT_MIN" rule; the codes are then
 * taken against the rounded pair, so the clamp does real work and the reconstruction
 * error is at most s/2 + 2^-8 (|m| + n s).  |m| above the largest bfloat16 is unspecified.
 * Also writes one summary key per (layer, frame-group, KV head): the mean over
 * the G tokens of the un-quantized keys (accumulated in float64, rounded once).
 *
 *   k, v           device; logical shape [n_frames][n_layers][H_k][G][d] of
 *                  cfg.in_dtype, element (f, l, h, tok, c) at
 *                  f*strides[0] + l*strides[1] + h*strides[2] + tok*strides[3] + c
 *                  (l relative to layer0; strides in elements, >= 0; rows of d
 *                  channels are contiguous and must start 16-byte aligned).
 *   k_for_summary  device, same shape/strides, or NULL to average `k` itself
 *                  (the paper averages the keys taken before the rotary
 *                  embedding; pass those here if `k` is post-rotary).
 *   commit         non-zero: advance the group counter by n_frames.  A model
 *                  that appends layer by layer passes 0 for all but its last
 *                  layer, so that every layer writes the same slots.
 *   first_group    host, may be NULL: receives T, the first slot written.
 *
 * Errors: INVALID_ARG (NULL k/v, bad layer range, n_frames < 0, misaligned
 * pointer or stride), CAPACITY (T + n_frames > capacity_groups; nothing is
 * evicted), NOT_BOUND, UNSUPPORTED (more than 65535 frames or 32767 layers in one
 * call, or n_frames * n_layers * H_k * (G + 1) above 2^31 - 1; a token stride so large that one head tile, (G + 1024) * strides[3]
 * elements, spans 2 GiB or more), HIP.  n_frames == 0 or n_layers == 0 is a
 * successful no-op.  first_group is written by successful calls only.
 */
tom_status_t tom_oqm_quantize_append(tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                     int32_t n_frames, const void* k_device,
                                     const void* v_device, const void* k_for_summary_device,
                                     const int64_t strides[4], int32_t commit,
                                     void* hip_stream, int32_t* first_group);

/* Bytes of device workspace tom_oqm_score_groups needs for this call shape
 * (0 on arguments that call would refuse).  `path` is a tom_score_path_t. */
size_t tom_oqm_score_workspace_bytes(const tom_oqm_t* h, int32_t n_layers, int32_t t_q,
                                     int32_t path, int32_t want_token_scores);

/*
 * Retrieval score (Sec. 3.4, Eq. 12; supplement "Question-guided single-pass
 * retrieval").  Per layer: average the r = H_q / H_k consecutive query heads
 * of each GQA block, average over the T_q query tokens, flatten [H_k][d], and
 * compare with each of the T stored summary keys flattened the same way:
 *   TOM_SIM_DOT     score = <q, key_t>
 *   TOM_SIM_COSINE  score = <q, key_t> / (max(|q|, 1e-12) * max(|key_t|, 1e-12))
 * Accumulation is float64 on both paths; the result is rounded once to float32.
 *
 *   q             device, [n_layers][H_q][T_q][d] contiguous, tom_dtype_t q_dtype
 *   scores        device, [n_layers][score_stride] float32; entries [0, T) of
 *                 each row are written, T = tom_oqm_num_groups(h)
 *   token_scores  device or NULL, [n_layers][T_q][T] float32: un-normalised dot
 *                 of query token j (GQA-folded) with key t.  Only produced by
 *                 the TOKEN_GEMM path.
 *   workspace     device, 16-byte aligned, at least
 *                 tom_oqm_score_workspace_bytes(...) bytes; scratch, contents
 *                 undefined afterwards; concurrent calls need separate ones.
 * Errors: INVALID_ARG, NOT_BOUND, UNSUPPORTED (more than 65535 layers or more than
 * 2^20 query tokens per call), HIP.  T == 0 is a no-op.
 */
tom_status_t tom_oqm_score_groups(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                  const void* q_device, int32_t q_dtype, int32_t t_q,
                                  float* scores_device, int64_t score_stride,
                                  float* token_scores_device, int32_t path,
                                  void* workspace_device, size_t workspace_bytes,
                                  void* hip_stream);

/*
 * Selection (Eq. 12 TopK; supplement: selected indices kept in sorted order).
 * For each of n_rows rows of `scores` (row stride score_stride, first
 * n_groups entries valid) picks the k_eff = min(k, n_groups) largest scores;
 * equal scores (-0 == +0) are taken by lower index first.  Writes k_eff
 * indices per row to idx[row * k .. row * k + k_eff), ascending index or
 * descending score per `order`; the rest of the row is left untouched.
 *   idx         device int32 [n_rows][k]
 *   k_eff_host  host, may be NULL: receives k_eff (known without a sync)
 * Errors: INVALID_ARG (k < 1, n_groups < 0, stride < n_groups, NULL),
 * UNSUPPORTED (SCORE_DESC with k_eff > 4096), HIP.  k_eff_host is written by
 * successful calls only.
 */
tom_status_t tom_oqm_topk(const float* scores_device, int64_t score_stride, int32_t n_rows,
                          int32_t n_groups, int32_t k, int32_t order, int32_t* idx_device,
                          int32_t* k_eff_host, void* hip_stream);

/*
 * Reconstruction (Eq. 11) of the selected groups into the bounded active KV
 * buffer (Eq. 13; supplement "Cache reconstruction for decoding").
 * For each layer li < n_layers and rank r < k_eff, frame-group
 * t = idx[li * k + r] of K and of V is dequantized, x = float(code) * s + m
 * (one fused float32 multiply-add, then rounded to cfg.out_dtype, ties to
 * even), into token rows [r * G, (r + 1) * G) of that layer's buffers.
 *   idx           device int32 [n_layers][k] (as written by tom_oqm_topk; it
 *                 stays on the device between the two calls)
 *   k_out, v_out  device, [n_layers][H_k][k * G][d] of cfg.out_dtype, 16-byte
 *                 aligned.  Rows >= k_eff * G are never written: the active
 *                 buffer is bounded by k * G tokens per layer whatever T is.
 * An index outside [0, T) is skipped by the kernel (its rows stay untouched).
 * Errors: INVALID_ARG, NOT_BOUND, UNSUPPORTED (more than 65535 layers per call,
 * more than 32767 KV heads, or k_eff * ceil(G / 3) above 2^31 - 1), HIP.
 * k_eff == 0 is a no-op.
 */
tom_status_t tom_oqm_dequant_gather(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                    const int32_t* idx_device, int32_t k, int32_t k_eff,
                                    void* k_out_device, void* v_out_device, void* hip_stream);

/*
 * Active-KV assembly with the system-token prefix (Sec. 3.4: the memory is a dual
 * structure, system tokens stay in 16 bits while visual groups are quantized; supplement
 * "Cache reconstruction for decoding": the KV slices of the selected groups and the system
 * prompt tokens are assembled into one cache).
 * Like tom_oqm_dequant_gather, but every head's buffer has prefix_rows extra token rows in
 * front of the gathered groups:
 *   k_out, v_out  device, [n_layers][H_k][prefix_rows + k * G][d] of cfg.out_dtype;
 *                 group of rank r goes to rows [prefix_rows + r*G, prefix_rows + (r+1)*G)
 *   sys_k, sys_v  device, [n_layers][H_k][prefix_rows][d] of cfg.out_dtype (already in the
 *                 model's 16-bit format: they are copied, not re-quantized), or both NULL
 *                 to leave rows [0, prefix_rows) as they are (e.g. written once per session).
 * Errors as for tom_oqm_dequant_gather; prefix_rows < 0 or only one of sys_k / sys_v given
 * is INVALID_ARG; with a prefix source, H_k * n_layers > 65535 is UNSUPPORTED.
 */
tom_status_t tom_oqm_assemble_active(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                     const int32_t* idx_device, int32_t k, int32_t k_eff,
                                     int32_t prefix_rows, const void* sys_k_device,
                                     const void* sys_v_device, void* k_out_device,
                                     void* v_out_device, void* hip_stream);

/*
 * One call per question (supplement "Question-guided single-pass retrieval" and "Cache
 * reconstruction for decoding": the matching cost is paid once per question and the
 * per-layer indices are reused for all decoding steps): tom_oqm_score_groups, then
 * tom_oqm_topk (ascending index order, k_eff = min(k, T)), then tom_oqm_assemble_active,
 * queued back to back on one stream.  All three argument sets are validated before the
 * first kernel is queued.  `scores` ([n_layers][score_stride]) and `idx` ([n_layers][k])
 * are outputs the caller may inspect or reuse; the other arguments are those of the three
 * calls.  No allocation, no memset, no synchronisation: the call can be captured in a HIP
 * graph.
 */
tom_status_t tom_oqm_retrieve(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                              const void* q_device, int32_t q_dtype, int32_t t_q, int32_t k,
                              int32_t path, float* scores_device, int64_t score_stride,
                              int32_t* idx_device, int32_t prefix_rows, const void* sys_k_device,
                              const void* sys_v_device, void* k_out_device, void* v_out_device,
                              void* workspace_device, size_t workspace_bytes, int32_t* k_eff_host,
                              void* hip_stream);

/*
 * tom_oqm_retrieve for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same steps, same kernels, same results as tom_oqm_retrieve; the score step's
 * scratch lives in a fixed device array inside the library (tom_oqm_static_scratch_bytes()
 * = 8 MiB, held on every GPU the library runs on until the process ends).  The call
 * allocates and frees nothing.  The array's device address is looked up at the first call
 * on each device (no allocation; make that first call outside a graph capture).
 *   - Shapes whose scratch (tom_oqm_score_workspace_bytes of the same n_layers, t_q, path)
 *     exceeds the array are refused with UNSUPPORTED before anything is queued: 8 MiB
 *     covers 28 layers x 64 query tokens x 512 flattened key channels on the TOKEN_GEMM path
 *     and any realistic shape on the MEAN_QUERY path.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap
 *     (different streams, or two threads) race on it.  Calls on one stream are safe.
 *     Nothing in the array has to start at zero; every call overwrites what it reads.
 * Other arguments, outputs and errors as for tom_oqm_retrieve.
 */
tom_status_t tom_oqm_retrieve_noalloc(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                      const void* q_device, int32_t q_dtype, int32_t t_q, int32_t k,
                                      int32_t path, float* scores_device, int64_t score_stride,
                                      int32_t* idx_device, int32_t prefix_rows,
                                      const void* sys_k_device, const void* sys_v_device,
                                      void* k_out_device, void* v_out_device, int32_t* k_eff_host,
                                      void* hip_stream);
/* Size in bytes of the static scratch array tom_oqm_retrieve_noalloc works in. */
size_t tom_oqm_static_scratch_bytes(void);

#ifdef __cplusplus
}
#endif
#endif /* TOM_OQM_H */

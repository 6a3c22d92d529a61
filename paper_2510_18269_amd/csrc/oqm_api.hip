// Host side of the C ABI declared in include/tom_oqm.h: handle management,
// argument validation, and dispatch to the gfx950 kernels.  Nothing here
// allocates device memory or synchronises with the GPU.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "oqm_common.h"

namespace oqm {

static thread_local char g_err[512] = "";

tom_status_t fail(tom_status_t st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

static bool dtype_ok(int32_t t) { return t == TOM_F32 || t == TOM_BF16 || t == TOM_F16; }
static int dtype_bytes(int32_t t) { return t == TOM_F32 ? 4 : 2; }
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static tom_status_t check_config(const tom_oqm_config_t* c) {
    if (!c) return fail(TOM_ERR_INVALID_ARG, "config is NULL");
    if (c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1)
        return fail(TOM_ERR_INVALID_ARG, "n_layers, n_kv_heads and n_q_heads must be >= 1");
    if (c->n_q_heads % c->n_kv_heads)
        return fail(TOM_ERR_INVALID_ARG, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)",
                    c->n_q_heads, c->n_kv_heads);
    if (c->head_dim < 8 || c->head_dim % 8 || c->head_dim > 2048)
        return fail(TOM_ERR_INVALID_ARG, "head_dim %d must be a multiple of 8 in [8, 2048]", c->head_dim);
    if (c->group_tokens < 1) return fail(TOM_ERR_INVALID_ARG, "group_tokens must be >= 1");
    if (((int64_t)c->group_tokens + 1024) * c->head_dim * 4 >= (1LL << 31))
        return fail(TOM_ERR_UNSUPPORTED, "group_tokens * head_dim is too large (one head tile must stay below 2 GiB)");
    if (c->capacity_groups < 1) return fail(TOM_ERR_INVALID_ARG, "capacity_groups must be >= 1");
    if (!dtype_ok(c->in_dtype) || !dtype_ok(c->out_dtype))
        return fail(TOM_ERR_INVALID_ARG, "in_dtype / out_dtype must be TOM_F32, TOM_BF16 or TOM_F16");
    if (c->sim != TOM_SIM_DOT && c->sim != TOM_SIM_COSINE)
        return fail(TOM_ERR_INVALID_ARG, "sim must be TOM_SIM_DOT or TOM_SIM_COSINE");
    if (c->bits != 4 && c->bits != 2) return fail(TOM_ERR_INVALID_ARG, "bits must be 4 or 2");
    if (c->meta_dtype == TOM_F16)
        return fail(TOM_ERR_UNSUPPORTED, "meta_dtype TOM_F16: binary16 cannot hold the scale of wide groups; use TOM_BF16");
    if (c->meta_dtype != TOM_F32 && c->meta_dtype != TOM_BF16)
        return fail(TOM_ERR_INVALID_ARG, "meta_dtype must be TOM_F32 or TOM_BF16");
    if (c->qaxis != TOM_QAXIS_HEAD_DIM && c->qaxis != TOM_QAXIS_TOKENS)
        return fail(TOM_ERR_INVALID_ARG, "qaxis is not a tom_qaxis_t");
    if (c->qaxis == TOM_QAXIS_HEAD_DIM) {
        const int gs = c->qgroup;
        if (gs < 1 || c->head_dim % gs)
            return fail(TOM_ERR_INVALID_ARG, "qgroup %d does not divide head_dim %d", gs, c->head_dim);
        if (gs != 8 && gs != 16 && gs != 32 && gs != 64 && gs != 128)
            return fail(TOM_ERR_UNSUPPORTED, "qgroup %d: the kernels cover 8, 16, 32, 64 and 128", gs);
    }
    if ((int64_t)c->n_kv_heads * c->head_dim > 8192)
        return fail(TOM_ERR_UNSUPPORTED, "n_kv_heads * head_dim > 8192 is not covered by the score kernels");
    // every storage array must have a byte size (and element offsets) that 64-bit arithmetic holds;
    // input elements (4 bytes at most) bound codes, metadata and keys alike
    const unsigned __int128 elems = (unsigned __int128)c->n_layers * 2 * (unsigned)c->capacity_groups *
                                    (unsigned)c->n_kv_heads * (unsigned)c->group_tokens * (unsigned)c->head_dim;
    if (elems * 8 >= ((unsigned __int128)1 << 62))
        return fail(TOM_ERR_UNSUPPORTED, "the storage arrays of this configuration would exceed 2^62 bytes");
    return TOM_OK;
}

// The launchers report hipGetLastError() after their launch.  An error that an unrelated,
// earlier HIP call of the process left behind must not be taken for this launch's: read it
// away first (reading resets it).
static void drop_stale_hip_error() { (void)hipGetLastError(); }

static tom_status_t check_layers(const tom_oqm_t* h, int32_t layer0, int32_t n_layers) {
    if (layer0 < 0 || n_layers < 0 || (int64_t)layer0 + n_layers > h->cfg.n_layers)
        return fail(TOM_ERR_INVALID_ARG, "layer range [%d, %lld) is outside [0, %d)", layer0,
                    (long long)layer0 + n_layers, h->cfg.n_layers);
    return TOM_OK;
}

// ---- scratch memory of the entry point that allocates nothing ---------------------------
// The score step's scratch (folded query, its squared norms, the per-token query block of
// the matrix-core path) for callers that can neither allocate nor hand over a workspace.
// The array's name is only a host-side stand-in: its device address is looked up once per
// device (each GPU holds its own copy) and that pointer is what the kernels get.
constexpr size_t kScratchBytes = size_t{8} << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

static tom_status_t static_scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(TOM_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(TOM_ERR_UNSUPPORTED, "device ordinal %d is outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> guard(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(TOM_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TOM_OK;
}

}  // namespace oqm

using namespace oqm;

extern "C" {

const char* tom_last_error(void) { return g_err; }

tom_status_t tom_oqm_query_sizes(const tom_oqm_config_t* cfg, tom_oqm_sizes_t* sizes) {
    if (!sizes) return fail(TOM_ERR_INVALID_ARG, "sizes is NULL");
    if (tom_status_t st = check_config(cfg)) return st;
    const Layout lay = layout_of(*cfg);
    const size_t tiles = (size_t)cfg->n_layers * 2 * (size_t)cfg->capacity_groups * cfg->n_kv_heads;
    sizes->codes = tiles * (size_t)lay.tile_code_bytes;
    sizes->meta = tiles * (size_t)lay.tile_meta * 2 * (cfg->meta_dtype == TOM_BF16 ? 2 : sizeof(float));
    sizes->keys = (size_t)cfg->n_layers * cfg->capacity_groups * cfg->n_kv_heads * cfg->head_dim *
                  sizeof(float);
    return TOM_OK;
}

tom_status_t tom_oqm_create(const tom_oqm_config_t* cfg, tom_oqm_t** out) {
    if (!out) return fail(TOM_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (tom_status_t st = check_config(cfg)) return st;
    tom_oqm_t* h = new (std::nothrow) tom_oqm_t();
    if (!h) return fail(TOM_ERR_INVALID_ARG, "out of host memory");
    h->cfg = *cfg;
    *out = h;
    return TOM_OK;
}

tom_status_t tom_oqm_bind(tom_oqm_t* h, void* codes, void* meta, void* keys) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    if (!codes || !meta || !keys)
        return fail(TOM_ERR_INVALID_ARG, "codes, meta and keys must all be non-NULL");
    if (!aligned16(codes) || !aligned16(meta) || !aligned16(keys))
        return fail(TOM_ERR_INVALID_ARG, "storage arrays must be 16-byte aligned");
    h->codes = static_cast<uint8_t*>(codes);
    h->meta = meta;
    h->keys = static_cast<float*>(keys);
    h->bound = true;
    return TOM_OK;
}

tom_status_t tom_oqm_reset(tom_oqm_t* h) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    h->n_groups = 0;
    return TOM_OK;
}

int32_t tom_oqm_num_groups(const tom_oqm_t* h) { return h ? h->n_groups : -1; }

tom_status_t tom_oqm_set_num_groups(tom_oqm_t* h, int32_t n) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    if (n < 0 || n > h->cfg.capacity_groups)
        return fail(TOM_ERR_INVALID_ARG, "n = %d is outside [0, capacity_groups = %d]", n,
                    h->cfg.capacity_groups);
    h->n_groups = n;
    return TOM_OK;
}

void tom_oqm_destroy(tom_oqm_t* h) { delete h; }

int32_t tom_oqm_k_from_budget(int64_t budget_tokens, int32_t group_tokens, int32_t stored_groups) {
    if (budget_tokens < 0 || group_tokens < 1 || stored_groups < 0) return 0;
    const int64_t a = budget_tokens / group_tokens + (budget_tokens % group_tokens != 0);  // ceil, no overflow
    return (int32_t)(a < stored_groups ? a : stored_groups);
}

tom_status_t tom_oqm_quantize_append(tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                     int32_t n_frames, const void* k, const void* v,
                                     const void* k_for_summary, const int64_t strides[4],
                                     int32_t commit, void* hip_stream, int32_t* first_group) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    if (!h->bound) return fail(TOM_ERR_NOT_BOUND, "tom_oqm_bind has not been called");
    if (tom_status_t st = check_layers(h, layer0, n_layers)) return st;
    if (n_frames < 0) return fail(TOM_ERR_INVALID_ARG, "n_frames < 0");
    if ((int64_t)h->n_groups + n_frames > h->cfg.capacity_groups)
        return fail(TOM_ERR_CAPACITY, "%d stored + %d new frame-groups exceed capacity %d",
                    h->n_groups, n_frames, h->cfg.capacity_groups);
    if (n_frames == 0 || n_layers == 0) {
        if (first_group) *first_group = h->n_groups;
        return TOM_OK;
    }
    if (!k || !v || !strides) return fail(TOM_ERR_INVALID_ARG, "k, v and strides must be non-NULL");
    const tom_oqm_config_t& c = h->cfg;
    const int eb = dtype_bytes(c.in_dtype);
    constexpr int64_t kMaxStride = int64_t{1} << 40;  // elements; far beyond any device tensor
    for (int i = 0; i < 4; ++i)
        if (strides[i] < 0 || strides[i] > kMaxStride || (strides[i] * eb) % 16)
            return fail(TOM_ERR_INVALID_ARG,
                        "strides[%d] = %lld must be in [0, 2^40] elements and a multiple of 16 bytes", i,
                        (long long)strides[i]);
    if (strides[3] < c.head_dim && c.group_tokens > 1)
        return fail(TOM_ERR_INVALID_ARG, "token stride %lld is smaller than head_dim", (long long)strides[3]);
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_for_summary))
        return fail(TOM_ERR_INVALID_ARG, "k, v and k_for_summary must be 16-byte aligned");
    if (n_frames > 65535 || 2 * n_layers > 65535)
        return fail(TOM_ERR_UNSUPPORTED, "at most 65535 frames and 32767 layers per call");
    // the head_dim-axis kernel takes up to G + 1 workgroups per (frame, layer, head) in a 1-D grid
    // (n_frames <= 65535 and n_layers * n_kv_heads < 2^25, so the first product fits 64 bits)
    if ((int64_t)n_frames * n_layers * c.n_kv_heads > 0x7fffffffLL / ((int64_t)c.group_tokens + 1))
        return fail(TOM_ERR_UNSUPPORTED, "n_frames * n_layers * n_kv_heads * (group_tokens + 1) exceeds 2^31 - 1: "
                                         "append fewer frames per call");
    if (strides[3] > ((1LL << 31) - 1) / eb / ((int64_t)c.group_tokens + 1024))
        return fail(TOM_ERR_UNSUPPORTED, "one head tile spans 2 GiB or more (token stride too large)");

    QuantArgs a{};
    a.k = k;
    a.v = v;
    a.ksum = k_for_summary ? k_for_summary : k;
    a.stride_frame = strides[0];
    a.stride_layer = strides[1];
    a.stride_head = strides[2];
    a.stride_token = strides[3];
    a.codes = h->codes;
    a.meta = h->meta;
    a.keys = h->keys;
    a.n_kv_heads = c.n_kv_heads;
    a.head_dim = c.head_dim;
    a.group_tokens = c.group_tokens;
    a.qgroup = c.qgroup;
    a.capacity_groups = c.capacity_groups;
    a.layer0 = layer0;
    a.n_layers = n_layers;
    a.n_frames = n_frames;
    a.first_group = h->n_groups;
    a.qaxis = c.qaxis;
    a.bits = c.bits;
    a.meta_bf16 = c.meta_dtype == TOM_BF16;
    drop_stale_hip_error();
    const hipError_t e = launch_quantize_append(a, c.in_dtype, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(TOM_ERR_HIP, "quantize_append launch: %s", hipGetErrorString(e));
    if (first_group) *first_group = h->n_groups;  // only a call that succeeds writes its output
    if (commit) h->n_groups += n_frames;
    return TOM_OK;
}

// Query tokens per call: keeps every workspace size and element offset of the score step far
// inside 64 bits (65535 layers x 2^20 tokens x 8192 channels x 8 bytes < 2^63).
constexpr int32_t kMaxQueryTokens = 1 << 20;

static int resolve_path(int32_t path, bool want_tokens) {
    if (path == TOM_SCORE_AUTO) return want_tokens ? TOM_SCORE_TOKEN_GEMM : TOM_SCORE_MEAN_QUERY;
    return path;
}

size_t tom_oqm_score_workspace_bytes(const tom_oqm_t* h, int32_t n_layers, int32_t t_q,
                                     int32_t path, int32_t want_token_scores) {
    if (!h || n_layers < 0 || n_layers > h->cfg.n_layers || t_q < 1 || t_q > kMaxQueryTokens) return 0;
    const size_t hd = (size_t)h->cfg.n_kv_heads * h->cfg.head_dim;
    size_t doubles = (size_t)n_layers * hd + (size_t)n_layers * h->cfg.n_kv_heads;
    doubles = (doubles + 1) & ~(size_t)1;
    if (resolve_path(path, want_token_scores != 0) == TOM_SCORE_TOKEN_GEMM)
        doubles += (size_t)n_layers * t_q * hd;
    return doubles * sizeof(double) + 16;
}

// Each hot-path call is "validate everything, then launch": `launch == false` stops after the
// validation, which lets tom_oqm_retrieve check all three steps before it queues the first.
static tom_status_t score_impl(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                               const void* q, int32_t q_dtype, int32_t t_q, float* scores,
                               int64_t score_stride, float* token_scores, int32_t path,
                               void* workspace, size_t workspace_bytes, void* hip_stream,
                               bool launch) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    if (!h->bound) return fail(TOM_ERR_NOT_BOUND, "tom_oqm_bind has not been called");
    if (tom_status_t st = check_layers(h, layer0, n_layers)) return st;
    if (t_q < 1) return fail(TOM_ERR_INVALID_ARG, "t_q must be >= 1");
    if (t_q > kMaxQueryTokens)
        return fail(TOM_ERR_UNSUPPORTED, "t_q = %d: at most %d query tokens per call", t_q, kMaxQueryTokens);
    if (!dtype_ok(q_dtype)) return fail(TOM_ERR_INVALID_ARG, "q_dtype is not a tom_dtype_t");
    if (path != TOM_SCORE_AUTO && path != TOM_SCORE_MEAN_QUERY && path != TOM_SCORE_TOKEN_GEMM)
        return fail(TOM_ERR_INVALID_ARG, "path is not a tom_score_path_t");
    const int T = h->n_groups;
    if (score_stride < T) return fail(TOM_ERR_INVALID_ARG, "score_stride %lld < stored groups %d",
                                      (long long)score_stride, T);
    if (T == 0 || n_layers == 0) return TOM_OK;
    if (n_layers > 65535) return fail(TOM_ERR_UNSUPPORTED, "at most 65535 layers per call");
    if (!q || !scores) return fail(TOM_ERR_INVALID_ARG, "q and scores must be non-NULL");
    if (!aligned16(q)) return fail(TOM_ERR_INVALID_ARG, "q must be 16-byte aligned");
    const int rpath = resolve_path(path, token_scores != nullptr);
    if (token_scores && rpath != TOM_SCORE_TOKEN_GEMM)
        return fail(TOM_ERR_INVALID_ARG, "token_scores are only produced by TOM_SCORE_TOKEN_GEMM");
    const size_t need = tom_oqm_score_workspace_bytes(h, n_layers, t_q, rpath, token_scores != nullptr);
    if (!workspace || workspace_bytes < need)
        return fail(TOM_ERR_INVALID_ARG, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    if (!aligned16(workspace)) return fail(TOM_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    if (!launch) return TOM_OK;

    const tom_oqm_config_t& c = h->cfg;
    const size_t hd = (size_t)c.n_kv_heads * c.head_dim;
    ScoreArgs a{};
    a.keys = h->keys;
    a.q = q;
    a.scores = scores;
    a.token_scores = token_scores;
    a.ws_qbar = static_cast<double*>(workspace);
    a.ws_qnorm2 = a.ws_qbar + (size_t)n_layers * hd;
    size_t used = (size_t)n_layers * hd + (size_t)n_layers * c.n_kv_heads;
    used = (used + 1) & ~(size_t)1;
    a.ws_qtok = a.ws_qbar + used;
    a.score_stride = score_stride;
    a.n_kv_heads = c.n_kv_heads;
    a.n_q_heads = c.n_q_heads;
    a.head_dim = c.head_dim;
    a.capacity_groups = c.capacity_groups;
    a.layer0 = layer0;
    a.n_layers = n_layers;
    a.t_q = t_q;
    a.n_groups = T;
    a.sim = c.sim;
    a.q_dtype = q_dtype;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    drop_stale_hip_error();
    hipError_t e = launch_query_fold(a, rpath == TOM_SCORE_TOKEN_GEMM, s);
    if (e != hipSuccess) return fail(TOM_ERR_HIP, "query_fold launch: %s", hipGetErrorString(e));
    e = rpath == TOM_SCORE_TOKEN_GEMM ? launch_score_token_gemm(a, s) : launch_score_mean_query(a, s);
    if (e != hipSuccess) return fail(TOM_ERR_HIP, "score launch: %s", hipGetErrorString(e));
    return TOM_OK;
}

tom_status_t tom_oqm_score_groups(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                  const void* q, int32_t q_dtype, int32_t t_q, float* scores,
                                  int64_t score_stride, float* token_scores, int32_t path,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
    return score_impl(h, layer0, n_layers, q, q_dtype, t_q, scores, score_stride, token_scores, path,
                      workspace, workspace_bytes, hip_stream, true);
}

static tom_status_t topk_impl(const float* scores, int64_t score_stride, int32_t n_rows,
                              int32_t n_groups, int32_t k, int32_t order, int32_t* idx,
                              int32_t* k_eff_host, void* hip_stream, bool launch) {
    if (k < 1) return fail(TOM_ERR_INVALID_ARG, "k must be >= 1");
    if (n_rows < 0 || n_groups < 0) return fail(TOM_ERR_INVALID_ARG, "n_rows and n_groups must be >= 0");
    if (score_stride < n_groups) return fail(TOM_ERR_INVALID_ARG, "score_stride < n_groups");
    if (order != TOM_ORDER_INDEX_ASC && order != TOM_ORDER_SCORE_DESC)
        return fail(TOM_ERR_INVALID_ARG, "order is not a tom_order_t");
    const int k_eff = k < n_groups ? k : n_groups;
    if (order == TOM_ORDER_SCORE_DESC && k_eff > kTopkMaxSortedK)
        return fail(TOM_ERR_UNSUPPORTED, "TOM_ORDER_SCORE_DESC supports k_eff <= %d", kTopkMaxSortedK);
    if ((n_rows > 0 && k_eff > 0) && (!scores || !idx))
        return fail(TOM_ERR_INVALID_ARG, "scores and idx must be non-NULL");
    if (!launch) return TOM_OK;  // validation pass of the one-call retrieval: no output yet
    if (k_eff_host) *k_eff_host = k_eff;
    if (n_rows == 0 || k_eff == 0) return TOM_OK;
    drop_stale_hip_error();
    const hipError_t e = launch_topk(scores, score_stride, n_rows, n_groups, k, k_eff, order, idx,
                                     static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(TOM_ERR_HIP, "topk launch: %s", hipGetErrorString(e));
    return TOM_OK;
}

tom_status_t tom_oqm_topk(const float* scores, int64_t score_stride, int32_t n_rows,
                          int32_t n_groups, int32_t k, int32_t order, int32_t* idx,
                          int32_t* k_eff_host, void* hip_stream) {
    return topk_impl(scores, score_stride, n_rows, n_groups, k, order, idx, k_eff_host, hip_stream, true);
}

static tom_status_t assemble_impl(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                  const int32_t* idx, int32_t k, int32_t k_eff, int32_t prefix_rows,
                                  const void* sys_k, const void* sys_v, void* k_out, void* v_out,
                                  void* hip_stream, bool launch) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    if (!h->bound) return fail(TOM_ERR_NOT_BOUND, "tom_oqm_bind has not been called");
    if (tom_status_t st = check_layers(h, layer0, n_layers)) return st;
    if (k < 1 || k_eff < 0 || k_eff > k)
        return fail(TOM_ERR_INVALID_ARG, "need k >= 1 and 0 <= k_eff <= k (k = %d, k_eff = %d)", k, k_eff);
    if (prefix_rows < 0) return fail(TOM_ERR_INVALID_ARG, "prefix_rows < 0");
    if ((sys_k == nullptr) != (sys_v == nullptr))
        return fail(TOM_ERR_INVALID_ARG, "sys_k and sys_v must both be given or both be NULL");
    const bool copy_prefix = prefix_rows > 0 && sys_k != nullptr;
    if (n_layers == 0 || (k_eff == 0 && !copy_prefix)) return TOM_OK;
    if (!k_out || !v_out) return fail(TOM_ERR_INVALID_ARG, "k_out and v_out must be non-NULL");
    if (k_eff > 0 && !idx) return fail(TOM_ERR_INVALID_ARG, "idx must be non-NULL");
    if (!aligned16(k_out) || !aligned16(v_out) || !aligned16(sys_k) || !aligned16(sys_v))
        return fail(TOM_ERR_INVALID_ARG, "k_out, v_out, sys_k and sys_v must be 16-byte aligned");
    const tom_oqm_config_t& c = h->cfg;
    if (2 * c.n_kv_heads > 65535 || n_layers > 65535)
        return fail(TOM_ERR_UNSUPPORTED, "at most 32767 KV heads and 65535 layers per call");
    // the gather takes up to ceil(G / 3) workgroups per selected tile along one grid dimension
    if ((int64_t)k_eff * (((int64_t)c.group_tokens + 2) / 3) > 0x7fffffffLL)
        return fail(TOM_ERR_UNSUPPORTED, "k_eff * group_tokens / 3 exceeds 2^31 - 1");
    if (copy_prefix) {  // grid of the prefix copy: (16-byte chunks / 256, H_k * n_layers, 2)
        const int64_t prefix_bytes = (int64_t)prefix_rows * c.head_dim * dtype_bytes(c.out_dtype);
        if ((int64_t)c.n_kv_heads * n_layers > 65535)
            return fail(TOM_ERR_UNSUPPORTED, "prefix copy: n_kv_heads * n_layers = %lld exceeds 65535",
                        (long long)c.n_kv_heads * n_layers);
        if ((prefix_bytes / 16 + kBlock - 1) / kBlock > 0x7fffffffLL)
            return fail(TOM_ERR_UNSUPPORTED, "prefix copy: prefix_rows * head_dim is too large");
    }
    if (!launch) return TOM_OK;
    DequantArgs a{};
    a.codes = h->codes;
    a.meta = h->meta;
    a.idx = idx;
    a.k_out = k_out;
    a.v_out = v_out;
    a.n_kv_heads = c.n_kv_heads;
    a.head_dim = c.head_dim;
    a.group_tokens = c.group_tokens;
    a.qgroup = c.qgroup;
    a.capacity_groups = c.capacity_groups;
    a.layer0 = layer0;
    a.n_layers = n_layers;
    a.k = k;
    a.k_eff = k_eff;
    a.n_groups = h->n_groups;
    a.qaxis = c.qaxis;
    a.bits = c.bits;
    a.meta_bf16 = c.meta_dtype == TOM_BF16;
    a.prefix_rows = prefix_rows;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    drop_stale_hip_error();
    if (copy_prefix) {
        const hipError_t e = launch_prefix_copy(a, sys_k, sys_v, c.out_dtype, s);
        if (e != hipSuccess) return fail(TOM_ERR_HIP, "prefix copy launch: %s", hipGetErrorString(e));
    }
    const hipError_t e = launch_dequant_gather(a, c.out_dtype, s);
    if (e != hipSuccess) return fail(TOM_ERR_HIP, "dequant_gather launch: %s", hipGetErrorString(e));
    return TOM_OK;
}

tom_status_t tom_oqm_dequant_gather(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                    const int32_t* idx, int32_t k, int32_t k_eff, void* k_out,
                                    void* v_out, void* hip_stream) {
    return assemble_impl(h, layer0, n_layers, idx, k, k_eff, 0, nullptr, nullptr, k_out, v_out,
                         hip_stream, true);
}

tom_status_t tom_oqm_assemble_active(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                     const int32_t* idx, int32_t k, int32_t k_eff,
                                     int32_t prefix_rows, const void* sys_k, const void* sys_v,
                                     void* k_out, void* v_out, void* hip_stream) {
    return assemble_impl(h, layer0, n_layers, idx, k, k_eff, prefix_rows, sys_k, sys_v, k_out, v_out,
                         hip_stream, true);
}

// One pass of the one-call retrieval over its three steps: validation only (go == false),
// or validation and launch.
static tom_status_t retrieve_pass(const tom_oqm_t* h, int32_t layer0, int32_t n_layers, const void* q,
                                  int32_t q_dtype, int32_t t_q, int32_t k, int32_t path, float* scores,
                                  int64_t score_stride, int32_t* idx, int32_t prefix_rows,
                                  const void* sys_k, const void* sys_v, void* k_out, void* v_out,
                                  void* workspace, size_t workspace_bytes, int32_t* k_eff_host,
                                  void* hip_stream, bool go) {
    const int T = h->n_groups;
    const int k_eff = k < T ? k : T;
    if (tom_status_t st = score_impl(h, layer0, n_layers, q, q_dtype, t_q, scores, score_stride, nullptr,
                                     path, workspace, workspace_bytes, hip_stream, go))
        return st;
    if (tom_status_t st = topk_impl(scores, score_stride, n_layers, T, k, TOM_ORDER_INDEX_ASC, idx,
                                    k_eff_host, hip_stream, go))
        return st;
    return assemble_impl(h, layer0, n_layers, idx, k, k_eff < 0 ? 0 : k_eff, prefix_rows, sys_k, sys_v,
                         k_out, v_out, hip_stream, go);
}

tom_status_t tom_oqm_retrieve(const tom_oqm_t* h, int32_t layer0, int32_t n_layers, const void* q,
                              int32_t q_dtype, int32_t t_q, int32_t k, int32_t path, float* scores,
                              int64_t score_stride, int32_t* idx, int32_t prefix_rows,
                              const void* sys_k, const void* sys_v, void* k_out, void* v_out,
                              void* workspace, size_t workspace_bytes, int32_t* k_eff_host,
                              void* hip_stream) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    for (int pass = 0; pass < 2; ++pass)  // pass 0 validates all three steps, pass 1 launches them
        if (tom_status_t st = retrieve_pass(h, layer0, n_layers, q, q_dtype, t_q, k, path, scores,
                                            score_stride, idx, prefix_rows, sys_k, sys_v, k_out, v_out,
                                            workspace, workspace_bytes, k_eff_host, hip_stream, pass == 1))
            return st;
    return TOM_OK;
}

size_t tom_oqm_static_scratch_bytes(void) { return kScratchBytes; }

tom_status_t tom_oqm_retrieve_noalloc(const tom_oqm_t* h, int32_t layer0, int32_t n_layers,
                                      const void* q, int32_t q_dtype, int32_t t_q, int32_t k,
                                      int32_t path, float* scores, int64_t score_stride, int32_t* idx,
                                      int32_t prefix_rows, const void* sys_k, const void* sys_v,
                                      void* k_out, void* v_out, int32_t* k_eff_host, void* hip_stream) {
    if (!h) return fail(TOM_ERR_INVALID_ARG, "handle is NULL");
    // Size check and full validation first, on the host alone (a stand-in pointer takes the
    // workspace's place): a call that fails here has not touched the GPU.
    // (arguments the validation pass below refuses give 0 here, and are then refused there)
    const size_t need = tom_oqm_score_workspace_bytes(h, n_layers, t_q, resolve_path(path, false), 0);
    if (need > kScratchBytes)
        return fail(TOM_ERR_UNSUPPORTED,
                    "the score step needs %zu bytes of scratch for %d layers and a %d-token query; the "
                    "library's static scratch array holds %zu (use tom_oqm_retrieve with a workspace)",
                    need, n_layers, t_q, kScratchBytes);
    void* const stand_in = reinterpret_cast<void*>(uintptr_t{256});
    if (tom_status_t st = retrieve_pass(h, layer0, n_layers, q, q_dtype, t_q, k, path, scores, score_stride,
                                        idx, prefix_rows, sys_k, sys_v, k_out, v_out, stand_in,
                                        kScratchBytes, k_eff_host, hip_stream, false))
        return st;
    void* ws = stand_in;  // an empty store or layer range launches no kernel that uses scratch
    if (h->n_groups > 0 && n_layers > 0)
        if (tom_status_t st = static_scratch_of_current_device(&ws)) return st;
    return retrieve_pass(h, layer0, n_layers, q, q_dtype, t_q, k, path, scores, score_stride, idx,
                         prefix_rows, sys_k, sys_v, k_out, v_out, ws, kScratchBytes, k_eff_host,
                         hip_stream, true);
}

}  // extern "C"

// Sanitizer driver for the host side of the C ABI (csrc/oqm_api.hip): built for the host with
// -fsanitize=address,undefined by tests/test_sanitizers.py, linked against launcher stubs
// instead of the GPU kernels.  Every call below is either refused by the host-side validation
// or a documented no-op, so no launcher may ever be reached (the stubs abort if one is) and no
// device pointer is ever dereferenced (they are fakes).  Exit status 0 = clean.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "oqm_common.h"

namespace oqm {
#define STUB(name, ...)                                                     \
    hipError_t name(__VA_ARGS__) {                                          \
        std::fprintf(stderr, "launcher " #name " reached: validation let a bad call through\n"); \
        std::abort();                                                       \
    }
STUB(launch_quantize_append, const QuantArgs&, int, hipStream_t)
STUB(launch_dequant_gather, const DequantArgs&, int, hipStream_t)
STUB(launch_prefix_copy, const DequantArgs&, const void*, const void*, int, hipStream_t)
STUB(launch_query_fold, const ScoreArgs&, bool, hipStream_t)
STUB(launch_score_mean_query, const ScoreArgs&, hipStream_t)
STUB(launch_score_token_gemm, const ScoreArgs&, hipStream_t)
STUB(launch_topk, const float*, int64_t, int, int, int, int, int, int32_t*, hipStream_t)
}  // namespace oqm

static int failures = 0;
#define EXPECT(call, want)                                                                   \
    do {                                                                                     \
        const tom_status_t got_ = (call);                                                    \
        if (got_ != (want)) {                                                                \
            std::fprintf(stderr, "line %d: %s -> %d (%s), wanted %d\n", __LINE__, #call, (int)got_, \
                         tom_last_error(), (int)(want));                                     \
            ++failures;                                                                      \
        }                                                                                    \
    } while (0)

int main() {
    void* const fake = reinterpret_cast<void*>(uintptr_t{0x10000});
    float* const ffake = static_cast<float*>(fake);
    int32_t* const ifake = static_cast<int32_t*>(fake);

    // configurations: every field at a bad value, and the shape limits
    tom_oqm_config_t good = {2, 2, 4, 64, 16, 32, TOM_QAXIS_HEAD_DIM, 4, 8, TOM_BF16, TOM_BF16, TOM_SIM_COSINE, TOM_F32};
    tom_oqm_sizes_t sizes;
    EXPECT(tom_oqm_query_sizes(&good, &sizes), TOM_OK);
    EXPECT(tom_oqm_query_sizes(nullptr, &sizes), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_query_sizes(&good, nullptr), TOM_ERR_INVALID_ARG);
    const int32_t bad_values[] = {INT32_MIN, -1, 0, 3, 7, 100, 65536, INT32_MAX};
    for (size_t field = 0; field < sizeof(good) / sizeof(int32_t); ++field)
        for (int32_t v : bad_values) {
            tom_oqm_config_t c = good;
            reinterpret_cast<int32_t*>(&c)[field] = v;
            tom_oqm_t* h = nullptr;
            const tom_status_t st = tom_oqm_create(&c, &h);   // any status is fine; no overflow, no crash
            if (st == TOM_OK) {
                if (tom_oqm_query_sizes(&c, &sizes) != TOM_OK) ++failures;
                tom_oqm_destroy(h);
            } else if (h != nullptr || std::strlen(tom_last_error()) == 0) {
                ++failures;
            }
        }
    tom_oqm_config_t huge = good;
    huge.group_tokens = INT32_MAX;  huge.head_dim = 2048;
    tom_oqm_t* h = nullptr;
    EXPECT(tom_oqm_create(&huge, &h), TOM_ERR_UNSUPPORTED);
    huge = good;  huge.n_kv_heads = 8;  huge.n_q_heads = 8;  huge.head_dim = 2048;
    EXPECT(tom_oqm_create(&huge, &h), TOM_ERR_UNSUPPORTED);

    EXPECT(tom_oqm_create(&good, &h), TOM_OK);
    const int64_t st[4] = {2 * 2 * 16 * 64, 2 * 16 * 64, 16 * 64, 64};
    int32_t first = -5, k_eff = -5;
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_NOT_BOUND);
    EXPECT(tom_oqm_bind(h, fake, static_cast<char*>(fake) + 4, fake), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_bind(h, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_bind(h, fake, fake, fake), TOM_OK);
    // store step
    EXPECT(tom_oqm_quantize_append(nullptr, 0, 2, 1, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 9, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_CAPACITY);
    EXPECT(tom_oqm_quantize_append(h, 1, 2, 1, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, INT32_MAX, 1, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 1, INT32_MAX, 1, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_dequant_gather(h, INT32_MAX, INT32_MAX, ifake, 4, 1, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, -1, fake, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, nullptr, fake, nullptr, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, nullptr, nullptr, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    const int64_t odd[4] = {st[0], st[1], st[2], 65}, neg[4] = {st[0], -8, st[2], 64}, wide[4] = {st[0], st[1], st[2], INT64_MAX / 8 * 8},
                  tall[4] = {st[0], st[1], st[2], int64_t{1} << 30};
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, nullptr, odd, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, nullptr, neg, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, nullptr, wide, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, nullptr, tall, 1, nullptr, &first), TOM_ERR_UNSUPPORTED);
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, static_cast<char*>(fake) + 2, st, 1, nullptr, &first), TOM_ERR_INVALID_ARG);
    if (first != -5) { std::fprintf(stderr, "first_group written by a failing call\n"); ++failures; }
    EXPECT(tom_oqm_quantize_append(h, 0, 2, 0, fake, fake, nullptr, st, 1, nullptr, &first), TOM_OK);
    if (first != 0) ++failures;
    // score / top-k / gather / assemble / one-call retrieval, empty store and bad arguments
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, 1, ffake, 0, nullptr, TOM_SCORE_AUTO, nullptr, 0, nullptr), TOM_OK);
    EXPECT(tom_oqm_set_num_groups(h, 9), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_set_num_groups(h, 8), TOM_OK);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, 1, ffake, 8, nullptr, TOM_SCORE_AUTO, nullptr, 0, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, 1, ffake, 7, nullptr, TOM_SCORE_AUTO, fake, 1 << 20, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, 9, 1, ffake, 8, nullptr, TOM_SCORE_AUTO, fake, 1 << 20, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, 0, ffake, 8, nullptr, TOM_SCORE_AUTO, fake, 1 << 20, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, 1, ffake, 8, ffake, TOM_SCORE_MEAN_QUERY, fake, 1 << 20, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, INT32_MAX, ffake, 8, nullptr, TOM_SCORE_TOKEN_GEMM, fake, 1 << 20, nullptr), TOM_ERR_UNSUPPORTED);
    EXPECT(tom_oqm_score_groups(h, 0, 2, fake, TOM_F32, 1 << 20, ffake, 8, nullptr, TOM_SCORE_TOKEN_GEMM, fake, 1 << 20, nullptr), TOM_ERR_INVALID_ARG);
    if (tom_oqm_score_workspace_bytes(h, 2, INT32_MAX, TOM_SCORE_TOKEN_GEMM, 0) != 0) ++failures;
    if (tom_oqm_score_workspace_bytes(h, INT32_MAX, 1, TOM_SCORE_TOKEN_GEMM, 0) != 0) ++failures;
    if (tom_oqm_score_workspace_bytes(h, 2, 1 << 20, TOM_SCORE_TOKEN_GEMM, 0) < ((size_t)1 << 31)) ++failures;
    EXPECT(tom_oqm_topk(ffake, 16, 1, 10, 0, TOM_ORDER_INDEX_ASC, ifake, &k_eff, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_topk(ffake, 5, 1, 10, 4, TOM_ORDER_INDEX_ASC, ifake, &k_eff, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_topk(nullptr, 16, 1, 10, 4, TOM_ORDER_INDEX_ASC, ifake, &k_eff, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_topk(ffake, 10000, 1, 10000, 5000, TOM_ORDER_SCORE_DESC, ifake, &k_eff, nullptr), TOM_ERR_UNSUPPORTED);
    if (k_eff != -5) { std::fprintf(stderr, "k_eff written by a failing call\n"); ++failures; }
    EXPECT(tom_oqm_topk(ffake, 16, 0, 10, 64, TOM_ORDER_INDEX_ASC, ifake, &k_eff, nullptr), TOM_OK);
    if (k_eff != 10) ++failures;
    EXPECT(tom_oqm_dequant_gather(h, 0, 2, ifake, 4, 5, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_dequant_gather(h, 0, 3, ifake, 4, 1, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_dequant_gather(h, 0, 2, nullptr, 4, 1, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_dequant_gather(h, 0, 2, ifake, 4, 0, fake, fake, nullptr), TOM_OK);
    EXPECT(tom_oqm_assemble_active(h, 0, 2, ifake, 4, 1, -1, nullptr, nullptr, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_assemble_active(h, 0, 2, ifake, 4, 1, 3, fake, nullptr, fake, fake, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_assemble_active(h, 0, 2, ifake, 4, 0, INT32_MAX, nullptr, nullptr, fake, fake, nullptr), TOM_OK);
    EXPECT(tom_oqm_retrieve(h, 0, 2, fake, TOM_F32, 1, 4, TOM_SCORE_AUTO, ffake, 8, ifake, 0, nullptr, nullptr, nullptr, fake,
                            fake, 1 << 20, &k_eff, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_retrieve_noalloc(h, 0, 2, fake, TOM_F32, 1 << 20, 4, TOM_SCORE_TOKEN_GEMM, ffake, 8, ifake, 0, nullptr,
                                    nullptr, fake, fake, &k_eff, nullptr), TOM_ERR_UNSUPPORTED);
    EXPECT(tom_oqm_retrieve_noalloc(h, 0, 2, fake, TOM_F32, 1, 4, TOM_SCORE_AUTO, ffake, 8, ifake, 0, nullptr, nullptr,
                                    nullptr, fake, &k_eff, nullptr), TOM_ERR_INVALID_ARG);
    EXPECT(tom_oqm_reset(h), TOM_OK);
    EXPECT(tom_oqm_retrieve(h, 0, 2, fake, TOM_F32, 1, 4, TOM_SCORE_AUTO, ffake, 8, ifake, 0, nullptr, nullptr, fake, fake,
                            nullptr, 0, &k_eff, nullptr), TOM_OK);
    if (k_eff != 0) ++failures;
    if (tom_oqm_k_from_budget(12544, 50, 1000000) != 251 || tom_oqm_k_from_budget(INT64_MAX, 1, 7) != 7 ||
        tom_oqm_k_from_budget(-1, 50, 7) != 0)
        ++failures;
    tom_oqm_destroy(h);
    tom_oqm_destroy(nullptr);
    if (failures) { std::fprintf(stderr, "%d failures\n", failures); return 2; }
    std::printf("abi sanitizer driver: clean\n");
    return 0;
}

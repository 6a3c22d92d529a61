/*
 * Sanitizer driver for the CPU oracle: one translation unit with oracle/oqm_oracle.c, built with
 * -fsanitize=address,undefined -fno-sanitize-recover=all by tests/test_sanitizers.py.
 * Every buffer is a heap block of exactly the documented size, so an out-of-bounds access
 * anywhere on the append -> score -> top-k -> gather -> assemble path aborts the program.
 * Shapes are ragged on purpose (G = 1, 7, 197; d = 8 and 24; both code widths, both axes, all
 * dtypes, both metadata precisions).  Exit status 0 = clean.
 */
#include "../../oracle/oqm_oracle.c"

#include <stdio.h>

static uint32_t rng_state = 12345u;
static float rnd(void) { /* uniform in [-2, 2), exactly representable in bfloat16 / binary16 */
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)((int)((rng_state >> 16) & 0xff) - 128) / 64.0f;
}

static void* blk(size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
    memset(p, 0x5a, bytes ? bytes : 1);
    return p;
}

#define REQUIRE(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s failed (G=%d d=%d bits=%d axis=%d dt=%d meta=%d)\n", \
    __LINE__, #cond, G, d, bits, qaxis, dt, meta); exit(2); } } while (0)

static void run_case(int G, int d, int gs, int bits, int qaxis, int dt, int meta) {
    const int L = 2, H = 2, Hq = 4, Tcap = 5, tq = 3, k = 3, prefix = 2;
    tomref_config c = {L, H, Hq, d, G, gs, qaxis, bits, Tcap, dt, dt, TOMREF_SIM_COSINE, meta};
    const int64_t tiles = (int64_t)L * 2 * Tcap * H;
    const int64_t cb = tomref_code_bytes_per_tile(G, d, bits), mt = tomref_meta_per_tile(G, d, gs, qaxis);
    uint8_t* codes = blk((size_t)(tiles * cb));
    float* scale = blk((size_t)(tiles * mt) * 4);
    float* zero = blk((size_t)(tiles * mt) * 4);
    float* keys = blk((size_t)L * Tcap * H * d * 4);
    const size_t es = dtype_size(dt);
    /* two appends: 3 frames, then 2; contiguous [F][L][H][G][d] */
    int first = 0;
    for (int call = 0; call < 2; ++call) {
        const int F = call ? 2 : 3;
        const int64_t n = (int64_t)F * L * H * G * d;
        float* tmp = blk((size_t)n * 4);
        void* kin = blk((size_t)n * es);
        void* vin = blk((size_t)n * es);
        void* ks = blk((size_t)n * es);
        for (int64_t i = 0; i < n; ++i) tmp[i] = rnd();
        tomref_from_f32(tmp, dt, n, kin);
        for (int64_t i = 0; i < n; ++i) tmp[i] = rnd() * 3.0f;
        tomref_from_f32(tmp, dt, n, vin);
        for (int64_t i = 0; i < n; ++i) tmp[i] = rnd();
        tomref_from_f32(tmp, dt, n, ks);
        const int64_t st[4] = {(int64_t)L * H * G * d, (int64_t)H * G * d, (int64_t)G * d, d};
        REQUIRE(tomref_quantize_append(&c, codes, scale, zero, keys, first, 0, L, F, kin, vin,
                                       call ? ks : NULL, st) == 0);
        first += F;
        free(tmp); free(kin); free(vin); free(ks);
    }
    REQUIRE(tomref_quantize_append(&c, codes, scale, zero, keys, first, 0, L, 1, codes, codes, NULL,
                                   (int64_t[4]){0, 0, 0, d}) == -2);   /* over capacity */
    const int T = first;
    /* score (with per-token scores), top-k in both orders, k > T */
    const int64_t qn = (int64_t)L * Hq * tq * d;
    float* qf = blk((size_t)qn * 4);
    void* q = blk((size_t)qn * es);
    for (int64_t i = 0; i < qn; ++i) qf[i] = rnd();
    tomref_from_f32(qf, dt, qn, q);
    float* scores = blk((size_t)L * T * 4);
    float* tok = blk((size_t)L * tq * T * 4);
    REQUIRE(tomref_score_groups(&c, keys, T, 0, L, q, dt, tq, scores, T, tok) == 0);
    int32_t* idx = blk((size_t)L * k * 4);
    REQUIRE(tomref_topk(scores, T, L, T, k, TOMREF_ORDER_SCORE_DESC, idx) == k);
    REQUIRE(tomref_topk(scores, T, L, T, k, TOMREF_ORDER_INDEX_ASC, idx) == k);
    int32_t* idx_all = blk((size_t)L * 9 * 4);
    REQUIRE(tomref_topk(scores, T, L, T, 9, TOMREF_ORDER_INDEX_ASC, idx_all) == T);
    /* gather and assemble (an index out of range is refused before its tile is read) */
    const size_t rows = (size_t)k * G, prow = (size_t)(prefix + k * G);
    void* ko = blk((size_t)L * H * rows * d * es);
    void* vo = blk((size_t)L * H * rows * d * es);
    REQUIRE(tomref_dequant_gather(&c, codes, scale, zero, T, 0, L, idx, k, k, ko, vo) == 0);
    const int32_t keep = idx[1];
    idx[1] = T + 3;
    REQUIRE(tomref_dequant_gather(&c, codes, scale, zero, T, 0, L, idx, k, k, ko, vo) == -1);
    idx[1] = keep;
    REQUIRE(tomref_dequant_gather(&c, codes, scale, zero, T, 0, L, idx, k, k - 1, ko, vo) == 0);
    void* sk = blk((size_t)L * H * prefix * d * es);
    void* sv = blk((size_t)L * H * prefix * d * es);
    void* kp = blk((size_t)L * H * prow * d * es);
    void* vp = blk((size_t)L * H * prow * d * es);
    REQUIRE(tomref_assemble_active(&c, codes, scale, zero, T, 0, L, idx, k, k, prefix, sk, sv, kp, vp) == 0);
    REQUIRE(tomref_assemble_active(&c, codes, scale, zero, T, 1, 1, idx, k, 0, prefix, NULL, NULL, kp, vp) == 0);
    free(codes); free(scale); free(zero); free(keys); free(qf); free(q); free(scores); free(tok);
    free(idx); free(idx_all); free(ko); free(vo); free(sk); free(sv); free(kp); free(vp);
}

int main(void) {
    static const int Gs[] = {1, 7, 197};
    int cases = 0;
    for (int gi = 0; gi < 3; ++gi)
        for (int d = 8; d <= 24; d += 16)
            for (int bits = 2; bits <= 4; bits += 2)
                for (int qaxis = 0; qaxis < 2; ++qaxis)
                    for (int dt = 0; dt < 3; ++dt)
                        for (int meta = 0; meta < 2; ++meta) {
                            run_case(Gs[gi], d, 8, bits, qaxis, dt, meta);
                            ++cases;
                        }
    /* the stand-alone tile functions and the closed-form helpers */
    {
        float x[7 * 8], out[7 * 8], sc[7], zr[7], key[8];
        uint8_t un[7 * 8], pk[7 * 8 / 2];
        for (int i = 0; i < 56; ++i) x[i] = rnd();
        if (tomref_quantize_tile(x, 7, 8, 8, 0, 4, 0, un, pk, sc, zr) != 0) return 2;
        if (tomref_dequant_tile(pk, sc, zr, 7, 8, 8, 0, 4, out) != 0) return 2;
        tomref_summary_key(x, 7, 8, key);
        if (tomref_k_from_budget(12544, 50, 1000000) != 251) return 2;
        if (tomref_kv_cache_bytes(28, 196, 4, 128, 2, 1800) <= 0) return 2;
    }
    printf("oracle sanitizer driver: %d cases clean\n", cases);
    return 0;
}

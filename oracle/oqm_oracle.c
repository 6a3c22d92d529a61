/*
 * oqm_oracle.c — CPU oracle for the Online Quantized Memory (OQM) hot path of
 * StreamingTOM (arxiv 2510.18269).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to say what the GPU library must
 * compute.  Only the tests, the smoke check and the benchmark's cpu_baseline
 * leg may load it; the product library never links, imports or calls it, and
 * it shares no source, header, table or helper with the HIP code.
 *
 * It is a plain, slow, step-by-step statement of the method: no blocking, no
 * fusion, no reordering beyond what the cited passages say.  Build:
 *     gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared oqm_oracle.c -lm
 * (-ffp-contract=off matters: every float operation below is one correctly
 * rounded IEEE-754 binary32 operation, which is what makes the 4-bit codes
 * reproducible bit for bit on another machine.)
 *
 * What each part follows (paper sections / equations):
 *   quantizer  Q_b      Sec. 3.4 "Online Quantized Memory", Eq. 8 and Eq. 9
 *   packing             Sec. 3.4, sentence after Eq. 9 (codes packed in uint8)
 *   summary key         Sec. 3.4 (mean of the keys before quantization) and
 *                       Supplement "Text-Video Retrieval / Layer-wise vision
 *                       memory" (one H_k x d key per layer and frame-group)
 *   dequantizer         Sec. 3.4, Eq. 11
 *   scoring             Sec. 3.4, Eq. 12; Supplement "Question-guided
 *                       single-pass retrieval" (GQA mean, token mean, flatten,
 *                       l2-normalise, cosine)
 *   top-K, K from B     Supplement, same paragraph (K = min(ceil(B/G), T/G),
 *                       indices kept in sorted order)
 *   active KV           Sec. 3.4, Eq. 13; Supplement "Cache reconstruction"
 *   footprint helpers   Sec. 3.1 Eq. 1 + footnote; Sec. 3.2 footnote; Eq. 10;
 *                       ablation table (ratio column)
 *
 * Readings taken where the paper is silent (each listed in the design notes):
 *   - rounding of "uint4(.)": round half to even, then clamp to [0, levels]
 *   - code = rne(d * inv) with d = float32(x - m), inv = float32(1/s) computed once
 *     per quant-group, and the product d * inv NOT rounded before the rounding to
 *     an integer (one rounding instead of two)
 *   - dequantized value = float32(code * s + m) with a single rounding
 *   - s < FLT_MIN (incl. max == min)  =>  s stored as 0, all codes 0
 *   - m = min + 0.0f so that a stored zero point is never -0
 *   - scale / zero stored as float32; meta_dtype = bfloat16 is a storage variant the paper
 *     does not describe (the paper only says the memory keeps non-quantized parts in 16
 *     bits): s and m are rounded to bfloat16 (nearest even) BEFORE the codes are computed,
 *     the codes are taken against the rounded pair (so quantizer and dequantizer agree)
 *     and the clamp to [0, levels] does real work (m may now lie above the minimum)
 *   - even channel -> low bits of the byte (little-endian nibbles)
 *   - quantization axis: the paper reduces over the G tokens of a channel
 *     (QAXIS_TOKENS); the benchmark configurations reduce over gs consecutive
 *     channels of one token (QAXIS_HEAD_DIM).  Both are implemented.
 *   - bits = 4 (paper default) or 2 (ablation table)
 *
 * Parity pins: tests/test_oracle_*.py (marked "not gpu") check every function
 * here against values the paper prints, closed forms, invariants, library
 * routines and brute force.  No function here is "parity unpinned"; what
 * cannot be pinned is the authors' own unpublished choices listed above.
 *
 * Storage layout used by the tomref_* mirrors (element offsets):
 *   codes [L][2 (0=K,1=V)][T_cap][H_k][G][d*bits/8]           uint8
 *   scale, zero: HEAD_DIM axis [L][2][T_cap][H_k][G][d/gs]    float32
 *                TOKENS   axis [L][2][T_cap][H_k][d]          float32
 *   keys  [L][T_cap][H_k][d]                                  float32
 *   active K / V out [n_layers][H_k][k*G][d]                  out_dtype
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { TOMREF_F32 = 0, TOMREF_BF16 = 1, TOMREF_F16 = 2 };
enum { TOMREF_QAXIS_HEAD_DIM = 0, TOMREF_QAXIS_TOKENS = 1 };
enum { TOMREF_SIM_DOT = 0, TOMREF_SIM_COSINE = 1 };
enum { TOMREF_ORDER_INDEX_ASC = 0, TOMREF_ORDER_SCORE_DESC = 1 };

typedef struct {
    int32_t n_layers;        /* L                                     */
    int32_t n_kv_heads;      /* H_k                                   */
    int32_t n_q_heads;       /* H_q, a multiple of H_k                */
    int32_t head_dim;        /* d                                     */
    int32_t group_tokens;    /* G: tokens of one frame-group          */
    int32_t qgroup;          /* gs: quant-group size (HEAD_DIM axis)  */
    int32_t qaxis;           /* TOMREF_QAXIS_*                        */
    int32_t bits;            /* 4 or 2                                */
    int32_t capacity_groups; /* T_cap                                 */
    int32_t in_dtype;        /* dtype of K/V handed to quantize       */
    int32_t out_dtype;       /* dtype of the active KV buffer         */
    int32_t sim;             /* TOMREF_SIM_*                          */
    int32_t meta_dtype;      /* TOMREF_F32 or TOMREF_BF16: precision scale / zero are kept in */
} tomref_config;

/* ------------------------------------------------------------------ */
/* dtype conversion (IEEE binary16 / bfloat16 <-> binary32)            */
/* ------------------------------------------------------------------ */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* bfloat16 is the upper half of a binary32: widening is exact. */
static float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/* binary32 -> bfloat16, round to nearest, ties to even. */
static uint16_t f32_to_bf16(float f) {
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* binary16 -> binary32 (exact). */
static float f16_to_f32(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    int32_t  e = (h >> 10) & 0x1f;
    uint32_t m = h & 0x3ffu;
    if (e == 0x1f) return bits_to_f32(sign | 0x7f800000u | (m << 13));
    if (e == 0) {
        /* zero or subnormal: value = m * 2^-24 */
        float v = (float)m * (1.0f / 16777216.0f);
        return sign ? -v : v;
    }
    return bits_to_f32(sign | ((uint32_t)(e - 15 + 127) << 23) | (m << 13));
}

/* binary32 -> binary16, round to nearest, ties to even (overflow -> inf). */
static uint16_t f32_to_f16(float f) {
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);               /* NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);              /* >= 65536 -> inf (65520.. rounds below) */
    if (a < 0x33000000u) return sign;                                     /* < 2^-25 -> 0 */
    int32_t e = (int32_t)(a >> 23) - 127;                                 /* unbiased */
    uint32_t m = (a & 0x7fffffu) | 0x800000u;                             /* 24-bit significand */
    int shift = (e >= -14) ? 13 : (13 + (-14 - e));                       /* bits dropped */
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept += 1u;
    uint32_t h;
    if (e >= -14) h = ((uint32_t)(e + 15 - 1) << 10) + kept;              /* kept carries the hidden bit */
    else          h = kept;                                               /* subnormal (may round up to normal) */
    if (h >= 0x7c00u) h = 0x7c00u;
    return (uint16_t)(sign | h);
}

static size_t dtype_size(int dtype) { return dtype == TOMREF_F32 ? 4u : 2u; }

/* Widen n elements of the given dtype to float32 (exact for all three). */
void tomref_to_f32(const void* src, int32_t dtype, int64_t n, float* dst) {
    for (int64_t i = 0; i < n; ++i) {
        if (dtype == TOMREF_F32)       dst[i] = ((const float*)src)[i];
        else if (dtype == TOMREF_BF16) dst[i] = bf16_to_f32(((const uint16_t*)src)[i]);
        else                           dst[i] = f16_to_f32(((const uint16_t*)src)[i]);
    }
}

/* Narrow n float32 values to the given dtype, round-to-nearest-even. */
void tomref_from_f32(const float* src, int32_t dtype, int64_t n, void* dst) {
    for (int64_t i = 0; i < n; ++i) {
        if (dtype == TOMREF_F32)       ((float*)dst)[i] = src[i];
        else if (dtype == TOMREF_BF16) ((uint16_t*)dst)[i] = f32_to_bf16(src[i]);
        else                           ((uint16_t*)dst)[i] = f32_to_f16(src[i]);
    }
}

static float load_elem(const void* p, int32_t dtype, int64_t i) {
    if (dtype == TOMREF_F32)  return ((const float*)p)[i];
    if (dtype == TOMREF_BF16) return bf16_to_f32(((const uint16_t*)p)[i]);
    return f16_to_f32(((const uint16_t*)p)[i]);
}

/* ------------------------------------------------------------------ */
/* footprint / budget helpers (closed forms the paper prints)          */
/* ------------------------------------------------------------------ */

/* Sec. 3.1, Eq. 1 integrated over `frames` frames: K and V, L layers, N tokens
 * per frame, H_kv heads of width d_h, elem_bytes per scalar. */
double tomref_kv_cache_bytes(int32_t L, int32_t N, int32_t H_kv, int32_t d_h,
                             int32_t elem_bytes, int64_t frames) {
    return 2.0 * (double)L * (double)frames * (double)N * (double)H_kv * (double)d_h * (double)elem_bytes;
}

/* Eq. 10 generalised to b bits: (N * 16) / (G * b).  b = 4 gives 4N/G. */
double tomref_compression_ratio(int32_t N, int32_t G, int32_t bits) {
    return ((double)N * 16.0) / ((double)G * (double)bits);
}

/* True stored bits per K/V scalar including float32 scale+zero metadata. */
double tomref_bits_per_element(int32_t bits, int32_t qaxis, int32_t gs, int32_t G) {
    double per_group = (qaxis == TOMREF_QAXIS_HEAD_DIM) ? (double)gs : (double)G;
    return (double)bits + 64.0 / per_group;
}

/* Supplement: K = min(ceil(B / G), T / G) with T the number of stored tokens. */
int32_t tomref_k_from_budget(int64_t budget_tokens, int32_t G, int64_t stored_tokens) {
    int64_t a = (budget_tokens + G - 1) / G;
    int64_t b = stored_tokens / G;
    return (int32_t)(a < b ? a : b);
}

/* ------------------------------------------------------------------ */
/* quantizer Q_b and its inverse on ONE head tile x[G][d] (float32)    */
/* ------------------------------------------------------------------ */

/* Eq. 9 on one quant-group: n values x[0], x[stride], ...  Writes the group's
 * scale and zero point and n unpacked codes c[0], c[cstride], ... */
static void quant_group(const float* x, int64_t stride, int n, int levels, int meta_dtype,
                        float* scale, float* zero, uint8_t* c, int64_t cstride) {
    float mn = x[0], mx = x[0];
    for (int i = 1; i < n; ++i) {
        float v = x[(int64_t)i * stride];
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    mn = mn + 0.0f;                                 /* -0 -> +0 */
    float s = (mx - mn) / (float)levels;            /* Eq. 9: (max - min) / 15 for 4 bits */
    float inv;
    if (!(s >= FLT_MIN)) s = 0.0f;                  /* flat or sub-normal range */
    if (meta_dtype == TOMREF_BF16) {                /* kept in 16 bits: round first, then use */
        s = bf16_to_f32(f32_to_bf16(s));
        mn = bf16_to_f32(f32_to_bf16(mn));
    }
    if (!(s >= FLT_MIN)) { s = 0.0f; inv = 0.0f; }
    else inv = 1.0f / s;
    *scale = s;
    *zero = mn;                                     /* Eq. 9: m = min */
    for (int i = 0; i < n; ++i) {
        float diff = x[(int64_t)i * stride] - mn;   /* one float32 subtraction */
        /* the product of two float32 values is exact in double, so this rounds the
         * exact product (x - m) * (1/s) once, to the nearest integer, ties to even */
        double r = nearbyint((double)diff * (double)inv);
        if (r < 0.0) r = 0.0;
        if (r > (double)levels) r = (double)levels;
        c[(int64_t)i * cstride] = (uint8_t)r;
    }
}

/* Number of (scale, zero) pairs of one head tile. */
int64_t tomref_meta_per_tile(int32_t G, int32_t d, int32_t gs, int32_t qaxis) {
    return qaxis == TOMREF_QAXIS_HEAD_DIM ? (int64_t)G * (d / gs) : (int64_t)d;
}

/* Bytes of packed codes of one head tile. */
int64_t tomref_code_bytes_per_tile(int32_t G, int32_t d, int32_t bits) {
    return (int64_t)G * d * bits / 8;
}

/* Quantize one head tile x[G][d].
 *   unpacked[G][d]  codes, one per byte (may be NULL)
 *   packed[G][d*bits/8]  channel 2j (4-bit) / 4j (2-bit) in the low bits of byte j
 *   scale/zero: HEAD_DIM -> [G][d/gs]; TOKENS -> [d]; float32 arrays that hold, with
 *               meta_dtype bfloat16, values already rounded to bfloat16
 * Returns 0, or -1 on a shape the definition does not cover. */
int32_t tomref_quantize_tile(const float* x, int32_t G, int32_t d, int32_t gs, int32_t qaxis,
                             int32_t bits, int32_t meta_dtype, uint8_t* unpacked, uint8_t* packed,
                             float* scale, float* zero) {
    if (G < 1 || d < 1 || (bits != 4 && bits != 2)) return -1;
    if (meta_dtype != TOMREF_F32 && meta_dtype != TOMREF_BF16) return -1;
    int per_byte = 8 / bits;
    if (d % per_byte) return -1;
    if (qaxis == TOMREF_QAXIS_HEAD_DIM && (gs < 1 || d % gs)) return -1;
    int levels = (1 << bits) - 1;
    uint8_t* c = (uint8_t*)malloc((size_t)G * d);
    if (!c) return -1;
    if (qaxis == TOMREF_QAXIS_HEAD_DIM) {
        /* one (scale, zero) per token and per block of gs consecutive channels */
        int ng = d / gs;
        for (int tok = 0; tok < G; ++tok)
            for (int g = 0; g < ng; ++g)
                quant_group(x + (int64_t)tok * d + g * gs, 1, gs, levels, meta_dtype,
                            &scale[(int64_t)tok * ng + g], &zero[(int64_t)tok * ng + g],
                            c + (int64_t)tok * d + g * gs, 1);
    } else {
        /* paper Eq. 9: one (scale, zero) per channel, over the G tokens */
        for (int ch = 0; ch < d; ++ch)
            quant_group(x + ch, d, G, levels, meta_dtype, &scale[ch], &zero[ch], c + ch, d);
    }
    if (unpacked) memcpy(unpacked, c, (size_t)G * d);
    if (packed) {
        int64_t nbytes = (int64_t)G * d / per_byte;
        for (int64_t j = 0; j < nbytes; ++j) {
            unsigned b = 0;
            for (int u = 0; u < per_byte; ++u) b |= (unsigned)c[j * per_byte + u] << (u * bits);
            packed[j] = (uint8_t)b;
        }
    }
    free(c);
    return 0;
}

/* Eq. 11 on one head tile: x_hat = float(code) * s + m evaluated exactly and
 * rounded once to float32 (a fused multiply-add). */
int32_t tomref_dequant_tile(const uint8_t* packed, const float* scale, const float* zero,
                            int32_t G, int32_t d, int32_t gs, int32_t qaxis, int32_t bits,
                            float* out) {
    if (G < 1 || d < 1 || (bits != 4 && bits != 2)) return -1;
    int per_byte = 8 / bits;
    unsigned mask = (1u << bits) - 1u;
    int ng = (qaxis == TOMREF_QAXIS_HEAD_DIM) ? d / gs : 0;
    for (int tok = 0; tok < G; ++tok)
        for (int ch = 0; ch < d; ++ch) {
            int64_t e = (int64_t)tok * d + ch;
            unsigned code = (packed[e / per_byte] >> ((e % per_byte) * bits)) & mask;
            int64_t mi = (qaxis == TOMREF_QAXIS_HEAD_DIM) ? (int64_t)tok * ng + ch / gs : ch;
            out[e] = fmaf((float)code, scale[mi], zero[mi]);   /* code*s + m, rounded once */
        }
    return 0;
}

/* Summary key of one head tile: mean over the G tokens, per channel, of the
 * keys BEFORE quantization.  Summed in double, rounded once to float32. */
void tomref_summary_key(const float* x, int32_t G, int32_t d, float* key) {
    for (int ch = 0; ch < d; ++ch) {
        double acc = 0.0;
        for (int tok = 0; tok < G; ++tok) acc += (double)x[(int64_t)tok * d + ch];
        key[ch] = (float)(acc / (double)G);
    }
}

/* ------------------------------------------------------------------ */
/* storage offsets                                                     */
/* ------------------------------------------------------------------ */

static int64_t tile_index(const tomref_config* c, int l, int kv, int64_t t, int h) {
    return ((((int64_t)l * 2 + kv) * c->capacity_groups + t) * c->n_kv_heads + h);
}

static int config_ok(const tomref_config* c) {
    if (c->n_layers < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1 || c->head_dim < 1) return 0;
    if (c->n_q_heads % c->n_kv_heads) return 0;
    if (c->group_tokens < 1 || c->capacity_groups < 1) return 0;
    if (c->bits != 4 && c->bits != 2) return 0;
    if (c->meta_dtype != TOMREF_F32 && c->meta_dtype != TOMREF_BF16) return 0;
    if (c->head_dim % (8 / c->bits)) return 0;
    if (c->qaxis == TOMREF_QAXIS_HEAD_DIM) {
        if (c->qgroup < 1 || c->head_dim % c->qgroup) return 0;
    } else if (c->qaxis != TOMREF_QAXIS_TOKENS) return 0;
    return 1;
}

/* ------------------------------------------------------------------ */
/* the four calls, on host pointers                                    */
/* ------------------------------------------------------------------ */

/* Store step (Eq. 8): quantize n_frames frame-groups of layers
 * [layer0, layer0 + n_layers) and write them at group slots
 * first_group .. first_group + n_frames - 1, plus one summary key per
 * (layer, frame-group, head).
 *   k, v          [n_frames][n_layers][H_k][G][d] in cfg->in_dtype, addressed by
 *                 strides[4] = {frame, layer, head, token} in elements
 *                 (channel stride 1); layer index relative to layer0
 *   k_for_summary same shape/strides, NULL => k
 * Returns 0; -1 bad argument; -2 over capacity. */
int32_t tomref_quantize_append(const tomref_config* cfg, uint8_t* codes, float* scale,
                               float* zero, float* keys, int32_t first_group,
                               int32_t layer0, int32_t n_layers, int32_t n_frames,
                               const void* k, const void* v, const void* k_for_summary,
                               const int64_t strides[4]) {
    if (!config_ok(cfg) || layer0 < 0 || n_layers < 0 || layer0 + n_layers > cfg->n_layers ||
        n_frames < 0 || first_group < 0)
        return -1;
    if ((int64_t)first_group + n_frames > cfg->capacity_groups) return -2;
    const int G = cfg->group_tokens, d = cfg->head_dim, H = cfg->n_kv_heads;
    const int64_t cb = tomref_code_bytes_per_tile(G, d, cfg->bits);
    const int64_t mt = tomref_meta_per_tile(G, d, cfg->qgroup, cfg->qaxis);
    float* x = (float*)malloc(sizeof(float) * (size_t)G * d);
    float* xs = (float*)malloc(sizeof(float) * (size_t)G * d);
    if (!x || !xs) { free(x); free(xs); return -1; }
    const void* ks = k_for_summary ? k_for_summary : k;
    for (int f = 0; f < n_frames; ++f)
        for (int li = 0; li < n_layers; ++li)
            for (int h = 0; h < H; ++h) {
                const int l = layer0 + li;
                const int64_t t = (int64_t)first_group + f;
                const int64_t base = f * strides[0] + li * strides[1] + h * strides[2];
                for (int kv = 0; kv < 2; ++kv) {
                    const void* src = kv == 0 ? k : v;
                    for (int tok = 0; tok < G; ++tok)
                        for (int ch = 0; ch < d; ++ch)
                            x[(int64_t)tok * d + ch] =
                                load_elem(src, cfg->in_dtype, base + tok * strides[3] + ch);
                    const int64_t ti = tile_index(cfg, l, kv, t, h);
                    tomref_quantize_tile(x, G, d, cfg->qgroup, cfg->qaxis, cfg->bits, cfg->meta_dtype, NULL,
                                         codes + ti * cb, scale + ti * mt, zero + ti * mt);
                }
                for (int tok = 0; tok < G; ++tok)
                    for (int ch = 0; ch < d; ++ch)
                        xs[(int64_t)tok * d + ch] =
                            load_elem(ks, cfg->in_dtype, base + tok * strides[3] + ch);
                tomref_summary_key(xs, G, d,
                                   keys + (((int64_t)l * cfg->capacity_groups + t) * H + h) * d);
            }
    free(x);
    free(xs);
    return 0;
}

/* Retrieval score (Eq. 12 + supplement): for each layer, fold the query to
 * the KV-head space by averaging the r = H_q/H_k consecutive query heads of a
 * GQA group, average over the T_q query tokens, flatten [H_k][d], and compare
 * with every stored summary key (flattened the same way).
 *   q            [n_layers][H_q][T_q][d] in q_dtype
 *   scores       [n_layers][score_stride] float32, entries [0, n_groups) written
 *   token_scores NULL or [n_layers][T_q][n_groups] float32: the un-normalised
 *                dot product of query token j (GQA-folded) with key t.  Their
 *                mean over j is the numerator of the score.
 * All accumulation in double; one rounding to float32 at the end. */
int32_t tomref_score_groups(const tomref_config* cfg, const float* keys, int32_t n_groups,
                            int32_t layer0, int32_t n_layers, const void* q, int32_t q_dtype,
                            int32_t t_q, float* scores, int64_t score_stride,
                            float* token_scores) {
    if (!config_ok(cfg) || layer0 < 0 || n_layers < 0 || layer0 + n_layers > cfg->n_layers ||
        t_q < 1 || n_groups < 0 || n_groups > cfg->capacity_groups || score_stride < n_groups)
        return -1;
    const int H = cfg->n_kv_heads, Hq = cfg->n_q_heads, d = cfg->head_dim, r = Hq / H;
    const int64_t hd = (int64_t)H * d;
    double* qt = (double*)malloc(sizeof(double) * (size_t)t_q * hd);  /* q~[j][h][ch] */
    double* qb = (double*)malloc(sizeof(double) * (size_t)hd);        /* q-bar[h][ch] */
    if (!qt || !qb) { free(qt); free(qb); return -1; }
    for (int li = 0; li < n_layers; ++li) {
        const int l = layer0 + li;
        for (int h = 0; h < H; ++h)
            for (int j = 0; j < t_q; ++j)
                for (int ch = 0; ch < d; ++ch) {
                    double acc = 0.0;
                    for (int g = 0; g < r; ++g)
                        acc += (double)load_elem(
                            q, q_dtype, (((int64_t)li * Hq + (h * r + g)) * t_q + j) * d + ch);
                    qt[(int64_t)j * hd + h * d + ch] = acc / (double)r;
                }
        for (int64_t e = 0; e < hd; ++e) {
            double acc = 0.0;
            for (int j = 0; j < t_q; ++j) acc += qt[(int64_t)j * hd + e];
            qb[e] = acc / (double)t_q;
        }
        double nq = 0.0;
        for (int64_t e = 0; e < hd; ++e) nq += qb[e] * qb[e];
        nq = sqrt(nq);
        for (int t = 0; t < n_groups; ++t) {
            const float* key = keys + ((int64_t)l * cfg->capacity_groups + t) * hd;
            double dot = 0.0, nk = 0.0;
            for (int64_t e = 0; e < hd; ++e) {
                dot += qb[e] * (double)key[e];
                nk += (double)key[e] * (double)key[e];
            }
            nk = sqrt(nk);
            double s = dot;
            if (cfg->sim == TOMREF_SIM_COSINE) {
                double a = nq > 1e-12 ? nq : 1e-12, b = nk > 1e-12 ? nk : 1e-12;
                s = dot / (a * b);
            }
            scores[(int64_t)li * score_stride + t] = (float)s;
            if (token_scores)
                for (int j = 0; j < t_q; ++j) {
                    double dj = 0.0;
                    for (int64_t e = 0; e < hd; ++e) dj += qt[(int64_t)j * hd + e] * (double)key[e];
                    token_scores[((int64_t)li * t_q + j) * n_groups + t] = (float)dj;
                }
        }
    }
    free(qt);
    free(qb);
    return 0;
}

/* Top-K per row: the k_eff = min(k, n_groups) largest scores, equal scores
 * ordered by lower index first (-0 == +0).  Output row r holds k_eff indices,
 * ascending (temporal order, the paper's "sorted order") or by decreasing
 * score; entries k_eff..k-1 of the row are left untouched.
 * Returns k_eff, or -1 on a bad argument.  Plain selection sort: O(k*T). */
int32_t tomref_topk(const float* scores, int64_t score_stride, int32_t n_rows, int32_t n_groups,
                    int32_t k, int32_t order, int32_t* idx) {
    if (n_rows < 0 || n_groups < 0 || k < 1 || score_stride < n_groups) return -1;
    const int k_eff = k < n_groups ? k : n_groups;
    uint8_t* taken = (uint8_t*)malloc((size_t)(n_groups > 0 ? n_groups : 1));
    if (!taken) return -1;
    for (int r = 0; r < n_rows; ++r) {
        const float* s = scores + (int64_t)r * score_stride;
        int32_t* out = idx + (int64_t)r * k;
        memset(taken, 0, (size_t)n_groups);
        for (int j = 0; j < k_eff; ++j) {
            int best = -1;
            for (int t = 0; t < n_groups; ++t) {
                if (taken[t]) continue;
                if (best < 0 || s[t] > s[best]) best = t;   /* strict '>' keeps the lowest index */
            }
            taken[best] = 1;
            out[j] = best;                                   /* decreasing score order so far */
        }
        if (order == TOMREF_ORDER_INDEX_ASC) {
            int w = 0;
            for (int t = 0; t < n_groups; ++t)
                if (taken[t]) out[w++] = t;
        }
    }
    free(taken);
    return k_eff;
}

/* Active KV with the system-token prefix (Sec. 3.4 dual-structure memory; supplement "Cache
 * reconstruction for decoding"): per layer and head the buffer holds prefix_rows rows of
 * system tokens, copied unchanged from sys_k / sys_v ([n_layers][H_k][prefix_rows][d], out
 * dtype; NULL = rows left untouched), followed by the gathered groups as in
 * tomref_dequant_gather.  k_out, v_out: [n_layers][H_k][prefix_rows + k*G][d]. */
int32_t tomref_dequant_gather(const tomref_config* cfg, const uint8_t* codes, const float* scale,
                              const float* zero, int32_t n_groups, int32_t layer0,
                              int32_t n_layers, const int32_t* idx, int32_t k, int32_t k_eff,
                              void* k_out, void* v_out);
int32_t tomref_assemble_active(const tomref_config* cfg, const uint8_t* codes, const float* scale,
                               const float* zero, int32_t n_groups, int32_t layer0,
                               int32_t n_layers, const int32_t* idx, int32_t k, int32_t k_eff,
                               int32_t prefix_rows, const void* sys_k, const void* sys_v,
                               void* k_out, void* v_out) {
    if (!config_ok(cfg) || prefix_rows < 0 || k < 1 || n_layers < 0) return -1;
    const int G = cfg->group_tokens, d = cfg->head_dim, H = cfg->n_kv_heads;
    const size_t es = dtype_size(cfg->out_dtype);
    const int64_t head_rows = (int64_t)prefix_rows + (int64_t)k * G;
    /* gather into a plain [n_layers][H][k*G][d] buffer, then place each head block */
    const size_t plain = (size_t)n_layers * H * (size_t)k * G * d * es;
    char* tk = (char*)malloc(plain ? plain : 1);
    char* tv = (char*)malloc(plain ? plain : 1);
    if (!tk || !tv) { free(tk); free(tv); return -1; }
    int32_t rc = tomref_dequant_gather(cfg, codes, scale, zero, n_groups, layer0, n_layers, idx, k,
                                       k_eff, tk, tv);
    if (rc == 0)
        for (int li = 0; li < n_layers; ++li)
            for (int h = 0; h < H; ++h) {
                const int64_t hb = (int64_t)li * H + h;
                char* dk = (char*)k_out + (size_t)(hb * head_rows) * d * es;
                char* dv = (char*)v_out + (size_t)(hb * head_rows) * d * es;
                if (sys_k && sys_v && prefix_rows > 0) {
                    memcpy(dk, (const char*)sys_k + (size_t)(hb * prefix_rows) * d * es, (size_t)prefix_rows * d * es);
                    memcpy(dv, (const char*)sys_v + (size_t)(hb * prefix_rows) * d * es, (size_t)prefix_rows * d * es);
                }
                const size_t used = (size_t)k_eff * G * d * es;   /* rows past k_eff*G stay untouched */
                memcpy(dk + (size_t)prefix_rows * d * es, tk + (size_t)(hb * k * G) * d * es, used);
                memcpy(dv + (size_t)prefix_rows * d * es, tv + (size_t)(hb * k * G) * d * es, used);
            }
    free(tk);
    free(tv);
    return rc;
}

/* Active-KV assembly (Eq. 13): for each layer and rank r < k_eff, dequantize
 * frame-group idx[layer][r] of K and of V (Eq. 11) into rows
 * [r*G, (r+1)*G) of the layer's active buffers.
 *   idx          [n_layers][k] (row stride k), entries < n_groups
 *   k_out, v_out [n_layers][H_k][k*G][d] in cfg->out_dtype; rows >= k_eff*G
 *                are not written. */
int32_t tomref_dequant_gather(const tomref_config* cfg, const uint8_t* codes, const float* scale,
                              const float* zero, int32_t n_groups, int32_t layer0,
                              int32_t n_layers, const int32_t* idx, int32_t k, int32_t k_eff,
                              void* k_out, void* v_out) {
    if (!config_ok(cfg) || layer0 < 0 || n_layers < 0 || layer0 + n_layers > cfg->n_layers ||
        k < 1 || k_eff < 0 || k_eff > k || n_groups > cfg->capacity_groups)
        return -1;
    const int G = cfg->group_tokens, d = cfg->head_dim, H = cfg->n_kv_heads;
    const int64_t cb = tomref_code_bytes_per_tile(G, d, cfg->bits);
    const int64_t mt = tomref_meta_per_tile(G, d, cfg->qgroup, cfg->qaxis);
    const size_t es = dtype_size(cfg->out_dtype);
    float* x = (float*)malloc(sizeof(float) * (size_t)G * d);
    if (!x) return -1;
    for (int li = 0; li < n_layers; ++li)
        for (int r = 0; r < k_eff; ++r) {
            const int32_t t = idx[(int64_t)li * k + r];
            if (t < 0 || t >= n_groups) { free(x); return -1; }
            for (int kv = 0; kv < 2; ++kv)
                for (int h = 0; h < H; ++h) {
                    const int64_t ti = tile_index(cfg, layer0 + li, kv, t, h);
                    tomref_dequant_tile(codes + ti * cb, scale + ti * mt, zero + ti * mt, G, d,
                                        cfg->qgroup, cfg->qaxis, cfg->bits, x);
                    char* out = (char*)(kv == 0 ? k_out : v_out);
                    int64_t row0 = ((int64_t)li * H + h) * ((int64_t)k * G) + (int64_t)r * G;
                    tomref_from_f32(x, cfg->out_dtype, (int64_t)G * d, out + (size_t)row0 * d * es);
                }
        }
    free(x);
    return 0;
}

// Retrieval scoring on gfx950 (paper Sec. 3.4, Eq. 12; supplement
// "Question-guided single-pass retrieval").
//
//   query_fold_kernel        Q [H_q][T_q][d] -> GQA mean over the r = H_q/H_k consecutive
//                            query heads of a block, then mean over the T_q tokens.
//   score_mean_query_kernel  one dot product (and one key norm) per stored frame-group
//                            against the folded query: a float64 GEMV that streams the
//                            summary keys once; HBM-bound (H_k*d*4 bytes per group).
//   score_token_gemm_kernel  per-token scores [T_q x H_k*d] x [H_k*d x T] on the matrix
//                            cores (v_mfma_f64_16x16x4_f64), then the token mean.
//
// Everything accumulates in float64 (the CDNA vector and matrix pipes run it at
// full rate), so the float32 scores handed to top-k agree with a float64
// reference up to the final rounding, and the selected indices with them.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

// ------------------------------------------------------------------ query fold
// grid (H_k, n_layers); 256 threads = (256 / (d/8)) token lanes x (d/8) channel lanes.
template <typename QT>
__global__ void __launch_bounds__(kBlock) query_fold_kernel(const ScoreArgs a, const int want_tokens) {
    constexpr int EB = elem_bytes<QT>::value;
    const int h = blockIdx.x, li = blockIdx.y;
    const int d = a.head_dim, H = a.n_kv_heads, Hq = a.n_q_heads, Tq = a.t_q;
    const int r = Hq / H;
    const int64_t HD = (int64_t)H * d;
    const int lpr = d >> 3;
    const int jn = kBlock / lpr;
    const int tid = threadIdx.x;
    const int jl = tid / lpr;
    const int slot = tid - jl * lpr;
    const bool active = jl < jn;
    const char* q = static_cast<const char*>(a.q);

    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.0;
    const double inv_r = 1.0 / (double)r;
    if (active) {
        // Two tokens per trip; for GQA blocks of up to 8 heads all their loads are issued
        // before the first is used (one memory round trip for T_q <= 2 * jn).
        constexpr int kTok = 2, kHeads = 8;
        for (int j0 = jl; j0 < Tq; j0 += kTok * jn) {
            double qt[kTok][8];
#pragma unroll
            for (int u = 0; u < kTok; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) qt[u][i] = 0.0;
            for (int g0 = 0; g0 < r; g0 += kHeads) {
                Raw8<QT> raw[kTok][kHeads];
#pragma unroll
                for (int u = 0; u < kTok; ++u) {
                    const int j = j0 + u * jn;
#pragma unroll
                    for (int g = 0; g < kHeads; ++g) {
                        zero_raw(raw[u][g]);
                        if (j < Tq && g0 + g < r) {
                            const int64_t off =
                                (((int64_t)li * Hq + (h * r + g0 + g)) * Tq + j) * d + slot * 8;
                            load_raw(q + off * EB, raw[u][g]);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kTok; ++u)
#pragma unroll
                    for (int g = 0; g < kHeads; ++g) {
                        float x[8];
                        widen(raw[u][g], x);  // heads past the block and tokens past T_q were zero-filled
#pragma unroll
                        for (int i = 0; i < 8; ++i) qt[u][i] += (double)x[i];
                    }
            }
#pragma unroll
            for (int u = 0; u < kTok; ++u) {
                const int j = j0 + u * jn;
                if (j >= Tq) break;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    qt[u][i] = qt[u][i] * inv_r;
                    acc[i] += qt[u][i];
                }
                if (want_tokens) {
                    double* dst = a.ws_qtok + ((int64_t)li * Tq + j) * HD + (int64_t)h * d + slot * 8;
#pragma unroll
                    for (int i = 0; i < 8; ++i) dst[i] = qt[u][i];
                }
            }
        }
    }
    __shared__ double red[kBlock * 8];
    __shared__ double wsum[kBlock / 64];
    if (active) {
#pragma unroll
        for (int i = 0; i < 8; ++i) red[jl * d + i * lpr + slot] = acc[i];  // position order: no bank conflicts
    }
    __syncthreads();
    double sq = 0.0;
    for (int p = tid; p < d; p += kBlock) {  // position p = i * lpr + slot holds channel slot * 8 + i
        double sum = 0.0;
        for (int j = 0; j < jn; ++j) sum += red[j * d + p];
        const double qb = sum * (1.0 / (double)Tq);
        const int c = (p % lpr) * 8 + p / lpr;
        a.ws_qbar[(int64_t)li * HD + (int64_t)h * d + c] = qb;
        sq += qb * qb;
    }
    sq = wave_sum_f64(sq);
    if ((tid & 63) == 0) wsum[tid >> 6] = sq;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int w = 0; w < kBlock / 64; ++w) tot += wsum[w];
        a.ws_qnorm2[(int64_t)li * H + h] = tot;  // this head's share of |q-bar|^2
    }
}

// ------------------------------------------------------------------ mean-query GEMV
// Sum of a double over an aligned set of 16 lanes (DPP swaps; valid in all 16 lanes).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double row16_sum_f64(double v) {
    v += dpp_f64<0xB1>(v);   // lane ^ 1
    v += dpp_f64<0x4E>(v);   // lane ^ 2
    v += dpp_f64<0x141>(v);  // the other quad of the 8
    v += dpp_f64<0x140>(v);  // the other half of the 16
    return v;
}

constexpr int kScoreChunks = 8;  // 16-byte key loads per lane that are in flight together

// grid (ceil(T / 16), n_layers); dynamic LDS: H_k*d doubles (q-bar).  16 lanes share one
// frame-group: lane i of them takes floats [64c + 4i, 64c + 4i + 4) of the key for
// c = 0, 1, ..., so every load instruction of the 16 lanes covers 256 contiguous bytes and a
// 512-float key is fetched by one batch of 8 loads per lane.
__global__ void __launch_bounds__(kBlock) score_mean_query_kernel(const ScoreArgs a) {
    extern __shared__ double qbar[];
    const int li = blockIdx.y;
    const int HD = a.n_kv_heads * a.head_dim;
    const int tid = threadIdx.x, sub = tid & 15;
    const float* keys = a.keys + ((int64_t)(a.layer0 + li) * a.capacity_groups) * HD;
    const int t = blockIdx.x * (kBlock / 16) + (tid >> 4);
    const int tc = min(t, a.n_groups - 1);  // the tail re-reads the last group
    const float* key = keys + (int64_t)tc * HD + sub * 4;
    // The first key loads do not depend on the query: issue them before q-bar is staged.
    f32x4 kx[kScoreChunks];
    auto load_keys = [&](int e0) {
#pragma unroll
        for (int c = 0; c < kScoreChunks; ++c) {
            kx[c] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (e0 + c * 64 + sub * 4 < HD) kx[c] = *reinterpret_cast<const f32x4*>(key + e0 + c * 64);
        }
    };
    load_keys(0);

    // q-bar is staged so that the 16 lanes of a frame-group read consecutive 16-byte pairs:
    // element e = 64c + 4s + i (chunk c, lane s, i < 4) sits at ((2c + i/2) * 16 + s) * 2 + i%2
    // (in element order the lanes' pairs would be 32 bytes apart: bank conflicts on every read)
    for (int e = tid; e < HD; e += kBlock) {
        const int c = e >> 6, sl = (e >> 2) & 15, i = e & 3;
        qbar[(((2 * c + (i >> 1)) * 16 + sl) << 1) + (i & 1)] = a.ws_qbar[(int64_t)li * HD + e];
    }
    double nq2 = 0.0;
    for (int hh = 0; hh < a.n_kv_heads; ++hh) nq2 += a.ws_qnorm2[(int64_t)li * a.n_kv_heads + hh];
    const double nq = sqrt(nq2);
    __syncthreads();

    double dot = 0.0, nk2 = 0.0;
    for (int e0 = 0; e0 < HD; e0 += kScoreChunks * 64) {
        f32x4 cur[kScoreChunks];
#pragma unroll
        for (int c = 0; c < kScoreChunks; ++c) cur[c] = kx[c];
        if (e0 + kScoreChunks * 64 < HD) load_keys(e0 + kScoreChunks * 64);  // uniform
#pragma unroll
        for (int c = 0; c < kScoreChunks; ++c) {
            const int e = e0 + c * 64 + sub * 4;
            if (e < HD) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const double kd = (double)cur[c][i];
                    const double qv = qbar[(((2 * ((e0 >> 6) + c) + (i >> 1)) * 16 + sub) << 1) + (i & 1)];
                    dot = fma(qv, kd, dot);
                    nk2 = fma(kd, kd, nk2);
                }
            }
        }
    }
    dot = row16_sum_f64(dot);
    nk2 = row16_sum_f64(nk2);
    if (sub == 0 && t < a.n_groups) {
        double s = dot;
        if (a.sim == TOM_SIM_COSINE) s = dot / (fmax(nq, 1e-12) * fmax(sqrt(nk2), 1e-12));
        a.scores[(int64_t)li * a.score_stride + t] = (float)s;
    }
}

// ------------------------------------------------------------------ per-token GEMM
// S[j][t] = sum_e qtok[j][e] * key[t][e], j < T_q query tokens, t < T groups, e < H_k*d.
// Unit of work = (layer, 64 consecutive groups): one workgroup of 4 waves; wave w owns groups
// n0 + 16w .. + 15 and up to four 16-token row tiles.  Operands are staged through LDS in
// chunks of kGemmK along e.
//
// Workgroup id -> unit.  Ids go round-robin over the eight XCDs, each with its own L2, so
// XCD x is given the contiguous run of units [x * per, (x + 1) * per): it then touches the
// folded query block (T_q x H_k*d float64, 256 KB at 64 x 512) of about n_layers / 8 + 1
// layers instead of every layer's (with a (tile, layer) grid every XCD fetched every layer's
// block: 118 MB of traffic for 72 MB of operands at 28 layers x 1024 groups).
//
// v_mfma_f64_16x16x4_f64 register layout (checked on hardware by the GPU tests through
// the per-token score output): lane = 16*kk + i supplies A[i][kk] and B[kk][i]; lane
// 16*g + j holds D[4*v + g][j] in accumulator register v.
constexpr int kGemmN = 64;
constexpr int kGemmM = 64;
constexpr int kGemmK = 32;
// Row pitches of the staged operands.  A fragment read takes element (row fi, column kk) per
// lane: with 34 doubles per row the 32 lanes of a half-wave fall on 4*fi + 2*kk, i.e. on all
// 32 even banks once (a pitch of 36 puts rows fi and fi + 8 on the same banks: measured 9 %
// slower); with 36 floats per row the 64 lanes of a B read fall on 64 different banks.
constexpr int kLdA = kGemmK + 2;  // doubles
constexpr int kLdB = kGemmK + 4;  // floats

__device__ __forceinline__ int mfma_d_row(int lane, int v) { return 4 * v + (lane >> 4); }

// One staged chunk: kGemmK/4 MFMA steps for MT row tiles of 16 tokens against the 16 groups
// of this wave.  No branches inside, so the LDS reads of a step are issued together.
template <int MT>
__device__ __forceinline__ void mma_chunk(const double* __restrict__ As, const float* __restrict__ Bs,
                                          f64x4 (&acc)[MT], double& nk2c, int wave, int fi,
                                          int kk) {
#pragma unroll
    for (int ks = 0; ks < kGemmK / 4; ++ks) {
        const double bv = (double)Bs[(wave * 16 + fi) * kLdB + ks * 4 + kk];
        double av[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) av[m] = As[(m * 16 + fi) * kLdA + ks * 4 + kk];
        nk2c = fma(bv, bv, nk2c);
#pragma unroll
        for (int m = 0; m < MT; ++m)
            acc[m] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[m], bv, acc[m], 0, 0, 0);
    }
}

// One block of up to 64 query rows: the chunk loop with the row-tile count fixed at compile
// time, so the accumulators stay in place across the whole contraction.
template <int MT>
__device__ __forceinline__ void gemm_rows(const ScoreArgs& a, double (&As)[2][kGemmM * kLdA], float (&Bs)[2][kGemmN * kLdB],
                                          const double* qtok, const float* keys, int m0, int n0, int li,
                                          double& colsum, double& nk2) {
    const int HD = a.n_kv_heads * a.head_dim;
    const int T = a.n_groups, Tq = a.t_q;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fi = lane & 15, kk = lane >> 4;
    const int n_chunks = (HD + kGemmK - 1) / kGemmK;
    constexpr int kALanes = kGemmK / 2, kBLanes = kGemmK / 4;
    constexpr int kAPass = kBlock / kALanes, kBPass = kBlock / kBLanes;
    constexpr int kARows = (MT * 16 + kAPass - 1) / kAPass, kBRows = kGemmN / kBPass;
    const int a_row = tid / kALanes, a_col = (tid % kALanes) * 2;
    const int b_row = tid / kBLanes, b_col = (tid % kBLanes) * 4;
    const int rows = min(kGemmM, Tq - m0);

    f64x4 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = f64x4{0.0, 0.0, 0.0, 0.0};
    double nk2c = 0.0;
    double ra[kARows][2];
    f32x4 rb[kBRows];
    auto load_chunk = [&](int c) {
        const int k0 = c * kGemmK;
#pragma unroll
        for (int i = 0; i < kARows; ++i) {
            const int rr = a_row + i * kAPass;
            ra[i][0] = 0.0;
            ra[i][1] = 0.0;
            if (rr < rows && k0 + a_col < HD) {
                const double* p = qtok + (int64_t)(m0 + rr) * HD + k0 + a_col;
                ra[i][0] = p[0];
                ra[i][1] = p[1];
            }
        }
#pragma unroll
        for (int i = 0; i < kBRows; ++i) {
            const int rr = b_row + i * kBPass;
            rb[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (n0 + rr < T && k0 + b_col < HD)
                rb[i] = *reinterpret_cast<const f32x4*>(keys + (int64_t)(n0 + rr) * HD + k0 + b_col);
        }
    };
    auto store_chunk = [&](int stage) {
#pragma unroll
        for (int i = 0; i < kARows; ++i) {
            const int rr = a_row + i * kAPass;
            if (rr < MT * 16) {
                As[stage][rr * kLdA + a_col] = ra[i][0];
                As[stage][rr * kLdA + a_col + 1] = ra[i][1];
            }
        }
#pragma unroll
        for (int i = 0; i < kBRows; ++i) {
            const int rr = b_row + i * kBPass;
#pragma unroll
            for (int j = 0; j < 4; ++j) Bs[stage][rr * kLdB + b_col + j] = rb[i][j];
        }
    };

    __syncthreads();  // the previous row block no longer reads LDS
    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        const int stage = c & 1;
        if (c + 1 < n_chunks) load_chunk(c + 1);  // in flight during the MFMAs below
        mma_chunk<MT>(As[stage], Bs[stage], acc, nk2c, wave, fi, kk);
        if (c + 1 < n_chunks) store_chunk(stage ^ 1);  // that stage was consumed before the last barrier
        __syncthreads();
    }
    if (m0 == 0) nk2 = nk2c;
    const int t = n0 + wave * 16 + fi;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int j = m0 + m * 16 + mfma_d_row(lane, v);
            colsum += acc[m][v];  // rows >= T_q were staged as zeros
            if (a.token_scores && j < Tq && t < T)
                a.token_scores[((int64_t)li * Tq + j) * T + t] = (float)acc[m][v];
        }
    }
}

__global__ void __launch_bounds__(kBlock) score_token_gemm_kernel(const ScoreArgs a) {
    // two LDS stages: chunk c is multiplied while chunk c+1 travels global -> registers -> LDS
    __shared__ double As[2][kGemmM * kLdA];
    __shared__ float Bs[2][kGemmN * kLdB];
    const int unit = (int)(blockIdx.x & 7u) * a.gemm_units_per_xcd + (int)(blockIdx.x >> 3);
    if (unit >= a.gemm_units) return;  // uniform per workgroup
    const int li = div_by(unit, a.gemm_tiles_per_layer, a.inv_gemm_tiles_per_layer);
    const int n0 = (unit - li * a.gemm_tiles_per_layer) * kGemmN;
    const int HD = a.n_kv_heads * a.head_dim;
    const int T = a.n_groups, Tq = a.t_q;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fi = lane & 15, kk = lane >> 4;
    const float* keys = a.keys + ((int64_t)(a.layer0 + li) * a.capacity_groups) * HD;
    const double* qtok = a.ws_qtok + (int64_t)li * Tq * HD;

    double colsum = 0.0, nk2 = 0.0;
    for (int m0 = 0; m0 < Tq; m0 += kGemmM) {
        const int mt = (min(kGemmM, Tq - m0) + 15) >> 4;
        switch (mt) {  // uniform
            case 1: gemm_rows<1>(a, As, Bs, qtok, keys, m0, n0, li, colsum, nk2); break;
            case 2: gemm_rows<2>(a, As, Bs, qtok, keys, m0, n0, li, colsum, nk2); break;
            case 3: gemm_rows<3>(a, As, Bs, qtok, keys, m0, n0, li, colsum, nk2); break;
            default: gemm_rows<4>(a, As, Bs, qtok, keys, m0, n0, li, colsum, nk2); break;
        }
    }
    // lanes fi, 16 + fi, 32 + fi, 48 + fi hold the partial sums of group n0 + 16*wave + fi
    colsum += __shfl_xor(colsum, 16, 64);
    colsum += __shfl_xor(colsum, 32, 64);
    nk2 += __shfl_xor(nk2, 16, 64);
    nk2 += __shfl_xor(nk2, 32, 64);
    const int t = n0 + wave * 16 + fi;
    if (kk == 0 && t < T) {
        double s = colsum / (double)Tq;
        if (a.sim == TOM_SIM_COSINE) {
            double nq2 = 0.0;
            for (int hh = 0; hh < a.n_kv_heads; ++hh) nq2 += a.ws_qnorm2[(int64_t)li * a.n_kv_heads + hh];
            s = s / (fmax(sqrt(nq2), 1e-12) * fmax(sqrt(nk2), 1e-12));
        }
        a.scores[(int64_t)li * a.score_stride + t] = (float)s;
    }
}

}  // namespace

hipError_t launch_query_fold(const ScoreArgs& a, bool want_tokens, hipStream_t s) {
    if (a.n_layers == 0) return hipSuccess;
    const dim3 grid(a.n_kv_heads, a.n_layers);
    switch (a.q_dtype) {
        case TOM_F32: query_fold_kernel<In_f32><<<grid, dim3(kBlock), 0, s>>>(a, want_tokens); break;
        case TOM_BF16: query_fold_kernel<In_bf16><<<grid, dim3(kBlock), 0, s>>>(a, want_tokens); break;
        case TOM_F16: query_fold_kernel<In_f16><<<grid, dim3(kBlock), 0, s>>>(a, want_tokens); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_score_mean_query(const ScoreArgs& a, hipStream_t s) {
    if (a.n_layers == 0 || a.n_groups == 0) return hipSuccess;
    const int per_block = kBlock / 16;
    const dim3 grid((a.n_groups + per_block - 1) / per_block, a.n_layers);
    // q-bar, padded to whole 64-element chunks (the staged order permutes within a chunk)
    const size_t lds = (size_t)((a.n_kv_heads * a.head_dim + 63) / 64 * 64) * sizeof(double);
    score_mean_query_kernel<<<grid, dim3(kBlock), lds, s>>>(a);
    return hipGetLastError();
}

}  // namespace oqm

namespace oqm {
hipError_t launch_score_token_gemm(const ScoreArgs& args, hipStream_t s) {
    if (args.n_layers == 0 || args.n_groups == 0) return hipSuccess;
    ScoreArgs a = args;
    a.gemm_tiles_per_layer = (a.n_groups + kGemmN - 1) / kGemmN;
    a.inv_gemm_tiles_per_layer = reciprocal_u32((uint32_t)a.gemm_tiles_per_layer);
    const int64_t units = (int64_t)a.gemm_tiles_per_layer * a.n_layers;
    if (units > 0x7fffffffLL - 8) return hipErrorInvalidValue;  // 2^25 tiles x 65535 layers at most: never
    a.gemm_units = (int32_t)units;
    a.gemm_units_per_xcd = (int32_t)((units + 7) / 8);
    score_token_gemm_kernel<<<dim3(8u * (unsigned)a.gemm_units_per_xcd), dim3(kBlock), 0, s>>>(a);
    return hipGetLastError();
}
}  // namespace oqm

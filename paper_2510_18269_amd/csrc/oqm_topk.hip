// Selection of the k best frame-groups per layer (paper Eq. 12 TopK; the
// supplement keeps the selected indices in sorted, i.e. temporal, order).
//
// One workgroup of 1024 threads per row.  The k-th largest score is found by a
// 4-pass, 8-bit most-significant-digit radix select over order-preserving
// 32-bit keys (LDS histograms), which is O(T) and exact.  The winners are then
// compacted in index order with wave ballots, which yields the ascending-index
// output directly and resolves equal scores by lowest index: of the entries
// equal to the threshold only the first `need` (by index) are taken.  For the
// score-descending order the k winners are sorted with an LDS bitonic network.
// The step is latency-bound: T <= a few thousand scores per row.
#include "oqm_common.h"
#include "oqm_device.h"

namespace oqm {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kCachedKeys = 2 * kTopkMaxSortedK;  // keys kept in LDS when the row fits

// Larger float <=> larger unsigned key; -0 and +0 map to the same key.
__device__ __forceinline__ uint32_t orderable(float s) {
    const uint32_t u = __float_as_uint(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(kTopkThreads)
topk_kernel(const float* __restrict__ scores, const int64_t stride, const int n, const int k,
            const int k_eff, const int order, int32_t* __restrict__ idx) {
    __shared__ uint64_t buf[kTopkMaxSortedK];  // cached keys first, sort buffer later
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wcnt_g[kTopkWaves], wcnt_e[kTopkWaves];
    __shared__ uint32_t s_prefix, s_remaining;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* s = scores + (int64_t)blockIdx.x * stride;
    int32_t* out = idx + (int64_t)blockIdx.x * k;
    uint32_t* skeys = reinterpret_cast<uint32_t*>(buf);
    const bool cached = n <= kCachedKeys;
    if (cached)
        for (int i = tid; i < n; i += kTopkThreads) skeys[i] = orderable(s[i]);
    __syncthreads();
    auto key_at = [&](int i) -> uint32_t { return cached ? skeys[i] : orderable(s[i]); };

    // ---- radix select: key value of the k_eff-th largest, and how many of its equals to take
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k_eff;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += kTopkThreads) {
            const uint32_t key = key_at(i);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane L owns bins 255-4L .. 252-4L; scan from the largest digit downwards
            uint32_t c[4], tot = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = hist[255 - (4 * lane + j)];
                tot += c[j];
            }
            uint32_t incl = tot;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t v = __shfl_up(incl, off, 64);
                if (lane >= off) incl += v;
            }
            const uint32_t excl = incl - tot;
            if (excl < remaining && remaining <= incl) {  // exactly one lane
                uint32_t cum = excl;
                int bsel = 3;
                bool found = false;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (!found) {
                        if (remaining <= cum + c[j]) {
                            bsel = j;
                            found = true;
                        } else {
                            cum += c[j];
                        }
                    }
                }
                s_prefix = prefix | ((uint32_t)(255 - (4 * lane + bsel)) << shift);
                s_remaining = remaining - cum;
            }
        }
        __syncthreads();
        prefix = s_prefix;
        remaining = s_remaining;
        mask |= 0xFFu << shift;
    }
    const uint32_t thr = prefix;
    const uint32_t need = remaining;  // entries equal to thr to take, lowest index first

    // ---- ordered compaction: winners in ascending index order
    uint32_t base_g = 0, base_e = 0;
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int c0 = 0; c0 < n; c0 += kTopkThreads) {
        const int i = c0 + tid;
        const bool valid = i < n;
        const uint32_t key = valid ? key_at(i) : 0u;
        const bool gt = valid && key > thr;
        const bool eq = valid && key == thr;
        const uint64_t bg = __ballot(gt), be = __ballot(eq);
        if (lane == 0) {
            wcnt_g[wave] = (uint32_t)__popcll(bg);
            wcnt_e[wave] = (uint32_t)__popcll(be);
        }
        __syncthreads();
        uint32_t og = base_g + (uint32_t)__popcll(bg & lt);
        uint32_t oe = base_e + (uint32_t)__popcll(be & lt);
        uint32_t tg = 0, te = 0;
#pragma unroll
        for (int w = 0; w < kTopkWaves; ++w) {
            const uint32_t g = wcnt_g[w], e = wcnt_e[w];
            if (w < wave) {
                og += g;
                oe += e;
            }
            tg += g;
            te += e;
        }
        if (gt)
            out[og + (oe < need ? oe : need)] = i;
        else if (eq && oe < need)
            out[og + oe] = i;
        base_g += tg;
        base_e += te;
        __syncthreads();
    }
    if (order != TOM_ORDER_SCORE_DESC) return;

    // ---- best-first order: bitonic sort of (key, ~index) pairs, descending
    int p2 = 1;
    while (p2 < k_eff) p2 <<= 1;
    uint64_t comp[kTopkMaxSortedK / kTopkThreads];
    __threadfence_block();
#pragma unroll
    for (int u = 0; u < kTopkMaxSortedK / kTopkThreads; ++u) {
        const int j = u * kTopkThreads + tid;
        comp[u] = 0;
        if (j < k_eff) {
            const int i = out[j];
            comp[u] = ((uint64_t)key_at(i) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)i);
        }
    }
    __syncthreads();  // all reads of the cached keys are done: the buffer changes role
#pragma unroll
    for (int u = 0; u < kTopkMaxSortedK / kTopkThreads; ++u) {
        const int j = u * kTopkThreads + tid;
        if (j < p2) buf[j] = comp[u];
    }
    __syncthreads();
    for (int size = 2; size <= p2; size <<= 1) {
        for (int strd = size >> 1; strd > 0; strd >>= 1) {
            for (int j = tid; j < p2; j += kTopkThreads) {
                const int partner = j ^ strd;
                if (partner > j) {
                    const bool desc = (j & size) == 0;
                    const uint64_t x = buf[j], y = buf[partner];
                    if ((x < y) == desc) {
                        buf[j] = y;
                        buf[partner] = x;
                    }
                }
            }
            __syncthreads();
        }
    }
    for (int j = tid; j < k_eff; j += kTopkThreads)
        out[j] = (int32_t)(0xFFFFFFFFu - (uint32_t)(buf[j] & 0xFFFFFFFFull));
}

}  // namespace

hipError_t launch_topk(const float* scores, int64_t stride, int n_rows, int n_groups, int k,
                       int k_eff, int order, int32_t* idx, hipStream_t s) {
    if (n_rows == 0 || k_eff == 0) return hipSuccess;
    topk_kernel<<<dim3(n_rows), dim3(kTopkThreads), 0, s>>>(scores, stride, n_groups, k, k_eff,
                                                            order, idx);
    return hipGetLastError();
}

}  // namespace oqm

// Selection (Alg. 1: recent set, TopK, union): per (batch, KV head) the
// budget - recent highest scores among the non-recent tokens, ties to the
// lower position, written as ascending token positions followed by the recent
// positions.
//
// One workgroup of 1024 threads per problem; each thread owns a contiguous
// range of token positions whose scores, turned into order-preserving 32-bit
// keys, stay in registers.  The key of the last selected element is found by
//   1. the key range [kmin, kmax] of the problem (one block reduction);
//   2. ONE histogram of 4096 bins that are linear in key - kmin over exactly
//      that range, so the keys spread over the bins whatever their exponents
//      (few same-address LDS atomics), and a block-wide suffix scan that finds
//      the bin holding the threshold;
//   3. an exact rank among the (typically few dozen) keys of that bin, kept in
//      LDS; if the bin is crowded (many equal or nearly equal scores) the low
//      bits are resolved by 8-bit radix rounds instead.
// An ordered compaction (one block-wide scan) then writes the indices in
// ascending order.  Sequences too long for the register file (more than 64
// keys per thread) re-read the scores from memory in every pass.
#include <type_traits>

#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;
constexpr int kBins = 4096;      // first-round bins
constexpr int kHistCopies = 2;   // waves alternate between copies
constexpr int kCandMax = 1024;   // keys of the threshold bin ranked directly

__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct TopkSmem {
    int hist[kHistCopies][kBins];
    unsigned long long cand[kCandMax];  // key << 32 | ~position: descending = selection order
    uint32_t red[2][kTopkWaves];
    int wsum[kTopkWaves];
    int scan[2][kTopkWaves];
    int bin, need, ncand;
    uint32_t T;
};

// Block-wide: given per-thread counts `loc` of consecutive, ascending key ranges (thread
// t covers lower keys than thread t+1), find the thread whose range holds the need-th
// largest key.  Returns the number of keys in the ranges above this thread's.
__device__ __forceinline__ int suffix_above(int loc, int lane, int wave, int *wsum) {
    int suf = loc;  // inclusive suffix sum within the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_down(suf, o);
        if (lane + o < 64) suf += t;
    }
    if (lane == 0) wsum[wave] = suf;
    __syncthreads();
    int above = suf - loc;
    for (int w = wave + 1; w < kTopkWaves; ++w) above += wsum[w];
    __syncthreads();
    return above;
}

// ITEMS > 0: keys of positions [tid*ITEMS, tid*ITEMS+ITEMS) live in registers.
// ITEMS == 0: keys are re-read (thread tid owns [tid*ipt, tid*ipt+ipt)).
// `sink`: positions below it are retained without being ranked (their keys are the padding
// key 0, which is never counted), like the `recent` last positions.
template <int ITEMS>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float *__restrict__ scores,
                                                            int n, int budget, int recent,
                                                            int sink, int32_t *__restrict__ idx) {
    extern __shared__ __attribute__((aligned(16))) char topk_smem[];
    TopkSmem &sm = *(TopkSmem *)topk_smem;

    const int z = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sc = scores + (int64_t)z * n;
    int32_t *out = idx + (int64_t)z * budget + sink;  // the ranked part starts behind the sinks
    const int n_cand = n - recent;
    const int k = budget - recent - sink;

    for (int t = tid; t < sink; t += kTopkThreads) out[t - sink] = t;
    for (int t = tid; t < recent; t += kTopkThreads) out[k + t] = n_cand + t;
    if (k == 0) return;

    constexpr int R = ITEMS > 0 ? ITEMS : 1;
    // one bit per register-resident key
    using Mask = std::conditional_t<(ITEMS > 32), unsigned long long, unsigned>;
    auto lowest = [](Mask m) { return sizeof(Mask) == 8 ? __ffsll((unsigned long long)m) - 1 : __ffs((unsigned)m) - 1; };
    auto popcount = [](Mask m) { return sizeof(Mask) == 8 ? __popcll((unsigned long long)m) : __popc((unsigned)m); };
    const int ipt = ITEMS > 0 ? ITEMS : (n_cand + kTopkThreads - 1) / kTopkThreads;
    const int j0 = min(tid * ipt, n_cand), j1 = min(j0 + ipt, n_cand);
    uint32_t key[R];
    if (ITEMS > 0) {
        // a key of 0 sorts below every real key (real keys have a bit set) and is never counted
        if (ITEMS % 4 == 0 && (((uintptr_t)(sc + j0)) & 15) == 0 && j0 + ITEMS <= n_cand) {
#pragma unroll
            for (int t = 0; t < R / 4; ++t) {
                const float4 v = *(const float4 *)(sc + j0 + 4 * t);
                key[4 * t] = order_key(v.x); key[4 * t + 1] = order_key(v.y);
                key[4 * t + 2] = order_key(v.z); key[4 * t + 3] = order_key(v.w);
            }
        } else {
#pragma unroll
            for (int t = 0; t < R; ++t) key[t] = j0 + t < j1 ? order_key(sc[j0 + t]) : 0u;
        }
        if (j0 < sink) {
#pragma unroll
            for (int t = 0; t < R; ++t) key[t] = j0 + t < sink ? 0u : key[t];
        }
    }
    // visit every owned key: f(key, position)
    auto for_keys = [&](auto f) {
        if (ITEMS > 0) {
#pragma unroll
            for (int t = 0; t < R; ++t)
                if (j0 + t < j1 && j0 + t >= sink) f(key[t], j0 + t);
        } else {
            for (int j = max(j0, sink); j < j1; ++j) f(order_key(sc[j]), j);
        }
    };

    // 1. range of the keys
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    for_keys([&](uint32_t u, int) { kmin = min(kmin, u); kmax = max(kmax, u); });
    kmin = reduce_lanes<1, 64>(kmin, OpMinU{});
    kmax = reduce_lanes<1, 64>(kmax, OpMaxU{});
    if (lane == 0) { sm.red[0][wave] = kmin; sm.red[1][wave] = kmax; }
    for (int t = tid; t < kHistCopies * kBins; t += kTopkThreads) (&sm.hist[0][0])[t] = 0;
    if (tid == 0) sm.ncand = 0;
    __syncthreads();
    kmin = sm.red[0][0]; kmax = sm.red[1][0];
#pragma unroll
    for (int w = 1; w < kTopkWaves; ++w) { kmin = min(kmin, sm.red[0][w]); kmax = max(kmax, sm.red[1][w]); }

    uint32_t T = kmax;  // key of the last selected element
    int need = k;       // how many keys equal to T are selected (lowest positions first)
    if (kmin != kmax) {
        // 2. one histogram, linear in key - kmin, over the occupied range only
        const uint32_t range = kmax - kmin;
        const int sh = max(0, 32 - __clz(range) - 12);  // (range >> sh) < 4096
        int *hist = sm.hist[wave & (kHistCopies - 1)];
        for_keys([&](uint32_t u, int) { atomicAdd(&hist[(u - kmin) >> sh], 1); });
        __syncthreads();
        int cb[4], loc = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            cb[t] = 0;
#pragma unroll
            for (int c = 0; c < kHistCopies; ++c) cb[t] += sm.hist[c][4 * tid + t];
            loc += cb[t];
        }
        int above = suffix_above(loc, lane, wave, sm.wsum);
        if (above < need && need <= above + loc) {
#pragma unroll
            for (int t = 3; t >= 0; --t) {
                if (above < need && need <= above + cb[t]) {
                    sm.bin = 4 * tid + t;
                    sm.need = need - above;
                    sm.ncand = cb[t];  // keys in the threshold bin
                }
                above += cb[t];
            }
        }
        __syncthreads();
        const uint32_t bin = (uint32_t)sm.bin;
        need = sm.need;
        const int nc = sm.ncand;
        __syncthreads();
        if (sh == 0) {
            T = kmin + bin;  // bins are single keys
        } else if (nc <= kCandMax) {
            // 3a. exact rank among the keys of the threshold bin
            if (tid == 0) sm.ncand = 0;
            __syncthreads();
            if (ITEMS > 0) {
                // mark the thread's keys of that bin, reserve their slots with one atomic
                Mask cm = 0;
#pragma unroll
                for (int t = 0; t < R; ++t)
                    cm |= (Mask)(key[t] != 0u && ((key[t] - kmin) >> sh) == bin) << t;
                if (cm) {
                    int slot = atomicAdd(&sm.ncand, popcount(cm));
                    while (cm) {
                        const int t = lowest(cm);
                        cm &= cm - 1;
                        uint32_t u = 0;
#pragma unroll
                        for (int q = 0; q < R; ++q) u = q == t ? key[q] : u;
                        sm.cand[slot++] = ((unsigned long long)u << 32) | (uint32_t)(~(j0 + t));
                    }
                }
            } else {
                for_keys([&](uint32_t u, int j) {
                    if (((u - kmin) >> sh) == bin) {
                        const int slot = atomicAdd(&sm.ncand, 1);
                        sm.cand[slot] = ((unsigned long long)u << 32) | (uint32_t)(~j);
                    }
                });
            }
            __syncthreads();
            if (tid < nc) {
                const unsigned long long mine = sm.cand[tid];
                int rank = 0;  // number of candidates selected before this one
                int u = 0;
                for (; u + 4 <= nc; u += 4)
                    rank += (sm.cand[u] > mine) + (sm.cand[u + 1] > mine) + (sm.cand[u + 2] > mine) +
                            (sm.cand[u + 3] > mine);
                for (; u < nc; ++u) rank += sm.cand[u] > mine;
                if (rank == need - 1) sm.T = (uint32_t)(mine >> 32);
            }
            __syncthreads();
            T = sm.T;
            need = -1;  // number of selected keys equal to T: known once the keys above T are counted
        } else {
            // 3b. crowded bin: 8-bit radix rounds over the low `sh` bits of key - kmin
            uint32_t prefix = bin << sh;
            for (int shift = ((sh - 1) / 8) * 8; shift >= 0; shift -= 8) {
                __syncthreads();
                if (tid < 256) { sm.hist[0][tid] = 0; sm.hist[1][tid] = 0; }
                __syncthreads();
                const uint32_t hi_mask = 0xffffffffu << min(shift + 8, 31);  // sh <= 20: never 32
                for_keys([&](uint32_t u, int) {
                    const uint32_t rel = u - kmin;
                    if ((rel >> sh) == bin && (rel & hi_mask) == (prefix & hi_mask))
                        atomicAdd(&hist[(rel >> shift) & 255u], 1);
                });
                __syncthreads();
                int c = 0;
                if (tid < 256) c = sm.hist[0][tid] + sm.hist[1][tid];
                const int ab = suffix_above(c, lane, wave, sm.wsum);  // threads >= 256 hold 0
                if (tid < 256 && ab < need && need <= ab + c) { sm.bin = tid; sm.need = need - ab; }
                __syncthreads();
                prefix |= (uint32_t)sm.bin << shift;
                need = sm.need;
            }
            T = kmin + prefix;
        }
    }

    // ordered compaction
    int gt = 0, eq = 0;
    Mask gtm = 0, eqm = 0;  // register-resident keys above / equal to T (padding keys are 0 < T)
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < R; ++t) {
            gtm |= (Mask)(key[t] > T) << t;
            eqm |= (Mask)(key[t] == T) << t;
        }
        gt = popcount(gtm);
        eq = popcount(eqm);
    } else {
        for_keys([&](uint32_t u, int) { gt += u > T; eq += u == T; });
    }
    // inclusive scans over the wave; with keys in registers both counts (at most 64 per
    // thread, 4096 per wave) share one word
    int gi = gt, ei = eq;
    if (ITEMS > 0) {
        int pk = gt | (eq << 16);
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int a = __shfl_up(pk, o);
            if (lane >= o) pk += a;
        }
        gi = pk & 0xffff;
        ei = pk >> 16;
    } else {
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int a = __shfl_up(gi, o), b = __shfl_up(ei, o);
            if (lane >= o) { gi += a; ei += b; }
        }
    }
    __syncthreads();
    if (lane == 63) { sm.scan[0][wave] = gi; sm.scan[1][wave] = ei; }
    __syncthreads();
    int gbase = 0, ebase = 0, gtotal = 0;
    for (int w = 0; w < kTopkWaves; ++w) {
        if (w < wave) { gbase += sm.scan[0][w]; ebase += sm.scan[1][w]; }
        gtotal += sm.scan[0][w];
    }
    if (need < 0) need = k - gtotal;
    int gtc = gbase + gi - gt, eqc = ebase + ei - eq;  // exclusive prefixes
    // the k indices are gathered in LDS (the histogram is dead by now) and then written out
    // with consecutive lanes on consecutive addresses; beyond the staging capacity each
    // thread writes its own
    int *stage = &sm.hist[0][0];
    const bool staged = k <= kHistCopies * kBins;
    auto emit = [&](auto *dst) {
        if (ITEMS > 0) {
            // selected keys of this thread: all above T and, among those equal to T, the
            // ones within the first `need` of the problem; visited in position order
            Mask sel = gtm;
            int quota = need - eqc;
            for (Mask m = eqm; m != 0 && quota > 0; m &= m - 1, --quota) sel |= m & (~m + 1);
            int o = gtc + min(eqc, need);
            while (sel) {
                dst[o++] = j0 + lowest(sel);
                sel &= sel - 1;
            }
        } else {
            for_keys([&](uint32_t u, int j) {
                if (u > T) {
                    dst[gtc + min(eqc, need)] = j;
                    ++gtc;
                } else if (u == T) {
                    if (eqc < need) dst[gtc + eqc] = j;
                    ++eqc;
                }
            });
        }
    };
    if (staged) {
        emit(stage);
        __syncthreads();
        for (int t = tid; t < k; t += kTopkThreads) out[t] = stage[t];
    } else {
        emit(out);
    }
}

template <int ITEMS>
static void launch_items(const float *scores, int Z, int n, int budget, int recent, int sink,
                         int32_t *idx, hipStream_t st) {
    hipLaunchKernelGGL(topk_kernel<ITEMS>, dim3(Z), dim3(kTopkThreads), sizeof(TopkSmem), st, scores,
                       n, budget, recent, sink, idx);
}

// Scores smoothed over tokens before the selection (caption of the method's overview
// figure): average pool of odd width, stride 1, mean over the taps inside the sequence.
// The pooled value decides which tokens are kept, so it is formed exactly as stated - the
// taps added left to right in fp32, then one division - and not by a running sum.
__global__ __launch_bounds__(256) void pool_scores_kernel(const float *__restrict__ scores, int n,
                                                          int half, float *__restrict__ pooled) {
    const int z = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const float *s = scores + (int64_t)z * n;
    const int lo = max(0, j - half), hi = min(n - 1, j + half);
    float acc = 0.f;
    for (int t = lo; t <= hi; ++t) acc = __fadd_rn(acc, s[t]);
    pooled[(int64_t)z * n + j] = __fdiv_rn(acc, (float)(hi - lo + 1));
}

hipError_t launch_topk(const float *scores, int Z, int n, int budget, int recent, int sink,
                       int pool, float *pooled, int32_t *idx, hipStream_t st) {
    static_assert(sizeof(TopkSmem) < 64 * 1024, "top-k LDS must fit the default dynamic limit");
    if (pool > 1) {
        hipLaunchKernelGGL(pool_scores_kernel, dim3((n + 255) / 256, Z), dim3(256), 0, st, scores, n,
                           (pool - 1) / 2, pooled);
        scores = pooled;
    }
    const int n_cand = n - recent;
    const int ipt = (n_cand + kTopkThreads - 1) / kTopkThreads;
    if (ipt <= 4) launch_items<4>(scores, Z, n, budget, recent, sink, idx, st);
    else if (ipt <= 8) launch_items<8>(scores, Z, n, budget, recent, sink, idx, st);
    else if (ipt <= 16) launch_items<16>(scores, Z, n, budget, recent, sink, idx, st);
    else if (ipt <= 32) launch_items<32>(scores, Z, n, budget, recent, sink, idx, st);
    else if (ipt <= 64) launch_items<64>(scores, Z, n, budget, recent, sink, idx, st);
    else launch_items<0>(scores, Z, n, budget, recent, sink, idx, st);
    return hipGetLastError();
}

}  // namespace aha

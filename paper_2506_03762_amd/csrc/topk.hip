// Selection (Alg. 1: recent set, TopK, union): per (batch, KV head) the
// budget - recent highest scores among the non-recent tokens, ties to the
// lower position, written as ascending token positions followed by the recent
// positions.
//
// One workgroup of 1024 threads per problem.  Scores become order-preserving
// 32-bit keys that stay in registers (each thread owns a contiguous range of
// token positions); a radix select (8-bit digits, per-wave LDS histograms)
// finds the key of the last selected element, starting at the highest bit in
// which the keys of this problem differ at all, so that the first digit
// already spreads over the bins.  An ordered compaction (one block-wide scan)
// then writes the indices in ascending order.  Sequences too long for the
// register file (more than 64 keys per thread) re-read the scores from memory
// in every round instead.
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;

__device__ __forceinline__ uint32_t order_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Histogram increment with wave-level aggregation: lanes that hit the bin of the first
// still-active lane are counted with one ballot and added by a single LDS atomic.  Two
// such rounds absorb the hot bins (scores of one head crowd into a few exponents); the
// lanes that are left add on their own.
__device__ __forceinline__ void hist_add(int *hist, uint32_t bin, bool valid, int lane) {
    unsigned long long active = __ballot(valid);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        if (active == 0) break;  // wave-uniform
        const int leader = __ffsll((long long)active) - 1;
        const uint32_t lbin = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
        const unsigned long long same = __ballot(valid && bin == lbin);
        if (lane == leader) atomicAdd(&hist[lbin], __popcll(same));
        if (bin == lbin) valid = false;
        active &= ~same;
    }
    if (valid) atomicAdd(&hist[bin], 1);
}

// ITEMS > 0: keys of positions [tid*ITEMS, tid*ITEMS+ITEMS) live in registers.
// ITEMS == 0: keys are re-read (thread tid owns [tid*ipt, tid*ipt+ipt)).
template <int ITEMS>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float *__restrict__ scores,
                                                            int n, int budget, int recent,
                                                            int32_t *__restrict__ idx) {
    __shared__ int s_hist[kTopkWaves][256];
    __shared__ int s_tot[256];
    __shared__ uint32_t s_red[2][kTopkWaves];
    __shared__ int s_digit, s_need;
    __shared__ int s_scan[2][kTopkWaves];

    const int z = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sc = scores + (int64_t)z * n;
    int32_t *out = idx + (int64_t)z * budget;
    const int n_cand = n - recent;
    const int k = budget - recent;

    for (int t = tid; t < recent; t += kTopkThreads) out[k + t] = n_cand + t;
    if (k == 0) return;

    constexpr int R = ITEMS > 0 ? ITEMS : 1;
    const int ipt = ITEMS > 0 ? ITEMS : (n_cand + kTopkThreads - 1) / kTopkThreads;
    const int j0 = min(tid * ipt, n_cand), j1 = min(j0 + ipt, n_cand);
    uint32_t key[R];
    if (ITEMS > 0) {
        // a key of 0 sorts below every real key (real keys have a bit set) and is never counted
#pragma unroll
        for (int t = 0; t < R; ++t) key[t] = j0 + t < j1 ? order_key(sc[j0 + t]) : 0u;
    }

    // range of the keys
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < R; ++t)
            if (j0 + t < j1) { kmin = min(kmin, key[t]); kmax = max(kmax, key[t]); }
    } else {
        for (int j = j0; j < j1; ++j) {
            const uint32_t u = order_key(sc[j]);
            kmin = min(kmin, u);
            kmax = max(kmax, u);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
    }
    if (lane == 0) { s_red[0][wave] = kmin; s_red[1][wave] = kmax; }
    __syncthreads();
    kmin = s_red[0][0]; kmax = s_red[1][0];
#pragma unroll
    for (int w = 1; w < kTopkWaves; ++w) { kmin = min(kmin, s_red[0][w]); kmax = max(kmax, s_red[1][w]); }

    uint32_t prefix = kmax;  // bits above the current digit are final
    int need = k;            // how many still to take among keys matching the prefix
    if (kmin != kmax) {
        const int hb = 31 - __clz(kmin ^ kmax);  // highest differing bit
        for (int shift = (hb / 8) * 8; shift >= 0; shift -= 8) {
            for (int t = tid; t < kTopkWaves * 256; t += kTopkThreads) (&s_hist[0][0])[t] = 0;
            __syncthreads();
            const uint32_t hi_mask = shift >= 24 ? 0u : (0xffffffffu << (shift + 8));
            const uint32_t want = prefix & hi_mask;
            if (ITEMS > 0) {
#pragma unroll
                for (int t = 0; t < R; ++t)
                    hist_add(s_hist[wave], (key[t] >> shift) & 255u,
                             j0 + t < j1 && (key[t] & hi_mask) == want, lane);
            } else {
                for (int t = 0; t < ipt; ++t) {  // same trip count in every lane
                    const int j = j0 + t;
                    const uint32_t u = j < j1 ? order_key(sc[j]) : 0u;
                    hist_add(s_hist[wave], (u >> shift) & 255u, j < j1 && (u & hi_mask) == want, lane);
                }
            }
            __syncthreads();
            if (tid < 256) {
                int c = 0;
#pragma unroll
                for (int w = 0; w < kTopkWaves; ++w) c += s_hist[w][tid];
                s_tot[tid] = c;
            }
            __syncthreads();
            if (wave == 0) {
                int cb[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) cb[t] = s_tot[4 * lane + t];
                const int loc = cb[0] + cb[1] + cb[2] + cb[3];
                int suf = loc;  // inclusive suffix sum over lanes
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const int t = __shfl_down(suf, o);
                    if (lane + o < 64) suf += t;
                }
                int above = suf - loc;
                if (above < need && need <= suf) {
#pragma unroll
                    for (int t = 3; t >= 0; --t) {
                        if (above < need && need <= above + cb[t]) {
                            s_digit = 4 * lane + t;
                            s_need = need - above;
                        }
                        above += cb[t];
                    }
                }
            }
            __syncthreads();
            const uint32_t dmask = 255u << shift;
            prefix = (prefix & ~dmask) | ((uint32_t)s_digit << shift);
            need = s_need;
            __syncthreads();
        }
    }
    const uint32_t T = prefix;  // key of the last selected element; take `need` of its equals

    // ordered compaction
    int gt = 0, eq = 0;
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < R; ++t) { gt += key[t] > T; eq += key[t] == T; }
    } else {
        for (int j = j0; j < j1; ++j) {
            const uint32_t u = order_key(sc[j]);
            gt += u > T;
            eq += u == T;
        }
    }
    int gi = gt, ei = eq;  // inclusive scans over the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int a = __shfl_up(gi, o), b = __shfl_up(ei, o);
        if (lane >= o) { gi += a; ei += b; }
    }
    if (lane == 63) { s_scan[0][wave] = gi; s_scan[1][wave] = ei; }
    __syncthreads();
    int gbase = 0, ebase = 0;
    for (int w = 0; w < wave; ++w) { gbase += s_scan[0][w]; ebase += s_scan[1][w]; }
    int gtc = gbase + gi - gt, eqc = ebase + ei - eq;  // exclusive prefixes
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < R; ++t) {
            if (key[t] > T) {
                out[gtc + min(eqc, need)] = j0 + t;
                ++gtc;
            } else if (key[t] == T) {
                if (eqc < need) out[gtc + eqc] = j0 + t;
                ++eqc;
            }
        }
    } else {
        for (int j = j0; j < j1; ++j) {
            const uint32_t u = order_key(sc[j]);
            if (u > T) {
                out[gtc + min(eqc, need)] = j;
                ++gtc;
            } else if (u == T) {
                if (eqc < need) out[gtc + eqc] = j;
                ++eqc;
            }
        }
    }
}

hipError_t launch_topk(const float *scores, int Z, int n, int budget, int recent, int32_t *idx,
                       hipStream_t st) {
    const int n_cand = n - recent;
    const int ipt = (n_cand + kTopkThreads - 1) / kTopkThreads;
    dim3 grid(Z), block(kTopkThreads);
    if (ipt <= 4)
        hipLaunchKernelGGL(topk_kernel<4>, grid, block, 0, st, scores, n, budget, recent, idx);
    else if (ipt <= 8)
        hipLaunchKernelGGL(topk_kernel<8>, grid, block, 0, st, scores, n, budget, recent, idx);
    else if (ipt <= 16)
        hipLaunchKernelGGL(topk_kernel<16>, grid, block, 0, st, scores, n, budget, recent, idx);
    else if (ipt <= 32)
        hipLaunchKernelGGL(topk_kernel<32>, grid, block, 0, st, scores, n, budget, recent, idx);
    else if (ipt <= 64)
        hipLaunchKernelGGL(topk_kernel<64>, grid, block, 0, st, scores, n, budget, recent, idx);
    else
        hipLaunchKernelGGL(topk_kernel<0>, grid, block, 0, st, scores, n, budget, recent, idx);
    return hipGetLastError();
}

}  // namespace aha

// fp32 eviction scores (Sec. 4.1 - 4.3; Alg. 1 Prefill), plain vector-ALU
// kernels.  This is the small-problem, high-accuracy path (fp32 Q/K/V); the
// bf16 path in score_bf16.hip carries the throughput.
//
// Pass 1: one workgroup per observed query row finds max_j and log2-sum-exp2
//         of t_ij = s_i * log2(e) * (Q_i . K_j) over j <= i.
// Pass 2: one thread per key keeps its K row in registers and sums
//         exp2(t_ij - L_i) over the observed rows i >= j.
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

// A running statistic (m, s, u) of scaled logits t: m = max t, s = sum exp2(t - m),
// u = sum exp2(t - m) (t - m).  The row's entropy is ln 2 * (log2 s - u / s) (Sec. 4.2).
// Re-referenced to a maximum M >= m it is (M, s f, (u + (m - M) s) f) with f = 2^(m - M).
__device__ __forceinline__ void reref_stat(float m, float M, float &s, float &u) {
    if (m == -INFINITY) { s = 0.f; u = 0.f; return; }
    const float f = exp2f(m - M);
    u = (u + (m - M) * s) * f;
    s *= f;
}

// `lse_out` / `ent_out` (either may be null): natural-log normaliser and entropy of every
// observed row, dense [batch, Hq, window].
template <int D>
__global__ __launch_bounds__(256) void f32_pass1_kernel(ScoreGeom g, float *rowL, float *lse_out,
                                                        float *ent_out) {
    const int z = blockIdx.y, rho = blockIdx.x, tid = threadIdx.x;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const RowMap rm{g.n, g.r, g.R,
                    g.rows ? g.rows + ((int64_t)b * g.Hq + (int64_t)h * g.G) * g.r : nullptr};
    const int i = rm.pos(rho);
    const int hq = h * g.G + rm.head(rho);
    const float *qrow = (const float *)g.q + b * g.qs[0] + hq * g.qs[1] + (int64_t)i * g.qs[2];
    const float *kbase = (const float *)g.k + b * g.ks[0] + h * g.ks[1];

    __shared__ float s_q[D];
    __shared__ float s_m[4], s_s[4], s_u[4];
    if (tid < D) s_q[tid] = qrow[tid];
    __syncthreads();
    const float lam = row_scale_log2(g.scale_mode, g.fixed_scale, g.lambda_floor, i + 1,
                                     g.budget, g.d);

    float m = -INFINITY, s = 0.f, u = 0.f;
    for (int j = tid; j <= i; j += 256) {
        const float4 *kr = (const float4 *)(kbase + (int64_t)j * g.ks[2]);
        float w = 0.f;
#pragma unroll 8
        for (int c = 0; c < D / 4; ++c) {
            const float4 kv = kr[c];
            w = fmaf(s_q[4 * c + 0], kv.x, w);
            w = fmaf(s_q[4 * c + 1], kv.y, w);
            w = fmaf(s_q[4 * c + 2], kv.z, w);
            w = fmaf(s_q[4 * c + 3], kv.w, w);
        }
        const float t = w * lam;
        const float mn = fmaxf(m, t);
        reref_stat(m, mn, s, u);
        const float e = exp2f(t - mn);
        s += e;
        u = fmaf(e, t - mn, u);
        m = mn;
    }
    // combine the per-thread statistics
    const float wm = wave_max(m);
    reref_stat(m, wm, s, u);
    const float ws = wave_sum(s), wu = wave_sum(u);
    if ((tid & 63) == 0) { s_m[tid >> 6] = wm; s_s[tid >> 6] = ws; s_u[tid >> 6] = wu; }
    __syncthreads();
    if (tid == 0) {
        const float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
        float S = 0.f, U = 0.f;
        for (int t = 0; t < 4; ++t) {
            float st = s_s[t], ut = s_u[t];
            reref_stat(s_m[t], M, st, ut);
            S += st;
            U += ut;
        }
        const float L = M + log2f(S);
        rowL[(int64_t)z * g.R + rho] = L;
        const int64_t o = ((int64_t)b * g.Hq + hq) * g.r + (rho % g.r);
        const float kLn2 = 0.69314718055994531f;
        if (lse_out) lse_out[o] = L * kLn2;
        if (ent_out) ent_out[o] = fmaxf(0.f, (log2f(S) - U / S) * kLn2);
    }
}

constexpr int kF32QRows = 16;  // query rows staged in LDS per step of pass 2

template <int D>
__global__ __launch_bounds__(256) void f32_pass2_kernel(ScoreGeom g, const float *rowL,
                                                        const float *gamma,
                                                        const float *gblockmax, int n_vtiles,
                                                        float *scores) {
    const int z = blockIdx.y, tid = threadIdx.x;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int j = blockIdx.x * 256 + tid;
    const RowMap rm{g.n, g.r, g.R,
                    g.rows ? g.rows + ((int64_t)b * g.Hq + (int64_t)h * g.G) * g.r : nullptr};
    const float *kbase = (const float *)g.k + b * g.ks[0] + h * g.ks[1];

    __shared__ float s_q[kF32QRows][D];
    __shared__ float s_lam[kF32QRows], s_L[kF32QRows];
    __shared__ int s_pos[kF32QRows];

    float kreg[D];
    {
        const int jj = j < g.n ? j : g.n - 1;
        const float4 *kr = (const float4 *)(kbase + (int64_t)jj * g.ks[2]);
#pragma unroll
        for (int c = 0; c < D / 4; ++c) {
            const float4 kv = kr[c];
            kreg[4 * c] = kv.x; kreg[4 * c + 1] = kv.y; kreg[4 * c + 2] = kv.z; kreg[4 * c + 3] = kv.w;
        }
    }
    const int j_lo = blockIdx.x * 256;  // smallest key of this workgroup
    float acc = 0.f;
    for (int r0 = 0; r0 < g.R; r0 += kF32QRows) {
        // rows of this step; skip steps whose rows all lie before the block's keys
        if (rm.max_pos(r0, r0 + kF32QRows) < j_lo) continue;
        __syncthreads();
        for (int t = tid; t < kF32QRows * D; t += 256) {
            const int rr = t / D, c = t % D, rho = r0 + rr;
            float qv = 0.f;
            if (rho < g.R) {
                const int hq = h * g.G + rm.head(rho);
                qv = ((const float *)g.q)[b * g.qs[0] + hq * g.qs[1] +
                                           (int64_t)rm.pos(rho) * g.qs[2] + c];
            }
            s_q[rr][c] = qv;
        }
        if (tid < kF32QRows) {
            const int rho = r0 + tid;
            const int i = rm.pos(rho);
            s_pos[tid] = i;
            s_lam[tid] = rho < g.R ? row_scale_log2(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                   i + 1, g.budget, g.d)
                                  : 0.f;
            s_L[tid] = rho < g.R ? rowL[(int64_t)z * g.R + rho] : INFINITY;
        }
        __syncthreads();
        for (int rr = 0; rr < kF32QRows; ++rr) {
            float w = 0.f;
#pragma unroll
            for (int c = 0; c < D; ++c) w = fmaf(s_q[rr][c], kreg[c], w);
            const float p = exp2f(fmaf(w, s_lam[rr], -s_L[rr]));
            acc += (j <= s_pos[rr]) ? p : 0.f;
        }
    }
    if (j < g.n) {
        float out = acc;
        if (g.value_prior) {
            float gm = 0.f;
            for (int t = 0; t < n_vtiles; ++t) gm = fmaxf(gm, gblockmax[z * n_vtiles + t]);
            out = gm > 0.f ? acc * (gamma[(int64_t)z * g.n + j] / gm) : acc;  // all-zero values: no prior
        }
        scores[(int64_t)z * g.n + j] = out;
    }
}

hipError_t launch_score_f32(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                            hipStream_t st, hipEvent_t mid, bool have_lse) {
    char *w = (char *)ws;
    float *rowL = (float *)(w + pl.off_rowL);
    const float *gamma = (const float *)(w + pl.off_gamma);
    const float *gbm = (const float *)(w + pl.off_gblockmax);
    dim3 g1(g.R, pl.Z), g2((g.n + 255) / 256, pl.Z);
    if (g.d == 64) {
        if (!have_lse)
            hipLaunchKernelGGL(f32_pass1_kernel<64>, g1, dim3(256), 0, st, g, rowL, (float *)nullptr,
                               (float *)nullptr);
        if (mid) (void)hipEventRecord(mid, st);
        hipLaunchKernelGGL(f32_pass2_kernel<64>, g2, dim3(256), 0, st, g, rowL, gamma, gbm,
                           pl.n_vtiles, scores);
    } else {
        if (!have_lse)
            hipLaunchKernelGGL(f32_pass1_kernel<128>, g1, dim3(256), 0, st, g, rowL, (float *)nullptr,
                               (float *)nullptr);
        if (mid) (void)hipEventRecord(mid, st);
        hipLaunchKernelGGL(f32_pass2_kernel<128>, g2, dim3(256), 0, st, g, rowL, gamma, gbm,
                           pl.n_vtiles, scores);
    }
    return hipGetLastError();
}

hipError_t launch_row_stats_f32(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *lse,
                                float *entropy, hipStream_t st) {
    float *rowL = (float *)((char *)ws + pl.off_rowL);
    dim3 g1(g.R, pl.Z);
    if (g.d == 64)
        hipLaunchKernelGGL(f32_pass1_kernel<64>, g1, dim3(256), 0, st, g, rowL, lse, entropy);
    else
        hipLaunchKernelGGL(f32_pass1_kernel<128>, g1, dim3(256), 0, st, g, rowL, lse, entropy);
    return hipGetLastError();
}

}  // namespace aha

// Value prior (Sec. 4.3): nu_j = ||V_j||^2, gamma = average pool of nu over
// tokens (odd width, stride 1, mean over the in-range taps), and the per-tile
// maxima of gamma from which the consumers form gamma / max(gamma).
//
// HBM-bound: V is read exactly once (plus (pool-1)/2 halo rows per tile).
// The windowed bf16 scores form the prior inside their row-statistics launch
// (score_bf16.hip) and do not use this kernel; it serves the fp32 path, full
// accumulation (where it also zeroes the scores) and the entry point that is
// handed the rows' normalisers (which it converts for the column-sum pass).
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

// One workgroup = kVTileRows consecutive tokens of one (batch, KV head).
// 16-byte loads; LPR lanes cover one row.
template <int ESIZE>
__global__ __launch_bounds__(256) void vprior_kernel(ScoreGeom g, int n_vtiles, float *gamma,
                                                     float *gblockmax,
                                                     float *zero_scores, const float *lse,
                                                     float *row_stats, int rows_pad) {
    const int z = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
    if (lse) {
        // the caller's row normalisers (natural log, [batch, Hq, window]) -> log2 domain, in
        // the order of the flattened query rows of each KV head (padding rows: unused)
        const int b = z / g.Hkv, h = z % g.Hkv;
        for (int rho = tile * 256 + tid; rho < rows_pad; rho += gridDim.x * 256) {
            float L = 0.f;
            if (rho < g.R) {
                const int gi = rho / g.r, ii = rho - gi * g.r;
                L = lse[((int64_t)b * g.Hq + h * g.G + gi) * g.r + ii] * kLog2e;
            }
            row_stats[(int64_t)z * rows_pad + rho] = L;
        }
    }
    if (zero_scores && tile < n_vtiles) {
        // full accumulation adds tile contributions atomically: the scores start from zero
        const int j = tile * kVTileRows + tid;
        if (j < g.n) zero_scores[(int64_t)z * g.n + j] = 0.f;
    }
    if (!g.value_prior || tile >= n_vtiles) return;

    __shared__ float s_nu[kVTileRows + 256];
    __shared__ float s_max[4];
    const int b = z / g.Hkv, h = z % g.Hkv;
    const char *vbase =
        (const char *)g.v + (int64_t)ESIZE * (b * g.vs[0] + h * g.vs[1]);
    const int half = (g.pool - 1) / 2;
    const int t0 = tile * kVTileRows;
    const int lo = max(0, t0 - half);
    const int hi = min(g.n, t0 + kVTileRows + half);  // exclusive
    value_norms_to_lds<ESIZE>(vbase, g.vs[2], g.d, lo, hi, s_nu, tid);
    __syncthreads();

    const int j = t0 + tid;
    float gam = 0.f;
    if (j < g.n) {
        const int a = max(0, j - half), e = min(g.n - 1, j + half);
        float s = 0.f;
        for (int t = a; t <= e; ++t) s += s_nu[t - lo];
        gam = s / (float)(e - a + 1);
        gamma[(int64_t)z * g.n + j] = gam;
    }
    float m = wave_max(gam);
    if ((tid & 63) == 0) s_max[tid >> 6] = m;
    __syncthreads();
    if (tid == 0)
        gblockmax[z * n_vtiles + tile] = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
}

hipError_t launch_value_prior(const ScoreGeom &g, const PrefillPlan &pl, void *ws,
                              float *scores, const float *lse, bool prior_here, hipStream_t st) {
    char *w = (char *)ws;
    float *gamma = (float *)(w + pl.off_gamma);
    float *gbm = (float *)(w + pl.off_gblockmax);
    // bf16 full accumulation (several query tiles) needs zeroed scores
    float *zero_scores = (g.dtype == AHA_BF16 && pl.n_qtiles > 1) ? scores : nullptr;
    if (!prior_here && !zero_scores && !lse) return hipSuccess;  // nothing for this launch to do
    ScoreGeom gl = g;
    gl.value_prior = prior_here ? 1 : 0;
    const int vt = (prior_here || zero_scores) ? pl.n_vtiles : 1;
    dim3 grid(vt, pl.Z);
    // where pass 2 reads the row statistics: one chunk per (problem, tile, row) on the bf16
    // path (rows padded to whole tiles), one value per row on the fp32 path
    float *row_stats = (float *)(w + (g.dtype == AHA_BF16 ? pl.off_partial : pl.off_rowL));
    const int rows_pad = g.dtype == AHA_BF16 ? pl.n_qtiles * pl.qtile : g.R;
    if (g.dtype == AHA_BF16)
        hipLaunchKernelGGL(vprior_kernel<2>, grid, dim3(256), 0, st, gl, pl.n_vtiles, gamma, gbm,
                           zero_scores, lse, row_stats, rows_pad);
    else
        hipLaunchKernelGGL(vprior_kernel<4>, grid, dim3(256), 0, st, gl, pl.n_vtiles, gamma, gbm,
                           zero_scores, lse, row_stats, rows_pad);
    return hipGetLastError();
}

}  // namespace aha

// Value prior (Sec. 4.3): nu_j = ||V_j||^2, gamma = average pool of nu over
// tokens (odd width, stride 1, mean over the in-range taps), and the per-tile
// maxima of gamma from which the consumers form gamma / max(gamma).
//
// HBM-bound: V is read exactly once (plus (pool-1)/2 halo rows per tile).
// The same launch tabulates the softmax scale of every window row (evaluated
// in double), so no separate set-up launch is needed.
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

// One workgroup = kVTileRows consecutive tokens of one (batch, KV head).
// 16-byte loads; LPR lanes cover one row.
template <int ESIZE>
__global__ __launch_bounds__(256) void vprior_kernel(ScoreGeom g, int n_vtiles, float *gamma,
                                                     float *gblockmax, float *lam_tab,
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
    if (z == 0) {
        // softmax scale of window row ii (token position n - r + ii, c = position + 1 keys)
        const int ii = tile * 256 + tid;
        if (ii < g.r)
            lam_tab[ii] = ESIZE == 2 ? row_scale_log2_f32(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                          g.n - g.r + ii + 1, g.budget, g.d)
                                     : row_scale_log2(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                      g.n - g.r + ii + 1, g.budget, g.d);
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
    const int lpr = g.d * ESIZE / 16;                 // lanes per row: 8, 16 or 32
    const int rows_per_pass = 256 / lpr;
    const int sub = tid % lpr, rloc = tid / lpr;

    // V is read exactly once, with streaming loads: kept out of the caches it leaves them to
    // the keys, which the two score passes read twice (pass 1 ran 5 % faster at the
    // full-depth shape; the same hint on pass 2's key loads made that pass 35 % slower).
    // nine independent 16-byte loads in flight per lane: with 16 lanes per row a tile and
    // its pooling halo (256 + 6 rows) then take two batches, not three (many more in flight
    // measured slower at the large shapes)
    constexpr int U = 9;
    for (int row0 = lo + rloc; row0 < hi; row0 += U * rows_per_pass) {
        u32x4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = min(row0 + u * rows_per_pass, hi - 1);
            w[u] = __builtin_nontemporal_load((const u32x4 *)(vbase + (int64_t)ESIZE * row * g.vs[2] + sub * 16));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float s = 0.f;
            if (ESIZE == 2) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    float a = bf16_lo(w[u][t]), c = bf16_hi(w[u][t]);
                    s = fmaf(a, a, s);
                    s = fmaf(c, c, s);
                }
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    float a = __uint_as_float(w[u][t]);
                    s = fmaf(a, a, s);
                }
            }
            // over the lanes of the row (8, 16 or 32 of them)
            s = reduce_lanes<1, 8>(s, OpSum{});
            if (lpr >= 16) s = combine_lane_xor<8>(s, OpSum{});
            if (lpr >= 32) s = combine_lane_xor<16>(s, OpSum{});
            const int row = row0 + u * rows_per_pass;
            if (sub == 0 && row < hi) s_nu[row - lo] = s;
        }
    }
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
                              float *scores, const float *lse, hipStream_t st) {
    char *w = (char *)ws;
    float *gamma = (float *)(w + pl.off_gamma);
    float *gbm = (float *)(w + pl.off_gblockmax);
    float *lam_tab = (float *)(w + pl.off_lam);
    const int lam_blocks = (g.r + 255) / 256;
    // bf16 full accumulation (several query tiles) needs zeroed scores
    float *zero_scores = (g.dtype == AHA_BF16 && pl.n_qtiles > 1) ? scores : nullptr;
    const int vt = (g.value_prior || zero_scores) ? pl.n_vtiles : 1;
    dim3 grid(vt > lam_blocks ? vt : lam_blocks, pl.Z);
    // where pass 2 reads the row statistics: one chunk per (problem, tile, row) on the bf16
    // path (rows padded to whole tiles), one value per row on the fp32 path
    float *row_stats = (float *)(w + (g.dtype == AHA_BF16 ? pl.off_partial : pl.off_rowL));
    const int rows_pad = g.dtype == AHA_BF16 ? pl.n_qtiles * pl.qtile : g.R;
    if (g.dtype == AHA_BF16)
        hipLaunchKernelGGL(vprior_kernel<2>, grid, dim3(256), 0, st, g, pl.n_vtiles, gamma, gbm,
                           lam_tab, zero_scores, lse, row_stats, rows_pad);
    else
        hipLaunchKernelGGL(vprior_kernel<4>, grid, dim3(256), 0, st, g, pl.n_vtiles, gamma, gbm,
                           lam_tab, zero_scores, lse, row_stats, rows_pad);
    return hipGetLastError();
}

}  // namespace aha

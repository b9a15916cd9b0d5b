// Compaction (Alg. 1 Generation: K_S, V_S; F_0 = refined prefill score):
// gather the retained K/V rows of every (batch, KV head) into the budgeted
// cache.  Pure copy, HBM-bound: each retained row is read once and written
// once with 16-byte accesses, the lanes of a row adjacent.
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

template <int ESIZE>
__global__ __launch_bounds__(256) void compact_kernel(ScoreGeom g, const float *__restrict__ scores,
                                                      const int32_t *__restrict__ idx, int budget,
                                                      int slots, char *__restrict__ kc,
                                                      char *__restrict__ vc, float *__restrict__ fc,
                                                      int32_t *__restrict__ pos,
                                                      int32_t *__restrict__ free_slot) {
    const int z = blockIdx.y, tid = threadIdx.x;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int row_bytes = g.d * ESIZE;
    const int lpr = row_bytes / 16;
    const int s = blockIdx.x * (256 / lpr) + tid / lpr, sub = tid % lpr;
    if (blockIdx.x == 0 && tid == 0) free_slot[z] = budget;
    if (s >= slots) return;
    u32x4 kw = {0u, 0u, 0u, 0u}, vw = {0u, 0u, 0u, 0u};
    int j = -1;
    if (s < budget) {
        j = idx[(int64_t)z * budget + s];
        const char *ks = (const char *)g.k + (int64_t)ESIZE * (b * g.ks[0] + h * g.ks[1] + (int64_t)j * g.ks[2]);
        const char *vs = (const char *)g.v + (int64_t)ESIZE * (b * g.vs[0] + h * g.vs[1] + (int64_t)j * g.vs[2]);
        kw = *(const u32x4 *)(ks + sub * 16);
        vw = *(const u32x4 *)(vs + sub * 16);
    }
    const int64_t drow = ((int64_t)z * slots + s) * row_bytes + sub * 16;
    // streaming stores: the cache rows are written once and not read back by this launch;
    // kept out of the caches they do not turn into write-backs under the next kernel's
    // reads (the value-prior launch of the next layer ran 30 % faster at the full-depth shape)
    __builtin_nontemporal_store(kw, (u32x4 *)(kc + drow));
    __builtin_nontemporal_store(vw, (u32x4 *)(vc + drow));
    if (sub == 0) {
        fc[(int64_t)z * slots + s] = j >= 0 ? scores[(int64_t)z * g.n + j] : 0.f;
        pos[(int64_t)z * slots + s] = j;
    }
}

hipError_t launch_compact(const ScoreGeom &g, const float *scores, const int32_t *idx, int budget,
                          int slots, int dtype, void *kc, void *vc, float *fc, int32_t *pos,
                          int32_t *free_slot, hipStream_t st) {
    const int esize = dtype == AHA_BF16 ? 2 : 4;
    const int rows_per_wg = 256 / (g.d * esize / 16);
    dim3 grid((slots + rows_per_wg - 1) / rows_per_wg, g.batch * g.Hkv);
    if (dtype == AHA_BF16)
        hipLaunchKernelGGL(compact_kernel<2>, grid, dim3(256), 0, st, g, scores, idx, budget, slots,
                           (char *)kc, (char *)vc, fc, pos, free_slot);
    else
        hipLaunchKernelGGL(compact_kernel<4>, grid, dim3(256), 0, st, g, scores, idx, budget, slots,
                           (char *)kc, (char *)vc, fc, pos, free_slot);
    return hipGetLastError();
}

}  // namespace aha

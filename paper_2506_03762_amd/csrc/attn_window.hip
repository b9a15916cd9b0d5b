// Attention output of the observed rows, O_i = sum_{j <= i} softmax_j(Q_i . K_j / sqrt(d)) V_j
// for the last `window` query positions, and those rows' log-sum-exp: the self-attention
// that the eviction score is computed beside (appendix on compatibility with
// FlashAttention; Alg. 1 Prefill forms both from the same logits).  The log-sum-exp is what
// aha_prefill_scores_lse takes, so this launch plus the column-sum pass give output and
// scores with one pass over the keys each.
//
// bf16: a flash-style single pass on the matrix cores, in the orientation of the score
// kernels (keys on M, queries on N).  A workgroup owns one block of 32 flattened query rows
// of a KV head and a range of keys; each of its four waves takes 64-key blocks:
//   S^T = K Q^T            v_mfma_f32_32x32x16_bf16, A = key fragments from global memory
//   online softmax         per query column = per lane (the two half-waves of a column share
//                          their running maximum every block)
//   O^T += V^T P^T         the same MFMA; B = the probabilities, converted to bf16 where they
//                          sit: accumulator elements 8 ks .. 8 ks + 7 of a lane are exactly the
//                          eight keys of contraction step ks that the lane supplies; A = V^T,
//                          gathered from a wave-private copy of the 64 value rows in LDS in
//                          that same key order (the contraction may run over the keys in any
//                          order as long as both operands agree).
// The waves' partial outputs (each relative to its own maximum) meet in LDS, the key ranges'
// in the workspace, and a small second launch normalises.
// fp32 (the small high-accuracy path): plain vector-ALU kernel, one workgroup per row.
#include "score_tile.h"

namespace aha {

template <int D>
struct AttnSmem {
    using T = TileSmem<D, 1>;
    static constexpr int LDV = D + 8;  // padded value row (elements): 16-byte aligned rows
    static constexpr size_t v_bytes = (size_t)kWaveKeys * LDV * 2;  // one wave's 64 value rows
    static constexpr size_t off_v = (T::bytes + 15) / 16 * 16;
    static constexpr size_t bytes = off_v + 4 * v_bytes;
    static constexpr int LDO = D + 1;  // padded row of a wave's partial output (floats)
    static_assert((size_t)32 * LDO * 4 <= v_bytes, "a wave's partial output reuses its value rows");
    static_assert(4 * 32 * sizeof(float2) <= T::q_bytes, "the waves' statistics reuse the query tile");
};

// The wave's 64 value rows [kb, kb + 64) -> its private LDS copy, row-major, 16-byte chunks,
// the lanes of a row adjacent.  Rows at or past `end` re-read row end - 1 (their
// probabilities are zero).  Request (global memory -> registers) and commit (-> LDS) are
// apart, so that the logits and the softmax of the step cover the round trip to memory.
template <int D>
struct ValueRows {
    static constexpr int CPR = D / 8, RPI = 64 / CPR, NI = kWaveKeys / RPI, LDV = AttnSmem<D>::LDV;
    u32x4 w[NI];
    __device__ __forceinline__ void request(const __bf16 *vbase, int64_t v_tstride, int kb, int end,
                                            int lane) {
        const int r0 = lane / CPR, c = lane % CPR;
#pragma unroll
        for (int t = 0; t < NI; ++t)
            w[t] = *(const u32x4 *)(vbase + (int64_t)min(kb + t * RPI + r0, end - 1) * v_tstride + c * 8);
    }
    __device__ __forceinline__ void commit(int lane, __bf16 *sV) const {
        const int r0 = lane / CPR, c = lane % CPR;
#pragma unroll
        for (int t = 0; t < NI; ++t) *(u32x4 *)(sV + (t * RPI + r0) * LDV + c * 8) = w[t];
    }
};

// A fragment of V^T for channel block cb, key block mb, contraction step ks: this lane's
// channel cb * 32 + lane % 32 of the eight keys that its accumulator elements 8 ks .. 8 ks + 7
// of key block mb stand for (rows mb * 32 + 16 ks + 8 (e / 4) + e % 4 + 4 (lane / 32)).
template <int D>
__device__ __forceinline__ bf16x8 value_fragment(const __bf16 *sV, int mb, int ks, int cb,
                                                 int lane) {
    constexpr int LDV = AttnSmem<D>::LDV;
    const uint16_t *p = (const uint16_t *)sV + (4 * (lane >> 5)) * LDV + (lane & 31);
    u32x4 w;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const int r0 = mb * 32 + 16 * ks + 8 * (e >> 2) + (e & 3);
        const uint32_t lo = p[r0 * LDV + cb * 32], hi = p[(r0 + 1) * LDV + cb * 32];
        w[e / 2] = lo | (hi << 16);
    }
    bf16x8 f;
    __builtin_memcpy(&f, &w, 16);
    return f;
}

template <int D>
__global__ __launch_bounds__(256, 2) void window_attn_kernel(ScoreGeom g, int n_blocks, int nparts,
                                                             int units, float *part_o,
                                                             float2 *part_ms) {
    using S = TileSmem<D, 1>;
    using A = AttnSmem<D>;
    constexpr int CB = D / 32;  // 32-channel blocks of the output
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __bf16 *sQ = (__bf16 *)smem;
    float *sLam = (float *)(smem + S::q_bytes);
    int *sPos = (int *)(sLam + S::ROWS);
    int *sBlk = sPos + 2 * S::ROWS;

    // The workgroups of one (problem, key range) - one per block of 32 query rows - re-read
    // the same keys and values: they get indices that are congruent modulo 8, i.e. one XCD
    // and one L2 (workgroups are dealt round-robin to the 8 XCDs).
    const int id = (int)blockIdx.x, xcd = id % kXcds, t = id / kXcds;
    const int nbk = t % n_blocks, u = (t / n_blocks) * kXcds + xcd;
    if (u >= units) return;
    const int part = u % nparts, z = u / nparts;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowMap rm{g.n, g.r, g.R, nullptr};
    const int rho0 = nbk * 32;
    const int end = rm.max_pos(rho0, rho0 + 32) + 1;  // the keys this block of rows may see
    const int steps = (end + kWgKeys - 1) / kWgKeys;
    const int key_begin = (int)((int64_t)part * steps / nparts) * kWgKeys;
    const int key_end = min(end, (int)((int64_t)(part + 1) * steps / nparts) * kWgKeys);
    const int64_t pidx = ((int64_t)(z * nparts + part) * n_blocks + nbk) * 32;
    if (key_begin >= key_end) {  // more ranges than this block has key steps: a neutral partial
        for (int i = tid; i < 32 * D; i += 256) part_o[pidx * D + i] = 0.f;
        if (tid < 32) part_ms[pidx + tid] = make_float2(-INFINITY, 0.f);
        return;
    }
    const __bf16 *kbase = (const __bf16 *)g.k + b * g.ks[0] + h * g.ks[1];
    const __bf16 *vbase = (const __bf16 *)g.v + b * g.vs[0] + h * g.vs[1];
    const float c_out = kLog2e * rsqrtf((float)D);
    {
        QTileRegs<D, 1> qt;
        q_tile_request<D, 1>(g, b, h, rho0, tid, qt);
        q_tile_meta<D, 1>(g, rm, rho0, tid, c_out, sLam, sPos, sBlk);
        q_tile_commit<D, 1>(qt, tid, sQ);
    }
    __syncthreads();
    const int pos = sPos[lane & 31];
    const int bmax = uniform(sBlk[0]), bmin = uniform(sBlk[1]);
    __bf16 *sV = (__bf16 *)(smem + A::off_v + wave * A::v_bytes);

    f32x16 O[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[cb][v] = 0.f;
    float m = -INFINITY, s = 0.f;  // running maximum (log2 domain) and sum of this lane's keys

    // The key fragments of a step are requested during the step before it, right after that
    // step's logits have consumed the registers; the value rows at the start of their step,
    // committed to LDS after its softmax.  (All requests are unconditional and clamped to the
    // key range: behind a branch the compiler would wait for them at once.)
    bf16x8 a[kMB][D / 16];
    load_a<D>(kbase, g.ks[2], min(key_begin + wave * kWaveKeys, key_end), key_end, lane, a);
    for (int kb0 = key_begin; kb0 < key_end; kb0 += kWgKeys) {
        const int kb = kb0 + wave * kWaveKeys;
        const bool live = kb < key_end && kb <= bmax;  // (wave-uniform; no barrier inside the loop)
        ValueRows<D> vr;
        vr.request(vbase, g.vs[2], min(kb, key_end), key_end, lane);
        f32x16 acc[kMB];
        mma_block<D, 1>(a, sQ, 0, lane, acc);
        __builtin_amdgcn_sched_barrier(0);
        load_a<D>(kbase, g.ks[2], min(kb + kWgKeys, key_end), key_end, lane, a);
        __builtin_amdgcn_sched_barrier(0);
        if (!live) continue;
        // causal limit and the ragged end of the key range
        if (kb + kWaveKeys - 1 > bmin || kb + kWaveKeys > key_end) {
#pragma unroll
            for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = acc_key(kb, mb, v, lane);
                    if (key > pos || key >= key_end) acc[mb][v] = -INFINITY;
                }
        }
        float amax = -INFINITY;
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) amax = fmaxf(amax, acc[mb][v]);
        // the two half-waves hold different keys of the same query column: one maximum
        amax = combine_lane_xor<32>(amax, OpMax{});
        const float mn = fmaxf(m, amax == -INFINITY ? -INFINITY : amax * c_out);
        const float mref = mn == -INFINITY ? 0.f : mn;
        const float corr = fast_exp2(m - mref);  // 0 while the column has seen no key
        float sum[2] = {0.f, 0.f};
        bf16x8 pf[kMB][2];  // the probabilities as B fragments of the two contraction steps
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float pr = fast_exp2(fmaf(acc[mb][8 * ks + e], c_out, -mref));
                    sum[e & 1] += pr;
                    pf[mb][ks][e] = (__bf16)pr;
                }
        s = s * corr + (sum[0] + sum[1]);
        m = mn;
        vr.commit(lane, sV);
        if (__builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {  // (rarely after the first blocks)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) O[cb][v] *= corr;
        }
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    O[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        value_fragment<D>(sV, mb, ks, cb, lane), pf[mb][ks], O[cb], 0, 0, 0);
    }

    // ---- the four waves' partials (different keys, own maxima) meet in LDS ----
    s += __shfl_xor(s, 32);  // the column's sum over both half-waves
    __syncthreads();         // the query tile and the value rows are done with
    float *sO = (float *)(smem + A::off_v + wave * A::v_bytes);
    float2 *sMS = (float2 *)smem;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            sO[(lane & 31) * A::LDO + cb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] = O[cb][v];
    if (lane < 32) sMS[wave * 32 + lane] = make_float2(m, s);
    __syncthreads();
    for (int i = tid; i < 32 * D; i += 256) {
        const int q = i / D, ch = i % D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sMS[w * 32 + q].x);
        const float mref = M == -INFINITY ? 0.f : M;
        float o = 0.f, ssum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float2 ms = sMS[w * 32 + q];
            const float f = fast_exp2(ms.x - mref);
            const float *wO = (const float *)(smem + A::off_v + w * A::v_bytes);
            o = fmaf(f, wO[q * A::LDO + ch], o);
            ssum = fmaf(f, ms.y, ssum);
        }
        part_o[(pidx + q) * D + ch] = o;
        if (ch == 0) part_ms[pidx + q] = make_float2(M, ssum);
    }
}

// Second launch: the key ranges' partials of every observed row -> the normalised output in
// the inputs' dtype and the row's natural-log normaliser.  256 / D rows per workgroup.
template <int D>
__global__ __launch_bounds__(256) void window_attn_merge_kernel(ScoreGeom g, int n_blocks,
                                                                int nparts, const float *part_o,
                                                                const float2 *part_ms,
                                                                uint16_t *out, float *lse) {
    const int z = blockIdx.y, rho = blockIdx.x * (256 / D) + threadIdx.x / D, ch = threadIdx.x % D;
    if (rho >= g.R) return;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int nbk = rho / 32, q = rho % 32;
    float M = -INFINITY;
    for (int p = 0; p < nparts; ++p)
        M = fmaxf(M, part_ms[((int64_t)(z * nparts + p) * n_blocks + nbk) * 32 + q].x);
    float o = 0.f, ssum = 0.f;
    for (int p = 0; p < nparts; ++p) {
        const int64_t pi = ((int64_t)(z * nparts + p) * n_blocks + nbk) * 32 + q;
        const float2 ms = part_ms[pi];
        const float f = exp2f(ms.x - M);  // (every row sees key 0: M is finite)
        o = fmaf(f, part_o[pi * D + ch], o);
        ssum = fmaf(f, ms.y, ssum);
    }
    const int gi = rho / g.r, ii = rho - gi * g.r;
    const int64_t row = ((int64_t)b * g.Hq + h * g.G + gi) * g.r + ii;
    out[row * D + ch] = (uint16_t)f32_to_bf16_rne(o / ssum);
    if (lse && ch == 0) lse[row] = (M + log2f(ssum)) * 0.69314718055994531f;
}

// ------------------------------------------------------------------ fp32 --
// One workgroup per observed row; keys in blocks of 256 (one per thread: dot product, block
// maximum, probabilities into LDS), then every thread adds its channel's share of the block
// (thread = channel c of key slice t / D) with the usual rescaling by the running maximum.
template <int D>
__global__ __launch_bounds__(256) void f32_window_attn_kernel(ScoreGeom g, float *out, float *lse) {
    constexpr int SL = 256 / D;  // key slices of a block
    const int z = blockIdx.y, rho = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const RowMap rm{g.n, g.r, g.R, nullptr};
    const int i = rm.pos(rho);
    const int hq = h * g.G + rm.head(rho);
    const float *qrow = (const float *)g.q + b * g.qs[0] + hq * g.qs[1] + (int64_t)i * g.qs[2];
    const float *kbase = (const float *)g.k + b * g.ks[0] + h * g.ks[1];
    const float *vbase = (const float *)g.v + b * g.vs[0] + h * g.vs[1];
    __shared__ float s_q[D], s_p[256], s_red[4], s_o[SL][D];
    if (tid < D) s_q[tid] = qrow[tid];
    __syncthreads();
    const float c_out = kLog2e * rsqrtf((float)D);
    const int c = tid % D, sl = tid / D;
    float m = -INFINITY, ssum = 0.f, o = 0.f;  // m, ssum uniform over the workgroup
    for (int j0 = 0; j0 <= i; j0 += 256) {
        const int j = j0 + tid;
        float t = -INFINITY;
        if (j <= i) {
            const float4 *kr = (const float4 *)(kbase + (int64_t)j * g.ks[2]);
            float w = 0.f;
#pragma unroll 8
            for (int cc = 0; cc < D / 4; ++cc) {
                const float4 kv = kr[cc];
                w = fmaf(s_q[4 * cc + 0], kv.x, w);
                w = fmaf(s_q[4 * cc + 1], kv.y, w);
                w = fmaf(s_q[4 * cc + 2], kv.z, w);
                w = fmaf(s_q[4 * cc + 3], kv.w, w);
            }
            t = w * c_out;
        }
        const float wm = wave_max(t);
        if (lane == 0) s_red[wave] = wm;
        __syncthreads();
        const float mn = fmaxf(m, fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3])));
        const float pr = exp2f(t - mn);  // 0 past the causal limit
        s_p[tid] = pr;
        const float ws = wave_sum(pr);
        __syncthreads();
        if (lane == 0) s_red[wave] = ws;
        __syncthreads();
        const float corr = exp2f(m - mn);  // 0 at the first block
        ssum = ssum * corr + (s_red[0] + s_red[1] + s_red[2] + s_red[3]);
        o *= corr;
        const int jn = min(256, i + 1 - j0);
        for (int jj = sl; jj < jn; jj += SL)
            o = fmaf(s_p[jj], vbase[(int64_t)(j0 + jj) * g.vs[2] + c], o);
        m = mn;
        __syncthreads();  // s_p and s_red are free again
    }
    s_o[sl][c] = o;
    __syncthreads();
    if (tid < D) {
        float tot = 0.f;
#pragma unroll
        for (int t2 = 0; t2 < SL; ++t2) tot += s_o[t2][tid];
        const int64_t row = ((int64_t)b * g.Hq + hq) * g.r + (rho % g.r);
        out[row * D + tid] = tot / ssum;
        if (lse && tid == 0) lse[row] = (m + log2f(ssum)) * 0.69314718055994531f;
    }
}

// ---------------------------------------------------------------- launch --
template <int D>
static hipError_t launch_attn_d(const ScoreGeom &g, const WindowAttnPlan &pl, void *ws, void *out,
                                float *lse, hipStream_t st) {
    using A = AttnSmem<D>;
    float *part_o = (float *)ws;
    float2 *part_ms = (float2 *)((char *)ws + pl.off_ms);
    static DeviceOnce once;
    const hipError_t ea = device_once(once, [] {
        return hipFuncSetAttribute((const void *)window_attn_kernel<D>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)A::bytes);
    });
    if (ea != hipSuccess) return ea;
    const int Z = g.batch * g.Hkv, units = Z * pl.nparts;
    const int64_t wgs = (int64_t)((units + kXcds - 1) / kXcds) * kXcds * pl.n_blocks;
    hipLaunchKernelGGL(window_attn_kernel<D>, dim3((unsigned)wgs), dim3(256), A::bytes, st, g,
                       pl.n_blocks, pl.nparts, units, part_o, part_ms);
    const hipError_t e1 = hipGetLastError();
    if (e1 != hipSuccess) return e1;
    const int rows_per_wg = 256 / D;
    hipLaunchKernelGGL(window_attn_merge_kernel<D>, dim3((g.R + rows_per_wg - 1) / rows_per_wg, Z),
                       dim3(256), 0, st, g, pl.n_blocks, pl.nparts, part_o, part_ms,
                       (uint16_t *)out, lse);
    return hipGetLastError();
}

hipError_t launch_window_attention(const ScoreGeom &g, const WindowAttnPlan &pl, void *ws,
                                   void *out, float *lse, hipStream_t st) {
    if (g.dtype == AHA_BF16)
        return g.d == 64 ? launch_attn_d<64>(g, pl, ws, out, lse, st)
                         : launch_attn_d<128>(g, pl, ws, out, lse, st);
    dim3 grid(g.R, g.batch * g.Hkv);
    if (g.d == 64)
        hipLaunchKernelGGL(f32_window_attn_kernel<64>, grid, dim3(256), 0, st, g, (float *)out, lse);
    else
        hipLaunchKernelGGL(f32_window_attn_kernel<128>, grid, dim3(256), 0, st, g, (float *)out, lse);
    return hipGetLastError();
}

}  // namespace aha

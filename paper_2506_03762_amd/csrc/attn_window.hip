// Attention output of the observed rows, O_i = sum_{j <= i} softmax_j(Q_i . K_j / sqrt(d)) V_j
// for the last `window` query positions, and those rows' log-sum-exp: the self-attention
// that the eviction score is computed beside (appendix on compatibility with
// FlashAttention; Alg. 1 Prefill forms both from the same logits).  The log-sum-exp is what
// aha_prefill_scores_lse takes, so this launch plus the column-sum pass give output and
// scores with one pass over the keys each.
//
// bf16: a flash-style single pass on the matrix cores, in the orientation of the score
// kernels (keys on M, queries on N).  A workgroup owns two blocks of 32 flattened query rows
// of a KV head (one block if there is only one) and a range of keys; each of its four waves
// takes 32-key blocks (64 with one row block) and runs, per row block:
//   S^T = K Q^T            v_mfma_f32_32x32x16_bf16, A = key fragments from global memory
//   online softmax         per query column = per lane (the two half-waves of a column share
//                          their running maximum every block)
//   O^T += V^T P^T         the same MFMA; B = the probabilities, converted to bf16 where they
//                          sit: accumulator elements 8 ks .. 8 ks + 7 of a lane are exactly the
//                          eight keys of contraction step ks that the lane supplies; A = V^T,
//                          gathered from a wave-private copy of the step's value rows in LDS
//                          in that same key order (the contraction may run over the keys in
//                          any order as long as both operands agree); a gathered fragment
//                          serves both row blocks.
// The waves' partial outputs (each relative to its own maximum) meet in LDS, the key ranges'
// in the workspace, and a small second launch normalises.
// fp32 (the small high-accuracy path): plain vector-ALU kernel, one workgroup per row.
#include "score_tile.h"

namespace aha {

// NQ blocks of 32 query rows per workgroup, MB blocks of 32 keys per wave and step.  Two
// shapes are built: (NQ, MB) = (2, 1) - a wave's key fragments, its value rows in LDS and the
// V^T fragments gathered from them serve two row blocks, which halves the traffic from the L2
// and the LDS reads per query-key pair - and (1, 2) for problems with a single block of rows.
// Padded value row in LDS (elements): rows 16-byte aligned.  With 32 keys per wave the four
// rows of a transposing read lie 16 banks apart (80 resp. 48 dwords per row), so that the
// 4 x 32 elements that a half-wave reads fall into 64 different banks; with 64 keys per wave
// (the single-row-block shape) only the smallest padding fits two workgroups per CU.
template <int D, int MB>
struct AttnLdv { static constexpr int value = MB == 1 ? D + 32 : D + 8; };

template <int D, int NQ, int MB>
struct AttnSmem {
    using T = TileSmem<D, NQ>;
    static constexpr int WK = 32 * MB;   // keys per wave and step
    static constexpr int LDV = AttnLdv<D, MB>::value;
    static constexpr size_t v_bytes = (size_t)WK * LDV * 2;  // one wave's value rows
    static constexpr size_t off_v = (T::bytes + 15) / 16 * 16;
    static constexpr int LDO = D + 1;    // padded row of a wave's partial output (floats)
    // after the main loop: the four waves' partial outputs of ONE row block, and all statistics
    static constexpr size_t o_bytes = (size_t)4 * 32 * LDO * 4;
    static constexpr size_t off_ms = o_bytes;
    static constexpr size_t merge_bytes = off_ms + (size_t)4 * NQ * 32 * sizeof(float2);
    static constexpr size_t loop_bytes = off_v + 4 * v_bytes;
    static constexpr size_t bytes = loop_bytes > merge_bytes ? loop_bytes : merge_bytes;
    static_assert(2 * bytes <= 160 * 1024, "two workgroups per CU");
};

// A wave's key fragments of a step: lane holds row kb + mb * 32 + lane % 32, channels
// ks * 16 + (lane / 32) * 8 .. + 8; rows at or past `end` re-read row end - 1.
template <int D, int MB>
__device__ __forceinline__ void load_keys(const __bf16 *kbase, int64_t k_tstride, int kb, int end,
                                          int lane, bf16x8 (&a)[MB][D / 16]) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int row = min(kb + mb * 32 + (lane & 31), end - 1);
        const __bf16 *p = kbase + (int64_t)row * k_tstride + (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) a[mb][ks] = *(const bf16x8 *)(p + ks * 16);
    }
}

// Logits of the wave's keys against one block of 32 query rows (sQb: that block's rows in LDS).
template <int D, int MB>
__device__ __forceinline__ void logits(const bf16x8 (&a)[MB][D / 16], const __bf16 *sQb, int lane,
                                       f32x16 (&acc)[MB]) {
    const __bf16 *bp = sQb + (lane & 31) * (D + 8) + (lane >> 5) * 8;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 bfrag = *(const bf16x8 *)(bp + ks * 16);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb][ks], bfrag, acc[mb], 0, 0, 0);
    }
}

// The wave's value rows [kb, kb + 32 MB) -> its private LDS copy, row-major, 16-byte chunks,
// the lanes of a row adjacent.  Rows at or past `end` re-read row end - 1 (their
// probabilities are zero).  Request (global memory -> registers) and commit (-> LDS) are
// apart, so that the logits and the softmax of the step cover the round trip to memory.
template <int D, int MB>
struct ValueRows {
    static constexpr int CPR = D / 8, RPI = 64 / CPR, NI = 32 * MB / RPI, LDV = AttnLdv<D, MB>::value;
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
// of key block mb stand for (rows mb * 32 + 16 ks + 8 (e / 4) + e % 4 + 4 (lane / 32)): two
// runs of four consecutive keys, eight rows apart, read with the transposing LDS load.
template <int LDV>
__device__ __forceinline__ bf16x8 value_fragment(const __bf16 *sV, int mb, int ks, int cb,
                                                 int lane) {
    return lds_transposed_fragment(sV, LDV, mb * 32 + 16 * ks, 8, cb * 32, lane);
}

template <int D, int NQ, int MB>
__global__ __launch_bounds__(256, 2) void window_attn_kernel(ScoreGeom g, int n_blocks, int nparts,
                                                             int units, float *part_o,
                                                             float2 *part_ms) {
    using S = TileSmem<D, NQ>;
    using A = AttnSmem<D, NQ, MB>;
    constexpr int CB = D / 32;          // 32-channel blocks of the output
    constexpr int WK = A::WK, WGK = 4 * WK;  // keys per wave / per workgroup and step
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __bf16 *sQ = (__bf16 *)smem;
    float *sLam = (float *)(smem + S::q_bytes);
    int *sPos = (int *)(sLam + S::ROWS);
    int *sBlk = sPos + 2 * S::ROWS;

    // The workgroups of one (problem, key range) - one per group of NQ row blocks - re-read
    // the same keys and values: they get indices that are congruent modulo 8, i.e. one XCD
    // and one L2 (workgroups are dealt round-robin to the 8 XCDs).
    const int n_groups = (n_blocks + NQ - 1) / NQ;
    const int id = (int)blockIdx.x, xcd = id % kXcds, t = id / kXcds;
    const int grp = t % n_groups, u = (t / n_groups) * kXcds + xcd;
    if (u >= units) return;
    const int part = u % nparts, z = u / nparts;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowMap rm{g.n, g.r, g.R, nullptr};
    const int rho0 = grp * S::ROWS;
    const int end = rm.max_pos(rho0, rho0 + S::ROWS) + 1;  // the keys these rows may see
    const int steps = (end + WGK - 1) / WGK;
    const int key_begin = (int)((int64_t)part * steps / nparts) * WGK;
    const int key_end = min(end, (int)((int64_t)(part + 1) * steps / nparts) * WGK);
    // partials are laid out per block of 32 rows; a group's last block may not exist
    auto pidx_of = [&](int nq) { return ((int64_t)(z * nparts + part) * n_blocks + grp * NQ + nq) * 32; };
    if (key_begin >= key_end) {  // more ranges than these rows have key steps: neutral partials
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            if (grp * NQ + nq >= n_blocks) break;
            for (int i = tid; i < 32 * D; i += 256) part_o[pidx_of(nq) * D + i] = 0.f;
            if (tid < 32) part_ms[pidx_of(nq) + tid] = make_float2(-INFINITY, 0.f);
        }
        return;
    }
    const __bf16 *kbase = (const __bf16 *)g.k + b * g.ks[0] + h * g.ks[1];
    const __bf16 *vbase = (const __bf16 *)g.v + b * g.vs[0] + h * g.vs[1];
    const float c_out = kLog2e * rsqrtf((float)D);
    {
        QTileRegs<D, NQ> qt;
        q_tile_request<D, NQ>(g, b, h, rho0, tid, qt);
        q_tile_meta<D, NQ>(g, rm, rho0, tid, c_out, sLam, sPos, sBlk);
        q_tile_commit<D, NQ>(qt, tid, sQ);
    }
    __syncthreads();
    int pos[NQ], bmin[NQ], bmax_all = -1;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        pos[nq] = sPos[nq * 32 + (lane & 31)];  // -1 for rows past the last one: every key masked
        bmin[nq] = uniform(sBlk[NQ + nq]);
        bmax_all = max(bmax_all, uniform(sBlk[nq]));
    }
    __bf16 *sV = (__bf16 *)(smem + A::off_v + wave * A::v_bytes);

    f32x16 O[NQ][CB];
    float m[NQ], s[NQ];  // running maximum (log2 domain) and sum of this lane's keys, per row block
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m[nq] = -INFINITY;
        s[nq] = 0.f;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) O[nq][cb][v] = 0.f;
    }

    // Per step: the value rows are requested at the start and committed to LDS after the
    // softmax (logits and softmax cover their round trip); the key fragments of the NEXT step
    // are requested right after that commit, into the registers this step's logits have
    // consumed, and the gathers and the second product cover theirs.  (Requested any earlier
    // they are live through the softmax, and the kernel no longer fits 256 registers.)  The
    // requests are clamped to the key range.
    bf16x8 a[MB][D / 16];
    load_keys<D, MB>(kbase, g.ks[2], min(key_begin + wave * WK, key_end), key_end, lane, a);
    for (int kb0 = key_begin; kb0 < key_end; kb0 += WGK) {
        const int kb = kb0 + wave * WK;
        const bool live = kb < key_end && kb <= bmax_all;  // (wave-uniform; no barrier in the loop)
        ValueRows<D, MB> vr;
        vr.request(vbase, g.vs[2], min(kb, key_end), key_end, lane);
        f32x16 acc[NQ][MB];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) logits<D, MB>(a, sQ + nq * 32 * S::LD, lane, acc[nq]);
        if (!live) {
            load_keys<D, MB>(kbase, g.ks[2], min(kb + WGK, key_end), key_end, lane, a);
            continue;
        }
        bf16x8 pf[NQ][MB][2];  // the probabilities as B fragments of the two contraction steps
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            // causal limit and the ragged end of the key range
            if (kb + WK - 1 > bmin[nq] || kb + WK > key_end) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = acc_key(kb, mb, v, lane);
                        if (key > pos[nq] || key >= key_end) acc[nq][mb][v] = -INFINITY;
                    }
            }
            float amax = -INFINITY;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) amax = fmaxf(amax, acc[nq][mb][v]);
            // the two half-waves hold different keys of the same query column: one maximum
            amax = combine_lane_xor<32>(amax, OpMax{});
            const float mn = fmaxf(m[nq], amax == -INFINITY ? -INFINITY : amax * c_out);
            const float mref = mn == -INFINITY ? 0.f : mn;
            const float corr = fast_exp2(m[nq] - mref);  // 0 while the column has seen no key
            float sum[2] = {0.f, 0.f};
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float pr = fast_exp2(fmaf(acc[nq][mb][8 * ks + e], c_out, -mref));
                        sum[e & 1] += pr;
                        pf[nq][mb][ks][e] = (__bf16)pr;
                    }
            s[nq] = s[nq] * corr + (sum[0] + sum[1]);
            m[nq] = mn;
            if (__builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {  // (rarely after the first blocks)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) O[nq][cb][v] *= corr;
            }
        }
        vr.commit(lane, sV);
        __builtin_amdgcn_sched_barrier(0);
        load_keys<D, MB>(kbase, g.ks[2], min(kb + WGK, key_end), key_end, lane, a);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const bf16x8 vf = value_fragment<A::LDV>(sV, mb, ks, cb, lane);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        O[nq][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nq][mb][ks],
                                                                            O[nq][cb], 0, 0, 0);
                }
    }

    // ---- the four waves' partials (different keys, own maxima) meet in LDS, one row block
    // at a time ----
    __syncthreads();  // the query tile and the value rows are done with
    float2 *sMS = (float2 *)(smem + A::off_ms);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float sc = s[nq] + __shfl_xor(s[nq], 32);  // the column's sum over both half-waves
        if (lane < 32) sMS[(wave * NQ + nq) * 32 + lane] = make_float2(m[nq], sc);
    }
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        if (grp * NQ + nq >= n_blocks) break;  // (workgroup-uniform)
        float *sO = (float *)smem + (size_t)wave * 32 * A::LDO;
        if (nq) __syncthreads();  // the previous block's partials are read
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                sO[(lane & 31) * A::LDO + cb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] = O[nq][cb][v];
        __syncthreads();
        const int64_t pidx = pidx_of(nq);
        for (int i = tid; i < 32 * D; i += 256) {
            const int q = i / D, ch = i % D;
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) M = fmaxf(M, sMS[(w * NQ + nq) * 32 + q].x);
            const float mref = M == -INFINITY ? 0.f : M;
            float o = 0.f, ssum = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float2 ms = sMS[(w * NQ + nq) * 32 + q];
                const float f = fast_exp2(ms.x - mref);
                const float *wO = (const float *)smem + (size_t)w * 32 * A::LDO;
                o = fmaf(f, wO[q * A::LDO + ch], o);
                ssum = fmaf(f, ms.y, ssum);
            }
            part_o[(pidx + q) * D + ch] = o;
            if (ch == 0) part_ms[pidx + q] = make_float2(M, ssum);
        }
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
    // (the loads of several key ranges in flight at once: the launch is bound by their latency)
    float M = -INFINITY;
#pragma unroll 8
    for (int p = 0; p < nparts; ++p)
        M = fmaxf(M, part_ms[((int64_t)(z * nparts + p) * n_blocks + nbk) * 32 + q].x);
    float o = 0.f, ssum = 0.f;
#pragma unroll 8
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
template <int D, int NQ, int MB>
static hipError_t launch_attn_t(const ScoreGeom &g, const WindowAttnPlan &pl, void *ws, void *out,
                                float *lse, hipStream_t st) {
    using A = AttnSmem<D, NQ, MB>;
    float *part_o = (float *)ws;
    float2 *part_ms = (float2 *)((char *)ws + pl.off_ms);
    static DeviceOnce once;
    const hipError_t ea = device_once(once, [] {
        return hipFuncSetAttribute((const void *)window_attn_kernel<D, NQ, MB>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)A::bytes);
    });
    if (ea != hipSuccess) return ea;
    const int Z = g.batch * g.Hkv, units = Z * pl.nparts;
    const int n_groups = (pl.n_blocks + NQ - 1) / NQ;
    const int64_t wgs = (int64_t)((units + kXcds - 1) / kXcds) * kXcds * n_groups;
    hipLaunchKernelGGL((window_attn_kernel<D, NQ, MB>), dim3((unsigned)wgs), dim3(256), A::bytes, st,
                       g, pl.n_blocks, pl.nparts, units, part_o, part_ms);
    const hipError_t e1 = hipGetLastError();
    if (e1 != hipSuccess) return e1;
    const int rows_per_wg = 256 / D;
    hipLaunchKernelGGL(window_attn_merge_kernel<D>, dim3((g.R + rows_per_wg - 1) / rows_per_wg, Z),
                       dim3(256), 0, st, g, pl.n_blocks, pl.nparts, part_o, part_ms,
                       (uint16_t *)out, lse);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_attn_d(const ScoreGeom &g, const WindowAttnPlan &pl, void *ws, void *out,
                                float *lse, hipStream_t st) {
    return pl.nq == 2 ? launch_attn_t<D, 2, 1>(g, pl, ws, out, lse, st)
                      : launch_attn_t<D, 1, 2>(g, pl, ws, out, lse, st);
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

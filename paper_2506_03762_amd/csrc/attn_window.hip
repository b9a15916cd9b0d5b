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
// takes 32-key blocks and runs, per row block:
//   S^T = K Q^T            v_mfma_f32_32x32x16_bf16, A = key fragments from global memory
//   online softmax         per query column = per lane (the two half-waves of a column share
//                          their reference, which follows the running maximum lazily)
//   O^T += V^T P^T         the same MFMA; B = the probabilities, converted to bf16 where they
//                          sit: accumulator elements 8 ks .. 8 ks + 7 of a lane are exactly the
//                          eight keys of contraction step ks that the lane supplies; A = V^T,
//                          read with transposing LDS loads from a wave-private copy of the
//                          step's value rows (loaded from global memory straight into LDS)
//                          in that same key order (the contraction may run over the keys in
//                          any order as long as both operands agree); a fragment serves
//                          both row blocks.
// The waves' partial outputs (each relative to its own reference) meet in LDS, the key ranges'
// in the workspace, and a small second launch normalises.
// fp32 (the small high-accuracy path): plain vector-ALU kernel, one workgroup per row.
#include "score_tile.h"

namespace aha {

// NQ blocks of 32 query rows per workgroup (two, or one for problems with a single block of
// rows); a wave takes 32 keys per step (MB = 1 block; the helpers keep the parameter).  With
// two row blocks a wave's key fragments, its value rows in LDS and the V^T fragments read
// from them serve both, which halves the traffic from the L2 and the LDS reads per query-key
// pair.
// LDS: the query tile (later the waves' partial outputs, half of the channels at a time) in
// the dynamic part, the waves' value rows in a static array of their own - so that the
// compiler can tell the direct loads into the value rows apart from the reads of the query
// tile, and does not wait for those loads before every such read.
template <int D, int NQ>
struct AttnSmem {
    using T = TileSmem<D, NQ>;
    static constexpr int WK = 32;                     // keys per wave and step
    static constexpr int v_elems = 4 * WK * D;        // the four waves' value rows (static LDS)
    static constexpr int HC = D / 2;                  // channels per pass of the waves' merge
    static constexpr int LDO = HC + 1;                // padded row of a wave's partial output (floats)
    // after the main loop: the four waves' partial outputs of ONE row block and half of its
    // channels, and all statistics
    static constexpr size_t o_bytes = (size_t)4 * 32 * LDO * 4;
    static constexpr size_t off_ms = o_bytes;
    static constexpr size_t merge_bytes = off_ms + (size_t)4 * NQ * 32 * sizeof(float2);
    static constexpr size_t bytes = T::bytes > merge_bytes ? T::bytes : merge_bytes;  // dynamic
    static_assert(2 * (bytes + v_elems * 2) <= 160 * 1024, "two workgroups per CU");
};

// The wave's value rows in LDS: row-major without padding (direct loads from global memory
// place the 64 lanes' 16-byte chunks back to back), the 16-byte chunks of row R permuted by
// XOR with swz(R), so that the four rows of a transposing read fall into different banks.
template <int D>
__device__ __forceinline__ int value_chunk_swizzle(int row) {
    return (4 * (row & 3)) % (D / 8);
}

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

// Logits of the wave's 32 keys against NQ blocks of 32 query rows (sQ: the tile in LDS, LD
// elements per row).  The query fragments are read kLogitsAhead products ahead of their use
// (a rolling window of registers): read right before its product, every fragment exposes the
// LDS latency, several times the 32 cycles of a product.
constexpr int kLogitsAhead = 4;
template <int D, int NQ, int LD>
__device__ __forceinline__ void logits(const bf16x8 (&a)[1][D / 16], const __bf16 *sQ, int lane,
                                       f32x16 (&acc)[NQ][1]) {
    constexpr int KS = D / 16, N = NQ * KS;
    const __bf16 *bp = sQ + (lane & 31) * LD + (lane >> 5) * 8;
    auto frag = [&](int i) { return *(const bf16x8 *)(bp + (i / KS) * 32 * LD + (i % KS) * 16); };
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nq][0][v] = 0.f;
    bf16x8 b[kLogitsAhead];
#pragma unroll
    for (int i = 0; i < kLogitsAhead; ++i) b[i] = frag(i);
#pragma unroll
    for (int i = 0; i < N; ++i) {
        acc[i / KS][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i % KS], b[i % kLogitsAhead],
                                                                 acc[i / KS][0], 0, 0, 0);
        if (i + kLogitsAhead < N) b[i % kLogitsAhead] = frag(i + kLogitsAhead);
    }
    // the order as written: the first reads, then one product and one read at a time
    __builtin_amdgcn_sched_group_barrier(0x100, kLogitsAhead, 0);
#pragma unroll
    for (int i = 0; i < N - kLogitsAhead; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, kLogitsAhead, 0);
}

// The wave's value rows [kb, kb + 32 MB) -> its private LDS copy, by loads that go from
// global memory straight to LDS (global_load_lds_dwordx4: no registers are held while the
// rows travel, and no LDS store instruction is issued): per instruction the 64 lanes' 16-byte
// chunks land back to back from a wave-uniform LDS address, i.e. 64 / (D / 8) whole rows; lane
// (row r, position c) fetches the chunk that the swizzle puts at position c.  Rows at or past
// `end` re-read row end - 1 (their probabilities are zero).
// The loads are written as assembly and the waits for them by hand (wait_loads): the
// compiler's own bookkeeping treats a load into LDS as one that may complete out of order
// with everything else and answers with full waits (vmcnt(0) lgkmcnt(0)) right behind it,
// which would expose the round trip this is meant to hide.  In the kernel's loop the loads
// into LDS are the OLDEST loads in flight whenever the compiler waits for loads it knows
// (the next step's key fragments, requested after them), so its counts stay on the safe side.
// Addresses: a step whose 32 MB rows all exist (every step but a ragged last one) uses the
// wave-uniform address of its first row as a scalar base, advanced per instruction on the
// scalar unit, and ONE loop-invariant 32-bit offset per lane (row within the instruction's
// rows, swizzled chunk); the ragged step clamps every lane's row to end - 1.
template <int D, int MB>
struct ValueRequest {
    static constexpr int CPR = D / 8, RPI = 64 / CPR, NI = 32 * MB / RPI;
    uint32_t lane_off;  // bytes from the first row of an instruction's rows
    uint32_t lds0;      // the wave's LDS copy (LDS addresses are the numeric values of LDS
                        // pointers; M0 carries the base of an instruction's rows)
    bool wide;          // the token stride does not fit the 32-bit lane offset
    __device__ __forceinline__ ValueRequest(int64_t v_tstride, int lane, __bf16 *sV) {
        const int r0 = lane / CPR, c = lane % CPR;
        // (the swizzle of row t RPI + r0 does not depend on t: RPI is a multiple of 4)
        lane_off = (uint32_t)(r0 * v_tstride * 2) + (c ^ value_chunk_swizzle<D>(r0)) * 16;
        lds0 = __builtin_amdgcn_readfirstlane(
            (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)sV);
        wide = v_tstride * 2 * RPI >= ((int64_t)1 << 31);
    }
    // kb: wave-uniform first row
    __device__ __forceinline__ void operator()(const __bf16 *vbase, int64_t v_tstride, int kb,
                                               int end, int lane) const {
        if (kb + 32 * MB <= end && !wide) {
            const __bf16 *row0 = vbase + (int64_t)kb * v_tstride;
#pragma unroll
            for (int t = 0; t < NI; ++t)
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :
                             : "v"(lane_off), "s"(row0 + (int64_t)t * RPI * v_tstride),
                               "s"(lds0 + t * RPI * D * 2)
                             : "memory");  // (M0 holds nothing else: gfx9 LDS instructions do not read it)
            return;
        }
        const int r0 = lane / CPR, c = lane % CPR;
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            const int row = t * RPI + r0;
            const __bf16 *src = vbase + (int64_t)min(kb + row, end - 1) * v_tstride +
                                (c ^ value_chunk_swizzle<D>(row)) * 8;
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                         :
                         : "v"(src), "s"(lds0 + t * RPI * D * 2)
                         : "memory");
        }
    }
};
// s_waitcnt vmcnt(N) alone (the other counters at their maxima): bits 3:0 and 15:14 hold
// vmcnt, 6:4 expcnt, 11:8 lgkmcnt.
template <int N>
__device__ __forceinline__ void wait_loads() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// A fragment of V^T for channel block cb, key block mb, contraction step ks: this lane's
// channel cb * 32 + lane % 32 of the eight keys that its accumulator elements 8 ks .. 8 ks + 7
// of key block mb stand for (rows mb * 32 + 16 ks + 8 (e / 4) + e % 4 + 4 (lane / 32)): two
// runs of four consecutive keys, eight rows apart.  A lane wants a COLUMN of four elements at
// a time: ds_read_b64_tr_b16 reads, per group of 16 lanes, a tile of 4 rows x 16 elements -
// lane s of the group supplies the address of row s / 4, elements 4 (s % 4) .. + 3 - and hands
// lane j of the group column j of that tile.  Two such reads make a fragment, with no
// repacking in the vector ALU.
template <int D>
__device__ __forceinline__ bf16x8 value_fragment(const __bf16 *sV, int mb, int ks, int cb,
                                                 int lane) {
    using lds_ptr = s16x4 __attribute__((address_space(3))) *;
    const int row = mb * 32 + 16 * ks + 4 * (lane >> 5) + ((lane >> 2) & 3);
    const int chunk = cb * 4 + ((lane & 16) >> 3) + ((lane & 3) >> 1);  // of elements 4 (s % 4) .. + 3
    // (rows 8 apart have the same swizzle)
    const __bf16 *p = sV + row * D + (chunk ^ value_chunk_swizzle<D>(row)) * 8 + 4 * (lane & 1);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * D));
    bf16x8 f;
    __builtin_memcpy(&f, &lo, 8);
    __builtin_memcpy((char *)&f + 8, &hi, 8);
    return f;
}

template <int D, int NQ>
__global__ __launch_bounds__(256, 2) void window_attn_kernel(ScoreGeom g, int n_blocks, int nparts,
                                                             int units, float *part_o,
                                                             float2 *part_ms) {
    constexpr int MB = 1;
    using S = TileSmem<D, NQ>;
    using A = AttnSmem<D, NQ>;
    __shared__ __attribute__((aligned(1024))) __bf16 sVall[A::v_elems];
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
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
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
    constexpr float kRefSlack = 8.f;  // log2 units
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
    __bf16 *sV = sVall + wave * (A::WK * D);

    f32x16 O[NQ][CB];
    float m[NQ], s[NQ];  // reference (log2 domain: at most kRefSlack below the running maximum) and
                         // sum of this lane's keys relative to it, per row block
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m[nq] = -INFINITY;
        s[nq] = 0.f;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) O[nq][cb][v] = 0.f;
    }

    // Per step: the value rows are requested at the start, straight into LDS, and the key
    // fragments of the NEXT step right after the logits, into the registers the logits have
    // consumed: the softmax covers the value rows' round trip, softmax and second product the
    // keys'.  The requests are clamped to the key range.
    const ValueRequest<D, MB> request_values(g.vs[2], lane, sV);
    bf16x8 a[MB][D / 16];
    load_keys<D, MB>(kbase, g.ks[2], min(key_begin + wave * WK, key_end), key_end, lane, a);
    for (int kb0 = key_begin; kb0 < key_end; kb0 += WGK) {
        const int kb = kb0 + wave * WK;
        const bool live = kb < key_end && kb <= bmax_all;  // (wave-uniform; no barrier in the loop)
        wait_loads<0>();  // this step's key fragments, requested a step ago, are here
        request_values(vbase, g.vs[2], min(kb, key_end), key_end, lane);
        f32x16 acc[NQ][MB];
        logits<D, NQ, S::LD>(a, sQ, lane, acc);
        __builtin_amdgcn_sched_barrier(0);
        load_keys<D, MB>(kbase, g.ks[2], min(kb + WGK, key_end), key_end, lane, a);
        __builtin_amdgcn_sched_barrier(0);
        if (!live) continue;
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
            // The reference that probabilities and sums are relative to follows the running
            // maximum lazily: it moves only when the block's maximum exceeds it by more than
            // kRefSlack (probabilities then stay below 2^kRefSlack, no loss in fp32 or bf16,
            // which share the exponent range).  After the first blocks that is rare, and a
            // block that moves no column's reference skips the rescaling of the outputs.
            const float bm = amax == -INFINITY ? -INFINITY : amax * c_out;
            const float mn = bm > m[nq] + kRefSlack ? bm : m[nq];  // (m = -inf: moves to any finite bm)
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
            if (__builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) O[nq][cb][v] *= corr;
            }
        }
        // the value rows are in LDS once at most the key fragments requested after them (D / 16
        // loads per key block) are still in flight
        __builtin_amdgcn_sched_barrier(0);
        wait_loads<MB * D / 16>();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const bf16x8 vf = value_fragment<D>(sV, mb, ks, cb, lane);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        O[nq][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nq][mb][ks],
                                                                            O[nq][cb], 0, 0, 0);
                }
    }

    // ---- the four waves' partials (different keys, own maxima) meet in LDS, one row block
    // and half of the channels at a time ----
    __syncthreads();  // the query tile is done with
    float2 *sMS = (float2 *)(smem + A::off_ms);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float sc = s[nq] + __shfl_xor(s[nq], 32);  // the column's sum over both half-waves
        if (lane < 32) sMS[(wave * NQ + nq) * 32 + lane] = make_float2(m[nq], sc);
    }
    constexpr int HC = A::HC, CBH = CB / 2;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        if (grp * NQ + nq >= n_blocks) break;  // (workgroup-uniform)
        const int64_t pidx = pidx_of(nq);
#pragma unroll
        for (int hc = 0; hc < 2; ++hc) {
            float *sO = (float *)smem + (size_t)wave * 32 * A::LDO;
            if (nq || hc) __syncthreads();  // the previous partials are read
#pragma unroll
            for (int cb = 0; cb < CBH; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    sO[(lane & 31) * A::LDO + cb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] =
                        O[nq][hc * CBH + cb][v];
            __syncthreads();
            for (int i = tid; i < 32 * HC; i += 256) {
                const int q = i / HC, ch = i % HC;
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
                part_o[(pidx + q) * D + hc * HC + ch] = o;
                if (hc == 0 && ch == 0) part_ms[pidx + q] = make_float2(M, ssum);
            }
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
    constexpr float kRefSlack = 8.f;  // log2 units
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
template <int D, int NQ>
static hipError_t launch_attn_t(const ScoreGeom &g, const WindowAttnPlan &pl, void *ws, void *out,
                                float *lse, hipStream_t st) {
    using A = AttnSmem<D, NQ>;
    float *part_o = (float *)ws;
    float2 *part_ms = (float2 *)((char *)ws + pl.off_ms);
    static DeviceOnce once;
    const hipError_t ea = device_once(once, [] {
        return hipFuncSetAttribute((const void *)window_attn_kernel<D, NQ>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)A::bytes);
    });
    if (ea != hipSuccess) return ea;
    const int Z = g.batch * g.Hkv, units = Z * pl.nparts;
    const int n_groups = (pl.n_blocks + NQ - 1) / NQ;
    const int64_t wgs = (int64_t)((units + kXcds - 1) / kXcds) * kXcds * n_groups;
    hipLaunchKernelGGL((window_attn_kernel<D, NQ>), dim3((unsigned)wgs), dim3(256), A::bytes, st,
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
    return pl.nq == 2 ? launch_attn_t<D, 2>(g, pl, ws, out, lse, st)
                      : launch_attn_t<D, 1>(g, pl, ws, out, lse, st);
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

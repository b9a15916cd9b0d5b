// bf16 eviction scores on the gfx950 matrix cores (Sec. 4.1 - 4.3; Alg. 1
// Prefill).  Two passes, both recomputing tiles of K Q^T with
// v_mfma_f32_32x32x16_bf16 (keys on M, queries on N); the n x n probability
// matrix never exists in memory.
//
//   pass 1: per observed query row, max and sum of exp2 over its keys
//           (log2 domain, scale applied in fp32 after the MFMA);
//   pass 2: per key, sum over the observed rows of exp2(t - L_row), times the
//           value prior.
//
// With keys on M the 32x32 accumulator gives every lane ONE query column
// (lane % 32) and 16 key rows, so the per-row scale, maximum and log-sum-exp
// are per-lane scalars in both passes; pass 1 reduces over keys in-lane, and
// pass 2 accumulates over query blocks in-lane and folds the 32 lanes of a
// half-wave once per key block.
//
// Work split: a workgroup keeps one tile of query rows (up to 256 flattened
// rows of a KV head's query group) in LDS as the B operand; each of its four
// waves owns 64-key blocks whose A fragments it loads straight from global
// memory into registers (each K byte is fetched once per tile), so waves run
// independently between the tile barriers; the A fragments are double-buffered so
// that the next key block is in flight while the current one multiplies.
#include "score_tile.h"

namespace aha {


// Online max / sum-of-exp2 of one 64 x 32 block for this lane's query column.
// The scale is non-negative, so the maximum of the scaled logits is the scale
// times the maximum raw dot.
// With ENT the first moment u = sum of exp2(t - m) * (t - m) is kept beside the sum: the
// row's entropy is ln 2 * (log2 s - u / s) (Sec. 4.2, entropy of a softmax row).
template <bool MASK, bool ENT, bool LAZY = false>
__device__ __forceinline__ void stats_update(const f32x16 (&acc)[kMB], float lam, int pos, int kb,
                                             int lane, float &m, float &s, float &u) {
    if (MASK) asm volatile("" ::: "memory");
    if constexpr (!MASK && LAZY) {
        // (LAZY: full accumulation, where this loop is the kernel; in the windowed kernel the
        // second code path costs registers that spill.)
        // Unmasked blocks: `m` is a REFERENCE that sum and moment are relative to, not
        // necessarily the running maximum (the final statistics m + log2 s and u / s do not
        // depend on it).  As long as every lane has one, the block is summed against it as it
        // stands - no maximum over the block's 32 elements - and the reference is only moved
        // (by the exact update below, which also redoes this block) when a block's sum says
        // that it has fallen more than 40 binades behind: fp32 has room for that, and a
        // reference never lies above the largest logit seen, so nothing underflows that the
        // exact update would have kept.
        if (__builtin_amdgcn_ballot_w64(m == -INFINITY) == 0) {
            float sum[4] = {0.f, 0.f, 0.f, 0.f}, mom[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float x = fmaf(acc[mb][v], lam, -m);
                    const float e = fast_exp2(x);
                    sum[v & 3] += e;
                    if (ENT) mom[v & 3] = fmaf(e, x, mom[v & 3]);
                }
            const float bs = (sum[0] + sum[1]) + (sum[2] + sum[3]);
            if (__builtin_amdgcn_ballot_w64(!(bs < 0x1p40f)) == 0) {  // (also: not a NaN)
                s += bs;
                if (ENT) u += (mom[0] + mom[1]) + (mom[2] + mom[3]);
                return;
            }
        }
    }
    float amax = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float x = acc[mb][v];
            if (MASK && acc_key(kb, mb, v, lane) > pos) x = -INFINITY;
            amax = fmaxf(amax, x);
        }
    const float tmax = amax == -INFINITY ? -INFINITY : amax * lam;
    const float mn = fmaxf(m, tmax);
    const float mref = mn == -INFINITY ? 0.f : mn;
    // four partial sums: independent chains, so that the exponentials' result latency is
    // covered by other work instead of wait states
    float sum[4] = {0.f, 0.f, 0.f, 0.f}, mom[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float x = fmaf(acc[mb][v], lam, -mref);
            float e = fast_exp2(x);
            if (MASK && acc_key(kb, mb, v, lane) > pos) e = 0.f;
            sum[v & 3] += e;
            // (e = 0 for masked or far-away keys: 0 * x, x finite, adds nothing)
            if (ENT) mom[v & 3] = fmaf(e, x, mom[v & 3]);
        }
    const float f = fast_exp2(m - mref);  // 0 while the row has seen no key
    if (ENT) {
        const float dm = m == -INFINITY ? 0.f : m - mref;
        u = (u + dm * s) * f + ((mom[0] + mom[1]) + (mom[2] + mom[3]));
    }
    s = s * f + ((sum[0] + sum[1]) + (sum[2] + sum[3]));
    m = mn;
}

template <bool MASK>
__device__ __forceinline__ void colsum_update(const f32x16 (&acc)[kMB], float lam, float L,
                                              int pos, int kb, int lane, f32x16 (&col)[kMB]) {
    // The empty asm keeps the masked and the unmasked instantiation apart: without it the
    // compiler merges the two branches and every block pays the per-element compare/select.
    if (MASK) asm volatile("" ::: "memory");
    if constexpr (!MASK) {
        // Four elements at a time - their scaled logits, their exponentials, their sums - and
        // the instructions kept in that order: scheduled by register pressure alone, every
        // exponential is followed at once by the addition that needs it, with a wait state
        // (an issue slot of the wave) in between.
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += 4) {
                float t[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] = fmaf(acc[mb][v0 + i], lam, -L);
                asm volatile("" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]));
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] = fast_exp2(t[i]);
                asm volatile("" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]));
#pragma unroll
                for (int i = 0; i < 4; ++i) col[mb][v0 + i] += t[i];
            }
        return;
    }
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float p = fast_exp2(fmaf(acc[mb][v], lam, -L));
            if (MASK && acc_key(kb, mb, v, lane) > pos) p = 0.f;
            col[mb][v] += p;
        }
    if (MASK) asm volatile("" ::: "memory");
}


// Work split shared by pass 1 and by pass 2 in full accumulation.  Query tile `pair` is
// teamed with tile T-1-pair: a tile of late rows sees many keys, its partner few, together
// about the same as any other pair.  The pair's work is laid out on a line - the first
// tile's 256-key steps, the set-up of the partner (loading a query tile costs about one
// step; every workgroup pays one set-up anyway, only a second one counts), the partner's
// steps - and the line is cut into `nparts` equal ranges.  Segment `seg` (0: first tile,
// 1: partner) of a workgroup is the part of its range that falls on that tile's steps.
// A single tile (windowed scores, or the middle tile of an odd count) is cut into equal
// ranges of steps.
struct Segment {
    int qt;          // query tile, -1: no such segment
    int kbeg, kend;  // keys [kbeg, kend); empty when kbeg >= kend
};
__device__ __forceinline__ Segment pair_segment(const RowMap &rm, int rows, int T, int pair,
                                                int part, int nparts, int seg) {
    const int tA = pair, tB = T - 1 - pair;
    const bool two = tB != tA;
    // (chosen accumulator rows - a single tile - may sit anywhere: the whole sequence)
    const int endA = rm.rows ? rm.n : rm.max_pos(tA * rows, (tA + 1) * rows) + 1;
    const int endB = two ? rm.max_pos(tB * rows, (tB + 1) * rows) + 1 : 0;
    const int sA = (endA + kWgKeys - 1) / kWgKeys, sB = (endB + kWgKeys - 1) / kWgKeys;
    // positions on the line: first tile's steps start at oA, the partner's at oB
    const int oA = 0, oB = sA + 1, V = two ? sA + sB + 1 : sA;
    const int v0 = (int)((int64_t)part * V / nparts), v1 = (int)((int64_t)(part + 1) * V / nparts);
    Segment r;
    if (seg == 0) {
        r.qt = tA;
        r.kbeg = (max(v0, oA) - oA) * kWgKeys;
        r.kend = min(endA, (min(v1, oA + sA) - oA) * kWgKeys);
    } else {
        r.qt = two ? tB : -1;
        r.kbeg = (max(v0, oB) - oB) * kWgKeys;
        r.kend = min(endB, (min(v1, oB + sB) - oB) * kWgKeys);
    }
    return r;
}

// ---------------------------------------------------------------- pass 1 --
// Value prior (Sec. 4.3) inside pass 1.  The value rows of the 64 keys a wave multiplies in a
// step are loaded with the addressing of the key fragments into the register buffer that is
// idle in the first half of the step (the next key block is requested at mid-step instead of
// at the start): a lane then holds one half (the channels of its half-wave) of two value rows.

// nu = ||V_row||^2 of those rows: squares summed in-lane, one exchange between the half-waves.
template <int D>
__device__ __forceinline__ void fragment_row_norms(const bf16x8 (&a)[kMB][D / 16],
                                                   float (&nu)[kMB]) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            const bf16x8 w = a[mb][ks];
            const bf16x2 p0 = {w[0], w[1]}, p1 = {w[2], w[3]}, p2 = {w[4], w[5]}, p3 = {w[6], w[7]};
            s0 = __builtin_amdgcn_fdot2_f32_bf16(p0, p0, s0, false);
            s1 = __builtin_amdgcn_fdot2_f32_bf16(p1, p1, s1, false);
            s0 = __builtin_amdgcn_fdot2_f32_bf16(p2, p2, s0, false);
            s1 = __builtin_amdgcn_fdot2_f32_bf16(p3, p3, s1, false);
        }
        const float h = s0 + s1;
        nu[mb] = combine_lane_xor<32>(h, OpSum{});
    }
}

// Pooling halo of a key range [kbeg, kend): the (pool - 1) / 2 value rows below and above it,
// one per group of d / 8 lanes (at most 256 / (d / 8) rows: the host checks the pool width).
// Requested right after the main loop, squared when the range is pooled.
template <int D>
struct PriorHalo {
    static constexpr int CPR = D / 8;  // 16-byte chunks per value row
    u32x4 w;
    int pos;     // token of this thread's halo row
    bool valid;  // the row exists (inside the sequence, inside the halo)
    bool below;
    __device__ __forceinline__ void request(const ScoreGeom &g, const __bf16 *vbase, int kbeg,
                                            int kend, int tid) {
        const int half = (g.pool - 1) / 2, hrow = tid / CPR;
        below = hrow < half;
        pos = below ? kbeg - half + hrow : kend + hrow - half;
        valid = hrow < 2 * half && pos >= 0 && pos < g.n;
        w = u32x4{0u, 0u, 0u, 0u};
        if (valid) w = *(const u32x4 *)(vbase + (int64_t)pos * g.vs[2] + (tid % CPR) * 8);
    }
    // ||row||^2 in the first lane of the row's group (every lane takes part)
    __device__ __forceinline__ float norm() const {
        float hn = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float x = bf16_lo(w[c]), y = bf16_hi(w[c]);
            hn = fmaf(x, x, fmaf(y, y, hn));
        }
        return reduce_lanes<1, CPR>(hn, OpSum{});
    }
};

// gamma = edge-truncated mean of nu over the pool window for the keys [kbeg, kend) of problem
// z, written to `gamma`; returns (in every thread) the largest gamma of the range.  The norms
// of the range's own rows were left by the workgroup's waves in `nu_g` (read past the L1:
// other waves of this workgroup wrote them); the range is worked through in pieces staged in
// s_nu.  The caller has passed a barrier since the last norm was written.
constexpr int kPriorPiece = 512;
constexpr int kPriorMaxHalo = 32;  // rows on both sides together
constexpr size_t kPriorSmem = (kPriorPiece + kPriorMaxHalo + 4) * sizeof(float);
template <int D>
__device__ __forceinline__ float pool_norms_of_range(const ScoreGeom &g, int z, int kbeg,
                                                     int kend, const float *nu_g,
                                                     const PriorHalo<D> &halo, float *s_nu,
                                                     float *gamma, int tid) {
    const int half = (g.pool - 1) / 2;
    float *s_max = s_nu + kPriorPiece + kPriorMaxHalo;
    const float hn = halo.norm();
    float gmax = 0.f;
    for (int t0 = kbeg; t0 < kend; t0 += kPriorPiece) {
        const int t1 = min(kend, t0 + kPriorPiece);
        const int lo = max(0, t0 - half), hi = min(g.n, t1 + half);  // hi exclusive
        for (int t = max(lo, kbeg) + tid; t < min(hi, kend); t += 256)
            s_nu[t - lo] = __hip_atomic_load(nu_g + (int64_t)z * g.n + t, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        // the halo rows that touch this piece (the first piece below, the last one above)
        if (halo.valid && tid % PriorHalo<D>::CPR == 0 && (halo.below ? t0 == kbeg : t1 == kend))
            s_nu[halo.pos - lo] = hn;
        __syncthreads();
        for (int j = t0 + tid; j < t1; j += 256) {
            const int a = max(0, j - half), e = min(g.n - 1, j + half);
            float s = 0.f;
            for (int t = a; t <= e; ++t) s += s_nu[t - lo];
            const float gam = s / (float)(e - a + 1);
            gamma[(int64_t)z * g.n + j] = gam;
            gmax = fmaxf(gmax, gam);
        }
        __syncthreads();
    }
    gmax = wave_max(gmax);
    if ((tid & 63) == 0) s_max[tid >> 6] = gmax;
    __syncthreads();
    gmax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    __syncthreads();
    return gmax;
}

// The prior of a key range formed AFTER the main loop, for tiles of fewer than 256 rows (see
// bf16_pass1_kernel): value rows of the keys [kbeg, kend) of problem z are streamed in a phase
// of their own: nu = ||V||^2 of the range and its pooling halo into
// LDS, gamma = edge-truncated mean over the pool window, written to `gamma`; returns (in
// every thread) the largest gamma of the range.  Works through the range in pieces of
// kPriorPiece keys so that the LDS it borrows (the query tile's, free at that time) stays
// small.  Ends with a barrier: the LDS may be reused at once.
// value rows a lane requests before it uses the first (9 and 33 measured slower here)
constexpr int kPriorLoads = 17;
constexpr size_t kPriorTailSmem = (kPriorPiece + 256 + 4) * sizeof(float);
__device__ __forceinline__ float value_prior_of_range(const ScoreGeom &g, int b, int h, int z,
                                                      int kbeg, int kend, float *s_nu,
                                                      float *gamma, int tid) {
    const char *vbase = (const char *)g.v + (int64_t)2 * (b * g.vs[0] + h * g.vs[1]);
    const int half = (g.pool - 1) / 2;
    float *s_max = s_nu + kPriorPiece + 256;
    float gmax = 0.f;
    for (int t0 = kbeg; t0 < kend; t0 += kPriorPiece) {
        const int t1 = min(kend, t0 + kPriorPiece);
        const int lo = max(0, t0 - half), hi = min(g.n, t1 + half);  // hi exclusive
        value_norms_to_lds<2, kPriorLoads>(vbase, g.vs[2], g.d, lo, hi, s_nu, tid);
        __syncthreads();
        for (int j = t0 + tid; j < t1; j += 256) {
            const int a = max(0, j - half), e = min(g.n - 1, j + half);
            float s = 0.f;
            for (int t = a; t <= e; ++t) s += s_nu[t - lo];
            const float gam = s / (float)(e - a + 1);
            gamma[(int64_t)z * g.n + j] = gam;
            gmax = fmaxf(gmax, gam);
        }
        __syncthreads();
    }
    gmax = wave_max(gmax);
    if ((tid & 63) == 0) s_max[tid >> 6] = gmax;
    __syncthreads();
    gmax = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    __syncthreads();
    return gmax;
}

// PRIOR (windowed scores with the value prior): the workgroup also forms the prior of its key
// range and leaves the range's maximum in gblockmax[z * nparts + part]: one launch less than
// a value-prior kernel of its own (a launch costs 4 - 5 us, a third of that kernel's time at
// 8 heads x 32K).  Where in the kernel depends on the tile:
//  - a full tile (256 rows, NB = 8): a step's arithmetic takes microseconds, long enough to
//    hide a load, so the value rows stream in under it.  Per step a wave loads the value rows
//    of its 64 keys into the idle register buffer, squares them at mid-step into `nu_g`
//    ([problem][token], workspace) and only then requests the next key block into that
//    buffer; after the main loop the range's norms are pooled (32K tokens x 8 KV heads:
//    pass 1 43.6 -> 39.5 us against a phase after the loop).
//  - smaller tiles: the steps are too short for that (the key prefetch would have half a
//    step to arrive), and the kernel is bound by the key stream: the value rows are streamed
//    in a phase of their own after the statistics (16K tokens x 128 heads x 64 rows: 183 us
//    against 215 us interleaved).
// ENT: the chunk's mean scaled logit under its own probabilities, E_c[t] = m + u / s, is
// written to `partial_mean` beside the chunk's log2-sum-exp2; entropy_merge_kernel turns the
// chunks of a row into its entropy.
template <int D, int NB, bool ENT, bool ROWS = false, bool PRIOR = false, bool LAZY = false>
__global__ __launch_bounds__(256, 2) void bf16_pass1_kernel(ScoreGeom g, int n_qtiles, int nparts,
                                                            int total_wgs, float *partial,
                                                            float *partial_mean, float *gamma,
                                                            float *gblockmax, float *nu_g) {
    using S = TileSmem<D, NB>;
    constexpr bool kInterleave = PRIOR && NB == 8;  // value rows under the tile arithmetic
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __bf16 *sQ = (__bf16 *)smem;
    float *sLam = (float *)(smem + S::q_bytes);
    int *sPos = (int *)(sLam + S::ROWS);
    int *sBlk = sPos + 2 * S::ROWS;
    float4 *sRed = (float4 *)smem;  // reuses the query tile after the main loop
    float *sNu = (float *)(smem + S::bytes);  // kInterleave: kPriorSmem bytes behind the tile

    // logical workgroup index -> (part, tile pair, problem)
    const int wg = logical_wg_index(total_wgs, n_qtiles > 1);
    if (wg >= total_wgs) return;
    const int npairs = (n_qtiles + 1) / 2;
    const int part = wg % nparts, pair = (wg / nparts) % npairs, z = wg / (nparts * npairs);
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowMap rm{g.n, g.r, g.R,
                    ROWS ? g.rows + ((int64_t)b * g.Hq + (int64_t)h * g.G) * g.r : nullptr};
    const __bf16 *kbase = (const __bf16 *)g.k + b * g.ks[0] + h * g.ks[1];

    for (int seg = 0; seg < 2; ++seg) {
        const Segment sg = pair_segment(rm, S::ROWS, n_qtiles, pair, part, nparts, seg);
        if (sg.qt < 0) break;
        const int qt = sg.qt, rho0 = qt * S::ROWS;
        const int64_t my_off = ((int64_t)(z * n_qtiles + qt) * nparts + part) * S::ROWS;
        float *my_partial = partial + my_off;
        const int key_begin = sg.kbeg, key_end = sg.kend;
        if (key_begin >= key_end) {
            // none of this part's steps fall on this tile: leave neutral statistics
            if (tid < S::ROWS) {
                my_partial[tid] = -INFINITY;
                if (ENT) partial_mean[my_off + tid] = 0.f;
            }
            if (PRIOR && tid == 0) gblockmax[z * nparts + part] = 0.f;  // no keys, no prior
            continue;
        }
        if (seg) __syncthreads();  // the previous tile (and its reduction buffer) is done with
        // The query tile (served by the L2 after its first touch) is requested first and the
        // first key block (from HBM, behind every other workgroup's) right after it: loads
        // return in order, so the tile is in LDS and the barrier passed while the keys are
        // still on their way.
        // The first tile of a pair walks its 256-key steps upwards, the partner downwards.
        // Step i of the pair's common clock is then key step i for every workgroup still on
        // its first tile and key step (steps of a full sequence) - i for every workgroup on
        // its partner tile, whatever the pair: the workgroups of a problem, which share an
        // XCD, read the same two key blocks at any time and find them in the L2.
        const int nsteps = (key_end - key_begin + kWgKeys - 1) / kWgKeys;
        const int kdir = seg ? -kWgKeys : kWgKeys;
        const int k_at0 = (seg ? key_begin + (nsteps - 1) * kWgKeys : key_begin) + wave * kWaveKeys;
        // this wave's key block of step i; past the last step: rows clamped to the range's end
        auto kb_of = [&](int i) { return i < nsteps ? k_at0 + i * kdir : key_end; };
        bf16x8 a0[kMB][D / 16], a1[kMB][D / 16];  // the next key block loads while one multiplies
        {
            // (the thread index goes through an opaque move: the set-up's addresses are then
            // recomputed per tile instead of being kept across the main loop, where they
            // would be spilled and their reload would wait for every load in flight)
            int tid_s = tid;
            asm volatile("" : "+v"(tid_s));
            QTileRegs<D, NB> qt_regs;
            q_tile_request<D, NB, ROWS>(g, b, h, rho0, tid_s, qt_regs);
            const float lam_req = q_tile_scale<D, NB>(g, rm, rho0, tid_s);
            __builtin_amdgcn_sched_barrier(0);  // the key block is requested last
            load_a<D>(kbase, g.ks[2], kb_of(0), key_end, lane, a0);
            q_tile_meta<D, NB>(g, rm, rho0, tid_s, lam_req, sLam, sPos, sBlk);
            q_tile_commit<D, NB>(qt_regs, tid_s, sQ);
        }
        __syncthreads();

        float lam[NB], m[NB], s[NB], u[ENT ? NB : 1];
        int pos[NB], bmax[NB], bmin[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            lam[nb] = sLam[nb * 32 + (lane & 31)];
            pos[nb] = sPos[nb * 32 + (lane & 31)];
            bmax[nb] = uniform(sBlk[nb]);
            bmin[nb] = uniform(sBlk[NB + nb]);
            m[nb] = -INFINITY;
            s[nb] = 0.f;
            u[ENT ? nb : 0] = 0.f;
        }

        const int tile_min = ROWS ? tile_min_pos<NB>(sBlk) : rm.min_pos(rho0, rho0 + S::ROWS);
        // blocks [nb0, nb1) of the tile against the 64 keys at kb
        auto blocks = [&](const bf16x8 (&a)[kMB][D / 16], int kb, int nb0, int nb1) {
            if (kb >= key_end) return;  // (a wave past the range's ragged end)
            if (kb + kWaveKeys - 1 <= tile_min) {
                // every row of the tile sees all 64 keys: no masks, no skipped blocks
                bf16x8 qf = query_fragment<D, NB>(sQ, nb0, 0, lane);
#pragma unroll
                for (int nb = nb0; nb < nb1; ++nb) {
                    f32x16 acc[kMB];
                    mma_block_stream<D, NB>(a, sQ, nb, nb + 1 < nb1 ? nb + 1 : nb0, lane, qf, acc);
                    stats_update<false, ENT, LAZY>(acc, lam[nb], 0, kb, lane, m[nb], s[nb], u[ENT ? nb : 0]);
                }
                return;
            }
#pragma unroll
            for (int nb = nb0; nb < nb1; ++nb) {
                if (bmax[nb] < kb) continue;  // nothing of this block sees these keys
                f32x16 acc[kMB];
                mma_block<D, NB>(a, sQ, nb, lane, acc);
                if (kb + kWaveKeys - 1 > bmin[nb])
                    stats_update<true, ENT>(acc, lam[nb], pos[nb], kb, lane, m[nb], s[nb], u[ENT ? nb : 0]);
                else
                    stats_update<false, ENT>(acc, lam[nb], pos[nb], kb, lane, m[nb], s[nb], u[ENT ? nb : 0]);
            }
        };
        // One step: the key block in `a` against the whole tile, while `nx` receives the next
        // key block.  The loads are issued unconditionally (past the range they re-read
        // clamped rows that are never used): behind a branch the compiler can no longer tell
        // how many loads are in flight and would wait for the prefetch itself.
        auto step = [&](const bf16x8 (&a)[kMB][D / 16], bf16x8 (&nx)[kMB][D / 16], int kb,
                        int kb_next) {
            if constexpr (!kInterleave) {
                load_a<D>(kbase, g.ks[2], kb_next, key_end, lane, nx);
                blocks(a, kb, 0, NB);
            } else {
                const __bf16 *vbase = (const __bf16 *)g.v + b * g.vs[0] + h * g.vs[1];
                load_a<D>(vbase, g.vs[2], kb, key_end, lane, nx);  // the value rows of these keys
                __builtin_amdgcn_sched_barrier(0);
                blocks(a, kb, 0, (NB + 1) / 2);
                __builtin_amdgcn_sched_barrier(0);
                float nu[kMB];
                fragment_row_norms<D>(nx, nu);
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb) {
                    const int row = kb + mb * 32 + lane;
                    if (lane < 32 && row < key_end) nu_g[(int64_t)z * g.n + row] = nu[mb];
                }
                __builtin_amdgcn_sched_barrier(0);
                load_a<D>(kbase, g.ks[2], kb_next, key_end, lane, nx);
                __builtin_amdgcn_sched_barrier(0);
                blocks(a, kb, (NB + 1) / 2, NB);
            }
        };
        for (int i = 0; i < nsteps; i += 2) {
            step(a0, a1, kb_of(i), kb_of(i + 1));
            if (i + 1 >= nsteps) break;
            step(a1, a0, kb_of(i + 1), kb_of(i + 2));
        }

        PriorHalo<D> halo;  // travels while the statistics are reduced
        if constexpr (kInterleave)
            halo.request(g, (const __bf16 *)g.v + b * g.vs[0] + h * g.vs[1], key_begin, key_end, tid);
        // fold the two half-waves (same query column, different key rows); a statistic
        // (m, s, u) re-referenced to a maximum M >= m is (M, s f, (u + (m - M) s) f), f = 2^(m - M)
        auto reref = [](float m_, float mref, float &s_, float &u_) {
            const float f = fast_exp2(m_ - mref);
            if (ENT) u_ = (u_ + (m_ == -INFINITY ? 0.f : m_ - mref) * s_) * f;
            s_ *= f;
        };
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float m2 = __shfl_xor(m[nb], 32), s2 = __shfl_xor(s[nb], 32);
            float u1 = u[ENT ? nb : 0], u2 = ENT ? __shfl_xor(u1, 32) : 0.f;
            const float mn = fmaxf(m[nb], m2);
            const float mref = mn == -INFINITY ? 0.f : mn;
            reref(m[nb], mref, s[nb], u1);
            reref(m2, mref, s2, u2);
            s[nb] += s2;
            u[ENT ? nb : 0] = u1 + u2;
            m[nb] = mn;
        }
        __syncthreads();  // everyone is done reading the query tile
        if (lane < 32) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                sRed[wave * S::ROWS + nb * 32 + lane] =
                    make_float4(m[nb], s[nb], u[ENT ? nb : 0], 0.f);
        }
        __syncthreads();
        if (tid < S::ROWS) {
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) M = fmaxf(M, sRed[w * S::ROWS + tid].x);
            const float mref = M == -INFINITY ? 0.f : M;
            float sum = 0.f, mom = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float4 e = sRed[w * S::ROWS + tid];
                float sw = e.y, uw = e.z;
                reref(e.x, mref, sw, uw);
                sum += sw;
                mom += uw;
            }
            my_partial[tid] = M + log2f(sum);  // -inf for a row that saw no key
            if (ENT) partial_mean[my_off + tid] = sum > 0.f ? mref + mom / sum : 0.f;
        }
        if constexpr (kInterleave) {
            // (every wave's norms were written before the barriers of the reduction above)
            const float gm = pool_norms_of_range<D>(g, z, key_begin, key_end, nu_g, halo, sNu,
                                                    gamma, tid);
            if (tid == 0) gblockmax[z * nparts + part] = gm;
        } else if constexpr (PRIOR) {
            __syncthreads();  // the reduction buffer is done with
            const float gm = value_prior_of_range(g, b, h, z, key_begin, key_end, (float *)smem,
                                                  gamma, tid);
            if (tid == 0) gblockmax[z * nparts + part] = gm;
        }
    }
}

// ---------------------------------------------------------------- pass 2 --
// Sum of 16 per-lane values over the 32 lanes of each half-wave by recursive
// halving: after the call lane l holds the total of element
// v = 8*bit4(l) + 4*bit3(l) + 2*bit2(l) + bit1(l)   (both lanes of a pair hold it).
__device__ __forceinline__ float fold16_over32(const f32x16 &xv, int lane) {
    // The elements go through an opaque move first: otherwise the compiler turns
    // "lane-dependent choice between two elements" into a dynamically indexed
    // vector access, which costs a 16-way compare/select chain per element.
    float x[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        x[t] = xv[t];
        asm volatile("" : "+v"(x[t]));
    }
    // lanes ^ 16: v_permlane16_swap exchanges the odd 16-lane rows of its first operand with
    // the even rows of its second, so the two results are (own, partner's) copies of
    // element t in the even rows and of element t + 8 in the odd rows
    float a[8], b4[4], c2[2];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x[t]),
                                                        __float_as_uint(x[t + 8]), false, false);
        a[t] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    bool hi = lane & 8;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float send = hi ? a[t] : a[t + 4], keep = hi ? a[t + 4] : a[t];
        b4[t] = keep + from_lane_xor<8>(send);
    }
    hi = lane & 4;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const float send = hi ? b4[t] : b4[t + 2], keep = hi ? b4[t + 2] : b4[t];
        c2[t] = keep + from_lane_xor<4>(send);
    }
    hi = lane & 2;
    const float send = hi ? c2[0] : c2[1], keep = hi ? c2[1] : c2[0];
    float d = keep + from_lane_xor<2>(send);
    d += from_lane_xor<1>(d);
    return d;
}

// Log2-sum-exp2 of one query row from the per-chunk log2-sum-exp2 values that pass 1 left.
// A batch of values is requested at once (request), so that it travels together with the
// other loads of the tile set-up, and merged later (merge) into the running (M, sum) with
// sum = sum over chunks of exp2(value - M).  Both go by groups of eight and skip the
// groups past the last chunk.
template <int BATCH>
__device__ __forceinline__ void chunk_request(const float *src, int stride, int c0, int nchunks,
                                              float (&e)[BATCH]) {
    static_assert(BATCH % 8 == 0, "groups of eight");
#pragma unroll
    for (int g8 = 0; g8 < BATCH; g8 += 8) {
        if (c0 + g8 >= nchunks) break;  // uniform
        // entries past the last chunk re-read it (branch-free, back-to-back loads) and are
        // neutralised in the merge
#pragma unroll
        for (int t = g8; t < g8 + 8; ++t) e[t] = src[(int64_t)min(c0 + t, nchunks - 1) * stride];
    }
}
template <int BATCH>
__device__ __forceinline__ void chunk_merge(const float (&e)[BATCH], int count, float &M,
                                            float &sum) {
    float bm = -INFINITY;
#pragma unroll
    for (int g8 = 0; g8 < BATCH; g8 += 8) {
        if (g8 >= count) break;  // uniform
#pragma unroll
        for (int t = g8; t < g8 + 8; ++t) bm = fmaxf(bm, t < count ? e[t] : -INFINITY);
    }
    const float mn = fmaxf(M, bm);
    const float mref = mn == -INFINITY ? 0.f : mn;
    sum *= fast_exp2(M - mref);
#pragma unroll
    for (int g8 = 0; g8 < BATCH; g8 += 8) {
        if (g8 >= count) break;
#pragma unroll
        for (int t = g8; t < g8 + 8; ++t) sum += t < count ? fast_exp2(e[t] - mref) : 0.f;
    }
    M = mn;
}

// SINGLE: all observed rows fit one query tile (the windowed score).  The tile is loaded
// once, the workgroup walks over several 256-key steps and the A fragments of the next
// step load while the current one multiplies; every score is written exactly once.
// Otherwise (full accumulation) the grid is (part, tile pair, problem) as in pass 1 and the
// tiles' contributions meet in the scores through float atomics.
template <int D, int NB, bool SINGLE, bool ROWS = false>
__global__ __launch_bounds__(256, 2) void bf16_pass2_kernel(ScoreGeom g, int n_qtiles,
                                                            int total_wgs, int wg_keys, int nchunks,
                                                            const float *partial,
                                                            const float *gamma,
                                                            const float *gblockmax,
                                                            int n_vtiles, float *scores) {
    using S = TileSmem<D, NB>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __bf16 *sQ = (__bf16 *)smem;
    float *sLam = (float *)(smem + S::q_bytes);
    int *sPos = (int *)(sLam + S::ROWS);
    float *sL = (float *)(sPos + S::ROWS);
    int *sBlk = (int *)(sL + S::ROWS);
    __shared__ float s_gmax[4];

    // logical workgroup index -> SINGLE: (key range, problem); else (part, tile pair, problem)
    const int wg = logical_wg_index(total_wgs, !SINGLE);
    if (wg >= total_wgs) return;
    const int per_problem = total_wgs / (g.batch * g.Hkv);
    const int z = wg / per_problem, wg_in_z = wg % per_problem;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowMap rm{g.n, g.r, g.R,
                    ROWS ? g.rows + ((int64_t)b * g.Hq + (int64_t)h * g.G) * g.r : nullptr};
    const __bf16 *kbase = (const __bf16 *)g.k + b * g.ks[0] + h * g.ks[1];
    // SINGLE: the workgroup's key range; otherwise ranges come per tile segment (below)
    int key_begin = wg_in_z * wg_keys;
    int key_end = min(g.n, key_begin + wg_keys);

    bf16x8 a0[kMB][D / 16];
    // (the windowed pass walks its key range from the last step to the first)
    const int last_step = key_begin + (key_end - key_begin - 1) / kWgKeys * kWgKeys;

    // this thread's share of the value prior's per-tile maxima (requested here, reduced
    // during the first tile set-up)
    float gm = (g.value_prior && tid < n_vtiles) ? gblockmax[z * n_vtiles + tid] : 0.f;
    bool gmax_pending = g.value_prior;
    float lamr[NB], Lr[NB];  // scale and log-sum-exp of this lane's query column, per block

    // query tile qt -> LDS, with the log-sum-exp of its rows folded from pass 1's chunks
    static_assert(S::ROWS <= 256, "one thread folds the statistics of one tile row");
    // `first_kb`: the wave's first key block of the tile, requested right behind the tile's
    // own (L2-served) loads so that those are not queued behind the keys coming from HBM
    int tile_min = 0;  // smallest position among the rows of the tile in LDS
    auto load_tile = [&](int qt, int first_kb) {
        const int rho0 = qt * S::ROWS;
        // Full accumulation sets up a tile per segment: there the thread index and the chunk
        // count go through an opaque move, so that the set-up's address arithmetic is
        // redone per tile instead of being kept (and spilled) across the main loop, where
        // a reload of a spilled address would have to wait for every load in flight.
        int tid = threadIdx.x, nchunks_t = nchunks;
        if (!SINGLE) {
            asm volatile("" : "+v"(tid));
            asm volatile("" : "+s"(nchunks_t));
        }
        {
            // tile rows, chunk statistics and scales are requested together, then used
            QTileRegs<D, NB> qt_regs;
            // (windowed mode has up to 64 chunks per row; full accumulation a few, and less
            // room in the register file at this point)
            constexpr int kChunkBatch = SINGLE ? 64 : 8;
            float ch[kChunkBatch];
            const bool row_ok = tid < S::ROWS && rho0 + tid < g.R;
            // (threads without a row of their own read row 0's statistics and drop them)
            const float *psrc = partial + ((int64_t)(z * n_qtiles + qt) * nchunks_t) * S::ROWS +
                                 (tid < S::ROWS ? tid : 0);
            q_tile_request<D, NB, ROWS>(g, b, h, rho0, tid, qt_regs);
            chunk_request(psrc, S::ROWS, 0, nchunks_t, ch);
            const float lam_req = q_tile_scale<D, NB>(g, rm, rho0, tid);
            __builtin_amdgcn_sched_barrier(0);  // the key block is requested last
            load_a<D>(kbase, g.ks[2], first_kb, key_end, lane, a0);
            q_tile_meta<D, NB>(g, rm, rho0, tid, lam_req, sLam, sPos, sBlk);
            if (gmax_pending) {
                for (int t = tid + 256; t < n_vtiles; t += 256)
                    gm = fmaxf(gm, gblockmax[z * n_vtiles + t]);
                gm = wave_max(gm);
                if (lane == 0) s_gmax[wave] = gm;
                gmax_pending = false;
            }
            float M = -INFINITY, sum = 0.f;
            chunk_merge(ch, nchunks_t, M, sum);
            for (int c0 = kChunkBatch; c0 < nchunks_t; c0 += kChunkBatch) {
                chunk_request(psrc, S::ROWS, c0, nchunks_t, ch);
                chunk_merge(ch, nchunks_t - c0, M, sum);
            }
            if (tid < S::ROWS) sL[tid] = row_ok ? M + log2f(sum) : INFINITY;
            q_tile_commit<D, NB>(qt_regs, tid, sQ);
        }
        __syncthreads();
        tile_min = ROWS ? tile_min_pos<NB>(sBlk) : rm.min_pos(rho0, rho0 + S::ROWS);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            lamr[nb] = sLam[nb * 32 + (tid & 31)];
            Lr[nb] = sL[nb * 32 + (tid & 31)];
        }
    };
    // this wave's 64 keys (A fragments a) against the query tile in LDS
    auto tile_times_keys = [&](const bf16x8 (&a)[kMB][D / 16], int kb, int rho0,
                               f32x16 (&col)[kMB]) {
        if (kb + kWaveKeys - 1 <= tile_min) {
            // all rows of the tile see all 64 keys: no masks, no skipped blocks
            bf16x8 qf = query_fragment<D, NB>(sQ, 0, 0, lane);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                f32x16 acc[kMB];
                mma_block_stream<D, NB>(a, sQ, nb, nb + 1 < NB ? nb + 1 : 0, lane, qf, acc);
                colsum_update<false>(acc, lamr[nb], Lr[nb], 0, kb, lane, col);
            }
            return;
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (uniform(sBlk[nb]) < kb) continue;
            f32x16 acc[kMB];
            mma_block<D, NB>(a, sQ, nb, lane, acc);
            const int pos = sPos[nb * 32 + (lane & 31)];
            if (kb + kWaveKeys - 1 > uniform(sBlk[NB + nb]))
                colsum_update<true>(acc, lamr[nb], Lr[nb], pos, kb, lane, col);
            else
                colsum_update<false>(acc, lamr[nb], Lr[nb], pos, kb, lane, col);
        }
    };
    // The value-prior factors of the (up to two) scores this lane will write are requested
    // when a step starts, so that their latency is hidden behind the step's arithmetic.
    const int my_v = ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 +
                     ((lane >> 1) & 1);
    auto request_gamma = [&](int kb, float (&gam)[kMB]) {
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            const int j = acc_key(kb, mb, my_v, lane);
            gam[mb] = (g.value_prior && j < g.n) ? gamma[(int64_t)z * g.n + j] : 1.f;
        }
    };
    // fold the 32 lanes of each half-wave and write the 64 scores of this wave's keys
    auto write_scores = [&](f32x16 (&col)[kMB], int kb, const float (&gam)[kMB]) {
        float ginv = 1.f;
        if (g.value_prior)  // s_gmax was published by the barrier of the first tile load
            ginv = prior_inverse(fmaxf(fmaxf(s_gmax[0], s_gmax[1]), fmaxf(s_gmax[2], s_gmax[3])));
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            const float tot = fold16_over32(col[mb], lane);
            const int j = acc_key(kb, mb, my_v, lane);
            if ((lane & 1) == 0 && j < g.n) scores[(int64_t)z * g.n + j] = tot * prior_factor(gam[mb], ginv);
        }
    };
    auto zero = [&](f32x16 (&col)[kMB]) {
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) col[mb][v] = 0.f;
    };

    if constexpr (SINGLE) {
        load_tile(0, last_step + wave * kWaveKeys);
        bf16x8 a1[kMB][D / 16];
        auto step = [&](const bf16x8 (&a)[kMB][D / 16], int kb0) {
            const int kb = kb0 + wave * kWaveKeys;
            if (kb >= g.n) return;
            float gam[kMB];
            request_gamma(kb, gam);
            f32x16 col[kMB];
            zero(col);
            tile_times_keys(a, kb, 0, col);
            write_scores(col, kb, gam);
        };
        // (unconditional prefetch, as in pass 1)
        for (int kb0 = last_step; kb0 >= key_begin; kb0 -= 2 * kWgKeys) {
            const int k1 = kb0 - kWgKeys, k2 = k1 - kWgKeys;
            // before the range: kb = key_end makes every row read the range's last one
            load_a<D>(kbase, g.ks[2], k1 >= key_begin ? k1 + wave * kWaveKeys : key_end, key_end,
                      lane, a1);
            step(a0, kb0);
            if (k1 < key_begin) break;
            load_a<D>(kbase, g.ks[2], k2 >= key_begin ? k2 + wave * kWaveKeys : key_end, key_end,
                      lane, a0);
            step(a1, k1);
        }
    } else {
        // full accumulation: this workgroup keeps ONE query tile in LDS and streams its keys
        // like pass 1; the 64 column sums of a wave step are this tile's contribution and are
        // added to the (zero-initialised) scores with hardware float atomics, already
        // multiplied by the value prior.  The order of the additions over the tiles is not
        // fixed, so repeated calls may differ in the last bits.
        // wg_keys carries the number of parts a tile pair's key steps are cut into
        const int nparts = wg_keys, part = wg_in_z % nparts, pair = wg_in_z / nparts;
        bf16x8 a1[kMB][D / 16];
        for (int seg = 0; seg < 2; ++seg) {
            const Segment sg = pair_segment(rm, S::ROWS, n_qtiles, pair, part, nparts, seg);
            if (sg.qt < 0) break;
            key_begin = sg.kbeg;
            key_end = sg.kend;
            if (key_begin >= key_end) continue;  // workgroup-uniform
            const int rho0 = sg.qt * S::ROWS;
            if (seg) __syncthreads();  // the previous tile is done with
            // (first tile upwards, partner downwards: see pass 1)
            const int nsteps = (key_end - key_begin + kWgKeys - 1) / kWgKeys;
            const int kdir = seg ? -kWgKeys : kWgKeys;
            const int k_at0 = seg ? key_begin + (nsteps - 1) * kWgKeys : key_begin;
            auto kb0_of = [&](int i) { return k_at0 + i * kdir; };
            auto load_kb_of = [&](int i) { return i < nsteps ? kb0_of(i) + wave * kWaveKeys : key_end; };
            load_tile(sg.qt, load_kb_of(0));
            float ginv = 1.f;
            if (g.value_prior)
                ginv = prior_inverse(fmaxf(fmaxf(s_gmax[0], s_gmax[1]), fmaxf(s_gmax[2], s_gmax[3])));
            auto step = [&](const bf16x8 (&a)[kMB][D / 16], int kb0) {
                const int kb = kb0 + wave * kWaveKeys;
                if (kb >= key_end) return;
                float gam[kMB];
                request_gamma(kb, gam);
                f32x16 col[kMB];
                zero(col);
                tile_times_keys(a, kb, rho0, col);
#pragma unroll
                for (int mb = 0; mb < kMB; ++mb) {
                    const float tot = fold16_over32(col[mb], lane);
                    const int j = acc_key(kb, mb, my_v, lane);
                    if ((lane & 1) == 0 && j < key_end)
                        unsafeAtomicAdd(&scores[(int64_t)z * g.n + j], tot * prior_factor(gam[mb], ginv));
                }
            };
            for (int i = 0; i < nsteps; i += 2) {
                load_a<D>(kbase, g.ks[2], load_kb_of(i + 1), key_end, lane, a1);
                step(a0, kb0_of(i));
                if (i + 1 >= nsteps) break;
                load_a<D>(kbase, g.ks[2], load_kb_of(i + 2), key_end, lane, a0);
                step(a1, kb0_of(i + 1));
            }
        }
    }
}

// Row statistics out (Sec. 4.2): from pass 1's per-chunk log2-sum-exp2 L_c and mean scaled
// logit E_c, the row's natural-log normaliser lse = ln 2 * L, L = log2 sum_c 2^L_c, and its
// entropy H = ln 2 * (L - sum_c 2^(L_c - L) E_c).  One thread per observed row.
__global__ __launch_bounds__(256) void row_stats_merge_kernel(ScoreGeom g, int rows_tile,
                                                              int n_qtiles, int nparts,
                                                              const float *partial,
                                                              const float *partial_mean,
                                                              float *lse, float *entropy) {
    const int z = blockIdx.y, rho = blockIdx.x * 256 + threadIdx.x;
    if (rho >= g.R) return;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int qt = rho / rows_tile, row = rho % rows_tile;
    const float *pl = partial + ((int64_t)(z * n_qtiles + qt) * nparts) * rows_tile + row;
    const float *pm = partial_mean + ((int64_t)(z * n_qtiles + qt) * nparts) * rows_tile + row;
    float M = -INFINITY;
    for (int c = 0; c < nparts; ++c) M = fmaxf(M, pl[(int64_t)c * rows_tile]);
    float sum = 0.f, mean = 0.f;
    for (int c = 0; c < nparts; ++c) {
        const float wgt = exp2f(pl[(int64_t)c * rows_tile] - M);  // 0 for a chunk without keys
        sum += wgt;
        mean = fmaf(wgt, pm[(int64_t)c * rows_tile], mean);
    }
    const float L = M + log2f(sum);
    const int gi = rho / g.r, ii = rho - gi * g.r;
    const int64_t o = ((int64_t)b * g.Hq + h * g.G + gi) * g.r + ii;
    const float kLn2 = 0.69314718055994531f;
    if (lse) lse[o] = L * kLn2;
    if (entropy) entropy[o] = fmaxf(0.f, (L - mean / sum) * kLn2);
}

// ---------------------------------------------------------------- launch --
template <int D, int NB>
static hipError_t launch_t(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                           hipStream_t st, hipEvent_t mid, bool have_lse, bool fold_prior) {
    using S = TileSmem<D, NB>;
    static_assert(2 * (S::bytes + kPriorSmem) <= 160 * 1024, "two workgroups per CU");
    static_assert(S::bytes >= kPriorTailSmem, "the prior's own phase borrows the query tile's LDS");
    char *w = (char *)ws;
    float *partial = (float *)(w + pl.off_partial);
    float *gamma = (float *)(w + pl.off_gamma);
    float *gbm = (float *)(w + pl.off_gblockmax);
    float *nu = (float *)(w + pl.off_nu);
    static DeviceOnce once;
    const hipError_t ea = device_once(once, [] {
        const void *kernels[8] = {(const void *)bf16_pass1_kernel<D, NB, false>,
                                  (const void *)bf16_pass1_kernel<D, NB, false, false, false, true>,
                                  (const void *)bf16_pass1_kernel<D, NB, false, false, true>,
                                  (const void *)bf16_pass1_kernel<D, NB, true>,
                                  (const void *)bf16_pass1_kernel<D, NB, false, true>,
                                  (const void *)bf16_pass2_kernel<D, NB, true>,
                                  (const void *)bf16_pass2_kernel<D, NB, true, true>,
                                  (const void *)bf16_pass2_kernel<D, NB, false>};
        for (const void *kf : kernels) {
            const hipError_t e = hipFuncSetAttribute(
                kf, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(S::bytes + kPriorSmem));
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    });
    if (ea != hipSuccess) return ea;
    // (part, tile pair, problem), part fastest
    const int64_t wgs1 = (int64_t)pl.nchunks * ((pl.n_qtiles + 1) / 2) * pl.Z;
    // windowed pass 2: (key range, problem)
    const int64_t wgs2 = (int64_t)((g.n + pl.p2_keys - 1) / pl.p2_keys) * pl.Z;
    // with the caller's row normalisers already in place (one "chunk" per row) pass 1 is skipped
    if (!have_lse) {
        if (g.rows)
            hipLaunchKernelGGL((bf16_pass1_kernel<D, NB, false, true>), xcd_grid(wgs1), dim3(256),
                               S::bytes, st, g, pl.n_qtiles, pl.nchunks, (int)wgs1, partial,
                               (float *)nullptr, (float *)nullptr, (float *)nullptr,
                               (float *)nullptr);
        else if (fold_prior)
            hipLaunchKernelGGL((bf16_pass1_kernel<D, NB, false, false, true>), xcd_grid(wgs1),
                               dim3(256), S::bytes + kPriorSmem, st, g, pl.n_qtiles, pl.nchunks, (int)wgs1,
                               partial, (float *)nullptr, gamma, gbm, nu);
        else if (pl.n_qtiles > 1)  // full accumulation: block sums against a lazy reference
            hipLaunchKernelGGL((bf16_pass1_kernel<D, NB, false, false, false, true>), xcd_grid(wgs1),
                               dim3(256), S::bytes, st, g, pl.n_qtiles, pl.nchunks, (int)wgs1,
                               partial, (float *)nullptr, (float *)nullptr, (float *)nullptr,
                               (float *)nullptr);
        else
            hipLaunchKernelGGL((bf16_pass1_kernel<D, NB, false>), xcd_grid(wgs1), dim3(256),
                               S::bytes, st, g, pl.n_qtiles, pl.nchunks, (int)wgs1, partial,
                               (float *)nullptr, (float *)nullptr, (float *)nullptr,
                               (float *)nullptr);
    }
    const int stat_chunks = have_lse ? 1 : pl.nchunks;
    // the prior's per-range maxima: one per key chunk when pass 1 formed it, else per tile
    const int n_maxima = fold_prior ? pl.nchunks : pl.n_vtiles;
    if (mid) (void)hipEventRecord(mid, st);
    if (pl.n_qtiles == 1 && g.rows)
        hipLaunchKernelGGL((bf16_pass2_kernel<D, NB, true, true>), xcd_grid(wgs2), dim3(256),
                           S::bytes, st, g, pl.n_qtiles, (int)wgs2, pl.p2_keys, stat_chunks,
                           partial, gamma, gbm, n_maxima, scores);
    else if (pl.n_qtiles == 1)
        hipLaunchKernelGGL((bf16_pass2_kernel<D, NB, true>), xcd_grid(wgs2), dim3(256), S::bytes,
                           st, g, pl.n_qtiles, (int)wgs2, pl.p2_keys, stat_chunks, partial,
                           gamma, gbm, n_maxima, scores);
    else
        hipLaunchKernelGGL((bf16_pass2_kernel<D, NB, false>), xcd_grid(wgs1), dim3(256), S::bytes,
                           st, g, pl.n_qtiles, (int)wgs1, pl.nchunks, stat_chunks, partial,
                           gamma, gbm, n_maxima, scores);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                           hipStream_t st, hipEvent_t mid, bool have_lse, bool fold_prior) {
    switch (pl.NB) {
        case 1: return launch_t<D, 1>(g, pl, ws, scores, st, mid, have_lse, fold_prior);
        case 2: return launch_t<D, 2>(g, pl, ws, scores, st, mid, have_lse, fold_prior);
        case 4: return launch_t<D, 4>(g, pl, ws, scores, st, mid, have_lse, fold_prior);
        default: return launch_t<D, 8>(g, pl, ws, scores, st, mid, have_lse, fold_prior);
    }
}

template <int D, int NB>
static hipError_t launch_stats_t(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *lse,
                                 float *entropy, hipStream_t st) {
    using S = TileSmem<D, NB>;
    char *w = (char *)ws;
    float *partial = (float *)(w + pl.off_partial);
    float *partial_mean = (float *)(w + pl.off_partial_mean);
    static DeviceOnce once;
    const hipError_t ea = device_once(once, [] {
        return hipFuncSetAttribute((const void *)bf16_pass1_kernel<D, NB, true>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::bytes);
    });
    if (ea != hipSuccess) return ea;
    const int64_t wgs1 = (int64_t)pl.nchunks * ((pl.n_qtiles + 1) / 2) * pl.Z;
    hipLaunchKernelGGL((bf16_pass1_kernel<D, NB, true>), xcd_grid(wgs1), dim3(256), S::bytes, st,
                       g, pl.n_qtiles, pl.nchunks, (int)wgs1, partial, partial_mean,
                       (float *)nullptr, (float *)nullptr, (float *)nullptr);
    const hipError_t e1 = hipGetLastError();
    if (e1 != hipSuccess) return e1;
    hipLaunchKernelGGL(row_stats_merge_kernel, dim3((g.R + 255) / 256, pl.Z), dim3(256), 0, st, g,
                       pl.qtile, pl.n_qtiles, pl.nchunks, partial, partial_mean, lse, entropy);
    return hipGetLastError();
}

hipError_t launch_row_stats_bf16(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *lse,
                                 float *entropy, hipStream_t st) {
#define AHA_STATS(DD)                                                         \
    switch (pl.NB) {                                                          \
        case 1: return launch_stats_t<DD, 1>(g, pl, ws, lse, entropy, st);    \
        case 2: return launch_stats_t<DD, 2>(g, pl, ws, lse, entropy, st);    \
        case 4: return launch_stats_t<DD, 4>(g, pl, ws, lse, entropy, st);    \
        default: return launch_stats_t<DD, 8>(g, pl, ws, lse, entropy, st);   \
    }
    if (g.d == 64) { AHA_STATS(64) }
    AHA_STATS(128)
#undef AHA_STATS
}

hipError_t launch_score_bf16(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                             hipStream_t st, hipEvent_t mid, bool have_lse, bool fold_prior) {
    return g.d == 64 ? launch_d<64>(g, pl, ws, scores, st, mid, have_lse, fold_prior)
                     : launch_d<128>(g, pl, ws, scores, st, mid, have_lse, fold_prior);
}

}  // namespace aha

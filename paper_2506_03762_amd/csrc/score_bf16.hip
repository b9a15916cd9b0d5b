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
// independently between the tile barriers.
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

constexpr int kMB = 2;                 // 32-key M blocks per wave step
constexpr int kWaveKeys = 32 * kMB;    // keys per wave step
constexpr int kWgKeys = 4 * kWaveKeys; // keys per workgroup step (= kP2Keys)
static_assert(kWgKeys == kP2Keys, "pass-2 grid assumes 256 keys per workgroup");

template <int D, int NB>
struct TileSmem {
    static constexpr int LD = D + 8;  // padded row, 16-byte aligned, conflict-free b128 reads
    static constexpr int ROWS = NB * 32;
    static constexpr size_t q_bytes = (size_t)ROWS * LD * 2;
    // query tile, then per row: scale, position, log-sum-exp; then per block: max / min position
    static constexpr size_t bytes = q_bytes + ROWS * 4 * 3 + NB * 4 * 2;
};

// Query tile -> LDS: rows rho0 .. rho0+ROWS of the KV head's flattened query
// rows (zero beyond R), per row the log2-domain scale and the position, and per
// 32-row block the largest and smallest position.  Two halves, so that other
// loads can be put in flight between the global requests and their use.
template <int D, int NB>
struct QTileRegs {
    static constexpr int UT = TileSmem<D, NB>::ROWS * (D / 8) / 256;  // 16-byte chunks per thread
    static_assert(TileSmem<D, NB>::ROWS * (D / 8) % 256 == 0, "tile chunks divide among 256 threads");
    static constexpr int U = UT < 8 ? UT : 8;   // chunks per batch (bounds the registers held)
    static constexpr int BATCHES = UT / U;
    u32x4 w[U];
};

template <int D, int NB>
__device__ __forceinline__ void q_tile_request(const ScoreGeom &g, int b, int h, int rho0,
                                               int batch, QTileRegs<D, NB> &t) {
    constexpr int CPR = D / 8;
    const int tid = threadIdx.x;
#pragma unroll
    for (int u = 0; u < QTileRegs<D, NB>::U; ++u) {
        const int i = tid + (batch * QTileRegs<D, NB>::U + u) * 256;
        const int rr = i / CPR, c = i % CPR, rho = rho0 + rr;
        t.w[u] = u32x4{0u, 0u, 0u, 0u};
        if (rho < g.R) {
            const int gi = rho / g.r, ii = rho - gi * g.r;
            const __bf16 *src = (const __bf16 *)g.q + b * g.qs[0] + (h * g.G + gi) * g.qs[1] +
                                (int64_t)(g.n - g.r + ii) * g.qs[2] + c * 8;
            t.w[u] = *(const u32x4 *)src;
        }
    }
}

template <int D, int NB>
__device__ __forceinline__ void q_tile_commit(int batch, const QTileRegs<D, NB> &t, __bf16 *sQ) {
    using S = TileSmem<D, NB>;
    constexpr int CPR = D / 8;
    const int tid = threadIdx.x;
#pragma unroll
    for (int u = 0; u < QTileRegs<D, NB>::U; ++u) {
        const int i = tid + (batch * QTileRegs<D, NB>::U + u) * 256;
        *(u32x4 *)(sQ + (i / CPR) * S::LD + (i % CPR) * 8) = t.w[u];
    }
}

template <int D, int NB>
__device__ __forceinline__ void q_tile_meta(const ScoreGeom &g, const RowMap &rm, int rho0,
                                            const float *lam_tab, float *sLam, int *sPos,
                                            int *sBlk) {
    using S = TileSmem<D, NB>;
    const int tid = threadIdx.x;
    for (int rr = tid; rr < S::ROWS; rr += 256) {
        const int rho = rho0 + rr;
        const bool ok = rho < g.R;
        const int ii = ok ? rho % g.r : 0;
        sPos[rr] = ok ? g.n - g.r + ii : -1;
        sLam[rr] = ok ? lam_tab[ii] : 0.f;
    }
    if (tid < NB) {
        sBlk[tid] = rm.max_pos(rho0 + tid * 32, rho0 + tid * 32 + 32);
        sBlk[NB + tid] = rm.min_pos(rho0 + tid * 32, rho0 + tid * 32 + 32);
    }
}

// A fragments of a wave's key block: lane holds row kb + mb*32 + lane%32,
// channels ks*16 + (lane/32)*8 .. +8.  Rows past the sequence are clamped
// (their results are masked or never written).
template <int D>
__device__ __forceinline__ void load_a(const __bf16 *kbase, int64_t k_tstride, int kb, int n,
                                       int lane, bf16x8 (&a)[kMB][D / 16]) {
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
        const int row = min(kb + mb * 32 + (lane & 31), n - 1);
        const __bf16 *p = kbase + (int64_t)row * k_tstride + (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) a[mb][ks] = *(const bf16x8 *)(p + ks * 16);
    }
}

template <int D, int NB>
__device__ __forceinline__ void mma_block(const bf16x8 (&a)[kMB][D / 16], const __bf16 *sQ,
                                          int nb, int lane, f32x16 (&acc)[kMB]) {
    using S = TileSmem<D, NB>;
    const __bf16 *bp = sQ + (nb * 32 + (lane & 31)) * S::LD + (lane >> 5) * 8;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 bfrag = *(const bf16x8 *)(bp + ks * 16);
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb][ks], bfrag, acc[mb], 0, 0, 0);
    }
}

// Key row of accumulator element v of M block mb, for this lane.
__device__ __forceinline__ int acc_key(int kb, int mb, int v, int lane) {
    return kb + mb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

// Online max / sum-of-exp2 of one 64 x 32 block for this lane's query column.
// The scale is non-negative, so the maximum of the scaled logits is the scale
// times the maximum raw dot.
template <bool MASK>
__device__ __forceinline__ void stats_update(const f32x16 (&acc)[kMB], float lam, int pos, int kb,
                                             int lane, float &m, float &s) {
    if (MASK) asm volatile("" ::: "memory");
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
    float sum = 0.f;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float e = fast_exp2(fmaf(acc[mb][v], lam, -mref));
            if (MASK && acc_key(kb, mb, v, lane) > pos) e = 0.f;
            sum += e;
        }
    s = s * fast_exp2(m - mref) + sum;
    m = mn;
}

template <bool MASK>
__device__ __forceinline__ void colsum_update(const f32x16 (&acc)[kMB], float lam, float L,
                                              int pos, int kb, int lane, f32x16 (&col)[kMB]) {
    // The empty asm keeps the masked and the unmasked instantiation apart: without it the
    // compiler merges the two branches and every block pays the per-element compare/select.
    if (MASK) asm volatile("" ::: "memory");
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

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// ---- straight-line (unmasked) wave step, software-pipelined by hand ----
// The matrix pipe needs 8 passes (32 cycles) per MFMA while issuing one takes a
// single slot, so the vector-ALU work on the PREVIOUS query block is placed
// between the MFMAs of the NEXT one: 16 slots per block, each one MFMA plus a
// fixed share of the exponentials.  sched_barrier(0) pins that order; the LDS
// fragment of k-step ks+2 is requested while k-step ks is being multiplied.
template <int D, int NB>
__device__ __forceinline__ bf16x8 ld_bfrag(const __bf16 *sQ, int nb, int ks, int lane) {
    using S = TileSmem<D, NB>;
    return *(const bf16x8 *)(sQ + (nb * 32 + (lane & 31)) * S::LD + (lane >> 5) * 8 + ks * 16);
}

// MFMAs of block nb into `nxt`, with work(slot) for slot = 0..2*KS-1 in between.
template <int D, int NB, typename F>
__device__ __forceinline__ void mma_block_with(const bf16x8 (&a)[kMB][D / 16], const __bf16 *sQ,
                                               int nb, int lane, f32x16 (&nxt)[kMB], F work) {
    constexpr int KS = D / 16;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) nxt[mb][v] = 0.f;
    bf16x8 bf[3];
    bf[0] = ld_bfrag<D, NB>(sQ, nb, 0, lane);
    bf[1] = ld_bfrag<D, NB>(sQ, nb, 1, lane);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (ks + 2 < KS) bf[(ks + 2) % 3] = ld_bfrag<D, NB>(sQ, nb, ks + 2, lane);
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            nxt[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb][ks], bf[ks % 3], nxt[mb], 0, 0, 0);
            float *pin = work(ks * kMB + mb);
            // tie this slot's vector work to the operand of the NEXT MFMA, so that it cannot
            // be deferred until all MFMAs of the block have been issued
            if (pin) {
                if (mb + 1 < kMB)
                    asm volatile("" : "+v"(*pin), "+v"(bf[ks % 3]));
                else if (ks + 1 < KS)
                    asm volatile("" : "+v"(*pin), "+v"(bf[(ks + 1) % 3]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Pass 2 keeps the plain order (all MFMAs of a block, then its exponentials): with the
// column sums, the A fragments and the per-block constants resident, a second accumulator
// set does not fit in 256 registers, and two waves per SIMD overlap the two pipes anyway.
template <int D, int NB>
__device__ __forceinline__ void fast_step_pass2(const bf16x8 (&a)[kMB][D / 16], const __bf16 *sQ,
                                                const float (&lamr)[NB], const float (&Lr)[NB],
                                                int lane, f32x16 (&col)[kMB]) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        f32x16 acc[kMB];
        mma_block<D, NB>(a, sQ, nb, lane, acc);
        colsum_update<false>(acc, lamr[nb], Lr[nb], 0, 0, lane, col);
    }
}

template <int D, int NB>
__device__ __forceinline__ void fast_step_pass1(const bf16x8 (&a)[kMB][D / 16], const __bf16 *sQ,
                                                const float (&lam)[NB], int lane, float (&m)[NB],
                                                float (&s)[NB]) {
    constexpr int SLOTS = kMB * (D / 16);
    // slots 0, 1: block maximum; slot 1 also rescales the running sum; the remaining
    // slots share the 32 exponentials
    constexpr int ES = SLOTS - 2;
    f32x16 acc[2][kMB];
    mma_block_with<D, NB>(a, sQ, 0, lane, acc[0], [](int) -> float * { return nullptr; });
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        f32x16(&cur)[kMB] = acc[nb & 1];
        const float lm = lam[nb];
        float amax0 = -INFINITY, amax1 = -INFINITY, mref = 0.f, sum = 0.f;
        auto work = [&](int slot) -> float * {
            if (slot == 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) amax0 = fmaxf(amax0, cur[0][v]);
                return &amax0;
            } else if (slot == 1) {
#pragma unroll
                for (int v = 0; v < 16; ++v) amax1 = fmaxf(amax1, cur[kMB - 1][v]);
                const float mn = fmaxf(m[nb], fmaxf(amax0, amax1) * lm);
                mref = mn;  // finite: every key of an unmasked block is visible
                s[nb] *= fast_exp2(m[nb] - mref);
                m[nb] = mn;
                return &mref;
            } else {
#pragma unroll
                for (int e = (slot - 2) * 32 / ES; e < (slot - 1) * 32 / ES; ++e)
                    sum += fast_exp2(fmaf(cur[e >> 4][e & 15], lm, -mref));
                return &sum;
            }
        };
        if (nb + 1 < NB) {
            mma_block_with<D, NB>(a, sQ, nb + 1, lane, acc[(nb + 1) & 1], work);
        } else {
#pragma unroll
            for (int slot = 0; slot < SLOTS; ++slot) work(slot);
        }
        s[nb] += sum;
    }
}

// ---------------------------------------------------------------- pass 1 --
template <int D, int NB>
__global__ __launch_bounds__(256, 2) void bf16_pass1_kernel(ScoreGeom g, int n_qtiles,
                                                            int chunk_keys, int nchunks,
                                                            const float *lam_tab,
                                                            float2 *partial) {
    using S = TileSmem<D, NB>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __bf16 *sQ = (__bf16 *)smem;
    float *sLam = (float *)(smem + S::q_bytes);
    int *sPos = (int *)(sLam + S::ROWS);
    int *sBlk = sPos + 2 * S::ROWS;
    float2 *sRed = (float2 *)smem;  // reuses the query tile after the main loop

    const int chunk = blockIdx.x, qt = blockIdx.y, z = blockIdx.z;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowMap rm{g.n, g.r, g.R};
    const int rho0 = qt * S::ROWS;
    const __bf16 *kbase = (const __bf16 *)g.k + b * g.ks[0] + h * g.ks[1];

    // the first key block is requested before the query tile, so both latencies overlap
    const int key_begin = chunk * chunk_keys;
    const int key_end = min(rm.max_pos(rho0, rho0 + S::ROWS) + 1, key_begin + chunk_keys);
    const int kb_first = key_begin + wave * kWaveKeys;
    bf16x8 a[kMB][D / 16];
    load_a<D>(kbase, g.ks[2], min(kb_first, g.n - 1), g.n, lane, a);
    {
        QTileRegs<D, NB> qt_regs;
#pragma unroll
        for (int bt = 0; bt < QTileRegs<D, NB>::BATCHES; ++bt) {
            q_tile_request<D, NB>(g, b, h, rho0, bt, qt_regs);
            q_tile_commit<D, NB>(bt, qt_regs, sQ);
        }
        q_tile_meta<D, NB>(g, rm, rho0, lam_tab, sLam, sPos, sBlk);
    }
    __syncthreads();

    float lam[NB], m[NB], s[NB];
    int pos[NB], bmax[NB], bmin[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        lam[nb] = sLam[nb * 32 + (lane & 31)];
        pos[nb] = sPos[nb * 32 + (lane & 31)];
        bmax[nb] = uniform(sBlk[nb]);
        bmin[nb] = uniform(sBlk[NB + nb]);
        m[nb] = -INFINITY;
        s[nb] = 0.f;
    }

    const int tile_min = rm.min_pos(rho0, rho0 + S::ROWS);
    for (int kb = kb_first; kb < key_end; kb += kWgKeys) {
        if (kb != kb_first) load_a<D>(kbase, g.ks[2], kb, g.n, lane, a);
        if (kb + kWaveKeys - 1 <= tile_min) {
            // every row of the tile sees all 64 keys: pipelined straight-line code
            fast_step_pass1<D, NB>(a, sQ, lam, lane, m, s);
            continue;
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (bmax[nb] < kb) continue;  // nothing of this block sees these keys
            f32x16 acc[kMB];
            mma_block<D, NB>(a, sQ, nb, lane, acc);
            if (kb + kWaveKeys - 1 > bmin[nb])
                stats_update<true>(acc, lam[nb], pos[nb], kb, lane, m[nb], s[nb]);
            else
                stats_update<false>(acc, lam[nb], pos[nb], kb, lane, m[nb], s[nb]);
        }
    }

    // fold the two half-waves (same query column, different key rows)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const float m2 = __shfl_xor(m[nb], 32), s2 = __shfl_xor(s[nb], 32);
        const float mn = fmaxf(m[nb], m2);
        const float mref = mn == -INFINITY ? 0.f : mn;
        s[nb] = s[nb] * fast_exp2(m[nb] - mref) + s2 * fast_exp2(m2 - mref);
        m[nb] = mn;
    }
    __syncthreads();  // everyone is done reading the query tile
    if (lane < 32) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) sRed[wave * S::ROWS + nb * 32 + lane] = make_float2(m[nb], s[nb]);
    }
    __syncthreads();
    float2 *my_partial = partial + ((int64_t)(z * n_qtiles + qt) * nchunks) * S::ROWS;
    if (tid < S::ROWS) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sRed[w * S::ROWS + tid].x);
        const float mref = M == -INFINITY ? 0.f : M;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float2 e = sRed[w * S::ROWS + tid];
            sum += e.y * fast_exp2(e.x - mref);
        }
        my_partial[(int64_t)chunk * S::ROWS + tid] = make_float2(M, sum);
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
    float a[8], b4[4], c2[2];
    bool hi = lane & 16;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const float send = hi ? x[t] : x[t + 8], keep = hi ? x[t + 8] : x[t];
        a[t] = keep + __shfl_xor(send, 16);
    }
    hi = lane & 8;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float send = hi ? a[t] : a[t + 4], keep = hi ? a[t + 4] : a[t];
        b4[t] = keep + __shfl_xor(send, 8);
    }
    hi = lane & 4;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const float send = hi ? b4[t] : b4[t + 2], keep = hi ? b4[t + 2] : b4[t];
        c2[t] = keep + __shfl_xor(send, 4);
    }
    hi = lane & 2;
    const float send = hi ? c2[0] : c2[1], keep = hi ? c2[1] : c2[0];
    float d = keep + __shfl_xor(send, 2);
    d += __shfl_xor(d, 1);
    return d;
}

// Log2-sum-exp2 of one query row from the per-chunk (max, sum) pairs that pass 1 left
// (16 independent loads in flight per batch).
__device__ __forceinline__ float fold_chunks(const float2 *src, int stride, int nchunks) {
    float M = -INFINITY, sum = 0.f;
    for (int c0 = 0; c0 < nchunks; c0 += 16) {
        float2 e[16];
#pragma unroll
        for (int t = 0; t < 16; ++t)
            e[t] = c0 + t < nchunks ? src[(int64_t)(c0 + t) * stride] : make_float2(-INFINITY, 0.f);
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const float mn = fmaxf(M, e[t].x);
            const float mref = mn == -INFINITY ? 0.f : mn;
            sum = sum * fast_exp2(M - mref) + e[t].y * fast_exp2(e[t].x - mref);
            M = mn;
        }
    }
    return M + log2f(sum);
}

template <int D, int NB>
__global__ __launch_bounds__(256, 2) void bf16_pass2_kernel(ScoreGeom g, int n_qtiles,
                                                            int wg_keys, int nchunks,
                                                            const float *lam_tab,
                                                            const float2 *partial,
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

    const int z = blockIdx.y;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const RowMap rm{g.n, g.r, g.R};
    const __bf16 *kbase = (const __bf16 *)g.k + b * g.ks[0] + h * g.ks[1];

    if (g.value_prior) {
        float gm = 0.f;
        for (int t = tid; t < n_vtiles; t += 256) gm = fmaxf(gm, gblockmax[z * n_vtiles + t]);
        gm = wave_max(gm);
        if (lane == 0) s_gmax[wave] = gm;
    }
    int loaded_qt = -1;
    float lamr[NB], Lr[NB];  // scale and log-sum-exp of this lane's query column, per block
    const int key_begin = blockIdx.x * wg_keys;
    const int key_end = min(g.n, key_begin + wg_keys);
    for (int kb0 = key_begin; kb0 < key_end; kb0 += kWgKeys) {
        const int kb = kb0 + wave * kWaveKeys;
        bf16x8 a[kMB][D / 16];
        load_a<D>(kbase, g.ks[2], kb, g.n, lane, a);
        f32x16 col[kMB];
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) col[mb][v] = 0.f;

        for (int qt = 0; qt < n_qtiles; ++qt) {
            const int rho0 = qt * S::ROWS;
            if (rm.max_pos(rho0, rho0 + S::ROWS) < kb0) continue;  // workgroup-uniform
            if (qt != loaded_qt) {
                __syncthreads();
                {
                    // tile rows and chunk statistics are requested together, then used
                    QTileRegs<D, NB> qt_regs;
                    q_tile_request<D, NB>(g, b, h, rho0, 0, qt_regs);
                    for (int rr = tid; rr < S::ROWS; rr += 256)
                        sL[rr] = rho0 + rr < g.R
                                     ? fold_chunks(partial + ((int64_t)(z * n_qtiles + qt) * nchunks) * S::ROWS + rr,
                                                   S::ROWS, nchunks)
                                     : INFINITY;
                    q_tile_commit<D, NB>(0, qt_regs, sQ);
#pragma unroll
                    for (int bt = 1; bt < QTileRegs<D, NB>::BATCHES; ++bt) {
                        q_tile_request<D, NB>(g, b, h, rho0, bt, qt_regs);
                        q_tile_commit<D, NB>(bt, qt_regs, sQ);
                    }
                    q_tile_meta<D, NB>(g, rm, rho0, lam_tab, sLam, sPos, sBlk);
                }
                __syncthreads();
                loaded_qt = qt;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    lamr[nb] = sLam[nb * 32 + (lane & 31)];
                    Lr[nb] = sL[nb * 32 + (lane & 31)];
                }
            }
            if (kb >= g.n) continue;  // wave-uniform; the barriers above were reached
            if (kb + kWaveKeys - 1 <= rm.min_pos(rho0, rho0 + S::ROWS)) {
                // all rows of the tile see all 64 keys: pipelined straight-line code
                fast_step_pass2<D, NB>(a, sQ, lamr, Lr, lane, col);
                continue;
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (uniform(sBlk[nb]) < kb) continue;
                f32x16 acc[kMB];
                mma_block<D, NB>(a, sQ, nb, lane, acc);
                const float lam = lamr[nb];
                const float L = Lr[nb];
                const int pos = sPos[nb * 32 + (lane & 31)];
                if (kb + kWaveKeys - 1 > uniform(sBlk[NB + nb]))
                    colsum_update<true>(acc, lam, L, pos, kb, lane, col);
                else
                    colsum_update<false>(acc, lam, L, pos, kb, lane, col);
            }
        }
        float ginv = 1.f;
        if (g.value_prior)  // s_gmax was published by the barrier of the first tile load
            ginv = 1.f / fmaxf(fmaxf(s_gmax[0], s_gmax[1]), fmaxf(s_gmax[2], s_gmax[3]));
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb) {
            const float tot = fold16_over32(col[mb], lane);
            const int v = ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 +
                          ((lane >> 1) & 1);
            const int j = acc_key(kb, mb, v, lane);
            if ((lane & 1) == 0 && j < g.n) {
                float out = tot;
                if (g.value_prior) out = tot * (gamma[(int64_t)z * g.n + j] * ginv);
                scores[(int64_t)z * g.n + j] = out;
            }
        }
    }
}

// ---------------------------------------------------------------- launch --
template <int D, int NB>
static hipError_t launch_t(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                           hipStream_t st, hipEvent_t mid) {
    using S = TileSmem<D, NB>;
    char *w = (char *)ws;
    float2 *partial = (float2 *)(w + pl.off_partial);
    const float *gamma = (const float *)(w + pl.off_gamma);
    const float *gbm = (const float *)(w + pl.off_gblockmax);
    const float *lam_tab = (const float *)(w + pl.off_lam);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)bf16_pass1_kernel<D, NB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)S::bytes);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void *)bf16_pass2_kernel<D, NB>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::bytes);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    dim3 g1(pl.nchunks, pl.n_qtiles, pl.Z);
    hipLaunchKernelGGL((bf16_pass1_kernel<D, NB>), g1, dim3(256), S::bytes, st, g, pl.n_qtiles,
                       pl.chunk_keys, pl.nchunks, lam_tab, partial);
    if (mid) (void)hipEventRecord(mid, st);
    dim3 g2((g.n + pl.p2_keys - 1) / pl.p2_keys, pl.Z);
    hipLaunchKernelGGL((bf16_pass2_kernel<D, NB>), g2, dim3(256), S::bytes, st, g, pl.n_qtiles,
                       pl.p2_keys, pl.nchunks, lam_tab, partial, gamma, gbm, pl.n_vtiles, scores);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                           hipStream_t st, hipEvent_t mid) {
    switch (pl.NB) {
        case 1: return launch_t<D, 1>(g, pl, ws, scores, st, mid);
        case 2: return launch_t<D, 2>(g, pl, ws, scores, st, mid);
        case 4: return launch_t<D, 4>(g, pl, ws, scores, st, mid);
        default: return launch_t<D, 8>(g, pl, ws, scores, st, mid);
    }
}

hipError_t launch_score_bf16(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *scores,
                             hipStream_t st, hipEvent_t mid) {
    return g.d == 64 ? launch_d<64>(g, pl, ws, scores, st, mid)
                     : launch_d<128>(g, pl, ws, scores, st, mid);
}

}  // namespace aha

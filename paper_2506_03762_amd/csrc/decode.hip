// One generation step with running eviction (Alg. 1 Generation, loop body).
//
// One workgroup of 1024 threads per (batch, KV head) streams that head's
// compact K cache once and its V cache once with 16-byte loads (the lanes of
// a row adjacent, 64 rows per sweep), so the step is bound by HBM bandwidth;
// the raw dots of all live slots stay in LDS, from which both the attention
// output (scale 1/sqrt(d)) and the score update (adaptive scale) are formed.
// No cross-workgroup exchange is needed: the whole head lives in one CU.
// With five or more query heads per KV head (bf16) the dots of whole 32-slot
// blocks come from the matrix core instead of per-query vector-ALU dots.
#include "aha_dev.h"
#include "aha_host.h"

namespace aha {

constexpr int kDecThreads = 1024;
constexpr int kDecWaves = kDecThreads / 64;

template <int ESIZE>
__device__ __forceinline__ void unpack(const u32x4 &w, float (&f)[16 / ESIZE]) {
    if constexpr (ESIZE == 2) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            f[2 * t] = bf16_lo(w[t]);
            f[2 * t + 1] = bf16_hi(w[t]);
        }
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) f[t] = __uint_as_float(w[t]);
    }
}

// Dot product of one 16-byte chunk of a key row with the same chunk of a query.  bf16: the
// packed pairs go through v_dot2c_f32_bf16 (exact products, fp32 accumulation) without
// being unpacked; fp32: four fused multiply-adds.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <int ESIZE>
__device__ __forceinline__ float chunk_dot(const u32x4 &kw, const u32x4 &qw) {
    if constexpr (ESIZE == 2) {
        float a = 0.f, b = 0.f;  // two chains
        auto pair = [](uint32_t w) {
            bf16x2 v;
            __builtin_memcpy(&v, &w, 4);
            return v;
        };
#pragma unroll
        for (int t = 0; t < 4; t += 2) {
            a = __builtin_amdgcn_fdot2_f32_bf16(pair(kw[t]), pair(qw[t]), a, false);
            b = __builtin_amdgcn_fdot2_f32_bf16(pair(kw[t + 1]), pair(qw[t + 1]), b, false);
        }
        return a + b;
    } else {
        float w = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) w = fmaf(__uint_as_float(kw[t]), __uint_as_float(qw[t]), w);
        return w;
    }
}

// Smallest (score bits << 32 | ~position) key of the wave, in two 32-bit reductions: the
// smallest score, then the smallest ~position among the lanes that hold it.
__device__ __forceinline__ unsigned long long wave_min_key(unsigned long long key) {
    const uint32_t hi = (uint32_t)(key >> 32), lo = (uint32_t)key;
    const uint32_t whi = reduce_lanes<1, 64>(hi, OpMinU{});
    const uint32_t wlo = reduce_lanes<1, 64>(hi == whi ? lo : 0xffffffffu, OpMinU{});
    return ((unsigned long long)whi << 32) | wlo;
}

template <int ESIZE, int D, int G>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(DecodeGeom g, int w_floats,
                                                             const float *ws_nu,
                                                             const float *ws_numax) {
    constexpr int CH = 16 / ESIZE;       // channels per 16-byte chunk
    constexpr int LPR = D / CH;          // lanes per row
    constexpr int RP = kDecThreads / LPR;  // rows per sweep
    constexpr int ROWB = D * ESIZE;
    constexpr bool kMfmaDots = ESIZE == 2 && G >= kDecodeMfmaGroup;  // dots on the matrix core
    constexpr bool kMfmaValues = ESIZE == 2 && G >= kDecodeMfmaValuesGroup;  // values too

    extern __shared__ __attribute__((aligned(16))) float dsm[];
    // (matrix-core dots: the query tile, 32 padded rows, comes first)
    float *s_w = dsm + (kMfmaDots ? kDecodeQTileBytes(D) / 4 : 0);  // [G][live] raw dots; later [waves][G][D] partial outputs
    float *s_p = s_w + w_floats;   // [G][live] output probabilities
    __shared__ float s_red[kDecWaves][2 * G];
    __shared__ float s_tot[3 * G];  // folded maxima [G], then reciprocal sums [2 G]
    __shared__ unsigned long long s_key[kDecWaves];

    const int z = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int live = g.budget + 1;
    const int fs = g.free_slot[z];
    const int rg = tid / LPR, sub = tid % LPR;
    char *kcz = (char *)g.kc + (int64_t)z * g.slots * ROWB;
    char *vcz = (char *)g.vc + (int64_t)z * g.slots * ROWB;
    float *fcz = g.fc + (int64_t)z * g.slots;
    int32_t *posz = g.pos + (int64_t)z * g.slots;

    // The new token's rows and the queries are requested together with the first cache rows:
    // the row of the free slot is read like any other and replaced afterwards, so no load
    // waits for the free-slot index.
    const u32x4 knw = *(const u32x4 *)((const char *)g.k_new + (int64_t)z * ROWB + sub * 16);
    const u32x4 vnw = *(const u32x4 *)((const char *)g.v_new + (int64_t)z * ROWB + sub * 16);
    u32x4 qw[G];  // (unused where the dots go through the matrix core)
    if constexpr (!kMfmaDots) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi)
            qw[gi] = *(const u32x4 *)((const char *)g.q + ((int64_t)(b * g.Hq + h * G + gi)) * ROWB + sub * 16);
    }

    // value prior inside the loop (an option): the slots' norms and their maximum come from
    // a launch of their own (decode_value_norms_kernel)
    const float ginv = g.value_prior ? prior_inverse(ws_numax[z]) : 1.f;
    // the running score and position of this thread's first slot (the later phase that updates
    // them would otherwise wait a full round trip to memory in the middle of the kernel)
    const float f_first = fcz[min(tid, live - 1)];
    const int p_first = posz[min(tid, live - 1)];
    const float f_second = fcz[min(tid + kDecThreads, live - 1)];
    const int p_second = posz[min(tid + kDecThreads, live - 1)];

    // ---- raw dots over the live slots (the new key stands in for slot fs) ----
    float mloc[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) mloc[gi] = -INFINITY;
    // dots of the 16-byte chunk `kw` of slot s with the queries' chunks `qw`, summed over the
    // lanes of the row
    auto dots = [&](int s, u32x4 kw, const u32x4 (&qc)[G]) {
        if (s == fs) {
            kw = knw;
            *(u32x4 *)(kcz + (int64_t)s * ROWB + sub * 16) = kw;
        }
        // (all heads' dots and lane reductions first, one guarded block of stores after them:
        // a store per head in between would fence the independent reduction chains apart,
        // and each chain alone waits out the data hazards between its lane exchanges)
        float w[G];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) w[gi] = chunk_dot<ESIZE>(kw, qc[gi]);
#pragma unroll
        for (int gi = 0; gi < G; ++gi) w[gi] = reduce_lanes<1, LPR>(w[gi], OpSum{});  // over the lanes of the row
        if (sub == 0) {
#pragma unroll
            for (int gi = 0; gi < G; ++gi) s_w[gi * live + s] = w[gi];
        }
#pragma unroll
        for (int gi = 0; gi < G; ++gi) mloc[gi] = fmaxf(mloc[gi], w[gi]);
    };
    if constexpr (!kMfmaDots) {
        // cache rows per thread requested before the first is used
        constexpr int PF = G <= 2 ? 8 : 4;
        u32x4 kpf[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u)
            kpf[u] = *(const u32x4 *)(kcz + (int64_t)min(rg + u * RP, live - 1) * ROWB + sub * 16);
#pragma unroll
        for (int u = 0; u < PF; ++u)
            if (rg + u * RP < live) dots(rg + u * RP, kpf[u], qw);
        // the rest in batches of PF rows per thread, requested together (written out by hand:
        // a loop with lane exchanges in its body is not unrolled by the compiler).  (A rolling
        // window - every used row's registers given at once to the row PF sweeps further on -
        // measured 10 % slower than whole batches.)
        for (int sb = rg + PF * RP; sb < live; sb += PF * RP) {
#pragma unroll
            for (int u = 0; u < PF; ++u)
                kpf[u] = *(const u32x4 *)(kcz + (int64_t)min(sb + u * RP, live - 1) * ROWB + sub * 16);
#pragma unroll
            for (int u = 0; u < PF; ++u)
                if (sb + u * RP < live) dots(sb + u * RP, kpf[u], qw);
        }
    } else {
        // Wide groups (bf16): with G queries per key row the dots are a small matrix product,
        // S^T = K Q^T, and per-query vector-ALU dots with their lane reductions cost more than
        // the key stream (and, with the value phase's G x 8 accumulators, more registers than
        // a thread of this workgroup has).  Blocks of 32 slots go through
        // v_mfma_f32_32x32x16_bf16 - slots on M, the G queries on N (columns >= G are zero) -
        // with the key fragments loaded straight into registers, a lane holding one half of a
        // row, and the queries read from a tile in LDS.  Whole blocks are dealt to the waves
        // round-robin; the slots past the last whole block and the free slot (whose cache row
        // is stale: the new key stands in for it) are done by 16-lane groups on the vector ALU
        // afterwards.
        constexpr int QLD = D + 8;  // padded row of the query tile: conflict-free b128 reads
        __bf16 *sQ = (__bf16 *)dsm;
        for (int i = tid; i < 32 * LPR; i += kDecThreads) {
            const int n = i / LPR, c = i % LPR;
            u32x4 w = {0u, 0u, 0u, 0u};
            if (n < G)
                w = *(const u32x4 *)((const char *)g.q + ((int64_t)(b * g.Hq + h * G + n)) * ROWB + c * 16);
            *(u32x4 *)(sQ + n * QLD + c * 8) = w;
        }
        // the leftover slots: group rg of 16 lanes takes slot nblk * 32 + rg, the group behind
        // them the free slot (unless it is one of the leftover slots); requested now, used last
        const int nblk = live / 32, ntail = live - nblk * 32;
        const int vrow = rg < ntail ? nblk * 32 + rg : (rg == ntail && fs < nblk * 32 ? fs : -1);
        u32x4 kv_row = {0u, 0u, 0u, 0u};
        if (vrow >= 0) kv_row = *(const u32x4 *)(kcz + (int64_t)vrow * ROWB + sub * 16);
        auto load_block = [&](int blk, bf16x8 (&dst)[D / 16]) {
            const int row = min(max(min(blk, nblk - 1), 0) * 32 + (lane & 31), live - 1);  // (any blk, any nblk)
            const char *pr = kcz + (int64_t)row * ROWB + (lane >> 5) * 16;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) dst[ks] = *(const bf16x8 *)(pr + ks * 32);
        };
        auto block_dots = [&](int blk, const bf16x8 (&a)[D / 16]) {
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const __bf16 *bp = sQ + (lane & 31) * QLD + (lane >> 5) * 8;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], *(const bf16x8 *)(bp + ks * 16), acc, 0, 0, 0);
            // lane: query column lane % 32, slots 8 * (v / 4) + 4 * (lane / 32) + v % 4 of the block
            if ((lane & 31) < G) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    s_w[(lane & 31) * live + blk * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)] = acc[v];
            }
        };
        // (The loads are issued unconditionally, clamped to the last whole block: behind a
        // branch the compiler would wait for a prefetch before the block in hand.)
        bf16x8 a0[D / 16], a1[D / 16];
        if (nblk <= 2 * kDecWaves) {
            // at most two blocks per wave (budgets up to 1024): both travel while the query
            // tile is set up, and nothing is requested that is not used
            load_block(wave, a0);
            load_block(wave + kDecWaves, a1);
            __syncthreads();  // the query tile is in LDS
            if (wave < nblk) block_dots(wave, a0);
            if (wave + kDecWaves < nblk) block_dots(wave + kDecWaves, a1);
        } else {
            load_block(wave, a0);
            __syncthreads();  // the query tile is in LDS
            for (int blk = wave; blk < nblk; blk += 2 * kDecWaves) {
                load_block(blk + kDecWaves, a1);
                block_dots(blk, a0);
                if (blk + kDecWaves >= nblk) break;
                load_block(blk + 2 * kDecWaves, a0);
                block_dots(blk + kDecWaves, a1);
            }
        }
        __syncthreads();  // the blocks' dots are written (the free slot's among them: stale)
        // (the lane reductions inside `dots` stay inside a row's group of lanes, which is
        // active or idle as a whole)
        if (vrow >= 0) {
            u32x4 qc[G];
#pragma unroll
            for (int gi = 0; gi < G; ++gi) qc[gi] = *(const u32x4 *)(sQ + gi * QLD + sub * 8);
            dots(vrow, kv_row, qc);
        }
        __syncthreads();
        // the maxima of the rows' dots, from LDS (the matrix blocks left none in registers)
        for (int s = tid; s < live; s += kDecThreads) {
#pragma unroll
            for (int gi = 0; gi < G; ++gi) mloc[gi] = fmaxf(mloc[gi], s_w[gi * live + s]);
        }
    }
    // the first value rows travel while the softmax statistics are formed (requesting more
    // of them here, or already behind the last batch of key rows, measured 6 % slower: the
    // key and value streams of the 256 workgroups then mix in memory)
    constexpr int VPF = kMfmaValues ? 1 : G <= 2 ? 8 : 4;
    u32x4 vpf[VPF];
    // (wide groups: the values go through the matrix core too, in blocks of 16 slots per wave:
    // block b of wave w is slots 16 (w + 16 b) ..; a lane holds the 16-byte chunk lane % LPR
    // of rows lane / LPR + t * (64 / LPR) of a block)
    constexpr int VB = 16, VRPI = 64 / LPR, VNI = VB / VRPI;
    u32x4 vblk[kMfmaValues ? VNI : 1];
    auto request_block = [&](int blk) {
#pragma unroll
        for (int t = 0; t < VNI; ++t)
            vblk[kMfmaValues ? t : 0] =
                *(const u32x4 *)(vcz + (int64_t)min(blk * VB + t * VRPI + lane / LPR, live - 1) * ROWB + sub * 16);
    };
    if constexpr (kMfmaValues) {
        request_block(wave);
    } else {
#pragma unroll
        for (int u = 0; u < VPF; ++u)
            vpf[u] = *(const u32x4 *)(vcz + (int64_t)min(rg + u * RP, live - 1) * ROWB + sub * 16);
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        const float m = wave_max(mloc[gi]);
        if (lane == 0) s_red[wave][gi] = m;
    }
    __syncthreads();
    // the waves' statistics are folded by one thread per value and published (every thread
    // folding for itself costs 48 LDS reads per head and thread: C4 decode 28.7 -> 28.4 us)
    float mx[G];
    if (tid < G) {
        float m = s_red[0][tid];
#pragma unroll
        for (int w = 1; w < kDecWaves; ++w) m = fmaxf(m, s_red[w][tid]);
        s_tot[tid] = m;
    }
    __syncthreads();
#pragma unroll
    for (int gi = 0; gi < G; ++gi) mx[gi] = s_tot[gi];
    // (no barrier: s_red and s_tot are next written behind the barrier that follows the sums)

    // ---- the two softmax denominators ----
    const float c_out = kLog2e * rsqrtf((float)D);
    const float c_sc = ESIZE == 2 ? row_scale_log2_f32(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                       g.logical_pos, g.budget, D)
                                  : row_scale_log2(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                   g.logical_pos, g.budget, D);
    float zo[G], zs[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) zo[gi] = zs[gi] = 0.f;
    for (int s = tid; s < live; s += kDecThreads) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const float d = s_w[gi * live + s] - mx[gi];
            zo[gi] += fast_exp2(d * c_out);
            zs[gi] += fast_exp2(d * c_sc);
        }
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        const float a = wave_sum(zo[gi]), c = wave_sum(zs[gi]);
        if (lane == 0) { s_red[wave][2 * gi] = a; s_red[wave][2 * gi + 1] = c; }
    }
    __syncthreads();
    if (tid < 2 * G) {
        float a = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) a += s_red[w][tid];
        s_tot[G + tid] = 1.f / a;  // (reciprocals: one division per head instead of two per slot)
    }
    __syncthreads();
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        zo[gi] = s_tot[G + 2 * gi];
        zs[gi] = s_tot[G + 2 * gi + 1];
    }

    // ---- probabilities, running score, eviction candidate ----
    unsigned long long best = ~0ull;
    int best_slot = -1;
    for (int s = tid; s < live; s += kDecThreads) {
        float add = 0.f;
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const float d = s_w[gi * live + s] - mx[gi];
            s_p[gi * live + s] = fast_exp2(d * c_out) * zo[gi];
            add += fast_exp2(d * c_sc) * zs[gi];
        }
        if (g.value_prior) add *= prior_factor(ws_nu[(int64_t)z * live + s], ginv);
        const float f = (s == fs ? 0.f : s == tid ? f_first : s == tid + kDecThreads ? f_second : fcz[s]) + add;
        fcz[s] = f;
        int ps;
        if (s == fs) { ps = g.logical_pos - 1; posz[s] = ps; } else { ps = s == tid ? p_first : s == tid + kDecThreads ? p_second : posz[s]; }
        if (ps < g.logical_pos - g.recent && ps >= g.sink) {
            const unsigned long long key =
                ((unsigned long long)__float_as_uint(f) << 32) | (uint32_t)(~ps);
            if (key < best) { best = key; best_slot = s; }
        }
    }
    const unsigned long long wbest = wave_min_key(best);  // every lane takes part
    if (lane == 0) s_key[wave] = wbest;
    __syncthreads();  // also: s_w is free from here on
    // (the waves' candidates are compared at the very end, off the path to the values)

    // ---- attention output: sum_s p_s V_s ----
    float *s_o = s_w;  // [waves][G][D]
    if constexpr (kMfmaValues) {
        // O^T += V^T P^T on the matrix core, 16 slots at a time: A = V^T (channels on M, a
        // lane gathers its channel of eight slots from the wave's copy of the block's rows in
        // LDS), B = the probabilities of those slots (query heads on N, columns >= G zero).
        // The wave's copy lies over the query tile (if any) and the dots, which are done with.
        constexpr int LDVS = D + 8, CB = D / 32;
        __bf16 *sVw = (__bf16 *)dsm + wave * VB * LDVS;
        f32x16 O[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) O[cb][v] = 0.f;
        const int nvb = (live + VB - 1) / VB, qn = lane & 31, hf = lane >> 5;
        for (int blk = wave; blk < nvb; blk += kDecWaves) {
            // this block's rows -> LDS (the new value row stands in for the free slot's and
            // goes to the cache), the next block's are requested (clamped: never past the last)
#pragma unroll
            for (int t = 0; t < VNI; ++t) {
                const int rin = t * VRPI + lane / LPR;
                u32x4 w = vblk[t];
                if (blk * VB + rin == fs) {
                    w = vnw;
                    *(u32x4 *)(vcz + (int64_t)fs * ROWB + sub * 16) = w;
                }
                *(u32x4 *)(sVw + rin * LDVS + sub * 8) = w;
            }
            request_block(min(blk + kDecWaves, nvb - 1));
            // probabilities of slots 8 hf .. 8 hf + 7 of the block for query head qn
            bf16x8 pfrag;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int sl = blk * VB + 8 * hf + e;
                pfrag[e] = (__bf16)((qn < G && sl < live) ? s_p[min(qn, G - 1) * live + min(sl, live - 1)] : 0.f);
            }
            // V^T fragments (slots 8 hf .. 8 hf + 7 of the block) by transposing LDS reads
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const bf16x8 vfrag = lds_transposed_fragment(sVw, LDVS, 4 * hf, 4, cb * 32, lane);
                O[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfrag, pfrag, O[cb], 0, 0, 0);
            }
        }
        __syncthreads();  // every wave is done with its rows: the partial outputs go on top
        if (qn < G) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    s_o[(wave * G + qn) * D + cb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3)] = O[cb][v];
        }
    } else {
    float o[G][CH];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int c = 0; c < CH; ++c) o[gi][c] = 0.f;
    auto weigh = [&](int s, u32x4 vw) {
        if (s == fs) {
            vw = vnw;
            *(u32x4 *)(vcz + (int64_t)s * ROWB + sub * 16) = vw;
        }
        float vf[CH];
        unpack<ESIZE>(vw, vf);
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const float p = s_p[gi * live + s];
#pragma unroll
            for (int c = 0; c < CH; ++c) o[gi][c] = fmaf(p, vf[c], o[gi][c]);
        }
    };
#pragma unroll
    for (int u = 0; u < VPF; ++u)
        if (rg + u * RP < live) weigh(rg + u * RP, vpf[u]);
#pragma unroll 8
    for (int s = rg + VPF * RP; s < live; s += RP)
        weigh(s, *(const u32x4 *)(vcz + (int64_t)s * ROWB + sub * 16));
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float v = o[gi][c];
            v = reduce_lanes<LPR, 64>(v, OpSum{});  // over the rows of the wave
            if (lane < LPR) s_o[(wave * G + gi) * D + sub * CH + c] = v;
        }
    }
    __syncthreads();
    for (int t = tid; t < G * D; t += kDecThreads) {
        const int gi = t / D, c = t % D;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) v += s_o[(w * G + gi) * D + c];
        const int64_t oi = ((int64_t)(b * g.Hq + h * G + gi)) * D + c;
        if constexpr (ESIZE == 2)
            ((uint16_t *)g.out)[oi] = (uint16_t)f32_to_bf16_rne(v);
        else
            ((float *)g.out)[oi] = v;
    }
    // positions are unique, so exactly one thread holds the victim: it retires the slot (only
    // the waves' own candidates look at the other waves' keys)
    if (best_slot >= 0 && best == wbest) {
        unsigned long long gbest = s_key[0];
#pragma unroll
        for (int w = 1; w < kDecWaves; ++w) gbest = s_key[w] < gbest ? s_key[w] : gbest;
        if (best == gbest) {
            posz[best_slot] = -1;
            g.free_slot[z] = best_slot;
        }
    }
}

// Value prior inside the generation loop (an option; Sec. 4.3 applied to the compact cache):
// nu_s = ||v_cache[s]||^2 of every live slot - the new token's row standing in for the free
// slot - and the largest of them, one workgroup per (batch, KV head).  A launch of its own, so
// that the decode kernels proper carry nothing of it.
template <int ESIZE, int D>
__global__ __launch_bounds__(256) void decode_value_norms_kernel(DecodeGeom g, float *ws_nu,
                                                                 float *ws_numax) {
    constexpr int CH = 16 / ESIZE, LPR = D / CH, RP = 256 / LPR, ROWB = D * ESIZE;
    __shared__ float s_max[4];
    const int z = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int live = g.budget + 1, fs = g.free_slot[z];
    const int rg = tid / LPR, sub = tid % LPR;
    const char *vcz = (const char *)g.vc + (int64_t)z * g.slots * ROWB;
    const u32x4 vnw = *(const u32x4 *)((const char *)g.v_new + (int64_t)z * ROWB + sub * 16);
    float numax = 0.f;
    for (int s = rg; s < live; s += RP) {
        const u32x4 vw = s == fs ? vnw : *(const u32x4 *)(vcz + (int64_t)s * ROWB + sub * 16);
        float vf[CH];
        unpack<ESIZE>(vw, vf);
        float nu = 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) nu = fmaf(vf[c], vf[c], nu);
        nu = reduce_lanes<1, LPR>(nu, OpSum{});  // over the lanes of the row
        if (sub == 0) ws_nu[(int64_t)z * live + s] = nu;
        numax = fmaxf(numax, nu);
    }
    numax = wave_max(numax);
    if (lane == 0) s_max[wave] = numax;
    __syncthreads();
    if (tid == 0) ws_numax[z] = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
}

// ---- few problems: split the slots of a head over several workgroups ----
// Stage 1, one workgroup per (slot range, batch, KV head): raw dots to the
// workspace, and the range's share of the attention output relative to the
// range's own maximum (flash-decoding style partials).
template <int ESIZE, int D, int G>
__global__ __launch_bounds__(256) void decode_split_kernel(DecodeGeom g, int nsplit, int sps,
                                                           float *ws_w, float *ws_part) {
    constexpr int CH = 16 / ESIZE, LPR = D / CH, RP = 256 / LPR, ROWB = D * ESIZE;
    constexpr int PF = 6;  // sweeps of the range whose K and V rows are requested at the start
    extern __shared__ __attribute__((aligned(16))) float dsm[];
    float *s_p = dsm;                 // [G][sps] dots, then unnormalised probabilities
    float *s_o = dsm + G * sps;       // [4 waves][G][D]
    __shared__ float s_red[4][G];

    const int split = blockIdx.x, z = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int live = g.budget + 1;
    const int s0 = split * sps, s1 = min(live, s0 + sps);
    const int rg = tid / LPR, sub = tid % LPR;
    char *kcz = (char *)g.kc + (int64_t)z * g.slots * ROWB;
    char *vcz = (char *)g.vc + (int64_t)z * g.slots * ROWB;

    // With so few workgroups the step is bound by memory latency, not bandwidth: everything
    // the first PF sweeps need is requested before anything is used - the free slot, the
    // queries, the new token's rows, the cached K and V rows (the row of the free slot is
    // read like any other and replaced afterwards) - so that the kernel waits for memory
    // once instead of once per dependent step.
    const int fs = g.free_slot[z];
    u32x4 qw[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
        qw[gi] = *(const u32x4 *)((const char *)g.q + ((int64_t)(b * g.Hq + h * G + gi)) * ROWB + sub * 16);
    const u32x4 knw = *(const u32x4 *)((const char *)g.k_new + (int64_t)z * ROWB + sub * 16);
    const u32x4 vnw = *(const u32x4 *)((const char *)g.v_new + (int64_t)z * ROWB + sub * 16);
    u32x4 kpf[PF], vpf[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) {
        const int sc = min(s0 + rg + u * RP, s1 - 1);  // past the range: a row that is there
        kpf[u] = *(const u32x4 *)(kcz + (int64_t)sc * ROWB + sub * 16);
        vpf[u] = *(const u32x4 *)(vcz + (int64_t)sc * ROWB + sub * 16);
    }
    float mloc[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) mloc[gi] = -INFINITY;
    auto dots = [&](int s, u32x4 kw) {
        if (s == fs) {
            kw = knw;
            *(u32x4 *)(kcz + (int64_t)s * ROWB + sub * 16) = kw;
        }
        // (dots and lane reductions of all heads first, then one guarded block of stores: the
        // independent reduction chains interleave instead of waiting out their hazards)
        float w[G];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) w[gi] = chunk_dot<ESIZE>(kw, qw[gi]);
#pragma unroll
        for (int gi = 0; gi < G; ++gi) w[gi] = reduce_lanes<1, LPR>(w[gi], OpSum{});  // over the lanes of the row
        if (sub == 0) {
#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                s_p[gi * sps + s - s0] = w[gi];
                ws_w[((int64_t)z * live + s) * G + gi] = w[gi];  // [head][slot][query]: a slot's dots together
            }
        }
#pragma unroll
        for (int gi = 0; gi < G; ++gi) mloc[gi] = fmaxf(mloc[gi], w[gi]);
    };
#pragma unroll
    for (int u = 0; u < PF; ++u) {
        const int s = s0 + rg + u * RP;
        if (s < s1) dots(s, kpf[u]);
    }
    // (the rest in batches written out by hand: a loop with lane exchanges in its body is
    // not unrolled by the compiler)
    for (int sb = s0 + rg + PF * RP; sb < s1; sb += PF * RP) {
#pragma unroll
        for (int u = 0; u < PF; ++u)
            kpf[u] = *(const u32x4 *)(kcz + (int64_t)min(sb + u * RP, s1 - 1) * ROWB + sub * 16);
#pragma unroll
        for (int u = 0; u < PF; ++u)
            if (sb + u * RP < s1) dots(sb + u * RP, kpf[u]);
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        const float m = wave_max(mloc[gi]);
        if (lane == 0) s_red[wave][gi] = m;
    }
    __syncthreads();
    float mx[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
        mx[gi] = fmaxf(fmaxf(s_red[0][gi], s_red[1][gi]), fmaxf(s_red[2][gi], s_red[3][gi]));
    __syncthreads();
    const float c_out = kLog2e * rsqrtf((float)D);
    float zo[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) zo[gi] = 0.f;
    for (int s = s0 + tid; s < s1; s += 256) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const float e = fast_exp2((s_p[gi * sps + s - s0] - mx[gi]) * c_out);
            s_p[gi * sps + s - s0] = e;
            zo[gi] += e;
        }
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        const float a = wave_sum(zo[gi]);
        if (lane == 0) s_red[wave][gi] = a;
    }
    __syncthreads();
    float o[G][CH];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int c = 0; c < CH; ++c) o[gi][c] = 0.f;
    auto weigh = [&](int s, u32x4 vw) {
        if (s == fs) {
            vw = vnw;
            *(u32x4 *)(vcz + (int64_t)s * ROWB + sub * 16) = vw;
        }
        float vf[CH];
        unpack<ESIZE>(vw, vf);
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const float p = s_p[gi * sps + s - s0];
#pragma unroll
            for (int c = 0; c < CH; ++c) o[gi][c] = fmaf(p, vf[c], o[gi][c]);
        }
    };
#pragma unroll
    for (int u = 0; u < PF; ++u) {
        const int s = s0 + rg + u * RP;
        if (s < s1) weigh(s, vpf[u]);
    }
#pragma unroll 4
    for (int s = s0 + rg + PF * RP; s < s1; s += RP)
        weigh(s, *(const u32x4 *)(vcz + (int64_t)s * ROWB + sub * 16));
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float v = o[gi][c];
            v = reduce_lanes<LPR, 64>(v, OpSum{});  // over the rows of the wave
            if (lane < LPR) s_o[(wave * G + gi) * D + sub * CH + c] = v;
        }
    __syncthreads();
    float *part = ws_part + ((int64_t)z * nsplit + split) * G * (D + 2);
    for (int t = tid; t < G * D; t += 256) {
        const int gi = t / D, c = t % D;
        part[gi * (D + 2) + c] = s_o[(0 * G + gi) * D + c] + s_o[(1 * G + gi) * D + c] +
                                 s_o[(2 * G + gi) * D + c] + s_o[(3 * G + gi) * D + c];
    }
    if (tid < G) {
        part[tid * (D + 2) + D] = mx[tid];
        part[tid * (D + 2) + D + 1] = s_red[0][tid] + s_red[1][tid] + s_red[2][tid] + s_red[3][tid];
    }
}

// Stage 2, two workgroups per (batch, KV head) that share nothing but their inputs: one
// merges the partial outputs, the other updates the running scores from the stored dots
// and picks the victim (side by side they take the time of the longer one).
constexpr int kMergeThreads = 1024;

template <int ESIZE, int D, int G>
__global__ __launch_bounds__(kMergeThreads) void decode_merge_kernel(DecodeGeom g, int nsplit,
                                                           const float *ws_w,
                                                           const float *ws_part,
                                                           const float *ws_nu,
                                                           const float *ws_numax) {
    static_assert(G * D <= kMergeThreads, "one output element per thread");
    static_assert(kMaxDecodeSplit * G <= kMergeThreads, "one (split, head) statistic per thread");
    __shared__ float s_pm[kMaxDecodeSplit][G], s_pz[kMaxDecodeSplit][G];
    __shared__ float s_red[kMergeThreads / 64][G];
    __shared__ unsigned long long s_key[kMergeThreads / 64];
    const int z = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = z / g.Hkv, h = z % g.Hkv;
    const int live = g.budget + 1;
    float *fcz = g.fc + (int64_t)z * g.slots;
    int32_t *posz = g.pos + (int64_t)z * g.slots;
    const float *part = ws_part + (int64_t)z * nsplit * G * (D + 2);
    const float c_out = kLog2e * rsqrtf((float)D);
    const float c_sc = ESIZE == 2 ? row_scale_log2_f32(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                       g.logical_pos, g.budget, D)
                                  : row_scale_log2(g.scale_mode, g.fixed_scale, g.lambda_floor,
                                                   g.logical_pos, g.budget, D);
    // slots per thread and batch fetched together (fewer for wide groups: G dots per slot)
    // slots per thread and batch (score role); splits whose outputs are requested up front
    // (output role: fewer for wide groups, where every split's address takes registers)
    constexpr int NT = kMergeThreads, U = 4, XB = G <= 4 ? 32 : 16;

    // Latency-bound like stage 1: every first-use load is requested here, before any result
    // is needed - the free slot, the splits' statistics, the first batch of stored dots with
    // their scores and positions (the free slot's stale entries are read like any other and
    // replaced afterwards), and this thread's output element of the first XB splits.
    const int fs = g.free_slot[z];
    float my_pm = -INFINITY, my_pz = 0.f;
    if (tid < nsplit * G) {
        my_pm = part[tid * (D + 2) + D];  // tid = split * G + head
        my_pz = part[tid * (D + 2) + D + 1];
    }
    // The score role goes through the query heads in groups of at most four (a slot's dots
    // lie together in the workspace: one 16-byte load per slot and whole group): with more
    // heads at once the per-head copies of four slots do not fit a thread of this workgroup.
    constexpr int GH = G < 4 ? G : 4, NG = (G + GH - 1) / GH;
    float wr[U][GH], fr[U], nur[U];
    int pr[U];
    // dots of head group `grp` (heads grp * GH ..; past G: -inf) of this thread's U slots
    auto fetch_dots = [&](int base, int grp) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = base + tid + u * NT;
            const bool ok = s < live;
            // (live * G floats of a head start 16-byte aligned when G is a multiple of four:
            // the workspace is 256-byte aligned)
            const float *wp = ws_w + ((int64_t)z * live + (ok ? s : 0)) * G + grp * GH;
            if constexpr (G % 4 == 0) {
                const f32x4 w4 = *(const f32x4 *)wp;
#pragma unroll
                for (int c = 0; c < 4; ++c) wr[u][c] = ok ? w4[c] : -INFINITY;
            } else {
#pragma unroll
                for (int c = 0; c < GH; ++c)
                    wr[u][c] = ok && grp * GH + c < G ? wp[grp * GH + c < G ? c : 0] : -INFINITY;
            }
        }
    };
    auto fetch = [&](int base) {  // the first group's dots, the scores, positions, value norms
        fetch_dots(base, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = base + tid + u * NT;
            const bool ok = s < live;
            fr[u] = ok ? fcz[s] : 0.f;
            pr[u] = ok ? posz[s] : 0x7fffffff;
            nur[u] = (ok && g.value_prior) ? ws_nu[(int64_t)z * live + s] : 0.f;
        }
    };
    auto patch_free_slot = [&](int base) {  // the new token: score 0, position logical_pos - 1
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + tid + u * NT == fs) {
                fr[u] = 0.f;
                pr[u] = g.logical_pos - 1;
            }
    };
    // The splits' statistics go to LDS and every wave folds the maxima by itself (one split
    // per lane).  (Written out in both roles, so that neither role's registers stay live
    // through the other's code: together they do not fit a thread of this workgroup.)
    auto fold_maxima = [&](float (&mx)[G]) {
        if (tid < nsplit * G) {
            s_pm[tid / G][tid % G] = my_pm;
            s_pz[tid / G][tid % G] = my_pz;
        }
        __syncthreads();
#pragma unroll
        for (int gi = 0; gi < G; ++gi) mx[gi] = wave_max(lane < nsplit ? s_pm[lane][gi] : -INFINITY);
    };
    if (blockIdx.y == 0) {  // (workgroup-uniform) the attention output
        const int ogi = tid / D, oc = tid % D;  // this thread's output element (tid < G * D)
        float x[XB];
#pragma unroll
        for (int u = 0; u < XB; ++u)
            x[u] = (tid < G * D && u < nsplit) ? part[(u * G + ogi) * (D + 2) + oc] : 0.f;
        float mx[G];
        fold_maxima(mx);
        if (tid >= G * D) return;
        float mxo = mx[0];  // this thread's head
#pragma unroll
        for (int gi = 1; gi < G; ++gi) mxo = ogi == gi ? mx[gi] : mxo;
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int u = 0; u < XB; ++u)
            if (u < nsplit) {
                const float sc = fast_exp2((s_pm[u][ogi] - mxo) * c_out);
                num = fmaf(x[u], sc, num);
                den = fmaf(s_pz[u][ogi], sc, den);
            }
#pragma unroll 8
        for (int sp = XB; sp < nsplit; ++sp) {
            const float sc = fast_exp2((s_pm[sp][ogi] - mxo) * c_out);
            num = fmaf(part[(sp * G + ogi) * (D + 2) + oc], sc, num);
            den = fmaf(s_pz[sp][ogi], sc, den);
        }
        const float v = num / den;
        const int64_t oi = ((int64_t)(b * g.Hq + h * G + ogi)) * D + oc;
        if constexpr (ESIZE == 2)
            ((uint16_t *)g.out)[oi] = (uint16_t)f32_to_bf16_rne(v);
        else
            ((float *)g.out)[oi] = v;
        return;
    }
    fetch(0);
    float mx[G];
    fold_maxima(mx);
    // score softmax over all live slots, from the stored raw dots; four slots per thread
    // and batch are fetched together so that the loads overlap
    float zs[G];
#pragma unroll
    for (int gi = 0; gi < G; ++gi) zs[gi] = 0.f;
    // one batch and one head group: the values stay in registers for pass two
    const bool keep = live <= U * NT && NG == 1;
    for (int base = 0; base < live; base += U * NT) {
        if (base) fetch(base);
#pragma unroll
        for (int grp = 0; grp < NG; ++grp) {
            if (grp) fetch_dots(base, grp);
            // (entries past the last slot are skipped, not fed as -inf: a scale of exactly 0
            // would turn them into 0 * inf)
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + tid + u * NT < live)
#pragma unroll
                    for (int c = 0; c < GH; ++c)
                        if (grp * GH + c < G)
                            zs[grp * GH + c] += fast_exp2((wr[u][c] - mx[grp * GH + c]) * c_sc);
        }
    }
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        const float a = wave_sum(zs[gi]);
        if (lane == 0) s_red[wave][gi] = a;
    }
    __syncthreads();
#pragma unroll
    for (int gi = 0; gi < G; ++gi) {
        float a = 0.f;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) a += s_red[w][gi];
        zs[gi] = 1.f / a;
    }
    const float ginv = g.value_prior ? prior_inverse(ws_numax[z]) : 1.f;
    unsigned long long best = ~0ull;
    int best_slot = -1;
    for (int base = 0; base < live; base += U * NT) {
        if (!keep) fetch(base);
        patch_free_slot(base);
        float add[U];
#pragma unroll
        for (int u = 0; u < U; ++u) add[u] = 0.f;
#pragma unroll
        for (int grp = 0; grp < NG; ++grp) {
            if (grp) fetch_dots(base, grp);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < GH; ++c)
                    if (grp * GH + c < G)
                        add[u] += fast_exp2((wr[u][c] - mx[grp * GH + c]) * c_sc) * zs[grp * GH + c];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = base + tid + u * NT;
            if (s >= live) continue;
            if (g.value_prior) add[u] *= prior_factor(nur[u], ginv);
            const float f = fr[u] + add[u];
            fcz[s] = f;
            const int ps = pr[u];
            if (s == fs) posz[s] = ps;
            if (ps < g.logical_pos - g.recent && ps >= g.sink) {
                const unsigned long long key =
                    ((unsigned long long)__float_as_uint(f) << 32) | (uint32_t)(~ps);
                if (key < best) { best = key; best_slot = s; }
            }
        }
    }
    const unsigned long long wbest = wave_min_key(best);  // every lane takes part
    if (lane == 0) s_key[wave] = wbest;
    __syncthreads();
    unsigned long long gbest = s_key[0];
#pragma unroll
    for (int w = 1; w < kMergeThreads / 64; ++w) gbest = s_key[w] < gbest ? s_key[w] : gbest;
    // positions are unique, so exactly one thread holds the victim: it retires the slot
    if (best_slot >= 0 && best == gbest) {
        posz[best_slot] = -1;
        g.free_slot[z] = best_slot;
    }
}

template <int ESIZE, int D>
static hipError_t launch_g(const DecodeGeom &g, const DecodePlan &pl, void *ws, hipStream_t st) {
    const int live = g.budget + 1;
    float *ws_nu = (float *)((char *)ws + pl.off_nu);
    float *ws_numax = ws_nu + (size_t)g.batch * g.Hkv * live;
    if (g.value_prior) {
        hipLaunchKernelGGL((decode_value_norms_kernel<ESIZE, D>), dim3(g.batch * g.Hkv), dim3(256),
                           0, st, g, ws_nu, ws_numax);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    if (pl.nsplit > 1) {
        float *ws_w = (float *)ws;
        float *ws_part = (float *)((char *)ws + pl.off_part);
        const size_t smem1 = (size_t)(g.G * pl.sps + 4 * g.G * D) * sizeof(float);
        dim3 g1(pl.nsplit, g.batch * g.Hkv), g2(g.batch * g.Hkv, 2);
#define AHA_DECS(GG)                                                                             \
    {                                                                                            \
        hipLaunchKernelGGL((decode_split_kernel<ESIZE, D, GG>), g1, dim3(256), smem1, st, g,     \
                           pl.nsplit, pl.sps, ws_w, ws_part);                                    \
        /* the merge rewrites the cache state: never after a refused first launch */             \
        const hipError_t e1 = hipGetLastError();                                                 \
        if (e1 != hipSuccess) return e1;                                                         \
        hipLaunchKernelGGL((decode_merge_kernel<ESIZE, D, GG>), g2, dim3(kMergeThreads), 0, st, g,         \
                           pl.nsplit, ws_w, ws_part, ws_nu, ws_numax);                           \
    }
        switch (g.G) {
            case 1: AHA_DECS(1) break;
            case 2: AHA_DECS(2) break;
            case 3: AHA_DECS(3) break;
            case 4: AHA_DECS(4) break;
            case 5: AHA_DECS(5) break;
            case 6: AHA_DECS(6) break;
            case 7: AHA_DECS(7) break;
            default: AHA_DECS(8) break;
        }
#undef AHA_DECS
        return hipGetLastError();
    }
    const bool mfma = ESIZE == 2 && g.G >= kDecodeMfmaGroup;
    const bool mfma_v = ESIZE == 2 && g.G >= kDecodeMfmaValuesGroup;
    const int w_floats = (int)decode_w_floats(g.G, live, D, mfma, mfma_v);
    const size_t smem = (size_t)(w_floats + g.G * live) * sizeof(float) +
                        (mfma ? kDecodeQTileBytes(D) : 0);
    dim3 grid(g.batch * g.Hkv);
#define AHA_DEC(GG)                                                                              \
    {                                                                                            \
        /* the largest dynamic LDS any accepted shape asks for, set once per device */          \
        static DeviceOnce once;                                                                  \
        const hipError_t ea = device_once(once, [] {                                             \
            return hipFuncSetAttribute((const void *)decode_kernel<ESIZE, D, GG>,                \
                                       hipFuncAttributeMaxDynamicSharedMemorySize,               \
                                       (int)kDecodeSingleLds);                                   \
        });                                                                                      \
        if (ea != hipSuccess) return ea;                                                         \
        hipLaunchKernelGGL((decode_kernel<ESIZE, D, GG>), grid, dim3(kDecThreads), smem, st, g,  \
                           w_floats, ws_nu, ws_numax);                                           \
    }
    switch (g.G) {
        case 1: AHA_DEC(1) break;
        case 2: AHA_DEC(2) break;
        case 3: AHA_DEC(3) break;
        case 4: AHA_DEC(4) break;
        case 5: AHA_DEC(5) break;
        case 6: AHA_DEC(6) break;
        case 7: AHA_DEC(7) break;
        default: AHA_DEC(8) break;
    }
#undef AHA_DEC
    return hipGetLastError();
}

hipError_t launch_decode(const DecodeGeom &g, const DecodePlan &pl, void *ws, int dtype,
                         hipStream_t st) {
    if (dtype == AHA_BF16)
        return g.d == 64 ? launch_g<2, 64>(g, pl, ws, st) : launch_g<2, 128>(g, pl, ws, st);
    return g.d == 64 ? launch_g<4, 64>(g, pl, ws, st) : launch_g<4, 128>(g, pl, ws, st);
}

}  // namespace aha

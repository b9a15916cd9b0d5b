// Tile machinery shared by the bf16 kernels that multiply a tile of query rows (kept in LDS
// as the B operand of v_mfma_f32_32x32x16_bf16) with blocks of keys (A operand, loaded from
// global memory straight into registers): the LDS layout of a query tile, its loading, the
// key-fragment loads, the 64-key x 32-query block product and the accumulator layout.
#pragma once

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
// 32-row block the largest and smallest position.  Request and commit are
// separate so that every other load of the tile set-up (first key block, row
// statistics, value-prior maxima) is in flight together with the tile: under
// load a dependent round trip to memory costs several microseconds.
template <int D, int NB>
struct QTileRegs {
    static constexpr int U = TileSmem<D, NB>::ROWS * (D / 8) / 256;  // 16-byte chunks per thread
    static_assert(TileSmem<D, NB>::ROWS * (D / 8) % 256 == 0, "tile chunks divide among 256 threads");
    u32x4 w[U];
    unsigned valid;  // bit u: chunk u belongs to a real row (others are stored as zero)
};

// ROWS: the accumulator rows were chosen by the caller (g.rows); a compile-time switch, so
// that the default kernels carry none of it.
template <int D, int NB, bool ROWS = false>
__device__ __forceinline__ void q_tile_request(const ScoreGeom &g, int b, int h, int rho0,
                                               int tid, QTileRegs<D, NB> &t) {
    constexpr int CPR = D / 8;        // 16-byte chunks per row
    constexpr int STEP = 256 / CPR;   // rows between a thread's consecutive chunks
    const int c = tid % CPR;
    // flattened row rho = gi * r + ii (query head of the group, window row); one division
    // for the first row, increments for the others
    int rho = rho0 + tid / CPR;
    int gi = rho / g.r, ii = rho - gi * g.r;
    const int step_g = STEP / g.r, step_i = STEP % g.r;
    const __bf16 *base = (const __bf16 *)g.q + b * g.qs[0] + (int64_t)h * g.G * g.qs[1] +
                         (int64_t)(g.n - g.r) * g.qs[2] + c * 8;
    // rows past the last one re-read the tile's first row (the tile has at least one real
    // row), so the loads need no branches and are all issued back to back
    const int gi0 = rho0 / g.r, ii0 = rho0 - gi0 * g.r;
    t.valid = 0u;
    if constexpr (ROWS) {
        // accumulator rows chosen by the caller: the position of every row comes from the list
        // (one more round trip to memory in the set-up; the default path below has none)
        const RowMap rm{g.n, g.r, g.R, g.rows + ((int64_t)b * g.Hq + (int64_t)h * g.G) * g.r};
        const __bf16 *b0 = (const __bf16 *)g.q + b * g.qs[0] + (int64_t)h * g.G * g.qs[1] + c * 8;
        int pos[QTileRegs<D, NB>::U];
#pragma unroll
        for (int u = 0; u < QTileRegs<D, NB>::U; ++u) {
            const int rr = rho + u * STEP;
            t.valid |= rr < g.R ? 1u << u : 0u;
            pos[u] = rm.pos(rr < g.R ? rr : rho0);
        }
#pragma unroll
        for (int u = 0; u < QTileRegs<D, NB>::U; ++u) {
            const int rr = rho + u * STEP < g.R ? rho + u * STEP : rho0;
            t.w[u] = *(const u32x4 *)(b0 + (rr / g.r) * g.qs[1] + (int64_t)pos[u] * g.qs[2]);
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < QTileRegs<D, NB>::U; ++u) {
        const bool ok = rho < g.R;
        t.valid |= ok ? 1u << u : 0u;
        t.w[u] = *(const u32x4 *)(base + (ok ? gi : gi0) * g.qs[1] + (ok ? ii : ii0) * g.qs[2]);
        rho += STEP;
        gi += step_g;
        ii += step_i;
        if (ii >= g.r) {
            ii -= g.r;
            ++gi;
        }
    }
}

template <int D, int NB>
__device__ __forceinline__ void q_tile_commit(const QTileRegs<D, NB> &t, int tid, __bf16 *sQ) {
    using S = TileSmem<D, NB>;
    constexpr int CPR = D / 8;
#pragma unroll
    for (int u = 0; u < QTileRegs<D, NB>::U; ++u) {
        const int i = tid + u * 256;
        *(u32x4 *)(sQ + (i / CPR) * S::LD + (i % CPR) * 8) =
            (t.valid >> u) & 1u ? t.w[u] : u32x4{0u, 0u, 0u, 0u};
    }
}

// Per-row scale and position of the tile (one row per thread: a tile has at most 256 rows).
// The scale of window row ii (token position n - r + ii, c = position + 1 keys) is a
// logarithm and a square root per row and tile: computed in place, no table.
template <int D, int NB>
__device__ __forceinline__ float q_tile_scale(const ScoreGeom &g, const RowMap &rm, int rho0,
                                              int tid) {
    static_assert(TileSmem<D, NB>::ROWS <= 256, "one tile row per thread");
    const int rho = rho0 + min(tid, TileSmem<D, NB>::ROWS - 1);
    const int i = rm.pos(rho < g.R ? rho : 0);
    return row_scale_log2_f32(g.scale_mode, g.fixed_scale, g.lambda_floor, i + 1, g.budget, g.d);
}
template <int D, int NB>
__device__ __forceinline__ void q_tile_meta(const ScoreGeom &g, const RowMap &rm, int rho0,
                                            int tid, float lam_requested, float *sLam, int *sPos,
                                            int *sBlk) {
    using S = TileSmem<D, NB>;
    const int rho = rho0 + tid;
    const bool ok = tid < S::ROWS && rho < g.R;
    const int pos = ok ? rm.pos(rho) : -1;
    if (tid < S::ROWS) {
        sPos[tid] = pos;
        sLam[tid] = ok ? lam_requested : 0.f;
    }
    if (rm.rows) {
        // chosen rows come in no particular pattern: the 32 rows of a block are 32 adjacent
        // threads, whose positions are reduced in the vector ALU (every thread takes part)
        const int mx = reduce_lanes<1, 32>(pos, OpMaxI{});
        const int mn = reduce_lanes<1, 32>(ok ? pos : g.n, OpMinI{});
        if ((tid & 31) == 0 && tid < S::ROWS) {
            sBlk[tid >> 5] = mx;
            sBlk[NB + (tid >> 5)] = mn;
        }
    } else if (tid < NB) {
        sBlk[tid] = rm.max_pos(rho0 + tid * 32, rho0 + tid * 32 + 32);
        sBlk[NB + tid] = rm.min_pos(rho0 + tid * 32, rho0 + tid * 32 + 32);
    }
}
// Smallest position of the tile's rows, from the per-block minima (after the tile's barrier).
template <int NB>
__device__ __forceinline__ int tile_min_pos(const int *sBlk) {
    int m = sBlk[NB];
#pragma unroll
    for (int nb = 1; nb < NB; ++nb) m = min(m, sBlk[NB + nb]);
    return m;
}

// A fragments of a wave's key block: lane holds row kb + mb*32 + lane%32,
// channels ks*16 + (lane/32)*8 .. +8.  Rows at or past `end` (the end of the
// workgroup's key range, at most the sequence length) read row end - 1 instead:
// their results are masked or never written, and a prefetch past the range then
// costs one row, not a block of somebody else's keys.
template <int D>
__device__ __forceinline__ void load_a(const __bf16 *kbase, int64_t k_tstride, int kb, int end,
                                       int lane, bf16x8 (&a)[kMB][D / 16]) {
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
        const int row = min(kb + mb * 32 + (lane & 31), end - 1);
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

// The same product with the query fragments read AHEAD of their use: each fragment one
// contraction step before its products, and fragment 0 of block `nb_next` behind the last
// products of this block, so that it travels under the block's vector work (`first`: fragment
// 0 of this block on entry, of block nb_next on exit).  A fragment read right before its
// products exposes the LDS latency to the wave eight times per block; the scheduling barriers
// keep the reads where they are written (the compiler would otherwise move each read back to
// its use to save its four registers).
template <int D, int NB>
__device__ __forceinline__ bf16x8 query_fragment(const __bf16 *sQ, int nb, int ks, int lane) {
    using S = TileSmem<D, NB>;
    return *(const bf16x8 *)(sQ + (nb * 32 + (lane & 31)) * S::LD + (lane >> 5) * 8 + ks * 16);
}
template <int D, int NB>
__device__ __forceinline__ void mma_block_stream(const bf16x8 (&a)[kMB][D / 16], const __bf16 *sQ,
                                                 int nb, int nb_next, int lane, bf16x8 &first,
                                                 f32x16 (&acc)[kMB]) {
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
    bf16x8 cur = first;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 nxt = ks + 1 < D / 16 ? query_fragment<D, NB>(sQ, nb, ks + 1, lane)
                                           : query_fragment<D, NB>(sQ, nb_next, 0, lane);
#pragma unroll
        for (int mb = 0; mb < kMB; ++mb)
            acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb][ks], cur, acc[mb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        cur = nxt;
    }
    first = cur;
}

// Key row of accumulator element v of M block mb, for this lane.
__device__ __forceinline__ int acc_key(int kb, int mb, int v, int lane) {
    return kb + mb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Workgroups are handed to the eight XCDs (each with an L2 of its own) round-robin by
// their linear index.  The score kernels are launched on a one-dimensional grid of
// 8 * ceil(total / 8) workgroups and work on the logical index returned here; indices
// >= total have no work.  In full accumulation (`contiguous`) the logical index runs
// contiguously over an XCD's share, so that the workgroups of one (batch, KV head)
// problem, which re-read the same keys many times, meet in one L2 (measured 4 % faster).
// The windowed scores stream every key once; there the plain order, which spreads a
// problem over all XCDs, is the faster one (measured 5 - 15 %).
constexpr int kXcds = 8;
__device__ __forceinline__ int logical_wg_index(int total, bool contiguous) {
    if (!contiguous) return (int)blockIdx.x;
    const int per = (total + kXcds - 1) / kXcds;
    return ((int)blockIdx.x % kXcds) * per + (int)blockIdx.x / kXcds;
}
static inline dim3 xcd_grid(int64_t total) {
    return dim3((unsigned)(((total + kXcds - 1) / kXcds) * kXcds));
}

}  // namespace aha

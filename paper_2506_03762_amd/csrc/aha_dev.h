// Device-side helpers shared by the gfx950 kernels of the AhaKV eviction path.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/aha.h"

namespace aha {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

// A^T fragment of v_mfma_f32_32x32x16_bf16 from a row-major bf16 matrix in LDS (the value rows
// [slot][channel], wanted as V^T with the channels on M): the lane's channel
// col0 + lane % 32 of the eight rows row0 + 4 (lane / 32) + {0..3} and row0 + gap + 4 (lane / 32) +
// {0..3}, ld elements per row.  A lane wants a COLUMN of four elements at a time:
// ds_read_b64_tr_b16 reads, per group of 16 lanes, a tile of 4 rows x 16 elements - lane s of
// the group supplies the address of row s / 4, elements 4 (s % 4) .. + 3 - and hands lane j of
// the group column j of that tile (its elements of rows 0 .. 3, in order).  Two such reads
// make a fragment, with no repacking in the vector ALU.
typedef short s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 lds_transposed_fragment(const __bf16 *base, int ld, int row0,
                                                          int gap, int col0, int lane) {
    using lds_ptr = s16x4 __attribute__((address_space(3))) *;
    const __bf16 *p = base + (row0 + 4 * (lane >> 5) + ((lane >> 2) & 3)) * ld + col0 + (lane & 16) +
                      4 * (lane & 3);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + gap * ld));
    bf16x8 f;
    __builtin_memcpy(&f, &lo, 8);
    __builtin_memcpy((char *)&f + 8, &hi, 8);
    return f;
}

// bf16 <-> fp32 on raw bits (bf16 is the upper half of an fp32).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}

// Softmax scale of a row that normalises over c keys, already multiplied by
// log2(e) so that exp2 can be used (Sec. 4.2: lambda = sqrt(2 ln(c/k)/d) with
// k the total budget; the logarithm is clamped at 0 and the result floored).
// Evaluated in double so that the fp32 value is correctly rounded.
__device__ __forceinline__ float row_scale_log2(int scale_mode, float fixed_scale,
                                                float lambda_floor, int c, int budget,
                                                int head_dim) {
    double s;
    if (scale_mode == AHA_SCALE_FIXED) {
        s = (double)fixed_scale;
    } else {
        double lg = log((double)c / (double)budget);
        if (lg < 0.0) lg = 0.0;
        s = sqrt(2.0 * lg / (double)head_dim);
        double fl = lambda_floor < 0.f ? 1.0 / sqrt((double)head_dim) : (double)lambda_floor;
        if (s < fl) s = fl;
    }
    return (float)(s * 1.4426950408889634074);
}

// The same scale in single precision (relative error ~1e-7), for the bf16 path whose
// tolerance is four orders of magnitude wider; avoids the slow double-precision log.
__device__ __forceinline__ float row_scale_log2_f32(int scale_mode, float fixed_scale,
                                                    float lambda_floor, int c, int budget,
                                                    int head_dim) {
    float s;
    if (scale_mode == AHA_SCALE_FIXED) {
        s = fixed_scale;
    } else {
        float lg = logf((float)c / (float)budget);
        if (lg < 0.f) lg = 0.f;
        s = sqrtf(2.f * lg / (float)head_dim);
        const float fl = lambda_floor < 0.f ? rsqrtf((float)head_dim) : lambda_floor;
        if (s < fl) s = fl;
    }
    return s * kLog2e;
}

// 2^x on the transcendental unit (v_exp_f32): no denormal results, exp2(-inf) = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- exchanges between lanes inside the vector ALU ----
// (a shuffle built on ds_bpermute goes through the LDS crossbar and costs its latency at
// every step of a reduction; the forms below are plain vector instructions)
// Data-parallel primitive with a fixed control word: a value from lane ^ 1, ^ 2, ^ 4, ^ 8.
template <int CTRL, int BANKS = 0xf>
__device__ __forceinline__ uint32_t dpp_move(uint32_t old, uint32_t x) {
    return __builtin_amdgcn_update_dpp(old, x, CTRL, 0xf, BANKS, false);
}
template <int M>
__device__ __forceinline__ uint32_t from_lane_xor(uint32_t x) {
    static_assert(M == 1 || M == 2 || M == 4 || M == 8, "within a row of 16 lanes");
    if constexpr (M == 1) return dpp_move<0xb1>(0u, x);       // quad_perm [1,0,3,2]
    else if constexpr (M == 2) return dpp_move<0x4e>(0u, x);  // quad_perm [2,3,0,1]
    else if constexpr (M == 4)  // row_shl:4 where bit 2 of the lane is clear (banks 0, 2), row_shr:4 elsewhere
        return dpp_move<0x114, 0xa>(dpp_move<0x104, 0x5>(0u, x), x);
    else return dpp_move<0x128>(0u, x);                       // row_ror:8
}
template <int M>
__device__ __forceinline__ float from_lane_xor(float x) {
    return __uint_as_float(from_lane_xor<M>(__float_as_uint(x)));
}
// op(x, x of lane ^ M) for any power of two M < 64.  Lanes ^ 16 and ^ 32 use
// v_permlane16_swap / v_permlane32_swap: applied to (x, x) they return the own and the
// partner's value in an order that depends on the lane, which a symmetric op does not mind.
template <int M, class T, class Op>
__device__ __forceinline__ T combine_lane_xor(T x, Op op) {
    static_assert(sizeof(T) == 4, "32-bit values");
    uint32_t bits;
    __builtin_memcpy(&bits, &x, 4);
    uint32_t o0, o1;
    if constexpr (M == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(bits, bits, false, false);
        o0 = r[0]; o1 = r[1];
    } else if constexpr (M == 32) {
        const auto r = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
        o0 = r[0]; o1 = r[1];
    } else {
        o0 = bits; o1 = from_lane_xor<M>(bits);
    }
    T a, b;
    __builtin_memcpy(&a, &o0, 4);
    __builtin_memcpy(&b, &o1, 4);
    return op(a, b);
}
// Reduction with a symmetric op over the lanes that differ in the bits LO <= bit < HI
// (powers of two): LO = 1, HI = 64 is the whole wave, LO = 1, HI = 16 an aligned group of
// 16 lanes, LO = 16, HI = 64 the four lanes with the same position in their row.
template <int LO, int HI, class T, class Op>
__device__ __forceinline__ T reduce_lanes(T v, Op op) {
    if constexpr (LO < HI) {
        v = combine_lane_xor<LO>(v, op);
        return reduce_lanes<LO * 2, HI>(v, op);
    } else {
        return v;
    }
}
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMinU { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; } };
struct OpMaxU { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };

__device__ __forceinline__ float wave_max(float v) { return reduce_lanes<1, 64>(v, OpMax{}); }
__device__ __forceinline__ float wave_sum(float v) { return reduce_lanes<1, 64>(v, OpSum{}); }

// Value prior gamma / max(gamma) (Sec. 4.3) as gamma * (1 / max).  A head whose value rows
// are all zero has max(gamma) = 0: the prior is then 1 everywhere (the inverse is stored as
// a negative number, which no real maximum produces, and tells the factor to be 1).
__device__ __forceinline__ float prior_inverse(float gmax) { return gmax > 0.f ? 1.f / gmax : -1.f; }
__device__ __forceinline__ float prior_factor(float gam, float ginv) {
    return ginv < 0.f ? 1.f : gam * ginv;
}

// nu = ||V_row||^2 (Sec. 4.3) of the value rows [lo, hi) of one head, into s_nu[row - lo]
// (LDS); called by all 256 threads of a workgroup, no barrier inside.  16-byte loads, the
// lanes of a row adjacent.  The rows are read with streaming (non-temporal) loads: they are
// used once, and kept out of the caches they leave them to the keys, which the two score
// passes read twice.  U independent loads are in flight per lane: nine for the stand-alone
// kernel, whose thousands of workgroups keep the memory system full (with 16 lanes per row a
// 256-row tile and its pooling halo take two batches; many more measured slower there).
template <int ESIZE, int U = 9>
__device__ __forceinline__ void value_norms_to_lds(const char *vbase, int64_t row_stride, int d,
                                                   int lo, int hi, float *s_nu, int tid) {
    const int lpr = d * ESIZE / 16;  // lanes per row: 8, 16 or 32
    const int rows_per_pass = 256 / lpr;
    const int sub = tid % lpr, rloc = tid / lpr;
    for (int row0 = lo + rloc; row0 < hi; row0 += U * rows_per_pass) {
        u32x4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = min(row0 + u * rows_per_pass, hi - 1);
            w[u] = __builtin_nontemporal_load(
                (const u32x4 *)(vbase + (int64_t)ESIZE * row * row_stride + sub * 16));
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
}

// Softmax geometry of the flattened query rows of one KV head: row rho of the
// group is query head g = rho / r, window row ii = rho % r, token position
// i = n - r + ii - or, when the caller chose the accumulator rows, rows[rho]
// (`rows` points at the positions of this KV head's first query head; the G heads'
// lists follow each other, which is the flattened order; positions are clamped to
// the sequence, so that a bad list cannot address memory outside the tensors).
struct RowMap {
    int n, r, R;  // sequence length, window, G * r
    const int32_t *rows;  // null: the r most recent rows
    __device__ __forceinline__ int pos(int rho) const {
        if (rho >= R) return -1;
        if (rows) return min(max(rows[rho], 0), n - 1);
        return n - r + rho % r;
    }
    __device__ __forceinline__ int head(int rho) const { return rho / r; }
    // largest / smallest position among rows [lo, hi) (hi > lo, clipped to R); closed forms
    // for the most recent rows, a scan for chosen rows (used on the small fp32 path only)
    __device__ __forceinline__ int max_pos(int lo, int hi) const {
        if (hi > R) hi = R;
        if (lo >= hi) return -1;
        if (rows) {
            int m = -1;
            for (int t = lo; t < hi; ++t) m = max(m, pos(t));
            return m;
        }
        return (lo / r != (hi - 1) / r) ? n - 1 : n - r + (hi - 1) % r;
    }
    __device__ __forceinline__ int min_pos(int lo, int hi) const {
        if (hi > R) hi = R;
        if (lo >= hi) return n;
        if (rows) {
            int m = n;
            for (int t = lo; t < hi; ++t) m = min(m, pos(t));
            return m;
        }
        return (lo / r != (hi - 1) / r) ? n - r : n - r + lo % r;
    }
};

struct OpMinI { __device__ __forceinline__ int operator()(int a, int b) const { return a < b ? a : b; } };
struct OpMaxI { __device__ __forceinline__ int operator()(int a, int b) const { return a > b ? a : b; } };

}  // namespace aha

// Host-side declarations shared by the kernel translation units and the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "../../include/aha.h"

namespace aha {

// One-time set-up per device (function attributes, symbol addresses): `fn` runs once on
// each device, with that device current, whatever thread gets there first; its result is
// kept and returned to every later caller on that device.
constexpr int kMaxDevices = 64;
struct DeviceOnce {
    std::once_flag flag[kMaxDevices];
    hipError_t err[kMaxDevices];
};
template <class F>
inline hipError_t device_once(DeviceOnce &o, F fn) {
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::call_once(o.flag[dev], [&] { o.err[dev] = fn(); });
    return o.err[dev];
}

// Geometry of one prefill call, passed by value to the kernels.
struct ScoreGeom {
    const void *q, *k, *v;
    const int32_t *rows;  // accumulator rows chosen by the caller [batch, Hq, r], or null
    int64_t qs[3], ks[3], vs[3];  // element strides: batch, head, token
    int batch, Hq, Hkv, G, d, n;
    int r;       // window
    int R;       // G * r flattened query rows per KV head
    int budget;
    int scale_mode;
    float fixed_scale, lambda_floor;
    int value_prior, pool;
    int dtype;   // AHA_F32 | AHA_BF16
};

// Where things live in the caller's workspace during aha_prefill_scores.
struct PrefillPlan {
    int Z;           // batch * Hkv problems
    int NB;          // 32-row blocks per query tile (bf16 path): 1, 2, 4 or 8
    int qtile;       // NB * 32 rows
    int n_qtiles;    // query tiles per problem
    int chunk_keys;  // keys per pass-1 workgroup
    int nchunks;     // pass-1 key chunks per (problem, query tile)
    int p2_keys;     // keys per pass-2 workgroup (a multiple of kP2Keys)
    int n_vtiles;    // value-prior tiles per problem (separate launch)
    bool can_fold;   // windowed bf16 scores: pass 1 can form the value prior per key chunk
    size_t off_rowL, off_partial, off_partial_mean, off_gamma, off_gblockmax, off_nu;
    size_t bytes;
};

constexpr int kVTileRows = 256;   // rows per value-prior workgroup
constexpr int kP2Keys = 256;      // keys per pass-2 workgroup (4 waves x 64)

// value_prior.hip
// `lse`, when not null, holds the caller's natural-log row normalisers
// [batch, Hq, window]; the launch then also writes them, in the log2 domain, where pass 2
// expects the row statistics (and the score launchers skip pass 1).
// `prior_here`: this launch forms the value prior (the windowed bf16 scores form it inside
// their row-statistics launch instead).  Launches nothing when there is nothing to do.
hipError_t launch_value_prior(const ScoreGeom &g, const PrefillPlan &pl, void *ws,
                              float *scores, const float *lse, bool prior_here, hipStream_t st);
// score_f32.hip
// `mid`, when not null, is recorded between the two passes; `have_lse`: the row statistics
// are already in the workspace, pass 1 is skipped.
hipError_t launch_score_f32(const ScoreGeom &g, const PrefillPlan &pl, void *ws,
                            float *scores, hipStream_t st, hipEvent_t mid, bool have_lse);
// score_bf16.hip
// `fold_prior`: pass 1 also forms the value prior of its key range (windowed scores only).
hipError_t launch_score_bf16(const ScoreGeom &g, const PrefillPlan &pl, void *ws,
                             float *scores, hipStream_t st, hipEvent_t mid, bool have_lse,
                             bool fold_prior);
// Row statistics of the observed rows out (pass 1 only): natural-log normaliser and entropy,
// dense [batch, Hq, window]; either pointer may be null.
hipError_t launch_row_stats_bf16(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *lse,
                                 float *entropy, hipStream_t st);
hipError_t launch_row_stats_f32(const ScoreGeom &g, const PrefillPlan &pl, void *ws, float *lse,
                                float *entropy, hipStream_t st);
// attn_window.hip
// Attention output of the observed rows: blocks of 32 flattened query rows per problem, each
// split over `nparts` key ranges whose partials (output rows + (max, sum) per row) sit in the
// workspace.
struct WindowAttnPlan {
    int n_blocks;   // blocks of 32 flattened query rows per (batch, KV head)
    int nparts;     // key ranges per block (bf16 path; 1 on the fp32 path, which needs no workspace)
    int nq;         // row blocks per workgroup: 2, or 1 when there is a single block
    size_t off_ms;  // (max, sum) pairs behind the partial outputs
    size_t bytes;
};
hipError_t launch_window_attention(const ScoreGeom &g, const WindowAttnPlan &pl, void *ws,
                                   void *out, float *lse, hipStream_t st);
// topk.hip
// `pool` > 1: the candidates are ranked by the scores pooled over `pool` tokens, which are
// written to `pooled` ([Z][n] floats) first.
// `sink`: the first positions, always retained and not ranked.
hipError_t launch_topk(const float *scores, int Z, int n, int budget, int recent, int sink,
                       int pool, float *pooled, int32_t *idx, hipStream_t st);
// compact.hip
hipError_t launch_compact(const ScoreGeom &g, const float *scores, const int32_t *idx,
                          int budget, int slots, int dtype, void *kc, void *vc, float *fc,
                          int32_t *pos, int32_t *free_slot, hipStream_t st);
// decode.hip
struct DecodeGeom {
    const void *q, *k_new, *v_new;
    void *kc, *vc, *out;
    float *fc;
    int32_t *pos, *free_slot;
    int batch, Hq, Hkv, G, d, budget, recent, slots, logical_pos;
    int scale_mode;
    float fixed_scale, lambda_floor;
    int sink;          // positions < sink are never evicted
    int value_prior;   // the added probabilities are refined by ||v||^2 / max over the live slots
};
// With few (batch, KV head) problems the slots of a head are split over nsplit workgroups
// (two launches, partials in the workspace); otherwise one workgroup handles a head.
constexpr int kMaxDecodeSplit = 64;  // most workgroups a head's slots are split over
constexpr size_t kDecodeSplitLds = 64 * 1024;    // dynamic LDS of a split workgroup, at most
constexpr size_t kDecodeSingleLds = 150 * 1024;  // dynamic LDS of the one-workgroup-per-head kernel, at most
// bf16 caches with at least this many query heads per KV head: the one-workgroup-per-head
// kernel forms the dots on the matrix core, from a query tile of 32 padded rows in LDS
constexpr int kDecodeMfmaGroup = 5;
constexpr size_t kDecodeQTileBytes(int d) { return (size_t)32 * (d + 8) * 2; }
// bf16 caches with at least this many query heads per KV head: the values are weighted on the
// matrix core as well (16 slots per wave at a time, staged through LDS)
constexpr int kDecodeMfmaValuesGroup = 4;  // (with 4 heads the dots stay in the vector ALU, with 3 the values too: measured faster)
// Floats of the first region of decode_kernel's dynamic LDS (raw dots of all live slots, later
// the waves' partial outputs [16][G][d]); with the values on the matrix core every wave also
// stages 16 value rows over the query tile (if any) and this region.
// Layout: [query tile][this region][G * live].
inline size_t decode_w_floats(int G, int live, int d, bool mfma_dots, bool mfma_values) {
    size_t w = (size_t)G * live > (size_t)16 * G * d ? (size_t)G * live : (size_t)16 * G * d;
    if (mfma_values) {
        const size_t staging = (size_t)16 * 16 * (d + 8) * 2, tile = mfma_dots ? kDecodeQTileBytes(d) : 0;
        const size_t need = staging > tile ? (staging - tile + 3) / 4 : 0;
        if (need > w) w = need;
    }
    return w;
}

struct DecodePlan {
    int nsplit;      // 1: single-launch path
    int sps;         // slots per split
    size_t off_part; // partial outputs behind the raw dots
    size_t off_nu;   // ||v||^2 of every live slot behind those (value prior in the loop)
    size_t bytes;    // workspace bytes (0 when nsplit == 1)
    bool fits;       // the LDS the chosen path needs is within its limit
};
hipError_t launch_decode(const DecodeGeom &g, const DecodePlan &pl, void *ws, int dtype,
                         hipStream_t st);

}  // namespace aha

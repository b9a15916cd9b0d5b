// C ABI of the AhaKV eviction path: argument checks, workspace layout and
// kernel launches.  Every check runs on the host before anything is
// enqueued, so the error paths need no GPU.
#include <stdarg.h>
#include <stdio.h>

#include "aha_host.h"

namespace aha {

static thread_local char g_err[512] = "";
static thread_local hipEvent_t g_stage_ev[4] = {nullptr, nullptr, nullptr, nullptr};
static thread_local bool g_stage_on = false;

static hipError_t stage(int i, hipStream_t st) {
    return g_stage_on ? hipEventRecord(g_stage_ev[i], st) : hipSuccess;
}

static int32_t fail(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int esize(int dtype) { return dtype == AHA_BF16 ? 2 : 4; }

// Checks shared by all entry points.
static int32_t check_common(const aha_params *p) {
    if (!p) return fail(AHA_ERR_INVALID_ARG, "params is null");
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1)
        return fail(AHA_ERR_INVALID_ARG, "batch, n_q_heads and n_kv_heads must be >= 1");
    if (p->n_q_heads % p->n_kv_heads != 0)
        return fail(AHA_ERR_INVALID_ARG, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)",
                    p->n_q_heads, p->n_kv_heads);
    if ((int64_t)p->batch * p->n_kv_heads > 65535)  // a grid's y dimension in several launches
        return fail(AHA_ERR_UNSUPPORTED, "batch * n_kv_heads (%lld) exceeds 65535",
                    (long long)p->batch * p->n_kv_heads);
    if (p->dtype != AHA_F32 && p->dtype != AHA_BF16)
        return fail(AHA_ERR_INVALID_ARG, "dtype %d is neither AHA_F32 nor AHA_BF16", p->dtype);
    if (p->head_dim != 64 && p->head_dim != 128)
        return fail(AHA_ERR_UNSUPPORTED, "head_dim %d: only 64 and 128 are built", p->head_dim);
    if (p->budget < 1) return fail(AHA_ERR_INVALID_ARG, "budget must be >= 1");
    if (p->budget > 1 << 30) return fail(AHA_ERR_UNSUPPORTED, "budget beyond 2^30");
    if (p->recent < 0 || p->recent > p->budget)
        return fail(AHA_ERR_INVALID_ARG, "recent (%d) must lie in [0, budget=%d]", p->recent,
                    p->budget);
    if (p->scale_mode != AHA_SCALE_FIXED && p->scale_mode != AHA_SCALE_ADAPTIVE)
        return fail(AHA_ERR_INVALID_ARG, "scale_mode %d is unknown", p->scale_mode);
    if (p->scale_mode == AHA_SCALE_FIXED && !(p->fixed_scale >= 0.f))
        return fail(AHA_ERR_INVALID_ARG, "fixed_scale must be >= 0");
    if (p->sink < 0 || (int64_t)p->sink + p->recent > p->budget)
        return fail(AHA_ERR_INVALID_ARG, "sink (%d) must be >= 0 and sink + recent (%d) <= budget (%d)",
                    p->sink, p->recent, p->budget);
    if (p->decode_value_prior != 0 && p->decode_value_prior != 1)
        return fail(AHA_ERR_INVALID_ARG, "decode_value_prior must be 0 or 1");
    if (p->reserved != 0) return fail(AHA_ERR_INVALID_ARG, "reserved must be 0");
    return AHA_OK;
}

static int32_t check_stride(const char *name, const int64_t s[3], int dtype, int d) {
    const int a = 16 / esize(dtype);
    for (int t = 0; t < 3; ++t)
        if (s[t] < 0 || s[t] % a != 0)
            return fail(AHA_ERR_INVALID_ARG, "%s_stride[%d]=%lld must be a non-negative multiple of %d elements",
                        name, t, (long long)s[t], a);
    if (s[2] < d)
        return fail(AHA_ERR_INVALID_ARG, "%s_stride[2]=%lld is smaller than head_dim", name,
                    (long long)s[2]);
    return AHA_OK;
}

static int32_t check_prefill(const aha_params *p, bool need_strides) {
    int32_t rc = check_common(p);
    if (rc) return rc;
    if (p->seq_len < 1) return fail(AHA_ERR_INVALID_ARG, "seq_len must be >= 1");
    if (p->seq_len > 1 << 30) return fail(AHA_ERR_UNSUPPORTED, "seq_len beyond 2^30");
    if (p->budget > p->seq_len)
        return fail(AHA_ERR_INVALID_ARG, "budget (%d) exceeds seq_len (%d)", p->budget, p->seq_len);
    if (p->window < 1 || p->window > p->seq_len)
        return fail(AHA_ERR_INVALID_ARG, "window (%d) must lie in [1, seq_len=%d]", p->window,
                    p->seq_len);
    if (p->value_prior != 0 && p->value_prior != 1)
        return fail(AHA_ERR_INVALID_ARG, "value_prior must be 0 or 1");
    if (p->value_prior && (p->pool_kernel < 1 || p->pool_kernel > 255 || p->pool_kernel % 2 == 0))
        return fail(AHA_ERR_INVALID_ARG, "pool_kernel (%d) must be odd and in [1, 255]",
                    p->pool_kernel);
    if ((int64_t)(p->n_q_heads / p->n_kv_heads) * p->window > (int64_t)1 << 30)
        return fail(AHA_ERR_UNSUPPORTED, "group * window is too large");
    if (p->score_pool < 0 || p->score_pool > 255 || (p->score_pool > 1 && p->score_pool % 2 == 0))
        return fail(AHA_ERR_INVALID_ARG, "score_pool (%d) must be 0 or odd and in [1, 255]",
                    p->score_pool);
    if (need_strides) {
        if ((rc = check_stride("q", p->q_stride, p->dtype, p->head_dim))) return rc;
        if ((rc = check_stride("k", p->k_stride, p->dtype, p->head_dim))) return rc;
        if ((rc = check_stride("v", p->v_stride, p->dtype, p->head_dim))) return rc;
    }
    return AHA_OK;
}

// Compaction reads K, V, the scores and the index list: only what those need is checked.
static int32_t check_compact(const aha_params *p) {
    int32_t rc = check_common(p);
    if (rc) return rc;
    if (p->seq_len < 1) return fail(AHA_ERR_INVALID_ARG, "seq_len must be >= 1");
    if (p->seq_len > 1 << 30) return fail(AHA_ERR_UNSUPPORTED, "seq_len beyond 2^30");
    if (p->budget > p->seq_len)
        return fail(AHA_ERR_INVALID_ARG, "budget (%d) exceeds seq_len (%d)", p->budget, p->seq_len);
    if ((rc = check_stride("k", p->k_stride, p->dtype, p->head_dim))) return rc;
    return check_stride("v", p->v_stride, p->dtype, p->head_dim);
}

static int32_t check_ptr(const char *name, const void *ptr, size_t align) {
    if (!ptr) return fail(AHA_ERR_INVALID_ARG, "%s is null", name);
    if ((uintptr_t)ptr % align != 0)
        return fail(AHA_ERR_INVALID_ARG, "%s is not %zu-byte aligned", name, align);
    return AHA_OK;
}

static ScoreGeom make_geom(const aha_params *p, const void *q, const void *k, const void *v) {
    ScoreGeom g{};
    g.q = q; g.k = k; g.v = v; g.rows = nullptr;
    for (int t = 0; t < 3; ++t) { g.qs[t] = p->q_stride[t]; g.ks[t] = p->k_stride[t]; g.vs[t] = p->v_stride[t]; }
    g.batch = p->batch; g.Hq = p->n_q_heads; g.Hkv = p->n_kv_heads; g.G = g.Hq / g.Hkv;
    g.d = p->head_dim; g.n = p->seq_len; g.r = p->window; g.R = g.G * g.r;
    g.budget = p->budget; g.scale_mode = p->scale_mode; g.fixed_scale = p->fixed_scale;
    g.lambda_floor = p->lambda_floor; g.value_prior = p->value_prior; g.pool = p->pool_kernel;
    g.dtype = p->dtype;
    return g;
}

// Workspace layout of aha_prefill_scores.
static PrefillPlan plan_prefill(const aha_params *p) {
    PrefillPlan pl{};
    const int G = p->n_q_heads / p->n_kv_heads;
    const int64_t R = (int64_t)G * p->window;
    const int n = p->seq_len;
    pl.Z = p->batch * p->n_kv_heads;
    pl.n_vtiles = (n + kVTileRows - 1) / kVTileRows;
    if (p->dtype == AHA_BF16) {
        const int blocks = (int)((R + 31) / 32);
        pl.NB = blocks >= 8 ? 8 : blocks > 2 ? 4 : blocks;  // 1, 2, 4, 8
        if (blocks == 3) pl.NB = 4;
        pl.qtile = pl.NB * 32;
        pl.n_qtiles = (int)((R + pl.qtile - 1) / pl.qtile);
        // Work units: query tiles are paired (first with last, ...) so that in full
        // accumulation every pair sees about the same number of keys, and the key steps of
        // a pair are cut into `nchunks` parts so that about 512 workgroups (two per CU) exist.
        const int64_t npairs = (pl.n_qtiles + 1) / 2;
        const int64_t units = (int64_t)pl.Z * npairs;
        const int target_wgs = 512;
        int64_t want = (target_wgs + units - 1) / units;
        const int64_t steps = (n + kP2Keys - 1) / kP2Keys;          // 256-key steps of a full tile
        const int64_t pair_steps = pl.n_qtiles > 1 ? steps + 1 : steps;
        if (want > pair_steps) want = pair_steps;
        if (want < 1) want = 1;
        pl.nchunks = (int)want;
        pl.chunk_keys = (int)(((steps + want - 1) / want) * kP2Keys);
        // windowed pass 2 (one tile) walks over the same key ranges, several steps per workgroup
        pl.p2_keys = pl.chunk_keys;
    } else {
        pl.NB = 0;
        pl.qtile = 1;
        pl.n_qtiles = 1;
        pl.chunk_keys = n;
        pl.nchunks = 1;
        pl.p2_keys = kP2Keys;
    }
    size_t off = 0;
    pl.off_rowL = off;  // fp32 path: log-sum-exp of every observed row
    const size_t rows = p->dtype == AHA_BF16 ? (size_t)pl.n_qtiles * pl.qtile : (size_t)R;
    if (p->dtype != AHA_BF16) off = align_up(off + sizeof(float) * (size_t)pl.Z * rows, 256);
    pl.off_partial = off;
    if (p->dtype == AHA_BF16)
        off = align_up(off + sizeof(float) * (size_t)pl.Z * rows * pl.nchunks, 256);
    pl.off_partial_mean = off;  // aha_prefill_row_stats: per-chunk mean scaled logit
    if (p->dtype == AHA_BF16)
        off = align_up(off + sizeof(float) * (size_t)pl.Z * rows * pl.nchunks, 256);
    pl.off_gamma = off;
    off = align_up(off + sizeof(float) * (size_t)pl.Z * n, 256);
    pl.off_gblockmax = off;  // per-range maxima of the value prior: per tile, or per key chunk
    const size_t n_maxima = (size_t)(pl.n_vtiles > pl.nchunks ? pl.n_vtiles : pl.nchunks);
    off = align_up(off + sizeof(float) * (size_t)pl.Z * n_maxima, 256);
    // windowed bf16 scores: pass 1 forms the value prior itself (the pooling halo it gathers
    // at a range's ends is bounded: pool widths up to 17)
    pl.can_fold = p->dtype == AHA_BF16 && pl.n_qtiles == 1 && p->pool_kernel <= 17;
    pl.off_nu = off;  // squared value norms [Z][n], pass 1 -> its own pooling
    if (pl.can_fold) off = align_up(off + sizeof(float) * (size_t)pl.Z * n, 256);
    pl.bytes = off;
    return pl;
}

// Attention output of the observed rows: about 512 workgroups over (block of 32 rows, key
// range, problem); the key ranges' partials go through the workspace.
static WindowAttnPlan plan_window_attn(const aha_params *p) {
    WindowAttnPlan pl{};
    const int64_t R = (int64_t)(p->n_q_heads / p->n_kv_heads) * p->window;
    const int64_t Z = (int64_t)p->batch * p->n_kv_heads;
    pl.n_blocks = (int)((R + 31) / 32);
    pl.nparts = 1;
    pl.nq = pl.n_blocks >= 2 ? 2 : 1;  // row blocks per workgroup
    if (p->dtype != AHA_BF16) return pl;  // fp32: one workgroup per row, no partials
    const int64_t wg_keys = kP2Keys / 2;  // a workgroup step: four waves of 32 keys
    const int64_t steps = (p->seq_len + wg_keys - 1) / wg_keys;
    const int64_t groups = (pl.n_blocks + pl.nq - 1) / pl.nq;
    int64_t want = (512 + Z * groups - 1) / (Z * groups);
    if (want > steps) want = steps;
    if (want > 64) want = 64;
    pl.nparts = (int)(want < 1 ? 1 : want);
    const size_t rows = (size_t)Z * pl.nparts * pl.n_blocks * 32;
    pl.off_ms = align_up(sizeof(float) * rows * p->head_dim, 256);
    pl.bytes = align_up(pl.off_ms + 2 * sizeof(float) * rows, 256);
    return pl;
}

// Decode: split a head's slots over workgroups when there are too few heads to fill the GPU.
// A split workgroup keeps group * (slots of its range) dots and 4 * group * head_dim partial
// outputs in LDS; the number of splits is raised until that fits kDecodeSplitLds (the limit
// a launch may ask for without an attribute), and `fits` says whether kMaxDecodeSplit
// splits were enough.
static DecodePlan plan_decode(const aha_params *p) {
    DecodePlan pl{};
    const int Z = p->batch * p->n_kv_heads, G = p->n_q_heads / p->n_kv_heads;
    const int live = p->budget + 1;
    pl.fits = true;
    int nsplit = 1;
    if (Z < 128) {
        nsplit = (256 + Z - 1) / Z;
        const int max_by_size = (live + 63) / 64;  // at least 64 slots per workgroup
        if (nsplit > max_by_size) nsplit = max_by_size;
        if (nsplit > kMaxDecodeSplit) nsplit = kMaxDecodeSplit;
        if (nsplit > 1) {
            const int64_t room = (int64_t)kDecodeSplitLds / 4 - 4 * (int64_t)G * p->head_dim;
            const int64_t max_sps = room / G;  // slots per split whose dots fit beside the outputs
            const int64_t need = max_sps > 0 ? (live + max_sps - 1) / max_sps : kMaxDecodeSplit + 1;
            if (need > nsplit) nsplit = need > kMaxDecodeSplit ? kMaxDecodeSplit : (int)need;
            if (need > kMaxDecodeSplit) pl.fits = false;
        }
    }
    pl.nsplit = nsplit < 1 ? 1 : nsplit;
    pl.sps = (live + pl.nsplit - 1) / pl.nsplit;
    pl.nsplit = (live + pl.sps - 1) / pl.sps;
    if (pl.nsplit > 1) {
        pl.off_part = align_up(sizeof(float) * (size_t)Z * G * live, 256);
        pl.off_nu = align_up(pl.off_part + sizeof(float) * (size_t)Z * pl.nsplit * G * (p->head_dim + 2), 256);
        pl.bytes = pl.off_nu;
    } else {
        // one workgroup per head: dots and output probabilities of all live slots in LDS
        const bool mfma = p->dtype == AHA_BF16 && G >= kDecodeMfmaGroup;
        const bool mfma_v = p->dtype == AHA_BF16 && G >= kDecodeMfmaValuesGroup;
        const size_t w_floats = decode_w_floats(G, live, p->head_dim, mfma, mfma_v);
        const size_t q_tile = mfma ? kDecodeQTileBytes(p->head_dim) : 0;
        if ((w_floats + (size_t)G * live) * 4 + q_tile > kDecodeSingleLds) pl.fits = false;
    }
    // value prior inside the loop: the live slots' value norms and their maximum per head
    if (p->decode_value_prior)
        pl.bytes = align_up(pl.off_nu + sizeof(float) * ((size_t)Z * live + Z), 256);
    return pl;
}

static int32_t check_ws(const void *ws, size_t have, size_t need) {
    if (need == 0) return AHA_OK;
    if (!ws) return fail(AHA_ERR_WORKSPACE, "workspace is null (%zu bytes needed)", need);
    if ((uintptr_t)ws % 256 != 0) return fail(AHA_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (have < need)
        return fail(AHA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
    return AHA_OK;
}

static int32_t hip_result(hipError_t e, const char *what) {
    if (e == hipSuccess) return AHA_OK;
    return fail(AHA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace aha

using namespace aha;

extern "C" {

// Selection: the pooled scores, when the scores are smoothed first.
static size_t topk_ws_bytes(const aha_params *p) {
    if (p->score_pool <= 1) return 0;
    return align_up(sizeof(float) * (size_t)p->batch * p->n_kv_heads * p->seq_len, 256);
}

int32_t aha_workspace_bytes(const aha_params *p, size_t *out_bytes) {
    if (!out_bytes) return fail(AHA_ERR_INVALID_ARG, "out_bytes is null");
    if (p && p->seq_len == 0) {  // a caller of aha_decode_step only
        const int32_t rc = check_common(p);
        if (rc) return rc;
        *out_bytes = plan_decode(p).bytes;
        return AHA_OK;
    }
    int32_t rc = check_prefill(p, false);
    if (rc) return rc;
    const size_t a = plan_prefill(p).bytes, d = plan_decode(p).bytes, t = topk_ws_bytes(p);
    *out_bytes = a > d ? (a > t ? a : t) : (d > t ? d : t);
    return AHA_OK;
}

// Shared by aha_prefill_scores (lse == nullptr), aha_prefill_scores_lse and
// aha_prefill_scores_rows (rows != nullptr).
static int32_t prefill_scores_impl(const aha_params *p, const void *q, const void *k,
                                   const void *v, const float *lse, bool with_lse,
                                   const int32_t *rows, float *scores, void *workspace,
                                   size_t workspace_bytes, void *stream) {
    int32_t rc = check_prefill(p, true);
    if (rc) return rc;
    if ((rc = check_ptr("q", q, 16)) || (rc = check_ptr("k", k, 16)) ||
        (rc = check_ptr("scores", scores, 4)))
        return rc;
    if (with_lse && (rc = check_ptr("lse", lse, 4))) return rc;
    if (p->value_prior && (rc = check_ptr("v", v, 16))) return rc;
    const PrefillPlan pl = plan_prefill(p);
    if ((rc = check_ws(workspace, workspace_bytes, pl.bytes))) return rc;
    // the bf16 score launches are one-dimensional over all their workgroups
    const int64_t score_wgs = (int64_t)pl.Z * ((pl.n_qtiles + 1) / 2) * pl.nchunks;
    if (score_wgs > (int64_t)1 << 30)
        return fail(AHA_ERR_UNSUPPORTED, "problem exceeds the launch grid limits");
    // chosen accumulator rows: the bf16 kernels keep them in one query tile
    if (rows && p->dtype == AHA_BF16 && pl.n_qtiles != 1)
        return fail(AHA_ERR_UNSUPPORTED,
                    "chosen accumulator rows: group * window (%d) must not exceed 256 for bf16",
                    (p->n_q_heads / p->n_kv_heads) * p->window);
    ScoreGeom g = make_geom(p, q, k, v);
    g.rows = rows;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = hip_result(stage(0, st), "stage event"))) return rc;
    // the windowed bf16 scores form the value prior inside their row-statistics launch
    const bool fold_prior = pl.can_fold && p->value_prior && !with_lse && !rows;
    if ((rc = hip_result(launch_value_prior(g, pl, workspace, scores, lse,
                                            p->value_prior && !fold_prior, st),
                         "value-prior kernel")))
        return rc;
    if ((rc = hip_result(stage(1, st), "stage event"))) return rc;
    hipEvent_t mid = g_stage_on ? g_stage_ev[2] : nullptr;
    if (p->dtype == AHA_BF16)
        rc = hip_result(launch_score_bf16(g, pl, workspace, scores, st, mid, with_lse, fold_prior),
                        "bf16 score kernels");
    else
        rc = hip_result(launch_score_f32(g, pl, workspace, scores, st, mid, with_lse),
                        "fp32 score kernels");
    if (rc) return rc;
    return hip_result(stage(3, st), "stage event");
}

int32_t aha_prefill_scores(const aha_params *p, const void *q, const void *k, const void *v,
                           float *scores, void *workspace, size_t workspace_bytes, void *stream) {
    return prefill_scores_impl(p, q, k, v, nullptr, false, nullptr, scores, workspace,
                               workspace_bytes, stream);
}

int32_t aha_prefill_scores_rows(const aha_params *p, const void *q, const void *k, const void *v,
                                const int32_t *rows, float *scores, void *workspace,
                                size_t workspace_bytes, void *stream) {
    const int32_t rc = check_ptr("rows", rows, 4);
    if (rc) return rc;
    return prefill_scores_impl(p, q, k, v, nullptr, false, rows, scores, workspace,
                               workspace_bytes, stream);
}

int32_t aha_prefill_scores_lse(const aha_params *p, const void *q, const void *k, const void *v,
                               const float *lse, float *scores, void *workspace,
                               size_t workspace_bytes, void *stream) {
    return prefill_scores_impl(p, q, k, v, lse, true, nullptr, scores, workspace, workspace_bytes,
                               stream);
}

int32_t aha_window_attention_workspace_bytes(const aha_params *p, size_t *out_bytes) {
    if (!out_bytes) return fail(AHA_ERR_INVALID_ARG, "out_bytes is null");
    const int32_t rc = check_prefill(p, false);
    if (rc) return rc;
    *out_bytes = plan_window_attn(p).bytes;
    return AHA_OK;
}

int32_t aha_prefill_window_attention(const aha_params *p, const void *q, const void *k,
                                     const void *v, void *out, float *lse, void *workspace,
                                     size_t workspace_bytes, void *stream) {
    int32_t rc = check_prefill(p, true);
    if (rc) return rc;
    if ((rc = check_ptr("q", q, 16)) || (rc = check_ptr("k", k, 16)) || (rc = check_ptr("v", v, 16)) ||
        (rc = check_ptr("out", out, 16)))
        return rc;
    if (lse && (rc = check_ptr("lse", lse, 4))) return rc;
    const WindowAttnPlan pl = plan_window_attn(p);
    if ((rc = check_ws(workspace, workspace_bytes, pl.bytes))) return rc;
    const int64_t Z = (int64_t)p->batch * p->n_kv_heads;
    const int64_t wgs = p->dtype == AHA_BF16 ? (Z * pl.nparts + 7) / 8 * 8 * pl.n_blocks
                                             : (int64_t)pl.n_blocks * 32;
    if (wgs > (int64_t)1 << 30 || (int64_t)pl.n_blocks * 32 > (int64_t)1 << 30)
        return fail(AHA_ERR_UNSUPPORTED, "problem exceeds the launch grid limits");
    const ScoreGeom g = make_geom(p, q, k, v);
    return hip_result(launch_window_attention(g, pl, workspace, out, lse, (hipStream_t)stream),
                      "window attention kernels");
}

int32_t aha_prefill_row_stats(const aha_params *p, const void *q, const void *k, float *lse,
                              float *entropy, void *workspace, size_t workspace_bytes,
                              void *stream) {
    int32_t rc = check_prefill(p, false);
    if (rc) return rc;
    if ((rc = check_stride("q", p->q_stride, p->dtype, p->head_dim)) ||
        (rc = check_stride("k", p->k_stride, p->dtype, p->head_dim)))
        return rc;
    if ((rc = check_ptr("q", q, 16)) || (rc = check_ptr("k", k, 16))) return rc;
    if (!lse && !entropy) return fail(AHA_ERR_INVALID_ARG, "lse and entropy are both null");
    if ((lse && (rc = check_ptr("lse", lse, 4))) || (entropy && (rc = check_ptr("entropy", entropy, 4))))
        return rc;
    const PrefillPlan pl = plan_prefill(p);
    if ((rc = check_ws(workspace, workspace_bytes, pl.bytes))) return rc;
    const int64_t score_wgs = (int64_t)pl.Z * ((pl.n_qtiles + 1) / 2) * pl.nchunks;
    if (score_wgs > (int64_t)1 << 30)
        return fail(AHA_ERR_UNSUPPORTED, "problem exceeds the launch grid limits");
    const ScoreGeom g = make_geom(p, q, k, nullptr);
    if (p->dtype == AHA_BF16)
        return hip_result(launch_row_stats_bf16(g, pl, workspace, lse, entropy, (hipStream_t)stream),
                          "bf16 row-statistics kernels");
    return hip_result(launch_row_stats_f32(g, pl, workspace, lse, entropy, (hipStream_t)stream),
                      "fp32 row-statistics kernel");
}

int32_t aha_select_topk(const aha_params *p, const float *scores, int32_t *idx, void *workspace,
                        size_t workspace_bytes, void *stream) {
    int32_t rc = check_prefill(p, false);
    if (rc) return rc;
    if ((rc = check_ptr("scores", scores, 4)) || (rc = check_ptr("idx", idx, 4))) return rc;
    const int pool = p->score_pool > 1 ? p->score_pool : 1;
    if (pool > 1 && (rc = check_ws(workspace, workspace_bytes, topk_ws_bytes(p)))) return rc;
    return hip_result(launch_topk(scores, p->batch * p->n_kv_heads, p->seq_len, p->budget,
                                  p->recent, p->sink, pool, (float *)workspace, idx,
                                  (hipStream_t)stream),
                      "top-k kernels");
}

int32_t aha_compact_kv(const aha_params *p, const void *k, const void *v, const float *scores,
                       const int32_t *idx, void *k_cache, void *v_cache, float *scores_c,
                       int32_t *pos_c, int32_t *free_slot, int32_t cache_slots, void *stream) {
    int32_t rc = check_compact(p);
    if (rc) return rc;
    if ((rc = check_ptr("k", k, 16)) || (rc = check_ptr("v", v, 16)) ||
        (rc = check_ptr("scores", scores, 4)) || (rc = check_ptr("idx", idx, 4)) ||
        (rc = check_ptr("k_cache", k_cache, 16)) || (rc = check_ptr("v_cache", v_cache, 16)) ||
        (rc = check_ptr("scores_c", scores_c, 4)) || (rc = check_ptr("pos_c", pos_c, 4)) ||
        (rc = check_ptr("free_slot", free_slot, 4)))
        return rc;
    if (cache_slots < p->budget + 1)
        return fail(AHA_ERR_INVALID_ARG, "cache_slots (%d) must be >= budget + 1 (%d)", cache_slots,
                    p->budget + 1);
    const ScoreGeom g = make_geom(p, nullptr, k, v);
    return hip_result(launch_compact(g, scores, idx, p->budget, cache_slots, p->dtype, k_cache,
                                     v_cache, scores_c, pos_c, free_slot, (hipStream_t)stream),
                      "compaction kernel");
}

// Host checks shared by aha_decode_step and its variant without a workspace argument
// (`scratch_limit` > 0: the scratch is the library's own and that many bytes long; the
// workspace arguments are then not looked at).  Nothing here touches the HIP runtime.
static int32_t decode_step_check(const aha_params *p, const void *q_new, const void *k_new,
                                 const void *v_new, void *k_cache, void *v_cache, float *scores_c,
                                 int32_t *pos_c, int32_t *free_slot, int32_t cache_slots,
                                 int32_t logical_pos, void *out, const void *workspace,
                                 size_t workspace_bytes, size_t scratch_limit, DecodePlan *plan) {
    int32_t rc = check_common(p);
    if (rc) return rc;
    if ((rc = check_ptr("q_new", q_new, 16)) || (rc = check_ptr("k_new", k_new, 16)) ||
        (rc = check_ptr("v_new", v_new, 16)) || (rc = check_ptr("k_cache", k_cache, 16)) ||
        (rc = check_ptr("v_cache", v_cache, 16)) || (rc = check_ptr("scores_c", scores_c, 4)) ||
        (rc = check_ptr("pos_c", pos_c, 4)) || (rc = check_ptr("free_slot", free_slot, 4)) ||
        (rc = check_ptr("out", out, 16)))
        return rc;
    if (cache_slots < p->budget + 1)
        return fail(AHA_ERR_INVALID_ARG, "cache_slots (%d) must be >= budget + 1 (%d)", cache_slots,
                    p->budget + 1);
    if (logical_pos < p->budget + 1)
        return fail(AHA_ERR_INVALID_ARG, "logical_pos (%d) must be >= budget + 1 (%d)", logical_pos,
                    p->budget + 1);
    const int G = p->n_q_heads / p->n_kv_heads;
    if (G > 8)
        return fail(AHA_ERR_UNSUPPORTED, "decode is built for query groups of up to 8 heads, not %d", G);
    *plan = plan_decode(p);
    if (!plan->fits)
        return fail(AHA_ERR_UNSUPPORTED,
                    "decode keeps group * (budget + 1) dots in LDS; %d * %d does not fit (%d splits)",
                    G, p->budget + 1, plan->nsplit);
    if (scratch_limit) {
        if (plan->bytes > scratch_limit)
            return fail(AHA_ERR_UNSUPPORTED,
                        "this shape needs %zu bytes of scratch, the built-in buffer holds %zu: use "
                        "aha_decode_step with a workspace", plan->bytes, scratch_limit);
        return AHA_OK;
    }
    return check_ws(workspace, workspace_bytes, plan->bytes);
}

static int32_t decode_step_launch(const aha_params *p, const DecodePlan &dpl, const void *q_new,
                                  const void *k_new, const void *v_new, void *k_cache,
                                  void *v_cache, float *scores_c, int32_t *pos_c,
                                  int32_t *free_slot, int32_t cache_slots, int32_t logical_pos,
                                  void *out, void *workspace, void *stream) {
    DecodeGeom g{};
    g.q = q_new; g.k_new = k_new; g.v_new = v_new; g.kc = k_cache; g.vc = v_cache; g.out = out;
    g.fc = scores_c; g.pos = pos_c; g.free_slot = free_slot;
    g.batch = p->batch; g.Hq = p->n_q_heads; g.Hkv = p->n_kv_heads; g.G = g.Hq / g.Hkv;
    g.d = p->head_dim;
    g.budget = p->budget; g.recent = p->recent; g.slots = cache_slots; g.logical_pos = logical_pos;
    g.scale_mode = p->scale_mode; g.fixed_scale = p->fixed_scale; g.lambda_floor = p->lambda_floor;
    g.sink = p->sink; g.value_prior = p->decode_value_prior;
    return hip_result(launch_decode(g, dpl, workspace, p->dtype, (hipStream_t)stream),
                      "decode kernel");
}

int32_t aha_decode_step(const aha_params *p, const void *q_new, const void *k_new,
                        const void *v_new, void *k_cache, void *v_cache, float *scores_c,
                        int32_t *pos_c, int32_t *free_slot, int32_t cache_slots,
                        int32_t logical_pos, void *out, void *workspace, size_t workspace_bytes,
                        void *stream) {
    DecodePlan dpl{};
    const int32_t rc = decode_step_check(p, q_new, k_new, v_new, k_cache, v_cache, scores_c, pos_c,
                                         free_slot, cache_slots, logical_pos, out, workspace,
                                         workspace_bytes, 0, &dpl);
    if (rc) return rc;
    return decode_step_launch(p, dpl, q_new, k_new, v_new, k_cache, v_cache, scores_c, pos_c,
                              free_slot, cache_slots, logical_pos, out, workspace, stream);
}

// ---- generation step without a workspace argument ----
// Scratch of the split decode path (raw dots and the splits' partial outputs) for callers
// that can neither allocate nor carry a workspace.  The array's name is only a host-side
// stand-in: its device address is asked for once per device (each GPU holds its own copy
// at its own address) and that pointer is what the kernels get.
constexpr size_t kScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static void *g_scratch_ptr[kMaxDevices];
static DeviceOnce g_scratch_once;

int32_t aha_decode_step_static(const aha_params *p, const void *q_new, const void *k_new,
                               const void *v_new, void *k_cache, void *v_cache, float *scores_c,
                               int32_t *pos_c, int32_t *free_slot, int32_t cache_slots,
                               int32_t logical_pos, void *out, void *stream) {
    DecodePlan dpl{};
    const int32_t rc = decode_step_check(p, q_new, k_new, v_new, k_cache, v_cache, scores_c, pos_c,
                                         free_slot, cache_slots, logical_pos, out, nullptr, 0,
                                         kScratchBytes, &dpl);
    if (rc) return rc;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_result(e, "hipGetDevice");
    e = device_once(g_scratch_once, [dev] {
        void *ptr = nullptr;
        const hipError_t es = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        g_scratch_ptr[dev] = es == hipSuccess ? ptr : nullptr;
        return es;
    });
    if (e != hipSuccess) return hip_result(e, "address of the built-in scratch buffer");
    // every value the kernels read from the scratch is written earlier in the same call:
    // nothing has to start from zero
    return decode_step_launch(p, dpl, q_new, k_new, v_new, k_cache, v_cache, scores_c, pos_c,
                              free_slot, cache_slots, logical_pos, out, g_scratch_ptr[dev], stream);
}

int32_t aha_profile_events(void *const *events, int32_t count) {
    if (count == 0 && !events) {
        g_stage_on = false;
        return AHA_OK;
    }
    if (count != 4 || !events) return fail(AHA_ERR_INVALID_ARG, "events must be NULL/0 or 4 handles");
    for (int i = 0; i < 4; ++i) {
        if (!events[i]) return fail(AHA_ERR_INVALID_ARG, "events[%d] is null", i);
        g_stage_ev[i] = (hipEvent_t)events[i];
    }
    g_stage_on = true;
    return AHA_OK;
}

const char *aha_last_error(void) { return g_err; }

const char *aha_version(void) { return "aha-gfx950 0.1"; }

}  // extern "C"

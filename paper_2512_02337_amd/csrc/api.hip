// C ABI of libspecpv: argument validation, workspace layout, split planning and
// the launch sequences of the four calls.  No kernels live here.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "internal.h"

namespace specpv {

static thread_local char g_hip_err[256] = "";

static int fail_hip(hipError_t e)
{
    snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
    return SPECPV_EHIP;
}

int device_cu_count()
{
    // per device, filled on first use; a racing first call writes the same value
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked) {
        const int c = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
        if (c > 0) return c;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
    if (tracked) __atomic_store_n(&cached[dev], cus, __ATOMIC_RELAXED);
    return cus;
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static int check_kv(const specpv_kv *kv)
{
    if (!kv || !kv->k || !kv->v || !kv->ctx_len) return SPECPV_EINVAL;
    if (kv->dtype != SPECPV_F32 && kv->dtype != SPECPV_BF16) return SPECPV_EINVAL;
    if (kv->head_dim != 64 && kv->head_dim != 128) return SPECPV_EINVAL;
    if (kv->batch < 1 || kv->n_kv_heads < 1 || kv->block_size < 1 || kv->max_blocks < 1) return SPECPV_EINVAL;
    const int64_t vec = kv->dtype == SPECPV_BF16 ? 8 : 4;  // elements per 16 bytes
    if (kv->stride_t < kv->head_dim || kv->stride_t % vec || kv->stride_h % vec || kv->stride_b % vec)
        return SPECPV_EINVAL;
    if (kv->stride_h < 0 || kv->stride_b < 0) return SPECPV_EINVAL;
    if (((uintptr_t)kv->k | (uintptr_t)kv->v) & 15) return SPECPV_EINVAL;
    if ((int64_t)kv->max_blocks * kv->block_size > ((int64_t)1 << 30)) return SPECPV_ELIMIT;
    return SPECPV_OK;
}

static int check_tree(const specpv_kv *kv, const specpv_tree *tree, bool need_draft_kv)
{
    if (!tree || !tree->q) return SPECPV_EINVAL;
    if (tree->M < 1 || tree->n_q_heads < 1) return SPECPV_EINVAL;
    if (tree->n_key_only < 0 || tree->n_key_only >= tree->M) return SPECPV_EINVAL;
    if (tree->n_q_heads % kv->n_kv_heads) return SPECPV_EINVAL;
    if (tree->M > SPECPV_MAX_M || tree->n_q_heads / kv->n_kv_heads > SPECPV_MAX_G) return SPECPV_ELIMIT;
    if ((uintptr_t)tree->q & 15) return SPECPV_EINVAL;
    if (need_draft_kv) {
        if (!tree->kd || !tree->vd || !tree->parent) return SPECPV_EINVAL;
        if (((uintptr_t)tree->kd | (uintptr_t)tree->vd) & 15) return SPECPV_EINVAL;
    }
    return SPECPV_OK;
}

static int check_cfg(const specpv_tree *tree, const specpv_select_cfg *cfg)
{
    if (!cfg) return SPECPV_EINVAL;
    if (cfg->n_sink_blocks < 0 || cfg->n_recent_blocks < 0 || cfg->k_blocks < 0) return SPECPV_EINVAL;
    if (cfg->reduce != SPECPV_REDUCE_MEAN && cfg->reduce != SPECPV_REDUCE_MAX && cfg->reduce != SPECPV_REDUCE_LAST)
        return SPECPV_EINVAL;
    if (cfg->reduce == SPECPV_REDUCE_LAST && (tree->last_node < tree->n_key_only || tree->last_node >= tree->M))
        return SPECPV_EINVAL;
    if (cfg->score != SPECPV_SCORE_EQ2 && cfg->score != SPECPV_SCORE_CHANNEL_BOUND) return SPECPV_EINVAL;
    if (cfg->n_extra_slots < 0) return SPECPV_EINVAL;
    if ((int64_t)cfg->n_sink_blocks + cfg->n_recent_blocks + cfg->k_blocks + cfg->n_extra_slots > ((int64_t)1 << 24))
        return SPECPV_ELIMIT;
    return SPECPV_OK;
}

static Shape make_shape(const specpv_kv *kv, const specpv_tree *tree)
{
    Shape s;
    memset(&s, 0, sizeof(s));
    s.k = kv->k; s.v = kv->v;
    s.sb = kv->stride_b; s.sh = kv->stride_h; s.st = kv->stride_t;
    s.ctx_len = kv->ctx_len;
    s.batch = kv->batch; s.Hkv = kv->n_kv_heads; s.D = kv->head_dim; s.B = kv->block_size;
    s.max_blocks = kv->max_blocks;
    if (tree) {
        s.q = tree->q; s.kd = tree->kd; s.vd = tree->vd; s.parent = tree->parent;
        s.Mk = tree->M; s.koff = tree->n_key_only; s.M = s.Mk - s.koff;
        s.Hq = tree->n_q_heads; s.G = s.Hq / s.Hkv;
    }
    return s;
}

// Which kernel the context part of the attention runs on and how many KV splits it uses when
// it covers n_blocks blocks per (sequence, KV head).  Host-only and deterministic in its
// arguments, so specpv_workspace_bytes and the calls agree.
static AttnPlan plan_attention(const Shape &s, int dtype, int64_t n_blocks)
{
    AttnPlan plan{1, attn_ctx_mfma_supported(s, dtype) ? kAttnSplit : kAttnGeneric};
    const int64_t tokens = n_blocks * s.B;
    if (tokens <= 0) return plan;
    if (plan.kind != kAttnGeneric) {
        const int64_t chunks = (tokens + 31) / 32;   // 32-token chunks per (sequence, KV head)
        const int64_t cus = device_cu_count();
        const int64_t row_tiles = (s.M + 63) / 64;
        // splits c that minimise the chunk-times on the critical path (one workgroup per CU, `base`
        // workgroups per split, `ranges` token ranges per workgroup), plus a charge for the
        // epilogue and the partials
        auto best_splits = [&](int64_t base, int64_t ranges, int64_t max_ns) {
            int64_t best = 1, best_cost = -1;
            for (int64_t c = 1; c <= max_ns; ++c) {
                const int64_t rounds = (base * c + cus - 1) / cus;
                const int64_t per_wave = (chunks + ranges * c - 1) / (ranges * c);
                const int64_t cost = rounds * (per_wave * 8 + 10) + c;
                if (best_cost < 0 || cost < best_cost) { best = c; best_cost = cost; }
            }
            return best;
        };
        // a workgroup per (sequence, query head, 64-node row tile, split), four token ranges each
        const int64_t max4 = chunks / 4 > 1 ? (chunks / 4 < 64 ? chunks / 4 : 64) : 1;
        int64_t ns = best_splits((int64_t)s.batch * s.Hq * row_tiles, 4, max4);
        // Long token ranges per wavefront amortise the longer prologue and epilogue of the kernels
        // with more rows per wavefront; at a handful of chunks the eight-wavefront kernel hides
        // latency better.
        if (chunks >= 8 * 4 * ns) {
            // a few workgroups per (sequence, KV head, split) that cover the group's query rows, one
            // token range each
            plan.kind = kAttnGroup;
            const int64_t max1 = chunks / 8 > 1 ? (chunks / 8 < 64 ? chunks / 8 : 64) : 1;
            const int64_t base1 = (int64_t)s.batch * s.Hkv * attn_group_parts(s);
            ns = best_splits(base1, 1, max1);
            if (s.batch > 1) {
                // The sequences of a batch may differ in length, and the lengths live on the device:
                // many small workgroups (about four per CU, 64 chunks or more each: shorter ones are
                // mostly prologue and epilogue) let the hardware scheduler even that out (measured on
                // 32K + 64K + 96K + 128K at G = 5: 1089 -> 841 us with eight workgroups of six wavefronts per
                // CU; with workgroups of ten, 752 us at eight per CU, 687 at four, 704 at two: every split
                // is another partial for the combine, 85 us at 64 splits against 37 at 32).
                int64_t c = (4 * cus + base1 - 1) / base1;
                if (c > max1) c = max1;
                while (c > ns && (chunks + c - 1) / c < 64) --c;
                if (c > ns) ns = c;
            }
        }
        plan.nsplit = (int)ns;
    } else {
        const int64_t rows = (int64_t)s.batch * s.Hq * s.M;
        const int64_t chunks = (tokens + 63) / 64;
        int64_t ns = (4096 + rows - 1) / rows;
        if (ns > chunks) ns = chunks;
        if (ns > 64) ns = 64;
        if (ns < 1) ns = 1;
        plan.nsplit = (int)ns;
    }
    return plan;
}

// Workspace layout: [arrival words, kArriveBytes, zero between calls][partial O][(m, l) pairs][scores],
// the partial arrays sized for nsplit + 1 slots (the context splits and the draft-tree segment).
struct Workspace {
    unsigned long long *arrive;
    float *part_o, *part_ml, *scores;
    size_t total;
};

static Workspace layout_workspace(const Shape &s, int nsplit, void *base)
{
    Workspace w;
    const size_t slots = (size_t)nsplit + 1;
    const size_t po = align_up((size_t)s.batch * s.Hq * slots * s.M * s.D * sizeof(float));
    const size_t pm = align_up((size_t)s.batch * s.Hq * slots * s.M * 2 * sizeof(float));
    const size_t sc = align_up((size_t)s.batch * s.Hkv * s.max_blocks * sizeof(float));
    char *p = (char *)base;
    w.arrive = (unsigned long long *)p;
    w.part_o = (float *)(p + kArriveBytes);
    w.part_ml = (float *)(p + kArriveBytes + po);
    w.scores = (float *)(p + kArriveBytes + po + pm);
    w.total = kArriveBytes + po + pm + sc;
    return w;
}

// Process-wide choice of how specpv_partial_verify_attn runs shapes that the eight-wavefront kernel
// takes (a testing aid, see specpv_debug_set_route).
static int g_route = 0;
static unsigned long long *g_timeline = nullptr;   // where instrumented builds (-DSPECPV_TIMELINE) put their time stamps

static int run_attention(const Shape &s_in, int dtype, const int32_t *sel_idx, const int32_t *sel_count,
                         int n_sel, void *out, float *lse, void *workspace, size_t workspace_bytes,
                         hipStream_t st)
{
    const AttnPlan plan = plan_attention(s_in, dtype, sel_idx ? n_sel : s_in.max_blocks);
    Shape s = s_in;
    // the matrix-core kernels take the partially verified tokens in front of the tree along with the cache
    // tokens (dense: every query row attends all of them); the vector-ALU kernel leaves them to the combine
    s.kctx = plan.kind != kAttnGeneric ? s.koff : 0;
    const int nsplit = plan.nsplit;
    const Workspace w = layout_workspace(s, nsplit, workspace);
    if (!workspace || workspace_bytes < w.total) return SPECPV_EWORKSPACE;
    const int route = __atomic_load_n(&g_route, __ATOMIC_RELAXED);
    // The single-kernel route is correct but measured slower than two launches (the last workgroup of a
    // tile reads all of the tile's partials through one CU): it runs only on request.
    const bool fused = plan.kind == kAttnSplit && route >= 2 && nsplit <= 64 &&
                       (size_t)s.batch * s.Hq * 2 * sizeof(unsigned long long) <= kArriveBytes;
    hipError_t e;
    if (fused) {
        Partials p{w.part_o, w.part_ml, nsplit + 1, 0, nullptr};
        const FusedArgs f{out, lse, w.arrive, route == 3 ? 1 : 0, g_timeline};
        e = launch_attn_ctx_mfma(s, sel_idx, sel_count, n_sel, p, nsplit, plan.kind, f, st);
        return e == hipSuccess ? SPECPV_OK : fail_hip(e);
    }
    Partials p{w.part_o, w.part_ml, nsplit, plan.kind != kAttnGeneric ? 1 : 0, g_timeline};
    const FusedArgs none{nullptr, nullptr, nullptr, 0, g_timeline};
    if (plan.kind != kAttnGeneric) e = launch_attn_ctx_mfma(s, sel_idx, sel_count, n_sel, p, nsplit, plan.kind, none, st);
    else e = launch_attn_ctx_generic(s, dtype, sel_idx, sel_count, n_sel, p, st);
    if (e != hipSuccess) return fail_hip(e);
    e = launch_combine(s, dtype, p, out, lse, st);
    if (e != hipSuccess) return fail_hip(e);
    return SPECPV_OK;
}

// Library-owned scratch for callers that cannot pass a workspace (specpv_partial_verify_attn_static).
// One copy per GPU, alive until the process ends.  In host code the array's name is only a handle:
// the device address comes from hipGetSymbolAddress, once per device, and is what the kernels get.
static __device__ __align__(256) unsigned char scratch[SPECPV_STATIC_SCRATCH_BYTES];

static hipError_t static_scratch(void **out)
{
    static void *ptr[64] = {};   // per device; a racing first call stores the same address
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    void *p = tracked ? __atomic_load_n(&ptr[dev], __ATOMIC_ACQUIRE) : nullptr;
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        if (tracked) __atomic_store_n(&ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return hipSuccess;
}

// Process-wide choice between one and two launches for scoring + selection (a testing aid, see
// specpv_debug_set_select_route).
static int g_select_route = 0;

// arrive: the zeroed arrival words at the head of a workspace, or nullptr where the caller gave none
static int run_select(const Shape &s, int dtype, const specpv_tree *tree, const void *kmax, const void *kmin,
                      const specpv_select_cfg *cfg, int32_t *sel_idx, int32_t *sel_count, float *scores,
                      unsigned long long *arrive, hipStream_t st)
{
    const int n_row = cfg->n_sink_blocks + cfg->k_blocks + cfg->n_recent_blocks + cfg->n_extra_slots;
    const TopkArgs sel{cfg->n_sink_blocks, cfg->n_recent_blocks, cfg->k_blocks, n_row, sel_idx, sel_count};
    // One launch (the last scoring workgroup of a (sequence, KV head) selects) only on request: it is the
    // slower of the two.  Measured per call at one 128K sequence 18.8 against 16.6 us, at 16K 11.0 against
    // 10.9, for a ragged batch of four 41.4 against 34.6: counting 64 workgroups in costs about what a launch
    // costs, and the last workgroup then starts its selection with cold reads like a fresh kernel would.
    const bool one = arrive && __atomic_load_n(&g_select_route, __ATOMIC_RELAXED) == 1 && score_select_supported(s, dtype);
    // the scoring kernels count query rows: node last_node is row last_node - n_key_only
    hipError_t e = launch_scores(s, dtype, kmax, kmin, (int)cfg->reduce, tree->last_node - tree->n_key_only,
                                 (int)cfg->score, scores, one ? &sel : nullptr, one ? arrive : nullptr, st);
    if (e != hipSuccess) return fail_hip(e);
    if (one) return SPECPV_OK;
    e = launch_topk(s, scores, sel.ns, sel.nr, sel.k, n_row, sel_idx, sel_count, st);
    if (e != hipSuccess) return fail_hip(e);
    return SPECPV_OK;
}

}  // namespace specpv

using namespace specpv;

extern "C" {

size_t specpv_workspace_bytes(const specpv_kv *kv, const specpv_tree *tree, const specpv_select_cfg *cfg)
{
    if (check_kv(kv) != SPECPV_OK) return 0;
    if (!tree) return kArriveBytes + align_up((size_t)kv->batch * sizeof(int32_t));
    if (check_tree(kv, tree, false) != SPECPV_OK) return 0;
    const Shape s = make_shape(kv, tree);
    int nsplit = plan_attention(s, kv->dtype, s.max_blocks).nsplit;
    if (cfg) {
        const int64_t n_sel = (int64_t)cfg->n_sink_blocks + cfg->k_blocks + cfg->n_recent_blocks + cfg->n_extra_slots;
        const int n2 = plan_attention(s, kv->dtype, n_sel).nsplit;
        if (n2 > nsplit) nsplit = n2;
    }
    return layout_workspace(s, nsplit, nullptr).total;
}

int specpv_block_summarize(const specpv_kv *kv, int32_t blk_begin, int32_t blk_end,
                           void *kmax, void *kmin, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if (!kmax || !kmin || blk_begin < 0) return SPECPV_EINVAL;
    if (((uintptr_t)kmax | (uintptr_t)kmin) & 15) return SPECPV_EINVAL;
    const Shape s = make_shape(kv, nullptr);
    const hipError_t e = launch_summarize(s, kv->dtype, blk_begin, blk_end, kmax, kmin, (hipStream_t)stream);
    return e == hipSuccess ? SPECPV_OK : fail_hip(e);
}

int specpv_select_blocks(const specpv_kv *kv, const specpv_tree *tree, const void *kmax, const void *kmin,
                         const specpv_select_cfg *cfg, int32_t *sel_idx, int32_t *sel_count, float *scores,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if ((rc = check_tree(kv, tree, false)) != SPECPV_OK) return rc;
    if ((rc = check_cfg(tree, cfg)) != SPECPV_OK) return rc;
    if (!kmax || !kmin || !sel_idx || !sel_count) return SPECPV_EINVAL;
    if (((uintptr_t)kmax | (uintptr_t)kmin) & 15) return SPECPV_EINVAL;
    const Shape s = make_shape(kv, tree);
    if (!scores) {
        // behind the arrival words
        const size_t need = kArriveBytes + align_up((size_t)s.batch * s.Hkv * s.max_blocks * sizeof(float));
        if (!workspace || workspace_bytes < need) return SPECPV_EWORKSPACE;
        scores = (float *)((char *)workspace + kArriveBytes);
    }
    unsigned long long *arrive = workspace && workspace_bytes >= kArriveBytes ? (unsigned long long *)workspace : nullptr;
    return run_select(s, kv->dtype, tree, kmax, kmin, cfg, sel_idx, sel_count, scores, arrive, (hipStream_t)stream);
}

int specpv_partial_verify_attn(const specpv_kv *kv, const specpv_tree *tree, const int32_t *sel_idx,
                               const int32_t *sel_count, int32_t n_sel, void *out, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if ((rc = check_tree(kv, tree, true)) != SPECPV_OK) return rc;
    if (!out || ((uintptr_t)out & 15)) return SPECPV_EINVAL;
    if (sel_idx && (!sel_count || n_sel < 0)) return SPECPV_EINVAL;
    if (sel_idx && n_sel > (1 << 24)) return SPECPV_ELIMIT;
    const Shape s = make_shape(kv, tree);
    return run_attention(s, kv->dtype, sel_idx, sel_count, n_sel, out, lse, workspace, workspace_bytes,
                         (hipStream_t)stream);
}

int specpv_partial_verify_attn_static(const specpv_kv *kv, const specpv_tree *tree, const int32_t *sel_idx,
                                      const int32_t *sel_count, int32_t n_sel, void *out, float *lse, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if ((rc = check_tree(kv, tree, true)) != SPECPV_OK) return rc;
    if (!out || ((uintptr_t)out & 15)) return SPECPV_EINVAL;
    if (sel_idx && (!sel_count || n_sel < 0)) return SPECPV_EINVAL;
    if (sel_idx && n_sel > (1 << 24)) return SPECPV_ELIMIT;
    const Shape s = make_shape(kv, tree);
    // the same plan as specpv_partial_verify_attn; its partial results must fit the static array
    const AttnPlan plan = plan_attention(s, kv->dtype, sel_idx ? n_sel : s.max_blocks);
    if (layout_workspace(s, plan.nsplit, nullptr).total > (size_t)SPECPV_STATIC_SCRATCH_BYTES) {
        snprintf(g_hip_err, sizeof(g_hip_err), "static scratch: the call needs %zu bytes, the array holds %zu",
                 layout_workspace(s, plan.nsplit, nullptr).total, (size_t)SPECPV_STATIC_SCRATCH_BYTES);
        return SPECPV_ELIMIT;
    }
    void *ws = nullptr;
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return fail_hip(e);
    return run_attention(s, kv->dtype, sel_idx, sel_count, n_sel, out, lse, ws, (size_t)SPECPV_STATIC_SCRATCH_BYTES,
                         (hipStream_t)stream);
}

int specpv_full_verify_refresh(const specpv_kv *kv, const specpv_tree *tree, void *kmax, void *kmin,
                               int32_t stale_blk_begin, const specpv_select_cfg *cfg, void *out, float *lse,
                               int32_t *sel_idx, int32_t *sel_count, float *scores,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if ((rc = check_tree(kv, tree, true)) != SPECPV_OK) return rc;
    if ((rc = check_cfg(tree, cfg)) != SPECPV_OK) return rc;
    if (!kmax || !kmin || !out || !sel_idx || !sel_count) return SPECPV_EINVAL;
    if (((uintptr_t)kmax | (uintptr_t)kmin | (uintptr_t)out) & 15) return SPECPV_EINVAL;
    const Shape s = make_shape(kv, tree);
    const int nsplit = plan_attention(s, kv->dtype, s.max_blocks).nsplit;
    const Workspace w = layout_workspace(s, nsplit, workspace);
    if (!workspace || workspace_bytes < w.total) return SPECPV_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (stale_blk_begin >= 0) {
        const hipError_t e = launch_summarize(s, kv->dtype, stale_blk_begin, -1, kmax, kmin, st);
        if (e != hipSuccess) return fail_hip(e);
    }
    rc = run_attention(s, kv->dtype, nullptr, nullptr, 0, out, lse, workspace, workspace_bytes, st);
    if (rc != SPECPV_OK) return rc;
    return run_select(s, kv->dtype, tree, kmax, kmin, cfg, sel_idx, sel_count, scores ? scores : w.scores, w.arrive, st);
}

int specpv_gather_blocks(const specpv_kv *kv, const int32_t *sel_idx, const int32_t *sel_count, int32_t n_sel,
                         void *out_k, void *out_v, int32_t *out_len, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if (!sel_idx || !sel_count || !out_k || !out_v || n_sel < 1) return SPECPV_EINVAL;
    if (((uintptr_t)out_k | (uintptr_t)out_v) & 15) return SPECPV_EINVAL;
    if (n_sel > (1 << 24) || (int64_t)n_sel * kv->block_size > ((int64_t)1 << 30)) return SPECPV_ELIMIT;
    if (kv->batch > 65535 || kv->n_kv_heads > 65535) return SPECPV_ELIMIT;   // grid limits, before anything is enqueued
    const Shape s = make_shape(kv, nullptr);
    const hipError_t e = launch_gather(s, kv->dtype, sel_idx, sel_count, n_sel, out_k, out_v, out_len, (hipStream_t)stream);
    return e == hipSuccess ? SPECPV_OK : fail_hip(e);
}

int specpv_select_mode(const specpv_policy *policy, int64_t seq_len, int32_t partial_ready, int32_t n_pending)
{
    if (!policy || policy->partial_budget_tokens < 0 || policy->pending_margin_tokens < 0 || seq_len < 0 || n_pending < 0)
        return SPECPV_EINVAL;
    if (seq_len <= policy->partial_budget_tokens) return SPECPV_MODE_FULL;
    if (!partial_ready) return SPECPV_MODE_FULL;
    if (n_pending > policy->pending_margin_tokens) return SPECPV_MODE_REFRESH;
    return SPECPV_MODE_PARTIAL;
}

int specpv_extend_parents(const int32_t *tree_parent, int32_t M_tree, int32_t n_pending, int32_t *out)
{
    if (!tree_parent || !out || M_tree < 1 || n_pending < 0) return SPECPV_EINVAL;
    if ((int64_t)M_tree + n_pending > SPECPV_MAX_M) return SPECPV_ELIMIT;
    for (int32_t i = 0; i < n_pending; ++i) out[i] = i - 1;
    for (int32_t j = 0; j < M_tree; ++j) {
        if (tree_parent[j] >= j) return SPECPV_EINVAL;
        out[n_pending + j] = tree_parent[j] < 0 ? n_pending - 1 : tree_parent[j] + n_pending;
    }
    return SPECPV_OK;
}

int specpv_commit_accepted(const specpv_kv *kv, void *buf_k, void *buf_v, int32_t pending_cap, int32_t M_tree,
                           int32_t *n_pending, const int32_t *accepted, const int32_t *n_accepted,
                           int32_t max_accept, specpv_mode mode, void *kmax, void *kmin,
                           const specpv_lists *lists, int32_t *dropped,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_kv(kv);
    if (rc != SPECPV_OK) return rc;
    if (!buf_k || !buf_v || !n_pending || !accepted || !n_accepted) return SPECPV_EINVAL;
    if (lists && (!lists->sel_idx || !lists->sel_count || lists->n_sel < 1)) return SPECPV_EINVAL;
    if (lists && lists->n_sel > (1 << 24)) return SPECPV_ELIMIT;
    if (pending_cap < 0 || M_tree < 1 || max_accept < 1) return SPECPV_EINVAL;
    if (mode != SPECPV_MODE_FULL && mode != SPECPV_MODE_PARTIAL && mode != SPECPV_MODE_REFRESH) return SPECPV_EINVAL;
    if (((uintptr_t)buf_k | (uintptr_t)buf_v) & 15) return SPECPV_EINVAL;
    if ((kmax || kmin) && (!kmax || !kmin || (((uintptr_t)kmax | (uintptr_t)kmin) & 15))) return SPECPV_EINVAL;
    if ((int64_t)pending_cap + max_accept > 128 || (int64_t)pending_cap + M_tree > SPECPV_MAX_M) return SPECPV_ELIMIT;
    if (!workspace || workspace_bytes < kArriveBytes + (size_t)kv->batch * sizeof(int32_t)) return SPECPV_EWORKSPACE;
    workspace = (char *)workspace + kArriveBytes;   // the arrival words stay zero
    const Shape s = make_shape(kv, nullptr);
    void *k1 = const_cast<void *>(kv->k), *v1 = const_cast<void *>(kv->v);
    const hipError_t e = launch_commit(s, kv->dtype, 1, &k1, &v1, &buf_k, &buf_v, pending_cap, M_tree, n_pending, accepted,
                                       n_accepted, max_accept, mode != SPECPV_MODE_PARTIAL, &kmax, &kmin,
                                       lists, dropped, (int32_t *)workspace, (hipStream_t)stream);
    return e == hipSuccess ? SPECPV_OK : fail_hip(e);
}

int specpv_commit_accepted_layers(const specpv_kv *const *kv, void *const *buf_k, void *const *buf_v, int32_t n_layers,
                                  int32_t pending_cap, int32_t M_tree, int32_t *n_pending, const int32_t *accepted,
                                  const int32_t *n_accepted, int32_t max_accept, specpv_mode mode,
                                  void *const *kmax, void *const *kmin, const specpv_lists *lists, int32_t *dropped,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!kv || !buf_k || !buf_v || n_layers < 1 || n_layers > SPECPV_MAX_LAYERS) return SPECPV_EINVAL;
    if (!n_pending || !accepted || !n_accepted) return SPECPV_EINVAL;
    if (pending_cap < 0 || M_tree < 1 || max_accept < 1) return SPECPV_EINVAL;
    if (mode != SPECPV_MODE_FULL && mode != SPECPV_MODE_PARTIAL && mode != SPECPV_MODE_REFRESH) return SPECPV_EINVAL;
    if ((int64_t)pending_cap + max_accept > 128 || (int64_t)pending_cap + M_tree > SPECPV_MAX_M) return SPECPV_ELIMIT;
    if ((kmax == nullptr) != (kmin == nullptr)) return SPECPV_EINVAL;
    void *kp[SPECPV_MAX_LAYERS], *vp[SPECPV_MAX_LAYERS];
    for (int l = 0; l < n_layers; ++l) {
        const specpv_kv *x = kv[l];
        const int rc = check_kv(x);
        if (rc != SPECPV_OK) return rc;
        // one shape, one set of strides, one dtype and the same length counters for all layers
        if (x->batch != kv[0]->batch || x->n_kv_heads != kv[0]->n_kv_heads || x->head_dim != kv[0]->head_dim ||
            x->block_size != kv[0]->block_size || x->max_blocks != kv[0]->max_blocks || x->dtype != kv[0]->dtype ||
            x->stride_b != kv[0]->stride_b || x->stride_h != kv[0]->stride_h || x->stride_t != kv[0]->stride_t ||
            x->ctx_len != kv[0]->ctx_len)
            return SPECPV_EINVAL;
        if (!buf_k[l] || !buf_v[l] || (((uintptr_t)buf_k[l] | (uintptr_t)buf_v[l]) & 15)) return SPECPV_EINVAL;
        if (kmax) {   // summaries for every layer or for none
            const bool want = kmax[0] != nullptr;
            if ((kmax[l] != nullptr) != want || (kmin[l] != nullptr) != want) return SPECPV_EINVAL;
            if (((uintptr_t)kmax[l] | (uintptr_t)kmin[l]) & 15) return SPECPV_EINVAL;
        }
        if (lists) {
            if (!lists[l].sel_idx || !lists[l].sel_count || lists[l].n_sel < 1 || lists[l].n_sel != lists[0].n_sel)
                return SPECPV_EINVAL;
            if (lists[l].n_sel > (1 << 24)) return SPECPV_ELIMIT;
        }
        kp[l] = const_cast<void *>(x->k);
        vp[l] = const_cast<void *>(x->v);
    }
    if (!workspace || workspace_bytes < kArriveBytes + (size_t)kv[0]->batch * sizeof(int32_t)) return SPECPV_EWORKSPACE;
    workspace = (char *)workspace + kArriveBytes;   // the arrival words stay zero
    const Shape s = make_shape(kv[0], nullptr);
    const hipError_t e = launch_commit(s, kv[0]->dtype, n_layers, kp, vp, buf_k, buf_v, pending_cap, M_tree, n_pending,
                                       accepted, n_accepted, max_accept, mode != SPECPV_MODE_PARTIAL, kmax, kmin,
                                       lists, dropped, (int32_t *)workspace, (hipStream_t)stream);
    return e == hipSuccess ? SPECPV_OK : fail_hip(e);
}

const char *specpv_strerror(int status)
{
    switch (status) {
    case SPECPV_OK: return "ok";
    case SPECPV_EINVAL: return "invalid argument (null pointer, shape, dtype, head dim, stride or alignment)";
    case SPECPV_EWORKSPACE: return "workspace missing or too small (see specpv_workspace_bytes)";
    case SPECPV_ELIMIT: return "size beyond the documented limits";
    case SPECPV_EHIP: return "HIP launch failed (see specpv_last_hip_error)";
    default: return "unknown status";
    }
}

const char *specpv_last_hip_error(void) { return g_hip_err; }

int specpv_debug_set_timeline(void *buf)
{
#ifndef SPECPV_TIMELINE
    if (buf) return SPECPV_EINVAL;   // this build takes no time stamps
#endif
    g_timeline = (unsigned long long *)buf;
    return SPECPV_OK;
}

int specpv_debug_set_route(int route)
{
    if (route < 0 || route > 3) return SPECPV_EINVAL;
    __atomic_store_n(&g_route, route, __ATOMIC_RELAXED);
    return SPECPV_OK;
}

int specpv_debug_set_select_route(int route)
{
    if (route < 0 || route > 2) return SPECPV_EINVAL;
    __atomic_store_n(&g_select_route, route, __ATOMIC_RELAXED);
    return SPECPV_OK;
}

int specpv_version(void) { return 202; }

}  // extern "C"

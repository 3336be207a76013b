// C ABI of the IST library: host-side plan, argument checks and kernel sequencing.
// See include/ist.h for the contract of every entry point.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "ist_internal.h"

namespace ist {
hipError_t launch_perm_check(const int32_t *perm, const int32_t *invpos, int64_t N, int32_t *err,
                             hipStream_t st);
}

using namespace ist;

namespace {

ist_status fail(ist_ctx *ctx, ist_status st, const std::string &msg)
{
    if (ctx) ctx->err = msg;
    return st;
}

ist_status hip_fail(ist_ctx *ctx, hipError_t e, const char *where)
{
    return fail(ctx, IST_EHIP, std::string(where) + ": " + hipGetErrorString(e));
}

#define IST_HIP(call, where)                                   \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, where); \
    } while (0)

}  // namespace
namespace ist {
thread_local KernelTag g_tag = {};
void tag_kernel(const char *label, double flops, double bytes)
{
    snprintf(g_tag.kernel, sizeof(g_tag.kernel), "%s", label);
    g_tag.flops = flops; g_tag.bytes = bytes;
}
}  // namespace ist
namespace {

const char *kClassNames[KC_COUNT] = {
    "perm_tables", "partition_copy", "merge_copy", "bias_copy", "gemm_forward", "gemm_backward_data",
    "gemm_update", "softmax_xent", "loss_reduce", "bias_update", "csr_forward", "csr_update", "norm", "resample_copy"};

hipEvent_t prof_event(ist_ctx *ctx)
{
    if (!ctx->prof_free.empty()) {
        hipEvent_t e = ctx->prof_free.back();
        ctx->prof_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void prof_begin(ist_ctx *ctx, int cls, hipStream_t st)
{
    if (!ctx->prof_on) return;
    ist_ctx::ProfRec r{};
    r.cls = cls; r.start = prof_event(ctx); r.stop = prof_event(ctx);
    if (!r.start || !r.stop) return;
    g_tag.kernel[0] = 0; g_tag.flops = 0.0; g_tag.bytes = 0.0;
    (void)hipEventRecord(r.start, st);
    ctx->prof_recs.push_back(r);
}

void prof_end(ist_ctx *ctx, hipStream_t st)
{
    if (!ctx->prof_on || ctx->prof_recs.empty()) return;
    ist_ctx::ProfRec &r = ctx->prof_recs.back();
    (void)hipEventRecord(r.stop, st);
    snprintf(r.kernel, sizeof(r.kernel), "%s", g_tag.kernel[0] ? g_tag.kernel : kClassNames[r.cls]);
    r.flops = g_tag.flops; r.bytes = g_tag.bytes;
}

// launch one kernel class, bracketed by events when profiling is on
#define IST_RUN(cls, call, where)                              \
    do {                                                       \
        prof_begin(ctx, cls, st);                              \
        hipError_t e_ = (call);                                \
        prof_end(ctx, st);                                     \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, where); \
    } while (0)

inline void set_split(const ist_ctx *ctx, GemmArgs &a)
{
    a.partial = ctx->partial_bytes ? reinterpret_cast<float *>(ctx->workspace + ctx->off_partial) : nullptr;
    a.partial_bytes = ctx->partial_bytes;
    a.zeros = ctx->workspace + ctx->off_zeros;
}

inline const int32_t *tbl(const char *base, size_t off)
{
    return reinterpret_cast<const int32_t *>(base + off);
}

// Arguments of the block copy of layer l (1-based) between `params` and a subnet buffer.
CopyArgs copy_args(const ist_ctx *ctx, char *base, int l, void *Wfull)
{
    const LayerPlan &L = ctx->layer[l - 1];
    CopyArgs a{};
    a.W = Wfull;
    a.ld = L.N_in;
    a.sub = base + L.off_W;
    a.rows = L.row_part ? tbl(base, ctx->hidden[l - 1].off_sorted) : nullptr;
    a.cols = L.col_part ? tbl(base, ctx->hidden[l - 2].off_sorted) : nullptr;
    a.slotr = L.row_part ? tbl(base, ctx->hidden[l - 1].off_slot) : nullptr;
    a.slotc = L.col_part ? tbl(base, ctx->hidden[l - 2].off_slot) : nullptr;
    a.maskc = L.col_part ? reinterpret_cast<const uint32_t *>(base + ctx->hidden[l - 2].off_mask) : nullptr;
    a.rankc = L.col_part ? tbl(base, ctx->hidden[l - 2].off_rank) : nullptr;
    a.wordsc = L.col_part ? ctx->hidden[l - 2].words : 0;
    a.nr = L.R;
    a.nc = L.C;
    a.N_out = L.N_out;
    a.N_in = L.N_in;
    a.G = ctx->S;
    a.esz = ctx->esz();
    a.transposed = L.transposed;
    return a;
}

}  // namespace

extern "C" {

const char *ist_version(void) { return "ist-gfx950 0.1"; }

const char *ist_last_error(const ist_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

ist_status ist_create(const ist_model_desc *d, int32_t max_B, ist_ctx **out)
{
    if (!d || !out || !d->dims) return IST_EINVAL;
    *out = nullptr;
    if (d->t < 2 || d->S < 1 || (d->dtype != IST_F32 && d->dtype != IST_BF16) ||
        (d->input != IST_DENSE && d->input != IST_CSR) || (d->has_bias != 0 && d->has_bias != 1) ||
        (d->normalize != 0 && d->normalize != 1) || !(d->norm_eps == d->norm_eps))
        return IST_EINVAL;
    if (d->layer_scale)
        for (int l = 0; l < d->t; ++l)
            if (!(d->layer_scale[l] > 0.0f) || !(d->layer_scale[l] <= 3.0e38f)) return IST_EINVAL;
    if (max_B < 1) return IST_ESHAPE;
    if (d->S > 4096) return IST_EUNSUPPORTED;   // the output-bias mean is a two-level tree of 64
    for (int l = 0; l <= d->t; ++l) {
        if (d->dims[l] < 1 || d->dims[l] > 0x7fffffffLL) return IST_ESHAPE;
        if (l > 0 && l < d->t && d->dims[l] < d->S) return IST_ESHAPE;   // every subnet owns at least one neuron
    }
    ist_ctx *ctx = new (std::nothrow) ist_ctx();
    if (!ctx) return IST_ENOMEM;
    ctx->t = d->t; ctx->S = d->S; ctx->dtype = d->dtype; ctx->input = d->input;
    ctx->has_bias = d->has_bias; ctx->max_B = max_B;
    ctx->normalize = d->normalize; ctx->norm_eps = d->norm_eps > 0.0f ? d->norm_eps : 1e-5f;
    ctx->dims.assign(d->dims, d->dims + d->t + 1);
    ctx->scale.assign((size_t)d->t, 1.0f);
    if (d->layer_scale) ctx->scale.assign(d->layer_scale, d->layer_scale + d->t);
    const int t = d->t, S = d->S, e = ctx->esz();

    // ---- subnet buffer: index tables, then per-layer blocks and biases ----
    size_t off = 0;
    ctx->hidden.resize(t - 1);
    for (int l = 1; l < t; ++l) {
        HiddenPlan &h = ctx->hidden[l - 1];
        h.N = ctx->dims[l];
        h.w = (h.N + S - 1) / S;
        h.off_sorted = off; off = align_up(off + sizeof(int32_t) * h.w * S);
        h.off_slot = off;   off = align_up(off + sizeof(int32_t) * h.N);
        h.off_p2q = off;    off = align_up(off + sizeof(int32_t) * h.N);
        h.words = (h.N + 31) / 32;
        h.off_mask = off;   off = align_up(off + sizeof(uint32_t) * S * h.words);
        h.off_rank = off;   off = align_up(off + sizeof(int32_t) * S * h.words);
    }
    const size_t tables_end = off;
    ctx->layer.resize(t);
    for (int l = 1; l <= t; ++l) {
        LayerPlan &L = ctx->layer[l - 1];
        L.N_out = ctx->dims[l]; L.N_in = ctx->dims[l - 1];
        L.row_part = l < t; L.col_part = l > 1;
        L.R = L.row_part ? ctx->hidden[l - 1].w : L.N_out;   // packed widths (the widest block's)
        L.C = L.col_part ? ctx->hidden[l - 2].w : L.N_in;
        L.transposed = (l == 1 && d->input == IST_CSR);
        L.ldr = (L.R + 7) / 8 * 8;
        L.off_W = off; off = align_up(off + (size_t)S * L.R * L.C * e);
        L.off_b = off; off = align_up(off + (size_t)S * L.R * e);
    }
    ctx->subnets_bytes = off;
    (void)tables_end;

    // ---- workspace ----
    // Output layers wider than 4096 classes use the two-pass cross-entropy that recomputes the
    // logits instead of storing them (B x N_t fp32 per subnet would dominate HBM traffic).
    ctx->fused_out = ctx->dims[t] > 4096;
    // a wide bf16 output layer behind a narrow hidden layer takes the two fused persistent launches of
    // ist_wideout.hip: dz_t then only ever exists tile by tile in LDS
    ctx->wide_out = ctx->fused_out && !ctx->layer[t - 1].transposed &&
                    wide_out_supported(ctx->dtype, max_B, ctx->layer[t - 1].C, ctx->dims[t]);
    size_t w = 0;
    for (int l = 1; l < t; ++l) {
        ctx->hidden[l - 1].off_invpos = w;
        w = align_up(w + sizeof(int32_t) * ctx->hidden[l - 1].N);
    }
    for (int l = 1; l <= t; ++l) {
        LayerPlan &L = ctx->layer[l - 1];
        size_t act_e = (l == t) ? sizeof(float) : (size_t)e;
        if (l == t && ctx->fused_out) act_e = 0;   // logits of a wide output layer are never stored
        L.off_act = w; w = align_up(w + (size_t)S * max_B * L.ldr * act_e);
        // the dz of a wide output layer is kept transposed, [S][N_t][max_B rounded up to 8]
        const size_t dz_elems = (l == t && ctx->wide_out) ? 0
                              : (l == t && ctx->fused_out) ? (size_t)S * L.R * ((max_B + 7) / 8 * 8) : (size_t)S * max_B * L.ldr;
        L.off_dz = w;  w = align_up(w + dz_elems * e);
        if (ctx->normalize && l < t) {
            L.off_z = w;   w = align_up(w + (size_t)S * max_B * L.ldr * sizeof(float));
            L.off_zh = w;  w = align_up(w + (size_t)S * max_B * L.ldr * e);
            L.off_isg = w; w = align_up(w + (size_t)S * L.ldr * sizeof(float));
        }
    }
    if (ctx->fused_out) {
        ctx->nb_max = (int32_t)((ctx->dims[t] + 31) / 32);
        const size_t rows = (size_t)S * max_B;
        ctx->off_pmax = w; w = align_up(w + sizeof(float) * rows * ctx->nb_max);
        ctx->off_psum = w; w = align_up(w + sizeof(float) * rows * ctx->nb_max);
        ctx->off_qmax = w; w = align_up(w + sizeof(float) * rows * kLseChunksHost);
        ctx->off_qsum = w; w = align_up(w + sizeof(float) * rows * kLseChunksHost);
        ctx->off_zlabel = w; w = align_up(w + sizeof(float) * rows);
        ctx->off_lse = w; w = align_up(w + sizeof(float) * rows);
        // bias gradient of the output layer as partial sums per class and block of >= 32 samples
        if (ctx->has_bias && !ctx->wide_out)
            { ctx->off_rsum = w; w = align_up(w + sizeof(float) * (size_t)S * ((max_B + 31) / 32) * ctx->dims[t]); }
    }
    ctx->off_zeros = w; w = align_up(w + 256);   // stays zero: source of out-of-range operand chunks
    ctx->off_rowloss = w; w = align_up(w + sizeof(float) * (size_t)kLossSlots * S * max_B);
    ctx->off_bitmap = w;
    if (d->input == IST_CSR)   // per (subnet, input column): one bit per sample, then one 64-bit "first occurrence" word
        w = align_up(w + csr_scratch_bytes(S, ctx->dims[0], max_B));
    ctx->off_err = w; w = align_up(w + sizeof(int32_t));
    // split-K scratch: the largest partial buffer any forward / backward-data product needs
    size_t pmax = 0;
    for (int l = 1; l <= t; ++l) {
        const LayerPlan &L = ctx->layer[l - 1];
        if (L.transposed) continue;
        SplitPlan f = plan_gemm(max_B, (int32_t)L.R, (int32_t)L.C, S, true, e);
        if (f.splits > 1) pmax = std::max(pmax, (size_t)S * f.splits * max_B * L.R * sizeof(float));
        if (l > 1) {
            SplitPlan b = plan_gemm(max_B, (int32_t)L.C, (int32_t)L.R, S, true, e);
            if (b.splits > 1) pmax = std::max(pmax, (size_t)S * b.splits * max_B * L.C * sizeof(float));
        }
    }
    // the workgroups of the fused wide-output launches leave their shares of dh in the same scratch
    if (ctx->wide_out) {
        ctx->wide_nb = wide_out_workgroups(S);
        pmax = std::max(pmax, (size_t)S * ctx->wide_nb * max_B * ctx->layer[t - 1].C * sizeof(float));
    }
    ctx->off_partial = w; ctx->partial_bytes = pmax; w = align_up(w + pmax);
    ctx->workspace_bytes = w;
    *out = ctx;
    return IST_OK;
}

ist_status ist_destroy(ist_ctx *ctx)
{
    if (ctx) {
        for (auto &r : ctx->prof_recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
        for (auto e : ctx->prof_free) (void)hipEventDestroy(e);
    }
    delete ctx;
    return IST_OK;
}

int32_t ist_profile_classes(void) { return KC_COUNT; }

const char *ist_profile_class_name(int32_t c) { return (c >= 0 && c < KC_COUNT) ? kClassNames[c] : ""; }

ist_status ist_profile_enable(ist_ctx *ctx, int32_t on)
{
    if (!ctx) return IST_EINVAL;
    ctx->prof_on = on != 0;
    return IST_OK;
}

ist_status ist_profile_reset(ist_ctx *ctx)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->prof_recs.empty()) IST_HIP(hipEventSynchronize(ctx->prof_recs.back().stop), "profile reset");
    for (auto &r : ctx->prof_recs) { ctx->prof_free.push_back(r.start); ctx->prof_free.push_back(r.stop); }
    ctx->prof_recs.clear();
    return IST_OK;
}

ist_status ist_profile_read(ist_ctx *ctx, int32_t cls, double *total_ms, int64_t *launches)
{
    if (!ctx || !total_ms || !launches || cls < 0 || cls >= KC_COUNT) return IST_EINVAL;
    double tot = 0.0;
    int64_t n = 0;
    if (!ctx->prof_recs.empty()) IST_HIP(hipEventSynchronize(ctx->prof_recs.back().stop), "profile read");
    for (auto &r : ctx->prof_recs) {
        if (r.cls != cls) continue;
        float ms = 0.0f;
        IST_HIP(hipEventElapsedTime(&ms, r.start, r.stop), "profile read");
        tot += ms;
        ++n;
    }
    *total_ms = tot;
    *launches = n;
    return IST_OK;
}

// Per-kernel view of the same records: launches grouped by kernel label.
namespace {
struct KernelAgg { std::string label; int cls; double ms, flops, bytes; int64_t n; };
ist_status aggregate(ist_ctx *ctx, std::vector<KernelAgg> &out)
{
    if (!ctx->prof_recs.empty()) IST_HIP(hipEventSynchronize(ctx->prof_recs.back().stop), "profile read");
    for (auto &r : ctx->prof_recs) {
        float ms = 0.0f;
        IST_HIP(hipEventElapsedTime(&ms, r.start, r.stop), "profile read");
        KernelAgg *k = nullptr;
        for (auto &a : out) if (a.cls == r.cls && a.label == r.kernel) { k = &a; break; }
        if (!k) { out.push_back(KernelAgg{r.kernel, r.cls, 0.0, 0.0, 0.0, 0}); k = &out.back(); }
        k->ms += ms; k->flops += r.flops; k->bytes += r.bytes; ++k->n;
    }
    return IST_OK;
}
}  // namespace

ist_status ist_profile_kernel_count(ist_ctx *ctx, int32_t *count)
{
    if (!ctx || !count) return IST_EINVAL;
    std::vector<KernelAgg> agg;
    const ist_status s = aggregate(ctx, agg);
    if (s != IST_OK) return s;
    *count = (int32_t)agg.size();
    return IST_OK;
}

ist_status ist_profile_kernel(ist_ctx *ctx, int32_t index, char *label, size_t label_cap, int32_t *kernel_class,
                              double *total_ms, int64_t *launches, double *flops, double *bytes)
{
    if (!ctx || !label || label_cap == 0 || !kernel_class || !total_ms || !launches || !flops || !bytes) return IST_EINVAL;
    std::vector<KernelAgg> agg;
    const ist_status s = aggregate(ctx, agg);
    if (s != IST_OK) return s;
    if (index < 0 || index >= (int32_t)agg.size()) return IST_EINVAL;
    const KernelAgg &k = agg[index];
    snprintf(label, label_cap, "%s", k.label.c_str());
    *kernel_class = k.cls; *total_ms = k.ms; *launches = k.n; *flops = k.flops; *bytes = k.bytes;
    return IST_OK;
}

ist_status ist_subnets_bytes(const ist_ctx *ctx, size_t *bytes)
{
    if (!ctx || !bytes) return IST_EINVAL;
    *bytes = ctx->subnets_bytes;
    return IST_OK;
}

ist_status ist_workspace_bytes(const ist_ctx *ctx, size_t *bytes)
{
    if (!ctx || !bytes) return IST_EINVAL;
    *bytes = ctx->workspace_bytes;
    return IST_OK;
}

ist_status ist_bind(ist_ctx *ctx, void *subnets, size_t sb, void *workspace, size_t wb)
{
    if (!ctx) return IST_EINVAL;
    if (!subnets || !workspace) return fail(ctx, IST_EINVAL, "ist_bind: null buffer");
    if (sb < ctx->subnets_bytes || wb < ctx->workspace_bytes)
        return fail(ctx, IST_ENOMEM, "ist_bind: buffer smaller than ist_*_bytes reports");
    if (reinterpret_cast<uintptr_t>(subnets) % kAlign || reinterpret_cast<uintptr_t>(workspace) % kAlign)
        return fail(ctx, IST_EINVAL, "ist_bind: buffers must be 256-byte aligned");
    ctx->subnets = static_cast<char *>(subnets);
    ctx->workspace = static_cast<char *>(workspace);
    ctx->partitioned = false;
    ctx->spare = nullptr;   // a spare bound earlier may be the buffer bound now: ask for it again
    // Index tables start as zeros so that they hold in-range values at all times,
    // also after a partition with an invalid permutation.
    const size_t tables = ctx->layer[0].off_W;
    IST_HIP(hipMemset(ctx->subnets, 0, tables), "ist_bind: clear tables");
    // scratch tables, and the activation / gradient buffers whose row padding must stay zero
    IST_HIP(hipMemset(ctx->workspace, 0, ctx->off_rowloss), "ist_bind: clear workspace");
    IST_HIP(hipMemset(ctx->workspace + ctx->off_err, 0, sizeof(int32_t)), "ist_bind: clear flag");
    ctx->bound = true;
    return IST_OK;
}

ist_status ist_set_checked(ist_ctx *ctx, int32_t checked)
{
    if (!ctx) return IST_EINVAL;
    ctx->checked = checked ? 1 : 0;
    return IST_OK;
}

// rows / columns of layer l held by subnet s itself (blocks may differ by one neuron)
static void own_shape(const ist_ctx *ctx, int32_t s, int32_t l, int64_t *rows, int64_t *cols)
{
    const LayerPlan &L = ctx->layer[l - 1];
    *rows = L.row_part ? ctx->hidden[l - 1].width(s, ctx->S) : L.N_out;
    *cols = L.col_part ? ctx->hidden[l - 2].width(s, ctx->S) : L.N_in;
}

ist_status ist_subnet_shape(const ist_ctx *ctx, int32_t l, int64_t *rows, int64_t *cols)
{
    if (!ctx || !rows || !cols || l < 1 || l > ctx->t) return IST_EINVAL;
    own_shape(ctx, 0, l, rows, cols);   // subnet 0 owns the widest blocks
    return IST_OK;
}

ist_status ist_subnet_shape_of(const ist_ctx *ctx, int32_t s, int32_t l, int64_t *rows, int64_t *cols)
{
    if (!ctx || !rows || !cols || l < 1 || l > ctx->t || s < 0 || s >= ctx->S) return IST_EINVAL;
    own_shape(ctx, s, l, rows, cols);
    return IST_OK;
}

static ist_status check_params(ist_ctx *ctx, const ist_params *p, const char *who)
{
    if (!p || !p->W) return fail(ctx, IST_EINVAL, std::string(who) + ": null params");
    if (ctx->has_bias && !p->b) return fail(ctx, IST_EINVAL, std::string(who) + ": null bias list");
    for (int l = 1; l <= ctx->t; ++l) {
        if (!p->W[l - 1]) return fail(ctx, IST_EINVAL, std::string(who) + ": null W_l");
        if (ctx->has_bias && !p->b[l - 1]) return fail(ctx, IST_EINVAL, std::string(who) + ": null b_l");
        if (reinterpret_cast<uintptr_t>(p->W[l - 1]) % ctx->esz())
            return fail(ctx, IST_EINVAL, std::string(who) + ": misaligned W_l");
    }
    return IST_OK;
}

// Block tables of every hidden layer from the permutations, into the subnet buffer at `base`;
// with checking on, IST_EPERM if some perm is not a permutation (synchronises the stream).
static ist_status build_tables(ist_ctx *ctx, char *base, const int32_t *const *perm, hipStream_t st, const char *who)
{
    const int t = ctx->t, S = ctx->S;
    if (ctx->checked) {
        // fills by a kernel, not memset nodes, so that a caller may record the call into a HIP graph
        IST_HIP(launch_fill_u32(ctx->errflag(), 1, 0u, st), "clear flag");
        for (int l = 1; l < t; ++l)
            IST_HIP(launch_fill_u32(ctx->workspace + ctx->hidden[l - 1].off_invpos, ctx->hidden[l - 1].N, 0xffffffffu, st),
                    "clear invpos");
    }
    for (int l0 = 1; l0 < t; l0 += kMaxPermJobs) {   // all hidden layers (8 at a time) in two launches
        PermJobs pj{};
        pj.S = S;
        for (int l = l0; l < t && l < l0 + kMaxPermJobs; ++l) {
            const HiddenPlan &h = ctx->hidden[l - 1];
            pj.job[pj.njobs++] = PermJob{perm[l - 1], reinterpret_cast<int32_t *>(ctx->workspace + h.off_invpos),
                                         reinterpret_cast<int32_t *>(base + h.off_sorted),
                                         reinterpret_cast<int32_t *>(base + h.off_slot),
                                         reinterpret_cast<int32_t *>(base + h.off_p2q),
                                         reinterpret_cast<uint32_t *>(base + h.off_mask),
                                         reinterpret_cast<int32_t *>(base + h.off_rank), h.N};
        }
        IST_RUN(KC_PERM_TABLES, launch_perm_tables(pj, ctx->errflag(), st), "perm tables");
    }
    if (ctx->checked)
        for (int l = 1; l < t; ++l) {
            const HiddenPlan &h = ctx->hidden[l - 1];
            IST_RUN(KC_PERM_TABLES, launch_perm_check(perm[l - 1], reinterpret_cast<const int32_t *>(ctx->workspace + h.off_invpos),
                                                      h.N, ctx->errflag(), st), "perm check");
        }
    if (ctx->checked) {
        int32_t flag = 0;
        IST_HIP(hipMemcpyAsync(&flag, ctx->errflag(), sizeof(flag), hipMemcpyDeviceToHost, st), "read flag");
        IST_HIP(hipStreamSynchronize(st), "sync");
        if (flag) return fail(ctx, IST_EPERM, std::string(who) + ": perm is not a permutation of 0..N_l-1");
    }

    return IST_OK;
}

ist_status ist_partition(ist_ctx *ctx, const ist_params *params, const int32_t *const *perm,
                         void *stream)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound) return fail(ctx, IST_ESTATE, "ist_partition: no buffers bound");
    ist_status ps = check_params(ctx, params, "ist_partition");
    if (ps != IST_OK) return ps;
    if (!perm) return fail(ctx, IST_EINVAL, "ist_partition: null perm list");
    for (int l = 1; l < ctx->t; ++l)
        if (!perm[l - 1]) return fail(ctx, IST_EINVAL, "ist_partition: null perm");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int t = ctx->t, S = ctx->S, e = ctx->esz();
    ctx->partitioned = false;

    ist_status ts = build_tables(ctx, ctx->subnets, perm, st, "ist_partition");
    if (ts != IST_OK) return ts;

    BiasCopyJobs bj{};
    for (int l = 1; l <= t; ++l) {
        const LayerPlan &L = ctx->layer[l - 1];
        CopyArgs a = copy_args(ctx, ctx->subnets, l, params->W[l - 1]);
        IST_RUN(KC_PARTITION_COPY, launch_partition_copy(a, st), "partition copy");
        if (ctx->has_bias) {   // hidden biases travel with their neuron, the output bias goes to every subnet
            if (bj.njobs == 16) { IST_RUN(KC_BIAS_COPY, launch_bias_jobs(bj, e, false, st), "partition biases"); bj.njobs = 0; }
            if (l < t) bj.job[bj.njobs++] = BiasCopyJob{params->b[l - 1], ctx->subnets + L.off_b, a.rows, L.R * S, S, 0};
            else bj.job[bj.njobs++] = BiasCopyJob{params->b[l - 1], ctx->subnets + L.off_b, nullptr, L.R, S, 0};
        }
    }
    if (bj.njobs) IST_RUN(KC_BIAS_COPY, launch_bias_jobs(bj, e, false, st), "partition biases");
    ctx->partitioned = true;
    return IST_OK;
}

ist_status ist_merge(ist_ctx *ctx, const ist_params *params, void *stream)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound || !ctx->partitioned) return fail(ctx, IST_ESTATE, "ist_merge: call ist_partition first");
    ist_status ps = check_params(ctx, params, "ist_merge");
    if (ps != IST_OK) return ps;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int t = ctx->t, S = ctx->S, e = ctx->esz();
    BiasCopyJobs bj{};
    for (int l = 1; l <= t; ++l) {
        const LayerPlan &L = ctx->layer[l - 1];
        CopyArgs a = copy_args(ctx, ctx->subnets, l, params->W[l - 1]);
        IST_RUN(KC_MERGE_COPY, launch_merge_copy(a, st), "merge copy");
        if (ctx->has_bias) {
            if (l < t) {
                if (bj.njobs == 16) { IST_RUN(KC_BIAS_COPY, launch_bias_jobs(bj, e, true, st), "merge biases"); bj.njobs = 0; }
                bj.job[bj.njobs++] = BiasCopyJob{params->b[l - 1], ctx->subnets + L.off_b, a.rows, L.R * S, S, 0};
            } else {
                IST_RUN(KC_BIAS_COPY, launch_bias_mean(params->b[l - 1], ctx->subnets + L.off_b, L.R, S, ctx->dtype, st),
                        "mean output bias");
            }
        }
    }
    if (bj.njobs) IST_RUN(KC_BIAS_COPY, launch_bias_jobs(bj, e, true, st), "merge biases");
    return IST_OK;
}

ist_status ist_bind_spare(ist_ctx *ctx, void *spare_subnets, size_t bytes)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound) return fail(ctx, IST_ESTATE, "ist_bind_spare: call ist_bind first");
    if (!spare_subnets) return fail(ctx, IST_EINVAL, "ist_bind_spare: null buffer");
    if (bytes < ctx->subnets_bytes) return fail(ctx, IST_ENOMEM, "ist_bind_spare: buffer smaller than ist_subnets_bytes reports");
    if (reinterpret_cast<uintptr_t>(spare_subnets) % kAlign) return fail(ctx, IST_EINVAL, "ist_bind_spare: buffer must be 256-byte aligned");
    if (spare_subnets == ctx->subnets) return fail(ctx, IST_EINVAL, "ist_bind_spare: the spare must be a second buffer");
    IST_HIP(hipMemset(spare_subnets, 0, ctx->layer[0].off_W), "ist_bind_spare: clear tables");
    ctx->spare = static_cast<char *>(spare_subnets);
    return IST_OK;
}

ist_status ist_resample(ist_ctx *ctx, const ist_params *params, const int32_t *const *perm, void *stream)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound || !ctx->partitioned) return fail(ctx, IST_ESTATE, "ist_resample: call ist_partition first");
    if (!ctx->spare) return fail(ctx, IST_ESTATE, "ist_resample: call ist_bind_spare first");
    ist_status ps = check_params(ctx, params, "ist_resample");
    if (ps != IST_OK) return ps;
    if (!perm) return fail(ctx, IST_EINVAL, "ist_resample: null perm list");
    for (int l = 1; l < ctx->t; ++l)
        if (!perm[l - 1]) return fail(ctx, IST_EINVAL, "ist_resample: null perm");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int t = ctx->t, S = ctx->S, e = ctx->esz();
    // tables of the new partition go to the spare buffer; a rejected perm leaves everything as it was
    ist_status ts = build_tables(ctx, ctx->spare, perm, st, "ist_resample");
    if (ts != IST_OK) return ts;
    for (int l = 1; l <= t; ++l) {
        const LayerPlan &L = ctx->layer[l - 1];
        CopyArgs o = copy_args(ctx, ctx->subnets, l, params->W[l - 1]);
        CopyArgs n = copy_args(ctx, ctx->spare, l, params->W[l - 1]);
        bool fused = false;
        IST_RUN(KC_RESAMPLE, launch_resample_copy(o, n, &fused, st), "resample copy");
        if (!fused) {
            IST_RUN(KC_MERGE_COPY, launch_merge_copy(o, st), "merge copy");
            IST_RUN(KC_PARTITION_COPY, launch_partition_copy(n, st), "partition copy");
        }
        if (ctx->has_bias) {
            if (l < t) {
                IST_RUN(KC_BIAS_COPY, launch_bias_rows(params->b[l - 1], ctx->subnets + L.off_b, o.rows, L.R * S, e, true, st),
                        "merge bias");
                IST_RUN(KC_BIAS_COPY, launch_bias_rows(params->b[l - 1], ctx->spare + L.off_b, n.rows, L.R * S, e, false, st),
                        "partition bias");
            } else {
                IST_RUN(KC_BIAS_COPY, launch_bias_mean(params->b[l - 1], ctx->subnets + L.off_b, L.R, S, ctx->dtype, st),
                        "mean output bias");
                IST_RUN(KC_BIAS_COPY, launch_bias_replicate(params->b[l - 1], ctx->spare + L.off_b, L.R, S, e, st),
                        "replicate output bias");
            }
        }
    }
    std::swap(ctx->subnets, ctx->spare);
    return IST_OK;
}

ist_status ist_subnet_export(ist_ctx *ctx, int32_t s, int32_t l, void *dstW, void *dstb, void *stream)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound || !ctx->partitioned) return fail(ctx, IST_ESTATE, "ist_subnet_export: call ist_partition first");
    if (s < 0 || s >= ctx->S || l < 1 || l > ctx->t || !dstW) return fail(ctx, IST_EINVAL, "ist_subnet_export: bad argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const LayerPlan &L = ctx->layer[l - 1];
    const int e = ctx->esz(), S = ctx->S;
    const int32_t *pr = L.row_part ? tbl(ctx->subnets, ctx->hidden[l - 1].off_p2q) : nullptr;
    const int32_t *pc = L.col_part ? tbl(ctx->subnets, ctx->hidden[l - 2].off_p2q) : nullptr;
    int64_t nr, nc;
    own_shape(ctx, s, l, &nr, &nc);
    const int64_t perm_r = L.row_part ? ctx->hidden[l - 1].perm_start(s, S) : 0, pack_r = L.row_part ? (int64_t)s * L.R : 0;
    const int64_t perm_c = L.col_part ? ctx->hidden[l - 2].perm_start(s, S) : 0, pack_c = L.col_part ? (int64_t)s * L.C : 0;
    const char *blk = ctx->subnets + L.off_W + (size_t)s * L.R * L.C * e;
    IST_HIP(launch_export(blk, dstW, nr, nc, L.R, L.C, pr, perm_r, pack_r, pc, perm_c, pack_c, L.transposed, e, st),
            "export W");
    if (dstb) {
        if (!ctx->has_bias) return fail(ctx, IST_EINVAL, "ist_subnet_export: model has no bias");
        const char *bb = ctx->subnets + L.off_b + (size_t)s * L.R * e;
        IST_HIP(launch_export(bb, dstb, nr, 1, L.R, 1, pr, perm_r, pack_r, nullptr, 0, 0, false, e, st), "export b");
    }
    return IST_OK;
}

// Where the full-network forward pass keeps its intermediate values: either regions of the bound
// workspace or a layout inside the library's own static scratch array.
struct FullFwdBuffers {
    char *act[64], *z[64], *zh[64], *isg[64];   // per layer l-1 (hidden layers; z / zh / isg with normalize only)
    int64_t pitch[64];                          // row pitch of layer l's activations, in elements
    float *partial; size_t partial_bytes;       // split-K scratch
    const void *zeros;                          // 256 zero bytes
};

static ist_status forward_full_checks(ist_ctx *ctx, const ist_params *params, const ist_batch *bt, float *logits,
                                      const char *who)
{
    if (!params || !params->W || !bt || !logits) return fail(ctx, IST_EINVAL, std::string(who) + ": null argument");
    if (ctx->has_bias && !params->b) return fail(ctx, IST_EINVAL, std::string(who) + ": null bias list");
    if (bt->B < 1 || bt->B > ctx->max_B) return fail(ctx, IST_ESHAPE, std::string(who) + ": B outside 1..max_B");
    if (ctx->input == IST_CSR) {
        if (!bt->rowptr || !bt->colidx || !bt->vals || bt->nnz < 0)
            return fail(ctx, IST_EINVAL, std::string(who) + ": incomplete CSR batch");
    } else if (!bt->x) {
        return fail(ctx, IST_EINVAL, std::string(who) + ": null x");
    }
    for (int l = 1; l <= ctx->t; ++l)
        if (!params->W[l - 1] || (ctx->has_bias && !params->b[l - 1]))
            return fail(ctx, IST_EINVAL, std::string(who) + ": null parameter array");
    if (ctx->t > 64) return fail(ctx, IST_EUNSUPPORTED, std::string(who) + ": more than 64 layers");
    return IST_OK;
}

static ist_status forward_full_run(ist_ctx *ctx, const ist_params *params, const ist_batch *bt, float *logits,
                                   const FullFwdBuffers &fb, hipStream_t st)
{
    const bool csr = ctx->input == IST_CSR;
    const int t = ctx->t, B = bt->B, dt = ctx->dtype;
    for (int l = 1; l <= t; ++l) {
        const LayerPlan &L = ctx->layer[l - 1];
        const void *bias = ctx->has_bias ? params->b[l - 1] : nullptr;
        const bool nrm = ctx->normalize && l < t;
        if (l == 1 && csr) {
            CsrArgs c{bt->rowptr, bt->colidx, bt->vals, bt->nnz, 0, 0, 1, B, L.N_in, L.N_out, fb.pitch[0]};
            IST_RUN(KC_CSR_FORWARD, launch_csr_forward(c, params->W[0], bias, fb.act[0],
                                       nrm ? reinterpret_cast<float *>(fb.z[0]) : nullptr, dt, st, true),
                    "csr forward (full network)");
        } else {
            GemmArgs a{};
            a.partial = fb.partial_bytes ? fb.partial : nullptr;
            a.partial_bytes = fb.partial_bytes;
            a.zeros = fb.zeros;
            if (l == 1) { a.A = bt->x; a.sam = L.N_in; }
            else { a.A = fb.act[l - 2]; a.sam = fb.pitch[l - 2]; }
            a.sak = 1; a.gA = 0;
            a.B = params->W[l - 1]; a.sbn = L.N_in; a.sbk = 1; a.gB = 0;
            a.M = B; a.N = (int32_t)L.N_out; a.K = (int32_t)L.N_in; a.G = 1;
            a.bias = bias; a.gBias = 0;
            if (l == t) { a.C = logits; a.ldc = L.N_out; }
            else if (nrm) { a.C = fb.z[l - 1]; a.ldc = fb.pitch[l - 1]; }
            else { a.C = fb.act[l - 1]; a.ldc = fb.pitch[l - 1]; }
            a.gC = 0;
            IST_RUN(KC_GEMM_FWD, launch_gemm(dt, (l == t || nrm) ? EPI_FWD_LOGITS : EPI_FWD_RELU, a, st),
                    "forward gemm (full network)");
        }
        if (nrm)
            IST_RUN(KC_NORM, launch_norm_forward(reinterpret_cast<const float *>(fb.z[l - 1]), fb.zh[l - 1],
                                fb.act[l - 1], reinterpret_cast<float *>(fb.isg[l - 1]), 1, B, L.N_out, fb.pitch[l - 1],
                                ctx->norm_eps, dt, st), "standardise (full network)");
    }
    return IST_OK;
}

ist_status ist_forward_full(ist_ctx *ctx, const ist_params *params, const ist_batch *bt, float *logits, void *stream)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound) return fail(ctx, IST_ESTATE, "ist_forward_full: call ist_bind first");
    ist_status cs = forward_full_checks(ctx, params, bt, logits, "ist_forward_full");
    if (cs != IST_OK) return cs;
    const int t = ctx->t, S = ctx->S;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = ctx->workspace;
    // One group of full width: the activation regions hold S subnets of max_B x ldr each, which is
    // exactly room for max_B rows of S * ldr >= N_l values.
    FullFwdBuffers fb{};
    for (int l = 1; l < t; ++l) {
        const LayerPlan &L = ctx->layer[l - 1];
        fb.act[l - 1] = ws + L.off_act; fb.z[l - 1] = ws + L.off_z; fb.zh[l - 1] = ws + L.off_zh;
        fb.isg[l - 1] = ws + L.off_isg;
        fb.pitch[l - 1] = (int64_t)S * L.ldr;
    }
    fb.partial = reinterpret_cast<float *>(ws + ctx->off_partial);
    fb.partial_bytes = ctx->partial_bytes;
    fb.zeros = ws + ctx->off_zeros;
    ist_status rs = forward_full_run(ctx, params, bt, logits, fb, st);
    if (rs != IST_OK) return rs;
    // Rows of full width overlay the subnets' padded rows: where a subnet row has padding columns
    // (R not a multiple of 8) they now hold values, and ist_subnet_steps relies on zeros there.
    bool padded = false;
    for (int l = 1; l <= t; ++l) padded = padded || ctx->layer[l - 1].ldr != ctx->layer[l - 1].R;
    if (padded)
        IST_RUN(KC_BIAS_COPY, launch_fill_zero(ws + ctx->layer[0].off_act, ctx->off_zeros - ctx->layer[0].off_act, st),
                "clear workspace");
    return IST_OK;
}

// ---- ist_forward_full_static: the same pass with its intermediate values in the library's own array ----
// (the array lives in this file so that its address can be asked for here)
constexpr size_t kStaticScratchBytes = IST_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device, asked for once per device (each GPU holds its
// own copy of the array at its own address).  Host code must use this pointer: the array's name is
// only a handle for hipGetSymbolAddress on the host side.
static hipError_t static_scratch_ptr(char **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = static_cast<char *>(ptr[dev]);
    return hipSuccess;
}

ist_status ist_forward_full_static(ist_ctx *ctx, const ist_params *params, const ist_batch *bt, float *logits,
                                   void *stream)
{
    if (!ctx) return IST_EINVAL;
    ist_status cs = forward_full_checks(ctx, params, bt, logits, "ist_forward_full_static");
    if (cs != IST_OK) return cs;
    const int t = ctx->t, e = ctx->esz();
    const size_t B = (size_t)bt->B;
    // layout inside the array, sized for this call's batch: zeros | per hidden layer h (and z, zh, 1/sigma) | split-K partials
    FullFwdBuffers fb{};
    size_t off = align_up(256);
    size_t offs[64][4] = {};
    for (int l = 1; l < t; ++l) {
        const size_t pitch = (size_t)(ctx->layer[l - 1].N_out + 7) / 8 * 8;
        fb.pitch[l - 1] = (int64_t)pitch;
        offs[l - 1][0] = off; off = align_up(off + B * pitch * e);
        if (ctx->normalize) {
            offs[l - 1][1] = off; off = align_up(off + B * pitch * sizeof(float));
            offs[l - 1][2] = off; off = align_up(off + B * pitch * e);
            offs[l - 1][3] = off; off = align_up(off + pitch * sizeof(float));
        }
        if (off > kStaticScratchBytes) break;   // (also keeps the sums far from overflow)
    }
    const size_t off_partial = off;
    off = align_up(off + ctx->partial_bytes);
    if (off > kStaticScratchBytes) {
        char msg[200];
        snprintf(msg, sizeof(msg), "ist_forward_full_static: this network and batch need more than the %zu bytes of the "
                                   "library's static scratch array; use ist_forward_full with a bound workspace",
                 kStaticScratchBytes);
        return fail(ctx, IST_ENOMEM, msg);
    }
    char *base = nullptr;
    IST_HIP(static_scratch_ptr(&base), "ist_forward_full_static: address of the scratch array");
    for (int l = 1; l < t; ++l) {
        fb.act[l - 1] = base + offs[l - 1][0]; fb.z[l - 1] = base + offs[l - 1][1];
        fb.zh[l - 1] = base + offs[l - 1][2]; fb.isg[l - 1] = base + offs[l - 1][3];
    }
    fb.partial = reinterpret_cast<float *>(base + off_partial);
    fb.partial_bytes = ctx->partial_bytes;
    fb.zeros = base;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The array keeps what the last call left: the zero block and the padding columns of the rows
    // (read by 16-byte operand loads) must be zero again, so the part in use is cleared, by a kernel.
    IST_HIP(launch_fill_zero(base, off_partial, st), "ist_forward_full_static: clear scratch");
    const bool prof = ctx->prof_on;   // per-launch events would have to be created: not here
    ctx->prof_on = false;
    const ist_status rs = forward_full_run(ctx, params, bt, logits, fb, st);
    ctx->prof_on = prof;
    return rs;
}

// One local step (step j of k) of every subnet on stream st: forward, loss, backward, update.
static ist_status one_step(ist_ctx *ctx, const ist_batch *bt, float lr, int32_t j, int32_t k, float *loss_out,
                           hipStream_t st)
{
    const bool csr = ctx->input == IST_CSR;
    const int t = ctx->t, S = ctx->S, e = ctx->esz(), B = bt->B, dt = ctx->dtype;
    char *ws = ctx->workspace, *sb = ctx->subnets;
    float *rowloss0 = reinterpret_cast<float *>(ws + ctx->off_rowloss);   // [kLossSlots][S][B]
    const int64_t ldb = (B + 7) / 8 * 8;   // row pitch of the transposed dz of a wide output layer
    std::vector<GemmArgs> upd;
    upd.reserve((size_t)t);
    {
        const int64_t row0 = (int64_t)j * bt->stride_k;
        float *rowloss = rowloss0 + (size_t)(j % kLossSlots) * S * B;
        int out_splits = 1, out_nrb = 0;
        WideOutArgs wide{};
        // ---------------- forward ----------------
        for (int l = 1; l <= t; ++l) {
            const LayerPlan &L = ctx->layer[l - 1];
            const void *bias = ctx->has_bias ? sb + L.off_b : nullptr;
            if (l == 1 && csr) {
                CsrArgs c{bt->rowptr, bt->colidx, bt->vals, bt->nnz, row0, bt->stride_s, S, B, L.C, L.R, L.ldr};
                c.alpha = ctx->scale[0];
                const bool nrm = ctx->normalize && l < t;
                IST_RUN(KC_CSR_FORWARD, launch_csr_forward(c, sb + L.off_W, bias, ws + L.off_act,
                                           nrm ? reinterpret_cast<float *>(ws + L.off_z) : nullptr, dt, st), "csr forward");
                if (nrm)
                    IST_RUN(KC_NORM, launch_norm_forward(reinterpret_cast<const float *>(ws + L.off_z), ws + L.off_zh,
                                        ws + L.off_act, reinterpret_cast<float *>(ws + L.off_isg), S, B, L.R, L.ldr,
                                        ctx->norm_eps, dt, st), "standardise (forward)");
                continue;
            }
            GemmArgs a{};
            set_split(ctx, a);
            if (l == 1) {
                a.A = static_cast<const char *>(bt->x) + (size_t)row0 * L.C * e;
                a.gA = bt->stride_s * L.C;
            } else {
                a.A = ws + ctx->layer[l - 2].off_act;
                a.gA = (int64_t)B * ctx->layer[l - 2].ldr;
            }
            a.sam = (l == 1) ? L.C : ctx->layer[l - 2].ldr; a.sak = 1;
            a.B = sb + L.off_W; a.sbn = L.C; a.sbk = 1; a.gB = L.R * L.C;
            a.C = ws + L.off_act; a.ldc = L.ldr; a.gC = (int64_t)B * L.ldr;
            a.M = B; a.N = (int32_t)L.R; a.K = (int32_t)L.C; a.G = S;
            a.bias = bias; a.gBias = L.R;
            a.alpha = ctx->scale[l - 1];
            if (l == t && ctx->wide_out) {
                // statistics launch, merge into log-sum-exp and loss; the backward launch follows below
                WideOutArgs wa{};
                wa.h = a.A; wa.ldh = a.sam; wa.gH = a.gA;
                wa.W = sb + L.off_W; wa.gW = L.R * L.C;
                wa.bias = ctx->has_bias ? sb + L.off_b : nullptr; wa.gBias = L.R;
                wa.y = bt->y + row0; wa.gY = bt->stride_s;
                wa.G = S; wa.B = B; wa.C = (int32_t)L.C; wa.N = L.R;
                wa.alpha = ctx->scale[t - 1]; wa.lr_w = lr * ctx->scale[t - 1]; wa.lr_b = lr; wa.invB = 1.0f / (float)B;
                wa.pmax = reinterpret_cast<float *>(ws + ctx->off_pmax);
                wa.psum = reinterpret_cast<float *>(ws + ctx->off_psum);
                wa.nb = ctx->wide_nb;
                wa.zlabel = reinterpret_cast<float *>(ws + ctx->off_zlabel);
                wa.lse = reinterpret_cast<float *>(ws + ctx->off_lse);
                wa.partial = reinterpret_cast<float *>(ws + ctx->off_partial);
                wa.zeros = ws + ctx->off_zeros;
                IST_RUN(KC_GEMM_FWD, launch_wide_out_stats(wa, st), "wide output layer: row statistics");
                IST_RUN(KC_SOFTMAX_XENT, launch_lse_combine(wa.pmax, wa.psum, wa.nb, reinterpret_cast<float *>(ws + ctx->off_qmax),
                                                           reinterpret_cast<float *>(ws + ctx->off_qsum), wa.zlabel, wa.y, wa.gY, L.R,
                                                           reinterpret_cast<float *>(ws + ctx->off_lse), rowloss, S, B, st),
                        "combine row statistics");
                wide = wa;
                continue;
            }
            if (l == t && ctx->fused_out) {
                // pass 1: per-row, per-column-block max / sum(exp); pass 2 (after the row
                // statistics are combined): recompute the logits and store dz_t directly
                const int bw = lse_block_width(dt, a.M, a.N, a.K, a.G);
                a.y = bt->y + row0; a.gY = bt->stride_s;
                a.pmax = reinterpret_cast<float *>(ws + ctx->off_pmax);
                a.psum = reinterpret_cast<float *>(ws + ctx->off_psum);
                a.nb = (int32_t)((L.R + bw - 1) / bw);
                a.zlabel = reinterpret_cast<float *>(ws + ctx->off_zlabel);
                a.lse = reinterpret_cast<float *>(ws + ctx->off_lse);
                a.invB = 1.0f / (float)B;
                IST_RUN(KC_GEMM_FWD, launch_gemm(dt, EPI_LSE, a, st), "forward gemm (row statistics)");
                IST_RUN(KC_SOFTMAX_XENT, launch_lse_combine(a.pmax, a.psum, a.nb, reinterpret_cast<float *>(ws + ctx->off_qmax),
                                                           reinterpret_cast<float *>(ws + ctx->off_qsum), a.zlabel, a.y, a.gY, L.R,
                                                           reinterpret_cast<float *>(ws + ctx->off_lse), rowloss, S, B, st),
                        "combine row statistics");
                // pass 2 with the operands exchanged: rows = classes, columns = samples, so that dz_t is
                // written (and later read) as dz_t^T [N_t][ldb], whole tiles contiguous in memory
                GemmArgs d{};
                set_split(ctx, d);
                d.A = a.B; d.sam = a.sbn; d.sak = 1; d.gA = a.gB;
                d.B = a.A; d.sbn = a.sam; d.sbk = 1; d.gB = a.gA;
                d.M = a.N; d.N = a.M; d.K = a.K; d.G = S;
                d.C = ws + L.off_dz; d.ldc = ldb; d.gC = L.R * ldb;
                d.bias = bias; d.gBias = L.R; d.alpha = a.alpha;
                d.y = a.y; d.gY = a.gY; d.lse = a.lse; d.invB = a.invB;
                if (ctx->has_bias) {
                    const int rw = dzt_block_width(dt, d.M, d.N, d.K, d.G);
                    d.pmax = reinterpret_cast<float *>(ws + ctx->off_rsum);   // here: partial bias gradients
                    d.nb = out_nrb = (B + rw - 1) / rw;
                }
                IST_RUN(KC_GEMM_FWD, launch_gemm(dt, EPI_DZT, d, st), "forward gemm (dz, transposed)");
                continue;
            }
            if (ctx->normalize && l < t) {
                // z_l in fp32, then standardise each neuron over the batch and apply the ReLU
                a.C = ws + L.off_z;
                IST_RUN(KC_GEMM_FWD, launch_gemm(dt, EPI_FWD_LOGITS, a, st), "forward gemm (pre-activation)");
                IST_RUN(KC_NORM, launch_norm_forward(reinterpret_cast<const float *>(ws + L.off_z), ws + L.off_zh,
                                    ws + L.off_act, reinterpret_cast<float *>(ws + L.off_isg), S, B, L.R, L.ldr,
                                    ctx->norm_eps, dt, st), "standardise (forward)");
                continue;
            }
            if (l == t && L.R <= kXentRowsMaxC) {
                // narrow output layer: a k-split product leaves its partial sums to the cross-entropy kernel
                a.keep_partial = 1;
                out_splits = gemm_splits(dt, EPI_FWD_LOGITS, a);
            }
            IST_RUN(KC_GEMM_FWD, launch_gemm(dt, l == t ? EPI_FWD_LOGITS : EPI_FWD_RELU, a, st), "forward gemm");
        }
        // ---------------- loss and dz_t ----------------
        if (!ctx->fused_out) {
            const LayerPlan &L = ctx->layer[t - 1];
            if (L.R > kXentRowsMaxC) {
                IST_RUN(KC_SOFTMAX_XENT, launch_softmax_xent(reinterpret_cast<const float *>(ws + L.off_act), bt->y + row0,
                                            bt->stride_s, ws + L.off_dz, rowloss, S, B, L.R, L.ldr, dt, st),
                        "softmax cross-entropy");
            } else if (out_splits > 1) {
                const int64_t mn = (int64_t)B * L.R;
                IST_RUN(KC_SOFTMAX_XENT, launch_xent_rows(reinterpret_cast<const float *>(ws + ctx->off_partial), out_splits, mn,
                                            out_splits * mn, L.R, ctx->has_bias ? sb + L.off_b : nullptr, L.R, bt->y + row0,
                                            bt->stride_s, ws + L.off_dz, L.ldr, rowloss, S, B, (int32_t)L.R, dt, st,
                                            ctx->scale[t - 1]),
                        "softmax cross-entropy (from partial products)");
            } else {
                IST_RUN(KC_SOFTMAX_XENT, launch_xent_rows(reinterpret_cast<const float *>(ws + L.off_act), 1, 0,
                                            (int64_t)B * L.ldr, L.ldr, nullptr, 0, bt->y + row0, bt->stride_s,
                                            ws + L.off_dz, L.ldr, rowloss, S, B, (int32_t)L.R, dt, st),
                        "softmax cross-entropy");
            }
        }
        // the row losses of up to kLossSlots steps are averaged by one launch
        if (loss_out && (j % kLossSlots == kLossSlots - 1 || j == k - 1)) {
            const int j0 = j - j % kLossSlots;
            IST_RUN(KC_LOSS_REDUCE, launch_loss_reduce(rowloss0, loss_out + j0, k, S, B, j - j0 + 1, st), "loss reduce");
        }
        // ---------------- backward + update, top layer first ----------------
        for (int l = t; l >= 1; --l) {
            const LayerPlan &L = ctx->layer[l - 1];
            if (l == t && ctx->wide_out) {
                // dz_t, the update of W_t and b_t and the workgroups' shares of dh in one launch; then their sum,
                // masked by h_{t-1} > 0, is dz_{t-1}
                const LayerPlan &P = ctx->layer[l - 2];
                IST_RUN(KC_GEMM_UPDATE, launch_wide_out_backward(wide, st), "wide output layer: backward and update");
                GemmArgs a{};
                set_split(ctx, a);
                a.C = ws + P.off_dz; a.ldc = P.ldr; a.gC = (int64_t)B * P.ldr;
                a.M = B; a.N = (int32_t)L.C; a.K = (int32_t)L.R; a.G = S;
                a.mask = ws + P.off_act; a.ldm = P.ldr; a.gMask = (int64_t)B * P.ldr;
                a.alpha = ctx->scale[l - 1];
                IST_RUN(KC_GEMM_BWD_DATA, launch_splitk_finish_bwd(dt, a, wide.partial, wide.nb, st),
                        "wide output layer: sum of the dh shares");
                if (ctx->normalize)
                    IST_RUN(KC_NORM, launch_norm_backward(ws + P.off_dz, ws + P.off_zh,
                                        reinterpret_cast<const float *>(ws + P.off_isg), S, B, P.R, P.ldr, dt, st),
                            "standardise (backward)");
                continue;
            }
            if (l > 1) {   // dz_{l-1} = (dz_l W_l) masked by h_{l-1} > 0, old W_l
                const LayerPlan &P = ctx->layer[l - 2];
                GemmArgs a{};
                set_split(ctx, a);
                a.A = ws + L.off_dz; a.sam = L.ldr; a.sak = 1; a.gA = (int64_t)B * L.ldr;
                if (l == t && ctx->fused_out) { a.sam = 1; a.sak = ldb; a.gA = L.R * ldb; }   // dz_t^T [N_t][ldb]
                a.B = sb + L.off_W; a.sbn = 1; a.sbk = L.C; a.gB = L.R * L.C;
                a.C = ws + P.off_dz; a.ldc = P.ldr; a.gC = (int64_t)B * P.ldr;
                a.M = B; a.N = (int32_t)L.C; a.K = (int32_t)L.R; a.G = S;
                a.mask = ws + P.off_act; a.ldm = P.ldr; a.gMask = (int64_t)B * P.ldr;
                a.alpha = ctx->scale[l - 1];
                IST_RUN(KC_GEMM_BWD_DATA, launch_gemm(dt, EPI_BWD_DATA, a, st), "backward-data gemm");
                if (ctx->normalize)   // what the product left is d loss / d zh_{l-1}: back through the standardisation
                    IST_RUN(KC_NORM, launch_norm_backward(ws + P.off_dz, ws + P.off_zh,
                                        reinterpret_cast<const float *>(ws + P.off_isg), S, B, P.R, P.ldr, dt, st),
                            "standardise (backward)");
            }
            if (l == 1 && csr) {
                CsrArgs c{bt->rowptr, bt->colidx, bt->vals, bt->nnz, row0, bt->stride_s, S, B, L.C, L.R, L.ldr};
                IST_RUN(KC_CSR_UPDATE, launch_csr_update(c, sb + L.off_W, ws + L.off_dz,
                                          reinterpret_cast<uint32_t *>(ws + ctx->off_bitmap), lr * ctx->scale[0], dt, st),
                        "csr update");
            } else {       // W_l <- W_l - lr * dz_l^T h_{l-1}
                GemmArgs a{};
                set_split(ctx, a);
                a.A = ws + L.off_dz; a.sam = 1; a.sak = L.ldr; a.gA = (int64_t)B * L.ldr;
                if (l == t && ctx->fused_out) { a.sam = ldb; a.sak = 1; a.gA = L.R * ldb; }   // dz_t^T [N_t][ldb]
                if (l == 1) {
                    a.B = static_cast<const char *>(bt->x) + (size_t)row0 * L.C * e;
                    a.gB = bt->stride_s * L.C;
                } else {
                    a.B = ws + ctx->layer[l - 2].off_act;
                    a.gB = (int64_t)B * ctx->layer[l - 2].ldr;
                }
                a.sbn = 1; a.sbk = (l == 1) ? L.C : ctx->layer[l - 2].ldr;
                a.C = sb + L.off_W; a.ldc = L.C; a.gC = L.R * L.C;
                a.M = (int32_t)L.R; a.N = (int32_t)L.C; a.K = B; a.G = S;
                a.lr = lr * ctx->scale[l - 1];   // dW_l = gamma_l dz_l^T h_{l-1}
                // small products wait for the end of the backward chain and share a launch (they only need
                // the dz_l, and nothing reads W_l any more in this step); the others go out now
                if (gemm_update_shares_launch(dt, a)) upd.push_back(a);
                else IST_RUN(KC_GEMM_UPDATE, launch_gemm(dt, EPI_UPDATE, a, st), "backward-weight gemm");
            }
        }
        // narrow bias updates (they only need the dz_l of this step) ride along with the shared update launch
        bool bias_done = false;
        BiasArgs ride{};
        if (ctx->has_bias && !ctx->fused_out && t <= kMaxBiasJobs && !upd.empty()) {
            ride.B = B; ride.G = S; ride.lr = lr;
            for (int l = 1; l <= t; ++l) {
                const LayerPlan &L = ctx->layer[l - 1];
                ride.job[ride.njobs++] = BiasJob{sb + L.off_b, ws + L.off_dz, L.R, L.ldr, 0};
            }
            if (!bias_jobs_all_narrow(ride, dt)) ride.njobs = 0;
        }
        for (size_t u0 = 0; u0 < upd.size(); u0 += 4) {
            const int nu = (int)std::min<size_t>(4, upd.size() - u0);
            bool rode = false;
            IST_RUN(KC_GEMM_UPDATE, launch_gemm_updates(dt, upd.data() + u0, nu, (ride.njobs && !bias_done) ? &ride : nullptr,
                                                        &rode, st), "backward-weight gemm");
            bias_done = bias_done || rode;
        }
        upd.clear();
        // all bias updates of the step in one launch (they only need the dz_l of this step)
        if (ctx->has_bias && !bias_done) {
            for (int l0 = 1; l0 <= t; l0 += kMaxBiasJobs) {
                BiasArgs ba{};
                ba.B = B; ba.G = S; ba.lr = lr;
                for (int l = l0; l <= t && l < l0 + kMaxBiasJobs; ++l) {
                    const LayerPlan &L = ctx->layer[l - 1];
                    if (l == t && ctx->wide_out) continue;   // updated by the backward launch
                    if (l == t && ctx->fused_out) {
                        IST_RUN(KC_BIAS_UPDATE, launch_bias_apply(sb + L.off_b, reinterpret_cast<const float *>(ws + ctx->off_rsum),
                                                                  out_nrb, L.R, S, lr, dt, st),
                                "bias update (from the partial sums of the dz pass)");
                        continue;
                    }
                    ba.job[ba.njobs++] = BiasJob{sb + L.off_b, ws + L.off_dz, L.R, L.ldr, 0};
                }
                IST_RUN(KC_BIAS_UPDATE, launch_bias_update(ba, dt, st), "bias update");
            }
        }
    }
    return IST_OK;
}

ist_status ist_subnet_steps(ist_ctx *ctx, const ist_batch *bt, float lr, int32_t k, float *loss_out,
                            void *stream)
{
    if (!ctx) return IST_EINVAL;
    if (!ctx->bound || !ctx->partitioned) return fail(ctx, IST_ESTATE, "ist_subnet_steps: call ist_partition first");
    if (!bt || !bt->y) return fail(ctx, IST_EINVAL, "ist_subnet_steps: null batch");
    if (k < 0) return fail(ctx, IST_EINVAL, "ist_subnet_steps: k < 0");
    if (bt->B < 1 || bt->B > ctx->max_B) return fail(ctx, IST_ESHAPE, "ist_subnet_steps: B outside 1..max_B");
    if (bt->stride_s < 0 || bt->stride_k < 0) return fail(ctx, IST_EINVAL, "ist_subnet_steps: negative stride");
    const bool csr = ctx->input == IST_CSR;
    if (csr) {
        if (!bt->rowptr || !bt->colidx || !bt->vals || bt->nnz < 0)
            return fail(ctx, IST_EINVAL, "ist_subnet_steps: incomplete CSR batch");
    } else if (!bt->x) {
        return fail(ctx, IST_EINVAL, "ist_subnet_steps: null x");
    }
    if (!(lr == lr)) return fail(ctx, IST_EINVAL, "ist_subnet_steps: lr is NaN");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (k == 0) return IST_OK;
    for (int j = 0; j < k; ++j) {
        const ist_status rs = one_step(ctx, bt, lr, j, k, loss_out, st);
        if (rs != IST_OK) return rs;
    }
    return IST_OK;
}


}  // extern "C"

// C ABI of the library: host-side argument checks and dispatch.  Nothing here touches device
// memory; every check runs before the first launch so that a failing call writes nothing.
#include "common.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>

// Scratch memory of specattn_sparse_decode_attn_static: the split partials and the cost prefix of one
// attention call.  Every GPU the library runs on holds its own copy of this array until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[SPECATTN_STATIC_SCRATCH_BYTES];

namespace specattn {

static thread_local char g_error[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}

void clear_error() { g_error[0] = '\0'; }

int cu_count()
{
    static int cached = 0;
    if (cached > 0) return cached;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) {
        cached = cus;
        return cus;
    }
    (void)hipGetLastError();
    return 256;
}

specattn_status check_launch(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return SPECATTN_OK;
    set_error("%s: %s", what, hipGetErrorString(e));
    return SPECATTN_EHIP;
}

namespace {

bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }
int log2i(int x) { int s = 0; while ((1 << s) < x) ++s; return s; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

specattn_status check_select(const specattn_select_args *s, bool fused)
{
    if (!s) { set_error("select args are NULL"); return SPECATTN_EINVAL; }
    if (!s->probs || !s->counts) { set_error("probs and counts must not be NULL"); return SPECATTN_EINVAL; }
    if (!fused && !s->indices && !s->block_counts && !s->kept_mask) { set_error("indices, block_counts and kept_mask must not all be NULL"); return SPECATTN_EINVAL; }
    if (s->B <= 0 || s->H_kv <= 0 || s->n_max <= 0) { set_error("B, H_kv and n_max must be positive"); return SPECATTN_EINVAL; }
    if (!(s->top_p > 0.0f && s->top_p <= 1.0f)) { set_error("top_p must lie in (0, 1]"); return SPECATTN_EINVAL; }
    if (s->n_max > SPECATTN_MAX_N) { set_error("n_max %d exceeds %d", s->n_max, SPECATTN_MAX_N); return SPECATTN_ESHAPE; }
    if ((int64_t)s->B * s->H_kv > (1 << 24)) { set_error("too many rows"); return SPECATTN_ESHAPE; }
    if (s->indices && !fused) {
        if (s->idx_capacity < 1) { set_error("idx_capacity must be at least 1"); return SPECATTN_ESHAPE; }
        if (s->idx_stride_row < s->idx_capacity) { set_error("idx_stride_row is smaller than idx_capacity"); return SPECATTN_ESHAPE; }
    }
    if (s->chunk_size < 0 || (s->chunk_size > 1 && (!is_pow2(s->chunk_size) || s->chunk_size > 1024))) { set_error("chunk_size must be 0, 1 or a power of two up to 1024"); return SPECATTN_ESHAPE; }
    if (s->chunk_size > 1 && (s->emit_physical || s->block_counts || s->kept_mask)) { set_error("chunk-granular selection is not available with emit_physical, block_counts or kept_mask"); return SPECATTN_EUNSUPPORTED; }
    if (s->bisect_iters < 0 || s->bisect_iters > 64) { set_error("bisect_iters must lie in 0..64"); return SPECATTN_ESHAPE; }
    if (s->bisect_iters > 0 && (fused || s->block_counts || s->kept_mask || s->chunk_size > 1 || !s->indices)) { set_error("the bisection mode needs an index list and is not available with the fused call, block_counts or chunks"); return SPECATTN_EUNSUPPORTED; }
    if (s->probs_stride_h < s->n_max || s->probs_stride_b < s->n_max) { set_error("probs strides are smaller than n_max"); return SPECATTN_ESHAPE; }
    if (s->emit_physical) {
        if (!s->page_table) { set_error("emit_physical needs a page table"); return SPECATTN_EINVAL; }
        if (!is_pow2(s->page_size)) { set_error("page_size must be a power of two"); return SPECATTN_ESHAPE; }
        if ((int64_t)s->max_pages_per_seq * s->page_size < s->n_max) { set_error("page table is shorter than n_max"); return SPECATTN_ESHAPE; }
    }
    return SPECATTN_OK;
}

specattn_status check_attn(const specattn_attn_args *a, bool fused)
{
    if (!a) { set_error("attention args are NULL"); return SPECATTN_EINVAL; }
    if (!a->q || !a->k || !a->v || !a->out) { set_error("q, k, v and out must not be NULL"); return SPECATTN_EINVAL; }
    const bool dense = !fused && !a->indices && !a->counts;     // no list: attend to every position
    if (!fused && !dense && (!a->indices || !a->counts)) { set_error("indices and counts must both be given, or both be NULL (dense)"); return SPECATTN_EINVAL; }
    if (dense && a->indices_are_physical) { set_error("indices_are_physical without an index list"); return SPECATTN_EINVAL; }
    if (a->B <= 0 || a->H_q <= 0 || a->H_kv <= 0 || a->T <= 0 || a->d <= 0 || a->n_max <= 0) { set_error("sizes must be positive"); return SPECATTN_EINVAL; }
    if (a->dtype != SPECATTN_F32 && a->dtype != SPECATTN_BF16 && a->dtype != SPECATTN_F16) { set_error("unknown dtype %d", (int)a->dtype); return SPECATTN_EUNSUPPORTED; }
    if (a->H_q % a->H_kv) { set_error("H_q is not a multiple of H_kv"); return SPECATTN_ESHAPE; }
    if (a->T > SPECATTN_MAX_T) { set_error("T exceeds %d", SPECATTN_MAX_T); return SPECATTN_ESHAPE; }
    if (a->d != 64 && a->d != 128) { set_error("d must be 64 or 128"); return SPECATTN_ESHAPE; }
    {
        // more than 64 query rows per kv head only fit the matrix-core route (the portable kernel's tables hold 64)
        AttnLaunch probe{};
        probe.dtype = (int)a->dtype; probe.d = a->d; probe.T = a->T; probe.H_kv = a->H_kv;
        if ((a->H_q / a->H_kv) * a->T > 64 && !attn_mfma_supported(probe)) { set_error("G*T exceeds 64 query rows per kv head (only bf16 / fp16 with d = 128 and H_kv <= %d take more)", ATTN_MFMA_MAX_ROWS); return SPECATTN_ESHAPE; }
    }
    if (!fused && !dense && a->idx_capacity < 1) { set_error("idx_capacity must be at least 1"); return SPECATTN_ESHAPE; }
    if (!fused && !dense && a->idx_stride_row < a->idx_capacity) { set_error("idx_stride_row is smaller than idx_capacity"); return SPECATTN_ESHAPE; }
    const bool paged = a->page_table != nullptr || a->indices_are_physical;
    if (paged) {
        if (!is_pow2(a->page_size)) { set_error("page_size must be a power of two"); return SPECATTN_ESHAPE; }
        if (a->page_table && (int64_t)a->max_pages_per_seq * a->page_size < a->n_max) { set_error("page table is shorter than n_max"); return SPECATTN_ESHAPE; }
        if (a->kv_stride_page <= 0) { set_error("kv_stride_page must be positive"); return SPECATTN_ESHAPE; }
    }
    if (a->chunk_size < 0 || (a->chunk_size > 1 && (!is_pow2(a->chunk_size) || a->chunk_size > 1024))) { set_error("chunk_size must be 0, 1 or a power of two up to 1024"); return SPECATTN_ESHAPE; }
    if (a->chunk_size > 1 && !fused && (dense || a->indices_are_physical)) { set_error("chunk lists are not available with dense calls or physical indices"); return SPECATTN_EUNSUPPORTED; }
    if (a->out_lowp && !aligned(a->out_lowp, 16)) { set_error("out_lowp must be 16-byte aligned"); return SPECATTN_EALIGN; }
    if ((a->k_new == nullptr) != (a->v_new == nullptr)) { set_error("k_new and v_new must both be given or both be NULL"); return SPECATTN_EINVAL; }
    if (a->k_new && (!aligned(a->k_new, 16) || !aligned(a->v_new, 16))) { set_error("k_new and v_new must be 16-byte aligned"); return SPECATTN_EALIGN; }
    if (a->kv_stride_n < a->d) { set_error("kv_stride_n is smaller than d"); return SPECATTN_ESHAPE; }
    const size_t es = a->dtype == SPECATTN_F32 ? 4 : 2;
    if (!aligned(a->q, 16) || !aligned(a->k, 16) || !aligned(a->v, 16) || !aligned(a->out, 16)) { set_error("q, k, v and out must be 16-byte aligned"); return SPECATTN_EALIGN; }
    const int64_t strides[] = {a->q_stride_b, a->q_stride_h, a->q_stride_t, a->kv_stride_b, a->kv_stride_h,
                               a->kv_stride_n, paged ? a->kv_stride_page : 0};
    for (int64_t st : strides)
        if ((st * (int64_t)es) % 16) { set_error("strides must be multiples of 16 bytes"); return SPECATTN_EALIGN; }
    return SPECATTN_OK;
}

specattn_status check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return SPECATTN_OK;
    if (!ws) { set_error("workspace is NULL, %zu bytes needed", need); return SPECATTN_EWORKSPACE; }
    if (!aligned(ws, 256)) { set_error("workspace must be 256-byte aligned"); return SPECATTN_EWORKSPACE; }
    if (have < need) { set_error("workspace has %zu bytes, %zu needed", have, need); return SPECATTN_EWORKSPACE; }
    return SPECATTN_OK;
}

// The fused call keeps the kept set on chip (mask source of the matrix-core kernel) for bf16 / fp16 with d = 128
// and single positions.  Everything else the two separate calls take (fp32, d = 64, chunk-granular selection)
// runs as those two calls with the list in the caller's workspace instead of caller-visible memory.
bool fused_on_chip(const specattn_select_args *s, const specattn_attn_args *a)
{
    AttnLaunch probe{};
    probe.dtype = (int)a->dtype; probe.d = a->d; probe.T = a->T; probe.H_kv = a->H_kv;
    return attn_mfma_supported(probe) && s->chunk_size <= 1;
}
size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

SelectLaunch make_select(const specattn_select_args *s)
{
    SelectLaunch l{};
    l.probs = s->probs;
    l.stride_b = s->probs_stride_b;
    l.stride_h = s->probs_stride_h;
    l.B = s->B; l.H_kv = s->H_kv; l.n_max = s->n_max;
    l.seq_lens = s->seq_lens;
    l.top_p = s->top_p;
    l.indices = s->indices;
    l.idx_stride = s->idx_stride_row;
    l.idx_capacity = s->indices ? s->idx_capacity : 0;
    l.counts = s->counts;
    l.thresholds = s->thresholds;
    l.row_flags = s->row_flags;
    l.page_table = s->page_table;
    l.page_shift = s->emit_physical ? log2i(s->page_size) : 0;
    l.max_pages = s->max_pages_per_seq;
    l.emit_physical = s->emit_physical;
    l.block_counts = s->block_counts;
    l.blocks_per_row = (s->n_max + SEL_BLOCK - 1) / SEL_BLOCK;
    l.n_tokens = s->n_max;
    l.chunk_shift = 0;
    l.kept_mask = s->kept_mask;
    return l;
}

AttnLaunch make_attn(const specattn_attn_args *a)
{
    AttnLaunch l{};
    l.q = a->q; l.k = a->k; l.v = a->v;
    l.dtype = (int)a->dtype;
    l.B = a->B; l.H_q = a->H_q; l.H_kv = a->H_kv; l.T = a->T; l.d = a->d; l.n_max = a->n_max;
    l.sm_scale = a->sm_scale > 0.0f ? a->sm_scale : 1.0f / std::sqrt((float)a->d);
    l.q_stride_b = a->q_stride_b; l.q_stride_h = a->q_stride_h; l.q_stride_t = a->q_stride_t;
    l.kv_stride_b = a->kv_stride_b; l.kv_stride_h = a->kv_stride_h; l.kv_stride_n = a->kv_stride_n;
    l.page_table = a->page_table;
    const bool paged = a->page_table != nullptr || a->indices_are_physical;
    l.page_shift = paged ? log2i(a->page_size) : 0;
    l.max_pages = a->max_pages_per_seq;
    l.kv_stride_page = a->kv_stride_page;
    l.indices = a->indices;
    l.idx_stride = a->idx_stride_row;
    l.counts = a->counts;
    l.idx_capacity = a->idx_capacity;
    l.indices_are_physical = a->indices_are_physical;
    l.chunk_shift = a->chunk_size > 1 ? log2i(a->chunk_size) : 0;
    l.dense = (!a->indices && !a->counts) ? 1 : 0;          // the fused call overwrites counts afterwards
    if (l.dense) l.idx_capacity = a->n_max;
    l.k_new = a->k_new;
    l.v_new = a->v_new;
    l.out = a->out;
    l.out_lowp = a->out_lowp;
    l.lse = a->lse;
    l.workspace = a->workspace;
    l.workspace_bytes = a->workspace_bytes;
    l.seq_lens = a->seq_lens;
    return l;
}

}  // namespace
}  // namespace specattn

using namespace specattn;

extern "C" {

specattn_status specattn_topp_select(const specattn_select_args *sel, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    clear_error();
    specattn_status st = check_select(sel, false);
    if (st != SPECATTN_OK) return st;
    const bool plain = sel->bisect_iters == 0 && sel->chunk_size <= 1;
    const size_t need = specattn_workspace_size(sel, nullptr);
    // the plain selection works without a workspace; with one, few long rows are split over many workgroups
    const bool split = plain && need > 0 && workspace && aligned(workspace, 256) && workspace_bytes >= need;
    if (split && sel->kept_mask) { set_error("kept_mask is not written by the split selection of few long rows: call without a workspace"); return SPECATTN_EUNSUPPORTED; }
    if (!plain) {
        st = check_workspace(workspace, workspace_bytes, need);
        if (st != SPECATTN_OK) return st;
    }
    SelectLaunch l = make_select(sel);
    if (split) {
        // workspace: [tau][valid][flags][block counts][ballots] as for the union with one member per row, then the
        // row histograms and locate states of the split passes
        const size_t rows = (size_t)sel->B * sel->H_kv, a256 = (rows * 4 + 255) & ~(size_t)255;
        char *ws = static_cast<char *>(workspace);
        float *tau = sel->thresholds ? sel->thresholds : reinterpret_cast<float *>(ws);
        int32_t *valid = reinterpret_cast<int32_t *>(ws + a256);
        uint32_t *mflags = reinterpret_cast<uint32_t *>(ws + 2 * a256);
        hipStream_t hs = static_cast<hipStream_t>(stream);
        st = launch_select_multi_wg(l, ws + union_workspace_bytes(sel->B, sel->H_kv, 1, sel->n_max), tau, valid, mflags, hs);
        if (st != SPECATTN_OK) return st;
        return launch_threshold_union(sel->probs, sel->probs_stride_b, sel->probs_stride_h, sel->B, sel->H_kv, 1, sel->n_max,
                                      sel->seq_lens, tau, valid, mflags, ws + 3 * a256, sel->indices, sel->idx_stride_row,
                                      sel->idx_capacity, sel->counts, sel->row_flags, sel->page_table, sel->page_size,
                                      sel->max_pages_per_seq, sel->emit_physical, hs);
    }
    if (sel->bisect_iters > 0) {                    // Algorithm 2 as the paper runs it, then the mask and compaction passes
        // workspace: [tau][valid][flags][block counts][ballots], the layout of the union with one member per row
        const size_t rows = (size_t)sel->B * sel->H_kv, a256 = (rows * 4 + 255) & ~(size_t)255;
        char *ws = static_cast<char *>(workspace);
        float *tau = sel->thresholds ? sel->thresholds : reinterpret_cast<float *>(ws);
        int32_t *valid = reinterpret_cast<int32_t *>(ws + a256);
        uint32_t *mflags = reinterpret_cast<uint32_t *>(ws + 2 * a256);
        hipStream_t hs = static_cast<hipStream_t>(stream);
        st = launch_bisect_thresholds(l, sel->bisect_iters, tau, valid, mflags, hs);
        if (st != SPECATTN_OK) return st;
        return launch_threshold_union(sel->probs, sel->probs_stride_b, sel->probs_stride_h, sel->B, sel->H_kv, 1, sel->n_max,
                                      sel->seq_lens, tau, valid, mflags, ws + 3 * a256, sel->indices, sel->idx_stride_row,
                                      sel->idx_capacity, sel->counts, sel->row_flags, sel->page_table, sel->page_size,
                                      sel->max_pages_per_seq, sel->emit_physical, hs);
    }
    if (sel->chunk_size > 1) {                      // reduce to chunk masses, then select over those
        const int cs = log2i(sel->chunk_size);
        const int nc = (sel->n_max + sel->chunk_size - 1) >> cs;
        float *mass = static_cast<float *>(workspace);
        st = launch_chunk_masses(sel->probs, sel->probs_stride_b, sel->probs_stride_h, sel->B, sel->H_kv, sel->n_max,
                                 sel->seq_lens, cs, nc, mass, static_cast<hipStream_t>(stream));
        if (st != SPECATTN_OK) return st;
        l.probs = mass;
        l.stride_b = (int64_t)sel->H_kv * nc;
        l.stride_h = nc;
        l.n_max = nc;
        l.chunk_shift = cs;
        l.blocks_per_row = (nc + SEL_BLOCK - 1) / SEL_BLOCK;
    }
    return launch_select(l, static_cast<hipStream_t>(stream));
}

static specattn_status check_union(const specattn_union_args *u)
{
    if (!u) { set_error("union args are NULL"); return SPECATTN_EINVAL; }
    if (!u->probs || !u->counts || !u->indices) { set_error("probs, indices and counts must not be NULL"); return SPECATTN_EINVAL; }
    if (!(u->top_p > 0.0f && u->top_p <= 1.0f)) { set_error("top_p must be in (0, 1]"); return SPECATTN_EINVAL; }
    if (u->B <= 0 || u->H_draft <= 0 || u->S <= 0 || u->H_kv <= 0 || u->n_max <= 0) { set_error("sizes must be positive"); return SPECATTN_EINVAL; }
    if (u->H_draft % u->H_kv) { set_error("H_draft is not a multiple of H_kv"); return SPECATTN_ESHAPE; }
    if (u->n_max > SPECATTN_MAX_N) { set_error("n_max exceeds %d", SPECATTN_MAX_N); return SPECATTN_ESHAPE; }
    if ((int64_t)u->B * u->H_draft * u->S > (1 << 24)) { set_error("too many rows"); return SPECATTN_ESHAPE; }
    if (u->probs_stride_row < u->n_max) { set_error("probs_stride_row is smaller than n_max"); return SPECATTN_ESHAPE; }
    if (u->idx_capacity < 1) { set_error("idx_capacity must be at least 1"); return SPECATTN_ESHAPE; }
    if (u->idx_stride_row < u->idx_capacity) { set_error("idx_stride_row is smaller than idx_capacity"); return SPECATTN_ESHAPE; }
    if (u->emit_physical && !u->page_table) { set_error("emit_physical needs a page table"); return SPECATTN_EINVAL; }
    if (u->page_table) {
        if (!is_pow2(u->page_size)) { set_error("page_size must be a power of two"); return SPECATTN_ESHAPE; }
        if ((int64_t)u->max_pages_per_seq * u->page_size < u->n_max) { set_error("page table is shorter than n_max"); return SPECATTN_ESHAPE; }
    }
    return SPECATTN_OK;
}

size_t specattn_union_workspace_size(const specattn_union_args *u)
{
    if (!u || u->B <= 0 || u->H_draft <= 0 || u->S <= 0 || u->H_kv <= 0 || u->n_max <= 0 || u->H_draft % u->H_kv) return 0;
    return union_workspace_bytes(u->B, u->H_kv, (u->H_draft / u->H_kv) * u->S, u->n_max);
}

specattn_status specattn_topp_select_union(const specattn_union_args *u, void *workspace, size_t workspace_bytes,
                                           void *stream)
{
    clear_error();
    specattn_status st = check_union(u);
    if (st != SPECATTN_OK) return st;
    st = check_workspace(workspace, workspace_bytes, specattn_union_workspace_size(u));
    if (st != SPECATTN_OK) return st;
    return launch_union(u, workspace, static_cast<hipStream_t>(stream));
}

specattn_status specattn_sparse_decode_attn(const specattn_attn_args *attn, void *stream)
{
    clear_error();
    specattn_status st = check_attn(attn, false);
    if (st != SPECATTN_OK) return st;
    st = check_workspace(attn->workspace, attn->workspace_bytes, specattn_workspace_size(nullptr, attn));
    if (st != SPECATTN_OK) return st;
    return launch_attn(make_attn(attn), static_cast<hipStream_t>(stream));
}

specattn_status specattn_lists_to_csr(const int32_t *indices, int64_t idx_stride_row, int32_t idx_capacity,
                                      const int32_t *counts, int32_t rows, int64_t *indptr, int32_t *packed, void *stream)
{
    clear_error();
    if (!counts || !indptr || (packed && !indices)) { set_error("counts and indptr must not be NULL, and packed needs indices"); return SPECATTN_EINVAL; }
    if (rows <= 0) { set_error("rows must be positive"); return SPECATTN_EINVAL; }
    if (idx_capacity < 1 || (packed && idx_stride_row < idx_capacity)) { set_error("idx_capacity must be at least 1 and idx_stride_row no smaller"); return SPECATTN_ESHAPE; }
    return launch_csr(indices, idx_stride_row, counts, rows, idx_capacity, indptr, packed, static_cast<hipStream_t>(stream));
}

specattn_status specattn_check_lists(const specattn_attn_args *attn, int64_t pool_slots, int32_t *n_bad, void *stream)
{
    clear_error();
    specattn_status st = check_attn(attn, false);
    if (st != SPECATTN_OK) return st;
    if (!attn->indices) { set_error("a dense call has no index list to check"); return SPECATTN_EINVAL; }
    if (!n_bad || pool_slots < 0) { set_error("n_bad must not be NULL and pool_slots must not be negative"); return SPECATTN_EINVAL; }
    return launch_check_lists(make_attn(attn), pool_slots, n_bad, static_cast<hipStream_t>(stream));
}

specattn_status specattn_fused(const specattn_select_args *sel, const specattn_attn_args *attn, void *stream)
{
    clear_error();
    specattn_status st = check_select(sel, true);
    if (st != SPECATTN_OK) return st;
    st = check_attn(attn, true);
    if (st != SPECATTN_OK) return st;
    if (sel->B != attn->B || sel->H_kv != attn->H_kv || sel->n_max != attn->n_max) {
        set_error("selection and attention arguments describe different rows");
        return SPECATTN_ESHAPE;
    }
    if (sel->reuse_selection && (!sel->kept_mask || !sel->block_counts)) {
        set_error("reuse_selection needs block_counts and kept_mask");
        return SPECATTN_EINVAL;
    }
    if (attn->indices_are_physical) {
        set_error("the fused call has no index list: indices_are_physical does not apply (pass the page table)");
        return SPECATTN_EUNSUPPORTED;
    }
    st = check_workspace(attn->workspace, attn->workspace_bytes, specattn_workspace_size(sel, attn));
    if (st != SPECATTN_OK) return st;
    const int rows = sel->B * sel->H_kv;
    if (!fused_on_chip(sel, attn)) {
        // selection into the workspace, then attention over that list
        if (sel->reuse_selection || sel->block_counts || sel->kept_mask) {
            set_error("reuse_selection, block_counts and kept_mask belong to the on-chip fused path (bf16 / fp16, d = 128, single positions)");
            return SPECATTN_EUNSUPPORTED;
        }
        const int chunk = sel->chunk_size > 1 ? sel->chunk_size : 1;
        const int cap = (sel->n_max + chunk - 1) / chunk;
        char *ws = static_cast<char *>(attn->workspace);
        const size_t attn_bytes = attn_workspace_bytes(rows, attn->H_q / attn->H_kv, attn->T, attn->d, attn->n_max);
        specattn_select_args s2 = *sel;
        s2.indices = reinterpret_cast<int32_t *>(ws + attn_bytes);
        s2.idx_stride_row = cap;
        s2.idx_capacity = cap;
        s2.emit_physical = 0;
        const size_t list_bytes = a256((size_t)rows * cap * sizeof(int32_t));
        const size_t sel_bytes = specattn_workspace_size(&s2, nullptr);
        st = specattn_topp_select(&s2, sel_bytes ? ws + attn_bytes + list_bytes : nullptr, sel_bytes, stream);
        if (st != SPECATTN_OK) return st;
        specattn_attn_args a2 = *attn;
        a2.indices = s2.indices;
        a2.idx_stride_row = cap;
        a2.idx_capacity = cap;
        a2.counts = sel->counts;
        a2.chunk_size = sel->chunk_size;
        a2.indices_are_physical = 0;
        a2.seq_lens = sel->seq_lens;
        a2.workspace_bytes = attn_bytes;
        return specattn_sparse_decode_attn(&a2, stream);
    }
    AttnLaunch al = make_attn(attn);
    const int blocks = (sel->n_max + SEL_BLOCK - 1) / SEL_BLOCK;
    // workspace: [attention partials][block counts: rows * blocks ints][kept mask: rows * blocks * 32 words]
    char *extra = static_cast<char *>(attn->workspace) +
                  attn_workspace_bytes(rows, attn->H_q / attn->H_kv, attn->T, attn->d, attn->n_max);
    int32_t *bc = sel->block_counts ? sel->block_counts : reinterpret_cast<int32_t *>(extra);
    extra += ((size_t)rows * blocks * sizeof(int32_t) + 255) & ~(size_t)255;
    uint32_t *mask = sel->kept_mask ? sel->kept_mask : reinterpret_cast<uint32_t *>(extra);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!sel->reuse_selection) {
        SelectLaunch sl = make_select(sel);
        sl.indices = nullptr;
        sl.idx_capacity = 0;
        sl.block_counts = bc;
        sl.blocks_per_row = blocks;
        sl.kept_mask = mask;
        st = launch_select(sl, s);
        if (st != SPECATTN_OK) return st;
    }
    al.indices = nullptr;
    al.dense = 0;
    al.counts = sel->counts;
    al.idx_capacity = sel->n_max;
    al.idx_stride = 0;
    al.seq_lens = sel->seq_lens;
    al.kept_mask = mask;
    al.block_counts = bc;
    al.blocks_per_row = blocks;
    return launch_attn_mfma(al, s);
}

size_t specattn_workspace_size(const specattn_select_args *sel, const specattn_attn_args *attn)
{
    if (!sel && !attn) return 0;
    if (sel && !attn) {                               // token selection keeps its state on chip;
        if (sel->bisect_iters > 0) {
            if (sel->B <= 0 || sel->H_kv <= 0 || sel->n_max <= 0) return 0;
            return union_workspace_bytes(sel->B, sel->H_kv, 1, sel->n_max);
        }
        if (sel->chunk_size <= 1) {                   // optional: lets few long rows be split over many workgroups
            if (sel->B <= 0 || sel->H_kv <= 0 || sel->n_max <= 0 || !sel->indices || sel->block_counts) return 0;
            if (!select_multi_wg_preferred(sel->B * sel->H_kv, sel->n_max)) return 0;
            return union_workspace_bytes(sel->B, sel->H_kv, 1, sel->n_max) + select_multi_wg_bytes(sel->B * sel->H_kv, sel->n_max);
        }
        if (sel->B <= 0 || sel->H_kv <= 0 || sel->n_max <= 0 || !is_pow2(sel->chunk_size)) return 0;
        const size_t nc = ((size_t)sel->n_max + sel->chunk_size - 1) / sel->chunk_size;
        return ((size_t)sel->B * sel->H_kv * nc * sizeof(float) + 255) & ~(size_t)255;
    }
    if (attn->B <= 0 || attn->H_kv <= 0 || attn->H_q <= 0 || attn->T <= 0 || attn->d <= 0) return 0;
    if (attn->H_q % attn->H_kv) return 0;
    const int rows = attn->B * attn->H_kv;
    const bool dense = !attn->indices && !attn->counts;
    const int cap = (sel || dense) ? attn->n_max : attn->idx_capacity * (attn->chunk_size > 1 ? attn->chunk_size : 1);
    if (cap <= 0) return 0;
    size_t bytes = attn_workspace_bytes(rows, attn->H_q / attn->H_kv, attn->T, attn->d, cap);
    if (sel && !fused_on_chip(sel, attn)) {           // fused by way of a list in the workspace
        if (sel->n_max <= 0) return 0;
        const int chunk = sel->chunk_size > 1 ? sel->chunk_size : 1;
        const int lcap = (sel->n_max + chunk - 1) / chunk;
        specattn_select_args s2 = *sel;
        s2.indices = reinterpret_cast<int32_t *>(0x1000);      // (only tested for NULL by the size query)
        bytes = a256(bytes) + a256((size_t)rows * lcap * sizeof(int32_t)) + specattn_workspace_size(&s2, nullptr);
        return bytes;
    }
    if (sel) {                                        // fused: room for the block counts and the kept mask
        const size_t blocks = ((size_t)attn->n_max + SEL_BLOCK - 1) / SEL_BLOCK;
        bytes += ((size_t)rows * blocks * sizeof(int32_t) + 255) & ~(size_t)255;
        bytes += ((size_t)rows * blocks * (SEL_BLOCK / 32) * sizeof(uint32_t) + 255) & ~(size_t)255;
    }
    return bytes;
}

// Device address of this GPU's copy of `scratch`, looked up once per device (any thread may call).
static specattn_status static_scratch(void **out)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void *ptr[MAX_DEVICES] = {nullptr};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        set_error("no current device, or its ordinal is beyond %d", MAX_DEVICES - 1);
        return SPECATTN_EHIP;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            set_error("hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
            return SPECATTN_EHIP;
        }
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return SPECATTN_OK;
}

specattn_status specattn_sparse_decode_attn_static(const specattn_attn_args *attn, void *stream)
{
    clear_error();
    specattn_status st = check_attn(attn, false);
    if (st != SPECATTN_OK) return st;
    // the least the call runs with: batches beyond 512 rows then go out in launches of 512 rows
    const bool dense = !attn->indices && !attn->counts;
    const int cap = dense ? attn->n_max : attn->idx_capacity * (attn->chunk_size > 1 ? attn->chunk_size : 1);
    const size_t need = cap <= 0 ? 0 : attn_workspace_min_bytes(attn->B * attn->H_kv, attn->H_q / attn->H_kv, attn->T, attn->d, cap);
    if (need == 0 || need > (size_t)SPECATTN_STATIC_SCRATCH_BYTES) {
        set_error("this call needs %zu bytes of scratch memory; the built-in buffer holds %zu", need,
                  (size_t)SPECATTN_STATIC_SCRATCH_BYTES);
        return SPECATTN_EWORKSPACE;
    }
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != SPECATTN_OK) return st;
    AttnLaunch l = make_attn(attn);
    l.workspace = ws;
    l.workspace_bytes = SPECATTN_STATIC_SCRATCH_BYTES;
    return launch_attn(l, static_cast<hipStream_t>(stream));
}

specattn_status specattn_init(void)
{
    clear_error();
    void *ws = nullptr;
    const specattn_status st = static_scratch(&ws);
    if (st != SPECATTN_OK) return st;
    const specattn_status sg = attn_generic_configure();
    if (sg != SPECATTN_OK) return sg;
    return attn_mfma_configure();
}

const char *specattn_last_error(void) { return g_error; }

int specattn_version(void) { return 1009; }

}  // extern "C"

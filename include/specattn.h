/*
 * specattn.h - C ABI of the MI355X (gfx950) SpecAttn hot path:
 * sorting-free top-p selection of KV positions from draft attention rows,
 * and sparse decode attention of the verifier's gamma+1 queries over the
 * selected K/V only.
 *
 * General rules for every entry point
 *  - Every pointer inside the argument structs is a DEVICE pointer owned by
 *    the caller.  The structs themselves are HOST memory, read during the
 *    call and not kept.
 *  - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL
 *    is the default stream).  The library never synchronises, never allocates
 *    and never frees device memory; scratch space comes in through the
 *    workspace arguments (size from specattn_workspace_size).
 *  - Return value: SPECATTN_OK or a negative specattn_status.  Argument
 *    errors are found on the host before anything is launched; on error no
 *    output is written.  specattn_last_error() gives a thread-local text.
 *  - "row" always means one (batch b, kv head h) pair, numbered r = b*H_kv+h.
 *  - GQA: query head h_q reads kv head h_q / (H_q / H_kv).
 */
#ifndef SPECATTN_H
#define SPECATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum specattn_status {
    SPECATTN_OK = 0,
    SPECATTN_EINVAL = -1,       /* NULL required pointer, top_p outside (0,1] or NaN, size <= 0 */
    SPECATTN_ESHAPE = -2,       /* H_q % H_kv != 0, unsupported d / T / n, capacity < 1, page size */
    SPECATTN_EALIGN = -3,       /* q/k/v base or strides not 16-byte aligned */
    SPECATTN_EWORKSPACE = -4,   /* workspace NULL, misaligned (256 B) or too small */
    SPECATTN_EUNSUPPORTED = -5, /* dtype / layout combination not built */
    SPECATTN_EHIP = -6          /* a launch failed; text in specattn_last_error() */
} specattn_status;

typedef enum specattn_dtype { SPECATTN_F32 = 0, SPECATTN_BF16 = 1, SPECATTN_F16 = 2 /* IEEE half */ } specattn_dtype;

/* bits of row_flags[r] */
#define SPECATTN_ROW_INVALID 1u        /* NaN / negative / infinite entry, zero row sum or length 0: count = 0 */
#define SPECATTN_ROW_NEAR_BOUNDARY 2u  /* kept or strictly-above mass within 1e-6 * row sum of the target */
#define SPECATTN_ROW_OVERFLOW 4u       /* count > idx_capacity: list truncated to the first idx_capacity */

/* limits */
#define SPECATTN_MAX_N (1 << 19)       /* longest row the selection handles */
#define SPECATTN_SEL_BLOCK 1024        /* positions per entry of block_counts */
#define SPECATTN_MAX_T 8               /* most verifier queries (gamma + 1) per head */
#define SPECATTN_STATIC_SCRATCH_BYTES (16u << 20)   /* built-in scratch of specattn_sparse_decode_attn_static */

/*
 * Selection (Section 3.4, Algorithm 2; objective: Appendix A, Eq. 8).
 *
 * For every row the call finds tau* = max{ t : sum of probs >= t is at least
 * top_p * (row sum) } exactly - tau* is always one of the row's values - and
 * emits { j : probs[j] >= tau* } in ascending j.  Entries tied with tau* are
 * all kept.  Exact zeros are never kept.  No sort is performed.
 */
typedef struct specattn_select_args {
    const float *probs;          /* [B][H_kv][n_max] fp32, non-negative; need not be normalised */
    int64_t probs_stride_b;      /* element strides; the last dimension is contiguous */
    int64_t probs_stride_h;
    int32_t B, H_kv, n_max;
    const int32_t *seq_lens;     /* [B] valid length per sequence, or NULL for n_max everywhere */
    float top_p;                 /* p in (0, 1] */

    int32_t *indices;            /* out [B*H_kv][idx_stride_row]: ascending positions; NULL = no list is
                                    written (then block_counts must be given, or the call is specattn_fused) */
    int64_t idx_stride_row;      /* elements between rows, >= idx_capacity */
    int32_t idx_capacity;        /* most entries written per row */
    int32_t *counts;             /* out [B*H_kv]: TRUE number kept, even when > idx_capacity */
    float *thresholds;           /* out [B*H_kv] tau*; optional (NULL) */
    uint32_t *row_flags;         /* out [B*H_kv] SPECATTN_ROW_* bits; optional (NULL) */

    /* optional paged output: emit pool slots instead of logical positions */
    const int32_t *page_table;   /* [B][max_pages_per_seq] page ids, or NULL */
    int32_t page_size;           /* tokens per page, power of two (16 in the paged workload) */
    int32_t max_pages_per_seq;
    int32_t emit_physical;       /* 1: indices[j] = page_table[b][pos/page_size]*page_size + pos%page_size
                                       (still in ascending pos order); needs page_table */

    /* selection state without an index list (what specattn_fused works from) */
    int32_t *block_counts;       /* out, optional: [B*H_kv][ceil(n_max / SPECATTN_SEL_BLOCK)] kept positions per block */
    int32_t reuse_selection;     /* specattn_fused only: 1 = counts, block_counts and kept_mask already hold the
                                    result of an earlier specattn_topp_select / specattn_fused call on these rows
                                    (e.g. one batched call for all layers); the selection phase is skipped */

    /* Chunk-granular selection (Section 4 evaluates with chunks of 16 tokens).  chunk_size 0 or 1: single
       positions.  A power of two >= 2: the row is first reduced to chunk masses - the sum of the chunk's
       entries, taken in fp64 in ascending position order and rounded once to fp32 - and the exact top-p
       selection runs over those; `indices` then holds ascending chunk numbers (chunk c stands for positions
       [c*chunk_size, min((c+1)*chunk_size, len))), idx_capacity and counts are in chunks, thresholds are
       chunk masses.  Needs workspace (specattn_workspace_size(sel, NULL)); not available together with
       emit_physical, block_counts or specattn_fused (SPECATTN_EUNSUPPORTED). */
    int32_t chunk_size;

    /* 0: the exact tau*.  k >= 1: Algorithm 2's value-space bisection with k halvings of [0, max] instead
       (the footnote of Section 3.4: the paper's implementation uses 10); the kept set is {a >= theta_low},
       the bracket end that always keeps mass >= top_p * (row sum), and `thresholds` receives theta_low
       rounded up to fp32.  theta_low = 0 keeps every position of the row.  ROW_NEAR_BOUNDARY then means
       that one of the k comparisons was decided by less than 1e-6 of the row sum.  Needs workspace; not
       available together with block_counts, chunk_size > 1 or specattn_fused (SPECATTN_EUNSUPPORTED). */
    int32_t bisect_iters;

    /* out, optional: the kept set as a bit mask (Algorithm 1 hands the verifier a binary mask per layer):
       [B*H_kv][ceil(n_max / SPECATTN_SEL_BLOCK) * SPECATTN_SEL_BLOCK / 32] words, bit i of word w of a row set
       iff position 32 * w + i is kept; bits at and beyond the row's length are 0.  Together with counts and
       block_counts this is the selection state specattn_fused works from (1 bit per position instead of the 32
       of a list entry per kept position).  Not available with chunk_size > 1, bisect_iters or the split path
       (a workspace handed to a plain selection of few long rows): SPECATTN_EUNSUPPORTED. */
    uint32_t *kept_mask;
} specattn_select_args;

/*
 * Sparse decode attention (Section 3.1.2, Eq. 2-3; Section 3.5).
 *
 * out[b][h_q][t] = softmax over the row's kept positions of
 *                  (q[b][h_q][t] . k[b][h_kv][j]) * sm_scale, times v.
 * All T queries of all G query heads of a kv head share that head's list.
 * A row with count 0 gives out = 0 and lse = -inf.  Accumulation is fp32;
 * `out` is fp32 whatever the input dtype.  Every sum is taken in a fixed order
 * (tiles are assigned to waves and workgroups by the counts alone), so repeated
 * calls on the same inputs give bit-identical out and lse.
 *
 * Shapes: bf16 and fp16 with d = 128 run on the matrix cores for any G = H_q / H_kv (up to 32 query rows
 * G*T per pass; larger groups are taken in equal shares of heads, each streaming the kept K/V
 * again).  fp32, and d = 64, run on a portable kernel limited to G*T <= 64.
 *
 * Dense layers (Section 4 keeps the first layers of the verifier dense): with
 * indices == NULL and counts == NULL every position below seq_lens[b] (n_max
 * when seq_lens is NULL) is attended to, through the same kernels, without
 * any list in memory.  idx_stride_row / idx_capacity are then ignored.
 */
typedef struct specattn_attn_args {
    const void *q;               /* [B][H_q][T][d] */
    const void *k, *v;           /* contiguous: [B][H_kv][n_max][d] via the strides below
                                    paged:      pool [pages][H_kv][page_size][d] */
    specattn_dtype dtype;        /* element type of q, k and v */
    int32_t B, H_q, H_kv, T, d, n_max;
    float sm_scale;              /* <= 0 selects 1/sqrt(d) (Eq. 1) */
    int64_t q_stride_b, q_stride_h, q_stride_t;        /* elements; last dim contiguous */
    int64_t kv_stride_b, kv_stride_h, kv_stride_n;     /* contiguous layout; kv_stride_n >= d */

    const int32_t *page_table;   /* NULL = contiguous layout */
    int32_t page_size, max_pages_per_seq;
    int64_t kv_stride_page;      /* paged: elements between pages; kv_stride_h / kv_stride_n then
                                    address head and in-page token */

    const int32_t *seq_lens;     /* [B] or NULL; used by specattn_fused (selection side) and by dense calls */
    const int32_t *indices;      /* [B*H_kv][idx_stride_row], as written by specattn_topp_select; NULL together
                                    with counts = dense */
    int64_t idx_stride_row;
    const int32_t *counts;       /* [B*H_kv]; values above idx_capacity are clamped to it */
    int32_t idx_capacity;
    int32_t indices_are_physical;/* 1: entries are pool slots (page*page_size + offset) */

    float *out;                  /* [B][H_q][T][d] fp32, contiguous */
    float *lse;                  /* [B][H_q][T] log-sum-exp of the kept scaled scores; optional */
    void *workspace;             /* split partials; 256-byte aligned */
    size_t workspace_bytes;

    /* optional: keys and values of the T tokens being verified (Algorithm 1 feeds the gamma draft
       tokens and the last accepted one through the verifier together).  [B][H_kv][T][d], contiguous,
       same dtype as k/v, 16-byte aligned; both NULL = the cache alone.  They sit behind the cache, are
       never subject to the selection, and are seen causally: query t also attends to new tokens 0..t. */
    const void *k_new, *v_new;

    /* 0 or 1: `indices` holds positions.  A power of two >= 2: `indices` holds chunk numbers as written by a
       chunk-granular specattn_topp_select (counts and idx_capacity in chunks); positions past seq_lens[b]
       in the last chunk are not attended to.  Not available with indices_are_physical or specattn_fused. */
    int32_t chunk_size;

    /* optional: a second copy of the output in the dtype of q/k/v (round to nearest even), [B][H_q][T][d]
       contiguous, 16-byte aligned - what a following projection in that dtype reads.  NULL = not written. */
    void *out_lowp;
} specattn_attn_args;

/*
 * Algorithm 2 as a whole (Section 3.4): top-p selection of the draft attention row of every
 * speculative step, then the union of the kept sets.  Every draft head that feeds a kv head
 * (draft heads h*H_draft/H_kv .. (h+1)*H_draft/H_kv - 1 feed kv head h) adds its rows to the same
 * union, so one ascending list per (sequence, kv head) comes out, ready for
 * specattn_sparse_decode_attn.  Each member row is cut at its own exact tau* (same rules as
 * specattn_topp_select); member rows that are invalid contribute nothing.
 */
typedef struct specattn_union_args {
    const float *probs;          /* [B][H_draft][S][n_max] fp32: row (b, h, s) starts at
                                    b*probs_stride_b + (h*S + s)*probs_stride_row */
    int64_t probs_stride_b;      /* elements */
    int64_t probs_stride_row;    /* elements between consecutive (head, step) rows, >= n_max */
    int32_t B, H_draft, S, H_kv, n_max;   /* S = gamma draft steps; H_draft % H_kv == 0 */
    const int32_t *seq_lens;     /* [B] common valid length, or NULL for n_max */
    float top_p;                 /* p in (0, 1] */

    int32_t *indices;            /* out [B*H_kv][idx_stride_row] ascending positions of the union */
    int64_t idx_stride_row;
    int32_t idx_capacity;
    int32_t *counts;             /* out [B*H_kv] TRUE size of the union, even when > idx_capacity */
    uint32_t *row_flags;         /* out, optional: INVALID if every member row is invalid (count 0),
                                    NEAR_BOUNDARY if any valid member row is, OVERFLOW as for the selection */
    float *member_thresholds;    /* out, optional: [B*H_draft*S] tau* of every member row */
    int32_t *member_counts;      /* out, optional: [B*H_draft*S] kept count of every member row */

    const int32_t *page_table;   /* optional paged output, as in specattn_select_args */
    int32_t page_size, max_pages_per_seq, emit_physical;
} specattn_union_args;

/* workspace: specattn_union_workspace_size(args) bytes, 256-byte aligned. */
specattn_status specattn_topp_select_union(const specattn_union_args *args, void *workspace,
                                           size_t workspace_bytes, void *stream);
size_t specattn_union_workspace_size(const specattn_union_args *args);

/* Selection alone.  The plain selection (single positions, exact tau*) never needs a workspace: without one
   every row is handled by one workgroup.  When specattn_workspace_size(sel, NULL) is not 0 for it (few, long
   rows) and a workspace of that size is given, each row is split over many workgroups instead; the results
   are the same.  The chunk and bisection modes need their workspace (SPECATTN_EWORKSPACE otherwise). */
specattn_status specattn_topp_select(const specattn_select_args *sel, void *workspace,
                                     size_t workspace_bytes, void *stream);

/*
 * Offline layer mapping (Section 3.3, Eq. 4; Appendix B, Algorithm 3): which draft layer's attention a verifier
 * layer's selection is taken from.  Run once per model pair on attention rows collected from a representative
 * data set; nothing of it runs during decoding.
 *
 * specattn_layer_similarity: attn_draft [m][rows][L], attn_verifier [n][rows][L], fp32 probabilities (>= 0;
 * positions a row cannot see hold 0), contiguous, device memory; row r of every layer of both models belongs to
 * the same query of the same text.  S [m][n] fp64 (device, out): S[i*n + j] = -(1/rows) * sum_r
 * D_KL(attn_verifier[j][r] || attn_draft[i][r]) - Eq. 4 averaged over the rows (natural logarithm; a verifier
 * entry of 0 adds nothing; a draft entry of 0 under verifier mass gives -infinity).  Workspace:
 * specattn_layer_similarity_workspace_size bytes, 256-byte aligned.  m*n <= 65535.
 *
 * specattn_layer_map: S [m][n] fp64 as above (device); f [n] int32 (device, out): the non-decreasing map from
 * verifier layer j to draft layer f[j] (0-based) that maximises sum_j S[f[j]*n + j] (draft layers may be
 * skipped or serve several verifier layers); *total (device, out) that maximum.  Among equal maxima the
 * recurrence of Algorithm 3 keeps the smallest draft index at every step.  m <= 1024, n <= 65535.  Workspace:
 * specattn_layer_map_workspace_size bytes, 256-byte aligned.
 *
 * Both: asynchronous on stream; SPECATTN_EINVAL / SPECATTN_ESHAPE / SPECATTN_EWORKSPACE before anything is
 * launched; the size queries return 0 for sizes the calls reject.
 */
size_t specattn_layer_similarity_workspace_size(int32_t m, int32_t n, int32_t rows, int32_t L);
specattn_status specattn_layer_similarity(const float *attn_draft, const float *attn_verifier, int32_t m, int32_t n,
                                          int32_t rows, int32_t L, double *S, void *workspace,
                                          size_t workspace_bytes, void *stream);
size_t specattn_layer_map_workspace_size(int32_t m, int32_t n);
specattn_status specattn_layer_map(const double *S, int32_t m, int32_t n, int32_t *f, double *total,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* Attention alone, over an index list already in device memory. */
specattn_status specattn_sparse_decode_attn(const specattn_attn_args *attn, void *stream);

/*
 * For callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same computation, arguments, checks and results as
 * specattn_sparse_decode_attn, except that attn->workspace / attn->workspace_bytes are ignored: the split
 * partials live in a buffer of SPECATTN_STATIC_SCRATCH_BYTES that is part of the library image (one copy per
 * GPU, held until the process ends).  The call allocates and frees nothing.  A call that cannot run in that
 * much is refused with SPECATTN_EWORKSPACE before anything is launched (batches of more than 512 rows run in
 * launches of 512 rows where the size specattn_workspace_size(NULL, attn) asks for would let them take 1536).  The buffer belongs to the device that is current when the call is made; `stream` must be a
 * stream of that device.  All calls on one GPU share the buffer: calls that overlap on one GPU (different
 * streams, or different threads without stream ordering between them) race on it and give wrong results;
 * calls ordered on one stream are safe, and nothing has to be cleared between them.
 */
specattn_status specattn_sparse_decode_attn_static(const specattn_attn_args *attn, void *stream);

/*
 * Selection + attention without an index list (Algorithm 1: the masks of all layers are created from the draft
 * model's attention before the verifier runs, and each verifier layer attends under its mask; Section 3.5: the
 * paper's implementation converts that mask to an index structure before its attention kernel can use it - this
 * call removes the conversion and the list's trip through memory).  The selection phase writes tau*, counts,
 * per-block counts and the kept-position mask (1 bit per position; into sel->thresholds / sel->block_counts /
 * sel->kept_mask when given, else into the workspace); the attention waves turn the mask words of a tile into
 * its 32 row addresses on chip.  sel->indices is ignored; attn->indices / attn->counts are ignored
 * (sel->counts is written and used).  attn->workspace serves both phases.
 * The kept set stays on chip for bf16 and fp16 with d = 128 and single positions, contiguous or page-table
 * layouts.  For what the two separate calls take beyond that - fp32, d = 64, chunk-granular selection
 * (sel->chunk_size > 1; attn->chunk_size is ignored) - the same entry point runs the selection into a list inside
 * attn->workspace and the attention over that list: same results, one call, nothing caller-visible in between;
 * reuse_selection, block_counts and kept_mask are not available then (SPECATTN_EUNSUPPORTED).  There is never a
 * caller-visible list, so attn->indices_are_physical does not apply (SPECATTN_EUNSUPPORTED; pass the page table).
 * What the on-chip route saves is memory (4 KiB of mask per row of 32768 positions instead of a list of up to
 * 128 KiB) and the list's write and read; decoding the mask costs the attention waves about as much time as the
 * selection saves, so where speed alone matters the two separate calls are the ones to use.
 */
specattn_status specattn_fused(const specattn_select_args *sel, const specattn_attn_args *attn,
                               void *stream);

/* Bytes of workspace needed: selection alone (attn NULL), attention alone (sel NULL), or the
   fused call (both).  0 is returned for invalid arguments. */
size_t specattn_workspace_size(const specattn_select_args *sel, const specattn_attn_args *attn);

/*
 * CSR form of the lists a selection call wrote (Section 3.5: in the paper the selection reaches the attention
 * kernel as a CSR structure).  indices [rows][idx_stride] and counts [rows] as written by specattn_topp_select /
 * specattn_topp_select_union (positions, chunk numbers or pool slots alike); counts above idx_capacity count as
 * idx_capacity, negative ones as 0.  indptr [rows + 1] (device, int64, out): indptr[0] = 0, indptr[r + 1] =
 * indptr[r] + length of list r.  packed (device, out, optional - NULL skips it): the entries of all lists back to
 * back, list r at packed[indptr[r] ...]; the caller sizes it for rows * idx_capacity entries or for the sum of the
 * counts it knows.  Asynchronous on stream; SPECATTN_EINVAL / SPECATTN_ESHAPE before anything is launched.
 */
specattn_status specattn_lists_to_csr(const int32_t *indices, int64_t idx_stride_row, int32_t idx_capacity,
                                      const int32_t *counts, int32_t rows, int64_t *indptr, int32_t *packed,
                                      void *stream);

/*
 * Debugging aid: checks, on the device and without touching K/V, the index lists that
 * specattn_sparse_decode_attn(attn) would read (Section 3.5: the selection reaches the attention kernel as an
 * index structure).  Counted as violations: a negative count or sequence length, an entry outside
 * [0, seq_len) (chunk lists: outside the sequence's chunks), a list that is not strictly ascending, a page-table
 * entry of a listed position that is negative or beyond the pool; for physical lists, an entry outside
 * [0, pool_slots).  pool_slots = pages * page_size of the pool, or 0 to skip the pool-size checks.
 * *n_bad (device int32) receives the number of violations; the caller reads it after synchronising.
 * Dense calls (no list) have nothing to check: SPECATTN_EINVAL.
 */
specattn_status specattn_check_lists(const specattn_attn_args *attn, int64_t pool_slots, int32_t *n_bad, void *stream);

/*
 * Measurement aid, not a step of the method: reads `bytes` of device memory at `src` once with plain
 * 16-byte-per-lane loads and discards them (`sink`, optional, is a device word that is almost never
 * written; it only keeps the loads alive).  Timed by the caller, it gives the read rate this machine
 * reaches, which is what the gather of selected K/V rows (Section 3.5) is compared against.
 * src and bytes must be multiples of 16: SPECATTN_EALIGN otherwise; NULL or 0: SPECATTN_EINVAL.
 */
specattn_status specattn_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

/*
 * Optional set-up of the current device: sets the attributes the attention kernels need (their LDS size) and
 * looks up the built-in scratch buffer.  Every attention entry point does the same on its first call on a
 * device; a caller that wants to record its FIRST attention call on a device in a HIP graph calls this before
 * the capture starts (setting kernel attributes is not a stream operation and is not captured).  Safe to call
 * any number of times, from any thread.  SPECATTN_OK or SPECATTN_EHIP.
 */
specattn_status specattn_init(void);

/* Text of the calling thread's last error ("" if none).  Never NULL. */
const char *specattn_last_error(void);

/* ABI version: major * 1000 + minor. */
int specattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECATTN_H */

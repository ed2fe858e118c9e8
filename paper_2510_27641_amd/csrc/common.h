// Shared host-side declarations of the HIP library (internal; the public ABI is include/specattn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "specattn.h"

namespace specattn {

// thread-local error text behind specattn_last_error()
void set_error(const char *fmt, ...);
void clear_error();

// number of compute units of the current device (256 when no device can be queried)
int cu_count();

// records a failed launch in the error text; returns SPECATTN_EHIP or SPECATTN_OK
specattn_status check_launch(const char *what);

// ---- selection -----------------------------------------------------------------------------
// Per-block kept counts for the fused path: block_counts[r][blk] = number kept among positions
// [blk*SEL_BLOCK, (blk+1)*SEL_BLOCK) of row r.
constexpr int SEL_BLOCK = 1024;

struct SelectLaunch {
    const float *probs;
    int64_t stride_b, stride_h;
    int B, H_kv, n_max;
    const int32_t *seq_lens;
    float top_p;
    int32_t *indices;        // may be null (fused path)
    int64_t idx_stride;
    int idx_capacity;
    int32_t *counts;
    float *thresholds;       // may be null
    uint32_t *row_flags;     // may be null
    const int32_t *page_table;
    int page_shift;          // log2(page_size)
    int max_pages;
    int emit_physical;
    int32_t *block_counts;   // may be null; [rows][blocks_per_row]
    int blocks_per_row;
#ifdef SPECATTN_TIMING
    long long *timing;
#endif
};
specattn_status launch_select(const SelectLaunch &a, hipStream_t stream);

// ---- attention -----------------------------------------------------------------------------
struct AttnLaunch {
    const void *q, *k, *v;
    int dtype;               // specattn_dtype
    int B, H_q, H_kv, T, d, n_max;
    float sm_scale;
    int64_t q_stride_b, q_stride_h, q_stride_t;
    int64_t kv_stride_b, kv_stride_h, kv_stride_n;
    const int32_t *page_table;
    int page_shift, max_pages;
    int64_t kv_stride_page;
    const int32_t *indices;
    int64_t idx_stride;
    const int32_t *counts;
    int idx_capacity;
    int indices_are_physical;
    int dense;               // 1: no list; every position below the sequence length is attended to
    float *out;
    float *lse;              // may be null
    void *workspace;
    size_t workspace_bytes;
    // fused path: the list is rebuilt on chip from probs / tau / block counts
    const float *probs;      // null = unfused
    int64_t probs_stride_b, probs_stride_h;
    const int32_t *seq_lens;
    const float *tau;
    const int32_t *block_counts;
    int blocks_per_row;
};
// Number of positions row r attends to: the kept count (clamped to the list capacity), or the
// sequence length when there is no list.
__device__ __forceinline__ int attn_row_count(const AttnLaunch &a, int r)
{
    if (a.dense) {
        const int len = a.seq_lens ? a.seq_lens[r / a.H_kv] : a.n_max;
        return len < 0 ? 0 : (len > a.n_max ? a.n_max : len);
    }
    const int c = a.counts[r];
    return c < 0 ? 0 : (c > a.idx_capacity ? a.idx_capacity : c);
}

// number of splits per row the attention launch will use for this shape
int attn_num_splits(int rows, int idx_capacity);
size_t attn_workspace_bytes(int rows, int G, int T, int d, int idx_capacity);
specattn_status launch_attn(const AttnLaunch &a, hipStream_t stream);

// matrix-core variant (bf16, d = 128, G*T <= 32)
bool attn_mfma_supported(const AttnLaunch &a);
size_t attn_mfma_workspace_bytes(int rows, int G, int T);
specattn_status launch_attn_mfma(const AttnLaunch &a, hipStream_t stream);

}  // namespace specattn

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
    int n_tokens;            // positions behind a row: seq_lens counts these (n_max << chunk_shift at most)
    int chunk_shift;         // log2 of the chunk size when the row holds chunk masses, else 0
    uint32_t *kept_mask;     // may be null; [rows][blocks_per_row * SEL_BLOCK / 32]: bit i of word w = position 32 w + i kept
};
specattn_status launch_select(const SelectLaunch &a, hipStream_t stream);
// Few long rows: each row split over many workgroups (thresholds only; the list comes from the mask and
// compaction passes).  `scratch` holds select_multi_wg_bytes(rows, n_max).
bool select_multi_wg_preferred(int rows, int n);
size_t select_multi_wg_bytes(int rows, int n);
specattn_status launch_select_multi_wg(const SelectLaunch &a, void *scratch, float *tau, int32_t *valid, uint32_t *flags,
                                       hipStream_t stream);
// mass[r][c] = fp32(sum in fp64 of the entries of chunk c of row r), NaN if the chunk holds an invalid entry
specattn_status launch_chunk_masses(const float *probs, int64_t stride_b, int64_t stride_h, int B, int H, int n_tokens,
                                    const int32_t *seq_lens, int chunk_shift, int n_chunks, float *mass,
                                    hipStream_t stream);

// union of the per-step selections (Algorithm 2 as a whole)
size_t union_workspace_bytes(int B, int H_kv, int M, int n_max);
specattn_status launch_union(const specattn_union_args *u, void *workspace, hipStream_t stream);
// mask + compaction passes alone, for rows whose thresholds are already known; `scratch` holds the block
// counts and ballots (the tail of union_workspace_bytes)
specattn_status launch_threshold_union(const float *probs, int64_t stride_b, int64_t stride_m, int B, int H_kv, int M,
                                       int n_max, const int32_t *seq_lens, const float *tau, const int32_t *mcounts,
                                       const uint32_t *mflags, void *scratch, int32_t *indices, int64_t idx_stride,
                                       int idx_capacity, int32_t *counts, uint32_t *row_flags,
                                       const int32_t *page_table, int page_size, int max_pages, int emit_physical,
                                       hipStream_t stream);
// Algorithm 2's fixed-iteration bisection: tau[r] = theta_low rounded up to fp32, valid[r] = 0/1, flags[r]
specattn_status launch_bisect_thresholds(const SelectLaunch &a, int iters, float *tau, int32_t *valid, uint32_t *flags,
                                         hipStream_t stream);

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
    int chunk_shift;         // > 0: list entries are chunk numbers of 1 << chunk_shift positions each
    const void *k_new, *v_new;   // [B][H_kv][T][d] new tokens behind the cache, or null
    int g_first, g_count;        // this launch handles query heads g_first .. g_first + g_count - 1 of every kv head's
                                 // group (g_count 0: all of them)
    float *out;
    void *out_lowp;          // may be null: the output once more in the input dtype
    float *lse;              // may be null
    void *workspace;
    size_t workspace_bytes;
    const int32_t *seq_lens;
    // fused path: the kept positions come from the selection's mask (one bit per position) and per-block counts
    const uint32_t *kept_mask;   // null = unfused; [rows][blocks_per_row * SEL_BLOCK / 32]
    const int32_t *block_counts; // [rows][blocks_per_row]
    int blocks_per_row;
};
__device__ __forceinline__ int attn_group_heads(const AttnLaunch &a) { return a.g_count ? a.g_count : a.H_q / a.H_kv; }
// query head behind head gh of this launch's share of kv head h's group
__device__ __forceinline__ int attn_query_head(const AttnLaunch &a, int h, int gh)
{
    return h * (a.H_q / a.H_kv) + a.g_first + gh;
}

// Inclusive prefix sum over the 64 lanes of a wave on the vector ALU (no LDS traffic): shifts by 1, 2, 4, 8 inside
// each row of 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);    // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);    // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);    // row_bcast:31 into rows 2 and 3
    return v;
}

// Number of positions row r attends to: the kept count (clamped to the list capacity), or the
// sequence length when there is no list.  With a chunk list: the kept chunks' positions, less the
// part of the last kept chunk that lies past the sequence length (the list is ascending, so only
// the last entry can be the partial chunk).
__device__ __forceinline__ int attn_row_count(const AttnLaunch &a, int r)
{
    int len = a.n_max;
    if (a.dense || a.chunk_shift) {
        len = a.seq_lens ? a.seq_lens[r / a.H_kv] : a.n_max;
        len = len < 0 ? 0 : (len > a.n_max ? a.n_max : len);
    }
    if (a.dense) return len;
    int c = a.counts[r];
    c = c < 0 ? 0 : (c > a.idx_capacity ? a.idx_capacity : c);
    if (!a.chunk_shift || c == 0) return c;
    const int last = a.indices[(int64_t)r * a.idx_stride + c - 1];
    const int end = (last + 1) << a.chunk_shift;
    int cut = end > len ? end - len : 0;
    cut = cut > (1 << a.chunk_shift) ? (1 << a.chunk_shift) : cut;
    return (c << a.chunk_shift) - cut;
}

// Position behind list rank jj of a row whose list starts at idx.
__device__ __forceinline__ int attn_list_pos(const AttnLaunch &a, const int32_t *idx, int jj)
{
    if (a.dense) return jj;
    if (a.chunk_shift) return (idx[jj >> a.chunk_shift] << a.chunk_shift) | (jj & ((1 << a.chunk_shift) - 1));
    return idx[jj];
}

// The same for N ranks at once, written so that all N loads are in flight together (a branch per rank would make
// every load wait for the one before).
template <int N>
__device__ __forceinline__ void attn_list_pos_n(const AttnLaunch &a, const int32_t *idx, const int (&jj)[N], int (&pos)[N])
{
    if (a.dense) {
#pragma unroll
        for (int i = 0; i < N; ++i) pos[i] = jj[i];
        return;
    }
    const int cs = a.chunk_shift, low = (1 << cs) - 1;
    int v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = idx[jj[i] >> cs];
#pragma unroll
    for (int i = 0; i < N; ++i) pos[i] = (v[i] << cs) | (jj[i] & low);
}
// In two steps, for callers that have other loads to issue before they need the positions: the raw list words
// first (nothing waits), the positions from them later.  Not for dense calls (no list).
template <int N>
__device__ __forceinline__ void attn_list_request_n(const AttnLaunch &a, const int32_t *idx, const int (&jj)[N], int (&raw)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) raw[i] = a.dense ? jj[i] : idx[jj[i] >> a.chunk_shift];
}
template <int N>
__device__ __forceinline__ void attn_list_finish_n(const AttnLaunch &a, const int (&jj)[N], const int (&raw)[N], int (&pos)[N])
{
    const int cs = a.chunk_shift, low = (1 << cs) - 1;
#pragma unroll
    for (int i = 0; i < N; ++i) pos[i] = a.dense ? jj[i] : ((raw[i] << cs) | (jj[i] & low));
}

__device__ __forceinline__ float ld_elem(const void *p, int64_t i, int dtype)
{
    if (dtype == SPECATTN_BF16) return __uint_as_float((uint32_t) static_cast<const uint16_t *>(p)[i] << 16);
    if (dtype == SPECATTN_F16) return (float) static_cast<const _Float16 *>(p)[i];
    return static_cast<const float *>(p)[i];
}

// Element i of the optional second output copy, in the input dtype (round to nearest even).
__device__ __forceinline__ void st_lowp(void *p, int64_t i, float x, int dtype)
{
    if (dtype == SPECATTN_BF16) {
        uint32_t u = __float_as_uint(x);
        u = ((u & 0x7fffffffu) > 0x7f800000u) ? (u | 0x00400000u) : (u + 0x7fffu + ((u >> 16) & 1u));     // NaN stays NaN
        static_cast<uint16_t *>(p)[i] = (uint16_t)(u >> 16);
    } else if (dtype == SPECATTN_F16) {
        static_cast<_Float16 *>(p)[i] = (_Float16)x;
    } else {
        static_cast<float *>(p)[i] = x;
    }
}

// Scores of query row (b, hq, t) against the keys of new tokens 0..t (unscaled dot products), computed
// by all threads of a workgroup of blockDim.x = max(64, d) threads together; `red` is LDS scratch of
// 2 * SPECATTN_MAX_T floats.  Every thread returns with all t + 1 values.  Contains a barrier.
__device__ __forceinline__ void tail_dots(const AttnLaunch &a, int b, int hq, int t, float *red,
                                          float (&dots)[SPECATTN_MAX_T])
{
    const int e = threadIdx.x, lane = e & 63, wave = e >> 6;
    const int hk = hq / (a.H_q / a.H_kv);
    const int64_t qoff = (int64_t)b * a.q_stride_b + (int64_t)hq * a.q_stride_h + (int64_t)t * a.q_stride_t;
    const int64_t noff = ((int64_t)b * a.H_kv + hk) * a.T * a.d;
    const float qe = e < a.d ? ld_elem(a.q, qoff + e, a.dtype) : 0.0f;
#pragma unroll
    for (int p = 0; p < SPECATTN_MAX_T; ++p) {
        float x = (p <= t && e < a.d) ? qe * ld_elem(a.k_new, noff + (int64_t)p * a.d + e, a.dtype) : 0.0f;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
        if (lane == 0 && wave < 2) red[wave * SPECATTN_MAX_T + p] = x;
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < SPECATTN_MAX_T; ++p)
        dots[p] = red[p] + (blockDim.x > 64 ? red[SPECATTN_MAX_T + p] : 0.0f);
}

// number of splits per row the attention launch will use for this shape
int attn_num_splits(int rows, int idx_capacity);
size_t attn_workspace_bytes(int rows, int G, int T, int d, int idx_capacity);
size_t attn_workspace_min_bytes(int rows, int G, int T, int d, int idx_capacity);   // the least the call runs with
specattn_status launch_attn(const AttnLaunch &a, hipStream_t stream);

// counts the index-list violations of an attention call into *n_bad (device memory)
specattn_status launch_check_lists(const AttnLaunch &a, int64_t pool_slots, int32_t *n_bad, hipStream_t stream);

// CSR row pointers (and, optionally, the packed entries) of padded index lists
specattn_status launch_csr(const int32_t *indices, int64_t idx_stride, const int32_t *counts, int rows, int capacity,
                           int64_t *indptr, int32_t *packed, hipStream_t stream);

// matrix-core variant (bf16 / fp16, d = 128)
constexpr int ATTN_MFMA_WAVES = 8;        // waves per workgroup (one workgroup per CU: two workgroups of four waves
                                          // do not share a CU's memory pipeline evenly - the one dispatched later
                                          // issues its gathers only when the earlier one's waves are waiting)
constexpr int ATTN_MFMA_MAX_ROWS = 512;   // rows per launch every call can count on (larger batches run as several launches); most kv heads
constexpr int ATTN_MFMA_MAX_ROWS_LIST = 1536;   // rows per launch when the workspace was sized for them
bool attn_mfma_supported(const AttnLaunch &a);
specattn_status attn_mfma_configure();    // one-time kernel attributes on the current device
specattn_status attn_generic_configure(); // the same for the fp32-ALU variants
size_t attn_mfma_workspace_bytes(int rows, int G, int T);       // what lets every launch take as many rows as it can
size_t attn_mfma_workspace_min_bytes(int rows, int G, int T);   // the least a call runs with
specattn_status launch_attn_mfma(const AttnLaunch &a, hipStream_t stream);

}  // namespace specattn

// Algorithm 2 as a whole (Section 3.4): the draft model's attention row of every speculative step
// (and of every draft head that feeds a kv head) is cut at its own exact top-p threshold, and the
// union of the kept sets is emitted as one ascending list per (sequence, kv head).
//
// Three launches: the selection kernel in threshold-only mode over all member rows; a mask pass in
// which every workgroup compares one block of positions of all member rows with their thresholds
// and leaves the kept bits (as wave ballots) and the block's count; a compaction pass that numbers
// the kept positions from the block counts and the ballots alone.
#include <hip/hip_runtime.h>

#include "common.h"

namespace specattn {
namespace {

constexpr int U_THREADS = 256;
constexpr int U_WAVES = U_THREADS / 64;
constexpr int U_ITERS = 4;                                  // float4 loads per thread and member row
constexpr int U_BLOCK = U_THREADS * 4 * U_ITERS;            // 4096 positions per workgroup
constexpr int U_WORDS = U_ITERS * U_WAVES * 4;              // ballots per block: [iter][wave][component]

struct UnionLaunch {
    const float *probs;
    int64_t stride_b, stride_m;     // elements between sequences / between consecutive member rows
    int B, H_kv, M, n_max;          // M member rows per (sequence, kv head), consecutive
    const int32_t *seq_lens;
    const float *tau;               // [B * H_kv * M] thresholds of the member rows
    const int32_t *mcounts;         // [B * H_kv * M] kept counts of the member rows (0 = contributes nothing)
    const uint32_t *mflags;         // [B * H_kv * M]
    int32_t *block_counts;          // [rows][blocks]
    unsigned long long *ballots;    // [rows][blocks][U_WORDS]
    int blocks;
    int32_t *indices;
    int64_t idx_stride;
    int idx_capacity;
    int32_t *counts;
    uint32_t *row_flags;
    const int32_t *page_table;
    int page_shift, max_pages, emit_physical;
};

// one workgroup per (row, block): kept bits of positions [blk * U_BLOCK, (blk + 1) * U_BLOCK) of row r.
// Position of (iter, thread, component): blk * U_BLOCK + iter * U_THREADS * 4 + thread * 4 + component.
__global__ __launch_bounds__(U_THREADS) void union_mask_kernel(UnionLaunch a)
{
    __shared__ int wave_cnt[U_WAVES];
    const int r = blockIdx.x / a.blocks, blk = blockIdx.x - r * a.blocks;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int len = a.seq_lens ? a.seq_lens[b] : a.n_max;
    len = len < 0 ? 0 : (len > a.n_max ? a.n_max : len);
    const float *rows = a.probs + (int64_t)b * a.stride_b + (int64_t)h * a.M * a.stride_m;
    const int64_t m0 = (int64_t)r * a.M;
    unsigned keep[U_ITERS] = {0u, 0u, 0u, 0u};                // 4 bits per iteration
    for (int m = 0; m < a.M; ++m) {
        if (a.mcounts[m0 + m] <= 0) continue;                 // invalid member rows keep nothing (uniform)
        const int t = __float_as_int(a.tau[m0 + m]);         // > 0 for every valid row: zeros are never kept
        const float *row = rows + (int64_t)m * a.stride_m;
        const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
#pragma unroll
        for (int it = 0; it < U_ITERS; ++it) {
            const int p = blk * U_BLOCK + it * U_THREADS * 4 + tid * 4;
            float4 v = make_float4(-1.f, -1.f, -1.f, -1.f);   // positions past the row's end: below any threshold
            if (p + 3 < len && aligned) {
                v = *reinterpret_cast<const float4 *>(row + p);
            } else {
                if (p < len) v.x = row[p];
                if (p + 1 < len) v.y = row[p + 1];
                if (p + 2 < len) v.z = row[p + 2];
                if (p + 3 < len) v.w = row[p + 3];
            }
            // compared as integers, like the selection itself: non-negative floats order like their bit
            // patterns; -0.0 (the only signed value a valid row can hold) counts as zero
            auto bits = [](float f) { const int i = __float_as_int(f); return i == (int)0x80000000 ? 0 : i; };
            const int x = bits(v.x), y = bits(v.y), z = bits(v.z), w = bits(v.w);
            keep[it] |= (x >= t ? 1u : 0u) | (y >= t ? 2u : 0u) | (z >= t ? 4u : 0u) | (w >= t ? 8u : 0u);
        }
    }
    unsigned long long *words = a.ballots + ((int64_t)r * a.blocks + blk) * U_WORDS;
    int cnt = 0;
#pragma unroll
    for (int it = 0; it < U_ITERS; ++it) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned long long w = __ballot((keep[it] >> c) & 1u);
            cnt += __popcll(w);
            if (lane == 0) words[(it * U_WAVES + wave) * 4 + c] = w;
        }
    }
    if (lane == 0) wave_cnt[wave] = cnt;
    __syncthreads();
    if (tid == 0) {
        int total = 0;
        for (int w = 0; w < U_WAVES; ++w) total += wave_cnt[w];
        a.block_counts[(int64_t)r * a.blocks + blk] = total;
    }
}

// one workgroup per (row, block): writes the positions of its block at their rank in the row's list.
__global__ __launch_bounds__(U_THREADS) void union_compact_kernel(UnionLaunch a)
{
    __shared__ int part[U_WAVES][2];
    __shared__ unsigned long long words[U_WORDS];
    __shared__ int group_base[U_ITERS * U_WAVES];
    const int r = blockIdx.x / a.blocks, blk = blockIdx.x - r * a.blocks;
    const int b = r / a.H_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // kept before this block, and in the whole row
    int before = 0, total = 0;
    for (int k = tid; k < a.blocks; k += U_THREADS) {
        const int c = a.block_counts[(int64_t)r * a.blocks + k];
        total += c;
        if (k < blk) before += c;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        before += __shfl_xor(before, off, 64);
        total += __shfl_xor(total, off, 64);
    }
    if (lane == 0) { part[wave][0] = before; part[wave][1] = total; }
    if (tid < U_WORDS) words[tid] = a.ballots[((int64_t)r * a.blocks + blk) * U_WORDS + tid];
    __syncthreads();
    before = total = 0;
#pragma unroll
    for (int w = 0; w < U_WAVES; ++w) { before += part[w][0]; total += part[w][1]; }
    if (tid == 0) {                                           // list position of every (iter, wave) group
        int run = before;
        for (int gidx = 0; gidx < U_ITERS * U_WAVES; ++gidx) {
            group_base[gidx] = run;
            for (int c = 0; c < 4; ++c) run += __popcll(words[gidx * 4 + c]);
        }
    }
    if (blk == 0 && tid == 0) {
        a.counts[r] = total;
        if (a.row_flags) {
            uint32_t any_valid = 0, near = 0;
            for (int m = 0; m < a.M; ++m) {
                const uint32_t f = a.mflags[(int64_t)r * a.M + m];
                if (!(f & SPECATTN_ROW_INVALID)) { any_valid = 1; near |= f & SPECATTN_ROW_NEAR_BOUNDARY; }
            }
            uint32_t f = any_valid ? near : SPECATTN_ROW_INVALID;
            if (total > a.idx_capacity) f |= SPECATTN_ROW_OVERFLOW;
            a.row_flags[r] = f;
        }
    }
    __syncthreads();
    int32_t *out = a.indices + (int64_t)r * a.idx_stride;
    const int32_t *ptab = (a.emit_physical && a.page_table) ? a.page_table + (int64_t)b * a.max_pages : nullptr;
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int it = 0; it < U_ITERS; ++it) {
        const unsigned long long *w = words + (it * U_WAVES + wave) * 4;
        int o = group_base[it * U_WAVES + wave] +
                __popcll(w[0] & below) + __popcll(w[1] & below) + __popcll(w[2] & below) + __popcll(w[3] & below);
        const int p = blk * U_BLOCK + it * U_THREADS * 4 + tid * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if ((w[c] >> lane) & 1ull) {
                if (o < a.idx_capacity) {
                    const int pos = p + c;
                    out[o] = ptab ? ((ptab[pos >> a.page_shift] << a.page_shift) | (pos & ((1 << a.page_shift) - 1))) : pos;
                }
                ++o;
            }
        }
    }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t union_blocks(int n_max) { return ((size_t)n_max + U_BLOCK - 1) / U_BLOCK; }

size_t union_workspace_bytes(int B, int H_kv, int M, int n_max)
{
    const size_t rows = (size_t)B * H_kv, members = rows * M, blocks = union_blocks(n_max);
    return 3 * align256(members * 4) + align256(rows * blocks * 4) + align256(rows * blocks * U_WORDS * 8);
}

// The mask and compaction passes for rows whose member thresholds are known.
specattn_status launch_threshold_union(const float *probs, int64_t stride_b, int64_t stride_m, int B, int H_kv, int M,
                                       int n_max, const int32_t *seq_lens, const float *tau, const int32_t *mcounts,
                                       const uint32_t *mflags, void *scratch, int32_t *indices, int64_t idx_stride,
                                       int idx_capacity, int32_t *counts, uint32_t *row_flags,
                                       const int32_t *page_table, int page_size, int max_pages, int emit_physical,
                                       hipStream_t stream)
{
    const size_t rows = (size_t)B * H_kv, blocks = union_blocks(n_max);
    char *ws = static_cast<char *>(scratch);
    UnionLaunch a{};
    a.probs = probs; a.stride_b = stride_b; a.stride_m = stride_m;
    a.B = B; a.H_kv = H_kv; a.M = M; a.n_max = n_max;
    a.seq_lens = seq_lens;
    a.tau = tau; a.mcounts = mcounts; a.mflags = mflags;
    a.block_counts = reinterpret_cast<int32_t *>(ws);
    a.ballots = reinterpret_cast<unsigned long long *>(ws + align256(rows * blocks * 4));
    a.blocks = (int)blocks;
    a.indices = indices; a.idx_stride = idx_stride; a.idx_capacity = idx_capacity;
    a.counts = counts; a.row_flags = row_flags;
    a.page_table = page_table; a.max_pages = max_pages; a.emit_physical = emit_physical;
    a.page_shift = 0;
    if (page_table) while ((1 << a.page_shift) < page_size) ++a.page_shift;
    const dim3 grid((unsigned)(blocks * rows));
    hipLaunchKernelGGL(union_mask_kernel, grid, dim3(U_THREADS), 0, stream, a);
    specattn_status st = check_launch("union_mask_kernel");
    if (st != SPECATTN_OK) return st;
    hipLaunchKernelGGL(union_compact_kernel, grid, dim3(U_THREADS), 0, stream, a);
    return check_launch("union_compact_kernel");
}

// workspace: [member tau][member counts][member flags][block counts][ballots]
specattn_status launch_union(const specattn_union_args *u, void *workspace, hipStream_t stream)
{
    const int per = u->H_draft / u->H_kv, M = per * u->S;
    const size_t members = (size_t)u->B * u->H_kv * M;
    char *ws = static_cast<char *>(workspace);
    float *tau = u->member_thresholds ? u->member_thresholds : reinterpret_cast<float *>(ws);
    ws += align256(members * 4);
    int32_t *mcounts = u->member_counts ? u->member_counts : reinterpret_cast<int32_t *>(ws);
    ws += align256(members * 4);
    uint32_t *mflags = reinterpret_cast<uint32_t *>(ws);
    ws += align256(members * 4);

    SelectLaunch s{};                                         // every member row on its own, thresholds only
    s.probs = u->probs;
    s.stride_b = u->probs_stride_b;
    s.stride_h = u->probs_stride_row;
    s.B = u->B;
    s.H_kv = u->H_draft * u->S;
    s.n_max = u->n_max;
    s.n_tokens = u->n_max;
    s.seq_lens = u->seq_lens;
    s.top_p = u->top_p;
    s.counts = mcounts;
    s.thresholds = tau;
    s.row_flags = mflags;
    const specattn_status st = launch_select(s, stream);
    if (st != SPECATTN_OK) return st;
    return launch_threshold_union(u->probs, u->probs_stride_b, u->probs_stride_row, u->B, u->H_kv, M, u->n_max,
                                  u->seq_lens, tau, mcounts, mflags, ws, u->indices, u->idx_stride_row, u->idx_capacity,
                                  u->counts, u->row_flags, u->page_table, u->page_size, u->max_pages_per_seq,
                                  u->emit_physical, stream);
}

}  // namespace specattn

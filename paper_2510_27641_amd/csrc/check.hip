// Debugging aid: the checks a bounds-asserting build of the attention kernels would make on its
// index lists, as a separate pass that reads no K/V (Section 3.5 hands the selection to the attention
// kernel as an index structure; a wrong entry there becomes a wild gather).  Violations are counted in
// device memory; nothing traps.
#include <hip/hip_runtime.h>

#include "common.h"

namespace specattn {
namespace {

__global__ void zero_word_kernel(int32_t *p) { *p = 0; }

// one workgroup per row
__global__ __launch_bounds__(256) void check_lists_kernel(AttnLaunch a, int64_t pool_slots, int32_t *n_bad)
{
    const int r = blockIdx.x, b = r / a.H_kv;
    int len = a.seq_lens ? a.seq_lens[b] : a.n_max;
    int bad = 0;
    if (len < 0 || len > a.n_max) { if (threadIdx.x == 0) ++bad; len = len < 0 ? 0 : a.n_max; }
    const int raw = a.counts[r];
    if (raw < 0 && threadIdx.x == 0) ++bad;
    const int c = raw < 0 ? 0 : (raw > a.idx_capacity ? a.idx_capacity : raw);       // what the kernels read
    const int32_t *idx = a.indices + (int64_t)r * a.idx_stride;
    const int units = a.chunk_shift ? (len + (1 << a.chunk_shift) - 1) >> a.chunk_shift : len;   // positions or chunks
    const int32_t *ptab = (a.page_table && !a.indices_are_physical) ? a.page_table + (int64_t)b * a.max_pages : nullptr;
    for (int j = threadIdx.x; j < c; j += blockDim.x) {
        const int e = idx[j];
        if (a.indices_are_physical) {
            if (e < 0 || (pool_slots > 0 && e >= pool_slots)) ++bad;
        } else {
            if (e < 0 || e >= units) { ++bad; continue; }
            if (j > 0 && idx[j - 1] >= e) ++bad;                                      // ascending, no repeats
            if (ptab) {
                // every page the entry's positions lie on (a chunk larger than a page spans several)
                const int first = a.chunk_shift ? e << a.chunk_shift : e;
                int last = a.chunk_shift ? first + (1 << a.chunk_shift) - 1 : first;
                last = last < len ? last : len - 1;
                for (int pg = first >> a.page_shift; pg <= (last >> a.page_shift); ++pg) {
                    const int page = ptab[pg];
                    if (page < 0 || (pool_slots > 0 && ((int64_t)page << a.page_shift) >= pool_slots)) ++bad;
                }
            }
        }
    }
    if (bad) atomicAdd(n_bad, bad);
}

// CSR form of the padded lists (Section 3.5: the mask reaches the paper's attention kernel as CSR): row pointers
// = exclusive prefix of the list lengths, by one workgroup (fixed order: deterministic).
__global__ __launch_bounds__(1024) void csr_indptr_kernel(const int32_t *counts, int rows, int capacity, int64_t *indptr)
{
    __shared__ long long wave_tot[16];
    __shared__ long long carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { carry = 0; indptr[0] = 0; }
    __syncthreads();
    for (int base = 0; base < rows; base += 1024) {
        const int r = base + tid;
        int c = r < rows ? counts[r] : 0;
        c = c < 0 ? 0 : (c > capacity ? capacity : c);
        long long inc = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long o = __shfl_up(inc, off, 64);
            if (lane >= off) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        long long before = carry;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        if (r < rows) indptr[r + 1] = before + inc;
        __syncthreads();
        if (tid == 1023) carry = before + inc;
        __syncthreads();
    }
}

// packed[indptr[r] + j] = indices[r][j]: one workgroup per row, contiguous reads and writes
__global__ __launch_bounds__(256) void csr_pack_kernel(const int32_t *indices, int64_t idx_stride, const int64_t *indptr,
                                                       int32_t *packed)
{
    const int r = blockIdx.x;
    const int64_t p0 = indptr[r], n = indptr[r + 1] - p0;
    const int32_t *src = indices + (int64_t)r * idx_stride;
    for (int64_t j = threadIdx.x; j < n; j += 256) packed[p0 + j] = src[j];
}

}  // namespace

specattn_status launch_csr(const int32_t *indices, int64_t idx_stride, const int32_t *counts, int rows, int capacity,
                           int64_t *indptr, int32_t *packed, hipStream_t stream)
{
    hipLaunchKernelGGL(csr_indptr_kernel, dim3(1), dim3(1024), 0, stream, counts, rows, capacity, indptr);
    specattn_status st = check_launch("csr_indptr_kernel");
    if (st != SPECATTN_OK || !packed) return st;
    hipLaunchKernelGGL(csr_pack_kernel, dim3(rows), dim3(256), 0, stream, indices, idx_stride, indptr, packed);
    return check_launch("csr_pack_kernel");
}

specattn_status launch_check_lists(const AttnLaunch &a, int64_t pool_slots, int32_t *n_bad, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, stream, n_bad);
    hipLaunchKernelGGL(check_lists_kernel, dim3(a.B * a.H_kv), dim3(256), 0, stream, a, pool_slots, n_bad);
    return check_launch("check_lists_kernel");
}

}  // namespace specattn

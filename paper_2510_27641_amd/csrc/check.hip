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
                const int first = a.chunk_shift ? e << a.chunk_shift : e;
                const int page = ptab[first >> a.page_shift];
                if (page < 0 || (pool_slots > 0 && ((int64_t)page << a.page_shift) >= pool_slots)) ++bad;
            }
        }
    }
    if (bad) atomicAdd(n_bad, bad);
}

}  // namespace

specattn_status launch_check_lists(const AttnLaunch &a, int64_t pool_slots, int32_t *n_bad, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, stream, n_bad);
    hipLaunchKernelGGL(check_lists_kernel, dim3(a.B * a.H_kv), dim3(256), 0, stream, a, pool_slots, n_bad);
    return check_launch("check_lists_kernel");
}

}  // namespace specattn

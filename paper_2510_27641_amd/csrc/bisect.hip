// Algorithm 2's inner loop as the paper's implementation runs it (Section 3.4 and its footnote): a
// fixed number of halvings of [0, max a] on the threshold value, each with a full masked row sum.
// Kept for comparison with the exact selection: with an attention sink at long context ten halvings
// cannot reach thresholds below max/1024 and the set degenerates to "everything".
//
// One workgroup per row.  The bracket ends and midpoints are fp64 (halving fp32 end points is exact
// in fp64 for far more steps than are ever asked for, so no rounding enters the thresholds); masses
// are fp64 sums in a fixed order.  The result is theta_low, the end that always keeps mass >= target,
// rounded up to fp32 so that {a >= tau} is the same set.
#include <hip/hip_runtime.h>

#include "common.h"

namespace specattn {
namespace {

constexpr int B_THREADS = 512;
constexpr int B_WAVES = B_THREADS / 64;

__device__ __forceinline__ double block_sum(double x, double *red)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();                                  // the previous round's readers are done
    if (lane == 0) red[wave] = x;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < B_WAVES; ++w) s += red[w];
    return s;
}

__global__ __launch_bounds__(B_THREADS) void bisect_threshold_kernel(SelectLaunch a, int iters, float *tau,
                                                                    int32_t *valid, uint32_t *flags)
{
    __shared__ double red[B_WAVES];
    __shared__ float red_max[B_WAVES];
    __shared__ int red_bad[B_WAVES];
    const int r = blockIdx.x;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int len = a.seq_lens ? a.seq_lens[b] : a.n_max;
    len = len < 0 ? 0 : (len > a.n_max ? a.n_max : len);
    const float *row = a.probs + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    const int n4 = aligned ? len / 4 : 0;             // float4 part; the rest goes one by one

    // every thread visits its entries in the same order in every pass
    auto for_mine = [&](auto &&fn) {
        for (int i = tid; i < n4; i += B_THREADS) {
            const float4 v = reinterpret_cast<const float4 *>(row)[i];
            fn(v.x); fn(v.y); fn(v.z); fn(v.w);
        }
        for (int i = n4 * 4 + tid; i < len; i += B_THREADS) fn(row[i]);
    };

    double total = 0.0;
    float mx = 0.0f;
    int bad = 0;
    for_mine([&](float x) {
        const uint32_t u = __float_as_uint(x);
        if (u > 0x80000000u || (u & 0x7fffffffu) >= 0x7f800000u) bad = 1;     // negative, infinite or NaN
        total += (double)x;
        mx = fmaxf(mx, x);
    });
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        bad |= __shfl_xor(bad, off, 64);
    }
    if (lane == 0) { red_max[wave] = mx; red_bad[wave] = bad; }
    total = block_sum(total, red);                    // its barriers also cover red_max / red_bad
#pragma unroll
    for (int w = 0; w < B_WAVES; ++w) { mx = fmaxf(mx, red_max[w]); bad |= red_bad[w]; }
    if (bad || len == 0 || !(total > 0.0)) {
        if (tid == 0) { tau[r] = 0.0f; valid[r] = 0; flags[r] = SPECATTN_ROW_INVALID; }
        return;
    }
    const double target = (double)a.top_p * total;    // M_target = p * sum a
    double lo = 0.0, hi = (double)mx, closest = INFINITY;
    for (int it = 0; it < iters; ++it) {
        const double mid = 0.5 * (hi + lo);
        double m = 0.0;
        for_mine([&](float x) { if ((double)x >= mid) m += (double)x; });
        m = block_sum(m, red);
        closest = fmin(closest, fabs(m - target));
        if (m < target) hi = mid; else lo = mid;
    }
    if (tid == 0) {
        float t = (float)lo;
        if ((double)t < lo) t = __uint_as_float(__float_as_uint(t) + 1u);      // next fp32 up (lo >= 0)
        tau[r] = t;
        valid[r] = 1;
        flags[r] = closest <= 1e-6 * total ? SPECATTN_ROW_NEAR_BOUNDARY : 0u;
    }
}

}  // namespace

specattn_status launch_bisect_thresholds(const SelectLaunch &a, int iters, float *tau, int32_t *valid, uint32_t *flags,
                                         hipStream_t stream)
{
    hipLaunchKernelGGL(bisect_threshold_kernel, dim3(a.B * a.H_kv), dim3(B_THREADS), 0, stream, a, iters, tau, valid, flags);
    return check_launch("bisect_threshold_kernel");
}

}  // namespace specattn

// Offline layer mapping (Section 3.3, Eq. 4; Appendix B, Algorithm 3).
//
// 1. Similarity: S[i][j] = -(1/rows) * sum_r D_KL(A^v_j[r] || A^d_i[r]) over aligned attention rows of the two
//    models (Eq. 4, averaged over the rows a representative data set yields).  fp32 probabilities in, fp64
//    logarithms and sums; every (i, j) pair is cut into chunks, one workgroup per (chunk, pair) adds its
//    terms in a fixed order, and a second small kernel adds the chunks in order - no atomics, so the result
//    does not depend on scheduling.  ALU-bound (two fp64 logarithms per term), and small: this runs once.
// 2. Alignment: the non-decreasing map f (verifier layer -> draft layer) that maximises sum_j S[f(j)][j],
//    by the recurrence of Algorithm 3 (its "above" transition contains the other two):
//    best[i][j] = S[i][j] + max_{k <= i} best[k][j-1], first maximum at ties.  One workgroup, thread i holds
//    draft layer i; every column is one prefix-maximum scan over the threads.
#include "common.h"

#include <cmath>

namespace specattn {
namespace {

constexpr int KL_THREADS = 256;
constexpr int MAP_THREADS = 1024;      // most draft layers the alignment kernel takes

__global__ __launch_bounds__(KL_THREADS) void layer_kl_kernel(const float *__restrict__ ad, const float *__restrict__ av,
                                                              int n, int64_t per_layer, int64_t chunk_len, int chunks,
                                                              double *__restrict__ partial)
{
    __shared__ double red[KL_THREADS / 64];
    const int pair = blockIdx.y, i = pair / n, j = pair - i * n;
    const int64_t begin = (int64_t)blockIdx.x * chunk_len;
    const int64_t end = (begin + chunk_len) < per_layer ? (begin + chunk_len) : per_layer;
    const float *pd = ad + (int64_t)i * per_layer, *pv = av + (int64_t)j * per_layer;
    double acc = 0.0;
    for (int64_t k = begin + threadIdx.x; k < end; k += KL_THREADS) {
        const float p = pv[k], q = pd[k];
        // 0 * log(0 / q) = 0; a draft entry of 0 under verifier mass gives +infinity through log(0)
        if (p > 0.0f) acc += (double)p * (log((double)p) - log((double)q));
    }
    // fixed-order reduction: lanes of a wave by xor butterflies, then the waves in order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < KL_THREADS / 64; ++w) s += red[w];
        partial[(int64_t)pair * chunks + blockIdx.x] = s;
    }
}

__global__ void layer_kl_finish_kernel(const double *__restrict__ partial, int pairs, int chunks, double rows,
                                       double *__restrict__ S)
{
    const int pair = blockIdx.x * blockDim.x + threadIdx.x;
    if (pair >= pairs) return;
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += partial[(int64_t)pair * chunks + c];
    S[pair] = -s / rows;
}

struct Best { double val; int idx; };

__global__ __launch_bounds__(MAP_THREADS) void layer_map_kernel(const double *__restrict__ S, int m, int n,
                                                                int32_t *__restrict__ back, int32_t *__restrict__ f,
                                                                double *__restrict__ total)
{
    __shared__ double sval[2][MAP_THREADS];
    __shared__ int sidx[2][MAP_THREADS];
    const int i = threadIdx.x;
    // prefix maximum over the threads with the first index at ties: Hillis-Steele over (value, index) pairs;
    // returns with the result of thread t in sval[b][t], sidx[b][t] and the buffer number b
    auto prefix_max = [&](double v) -> int {
        int b = 0;
        sval[0][i] = v;
        sidx[0][i] = i;
        __syncthreads();
        for (int off = 1; off < MAP_THREADS; off <<= 1) {
            double mv = sval[b][i];
            int mi = sidx[b][i];
            if (i >= off) {
                const double lv = sval[b][i - off];          // the candidates with lower indices win ties
                if (!(mv > lv)) { mv = lv; mi = sidx[b][i - off]; }
            }
            sval[b ^ 1][i] = mv;
            sidx[b ^ 1][i] = mi;
            b ^= 1;
            __syncthreads();
        }
        return b;
    };
    double best = i < m ? S[(int64_t)i * n] : -INFINITY;       // column 0; threads past m never win a maximum
    for (int j = 1; j < n; ++j) {
        const int b = prefix_max(best);
        if (i < m) {
            const int k = sidx[b][i];
            back[(int64_t)i * n + j] = k;
            best = S[(int64_t)i * n + j] + sval[b][i];
        }
        __syncthreads();                                       // everyone has read the scan result
    }
    const int b = prefix_max(best);
    if (i == 0) {
        int at = sidx[b][MAP_THREADS - 1];                     // first maximum of the last column
        at = at < m ? at : 0;                                  // all entries -infinity or NaN: layer 0
        *total = sval[b][MAP_THREADS - 1];
        f[n - 1] = at;
        __threadfence_block();
        for (int j = n - 1; j > 0; --j) {
            at = __hip_atomic_load(&back[(int64_t)at * n + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            f[j - 1] = at;
        }
    }
}

int kl_chunks(int pairs, int64_t per_layer)
{
    // enough workgroups to fill the chip, chunks of at least 4096 terms
    int64_t want = (4 * (int64_t)cu_count() + pairs - 1) / pairs;
    const int64_t most = (per_layer + 4095) / 4096;
    if (want > most) want = most;
    if (want > 1024) want = 1024;
    return want < 1 ? 1 : (int)want;
}

bool bad_dims(int m, int n, int rows, int L)
{
    return m <= 0 || n <= 0 || rows <= 0 || L <= 0 || (int64_t)m * n > 65535 || (int64_t)rows * L > ((int64_t)1 << 40);
}

}  // namespace
}  // namespace specattn

using namespace specattn;

extern "C" {

size_t specattn_layer_similarity_workspace_size(int32_t m, int32_t n, int32_t rows, int32_t L)
{
    if (bad_dims(m, n, rows, L)) return 0;
    const size_t bytes = (size_t)m * n * kl_chunks(m * n, (int64_t)rows * L) * sizeof(double);
    return (bytes + 255) & ~(size_t)255;
}

specattn_status specattn_layer_similarity(const float *attn_draft, const float *attn_verifier, int32_t m, int32_t n,
                                          int32_t rows, int32_t L, double *S, void *workspace, size_t workspace_bytes,
                                          void *stream)
{
    clear_error();
    if (!attn_draft || !attn_verifier || !S) { set_error("attn_draft, attn_verifier and S must not be NULL"); return SPECATTN_EINVAL; }
    if (m <= 0 || n <= 0 || rows <= 0 || L <= 0) { set_error("m, n, rows and L must be positive"); return SPECATTN_EINVAL; }
    if (bad_dims(m, n, rows, L)) { set_error("at most 65535 layer pairs and 2^40 entries per layer"); return SPECATTN_ESHAPE; }
    const size_t need = specattn_layer_similarity_workspace_size(m, n, rows, L);
    if (!workspace) { set_error("workspace is NULL, %zu bytes needed", need); return SPECATTN_EWORKSPACE; }
    if (reinterpret_cast<uintptr_t>(workspace) % 256) { set_error("workspace must be 256-byte aligned"); return SPECATTN_EWORKSPACE; }
    if (workspace_bytes < need) { set_error("workspace has %zu bytes, %zu needed", workspace_bytes, need); return SPECATTN_EWORKSPACE; }
    const int pairs = m * n;
    const int64_t per_layer = (int64_t)rows * L;
    const int chunks = kl_chunks(pairs, per_layer);
    const int64_t chunk_len = (per_layer + chunks - 1) / chunks;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    double *partial = static_cast<double *>(workspace);
    hipLaunchKernelGGL(layer_kl_kernel, dim3(chunks, pairs), dim3(KL_THREADS), 0, hs, attn_draft, attn_verifier, n, per_layer,
                       chunk_len, chunks, partial);
    specattn_status st = check_launch("layer_kl_kernel");
    if (st != SPECATTN_OK) return st;
    hipLaunchKernelGGL(layer_kl_finish_kernel, dim3((pairs + 255) / 256), dim3(256), 0, hs, partial, pairs, chunks, (double)rows, S);
    return check_launch("layer_kl_finish_kernel");
}

size_t specattn_layer_map_workspace_size(int32_t m, int32_t n)
{
    if (m <= 0 || n <= 0 || m > MAP_THREADS || n > 65535) return 0;
    return (((size_t)m * n * sizeof(int32_t)) + 255) & ~(size_t)255;
}

specattn_status specattn_layer_map(const double *S, int32_t m, int32_t n, int32_t *f, double *total, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    clear_error();
    if (!S || !f || !total) { set_error("S, f and total must not be NULL"); return SPECATTN_EINVAL; }
    if (m <= 0 || n <= 0) { set_error("m and n must be positive"); return SPECATTN_EINVAL; }
    if (m > MAP_THREADS || n > 65535) { set_error("at most %d draft layers and 65535 verifier layers", MAP_THREADS); return SPECATTN_ESHAPE; }
    const size_t need = specattn_layer_map_workspace_size(m, n);
    if (!workspace) { set_error("workspace is NULL, %zu bytes needed", need); return SPECATTN_EWORKSPACE; }
    if (reinterpret_cast<uintptr_t>(workspace) % 256) { set_error("workspace must be 256-byte aligned"); return SPECATTN_EWORKSPACE; }
    if (workspace_bytes < need) { set_error("workspace has %zu bytes, %zu needed", workspace_bytes, need); return SPECATTN_EWORKSPACE; }
    hipLaunchKernelGGL(layer_map_kernel, dim3(1), dim3(MAP_THREADS), 0, static_cast<hipStream_t>(stream), S, m, n,
                       static_cast<int32_t *>(workspace), f, total);
    return check_launch("layer_map_kernel");
}

}  // extern "C"

// Sparse decode attention over a selected index list (Section 3.1.2, Eq. 2-3; Section 3.5):
// portable fp32-ALU variant for any supported shape and dtype (fp32 or bf16 inputs), plus the
// split merge used by every variant.
//
// Work split: one workgroup per (row, split); a split is a contiguous slice of the row's index
// list.  Each workgroup streams its slice in tiles of 32 positions through LDS, keeps the
// running softmax state (max m, sum l, un-normalised output o) for all G*T query rows of the
// kv head, and writes one partial (m, l, o).  merge_kernel combines the partials of a row:
//   O = sum_s exp(m_s - m) o_s / sum_s exp(m_s - m) l_s,  lse = m + log(sum_s exp(m_s - m) l_s).
#include "common.h"

#include <hip/hip_bf16.h>

#include <mutex>

namespace specattn {
namespace {

constexpr int GEN_THREADS = 256;
constexpr int GEN_TILE = 32;
constexpr int MAX_QT = 64;            // G*T query rows per kv head handled by the generic kernel

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float ld(const void *p, int64_t i) { return static_cast<const float *>(p)[i]; }
};
template <> struct Elem<_Float16> {
    static __device__ __forceinline__ float ld(const void *p, int64_t i) { return (float) static_cast<const _Float16 *>(p)[i]; }
};
template <> struct Elem<__hip_bfloat16> {
    static __device__ __forceinline__ float ld(const void *p, int64_t i)
    {
        return __uint_as_float((uint32_t) static_cast<const uint16_t *>(p)[i] << 16);
    }
};

// element offset of position/slot `idx` of (b, h) inside k or v
struct KvMap {
    int64_t base;            // b / h part (contiguous) or h part (paged)
    int64_t stride_n, stride_page;
    const int32_t *ptab;     // this sequence's page table row, or null
    int page_shift;
    bool physical;
    __device__ __forceinline__ int64_t off(int idx) const
    {
        if (!ptab && !physical) return base + (int64_t)idx * stride_n;
        const int mask = (1 << page_shift) - 1;
        const int page = physical ? (idx >> page_shift) : ptab[idx >> page_shift];
        return base + (int64_t)page * stride_page + (int64_t)(idx & mask) * stride_n;
    }
};

__device__ __forceinline__ KvMap make_map(const AttnLaunch &a, int b, int h)
{
    KvMap m;
    const bool paged = a.page_table != nullptr || a.indices_are_physical;
    m.base = paged ? (int64_t)h * a.kv_stride_h : (int64_t)b * a.kv_stride_b + (int64_t)h * a.kv_stride_h;
    m.stride_n = a.kv_stride_n;
    m.stride_page = a.kv_stride_page;
    m.ptab = (a.page_table && !a.indices_are_physical) ? a.page_table + (int64_t)b * a.max_pages : nullptr;
    m.page_shift = a.page_shift;
    m.physical = a.indices_are_physical != 0;
    return m;
}

template <typename T, int D>
__global__ __launch_bounds__(GEN_THREADS) void attn_generic_kernel(AttnLaunch a, int n_splits, float *part_o,
                                                                  float *part_ml)
{
    extern __shared__ float smem[];
    const int QT = (a.H_q / a.H_kv) * a.T;
    float *Qs = smem;                       // [QT][D]
    float *Ks = Qs + MAX_QT * D;            // [TILE][D+1]
    float *Vs = Ks + GEN_TILE * (D + 1);    // [TILE][D]
    float *Ss = Vs + GEN_TILE * D;          // [QT][TILE+1]
    float *alpha = Ss + MAX_QT * (GEN_TILE + 1);   // [QT]
    float *m_run = alpha + MAX_QT;          // [QT]
    float *l_run = m_run + MAX_QT;          // [QT]

    const int r = blockIdx.x / n_splits, s = blockIdx.x - r * n_splits;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int G = a.H_q / a.H_kv;
    const int tid = threadIdx.x;
    const int count = attn_row_count(a, r);
    const int tiles = (count + GEN_TILE - 1) / GEN_TILE;
    const int tiles_per_split = (tiles + n_splits - 1) / n_splits;
    const int j_begin = s * tiles_per_split * GEN_TILE;
    int j_end = j_begin + tiles_per_split * GEN_TILE;
    j_end = j_end > count ? count : j_end;
    const int32_t *idx = a.dense ? nullptr : a.indices + (int64_t)r * a.idx_stride;
    const KvMap map = make_map(a, b, h);
    const float scale = a.sm_scale;

    for (int e = tid; e < QT * D; e += GEN_THREADS) {
        const int qi = e / D, dd = e - qi * D;
        const int g = qi / a.T, t = qi - g * a.T;
        const int64_t qo = (int64_t)b * a.q_stride_b + (int64_t)(h * G + g) * a.q_stride_h + (int64_t)t * a.q_stride_t + dd;
        Qs[e] = Elem<T>::ld(a.q, qo);
    }
    if (tid < QT) { m_run[tid] = -INFINITY; l_run[tid] = 0.0f; }
    constexpr int OPT = (MAX_QT * D) / GEN_THREADS;      // outputs owned per thread (upper bound)
    float acc[OPT];
#pragma unroll
    for (int k = 0; k < OPT; ++k) acc[k] = 0.0f;
    __syncthreads();

    for (int j0 = j_begin; j0 < j_end; j0 += GEN_TILE) {
        const int np = (j_end - j0) < GEN_TILE ? (j_end - j0) : GEN_TILE;
        for (int e = tid; e < GEN_TILE * D; e += GEN_THREADS) {
            const int p = e / D, dd = e - p * D;
            float kv = 0.0f, vv = 0.0f;
            if (p < np) {
                const int64_t o = map.off(attn_list_pos(a, idx, j0 + p)) + dd;
                kv = Elem<T>::ld(a.k, o);
                vv = Elem<T>::ld(a.v, o);
            }
            Ks[p * (D + 1) + dd] = kv;
            Vs[p * D + dd] = vv;
        }
        __syncthreads();
        for (int e = tid; e < QT * GEN_TILE; e += GEN_THREADS) {
            const int qi = e / GEN_TILE, p = e - qi * GEN_TILE;
            float dot = 0.0f;
#pragma unroll 8
            for (int dd = 0; dd < D; ++dd) dot = fmaf(Qs[qi * D + dd], Ks[p * (D + 1) + dd], dot);
            Ss[qi * (GEN_TILE + 1) + p] = p < np ? dot * scale : -INFINITY;
        }
        __syncthreads();
        if (tid < QT) {
            float mx = m_run[tid];
            for (int p = 0; p < np; ++p) mx = fmaxf(mx, Ss[tid * (GEN_TILE + 1) + p]);
            const float al = (m_run[tid] == -INFINITY) ? 0.0f : __expf(m_run[tid] - mx);
            float sum = 0.0f;
            for (int p = 0; p < GEN_TILE; ++p) {
                const float w = p < np ? __expf(Ss[tid * (GEN_TILE + 1) + p] - mx) : 0.0f;
                Ss[tid * (GEN_TILE + 1) + p] = w;
                sum += w;
            }
            alpha[tid] = al;
            l_run[tid] = l_run[tid] * al + sum;
            m_run[tid] = mx;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < OPT; ++k) {
            const int e = tid + k * GEN_THREADS;
            if (e < QT * D) {
                const int qi = e / D, dd = e - qi * D;
                float o = acc[k] * alpha[qi];
                for (int p = 0; p < GEN_TILE; ++p) o = fmaf(Ss[qi * (GEN_TILE + 1) + p], Vs[p * D + dd], o);
                acc[k] = o;
            }
        }
        __syncthreads();
    }

    float *po = part_o + ((int64_t)r * n_splits + s) * QT * D;
    float *pml = part_ml + ((int64_t)r * n_splits + s) * QT * 2;
#pragma unroll
    for (int k = 0; k < OPT; ++k) {
        const int e = tid + k * GEN_THREADS;
        if (e < QT * D) po[e] = acc[k];
    }
    if (tid < QT) { pml[2 * tid] = m_run[tid]; pml[2 * tid + 1] = l_run[tid]; }
}

// One workgroup per (row, query row): combine the partials of all splits, then the new tokens
// behind the cache (query t sees new tokens 0..t), if the caller gave any.
__global__ void merge_kernel(AttnLaunch a, int n_splits, const float *part_o, const float *part_ml)
{
    __shared__ float red[2 * SPECATTN_MAX_T];
    const int G = a.H_q / a.H_kv;
    const int QT = G * a.T;
    const int r = blockIdx.x / QT, qi = blockIdx.x - r * QT;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int g = qi / a.T, t = qi - g * a.T;
    const int D = a.d;
    float dots[SPECATTN_MAX_T];
    const int n_tail = a.k_new ? t + 1 : 0;
    if (n_tail) tail_dots(a, b, h * G + g, t, red, dots);
    float m = -INFINITY;
    for (int s = 0; s < n_splits; ++s) m = fmaxf(m, part_ml[(((int64_t)r * n_splits + s) * QT + qi) * 2]);
#pragma unroll
    for (int p = 0; p < SPECATTN_MAX_T; ++p)
        if (p < n_tail) m = fmaxf(m, dots[p] * a.sm_scale);
    float l = 0.0f;
    for (int s = 0; s < n_splits; ++s) {
        const float *p = part_ml + (((int64_t)r * n_splits + s) * QT + qi) * 2;
        if (p[0] != -INFINITY) l += __expf(p[0] - m) * p[1];
    }
    float wt[SPECATTN_MAX_T];
#pragma unroll
    for (int p = 0; p < SPECATTN_MAX_T; ++p) {
        wt[p] = p < n_tail ? __expf(dots[p] * a.sm_scale - m) : 0.0f;
        l += wt[p];
    }
    const int64_t orow = ((int64_t)b * a.H_q + (h * G + g)) * a.T + t;
    const int64_t noff = ((int64_t)b * a.H_kv + h) * a.T * D;
    for (int dd = threadIdx.x; dd < D; dd += blockDim.x) {
        float o = 0.0f;
        for (int s = 0; s < n_splits; ++s) {
            const float ms = part_ml[(((int64_t)r * n_splits + s) * QT + qi) * 2];
            if (ms != -INFINITY) o += __expf(ms - m) * part_o[(((int64_t)r * n_splits + s) * QT + qi) * D + dd];
        }
#pragma unroll
        for (int p = 0; p < SPECATTN_MAX_T; ++p)
            if (p < n_tail) o += wt[p] * ld_elem(a.v_new, noff + (int64_t)p * D + dd, a.dtype);
        const float res = l > 0.0f ? o / l : 0.0f;
        a.out[orow * D + dd] = res;
        if (a.out_lowp) st_lowp(a.out_lowp, orow * D + dd, res, a.dtype);
    }
    if (a.lse && threadIdx.x == 0) a.lse[orow] = l > 0.0f ? m + __logf(l) : -INFINITY;
}

constexpr size_t generic_lds_bytes(int d)
{
    return sizeof(float) * (size_t)(MAX_QT * d + GEN_TILE * (d + 1) + GEN_TILE * d + MAX_QT * (GEN_TILE + 1) + 3 * MAX_QT);
}

template <typename T, int D>
specattn_status run_generic(const AttnLaunch &a, int rows, int n_splits, float *part_o, float *part_ml,
                            hipStream_t stream)
{
    const specattn_status st = attn_generic_configure();
    if (st != SPECATTN_OK) return st;
    hipLaunchKernelGGL((attn_generic_kernel<T, D>), dim3(rows * n_splits), dim3(GEN_THREADS), generic_lds_bytes(D), stream, a,
                       n_splits, part_o, part_ml);
    return check_launch("attn_generic_kernel");
}

}  // namespace

// The LDS size of every variant, set once per device (not on a variant's first launch: a first call may be
// recorded in a graph, and a process may use several devices).
specattn_status attn_generic_configure()
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static bool done[MAX_DEVICES] = {false};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        set_error("no current device");
        return SPECATTN_EHIP;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (done[dev]) return SPECATTN_OK;
    const struct { const void *fn; size_t lds; } variants[] = {
        {reinterpret_cast<const void *>(&attn_generic_kernel<float, 64>), generic_lds_bytes(64)},
        {reinterpret_cast<const void *>(&attn_generic_kernel<float, 128>), generic_lds_bytes(128)},
        {reinterpret_cast<const void *>(&attn_generic_kernel<__hip_bfloat16, 64>), generic_lds_bytes(64)},
        {reinterpret_cast<const void *>(&attn_generic_kernel<__hip_bfloat16, 128>), generic_lds_bytes(128)},
        {reinterpret_cast<const void *>(&attn_generic_kernel<_Float16, 64>), generic_lds_bytes(64)},
        {reinterpret_cast<const void *>(&attn_generic_kernel<_Float16, 128>), generic_lds_bytes(128)},
    };
    for (const auto &v : variants) {
        if (hipFuncSetAttribute(v.fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)v.lds) != hipSuccess) {
            (void)hipGetLastError();
            set_error("cannot reserve %zu bytes of LDS", v.lds);
            return SPECATTN_EHIP;
        }
    }
    done[dev] = true;
    return SPECATTN_OK;
}

int attn_num_splits(int rows, int idx_capacity)
{
    const int want = 4 * cu_count();                          // workgroups in flight to aim for
    int s = (want + rows - 1) / rows;
    const int max_s = (idx_capacity + 255) / 256;             // at least 256 positions per split
    if (s > max_s) s = max_s;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return s;
}

static size_t workspace_bytes(int rows, int G, int T, int d, int idx_capacity, bool least)
{
    const size_t ns = (size_t)attn_num_splits(rows, idx_capacity);
    const size_t qt = (size_t)G * T;
    size_t bytes = (size_t)rows * ns * qt * (size_t)(d + 2) * sizeof(float);
    bytes = (bytes + 255) & ~(size_t)255;
    if (d == 128) {                                  // the matrix-core variant may take this shape (larger groups of
        const size_t other = least ? attn_mfma_workspace_min_bytes(rows, G, T)   // query heads run as several launches over it)
                                   : attn_mfma_workspace_bytes(rows, G, T);
        if (other > bytes) bytes = other;
    }
    return bytes;
}
size_t attn_workspace_bytes(int rows, int G, int T, int d, int idx_capacity) { return workspace_bytes(rows, G, T, d, idx_capacity, false); }
size_t attn_workspace_min_bytes(int rows, int G, int T, int d, int idx_capacity) { return workspace_bytes(rows, G, T, d, idx_capacity, true); }

specattn_status launch_attn(const AttnLaunch &a, hipStream_t stream)
{
    if (attn_mfma_supported(a)) return launch_attn_mfma(a, stream);
    const int rows = a.B * a.H_kv;
    const int G = a.H_q / a.H_kv;
    const int QT = G * a.T;
    const int ns = attn_num_splits(rows, a.idx_capacity << a.chunk_shift);
    float *part_o = static_cast<float *>(a.workspace);
    float *part_ml = part_o + (size_t)rows * ns * QT * a.d;
    specattn_status st;
    if (a.dtype == SPECATTN_F32 && a.d == 64) st = run_generic<float, 64>(a, rows, ns, part_o, part_ml, stream);
    else if (a.dtype == SPECATTN_F32 && a.d == 128) st = run_generic<float, 128>(a, rows, ns, part_o, part_ml, stream);
    else if (a.dtype == SPECATTN_BF16 && a.d == 64) st = run_generic<__hip_bfloat16, 64>(a, rows, ns, part_o, part_ml, stream);
    else if (a.dtype == SPECATTN_BF16 && a.d == 128) st = run_generic<__hip_bfloat16, 128>(a, rows, ns, part_o, part_ml, stream);
    else if (a.dtype == SPECATTN_F16 && a.d == 64) st = run_generic<_Float16, 64>(a, rows, ns, part_o, part_ml, stream);
    else if (a.dtype == SPECATTN_F16 && a.d == 128) st = run_generic<_Float16, 128>(a, rows, ns, part_o, part_ml, stream);
    else { set_error("no attention kernel for dtype %d, d %d", a.dtype, a.d); return SPECATTN_EUNSUPPORTED; }
    if (st != SPECATTN_OK) return st;
    hipLaunchKernelGGL(merge_kernel, dim3(rows * QT), dim3(a.d < 64 ? 64 : a.d), 0, stream, a, ns, part_o, part_ml);
    return check_launch("merge_kernel");
}

}  // namespace specattn

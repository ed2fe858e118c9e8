// Sorting-free exact top-p selection (Section 3.4, Algorithm 2; objective Appendix A, Eq. 8).
//
// Algorithm 2 bisects the threshold in value space and evaluates the kept mass once per step.
// This kernel reaches the exact threshold tau* = max{t : mass{a >= t} >= p * sum a} with three
// radix passes over the fp32 bit pattern instead (non-negative floats order like their bits):
//   pass 1: 2048 bins on bits[30:20], pass 2: 1024 bins on bits[19:10] inside the boundary bin,
//   pass 3: 1024 bins on bits[9:0]  ->  all 31 bits of tau*.
// All entries of one bin share their exponent, so a bin's mass is kept as an exact integer sum
// of 24-bit significands next to the count in one 64-bit LDS counter; bin masses are therefore
// independent of summation order and the result is deterministic.  fp64 appears only in the
// suffix sums over bins.  The kept positions are then written in ascending order by
// ballot + popcount prefix (no dense mask, no CSR conversion as in Section 3.5).
//
// One workgroup owns one row.  Rows up to THREADS*4*NV4 entries live in registers for all four
// passes (one HBM read); longer rows are re-read from L2/HBM each pass.
#include "common.h"

namespace specattn {
namespace {

constexpr int NB1 = 2048;                     // bins of pass 1
constexpr int NB2 = 1024;                     // bins of passes 2 and 3
constexpr int CNT_SHIFT = 44;                 // counter = count << 44 | sum of significands
constexpr unsigned long long CNT_ONE = 1ull << CNT_SHIFT;
constexpr unsigned long long SIG_MASK = CNT_ONE - 1;

struct RowShared {
    unsigned long long hist[NB1];
    double wave_m[16];
    unsigned wave_c[16];
    unsigned wave_tot[2][16];
    double total_m;
    double m_above;
    unsigned c_above;
    unsigned long long bin_packed;
    int best;
    int lowest;
    unsigned running;
};

__device__ __forceinline__ unsigned long long packed_entry(uint32_t u)
{
    const uint32_t sig = (u & 0x7fffffu) | ((u >> 23) ? 0x800000u : 0u);
    return CNT_ONE | sig;
}

// value of a significand sum whose entries all carry biased exponent field e: sum * 2^(max(e,1)-150)
__device__ __forceinline__ double mass_of(unsigned long long packed, int e_field)
{
    const double s = (double)(long long)(packed & SIG_MASK);     // < 2^44: exact
    return ldexp(s, (e_field > 0 ? e_field : 1) - 150);
}

// Suffix sums over threads (thread t gets the sum over threads > t) of a double and a count.
template <int THREADS>
__device__ __forceinline__ void suffix_scan(double lm, unsigned lc, RowShared &sh, double &excl_m,
                                            unsigned &excl_c, double &total_m)
{
    constexpr int NW = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double im = lm;
    unsigned ic = lc;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double om = __shfl_down(im, off, 64);
        const unsigned oc = __shfl_down(ic, off, 64);
        if (lane + off < 64) { im += om; ic += oc; }
    }
    if (lane == 0) { sh.wave_m[wave] = im; sh.wave_c[wave] = ic; }
    const double nm = __shfl_down(im, 1, 64);          // inclusive sum of the lanes above
    const unsigned nc = __shfl_down(ic, 1, 64);
    __syncthreads();
    double hm = 0.0;
    unsigned hc = 0;
    for (int w = NW - 1; w > wave; --w) { hm += sh.wave_m[w]; hc += sh.wave_c[w]; }
    excl_m = (lane < 63 ? nm : 0.0) + hm;
    excl_c = (lane < 63 ? nc : 0u) + hc;
    double tot = 0.0;
    for (int w = NW - 1; w >= 0; --w) tot += sh.wave_m[w];
    total_m = tot;
    __syncthreads();
}

// One radix pass decision.  hist[0..NB) holds the packed counters of this pass.
// On return (uniform over the block): bin = highest non-empty bin b with
// m_above + mass(bins >= b) >= target (lowest non-empty bin if rounding leaves none),
// and m_above / c_above advanced to cover the bins above it.
template <int THREADS, int NB, bool FIRST>
__device__ __forceinline__ int locate_bin(RowShared &sh, int e_field_fixed, float top_p, double &target,
                                          double &m_above, unsigned &c_above,
                                          unsigned long long &bin_packed)
{
    constexpr int BPT = NB / THREADS;
    static_assert(BPT >= 1, "more threads than bins");
    const int b0 = threadIdx.x * BPT;
    double lm = 0.0;
    unsigned lc = 0;
    double mass[BPT];
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        const unsigned long long h = sh.hist[b0 + j];
        const int e = FIRST ? ((b0 + j) >> 3) : e_field_fixed;
        mass[j] = mass_of(h, e);
        lm += mass[j];
        lc += (unsigned)(h >> CNT_SHIFT);
    }
    double excl_m, total;
    unsigned excl_c;
    if (threadIdx.x == 0) { sh.best = -1; sh.lowest = NB; }
    suffix_scan<THREADS>(lm, lc, sh, excl_m, excl_c, total);
    if (FIRST) target = (double)top_p * total;     // Algorithm 2: M_target = p * sum a
    if (FIRST && !(total > 0.0)) return -1;        // no mass at all (uniform decision)

    int mine = -1, low = NB;
    double run = excl_m;
#pragma unroll
    for (int j = BPT - 1; j >= 0; --j) {
        const bool nonempty = (sh.hist[b0 + j] >> CNT_SHIFT) != 0;
        if (nonempty) {
            low = b0 + j;
            if (mine < 0 && (m_above + (run + mass[j])) >= target) mine = b0 + j;
        }
        run += mass[j];
    }
    if (mine >= 0) atomicMax(&sh.best, mine);
    if (low < NB) atomicMin(&sh.lowest, low);
    __syncthreads();
    const int bin = sh.best >= 0 ? sh.best : sh.lowest;
    if (bin >= b0 && bin < b0 + BPT) {
        double r = excl_m;
        unsigned c = excl_c;
#pragma unroll
        for (int j = BPT - 1; j >= 0; --j) {
            if (b0 + j > bin) { r += mass[j]; c += (unsigned)(sh.hist[b0 + j] >> CNT_SHIFT); }
        }
        sh.m_above = m_above + r;
        sh.c_above = c_above + c;
        sh.bin_packed = sh.hist[bin];
    }
    __syncthreads();
    m_above = sh.m_above;
    c_above = sh.c_above;
    bin_packed = sh.bin_packed;
    return bin;
}

template <int THREADS, int NB>
__device__ __forceinline__ void clear_hist(RowShared &sh)
{
    for (int b = threadIdx.x; b < NB; b += THREADS) sh.hist[b] = 0ull;
    __syncthreads();
}

// THREADS threads per row; RESIDENT: the row sits in NV4 uint4 registers per thread.
template <int THREADS, int NV4, bool RESIDENT>
__global__ __launch_bounds__(THREADS) void topp_select_kernel(SelectLaunch a)
{
    __shared__ RowShared sh;
    constexpr int NW = THREADS / 64;
    constexpr int ITEM = THREADS * 4;                 // positions per item (one uint4 per thread)
    const int r = blockIdx.x;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int len = a.seq_lens ? a.seq_lens[b] : a.n_max;
    len = len < 0 ? 0 : (len > a.n_max ? a.n_max : len);
    const float *row = a.probs + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    const int n_items = (len + ITEM - 1) / ITEM;

    bool bad = false;
    auto load_item = [&](int i) -> uint4 {
        const int p = (i * THREADS + tid) * 4;
        uint4 u = make_uint4(0, 0, 0, 0);
        if (p + 3 < len && aligned) {
            u = *reinterpret_cast<const uint4 *>(row + p);
        } else {
            if (p < len) u.x = __float_as_uint(row[p]);
            if (p + 1 < len) u.y = __float_as_uint(row[p + 1]);
            if (p + 2 < len) u.z = __float_as_uint(row[p + 2]);
            if (p + 3 < len) u.w = __float_as_uint(row[p + 3]);
        }
        // -0.0 is zero; negative, infinite and NaN entries make the row invalid
        auto clean = [&](uint32_t x) -> uint32_t {
            if (x == 0x80000000u) return 0u;
            if (x >= 0x7f800000u) { bad = true; return 0u; }
            return x;
        };
        u.x = clean(u.x); u.y = clean(u.y); u.z = clean(u.z); u.w = clean(u.w);
        return u;
    };

    uint4 data[RESIDENT ? NV4 : 1];
    if (RESIDENT) {
#pragma unroll
        for (int i = 0; i < NV4; ++i) data[i] = (i < n_items) ? load_item(i) : make_uint4(0, 0, 0, 0);
    }
    auto for_items = [&](auto &&fn) {
        if (RESIDENT) {
#pragma unroll
            for (int i = 0; i < NV4; ++i)
                if (i < n_items) fn(i, data[i]);
        } else {
            for (int i = 0; i < n_items; ++i) fn(i, load_item(i));
        }
    };

    // ---- pass 1: bits[30:20] -----------------------------------------------------------------
    clear_hist<THREADS, NB1>(sh);
    for_items([&](int, uint4 u) {
        if (u.x) atomicAdd(&sh.hist[u.x >> 20], packed_entry(u.x));
        if (u.y) atomicAdd(&sh.hist[u.y >> 20], packed_entry(u.y));
        if (u.z) atomicAdd(&sh.hist[u.z >> 20], packed_entry(u.z));
        if (u.w) atomicAdd(&sh.hist[u.w >> 20], packed_entry(u.w));
    });
    const bool any_bad = __syncthreads_or(bad ? 1 : 0) != 0;     // also orders the atomics

    double target = 0.0, m_above = 0.0;
    unsigned c_above = 0;
    unsigned long long bin_packed = 0;
    const int b1 = locate_bin<THREADS, NB1, true>(sh, 0, a.top_p, target, m_above, c_above, bin_packed);
    const double row_sum = (double)target / (double)a.top_p;     // only used for the boundary flag
    if (any_bad || b1 < 0 || len == 0) {
        if (tid == 0) {
            a.counts[r] = 0;
            if (a.thresholds) a.thresholds[r] = 0.0f;
            if (a.row_flags) a.row_flags[r] = SPECATTN_ROW_INVALID;
        }
        if (a.block_counts)
            for (int k = tid; k < a.blocks_per_row; k += THREADS) a.block_counts[(int64_t)r * a.blocks_per_row + k] = 0;
        return;
    }
    const int e_field = b1 >> 3;

    // ---- pass 2: bits[19:10] inside bin b1 ---------------------------------------------------
    clear_hist<THREADS, NB2>(sh);
    for_items([&](int, uint4 u) {
        if ((u.x >> 20) == (uint32_t)b1 && u.x) atomicAdd(&sh.hist[(u.x >> 10) & 1023u], packed_entry(u.x));
        if ((u.y >> 20) == (uint32_t)b1 && u.y) atomicAdd(&sh.hist[(u.y >> 10) & 1023u], packed_entry(u.y));
        if ((u.z >> 20) == (uint32_t)b1 && u.z) atomicAdd(&sh.hist[(u.z >> 10) & 1023u], packed_entry(u.z));
        if ((u.w >> 20) == (uint32_t)b1 && u.w) atomicAdd(&sh.hist[(u.w >> 10) & 1023u], packed_entry(u.w));
    });
    __syncthreads();
    const int b2 = locate_bin<THREADS, NB2, false>(sh, e_field, a.top_p, target, m_above, c_above, bin_packed);

    // ---- pass 3: bits[9:0] inside (b1, b2) ---------------------------------------------------
    const uint32_t prefix = ((uint32_t)b1 << 10) | (uint32_t)b2;
    clear_hist<THREADS, NB2>(sh);
    for_items([&](int, uint4 u) {
        if ((u.x >> 10) == prefix && u.x) atomicAdd(&sh.hist[u.x & 1023u], packed_entry(u.x));
        if ((u.y >> 10) == prefix && u.y) atomicAdd(&sh.hist[u.y & 1023u], packed_entry(u.y));
        if ((u.z >> 10) == prefix && u.z) atomicAdd(&sh.hist[u.z & 1023u], packed_entry(u.z));
        if ((u.w >> 10) == prefix && u.w) atomicAdd(&sh.hist[u.w & 1023u], packed_entry(u.w));
    });
    __syncthreads();
    const int b3 = locate_bin<THREADS, NB2, false>(sh, e_field, a.top_p, target, m_above, c_above, bin_packed);
    const uint32_t tau_bits = (prefix << 10) | (uint32_t)b3;     // >= 1: zeros never enter a bin
    const unsigned kept = c_above + (unsigned)(bin_packed >> CNT_SHIFT);

    if (tid == 0) {
        a.counts[r] = (int32_t)kept;
        if (a.thresholds) a.thresholds[r] = __uint_as_float(tau_bits);
        if (a.row_flags) {
            const double m_excl = m_above, m_incl = m_above + mass_of(bin_packed, e_field);
            const double band = 1e-6 * row_sum;
            uint32_t f = 0;
            if (fabs(m_incl - target) <= band || fabs(m_excl - target) <= band) f |= SPECATTN_ROW_NEAR_BOUNDARY;
            if (a.indices && kept > (unsigned)a.idx_capacity) f |= SPECATTN_ROW_OVERFLOW;
            a.row_flags[r] = f;
        }
        sh.running = 0;
    }
    if (!a.indices && !a.block_counts) return;

    // ---- ordered compaction: {j : a_j >= tau*}, ascending (Algorithm 2, last step) -------------
    int32_t *out = a.indices ? a.indices + (int64_t)r * a.idx_stride : nullptr;
    const int32_t *ptab = (a.emit_physical && a.page_table) ? a.page_table + (int64_t)b * a.max_pages : nullptr;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    __syncthreads();
    int it = 0;
    auto compact_item = [&](int i, uint4 u) {
        const bool f0 = u.x >= tau_bits, f1 = u.y >= tau_bits, f2 = u.z >= tau_bits, f3 = u.w >= tau_bits;
        const unsigned long long m0 = __ballot(f0), m1 = __ballot(f1), m2 = __ballot(f2), m3 = __ballot(f3);
        const unsigned before = __popcll(m0 & lt_mask) + __popcll(m1 & lt_mask) + __popcll(m2 & lt_mask) +
                                __popcll(m3 & lt_mask);
        const unsigned wtot = __popcll(m0) + __popcll(m1) + __popcll(m2) + __popcll(m3);
        const int buf = it & 1;
        if (lane == 0) sh.wave_tot[buf][wave] = wtot;
        __syncthreads();
        unsigned base = sh.running, all = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const unsigned t = sh.wave_tot[buf][w];
            if (w < wave) base += t;
            all += t;
        }
        if (a.block_counts) {
            constexpr int BPI = ITEM / SEL_BLOCK;              // selection blocks per item
            constexpr int WPB = NW / BPI;                      // waves per block
            if (tid < BPI) {
                unsigned c = 0;
                for (int w = 0; w < WPB; ++w) c += sh.wave_tot[buf][tid * WPB + w];
                const int blk = i * BPI + tid;
                if (blk < a.blocks_per_row) a.block_counts[(int64_t)r * a.blocks_per_row + blk] = (int32_t)c;
            }
        }
        if (out) {
            unsigned o = base + before;
            const int p = (i * THREADS + tid) * 4;
            auto emit = [&](bool f, int pos) {
                if (f) {
                    if (o < (unsigned)a.idx_capacity) {
                        int32_t val = pos;
                        if (ptab) val = (ptab[pos >> a.page_shift] << a.page_shift) | (pos & ((1 << a.page_shift) - 1));
                        out[o] = val;
                    }
                    ++o;
                }
            };
            emit(f0, p); emit(f1, p + 1); emit(f2, p + 2); emit(f3, p + 3);
        }
        __syncthreads();                                       // everyone has read `running`
        if (tid == 0) sh.running = base + all;                 // wave 0: base == running
        ++it;
    };
    for_items(compact_item);
    if (a.block_counts) {                                      // blocks past the row's end
        constexpr int BPI = ITEM / SEL_BLOCK;
        for (int k = n_items * BPI + tid; k < a.blocks_per_row; k += THREADS)
            a.block_counts[(int64_t)r * a.blocks_per_row + k] = 0;
    }
}

template <int THREADS, int NV4, bool RESIDENT>
specattn_status launch_one(const SelectLaunch &a, hipStream_t stream)
{
    const int rows = a.B * a.H_kv;
    hipLaunchKernelGGL((topp_select_kernel<THREADS, NV4, RESIDENT>), dim3(rows), dim3(THREADS), 0, stream, a);
    return check_launch("topp_select_kernel");
}

}  // namespace

specattn_status launch_select(const SelectLaunch &a, hipStream_t stream)
{
    const int n = a.n_max;
    // block counts are per 1024 positions, so every variant has THREADS*4 a multiple of 1024
    if (n <= 1024) return launch_one<256, 1, true>(a, stream);
    if (n <= 2048) return launch_one<256, 2, true>(a, stream);
    if (n <= 4096) return launch_one<256, 4, true>(a, stream);
    if (n <= 8192) return launch_one<512, 4, true>(a, stream);
    if (n <= 16384) return launch_one<1024, 4, true>(a, stream);
    if (n <= 32768) return launch_one<1024, 8, true>(a, stream);
    if (n <= 65536) return launch_one<1024, 16, true>(a, stream);
    return launch_one<1024, 1, false>(a, stream);
}

}  // namespace specattn

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

struct LocSlot {                 // a candidate outcome of one locate step
    unsigned long long packed;
    double m_above;
    unsigned c_above;
    int bin;
};

struct RowShared {
    unsigned long long hist[NB1];
    LocSlot loc[16];
    int loc_state[16];
    double wave_m[16];
    unsigned wave_c[16];
    unsigned wave_tot[2][16];
    unsigned wt[256];            // kept entries per (item, wave), then their exclusive prefix
    double total_m;
    double m_above;
    unsigned c_above;
    unsigned long long bin_packed;
    int best;
    int lowest;
    unsigned running;
};

// What an entry adds to its bin's counter: one to the count, and its 23 significand bits with bit 23 set.  For
// normal numbers that is the significand; subnormal ones (exponent field 0) have no hidden bit, which mass_of
// takes back out for the bins they fall into - cheaper than a compare and a select for every entry.
__device__ __forceinline__ unsigned long long packed_entry(uint32_t u)
{
    return CNT_ONE | ((u & 0x7fffffu) | 0x800000u);
}

// value of a bin whose entries all carry biased exponent field e: (significand sum) * 2^(max(e,1)-150),
// exact (the sum is below 2^44 and the scale is a power of two well inside the fp64 range)
__device__ __forceinline__ double mass_of(unsigned long long packed, int e_field)
{
    long long sig = (long long)(packed & SIG_MASK);
    if (e_field == 0) sig -= (long long)(packed >> CNT_SHIFT) << 23;       // subnormal entries: no hidden bit
    const double s = (double)sig;
    const int e = (e_field > 0 ? e_field : 1) - 150;
    return s * __hiloint2double((1023 + e) << 20, 0);
}

// Cross-lane moves on the vector ALU (no LDS traffic): lanes without a source lane receive 0.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ int dpp_int(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK> __device__ __forceinline__ double dpp_double(double v)
{
    return __hiloint2double(dpp_int<CTRL, ROW_MASK>(__double2hiint(v)), dpp_int<CTRL, ROW_MASK>(__double2loint(v)));
}
// Inclusive prefix sums over the 64 lanes of a wave: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then
// lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ void wave_prefix(double &m, unsigned &c)
{
#define SPECATTN_SCAN_STEP(CTRL, RM) \
    do { m += dpp_double<CTRL, RM>(m); c += (unsigned)dpp_int<CTRL, RM>((int)c); } while (0)
    SPECATTN_SCAN_STEP(0x111, 0xf);    // row_shr:1
    SPECATTN_SCAN_STEP(0x112, 0xf);    // row_shr:2
    SPECATTN_SCAN_STEP(0x114, 0xf);    // row_shr:4
    SPECATTN_SCAN_STEP(0x118, 0xf);    // row_shr:8
    SPECATTN_SCAN_STEP(0x142, 0xa);    // row_bcast:15 into rows 1 and 3
    SPECATTN_SCAN_STEP(0x143, 0xc);    // row_bcast:31 into rows 2 and 3
#undef SPECATTN_SCAN_STEP
}

// Kept-position mask: every lane holds the keep flags of four consecutive positions (bit c = position 4 * lane + c
// of a run of 256); the eight lanes that share a 32-position word combine their nibbles on the vector ALU
// (neighbour, pair and half-row exchanges), after which each of them holds the whole word.
__device__ __forceinline__ uint32_t mask_word(uint32_t nibble, int lane)
{
    int v = (int)(nibble << (4 * (lane & 7)));
    v |= __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);     // quad_perm [1,0,3,2]
    v |= __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);     // quad_perm [2,3,0,1]
    v |= __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);    // row_half_mirror: lane i <-> 7 - i of its eight
    return (uint32_t)v;
}

// One radix pass decision.  hist[0..NB) holds the packed counters of this pass.
// On return (uniform over the block): bin = highest non-empty bin b with
// m_above + mass(bins >= b) >= target (lowest non-empty bin if rounding leaves none),
// and m_above / c_above advanced to cover the bins above it.
// Threads own bins from the top down (thread 0 the highest BPT bins), so "the bins above mine" is a
// prefix over threads: a wave-wide scan, the wave totals through LDS, and every thread knows the mass
// above its own bins; the one thread whose bins hold the boundary finds it among them.
template <int THREADS, int NB, bool FIRST>
__device__ __forceinline__ int locate_bin(RowShared &sh, int e_field_fixed, float top_p, double &target,
                                          double &m_above, unsigned &c_above,
                                          unsigned long long &bin_packed)
{
    constexpr int NW = THREADS / 64;
    constexpr int BPT = NB / THREADS;
    static_assert(BPT >= 1, "more threads than bins");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int top = NB - 1 - (int)threadIdx.x * BPT;           // this thread's highest bin
    // (bins are re-read from LDS wherever they are needed again, rather than kept in registers: the caller holds
    // the whole row in registers and has none to spare)
    auto bin_entry = [&](int j) -> unsigned long long { return sh.hist[top - j]; };
    auto bin_mass = [&](int j, unsigned long long hj) -> double {
        return mass_of(hj, FIRST ? ((top - j) >> 3) : e_field_fixed);
    };
    double lm = 0.0;
    unsigned lc = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        const unsigned long long hj = bin_entry(j);
        lm += bin_mass(j, hj);
        lc += (unsigned)(hj >> CNT_SHIFT);
    }
    double incl_m = lm;
    unsigned incl_c = lc;
    wave_prefix(incl_m, incl_c);
    if (lane == 63) { sh.wave_m[wave] = incl_m; sh.wave_c[wave] = incl_c; }
    // mass and count of the lanes before this one (wave_shr:1)
    double above = dpp_double<0x138, 0xf>(incl_m);
    unsigned above_c = (unsigned)dpp_int<0x138, 0xf>((int)incl_c);
    __syncthreads();
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const double wm = sh.wave_m[w];
        if (w < wave) { above += wm; above_c += sh.wave_c[w]; }
        total += wm;
    }
    if (FIRST) target = (double)top_p * total;     // Algorithm 2: M_target = p * sum a
    if (FIRST && !(total > 0.0)) return -1;        // no mass at all (uniform decision)

    // Masses are non-negative, so the running sum over a thread's bins never decreases: the thread holds a
    // feasible non-empty bin exactly if the sum after its last bin reaches the target.
    double run_end = above;
#pragma unroll
    for (int j = 0; j < BPT; ++j) run_end += bin_mass(j, bin_entry(j));
    const bool holds = lc > 0 && (m_above + run_end) >= target;
    const unsigned long long has = __ballot(holds);
    // per wave: the first lane (highest bins) that holds a feasible bin looks for the highest one among its own
    if (has && lane == __ffsll((unsigned long long)has) - 1) {
        double run = above;
        unsigned runc = above_c;
        bool found = false;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const unsigned long long hj = bin_entry(j);
            const double mj = bin_mass(j, hj);
            const unsigned cj = (unsigned)(hj >> CNT_SHIFT);
            if (!found && cj && (m_above + (run + mj)) >= target) {
                found = true;
                sh.loc[wave].bin = top - j; sh.loc[wave].m_above = run; sh.loc[wave].c_above = runc; sh.loc[wave].packed = hj;
            }
            run += mj;
            runc += cj;
        }
    }
    if (lane == 0) sh.loc_state[wave] = has ? 1 : 0;
    __syncthreads();
    int pick = -1;                                 // first wave with a feasible bin
#pragma unroll
    for (int w = NW - 1; w >= 0; --w)
        if (sh.loc_state[w]) pick = w;
    if (pick < 0) {
        // Rounding left no feasible bin (the row total itself fell short of the target by an ulp): take the
        // lowest non-empty bin.  Uniform over the block, and rare.
        int low = -1;
        double run = above, low_above = 0.0;
        unsigned runc = above_c, low_c = 0;
        unsigned long long low_h = 0;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const unsigned long long hj = bin_entry(j);
            const unsigned cj = (unsigned)(hj >> CNT_SHIFT);
            if (cj) { low = top - j; low_above = run; low_c = runc; low_h = hj; }
            run += bin_mass(j, hj);
            runc += cj;
        }
        const unsigned long long has_low = __ballot(low >= 0);
        if (has_low && lane == 63 - __clzll(has_low)) {
            sh.loc[wave].bin = low; sh.loc[wave].m_above = low_above; sh.loc[wave].c_above = low_c; sh.loc[wave].packed = low_h;
        }
        __syncthreads();                           // every thread has read loc_state
        if (lane == 0) sh.loc_state[wave] = has_low ? 1 : 0;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w)
            if (sh.loc_state[w]) pick = w;         // last wave (lowest bins) with any entry
    }
    const LocSlot &slot = sh.loc[pick];
    const int bin = slot.bin;
    m_above += slot.m_above;
    c_above += slot.c_above;
    bin_packed = slot.packed;
    return bin;
}

template <int THREADS, int NB>
__device__ __forceinline__ void clear_hist(RowShared &sh)
{
    for (int b = threadIdx.x; b < NB; b += THREADS) sh.hist[b] = 0ull;
    __syncthreads();
}

// THREADS threads per row; RESIDENT: the row sits in NV4 uint4 registers per thread.
// Entries of the buffer in which a row's list is staged in list order for contiguous stores (dynamic LDS, so that
// the small workgroups, which are meant to run four to a CU, are not held to three by a buffer sized for the large
// ones; longer lists take several rounds).
constexpr unsigned stage_entries(int threads) { return threads <= 256 ? 4096u : 8192u; }

template <int THREADS, int NV4, bool RESIDENT>
__global__ __launch_bounds__(THREADS, 4) void topp_select_kernel(SelectLaunch a)
{
    __shared__ RowShared sh;
    extern __shared__ __align__(16) int32_t stage_dyn[];
    constexpr int NW = THREADS / 64;
    constexpr int ITEM = THREADS * 4;                 // positions per item (one uint4 per thread)
    const int r = blockIdx.x;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int len = a.seq_lens ? a.seq_lens[b] : a.n_tokens;
    len = len < 0 ? 0 : (len > a.n_tokens ? a.n_tokens : len);
    len = (len + (1 << a.chunk_shift) - 1) >> a.chunk_shift;     // rows of chunk masses: length in chunks
    len = len > a.n_max ? a.n_max : len;
    const float *row = a.probs + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    const int n_items = (len + ITEM - 1) / ITEM;

    // -0.0 is zero; negative, infinite and NaN entries make the row invalid.  Branch-free: the largest bit pattern
    // seen is tested once per thread, and an invalid entry is clamped to the largest finite value so that its bin
    // stays inside the histogram (the row's result is discarded anyway).
    uint32_t worst = 0u;
    auto clean = [&](uint32_t x) -> uint32_t {
        x = (x == 0x80000000u) ? 0u : x;
        worst = worst > x ? worst : x;
        return x < 0x7f7fffffu ? x : 0x7f7fffffu;
    };
    auto clean4 = [&](uint4 u) -> uint4 { return make_uint4(clean(u.x), clean(u.y), clean(u.z), clean(u.w)); };
    // Slow form of an item's load (rows that are not 16-byte aligned or hold fewer than four entries).
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
        return clean4(u);
    };
    // Fast form: every thread issues plain 16-byte loads with nothing between them that waits for data, so
    // all of a thread's loads are in flight together.  An item that reaches past the row's end loads the
    // row's last whole vector instead (in bounds) and is masked afterwards; the at most three entries behind
    // the last whole vector are fetched once, by the thread that owns them.
    const bool vec_ok = aligned && len >= 4;                   // uniform
    const int last4 = (len - 4) & ~3;                          // start of the row's last whole vector
    const int tail_p = (len & 3) ? (len & ~3) : -1;            // start of the partial vector, if any
    uint4 tailv = make_uint4(0, 0, 0, 0);
    if (vec_ok && tail_p >= 0 && tid == (tail_p % ITEM) / 4) {
        tailv.x = __float_as_uint(row[tail_p]);
        if (tail_p + 1 < len) tailv.y = __float_as_uint(row[tail_p + 1]);
        if (tail_p + 2 < len) tailv.z = __float_as_uint(row[tail_p + 2]);
    }
    auto raw_load = [&](int i) -> uint4 {
        const int p = (i * THREADS + tid) * 4;
        // streaming load: a row is read once and should not displace anything in the caches
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + (p < last4 ? p : last4)));
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    auto finish_item = [&](int i, uint4 u) -> uint4 {
        const int p = (i * THREADS + tid) * 4;
        if (p + 3 >= len) u = (p == tail_p) ? tailv : make_uint4(0, 0, 0, 0);
        return clean4(u);
    };

    uint4 data[RESIDENT ? NV4 : 1];
    if (RESIDENT) {
        if (vec_ok) {
#pragma unroll
            for (int i = 0; i < NV4; ++i) data[i] = raw_load(i);
        } else {
#pragma unroll
            for (int i = 0; i < NV4; ++i) data[i] = (i < n_items) ? load_item(i) : make_uint4(0, 0, 0, 0);
        }
    }
    // the histogram is cleared while the loads are in flight
    clear_hist<THREADS, NB1>(sh);
    if (RESIDENT && vec_ok) {
        // Common case first: no sign bit among the thread's entries.  Then nothing needs cleaning, an entry is invalid
        // exactly if its exponent field is all ones, and every bin index stays below NB1 - one OR and one maximum per
        // entry instead of a compare, two selects and a maximum.
        uint32_t any = 0u, top = 0u;
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            const int p = (i * THREADS + tid) * 4;
            uint4 u = data[i];
            if (p + 3 >= len) u = (p == tail_p) ? tailv : make_uint4(0, 0, 0, 0);
            data[i] = u;
            any |= u.x | u.y | u.z | u.w;
            const uint32_t m01 = u.x > u.y ? u.x : u.y, m23 = u.z > u.w ? u.z : u.w;
            const uint32_t m = m01 > m23 ? m01 : m23;
            top = top > m ? top : m;
        }
        if (any & 0x80000000u) {                 // -0.0 or a negative entry somewhere
#pragma unroll
            for (int i = 0; i < NV4; ++i) data[i] = clean4(data[i]);
        } else {
            worst = top;
        }
    }
    auto for_items = [&](auto &&fn) {
        if (RESIDENT) {
#pragma unroll
            for (int i = 0; i < NV4; ++i)
                if (i < n_items) fn(i, data[i]);
        } else {
            // rows too long for the registers: stream them, four loads in flight per thread
            for (int i0 = 0; i0 < n_items; i0 += 4) {
                uint4 u[4];
                if (vec_ok) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) u[k] = raw_load(i0 + k);
#pragma unroll
                    for (int k = 0; k < 4; ++k) u[k] = finish_item(i0 + k, u[k]);
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) u[k] = (i0 + k < n_items) ? load_item(i0 + k) : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (i0 + k < n_items) fn(i0 + k, u[k]);
            }
        }
    };

    // ---- pass 1: bits[30:20] -----------------------------------------------------------------
    // (one histogram per pair of waves instead of one per workgroup measured slower: the atomics of a row's few
    // dozen busy bins are not what bounds this pass)
    for_items([&](int, uint4 u) {
        if (u.x) atomicAdd(&sh.hist[u.x >> 20], packed_entry(u.x));
        if (u.y) atomicAdd(&sh.hist[u.y >> 20], packed_entry(u.y));
        if (u.z) atomicAdd(&sh.hist[u.z >> 20], packed_entry(u.z));
        if (u.w) atomicAdd(&sh.hist[u.w >> 20], packed_entry(u.w));
    });
    const bool any_bad = __syncthreads_or(worst >= 0x7f800000u ? 1 : 0) != 0;     // also orders the atomics

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
        if (a.kept_mask)
            for (int k = tid; k < a.blocks_per_row * (SEL_BLOCK / 32); k += THREADS)
                a.kept_mask[(int64_t)r * a.blocks_per_row * (SEL_BLOCK / 32) + k] = 0u;
        return;
    }
    const int e_field = b1 >> 3;

    // A boundary bin that holds a single entry pins tau*: the bin's significand sum is that entry's
    // significand, and the exponent is the bin's.  Otherwise refine inside the bin.
    auto single_entry_bits = [&](unsigned long long packed) -> uint32_t {
        return ((uint32_t)e_field << 23) | ((uint32_t)packed & 0x7fffffu);
    };
    uint32_t tau_bits;
    if ((bin_packed >> CNT_SHIFT) == 1) {
        tau_bits = single_entry_bits(bin_packed);
    } else {
        // ---- pass 2: bits[19:10] inside bin b1 -----------------------------------------------
        clear_hist<THREADS, NB2>(sh);
        for_items([&](int, uint4 u) {
            if ((u.x >> 20) == (uint32_t)b1 && u.x) atomicAdd(&sh.hist[(u.x >> 10) & 1023u], packed_entry(u.x));
            if ((u.y >> 20) == (uint32_t)b1 && u.y) atomicAdd(&sh.hist[(u.y >> 10) & 1023u], packed_entry(u.y));
            if ((u.z >> 20) == (uint32_t)b1 && u.z) atomicAdd(&sh.hist[(u.z >> 10) & 1023u], packed_entry(u.z));
            if ((u.w >> 20) == (uint32_t)b1 && u.w) atomicAdd(&sh.hist[(u.w >> 10) & 1023u], packed_entry(u.w));
        });
        __syncthreads();
        const int b2 = locate_bin<THREADS, NB2, false>(sh, e_field, a.top_p, target, m_above, c_above, bin_packed);
        const uint32_t prefix = ((uint32_t)b1 << 10) | (uint32_t)b2;
        if ((bin_packed >> CNT_SHIFT) == 1) {
            tau_bits = single_entry_bits(bin_packed);
        } else {
            // ---- pass 3: bits[9:0] inside (b1, b2) -------------------------------------------
            clear_hist<THREADS, NB2>(sh);
            for_items([&](int, uint4 u) {
                if ((u.x >> 10) == prefix && u.x) atomicAdd(&sh.hist[u.x & 1023u], packed_entry(u.x));
                if ((u.y >> 10) == prefix && u.y) atomicAdd(&sh.hist[u.y & 1023u], packed_entry(u.y));
                if ((u.z >> 10) == prefix && u.z) atomicAdd(&sh.hist[u.z & 1023u], packed_entry(u.z));
                if ((u.w >> 10) == prefix && u.w) atomicAdd(&sh.hist[u.w & 1023u], packed_entry(u.w));
            });
            __syncthreads();
            const int b3 = locate_bin<THREADS, NB2, false>(sh, e_field, a.top_p, target, m_above, c_above, bin_packed);
            tau_bits = (prefix << 10) | (uint32_t)b3;             // >= 1: zeros never enter a bin
        }
    }
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
    if (!a.indices && !a.block_counts && !a.kept_mask) return;
    uint32_t *mask_out = a.kept_mask ? a.kept_mask + (int64_t)r * a.blocks_per_row * (SEL_BLOCK / 32) : nullptr;
    const int mask_words = a.blocks_per_row * (SEL_BLOCK / 32);
    // word (i * THREADS + tid) / 8 of the mask covers this thread's four positions of item i; the lane that
    // holds the word's first nibble stores it
    auto emit_mask = [&](int i, uint32_t nibble) {
        const uint32_t word = mask_word(nibble, lane);
        const int w = (i * THREADS + tid) >> 3;
        if ((lane & 7) == 0 && w < mask_words) mask_out[w] = word;
    };

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
        if (mask_out) emit_mask(i, (f0 ? 1u : 0u) | (f1 ? 2u : 0u) | (f2 ? 4u : 0u) | (f3 ? 8u : 0u));
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
    if (RESIDENT) {
        // All items at once.  First only counts: every wave's kept entries per item (four compares and four scalar
        // bit counts; the keep flags are not stored anywhere - comparing again later is cheaper than packing
        // them away and unpacking them), then one workgroup-wide exclusive prefix over the (item, wave) counts,
        // which gives every wave its place in the list.
        constexpr int NE = NV4 * NW;
        static_assert(NE <= 256 && NE <= THREADS && NV4 <= 64, "prefix table too small");
        unsigned my_tot = 0;                                   // lane i: this wave's kept entries of item i
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            const uint4 u = data[i];
            const bool f0 = u.x >= tau_bits, f1 = u.y >= tau_bits, f2 = u.z >= tau_bits, f3 = u.w >= tau_bits;
            const unsigned wtot = __popcll(__ballot(f0)) + __popcll(__ballot(f1)) + __popcll(__ballot(f2)) + __popcll(__ballot(f3));
            if (lane == i) my_tot = wtot;
            if (mask_out) emit_mask(i, (f0 ? 1u : 0u) | (f1 ? 2u : 0u) | (f2 ? 4u : 0u) | (f3 ? 8u : 0u));
        }
        if (lane < NV4) sh.wt[lane * NW + wave] = my_tot;
        __syncthreads();
        if (a.block_counts) {
            constexpr int BPI = ITEM / SEL_BLOCK;              // selection blocks per item
            constexpr int WPB = NW / BPI;                      // waves per block
            for (int blk = tid; blk < NV4 * BPI && blk < a.blocks_per_row; blk += THREADS) {
                unsigned c = 0;
                for (int w = 0; w < WPB; ++w) c += sh.wt[(blk / BPI) * NW + (blk % BPI) * WPB + w];
                a.block_counts[(int64_t)r * a.blocks_per_row + blk] = (int32_t)c;
            }
        }
        if (out) {
            unsigned v = tid < NE ? sh.wt[tid] : 0u, inc = v;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned o = __shfl_up(inc, off, 64);
                if (lane >= off) inc += o;
            }
            if (lane == 63) sh.wave_c[wave] = inc;
            __syncthreads();
            if (tid < NE) {
                unsigned base = 0;
                for (int w = 0; w < wave; ++w) base += sh.wave_c[w];
                sh.wt[tid] = base + inc - v;
            }
            __syncthreads();
            // The row's list is put together in LDS, in list order (a kept entry's rank is its wave's place for the
            // item, plus the kept entries of the lanes before, plus the kept ones before it in its own lane), and goes
            // out with contiguous stores over the whole workgroup: whole cache lines, whatever the kept counts of the
            // single waves are.  Lists longer than the buffer take several rounds.
            constexpr unsigned CH = stage_entries(THREADS);
            int32_t *stage = stage_dyn;
            const unsigned cap = kept < (unsigned)a.idx_capacity ? kept : (unsigned)a.idx_capacity;
            const unsigned my_base = lane < NV4 ? sh.wt[lane * NW + wave] : 0u;    // lane i: this wave's place for item i
            for (unsigned c0 = 0; c0 < cap; c0 += CH) {
                if (c0) __syncthreads();                               // the round before has been read out
                const bool one_round = kept <= CH;                     // (uniform) every rank of the row fits the buffer,
                                                                       // also those beyond a smaller capacity
#pragma unroll
                for (int i = 0; i < NV4; ++i) {
                    const uint4 u = data[i];
                    const bool f0 = u.x >= tau_bits, f1 = u.y >= tau_bits, f2 = u.z >= tau_bits, f3 = u.w >= tau_bits;
                    const unsigned long long m0 = __ballot(f0), m1 = __ballot(f1), m2 = __ballot(f2), m3 = __ballot(f3);
                    if ((m0 | m1 | m2 | m3) == 0ull) continue;         // (uniform over the wave)
                    const unsigned before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m3 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m3,
                                            __builtin_amdgcn_mbcnt_hi((uint32_t)(m2 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m2,
                                            __builtin_amdgcn_mbcnt_hi((uint32_t)(m1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m1,
                                            __builtin_amdgcn_mbcnt_hi((uint32_t)(m0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m0, 0u))))))));
                    const unsigned o0 = (unsigned)__builtin_amdgcn_readlane((int)my_base, i) - c0 + before;   // (wraps around below c0)
                    const unsigned o1 = o0 + (f0 ? 1u : 0u), o2 = o1 + (f1 ? 1u : 0u), o3 = o2 + (f2 ? 1u : 0u);
                    const int p = (i * THREADS + tid) * 4;
                    if (one_round) {
                        if (f0) stage[o0] = p;
                        if (f1) stage[o1] = p + 1;
                        if (f2) stage[o2] = p + 2;
                        if (f3) stage[o3] = p + 3;
                    } else {
                        if (f0 && o0 < CH) stage[o0] = p;
                        if (f1 && o1 < CH) stage[o1] = p + 1;
                        if (f2 && o2 < CH) stage[o2] = p + 2;
                        if (f3 && o3 < CH) stage[o3] = p + 3;
                    }
                }
                __syncthreads();
                const unsigned nround = (cap - c0) < CH ? (cap - c0) : CH;
                for (unsigned k = tid; k < nround; k += THREADS) {
                    int32_t val = stage[k];
                    if (ptab) val = (ptab[val >> a.page_shift] << a.page_shift) | (val & ((1 << a.page_shift) - 1));
                    out[c0 + k] = val;
                }
            }
        }
    } else {
        for_items(compact_item);
    }
    if (a.block_counts) {                                      // blocks past the row's end
        constexpr int BPI = ITEM / SEL_BLOCK;
        for (int k = (RESIDENT ? NV4 : n_items) * BPI + tid; k < a.blocks_per_row; k += THREADS)
            a.block_counts[(int64_t)r * a.blocks_per_row + k] = 0;
    }
    if (mask_out)                                              // words past the last item
        for (int k = (RESIDENT ? NV4 : n_items) * (ITEM / 32) + tid; k < mask_words; k += THREADS) mask_out[k] = 0u;
}

template <int THREADS, int NV4, bool RESIDENT>
specattn_status launch_one(const SelectLaunch &a, hipStream_t stream)
{
    const int rows = a.B * a.H_kv;
    hipLaunchKernelGGL((topp_select_kernel<THREADS, NV4, RESIDENT>), dim3(rows), dim3(THREADS), stage_entries(THREADS) * sizeof(int32_t),
                       stream, a);
    return check_launch("topp_select_kernel");
}

// ---- few long rows: one row split over many workgroups ------------------------------------------------
// The same three radix passes, but every workgroup histograms one slice (a multiple of MW_SLICE positions,
// chosen so that about two workgroups per CU are in flight) in LDS and
// adds its non-empty bins to the row's histogram in memory (64-bit integer atomics: the sums stay exact and
// independent of order).  Kernel boundaries separate the passes; at the start of the next pass every
// workgroup of a row locates the boundary bin from the finished histogram by itself (identical code on
// identical data), and slice 0 records the outcome for the kernels that follow.
constexpr int MW_THREADS = 256;
constexpr int MW_SLICE = 4096;

struct MwStage {                     // outcome of one locate step
    unsigned long long bin_packed;
    double target, m_above;
    unsigned c_above;
    int bin;
    int done;                        // the boundary bin held a single entry: tau_bits is final
    uint32_t tau_bits;
};
struct MwState {
    MwStage s1, s2;
    int bad;                         // an entry was NaN, negative or infinite
    int invalid;                     // no mass at all
};
struct MwLaunch {
    SelectLaunch a;
    unsigned long long *h1, *h2, *h3;    // [rows][NB1], [rows][NB2], [rows][NB2]
    MwState *state;                      // [rows]
    int slices, slice_len;               // workgroups per row; positions per workgroup (a multiple of MW_SLICE)
    float *tau;                          // [rows] out
    int32_t *valid;                      // [rows] out: 1 unless the row is invalid
    uint32_t *flags;                     // [rows] out
};

__global__ void mw_clear_kernel(unsigned long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}

__device__ __forceinline__ int mw_row_len(const SelectLaunch &a, int b)
{
    int len = a.seq_lens ? a.seq_lens[b] : a.n_tokens;
    len = len < 0 ? 0 : (len > a.n_tokens ? a.n_tokens : len);
    return len > a.n_max ? a.n_max : len;
}

template <int PASS>
__global__ __launch_bounds__(MW_THREADS) void mw_pass_kernel(MwLaunch w)
{
    __shared__ RowShared sh;
    const SelectLaunch &a = w.a;
    const int r = blockIdx.x / w.slices, sl = blockIdx.x - r * w.slices;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int tid = threadIdx.x;
    const int len = mw_row_len(a, b);
    MwState &st = w.state[r];
    uint32_t want = 0;                 // PASS 2: bits[30:20] == want; PASS 3: bits[30:10] == want
    if (PASS >= 2) {
        if (st.bad || len == 0) return;
        const unsigned long long *hg = PASS == 2 ? w.h1 + (size_t)r * NB1 : w.h2 + (size_t)r * NB2;
        for (int k = tid; k < (PASS == 2 ? NB1 : NB2); k += MW_THREADS) sh.hist[k] = hg[k];
        __syncthreads();
        double target = 0.0, m_above = 0.0;
        unsigned c_above = 0;
        unsigned long long bin_packed = 0;
        int bin, e_field;
        if (PASS == 2) {
            bin = locate_bin<MW_THREADS, NB1, true>(sh, 0, a.top_p, target, m_above, c_above, bin_packed);
            if (bin < 0) {
                if (sl == 0 && tid == 0) st.invalid = 1;
                return;
            }
            e_field = bin >> 3;
            want = (uint32_t)bin;
        } else {
            if (st.invalid || st.s1.done) return;
            target = st.s1.target; m_above = st.s1.m_above; c_above = st.s1.c_above;
            e_field = st.s1.bin >> 3;
            bin = locate_bin<MW_THREADS, NB2, false>(sh, e_field, a.top_p, target, m_above, c_above, bin_packed);
            want = ((uint32_t)st.s1.bin << 10) | (uint32_t)bin;
        }
        const bool single = (bin_packed >> CNT_SHIFT) == 1;
        if (sl == 0 && tid == 0) {
            MwStage &o = PASS == 2 ? st.s1 : st.s2;
            o.bin_packed = bin_packed; o.target = target; o.m_above = m_above; o.c_above = c_above; o.bin = bin;
            o.done = single ? 1 : 0;
            o.tau_bits = ((uint32_t)e_field << 23) | ((uint32_t)bin_packed & 0x7fffffu);
        }
        if (single) return;
        __syncthreads();               // locate_bin's readers of sh.hist are done
    }
    constexpr int NB = PASS == 1 ? NB1 : NB2;
    for (int k = tid; k < NB; k += MW_THREADS) sh.hist[k] = 0ull;
    __syncthreads();
    const float *row = a.probs + (int64_t)b * a.stride_b + (int64_t)h * a.stride_h;
    const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    bool bad = false;
    int p_end = (sl + 1) * w.slice_len;
    p_end = p_end > len ? len : p_end;
    for (int p = sl * w.slice_len + tid * 4; p < p_end; p += MW_THREADS * 4) {
        uint4 u = make_uint4(0, 0, 0, 0);
        if (p + 3 < len && aligned) {
            u = *reinterpret_cast<const uint4 *>(row + p);
        } else {
            if (p < len) u.x = __float_as_uint(row[p]);
            if (p + 1 < len) u.y = __float_as_uint(row[p + 1]);
            if (p + 2 < len) u.z = __float_as_uint(row[p + 2]);
            if (p + 3 < len) u.w = __float_as_uint(row[p + 3]);
        }
        auto visit = [&](uint32_t x) {
            if (x == 0x80000000u) x = 0u;                               // -0.0 is zero
            if (x >= 0x7f800000u) { bad = true; return; }               // negative, infinite, NaN
            if (!x) return;
            if (PASS == 1) atomicAdd(&sh.hist[x >> 20], packed_entry(x));
            else if (PASS == 2) { if ((x >> 20) == want) atomicAdd(&sh.hist[(x >> 10) & 1023u], packed_entry(x)); }
            else { if ((x >> 10) == want) atomicAdd(&sh.hist[x & 1023u], packed_entry(x)); }
        };
        visit(u.x); visit(u.y); visit(u.z); visit(u.w);
    }
    const bool any_bad = __syncthreads_or(bad ? 1 : 0) != 0;             // also orders the LDS atomics
    if (PASS == 1 && any_bad && tid == 0) atomicOr(&st.bad, 1);
    unsigned long long *hg = (PASS == 1 ? w.h1 + (size_t)r * NB1 : PASS == 2 ? w.h2 + (size_t)r * NB2 : w.h3 + (size_t)r * NB2);
    for (int k = tid; k < NB; k += MW_THREADS) {
        const unsigned long long v = sh.hist[k];
        if (v) atomicAdd(&hg[k], v);
    }
}

// One workgroup per row: the last locate step, tau*, validity and the boundary flag.
__global__ __launch_bounds__(MW_THREADS) void mw_final_kernel(MwLaunch w)
{
    __shared__ RowShared sh;
    const SelectLaunch &a = w.a;
    const int r = blockIdx.x, b = r / a.H_kv, tid = threadIdx.x;
    const int len = mw_row_len(a, b);
    const MwState &st = w.state[r];
    if (st.bad || st.invalid || len == 0) {
        if (tid == 0) { w.tau[r] = 0.0f; w.valid[r] = 0; w.flags[r] = SPECATTN_ROW_INVALID; }
        return;
    }
    const int e_field = st.s1.bin >> 3;
    double target = st.s1.target, m_above;
    unsigned long long bin_packed;
    uint32_t tau_bits;
    if (st.s1.done) {
        tau_bits = st.s1.tau_bits; m_above = st.s1.m_above; bin_packed = st.s1.bin_packed;
    } else if (st.s2.done) {
        tau_bits = st.s2.tau_bits; m_above = st.s2.m_above; bin_packed = st.s2.bin_packed;
    } else {
        for (int k = tid; k < NB2; k += MW_THREADS) sh.hist[k] = w.h3[(size_t)r * NB2 + k];
        __syncthreads();
        m_above = st.s2.m_above;
        unsigned c_above = st.s2.c_above;
        const int b3 = locate_bin<MW_THREADS, NB2, false>(sh, e_field, a.top_p, target, m_above, c_above, bin_packed);
        tau_bits = ((uint32_t)st.s1.bin << 20) | ((uint32_t)st.s2.bin << 10) | (uint32_t)b3;
    }
    if (tid == 0) {
        const double row_sum = target / (double)a.top_p;
        const double m_incl = m_above + mass_of(bin_packed, e_field), band = 1e-6 * row_sum;
        w.tau[r] = __uint_as_float(tau_bits);
        w.valid[r] = 1;
        w.flags[r] = (fabs(m_incl - target) <= band || fabs(m_above - target) <= band) ? SPECATTN_ROW_NEAR_BOUNDARY : 0u;
    }
}

inline size_t mw_align(size_t x) { return (x + 255) & ~(size_t)255; }

// One thread per (row, chunk): the chunk's entries are added up in fp64 in ascending position order and
// the sum is rounded once to fp32 (Section 4: chunk-granular selection; the score of a chunk is its mass).
__global__ __launch_bounds__(256) void chunk_mass_kernel(const float *__restrict__ probs, int64_t stride_b,
                                                         int64_t stride_h, int H, int n_tokens,
                                                         const int32_t *__restrict__ seq_lens, int chunk_shift,
                                                         int n_chunks, int64_t total, float *__restrict__ mass)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    const int64_t r = gid / n_chunks;
    const int c = (int)(gid - r * n_chunks);
    const int b = (int)(r / H), h = (int)(r - (int64_t)b * H);
    int len = seq_lens ? seq_lens[b] : n_tokens;
    len = len < 0 ? 0 : (len > n_tokens ? n_tokens : len);
    const float *row = probs + (int64_t)b * stride_b + (int64_t)h * stride_h;
    const int chunk = 1 << chunk_shift;
    const int p0 = c << chunk_shift;
    int p1 = p0 + chunk;
    p1 = p1 > len ? len : p1;
    double sum = 0.0;
    bool bad = false;
    auto add = [&](float x) {
        const uint32_t u = __float_as_uint(x);
        if (u > 0x80000000u || (u & 0x7fffffffu) >= 0x7f800000u) bad = true;     // negative, infinite or NaN
        sum += (double)x;
    };
    if (p1 == p0 + chunk && chunk >= 4 && (reinterpret_cast<uintptr_t>(row + p0) & 15) == 0) {
        for (int p = p0; p < p1; p += 4) {
            const float4 v = *reinterpret_cast<const float4 *>(row + p);
            add(v.x); add(v.y); add(v.z); add(v.w);
        }
    } else {
        for (int p = p0; p < p1; ++p) add(row[p]);
    }
    mass[gid] = bad ? __uint_as_float(0x7fc00000u) : (float)sum;
}

}  // namespace

specattn_status launch_chunk_masses(const float *probs, int64_t stride_b, int64_t stride_h, int B, int H, int n_tokens,
                                    const int32_t *seq_lens, int chunk_shift, int n_chunks, float *mass,
                                    hipStream_t stream)
{
    const int64_t total = (int64_t)B * H * n_chunks;
    const unsigned grid = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(chunk_mass_kernel, dim3(grid), dim3(256), 0, stream, probs, stride_b, stride_h, H, n_tokens,
                       seq_lens, chunk_shift, n_chunks, total, mass);
    return check_launch("chunk_mass_kernel");
}

bool select_multi_wg_preferred(int rows, int n)
{
    // One workgroup per row leaves most of the chip idle when there are few rows, and rows beyond 65536
    // entries do not fit its registers; the split path costs six more launches and re-reads the rows from
    // L2 in every pass.  Measured crossover: 32 rows at 65536 entries, 64 at 131072, 128 at 262144.
    return n >= 65536 && (int64_t)rows * 2048 <= n;
}

size_t select_multi_wg_bytes(int rows, int n)
{
    const size_t R = (size_t)rows;
    return mw_align(R * NB1 * 8) + 2 * mw_align(R * NB2 * 8) + mw_align(R * sizeof(MwState));
}

// tau / valid / flags of every row by the split path; `scratch` holds select_multi_wg_bytes
specattn_status launch_select_multi_wg(const SelectLaunch &a, void *scratch, float *tau, int32_t *valid, uint32_t *flags,
                                       hipStream_t stream)
{
    const int rows = a.B * a.H_kv;
    const size_t R = (size_t)rows;
    MwLaunch w;
    w.a = a;
    char *p = static_cast<char *>(scratch);
    w.h1 = reinterpret_cast<unsigned long long *>(p); p += mw_align(R * NB1 * 8);
    w.h2 = reinterpret_cast<unsigned long long *>(p); p += mw_align(R * NB2 * 8);
    w.h3 = reinterpret_cast<unsigned long long *>(p); p += mw_align(R * NB2 * 8);
    w.state = reinterpret_cast<MwState *>(p);
    {
        const int blocks = (a.n_max + MW_SLICE - 1) / MW_SLICE;
        int k = (int)((R * blocks + 2 * cu_count() - 1) / (2 * cu_count()));      // blocks per workgroup
        k = k < 1 ? 1 : (k > 16 ? 16 : k);
        w.slice_len = k * MW_SLICE;
        w.slices = (a.n_max + w.slice_len - 1) / w.slice_len;
    }
    w.tau = tau; w.valid = valid; w.flags = flags;
    const size_t words = select_multi_wg_bytes(rows, a.n_max) / 8;
    hipLaunchKernelGGL(mw_clear_kernel, dim3((unsigned)((words + 1023) / 1024 < 2048 ? (words + 1023) / 1024 : 2048)), dim3(256), 0,
                       stream, w.h1, words);
    specattn_status st = check_launch("mw_clear_kernel");
    if (st != SPECATTN_OK) return st;
    const dim3 grid((unsigned)(R * w.slices));
    hipLaunchKernelGGL(mw_pass_kernel<1>, grid, dim3(MW_THREADS), 0, stream, w);
    hipLaunchKernelGGL(mw_pass_kernel<2>, grid, dim3(MW_THREADS), 0, stream, w);
    hipLaunchKernelGGL(mw_pass_kernel<3>, grid, dim3(MW_THREADS), 0, stream, w);
    st = check_launch("mw_pass_kernel");
    if (st != SPECATTN_OK) return st;
    hipLaunchKernelGGL(mw_final_kernel, dim3(rows), dim3(MW_THREADS), 0, stream, w);
    return check_launch("mw_final_kernel");
}

specattn_status launch_select(const SelectLaunch &a, hipStream_t stream)
{
    const int n = a.n_max;
    // Many rows: small workgroups, several per CU, so that one row's load overlaps another row's
    // passes.  Few rows: as many threads per row as its length allows, for latency.
    const bool many = a.B * a.H_kv >= 2 * cu_count();
    // block counts are per 1024 positions, so every variant has THREADS*4 a multiple of 1024
    if (n <= 1024) return launch_one<256, 1, true>(a, stream);
    if (n <= 2048) return launch_one<256, 2, true>(a, stream);
    if (n <= 4096) return launch_one<256, 4, true>(a, stream);
    if (n <= 8192) return many ? launch_one<256, 8, true>(a, stream) : launch_one<512, 4, true>(a, stream);
    if (n <= 16384) return many ? launch_one<256, 16, true>(a, stream) : launch_one<1024, 4, true>(a, stream);
    if (n <= 32768) return many ? launch_one<512, 16, true>(a, stream) : launch_one<1024, 8, true>(a, stream);
    if (n <= 65536) return launch_one<1024, 16, true>(a, stream);
    return launch_one<1024, 1, false>(a, stream);
}

}  // namespace specattn

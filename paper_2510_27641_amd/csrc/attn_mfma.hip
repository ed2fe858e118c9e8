// Sparse decode attention over a selected index list or kept-position mask (Section 3.1.2, Eq. 2-3;
// Section 3.5), bf16 or fp16, d = 128, up to 32 query rows per kv head and launch: the gfx950
// matrix-core variant.
//
// Work split ("stream-K" over kept positions): the kept positions of all rows, in 32-position
// tiles, form one line; the line is cut into equal shares, one per workgroup (one workgroup of eight waves
// per CU), so the split is balanced by the *kept* count whatever the per-row counts are.  A fixed
// permutation of the workgroup numbers puts the owners of consecutive shares on different XCDs.  A share
// that crosses row boundaries yields one partial (m, l, o) per (row, workgroup); partial (r, w) lives in
// slot w + r.  merge_partials_kernel combines a row's partials, in workgroup order.  Inside a share tile k goes
// to wave k mod 8, so every sum is taken in a fixed order and the outputs are bit-identical from run to run.
// Measured and dropped: waves claiming the tiles of a share from an LDS counter as their data arrives (no
// faster on any workload, 1.3 us slower on the 32K layer, and it gives the fixed summation order up); tiles of
// a row claimed by all of its workgroups from a counter in memory (a device-scope atomic takes about as long
// as a tile under load - 5 us - and claims made that far ahead leave as much unbalanced work at the end as they
// remove); the merge folded into this kernel (last arriver per row: write-through stores, an atomic and
// device-scope loads in a row cost 14 us after the last tile, against 8 us for the wrap-up plus the second
// launch).
//
// Data path per wave and tile: the 32 gathered K rows and the 32 V rows (256 B each) go from HBM
// straight into LDS (global_load_lds: 16 lanes fetch one full row, four rows per instruction,
// XOR-swizzled chunk order).  Each wave owns one K buffer and one V buffer; the next tile's K is
// requested as soon as this tile's K fragments are in registers, the next V as soon as this tile's
// V has been consumed.  The list words of a tile (or the words of the kept mask) are fetched the same way,
// by LDS-DMA into two small slots per wave, one iteration ahead of the gathers that need them: nothing a
// tile needs is waited for when its turn comes, and no barrier separates the tiles of a share.
//   S^T = K Q^T    : mfma 16x16x32 bf16, A = K fragment (ds_read_b128), B = Q fragment (Q tile in LDS)
//   softmax        : running reference max per query row, rescaled only when exceeded by 2^8
//   O^T += V^T P^T : A = V^T fragment (ds_read_b64_tr_b16), B = P split into bf16 hi + lo parts
// The mfma output layout puts each query row in a fixed lane, so scores, weights and output
// accumulators of that row never leave the lane.
#include "common.h"

#include <mutex>

namespace specattn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// The two 16-bit element types the matrix cores take here.  Both contractions use the 16x16x32 shape;
// the softmax weights are handed over as a high part (the weight rounded to the element type) and a low
// part (the rounding error, rounded again), so that the type's short significand costs no accuracy.
template <bool F16> struct Half;
template <> struct Half<false> {
    typedef bf16x8 x8;
    typedef bf16x2 x2;
    static __device__ __forceinline__ f32x4 mfma(x8 a, x8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
};
template <> struct Half<true> {
    typedef f16x8 x8;
    typedef f16x2 x2;
    static __device__ __forceinline__ f32x4 mfma(x8 a, x8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
};

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int NW = ATTN_MFMA_WAVES;   // waves per workgroup
constexpr int THREADS = NW * 64;
constexpr int WG_PER_CU = 8 / NW;     // eight waves per CU in all
constexpr int TILE = 32;              // positions per tile
constexpr int D = 128;
constexpr int ROW_BYTES = D * 2;      // one K or V row
constexpr int TILE_BYTES = TILE * ROW_BYTES;          // 8 KiB per tensor
constexpr int WAVE_LDS = 2 * TILE_BYTES;              // K buffer, V buffer
constexpr int MAX_ROWS = ATTN_MFMA_MAX_ROWS;          // rows whose cost prefix fits the LDS table
constexpr int MAX_BLOCKS = SPECATTN_MAX_N / SEL_BLOCK;   // selection blocks per row, at most
constexpr int SLOT_BYTES = 256;       // one wave-wide LDS-DMA of 4 bytes per lane
constexpr int KV_AUX = 2;             // cache policy of the K/V gathers: non-temporal (each row is used once)
constexpr int SEG_COST = 12;          // cost of picking a row up, in tiles
constexpr float RESCALE_SLACK = 8.0f; // log2 units the running max may exceed the reference by

// dynamic LDS, in bytes from the start
constexpr int OFF_WSUM = NW * WAVE_LDS;                         // int[NW]
constexpr int OFF_MISC = OFF_WSUM + NW * 4;                     // int[4]: spare
constexpr int OFF_SLOT = (OFF_MISC + 16 + 255) & ~255;          // [NW][2][SLOT_BYTES] list / mask words in flight;
                                                                // a wave's (m, l) table of the wave merge uses its first slot
constexpr int OFF_SCAT = OFF_SLOT + NW * 2 * SLOT_BYTES;        // uint[NW][2][32] positions of a tile (mask source)
constexpr int OFF_Q = OFF_SCAT + NW * 256;                      // Q tile [2 * 16][256 B], chunks swizzled like K
// Behind Q: the row tables (cost prefix and kept counts of up to MAX_ROWS_LIST rows), then a row's block prefix (mask
// source).  Calls of up to 64 rows keep their row tables in the first kilobyte, and the mask source then uses the
// rest of the region for the block counts of all rows.
constexpr int OFF_TAB = OFF_Q + 2 * 16 * ROW_BYTES;
constexpr int MAX_ROWS_LIST = ATTN_MFMA_MAX_ROWS_LIST;
constexpr int BC_ALL = 2048;
constexpr int FEW_ROWS = 64;                                    // rows a single wave scans by itself
constexpr int OFF_BC = OFF_TAB + 1024;                          // int[BC_ALL] block counts of all rows (mask source, <= FEW_ROWS rows)
constexpr int TAB_BYTES = (2 * MAX_ROWS_LIST + 1) * 4;          // int[rows + 1] cost prefix, int[rows] kept counts, clamped
constexpr int OFF_BLK = OFF_TAB + TAB_BYTES;                    // int[MAX_BLOCKS + 1] kept before block (mask source)
constexpr int LDS_BYTES = OFF_BLK + (MAX_BLOCKS + 1) * 4;
static_assert((2 * FEW_ROWS + 1) * 4 <= 1024 && 1024 + BC_ALL * 4 <= TAB_BYTES, "the block counts must fit behind the tables of a small call");
static_assert(16 * 2 * 2 * 4 <= SLOT_BYTES, "a wave's (m, l) table must fit its first slot");
static_assert(LDS_BYTES * WG_PER_CU <= 160 * 1024, "the workgroups of a CU must fit its LDS");

// 16-byte chunk c of row `row` is stored in slot c ^ swz(row): makes both the K fragment reads
// (16 rows x one chunk) and the V transpose reads (8 rows x 32 B) spread over all banks.
__device__ __forceinline__ int swz(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }

// Where the gathered rows live.  A list entry is a logical position (contiguous layout) or a pool
// slot page * page_size + offset (paged layouts; logical positions are mapped through the page
// table when the tile's row offsets are formed).
enum Layout { CONTIGUOUS = 0, PAGE_TABLE = 1, PHYSICAL = 2 };
// Where a row's kept positions come from: an index list in memory (also chunk lists and dense calls, which
// have no list at all), or the kept-position mask and per-block counts of the selection (fused call).
enum Source { LIST = 0, MASK = 1 };

struct KvMap {
    int64_t base, stride_n, stride_page;
    const int32_t *ptab;
    int page_shift;
    // row offsets (16-byte units, relative to `base`) of N positions, the page-table loads (if any) in flight together
    template <int LAYOUT, int N> __device__ __forceinline__ void rel_n(const int (&idx)[N], uint32_t (&off16)[N]) const
    {
        if (LAYOUT == CONTIGUOUS) {
#pragma unroll
            for (int i = 0; i < N; ++i) off16[i] = (uint32_t)(((int64_t)idx[i] * stride_n) >> 3);
            return;
        }
        const int mask = (1 << page_shift) - 1;
        int page[N];
#pragma unroll
        for (int i = 0; i < N; ++i) page[i] = LAYOUT == PAGE_TABLE ? ptab[idx[i] >> page_shift] : (idx[i] >> page_shift);
#pragma unroll
        for (int i = 0; i < N; ++i) off16[i] = (uint32_t)(((int64_t)page[i] * stride_page + (int64_t)(idx[i] & mask) * stride_n) >> 3);
    }
};

template <int LAYOUT> __device__ __forceinline__ KvMap make_map(const AttnLaunch &a, int b, int h)
{
    KvMap m;
    m.base = LAYOUT == CONTIGUOUS ? (int64_t)b * a.kv_stride_b + (int64_t)h * a.kv_stride_h : (int64_t)h * a.kv_stride_h;
    m.stride_n = a.kv_stride_n;
    m.stride_page = a.kv_stride_page;
    m.ptab = LAYOUT == PAGE_TABLE ? a.page_table + (int64_t)b * a.max_pages : nullptr;
    m.page_shift = a.page_shift;
    return m;
}

// LDS reads are issued by hand, each batch together with its wait in one asm block: the compiler
// then neither adds waits for the gathers still in flight (it cannot tell them from the data being
// read) nor touches a result register before the data has arrived.
struct KFrags { u32x4 f[2][4]; };     // [position tile][k-step]
__device__ __forceinline__ void lds_read_k(KFrags &k, const uint32_t (&addr)[4])
{
    asm volatile(
        "ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n"
        "ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %9 offset:4096\n"
        "ds_read_b128 %6, %10 offset:4096\n ds_read_b128 %7, %11 offset:4096\n"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(k.f[0][0]), "=&v"(k.f[0][1]), "=&v"(k.f[0][2]), "=&v"(k.f[0][3]),
          "=&v"(k.f[1][0]), "=&v"(k.f[1][1]), "=&v"(k.f[1][2]), "=&v"(k.f[1][3])
        : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3])
        : "memory");
}
// The Q fragments of one 16-row query tile (k-steps 0..3) from the Q tile staged in LDS.
struct QFrags { u32x4 f[4]; };
__device__ __forceinline__ void lds_read_q(QFrags &q, const uint32_t (&addr)[4], bool second_tile)
{
    if (!second_tile)
        asm volatile(
            "ds_read_b128 %0, %4\n ds_read_b128 %1, %5\n ds_read_b128 %2, %6\n ds_read_b128 %3, %7\n"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(q.f[0]), "=&v"(q.f[1]), "=&v"(q.f[2]), "=&v"(q.f[3])
            : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3])
            : "memory");
    else
        asm volatile(
            "ds_read_b128 %0, %4 offset:4096\n ds_read_b128 %1, %5 offset:4096\n"
            "ds_read_b128 %2, %6 offset:4096\n ds_read_b128 %3, %7 offset:4096\n"
            "s_waitcnt lgkmcnt(0)"
            : "=&v"(q.f[0]), "=&v"(q.f[1]), "=&v"(q.f[2]), "=&v"(q.f[3])
            : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3])
            : "memory");
}
// Transposing reads: within each group of 16 lanes, lane i receives element i%4 of the four 8-byte
// rows addressed by lanes i/4, i/4+4, i/4+8 and i/4+12.  Four dv tiles, both halves of the tile.
struct VFrags { u32x2 f[4][2]; };     // [dv tile][half]
__device__ __forceinline__ void lds_read_v(VFrags &v, uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3)
{
    asm volatile(
        "ds_read_b64_tr_b16 %0, %8\n ds_read_b64_tr_b16 %1, %8 offset:4096\n"
        "ds_read_b64_tr_b16 %2, %9\n ds_read_b64_tr_b16 %3, %9 offset:4096\n"
        "ds_read_b64_tr_b16 %4, %10\n ds_read_b64_tr_b16 %5, %10 offset:4096\n"
        "ds_read_b64_tr_b16 %6, %11\n ds_read_b64_tr_b16 %7, %11 offset:4096\n"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(v.f[0][0]), "=&v"(v.f[0][1]), "=&v"(v.f[1][0]), "=&v"(v.f[1][1]),
          "=&v"(v.f[2][0]), "=&v"(v.f[2][1]), "=&v"(v.f[3][0]), "=&v"(v.f[3][1])
        : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
        : "memory");
}
// The 8 words a lane needs of a tile's 32: words addr/4, addr/4 + 4, ...
__device__ __forceinline__ void lds_read_entries(uint32_t (&e)[8], uint32_t addr)
{
    asm volatile(
        "ds_read_b32 %0, %8\n ds_read_b32 %1, %8 offset:16\n ds_read_b32 %2, %8 offset:32\n"
        "ds_read_b32 %3, %8 offset:48\n ds_read_b32 %4, %8 offset:64\n ds_read_b32 %5, %8 offset:80\n"
        "ds_read_b32 %6, %8 offset:96\n ds_read_b32 %7, %8 offset:112\n"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(e[0]), "=&v"(e[1]), "=&v"(e[2]), "=&v"(e[3]), "=&v"(e[4]), "=&v"(e[5]), "=&v"(e[6]), "=&v"(e[7])
        : "v"(addr)
        : "memory");
}
__device__ __forceinline__ uint32_t lds_read_word(uint32_t addr)
{
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1\n s_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ void lds_write_word(uint32_t addr, uint32_t v)
{
    asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// value of `v` in lane `src_lane` (a cross-lane read through the LDS crossbar; no memory is touched)
__device__ __forceinline__ uint32_t lane_read(uint32_t v, int src_lane)
{
    uint32_t r;
    asm volatile("ds_bpermute_b32 %0, %1, %2\n s_waitcnt lgkmcnt(0)" : "=&v"(r) : "v"(src_lane << 2), "v"(v) : "memory");
    return r;
}
// One word from global memory, waited for on the spot.  Written out because a load the compiler tracks makes it wait
// for everything in flight (the gathers included) wherever the loaded value may be used, taken or not.
__device__ __forceinline__ uint32_t global_read_word(const uint32_t *p)
{
    uint32_t r;
    asm volatile("global_load_dword %0, %1, off\n s_waitcnt vmcnt(0)" : "=&v"(r) : "v"(p) : "memory");
    return r;
}
// The same for two values at once (one round trip through the crossbar instead of two).
__device__ __forceinline__ void lane_read2(uint32_t a, uint32_t b, int src_lane, uint32_t &ra, uint32_t &rb)
{
    asm volatile("ds_bpermute_b32 %0, %2, %3\n ds_bpermute_b32 %1, %2, %4\n s_waitcnt lgkmcnt(0)"
                 : "=&v"(ra), "=&v"(rb) : "v"(src_lane << 2), "v"(a), "v"(b) : "memory");
}
// Forward permute: every lane pushes `v` to lane `dst_lane`; a lane nobody pushes to receives 0, and of several
// pushes to one lane the highest pushing lane's value arrives.
__device__ __forceinline__ uint32_t lane_push(uint32_t v, int dst_lane)
{
    uint32_t r;
    asm volatile("ds_permute_b32 %0, %1, %2\n s_waitcnt lgkmcnt(0)" : "=&v"(r) : "v"(dst_lane << 2), "v"(v) : "memory");
    return r;
}
// Inclusive prefix maximum over lanes 0..31 (the two lower rows of 16 lanes) on the vector ALU.
__device__ __forceinline__ int prefix_max32(int v)
{
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false));    // row_shr:1
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false));    // row_shr:2
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false));    // row_shr:4
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false));    // row_shr:8
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false));    // row_bcast:15 into rows 1 and 3
    return v;
}
// Index of the k-th set bit of x (k = 0 is the lowest; k must be below the number of set bits).
__device__ __forceinline__ int kth_set_bit(uint32_t x, int k)
{
    int r = 0, c;
    c = __popc(x & 0xffffu); if (k >= c) { k -= c; r = 16; x >>= 16; }
    c = __popc(x & 0xffu);   if (k >= c) { k -= c; r += 8; x >>= 8; }
    c = __popc(x & 0xfu);    if (k >= c) { k -= c; r += 4; x >>= 4; }
    c = __popc(x & 0x3u);    if (k >= c) { k -= c; r += 2; x >>= 2; }
    c = (int)(x & 1u);       if (k >= c) { r += 1; }
    return r;
}
// Workgroup barrier for data handed over through LDS only: waits for this wave's LDS operations, not for its
// outstanding global loads (a plain __syncthreads() also waits for every gather and prefetch still in flight).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n s_barrier" ::: "memory"); }

// Waits on the vector-memory counter with a run-time count (the instruction takes an immediate).
__device__ __forceinline__ void vm_wait(int n)
{
    switch (n) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
    case 9: asm volatile("s_waitcnt vmcnt(9)" ::: "memory"); break;
    case 10: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
    case 17: asm volatile("s_waitcnt vmcnt(17)" ::: "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}

struct Plan {
    float *part_ml;           // [slots][QTP][2]
    float *part_o;            // [slots][QTP][D]
    int32_t *cost_prefix;     // [rows + 1] in the workspace (written by workgroup 0, read by the merge kernel)
    int n_wg;
};

// Cost of a row on the line the workgroups share out: its tiles, plus SEG_COST for picking the row up
// (fresh Q, partial write), so that workgroups holding many short rows get fewer tiles.
__device__ __forceinline__ int row_cost(int count) { return count > 0 ? (count + TILE - 1) / TILE + SEG_COST : 0; }

// Exclusive prefix of the row costs into pre[0..rows], every workgroup for itself.
__device__ __forceinline__ void cost_prefix(const AttnLaunch &a, int rows, int *pre, int *cnt, int *wsum)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (rows <= FEW_ROWS) {
        // Few rows: every wave scans all of them by itself and writes the (identical) tables; a wave reads
        // back only after its own writes (LDS operations of a wave complete in order), so no barrier is needed.
        const int c = lane < rows ? attn_row_count(a, lane) : 0;
        const int cost = row_cost(c);
        const int inc = wave_inclusive_sum(cost);
        if (lane < rows) { cnt[lane] = c; pre[lane] = inc - cost; }
        if (lane == 63) pre[rows] = inc;                  // lanes past the last row add nothing
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        return;
    }
    // Many rows: THREADS rows per round (the counts of all rounds are requested at once), a wave-wide scan, the
    // wave totals through LDS, the rounds before carried along.
    constexpr int ROUNDS = (MAX_ROWS_LIST + THREADS - 1) / THREADS;
    int c[ROUNDS];
#pragma unroll
    for (int k = 0; k < ROUNDS; ++k) {
        const int rr = k * THREADS + tid;
        c[k] = rr < rows ? attn_row_count(a, rr) : 0;
    }
    int carry = 0;
#pragma unroll
    for (int k = 0; k < ROUNDS; ++k) {
        if (k * THREADS >= rows) break;                  // (uniform)
        const int rr = k * THREADS + tid;
        const int cost = row_cost(c[k]);
        const int inc = wave_inclusive_sum(cost);
        if (rr < rows) cnt[rr] = c[k];
        if (lane == 63) wsum[wave] = inc;
        lds_barrier();
        int base = carry, all = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const int s = wsum[w];
            if (w < wave) base += s;
            all += s;
        }
        if (rr < rows) pre[rr] = base + inc - cost;
        carry += all;
        lds_barrier();                                   // the wave totals are rewritten by the next round
    }
    if (tid == 0) pre[rows] = carry;
    lds_barrier();
}

// The share [c0, c1) of the cost line a workgroup takes, and where a row's tiles fall inside it: tile k of
// row r sits at pre[r] + SEG_COST + k.
struct Share {
    int c0, c1;
    // local tile range of row r inside the share; empty when lt_begin >= lt_end
    __device__ __forceinline__ void seg_range(const int *pre, const int *cnt, int r, int &lt_begin, int &lt_end) const
    {
        const int tiles = (cnt[r] + TILE - 1) / TILE;
        const int lo = c0 - pre[r] - SEG_COST, hi = c1 - pre[r] - SEG_COST;
        lt_begin = lo < 0 ? 0 : (lo > tiles ? tiles : lo);
        lt_end = hi < 0 ? 0 : (hi > tiles ? tiles : hi);
    }
    // first row at or after r with work for this workgroup, or `rows`
    __device__ __forceinline__ int next_seg(const int *pre, const int *cnt, int rows, int r) const
    {
        for (; r < rows && pre[r] < c1; ++r) {
            int lb, le;
            seg_range(pre, cnt, r, lb, le);
            if (lb < le) return r;
        }
        return rows;
    }
    // first row with work for this workgroup, or `rows`
    __device__ __forceinline__ int first_seg(const int *pre, const int *cnt, int rows) const
    {
        int lo = 0, hi = rows;                      // row holding cost c0: pre[r] <= c0 < pre[r+1]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= c0) lo = mid; else hi = mid;
        }
        return next_seg(pre, cnt, rows, lo);
    }
};
// floor(a / b) for 0 <= a < 2^52, 0 < b < 2^31 in one fp64 division instead of the long 64-bit integer division
// sequence: both operands are exact in fp64, the correctly rounded quotient can only reach the next integer from
// below when a / b is within 2^-53 of it, and a true quotient that is no integer lies at least 1 / b below it.
__device__ __forceinline__ int floor_div(int64_t a, int b)
{
    return (int)floor((double)a / (double)b);
}

// The first min(n_wg, total) workgroups share the line: workgroup w takes [w * total / n, (w + 1) * total / n),
// so shares differ by at most one unit and none of them is empty (every workgroup between the first and the
// last of a row therefore holds tiles of that row, which the merge relies on).
__device__ __forceinline__ int share_start(int total, int n_wg, int w)
{
    const int n = n_wg < total ? n_wg : total;
    if (w >= n) return total;
    // (a power of two - the usual 256 workgroups - divides exactly in any arithmetic: a shift then gives the same
    // floor as the division below at a tenth of the instructions, on the way to a workgroup's first request)
    if ((n & (n - 1)) == 0) return (int)(((int64_t)w * total) >> (31 - __clz(n)));
    return floor_div((int64_t)w * total, n);
}
__device__ __forceinline__ Share make_share(int total, int n_wg, int w)
{
    Share s;
    s.c0 = share_start(total, n_wg, w);
    s.c1 = share_start(total, n_wg, w + 1);
    return s;
}
// the workgroup whose share holds cost position c (0 <= c < total)
__device__ __forceinline__ int share_of(int total, int n_wg, int c)
{
    const int n = n_wg < total ? n_wg : total;
    return floor_div(((int64_t)c + 1) * n - 1, total);
}

// Which share of the line a workgroup takes.  The hardware deals workgroup i to XCD i mod 8; the owners of
// four consecutive shares (the usual team of a row) are four workgroups on four different XCDs, and the sets
// {x, x+1, x+3, x+6} rotate from team to team, so that every XCD serves half of the teams and a difference in
// speed between XCDs is spread over all rows.  (A bijection of 0 .. n_wg - 1 when n_wg is a multiple of 32.)
__device__ __forceinline__ int share_index(int wg, int n_wg)
{
    if (n_wg & 31) return wg;
    const int x = wg & 7, c = wg >> 3, m = c & 3;
    const int off = m == 0 ? 0 : (m == 1 ? 1 : (m == 2 ? 3 : 6));
    const int team = ((c >> 2) << 3) | ((x - off) & 7);
    return (team << 2) | m;
}

// One step of merging partial (m, l, o) triples that share the log2-unit convention.
struct Merge {
    float m = -INFINITY, l = 0.0f, o = 0.0f;
    __device__ __forceinline__ void add(float mw, float lw, float ow)
    {
        const float mn = fmaxf(m, mw);
        const float fa = (m == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m - mn);
        const float fb = (mw == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw - mn);
        l = l * fa + lw * fb;
        o = o * fa + ow * fb;
        m = mn;
    }
};
template <int NQT, int LAYOUT, int SRC, bool F16>
__global__ __launch_bounds__(THREADS, WG_PER_CU) void attn_mfma_kernel(AttnLaunch a, Plan plan)
{
    typedef typename Half<F16>::x8 h16x8;
    typedef typename Half<F16>::x2 h16x2;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int QTP = NQT * 16;
    constexpr int QROUNDS = (NQT * 16 * 16 + THREADS - 1) / THREADS;    // 16-byte chunks of the Q tile per thread
    const int rows = a.B * a.H_kv;
    int *pre = reinterpret_cast<int *>(smem + OFF_TAB);
    int *cnt_lds = pre + ((a.B * a.H_kv <= FEW_ROWS ? FEW_ROWS : MAX_ROWS_LIST) + 1);
    int *wsum = reinterpret_cast<int *>(smem + OFF_WSUM);
    int *blk_pre = reinterpret_cast<int *>(smem + OFF_BLK);
    char *q_lds = smem + OFF_Q;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    char *wave_lds = smem + wave * WAVE_LDS;
    char *slot_lds = smem + OFF_SLOT + wave * 2 * SLOT_BYTES;
    float *mlw = reinterpret_cast<float *>(smem + OFF_SLOT);            // wave w's (m, l): [w * 128 + q * 2 * NQT + ...]
    const uint32_t ks_addr = (uint32_t)(uintptr_t)LDS_PTR(char, wave_lds);
    const uint32_t vs_addr = ks_addr + TILE_BYTES;
    const uint32_t slot_addr = (uint32_t)(uintptr_t)LDS_PTR(char, slot_lds);
    const uint32_t scat_addr = (uint32_t)(uintptr_t)LDS_PTR(char, smem + OFF_SCAT + wave * 256);
    const uint32_t blk_addr = (uint32_t)(uintptr_t)LDS_PTR(int, blk_pre);
    const uint32_t q_addr = (uint32_t)(uintptr_t)LDS_PTR(char, q_lds);
    // K fragment of k-step c: row l16 (+16 per position tile), 16-byte chunk 4c + g
    uint32_t k_off[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) k_off[c] = ks_addr + (uint32_t)(l16 * ROW_BYTES + (((4 * c + g) ^ swz(l16)) << 4));
    // Q fragment of k-step c: same pattern on the Q tile (row = query row l16, +16 for the second tile)
    uint32_t q_off[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) q_off[c] = q_addr + (k_off[c] - ks_addr);
    // V^T fragment of dv tile t: source lane points at row 4g + l16/4 (+16 per half), 4 values from
    // column 16t + 4*(l16%4)
    uint32_t v_off[8];
    {
        const int row = 4 * g + (l16 >> 2);
#pragma unroll
        for (int t = 0; t < 8; ++t)
            v_off[t] = vs_addr + (uint32_t)(row * ROW_BYTES + (((2 * t + ((l16 & 3) >> 1)) ^ swz(row)) << 4) + ((l16 & 1) << 3));
    }
    // gather instruction i moves rows 4i .. 4i+3; this lane fetches chunk l16 ^ swz(4i + g), which
    // depends on i only through i % 4
    int64_t lane_chunk[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) lane_chunk[j] = (int64_t)((l16 ^ swz(4 * j + g)) << 4);

    // Every kernel argument the main path uses is fetched here, in one batch: left to the compiler, the
    // argument loads are issued where each is first needed, and every such group is one more round trip to
    // memory on the way to the first gather.
#define SPECATTN_PRELOAD(x) asm volatile("" ::"s"(x))
    SPECATTN_PRELOAD(a.q); SPECATTN_PRELOAD(a.k); SPECATTN_PRELOAD(a.v);
    SPECATTN_PRELOAD(a.B); SPECATTN_PRELOAD(a.H_q); SPECATTN_PRELOAD(a.H_kv); SPECATTN_PRELOAD(a.T);
    SPECATTN_PRELOAD(a.sm_scale);
    SPECATTN_PRELOAD(a.q_stride_b); SPECATTN_PRELOAD(a.q_stride_h); SPECATTN_PRELOAD(a.q_stride_t);
    SPECATTN_PRELOAD(a.kv_stride_b); SPECATTN_PRELOAD(a.kv_stride_h); SPECATTN_PRELOAD(a.kv_stride_n);
    SPECATTN_PRELOAD(a.counts); SPECATTN_PRELOAD(a.idx_capacity); SPECATTN_PRELOAD(a.dense); SPECATTN_PRELOAD(a.chunk_shift);
    SPECATTN_PRELOAD(a.g_first); SPECATTN_PRELOAD(a.g_count); SPECATTN_PRELOAD(a.k_new);
    SPECATTN_PRELOAD(a.out); SPECATTN_PRELOAD(a.out_lowp); SPECATTN_PRELOAD(a.lse);
    SPECATTN_PRELOAD(plan.part_ml); SPECATTN_PRELOAD(plan.part_o); SPECATTN_PRELOAD(plan.cost_prefix);
    SPECATTN_PRELOAD(plan.n_wg);
    if (LAYOUT != CONTIGUOUS) { SPECATTN_PRELOAD(a.page_table); SPECATTN_PRELOAD(a.page_shift); SPECATTN_PRELOAD(a.max_pages); SPECATTN_PRELOAD(a.kv_stride_page); }
    if (SRC == LIST) { SPECATTN_PRELOAD(a.indices); SPECATTN_PRELOAD(a.idx_stride); }
    if (SRC == MASK) { SPECATTN_PRELOAD(a.kept_mask); SPECATTN_PRELOAD(a.block_counts); SPECATTN_PRELOAD(a.blocks_per_row); SPECATTN_PRELOAD(a.n_max); }
#undef SPECATTN_PRELOAD
    // Mask source, small calls: the per-block kept counts of all rows are requested together with the counts (the row
    // this workgroup starts in is not known yet), so that its first segment need not go to memory for them again.
    constexpr int BC_PT = BC_ALL / THREADS;
    int *bc_lds = reinterpret_cast<int *>(smem + OFF_BC);
    const bool bc_all = SRC == MASK && rows <= FEW_ROWS && rows * a.blocks_per_row <= BC_ALL;
    int bc_pf[BC_PT];
    if (bc_all) {
#pragma unroll
        for (int k = 0; k < BC_PT; ++k) {
            const int j = tid + k * THREADS;
            bc_pf[k] = a.block_counts[j < rows * a.blocks_per_row ? j : 0];
        }
    }
    cost_prefix(a, rows, pre, cnt_lds, wsum);
    if (blockIdx.x == 0)
        for (int rr = tid; rr <= rows; rr += THREADS) plan.cost_prefix[rr] = pre[rr];
    if (bc_all) {
#pragma unroll
        for (int k = 0; k < BC_PT; ++k) bc_lds[tid + k * THREADS] = bc_pf[k];   // (read behind the first segment's barrier)
    }
    const int G = attn_group_heads(a);
    const int QT = G * a.T;
    const float scale2 = a.sm_scale * 1.4426950408889634f;            // scores in log2 units

    // ---- per-segment inputs that are fetched ahead of time -------------------------------------------
    // The Q tile of a segment goes through LDS: thread t fetches 16-byte chunk t%16 of query rows t/16 (+16 ...)
    // ahead of time and stores it (swizzled like a K row) when the segment starts.
    u32x4 q_pf[QROUNDS];
    auto fetch_q = [&](int rr) {
        const int b = rr / a.H_kv, h = rr - b * a.H_kv;
#pragma unroll
        for (int k = 0; k < QROUNDS; ++k) {
            const int qi = (tid >> 4) + k * (THREADS / 16), ch = tid & 15;
            q_pf[k] = (u32x4){0u, 0u, 0u, 0u};
            if (qi < QT) {
                const int gh = qi / a.T, tt = qi - gh * a.T;
                const uint16_t *qp = static_cast<const uint16_t *>(a.q) + (int64_t)b * a.q_stride_b +
                                     (int64_t)attn_query_head(a, h, gh) * a.q_stride_h + (int64_t)tt * a.q_stride_t;
                q_pf[k] = *reinterpret_cast<const u32x4 *>(qp + ch * 8);
            }
        }
    };
    auto store_q = [&]() {
#pragma unroll
        for (int k = 0; k < QROUNDS; ++k) {
            const int qi = (tid >> 4) + k * (THREADS / 16), ch = tid & 15;
            if (qi < NQT * 16) *reinterpret_cast<u32x4 *>(q_lds + qi * ROW_BYTES + ((ch ^ swz(qi & 15)) << 4)) = q_pf[k];
        }
    };

    // This workgroup's share of the cost line, and the rows of which it holds tiles.  Up to 64 rows, lane i looks
    // at row i: one LDS round trip, the share, every row's local tile range at once and a ballot, instead of a
    // binary search and a row-by-row walk over the table, each step of which waits for an LDS read.
    const bool few_rows = rows <= FEW_ROWS;              // uniform
    int row_lo = 0, row_cnt = 0, row_hi = 0;
    if (few_rows) {
        row_lo = lane < rows ? pre[lane] : 0;
        row_hi = lane < rows ? pre[lane + 1] : 0;
        row_cnt = lane < rows ? cnt_lds[lane] : 0;
    }
    const int total = few_rows ? __builtin_amdgcn_readlane(row_hi, rows - 1) : pre[rows];
    const int my_share = share_index(blockIdx.x, plan.n_wg);
    const Share sh = make_share(total, plan.n_wg, my_share);
    const int c0 = sh.c0, c1 = sh.c1;
    if (c0 >= c1) return;                                // more workgroups than units of work
    int my_lb = 0, my_le = 0;                            // few rows: local tile range of row `lane`
    unsigned long long seg_mask = 0;                     // few rows: the rows with tiles in this share
    if (few_rows) {
        const int tiles = (row_cnt + TILE - 1) / TILE;
        const int lo = c0 - row_lo - SEG_COST, hi = c1 - row_lo - SEG_COST;
        my_lb = lo < 0 ? 0 : (lo > tiles ? tiles : lo);
        my_le = hi < 0 ? 0 : (hi > tiles ? tiles : hi);
        seg_mask = __ballot(lane < rows && my_lb < my_le);
    }
    auto seg_range = [&](int r, int &lt_begin, int &lt_end) {
        if (few_rows) {
            const int ru = __builtin_amdgcn_readfirstlane(r);
            lt_begin = __builtin_amdgcn_readlane(my_lb, ru);
            lt_end = __builtin_amdgcn_readlane(my_le, ru);
        } else {
            sh.seg_range(pre, cnt_lds, r, lt_begin, lt_end);
        }
    };
    // first row at or after r with work for this workgroup, or `rows`
    auto next_seg = [&](int r) {
        if (few_rows) {
            const unsigned long long m = r < 64 ? (seg_mask >> r) << r : 0ull;
            return m ? (int)__ffsll((long long)m) - 1 : rows;
        }
        return sh.next_seg(pre, cnt_lds, rows, r);
    };
    int r = few_rows ? next_seg(0) : sh.first_seg(pre, cnt_lds, rows);

    bool first_seg = true;
    if (r < rows) fetch_q(r);

    while (r < rows) {
        int lt_begin, lt_end;
        seg_range(r, lt_begin, lt_end);
        const int r_next = next_seg(r + 1);
        const int b = r / a.H_kv, h = r - b * a.H_kv;
        const int count = few_rows ? __builtin_amdgcn_readlane(row_cnt, __builtin_amdgcn_readfirstlane(r)) : cnt_lds[r];
        const int p_lo = few_rows ? __builtin_amdgcn_readlane(row_lo, __builtin_amdgcn_readfirstlane(r)) : pre[r];
        const int p_hi = few_rows ? __builtin_amdgcn_readlane(row_hi, __builtin_amdgcn_readfirstlane(r)) : pre[r + 1];
        const int tiles = (count + TILE - 1) / TILE;
        const int tile_end = lt_end;             // the tiles [lt_begin, lt_end) of the row are this workgroup's
        const KvMap map = make_map<LAYOUT>(a, b, h);
        const char *kbh = static_cast<const char *>(a.k) + map.base * 2;
        const char *vbh = static_cast<const char *>(a.v) + map.base * 2;
        const int32_t *idx_row = (SRC == LIST && !a.dense) ? a.indices + (int64_t)r * a.idx_stride : nullptr;
        const uint32_t *mask_row = SRC == MASK ? a.kept_mask + (int64_t)r * a.blocks_per_row * (SEL_BLOCK / 32) : nullptr;
        const int n_idx = (SRC == MASK || !a.dense) ? 1 : 0;            // LDS-DMA instructions per tile for list / mask words

        // ---- the wave's tiles --------------------------------------------------------------------------
        // tile k of the share goes to wave k mod NW
        int t_cur = lt_begin + wave, t_nxt = t_cur + NW, t_nn = t_nxt + NW;
        // Mask source: where a tile's 32 kept positions start.  Returns the block b that holds rank 32 t and
        // leaves in `skip` the kept positions of b that come before that rank.  (LDS reads by hand, see above.)
        auto mask_locate = [&](int t, int &skip) -> int {
            const int rank = t * TILE;
            const int nb = a.blocks_per_row;
            const int stride = (nb + 63) >> 6;                          // blocks per lane of the coarse step
            int lo = lane * stride < nb ? (int)lds_read_word(blk_addr + (uint32_t)(lane * stride) * 4) : 0x7fffffff;
            int cnum = __popcll(__ballot(lo <= rank));                  // blk_pre[0] = 0 <= rank: at least 1
            int bb = (cnum > 0 ? cnum - 1 : 0) * stride;
            if (stride > 1) {
                lo = (lane < stride && bb + lane < nb) ? (int)lds_read_word(blk_addr + (uint32_t)(bb + lane) * 4) : 0x7fffffff;
                cnum = __popcll(__ballot(lo <= rank));
                bb += cnum > 0 ? cnum - 1 : 0;
            }
            bb = __builtin_amdgcn_readfirstlane(bb);
            skip = rank - (int)__builtin_amdgcn_readfirstlane(lds_read_word(blk_addr + (uint32_t)bb * 4));
            return bb;
        };
        // Requests the words tile t needs into slot s (one LDS-DMA instruction): its 32 list words, or 64 words of
        // the kept mask from the block that holds its first rank.  Tiles past the end request the last tile's.
        int m_blk0 = 0, m_blk1 = 0, m_skip0 = 0, m_skip1 = 0;           // mask source: what slots 0 and 1 hold
        auto request = [&](int t, int s) {
            if (t >= tiles) t = tiles - 1;
            if (SRC == MASK) {
                int skip;
                const int bb = mask_locate(t, skip);
                if (s) { m_blk1 = bb; m_skip1 = skip; } else { m_blk0 = bb; m_skip0 = skip; }
                const int nw = a.blocks_per_row * (SEL_BLOCK / 32);
                int w = bb * (SEL_BLOCK / 32) + lane;
                w = w < nw ? w : nw - 1;
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(mask_row + w), LDS_PTR(void, slot_lds + s * SLOT_BYTES), 4, 0, 0);
            } else if (!a.dense) {
                int jj = t * TILE + (lane & 31);
                jj = jj < count ? jj : count - 1;
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(idx_row + (jj >> a.chunk_shift)),
                                                 LDS_PTR(void, slot_lds + s * SLOT_BYTES), 4, 0, 0);
            }
        };
        // Mask source: turns the 64 mask words in slot s into the 32 positions of tile t (table s of the wave).  The
        // words start at block m_blk; the tile's ranks start m_skip kept positions into them.  Lane w counts its
        // word's bits and a wave-wide prefix gives the rank of its first bit; every word that holds ranks of the
        // tile marks the first of them, a prefix maximum over the marks tells lane j (< 32) which word holds rank
        // j, and the lane picks its bit out of that word: no loop over bits.  Done one iteration before the
        // tile's gathers are issued.  (A row so sparse that 2048 positions hold fewer than 32 kept ones takes
        // further rounds over the next 64 words.)
        auto decode = [&](int t, int s) {
            if (t >= tiles) t = tiles - 1;
            const int need = (count - t * TILE) < TILE ? (count - t * TILE) : TILE;
            int have = 0;                                               // ranks of the tile found so far
            int word0 = (s ? m_blk1 : m_blk0) * (SEL_BLOCK / 32);
            int skip = s ? m_skip1 : m_skip0;
            const int nw = a.blocks_per_row * (SEL_BLOCK / 32);
            const uint32_t table = scat_addr + (uint32_t)s * 128;
            uint32_t bits = lds_read_word(slot_addr + (uint32_t)(s * SLOT_BYTES + lane * 4));
            for (;;) {
                if (word0 + lane >= nw) bits = 0u;
                const int pc = __popc(bits);
                const int inc = wave_inclusive_sum(pc);
                const int ex = inc - pc;
                const int got = __builtin_amdgcn_readlane(inc, 63) - skip;     // ranks of the tile among these words
                if (got > 0) {
                    const int lo = ex - skip + have, hi = lo + pc;      // table slots this word's bits would take
                    // every word that holds ranks of the tile pushes its number to the lane of its first such rank
                    // (the others push to lane 63, which stands for no rank)
                    const bool holds = pc > 0 && hi > have && lo < need;
                    const int mark = (int)lane_push(holds ? (uint32_t)lane + 1u : 0u, holds ? (lo > have ? lo : have) : 63);
                    const int owner = prefix_max32((lane >= have && lane < 32) ? mark : 0) - 1;   // the word that holds rank `lane`
                    const int src = owner >= 0 ? owner : 0;
                    uint32_t wbits, wex;
                    lane_read2(bits, (uint32_t)ex, src, wbits, wex);
                    const int top = (have + got) < need ? (have + got) : need;
                    if (lane >= have && lane < top && owner >= 0) {
                        const int k = lane - have + skip - (int)wex;    // which of the word's bits
                        lds_write_word(table + (uint32_t)lane * 4, (uint32_t)((word0 + src) * 32 + kth_set_bit(wbits, k)));
                    }
                }
                have += got > 0 ? got : 0;
                skip = got < 0 ? -got : 0;
                word0 += 64;
                if (have >= need || word0 >= nw) break;
                bits = global_read_word(mask_row + (word0 + lane < nw ? word0 + lane : nw - 1));   // sparse row: the tile reaches further
            }
            // (no wait: the table is read by this wave's own later LDS reads, which the LDS unit serves in order)
            if (need < TILE) {
                lds_wait();                                          // ranks past the end repeat the last kept position
                const uint32_t last_pos = lds_read_word(table + (uint32_t)((need > 0 ? need : 1) - 1) * 4);
                if (lane >= need && lane < TILE) lds_write_word(table + (uint32_t)lane * 4, last_pos);
                lds_wait();
            }
        };
        // Row offsets (16-byte units) of the 8 rows this lane helps to fetch for tile t, whose list words (or decoded
        // positions) are in slot / table s.
        auto entries = [&](int t, int s, uint32_t (&ent)[8]) {
            int pos[8], jj[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                jj[i] = t * TILE + 4 * i + g;
                jj[i] = jj[i] < count ? jj[i] : count - 1;              // ranks past the end repeat the last kept position
            }
            if (SRC == MASK) {
                uint32_t e[8];
                lds_read_entries(e, scat_addr + (uint32_t)(s * 128 + g * 4));
                // (a mask that does not hold `count` bits would leave table entries unwritten: stay inside the row)
#pragma unroll
                for (int i = 0; i < 8; ++i) pos[i] = e[i] < (uint32_t)a.n_max ? (int)e[i] : a.n_max - 1;
            } else if (a.dense) {
#pragma unroll
                for (int i = 0; i < 8; ++i) pos[i] = jj[i];
            } else {
                uint32_t e[8];
                lds_read_entries(e, slot_addr + (uint32_t)(s * SLOT_BYTES + g * 4));
                const int cs = a.chunk_shift, low = (1 << cs) - 1;
#pragma unroll
                for (int i = 0; i < 8; ++i) pos[i] = (int)(e[i] << cs) | (jj[i] & low);
            }
            map.rel_n<LAYOUT>(pos, ent);
        };
        // gather 32 rows of one tensor into this wave's buffer: 8 instructions of 4 rows x 256 B
        auto issue = [&](const char *base, char *buf, const uint32_t (&ent)[8]) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const char *src = base + ((int64_t)ent[i] << 4) + lane_chunk[i & 3];
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(void, buf + i * 1024), 16, 0, KV_AUX);
            }
        };

        // ---- start of the segment: the words of the wave's first two tiles are requested before anything else the
        //      segment needs, since the first gathers wait for them (counts -> list words -> K/V rows are three
        //      dependent trips to memory); then Q goes into LDS ---------------------------------------------------
        if (!first_seg) lds_barrier();           // the previous segment's readers of the wave buffers, slots and Q are done
        if (SRC == MASK) {
            // the row's block prefix first: a tile's mask words are found through it
            if (first_seg && bc_all) lds_barrier();                     // the block counts of all rows are in LDS
            {
                if (wave == 0) {                                        // (a scan per wave into a register was slower)
                    const int32_t *bc = a.block_counts + (int64_t)r * a.blocks_per_row;
                    int running = 0;
                    for (int base = 0; base < a.blocks_per_row; base += 64) {
                        const int c = (base + lane < a.blocks_per_row) ? (bc_all ? bc_lds[r * a.blocks_per_row + base + lane] : bc[base + lane]) : 0;
                        const int inc = wave_inclusive_sum(c);
                        if (base + lane < a.blocks_per_row) blk_pre[base + lane + 1] = running + inc;
                        running += __builtin_amdgcn_readlane(inc, 63);
                    }
                    if (lane == 0) blk_pre[0] = 0;
                }
                lds_barrier();
            }
        }
        if (t_cur < tile_end) { request(t_cur, 0); request(t_nxt, 1); }
        store_q();
        lds_barrier();

        f32x4 o[NQT][8];                     // O^T[dv = 16t + 4g + i][q = l16]
        float m_ref[NQT], l_sum[NQT];        // reference max (log2 units) and sum of weights
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            m_ref[qt] = -INFINITY;
            l_sum[qt] = 0.0f;
#pragma unroll
            for (int t = 0; t < 8; ++t) o[qt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }

        if (t_cur < tile_end) {
            // The gathers and word requests are not tracked by the compiler's wait insertion; every wait on them is
            // written out.  Order of issue per wave and iteration: K(next) ... V(next) words(third).
            uint32_t ent[8];
            vm_wait(0);                                                 // the words of the first two tiles are there
            if (SRC == MASK) decode(t_cur, 0);
            entries(t_cur, 0, ent);
            issue(kbh, wave_lds, ent);
            issue(vbh, wave_lds + TILE_BYTES, ent);
            if (SRC == MASK) decode(t_nxt, 1);                          // (behind the first gathers, not ahead of them)
            request(t_nn, 0);
            int s_nxt = 1;                                              // slot with the words of t_nxt; t_nn's is the other
            while (t_cur < tile_end) {
                const bool has_next = t_nxt < tile_end;
                vm_wait(8 + n_idx);                                     // K(cur) landed; V(cur) and the last request may be in flight

                // ---- S^T[pos][q] = K Q^T -----------------------------------------------------------
                f32x4 s[NQT][2];
                {
                    KFrags kf;
                    lds_read_k(kf, k_off);
                    if (has_next) {                                    // the K buffer is free again
                        entries(t_nxt, s_nxt, ent);
                        issue(kbh, wave_lds, ent);
                    }
#pragma unroll
                    for (int qt = 0; qt < NQT; ++qt) {
                        QFrags qf;
                        lds_read_q(qf, q_off, qt == 1);
#pragma unroll
                        for (int pt = 0; pt < 2; ++pt) {
                            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                acc = Half<F16>::mfma(__builtin_bit_cast(h16x8, kf.f[pt][c]),
                                                      __builtin_bit_cast(h16x8, qf.f[c]), acc);
                            s[qt][pt] = acc;
                        }
                    }
                }

                // ---- softmax weights; lane (q = l16, g) holds positions 16pt + 4g + i ---------------
                const int remaining = count - t_cur * TILE;            // > 0; < TILE only on a row's last tile
                h16x8 p_hi[NQT], p_lo[NQT];
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt) {
                    float x[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[e] = s[qt][e >> 2][e & 3];
                    if (remaining < TILE) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (16 * (e >> 2) + 4 * g + (e & 3) >= remaining) x[e] = -INFINITY;
                    }
                    const float mloc = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                                             fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7]))) * scale2;
                    if (__any(mloc > m_ref[qt] + RESCALE_SLACK)) {     // first tile, then rare
                        float mx = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
                        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                        const float mnew = fmaxf(m_ref[qt], mx);
                        const float alpha = (m_ref[qt] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(m_ref[qt] - mnew);
                        l_sum[qt] *= alpha;
#pragma unroll
                        for (int t = 0; t < 8; ++t) o[qt][t] *= alpha;
                        m_ref[qt] = mnew;
                    }
                    const float mr = (m_ref[qt] == -INFINITY) ? 0.0f : m_ref[qt];
                    float psum = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(x[e], scale2, -mr));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(x[e + 1], scale2, -mr));
                        psum += p0 + p1;
                        const h16x2 hi = __builtin_convertvector((f32x2){p0, p1}, h16x2);
                        const f32x2 back = __builtin_convertvector(hi, f32x2);
                        const h16x2 lo = __builtin_convertvector((f32x2){p0 - back[0], p1 - back[1]}, h16x2);
                        p_hi[qt][e] = hi[0]; p_hi[qt][e + 1] = hi[1];
                        p_lo[qt][e] = lo[0]; p_lo[qt][e + 1] = lo[1];
                    }
                    l_sum[qt] += psum;
                }

                // ---- O^T += V^T P^T -----------------------------------------------------------------
                if (has_next) vm_wait(8 + n_idx);                      // V(cur) landed; the last request and K(next) in flight
                else vm_wait(0);
#pragma unroll
                for (int tb = 0; tb < 8; tb += 4) {                    // four 16-wide dv tiles per batch
                    VFrags vh;
                    lds_read_v(vh, v_off[tb], v_off[tb + 1], v_off[tb + 2], v_off[tb + 3]);
                    if (tb == 4 && has_next) issue(vbh, wave_lds + TILE_BYTES, ent);   // the V buffer is free again
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const u32x4 both = (u32x4){vh.f[t][0][0], vh.f[t][0][1], vh.f[t][1][0], vh.f[t][1][1]};
                        const h16x8 vf = __builtin_bit_cast(h16x8, both);
#pragma unroll
                        for (int qt = 0; qt < NQT; ++qt) {
                            o[qt][tb + t] = Half<F16>::mfma(vf, p_hi[qt], o[qt][tb + t]);
                            o[qt][tb + t] = Half<F16>::mfma(vf, p_lo[qt], o[qt][tb + t]);
                        }
                    }
                }
                // ---- the tile after the next two: request its words -------------------------------------------
                const int t_new = t_nn + NW;
                if (has_next) {
                    request(t_new, s_nxt);                             // the slot t_nxt's words were read from
                    if (SRC == MASK && t_nn < tile_end) {              // the positions of the tile that is next but one
                        vm_wait(17);                                   // its words (requested an iteration ago) are there
                        decode(t_nn, s_nxt ^ 1);
                    }
                }
                t_cur = t_nxt; t_nxt = t_nn; t_nn = t_new;
                s_nxt ^= 1;
            }
        }
        vm_wait(0);                              // nothing of this wave's is in flight any more (the slots are reused below)

        // ---- request what the next segment needs, to arrive while this one is wrapped up --------------
        if (r_next < rows) fetch_q(r_next);

        // ---- combine the waves of this workgroup: every wave hands its state over lane by lane through its
        //      own tile buffers, which are idle as soon as the wave itself has no tile left - before the barrier,
        //      so that only the last wave's hand-over is waited for; wave w then reduces and writes the
        //      (query tile, dv tile) blocks k = w * KPW .. of all states.  (m, l) per query row go into the
        //      wave's first word slot. ----------------------------------------------------------------------
        {
            float *dmp = reinterpret_cast<float *>(wave_lds);                  // [NQT * 8][64 lanes] float4
#pragma unroll
            for (int qt = 0; qt < NQT; ++qt) {
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    *reinterpret_cast<f32x4 *>(dmp + ((qt * 8 + t) * 64 + lane) * 4) = o[qt][t];
                float l = l_sum[qt];
                l += __shfl_xor(l, 16, 64);
                l += __shfl_xor(l, 32, 64);
                if (g == 0) {
                    mlw[wave * 128 + l16 * 2 * NQT + 2 * qt] = m_ref[qt];
                    mlw[wave * 128 + l16 * 2 * NQT + 2 * qt + 1] = l;
                }
            }
        }
        lds_barrier();                         // every wave has handed over, and is done with Q
        // Workgroups w_first..w_last share row r: a row owned by one workgroup is finished here; otherwise the
        // partial goes to slot (share + r) for the merge kernel.
        const int w_first = share_of(total, plan.n_wg, p_lo + SEG_COST), w_last = share_of(total, plan.n_wg, p_hi - 1);
        const bool final_here = w_first == w_last && !a.k_new;
        {
            constexpr int KPW = NQT * 8 / NW;    // blocks per wave
            static_assert(KPW >= 1, "more waves than blocks to reduce");
            const int slot = my_share + r;
            float *po = plan.part_o + (int64_t)slot * QTP * D;
            float *pml = plan.part_ml + (int64_t)slot * QTP * 2;
#pragma unroll
            for (int kk = 0; kk < KPW; ++kk) {
                const int k = wave * KPW + kk;   // uniform
                const int qt = k >> 3, t = k & 7;
                float m = -INFINITY;
#pragma unroll
                for (int w = 0; w < NW; ++w) m = fmaxf(m, mlw[w * 128 + l16 * 2 * NQT + 2 * qt]);
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                float l = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float mw = mlw[w * 128 + l16 * 2 * NQT + 2 * qt];
                    const float f = (mw == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw - m);
                    l += f * mlw[w * 128 + l16 * 2 * NQT + 2 * qt + 1];
                    acc += f * *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(smem + w * WAVE_LDS) +
                                                                (k * 64 + lane) * 4);
                }
                const int q = qt * 16 + l16;
                if (q < QT) {
                    if (final_here) {
                        const int gh = q / a.T, tt = q - gh * a.T;
                        const int64_t orow = ((int64_t)b * a.H_q + attn_query_head(a, h, gh)) * a.T + tt;
                        const f32x4 res = l > 0.0f ? acc / l : (f32x4){0.f, 0.f, 0.f, 0.f};
                        *reinterpret_cast<f32x4 *>(a.out + orow * D + 16 * t + 4 * g) = res;
                        if (a.out_lowp) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) st_lowp(a.out_lowp, orow * D + 16 * t + 4 * g + i, res[i], a.dtype);
                        }
                        if (a.lse && g == 0 && t == 0)
                            a.lse[orow] = l > 0.0f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
                    } else {
                        *reinterpret_cast<f32x4 *>(po + q * D + 16 * t + 4 * g) = acc;
                        if (g == 0 && t == 0) { pml[2 * q] = m; pml[2 * q + 1] = l; }
                    }
                }
            }
        }
        first_seg = false;
        r = r_next;                              // the next segment starts with a barrier of its own
    }

}

// After the main kernel, one workgroup per (row, query row): rows shared by several workgroups get
// their partials (r, w) combined; rows without any kept position get out = 0, lse = -inf.  When the
// caller gave the new tokens behind the cache, every row goes through here (the main kernel then
// leaves partials only) and query t also attends to new tokens 0..t.
__global__ void merge_partials_kernel(AttnLaunch a, Plan plan, int qtp)
{
    __shared__ float red[2 * SPECATTN_MAX_T];
    const int G = attn_group_heads(a);
    const int QT = G * a.T;
    const int rows = a.B * a.H_kv;
    const int r = blockIdx.x / QT, q = blockIdx.x - r * QT;
    const int b = r / a.H_kv, h = r - b * a.H_kv;
    const int gh = q / a.T, t = q - gh * a.T;
    const int64_t orow = ((int64_t)b * a.H_q + attn_query_head(a, h, gh)) * a.T + t;
    const int dv = threadIdx.x;
    const bool tail = a.k_new != nullptr;
    const int total = plan.cost_prefix[rows];
    const int p0 = plan.cost_prefix[r], p1 = plan.cost_prefix[r + 1];
    if (p0 == p1 && !tail) {
        a.out[orow * D + dv] = 0.0f;
        if (a.out_lowp) st_lowp(a.out_lowp, orow * D + dv, 0.0f, a.dtype);
        if (a.lse && dv == 0) a.lse[orow] = -INFINITY;
        return;
    }
    Merge acc;
    if (p0 != p1) {
        const int w0 = share_of(total, plan.n_wg, p0 + SEG_COST), w1 = share_of(total, plan.n_wg, p1 - 1);
        if (w0 == w1 && !tail) return;              // finished by its only workgroup
        for (int wb = w0; wb <= w1; wb += 8) {      // eight partials per round trip
            float mw[8], lw[8], ow[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int64_t s = (int64_t)(wb + k + r) * qtp + q;
                const bool ok = wb + k <= w1;
                mw[k] = ok ? plan.part_ml[s * 2] : -INFINITY;
                lw[k] = ok ? plan.part_ml[s * 2 + 1] : 0.0f;
                ow[k] = ok ? plan.part_o[s * D + dv] : 0.0f;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) acc.add(mw[k], lw[k], ow[k]);
        }
    }
    if (tail) {
        float dots[SPECATTN_MAX_T];
        tail_dots(a, b, attn_query_head(a, h, gh), t, red, dots);
        const float scale2 = a.sm_scale * 1.4426950408889634f;       // m is in log2 units
        const int64_t noff = ((int64_t)b * a.H_kv + h) * a.T * D;
#pragma unroll
        for (int p = 0; p < SPECATTN_MAX_T; ++p)
            if (p <= t) acc.add(dots[p] * scale2, 1.0f, ld_elem(a.v_new, noff + (int64_t)p * D + dv, a.dtype));
    }
    const float res = acc.l > 0.0f ? acc.o / acc.l : 0.0f;
    a.out[orow * D + dv] = res;
    if (a.out_lowp) st_lowp(a.out_lowp, orow * D + dv, res, a.dtype);
    // m is in log2 units of the scaled scores
    if (a.lse && dv == 0) a.lse[orow] = acc.l > 0.0f ? (acc.m + log2f(acc.l)) * 0.6931471805599453f : -INFINITY;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// every kernel variant, for the one-time LDS-size attribute
struct Variant { int nqt, layout, src; bool f16; const void *fn; };
#define V4(NQT, LAY, SRC) \
    {NQT, LAY, SRC, false, reinterpret_cast<const void *>(&attn_mfma_kernel<NQT, LAY, SRC, false>)}, \
    {NQT, LAY, SRC, true, reinterpret_cast<const void *>(&attn_mfma_kernel<NQT, LAY, SRC, true>)}
const Variant g_variants[] = {
    V4(1, CONTIGUOUS, LIST), V4(1, PAGE_TABLE, LIST), V4(1, PHYSICAL, LIST),
    V4(2, CONTIGUOUS, LIST), V4(2, PAGE_TABLE, LIST), V4(2, PHYSICAL, LIST),
    V4(1, CONTIGUOUS, MASK), V4(1, PAGE_TABLE, MASK), V4(2, CONTIGUOUS, MASK), V4(2, PAGE_TABLE, MASK),
};
#undef V4

}  // namespace

bool attn_mfma_supported(const AttnLaunch &a)
{
    // any number of query heads per kv head: groups of more than 32 query rows run as several launches
    return (a.dtype == SPECATTN_BF16 || a.dtype == SPECATTN_F16) && a.d == 128 && a.T <= 32 && a.H_kv <= MAX_ROWS;
}

int attn_mfma_workgroups() { return cu_count() * WG_PER_CU; }

// The kernels use more LDS than the default limit: raise it for every variant, once per device.
specattn_status attn_mfma_configure()
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
    for (const Variant &v : g_variants) {
        if (hipFuncSetAttribute(v.fn, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess) {
            (void)hipGetLastError();
            set_error("cannot reserve %d bytes of LDS", LDS_BYTES);
            return SPECATTN_EHIP;
        }
    }
    done[dev] = true;
    return SPECATTN_OK;
}

static size_t workspace_for(int rows, int G, int T)
{
    const size_t qtp = (G * T <= 16) ? 16 : 32;
    const size_t slots = (size_t)attn_mfma_workgroups() + rows;
    size_t bytes = align256(((size_t)rows + 1) * sizeof(int32_t));                        // cost prefix
    bytes += slots * qtp * (D + 2) * sizeof(float);
    return align256(bytes);
}
// larger batches run as several launches over the same workspace
size_t attn_mfma_workspace_bytes(int rows, int G, int T) { return workspace_for(rows < MAX_ROWS_LIST ? rows : MAX_ROWS_LIST, G, T); }
size_t attn_mfma_workspace_min_bytes(int rows, int G, int T) { return workspace_for(rows < MAX_ROWS ? rows : MAX_ROWS, G, T); }

static specattn_status launch_chunk(const AttnLaunch &a, hipStream_t stream)
{
    const int rows = a.B * a.H_kv;
    const int G = a.g_count ? a.g_count : a.H_q / a.H_kv;
    const int QT = G * a.T;
    const int qtp = QT <= 16 ? 16 : 32;
    Plan plan;
    plan.n_wg = attn_mfma_workgroups();
    const size_t slots = (size_t)plan.n_wg + rows;
    // every workgroup may leave a partial in slot (workgroup + row): never launch over a workspace that cannot hold them
    if (!a.workspace || a.workspace_bytes < workspace_for(rows, G, a.T)) {
        set_error("attention workspace has %zu bytes, %zu needed", a.workspace_bytes, workspace_for(rows, G, a.T));
        return SPECATTN_EWORKSPACE;
    }
    char *ws = static_cast<char *>(a.workspace);
    plan.cost_prefix = reinterpret_cast<int32_t *>(ws);
    ws += align256(((size_t)rows + 1) * sizeof(int32_t));
    plan.part_ml = reinterpret_cast<float *>(ws);
    plan.part_o = plan.part_ml + slots * qtp * 2;
    const int layout = a.indices_are_physical ? PHYSICAL : (a.page_table ? PAGE_TABLE : CONTIGUOUS);
    const int src = a.kept_mask ? MASK : LIST;
    const bool f16 = a.dtype == SPECATTN_F16;
    const void *fn = nullptr;
    for (const Variant &v : g_variants)
        if (v.nqt * 16 == qtp && v.layout == layout && v.src == src && v.f16 == f16) fn = v.fn;
    if (!fn) { set_error("the fused path takes logical positions, not pool slots"); return SPECATTN_EUNSUPPORTED; }
    specattn_status st = attn_mfma_configure();
    if (st != SPECATTN_OK) return st;
    void *kargs[] = {const_cast<AttnLaunch *>(&a), &plan};
    if (hipLaunchKernel(fn, dim3(plan.n_wg), dim3(THREADS), kargs, LDS_BYTES, stream) != hipSuccess) {
        set_error("attn_mfma_kernel: launch failed");
        (void)hipGetLastError();
        return SPECATTN_EHIP;
    }
    st = check_launch("attn_mfma_kernel");
    if (st != SPECATTN_OK) return st;
    hipLaunchKernelGGL(merge_partials_kernel, dim3(rows * QT), dim3(D), 0, stream, a, plan, qtp);
    return check_launch("merge_partials_kernel");
}

// Batches with more rows than the kernel's LDS tables hold go out as several launches over
// consecutive sequences (rows are independent; the workspace is reused, the stream orders them).
// Likewise the query heads of a kv head: at most 32 query rows (heads x T) fit one launch, larger groups
// are cut into equal shares of heads, each streaming the kept K/V again.
static specattn_status launch_batch(const AttnLaunch &a, hipStream_t stream);

specattn_status launch_attn_mfma(const AttnLaunch &a, hipStream_t stream)
{
    const int G = a.H_q / a.H_kv;
    if (G * a.T <= 32) return launch_batch(a, stream);
    const int per_launch = 32 / a.T;
    const int shares = (G + per_launch - 1) / per_launch;
    const int heads = (G + shares - 1) / shares;
    for (int g0 = 0; g0 < G; g0 += heads) {
        AttnLaunch c = a;
        c.g_first = g0;
        c.g_count = (G - g0) < heads ? (G - g0) : heads;
        const specattn_status st = launch_batch(c, stream);
        if (st != SPECATTN_OK) return st;
    }
    return SPECATTN_OK;
}

static specattn_status launch_batch(const AttnLaunch &a, hipStream_t stream)
{
    // rows per launch: what the kernel's tables hold for this source, or - when the workspace was sized for
    // less (the built-in scratch buffer) - what every source can count on
    const int G = a.g_count ? a.g_count : a.H_q / a.H_kv;
    int cap = MAX_ROWS_LIST;
    if (a.B * a.H_kv > MAX_ROWS && a.workspace_bytes < workspace_for(a.B * a.H_kv < cap ? a.B * a.H_kv : cap, G, a.T)) cap = MAX_ROWS;
    const int b_max = cap / a.H_kv;
    if (a.B <= b_max) return launch_chunk(a, stream);
    const int es = 2;                                       // bf16 or fp16
    for (int b0 = 0; b0 < a.B; b0 += b_max) {
        AttnLaunch c = a;
        c.B = (a.B - b0) < b_max ? (a.B - b0) : b_max;
        const int64_t r0 = (int64_t)b0 * a.H_kv;
        c.q = static_cast<const char *>(a.q) + (int64_t)b0 * a.q_stride_b * es;
        const bool paged = a.page_table != nullptr || a.indices_are_physical;
        if (!paged) {
            c.k = static_cast<const char *>(a.k) + (int64_t)b0 * a.kv_stride_b * es;
            c.v = static_cast<const char *>(a.v) + (int64_t)b0 * a.kv_stride_b * es;
        }
        if (a.page_table) c.page_table = a.page_table + (int64_t)b0 * a.max_pages;
        if (a.indices) c.indices = a.indices + r0 * a.idx_stride;
        if (a.counts) c.counts = a.counts + r0;
        c.out = a.out + (int64_t)b0 * a.H_q * a.T * a.d;
        if (a.out_lowp) c.out_lowp = static_cast<char *>(a.out_lowp) + (int64_t)b0 * a.H_q * a.T * a.d * es;
        if (a.lse) c.lse = a.lse + (int64_t)b0 * a.H_q * a.T;
        if (a.seq_lens) c.seq_lens = a.seq_lens + b0;
        if (a.k_new) {
            c.k_new = static_cast<const char *>(a.k_new) + r0 * a.T * a.d * es;
            c.v_new = static_cast<const char *>(a.v_new) + r0 * a.T * a.d * es;
        }
        if (a.kept_mask) {
            c.kept_mask = a.kept_mask + r0 * a.blocks_per_row * (SEL_BLOCK / 32);
            c.block_counts = a.block_counts + r0 * a.blocks_per_row;
        }
        const specattn_status st = launch_chunk(c, stream);
        if (st != SPECATTN_OK) return st;
    }
    return SPECATTN_OK;
}

}  // namespace specattn

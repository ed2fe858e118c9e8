// Sparse decode attention over a selected index list (Section 3.1.2, Eq. 2-3; Section 3.5),
// bf16 or fp16, d = 128, up to 32 query rows per kv head and launch: the gfx950 matrix-core variant.
//
// Work split ("stream-K" over kept positions): the kept positions of all rows, in 32-position
// tiles, form one sequence; workgroup w takes an equal contiguous share of it, so the split is
// balanced by the *kept* count whatever the per-row counts are.  A share that crosses row
// boundaries yields one partial (m, l, o) per (row, workgroup); partial (r, w) lives in slot w + r.
// merge_partials_kernel combines a row's partials.
//
// Data path per wave and tile: the 32 gathered K rows and the 32 V rows (256 B each) go from HBM
// straight into LDS (global_load_lds: 16 lanes fetch one full row, four rows per instruction,
// XOR-swizzled chunk order).  Each wave owns one K buffer and one V buffer; the next tile's K is
// requested as soon as this tile's K fragments are in registers, the next V as soon as this tile's
// V has been consumed, so 8-16 KiB per wave (64-128 KiB per CU) are always in flight.
//   S^T = K Q^T    : mfma 16x16x32 bf16, A = K fragment (ds_read_b128), B = Q fragment (registers)
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

constexpr int NW = 8;                 // waves per workgroup
constexpr int THREADS = NW * 64;
constexpr int TILE = 32;              // positions per tile
constexpr int D = 128;
constexpr int ROW_BYTES = D * 2;      // one K or V row
constexpr int TILE_BYTES = TILE * ROW_BYTES;          // 8 KiB per tensor
constexpr int WAVE_LDS = 2 * TILE_BYTES;              // K buffer, V buffer
constexpr int MAX_ROWS = 1536;        // rows whose cost prefix fits the LDS table
constexpr int CHUNK_TILES = 64;       // tiles whose row offsets are staged in LDS at a time
constexpr int MAX_BLOCKS = SPECATTN_MAX_N / SEL_BLOCK;   // selection blocks per row, at most
// dynamic LDS: wave buffers, cost prefix, counts, wave sums, tile counter, list entries, block prefix,
// scan scratch, and the Q tile (two 16-row tiles at most) at the end
constexpr int LDS_MAIN = NW * WAVE_LDS +
                         (2 * MAX_ROWS + 1 + NW + 1 + CHUNK_TILES * TILE + MAX_BLOCKS + 1 + 2 * (NW + 1)) * 4 + 48 +
                         2 * 16 * ROW_BYTES;
#ifdef SPECATTN_TIMING
constexpr int LDS_BYTES = LDS_MAIN + 256;             // development builds: room for the wall-clock stamps
#else
constexpr int LDS_BYTES = LDS_MAIN;
#endif
// the waves' (m, l) of two query tiles fit the block-prefix array and the scratch behind it
static_assert(NW * 16 * 2 * 2 <= MAX_BLOCKS + 1 + 2 * (NW + 1), "no room for the wave merge's (m, l) table");
#ifndef SPECATTN_KV_AUX
#define SPECATTN_KV_AUX 2
#endif
constexpr int KV_AUX = SPECATTN_KV_AUX;   // cache policy bits of the K/V gathers
#ifndef SPECATTN_SEG_COST
#define SPECATTN_SEG_COST 12
#endif
constexpr int SEG_COST = SPECATTN_SEG_COST;          // cost of starting a row segment, in tiles
constexpr float RESCALE_SLACK = 8.0f; // log2 units the running max may exceed the reference by

// 16-byte chunk c of row `row` is stored in slot c ^ swz(row): makes both the K fragment reads
// (16 rows x one chunk) and the V transpose reads (8 rows x 32 B) spread over all banks.
__device__ __forceinline__ int swz(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }

// Where the gathered rows live.  A list entry is a logical position (contiguous layout) or a pool
// slot page * page_size + offset (paged layouts; logical positions are mapped through the page
// table once, when the chunk's list is staged).
enum Layout { CONTIGUOUS = 0, PAGE_TABLE = 1, PHYSICAL = 2 };

struct KvMap {
    int64_t base, stride_n, stride_page;
    const int32_t *ptab;
    int page_shift;
    // element offset of the row, relative to `base`
    template <int LAYOUT> __device__ __forceinline__ int64_t rel(int idx) const
    {
        if (LAYOUT == CONTIGUOUS) return (int64_t)idx * stride_n;
        const int mask = (1 << page_shift) - 1;
        const int page = LAYOUT == PAGE_TABLE ? ptab[idx >> page_shift] : (idx >> page_shift);
        return (int64_t)page * stride_page + (int64_t)(idx & mask) * stride_n;
    }
    // the same for N positions, with the page-table loads (if any) in flight together
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
// Row offsets of the 8 rows a lane helps to fetch: entries addr, addr + 16 B, ...
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
// Wave-wide fetch-and-add on an LDS counter: lane 0 adds 1, the others add 0, so lane 0 reads the
// value before the wave's own increment; that value is returned to the whole wave.
__device__ __forceinline__ int lds_claim(uint32_t addr, int lane)
{
    uint32_t v;
    const uint32_t inc = lane == 0 ? 1u : 0u;
    asm volatile("ds_add_rtn_u32 %0, %1, %2\n s_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(addr), "v"(inc) : "memory");
    return (int)__builtin_amdgcn_readfirstlane(v);
}

// Workgroup barrier for data handed over through LDS only: waits for this wave's LDS operations, not for its
// outstanding global loads (a plain __syncthreads() also waits for every gather and prefetch still in flight).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n s_barrier" ::: "memory"); }

struct Plan {
    float *part_ml;           // [slots][QTP][2]
    float *part_o;            // [slots][QTP][D]
    int32_t *cost_prefix;     // [rows + 1] in the workspace (written by workgroup 0, read by the merge)
    int n_wg;
#ifdef SPECATTN_TIMING
    long long *timing;        // [n_wg][8] wall-clock stamps (development builds only)
#endif
};

#ifdef SPECATTN_TIMING
// Development builds: thread 0 keeps wall-clock stamps in LDS (a store to memory here would make the compiler
// place waits on outstanding loads around it, and so change what is measured) and writes them out when it ends.
#define STAMP_PUT(k) do { const long long t_ = wall_clock64(); asm volatile("ds_write_b64 %0, %1 offset:%2\n s_waitcnt lgkmcnt(0)" ::"v"(stamp_addr), "v"(t_), "n"(8 * (k)) : "memory"); } while (0)
#define STAMP(k) do { if (threadIdx.x == 0) STAMP_PUT(k); } while (0)
#define STAMP_ONCE(k) do { if (threadIdx.x == 0 && !(stamped & (1u << (k)))) { stamped |= 1u << (k); STAMP_PUT(k); } } while (0)
#define STAMP_DUMP() do { if (threadIdx.x == 0) for (int k_ = 0; k_ < 16; ++k_) plan.timing[blockIdx.x * 16 + k_] = ((long long)stamp_lds[2 * k_ + 1] << 32) | (unsigned)stamp_lds[2 * k_]; } while (0)
#else
#define STAMP_ONCE(k) do { } while (0)
#define STAMP(k) do { } while (0)
#define STAMP_DUMP() do { } while (0)
#endif

// Cost of a row on the line the workgroups share out: its tiles, plus SEG_COST for picking the row up
// (fresh Q, pipeline refill, partial write) so that workgroups crossing a row boundary get fewer tiles.
__device__ __forceinline__ int row_cost(int count) { return count > 0 ? (count + TILE - 1) / TILE + SEG_COST : 0; }

// Exclusive prefix of the row costs into pre[0..rows], every workgroup for itself.
__device__ __forceinline__ void cost_prefix(const AttnLaunch &a, int rows, int *pre, int *cnt, int *wsum)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (rows <= 64) {
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
    const int per = (rows + THREADS - 1) / THREADS;
    const int r0 = tid * per;
    int local = 0;
    for (int k = 0; k < per; ++k) {
        const int r = r0 + k;
        if (r < rows) {
            const int c = attn_row_count(a, r);
            cnt[r] = c;
            local += row_cost(c);
        }
    }
    const int inc = wave_inclusive_sum(local);
    if (lane == 63) wsum[wave] = inc;
    lds_barrier();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    int run = base + inc - local;
    for (int k = 0; k < per; ++k) {
        const int r = r0 + k;
        if (r < rows) {
            pre[r] = run;
            run += row_cost(cnt[r]);
        }
    }
    if (tid == THREADS - 1) pre[rows] = base + inc;
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
__device__ __forceinline__ Share make_share(int total, int n_wg, int w)
{
    const int n = n_wg < total ? n_wg : total;
    Share s;
    s.c0 = w < n ? floor_div((int64_t)w * total, n) : total;
    s.c1 = w < n ? floor_div((int64_t)(w + 1) * total, n) : total;
    return s;
}
// the workgroup whose share holds cost position c (0 <= c < total)
__device__ __forceinline__ int share_of(int total, int n_wg, int c)
{
    const int n = n_wg < total ? n_wg : total;
    return floor_div(((int64_t)c + 1) * n - 1, total);
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

template <int NQT, int LAYOUT, bool FUSED, bool F16>
__global__ __launch_bounds__(THREADS) void attn_mfma_kernel(AttnLaunch a, Plan plan)
{
    typedef typename Half<F16>::x8 h16x8;
    typedef typename Half<F16>::x2 h16x2;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    constexpr int QTP = NQT * 16;
    constexpr int EPT = CHUNK_TILES * TILE / THREADS;                   // list entries staged per thread
    const int rows = a.B * a.H_kv;
    int *pre = reinterpret_cast<int *>(smem + NW * WAVE_LDS);          // [MAX_ROWS + 1] cost prefix
    int *cnt_lds = pre + MAX_ROWS + 1;                                  // [MAX_ROWS] kept counts, clamped
    int *wsum = cnt_lds + MAX_ROWS;                                     // [NW]
    int *tile_ctr = wsum + NW;                                          // tiles of the current chunk claimed so far
    uint32_t *ent_lds = reinterpret_cast<uint32_t *>(tile_ctr + 1);       // [CHUNK_TILES * TILE] row offsets / 16 B
    int *blk_pre = reinterpret_cast<int *>(ent_lds + CHUNK_TILES * TILE);   // fused: [MAX_BLOCKS + 1] kept before block
    float *ml_lds = reinterpret_cast<float *>(blk_pre);                 // wave merge: [NW][16 query rows][2 * NQT], same space
    char *q_lds = smem + LDS_MAIN - NQT * 16 * ROW_BYTES;              // Q tile [NQT*16][256 B], chunks swizzled like K
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    char *wave_lds = smem + wave * WAVE_LDS;
    const uint32_t ks_addr = (uint32_t)(uintptr_t)LDS_PTR(char, wave_lds);
    const uint32_t vs_addr = ks_addr + TILE_BYTES;
    const uint32_t ent_addr = (uint32_t)(uintptr_t)LDS_PTR(uint32_t, ent_lds);
    const uint32_t ctr_addr = (uint32_t)(uintptr_t)LDS_PTR(int, tile_ctr);
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

#ifdef SPECATTN_TIMING
    unsigned stamped = 0;
    int *stamp_lds = reinterpret_cast<int *>(smem + LDS_MAIN);
    const uint32_t stamp_addr = (uint32_t)(uintptr_t)LDS_PTR(int, stamp_lds);
    if (tid == 0) for (int k = 0; k < 32; ++k) stamp_lds[k] = 0;
#endif
    // Every kernel argument the main path uses is fetched here, in one batch: left to the compiler, the
    // argument loads are issued where each is first needed, and every such group is one more round trip to
    // memory on the way to the first gather.
#define SPECATTN_PRELOAD(x) asm volatile("" ::"s"(x))
    SPECATTN_PRELOAD(a.q); SPECATTN_PRELOAD(a.k); SPECATTN_PRELOAD(a.v);
    SPECATTN_PRELOAD(a.B); SPECATTN_PRELOAD(a.H_q); SPECATTN_PRELOAD(a.H_kv); SPECATTN_PRELOAD(a.T);
    SPECATTN_PRELOAD(a.sm_scale);
    SPECATTN_PRELOAD(a.q_stride_b); SPECATTN_PRELOAD(a.q_stride_h); SPECATTN_PRELOAD(a.q_stride_t);
    SPECATTN_PRELOAD(a.kv_stride_b); SPECATTN_PRELOAD(a.kv_stride_h); SPECATTN_PRELOAD(a.kv_stride_n);
    SPECATTN_PRELOAD(a.indices); SPECATTN_PRELOAD(a.idx_stride); SPECATTN_PRELOAD(a.counts);
    SPECATTN_PRELOAD(a.idx_capacity); SPECATTN_PRELOAD(a.dense); SPECATTN_PRELOAD(a.chunk_shift);
    SPECATTN_PRELOAD(a.g_first); SPECATTN_PRELOAD(a.g_count); SPECATTN_PRELOAD(a.k_new);
    SPECATTN_PRELOAD(a.out); SPECATTN_PRELOAD(a.out_lowp); SPECATTN_PRELOAD(a.lse);
    SPECATTN_PRELOAD(plan.part_ml); SPECATTN_PRELOAD(plan.part_o); SPECATTN_PRELOAD(plan.cost_prefix);
    SPECATTN_PRELOAD(plan.n_wg);
    if (LAYOUT != CONTIGUOUS) { SPECATTN_PRELOAD(a.page_table); SPECATTN_PRELOAD(a.page_shift); SPECATTN_PRELOAD(a.max_pages); SPECATTN_PRELOAD(a.kv_stride_page); }
    if (FUSED) { SPECATTN_PRELOAD(a.probs); SPECATTN_PRELOAD(a.probs_stride_b); SPECATTN_PRELOAD(a.probs_stride_h); SPECATTN_PRELOAD(a.seq_lens); SPECATTN_PRELOAD(a.tau); SPECATTN_PRELOAD(a.block_counts); SPECATTN_PRELOAD(a.blocks_per_row); SPECATTN_PRELOAD(a.n_max); }
#undef SPECATTN_PRELOAD
    STAMP(0);
    // Fused path, small calls: the per-block kept counts and thresholds of all rows are requested together with
    // the counts (the row this workgroup starts in is not known yet), so that its first segment need not wait
    // for them again.  The block counts pass through the list buffer, which is free until the first chunk.
    constexpr int EPT0 = CHUNK_TILES * TILE / THREADS;
    const bool bc_all = FUSED && rows <= 64 && rows * a.blocks_per_row <= CHUNK_TILES * TILE;
    int bc_pf[EPT0];
    uint32_t tau_pf = 0;
    if (bc_all) {
#pragma unroll
        for (int k = 0; k < EPT0; ++k) {
            const int j = tid + k * THREADS;
            bc_pf[k] = a.block_counts[j < rows * a.blocks_per_row ? j : 0];
        }
        tau_pf = __float_as_uint(a.tau[lane < rows ? lane : 0]);
    }
    cost_prefix(a, rows, pre, cnt_lds, wsum);
    STAMP(1);
    if (blockIdx.x == 0)
        for (int rr = tid; rr <= rows; rr += THREADS) plan.cost_prefix[rr] = pre[rr];
    const int G = attn_group_heads(a);
    const int QT = G * a.T;
    const float scale2 = a.sm_scale * 1.4426950408889634f;            // scores in log2 units

    // ---- per-segment inputs that are fetched ahead of time -------------------------------------------
    // The Q tile of a segment goes through LDS: thread t fetches 16-byte chunk t%16 of query row t/16
    // ahead of time and stores it (swizzled like a K row) when the segment is staged.
    uint32_t ent_pf[EPT];                    // this thread's entries of the segment's first chunk
    u32x4 q_pf = (u32x4){0u, 0u, 0u, 0u};
    auto fetch_q = [&](int rr) {
        const int b = rr / a.H_kv, h = rr - b * a.H_kv;
        const int qi = tid >> 4, ch = tid & 15;
        q_pf = (u32x4){0u, 0u, 0u, 0u};
        if (qi < QT) {
            const int gh = qi / a.T, tt = qi - gh * a.T;
            const uint16_t *qp = static_cast<const uint16_t *>(a.q) + (int64_t)b * a.q_stride_b +
                                 (int64_t)attn_query_head(a, h, gh) * a.q_stride_h + (int64_t)tt * a.q_stride_t;
            q_pf = *reinterpret_cast<const u32x4 *>(qp + ch * 8);
        }
    };
    auto store_q = [&]() {
        const int qi = tid >> 4, ch = tid & 15;
        if (qi < NQT * 16)
            *reinterpret_cast<u32x4 *>(q_lds + qi * ROW_BYTES + ((ch ^ swz(qi & 15)) << 4)) = q_pf;
    };
    // row offsets (16-byte units) of list entries [first, first + n) of row rr; entries past the end of
    // the list repeat the last kept position (their scores are masked), so every gather stays in bounds
    auto fetch_entries = [&](int rr, int first, int n, uint32_t (&out)[EPT]) {
        const int b = rr / a.H_kv, h = rr - b * a.H_kv;
        const KvMap map = make_map<LAYOUT>(a, b, h);
        const int32_t *idx = a.indices + (int64_t)rr * a.idx_stride;
        const int count = cnt_lds[rr];
        int jj[EPT], pos[EPT];
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            jj[k] = first + tid + k * THREADS;
            jj[k] = jj[k] < count ? jj[k] : count - 1;
        }
        attn_list_pos_n(a, idx, jj, pos);
        map.rel_n<LAYOUT>(pos, out);
        (void)n;                                   // entries past n are computed (in bounds) and never stored
    };
    auto store_entries = [&](int n, const uint32_t (&in)[EPT]) {
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            const int j = tid + k * THREADS;
            if (j < n) ent_lds[j] = in[k];
        }
    };
    // ---- fused path: the list is never read from memory; it is rebuilt from the draft row ----------
    // blk_pre[b] = number of kept positions of row rr before block b (blocks of SEL_BLOCK positions)
    uint32_t seg_tau = 0;                    // tau* of the current segment's row, as bits
    bool bc_in_lds = false;                  // the list buffer holds the block counts of all rows
    auto fused_prepare_row = [&](int rr) {
        lds_barrier();
        const int32_t *bc = a.block_counts + (int64_t)rr * a.blocks_per_row;
        const int *bc_lds = reinterpret_cast<const int *>(ent_lds) + rr * a.blocks_per_row;
        seg_tau = bc_in_lds ? (uint32_t)__builtin_amdgcn_readlane((int)tau_pf, __builtin_amdgcn_readfirstlane(rr)) : __float_as_uint(a.tau[rr]);
        if (wave == 0) {
            int running = 0;
            for (int base = 0; base < a.blocks_per_row; base += 64) {
                const int c = (base + lane < a.blocks_per_row) ? (bc_in_lds ? bc_lds[base + lane] : bc[base + lane]) : 0;
                const int inc = wave_inclusive_sum(c);
                if (base + lane < a.blocks_per_row) blk_pre[base + lane + 1] = running + inc;
                running += __builtin_amdgcn_readlane(inc, 63);
            }
            if (lane == 0) blk_pre[0] = 0;
        }
        lds_barrier();
        bc_in_lds = false;                   // the list buffer is about to be overwritten
    };
    // ent_lds[0 .. n) <- row offsets of the kept positions of rank first .. first + n - 1 of row rr.  The block
    // prefix gives the rank at which every block of SEL_BLOCK positions starts, so the blocks that hold those
    // ranks are independent: each wave takes every NW-th of them, compares the block's draft probabilities
    // with tau* (16 positions per lane, as four coalesced 16-byte loads) and numbers the kept ones with
    // wave-wide prefix sums - no workgroup-wide scan, no barrier between blocks, nothing scanned in vain.
    auto fused_stage = [&](int rr, int first, int n) {
        const int b = rr / a.H_kv, h = rr - b * a.H_kv;
        const KvMap map = make_map<LAYOUT>(a, b, h);
        const float *row = a.probs + (int64_t)b * a.probs_stride_b + (int64_t)h * a.probs_stride_h;
        const bool aligned = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
        int len = a.seq_lens ? a.seq_lens[b] : a.n_max;
        len = len < 0 ? 0 : (len > a.n_max ? a.n_max : len);
        const uint32_t tau_bits = seg_tau;
        const int count = cnt_lds[rr];
        const int last = (first + n) < count ? (first + n) : count;      // ranks [first, last) exist
        // blocks that hold ranks `first` and `last - 1`: blk_pre[b] <= rank < blk_pre[b + 1].  Up to 64 blocks per
        // row every lane looks at one block (one LDS round trip instead of a chain of dependent ones).
        int b0, b1;
        if (a.blocks_per_row <= 64) {
            const int lo = lane < a.blocks_per_row ? blk_pre[lane] : 0x7fffffff;
            const int b0m = __popcll(__ballot(lo <= first)), b1m = __popcll(__ballot(lo <= last - 1));
            b0 = (b0m > 0 ? b0m : 1) - 1;                                // blk_pre[0] = 0 <= any rank
            b1 = (b1m > 0 ? b1m : 1) - 1;
        } else {
            auto block_of = [&](int rank) {
                int lo = 0, hi = a.blocks_per_row;
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (blk_pre[mid] <= rank) lo = mid; else hi = mid;
                }
                return lo;
            };
            b0 = block_of(first); b1 = block_of(last - 1);
        }
        constexpr int QUARTER = SEL_BLOCK / 4;                           // positions one load instruction covers
        static_assert(QUARTER == 64 * 4, "a wave covers a quarter block with one 16-byte load per lane");
        const bool vec_ok = aligned && len >= 4;
        const int last4 = (len - 4) & ~3;                                // start of the row's last whole vector
        for (int blk = b0 + wave; blk <= b1; blk += 2 * NW) {            // two blocks per round and wave
            uint4 u[2][4];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int p0 = (blk + t * NW) * SEL_BLOCK + k * QUARTER + lane * 4;
                    if (vec_ok) {
                        u[t][k] = *reinterpret_cast<const uint4 *>(row + (p0 < last4 ? p0 : last4));   // inside the row
                    } else {
                        u[t][k].x = p0 < len ? __float_as_uint(row[p0]) : 0u;
                        u[t][k].y = p0 + 1 < len ? __float_as_uint(row[p0 + 1]) : 0u;
                        u[t][k].z = p0 + 2 < len ? __float_as_uint(row[p0 + 2]) : 0u;
                        u[t][k].w = p0 + 3 < len ? __float_as_uint(row[p0 + 3]) : 0u;
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int bb = blk + t * NW;
                if (bb > b1) break;                                      // uniform over the wave
                int rk = blk_pre[bb];                                    // rank of the block's first kept position
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int p0 = bb * SEL_BLOCK + k * QUARTER + lane * 4;
                    uint32_t x[4] = {u[t][k].x, u[t][k].y, u[t][k].z, u[t][k].w};
                    if (vec_ok && p0 + 3 >= len) {                       // reaches past the row's end: entry by entry
#pragma unroll
                        for (int i = 0; i < 4; ++i) x[i] = (p0 + i < len) ? __float_as_uint(row[p0 + i]) : 0u;
                    }
                    // kept entries before this lane's four: ballots and per-lane bit counts (no scan)
                    bool keep[4];
                    unsigned long long m[4];
                    int before = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        keep[i] = x[i] != 0x80000000u && x[i] >= tau_bits;       // -0.0 is zero, as in the selection
                        m[i] = __ballot(keep[i]);
                        before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m[i] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m[i], before));
                    }
                    int mine = rk + before - first;                      // slot of this lane's first kept entry
                    const uint32_t off0 = LAYOUT == CONTIGUOUS ? (uint32_t)(map.rel<LAYOUT>(p0) >> 3) : 0u;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        // (kept positions lie below the row's length, so the page-table lookup stays inside the table)
                        if (keep[i] && mine >= 0 && mine < last - first)
                            ent_lds[mine] = LAYOUT == CONTIGUOUS ? off0 + (uint32_t)i * (uint32_t)(map.stride_n >> 3)
                                                                 : (uint32_t)(map.rel<LAYOUT>(p0 + i) >> 3);
                        mine += keep[i] ? 1 : 0;
                    }
                    rk += __popcll(m[0]) + __popcll(m[1]) + __popcll(m[2]) + __popcll(m[3]);
                }
            }
        }
        STAMP_ONCE(8);
        lds_barrier();
        STAMP_ONCE(10);
        // ranks past the end of the list repeat the last kept position (their scores are masked)
        for (int j = last - first + tid; j < n; j += THREADS) ent_lds[j] = ent_lds[last - first - 1];
    };

    // This workgroup's share of the cost line, and the rows of which it holds tiles.  Up to 64 rows, lane i looks
    // at row i: one LDS round trip, the share, every row's local tile range at once and a ballot, instead of a
    // binary search and a row-by-row walk over the table, each step of which waits for an LDS read.
    const bool few_rows = rows <= 64;                    // uniform
    int row_lo = 0, row_cnt = 0, row_hi = 0;
    if (few_rows) {
        row_lo = lane < rows ? pre[lane] : 0;
        row_hi = lane < rows ? pre[lane + 1] : 0;
        row_cnt = lane < rows ? cnt_lds[lane] : 0;
    }
    const int total = few_rows ? __builtin_amdgcn_readlane(row_hi, rows - 1) : pre[rows];
    const Share sh = make_share(total, plan.n_wg, blockIdx.x);
    const int c0 = sh.c0, c1 = sh.c1;
    if (c0 >= c1) { STAMP_DUMP(); return; }
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
    if (r >= rows) { STAMP_DUMP(); return; }

    bool first_staged = false;               // the first chunk's list, Q and the tile counter are already in LDS
    if (bc_all) {
#pragma unroll
        for (int k = 0; k < EPT0; ++k) reinterpret_cast<int *>(ent_lds)[tid + k * THREADS] = bc_pf[k];
        bc_in_lds = true;                    // visible after the barrier that fused_prepare_row starts with
    }
    {
        int lb, le;
        seg_range(r, lb, le);
        STAMP_ONCE(12);
        const int n0 = ((le - lb) < CHUNK_TILES ? (le - lb) : CHUNK_TILES) * TILE;
        // Head start: wave w fetches the indices of tile w of the first chunk itself and requests that
        // tile's rows at once, instead of waiting until the whole chunk's list is staged in LDS.  These index
        // loads go out before everything else the segment needs, since the first gathers wait for them.
        const int n_ahead = (n0 / TILE) < NW ? (n0 / TILE) : NW;
        const bool ahead = !FUSED && wave < n_ahead;
        const int b_first = r / a.H_kv, h_first = r - b_first * a.H_kv;
        const KvMap map_first = make_map<LAYOUT>(a, b_first, h_first);
        int jj_first[8], raw_first[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) jj_first[i] = raw_first[i] = 0;
        // Everything the ordinary start requests is requested and taken in inside this one block, before any
        // gather goes out: loads return in order, so a value left outstanding here - even one that only the
        // compiler's bookkeeping believes outstanding on some path - could later only be waited for together with
        // the gathers issued behind it, and such a wait holds the wave until its first tile has landed.
        if (!FUSED) {
            if (ahead) {
                const int32_t *idx = a.indices + (int64_t)r * a.idx_stride;
                const int count = cnt_lds[r];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    jj_first[i] = (lb + wave) * TILE + 4 * i + g;
                    jj_first[i] = jj_first[i] < count ? jj_first[i] : count - 1;
                }
                attn_list_request_n(a, idx, jj_first, raw_first);
            }
            fetch_q(r);
            fetch_entries(r, lb * TILE, n0, ent_pf);
            asm volatile("" ::"v"(q_pf));
#pragma unroll
            for (int k = 0; k < EPT; ++k) asm volatile("" ::"v"(ent_pf[k]));
#pragma unroll
            for (int i = 0; i < 8; ++i) asm volatile("" ::"v"(raw_first[i]));
        }
        if (FUSED) {
            fetch_q(r);
            // The first chunk of the first segment is staged right here, ahead of the set-up code of the tile loop
            // (several hundred instructions that the unfused path runs while its first gathers are in flight).
            fused_prepare_row(r);
            STAMP_ONCE(14);
            fused_stage(r, lb * TILE, n0);
            first_staged = true;
            // Head start as on the unfused path: wave w requests tile w of the staged chunk at once.
            asm volatile("" ::"v"(q_pf));        // Q has arrived long ago; taken in before the gathers (see below)
            store_q();
            if (tid == 0) *tile_ctr = n_ahead;
            lds_barrier();                       // the padding entries behind the end of the list, Q and the counter are in place
            if (wave < n_ahead) {
                uint32_t e[8];
                lds_read_entries(e, ent_addr + (uint32_t)((wave * TILE + g) << 2));
                const char *kb0 = static_cast<const char *>(a.k) + map_first.base * 2;
                const char *vb0 = static_cast<const char *>(a.v) + map_first.base * 2;
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    __builtin_amdgcn_global_load_lds(GLOBAL_PTR(kb0 + ((int64_t)e[i] << 4) + lane_chunk[i & 3]),
                                                     LDS_PTR(void, wave_lds + i * 1024), 16, 0, KV_AUX);
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    __builtin_amdgcn_global_load_lds(GLOBAL_PTR(vb0 + ((int64_t)e[i] << 4) + lane_chunk[i & 3]),
                                                     LDS_PTR(void, wave_lds + TILE_BYTES + i * 1024), 16, 0, KV_AUX);
            }
        }
        // Q goes into LDS right here.  Inside the segment loop the same store comes after a point where Q may
        // have been requested again (for the next segment) with gathers behind it, and the wait placed there
        // would, on the first pass, hold every wave until its head-start gathers had landed.
        // The first chunk's list goes in with it, and the one barrier that makes both visible comes before the
        // gathers: behind them every wave then runs on to its first tile without meeting the others again.
        if (!FUSED) {
            store_q();
            store_entries(n0, ent_pf);
            if (tid == 0) *tile_ctr = n_ahead;
            first_staged = true;
            lds_barrier();
        }
        STAMP_ONCE(13);
        if (ahead) {
            const KvMap &map = map_first;
            int pos_first[8];
            attn_list_finish_n(a, jj_first, raw_first, pos_first);
            uint32_t e[8];
            map.rel_n<LAYOUT>(pos_first, e);
            const char *kb0 = static_cast<const char *>(a.k) + map.base * 2;
            const char *vb0 = static_cast<const char *>(a.v) + map.base * 2;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(kb0 + ((int64_t)e[i] << 4) + lane_chunk[i & 3]),
                                                 LDS_PTR(void, wave_lds + i * 1024), 16, 0, KV_AUX);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(vb0 + ((int64_t)e[i] << 4) + lane_chunk[i & 3]),
                                                 LDS_PTR(void, wave_lds + TILE_BYTES + i * 1024), 16, 0, KV_AUX);
        }
    }
    if (!FUSED) STAMP_ONCE(8);
    bool head_start = true;                   // true until the first chunk of the first segment has begun

    while (r < rows) {
        int lt_begin, lt_end;
        seg_range(r, lt_begin, lt_end);
        const int r_next = next_seg(r + 1);
        const int b = r / a.H_kv, h = r - b * a.H_kv;
        const int count = cnt_lds[r];
        const KvMap map = make_map<LAYOUT>(a, b, h);
        const char *kbh = static_cast<const char *>(a.k) + map.base * 2;
        const char *vbh = static_cast<const char *>(a.v) + map.base * 2;
        STAMP_ONCE(15);

        f32x4 o[NQT][8];                     // O^T[dv = 16t + 4g + i][q = l16]
        float m_ref[NQT], l_sum[NQT];        // reference max (log2 units) and sum of weights
                                             // (zeroed once the first chunk is staged, which keeps the
                                             //  registers free during the staging)

        // row offsets (in 16-byte units) of the 8 rows this lane helps to fetch for one tile
        auto read_entries = [&](int tile_in_chunk, uint32_t (&ent)[8]) {
            lds_read_entries(ent, ent_addr + (uint32_t)((tile_in_chunk * TILE + g) << 2));
        };
        // gather 32 rows of one tensor into this wave's buffer: 8 instructions of 4 rows x 256 B
        auto issue = [&](const char *base, char *buf, const uint32_t (&ent)[8]) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const char *src = base + ((int64_t)ent[i] << 4) + lane_chunk[i & 3];
                __builtin_amdgcn_global_load_lds(GLOBAL_PTR(src), LDS_PTR(void, buf + i * 1024), 16, 0, KV_AUX);
            }
        };

        for (int ch_begin = lt_begin; ch_begin < lt_end; ch_begin += CHUNK_TILES) {
            const int ch_end = (ch_begin + CHUNK_TILES) < lt_end ? (ch_begin + CHUNK_TILES) : lt_end;
            // ---- stage this chunk's row offsets in LDS (the first chunk's were fetched ahead) ----------
            if (FUSED && !first_staged) {
                if (ch_begin == lt_begin) fused_prepare_row(r); else lds_barrier();
                fused_stage(r, ch_begin * TILE, (ch_end - ch_begin) * TILE);
                if (ch_begin == lt_begin) store_q();
                if (tid == 0) *tile_ctr = 0;
                lds_barrier();
            } else if (!first_staged) {
                if (ch_begin != lt_begin) fetch_entries(r, ch_begin * TILE, (ch_end - ch_begin) * TILE, ent_pf);
                lds_barrier();                                       // previous users of ent_lds / q_lds are done
                store_entries((ch_end - ch_begin) * TILE, ent_pf);
                if (ch_begin == lt_begin) store_q();
                if (tid == 0) *tile_ctr = 0;
                lds_barrier();
            } else {
                first_staged = false;                                // staged, and made visible, before the loop
                STAMP_ONCE(2);
            }
            STAMP_ONCE(9);
            if (ch_begin == lt_begin) {
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt) {
                    m_ref[qt] = -INFINITY;
                    l_sum[qt] = 0.0f;
#pragma unroll
                    for (int t = 0; t < 8; ++t) o[qt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
                }
            }

            // The gathers are not tracked by the compiler's wait insertion; every wait on them is
            // written out.  Per wave the order of issue is K(t), V(t), K(t+1), V(t+1), ...
            // Tiles of the chunk are claimed by the waves as they go (a wave that gets its data later
            // simply takes fewer), one claim ahead of the tile whose gathers are being issued.
            uint32_t ent[8];
            const int n_ch = ch_end - ch_begin;
            int cur;
            if (head_start && wave < n_ch) {
                cur = wave;                                            // already requested above
            } else {
                cur = lds_claim(ctr_addr, lane);
                if (cur < n_ch) {
                    read_entries(cur, ent);
                    issue(kbh, wave_lds, ent);
                    issue(vbh, wave_lds + TILE_BYTES, ent);
                }
            }
            head_start = false;
            int nxt = lds_claim(ctr_addr, lane);
            while (cur < n_ch) {
                const int lt = ch_begin + cur;
                const bool has_next = nxt < n_ch;
                asm volatile("s_waitcnt vmcnt(8)" ::: "memory");        // K(t) landed; V(t) may be in flight
                if (!FUSED) STAMP_ONCE(10);

                // ---- S^T[pos][q] = K Q^T -----------------------------------------------------------
                f32x4 s[NQT][2];
                {
                    KFrags kf;
                    lds_read_k(kf, k_off);
                    if (has_next) {                                    // the K buffer is free again
                        read_entries(nxt, ent);
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
                const int remaining = count - lt * TILE;               // > 0; < TILE only on a row's last tile
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
                if (has_next) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // V(t) landed; K(t+1) in flight
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
                cur = nxt;
                if (has_next) nxt = lds_claim(ctr_addr, lane);
            }
        }   // chunks
        STAMP(3);
        STAMP_ONCE(11);

        // ---- request what the next segment needs, to arrive while this one is wrapped up --------------
        if (r_next < rows) {
            int lb, le;
            seg_range(r_next, lb, le);
            fetch_q(r_next);
            const int n0 = ((le - lb) < CHUNK_TILES ? (le - lb) : CHUNK_TILES) * TILE;
            if (!FUSED) fetch_entries(r_next, lb * TILE, n0, ent_pf);
        }

        // ---- combine the waves of this workgroup: every wave hands its state over lane by lane through its
        //      own tile buffers, which are idle as soon as the wave itself has no tile left - before the barrier,
        //      so that only the last wave's hand-over is waited for; wave w then reduces and writes the
        //      (query tile, dv tile) blocks k = w * KPW .. of all eight states.  (m, l) per query row go into the
        //      block-prefix array, which nobody reads while tiles are processed. -----------------------------
        float *mlw = ml_lds;                     // [NW][16 query rows][2 * NQT]: m, l (summed over the lane groups)
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
                    mlw[(wave * 16 + l16) * 2 * NQT + 2 * qt] = m_ref[qt];
                    mlw[(wave * 16 + l16) * 2 * NQT + 2 * qt + 1] = l;
                }
            }
        }
        lds_barrier();                         // every wave has handed over, and is done with ent_lds and Q
        STAMP(4);
        STAMP(5);
        // Workgroups w0..w1 share row r: a row owned by one workgroup is finished here; otherwise the
        // partial goes to slot w + r for the merge kernel.
        const int w0 = share_of(total, plan.n_wg, pre[r] + SEG_COST), w1 = share_of(total, plan.n_wg, pre[r + 1] - 1);
        {
            constexpr int KPW = NQT * 8 / NW;    // blocks per wave (2 or 1)
            const int slot = blockIdx.x + r;
            float *po = plan.part_o + (int64_t)slot * QTP * D;
            float *pml = plan.part_ml + (int64_t)slot * QTP * 2;
#pragma unroll
            for (int kk = 0; kk < KPW; ++kk) {
                const int k = wave * KPW + kk;   // uniform
                const int qt = k >> 3, t = k & 7;
                float m = -INFINITY;
#pragma unroll
                for (int w = 0; w < NW; ++w) m = fmaxf(m, mlw[(w * 16 + l16) * 2 * NQT + 2 * qt]);
                f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                float l = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float mw = mlw[(w * 16 + l16) * 2 * NQT + 2 * qt];
                    const float f = (mw == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f(mw - m);
                    l += f * mlw[(w * 16 + l16) * 2 * NQT + 2 * qt + 1];
                    acc += f * *reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(smem + w * WAVE_LDS) +
                                                                (k * 64 + lane) * 4);
                }
                const int q = qt * 16 + l16;
                if (q < QT) {
                    if (w0 == w1 && !a.k_new) {
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
        STAMP(6);
        r = r_next;                              // the next segment starts with a barrier of its own
    }
    STAMP(7);
    STAMP_DUMP();
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

}  // namespace

bool attn_mfma_supported(const AttnLaunch &a)
{
    // any number of query heads per kv head: groups of more than 32 query rows run as several launches
    return (a.dtype == SPECATTN_BF16 || a.dtype == SPECATTN_F16) && a.d == 128 && a.T <= 32 && a.H_kv <= MAX_ROWS;
}

int attn_mfma_workgroups() { return cu_count(); }

size_t attn_mfma_workspace_bytes(int rows, int G, int T)
{
    if (rows > MAX_ROWS) rows = MAX_ROWS;                 // larger batches run as several launches
    const size_t qtp = (G * T <= 16) ? 16 : 32;
    const size_t slots = (size_t)attn_mfma_workgroups() + rows;
    size_t bytes = (((size_t)rows + 1) * sizeof(int32_t) + 255) & ~(size_t)255;        // cost prefix
    bytes += slots * qtp * (D + 2) * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

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
    if (!a.workspace || a.workspace_bytes < attn_mfma_workspace_bytes(rows, G, a.T)) {
        set_error("attention workspace has %zu bytes, %zu needed", a.workspace_bytes, attn_mfma_workspace_bytes(rows, G, a.T));
        return SPECATTN_EWORKSPACE;
    }
    char *ws = static_cast<char *>(a.workspace);
    plan.cost_prefix = reinterpret_cast<int32_t *>(ws);
    ws += (((size_t)rows + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
    plan.part_ml = reinterpret_cast<float *>(ws);
    plan.part_o = plan.part_ml + slots * qtp * 2;
    const size_t lds = LDS_BYTES;
    const int layout = a.indices_are_physical ? PHYSICAL : (a.page_table ? PAGE_TABLE : CONTIGUOUS);
    const void *fn = nullptr;
    const bool fused = a.probs != nullptr;
    const bool f16 = a.dtype == SPECATTN_F16;
#define PICK(NQT, LAY, FUS)                                                                                      \
    if (qtp == 16 * NQT && layout == LAY && fused == FUS)                                                        \
        fn = f16 ? reinterpret_cast<const void *>(&attn_mfma_kernel<NQT, LAY, FUS, true>)                        \
                 : reinterpret_cast<const void *>(&attn_mfma_kernel<NQT, LAY, FUS, false>);
    PICK(1, CONTIGUOUS, false) PICK(1, PAGE_TABLE, false) PICK(1, PHYSICAL, false)
    PICK(2, CONTIGUOUS, false) PICK(2, PAGE_TABLE, false) PICK(2, PHYSICAL, false)
    PICK(1, CONTIGUOUS, true) PICK(1, PAGE_TABLE, true) PICK(2, CONTIGUOUS, true) PICK(2, PAGE_TABLE, true)
    if (!fn) { set_error("the fused path takes logical positions, not pool slots"); return SPECATTN_EUNSUPPORTED; }
#undef PICK
    {
        // the kernels use more LDS than the default limit; raise it once per kernel (any thread may call)
        static std::mutex mu;
        static const void *configured[32] = {nullptr};
        std::lock_guard<std::mutex> lock(mu);
        bool seen = false;
        for (const void *c : configured) seen = seen || c == fn;
        if (!seen) {
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
                set_error("cannot reserve %zu bytes of LDS", lds);
                return SPECATTN_EHIP;
            }
            for (const void *&c : configured) if (!c) { c = fn; break; }
        }
    }
#ifdef SPECATTN_TIMING
    extern long long *g_specattn_timing;      // development builds: set by the timing harness
    plan.timing = g_specattn_timing;
    if (!plan.timing) { set_error("timing build without a timing buffer"); return SPECATTN_EINVAL; }
#endif
    void *kargs[] = {const_cast<AttnLaunch *>(&a), &plan};
    if (hipLaunchKernel(fn, dim3(plan.n_wg), dim3(THREADS), kargs, lds, stream) != hipSuccess) {
        set_error("attn_mfma_kernel: launch failed");
        (void)hipGetLastError();
        return SPECATTN_EHIP;
    }
    specattn_status st = check_launch("attn_mfma_kernel");
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
    const int b_max = MAX_ROWS / a.H_kv;
    if (a.B <= b_max) return launch_chunk(a, stream);
    const int es = 2;                                       // bf16 or fp16
    const int G = a.H_q / a.H_kv;
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
        if (a.probs) {
            c.probs = a.probs + (int64_t)b0 * a.probs_stride_b;
            c.tau = a.tau + r0;
            c.block_counts = a.block_counts + r0 * a.blocks_per_row;
        }
        (void)G;
        const specattn_status st = launch_chunk(c, stream);
        if (st != SPECATTN_OK) return st;
    }
    return SPECATTN_OK;
}

}  // namespace specattn

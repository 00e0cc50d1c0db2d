// MM-DiT joint attention for MI355X (gfx950): dense and block-sparse, flash-style.
//
// Operation: RAPID^3 Sec. 3.1 Eq. 1 (self-attention block of a DiT layer) and
// Sec. 3.2 Level-3 / Eq. 4 (the same block restricted to a pruned attention map,
// per layer and per head).  The pruned map is given as a block mask; pruned tiles
// are never read.
//
// Building blocks (a wavefront always owns 32 queries and walks over 64-key tiles):
//   S^T = K Q^T    v_mfma_f32_32x32x16_bf16, A = K tile rows from LDS (128-bit
//                  reads), B = the wavefront's Q rows held in registers for the
//                  whole kernel.  Computing the TRANSPOSED score tile puts one
//                  query per lane: the running max / sum are per-lane scalars, the
//                  row reductions are in-register plus ONE cross-half exchange
//                  (v_permlane32_swap), and the fp32 accumulator registers of a
//                  lane are, after conversion to bf16, exactly the B operand of
//                  the next product -- P never touches LDS.
//   O^T += V^T P^T same MFMA; A = V^T fragments fetched straight out of the
//                  row-major V tile with the LDS transpose read
//                  (ds_read_b64_tr_b16), B = P^T from the registers above.
//                  The contraction index is a dummy, so the key order inside a
//                  16-key step is whatever the accumulator layout yields (keys
//                  4h+r and 8+4h+r for lane half h); V^T is fetched in that order.
//   tiles          global -> LDS directly (global_load_lds_dwordx4), chunk-swizzled,
//                  several tiles ahead of their use.
// Kernels:
//   attn_dense_pp_kernel<D>     dense: 256 queries per workgroup, 8 wavefronts in two groups that
//                               alternate a softmax phase and an MFMA phase in anti-phase
//   attn_sparse_sg_kernel<D>    sparse, 128-token mask tiles: one four-wavefront workgroup per plan
//                               record (a query-block or a piece of its kept list); pieces are
//                               merged by the last one to finish
//   attn_sparse_pp_kernel<D,2>  sparse, 64-token mask tiles: one query-block per workgroup, the kept
//                               list split between two wavefront groups and merged through LDS
//   plan_small_kernel           mask compaction and launch plan in one launch (up to 64 blocks per side)
//   compact_mask_kernel, plan_split_kernel (128-token tiles), plan_kernel (64-token tiles)
//                               the same in two launches for larger problems
// Entry points (C ABI, bottom of the file): rapid_attn_dense, rapid_attn_block_sparse,
// rapid_attn_block_sparse_static (scratch in a fixed array of this file), rapid_attn_joint,
// rapid_attn_joint_select (selection kernels of rapid_mask.hip write the kept lists).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <initializer_list>

#include "rapid_attn.h"
#include "rapid_internal.h"
#include "rapid_mask.h"

// Scratch of the entry point that allocates nothing (see static_scratch below).
static __device__ __align__(256) unsigned char scratch[RAPID_ATTN_STATIC_SCRATCH_BYTES];

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Whether the common path of the softmax computes no row maximum (softmax_tile).  At D = 64 the
// vector unit is the busiest one (half as many MFMA cycles per score as at D = 128) and every
// instruction taken out of the softmax phase shows; at D = 128 it made no difference.
template <int D> struct Optimistic { static constexpr bool value = D == 64; };

constexpr int KT = 64;          // keys per LDS tile
constexpr int XCDS = 8;         // L2 domains the dispatcher deals workgroups over
constexpr int DENSE_QT = 256;    // query rows per workgroup on the dense path
constexpr float LOG2E = 1.44269504088896340736f;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// A [B, H, tokens, D] tensor handed over as one or two token segments: token t < n0 is row t
// of segment 0, any other token is row t - n0 of segment 1 (MM-DiT keeps the image and the
// text stream in separate tensors and joins them only for attention).  Strides in elements,
// D contiguous; head and token strides are common to both segments.
struct SegTensor {
    const __bf16* seg0;
    const __bf16* seg1;      // null when there is one segment
    long long sb0, sb1;      // batch strides
    long long sh, sn;        // head stride, token stride
};

// The token rows of one (sample, head): row r starts at (r < n0 ? base0 : base1) + r * row_bytes
// (base1 is biased by -n0 rows so that both segments are indexed by the joint token number).
struct Rows {
    const char* base0;
    const char* base1;
    int n0;
    unsigned row_bytes;
    __device__ __forceinline__ const char* row(int r) const { return (r < n0 ? base0 : base1) + (size_t)r * row_bytes; }
};

__device__ __forceinline__ Rows rows_of(const SegTensor& t, int b, int h, int n0)
{
    Rows r;
    r.base0 = (const char*)(t.seg0 + (size_t)b * t.sb0 + (size_t)h * t.sh);
    r.base1 = t.seg1 ? (const char*)(t.seg1 + (size_t)b * t.sb1 + (size_t)h * t.sh) - (size_t)n0 * t.sn * 2 : r.base0;
    r.n0 = n0;
    r.row_bytes = (unsigned)(t.sn * 2);
    return r;
}

struct AttnParams {
    SegTensor q, k, v, o;
    const int32_t* kv_lens;  // per-sample valid tokens (device, [B]) or null: kv_len for all
    int n0;                  // tokens in the first segment (N when there is one)
    const int32_t* counts;   // sparse: kept key-blocks per (b,h,query-block); dense: null
    const int32_t* order;    // sparse: launch plan (64-token tiles: item ids; 128-token tiles: PlanRec records)
    const int32_t* index;    // sparse: kept key-block lists, nb per row
    int32_t* arrived;        // sparse, 128-token tiles: finished pieces per split item
    char* partial;           // sparse, 128-token tiles: partial results of the pieces of split items
    int H, N, kv_len;
    int nq;                  // query tiles per (sample, head)
    int items;               // B*H*nq
    int chunk;               // ceil(items / XCDS)
    int block, nb;           // mask tile edge, N / block (sparse only)
    int sub_shift;           // log2(block / 64)
    float c;                 // scale * log2(e)
};

// ---------------------------------------------------------------------------
// Mask compaction: one wavefront per (b, h, query-block) row of the mask.
// counts[row] = number of kept key-blocks whose first token is below kv_len;
// index[row*nb + 0..count) = those key-blocks, ascending.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void compact_mask_kernel(
    const unsigned char* __restrict__ mask, int rows, int nb, int block, int kv_len,
    const int32_t* __restrict__ kv_lens, int rows_per_sample, int N,
    int32_t* __restrict__ counts, int32_t* __restrict__ index)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    if (kv_lens != nullptr) {
        kv_len = kv_lens[row / rows_per_sample];
        kv_len = kv_len < 0 ? 0 : (kv_len > N ? N : kv_len);
    }
    const unsigned char* mrow = mask + (size_t)row * nb;
    int32_t* irow = index + (size_t)row * nb;
    int base = 0;
    for (int j0 = 0; j0 < nb; j0 += 64) {
        const int j = j0 + lane;
        const bool keep = (j < nb) && (mrow[j] != 0) && ((long long)j * block < kv_len);
        const unsigned long long bal = __ballot(keep);
        if (keep) irow[base + __popcll(bal & ((1ull << lane) - 1ull))] = j;
        base += __popcll(bal);
    }
    if (lane == 0) counts[row] = base;
}

// ---------------------------------------------------------------------------
// Launch plans of the sparse path.  Items = (b, h, query-block).  All items of one (b,h)
// go to XCD (b*H + h) % 8, so the K/V of a head stay in one L2; inside an XCD the entries
// are ordered by length, longest first (the dispatcher hands out workgroups in id order, so
// this is longest-processing-time-first scheduling of a ragged batch).  One workgroup per
// XCD: counting sort over the lengths.  Entries of equal length land in arbitrary order;
// that only changes which workgroup computes an entry, never its value.
// ---------------------------------------------------------------------------
constexpr int PLAN_MAX_NB = 8176;                // bins 0 .. nb fit the scan below
constexpr int PLAN_BINS = 8192;                  // 8 bins per thread

constexpr int PLAN_CACHE = 4096;                 // counts of this many items are kept in LDS

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves:
// four shifts inside each row of 16 lanes, then lane 15 of rows 0 and 2 is added to rows 1
// and 3, then lane 31 to rows 2 and 3.  A lane without a source takes 0.  All lanes active.
__device__ __forceinline__ int wave_scan_inclusive(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2, 3
    return v;
}

// Maximum over the 64 lanes, valid in lane 63 (same moves; a lane without a source keeps its own).
__device__ __forceinline__ int wave_max_to_last(int v)
{
    auto step = [&](int t) { v = t > v ? t : v; };
    step(__builtin_amdgcn_update_dpp(v, v, 0x111, 0xf, 0xf, false));
    step(__builtin_amdgcn_update_dpp(v, v, 0x112, 0xf, 0xf, false));
    step(__builtin_amdgcn_update_dpp(v, v, 0x114, 0xf, 0xf, false));
    step(__builtin_amdgcn_update_dpp(v, v, 0x118, 0xf, 0xf, false));
    step(__builtin_amdgcn_update_dpp(v, v, 0x142, 0xa, 0xf, false));
    step(__builtin_amdgcn_update_dpp(v, v, 0x143, 0xc, 0xf, false));
    return v;
}

// Exclusive prefix sum of one value per thread over the 1024 threads of the block: a scan
// inside each wavefront, then the 16 wavefront totals through LDS.  Two barriers.
__device__ __forceinline__ int plan_block_scan(int v, int* wave_sum, int tid)
{
    const int lane = tid & 63, wv = tid >> 6;
    const int incl = wave_scan_inclusive(v);
    if (lane == 63) wave_sum[wv] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {                // all 16 reads in flight, none depends on wv
        const int t = wave_sum[w];
        before += w < wv ? t : 0;
    }
    __syncthreads();
    return before + incl - v;
}

// Exclusive prefix sum of hist[0 .. PLAN_BINS) in place (thread t owns bins 8t..8t+7).
__device__ __forceinline__ void plan_scan_bins(int* hist, int* wave_sum, int tid)
{
    int own[8], sum = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) { own[j] = hist[8 * tid + j]; sum += own[j]; }
    int run = plan_block_scan(sum, wave_sum, tid);
#pragma unroll
    for (int j = 0; j < 8; ++j) { hist[8 * tid + j] = run; run += own[j]; }
    __syncthreads();
}

// 64-token mask tiles: order[x * chunk + i] = i-th item of XCD x, -1 past the end.
__global__ __launch_bounds__(1024) void plan_kernel(const int32_t* __restrict__ counts, int BH, int nb, int chunk,
                                                    int32_t* __restrict__ order)
{
    __shared__ int hist[PLAN_BINS];              // by r = nb - count (r = 0: longest)
    __shared__ int wave_sum[16];
    const int x = blockIdx.x, tid = threadIdx.x;
    const int n_bh = (BH - x + XCDS - 1) / XCDS;  // (b,h) pairs with index % 8 == x
    const int n_items = n_bh > 0 ? n_bh * nb : 0;
    int32_t* out = order + (size_t)x * chunk;
    auto item_of = [&](int i) { return ((i / nb) * XCDS + x) * nb + i % nb; };
    if (nb > PLAN_MAX_NB) {                       // no sort: natural order
        for (int i = tid; i < chunk; i += 1024) out[i] = i < n_items ? item_of(i) : -1;
        return;
    }
    for (int i = tid; i < chunk; i += 1024) out[i] = -1;
#pragma unroll
    for (int j = 0; j < 8; ++j) hist[8 * tid + j] = 0;
    __syncthreads();
    for (int i = tid; i < n_items; i += 1024) atomicAdd(&hist[nb - counts[item_of(i)]], 1);
    __syncthreads();
    plan_scan_bins(hist, wave_sum, tid);
    for (int i = tid; i < n_items; i += 1024) {
        const int item = item_of(i);
        out[atomicAdd(&hist[nb - counts[item]], 1)] = item;
    }
}

// 128-token mask tiles: the plan is a list of records, one per workgroup.  The dispatcher
// fills the CUs entry by entry, so an entry that is long against a CU's share of the work
// leaves most of the chip idle at the end: an item can be cut into P pieces (SplitRule
// below).  Each piece is a record of its own; the pieces leave partial results in the
// workspace and the last one to finish combines them.  A piece is expensive (its partial
// result goes through memory: measured at D = 128, an entry costs about two key-blocks of
// time and a piece two more), so only rows several times the average (the text rows of a
// sparse mask) are worth cutting.  Partial-result slots are handed out in item order (a
// prefix sum, so the plan does not depend on timing); an item that no longer fits in the
// XCD's pmax slots stays whole.
struct PlanRec {
    int item;     // b*H*nb + h*nb + query-block, or -1: no work
    int blk0;     // first position of the piece in the item's kept list
    int nblk;     // kept key-blocks of the piece
    int w;        // -1: the whole item; else (first partial slot << 8) | (piece << 4) | (P - 1)
};
constexpr int CUS_PER_XCD = 32;                  // MI355X: 256 CUs in 8 XCDs
constexpr int SPLIT_MIN_BLOCKS = 8;
constexpr int SPLIT_MAX_PIECES = 16;
constexpr int SPLIT_SLOTS = 256;                 // partial-result slots per XCD (the rule needs < 256)
constexpr int ENTRY_COST = 2, PIECE_COST = 2;    // measured, in key-blocks of time at D = 128

// The rule of one XCD.  P(c) = round(c * g / total) pieces for an item with c kept key-blocks
// (g granules: pieces of about total / g), or p_all pieces for every item when that is set;
// in both cases at most c / SPLIT_MIN_BLOCKS and SPLIT_MAX_PIECES, at least 1.
//   D = 128: g = 32 CUs x 2.5.  Rows that are all about alike (the longest within 1/9 of the
//     mean: an all-ones mask) are not told apart by their lengths; what matters then is how
//     many rounds the 64 places of the XCD need, so p_all is the P that minimises
//     rounds(P) * (piece length + cost of an entry), the first such P.
//   D = 64: g = 32 x 4; rows all alike: 32 x 12 (fewer items than the 128 places: cut them all).
struct SplitRule {
    int g;
    int p_all;     // 0: by length
};

// cost of cutting every one of n_items rows of max_c blocks into P pieces, D = 128
__device__ __forceinline__ long long split_alike_cost(int n_items, int max_c, int P)
{
    const long long places = CUS_PER_XCD * 2;
    const long long rounds = ((long long)n_items * P + places - 1) / places;
    return rounds * ((max_c + P - 1) / P + ENTRY_COST + (P > 1 ? PIECE_COST : 0));
}

__device__ __forceinline__ bool rows_alike(int n_items, int max_c, unsigned long long total)
{
    return 8ull * (unsigned long long)n_items * (unsigned)max_c <= 9ull * total;
}

// `costs` holds split_alike_cost for P = 1 .. SPLIT_MAX_PIECES (used at D = 128 when the rows are alike)
__device__ __forceinline__ SplitRule split_rule(int D, int n_items, int max_c, unsigned long long total,
                                                const long long* costs)
{
    SplitRule r;
    r.p_all = 0;
    const bool alike = rows_alike(n_items, max_c, total);
    if (D == 128) {
        r.g = CUS_PER_XCD * 5 / 2;
        if (alike && total != 0ull) {
            long long best = costs[0];
            r.p_all = 1;
            const int top = max_c / SPLIT_MIN_BLOCKS < SPLIT_MAX_PIECES ? max_c / SPLIT_MIN_BLOCKS : SPLIT_MAX_PIECES;
            for (int P = 2; P <= top; ++P)
                if (costs[P - 1] < best) { best = costs[P - 1]; r.p_all = P; }
        }
    } else {
        r.g = CUS_PER_XCD * (alike ? 12 : 4);
    }
    return r;
}

__device__ __forceinline__ int split_pieces(int c, unsigned long long total, const SplitRule& rule)
{
    if (total == 0ull) return 1;
    unsigned long long P = rule.p_all ? (unsigned long long)rule.p_all
                                      : (2ull * (unsigned)c * (unsigned)rule.g + total) / (2ull * total);
    const unsigned long long by_len = (unsigned)c / SPLIT_MIN_BLOCKS;
    if (P > by_len) P = by_len;
    if (P > (unsigned long long)SPLIT_MAX_PIECES) P = SPLIT_MAX_PIECES;
    return P < 1ull ? 1 : (int)P;
}

__global__ __launch_bounds__(1024) void plan_split_kernel(const int32_t* __restrict__ counts, int BH, int nb, int cap,
                                                          int pmax, int D, PlanRec* __restrict__ recs,
                                                          int32_t* __restrict__ arrived)
{
    __shared__ int hist[PLAN_BINS];              // by r = nb - length (r = 0: longest)
    __shared__ int ccache[PLAN_CACHE];           // counts of the first items, read once
    __shared__ int wave_sum[16];
    __shared__ unsigned long long total;          // kept key-blocks of this XCD's items
    __shared__ int longest;                       // of its rows
    __shared__ long long alike_cost[SPLIT_MAX_PIECES];
    const int x = blockIdx.x, tid = threadIdx.x;
    const int n_bh = (BH - x + XCDS - 1) / XCDS;
    const int n_items = n_bh > 0 ? n_bh * nb : 0;
    PlanRec* out = recs + (size_t)x * cap;
    auto item_of = [&](int i) { return ((i / nb) * XCDS + x) * nb + i % nb; };
    auto count_of = [&](int i) { return i < PLAN_CACHE ? ccache[i] : counts[item_of(i)]; };
    const PlanRec none = {-1, 0, 0, -1};
    for (int i = tid; i < pmax; i += 1024) arrived[(size_t)x * pmax + i] = 0;
    if (nb > PLAN_MAX_NB) {                       // no sort, no pieces: natural order
        for (int i = tid; i < cap; i += 1024) {
            PlanRec r = none;
            if (i < n_items) { r.item = item_of(i); r.nblk = counts[r.item]; }
            out[i] = r;
        }
        return;
    }
    if (tid == 0) { total = 0ull; longest = 0; }
#pragma unroll
    for (int j = 0; j < 8; ++j) hist[8 * tid + j] = 0;
    __syncthreads();
    {
        unsigned long long mine = 0ull;
        int mx = 0;
        for (int i = tid; i < n_items; i += 1024) {
            const int c = counts[item_of(i)];
            if (i < PLAN_CACHE) ccache[i] = c;
            mine += (unsigned long long)c;
            mx = c > mx ? c : mx;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            mine += __shfl_down(mine, d, 64);
            const int o = __shfl_down(mx, d, 64);
            mx = o > mx ? o : mx;
        }
        if ((tid & 63) == 0) { atomicAdd(&total, mine); atomicMax(&longest, mx); }
    }
    for (int i = tid; i < cap; i += 1024) out[i] = none;
    __syncthreads();
    const unsigned long long tot = total;
    if (tid < SPLIT_MAX_PIECES) alike_cost[tid] = split_alike_cost(n_items, longest, tid + 1);
    __syncthreads();
    const SplitRule rule = split_rule(D, n_items, longest, tot, alike_cost);
    // partial-result slots in item order: thread t owns the items [lo, hi)
    const int per = (n_items + 1023) / 1024;
    const int lo = tid * per < n_items ? tid * per : n_items;
    const int hi = lo + per < n_items ? lo + per : n_items;
    int mine = 0;
    for (int i = lo; i < hi; ++i) {
        const int P = split_pieces(count_of(i), tot, rule);
        if (P > 1) mine += P;
    }
    const int first_slot = plan_block_scan(mine, wave_sum, tid);
    // pieces of item i: P (1 = whole) and the first partial slot
    auto pieces_of = [&](int c, int& run, int& P, int& slot0) {
        const int want = split_pieces(c, tot, rule);
        P = want;
        slot0 = -1;
        if (want > 1) {
            if (run + want <= pmax) slot0 = run; else P = 1;
            run += want;                          // the prefix counts every candidate
        }
    };
    {
        int run = first_slot;
        for (int i = lo; i < hi; ++i) {
            const int c = count_of(i);
            int P, slot0;
            pieces_of(c, run, P, slot0);
            for (int k = 0; k < P; ++k) atomicAdd(&hist[nb - (c * (k + 1) / P - c * k / P)], 1);
        }
    }
    __syncthreads();
    plan_scan_bins(hist, wave_sum, tid);
    {
        int run = first_slot;
        for (int i = lo; i < hi; ++i) {
            const int item = item_of(i);
            const int c = count_of(i);
            int P, slot0;
            pieces_of(c, run, P, slot0);
            for (int k = 0; k < P; ++k) {
                PlanRec r;
                r.item = item;
                r.blk0 = c * k / P;
                r.nblk = c * (k + 1) / P - r.blk0;
                r.w = (P > 1) ? (((x * pmax + slot0) << 8) | (k << 4) | (P - 1)) : -1;
                out[atomicAdd(&hist[nb - r.nblk], 1)] = r;
            }
        }
    }
}

// Small problems (the 1024x1024-image shapes: about a hundred items per XCD): compaction and
// plan in ONE launch, written for latency.  Two launches with a trip through memory between
// them cost 11 us of a sparse call that takes 80 .. 130 us.  Here every thread loads its
// bytes of the XCD's mask rows at once and keeps them in registers; a kept block sets its
// bit in the row's 64-bit word in LDS (nb <= 64), the rank of a block in its row's list is a
// population count below its bit, and the plan is made one thread per item in 32-bit
// arithmetic (same rule, same records as plan_split_kernel: the limits below keep every
// intermediate below 2^32).  No loop in it depends on memory more than once.
constexpr int SMALL_NB = 64;                     // mask blocks per side
constexpr int SMALL_ITEMS = 1024;                // items of one XCD
constexpr int SMALL_SWEEPS = 8;                  // mask bytes of one XCD's items: 1024 per sweep
constexpr int SMALL_BYTES = 1024 * SMALL_SWEEPS;

__global__ __launch_bounds__(1024) void plan_small_kernel(
    const unsigned char* __restrict__ mask, const int32_t* __restrict__ kv_lens, int kv_len, int N, int block,
    int H, int BH, int nb, int cap, int pmax, int D,
    int32_t* __restrict__ counts, int32_t* __restrict__ index, PlanRec* __restrict__ recs,
    int32_t* __restrict__ arrived)
{
    __shared__ unsigned rowbits[2 * SMALL_ITEMS]; // kept key-blocks of item i: bits of words 2i, 2i+1
    __shared__ int live[SMALL_ITEMS];            // per (b,h) pair: key-blocks that start below kv_len
    __shared__ int hist[128];                    // by r = nb - length; hist[nb + 1] = number of records
    __shared__ int wave_sum[16], kept_sum[16], wave_max[16];
    __shared__ long long alike_cost[SPLIT_MAX_PIECES];
    const int x = blockIdx.x, tid = threadIdx.x;
    const int n_bh = BH > x ? (BH - x + XCDS - 1) / XCDS : 0;
    const int n_items = n_bh * nb;
    const unsigned per_bh = (unsigned)(nb * nb);
    const unsigned bytes = (unsigned)n_bh * per_bh;
    PlanRec* out = recs + (size_t)x * cap;
    // f / nb^2 for f * nb^2 < 2^32 by one multiplication (nb = 1: the product wraps, handled
    // apart); f / nb for f < 2^13, nb <= 64 by a full-rate 24-bit multiplication: with
    // m = ceil(2^19 / nb), f * (m * nb - 2^19) < 2^13 * 64 = 2^19, so the quotient is exact
    const unsigned magic_bh = 0xffffffffu / per_bh + 1u, magic_nb = ((1u << 19) + (unsigned)nb - 1u) / (unsigned)nb;
    auto div_bh = [&](unsigned f) { return per_bh == 1u ? f : __umulhi(f, magic_bh); };
    auto div_nb = [&](unsigned f) { return __umul24(f, magic_nb) >> 19; };

    // byte f of this XCD's rows: pair g = f / nb^2, then row-major inside the pair.  Lanes past
    // the end load the last byte again, so that no load sits behind a branch.
    unsigned v[SMALL_SWEEPS];
#pragma unroll
    for (int t = 0; t < SMALL_SWEEPS; ++t) {
        v[t] = 0;
        if (1024u * t < bytes) {                  // the same for the whole workgroup
            const unsigned f = (unsigned)tid + 1024u * t, fc = f < bytes ? f : bytes - 1u;
            const unsigned g = div_bh(fc);
            v[t] = mask[(size_t)(g * XCDS + x) * per_bh + (fc - g * per_bh)];
        }
    }
    for (int g = tid; g < n_bh; g += 1024) {
        int len = kv_len;
        if (kv_lens != nullptr) {
            len = kv_lens[(g * XCDS + x) / H];
            len = len < 0 ? 0 : (len > N ? N : len);
        }
        const int lv = (len + block - 1) / block;
        live[g] = lv < nb ? lv : nb;
    }
    for (int i = tid; i < pmax; i += 1024) arrived[(size_t)x * pmax + i] = 0;
    rowbits[tid] = 0u;
    rowbits[tid + 1024] = 0u;
    if (tid < 128) hist[tid] = 0;
    __syncthreads();

    // 64 consecutive bytes are the ends of at most a few rows: one ballot, and the first lane
    // of each row's stretch adds the stretch to the row's word (same-address LDS atomics from
    // every lane would serialise)
    int kept = 0;                                 // kept blocks seen by this wavefront
#pragma unroll
    for (int t = 0; t < SMALL_SWEEPS; ++t) {
        if (1024u * t < bytes) {                  // the same for the whole workgroup
            const unsigned f = (unsigned)tid + 1024u * t;
            const bool in = f < bytes;
            const unsigned i = div_nb(in ? f : 0u), j = (in ? f : 0u) - __umul24(i, nb);
            const bool keep = in && v[t] != 0u && (int)j < live[div_nb(i)];
            const unsigned long long bal = __ballot(keep);
            const unsigned lane = (unsigned)tid & 63u;
            kept += __popcll(bal);
            if (in && (j == 0u || lane == 0u)) {
                const unsigned left = (unsigned)nb - j, room = 64u - lane;
                const unsigned len = left < room ? left : room;
                const unsigned long long seg = (bal >> lane) & (len >= 64u ? ~0ull : (1ull << len) - 1ull);
                const unsigned long long word = seg << j;                      // j + len <= nb <= 64
                if ((unsigned)word) atomicOr(&rowbits[2u * i], (unsigned)word);
                if ((unsigned)(word >> 32)) atomicOr(&rowbits[2u * i + 1u], (unsigned)(word >> 32));
            }
        }
    }
    if ((tid & 63) == 0) kept_sum[tid >> 6] = kept;
    __syncthreads();
    unsigned tot = 0u;                            // kept key-blocks of this XCD's items
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += (unsigned)kept_sum[w];

#pragma unroll
    for (int t = 0; t < SMALL_SWEEPS; ++t) {
        const unsigned f = (unsigned)tid + 1024u * t;
        if (f < bytes && v[t] != 0u) {
            const unsigned i = div_nb(f), j = f - __umul24(i, nb), g = div_nb(i);
            const unsigned lo = rowbits[2u * i], hi = rowbits[2u * i + 1u];
            const unsigned long long bits = ((unsigned long long)hi << 32) | lo;
            if ((bits >> j) & 1ull) {
                const unsigned row = __umul24(g * XCDS + x, nb) + (i - __umul24(g, nb));   // < 2^13
                index[__umul24(row, nb) + __popcll(bits & ((1ull << j) - 1ull))] = (int)j;
            }
        }
    }

    // plan: thread i takes item i.  Pieces as in split_pieces(), in 32 bits.
    const bool has = tid < n_items;
    const int item = has ? (int)(__umul24(div_nb(tid) * XCDS + x, nb) + (tid - __umul24(div_nb(tid), nb))) : 0;
    const int c = has ? __popc(rowbits[2 * tid]) + __popc(rowbits[2 * tid + 1]) : 0;
    if (has) counts[item] = c;
    {                                             // the longest row, to every thread
        const int mx = wave_max_to_last(c);
        if ((tid & 63) == 63) wave_max[tid >> 6] = mx;
    }
    __syncthreads();
    int longest = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) longest = wave_max[w] > longest ? wave_max[w] : longest;
    if (D == 128 && rows_alike(n_items, longest, tot)) {   // the same for the whole workgroup
        if (tid < SPLIT_MAX_PIECES) alike_cost[tid] = split_alike_cost(n_items, longest, tid + 1);
        __syncthreads();
    }
    const SplitRule rule = split_rule(D, n_items, longest, tot, alike_cost);
    int want = 1;
    if (has && tot != 0u) {
        unsigned P = rule.p_all ? (unsigned)rule.p_all : (2u * (unsigned)c * (unsigned)rule.g + tot) / (2u * tot);
        const unsigned by_len = (unsigned)c / SPLIT_MIN_BLOCKS;
        P = P > by_len ? by_len : P;
        P = P > (unsigned)SPLIT_MAX_PIECES ? SPLIT_MAX_PIECES : P;
        want = P < 1u ? 1 : (int)P;
    }
    const int first_slot = plan_block_scan(want > 1 ? want : 0, wave_sum, tid);
    int P = want, slot0 = -1;
    if (want > 1) {
        if (first_slot + want <= pmax) slot0 = first_slot; else P = 1;
    }
    // piece k holds c(k+1)/P - ck/P key-blocks: c/P, plus one whenever the running remainder wraps
    const int q = c / P, r = c - q * P;
    if (has) {
        int e = 0;
        for (int k = 0; k < P; ++k) {
            e += r;
            const int extra = e >= P;
            e -= extra ? P : 0;
            atomicAdd(&hist[nb - (q + extra)], 1);
        }
    }
    __syncthreads();
    {
        const int mine = tid <= nb ? hist[tid] : 0;
        const int before = plan_block_scan(mine, wave_sum, tid);
        if (tid <= nb + 1) hist[tid] = before;   // entry nb + 1: all records
    }
    __syncthreads();
    const int n_rec = hist[nb + 1];
    __syncthreads();                              // everyone has read it before the bins move
    if (has) {
        int e = 0, b0 = 0;
        for (int k = 0; k < P; ++k) {
            e += r;
            const int extra = e >= P;
            e -= extra ? P : 0;
            PlanRec rec;
            rec.item = item;
            rec.blk0 = b0;
            rec.nblk = q + extra;
            rec.w = (P > 1) ? (((x * pmax + slot0) << 8) | (k << 4) | (P - 1)) : -1;
            b0 += rec.nblk;
            // At launch the dispatcher deals the XCD's workgroups out to its 32 CUs in turn (seen in
            // the hardware ids of traced launches): CU i starts with the records i, i + 32, ...
            // Longest-first order would give CU 0 the longest record of every round of 32, so the
            // odd rounds of the first wave (as many records as the XCD has places) run backwards.
            // Later records go wherever a place frees up first and stay longest first.
            int pos = atomicAdd(&hist[nb - rec.nblk], 1);
            const int round = pos >> 5;
            if (pos < CUS_PER_XCD * (D == 128 ? 2 : 4) && (round & 1)) {
                const int left = n_rec - (round << 5);
                pos = (round << 5) + (left < 32 ? left : 32) - 1 - (pos & 31);
            }
            out[pos] = rec;
        }
    }
    const PlanRec none = {-1, 0, 0, -1};
    for (int i = n_rec + tid; i < cap; i += 1024) out[i] = none;
}

// ---------------------------------------------------------------------------
// Attention.  D in {64,128}; NW wavefronts; query tile = 32*NW rows.
// ---------------------------------------------------------------------------
// LDS tile geometry.  A 64 x D bf16 tile is stored row-major WITHOUT padding, because
// it is filled by direct global->LDS loads (global_load_lds_dwordx4: one instruction
// writes 64 lanes x 16 B = 1 KB of consecutive LDS).  Bank conflicts are avoided by
// permuting the 16-byte chunks inside each row: physical chunk = logical chunk ^ swz(row).
// The permutation is applied on the global side of the copy (each lane chooses which
// chunk of the row it fetches), so the copy stays fully coalesced.
template <int D>
struct Geo {
    static constexpr int ROW_BYTES = D * 2;                 // 256 | 128
    static constexpr int CPR = D / 8;                       // chunks per row: 16 | 8
    static constexpr int TILE_BYTES = KT * ROW_BYTES;       // 16384 | 8192
    static constexpr int ROWS_PER_LOAD = 1024 / ROW_BYTES;  // 4 | 8
    static constexpr int LOADS = TILE_BYTES / 1024;         // 16 | 8
    // K is read 16 bytes per lane, lanes = consecutive rows at one logical chunk:
    // 16 consecutive rows must land on 16 different chunks of the 256-byte bank line.
    static __device__ __forceinline__ int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
    // V is read by the transpose read as 4-row x 64-byte patches: consecutive rows must
    // land on different 64-byte groups of the bank line.
    static __device__ __forceinline__ int swz_v(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

// Issue the asynchronous copy of rows key0..key0+63 of `src` into an LDS tile.  Rows at or
// beyond kv_len are replaced by row kv_len-1 (finite data; their probabilities are exactly
// 0, and their scores are overwritten with -inf, so they never contribute).
template <int D, int NW, bool IS_V>
__device__ __forceinline__ void issue_tile(const Rows& src, int key0, int kv_len,
                                           char* lds, int wave, int lane)
{
    typedef Geo<D> G;
    constexpr int PER_WAVE = G::LOADS / NW;
    // global_load_lds_dwordx4: LDS address = M0 + 16 * lane.  Written as assembly so that the
    // copy pipeline is ordered only by the explicit vmcnt waits and barriers of the main loop
    // (the compiler would otherwise wait for all copies before LDS reads it cannot
    // disambiguate).  M0 has no other user in these kernels.
    if (key0 + KT <= kv_len) {
        // whole tile valid: scalar tile base + a per-lane byte offset that does not depend
        // on the tile (no vector arithmetic per copy)
        const char* tile = src.row(key0);                  // a tile never straddles the segments
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int ld = wave * PER_WAVE + i;             // wave-uniform
            const int row = ld * G::ROWS_PER_LOAD + lane / G::CPR;
            const int logical = (lane % G::CPR) ^ (IS_V ? G::swz_v(row) : G::swz_k(row));
            const unsigned off = (unsigned)row * src.row_bytes + (unsigned)logical * 16u;
            const unsigned dst = (unsigned)(size_t)LDS_PTR(char, lds + ld * 1024);
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(off), "s"(tile));
        }
    } else {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int ld = wave * PER_WAVE + i;
            const int row = ld * G::ROWS_PER_LOAD + lane / G::CPR;
            const int logical = (lane % G::CPR) ^ (IS_V ? G::swz_v(row) : G::swz_k(row));
            int grow = key0 + row;
            grow = grow < kv_len ? grow : kv_len - 1;
            const char* g = (key0 < src.n0 ? src.base0 : src.base1) + (size_t)grow * src.row_bytes + logical * 16;
            const unsigned dst = (unsigned)(size_t)LDS_PTR(char, lds + ld * 1024);
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(g));
        }
    }
}

struct SoftmaxState {
    float m;      // reference of the exponents, in units of scale * log2(e); same in both lane halves
    float l;      // this lane's partial sum of probabilities
};

// ---------------------------------------------------------------------------
// The matrix work of one tile as a stream of ITEMS.  An item is one MFMA together with
// the LDS read(s) of its A operand:
//   items 0 .. NPV-1     O^T += V^T P^T   item = (g, db): 16-key group g = 2 rb + t, 32-row
//                        block db of O^T; two transpose reads (keys 4h+r and 8+4h+r)
//   items NPV .. NI-1    S^T += K Q^T     item = (t, rb): k-step t, 32-key row block rb;
//                        one 128-bit read
// The reads of item i+PD are requested before the MFMA of item i is issued, so every
// operand has PD MFMAs (about 200 cycles) of lead.  The reads are inline assembly with
// their own s_waitcnt: issued through compiler builtins the transpose reads carry no
// alias scope and each of them would wait for ALL outstanding global->LDS copies.  LDS
// returns data in order, so "lgkmcnt(N)" = everything but the newest N requests has
// arrived; the counter has 4 bits, which bounds PD (at most 15 requests in flight).
// ---------------------------------------------------------------------------
template <int D, int PD_>
struct TileItems {
    static constexpr int DB = D / 32, KS = D / 16;
    static constexpr int NPV = 4 * DB;
    static constexpr int NQK = 2 * KS;
    static constexpr int NI = NPV + NQK;
    static constexpr int PD = PD_;             // how many items ahead the LDS reads are requested
    static constexpr int NBUF = PD + 1;
    static constexpr int reads(int i) { return i < NPV ? 2 : 1; }
    // LDS requests of the items after i that are in flight while item i is awaited
    static constexpr int newer(int i, int last)
    {
        int s = 0;
        for (int k = i + 1; k <= i + PD && k < last; ++k) s += reads(k);
        return s;
    }
};

template <int D, int PD>
struct TileCtx {
    unsigned vaddr[D / 32];                    // LDS byte address of this lane's transpose-read patch, per O^T block
    unsigned kbase;                            // LDS byte address of row n of the K tile
    unsigned kxor;                             // (h ^ swz_k(n)) << 4: chunk (2t+h) ^ swz == (2t) ^ (kxor >> 4)
    u32x2 lo[TileItems<D, PD>::NBUF];              // item i lives in slot i % NBUF
    u32x2 hi[TileItems<D, PD>::NBUF];
    u32x4 kf[TileItems<D, PD>::NBUF];
};

template <int D, int PD, int I>
__device__ __forceinline__ void item_request(TileCtx<D, PD>& c)
{
    typedef TileItems<D, PD> TI;
    constexpr int RB = Geo<D>::ROW_BYTES;
    constexpr int slot = I % TI::NBUF;
    if constexpr (I < TI::NPV) {
        constexpr int g = I / TI::DB, db = I % TI::DB;
        constexpr int row0 = (g >> 1) * 32 + (g & 1) * 16;
        asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                     : "=&v"(c.lo[slot]), "=&v"(c.hi[slot])
                     : "v"(c.vaddr[db]), "i"(row0 * RB), "i"((row0 + 8) * RB));
    } else {
        constexpr int t = (I - TI::NPV) / 2, rb = (I - TI::NPV) % 2;
        const unsigned ka = c.kbase + ((unsigned)(t << 5) ^ c.kxor);
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(c.kf[slot]) : "v"(ka), "i"(rb * 32 * RB));
    }
}

// Wait for item I; LAST = end of the run of items whose requests may be in flight.  The
// fragment is an in/out operand so that its use is ordered after the wait.
template <int D, int PD, int I, int LAST>
__device__ __forceinline__ void item_wait(TileCtx<D, PD>& c)
{
    typedef TileItems<D, PD> TI;
    constexpr int slot = I % TI::NBUF;
    constexpr int N = TI::newer(I, LAST);
    static_assert(N + TI::reads(I) <= 15, "lgkmcnt is a 4-bit counter");
    if constexpr (I < TI::NPV) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(c.lo[slot]), "+v"(c.hi[slot]) : "i"(N));
    else asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(c.kf[slot]) : "i"(N));
}

template <int D, int PD, int I>
__device__ __forceinline__ void item_mfma(const TileCtx<D, PD>& c, const bf16x8 (&pb)[4], const bf16x8 (&qf)[D / 16],
                                          f32x16 (&acc)[D / 32], f32x16 (&st)[2])
{
    typedef TileItems<D, PD> TI;
    constexpr int slot = I % TI::NBUF;
    if constexpr (I < TI::NPV) {
        constexpr int g = I / TI::DB, db = I % TI::DB;
        const u32x4 both = __builtin_shufflevector(c.lo[slot], c.hi[slot], 0, 1, 2, 3);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb[g], acc[db], 0, 0, 0);
    } else {
        constexpr int t = (I - TI::NPV) / 2, rb = (I - TI::NPV) % 2;
        f32x16 cin = st[rb];
        if constexpr (t == 0) {                            // first k-step starts from zero
#pragma unroll
            for (int j = 0; j < 16; ++j) cin[j] = 0.f;
        }
        st[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, c.kf[slot]), qf[t], cin, 0, 0, 0);
    }
}

// Request the first PD items of the run [FROM, TO).
template <int D, int PD, int FROM, int TO, int I = FROM>
__device__ __forceinline__ void items_prefetch(TileCtx<D, PD>& c)
{
    if constexpr (I < TO && I < FROM + PD) {
        item_request<D, PD, I>(c);
        items_prefetch<D, PD, FROM, TO, I + 1>(c);
    }
}

// Issue items [I, TO); items_prefetch<D, PD, I, TO> must have been called before.
template <int D, int PD, int I, int TO>
__device__ __forceinline__ void items_run(TileCtx<D, PD>& c, const bf16x8 (&pb)[4], const bf16x8 (&qf)[D / 16],
                                          f32x16 (&acc)[D / 32], f32x16 (&st)[2])
{
    if constexpr (I < TO) {
        if constexpr (I + PD < TO) item_request<D, PD, I + PD>(c);
        item_wait<D, PD, I, TO>(c);
        item_mfma<D, PD, I>(c, pb, qf, acc, st);
        items_run<D, PD, I + 1, TO>(c, pb, qf, acc, st);
    }
}

// Lane addresses for the tile held in (lds_k, lds_v).
//   K: lane (n, h) reads row n (+32 rb), logical chunk 2t + h of k-step t.
//   V: within a 16-lane group, lane j points at row j/4, columns 4 (j%4)..+3 of a 4 x 16
//      patch of the transpose read and lane i receives column i; lane half h covers rows +4h.
template <int D, int PD>
__device__ __forceinline__ void k_addresses(const char* lds_k, int n, int h, TileCtx<D, PD>& c)
{
    typedef Geo<D> G;
    c.kbase = (unsigned)(size_t)LDS_PTR(const char, lds_k) + n * G::ROW_BYTES;
    c.kxor = (unsigned)(h ^ G::swz_k(n)) << 4;
}

template <int D>
__device__ __forceinline__ void v_addresses(const char* lds_v, int h, int tr_row, int tr_col, unsigned (&vaddr)[D / 32])
{
    typedef Geo<D> G;
    const unsigned vbase = (unsigned)(size_t)LDS_PTR(const char, lds_v) + (4 * h + tr_row) * G::ROW_BYTES + tr_col * 2;
    const int vx = G::swz_v(tr_row) >> 2;                  // 64-byte group swizzle of this lane's rows
#pragma unroll
    for (int db = 0; db < D / 32; ++db) vaddr[db] = vbase + ((db ^ vx) << 6);
}

// Keys at or beyond kv_len -> -inf.  Register i of row block rb of S^T holds key
// key0 + 32 rb + 8 (i/4) + 4 h + i%4  of query n.
__device__ __forceinline__ void mask_tail(f32x16 (&st)[2], int key0, int kv_len, int h)
{
    if (key0 + KT > kv_len) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = key0 + 32 * rb + 8 * (i >> 2) + 4 * h + (i & 3);
                if (key >= kv_len) st[rb][i] = -INFINITY;
            }
    }
}

// Online softmax of one tile (one query per lane; the two lane halves hold disjoint keys).
// Probabilities are exp2(c * s - m) with c = scale * log2(e) and a per-query reference m (kept in
// exponent units); any m gives the same quotient acc / l, and bf16 and fp32 share their exponent
// range, so m need not be the running maximum.  Two ways to keep it in range:
//   lazy (D = 128): the tile's maximum is computed, and m moves up to it only when it lies more
//     than 8 above m (probabilities stay below 2^8);
//   optimistic (D = 64): no maximum on the common path.  m comes from the first tile and moves
//     only when a later tile's probabilities get large: their sum, which is needed anyway,
//     exceeds 2^60 (or is not a number).  Then the tile's maximum becomes the reference and the
//     tile's probabilities are computed again.
// When m moves, l and the accumulators are rescaled.  Leaves the probabilities as bf16 MFMA
// operands: pb[2 rb + t] = keys 16t + {4h..4h+3, 8+4h..8+4h+3} of row block rb.
template <int D>
__device__ __forceinline__ void softmax_tile(const f32x16 (&st)[2], f32x16 (&acc)[D / 32], SoftmaxState& st_,
                                             float c, bool first, bf16x8 (&pb)[4])
{
    constexpr int DB = D / 32;
    // The row sum adds up the probabilities two per instruction (v_dot2 of the bf16 pair against
    // 1.0): it is then over the probabilities as rounded to bf16, the weights the PV product applies.
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;
    auto probabilities = [&]() -> float {
        float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int rb = g >> 1, t = g & 1;
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                bf16x2 pr;
                pr[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(st[rb][8 * t + i], c, -st_.m));
                pr[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(st[rb][8 * t + i + 1], c, -st_.m));
                pb[g][i] = pr[0];
                pb[g][i + 1] = pr[1];
                if (i & 2) rs1 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs1, false);
                else rs0 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs0, false);
            }
        }
        return rs0 + rs1;
    };
    // the tile's largest exponent relative to m (on the first tile: the exponent itself)
    auto tile_max = [&]() -> float {
        float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(fmaxf(mx, st[0][i]), st[1][i]);
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        return first ? mx * c : __builtin_fmaf(mx, c, -st_.m);
    };
    float rs = 0.f, mx = 0.f;
    bool move = first;
    if constexpr (Optimistic<D>::value) {
        if (!first) {
            rs = probabilities();
            move = __builtin_amdgcn_ballot_w64(!(rs <= 0x1p60f)) != 0ull;     // also true for inf and NaN
        }
        if (move) mx = tile_max();
    } else {
        mx = tile_max();
        if (!first) move = __builtin_amdgcn_ballot_w64(mx > 8.0f) != 0ull;
    }
    if (move) {
        // mx is finite: every visited tile has a valid key.  On the first tile nothing has been
        // accumulated yet; later the reference only moves up.
        const float delta = first ? mx : fmaxf(mx, 0.f);
        const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta);
        st_.m = first ? mx : st_.m + delta;
        st_.l *= alpha;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[i][j] *= alpha;
    }
    if (!Optimistic<D>::value || move) rs = probabilities();
    st_.l += rs;
}

// Epilogue: O = acc / l as bf16.  Register 4j+r of block db holds d = 32 db + 8 j + 4 h + r
// of this lane's query; rows at or beyond kv_len and rows without any kept key become 0.
template <int D>
__device__ __forceinline__ void write_output(const Rows& O, const f32x16 (&acc)[D / 32], float l_part,
                                             int qrow, bool qvalid, int N, int h)
{
    float l_run = l_part;
    {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_run = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float inv = (qvalid && l_run > 0.f) ? 1.0f / l_run : 0.f;
    if (qrow < N) {
        __bf16* orow = (__bf16*)const_cast<char*>(O.row(qrow));
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x4 ov;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float x = acc[db][4 * j + r] * inv;
                    ov[r] = (__bf16)((inv != 0.f) ? x : 0.f);
                }
                *(bf16x4*)(orow + 32 * db + 8 * j + 4 * h) = ov;
            }
    }
}

// The same output through LDS, for a wavefront whose 32 queries are the rows row0 .. row0 + 31.
// A lane holds 8-byte pieces of ONE row, so storing from registers sends 32 short stretches of
// 32 different rows with every instruction (16 instructions, 512 memory requests per
// wavefront); written to `stage` first (row stride D*2 + 16 bytes: the 8-byte writes of the
// 32 rows spread over the banks) and read back 16 bytes per lane along the rows, a store
// instruction covers whole rows (8 or 4 instructions, a quarter of the requests).  `stage`
// is this wavefront's own region of (D*2 + 16) * 32 bytes; nobody else may still be reading it.
template <int D>
__device__ __forceinline__ void write_output_rows(const Rows& O, const f32x16 (&acc)[D / 32], float l_part,
                                                  int row0, bool qvalid, int N, int lane, char* stage)
{
    constexpr int RS = D * 2 + 16;
    const int n = lane & 31, h = lane >> 5;
    float l_run = l_part;
    {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_run = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float inv = (qvalid && l_run > 0.f) ? 1.0f / l_run : 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bf16x4 ov;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float x = acc[db][4 * j + r] * inv;
                ov[r] = (__bf16)((inv != 0.f) ? x : 0.f);
            }
            *(bf16x4*)(stage + n * RS + (32 * db + 8 * j + 4 * h) * 2) = ov;
        }
    constexpr int CH = D * 2 / 16;                // 16-byte chunks of a row
    constexpr int RPI = 64 / CH;                  // rows per store instruction
    const int rr = lane / CH, cc = lane % CH;
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
        const int r = i * RPI + rr;
        const u32x4 v = *(const u32x4*)(stage + r * RS + cc * 16);
        if (row0 + r < N) *(u32x4*)(const_cast<char*>(O.row(row0 + r)) + cc * 16) = v;
    }
}

// Q^T fragments (B operand of S^T = K Q^T): lane (n, h) holds Q[qrow][16t + 8h .. +8].
template <int D>
__device__ __forceinline__ void load_q(const Rows& Q, int qrow, bool qvalid, int h, bf16x8 (&qf)[D / 16])
{
    const __bf16* qr = (const __bf16*)Q.row(qvalid ? qrow : 0);
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (qvalid) raw = *(const u32x4*)(qr + 16 * t + 8 * h);
        qf[t] = __builtin_bit_cast(bf16x8, raw);
    }
}

// The same fragments requested by explicit assembly: the compiler then places no waits of
// its own for them (it cannot count the tile copies issued around them and would wait for
// everything); the caller waits with wait_vmcnt and then passes the fragments through
// q_arrived so that their uses stay behind that wait.  Rows that are not valid read row 0
// of the (sample, head) and are zeroed afterwards.
template <int D>
__device__ __forceinline__ void load_q_async(const Rows& Q, int qrow, bool qvalid, int h, u32x4 (&raw)[D / 16])
{
    const __bf16* src = (const __bf16*)Q.row(qvalid ? qrow : 0) + 8 * h;
#pragma unroll
    for (int t = 0; t < D / 16; ++t)
        asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(raw[t]) : "v"(src), "i"(32 * t));
}

template <int D>
__device__ __forceinline__ void q_arrived(u32x4 (&raw)[D / 16], bool qvalid, bf16x8 (&qf)[D / 16])
{
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        asm volatile("" : "+v"(raw[t]));
        const u32x4 zero = {0u, 0u, 0u, 0u};
        qf[t] = __builtin_bit_cast(bf16x8, qvalid ? raw[t] : zero);
    }
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in
// bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima)
template <int VM>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(VM >= 0 && VM < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (VM & 15) | ((VM >> 4) << 14));
}

// Values computed from registers only carry no ordering against a barrier; an empty volatile
// assembly statement that "modifies" them makes them complete before whatever follows it.
__device__ __forceinline__ void pin_in_phase(bf16x8 (&pb)[4], float& l)
{
    u32x4 a = __builtin_bit_cast(u32x4, pb[0]), b = __builtin_bit_cast(u32x4, pb[1]);
    u32x4 c = __builtin_bit_cast(u32x4, pb[2]), d = __builtin_bit_cast(u32x4, pb[3]);
    asm volatile("" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(l));
    pb[0] = __builtin_bit_cast(bf16x8, a); pb[1] = __builtin_bit_cast(bf16x8, b);
    pb[2] = __builtin_bit_cast(bf16x8, c); pb[3] = __builtin_bit_cast(bf16x8, d);
}

// Workgroup barrier that is also a boundary for the instruction scheduler: register-only
// work (the softmax arithmetic) must not drift from its phase into the neighbouring one.
__device__ __forceinline__ void phase_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------------------------
// Dense path: 256 queries per workgroup, 8 wavefronts in two groups of four (one wavefront
// of each group on every SIMD), 4 LDS stages, tile copies issued 3 tiles ahead.
//
// Per tile a wavefront alternates two phases separated by workgroup barriers:
//   B(j)  softmax of S_j                      -- VALU / transcendental work
//   A(j)  O^T += V_j^T P_j^T ; S_{j+1} = K_{j+1} Q^T   -- 32 MFMAs, LDS reads
// Group 1 enters the loop one barrier later than group 0, so between any two barriers one
// group is in a B phase while the other is in an A phase: the two wavefronts that share a
// SIMD are held in anti-phase and the matrix pipe of one overlaps the vector work of the
// other, instead of both running the same phase in lock-step after every barrier.
// Every barrier is executed by all wavefronts (group 0 makes up its missing one at the end).
// Copy bookkeeping (slot = interval between two barriers; group 0 runs A(j) in slot 2j+2,
// group 1 in slot 2j+3): tile j+3 is issued at the start of A(j) into the stage of tile j-1,
// which both groups have finished (group 1's A(j-1) is slot 2j+1); every wavefront waits for
// its share of tile j+1 before its first barrier of iteration j, i.e. before barrier 2j+2 at
// the latest, which precedes the first use of tile j+1 (group 0's A(j)).
// ---------------------------------------------------------------------------
// The body, for the 256 queries starting at row q0 of (sample, head) bh.  `lds` = 8 tile
// stages: K stages 0..3, V stages 4..7; tile t lives in stage t % 4.  All LDS traffic of the
// loop is explicit assembly, so the stages are plain runtime offsets into one array.
template <int D>
__device__ __forceinline__ void dense_item(const AttnParams& p, char* lds, int bh, int q0)
{
    typedef Geo<D> G;
    // How far ahead the LDS reads run (TileItems).  At D = 64 four wavefronts share a SIMD on 128
    // registers each; the depth is the largest at which this kernel keeps everything in registers
    // (a few values in scratch memory inside the loop cost 4-8 %); the other wavefronts cover the latency.
    constexpr int PD = D == 64 ? 2 : 6;
    typedef TileItems<D, PD> TI;
    constexpr int NW = 8, KS = D / 16, DB = D / 32;
    constexpr int LPT = 2 * G::LOADS / NW;        // copy instructions per wavefront per tile (K + V), all copying
    auto k_stage = [&](int t) -> char* { return lds + (t & 3) * G::TILE_BYTES; };
    auto v_stage = [&](int t) -> char* { return lds + (4 + (t & 3)) * G::TILE_BYTES; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = wave >> 2;
    const int n = lane & 31;                      // query within the wavefront / MFMA column
    const int h = lane >> 5;                      // lane half
    int kv_len = p.kv_len;
    if (p.kv_lens != nullptr) {                   // per-sample length, clamped to 0..N
        kv_len = ((const __attribute__((address_space(4))) int32_t*)p.kv_lens)[bh / p.H];
        kv_len = kv_len < 0 ? 0 : (kv_len > p.N ? p.N : kv_len);
    }

    const int smp = bh / p.H, head = bh % p.H;
    const Rows Q = rows_of(p.q, smp, head, p.n0), K = rows_of(p.k, smp, head, p.n0);
    const Rows V = rows_of(p.v, smp, head, p.n0), O = rows_of(p.o, smp, head, p.n0);

    const int T = (kv_len + KT - 1) / KT;
    if (T == 0) {                                 // a sample without valid tokens: its rows are zero
        f32x16 zero[DB];
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) zero[i][j] = 0.f;
        write_output<D>(O, zero, 0.f, q0 + (threadIdx.x >> 6) * 32 + (threadIdx.x & 31), false, p.N, (threadIdx.x & 63) >> 5);
        return;
    }

#pragma unroll
    for (int t = 0; t < 3; ++t) {
        if (t < T) {
            issue_tile<D, NW, false>(K, t * KT, kv_len, k_stage(t), wave, lane);
            issue_tile<D, NW, true>(V, t * KT, kv_len, v_stage(t), wave, lane);
        }
    }

    const int qrow = q0 + wave * 32 + n;          // this lane's query row
    const bool qvalid = qrow < kv_len;            // kv_len <= N
    bf16x8 qf[KS];
    load_q<D>(Q, qrow, qvalid, h, qf);

    f32x16 acc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    SoftmaxState sm;
    sm.m = -INFINITY;
    sm.l = 0.f;
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = ((lane & 3) << 2) + (((lane >> 4) & 1) << 4);

    // The Q fragments and the first tiles must have arrived before the loop (a wait for
    // the Q loads inside the loop would also wait for every tile copy in flight).
    wait_vmcnt<0>();
    __syncthreads();
    if (group == 1) __syncthreads();              // group 1 runs one barrier behind

    TileCtx<D, PD> ctx;
    bf16x8 pb[4];
    f32x16 st[2];
    k_addresses<D>(k_stage(0), n, h, ctx);
    items_prefetch<D, PD, TI::NPV, TI::NI>(ctx);
    items_run<D, PD, TI::NPV, TI::NI>(ctx, pb, qf, acc, st);   // S_0
    mask_tail(st, 0, kv_len, h);

    // Where the tile copies are issued.  At D = 128 the A phase is the critical one (measured per
    // phase: the copy instructions cost it ~270 cycles while the B phase had ~550 cycles of
    // slack), so the copies go to the start of the B phases, split between the groups: in its
    // B(j) group 0 copies K_{j+3} and group 1 copies V_{j+3}.  With b(n) the n-th barrier of the
    // loop, group 0 runs B(j) after b(2j+1) and A(j) after b(2j+2), group 1 one barrier later.
    //   K_{j+3} overwrites K_{j-1}, last read by S_{j-1} = K_{j-1} Q^T in A(j-2) (both groups are
    //   through it before b(2j)); K_t is first read in group 0's A(t-1) after b(2t): group 0
    //   waits for its K_{j+1} at the end of B(j), before b(2j+2).
    //   V_{j+3} overwrites V_{j-1}, last read in group 1's A(j-1) (done before b(2j+2)); V_t is
    //   first read in group 0's B(t) after b(2t+1), the barrier that ends group 1's B(t-1):
    //   group 1 waits for its V_{j+1} at the end of B(j).
    // At D = 64 the B phase is the longer one and every wavefront issues its share of tile j+3
    // at the start of A(j).
    constexpr bool COPY_IN_B = (D == 128);
    constexpr int LC = G::LOADS / 4;              // copy instructions per wavefront for one K or V tile by one group
    for (int j = 0; j < T; ++j) {
        if constexpr (!COPY_IN_B) {
            // my share of tile j+1 (outstanding: tiles j+1 and j+2, completing in order)
            if (j + 2 < T) wait_vmcnt<LPT>();
            else wait_vmcnt<0>();
        }
        phase_barrier();

        // ---- B(j)
        if constexpr (COPY_IN_B) {
            if (j + 3 < T) {
                if (group == 0) issue_tile<D, 4, false>(K, (j + 3) * KT, kv_len, k_stage(j + 3), wave, lane);
                else issue_tile<D, 4, true>(V, (j + 3) * KT, kv_len, v_stage(j + 3), wave - 4, lane);
            }
        }
        v_addresses<D>(v_stage(j), h, tr_row, tr_col, ctx.vaddr);
        softmax_tile<D>(st, acc, sm, p.c, j == 0, pb);
        pin_in_phase(pb, sm.l);
        items_prefetch<D, PD, 0, TI::NI>(ctx);        // first V_j^T fragments of A(j)
        if constexpr (COPY_IN_B) {
            // my group's tile j+1 has landed; its tiles j+2 and j+3 may still be on their way
            // (tiles 0..2 came with the prologue: in the loop tile t is issued in B(t-3))
            const int newer = ((j >= 1 && j + 2 < T) ? 1 : 0) + ((j + 3 < T) ? 1 : 0);
            if (newer == 2) wait_vmcnt<2 * LC>();
            else if (newer == 1) wait_vmcnt<LC>();
            else wait_vmcnt<0>();
        }
        phase_barrier();

        // ---- A(j): matrix work first in line at the SIMD's issue arbiter
        __builtin_amdgcn_s_setprio(3);
        if constexpr (!COPY_IN_B) {
            if (j + 3 < T) {
                issue_tile<D, NW, false>(K, (j + 3) * KT, kv_len, k_stage(j + 3), wave, lane);
                issue_tile<D, NW, true>(V, (j + 3) * KT, kv_len, v_stage(j + 3), wave, lane);
            }
        }
        // PV(j) then QK(j+1) as one stream.  For the last tile the QK half re-reads a
        // landed stage and its result is never used.
        k_addresses<D>(k_stage((j + 1 < T) ? j + 1 : j), n, h, ctx);
        items_run<D, PD, 0, TI::NI>(ctx, pb, qf, acc, st);
        mask_tail(st, (j + 1) * KT, kv_len, h);
        __builtin_amdgcn_s_setprio(0);
    }
    if (group == 0) __syncthreads();              // same number of barriers for every wavefront

    if constexpr (D == 128) {
        // row-wise through LDS (see write_output_rows); group 0 waits here until group 1 is
        // through its last matrix phase and the stages are free, which costs nothing: the
        // workgroup ends, and its CU takes the next one, when group 1 is done either way
        __syncthreads();
        write_output_rows<D>(O, acc, sm.l, q0 + wave * 32, qvalid, p.N, lane, lds + wave * ((D * 2 + 16) * 32));
    } else {
        write_output<D>(O, acc, sm.l, qrow, qvalid, p.N, h);
    }
}

// (D = 64: 64 KB of LDS and <= 128 VGPRs, so two workgroups share a CU: four wavefronts per
// SIMD hide more of the softmax phase, which is the longer one at D = 64.)
template <int D>
__global__ __launch_bounds__(512, (D == 64 ? 4 : 2)) void attn_dense_pp_kernel(const AttnParams p)
{
    __shared__ __attribute__((aligned(1024))) char lds[8 * Geo<D>::TILE_BYTES];
    // XCD-aware work mapping: the dispatcher deals consecutive workgroup ids round-robin
    // over the 8 XCDs, so give each XCD a contiguous run of items (query tiles of the same
    // head then share K/V in that XCD's L2).
    const int wg = blockIdx.x;
    const int item = (wg % XCDS) * p.chunk + wg / XCDS;
    if (item >= p.items) return;
    dense_item<D>(p, lds, item / p.nq, (item % p.nq) * DENSE_QT);
}

// ---------------------------------------------------------------------------
// Sparse path: one workgroup per (b, h, query-block); its kept-tile list is split between
// two wavefront groups (even tiles -> group 0, odd tiles -> group 1) that work on the SAME
// queries with separate softmax states and are merged through LDS at the end.  This halves
// the critical path of a long list (a text row keeps every tile) and gives the same
// anti-phase pairing of softmax and MFMA phases as the dense path.
//
// Time is divided into slots by workgroup barriers; tile t (64 keys) is handled as
//   slot t      S_t = K_t Q^T          (inside the A phase of tile t-2, or alone for t = 0, 1)
//   slot t+1    B(t): softmax of S_t, first V_t^T fragments requested
//   slot t+2    A(t): O^T += V_t^T P_t^T ; S_{t+2}
// by group t % 2, so in every slot one group is in an A phase and the other in a B phase.
// Every wavefront passes T+2 slot barriers (a group without work in a slot only does its
// share of the copies and waits).  Copies: in slot s every wavefront issues its share of
// K_{s+3} (4-stage ring) and V_{s+2} (5-stage ring) and, before the barrier that ends the
// slot, waits for its share of K_{s+1} and V_s (both issued in slot s-2; copies complete
// in order).  K_t is therefore complete at the start of slot t and V_t at the start of
// slot t+1; stage reuse: K_{t+4} is issued in slot t+1 > t, V_{t+5} in slot t+3 > t+2.
// All LDS traffic of the main loop is explicit assembly, so stages are plain runtime
// offsets into one array.
// ---------------------------------------------------------------------------
// (Waves per SIMD the register budget is set for: the 144 KB of stages at D = 128 leave room for
// one workgroup per CU, 72 KB at D = 64 for two.)
template <int D, int WPG>
__global__ __launch_bounds__(128 * WPG, (D == 64 ? (WPG == 4 ? 4 : 2) : 1)) void attn_sparse_pp_kernel(const AttnParams p)
{
    typedef Geo<D> G;
    constexpr int PD = 6;
    typedef TileItems<D, PD> TI;
    constexpr int NW = 2 * WPG, QT = 32 * WPG, KS = D / 16, DB = D / 32;
    constexpr int NSK = 4, NSV = 5;
    constexpr int LPT = 2 * G::LOADS / NW;        // copy instructions per wavefront per slot (K + V)
    static_assert(WPG * DB * 16 * 64 * 4 + WPG * 64 * 8 <= (NSK + NSV) * G::TILE_BYTES, "merge buffer fits the rings");

    __shared__ __attribute__((aligned(1024))) char lds[(NSK + NSV) * G::TILE_BYTES];

    typedef const __attribute__((address_space(4))) int32_t* cptr_t;
    const int wg = blockIdx.x;
    const int item = ((cptr_t)p.order)[(size_t)(wg % XCDS) * p.chunk + wg / XCDS];
    if (item < 0) return;
    const int bh = item / p.nq;
    const int qi = item % p.nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = wave / WPG;
    const int wq = wave % WPG;
    const int n = lane & 31;
    const int h = lane >> 5;
    int kv_len = p.kv_len;
    if (p.kv_lens != nullptr) {                   // per-sample length, clamped to 0..N
        kv_len = ((const __attribute__((address_space(4))) int32_t*)p.kv_lens)[bh / p.H];
        kv_len = kv_len < 0 ? 0 : (kv_len > p.N ? p.N : kv_len);
    }

    const int smp = bh / p.H, head = bh % p.H;
    const Rows Q = rows_of(p.q, smp, head, p.n0), K = rows_of(p.k, smp, head, p.n0);
    const Rows V = rows_of(p.v, smp, head, p.n0), O = rows_of(p.o, smp, head, p.n0);

    const int qrow = qi * QT + wq * 32 + n;       // groups share the queries
    const bool qvalid = qrow < kv_len;

    // 64-key tiles of this item: tile t -> first key
    const int ss = p.sub_shift;
    cptr_t list = (cptr_t)(p.index + (size_t)item * p.nb);
    int T;
    {
        const int n_blocks = ((cptr_t)p.counts)[item];
        T = n_blocks << ss;
        if (n_blocks > 0 && (((list[n_blocks - 1] + 1) << ss) - 1) * KT >= kv_len) T -= 1;
    }
    f32x16 acc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    if (T <= 0) {                                 // nothing kept: the rows are zero
        if (group == 0) write_output<D>(O, acc, 0.f, qrow, false, p.N, h);
        return;
    }
    auto key_of = [&](int t) -> int { return ((list[t >> ss] << ss) + (t & ((1 << ss) - 1))) * KT; };
    auto k_stage = [&](int t) -> char* { return lds + (t & (NSK - 1)) * G::TILE_BYTES; };
    // kq[i] = first key of tile s+i for the current slot s (0 past the end); kq4 is loaded a slot ahead
    int kq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) kq[i] = (i < T) ? key_of(i) : 0;
    int kq4 = (4 < T) ? key_of(4) : 0;
    int vst_issue = 2;                            // V stage of tile s+2
    int vst_use = 0;                              // V stage of this group's current tile

    // prologue: K_0..K_2, V_0, V_1
#pragma unroll
    for (int t = 0; t < 3; ++t)
        if (t < T) issue_tile<D, NW, false>(K, kq[t], kv_len, k_stage(t), wave, lane);
#pragma unroll
    for (int t = 0; t < 2; ++t)
        if (t < T) issue_tile<D, NW, true>(V, kq[t], kv_len, lds + (NSK + t) * G::TILE_BYTES, wave, lane);

    bf16x8 qf[KS];
    load_q<D>(Q, qrow, qvalid, h, qf);
    SoftmaxState sm;
    sm.m = -INFINITY;
    sm.l = 0.f;
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = ((lane & 3) << 2) + (((lane >> 4) & 1) << 4);
    wait_vmcnt<0>();
    __syncthreads();

    int s = 0;                                    // current slot = slot barriers passed
    auto slot_begin = [&]() {                     // my share of K_{s+3} and V_{s+2}
        if (s + 3 < T) issue_tile<D, NW, false>(K, kq[3], kv_len, k_stage(s + 3), wave, lane);
        if (s + 2 < T) issue_tile<D, NW, true>(V, kq[2], kv_len, lds + (NSK + vst_issue) * G::TILE_BYTES, wave, lane);
    };
    auto slot_end = [&]() {                       // K_{s+1} and V_s complete, then the barrier
        if (s + 3 < T) wait_vmcnt<2 * LPT>();
        else wait_vmcnt<0>();
        phase_barrier();
        ++s;
        kq[0] = kq[1]; kq[1] = kq[2]; kq[2] = kq[3]; kq[3] = kq4;
        kq4 = (s + 4 < T) ? key_of(s + 4) : 0;
        vst_issue = (vst_issue == NSV - 1) ? 0 : vst_issue + 1;
    };

    TileCtx<D, PD> ctx;
    bf16x8 pb[4];
    f32x16 st[2];

    if (group == 1) { slot_begin(); slot_end(); vst_use = 1; }   // group 1 runs one slot behind
    int t = group;                                // this group's tiles: group, group + 2, ...
    if (t < T) {                                  // slot t: S_t on its own
        slot_begin();
        k_addresses<D>(k_stage(t), n, h, ctx);
        items_prefetch<D, PD, TI::NPV, TI::NI>(ctx);
        items_run<D, PD, TI::NPV, TI::NI>(ctx, pb, qf, acc, st);
        mask_tail(st, kq[0], kv_len, h);
        slot_end();
    }
    while (t < T) {
        // ---- slot t+1: B(t)
        slot_begin();
        v_addresses<D>(lds + (NSK + vst_use) * G::TILE_BYTES, h, tr_row, tr_col, ctx.vaddr);
        softmax_tile<D>(st, acc, sm, p.c, t == group, pb);
        pin_in_phase(pb, sm.l);
        items_prefetch<D, PD, 0, TI::NI>(ctx);        // first V_t^T fragments of A(t)
        slot_end();
        // ---- slot t+2: A(t)
        __builtin_amdgcn_s_setprio(3);
        slot_begin();
        // (without a tile t+2 the QK half re-reads K_t, which is landed, and is dropped)
        k_addresses<D>(k_stage((t + 2 < T) ? t + 2 : t), n, h, ctx);
        items_run<D, PD, 0, TI::NI>(ctx, pb, qf, acc, st);
        mask_tail(st, kq[0], kv_len, h);
        __builtin_amdgcn_s_setprio(0);
        slot_end();
        t += 2;
        vst_use += 2;
        if (vst_use >= NSV) vst_use -= NSV;
    }
    while (s < T + 2) { slot_begin(); slot_end(); }

    // ---- merge the two groups (same queries, same register layout) through LDS
    u32x4* mbuf = (u32x4*)lds;                                    // [wq][DB*4][64 lanes]
    float* mlbuf = (float*)(lds + WPG * DB * 4 * 64 * 16);        // [wq][64 lanes][m, l]
    if (group == 1) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32x4 v;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = __float_as_uint(acc[db][4 * j + r]);
                mbuf[(wq * DB * 4 + db * 4 + j) * 64 + lane] = v;
            }
        mlbuf[(wq * 64 + lane) * 2] = sm.m;
        mlbuf[(wq * 64 + lane) * 2 + 1] = sm.l;
    }
    __syncthreads();
    if (group == 0) {
        const float m1 = mlbuf[(wq * 64 + lane) * 2];
        const float l1 = mlbuf[(wq * 64 + lane) * 2 + 1];
        const float m = fmaxf(sm.m, m1);                          // group 0 always has tile 0: finite
        const float a0 = __builtin_amdgcn_exp2f(sm.m - m);
        const float a1 = __builtin_amdgcn_exp2f(m1 - m);         // 0 if group 1 had no tile
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4 v = mbuf[(wq * DB * 4 + db * 4 + j) * 64 + lane];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[db][4 * j + r] = acc[db][4 * j + r] * a0 + __uint_as_float(v[r]) * a1;
            }
        write_output<D>(O, acc, sm.l * a0 + l1 * a1, qrow, qvalid, p.N, h);
    }
}

// Partial result of one piece of a split item: the fp32 accumulators in register order
// ([wavefront][register pair][lane], 8 bytes each), then (m, l) per lane.
template <int D>
struct PartialSlot {
    static constexpr size_t ML_OFF = (size_t)4 * (D / 32) * 4 * 64 * 16;      // 64 KB | 32 KB
    static constexpr size_t BYTES = ML_OFF + 4 * 64 * 2 * 4;                  // + 2 KB
};

// ---------------------------------------------------------------------------
// Sparse path, 128-token mask tiles: one workgroup of FOUR wavefronts per (b, h, query-block)
// walks the whole kept-tile list of its item; 64 KB of LDS (32 KB at D = 64) and one
// wavefront per SIMD, so two such workgroups (four at D = 64) share a CU.  The fixed cost
// of an item (list lookup, first copies, Q load, output) is then hidden behind the tile loop
// of the neighbour instead of leaving the CU idle, which is what matters when the lists are
// short; the two wavefronts on a SIMD belong to different items and fall into the same
// softmax-against-MFMA overlap as the two groups of the dense kernel.
//
// Per tile j two slots separated by workgroup barriers:
//   B(j)  softmax of S_j; copies of V_{j+1} and K_{j+2} issued; first V_j^T fragments requested
//   A(j)  O^T += V_j^T P_j^T ; S_{j+1} = K_{j+1} Q^T
// LDS: K stages 0,1 and V stages 2,3; tile t in stage t % 2.  When B(j) starts every
// wavefront has finished A(j-1), the last reader of V_{j-1} and K_j, whose stages take
// V_{j+1} and K_{j+2}.  Copies complete in issue order, so "all but the newest n" is a wait
// for everything older: K_{j+1} (issued in B(j-1)) is awaited at the end of B(j) with this
// slot's copies still in flight, V_{j+1} at the end of A(j) with K_{j+2} still in flight.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, (D == 64 ? 4 : 2)) void attn_sparse_sg_kernel(const AttnParams p)
{
    typedef Geo<D> G;
    constexpr int PD = D == 64 ? 3 : 6;           // see dense_item
    typedef TileItems<D, PD> TI;
    constexpr int NW = 4, QT = 128, KS = D / 16, DB = D / 32;
    constexpr int LPT = G::LOADS / NW;            // copy instructions per wavefront per tile (K or V)

    __shared__ __attribute__((aligned(1024))) char lds[4 * G::TILE_BYTES];

    typedef const __attribute__((address_space(4))) int32_t* cptr_t;
    const int wg = blockIdx.x;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(4))) i32x4* rptr_t;
    static_assert(sizeof(PlanRec) == sizeof(i32x4), "one record = one 16-byte scalar load");
    const i32x4 raw = ((rptr_t)p.order)[(size_t)(wg % XCDS) * p.chunk + wg / XCDS];
    const PlanRec rec = {raw[0], raw[1], raw[2], raw[3]};
    const int item = rec.item;
    if (item < 0) return;
    const int bh = item / p.nq;
    const int qi = item % p.nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31;
    const int h = lane >> 5;
    int kv_len = p.kv_len;
    if (p.kv_lens != nullptr) {                   // per-sample length, clamped to 0..N
        kv_len = ((const __attribute__((address_space(4))) int32_t*)p.kv_lens)[bh / p.H];
        kv_len = kv_len < 0 ? 0 : (kv_len > p.N ? p.N : kv_len);
    }

    const int smp = bh / p.H, head = bh % p.H;
    const Rows Q = rows_of(p.q, smp, head, p.n0), K = rows_of(p.k, smp, head, p.n0);
    const Rows V = rows_of(p.v, smp, head, p.n0), O = rows_of(p.o, smp, head, p.n0);

    const int qrow = qi * QT + wave * 32 + n;
    const bool qvalid = qrow < kv_len;

    // 64-key tiles of this piece (two per kept 128-key block; the item's last block may have one)
    cptr_t list = (cptr_t)(p.index + (size_t)item * p.nb + rec.blk0);
    int T = rec.nblk * 2;
    if (rec.nblk > 0 && (list[rec.nblk - 1] * 2 + 1) * KT >= kv_len) T -= 1;
    f32x16 acc[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    if (T <= 0) {                                 // nothing kept: the rows are zero
        write_output<D>(O, acc, 0.f, qrow, false, p.N, h);
        return;
    }
    auto key_of = [&](int t) -> int { return (list[t >> 1] * 2 + (t & 1)) * KT; };
    auto k_stage = [&](int t) -> char* { return lds + (t & 1) * G::TILE_BYTES; };
    auto v_stage = [&](int t) -> char* { return lds + (2 + (t & 1)) * G::TILE_BYTES; };
    // first keys of tiles j+1, j+2, j+3 (0 past the end), fetched ahead of their use
    const int key0 = key_of(0);
    int kn1 = (1 < T) ? key_of(1) : 0;
    int kn2 = (2 < T) ? key_of(2) : 0;
    int kn3 = (3 < T) ? key_of(3) : 0;

    // Q and K_0 first: S_0 needs only these; V_0 and K_1 land while it is computed.
    u32x4 qraw[KS];
    load_q_async<D>(Q, qrow, qvalid, h, qraw);
    issue_tile<D, NW, false>(K, key0, kv_len, k_stage(0), wave, lane);
    issue_tile<D, NW, true>(V, key0, kv_len, v_stage(0), wave, lane);
    if (1 < T) issue_tile<D, NW, false>(K, kn1, kv_len, k_stage(1), wave, lane);

    SoftmaxState sm;
    sm.m = -INFINITY;
    sm.l = 0.f;
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = ((lane & 3) << 2) + (((lane >> 4) & 1) << 4);
    if (1 < T) wait_vmcnt<2 * LPT>();
    else wait_vmcnt<LPT>();
    bf16x8 qf[KS];
    q_arrived<D>(qraw, qvalid, qf);
    __syncthreads();

    TileCtx<D, PD> ctx;
    bf16x8 pb[4];
    f32x16 st[2];
    k_addresses<D>(k_stage(0), n, h, ctx);
    items_prefetch<D, PD, TI::NPV, TI::NI>(ctx);
    items_run<D, PD, TI::NPV, TI::NI>(ctx, pb, qf, acc, st);   // S_0
    mask_tail(st, key0, kv_len, h);
    if (1 < T) wait_vmcnt<LPT>();                 // V_0 landed (K_1 may still be on its way)
    else wait_vmcnt<0>();

    for (int j = 0; j < T; ++j) {
        phase_barrier();                          // A(j-1) (or S_0) finished by every wavefront; V_j landed

        // ---- B(j)
        if (j + 1 < T) issue_tile<D, NW, true>(V, kn1, kv_len, v_stage(j + 1), wave, lane);
        if (j + 2 < T) issue_tile<D, NW, false>(K, kn2, kv_len, k_stage(j), wave, lane);
        v_addresses<D>(v_stage(j), h, tr_row, tr_col, ctx.vaddr);
        softmax_tile<D>(st, acc, sm, p.c, j == 0, pb);
        pin_in_phase(pb, sm.l);
        items_prefetch<D, PD, 0, TI::NI>(ctx);        // first V_j^T fragments of A(j)
        if (j + 2 < T) wait_vmcnt<2 * LPT>();     // K_{j+1} landed
        else if (j + 1 < T) wait_vmcnt<LPT>();
        else wait_vmcnt<0>();
        phase_barrier();

        // ---- A(j): PV(j) then QK(j+1) as one stream (without a tile j+1 the QK half re-reads
        // K_j, which is still in its stage, and its result is never used)
        __builtin_amdgcn_s_setprio(3);
        k_addresses<D>(k_stage((j + 1 < T) ? j + 1 : j), n, h, ctx);
        items_run<D, PD, 0, TI::NI>(ctx, pb, qf, acc, st);
        mask_tail(st, kn1, kv_len, h);
        __builtin_amdgcn_s_setprio(0);
        if (j + 2 < T) wait_vmcnt<LPT>();         // V_{j+1} landed
        else wait_vmcnt<0>();
        kn1 = kn2; kn2 = kn3;
        kn3 = (j + 4 < T) ? key_of(j + 4) : 0;
    }

    // At D = 128 the output goes out row-wise through LDS (-1.5 % on a sparse call); at D = 64,
    // with four workgroups on the CU and rows half as long, that was 2-3 % slower than direct.
    char* out_stage = lds + wave * ((D * 2 + 16) * 32);
    if (rec.w < 0) {                              // the whole item
        if constexpr (D == 128) {
            __syncthreads();                      // every wavefront has read its last tiles
            write_output_rows<D>(O, acc, sm.l, qi * QT + wave * 32, qvalid, p.N, lane, out_stage);
        } else {
            write_output<D>(O, acc, sm.l, qrow, qvalid, p.N, h);
        }
        return;
    }

    // ---- a piece of a split item: leave (acc, m, l) in this piece's slot; the piece that
    // finishes last adds all of them up, in piece order (so the sum does not depend on which
    // one that is).  A piece has at least one valid key per query, so every m is finite.
    // The slots are written and read with device-scope relaxed atomic accesses, each of which
    // is coherent across the chip by itself, instead of plain accesses between device-scope
    // fences: a release fence would write back every dirty line of the XCD's L2.  Order: a
    // wavefront's stores are acknowledged (vmcnt 0) before the barrier after which one thread
    // counts the piece in; the last piece reads only after it has seen the full count.
    typedef unsigned long long u64;
    constexpr size_t SLOT_BYTES = PartialSlot<D>::BYTES;
    constexpr int PAIRS = DB * 8;                 // 64-bit words of accumulators per lane
    const int P = (rec.w & 15) + 1;
    const int piece = (rec.w >> 4) & 15;
    const int slot0 = rec.w >> 8;
    auto slot_acc = [&](int k) -> u64* { return (u64*)(p.partial + (size_t)(slot0 + k) * SLOT_BYTES) + (size_t)wave * PAIRS * 64 + lane; };
    auto slot_ml = [&](int k) -> u64* { return (u64*)(p.partial + (size_t)(slot0 + k) * SLOT_BYTES + PartialSlot<D>::ML_OFF) + wave * 64 + lane; };
    {
        u64* pacc = slot_acc(piece);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u64 v = (u64)__float_as_uint(acc[db][2 * j]) | ((u64)__float_as_uint(acc[db][2 * j + 1]) << 32);
                __hip_atomic_store(pacc + (db * 8 + j) * 64, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        const u64 ml = (u64)__float_as_uint(sm.m) | ((u64)__float_as_uint(sm.l) << 32);
        __hip_atomic_store(slot_ml(piece), ml, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __shared__ int arrived_before;
    wait_vmcnt<0>();
    __syncthreads();
    if (tid == 0) arrived_before = __hip_atomic_fetch_add(&p.arrived[slot0], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (arrived_before != P - 1) return;

    float m = -INFINITY;
    for (int k = 0; k < P; ++k) {
        const u64 ml = __hip_atomic_load(slot_ml(k), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        m = fmaxf(m, __uint_as_float((unsigned)ml));
    }
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    float l = 0.f;
    for (int k = 0; k < P; ++k) {
        const u64 ml = __hip_atomic_load(slot_ml(k), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float a = __builtin_amdgcn_exp2f(__uint_as_float((unsigned)ml) - m);
        l += __uint_as_float((unsigned)(ml >> 32)) * a;
        const u64* pacc = slot_acc(k);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const u64 v = __hip_atomic_load(pacc + (db * 8 + j) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                acc[db][2 * j] += __uint_as_float((unsigned)v) * a;
                acc[db][2 * j + 1] += __uint_as_float((unsigned)(v >> 32)) * a;
            }
    }
    if constexpr (D == 128) write_output_rows<D>(O, acc, l, qi * QT + wave * 32, qvalid, p.N, lane, out_stage);   // after the barriers above
    else write_output<D>(O, acc, l, qrow, qvalid, p.N, h);
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct WorkspaceLayout {
    size_t counts_off, order_off, index_off, arrived_off, partial_off, total;
    int chunk;    // plan entries per XCD
    int pmax;     // partial-result slots per XCD (128-token tiles)
};

// items of one XCD: (b,h) pairs are dealt round-robin over the XCDs
inline int plan_items(int B, int H, int nb) { return ((B * H + XCDS - 1) / XCDS) * nb; }

// 64-token tiles:  counts | order int32[8*chunk]   | index
// 128-token tiles: counts | records PlanRec[8*chunk] | index | arrived int32[8*pmax] | partial slots [8*pmax]
// `slots` < 0: as many partial-result slots per XCD as the split rule can ever use
// (min(256, items)); otherwise that many at most (fewer slots = fewer items cut).
inline WorkspaceLayout workspace_layout(int B, int H, int nb, int D, int block, int slots = -1)
{
    const size_t rows = (size_t)B * H * nb;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    WorkspaceLayout w;
    const int items = plan_items(B, H, nb);
    w.counts_off = 0;
    w.order_off = up(rows * 4);
    if (block == 128) {
        w.pmax = SPLIT_SLOTS < items ? SPLIT_SLOTS : items;
        if (slots >= 0 && slots < w.pmax) w.pmax = slots;
        w.chunk = items + w.pmax;
        w.index_off = w.order_off + up((size_t)XCDS * w.chunk * sizeof(PlanRec));
        w.arrived_off = w.index_off + up(rows * (size_t)nb * 4);
        w.partial_off = w.arrived_off + up((size_t)XCDS * w.pmax * 4);
        const size_t slot = D == 64 ? PartialSlot<64>::BYTES : PartialSlot<128>::BYTES;
        w.total = w.partial_off + up((size_t)XCDS * w.pmax * slot);
    } else {
        w.pmax = 0;
        w.chunk = items;
        w.index_off = w.order_off + up((size_t)XCDS * w.chunk * 4);
        w.arrived_off = w.partial_off = w.total = w.index_off + up(rows * (size_t)nb * 4);
    }
    return w;
}

int check_common(const void* q, const void* k, const void* v, const void* o,
                 int B, int H, int N, int D, int kv_len)
{
    if (!q || !k || !v || !o) return RAPID_ERR_NULL;
    if (B <= 0 || H <= 0 || N <= 0) return RAPID_ERR_SHAPE;
    if (kv_len < 1 || kv_len > N) return RAPID_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL / 4096) return RAPID_ERR_SHAPE;
    if (N > (1 << 22)) return RAPID_ERR_SHAPE;
    if (D != 64 && D != 128) return RAPID_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return RAPID_ERR_ALIGN;
    // O is written while other workgroups still read Q, K and V: it must not share a byte with them
    const uintptr_t bytes = (uintptr_t)B * H * N * D * 2, ob = (uintptr_t)o;
    for (const void* in : {q, k, v}) {
        const uintptr_t ib = (uintptr_t)in;
        if (ob < ib + bytes && ib < ob + bytes) return RAPID_ERR_ALIAS;
    }
    return RAPID_OK;
}

// One validated call: tensors as segment views, sizes, lengths.
struct Problem {
    SegTensor q, k, v, o;
    int n0;
    int B, H, N, D;
    int kv_len;
    const int32_t* kv_lens;
    float scale;
};

SegTensor contiguous_bhnd(const void* ptr, int H, int N, int D)
{
    SegTensor t;
    t.seg0 = (const __bf16*)ptr; t.seg1 = nullptr;
    t.sb0 = (long long)H * N * D; t.sb1 = 0;
    t.sh = (long long)N * D; t.sn = D;
    return t;
}

void fill_common(AttnParams& p, const Problem& pr)
{
    p.q = pr.q; p.k = pr.k; p.v = pr.v; p.o = pr.o;
    p.kv_lens = pr.kv_lens;
    p.n0 = pr.n0;
    p.H = pr.H; p.N = pr.N; p.kv_len = pr.kv_len;
    p.c = pr.scale * LOG2E;
}

int run_dense(const Problem& pr, void* stream)
{
    AttnParams p{};
    fill_common(p, pr);
    p.counts = nullptr; p.order = nullptr; p.index = nullptr;
    p.nq = (pr.N + DENSE_QT - 1) / DENSE_QT;
    const long long items = (long long)pr.B * pr.H * p.nq;
    if (items > 0x7fffffffLL / 2) return RAPID_ERR_SHAPE;
    p.items = (int)items;
    p.chunk = (p.items + XCDS - 1) / XCDS;
    p.block = 0; p.nb = 0; p.sub_shift = 0;
    hipStream_t s = (hipStream_t)stream;
    const int grid = p.chunk * XCDS;
    if (pr.D == 64) hipLaunchKernelGGL((attn_dense_pp_kernel<64>), dim3(grid), dim3(512), 0, s, p);
    else hipLaunchKernelGGL((attn_dense_pp_kernel<128>), dim3(grid), dim3(512), 0, s, p);
    return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
}

// nb = ceil(N / block): the last mask block may be ragged (it then ends at N)
// `mask` null: counts and lists are already in the workspace (written by the selection kernels)
int run_sparse(const Problem& pr, int block, const unsigned char* mask, void* workspace, size_t workspace_bytes,
               void* stream, int slots = -1)
{
    const int B = pr.B, H = pr.H, N = pr.N, D = pr.D;
    const int nb = (N + block - 1) / block;
    const long long rows = (long long)B * H * nb;
    if (rows > 0x7fffffffLL / 16) return RAPID_ERR_SHAPE;
    const WorkspaceLayout w = workspace_layout(B, H, nb, D, block, slots);
    if (!workspace || workspace_bytes < w.total) return RAPID_ERR_WORKSPACE;
    if (!aligned16(workspace)) return RAPID_ERR_ALIGN;

    char* ws = (char*)workspace;
    int32_t* counts = (int32_t*)(ws + w.counts_off);
    int32_t* order = (int32_t*)(ws + w.order_off);
    int32_t* index = (int32_t*)(ws + w.index_off);
    hipStream_t s = (hipStream_t)stream;

    const int xcd_items = plan_items(B, H, nb);
    if (mask != nullptr && block == 128 && nb <= SMALL_NB && xcd_items <= SMALL_ITEMS && xcd_items * nb <= SMALL_BYTES) {
        hipLaunchKernelGGL(plan_small_kernel, dim3(XCDS), dim3(1024), 0, s, mask, pr.kv_lens, pr.kv_len, N, block,
                           H, B * H, nb, w.chunk, w.pmax, D, counts, index, (PlanRec*)order,
                           (int32_t*)(ws + w.arrived_off));
    } else {
        if (mask != nullptr) {
            hipLaunchKernelGGL(compact_mask_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                               mask, (int)rows, nb, block, pr.kv_len, pr.kv_lens, H * nb, N, counts, index);
            if (hipGetLastError() != hipSuccess) return RAPID_ERR_DEVICE;
        }
        if (block == 128)
            hipLaunchKernelGGL(plan_split_kernel, dim3(XCDS), dim3(1024), 0, s, counts, B * H, nb, w.chunk,
                               w.pmax, D, (PlanRec*)order, (int32_t*)(ws + w.arrived_off));
        else
            hipLaunchKernelGGL(plan_kernel, dim3(XCDS), dim3(1024), 0, s, counts, B * H, nb, w.chunk, order);
    }
    if (hipGetLastError() != hipSuccess) return RAPID_ERR_DEVICE;

    AttnParams p{};
    fill_common(p, pr);
    p.counts = counts; p.order = order; p.index = index;
    p.arrived = (int32_t*)(ws + w.arrived_off);
    p.partial = ws + w.partial_off;
    p.nq = nb;
    p.items = (int)rows;
    p.chunk = w.chunk;
    p.block = block; p.nb = nb; p.sub_shift = block == 128 ? 1 : 0;
    const dim3 grid((unsigned)w.chunk * XCDS);
    if (block == 128) {
        if (D == 64) hipLaunchKernelGGL((attn_sparse_sg_kernel<64>), grid, dim3(256), 0, s, p);
        else hipLaunchKernelGGL((attn_sparse_sg_kernel<128>), grid, dim3(256), 0, s, p);
    } else {
        if (D == 64) hipLaunchKernelGGL((attn_sparse_pp_kernel<64, 2>), grid, dim3(256), 0, s, p);
        else hipLaunchKernelGGL((attn_sparse_pp_kernel<128, 2>), grid, dim3(256), 0, s, p);
    }
    return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
}

Problem contiguous_problem(const void* q, const void* k, const void* v, void* o, int B, int H, int N, int D,
                           int kv_len, float scale)
{
    Problem pr;
    pr.q = contiguous_bhnd(q, H, N, D); pr.k = contiguous_bhnd(k, H, N, D);
    pr.v = contiguous_bhnd(v, H, N, D); pr.o = contiguous_bhnd(o, H, N, D);
    pr.n0 = N;
    pr.B = B; pr.H = H; pr.N = N; pr.D = D;
    pr.kv_len = kv_len; pr.kv_lens = nullptr;
    pr.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    return pr;
}

// The segments of rapid_attn_joint as a validated Problem.
int joint_problem(const rapid_attn_segment* segments, int n_segments, int B, int H, int D, int block, bool sparse,
                  int kv_len, const int* kv_lens, float scale, Problem& pr)
{
    if (!segments) return RAPID_ERR_NULL;
    if (n_segments != 1 && n_segments != 2) return RAPID_ERR_SHAPE;
    if (B <= 0 || H <= 0) return RAPID_ERR_SHAPE;
    if (D != 64 && D != 128) return RAPID_ERR_UNSUPPORTED;
    if (sparse && block != 64 && block != 128) return RAPID_ERR_UNSUPPORTED;
    long long N = 0;
    rapid_attn_segment seg[2];                    // strides of size-1 dimensions are not looked at
    for (int i = 0; i < n_segments; ++i) seg[i] = rapid_internal::normalised_segment(segments[i], B, H, i == 1 ? &seg[0] : nullptr);
    segments = seg;
    for (int i = 0; i < n_segments; ++i) {
        const rapid_attn_segment& g = segments[i];
        if (!g.q || !g.k || !g.v || !g.o) return RAPID_ERR_NULL;
        if (g.n <= 0) return RAPID_ERR_SHAPE;
        if (!aligned16(g.q) || !aligned16(g.k) || !aligned16(g.v) || !aligned16(g.o)) return RAPID_ERR_ALIGN;
        const long long st[6] = {g.in_stride_b, g.in_stride_h, g.in_stride_n, g.out_stride_b, g.out_stride_h, g.out_stride_n};
        for (int j = 0; j < 6; ++j) {
            if (st[j] < 0 || st[j] > (1LL << 40)) return RAPID_ERR_SHAPE;
            if (st[j] % 8 != 0) return RAPID_ERR_ALIGN;            // every row starts on 16 bytes
        }
        // rows are D contiguous elements; byte offsets inside a 64-row tile stay below 2^31
        if (g.in_stride_n < D || g.out_stride_n < D || g.in_stride_n > (1LL << 23) || g.out_stride_n > (1LL << 23)) return RAPID_ERR_SHAPE;
        N += g.n;
    }
    if (N > (1 << 22)) return RAPID_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL / 4096) return RAPID_ERR_SHAPE;
    if (n_segments == 2) {
        // tiles of 64 keys and mask blocks of 128 queries must not straddle the two tensors
        if (segments[0].n % 128 != 0) return RAPID_ERR_SHAPE;
        if (segments[0].in_stride_h != segments[1].in_stride_h || segments[0].in_stride_n != segments[1].in_stride_n ||
            segments[0].out_stride_h != segments[1].out_stride_h || segments[0].out_stride_n != segments[1].out_stride_n)
            return RAPID_ERR_SHAPE;
    }
    if (kv_len == 0) kv_len = (int)N;
    if (kv_len < 1 || kv_len > N) return RAPID_ERR_SHAPE;

    auto view = [&](int which) {
        SegTensor t;
        const rapid_attn_segment& a = segments[0];
        const rapid_attn_segment* b2 = n_segments == 2 ? &segments[1] : nullptr;
        const void* p0 = which == 0 ? a.q : which == 1 ? a.k : which == 2 ? a.v : (const void*)a.o;
        const void* p1 = !b2 ? nullptr : which == 0 ? b2->q : which == 1 ? b2->k : which == 2 ? b2->v : (const void*)b2->o;
        t.seg0 = (const __bf16*)p0; t.seg1 = (const __bf16*)p1;
        const bool out = which == 3;
        t.sb0 = out ? a.out_stride_b : a.in_stride_b;
        t.sb1 = !b2 ? 0 : (out ? b2->out_stride_b : b2->in_stride_b);
        t.sh = out ? a.out_stride_h : a.in_stride_h;
        t.sn = out ? a.out_stride_n : a.in_stride_n;
        return t;
    };
    pr.q = view(0); pr.k = view(1); pr.v = view(2); pr.o = view(3);
    pr.n0 = n_segments == 2 ? segments[0].n : (int)N;
    pr.B = B; pr.H = H; pr.N = (int)N; pr.D = D;
    pr.kv_len = kv_len; pr.kv_lens = kv_lens;
    pr.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    return RAPID_OK;
}

// The scratch of rapid_attn_block_sparse_static: one array per GPU, part of the loaded code
// object, alive until the process ends.  In host code `scratch` is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device, with that device
// current, and kept.
constexpr int MAX_DEVICES = 64;
std::atomic<void*> scratch_ptr[MAX_DEVICES];

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return RAPID_ERR_DEVICE;
    void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return RAPID_ERR_DEVICE;
        scratch_ptr[dev].store(ptr, std::memory_order_release);   // two threads racing store the same address
    }
    *out = ptr;
    return RAPID_OK;
}

}  // namespace

extern "C" {

int rapid_attn_dense(const void* q, const void* k, const void* v, void* o,
                     int B, int H, int N, int D, int kv_len, float scale,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    (void)workspace; (void)workspace_bytes;
    const int rc = check_common(q, k, v, o, B, H, N, D, kv_len);
    if (rc != RAPID_OK) return rc;
    return run_dense(contiguous_problem(q, k, v, o, B, H, N, D, kv_len, scale), stream);
}

int rapid_attn_block_sparse(const void* q, const void* k, const void* v, void* o,
                            int B, int H, int N, int D, int block,
                            const unsigned char* mask, int kv_len, float scale,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    if (!mask) return RAPID_ERR_NULL;
    const int rc = check_common(q, k, v, o, B, H, N, D, kv_len);
    if (rc != RAPID_OK) return rc;
    if (block != 64 && block != 128) return RAPID_ERR_UNSUPPORTED;
    if (N % block != 0) return RAPID_ERR_SHAPE;
    return run_sparse(contiguous_problem(q, k, v, o, B, H, N, D, kv_len, scale), block, mask, workspace,
                      workspace_bytes, stream);
}

int rapid_attn_joint(const rapid_attn_segment* segments, int n_segments, int B, int H, int D,
                     int block, const unsigned char* mask, int kv_len, const int* kv_lens, float scale,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    Problem pr;
    const int rc = joint_problem(segments, n_segments, B, H, D, block, mask != nullptr, kv_len, kv_lens, scale, pr);
    if (rc != RAPID_OK) return rc;
    if (!mask) return run_dense(pr, stream);
    return run_sparse(pr, block, mask, workspace, workspace_bytes, stream);
}

// Selection and attention in one call: the selection kernels write counts and kept lists where the
// attention's own compaction would have put them; the block means go behind the attention workspace.
int rapid_attn_joint_select(const rapid_attn_segment* segments, int n_segments, int B, int H, int D, int block,
                            int kv_len, const int* kv_lens, int text_start, float tau, float scale,
                            unsigned char* mask_out, void* workspace, size_t workspace_bytes, void* stream)
{
    Problem pr;
    const int rc = joint_problem(segments, n_segments, B, H, D, block, true, kv_len, kv_lens, scale, pr);
    if (rc != RAPID_OK) return rc;
    const int nb = (pr.N + block - 1) / block;
    if ((long long)B * H * nb > 0x7fffffffLL / 16) return RAPID_ERR_SHAPE;
    const WorkspaceLayout w = workspace_layout(B, H, nb, D, block);
    const size_t means = rapid_internal::select_scratch_bytes(B, H, nb, D);
    if (!workspace || workspace_bytes < w.total + means) return RAPID_ERR_WORKSPACE;
    if (!aligned16(workspace)) return RAPID_ERR_ALIGN;
    char* ws = (char*)workspace;
    const int rs = rapid_internal::select_to_lists(segments, n_segments, B, H, D, block, kv_len, kv_lens, text_start, tau,
                                                   scale, mask_out, (int32_t*)(ws + w.counts_off),
                                                   (int32_t*)(ws + w.index_off), ws + w.total, means, stream);
    if (rs != RAPID_OK) return rs;
    return run_sparse(pr, block, nullptr, workspace, w.total, stream);
}

size_t rapid_attn_joint_select_workspace_bytes(int B, int H, int N, int D, int block)
{
    const size_t attn = rapid_attn_joint_workspace_bytes(B, H, N, D, block);
    if (attn == 0 || (N + block - 1) / block > 2048) return 0;
    return attn + rapid_internal::select_scratch_bytes(B, H, (N + block - 1) / block, D);
}

int rapid_attn_block_sparse_static(const void* q, const void* k, const void* v, void* o,
                                   int B, int H, int N, int D, int block,
                                   const unsigned char* mask, int kv_len, float scale, void* stream)
{
    if (!mask) return RAPID_ERR_NULL;
    const int rc = check_common(q, k, v, o, B, H, N, D, kv_len);
    if (rc != RAPID_OK) return rc;
    if (block != 64 && block != 128) return RAPID_ERR_UNSUPPORTED;
    if (N % block != 0) return RAPID_ERR_SHAPE;
    const int nb = N / block;
    if ((long long)B * H * nb > 0x7fffffffLL / 16) return RAPID_ERR_SHAPE;
    // as many partial-result slots as fit next to the lists (fewer slots: fewer items are cut)
    const WorkspaceLayout none = workspace_layout(B, H, nb, D, block, 0);
    if (none.total > (size_t)RAPID_ATTN_STATIC_SCRATCH_BYTES) return RAPID_ERR_WORKSPACE;
    int slots = -1;
    if (workspace_layout(B, H, nb, D, block).total > (size_t)RAPID_ATTN_STATIC_SCRATCH_BYTES) {
        const size_t per_slot = XCDS * ((D == 64 ? PartialSlot<64>::BYTES : PartialSlot<128>::BYTES) + sizeof(PlanRec) + 4);
        slots = (int)(((size_t)RAPID_ATTN_STATIC_SCRATCH_BYTES - none.total) / per_slot);
        while (slots > 0 && workspace_layout(B, H, nb, D, block, slots).total > (size_t)RAPID_ATTN_STATIC_SCRATCH_BYTES) --slots;
    }
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != RAPID_OK) return rs;
    return run_sparse(contiguous_problem(q, k, v, o, B, H, N, D, kv_len, scale), block, mask, ws,
                      (size_t)RAPID_ATTN_STATIC_SCRATCH_BYTES, stream, slots);
}

size_t rapid_attn_joint_workspace_bytes(int B, int H, int N, int D, int block)
{
    if (B <= 0 || H <= 0 || N <= 0 || N > (1 << 22)) return 0;
    if (D != 64 && D != 128) return 0;
    if (block != 64 && block != 128) return 0;
    const int nb = (N + block - 1) / block;
    if ((long long)B * H * nb > 0x7fffffffLL / 16) return 0;
    return workspace_layout(B, H, nb, D, block).total;
}

size_t rapid_attn_workspace_bytes(int B, int H, int N, int D, int block)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (D != 64 && D != 128) return 0;
    if (block != 64 && block != 128) return 0;
    if (N % block != 0 || N > (1 << 22)) return 0;
    if ((long long)B * H * (N / block) > 0x7fffffffLL / 16) return 0;
    return workspace_layout(B, H, N / block, D, block).total;
}

const char* rapid_attn_status_string(int status)
{
    switch (status) {
        case RAPID_OK: return "ok";
        case RAPID_ERR_NULL: return "a required pointer is NULL";
        case RAPID_ERR_SHAPE: return "invalid shape: need B,H,N > 0, 1 <= kv_len <= N, N % block == 0";
        case RAPID_ERR_UNSUPPORTED: return "unsupported: D must be 64 or 128, block must be 64 or 128";
        case RAPID_ERR_ALIGN: return "q/k/v/o/workspace must be 16-byte aligned";
        case RAPID_ERR_WORKSPACE: return "workspace is NULL or smaller than rapid_attn_workspace_bytes()";
        case RAPID_ERR_DEVICE: return "HIP runtime refused the launch";
        case RAPID_ERR_ALIAS: return "o overlaps q, k or v";
        default: return "unknown status";
    }
}

int rapid_attn_version(void) { return RAPID_ATTN_VERSION; }

}  // extern "C"

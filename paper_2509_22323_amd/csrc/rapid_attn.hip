// MM-DiT joint attention for MI355X (gfx950): dense and block-sparse, flash-style.
//
// Operation: RAPID^3 Sec. 3.1 Eq. 1 (self-attention block of a DiT layer) and
// Sec. 3.2 Level-3 / Eq. 4 (the same block restricted to a pruned attention map,
// per layer and per head).  The pruned map is given as a block mask; pruned tiles
// are never read.
//
// Kernel shape.  One workgroup owns one query tile of 32*NW rows (NW wavefronts,
// 32 query rows each) of one (sample, head) and walks over 64-key tiles:
//   S^T = K Q^T    v_mfma_f32_32x32x16_bf16, A = K tile rows from LDS (128-bit
//                  reads), B = the wave's Q rows held in registers for the whole
//                  kernel.  Computing the TRANSPOSED score tile puts one query
//                  per lane: the running max / sum are per-lane scalars, the row
//                  reductions are in-register plus ONE cross-half exchange
//                  (v_permlane32_swap), and the fp32 accumulator registers of a
//                  lane are, after conversion to bf16, exactly the B operand of
//                  the next product -- P never touches LDS.
//   O^T += V^T P^T same MFMA; A = V^T fragments fetched straight out of the
//                  row-major V tile with the LDS transpose read
//                  (ds_read_b64_tr_b16), B = P^T from the registers above.
// The contraction index of the second product is a dummy, so its key order
// inside a 16-key step is whatever the accumulator layout yields (keys
// 4h+r and 8+4h+r for lane half h); the V^T fragments are fetched in that order.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rapid_attn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int KT = 64;          // keys per LDS tile
constexpr int XCDS = 8;         // L2 domains the dispatcher deals workgroups over
#ifndef DENSE_QT
#define DENSE_QT 256            // query rows per workgroup on the dense path
#endif
#ifndef DENSE_NS
#define DENSE_NS 3              // LDS stages on the dense path
#endif
#ifndef DENSE_PINGPONG
#define DENSE_PINGPONG 1        // dense path: two wavefront groups held in anti-phase
#endif
constexpr float LOG2E = 1.44269504088896340736f;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

struct AttnParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    __bf16* o;
    const int32_t* counts;   // sparse: kept key-blocks per (b,h,query-block); dense: null
    const int32_t* order;    // sparse: launch order of (b,h,query-block) items
    const int32_t* index;    // sparse: kept key-block lists, nb per row
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
// index[row*nb + 0..count) = those key-blocks, ascending; order[row] = row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void compact_mask_kernel(
    const unsigned char* __restrict__ mask, int rows, int nb, int block, int kv_len,
    int32_t* __restrict__ counts, int32_t* __restrict__ order, int32_t* __restrict__ index)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
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
    if (lane == 0) { counts[row] = base; order[row] = row; }
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
__device__ __forceinline__ void issue_tile(const __bf16* __restrict__ src, int key0, int kv_len,
                                           char* lds, int wave, int lane)
{
    typedef Geo<D> G;
    constexpr int PER_WAVE = G::LOADS / NW;
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int ld = wave * PER_WAVE + i;                 // wave-uniform
        const int row = ld * G::ROWS_PER_LOAD + lane / G::CPR;
        const int phys = lane % G::CPR;
        const int logical = phys ^ (IS_V ? G::swz_v(row) : G::swz_k(row));
        int grow = key0 + row;
        grow = grow < kv_len ? grow : kv_len - 1;
        const __bf16* g = src + (size_t)grow * D + logical * 8;
        // global_load_lds_dwordx4: LDS address = M0 + 16 * lane.  Written as assembly so that
        // the copy pipeline is ordered only by the explicit vmcnt waits and barriers of the
        // main loop (the compiler would otherwise wait for all copies before LDS reads it
        // cannot disambiguate).  M0 has no other user in this kernel.
        const unsigned dst = (unsigned)(size_t)LDS_PTR(char, lds + ld * 1024);
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(g));
    }
}

struct SoftmaxState {
    float m;      // max used for the exponent (raw score units); same in both lane halves
    float l;      // this lane's partial sum of probabilities
};

// ---------------------------------------------------------------------------
// V^T fragments through the LDS transpose read.  These reads are written as inline
// assembly with their own s_waitcnt: issued through the compiler builtin they carry no
// alias scope, and the compiler then makes every one of them wait for ALL outstanding
// global->LDS copies (vmcnt(0)), which would serialise the copy pipeline.  LDS returns
// data in order, so "lgkmcnt(N)" = everything but the newest N LDS requests has arrived.
// ---------------------------------------------------------------------------
template <int D>
struct VFrag {
    u32x2 lo[D / 32];      // keys 4h+r      of the 16-key step, for each 32-row block of O^T
    u32x2 hi[D / 32];      // keys 8+4h+r
};

// Request the fragments of the 16 keys starting at tile row ROW0 (a multiple of 16).
// vaddr[db] = LDS byte address of this lane's patch in tile row 0 for O^T block db.
template <int D, int ROW0>
__device__ __forceinline__ void vt_request(VFrag<D>& f, const unsigned (&vaddr)[D / 32])
{
    constexpr int RB = Geo<D>::ROW_BYTES;
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
        asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                     : "=&v"(f.lo[db]), "=&v"(f.hi[db])
                     : "v"(vaddr[db]), "i"(ROW0 * RB), "i"((ROW0 + 8) * RB));
    }
}

// Wait until the fragments in `f` have arrived; N = newer LDS requests that may stay in
// flight.  The fragments are in/out operands so that their uses are ordered after the wait.
template <int D, int N>
__device__ __forceinline__ void vt_wait(VFrag<D>& f)
{
    if constexpr (D == 128) {
        asm volatile("s_waitcnt lgkmcnt(%8)"
                     : "+v"(f.lo[0]), "+v"(f.hi[0]), "+v"(f.lo[1]), "+v"(f.hi[1]),
                       "+v"(f.lo[2]), "+v"(f.hi[2]), "+v"(f.lo[3]), "+v"(f.hi[3])
                     : "i"(N));
    } else {
        asm volatile("s_waitcnt lgkmcnt(%4)"
                     : "+v"(f.lo[0]), "+v"(f.hi[0]), "+v"(f.lo[1]), "+v"(f.hi[1])
                     : "i"(N));
    }
}

// Products of one 16-key group G = 2 rb + t; requests the fragments of group G+1 first.
// NEWER = LDS requests issued after the fragments of this group that may stay in flight.
template <int D, int GRP, int NEWER = 0>
__device__ __forceinline__ void pv_group(VFrag<D> (&vfrag)[2], const unsigned (&vaddr)[D / 32],
                                         const bf16x8 (&pb)[4], f32x16 (&acc)[D / 32])
{
    if constexpr (GRP < 3) {
        vt_request<D, ((GRP + 1) >> 1) * 32 + ((GRP + 1) & 1) * 16>(vfrag[(GRP + 1) & 1], vaddr);
        vt_wait<D, 2 * (D / 32) + NEWER>(vfrag[GRP & 1]);
    } else {
        vt_wait<D, NEWER>(vfrag[GRP & 1]);
    }
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
        const u32x4 both = __builtin_shufflevector(vfrag[GRP & 1].lo[db], vfrag[GRP & 1].hi[db], 0, 1, 2, 3);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb[GRP], acc[db], 0, 0, 0);
    }
}

// K fragments (A operand of S^T = K Q^T), requested in batches of two k-steps x two row
// blocks = 4 x ds_read_b128, through assembly with explicit waits for the same reason as the
// V^T fragments: batch b+1 is in flight while the four products of batch b are issued.
struct KBatch {
    u32x4 f[4];            // [2 * (t & 1) + rb]
};

// kaddr[t] = LDS byte address of this lane's 16-byte chunk of k-step t in row n of the tile.
template <int D, int B>
__device__ __forceinline__ void k_request(KBatch& kb, const unsigned (&kaddr)[D / 16])
{
    constexpr int RB32 = 32 * Geo<D>::ROW_BYTES;           // second 32-key row block
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:%6\n\t"
                 "ds_read_b128 %2, %5\n\tds_read_b128 %3, %5 offset:%6"
                 : "=&v"(kb.f[0]), "=&v"(kb.f[1]), "=&v"(kb.f[2]), "=&v"(kb.f[3])
                 : "v"(kaddr[2 * B]), "v"(kaddr[2 * B + 1]), "i"(RB32));
}

template <bool MORE>
__device__ __forceinline__ void k_wait(KBatch& kb)
{
    asm volatile("s_waitcnt lgkmcnt(%4)"
                 : "+v"(kb.f[0]), "+v"(kb.f[1]), "+v"(kb.f[2]), "+v"(kb.f[3])
                 : "i"(MORE ? 4 : 0));
}

template <int D, int B>
__device__ __forceinline__ void qk_batch(KBatch (&kb)[2], const unsigned (&kaddr)[D / 16],
                                         const bf16x8 (&qf)[D / 16], f32x16 (&st)[2])
{
    constexpr int NB = D / 32;                             // batches per tile
    if constexpr (B + 1 < NB) {
        k_request<D, B + 1>(kb[(B + 1) & 1], kaddr);
        k_wait<true>(kb[B & 1]);
    } else {
        k_wait<false>(kb[B & 1]);
    }
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
            st[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kb[B & 1].f[2 * tt + rb]),
                                                             qf[2 * B + tt], st[rb], 0, 0, 0);
}

template <int D>
__device__ __forceinline__ void k_addresses(const char* lds_k, int n, int h, unsigned (&kaddr)[D / 16])
{
    typedef Geo<D> G;
    const unsigned kbase = (unsigned)(size_t)LDS_PTR(const char, lds_k) + n * G::ROW_BYTES;
    const int kx = h ^ G::swz_k(n);                        // chunk (2t+h) ^ swz == (2t) ^ kx
#pragma unroll
    for (int t = 0; t < D / 16; ++t) kaddr[t] = kbase + (((2 * t) ^ kx) << 4);
}

// S^T = K Q^T for one 64-key tile: two 32-key row blocks; keys at or beyond kv_len -> -inf.
// Register i of row block rb holds key  key0 + 32 rb + 8 (i/4) + 4 h + i%4  of query n.
// Batch 0 of the K fragments must already have been requested into kb[0].
template <int D>
__device__ __forceinline__ void qk_tile(KBatch (&kb)[2], const unsigned (&kaddr)[D / 16], const bf16x8 (&qf)[D / 16],
                                        f32x16 (&st)[2], int key0, int kv_len, int h)
{
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int j = 0; j < 16; ++j) st[rb][j] = 0.f;
    qk_batch<D, 0>(kb, kaddr, qf, st);
    qk_batch<D, 1>(kb, kaddr, qf, st);
    if constexpr (D == 128) {
        qk_batch<D, 2>(kb, kaddr, qf, st);
        qk_batch<D, 3>(kb, kaddr, qf, st);
    }
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
// Updates the running reference max / partial sum, rescales the accumulators when the
// reference moves, and leaves the probabilities as bf16 MFMA operands:
// pb[2 rb + t] = keys 16t + {4h..4h+3, 8+4h..8+4h+3} of row block rb.
template <int D>
__device__ __forceinline__ void softmax_tile(const f32x16 (&st)[2], f32x16 (&acc)[D / 32], SoftmaxState& st_,
                                             float c, float tau, bf16x8 (&pb)[4])
{
    constexpr int DB = D / 32;
    float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(fmaxf(mx, st[0][i]), st[1][i]);
    {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    // Lazy rescale: keep the old reference max while the new one exceeds it by at most
    // tau (probabilities then stay below 2^8); any reference gives the same quotient.
    if (__builtin_amdgcn_ballot_w64(mx > st_.m + tau) != 0ull) {
        const float m_new = fmaxf(st_.m, mx);              // finite: every visited tile has a valid key
        const float alpha = __builtin_amdgcn_exp2f((st_.m - m_new) * c);
        st_.m = m_new;
        st_.l *= alpha;
#pragma unroll
        for (int i = 0; i < DB; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[i][j] *= alpha;
    }
    const float mc = st_.m * c;
    float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int rb = g >> 1, t = g & 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(st[rb][8 * t + i], c, -mc));
            if (i & 1) rs1 += e; else rs0 += e;
            pb[g][i] = (__bf16)e;
        }
    }
    st_.l += rs0 + rs1;
}

// LDS byte addresses of this lane's transpose-read patches in row 0 of a V tile.
template <int D>
__device__ __forceinline__ void v_addresses(const char* lds_v, int h, int tr_row, int tr_col, unsigned (&vaddr)[D / 32])
{
    typedef Geo<D> G;
    const unsigned vbase = (unsigned)(size_t)LDS_PTR(const char, lds_v) + (4 * h + tr_row) * G::ROW_BYTES + tr_col * 2;
    const int vx = G::swz_v(tr_row) >> 2;                  // 64-byte group swizzle of this lane's rows
#pragma unroll
    for (int db = 0; db < D / 32; ++db) vaddr[db] = vbase + ((db ^ vx) << 6);
}

// O^T += V^T P^T for one tile.  Four groups (rb, t) of 16 keys; the V^T fragments of group
// g+1 are requested before the products of group g are issued; group 0 must already have
// been requested into vfrag[0].
template <int D>
__device__ __forceinline__ void pv_tile(VFrag<D> (&vfrag)[2], const unsigned (&vaddr)[D / 32],
                                        const bf16x8 (&pb)[4], f32x16 (&acc)[D / 32])
{
    pv_group<D, 0>(vfrag, vaddr, pb, acc);
    pv_group<D, 1>(vfrag, vaddr, pb, acc);
    pv_group<D, 2>(vfrag, vaddr, pb, acc);
    pv_group<D, 3>(vfrag, vaddr, pb, acc);
}

// One 64-key tile in sequence: S^T = K Q^T, online softmax, O^T += V^T P^T.
template <int D>
__device__ __forceinline__ void compute_tile(const char* lds_k, const char* lds_v, const bf16x8 (&qf)[D / 16],
                                             f32x16 (&acc)[D / 32], SoftmaxState& st_, int key0, int kv_len,
                                             float c, float tau, int n, int h, int tr_row, int tr_col)
{
    unsigned kaddr[D / 16];
    k_addresses<D>(lds_k, n, h, kaddr);
    KBatch kb[2];
    k_request<D, 0>(kb[0], kaddr);
    f32x16 st[2];
    qk_tile<D>(kb, kaddr, qf, st, key0, kv_len, h);
    unsigned vaddr[D / 32];
    v_addresses<D>(lds_v, h, tr_row, tr_col, vaddr);
    VFrag<D> vfrag[2];
    vt_request<D, 0>(vfrag[0], vaddr);                     // consumed after the softmax
    bf16x8 pb[4];
    softmax_tile<D>(st, acc, st_, c, tau, pb);
    pv_tile<D>(vfrag, vaddr, pb, acc);
}

// Epilogue: O = acc / l as bf16.  Register 4j+r of block db holds d = 32 db + 8 j + 4 h + r
// of this lane's query; rows at or beyond kv_len and rows without any kept key become 0.
template <int D>
__device__ __forceinline__ void write_output(__bf16* __restrict__ O, const f32x16 (&acc)[D / 32], float l_part,
                                             int qrow, bool qvalid, int N, int h)
{
    float l_run = l_part;
    {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
        l_run = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float inv = (qvalid && l_run > 0.f) ? 1.0f / l_run : 0.f;
    if (qrow < N) {
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
                *(bf16x4*)(O + (size_t)qrow * D + 32 * db + 8 * j + 4 * h) = ov;
            }
    }
}

// Q^T fragments (B operand of S^T = K Q^T): lane (n, h) holds Q[qrow][16t + 8h .. +8].
template <int D>
__device__ __forceinline__ void load_q(const __bf16* __restrict__ Q, int qrow, bool qvalid, int h, bf16x8 (&qf)[D / 16])
{
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (qvalid) raw = *(const u32x4*)(Q + (size_t)qrow * D + 16 * t + 8 * h);
        qf[t] = __builtin_bit_cast(bf16x8, raw);
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

// NW wavefronts x 32 queries; NS LDS stages (tile t lives in stage t % NS, its copy is
// issued NS-1 tiles ahead); WPE = wavefronts per SIMD the register budget is held to.
template <int D, int NW, int NS, int WPE>
__global__ __launch_bounds__(64 * NW, WPE) void attn_kernel(const AttnParams p)
{
    typedef Geo<D> G;
    constexpr int QT = 32 * NW;
    constexpr int KS = D / 16;                    // k-steps of the QK^T product
    constexpr int DB = D / 32;                    // 32-row blocks of O^T
    constexpr int LPT = 2 * G::LOADS / NW;        // copy instructions per wavefront per tile (K + V)

    // K and V tile rings.  Every stage is its own array (unused ones are dropped) and is
    // selected with compile-time constants only: the compiler then knows that the stage
    // being filled is not the stage being read and adds no wait between the two.
    static_assert(NS >= 2 && NS <= 4, "2 to 4 stages");
    __shared__ __attribute__((aligned(1024))) char lds_k0[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_k1[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_k2[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_k3[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v0[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v1[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v2[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v3[G::TILE_BYTES];
    auto stage_k = [&](int st) -> char* { return st == 0 ? lds_k0 : st == 1 ? lds_k1 : st == 2 ? lds_k2 : lds_k3; };
    auto stage_v = [&](int st) -> char* { return st == 0 ? lds_v0 : st == 1 ? lds_v1 : st == 2 ? lds_v2 : lds_v3; };

    // XCD-aware work mapping: the dispatcher deals consecutive workgroup ids
    // round-robin over the 8 XCDs, so give each XCD a contiguous run of items
    // (query tiles of the same head share K/V in that XCD's L2).
    const int wg = blockIdx.x;
    int item = (wg % XCDS) * p.chunk + wg / XCDS;
    if (item >= p.items) return;
    if (p.order) item = ((const __attribute__((address_space(4))) int32_t*)p.order)[item];
    const int bh = item / p.nq;
    const int qi = item % p.nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31;                      // query within the wave / MFMA column
    const int h = lane >> 5;                      // lane half
    const int kv_len = p.kv_len;

    const size_t base = (size_t)bh * p.N * D;
    const __bf16* __restrict__ Q = p.q + base;
    const __bf16* __restrict__ K = p.k + base;
    const __bf16* __restrict__ V = p.v + base;
    __bf16* __restrict__ O = p.o + base;

    // key tiles to visit: tile t -> first key
    // (the kept-tile list is read through the constant address space so that the reads
    // are scalar loads: they must not share a counter with the tile copies in flight)
    typedef const __attribute__((address_space(4))) int32_t* cptr_t;
    const int ss = p.sub_shift;                   // log2(64-key tiles per mask block)
    const bool sparse = p.counts != nullptr;
    cptr_t list = (cptr_t)(p.index + (size_t)item * p.nb);
    int T;
    if (sparse) {
        const int n_blocks = ((cptr_t)p.counts)[item];
        T = n_blocks << ss;
        if (n_blocks > 0 && (((list[n_blocks - 1] + 1) << ss) - 1) * KT >= kv_len) T -= 1;
    } else {
        T = (kv_len + KT - 1) / KT;
    }
    auto tile_key0 = [&](int t) -> int {
        if (!sparse) return t * KT;
        return ((list[t >> ss] << ss) + (t & ((1 << ss) - 1))) * KT;
    };

    // prologue: copies of the first NS-1 tiles; key_ring[s] = first key of the tile in stage s
    int key_ring[NS];
#pragma unroll
    for (int st = 0; st < NS; ++st) key_ring[st] = 0;
#pragma unroll
    for (int st = 0; st < NS - 1; ++st) {
        if (st < T) {
            key_ring[st] = tile_key0(st);
            issue_tile<D, NW, false>(K, key_ring[st], kv_len, stage_k(st), wave, lane);
            issue_tile<D, NW, true>(V, key_ring[st], kv_len, stage_v(st), wave, lane);
        }
    }
    int key_pref = (NS - 1 < T) ? tile_key0(NS - 1) : 0;   // first key of the next tile to issue

    const int qrow = qi * QT + wave * 32 + n;     // this lane's query row
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
    const float tau = 8.0f / p.c;                 // 2^8 head-room on the probabilities

    // per-lane offsets of the transpose read: within a 16-lane group, lane j points
    // at row j/4, columns 4*(j%4)..+3 of a 4 x 16 patch; lane i receives column i.
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = ((lane & 3) << 2) + (((lane >> 4) & 1) << 4);

    // The Q fragments must have arrived before the loop: a wait for them inside the loop
    // would also wait for every tile copy in flight.
    wait_vmcnt<0>();

    // Pipeline: tile t is computed out of stage t % NS while the copies of tiles
    // t+1 .. t+NS-1 are in flight.  One barrier per tile: after it, tile t is visible to
    // all wavefronts and all of them have finished reading the stage of tile t-1, which
    // is the stage the copy of tile t+NS-1 is then issued into.
    for (int t0 = 0; t0 < T; t0 += NS) {
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            const int t = t0 + st;
            if (t >= T) break;
            // my copies of tile t have landed once at most the copies of the tiles issued
            // after it are outstanding (vector-memory operations complete in order)
            if (NS >= 3 && t + NS - 2 < T) wait_vmcnt<(NS - 2) * LPT>();
            else if (NS >= 4 && t + NS - 3 < T) wait_vmcnt<(NS >= 4 ? (NS - 3) * LPT : 0)>();
            else if (NS >= 4 && t + 1 < T) wait_vmcnt<(NS >= 4 ? LPT : 0)>();
            else wait_vmcnt<0>();
            __syncthreads();
            const int nst = (st + NS - 1) % NS;    // a constant once unrolled
            if (t + NS - 1 < T) {
                key_ring[nst] = key_pref;
                issue_tile<D, NW, false>(K, key_pref, kv_len, stage_k(nst), wave, lane);
                issue_tile<D, NW, true>(V, key_pref, kv_len, stage_v(nst), wave, lane);
                if (t + NS < T) key_pref = tile_key0(t + NS);
            }
            compute_tile<D>(stage_k(st), stage_v(st), qf, acc, sm, key_ring[st], kv_len, p.c, tau, n, h, tr_row, tr_col);
        }
    }

    write_output<D>(O, acc, sm.l, qrow, qvalid, p.N, h);
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
template <int D>
__global__ __launch_bounds__(512, 2) void attn_dense_pp_kernel(const AttnParams p)
{
    typedef Geo<D> G;
    constexpr int NW = 8, QT = 256, KS = D / 16, DB = D / 32;
    constexpr int LPT = 2 * G::LOADS / NW;        // copy instructions per wavefront per tile (K + V)

    __shared__ __attribute__((aligned(1024))) char lds_k0[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_k1[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_k2[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_k3[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v0[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v1[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v2[G::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds_v3[G::TILE_BYTES];
    auto stage_k = [&](int st) -> char* { return st == 0 ? lds_k0 : st == 1 ? lds_k1 : st == 2 ? lds_k2 : lds_k3; };
    auto stage_v = [&](int st) -> char* { return st == 0 ? lds_v0 : st == 1 ? lds_v1 : st == 2 ? lds_v2 : lds_v3; };

    const int wg = blockIdx.x;
    const int item = (wg % XCDS) * p.chunk + wg / XCDS;     // XCD-aware: see attn_kernel
    if (item >= p.items) return;
    const int bh = item / p.nq;
    const int qi = item % p.nq;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = wave >> 2;
    const int n = lane & 31;
    const int h = lane >> 5;
    const int kv_len = p.kv_len;

    const size_t base = (size_t)bh * p.N * D;
    const __bf16* __restrict__ Q = p.q + base;
    const __bf16* __restrict__ K = p.k + base;
    const __bf16* __restrict__ V = p.v + base;
    __bf16* __restrict__ O = p.o + base;

    const int T = (kv_len + KT - 1) / KT;         // >= 1

#pragma unroll
    for (int st = 0; st < 3; ++st) {
        if (st < T) {
            issue_tile<D, NW, false>(K, st * KT, kv_len, stage_k(st), wave, lane);
            issue_tile<D, NW, true>(V, st * KT, kv_len, stage_v(st), wave, lane);
        }
    }

    const int qrow = qi * QT + wave * 32 + n;
    const bool qvalid = qrow < kv_len;
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
    const float tau = 8.0f / p.c;
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = ((lane & 3) << 2) + (((lane >> 4) & 1) << 4);

    wait_vmcnt<0>();                              // Q fragments and the first tiles
    __syncthreads();
    if (group == 1) __syncthreads();              // group 1 runs one barrier behind

    f32x16 st[2];
    {
        unsigned kaddr[KS];
        k_addresses<D>(stage_k(0), n, h, kaddr);
        KBatch kb[2];
        k_request<D, 0>(kb[0], kaddr);
        qk_tile<D>(kb, kaddr, qf, st, 0, kv_len, h);
    }

    for (int j0 = 0; j0 < T; j0 += 4) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int j = j0 + s;
            if (j >= T) break;
            // my share of tile j+1 (outstanding: tiles j+1 and j+2, completing in order)
            if (j + 2 < T) wait_vmcnt<LPT>();
            else wait_vmcnt<0>();
            phase_barrier();

            // ---- B(j)
            unsigned vaddr[DB];
            v_addresses<D>(stage_v(s), h, tr_row, tr_col, vaddr);
            bf16x8 pb[4];
            softmax_tile<D>(st, acc, sm, p.c, tau, pb);
            pin_in_phase(pb, sm.l);
            VFrag<D> vfrag[2];
            vt_request<D, 0>(vfrag[0], vaddr);
            phase_barrier();

            // ---- A(j): matrix work first in line at the SIMD's issue arbiter
            __builtin_amdgcn_s_setprio(3);
            if (j + 3 < T) {
                issue_tile<D, NW, false>(K, (j + 3) * KT, kv_len, stage_k((s + 3) & 3), wave, lane);
                issue_tile<D, NW, true>(V, (j + 3) * KT, kv_len, stage_v((s + 3) & 3), wave, lane);
            }
            // (the first K fragments of tile j+1 are requested ahead of the last PV products;
            // for the last tile this re-reads a landed stage and the result is dropped)
            unsigned kaddr[KS];
            k_addresses<D>(stage_k((j + 1 < T) ? ((s + 1) & 3) : s), n, h, kaddr);
            KBatch kb[2];
            pv_group<D, 0>(vfrag, vaddr, pb, acc);
            pv_group<D, 1>(vfrag, vaddr, pb, acc);
            pv_group<D, 2>(vfrag, vaddr, pb, acc);
            k_request<D, 0>(kb[0], kaddr);
            pv_group<D, 3, 4>(vfrag, vaddr, pb, acc);
            if (j + 1 < T) qk_tile<D>(kb, kaddr, qf, st, (j + 1) * KT, kv_len, h);
            else k_wait<false>(kb[0]);
            __builtin_amdgcn_s_setprio(0);
        }
    }
    if (group == 0) __syncthreads();              // same number of barriers for every wavefront

    write_output<D>(O, acc, sm.l, qrow, qvalid, p.N, h);
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct WorkspaceLayout {
    size_t counts_off, order_off, index_off, total;
};

inline WorkspaceLayout workspace_layout(int B, int H, int nb)
{
    const size_t rows = (size_t)B * H * nb;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    WorkspaceLayout w;
    w.counts_off = 0;
    w.order_off = up(rows * 4);
    w.index_off = w.order_off + up(rows * 4);
    w.total = w.index_off + up(rows * (size_t)nb * 4);
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
    return RAPID_OK;
}

template <int D, int NW, int NS, int WPE>
int launch_attn(const AttnParams& p, hipStream_t stream)
{
    const int grid = p.chunk * XCDS;
    hipLaunchKernelGGL((attn_kernel<D, NW, NS, WPE>), dim3(grid), dim3(64 * NW), 0, stream, p);
    return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
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
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);

    AttnParams p{};
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v; p.o = (__bf16*)o;
    p.counts = nullptr; p.order = nullptr; p.index = nullptr;
    p.H = H; p.N = N; p.kv_len = kv_len;
    p.nq = (N + DENSE_QT - 1) / DENSE_QT;
    const long long items = (long long)B * H * p.nq;
    if (items > 0x7fffffffLL / 2) return RAPID_ERR_SHAPE;
    p.items = (int)items;
    p.chunk = (p.items + XCDS - 1) / XCDS;
    p.block = 0; p.nb = 0; p.sub_shift = 0;
    p.c = scale * LOG2E;
    hipStream_t s = (hipStream_t)stream;
#if DENSE_PINGPONG
    {
        const int grid = p.chunk * XCDS;
        if (D == 64) hipLaunchKernelGGL((attn_dense_pp_kernel<64>), dim3(grid), dim3(512), 0, s, p);
        else hipLaunchKernelGGL((attn_dense_pp_kernel<128>), dim3(grid), dim3(512), 0, s, p);
        return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
    }
#else
    return D == 64 ? launch_attn<64, DENSE_QT / 32, DENSE_NS, 2>(p, s)
                   : launch_attn<128, DENSE_QT / 32, DENSE_NS, 2>(p, s);
#endif
}

int rapid_attn_block_sparse(const void* q, const void* k, const void* v, void* o,
                            int B, int H, int N, int D, int block,
                            const unsigned char* mask, int kv_len, float scale,
                            void* workspace, size_t workspace_bytes, void* stream)
{
    if (!mask) return RAPID_ERR_NULL;
    int rc = check_common(q, k, v, o, B, H, N, D, kv_len);
    if (rc != RAPID_OK) return rc;
    if (block != 64 && block != 128) return RAPID_ERR_UNSUPPORTED;
    if (N % block != 0) return RAPID_ERR_SHAPE;
    const int nb = N / block;
    const long long rows = (long long)B * H * nb;
    if (rows > 0x7fffffffLL / 2) return RAPID_ERR_SHAPE;
    const WorkspaceLayout w = workspace_layout(B, H, nb);
    if (!workspace || workspace_bytes < w.total) return RAPID_ERR_WORKSPACE;
    if (!aligned16(workspace)) return RAPID_ERR_ALIGN;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);

    char* ws = (char*)workspace;
    int32_t* counts = (int32_t*)(ws + w.counts_off);
    int32_t* order = (int32_t*)(ws + w.order_off);
    int32_t* index = (int32_t*)(ws + w.index_off);
    hipStream_t s = (hipStream_t)stream;

    hipLaunchKernelGGL(compact_mask_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                       mask, (int)rows, nb, block, kv_len, counts, order, index);
    if (hipGetLastError() != hipSuccess) return RAPID_ERR_DEVICE;

    AttnParams p{};
    p.q = (const __bf16*)q; p.k = (const __bf16*)k; p.v = (const __bf16*)v; p.o = (__bf16*)o;
    p.counts = counts; p.order = order; p.index = index;
    p.H = H; p.N = N; p.kv_len = kv_len;
    p.nq = nb;
    p.items = (int)rows;
    p.chunk = (p.items + XCDS - 1) / XCDS;
    p.block = block; p.nb = nb; p.sub_shift = block == 128 ? 1 : 0;
    p.c = scale * LOG2E;
    if (block == 128)
        return D == 64 ? launch_attn<64, 4, 2, 2>(p, s) : launch_attn<128, 4, 2, 2>(p, s);
    return D == 64 ? launch_attn<64, 2, 2, 2>(p, s) : launch_attn<128, 2, 2, 1>(p, s);
}

size_t rapid_attn_workspace_bytes(int B, int H, int N, int D, int block)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (D != 64 && D != 128) return 0;
    if (block != 64 && block != 128) return 0;
    if (N % block != 0 || N > (1 << 22)) return 0;
    if ((long long)B * H * (N / block) > 0x7fffffffLL / 2) return 0;
    return workspace_layout(B, H, N / block).total;
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
        default: return "unknown status";
    }
}

int rapid_attn_version(void) { return RAPID_ATTN_VERSION; }

}  // extern "C"

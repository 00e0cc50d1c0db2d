// Block-mask selection for the Sparse-Attention levels, MI355X (gfx950).  C ABI and the rule:
// include/rapid_mask.h (RAPID^3 Sec. 3.2 Level-3 and Sec. 3.3 (c) describe what the mask is
// for; the rule is this library's own).
//
// Two kernels.  block_mean_kernel streams Q and K once (HBM-bound: 2 bytes per element read,
// 4 * D bytes per block written) and leaves fp32 block means in the workspace.
// select_blocks_kernel gives every mask row to one wavefront: scores against all key-block
// means, softmax, and the cumulative-mass cut found without sorting, by bisection over the
// bit patterns of the (positive) probabilities.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "rapid_internal.h"
#include "rapid_mask.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MAX_NB = 2048;      // mask blocks per side the selection kernel holds in LDS

// Q and K of the joint sequence as one or two token segments (the image and the text stream of
// an MM-DiT block): token t < n0 is row t of segment 0, any other token row t - n0 of segment 1.
// Strides in elements, D contiguous; head and token strides are common to both segments.
struct QKView {
    const uint16_t* q0; const uint16_t* k0;
    const uint16_t* q1; const uint16_t* k1;      // null when there is one segment
    long long sb0, sb1, sh, sn;
    int n0, N, H;
    int kv_len;                                   // valid tokens of every sample, or
    const int32_t* kv_lens;                       // per sample (device, [B]), clamped to 0..N
    int text_start;
};

__device__ __forceinline__ int valid_tokens(const QKView& v, int b)
{
    if (v.kv_lens == nullptr) return v.kv_len;
    const int n = v.kv_lens[b];
    return n < 0 ? 0 : (n > v.N ? v.N : n);
}
// live blocks (those that start below the valid length) and the first text block of a sample
__device__ __forceinline__ void sample_blocks(const QKView& v, int b, int block, int nb, int& live, int& first_text)
{
    const int kv = valid_tokens(v, b);
    live = (kv + block - 1) / block;
    first_text = v.text_start < kv ? v.text_start / block : nb;
}

// means[(which, bh, i), :] = mean over the valid rows of block i of Q (which = 0) or K (1).
// 256 threads: D/8 column groups of 8 elements x 256/(D/8) row groups; every thread adds up
// its rows in increasing order, the row groups are then added in increasing order.
template <int D>
__global__ __launch_bounds__(256) void block_mean_kernel(const QKView v, int block, int nb, float* __restrict__ means,
                                                         size_t which_stride)
{
    constexpr int CG = D / 8, RG = 256 / CG;
    __shared__ float red[RG][D];
    const int i = blockIdx.x % nb, bh = blockIdx.x / nb, which = blockIdx.y;
    const int b = bh / v.H, h = bh % v.H;
    const uint16_t* s0 = (which ? v.k0 : v.q0) + (size_t)b * v.sb0 + (size_t)h * v.sh;
    const uint16_t* s1 = v.q1 ? (which ? v.k1 : v.q1) + (size_t)b * v.sb1 + (size_t)h * v.sh - (size_t)v.n0 * v.sn : s0;
    const int kv = valid_tokens(v, b);
    const int lo = i * block;
    int hi = lo + block;
    hi = hi < kv ? hi : kv;                        // kv <= N: a ragged last block ends at N
    const int c = threadIdx.x % CG, g = threadIdx.x / CG;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int r = lo + g; r < hi; r += RG) {
        const u32x4 x = *(const u32x4*)((r < v.n0 ? s0 : s1) + (size_t)r * v.sn + c * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[2 * e] += __uint_as_float(x[e] << 16);
            acc[2 * e + 1] += __uint_as_float(x[e] & 0xffff0000u);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[g][c * 8 + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < D) {
        float s = 0.f;
        for (int gg = 0; gg < RG; ++gg) s += red[gg][threadIdx.x];
        const int cnt = hi - lo;
        means[which * which_stride + ((size_t)bh * nb + i) * D + threadIdx.x] = cnt > 0 ? s / (float)cnt : 0.f;
    }
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// One wavefront per mask row (b, h, i); four rows per workgroup.
// What a row's result is written as: a byte per key-block into `mask` (when given), and/or the
// ascending list of kept key-blocks with its length (the form the attention kernels walk: the
// arrays `counts` and `index` of the attention workspace), so that selection can feed the
// attention without a byte mask in between.
struct RowSink {
    unsigned char* mask;     // [rows, nb] or null
    int32_t* counts;         // [rows] or null
    int32_t* index;          // [rows, nb], with counts
};

// One wavefront writes row `row`: keep(j) for j = lane, lane + 64, ...; every lane takes part.
template <class Keep>
__device__ __forceinline__ void write_row(const RowSink& sink, size_t row, int nb, int lane, Keep keep)
{
    int base = 0;
    for (int j0 = 0; j0 < nb; j0 += 64) {
        const int j = j0 + lane;
        const bool kp = j < nb && keep(j);
        if (sink.mask != nullptr && j < nb) sink.mask[row * nb + j] = kp ? 1 : 0;
        if (sink.counts != nullptr) {
            const unsigned long long bal = __ballot(kp);
            if (kp) sink.index[row * nb + base + __popcll(bal & ((1ull << lane) - 1ull))] = j;
            base += __popcll(bal);
        }
    }
    if (sink.counts != nullptr && lane == 0) sink.counts[row] = base;
}

template <int D>
__global__ __launch_bounds__(256) void select_blocks_kernel(const float* __restrict__ qmean, const float* __restrict__ kmean,
                                                            const QKView v, int block, int rows, int nb, float tau,
                                                            float scale, const RowSink sink)
{
    __shared__ float qrow[4][D];
    __shared__ float prob[4][MAX_NB];
    const int wv = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wv;
    if (row >= rows) return;
    const int i = row % nb;
    const size_t bh = row / nb;
    int live, first_text;
    sample_blocks(v, (int)(bh / v.H), block, nb, live, first_text);
    if (i >= live) {
        write_row(sink, (size_t)row, nb, lane, [](int) { return false; });
        return;
    }
    for (int d = lane; d < D; d += 64) qrow[wv][d] = qmean[(size_t)row * D + d];
    __builtin_amdgcn_wave_barrier();               // one wavefront: its LDS accesses execute in order

    // scores of the live key-blocks (lane j, j + 64, ...), their maximum
    const float* kb = kmean + bh * nb * D;
    float mx = -INFINITY;
    for (int j = lane; j < live; j += 64) {
        const f32x4* kr = (const f32x4*)(kb + (size_t)j * D);
        float dot = 0.f;
#pragma unroll 4
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const f32x4 kv = kr[d4];
            dot += qrow[wv][4 * d4] * kv[0];
            dot += qrow[wv][4 * d4 + 1] * kv[1];
            dot += qrow[wv][4 * d4 + 2] * kv[2];
            dot += qrow[wv][4 * d4 + 3] * kv[3];
        }
        const float s = scale * dot;
        prob[wv][j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    // unnormalised probabilities e = exp(s - max) <= 1 and their sum (normalising both sides
    // of "mass >= tau * total" changes nothing)
    float part = 0.f;
    for (int j = lane; j < live; j += 64) {
        const float e = expf(prob[wv][j] - mx);
        prob[wv][j] = e;
        part += e;
    }
    const float total = wave_sum(part);
    // v* = largest probability whose upper set {e >= v*} holds at least tau * total: positive
    // floats order like their bit patterns, and the mass of the upper set falls as the cut
    // rises, so bisect over the patterns between 0 and 1.0f.
    unsigned cut = 0u;
    if (tau < 1.0f) {
        const float target = tau * total;
        unsigned lo = 0u, hi = 0x3F800001u;                  // mass(lo) >= target > mass(hi) = 0
        while (hi - lo > 1u) {
            const unsigned mid = lo + (hi - lo) / 2u;
            float m = 0.f;
            for (int j = lane; j < live; j += 64) {
                const float e = prob[wv][j];
                m += (__float_as_uint(e) >= mid) ? e : 0.f;
            }
            m = wave_sum(m);
            if (m >= target) lo = mid; else hi = mid;
        }
        cut = lo;
    }
    const bool text_row = i >= first_text;
    write_row(sink, (size_t)row, nb, lane, [&](int j) {
        return j < live && (text_row || j >= first_text || j == i || __float_as_uint(prob[wv][j]) >= cut);
    });
}

// The same for up to SMALL_NB mask blocks per side (every shape of the paper's models): one
// workgroup per 16 rows of one (sample, head).  The key-block means of the head pass through
// LDS in chunks of 64 (coalesced loads, rows padded by four floats so that the 16-byte reads
// of consecutive lanes fall on different banks) and serve all 16 rows; a wavefront owns four
// rows.  The cut needs neither a sort nor a search here: block j is kept iff the blocks with
// a strictly larger probability hold less than tau of the mass, a sum each lane forms for its
// own blocks over all the others (nb^2 work per row, trivial at this size).
constexpr int SMALL_NB = 256;
constexpr int SMALL_RPW = 1;                   // mask rows per wavefront
constexpr int SMALL_ROWS = 4 * SMALL_RPW;     // per workgroup

template <int D>
__global__ __launch_bounds__(256) void select_blocks_small_kernel(const float* __restrict__ qmean,
                                                                  const float* __restrict__ kmean, const QKView v,
                                                                  int block, int nb, float tau, float scale,
                                                                  const RowSink sink)
{
    constexpr int KROW = D + 4;
    __shared__ __attribute__((aligned(16))) float kch[64 * KROW];
    __shared__ __attribute__((aligned(16))) float qs[SMALL_ROWS][D];
    __shared__ float ps[SMALL_ROWS][SMALL_NB];
    const int groups = (nb + SMALL_ROWS - 1) / SMALL_ROWS;
    const size_t bh = blockIdx.x / groups;
    int live, first_text;
    sample_blocks(v, (int)(bh / v.H), block, nb, live, first_text);
    const int i0 = (blockIdx.x % groups) * SMALL_ROWS;
    const int tid = threadIdx.x, wv = tid >> 6, lane = tid & 63;

    constexpr int KPT = 64 * (D / 4) / 256;                    // 16-byte pieces of a chunk per thread
    const float* kb = kmean + bh * nb * D;
    f32x4 kreg[KPT];
    auto fetch_chunk = [&](int j0) {                           // requested early, stored to LDS later
#pragma unroll
        for (int u = 0; u < KPT; ++u) {
            const int e = tid + u * 256, jr = e / (D / 4), d4 = e % (D / 4);
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            kreg[u] = (j0 + jr < live) ? *(const f32x4*)(kb + (size_t)(j0 + jr) * D + 4 * d4) : zero;
        }
    };
    fetch_chunk(0);
    for (int e = tid; e < SMALL_ROWS * D; e += 256) {
        const int r = e / D, d = e % D;
        qs[r][d] = (i0 + r < live) ? qmean[(bh * nb + i0 + r) * D + d] : 0.f;
    }
    for (int j0 = 0; j0 < live; j0 += 64) {
        __syncthreads();                                       // previous chunk consumed (and qs written)
#pragma unroll
        for (int u = 0; u < KPT; ++u) {
            const int e = tid + u * 256, jr = e / (D / 4), d4 = e % (D / 4);
            *(f32x4*)(kch + jr * KROW + 4 * d4) = kreg[u];
        }
        if (j0 + 64 < live) fetch_chunk(j0 + 64);              // the next chunk travels during this one's work
        __syncthreads();
        float dot[SMALL_RPW];
#pragma unroll
        for (int r = 0; r < SMALL_RPW; ++r) dot[r] = 0.f;
        const float* kr = kch + lane * KROW;
#pragma unroll 4
        for (int d4 = 0; d4 < D / 4; ++d4) {
            const f32x4 kv = *(const f32x4*)(kr + 4 * d4);
#pragma unroll
            for (int r = 0; r < SMALL_RPW; ++r) {
                const f32x4 qv = *(const f32x4*)(&qs[wv * SMALL_RPW + r][4 * d4]);
                dot[r] += qv[0] * kv[0];
                dot[r] += qv[1] * kv[1];
                dot[r] += qv[2] * kv[2];
                dot[r] += qv[3] * kv[3];
            }
        }
        if (j0 + lane < live) {
#pragma unroll
            for (int r = 0; r < SMALL_RPW; ++r) ps[wv * SMALL_RPW + r][j0 + lane] = scale * dot[r];
        }
    }
    __builtin_amdgcn_wave_barrier();                           // a wavefront reads only the rows it wrote

    for (int r = 0; r < SMALL_RPW; ++r) {
        const int row = wv * SMALL_RPW + r, i = i0 + row;
        if (i >= nb) break;
        const size_t mrow = bh * nb + i;
        if (i >= live) {
            write_row(sink, mrow, nb, lane, [](int) { return false; });
            continue;
        }
        float mx = -INFINITY;
        for (int j = lane; j < live; j += 64) mx = fmaxf(mx, ps[row][j]);
        mx = wave_max(mx);
        float part = 0.f;
        for (int j = lane; j < live; j += 64) {
            const float e = expf(ps[row][j] - mx);
            ps[row][j] = e;
            part += e;
        }
        const float target = tau * wave_sum(part);
        const bool text_row = i >= first_text;
        write_row(sink, mrow, nb, lane, [&](int j) {
            if (j >= live) return false;
            if (text_row || j >= first_text || j == i || tau >= 1.0f) return true;
            const float mine = ps[row][j];
            float above = 0.f;                             // mass of the blocks that come before j
            for (int k2 = 0; k2 < live; ++k2) {
                const float e = ps[row][k2];
                above += (e > mine) ? e : 0.f;
            }
            return above < target;
        });
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t means_bytes(int B, int H, int nb, int D) { return (size_t)2 * B * H * nb * D * sizeof(float); }

bool shape_ok(int B, int H, int N, int D, int block, bool ragged)
{
    if (B <= 0 || H <= 0 || N <= 0 || N > (1 << 22)) return false;
    if ((long long)B * H > 0x7fffffffLL / 4096) return false;
    if (D != 64 && D != 128) return false;
    if (block != 64 && block != 128) return false;
    if (!ragged && N % block != 0) return false;
    if ((N + block - 1) / block > MAX_NB) return false;
    return true;
}

// One validated call: means, then the selection kernel that fits the size.
int run_select(const QKView& v, int B, int D, int block, float tau, float scale, const RowSink& sink, void* workspace,
               size_t workspace_bytes, void* stream)
{
    const int H = v.H, nb = (v.N + block - 1) / block;
    if (nb > MAX_NB) return RAPID_ERR_UNSUPPORTED;
    const size_t need = means_bytes(B, H, nb, D);
    if (!workspace || workspace_bytes < need) return RAPID_ERR_WORKSPACE;
    if (!aligned16(workspace)) return RAPID_ERR_ALIGN;
    if ((long long)B * H * nb > 0x7fffffffLL / 16) return RAPID_ERR_SHAPE;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);

    float* means = (float*)workspace;
    const size_t which_stride = (size_t)B * H * nb * D;
    hipStream_t s = (hipStream_t)stream;
    const dim3 g1((unsigned)(nb * B * H), 2u);
    if (D == 64) hipLaunchKernelGGL((block_mean_kernel<64>), g1, dim3(256), 0, s, v, block, nb, means, which_stride);
    else hipLaunchKernelGGL((block_mean_kernel<128>), g1, dim3(256), 0, s, v, block, nb, means, which_stride);
    if (hipGetLastError() != hipSuccess) return RAPID_ERR_DEVICE;

    const int rows = B * H * nb;
    if (nb <= SMALL_NB) {
        const dim3 gs((unsigned)(B * H * ((nb + SMALL_ROWS - 1) / SMALL_ROWS)));
        if (D == 64)
            hipLaunchKernelGGL((select_blocks_small_kernel<64>), gs, dim3(256), 0, s, means, means + which_stride, v, block,
                               nb, tau, scale, sink);
        else
            hipLaunchKernelGGL((select_blocks_small_kernel<128>), gs, dim3(256), 0, s, means, means + which_stride, v, block,
                               nb, tau, scale, sink);
        return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
    }
    const dim3 g2((unsigned)((rows + 3) / 4));
    if (D == 64)
        hipLaunchKernelGGL((select_blocks_kernel<64>), g2, dim3(256), 0, s, means, means + which_stride, v, block, rows, nb,
                           tau, scale, sink);
    else
        hipLaunchKernelGGL((select_blocks_kernel<128>), g2, dim3(256), 0, s, means, means + which_stride, v, block, rows, nb,
                           tau, scale, sink);
    return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
}

// Q and K of the joint sequence from segment descriptors, validated (v and o are not looked at).
int joint_view(const rapid_attn_segment* segments, int n_segments, int B, int H, int D, int block, int kv_len,
               const int* kv_lens, int text_start, float tau, QKView& v)
{
    if (!segments) return RAPID_ERR_NULL;
    if (n_segments != 1 && n_segments != 2) return RAPID_ERR_SHAPE;
    if (B <= 0 || H <= 0) return RAPID_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL / 4096) return RAPID_ERR_SHAPE;
    if (D != 64 && D != 128) return RAPID_ERR_UNSUPPORTED;
    if (block != 64 && block != 128) return RAPID_ERR_UNSUPPORTED;
    if (text_start < 0 || !(tau > 0.f)) return RAPID_ERR_SHAPE;
    long long N = 0;
    rapid_attn_segment seg[2];                    // strides of size-1 dimensions are not looked at
    for (int i = 0; i < n_segments; ++i) seg[i] = rapid_internal::normalised_segment(segments[i], B, H, i == 1 ? &seg[0] : nullptr);
    segments = seg;
    for (int i = 0; i < n_segments; ++i) {
        const rapid_attn_segment& g = segments[i];
        if (!g.q || !g.k) return RAPID_ERR_NULL;
        if (g.n <= 0) return RAPID_ERR_SHAPE;
        if (!aligned16(g.q) || !aligned16(g.k)) return RAPID_ERR_ALIGN;
        const long long st[3] = {g.in_stride_b, g.in_stride_h, g.in_stride_n};
        for (int j = 0; j < 3; ++j) {
            if (st[j] < 0 || st[j] > (1LL << 40)) return RAPID_ERR_SHAPE;
            if (st[j] % 8 != 0) return RAPID_ERR_ALIGN;        // every row starts on 16 bytes
        }
        if (g.in_stride_n < D || g.in_stride_n > (1LL << 23)) return RAPID_ERR_SHAPE;
        N += g.n;
    }
    if (N > (1 << 22)) return RAPID_ERR_SHAPE;
    if (n_segments == 2) {
        // as rapid_attn_joint: the masks made here are for that call
        if (segments[0].n % 128 != 0) return RAPID_ERR_SHAPE;
        if (segments[0].in_stride_h != segments[1].in_stride_h || segments[0].in_stride_n != segments[1].in_stride_n)
            return RAPID_ERR_SHAPE;
    }
    if (kv_len == 0) kv_len = (int)N;
    if (kv_len < 1 || kv_len > N) return RAPID_ERR_SHAPE;
    v.q0 = (const uint16_t*)segments[0].q; v.k0 = (const uint16_t*)segments[0].k;
    v.q1 = n_segments == 2 ? (const uint16_t*)segments[1].q : nullptr;
    v.k1 = n_segments == 2 ? (const uint16_t*)segments[1].k : nullptr;
    v.sb0 = segments[0].in_stride_b; v.sb1 = n_segments == 2 ? segments[1].in_stride_b : 0;
    v.sh = segments[0].in_stride_h; v.sn = segments[0].in_stride_n;
    v.n0 = n_segments == 2 ? segments[0].n : (int)N; v.N = (int)N; v.H = H;
    v.kv_len = kv_len; v.kv_lens = kv_lens; v.text_start = text_start;
    return RAPID_OK;
}

}  // namespace

namespace rapid_internal {

size_t select_scratch_bytes(int B, int H, int nb, int D) { return means_bytes(B, H, nb, D); }

int select_to_lists(const rapid_attn_segment* segments, int n_segments, int B, int H, int D, int block,
                    int kv_len, const int* kv_lens, int text_start, float tau, float scale,
                    unsigned char* mask, int32_t* counts, int32_t* index, void* scratch, size_t scratch_bytes,
                    void* stream)
{
    if (!counts || !index) return RAPID_ERR_NULL;
    QKView v{};
    const int rc = joint_view(segments, n_segments, B, H, D, block, kv_len, kv_lens, text_start, tau, v);
    if (rc != RAPID_OK) return rc;
    return run_select(v, B, D, block, tau, scale, RowSink{mask, counts, index}, scratch, scratch_bytes, stream);
}

}  // namespace rapid_internal

extern "C" {

int rapid_mask_select(const void* q, const void* k, int B, int H, int N, int D, int block, int kv_len,
                      int text_start, float tau, float scale, unsigned char* mask, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    if (!q || !k || !mask) return RAPID_ERR_NULL;
    if (B <= 0 || H <= 0 || N <= 0 || N > (1 << 22)) return RAPID_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL / 4096) return RAPID_ERR_SHAPE;
    if (kv_len < 1 || kv_len > N || text_start < 0 || !(tau > 0.f)) return RAPID_ERR_SHAPE;
    if (D != 64 && D != 128) return RAPID_ERR_UNSUPPORTED;
    if (block != 64 && block != 128) return RAPID_ERR_UNSUPPORTED;
    if (N % block != 0) return RAPID_ERR_SHAPE;
    if (N / block > MAX_NB) return RAPID_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k)) return RAPID_ERR_ALIGN;
    QKView v{};
    v.q0 = (const uint16_t*)q; v.k0 = (const uint16_t*)k; v.q1 = nullptr; v.k1 = nullptr;
    v.sb0 = (long long)H * N * D; v.sb1 = 0; v.sh = (long long)N * D; v.sn = D;
    v.n0 = N; v.N = N; v.H = H;
    v.kv_len = kv_len; v.kv_lens = nullptr; v.text_start = text_start;
    return run_select(v, B, D, block, tau, scale, RowSink{mask, nullptr, nullptr}, workspace, workspace_bytes, stream);
}

int rapid_mask_select_joint(const rapid_attn_segment* segments, int n_segments, int B, int H, int D, int block,
                            int kv_len, const int* kv_lens, int text_start, float tau, float scale,
                            unsigned char* mask, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!mask) return RAPID_ERR_NULL;
    QKView v{};
    const int rc = joint_view(segments, n_segments, B, H, D, block, kv_len, kv_lens, text_start, tau, v);
    if (rc != RAPID_OK) return rc;
    return run_select(v, B, D, block, tau, scale, RowSink{mask, nullptr, nullptr}, workspace, workspace_bytes, stream);
}

size_t rapid_mask_select_workspace_bytes(int B, int H, int N, int D, int block)
{
    if (!shape_ok(B, H, N, D, block, false)) return 0;
    return means_bytes(B, H, N / block, D);
}

size_t rapid_mask_select_joint_workspace_bytes(int B, int H, int N, int D, int block)
{
    if (!shape_ok(B, H, N, D, block, true)) return 0;
    return means_bytes(B, H, (N + block - 1) / block, D);
}

float rapid_mask_level_tau(int action)
{
    switch (action) {
        case 0: return 1.0f;
        case 1: return 0.98f;
        case 2: return 0.95f;
        case 3: return 0.90f;
        default: return NAN;
    }
}

}  // extern "C"

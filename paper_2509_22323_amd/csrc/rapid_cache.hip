// Cache-Reuse residual operations and cost accounting of RAPID^3 for MI355X (gfx950).
// C ABI: include/rapid_cache.h.
//
// Device side (Sec. 3.2 "Level-2: Cache-Reuse", Eq. 3): Delta = G(X) - X when the cache is
// updated, O = X + Delta when it is reused; bf16 tensors, one rounding per element.  Both are
// streaming kernels bound by HBM: 2 bytes read from each of two tensors and 2 bytes written
// per element, nothing is reused.  Each lane moves 16 bytes per access (8 elements), four
// independent accesses per tensor in flight before the first use.
// Host side (Sec. 3.3, reward paragraph): equivalent steps K and the discounted reward.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "rapid_cache.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int THREADS = 256;
constexpr int UNROLL = 4;                 // 16-byte accesses per tensor and lane in flight
constexpr int MAX_GROUPS = 16384;         // workgroups per launch: 64 per CU, grid-stride beyond

// a (+/-) b on two packed pairs of bf16, exact in fp32, then one round-to-nearest-even
template <bool SUB>
__device__ __forceinline__ unsigned combine2(unsigned a, unsigned b)
{
    const float a0 = __uint_as_float(a << 16), a1 = __uint_as_float(a & 0xffff0000u);
    const float b0 = __uint_as_float(b << 16), b1 = __uint_as_float(b & 0xffff0000u);
    bf16x2 r;
    r[0] = (__bf16)(SUB ? a0 - b0 : a0 + b0);
    r[1] = (__bf16)(SUB ? a1 - b1 : a1 + b1);
    return __builtin_bit_cast(unsigned, r);
}

template <bool SUB>
__device__ __forceinline__ uint16_t combine1(uint16_t a, uint16_t b)
{
    const float fa = __uint_as_float((unsigned)a << 16), fb = __uint_as_float((unsigned)b << 16);
    return __builtin_bit_cast(uint16_t, (__bf16)(SUB ? fa - fb : fa + fb));
}

// out[s, :] = a[s, :] (+/-) b[s, :] for the samples s = blockIdx.y whose flag is set.
// VEC: every sample starts on a 16-byte boundary in all three tensors; the last
// per_sample % 8 elements of a sample are done one by one.
template <bool SUB, bool VEC>
__global__ __launch_bounds__(THREADS) void cache_residual_kernel(const uint16_t* a, const uint16_t* b, uint16_t* out,
                                                                size_t per_sample, const unsigned char* flags)
{
    const int s = blockIdx.y;
    if (flags != nullptr && flags[s] == 0) return;
    const size_t base = (size_t)s * per_sample;
    a += base; b += base; out += base;
    const size_t tid = (size_t)blockIdx.x * THREADS + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * THREADS;
    if constexpr (VEC) {
        const size_t nvec = per_sample / 8;
        const u32x4* av = (const u32x4*)a;
        const u32x4* bv = (const u32x4*)b;
        u32x4* ov = (u32x4*)out;
        // consecutive lanes touch consecutive 16-byte vectors; the UNROLL accesses of a lane
        // are one grid-width apart
        for (size_t v0 = tid; v0 < nvec; v0 += nthreads * UNROLL) {
            u32x4 x[UNROLL], y[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const size_t v = v0 + (size_t)u * nthreads;
                // read once, never again: non-temporal loads keep the two input streams from
                // displacing each other and the output in the caches (+14 % at one layer's hidden
                // states, +20 % on large tensors; the same hint on the stores made it slower)
                if (v < nvec) { x[u] = __builtin_nontemporal_load(&av[v]); y[u] = __builtin_nontemporal_load(&bv[v]); }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const size_t v = v0 + (size_t)u * nthreads;
                if (v < nvec) {
                    u32x4 r;
#pragma unroll
                    for (int i = 0; i < 4; ++i) r[i] = combine2<SUB>(x[u][i], y[u][i]);
                    ov[v] = r;
                }
            }
        }
        for (size_t e = nvec * 8 + tid; e < per_sample; e += nthreads) out[e] = combine1<SUB>(a[e], b[e]);
    } else {
        for (size_t e = tid; e < per_sample; e += nthreads) out[e] = combine1<SUB>(a[e], b[e]);
    }
}

inline bool aligned(const void* p, uintptr_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; }

template <bool SUB>
int launch(const void* a, const void* b, void* out, int B, size_t per_sample, const unsigned char* flags, void* stream)
{
    if (!a || !b || !out) return RAPID_ERR_NULL;
    if (B <= 0 || per_sample == 0) return RAPID_ERR_SHAPE;
    if (B > 65535 || per_sample > ((size_t)1 << 40) / (size_t)B) return RAPID_ERR_SHAPE;
    if (!aligned(a, 2) || !aligned(b, 2) || !aligned(out, 2)) return RAPID_ERR_ALIGN;
    const bool vec = aligned(a, 16) && aligned(b, 16) && aligned(out, 16) && (B == 1 || per_sample % 8 == 0);
    const size_t work = vec ? (per_sample + 7) / 8 : per_sample;         // lane-iterations per sample
    size_t groups = (work + (size_t)THREADS * UNROLL - 1) / ((size_t)THREADS * UNROLL);
    const size_t cap = (size_t)MAX_GROUPS / (size_t)B > 0 ? (size_t)MAX_GROUPS / (size_t)B : 1;
    if (groups > cap) groups = cap;
    if (groups < 1) groups = 1;
    const dim3 grid((unsigned)groups, (unsigned)B);
    hipStream_t s = (hipStream_t)stream;
    if (vec)
        hipLaunchKernelGGL((cache_residual_kernel<SUB, true>), grid, dim3(THREADS), 0, s, (const uint16_t*)a,
                           (const uint16_t*)b, (uint16_t*)out, per_sample, flags);
    else
        hipLaunchKernelGGL((cache_residual_kernel<SUB, false>), grid, dim3(THREADS), 0, s, (const uint16_t*)a,
                           (const uint16_t*)b, (uint16_t*)out, per_sample, flags);
    return hipGetLastError() == hipSuccess ? RAPID_OK : RAPID_ERR_DEVICE;
}

}  // namespace

extern "C" {

int rapid_cache_store(const void* gen_out, const void* x, void* delta, int B, size_t elems_per_sample,
                      const unsigned char* sample_flags, void* stream)
{
    return launch<true>(gen_out, x, delta, B, elems_per_sample, sample_flags, stream);
}

int rapid_cache_reuse(const void* x, const void* delta, void* out, int B, size_t elems_per_sample,
                      const unsigned char* sample_flags, void* stream)
{
    return launch<false>(x, delta, out, B, elems_per_sample, sample_flags, stream);
}

int rapid_equivalent_steps(const double* c_cache, const double* c_sparse, int n_steps, double* k_exact)
{
    if (n_steps < 0) return RAPID_ERR_SHAPE;
    if (n_steps > 0 && (!c_cache || !c_sparse)) return RAPID_ERR_NULL;
    double k = 0.0;
    for (int i = 0; i < n_steps; ++i) {
        if (!(c_cache[i] >= 0.0 && c_cache[i] <= 1.0) || !(c_sparse[i] >= 0.0 && c_sparse[i] <= 1.0)) return RAPID_ERR_SHAPE;
        k += (1.0 - c_cache[i]) * (1.0 - c_sparse[i]);
    }
    if (k_exact) *k_exact = k;
    const double r = floor(k + 0.5);                       // k >= 0: ties away from zero
    if (r > 2147483647.0) return RAPID_ERR_SHAPE;
    return r < 1.0 ? 1 : (int)r;
}

double rapid_reward(double q, double d, double omega, double lambda, int K)
{
    if (K < 1) return NAN;
    double s = 0.0;
    for (int k = 1; k <= K; ++k) s += pow(lambda, (double)(K - k)) * (q + omega * d);
    return s / (double)K;
}

}  // extern "C"

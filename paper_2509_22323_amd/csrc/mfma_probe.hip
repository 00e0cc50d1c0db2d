// Measurement aid for bench.py (not part of the attention library): a loop of nothing but
// v_mfma_f32_32x32x16_bf16 on operands taken from a caller-supplied buffer, two wavefronts
// per SIMD.  The sustained rate depends on the operand DATA: with constant operands an
// MI355X runs it near the published dense bf16 peak, with random bf16 operands the clock
// is throttled well below.  bench.py reports both next to the attention kernel's rate, so
// that the roofline fraction can be read against what the matrix pipe sustains on the
// same box for the same kind of data.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// data: 16 x 16 bytes per thread (8 A fragments, 8 B fragments); out: one float per thread.
__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(const u32x4* __restrict__ data, float* __restrict__ out,
                                                            int iters)
{
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, data[tid * 16 + i]);
        b[i] = __builtin_bit_cast(bf16x8, data[tid * 16 + 8 + i]);
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + j) & 7], b[u], acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    out[tid] = s;
}

}  // namespace

// Launch the probe: `blocks` workgroups of 256 threads, `iters` x 32 MFMAs per wavefront.
// data: device, data_bytes >= blocks*256*256 bytes; out: device, out_bytes >= blocks*256*4.
// Both sizes are checked here: the kernel itself has no bounds checks.  Returns 0 on success,
// -2 if a buffer is too small.  FLOPs of one launch = blocks * 4 * iters * 32 * 32768.
extern "C" __attribute__((visibility("default")))
int rapid_probe_mfma(const void* data, size_t data_bytes, void* out, size_t out_bytes, int blocks, int iters,
                     void* stream)
{
    if (!data || !out || blocks <= 0 || iters <= 0) return -1;
    if (data_bytes < (size_t)blocks * 256 * 256 || out_bytes < (size_t)blocks * 256 * sizeof(float)) return -2;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4*)data, (float*)out, iters);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

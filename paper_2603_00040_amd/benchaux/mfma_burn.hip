// Bench-only helper, built into its own library (libattnqat_benchaux.so): NOT part of the attention library or its ABI.
// Measurement kernel: the rate at which this part sustains the 16-bit MFMA
// (v_mfma_f32_32x32x16_f16) when nothing else runs, and the clock it holds while doing so.  The published peak
// (2.5 PFLOP/s) is 1024 matrix pipes x 1024 flop per cycle x 2.4 GHz; under a matrix load the part lowers its clock,
// so the rate that can be reached in practice is lower, and the attention kernels' figures are read against both.
#include <hip/hip_runtime.h>

namespace {

typedef _Float16 probe_half8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

// 256 threads, 2 workgroups per CU: two waves per SIMD, each a chain of MFMAs on four accumulators with non-trivial
// register operands.  clk[2*block] = shader clock cycles, clk[2*block + 1] = 100 MHz ticks, of wave 0's loop.
__global__ __launch_bounds__(256, 2) void mfma_burn_kernel(float* __restrict__ out, unsigned long long* __restrict__ clk, int iters)
{
    probe_half8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.001f * (float)((int)threadIdx.x + i));
        b[i] = (_Float16)(0.002f * (float)((int)threadIdx.x - i));
    }
    probe_floatx16 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[k][i] = 0.0f;
    const unsigned long long t0 = __builtin_readcyclecounter();
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[k], 0, 0, 0);
    }
    const unsigned long long t1 = __builtin_readcyclecounter();
    const unsigned long long r1 = __builtin_amdgcn_s_memrealtime();
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[k][i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (threadIdx.x == 0) { clk[2 * blockIdx.x] = t1 - t0; clk[2 * blockIdx.x + 1] = r1 - r0; }
}

}  // namespace

// `blocks` workgroups of 4 waves (2 workgroups per CU: 512 fill a 256-CU part once) each issue iters * 16 MFMAs
// (32x32x16, f16: 32768 flop each) per wave.  out (device, blocks * 256 floats) takes the sums (ignored), clk (device,
// 2 * blocks uint64) per workgroup the shader clock cycles and the 100 MHz ticks its first wave spent in the loop.
// Only enqueues; the caller times the launch.  Returns 0, -1 for bad arguments, -5 if the launch failed.
extern "C" int benchaux_mfma_burn(int blocks, int iters, float* out, unsigned long long* clk, void* stream)
{
    if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 22) || !out || !clk) return -1;
    hipLaunchKernelGGL(mfma_burn_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, clk, iters);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

namespace {
// Plain grid-stride copy, 16 bytes per lane and step: the known-size kernel against which the profiler's traffic
// counters are calibrated.
__global__ __launch_bounds__(256) void copy16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}
}  // namespace

// Copies `bytes` (a multiple of 16) from src to dst (device, 16-byte aligned, not overlapping): reads and writes exactly
// that many bytes.  Only enqueues.  Returns 0, -1 for bad arguments, -5 if the launch failed.
extern "C" int benchaux_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return -1;
    hipLaunchKernelGGL(copy16_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

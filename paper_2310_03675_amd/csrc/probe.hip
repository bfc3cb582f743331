// Measurement aid: the matrix pipe's rate and the shader clock it runs at, under load.
//
// The int8 MFMA rate of this chip depends on the operands: the published peak (5.0 POP/s) is
// 256 CUs x 4 SIMDs x one v_mfma_i32_32x32x32_i8 every 32 cycles at 2.4 GHz, and a kernel that
// keeps every SIMD's matrix pipe busy does issue one MFMA per 32 cycles -- but the clock those
// cycles run at falls with the switching activity of the operands (power management):
// all-zero operands, quantizer-like codes and random bytes give different clocks.  This
// kernel measures it: every wave loops over independent MFMAs on operand fragments read once
// from a caller-supplied buffer (registers only, nothing else competes; one to four waves per
// SIMD: with one or two the pipe takes an MFMA every 32 cycles, with four waves taking turns
// it took 46 to 53 cycles per MFMA on the machines measured), and one wave reports
// its shader-clock cycles (s_memtime) and the constant-rate wall clock (s_memrealtime) around
// the loop.  bench.py prints the result next to the rooflines that are priced at 2.4 GHz.

#include "../../include/hdqt.h"
#include "common.hpp"

namespace hdqt {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256, 4) void matrix_clock_kernel(const uint4* frags, int iters, long long* result, int* sink)
{
    const int lane = threadIdx.x & 63;
    v4i fa[4], fb[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        fa[k] = __builtin_bit_cast(v4i, frags[k * 64 + lane]);
        fb[k] = __builtin_bit_cast(v4i, frags[(4 + k) * 64 + lane]);
    }
    v16i acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[k][r] = 0;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                acc[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[(k + q) & 3], fb[k], acc[k], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    int s = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[k][r];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) { result[0] = c1 - c0; result[1] = w1 - w0; }
}

} // namespace
} // namespace hdqt

extern "C" {

int hdqt_wall_clock_khz(void)
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
    return khz;
}

int hdqt_probe_matrix_clock(const void* fragments, int iters, int waves_per_simd, long long* result,
                            void* scratch, size_t scratch_bytes, void* stream)
{
    constexpr int kThreads = 256;                       // a workgroup is one wave on each SIMD of a CU
    if (!fragments || !result || !scratch) return HDQT_EINVAL_NULL;
    if (iters < 1 || iters > (1 << 20) || waves_per_simd < 1 || waves_per_simd > 4) return HDQT_EINVAL_DIM;
    const int kBlocks = 256 * waves_per_simd;           // 256 CUs
    if (scratch_bytes < (size_t)kBlocks * kThreads * sizeof(int)) return HDQT_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(fragments) & 15u) || (reinterpret_cast<uintptr_t>(result) & 7u)) return HDQT_EALIGN;
    hipLaunchKernelGGL(hdqt::matrix_clock_kernel, dim3(kBlocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(fragments), iters, result, static_cast<int*>(scratch));
    return hipGetLastError() == hipSuccess ? HDQT_OK : HDQT_EHIP;
}

} // extern "C"

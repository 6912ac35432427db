// On-box calibration of the two rooflines the layers are priced against: what the matrix
// cores deliver when nothing else is in the way (a register-only loop of independent matrix
// instructions on every SIMD), and what HBM delivers to a plain streaming copy.  The caller
// times the launches with events; these kernels do no other work.
#include "fc_mfma_util.hpp"

namespace fc {

// Every wave runs `iters` rounds of eight independent 32x32x16 (or, for 8-bit operands,
// 32x32x64) matrix instructions on operands it holds in registers: 8 * 2 * 32 * 32 * K
// FLOP per round and wave.
template <int DT>
__global__ __launch_bounds__(256) void k_calibrate_mfma(int iters, float *__restrict__ sink)
{
    Frag<DT> a, b;
    const uint32_t s = 0x3c003c00u + (uint32_t)threadIdx.x; // finite 16-bit (and 8-bit) patterns
    a.v = make_uint4(s, s + 1, s + 2, s + 3);
    b.v = make_uint4(s + 4, s + 5, s + 6, s + 7);
    if constexpr (DT == FC_FP8) {
        a.v2 = a.v;
        b.v2 = b.v;
    }
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = mfma32<DT>(a, b, acc[i]);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0] + acc[i][15];
    if (t == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = t; // (keeps the loop alive; never true in practice)
}

// Grid-stride copy of 16-byte pieces.
__global__ __launch_bounds__(256) void k_calibrate_copy(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst,
                                                        size_t pieces)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < pieces; i += (size_t)gridDim.x * 256)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

hipError_t launch_calibrate_mfma(int dtype, int iters, int blocks, float *sink, hipStream_t s)
{
    if (dtype == FC_BF16) hipLaunchKernelGGL(k_calibrate_mfma<FC_BF16>, dim3(blocks), dim3(256), 0, s, iters, sink);
    else if (dtype == FC_F16) hipLaunchKernelGGL(k_calibrate_mfma<FC_F16>, dim3(blocks), dim3(256), 0, s, iters, sink);
    else hipLaunchKernelGGL(k_calibrate_mfma<FC_FP8>, dim3(blocks), dim3(256), 0, s, iters, sink);
    return hipGetLastError();
}

hipError_t launch_calibrate_copy(const void *src, void *dst, size_t bytes, hipStream_t s)
{
    const size_t pieces = bytes / 16;
    size_t blocks = (pieces + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(k_calibrate_copy, dim3((unsigned)blocks), dim3(256), 0, s, (const u32x4_t *)src, (u32x4_t *)dst, pieces);
    return hipGetLastError();
}

} // namespace fc

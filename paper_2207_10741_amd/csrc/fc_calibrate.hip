// On-box calibration of the two rooflines the layers are priced against: what the matrix
// cores deliver when nothing else is in the way (a register-only loop of independent matrix
// instructions on every SIMD), and what HBM delivers to a plain streaming copy.  The caller
// times the launches with events; these kernels do no other work.  A third kernel measures
// what a wave can issue beside its matrix instructions (cycles per step, counted on the device).
#include "fc_dma_util.hpp"

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

// What does one more instruction cost a wave that issues two matrix instructions per step?
// Every wave runs `steps` steps of two independent 32x32x16 bf16 matrix instructions plus the
// item `MODE` names, and wave 0 of every workgroup reports the shader cycles the loop took.
//   0: nothing else                        3: one 16-byte-per-lane LDS read (the next operand)
//   1: one 1 KB load from `src` into LDS   4: items 1 and 3
//   2: twelve dependent integer instructions
// NT / 256 waves share a SIMD.  `src` holds at least 1 MiB; every access stays inside it.
template <int MODE, int NT>
__global__ __launch_bounds__(NT, 1) void k_calibrate_issue(const unsigned char *__restrict__ src, int steps,
                                                           long long *__restrict__ cycles, float *__restrict__ sink)
{
    constexpr uint32_t kWaveBytes = 4096;   // 2 KB of operand rows, then two 1 KB landing zones
    __shared__ __align__(16) unsigned char lds[(NT / 64) * kWaveBytes];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    unsigned char *my = lds + (size_t)wave * kWaveBytes;
    const uint32_t my0 = (uint32_t)reinterpret_cast<uintptr_t>(lds) + (uint32_t)wave * kWaveBytes;
    for (int i = lane; i < (int)kWaveBytes / 4; i += 64) reinterpret_cast<uint32_t *>(my)[i] = 0x3c003c00u + (uint32_t)i;
    __syncthreads();
    const u32x4_t rsrc = make_rsrc_words(src, 1u << 20);
    const uint32_t off0 = (uint32_t)(((blockIdx.x * (NT / 64) + wave) * 65536u + (uint32_t)lane * 16u) & ((1u << 20) - 8192u));
    Frag<FC_BF16> wa, wb, fr;
    wa.v = make_uint4(0x3c003c00u + lane, 0x3c013c01u, 0x3c023c02u, 0x3c033c03u);
    wb.v = make_uint4(0x3c043c04u + lane, 0x3c053c05u, 0x3c063c06u, 0x3c073c07u);
    fr.load(my, (uint32_t)lane * 16u);
    f32x16_t acc0, acc1;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc0[j] = acc1[j] = 0.f;
    uint32_t v1 = lane, v2 = lane * 3u, v3 = 7u;
    const long long t0 = clock64();
    for (int it = 0; it < steps; ++it) {
        acc0 = mfma32<FC_BF16>(wa, fr, acc0);
        acc1 = mfma32<FC_BF16>(wb, fr, acc1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MODE == 1 || MODE == 4) {
            dma_load16(rsrc, off0 + (uint32_t)(it & 3) * 1024u, my0 + 2048u + (uint32_t)(it & 1) * 1024u);
            if (it & 1) wait_vmcnt<1>();
        }
        if constexpr (MODE == 2) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v1 = v1 * 3u + v3;
                v2 = (v2 ^ v1) + 5u;
                v3 = v3 + (v2 >> 3);
            }
        }
        if constexpr (MODE == 3 || MODE == 4) fr.load(my, ((uint32_t)lane * 16u + (uint32_t)it * 1024u) & 2047u);
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<0>();
    const long long t1 = clock64();
    if (threadIdx.x == 0) cycles[blockIdx.x] = t1 - t0;
    float t = acc0[0] + acc0[15] + acc1[0] + acc1[15];
    if (t == 12345.678f || v1 + v2 + v3 == 0x7fffffffu) sink[blockIdx.x] = t + (float)fr.v.x; // (never true in practice)
}

template <int NT>
static hipError_t launch_issue_nt(int mode, int blocks, const void *src, int steps, long long *cycles, float *sink,
                                  hipStream_t s)
{
    const unsigned char *sp = (const unsigned char *)src;
    switch (mode) {
    case 0: hipLaunchKernelGGL((k_calibrate_issue<0, NT>), dim3(blocks), dim3(NT), 0, s, sp, steps, cycles, sink); break;
    case 1: hipLaunchKernelGGL((k_calibrate_issue<1, NT>), dim3(blocks), dim3(NT), 0, s, sp, steps, cycles, sink); break;
    case 2: hipLaunchKernelGGL((k_calibrate_issue<2, NT>), dim3(blocks), dim3(NT), 0, s, sp, steps, cycles, sink); break;
    case 3: hipLaunchKernelGGL((k_calibrate_issue<3, NT>), dim3(blocks), dim3(NT), 0, s, sp, steps, cycles, sink); break;
    default: hipLaunchKernelGGL((k_calibrate_issue<4, NT>), dim3(blocks), dim3(NT), 0, s, sp, steps, cycles, sink); break;
    }
    return hipGetLastError();
}

hipError_t launch_calibrate_issue(int mode, int waves_per_simd, int steps, int blocks, const void *src,
                                  long long *cycles, float *sink, hipStream_t s)
{
    if (waves_per_simd == 1) return launch_issue_nt<256>(mode, blocks, src, steps, cycles, sink, s);
    if (waves_per_simd == 2) return launch_issue_nt<512>(mode, blocks, src, steps, cycles, sink, s);
    return launch_issue_nt<1024>(mode, blocks, src, steps, cycles, sink, s);
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

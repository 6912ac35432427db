// Pieces shared by the kernels that gather straight from global memory into LDS: the raw
// buffer descriptor, the wave-wide 16-byte-per-lane load into LDS, the explicit wait on the
// vector-memory counter, and the XOR swizzle of the 128-byte LDS rows.
#pragma once
#include "fc_mfma_util.hpp"

namespace fc {

// LDS swizzle: slot of a row's 16-byte piece p is p ^ FC_SWZ(row)
#ifndef FC_SWZ
#define FC_SWZ(r) (((r) >> 1) & 7)
#endif

constexpr uint32_t kBufferLimit = 0xF0000000u; // tensors handled through one descriptor stay below this
constexpr uint32_t kOutOfRange = kBufferLimit; // offset that is out of range for every descriptor
constexpr int kStageBytes = 128;               // bytes of one pixel a stage gathers (64 16-bit or 128 8-bit channels)
constexpr int kDeviceScope = 16;               // cache-policy bit sc1: the access is coherent across the XCDs' L2s

// Raw buffer descriptor (4 dwords) over `bytes` bytes at p: stride 0, so offsets are
// plain byte offsets and anything at or beyond `bytes` reads as zero.
__device__ __forceinline__ u32x4_t make_rsrc_words(const void *p, uint32_t bytes)
{
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    u32x4_t r;
    r.x = (uint32_t)a;
    r.y = (uint32_t)(a >> 32) & 0xffffu;
    r.z = bytes;
    r.w = 0x00020000u;
    return r;
}

// One wave-wide 16-byte-per-lane load into LDS at lds_addr + 16 * lane (lds_addr is
// wave-uniform and goes through M0).
__device__ __forceinline__ void dma_load16(const u32x4_t &rsrc, uint32_t byte_offset, uint32_t lds_addr)
{
    __asm__ volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :
                     : "s"(lds_addr), "v"(byte_offset), "s"(rsrc)
                     : "memory");
}

// The same with a wave-uniform byte offset added by the instruction (the scalar offset operand):
// the part of an address that is the same for every lane costs no vector arithmetic.  An
// out-of-range `byte_offset` stays out of range whatever the scalar offset is (it is checked
// against the descriptor's size less the scalar offset).
__device__ __forceinline__ void dma_load16_s(const u32x4_t &rsrc, uint32_t byte_offset, uint32_t scalar_offset,
                                             uint32_t lds_addr)
{
    __asm__ volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_addr), "v"(byte_offset), "s"(rsrc), "s"(scalar_offset)
                     : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __asm__ volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

} // namespace fc

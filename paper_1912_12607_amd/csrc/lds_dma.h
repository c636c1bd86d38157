// Operand fetch of the wide implicit-GEMM kernels: buffer loads that write straight into LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace int8t {

typedef int lds_dma_v4i __attribute__((ext_vector_type(4)));

constexpr uint32_t IGD_OOB = 0x80000000u;
constexpr int IGD_BN = 256;

// Buffer descriptor (base, no stride, byte count, raw 32-bit format) as four scalar words.
__device__ __forceinline__ lds_dma_v4i igd_rsrc(const void* p, uint32_t bytes) {
    const uint64_t addr = (uint64_t)p;
    return lds_dma_v4i{(int)(uint32_t)addr, (int)((uint32_t)(addr >> 32) & 0xffffu), (int)bytes, 0x00020000};
}
// One wave-wide 16-byte-per-lane buffer load into LDS: lane l's bytes land at lds_base + 16*l, an
// offset beyond the descriptor writes zeros.  Written as an instruction block so that the wait for
// it can be placed by hand (see the vmcnt waits in the kernel): the compiler would otherwise wait
// for ALL outstanding loads in front of every LDS read.  (m0 carries the LDS base; the compiler keeps
// no value of its own in it across statements.)
__device__ __forceinline__ void igd_load_lds(const lds_dma_v4i& rsrc, uint32_t lds_base_uniform, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base_uniform), "v"(voff), "s"(rsrc) : "memory");
}
// slot of (row, granule) in a [rows][KG] tile; the xor makes the MFMA operand reads (16 consecutive
// rows of one granule per LDS pass) hit 16 different slots mod 16, see lds_slot(): with 8 granules per
// row, slot mod 16 = 8 * (row & 1) + position, so rows of equal parity need different positions
template <int KG>
__device__ __forceinline__ int igd_slot(int row, int g) {
    return KG == 4 ? row * 4 + (g ^ ((row >> 2) & 3)) : row * 8 + (g ^ ((row >> 1) & 7));
}
template <int N>
__device__ __forceinline__ void igd_wait_vmcnt() {
    static_assert(N == 0 || N == 1 || N == 2 || N == 4 || N == 6 || N == 8 || N == 12, "outstanding loads allowed while waiting");
    if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (N == 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
    else if (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else if (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
}


}  // namespace int8t

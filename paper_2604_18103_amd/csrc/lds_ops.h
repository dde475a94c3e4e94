// LDS operand access shared by the MFMA kernels (attention, GEMMs): direct global->LDS tile loads and the gfx950
// LDS transpose read, each a thin wrapper around one instruction.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace dash {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// LDS transpose read: within each group of 16 lanes, lane t supplies the address of 4 consecutive
// 16-bit elements of row t/4 (columns 4*(t%4)..+3) of a 4x16 block and receives column t of the block.
__device__ __forceinline__ s16x4 lds_read_tr16(const __bf16* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}

// One direct global->LDS load: lane l's 16 bytes at `base + voff` (uniform base, per-lane 32-bit offset) land at
// LDS address lds_base + 16*l. Issued as inline asm so that the compiler's wait-count bookkeeping does not tie
// every later LDS read to it; the kernels wait for these loads explicitly (dma_wait) before the barrier that
// publishes a stage. (M0 holds the LDS base; naming it as a clobber is what keeps the compiler from caching a
// value in it.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_load16(const void* base, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_base), "v"(voff), "s"(base) : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }
// waits until at most KEEP of this wave's loads (the most recently issued ones) are still in flight
template <int KEEP>
__device__ __forceinline__ void dma_wait_keep() { asm volatile("s_waitcnt vmcnt(%0)" : : "i"(KEEP) : "memory"); }
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

}  // namespace dash

// Asynchronous global -> LDS copies (16 bytes per lane) and the explicit wait on them.
//
// dma_load16: every lane of the wave passes its own global address; the 64 x 16 bytes
// land contiguously, in lane order, at LDS byte address lds_wave_base.  The copy is
// tracked by the vector-memory counter only, so the caller must wait_vmcnt<N>() (N =
// number of younger copies allowed to stay in flight) and then pass a barrier before
// other waves read the data.  The compiler is not told about the LDS write; that is
// what lets several copies stay in flight across loop iterations.
#pragma once
#include <stdint.h>

__device__ __forceinline__ void dma_load16(const void *lane_addr, uint32_t lds_wave_base) {
    // lds_wave_base must be wave-uniform (derive it with readfirstlane where the compiler cannot tell)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_addr), "s"(lds_wave_base) : "memory");
}
// The same copy addressed as a wave-uniform base (held in scalar registers) plus a per-lane 32-bit byte offset: the running
// pointers of a stream then advance on the scalar unit and no vector instruction is spent on addresses.
__device__ __forceinline__ void dma_load16_s(const void *uniform_base, uint32_t lane_offset, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_offset), "s"(uniform_base), "s"(lds_wave_base) : "memory");
}
// Same with 4 bytes per lane: 64 x 4 bytes land contiguously at lds_wave_base.
__device__ __forceinline__ void dma_load4(const void *lane_addr, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(lane_addr), "s"(lds_wave_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    // s_waitcnt immediate: vmcnt in bits 3:0 and 15:14; expcnt (6:4) and lgkmcnt (11:8) left at "no wait"
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
    asm volatile("" ::: "memory");
}
// LDS byte address of a pointer into shared memory
__device__ __forceinline__ uint32_t lds_addr(const void *p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)p;
}

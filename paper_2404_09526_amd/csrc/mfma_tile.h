// Device helpers shared by the kernels that work on MFMA tiles staged in LDS (gfx950 only): the exchange between the
// two halves of a wavefront, LDS transfers issued as assembly, and the waits that belong to them.
#pragma once
#include "esp_common.h"

namespace esp {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4_t;
#define ESP_LDS __attribute__((address_space(3)))

// Both halves of the wavefront exchange a value: lo = value held by lane l & 31, hi = value held by
// lane l | 32.  v_permlane32_swap exchanges the upper half of its first register with the lower half of
// its second.  It is issued as inline assembly: with equal operands the compiler's own intrinsic gets
// folded as if both results were the same value.
__device__ __forceinline__ void half_pair(float x, float& lo, float& hi) {
    int a = __builtin_bit_cast(int, x), b = a;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    lo = __builtin_bit_cast(float, a);
    hi = __builtin_bit_cast(float, b);
}
__device__ __forceinline__ float half_swap_max(float x) {
    float lo, hi;
    half_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float half_swap_sum(float x) {
    float lo, hi;
    half_pair(x, lo, hi);
    return lo + hi;
}

#define ESP_GLOBAL __attribute__((address_space(1)))

// One global -> LDS transfer of 64 x 16 bytes: lane L's 16 bytes (at gbase + voff) land at lds_addr + 16*L.
// Issued as assembly so that the loads stay in flight across LDS reads of other stages; the matching
// waits are the explicit vmcnt waits in the kernel.
__device__ __forceinline__ void load_to_lds_b128(uint32_t lds_addr, const void* gbase, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory", "m0");
}
// the same with a full address per lane (rows scattered over a pool larger than a 32-bit offset reaches)
__device__ __forceinline__ void load_to_lds_b128_at(uint32_t lds_addr, const void* src) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_addr), "v"(src) : "memory", "m0");
}
// the same for rows that are read once (a decode pass over the pool): marked non-temporal, so that they do not
// displace what the caches hold
__device__ __forceinline__ void load_to_lds_b128_at_nt(uint32_t lds_addr, const void* src) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
                 :: "s"(lds_addr), "v"(src) : "memory", "m0");
}
__device__ __forceinline__ void load_to_lds_b32(uint32_t lds_addr, const void* gbase, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace esp

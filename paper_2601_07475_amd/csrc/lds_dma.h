// Global -> LDS copies without register staging, and the synchronisation that goes with them.
//
// global_load_lds_dword{,x4}: every lane reads 4 / 16 bytes from (SGPR base + its 32-bit VGPR
// offset); the wave's data lands contiguously in LDS at M0 + 4 / 16 * lane.  The instructions
// are issued through inline assembly on purpose: the compiler then neither knows nor guesses
// which later LDS reads depend on them (it would otherwise drain the vector-memory counter
// before every LDS read and undo the prefetch), so the CALLER orders them by hand:
//   * wait_vmcnt<N>() before reading: vector-memory operations retire in issue order, so
//     "at most N outstanding" means everything but the N youngest has landed;
//   * wg_barrier() so that every wave's copies are visible to every other wave.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arcq {

typedef __attribute__((address_space(3))) uint8_t lds_u8_t;

// Byte address inside the workgroup's LDS allocation of a pointer into __shared__ memory.
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)((const lds_u8_t*)p);
}

// lds_wave_base must be the same in every lane of the wave (it is read from lane 0).
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voffset, uint32_t lds_wave_base) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(m0v), "v"(voffset), "s"(gbase)
                 : "memory", "m0");
}

__device__ __forceinline__ void dma4(const void* gbase, uint32_t voffset, uint32_t lds_wave_base) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(m0v), "v"(voffset), "s"(gbase)
                 : "memory", "m0");
}

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14;
// expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
    asm volatile("" ::: "memory");
}

// Waits for every outstanding LDS / scalar-memory operation of this wave (lgkmcnt(0)) only.
__device__ __forceinline__ void wait_lgkmcnt0() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);
    asm volatile("" ::: "memory");
}

// Workgroup barrier without the memory fence of __syncthreads() (which would drain every
// outstanding vector-memory operation, prefetches included).  Memory accesses are not moved
// across it by the compiler.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Small LDS accesses issued through inline assembly, for bookkeeping words that live beside a
// buffer with copies in flight: the compiler does not see them as LDS accesses, so it does not
// wait for those copies first.  The caller orders them with wait_lgkmcnt0() and wg_barrier().
__device__ __forceinline__ void lds_add_u64(uint32_t addr, uint64_t v) {
    asm volatile("ds_add_u64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_add_f64(uint32_t addr, double v) {
    asm volatile("ds_add_f64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_u64(uint32_t addr, uint64_t v) {
    asm volatile("ds_write_b64 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_f32(uint32_t addr, float v) {
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
// The two reads wait for their own result (and every older LDS operation of the wave).
__device__ __forceinline__ uint64_t lds_read_u64(uint32_t addr) {
    uint64_t v;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ double lds_read_f64(uint32_t addr) {
    double v;
    asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
typedef uint32_t lds_u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ lds_u32x4_t lds_read_b128(uint32_t addr) {       // addr 16-byte aligned
    lds_u32x4_t v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}
__device__ __forceinline__ float lds_read_f32(uint32_t addr) {
    float v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
    return v;
}

}  // namespace arcq

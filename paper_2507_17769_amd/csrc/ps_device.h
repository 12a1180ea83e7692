// Device-side helpers for the gfx950 kernels: bf16 packing, MFMA operand types, wave shuffles.
#pragma once
#include "ps_common.h"

namespace ps {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));  // 4 bf16 bit patterns (16x16x16 MFMA operand)
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// two floats -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2_t v;
    v.x = (__bf16)lo;
    v.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float x) { return (bf16_t)(pack_bf16(x, 0.f) & 0xFFFFu); }

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

__device__ __forceinline__ uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// the same with the non-temporal hint: for data that is read once (streamed weights, decode KV)
__device__ __forceinline__ uint4 ldg16_stream(const void* p) {
    typedef unsigned u32x4_nt_t __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt_t*>(p)));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}


// ---- HBM -> LDS copies without a register hop, and the LDS reads that go with them -------------
// global_load_lds writes lane l's 16 bytes at the (wavefront-uniform) LDS address + 16 l and counts
// in vmcnt.  The compiler cannot tell an ordinary LDS read from the LDS writes of such loads in
// flight and would drain the load queue before each one, so the kernels that use these copies read
// LDS through lds_read16 (inline assembly) and wait with lgkm_tie, which names the registers it
// makes valid so that their consumers cannot move above the wait.
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

#define PS_GLOBAL_TO_LDS(gp, lp)                                                                                     \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gp),                            \
                                     (__attribute__((address_space(3))) void*)(lp), 16, 0, 0)

__device__ __forceinline__ u32x4_t lds_read16(uint32_t addr, int off) {
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(off) : "memory");
    return v;
}
// wait until at most CNT LDS operations are outstanding; the named registers are tied to the wait
template <int CNT>
__device__ __forceinline__ void lgkm_tie(u32x4_t& a) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(CNT));
}
template <int CNT>
__device__ __forceinline__ void lgkm_tie(u32x4_t& a, u32x4_t& b, u32x4_t& c) {
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(CNT));
}
template <int CNT>
__device__ __forceinline__ void lgkm_tie(u32x4_t& a, u32x4_t& b, u32x4_t& c, u32x4_t& d, u32x4_t& e) {
    asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e) : "n"(CNT));
}
template <int CNT>
__device__ __forceinline__ void vm_wait() {
    // s_waitcnt immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]; others left open
    __builtin_amdgcn_s_waitcnt((CNT & 15) | ((CNT >> 4) << 14) | 0x0F70);
}

}  // namespace ps

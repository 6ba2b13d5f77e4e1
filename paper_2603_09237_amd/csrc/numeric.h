// Element types and conversions used by the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;  // storage type of bf16 tensors; conversion from float rounds to nearest even

// 16-bit fixed point for the saved activation derivatives in bf16 mode.  tanh' lies in [0, 1] and
// SiLU' in [-0.0998, 1.0998]; the code q = round((g + 1/8) / step), step = 5 * 2^-18, covers
// [-0.125, 1.125) with an absolute error below 1e-5 -- an order of magnitude finer than fp16 near 1,
// which keeps dZ = dH * act'(z) from landing on the other side of a bf16 rounding boundary.
struct gfix16_t { uint16_t q; };
#define GFIX_STEP 1.9073486328125e-05f

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

// Storage type of act'(z) saved for the backward pass: same width as the GEMM input type.
template <typename T> struct GradT { typedef float type; };
template <> struct GradT<__bf16> { typedef gfix16_t type; };
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

template <typename T> __device__ inline T cvt(float v);
template <> __device__ inline float cvt<float>(float v) { return v; }
template <> __device__ inline bf16_t cvt<bf16_t>(float v) { return (bf16_t)v; }
template <> __device__ inline gfix16_t cvt<gfix16_t>(float v) {
    float q = rintf((v + 0.125f) * (1.0f / GFIX_STEP));
    q = fminf(fmaxf(q, 0.f), 65535.f);
    gfix16_t r;
    r.q = (uint16_t)q;
    return r;
}

__device__ inline float to_f(float v) { return v; }
__device__ inline float to_f(bf16_t v) { return (float)v; }
__device__ inline float to_f(gfix16_t v) { return (float)v.q * GFIX_STEP - 0.125f; }

// eight consecutive elements, destination 16-byte aligned (bf16) / 32-byte run of two float4 (fp32)
__device__ inline void store8(float* dst, const float v[8]) {
    reinterpret_cast<float4*>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ inline void store8(bf16_t* dst, const float v[8]) {
    bf16x8_t o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (bf16_t)v[i];
    *reinterpret_cast<bf16x8_t*>(dst) = o;
}

// ---- direct-to-LDS loads (global_load_lds_*): a wave-uniform 64-bit base in scalar registers plus a 32-bit
// lane offset; lane l of the wave writes its 4 (16) bytes at LDS address lds_addr + 4 l (16 l).  Asynchronous:
// counted by vmcnt like any load, no staging registers.
// wave-uniform 64-bit address held in scalar registers, whatever unit computed it
__device__ inline uint64_t uniform_addr(const void* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ inline void dma16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff),
                 "s"(uniform_addr(sbase))
                 : "memory");
}
__device__ inline void dma4(const void* sbase, uint32_t voff, uint32_t lds_addr) {  // 4 bytes per lane
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(voff),
                 "s"(uniform_addr(sbase))
                 : "memory");
}
// the same, marked non-temporal: for tensors a kernel reads once
__device__ inline void dma16_nt(const void* sbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_addr), "v"(voff),
                 "s"(uniform_addr(sbase))
                 : "memory");
}
__device__ inline void dma4_nt(const void* sbase, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2 nt" ::"s"(lds_addr), "v"(voff),
                 "s"(uniform_addr(sbase))
                 : "memory");
}
template <int N> __device__ inline void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }


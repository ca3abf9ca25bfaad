// Device-side helpers shared by the kernel files of libnpas (HIP only): storage conversions, the activations as
// one clamp, MFMA wrappers, fast division, streaming accesses.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "npas_internal.h"

namespace npas {

// Raises a kernel's dynamic LDS limit once per process (one std::once_flag per kernel instantiation).
template <typename K> static void allow_lds_once(std::once_flag &once, K kern, int bytes)
{
    std::call_once(once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    });
}

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

__device__ __forceinline__ uint32_t fastdiv(uint32_t n, uint32_t magic)
{
    return magic ? __umulhi(n, magic) : n; // magic = ceil(2^32 / d), 0 for d == 1
}

// Streaming (non-temporal) 8-byte accesses for tensors that are written or read once per launch and
// are far larger than the L2: they leave the cache to the operands that are reused.
__device__ __forceinline__ void store_stream8(void *p, uint2 v)
{
    __builtin_nontemporal_store(__builtin_bit_cast(unsigned long long, v), reinterpret_cast<unsigned long long *>(p));
}
__device__ __forceinline__ uint2 load_stream8(const void *p)
{
    return __builtin_bit_cast(uint2, __builtin_nontemporal_load(reinterpret_cast<const unsigned long long *>(p)));
}
__device__ __forceinline__ void store_stream16(void *p, uint4 v)
{
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4 *>(p));
}
__device__ __forceinline__ uint4 load_stream16(const void *p)
{
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)));
}

__device__ __forceinline__ float act_apply(float v, int act)
{
    if (act == NPAS_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == NPAS_ACT_RELU6) return fminf(fmaxf(v, 0.0f), 6.0f);
    if (act == NPAS_ACT_HARDSWISH) return v * fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
    return v;
}

// The activations as one clamp to [lo, hi] (none: +-inf, ReLU: [0, inf), ReLU6: [0, 6]); hard-swish
// (v * clamp(v + 3, 0, 6) / 6) is that clamp of v + 3 times v / 6, behind a wave-uniform flag.
struct Clamp {
    float lo, hi;
    bool hs;
};
__device__ __forceinline__ Clamp clamp_of(int act)
{
    return Clamp{act == NPAS_ACT_NONE ? -INFINITY : 0.0f, (act == NPAS_ACT_RELU6 || act == NPAS_ACT_HARDSWISH) ? 6.0f : INFINITY,
                 act == NPAS_ACT_HARDSWISH};
}
// HSW: the launch has a hard-swish somewhere (a kernel body is instantiated with and without; without, an activation
// is the one clamp instruction and nothing else)
template <bool HSW = true> __device__ __forceinline__ float clampf(float v, Clamp c)
{
    if (HSW && c.hs) return v * __builtin_amdgcn_fmed3f(v + 3.0f, 0.0f, 6.0f) * (1.0f / 6.0f);
    return __builtin_amdgcn_fmed3f(v, c.lo, c.hi);
}

// fp32 -> 16-bit storage, round to nearest even.
template <int DT> __device__ __forceinline__ uint16_t to_storage(float v)
{
    if (DT == NPAS_BF16) {
        uint32_t u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40); // NaN stays NaN
        u += 0x7fffu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    } else {
        _Float16 h = (_Float16)v;
        return __builtin_bit_cast(uint16_t, h);
    }
}

// two fp32 -> one dword of two 16-bit storage values (lo, hi), round to nearest even
template <int DT> __device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    if (DT == NPAS_BF16) {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
    } else {
        typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, f16x2));
    }
}

template <int DT> __device__ __forceinline__ float from_storage(uint16_t b)
{
    if (DT == NPAS_BF16) return __uint_as_float((uint32_t)b << 16);
    return (float)__builtin_bit_cast(_Float16, b);
}

// element i of an activation tensor of storage type DT as fp32, and back
template <int DT> __device__ __forceinline__ float ld_act(const void *p, size_t i)
{
    if (DT == NPAS_F32) return reinterpret_cast<const float *>(p)[i];
    return from_storage<DT>(reinterpret_cast<const uint16_t *>(p)[i]);
}
template <int DT> __device__ __forceinline__ void st_act(void *p, size_t i, float v)
{
    if (DT == NPAS_F32) reinterpret_cast<float *>(p)[i] = v;
    else reinterpret_cast<uint16_t *>(p)[i] = to_storage<DT>(v);
}

template <int DT> __device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c)
{
    if (DT == NPAS_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run
// of logical ids so that workgroups sharing an activation patch share an L2.
__device__ __forceinline__ uint32_t xcd_remap(uint32_t wg, uint32_t nwg)
{
    uint32_t xcd = wg & 7u, idx = wg >> 3, q = nwg >> 3, r = nwg & 7u;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

// Direct global -> LDS load: 64 lanes x 16 bytes land lane-linearly in the 1 KB block at lds_addr; nothing is held in registers.
__device__ __forceinline__ void lds_dma16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(gptr)
                 : "memory"); // m0 is reserved: the compiler keeps nothing in it across statements
}

// "At most n vector-memory operations of this wave outstanding" for a wave-uniform n < 64
// (the instruction takes an immediate).
__device__ __forceinline__ void wait_vmcnt(uint32_t n)
{
#define NPAS_W(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
    switch (n) {
        NPAS_W(0) NPAS_W(1) NPAS_W(2) NPAS_W(3) NPAS_W(4) NPAS_W(5) NPAS_W(6) NPAS_W(7) NPAS_W(8) NPAS_W(9) NPAS_W(10)
        NPAS_W(11) NPAS_W(12) NPAS_W(13) NPAS_W(14) NPAS_W(15) NPAS_W(16) NPAS_W(17) NPAS_W(18) NPAS_W(19) NPAS_W(20)
        NPAS_W(21) NPAS_W(22) NPAS_W(23) NPAS_W(24) NPAS_W(25) NPAS_W(26) NPAS_W(27) NPAS_W(28) NPAS_W(29) NPAS_W(30)
        NPAS_W(31) NPAS_W(32) NPAS_W(33) NPAS_W(34) NPAS_W(35) NPAS_W(36) NPAS_W(37) NPAS_W(38) NPAS_W(39) NPAS_W(40)
        NPAS_W(41) NPAS_W(42) NPAS_W(43) NPAS_W(44) NPAS_W(45) NPAS_W(46) NPAS_W(47) NPAS_W(48) NPAS_W(49) NPAS_W(50)
        NPAS_W(51) NPAS_W(52) NPAS_W(53) NPAS_W(54) NPAS_W(55) NPAS_W(56) NPAS_W(57) NPAS_W(58) NPAS_W(59) NPAS_W(60)
        NPAS_W(61) NPAS_W(62)
    default: asm volatile("s_waitcnt vmcnt(63)" ::: "memory"); break;
    }
#undef NPAS_W
}

} // namespace npas

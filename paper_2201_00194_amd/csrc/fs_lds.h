// Device helpers shared by the LDS-staged kernels: absolute LDS addressing and explicit
// address spaces for pointers that arrive inside descriptors.
#ifndef FS_LDS_H
#define FS_LDS_H

#include "fs_internal.h"

namespace fs {

extern __shared__ __attribute__((aligned(16))) unsigned char fs_lds[];   // sized at launch

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// LDS accesses by absolute byte address (the dynamic LDS block starts at address 0: the
// kernel has no static LDS).
// Pointers that arrive inside a descriptor are generic to the compiler; FS_GLOBAL / FS_CONST
// tell it they are global memory (plain global loads that do not tie up the LDS counter) or
// read-only uniform data (scalar loads).
#if defined(__HIP_DEVICE_COMPILE__)
#define FS_LDS_PTR(T, a) ((__attribute__((address_space(3))) T *)(uint32_t)(a))
#define FS_GLOBAL(T, p) ((__attribute__((address_space(1))) T *)(uintptr_t)(p))
#define FS_CONST(T, p) ((__attribute__((address_space(4))) const T *)(uintptr_t)(p))
#else
#define FS_LDS_PTR(T, a) ((T *)(uintptr_t)(a))   // host pass only parses the kernels
#define FS_GLOBAL(T, p) ((T *)(uintptr_t)(p))
#define FS_CONST(T, p) ((const T *)(uintptr_t)(p))
#endif
static __device__ __forceinline__ u32x2 lds_u2(uint32_t a) { return *FS_LDS_PTR(const u32x2, a); }
static __device__ __forceinline__ float lds_f(uint32_t a) { return *FS_LDS_PTR(const float, a); }
static __device__ __forceinline__ uint32_t lds_u(uint32_t a) { return *FS_LDS_PTR(const uint32_t, a); }
static __device__ __forceinline__ void lds_store_u4(uint32_t a, u32x4 v) { *FS_LDS_PTR(u32x4, a) = v; }
static __device__ __forceinline__ void lds_store_f(uint32_t a, float v) { *FS_LDS_PTR(float, a) = v; }
static __device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

static __device__ __forceinline__ uint32_t lds_u16(uint32_t a) { return *FS_LDS_PTR(const uint16_t, a); }

// Linear copy global -> LDS without registers: every wavefront-wide group of 64 consecutive
// 16-byte pieces (1 KB) goes out as one load whose data the memory pipeline writes straight to
// LDS, lane l's piece at dst + 16*l (gfx950).  Wavefront `wave` of `n_waves` issues groups wave,
// wave + n_waves, ...; returns the number of pieces covered (n16 rounded down to 64) -- the
// caller copies the rest through registers.  Nothing is waited for: lds_direct_wait() before
// the barrier that publishes the data.  `dst` must be the same in all lanes.
// `src`: what FS_GLOBAL(const u32x4, ...) gives.
template <class P>
static __device__ __forceinline__ int lds_fill_direct(P src, uint32_t dst, int n16, int wave, int n_waves,
                                                      int lane)
{
    const int n_groups = n16 >> 6;
#if defined(__HIP_DEVICE_COMPILE__)
    for (int g = wave; g < n_groups; g += n_waves)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(src + (g << 6) + lane),
            (__attribute__((address_space(3))) void *)(uint32_t)(dst + 1024u * (uint32_t)g), 16, 0, 0);
#else
    (void)src; (void)dst; (void)wave; (void)n_waves; (void)lane;   // host pass only parses the kernels
#endif
    return n_groups << 6;
}

static __device__ __forceinline__ void lds_direct_wait()
{
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_s_waitcnt(0);
#endif
}

// acc += B parked values, `stride` bytes apart from LDS address `va` on, in that order: all B
// loads go out before the first add (their addresses are immediates), so the ordered sum
// exposes the LDS latency once per call.  The caller takes the largest B that fits first.
template <int B>
__device__ __forceinline__ void ordered_add(float &acc, uint32_t &va, uint32_t stride)
{
    float v[B];
#pragma unroll
    for (int k = 0; k < B; ++k)
        v[k] = lds_f(va + (uint32_t)k * stride);
#pragma unroll
    for (int k = 0; k < B; ++k)
        acc = acc + v[k];
    va += (uint32_t)B * stride;
}

// The same for n values, n >= 0.
__device__ __forceinline__ void ordered_add_n(float &acc, uint32_t va, uint32_t stride, int n)
{
    while (n >= 32) {
        ordered_add<32>(acc, va, stride);
        n -= 32;
    }
    if (n >= 24) {
        ordered_add<24>(acc, va, stride);
        n -= 24;
    }
    if (n >= 16) {
        ordered_add<16>(acc, va, stride);
        n -= 16;
    }
    if (n >= 8) {
        ordered_add<8>(acc, va, stride);
        n -= 8;
    }
    if (n >= 4) {
        ordered_add<4>(acc, va, stride);
        n -= 4;
    }
    if (n >= 2) {
        ordered_add<2>(acc, va, stride);
        n -= 2;
    }
    if (n >= 1)
        ordered_add<1>(acc, va, stride);
}

}  // namespace fs
#endif

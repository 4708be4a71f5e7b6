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

}  // namespace fs
#endif

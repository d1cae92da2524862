// Shared pieces of the bf16 MFMA kernels (decode-shaped tiles, streaming kernels): the 16-byte operand type,
// loads, the 16x16x32 MFMA, the split of fp32 values into two bf16 terms, a block of zeros.
//
// Lane roles in v_mfma_f32_16x16x32_bf16 (D = A*B + C, A 16x32, B 32x16):
//   lane l supplies A[row l%16][k 8*(l/16) .. +7] and B[k 8*(l/16) .. +7][col l%16]
//   and receives D[row 4*(l/16)+i][col l%16], i = 0..3.
#pragma once
#include "device_util.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

union op16 {            // one 16-byte MFMA operand
    uint4 u;
    bf16x8 v;
};

// 16-byte load from global memory.  Pointers fetched from a pointer table cannot be traced back to a
// kernel argument by the compiler, which would make their loads flat ones (counted as LDS traffic too,
// so that waits on them are coarse); the address space is therefore stated here.
__device__ __forceinline__ uint4 ld16(const bf16_t* p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const u32x4 r = *(const __attribute__((address_space(1))) u32x4*)(uintptr_t)p;
    return uint4{r[0], r[1], r[2], r[3]};
#else       // the host pass only parses device functions
    return *reinterpret_cast<const uint4*>(p);
#endif
}
__device__ __forceinline__ uint4 ld16_global(const bf16_t* p) { return ld16(p); }

// the same for data that is read (or written) exactly once by the whole launch: marked non-temporal, so that
// it does not displace what the launch re-reads (adapter matrices) from the caches
__device__ __forceinline__ uint4 ld16_stream(const bf16_t* p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const u32x4 r = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4*)(uintptr_t)p);
    return uint4{r[0], r[1], r[2], r[3]};
#else
    return *reinterpret_cast<const uint4*>(p);
#endif
}
__device__ __forceinline__ void st16_stream(bf16_t* p, uint4 val)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const u32x4 r = {val.x, val.y, val.z, val.w};
    __builtin_nontemporal_store(r, (__attribute__((address_space(1))) u32x4*)(uintptr_t)p);
#else
    *reinterpret_cast<uint4*>(p) = val;
#endif
}

__device__ __forceinline__ floatx4 mfma(const op16& a, const op16& b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

static __device__ __align__(256) uint32_t lora_zero_block[64];       // what masked-out loads read (never written)
__device__ __forceinline__ void split_bf16(const float* f, op16& hi, op16& lo)
{
    uint32_t h[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const bf16_t hb = f32_to_bf16(f[i]);
        h[i] = hb;
        l[i] = f32_to_bf16(f[i] - bf16_to_f32(hb));
    }
    hi.u = uint4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    lo.u = uint4{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
}

// NP = number of v parts when known at compile time (0: read it from vsp, up to 4)

// Device helpers for IEEE half-precision payloads, shared by the FP16 contrast
// kernels and the half-payload mode of the COVAP path.
#ifndef COVAP_HALF_UTIL_H
#define COVAP_HALF_UTIL_H

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

namespace covap_dev {

// Pins a value in a register.  Without it the compiler folds fp16(fma(c, r, g))
// into one v_fma_mixlo_f16, which rounds the exact sum straight to fp16 and so
// differs from "round to fp32, then to fp16" whenever the fp32 value is a tie.
__device__ __forceinline__ float pinned(float x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// Two fp32 values to two halves in one word: round to nearest even; fp16
// denormals are produced, overflow gives Inf.
__device__ __forceinline__ uint32_t pack_half2(float a, float b)
{
    return (uint32_t)__half_as_ushort(__float2half_rn(a)) |
           ((uint32_t)__half_as_ushort(__float2half_rn(b)) << 16);
}
__device__ __forceinline__ float half_lo(uint32_t w)
{
    return __half2float(__ushort_as_half((uint16_t)(w & 0xffffu)));
}
__device__ __forceinline__ float half_hi(uint32_t w)
{
    return __half2float(__ushort_as_half((uint16_t)(w >> 16)));
}

}  // namespace covap_dev

#endif  // COVAP_HALF_UTIL_H

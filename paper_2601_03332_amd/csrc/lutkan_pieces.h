// Device helper shared by the locate kernel (lutkan_kernels.hip) and the base-branch product (lutkan_base_gemm.hip).
#pragma once

#include <hip/hip_runtime.h>

// The three bf16 pieces (bit patterns) of an fp32 value, by truncation: a = h + m + l exactly for finite a (24
// significand bits = 3 x 8).  inf and NaN keep their class in the high piece, the other two are zero.
__device__ __forceinline__ void lutkan_cut3(float a, unsigned &h, unsigned &m, unsigned &l) {
  const unsigned ab = __float_as_uint(a);
  if ((ab & 0x7f800000u) == 0x7f800000u) {
    h = (ab >> 16) | ((ab & 0x007fffffu) ? 0x0040u : 0u);
    m = l = 0u;
    return;
  }
  const float r = a - __uint_as_float(ab & 0xffff0000u);          // exact: the low 16 significand bits
  const unsigned rb = __float_as_uint(r);
  const float r2 = r - __uint_as_float(rb & 0xffff0000u);         // exact: at most 8 significand bits are left
  h = ab >> 16;
  m = rb >> 16;
  l = __float_as_uint(r2) >> 16;
}

// Measurement aids of liblutkan: kernels of known work, one per resource the LUT layer forward can be bound by
// (vector-ALU FMA issue, the issue rate of the tiled kernel's own instruction mix, LDS read bandwidth, L2 read
// bandwidth, HBM read bandwidth).  A caller times a launch
// and divides the reported work by the duration to get the rate this machine actually sustains, which is what
// the roofline terms of the layer kernels are compared with.  They are not part of the method.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lutkan_internal.h"

using lutkan::fail;

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 1024;     // 16 waves, like the tiled layer kernels
constexpr int kFmaChains = 16;          // independent FMA chains per thread (hides the FMA latency at 4 waves / SIMD)
constexpr int kLdsProbeBytes = 64 * 1024;
constexpr int kL2ProbeBytes = 2 * 1024 * 1024;   // per pass; fits every XCD's L2, exceeds every CU's L1

// fp32 FMA issue rate: every lane runs kFmaChains dependent chains of `iters` FMAs (non-packed form).  The compiler
// emits the three-operand encoding with one scalar operand (x = x * a + b), which issues every 4.1-4.3 cycles per wave
// and SIMD like the permutes, packed-fp16 and mixed-precision instructions of the layer kernels: the yardstick for
// their vector-instruction count.  (The two-operand v_fmac_f32 on registers alone issues every 2.8 cycles.)
__global__ __launch_bounds__(kProbeThreads) void probe_valu_fma_kernel(float *sink, int iters, float a, float b) {
  float x[kFmaChains];
#pragma unroll
  for (int c = 0; c < kFmaChains; ++c) x[c] = (float)(threadIdx.x + c);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kFmaChains; ++c) x[c] = fmaf(x[c], a, b);
  }
  float s = 0.0f;
#pragma unroll
  for (int c = 0; c < kFmaChains; ++c) s += x[c];
  if (s == 123456.789f) sink[0] = s;     // keeps the chains alive; practically never taken
}

// The same count of fp32 FMAs in the two-operand encoding on registers only (x += b * y, y another running value):
// on gfx950 this form issues every 2.8 cycles per wave and SIMD, i.e. above the 4-cycle rate that every other
// instruction of the layer kernels has.  Reported beside the rate above so that nobody takes the 4-cycle figure for
// the ceiling of the fp32 units.
__global__ __launch_bounds__(kProbeThreads) void probe_valu_fmac_kernel(float *sink, int iters, float b) {
  float x[kFmaChains];
#pragma unroll
  for (int c = 0; c < kFmaChains; ++c) x[c] = (float)(threadIdx.x + c) * 1e-3f;
  float bv = b;
  asm volatile("" : "+v"(bv));                         // the multiplier in a vector register
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kFmaChains; ++c) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[c]) : "v"(bv), "v"(x[(c + 1) % kFmaChains]));
  }
  float s = 0.0f;
#pragma unroll
  for (int c = 0; c < kFmaChains; ++c) s += x[c];
  if (s == 123456.789f) sink[0] = s;
}

// Issue rate of the instruction mix of the tiled LUT kernel (int8 codes, value_repr = phi): per row step a lane
// issues 2 16-bit multiply-adds (addresses), 4 byte permutes, 4 packed-fp16 adds, 4 mixed-precision FMAs and 4 fp32
// FMAs, with the data dependences of the kernel (permutes -> packed adds -> mixed FMAs -> FMAs, four columns side by
// side).  On gfx950 these kinds do not all issue in four cycles per wave, so the rate of the mix, not the FMA rate,
// is the vector-ALU bound of that kernel.  The probe runs one 16-wave work-group per compute unit, like the kernel
// (the dynamic LDS it asks for, and never touches, keeps a second work-group off the compute unit).
constexpr int kMixLdsBytes = 96 * 1024;
constexpr int kMixInstructionsPerStep = 18;

__global__ __launch_bounds__(kProbeThreads) void probe_valu_mix_kernel(float *sink, int iters, unsigned seed, float w) {
  unsigned rec = seed + threadIdx.x, c0 = seed * 3u + threadIdx.x, c1 = seed * 7u + threadIdx.x;
  unsigned base0 = threadIdx.x * 4u, base1 = threadIdx.x * 16u;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const float alpha[4] = {w, w * 0.5f, w * 0.25f, w * 0.125f};
  const unsigned bias = 0x00800080u, rows = 64u;
  for (int it = 0; it < iters; ++it) {
    unsigned a0, a1, q0lo, q0hi, q1lo, q1hi, dlo, dhi;
    float t0, t1, t2, t3;
    asm volatile("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[0,0,0,0]" : "=v"(a0) : "v"(rec), "v"(rows), "v"(base0));
    asm volatile("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(a1) : "v"(rec), "v"(rows), "v"(base1));
    asm volatile("v_perm_b32 %0, %1, %1, %2" : "=v"(q0lo) : "v"(c0), "v"(0x0c010c00u));
    asm volatile("v_perm_b32 %0, %1, %1, %2" : "=v"(q0hi) : "v"(c0), "v"(0x0c030c02u));
    asm volatile("v_perm_b32 %0, %1, %1, %2" : "=v"(q1lo) : "v"(c1), "v"(0x0c010c00u));
    asm volatile("v_perm_b32 %0, %1, %1, %2" : "=v"(q1hi) : "v"(c1), "v"(0x0c030c02u));
    asm volatile("v_pk_add_f16 %0, %1, %2 neg_lo:[0,1] neg_hi:[0,1]" : "=v"(dlo) : "v"(q1lo), "v"(q0lo));
    asm volatile("v_pk_add_f16 %0, %1, %2 neg_lo:[0,1] neg_hi:[0,1]" : "=v"(dhi) : "v"(q1hi), "v"(q0hi));
    asm volatile("v_pk_add_f16 %0, %0, %1 neg_lo:[0,1] neg_hi:[0,1]" : "+v"(q0lo) : "v"(bias));
    asm volatile("v_pk_add_f16 %0, %0, %1 neg_lo:[0,1] neg_hi:[0,1]" : "+v"(q0hi) : "v"(bias));
    asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,1,1]" : "=v"(t0) : "v"(w), "v"(dlo), "v"(q0lo));
    asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,1,1] op_sel_hi:[0,1,1]" : "=v"(t1) : "v"(w), "v"(dlo), "v"(q0lo));
    asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[0,1,1]" : "=v"(t2) : "v"(w), "v"(dhi), "v"(q0hi));
    asm volatile("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,1,1] op_sel_hi:[0,1,1]" : "=v"(t3) : "v"(w), "v"(dhi), "v"(q0hi));
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[0]) : "v"(alpha[0]), "v"(t0));
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[1]) : "v"(alpha[1]), "v"(t1));
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[2]) : "v"(alpha[2]), "v"(t2));
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[3]) : "v"(alpha[3]), "v"(t3));
    // the next step's "loads" are this step's addresses: everything above stays live and changes every step
    c0 = a0;
    c1 = a1;
    rec = a0 ^ a1;
  }
  if (acc[0] + acc[1] + acc[2] + acc[3] == 123456.789f) sink[0] = acc[0];
}

// LDS read bandwidth: a work-group fills 64 KiB of LDS once, then every lane reads 16 bytes per step, lanes on
// consecutive addresses (conflict-free), walking the four 16 KiB quarters of the buffer.
__global__ __launch_bounds__(kProbeThreads) void probe_lds_read_kernel(const float *src, float *sink, int iters) {
  extern __shared__ __align__(16) unsigned char lds[];
  f32x4 *cells = reinterpret_cast<f32x4 *>(lds);
  for (int v = threadIdx.x; v < kLdsProbeBytes / 16; v += kProbeThreads)
    cells[v] = *reinterpret_cast<const f32x4 *>(src + 4 * (v & 1023));
  __syncthreads();
  typedef const __attribute__((address_space(3))) f32x4 *lds_vec;
  unsigned addr = (unsigned)(uintptr_t)(lds_vec)(cells + threadIdx.x);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    asm volatile("" : "+v"(addr));          // opaque to the optimiser: the four reads are issued again every pass
#pragma unroll
    for (int q = 0; q < 4; ++q) acc += *(lds_vec)(uintptr_t)(addr + q * (kProbeThreads * 16));
  }
  if (acc.x + acc.y + acc.z + acc.w == 123456.789f) sink[0] = acc.x;
}

// L2 read bandwidth: every work-group streams the same 2 MiB (coalesced 16-byte loads) `iters` times; after the
// first pass the data sits in every XCD's L2 and is too large for a CU's L1.
// HBM read bandwidth: the same kernel over a buffer far larger than the caches, each 16-byte vector read once per pass.
__global__ __launch_bounds__(kProbeThreads) void probe_global_read_kernel(const f32x4 *src, float *sink, int64_t n16_per_group,
                                                                           int64_t group_stride16, int iters) {
  const f32x4 *base = src + (int64_t)blockIdx.x * group_stride16;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    for (int64_t v = threadIdx.x; v < n16_per_group; v += 4 * kProbeThreads) {
      // four independent loads per step keep enough requests in flight
      f32x4 r[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int64_t e = v + (int64_t)q * kProbeThreads;
        r[q] = (e < n16_per_group) ? base[e] : f32x4{0.f, 0.f, 0.f, 0.f};
      }
      acc += (r[0] + r[1]) + (r[2] + r[3]);
    }
  }
  if (acc.x + acc.y + acc.z + acc.w == 123456.789f) sink[0] = acc.x;
}

}  // namespace

extern "C" int lutkan_probe_launch(int32_t kind, void *buffer, size_t buffer_bytes, int32_t iters, double *work_out,
                                   void *hip_stream) {
  const char *who = "lutkan_probe_launch";
  if (!buffer || !work_out) return fail(LUTKAN_EINVAL, "%s: null buffer or work_out", who);
  if ((reinterpret_cast<uintptr_t>(buffer) & 15) != 0) return fail(LUTKAN_EINVAL, "%s: buffer must be 16-byte aligned", who);
  if (iters < 1 || iters > (1 << 20)) return fail(LUTKAN_EINVAL, "%s: iters=%d outside [1, 2^20]", who, iters);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  float *fbuf = static_cast<float *>(buffer);
  const int groups = 256 * 8;                 // eight work-groups per compute unit's worth of work
  switch (kind) {
    case LUTKAN_PROBE_VALU_FMA: {
      if (buffer_bytes < 16) return fail(LUTKAN_ESHAPE, "%s: buffer too small", who);
      hipLaunchKernelGGL(probe_valu_fma_kernel, dim3(groups), dim3(kProbeThreads), 0, s, fbuf, iters, 0.999f, 0.001f);
      *work_out = 2.0 * kFmaChains * (double)iters * kProbeThreads * groups;            // flop
      break;
    }
    case LUTKAN_PROBE_VALU_FMAC: {
      if (buffer_bytes < 16) return fail(LUTKAN_ESHAPE, "%s: buffer too small", who);
      hipLaunchKernelGGL(probe_valu_fmac_kernel, dim3(groups), dim3(kProbeThreads), 0, s, fbuf, iters, 1e-9f);
      *work_out = 2.0 * kFmaChains * (double)iters * kProbeThreads * groups;            // flop
      break;
    }
    case LUTKAN_PROBE_VALU_MIX: {
      if (buffer_bytes < 16) return fail(LUTKAN_ESHAPE, "%s: buffer too small", who);
      static bool raised_mix = false;
      if (!raised_mix) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(probe_valu_mix_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMixLdsBytes);
        if (e != hipSuccess) return fail(LUTKAN_EHIP, "hipFuncSetAttribute(LDS): %s", hipGetErrorString(e));
        raised_mix = true;
      }
      hipLaunchKernelGGL(probe_valu_mix_kernel, dim3(groups), dim3(kProbeThreads), kMixLdsBytes, s, fbuf, iters, 12345u, 0.37f);
      *work_out = (double)kMixInstructionsPerStep * (double)iters * kProbeThreads * groups;   // lane-instructions
      break;
    }
    case LUTKAN_PROBE_LDS_READ: {
      if (buffer_bytes < 16 * 1024 + 16) return fail(LUTKAN_ESHAPE, "%s: buffer needs 16 KiB + 16 B", who);
      static bool raised = false;
      if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(probe_lds_read_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsProbeBytes);
        if (e != hipSuccess) return fail(LUTKAN_EHIP, "hipFuncSetAttribute(LDS): %s", hipGetErrorString(e));
        raised = true;
      }
      hipLaunchKernelGGL(probe_lds_read_kernel, dim3(groups), dim3(kProbeThreads), kLdsProbeBytes, s, fbuf + 4, fbuf, iters);
      *work_out = 4.0 * 16.0 * (double)iters * kProbeThreads * groups;                  // bytes read from LDS
      break;
    }
    case LUTKAN_PROBE_L2_READ: {
      if (buffer_bytes < (size_t)kL2ProbeBytes + 16) return fail(LUTKAN_ESHAPE, "%s: buffer needs 2 MiB + 16 B", who);
      hipLaunchKernelGGL(probe_global_read_kernel, dim3(groups), dim3(kProbeThreads), 0, s,
                         reinterpret_cast<const f32x4 *>(fbuf + 4), fbuf, (int64_t)(kL2ProbeBytes / 16), (int64_t)0, iters);
      *work_out = (double)kL2ProbeBytes * iters * groups;                               // bytes read through L2
      break;
    }
    case LUTKAN_PROBE_HBM_READ: {
      if (buffer_bytes < ((size_t)1 << 30)) return fail(LUTKAN_ESHAPE, "%s: buffer must be at least 1 GiB to defeat the caches", who);
      const int64_t per_group16 = (int64_t)((buffer_bytes - 16) / 16 / groups);
      hipLaunchKernelGGL(probe_global_read_kernel, dim3(groups), dim3(kProbeThreads), 0, s,
                         reinterpret_cast<const f32x4 *>(fbuf + 4), fbuf, per_group16, per_group16, iters);
      *work_out = 16.0 * (double)per_group16 * groups * iters;                          // bytes read from HBM
      break;
    }
    default:
      return fail(LUTKAN_EINVAL, "%s: unknown kind %d", who, kind);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: %s", who, hipGetErrorString(e));
  return LUTKAN_OK;
}

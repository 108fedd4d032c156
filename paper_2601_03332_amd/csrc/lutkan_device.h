// Device helpers and launch helpers shared by the LUT kernels (lutkan_kernels.hip) and the B-spline kernels
// (bspline_kernels.hip) of liblutkan.  Everything sits in an unnamed namespace: each of the two files gets its own
// copy, nothing here is visible outside the library.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <type_traits>

#include "lutkan_internal.h"

using lutkan::fail;

namespace {

constexpr int kWave = 64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte load/store
typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr float kTwoTo24 = 16777216.0f;
constexpr float kTwoToMinus24 = 1.0f / 16777216.0f;

// A LUT lookup record, one per (input, row), stored [input][row].  value_repr = phi: 8 bytes
//   x = table row k*L+l0 in bits 0..15, segment k in bits 16..31   (the all-zero rows K*L and K when masked)
//   y = interpolation weight w as fp32 bits                        (0 when masked, NaN for a NaN input)
// value_repr = spline_component: 16 bytes, the same two words, then
//   z = SiLU(x) of the raw input as fp32 bits, w = 0.
// The two 16-bit halves of x are what the tiled kernel scales (by the bytes of a code row resp. a parameter row)
// and adds to a lane's column address, one multiply-add each; nothing else is computed per row.

// The largest float below a finite t: nextafter(t, -inf), the safe upper clip value of Eq. 13 in half-open mode.
__device__ __forceinline__ float next_float_below(float t) {
  const unsigned bits = __float_as_uint(t);
  if (t > 0.0f) return __uint_as_float(bits - 1u);
  if (t < 0.0f) return __uint_as_float(bits + 1u);
  return __uint_as_float(0x80000001u);                 // below +-0: the smallest negative subnormal
}

// Asynchronous global -> LDS copy of 16 bytes per lane (gfx950 LDS-DMA form of the global load): the wave's active
// lanes each fetch 16 bytes from (a wave-uniform 64-bit base in scalar registers) + (their own 32-bit byte offset)
// and the data lands at lds_dst + 16*lane.  With the lane offsets of a wave fixed (16 * lane) the address of every
// copy of a walk is scalar arithmetic only: no vector instruction is spent on staging.
// lds_dst must be wave-uniform (it travels in M0; one wait state separates the M0 write from the load).
// Completion is tracked by vmcnt like any other vector memory load.  The copy is written out as instructions
// rather than through the compiler's builtin: for the builtin the compiler makes the wave wait for all its
// outstanding copies before any later LDS read and before every barrier, because it cannot tell the stage
// buffers apart; here the kernel waits itself (wait_all_vector_loads) before it reads what a copy wrote.
//
// M0: by default the helper overwrites it and declares it clobbered, which is sound as long as nothing else in these
// kernels keeps a value in M0 across a copy (a CPU-side test checks the generated code for that).  Should a compiler
// ever start doing so, set kLdsDmaPreservesM0: the copy then saves M0 in a scalar register and restores it (measured
// 1.3 % slower on the widest layer).
constexpr bool kLdsDmaPreservesM0 = false;

__device__ __forceinline__ void copy16_global_to_lds_at(const void *uniform_base, unsigned lane_byte_offset, void *lds_dst) {
  const unsigned dst = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds_dst);
  if constexpr (kLdsDmaPreservesM0) {
    unsigned saved;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved) : "s"(dst), "v"(lane_byte_offset), "s"(uniform_base) : "memory");
  } else {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(lane_byte_offset), "s"(uniform_base) : "m0", "memory");
  }
}

__device__ __forceinline__ void wait_all_vector_loads() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0)
// Waits until at most n (wave-uniform, 0..7; more counts as 0) of the wave's vector memory loads are outstanding.  The
// count is an immediate of the wait instruction, hence the switch.
__device__ __forceinline__ void wait_until_vector_loads_outstanding(int n) {
  switch (n) {
    case 1: __builtin_amdgcn_s_waitcnt(0x0f71); break;
    case 2: __builtin_amdgcn_s_waitcnt(0x0f72); break;
    case 3: __builtin_amdgcn_s_waitcnt(0x0f73); break;
    case 4: __builtin_amdgcn_s_waitcnt(0x0f74); break;
    case 5: __builtin_amdgcn_s_waitcnt(0x0f75); break;
    case 6: __builtin_amdgcn_s_waitcnt(0x0f76); break;
    case 7: __builtin_amdgcn_s_waitcnt(0x0f77); break;
    default: __builtin_amdgcn_s_waitcnt(0x0f70); break;
  }
}

// Work-group barrier that orders LDS traffic only (__syncthreads() also drains the wave's global-memory traffic).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Copies n16 16-byte vectors from gsrc (wave-uniform) to lds_dst with all NW waves of the work-group, 1 KiB per wave
// step: wave w takes the whole chunks w, w + NW, ...; the last, partial chunk goes to the wave whose turn it is.
// lane_off = 16 * lane.
template <int NW>
__device__ __forceinline__ void stage_slice(const unsigned char *gsrc, unsigned char *lds_dst, int n16, int wave, int lane, unsigned lane_off) {
  const int whole = n16 >> 6;
  for (int c = wave; c < whole; c += NW) copy16_global_to_lds_at(gsrc + c * 1024, lane_off, lds_dst + c * 1024);
  const int tail = n16 & 63;
  if (tail != 0 && wave == (whole % NW) && lane < tail) copy16_global_to_lds_at(gsrc + whole * 1024, lane_off, lds_dst + whole * 1024);
}

// Sums the n_split partial outputs of the tiled kernels in ascending chunk order (deterministic): y = sum_s part[s],
// or y = y + sum_s part[s] with `accumulate` (y then already holds the base branch of the layer).
__global__ __launch_bounds__(256) void sum_partials_kernel(const float *part, float *y, int64_t n, int n_split, int accumulate) {
  const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e + 3 < n && (n & 3) == 0) {                   // 16-byte path needs every chunk's base aligned
    f32x4 acc = *reinterpret_cast<const f32x4 *>(part + e);
#pragma unroll 8
    for (int s = 1; s < n_split; ++s) acc += *reinterpret_cast<const f32x4 *>(part + (int64_t)s * n + e);   // loads of 8 chunks in flight
    if (accumulate) acc = *reinterpret_cast<const f32x4 *>(y + e) + acc;
    *reinterpret_cast<f32x4 *>(y + e) = acc;
  } else {
    for (int64_t q = e; q < n && q < e + 4; ++q) {
      float acc = part[q];
      for (int s = 1; s < n_split; ++s) acc += part[(int64_t)s * n + q];
      y[q] = accumulate ? y[q] + acc : acc;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Host launchers.
// ------------------------------------------------------------------------------------------------
constexpr int kTileWaves = 16;          // waves per tiled work-group (1024 threads, one work-group per CU)
constexpr int kMaxTileRows = kTileWaves * 64;   // largest row tile of any tiled variant; Bp is a multiple of it
constexpr int kMaxTiledLds = lutkan::kLdsPerWorkGroup;

inline int64_t round_up(int64_t v, int64_t q) { return (v + q - 1) / q * q; }
inline int64_t padded_rows(int64_t B) { return round_up(B, kMaxTileRows); }
inline int lut_record_bytes(int value_repr) { return value_repr == LUTKAN_REPR_SPLINE_COMPONENT ? 16 : 8; }
inline size_t record_bytes(int d, int64_t Bp, int bytes_per_record) { return (size_t)round_up((int64_t)d * Bp * bytes_per_record, 256); }

int check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: %s", what, hipGetErrorString(e));
  return LUTKAN_OK;
}

enum { kLocate = 1, kEdges = 2 };      // the two phases of a forward call

int gather_jx_log2(int m) {
  int lg = 2;
  while ((1 << lg) < m && lg < 8) ++lg;
  return lg;
}

// Launch shape of the tiled kernels for B rows: NP row steps per wave (16/8/4/2/1, at most 64 rows per wave) and
// the number of chunks the d inputs are split into (each with its own work-groups and its own set of partial sums).
// Chosen by a small cost model, in microseconds, over every (NP, chunk count) pair:
//   one input of one work-group   max(0.55 + 0.11 * NP, slice bytes at 100 GB/s) + 0.1
//                                 (barrier and address set-up, NP row steps of 256 edges per wave, the slice's
//                                 global -> LDS copy when that is the longer of the two)
//   one work-group                3 + its inputs (pipeline fill, accumulator write-back); a wide form of the table
//                                 (16-bit codes: 0.095 * NP per input, fp32 values: 0.070 * NP) adds half its slice
//                                 at 21 GB/s to the fill
//   the launch                    rounds of 256 work-groups (one per compute unit), one after the other
//   the partial sums              4 + their bytes at 3 TB/s, when there is more than one chunk
//   a table of more than 128 MiB  at least its bytes at 21 GB/s per work-group and 5.3 TB/s in all (it streams from
//                                 HBM on every launch; smaller tables are served by the caches after the first)
// The constants come from the widest workload (2.4 us per input at NP = 16), a 64x1024 layer at NP = 4 (1.1 us) and
// sweeps over batch sizes of 78x16 ... 4096x256 layers; the model replaced a rule (largest row tile first, split the inputs until 256
// work-groups, at most 32 chunks) that lost up to 40 % on wide-input, narrow-output layers at a few hundred rows.
struct TilePlan {
  int np, n_split, chunk;
  double cost;       // the model's estimate for the launch (and its summing pass), microseconds
  bool hbm_bound;    // the estimate is the time the table takes to stream from HBM, not the work-groups' own time
};

// code_bytes: 1 for the table as compiled; 2 or 4 when the slices are those of a wide form of the table, whose row
// steps take fewer instructions.
inline double row_step_us(int code_bytes) { return code_bytes == 4 ? 0.070 : code_bytes == 2 ? 0.095 : 0.11; }
TilePlan plan_tiles(int64_t B, int d, int m, int n_tiles, int rps, int slice_bytes, int code_bytes = 1) {
  const int np_max = std::min(16, 64 / rps);
  const int max_split = std::max(1, std::min(128, d / 8));
  TilePlan best{np_max, 1, d, 1e300, false};
  double best_cost = 1e300;
  // a table beyond what the caches hold streams from HBM once per launch: about 21 GB/s per streaming work-group,
  // 5.3 TB/s for the whole chip
  const double table_bytes = (double)n_tiles * d * slice_bytes;
  const bool streams_from_hbm = table_bytes > 128.0 * 1024 * 1024;
  // a work-group's first slice arrives before it computes anything; the wide form's is twice as long (measured on a
  // 256x256 layer at 512 rows, 8 inputs per work-group: 0.030 -> 0.037 ms on the wide form)
  const double fill = 3.0 + (code_bytes > 1 ? 0.5 * slice_bytes / 21e3 : 0.0);
  for (int np = np_max; np >= 1; np >>= 1) {
    const int64_t rows = (int64_t)kTileWaves * rps * np;
    const int64_t groups = (B + rows - 1) / rows * n_tiles;
    const double per_input = std::max(0.55 + row_step_us(code_bytes) * np, slice_bytes / 100e3) + 0.1;
    // candidate chunk counts: 1 .. 8, then the counts that fill whole rounds of 256 work-groups, and the cap
    int candidates[16];
    int n_candidates = 0;
    for (int c = 1; c <= 8; ++c) candidates[n_candidates++] = c;
    for (int rounds = 1; rounds <= 4; ++rounds) candidates[n_candidates++] = (int)std::min<int64_t>(max_split, (256 * rounds + groups - 1) / groups);
    candidates[n_candidates++] = max_split;
    for (int q = 0; q < n_candidates; ++q) {
      const int want = std::min(candidates[q], max_split);
      const int chunk = (d + want - 1) / want;
      const int split = (d + chunk - 1) / chunk;      // no empty trailing chunks
      const double rounds = (double)((groups * split + 255) / 256);
      double cost = rounds * (fill + chunk * per_input);
      bool hbm_bound = false;
      if (streams_from_hbm) {         // ties go to the smaller row tile (fewer padding rows)
        // within one round of work-groups: once per row tile (measured at a few hundred to a few thousand rows);
        // over several rounds: once per round, the row tiles of a round walk the inputs together and share what
        // they read through the caches
        const double passes = rounds > 1.0 ? rounds : (double)(groups / n_tiles);
        const double stream = passes * table_bytes / std::min(5.3e6, 21e3 * (double)std::min<int64_t>(256, groups * split));
        hbm_bound = stream > cost;
        cost = std::max(cost, stream) + 0.01 * np;
      }
      if (split > 1) cost += 4.0 + (double)split * (double)B * m * 4.0 / 3e6;
      if (cost < best_cost) { best_cost = cost; best = TilePlan{np, split, chunk, cost, hbm_bound}; }
    }
  }
  return best;
}

// Launch shape of the gather kernels (lanes_per_row = m with one column per lane, a quarter of the padded width with
// four): the d inputs are cut into chunks (at least 4 inputs each, at most 64 chunks)
// until the launch has about a million threads: a thread's walk over its inputs is a chain of dependent reads,
// four inputs per round trip, so short chunks matter more than full compute units.
struct GatherPlan {
  int n_split, chunk;
};

GatherPlan plan_gather(int64_t B, int d, int lanes_per_row) {
  const int64_t threads = B * (int64_t)lanes_per_row;
  int64_t want = (threads >= (1 << 20)) ? 1 : ((1 << 20) + threads - 1) / threads;
  want = std::min<int64_t>(want, std::min(64, std::max(1, d / 4)));
  const int chunk = (int)((d + want - 1) / want);
  return GatherPlan{(d + chunk - 1) / chunk, chunk};
}

// The default cap on a kernel's dynamic LDS (64 KiB) is below the 160 KiB a gfx950 CU has.  Raising it is a
// per-kernel, per-device setting: one of these per kernel remembers which devices have it (bit = device ordinal).
struct LdsCap {
  std::atomic<uint64_t> devices{0};
};

template <typename Kern>
int raise_lds_cap(Kern kern, LdsCap *cap, const char *what) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: hipGetDevice: %s", what, hipGetErrorString(e));
  if (dev < 0 || dev >= 64) return fail(LUTKAN_EUNSUPPORTED, "%s: device ordinal %d", what, dev);
  const uint64_t bit = 1ull << dev;
  if (cap->devices.load(std::memory_order_acquire) & bit) return LUTKAN_OK;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxTiledLds);
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: hipFuncSetAttribute(LDS): %s", what, hipGetErrorString(e));
  cap->devices.fetch_or(bit, std::memory_order_release);
  return LUTKAN_OK;
}

template <typename Kern, typename Args>
int launch_with_lds(Kern kern, LdsCap *cap, const dim3 &grid, size_t lds, hipStream_t s, const Args &args, const char *what) {
  if (lds > (size_t)kMaxTiledLds) return fail(LUTKAN_EUNSUPPORTED, "%s: needs %zu bytes of LDS", what, lds);
  if (int rc = raise_lds_cap(kern, cap, what)) return rc;
  hipLaunchKernelGGL(kern, grid, dim3(kTileWaves * 64), lds, s, args);
  return check_launch(what);
}

// Records for every (input, padded row), then room for the partial sums when the inputs are split into chunks.
size_t tiled_workspace_bytes(int d, int m, int jt, int n_tiles, int64_t B, int bytes_per_record, int slice_bytes, int code_bytes = 1) {
  size_t bytes = record_bytes(d, padded_rows(B), bytes_per_record);
  const TilePlan tp = plan_tiles(B, d, m, n_tiles, 64 / (jt / 4), slice_bytes, code_bytes);
  // any of the kernels may run (tiled, gather with one column per lane, gather with four): room for the largest set
  const GatherPlan gp = plan_gather(B, d, m), gp4 = plan_gather(B, d, n_tiles * jt / 4);
  const int n_split = std::max(tp.n_split, std::max(gp.n_split, gp4.n_split));
  if (n_split > 1) bytes += (size_t)n_split * (size_t)B * (size_t)m * 4;
  return bytes;
}

}  // namespace

// Error statistics of the OOB evaluation protocol (Sec. 5.6, Sec. 6.5): |y - y_ref| over the outputs of the
// in-range samples (every input satisfies the domain predicate of Sec. 5.2) and of the OOB-only samples (at least
// one input does not), as sums, maxima and counts, in one pass over x, y and y_ref.
//
// One wave per row at a time: the 64 lanes read the row's inputs and outputs as contiguous runs, the row's subset is
// a wave-uniform flag, every lane keeps fp64 sums and maxima for both subsets.  A work-group writes one partial
// record; a second, single work-group kernel adds the partials in a fixed order, so the result does not depend on
// scheduling.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "lutkan_internal.h"

using lutkan::fail;

namespace {

constexpr int kStatWaves = 4;
constexpr int kStatRowsPerWave = 16;
constexpr int kStatRowsPerGroup = kStatWaves * kStatRowsPerWave;

struct Partial {
  double sum_in, sum_oob, max_in, max_oob;
  unsigned long long rows_in, rows_oob, nan_in, nan_oob;
};
static_assert(sizeof(Partial) == 64, "one partial record is 64 bytes");

struct Acc {
  double sum_in, sum_oob, max_in, max_oob;
  unsigned long long rows_in, rows_oob, nan_in, nan_oob;
};

__device__ __forceinline__ Acc empty_acc() { return Acc{0.0, 0.0, 0.0, 0.0, 0ull, 0ull, 0ull, 0ull}; }

__device__ __forceinline__ void merge(Acc &a, const Acc &b) {
  a.sum_in += b.sum_in;
  a.sum_oob += b.sum_oob;
  a.max_in = fmax(a.max_in, b.max_in);
  a.max_oob = fmax(a.max_oob, b.max_oob);
  a.rows_in += b.rows_in;
  a.rows_oob += b.rows_oob;
  a.nan_in += b.nan_in;
  a.nan_oob += b.nan_oob;
}

__device__ __forceinline__ Acc shuffle_down(const Acc &a, int off) {
  Acc o;
  o.sum_in = __shfl_down(a.sum_in, off, 64);
  o.sum_oob = __shfl_down(a.sum_oob, off, 64);
  o.max_in = __shfl_down(a.max_in, off, 64);
  o.max_oob = __shfl_down(a.max_oob, off, 64);
  o.rows_in = __shfl_down(a.rows_in, off, 64);
  o.rows_oob = __shfl_down(a.rows_oob, off, 64);
  o.nan_in = __shfl_down(a.nan_in, off, 64);
  o.nan_oob = __shfl_down(a.nan_oob, off, 64);
  return o;
}

__global__ __launch_bounds__(kStatWaves * 64) void error_stats_partial_kernel(const float *y, const float *y_ref, const float *x,
                                                                              int64_t B, int m, int d, float t0, float tK,
                                                                              const float *input_domain, int closed,
                                                                              Partial *partials) {
  __shared__ Acc s_acc[kStatWaves];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  Acc acc = empty_acc();
  for (int r = 0; r < kStatRowsPerWave; ++r) {
    const int64_t b = (int64_t)blockIdx.x * kStatRowsPerGroup + r * kStatWaves + wave;
    if (b >= B) break;                                  // wave-uniform
    // In(x) of Sec. 5.2 for every input of the row; NaN is out of domain
    int outside = 0;
    for (int i = lane; i < d; i += 64) {
      const float v = x[b * d + i];
      const float lo = input_domain ? input_domain[2 * i] : t0;
      const float hi = input_domain ? input_domain[2 * i + 1] : tK;
      const bool in = closed ? (v >= lo && v <= hi) : (v >= lo && v < hi);
      outside |= in ? 0 : 1;
    }
    const bool row_in = (__ballot(outside != 0) == 0ull);
    double sum = 0.0, mx = 0.0;
    unsigned long long nans = 0;
    for (int j = lane; j < m; j += 64) {
      const double e = fabs((double)y[b * m + j] - (double)y_ref[b * m + j]);
      if (e != e) { ++nans; continue; }
      sum += e;
      mx = fmax(mx, e);
    }
    if (row_in) {
      acc.nan_in += nans;
      acc.sum_in += sum;
      acc.max_in = fmax(acc.max_in, mx);
      if (lane == 0) ++acc.rows_in;
    } else {
      acc.nan_oob += nans;
      acc.sum_oob += sum;
      acc.max_oob = fmax(acc.max_oob, mx);
      if (lane == 0) ++acc.rows_oob;
    }
  }
  for (int off = 32; off > 0; off >>= 1) merge(acc, shuffle_down(acc, off));
  if (lane == 0) s_acc[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    Acc t = s_acc[0];
    for (int w = 1; w < kStatWaves; ++w) merge(t, s_acc[w]);
    Partial p;
    p.sum_in = t.sum_in; p.sum_oob = t.sum_oob; p.max_in = t.max_in; p.max_oob = t.max_oob;
    p.rows_in = t.rows_in; p.rows_oob = t.rows_oob; p.nan_in = t.nan_in; p.nan_oob = t.nan_oob;
    partials[blockIdx.x] = p;
  }
}

// MAE of a subset (Sec. 6.5 over the subsets of Sec. 5.6): the mean of its differences that are not NaN.
__device__ __forceinline__ double subset_mae(double sum_abs, unsigned long long rows, int m, unsigned long long nans) {
  const unsigned long long counted = rows * (unsigned long long)m - nans;
  return counted ? sum_abs / (double)counted : __builtin_nan("");
}

__global__ __launch_bounds__(256) void error_stats_final_kernel(const Partial *partials, int64_t n, int64_t B, int m,
                                                                lutkan_error_summary *out) {
  __shared__ Acc s_acc[256];
  Acc acc = empty_acc();
  for (int64_t q = threadIdx.x; q < n; q += 256) {      // fixed assignment of partials to threads
    const Partial p = partials[q];
    Acc t = empty_acc();
    t.sum_in = p.sum_in; t.sum_oob = p.sum_oob; t.max_in = p.max_in; t.max_oob = p.max_oob;
    t.rows_in = p.rows_in; t.rows_oob = p.rows_oob; t.nan_in = p.nan_in; t.nan_oob = p.nan_oob;
    merge(acc, t);
  }
  s_acc[threadIdx.x] = acc;
  __syncthreads();
  for (int half = 128; half > 0; half >>= 1) {          // fixed tree
    if ((int)threadIdx.x < half) merge(s_acc[threadIdx.x], s_acc[threadIdx.x + half]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const Acc t = s_acc[0];
    out->rows_in = t.rows_in; out->rows_oob = t.rows_oob; out->nan_in = t.nan_in; out->nan_oob = t.nan_oob;
    out->sum_abs_in = t.sum_in; out->sum_abs_oob = t.sum_oob;
    out->max_abs_in = t.max_in; out->max_abs_oob = t.max_oob;
    out->mae_in = subset_mae(t.sum_in, t.rows_in, m, t.nan_in);
    out->mae_oob = subset_mae(t.sum_oob, t.rows_oob, m, t.nan_oob);
    out->oob_any_frac = (double)t.rows_oob / (double)B;
  }
}

inline int64_t stat_groups(int64_t B) { return (B + kStatRowsPerGroup - 1) / kStatRowsPerGroup; }

}  // namespace

extern "C" size_t lutkan_error_stats_workspace_bytes(int64_t B) {
  return B > 0 ? (size_t)stat_groups(B) * sizeof(Partial) : 0;
}

extern "C" int lutkan_error_stats(const float *y, const float *y_ref, int64_t B, int32_t m, const float *x, int32_t d,
                                  float t0, float tK, const float *input_domain, int32_t boundary,
                                  lutkan_error_summary *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  const char *who = "lutkan_error_stats";
  if (!y || !y_ref || !x || !out) return fail(LUTKAN_EINVAL, "%s: null y / y_ref / x / out", who);
  if (B < 1 || m < 1 || d < 1) return fail(LUTKAN_EINVAL, "%s: B, m, d must be >= 1", who);
  if (!input_domain && !(t0 < tK)) return fail(LUTKAN_EINVAL, "%s: need t0 < tK", who);
  if (boundary != LUTKAN_HALF_OPEN && boundary != LUTKAN_CLOSED) return fail(LUTKAN_EINVAL, "%s: bad boundary_mode %d", who, boundary);
  if ((reinterpret_cast<uintptr_t>(out) & 7) != 0) return fail(LUTKAN_EINVAL, "%s: out must be 8-byte aligned", who);
  const size_t need = lutkan_error_stats_workspace_bytes(B);
  if (!workspace || workspace_bytes < need) return fail(LUTKAN_ESHAPE, "%s: workspace of %zu bytes, need %zu", who, workspace_bytes, need);
  if ((reinterpret_cast<uintptr_t>(workspace) & 15) != 0) return fail(LUTKAN_EINVAL, "%s: workspace must be 16-byte aligned", who);
  const int64_t groups = stat_groups(B);
  if (groups > 0x7fffffff) return fail(LUTKAN_EUNSUPPORTED, "%s: B too large", who);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Partial *partials = static_cast<Partial *>(workspace);
  hipLaunchKernelGGL(error_stats_partial_kernel, dim3((unsigned)groups), dim3(kStatWaves * 64), 0, s, y, y_ref, x, B, m, d, t0, tK,
                     input_domain, boundary == LUTKAN_CLOSED ? 1 : 0, partials);
  hipLaunchKernelGGL(error_stats_final_kernel, dim3(1), dim3(256), 0, s, partials, groups, B, (int)m, out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: %s", who, hipGetErrorString(e));
  return LUTKAN_OK;
}

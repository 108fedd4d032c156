// gfx950 kernels and launchers of the B-spline baseline layer of liblutkan (Sec. 3.2-3.3): the same work split as
// the LUT layer (lutkan_kernels.hip) -- per (row, input) the span and the four non-zero cubic basis values, then
// per edge four coefficient FMAs -- with the same tiling, staging and launch planning.
// The file is compiled with -ffp-contract=off; every fused multiply-add below is written out as fmaf().
#include "lutkan_device.h"

namespace {

// ------------------------------------------------------------------------------------------------
// B-spline baseline (Sec. 3.2-3.3).
// ------------------------------------------------------------------------------------------------
// A B-spline record is 32 bytes per (input, row), stored [input][row] as two 16-byte halves:
//   {byte offset of coefficient row k inside the input's coefficient slice, N0, N1, N2}, {N3, SiLU(x), 0, 0}
// where N0..N3 are the four non-zero cubic basis values (all 0 when masked, NaN for a NaN input) and SiLU(x) of
// the raw input is present for value_repr = spline_component (else 0).
struct SplineLocateArgs {
  const float *x;
  u32x4 *rec;            // [d][Bp][2]
  int64_t B, Bp;
  int32_t d, G, jt;
  int32_t closed, zero_spline, with_base;
  int32_t extended;      // the domain is the whole extended knot vector (else its inner G intervals)
  float tKs;
  float ext_knots[LUTKAN_MAX_K + 7];
  const float *input_ext_knots;   // [d][G+7]: one knot vector per input (then ext_knots and tKs are not used)
};

constexpr int kSplTile = 1024;  // (row, input) pairs per block of the B-spline locate kernel (32-byte records)

// Same tiling as the LUT locate kernel: blockIdx.x = tile of ROWS rows, blockIdx.y = tile of COLS inputs
// (COLS = 32 or 16, ROWS * COLS = 1024).  PERIN: one knot vector per input, the block keeps those of its COLS inputs.
template <int COLS, bool PERIN>
__global__ __launch_bounds__(256) void bspline_locate_kernel(const SplineLocateArgs a) {
  constexpr int ROWS = kSplTile / COLS;
  constexpr int PSTRIDE = LUTKAN_MAX_K + 13;
  static_assert(PSTRIDE % 2 == 1, "odd stride between the knot rows");
  __shared__ u32x4 s_rec[2][COLS][ROWS + 1];
  // the extended knots with three made-up knots on either side: s_pad[3 + r] = ext_knots[r].  A basis function that
  // exists (index 0 .. G+2) only ever touches real knots; the padding keeps the recursion of the others in bounds.
  __shared__ float s_pad[(PERIN ? COLS : 1) * PSTRIDE];
  const int tid = threadIdx.x;
  const int64_t b0 = (int64_t)blockIdx.x * ROWS;
  const int i0 = blockIdx.y * COLS;
  const int n = a.G + 7;
  for (int q = tid; q < (PERIN ? COLS : 1) * (n + 6); q += 256) {
    const int c = q / (n + 6), r = q - c * (n + 6);
    float v = 0.0f;
    if (!PERIN || i0 + c < a.d) {
      const float *src = PERIN ? a.input_ext_knots + (int64_t)(i0 + c) * n : a.ext_knots;
      if (r < 3) v = src[0] - (float)(3 - r) * (src[1] - src[0]);
      else if (r >= n + 3) v = src[n - 1] + (float)(r - n - 2) * (src[n - 1] - src[n - 2]);
      else v = src[r - 3];
    }
    s_pad[c * PSTRIDE + r] = v;
  }
  __syncthreads();
  const int first_knot = a.extended ? 0 : 3;           // domain knot kappa is extended knot first_knot + kappa
  const int segments = a.extended ? a.G + 6 : a.G;
  const int R = a.G + 3;
  {
    const int il = tid % COLS;
    const int i = i0 + il;
    const float *s_tau = s_pad + (PERIN ? il * PSTRIDE : 0) + 3;
    const float t0 = s_tau[first_knot], tK = s_tau[first_knot + segments];
    const float tKs = PERIN ? (a.closed ? tK : next_float_below(tK)) : a.tKs;
#pragma unroll 1
    for (int p = 0; p < kSplTile / 256; ++p) {
      const int bl = p * (256 / COLS) + tid / COLS;
      const int64_t b = b0 + bl;
      int k = 0;
      float n0 = 0.f, n1 = 0.f, n2 = 0.f, n3 = 0.f, base = 0.f;
      if (b < a.B && i < a.d) {
        const float x = a.x[b * a.d + i];
        if (a.with_base) base = __fdiv_rn(x, 1.0f + expf(-x));             // SiLU at the raw input, never masked
        const bool is_nan = (x != x);
        const bool inside = a.closed ? (x >= t0 && x <= tK) : (x >= t0 && x < tK);
        float xc = is_nan ? t0 : x;
        xc = (xc < t0) ? t0 : xc;
        xc = (xc > tKs) ? tKs : xc;
        for (int kappa = 1; kappa < segments; ++kappa) k += (s_tau[first_knot + kappa] <= xc) ? 1 : 0;
        // Cox-de Boor on the span mu = first_knot + k, non-zero entries only (Eq. 4-5); knots are distinct.
        const int mu = first_knot + k;
        const float *tau = s_tau + (mu - 3);        // tau[0..7] = ext_knots[mu-3 .. mu+4] (padding beyond the ends)
        float lower[5] = {0.f, 0.f, 0.f, 1.f, 0.f};
#pragma unroll
        for (int q = 1; q <= 3; ++q) {
          float next[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 3 - q; s <= 3; ++s) {
            const float left = (xc - tau[s]) / (tau[s + q] - tau[s]) * lower[s];
            const float right = (tau[s + q + 1] - xc) / (tau[s + q + 1] - tau[s + 1]) * lower[s + 1];
            next[s] = left + right;
          }
#pragma unroll
          for (int s = 0; s < 5; ++s) lower[s] = next[s];
        }
        // oob_policy zero_spline: all four weights 0 (the contribution is then exactly zero); NaN poisons them
        const bool masked = a.zero_spline && !inside && !is_nan;
        float gate = is_nan ? __builtin_nanf("") : (masked ? 0.0f : 1.0f);
        // at the last extended knot itself every basis function is 0 (half-open degree-0 indicator, Eq. 4)
        if (a.extended && xc == tK && !is_nan) gate = 0.0f;
        // lower[e] belongs to function mu-3+e.  The four coefficient rows read are first .. first+3 with first
        // clamped into [0, R-4]; a slot whose function does not exist (outer spans of the extended range) gets 0.
        const int first = min(max(mu - 3, 0), R - 4);
        const int shift = first - (mu - 3);          // -3 .. 3, 0 on the inner grid
        float slot[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int from = e + shift;
          float v = 0.0f;
#pragma unroll
          for (int f = 0; f < 4; ++f) v = (from == f) ? lower[f] : v;
          slot[e] = v * gate;
        }
        n0 = slot[0]; n1 = slot[1]; n2 = slot[2]; n3 = slot[3];
        k = first;
      }
      s_rec[0][il][bl] = u32x4{(unsigned)((k + a.with_base) * a.jt * 4), __float_as_uint(n0), __float_as_uint(n1), __float_as_uint(n2)};
      s_rec[1][il][bl] = u32x4{__float_as_uint(n3), __float_as_uint(base), 0u, 0u};
    }
    __syncthreads();
    const int bl2 = tid % ROWS;
#pragma unroll 1
    for (int p = 0; p < kSplTile / 256; ++p) {
      const int il2 = p * (256 / ROWS) + tid / ROWS;
      const int i2 = i0 + il2;
      if (i2 < a.d && b0 + bl2 < a.Bp) {
        const int64_t o = ((int64_t)i2 * a.Bp + b0 + bl2) * 2;
        a.rec[o] = s_rec[0][il2][bl2];
        a.rec[o + 1] = s_rec[1][il2][bl2];
      }
    }
  }
}

struct SplineEdgeArgs {
  const float *coef_table;   // [t][i][rows][jt]
  const u32x4 *rec;          // [d][Bp][2]
  float *y;
  int64_t B, Bp;
  int32_t d, m, rows;        // rows of a coefficient slice: R, plus the leading s_out*s_base row with spline_component
  int32_t with_base;
  int32_t jt, n_tiles;
  int32_t chunk;
  int64_t split_stride;
};

__global__ __launch_bounds__(256) void bspline_gather_kernel(const SplineEdgeArgs a, const int jx_log2) {
  constexpr int U = 4;                      // inputs per batch of independent loads, as in the LUT gather kernel
  const int jx = 1 << jx_log2;
  const int tx = threadIdx.x & (jx - 1);
  const int ty = threadIdx.x >> jx_log2;
  const int j = blockIdx.y * jx + tx;
  const int64_t b = (int64_t)blockIdx.x * (256 >> jx_log2) + ty;
  if (j >= a.m || b >= a.B) return;
  const int t = j / a.jt, jj = j - t * a.jt;
  const float *tile = a.coef_table + (size_t)t * a.d * a.rows * a.jt;
  const int i_begin = blockIdx.z * a.chunk;            // chunks of inputs and partial sums as in the LUT gather kernel
  const int i_end = min(a.d, i_begin + a.chunk);
  float acc = 0.0f;
  for (int i0 = i_begin; i0 < i_end; i0 += U) {
    u32x4 r0[U], r1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t o = ((int64_t)min(i0 + u, i_end - 1) * a.Bp + b) * 2;
      r0[u] = a.rec[o];
      r1[u] = a.rec[o + 1];
    }
    float cf[U][4], bg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float *sl = tile + (size_t)min(i0 + u, i_end - 1) * a.rows * a.jt;
      const float *c = sl + (r0[u].x >> 2) + jj;
#pragma unroll
      for (int q = 0; q < 4; ++q) cf[u][q] = c[q * a.jt];
      bg[u] = a.with_base ? sl[jj] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (i0 + u < i_end) {
        acc = fmaf(__uint_as_float(r0[u].y), cf[u][0], acc);
        acc = fmaf(__uint_as_float(r0[u].z), cf[u][1], acc);
        acc = fmaf(__uint_as_float(r0[u].w), cf[u][2], acc);
        acc = fmaf(__uint_as_float(r1[u].x), cf[u][3], acc);
        if (a.with_base) acc = fmaf(bg[u], __uint_as_float(r1[u].y), acc);
      }
    }
  }
  a.y[(int64_t)blockIdx.z * a.split_stride + b * a.m + j] = acc;
}

// Tiled B-spline kernel: same ownership and streaming as the LUT tiled kernel; the staged slice is the input's
// coefficient matrix c[R][JT]; per row four contiguous coefficient runs (rows k..k+3) are read and weighted by
// the row's four basis values.
template <int LPR, int NP, int NW, bool BASE>
__global__ __launch_bounds__(NW * 64) void bspline_tiled_kernel(const SplineEdgeArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int JT = 4 * LPR;
  constexpr int RPS = 64 / LPR;
  constexpr int RW = RPS * NP;
  static_assert(RW <= 64, "a wave's records for one input must fit two 1 KiB copy steps");
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sub = lane & (LPR - 1);
  const int hrow = lane / LPR;
  const int t = blockIdx.x % a.n_tiles;
  const int64_t rt = blockIdx.x / a.n_tiles;
  const int64_t b0 = rt * (NW * RW) + (int64_t)wave * RW;
  const int blob_bytes = a.rows * JT * 4;
  const int nvec = blob_bytes >> 4;

  float acc[NP][4];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[p][c] = 0.0f;

  const unsigned char *src = reinterpret_cast<const unsigned char *>(a.coef_table + (size_t)t * a.d * a.rows * JT);   // slice (t, 0); wave-uniform
  // a wave's RW 32-byte records are 2*RW consecutive 16-byte vectors: lanes 0..63 take the first 64, then the rest
  const unsigned char *rec_src = reinterpret_cast<const unsigned char *>(a.rec + b0 * 2);                            // wave-uniform
  const unsigned lane_off = lane * 16;
  unsigned char *rec_area = lds + 2 * blob_bytes + wave * (2 * RW * 32);
  auto stage_records = [&](int i, unsigned char *dst) {
    const unsigned char *g = rec_src + (int64_t)i * a.Bp * 32;
    if (lane < 2 * RW) copy16_global_to_lds_at(g, lane_off, dst);
    if (2 * RW > 64 && lane + 64 < 2 * RW) copy16_global_to_lds_at(g + 1024, lane_off, dst + 1024);
  };

  const int i_begin = blockIdx.y * a.chunk;
  const int i_end = min(a.d, i_begin + a.chunk);
  float *yout = a.y + (int64_t)blockIdx.y * a.split_stride;

  stage_slice<NW>(src + (size_t)i_begin * blob_bytes, lds, nvec, wave, lane, lane_off);
  stage_records(i_begin, rec_area);
  wait_all_vector_loads();
  __syncthreads();

  for (int i = i_begin; i < i_end; ++i) {
    const int cur = (i - i_begin) & 1;
    if (i + 1 < i_end) {
      stage_slice<NW>(src + (size_t)(i + 1) * blob_bytes, lds + (cur ^ 1) * blob_bytes, nvec, wave, lane, lane_off);
      stage_records(i + 1, rec_area + (cur ^ 1) * (RW * 32));
    }
    const unsigned char *rec_buf = rec_area + cur * (RW * 32) + hrow * 32;
    const unsigned char *col_coef = lds + cur * blob_bytes + sub * 16;
    // Same software pipeline as the LUT kernel: wait once per step, then issue the coefficient reads of step
    // p+1 and the record of step p+2, then do the arithmetic of step p.
    struct Rec { u32x4 a; float n3, base; };
    struct Coefs { f32x4 c[4]; };
    f32x4 base_gain = {0.f, 0.f, 0.f, 0.f};
    if (BASE) base_gain = *reinterpret_cast<const f32x4 *>(col_coef);        // row 0 of the slice: s_out*s_base
    auto read_rec = [&](int p) {
      Rec r;
      r.a = *reinterpret_cast<const u32x4 *>(rec_buf + p * (RPS * 32));
      if (BASE) {
        const f32x2 t2 = *reinterpret_cast<const f32x2 *>(rec_buf + p * (RPS * 32) + 16);
        r.n3 = t2.x;
        r.base = t2.y;
      } else {
        r.n3 = *reinterpret_cast<const float *>(rec_buf + p * (RPS * 32) + 16);
        r.base = 0.0f;
      }
      return r;
    };
    auto fetch = [&](const Rec &r) {
      Coefs f;
      const unsigned char *cp = col_coef + r.a.x;
#pragma unroll
      for (int q = 0; q < 4; ++q) f.c[q] = *reinterpret_cast<const f32x4 *>(cp + q * (JT * 4));
      return f;
    };
    Rec rc_cur = read_rec(0);
    Rec rc_nxt = read_rec(NP > 1 ? 1 : 0);
    Coefs f_cur = fetch(rc_cur);
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      Coefs f_nxt = f_cur;
      Rec rc_nn = rc_nxt;
      asm volatile("" ::"v"(f_cur.c[3]), "v"(rc_nxt.n3));                       // first touch of step p's data
      __builtin_amdgcn_sched_barrier(0);
      if (p + 2 < NP) rc_nn = read_rec(p + 2);
      if (p + 1 < NP) f_nxt = fetch(rc_nxt);
      __builtin_amdgcn_sched_barrier(0);
      const float n[4] = {__uint_as_float(rc_cur.a.y), __uint_as_float(rc_cur.a.z), __uint_as_float(rc_cur.a.w), rc_cur.n3};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc[p][0] = fmaf(n[q], f_cur.c[q].x, acc[p][0]);
        acc[p][1] = fmaf(n[q], f_cur.c[q].y, acc[p][1]);
        acc[p][2] = fmaf(n[q], f_cur.c[q].z, acc[p][2]);
        acc[p][3] = fmaf(n[q], f_cur.c[q].w, acc[p][3]);
      }
      if constexpr (BASE) {
        acc[p][0] = fmaf(base_gain.x, rc_cur.base, acc[p][0]);
        acc[p][1] = fmaf(base_gain.y, rc_cur.base, acc[p][1]);
        acc[p][2] = fmaf(base_gain.z, rc_cur.base, acc[p][2]);
        acc[p][3] = fmaf(base_gain.w, rc_cur.base, acc[p][3]);
      }
      __builtin_amdgcn_sched_barrier(0);
      rc_cur = rc_nxt;
      rc_nxt = rc_nn;
      f_cur = f_nxt;
    }
    wait_all_vector_loads();
    lds_barrier();
  }

  const int j = t * JT + sub * 4;
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const int64_t b = b0 + p * RPS + hrow;
    if (b < a.B) {
      if (j + 3 < a.m && (a.m & 3) == 0) {
        *reinterpret_cast<f32x4 *>(yout + b * a.m + j) = f32x4{acc[p][0], acc[p][1], acc[p][2], acc[p][3]};
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (j + c < a.m) yout[b * a.m + j + c] = acc[p][c];
      }
    }
  }
}

template <int LPR, int NP>
int launch_spline_tiled_np(const SplineEdgeArgs &ea, hipStream_t s) {
  constexpr int NW = kTileWaves;
  constexpr int RW = (64 / LPR) * NP;
  const int bytes = ea.rows * 4 * LPR * 4;
  const int64_t row_tiles = (ea.B + NW * RW - 1) / (NW * RW);
  if (row_tiles * ea.n_tiles > 0x7fffffffLL) return fail(LUTKAN_EUNSUPPORTED, "bspline_tiled_kernel: B * m too large for one launch");
  const dim3 grid((unsigned)(row_tiles * ea.n_tiles), (unsigned)((ea.d + ea.chunk - 1) / ea.chunk));
  const size_t lds = 2 * (size_t)bytes + (size_t)NW * 2 * RW * 32;
  static LdsCap raised, raised_base;
  if (ea.with_base) return launch_with_lds(bspline_tiled_kernel<LPR, NP, NW, true>, &raised_base, grid, lds, s, ea, "bspline_tiled_kernel");
  return launch_with_lds(bspline_tiled_kernel<LPR, NP, NW, false>, &raised, grid, lds, s, ea, "bspline_tiled_kernel");
}

template <int LPR>
int launch_spline_tiled(const SplineEdgeArgs &ea, int np, hipStream_t s) {
  constexpr int kMaxNp = (64 / (64 / LPR) < 16) ? 64 / (64 / LPR) : 16;
  if constexpr (kMaxNp >= 16) { if (np >= 16) return launch_spline_tiled_np<LPR, 16>(ea, s); }
  if constexpr (kMaxNp >= 8) { if (np >= 8) return launch_spline_tiled_np<LPR, 8>(ea, s); }
  if constexpr (kMaxNp >= 4) { if (np >= 4) return launch_spline_tiled_np<LPR, 4>(ea, s); }
  if constexpr (kMaxNp >= 2) { if (np >= 2) return launch_spline_tiled_np<LPR, 2>(ea, s); }
  return launch_spline_tiled_np<LPR, 1>(ea, s);
}

int launch_spline_tiled_jt(const SplineEdgeArgs &ea, int np, hipStream_t s) {
  switch (ea.jt) {
    case 128: return launch_spline_tiled<32>(ea, np, s);
    case 64: return launch_spline_tiled<16>(ea, np, s);
    case 32: return launch_spline_tiled<8>(ea, np, s);
    case 16: return launch_spline_tiled<4>(ea, np, s);
    case 8: return launch_spline_tiled<2>(ea, np, s);
    default: return launch_spline_tiled<1>(ea, np, s);
  }
}

int bspline_impl(const bspline_dev_layer *l, const float *x, int64_t B, float *y, void *workspace,
                 size_t workspace_bytes, void *hip_stream, const char *who, int phases) {
  if (!l) return fail(LUTKAN_EINVAL, "%s: null layer", who);
  if (!l->coef_table) return fail(LUTKAN_EINVAL, "%s: layer.coef_table is null", who);
  if (l->knots_per_input != 0 && l->knots_per_input != 1) return fail(LUTKAN_EINVAL, "%s: bad knots_per_input %d", who, l->knots_per_input);
  if (l->knots_per_input && (!l->input_ext_knots || (reinterpret_cast<uintptr_t>(l->input_ext_knots) & 3) != 0))
    return fail(LUTKAN_EINVAL, "%s: knots_per_input needs layer.input_ext_knots (device, 4-byte aligned)", who);
  if (l->d < 1 || l->m < 1 || l->G < 1 || l->G > LUTKAN_MAX_K) return fail(LUTKAN_EINVAL, "%s: bad d/m/G", who);
  if (l->degree != 3) return fail(LUTKAN_EUNSUPPORTED, "%s: only cubic splines", who);
  if (l->boundary != LUTKAN_HALF_OPEN && l->boundary != LUTKAN_CLOSED) return fail(LUTKAN_EINVAL, "%s: bad boundary_mode", who);
  if (l->oob != LUTKAN_CLIP_X && l->oob != LUTKAN_ZERO_SPLINE) return fail(LUTKAN_EINVAL, "%s: bad oob_policy", who);
  if (l->algo < LUTKAN_ALGO_AUTO || l->algo > LUTKAN_ALGO_TILED) return fail(LUTKAN_EINVAL, "%s: bad algo", who);
  if (l->value_repr != LUTKAN_REPR_PHI && l->value_repr != LUTKAN_REPR_SPLINE_COMPONENT) return fail(LUTKAN_EINVAL, "%s: bad value_repr", who);
  if (l->knot_span != LUTKAN_SPAN_DOMAIN && l->knot_span != LUTKAN_SPAN_EXTENDED) return fail(LUTKAN_EINVAL, "%s: bad knot_span", who);
  for (int r = 0; r < l->G + 6; ++r)
    if (!(l->ext_knots[r] < l->ext_knots[r + 1])) return fail(LUTKAN_EINVAL, "%s: knots not strictly increasing at %d", who, r);
  if (l->jt < 4 || l->jt > 128 || (l->jt & (l->jt - 1))) return fail(LUTKAN_EINVAL, "%s: bad jt", who);
  if (l->n_tiles != (l->m + l->jt - 1) / l->jt) return fail(LUTKAN_ESHAPE, "%s: n_tiles does not match m and jt", who);
  if ((reinterpret_cast<uintptr_t>(l->coef_table) & 15) != 0) return fail(LUTKAN_EINVAL, "%s: coef_table must be 16-byte aligned", who);
  if (l->coef_blob_bytes != lutkan::coef_slice_rows(l->G + 3, l->value_repr) * l->jt * 4) return fail(LUTKAN_ESHAPE, "%s: coef_blob_bytes does not match G, jt, value_repr", who);
  if (B < 0) return fail(LUTKAN_EINVAL, "%s: B < 0", who);
  if (B == 0) return LUTKAN_OK;
  if (((phases & kLocate) && !x) || ((phases & kEdges) && !y) || x == y) return fail(LUTKAN_EINVAL, "%s: null or aliased x / y", who);
  const size_t need = bspline_forward_workspace_bytes(l, B);
  if (!workspace || workspace_bytes < need) return fail(LUTKAN_ESHAPE, "%s: workspace of %zu bytes, need %zu", who, workspace_bytes, need);
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return fail(LUTKAN_EINVAL, "%s: workspace must be 256-byte aligned", who);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t Bp = padded_rows(B);
  const int G = l->G;

  SplineLocateArgs la;
  la.x = x;
  la.rec = static_cast<u32x4 *>(workspace);
  la.B = B; la.Bp = Bp; la.d = l->d; la.G = G; la.jt = l->jt;
  la.with_base = (l->value_repr == LUTKAN_REPR_SPLINE_COMPONENT);
  la.closed = (l->boundary == LUTKAN_CLOSED);
  la.zero_spline = (l->oob == LUTKAN_ZERO_SPLINE);
  la.extended = (l->knot_span == LUTKAN_SPAN_EXTENDED);
  const float domain_end = la.extended ? l->ext_knots[G + 6] : l->ext_knots[3 + G];
  la.tKs = la.closed ? domain_end : std::nextafterf(domain_end, -INFINITY);
  for (int r = 0; r < G + 7; ++r) la.ext_knots[r] = l->ext_knots[r];
  la.input_ext_knots = l->knots_per_input ? l->input_ext_knots : nullptr;
  if (phases & kLocate) {
    const int cols = ((l->d + 15) / 16 * 16 < (l->d + 31) / 32 * 32) ? 16 : 32;      // the width that pads d least
    const dim3 lgrid((unsigned)(Bp / (kSplTile / cols)), (unsigned)((l->d + cols - 1) / cols));
    if (lgrid.y > 65535u) return fail(LUTKAN_EUNSUPPORTED, "%s: d too large", who);
    if (l->knots_per_input) {
      if (cols == 32) hipLaunchKernelGGL((bspline_locate_kernel<32, true>), lgrid, dim3(256), 0, s, la);
      else hipLaunchKernelGGL((bspline_locate_kernel<16, true>), lgrid, dim3(256), 0, s, la);
    } else {
      if (cols == 32) hipLaunchKernelGGL((bspline_locate_kernel<32, false>), lgrid, dim3(256), 0, s, la);
      else hipLaunchKernelGGL((bspline_locate_kernel<16, false>), lgrid, dim3(256), 0, s, la);
    }
    if (int rc = check_launch("bspline_locate_kernel")) return rc;
    lutkan::plan_note("bspline_locate; ");
  }
  if (!(phases & kEdges)) return LUTKAN_OK;

  SplineEdgeArgs ea;
  ea.coef_table = l->coef_table; ea.rec = la.rec; ea.y = y;
  ea.B = B; ea.Bp = Bp; ea.d = l->d; ea.m = l->m; ea.rows = lutkan::coef_slice_rows(G + 3, l->value_repr);
  ea.with_base = la.with_base; ea.jt = l->jt; ea.n_tiles = l->n_tiles;
  bool tiled = true;                                   // a coefficient slice always fits LDS (R <= 67)
  if (l->algo == LUTKAN_ALGO_GATHER) tiled = false;
  // up to 16 rows the gather kernel with the inputs split over the GPU is the faster one (measured on 256x256 and
  // 1024x1024 layers): the tiled kernel's walk over all inputs is then a longer chain than the arithmetic
  if (l->algo == LUTKAN_ALGO_AUTO && B <= 16) tiled = false;
  if (l->algo == LUTKAN_ALGO_TILED && !tiled) return fail(LUTKAN_EUNSUPPORTED, "%s: tiled kernel unavailable", who);
  ea.chunk = l->d;
  ea.split_stride = 0;
  if (tiled) {
    const TilePlan tp = plan_tiles(B, l->d, l->m, l->n_tiles, 64 / (l->jt / 4), l->coef_blob_bytes);
    float *partials = reinterpret_cast<float *>(static_cast<char *>(workspace) + record_bytes(l->d, Bp, 32));
    ea.chunk = tp.chunk;
    if (tp.n_split > 1) { ea.y = partials; ea.split_stride = B * l->m; }
    const int rc = launch_spline_tiled_jt(ea, tp.np, s);
    if (rc) return rc;
    lutkan::plan_note("bspline_tiled np=%d split=%d; ", tp.np, tp.n_split);
    if (tp.n_split == 1) return rc;
    const int64_t n = B * l->m;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, partials, y, n, tp.n_split, 0);
    lutkan::plan_note("sum; ");
    return check_launch("sum_partials_kernel");
  }
  const int lg = gather_jx_log2(l->m);
  const GatherPlan gp = plan_gather(B, l->d, l->m);
  float *partials = reinterpret_cast<float *>(static_cast<char *>(workspace) + record_bytes(l->d, Bp, 32));
  ea.chunk = gp.chunk;
  if (gp.n_split > 1) { ea.y = partials; ea.split_stride = B * l->m; }
  const dim3 grid((unsigned)((B + (256 >> lg) - 1) / (256 >> lg)), (unsigned)((l->m + (1 << lg) - 1) >> lg), (unsigned)gp.n_split);
  hipLaunchKernelGGL(bspline_gather_kernel, grid, dim3(256), 0, s, ea, lg);
  if (int rc = check_launch("bspline_gather_kernel")) return rc;
  lutkan::plan_note("bspline_gather split=%d; ", gp.n_split);
  if (gp.n_split == 1) return LUTKAN_OK;
  const int64_t n = B * l->m;
  hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, partials, y, n, gp.n_split, 0);
  lutkan::plan_note("sum; ");
  return check_launch("sum_partials_kernel");
}

}  // namespace

extern "C" size_t bspline_forward_workspace_bytes(const bspline_dev_layer *layer, int64_t B) {
  if (!layer || B <= 0 || layer->d < 1 || layer->m < 1 || layer->n_tiles < 1 || layer->coef_blob_bytes < 1) return 0;
  if (layer->jt < 4 || layer->jt > 128 || (layer->jt & (layer->jt - 1))) return 0;     // as bspline_kan_forward refuses it
  return tiled_workspace_bytes(layer->d, layer->m, layer->jt, layer->n_tiles, B, 32, layer->coef_blob_bytes);
}

extern "C" int bspline_kan_forward(const bspline_dev_layer *l, const float *x, int64_t B, float *y,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return bspline_impl(l, x, B, y, workspace, workspace_bytes, hip_stream, "bspline_kan_forward", kLocate | kEdges);
}

extern "C" int bspline_forward_locate(const bspline_dev_layer *l, const float *x, int64_t B, void *workspace,
                                      size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return bspline_impl(l, x, B, nullptr, workspace, workspace_bytes, hip_stream, "bspline_forward_locate", kLocate);
}

extern "C" int bspline_forward_edges(const bspline_dev_layer *l, int64_t B, float *y, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return bspline_impl(l, nullptr, B, y, workspace, workspace_bytes, hip_stream, "bspline_forward_edges", kEdges);
}


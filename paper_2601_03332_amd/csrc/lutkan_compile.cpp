// Host-side LUT compiler of liblutkan: B-spline KAN layer -> segment-wise int8/uint8 tables.
//
// Follows Sec. 4.2 (half-open per-segment sampling, Eq. 7), Sec. 3.2 (Cox-de Boor, Eq. 3-5),
// Sec. 4.4 (symmetric int8 / asymmetric uint8 affine quantisation, Eq. 10-12) and Sec. 4.6 (artifact
// arrays), then re-lays the tables out for the gfx950 kernels: column tiles of jt outputs, one
// contiguous slice per (tile, input) holding that input's dequantisation parameters and its
// [segment][sample][column] codes.
//
// Numerics: the spline is evaluated in double from the fp32 knots and coefficients and rounded once to
// fp32; quantisation is fp32 with one rounding per operation and round-half-to-even.  This file must be
// compiled without FMA contraction.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <thread>

#include "lutkan_internal.h"

namespace lutkan {

static thread_local char g_err[512] = "";
static thread_local char g_plan[1024] = "";
static thread_local size_t g_plan_len = 0;

void plan_clear() {
  g_plan[0] = 0;
  g_plan_len = 0;
}

void plan_note(const char *fmt, ...) {
  if (g_plan_len + 1 >= sizeof(g_plan)) return;
  va_list ap;
  va_start(ap, fmt);
  const int n = vsnprintf(g_plan + g_plan_len, sizeof(g_plan) - g_plan_len, fmt, ap);
  va_end(ap);
  if (n > 0) g_plan_len = std::min(sizeof(g_plan) - 1, g_plan_len + (size_t)n);
}

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int choose_jt(int m, int K, int L, int scheme, int value_repr, int param_dtype) {
  int jt = 4;
  while (jt < m && jt < 64) jt *= 2;
  int fit = jt;
  while (fit > 4 && blob_layout(K, L, fit, scheme, value_repr, param_dtype).bytes > lds_slice_budget(value_repr)) fit /= 2;
  if (blob_layout(K, L, fit, scheme, value_repr, param_dtype).bytes <= lds_slice_budget(value_repr)) return fit;
  return jt < 32 ? jt : 32;   // no width fits: the gather kernel, which is fastest on 32-column tiles
}

int choose_coef_jt(int m) {
  int jt = 4;
  while (jt < m && jt < 128) jt *= 2;
  return jt;
}

namespace {

constexpr int P = 3;  // cubic

// The four cubic B-spline basis functions that are non-zero on the span [tau[mu], tau[mu+1]), by the
// Cox-de Boor recursion restricted to its non-zero entries.  out[a] = B_{mu-3+a, 3}(x).
// Each term is (numerator / knot difference) * lower-degree value, left term plus right term, and a
// zero-length knot difference contributes 0.
void nonzero_cubic_basis(const double *tau, int mu, double x, double out[4]) {
  double lower[5] = {0.0, 0.0, 0.0, 1.0, 0.0};  // lower[a] = B_{mu-3+a, q-1}(x); slot 4 is always 0
  for (int q = 1; q <= P; ++q) {
    double next[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int a = P - q; a <= P; ++a) {
      const int r = mu - P + a;
      double acc = 0.0;
      bool have = false;
      if (lower[a] != 0.0) {
        const double span = tau[r + q] - tau[r];
        if (span != 0.0) { acc = (x - tau[r]) / span * lower[a]; have = true; }
      }
      if (lower[a + 1] != 0.0) {
        const double span = tau[r + q + 1] - tau[r + 1];
        if (span != 0.0) {
          const double term = (tau[r + q + 1] - x) / span * lower[a + 1];
          acc = have ? acc + term : term;
        }
      }
      next[a] = acc;
    }
    std::memcpy(lower, next, sizeof(lower));
  }
  for (int a = 0; a < 4; ++a) out[a] = lower[a];
}

// The same four values for a span anywhere in the extended knot vector (mu = 0 .. n-2): out[a] = B_{mu-3+a, 3}(x)
// where that function exists (0 <= mu-3+a < R), else 0.  The recursion is run on a copy of the knots padded by three
// made-up knots per side; an existing function only ever touches real knots, and the others are dropped.
void cubic_basis_on_any_span(const std::vector<double> &tau, int R, int mu, double x, double out[4]) {
  const int n = (int)tau.size();
  std::vector<double> padded((size_t)n + 6);
  for (int r = 0; r < n; ++r) padded[(size_t)r + 3] = tau[r];
  for (int t = 1; t <= 3; ++t) {
    padded[(size_t)3 - t] = tau[0] - t * (tau[1] - tau[0]);
    padded[(size_t)n + 2 + t] = tau[n - 1] + t * (tau[n - 1] - tau[n - 2]);
  }
  nonzero_cubic_basis(padded.data(), mu + 3, x, out);
  for (int a = 0; a < 4; ++a)
    if (mu - 3 + a < 0 || mu - 3 + a >= R) out[a] = 0.0;
}

struct SegmentCodes {
  float alpha, ymin;
};

// Eq. 11: q in [-127,127], y_min = 0, alpha = max|v| / 127.  A zero segment stores alpha = 1, q = 0.
SegmentCodes quantise_symmetric(const float *v, int L, int8_t *q) {
  float peak = 0.0f;
  for (int l = 0; l < L; ++l) peak = std::max(peak, std::fabs(v[l]));
  if (peak == 0.0f) {
    std::memset(q, 0, (size_t)L);
    return {1.0f, 0.0f};
  }
  const float alpha = peak / 127.0f;
  for (int l = 0; l < L; ++l) {
    const float code = std::nearbyintf(v[l] / alpha);
    q[l] = (int8_t)std::min(127.0f, std::max(-127.0f, code));
  }
  return {alpha, 0.0f};
}

// Eq. 12: q in [0,255], y_min = min v, alpha = (max v - y_min) / 255.  A flat segment stores alpha = 1, q = 0.
SegmentCodes quantise_asymmetric(const float *v, int L, uint8_t *q) {
  const float lo = *std::min_element(v, v + L);
  const float hi = *std::max_element(v, v + L);
  if (hi == lo) {
    std::memset(q, 0, (size_t)L);
    return {1.0f, lo};
  }
  const float width = hi - lo;
  const float alpha = width / 255.0f;
  for (int l = 0; l < L; ++l) {
    const float shifted = v[l] - lo;
    const float code = std::nearbyintf(shifted / alpha);
    q[l] = (uint8_t)std::min(255.0f, std::max(0.0f, code));
  }
  return {alpha, lo};
}

// Sec. 4.6 lets scale and y_min be stored as float16: the nearest binary16 value (the conversion rounds to nearest,
// ties to even) and its bit pattern for the device table.
struct HalfValue {
  float value;
  uint16_t bits;
};

HalfValue to_binary16(float x) {
  const _Float16 h = (_Float16)x;
  HalfValue out;
  out.value = (float)h;
  std::memcpy(&out.bits, &h, sizeof(out.bits));
  return out;
}

// Writes one edge's share of a (tile, input) slice of the LUT device table (layout in lutkan.h).
struct SlicePacker {
  BlobLayout lay;
  int jt, L, scheme;
  bool half_params;

  // s_out * s_base of the edge in column jj (spline_component only)
  void put_base(uint8_t *slice, int jj, float base_gain) const { reinterpret_cast<float *>(slice)[jj] = base_gain; }

  // Segment k of the edge in column jj: its dequantisation parameters (times gain = s_out * s_spline with
  // spline_component, else exactly as given; float16 parameters arrive already rounded) and its L codes.
  void put_segment(uint8_t *slice, int jj, int k, float alpha, float ymin, bool with_gain, float gain, const uint8_t *codes) const {
    // parameter row k: the alpha of every column, then (asymmetric only) the y_min of every column
    uint8_t *row = slice + lay.params_off + (size_t)k * lay.param_row_bytes;
    if (half_params) {
      uint16_t *p16 = reinterpret_cast<uint16_t *>(row);
      p16[jj] = to_binary16(alpha).bits;
      if (scheme == LUTKAN_ASYM_UINT8) p16[jt + jj] = to_binary16(ymin).bits;
    } else {
      float *p32 = reinterpret_cast<float *>(row);
      p32[jj] = with_gain ? gain * alpha : alpha;
      if (scheme == LUTKAN_ASYM_UINT8) p32[jt + jj] = with_gain ? gain * ymin : ymin;
    }
    // device codes: uint8 as is; int8 stored excess-128 (q + 128), which the kernels undo exactly
    const uint8_t flip = (scheme == LUTKAN_SYM_INT8) ? 0x80 : 0x00;
    uint8_t *dst = slice + lay.codes_off;
    for (int l = 0; l < L; ++l) dst[((size_t)k * L + l) * jt + jj] = codes[l] ^ flip;
  }
};

// Fills the size and contract fields of an artifact's info once its arrays and tables are in place.
void fill_info(lutkan_artifact *a, int d, int m, int K, int L, int G, int scheme, int boundary, int oob, int repr,
               int param_dtype, int knots_per_input, int jt, int n_tiles, const BlobLayout &lay, int coef_jt, int coef_blob) {
  const size_t E = (size_t)d * m;
  lutkan_info &I = a->info;
  std::memset(&I, 0, sizeof(I));
  I.d = d; I.m = m; I.K = K; I.L = L; I.G = G; I.degree = P;
  I.scheme = scheme; I.boundary = boundary; I.oob = oob; I.value_repr = repr; I.param_dtype = param_dtype;
  I.knots_per_input = knots_per_input;
  I.jt = jt; I.n_tiles = n_tiles; I.blob_bytes = lay.bytes;
  I.coef_jt = coef_blob ? coef_jt : 0; I.coef_n_tiles = coef_blob ? (m + coef_jt - 1) / coef_jt : 0; I.coef_blob_bytes = coef_blob;
  I.t0 = a->knots[0]; I.tK = a->knots[K];
  I.tK_star = (boundary == LUTKAN_CLOSED) ? I.tK : std::nextafterf(I.tK, -INFINITY);  // Eq. 13
  I.q_canonical_bytes = E * K * L;
  I.params_canonical_bytes = E * K * (param_dtype == LUTKAN_PARAM_FP16 ? 2 : 4);
  I.table_bytes = a->table.size();
  I.coef_table_bytes = a->coef_table.size() * 4;
  I.artifact_bytes = I.q_canonical_bytes + 2 * I.params_canonical_bytes + 4 * (size_t)(K + 1) * (knots_per_input ? d : 1) +
                     (repr == LUTKAN_REPR_SPLINE_COMPONENT ? 12 * E : 0);
}

}  // namespace
}  // namespace lutkan

using namespace lutkan;

extern "C" const char *lutkan_last_error(void) { return g_err; }
extern "C" const char *lutkan_last_plan(void) { return g_plan; }
extern "C" const char *lutkan_version(void) { return "lutkan-gfx950 0.1"; }

extern "C" int lutkan_compile(const lutkan_layer_desc *desc, int32_t n_threads, lutkan_artifact **out) {
  if (!desc || !out) return fail(LUTKAN_EINVAL, "lutkan_compile: null argument");
  if (!desc->ext_knots || !desc->coef) return fail(LUTKAN_EINVAL, "lutkan_compile: null knots/coef");
  const int d = desc->d, m = desc->m, G = desc->G, L = desc->L;
  if (d < 1 || m < 1 || G < 1) return fail(LUTKAN_EINVAL, "lutkan_compile: d, m, G must be >= 1");
  if (L < 2) return fail(LUTKAN_EINVAL, "lutkan_compile: L must be >= 2 (got %d)", L);
  if (desc->degree != P) return fail(LUTKAN_EUNSUPPORTED, "lutkan_compile: only cubic splines (degree 3), got %d", desc->degree);
  if (desc->scheme != LUTKAN_SYM_INT8 && desc->scheme != LUTKAN_ASYM_UINT8) return fail(LUTKAN_EINVAL, "lutkan_compile: bad scheme %d", desc->scheme);
  if (desc->boundary != LUTKAN_HALF_OPEN && desc->boundary != LUTKAN_CLOSED) return fail(LUTKAN_EINVAL, "lutkan_compile: bad boundary_mode %d", desc->boundary);
  if (desc->oob != LUTKAN_CLIP_X && desc->oob != LUTKAN_ZERO_SPLINE) return fail(LUTKAN_EINVAL, "lutkan_compile: bad oob_policy %d", desc->oob);
  if (desc->value_repr != LUTKAN_REPR_PHI && desc->value_repr != LUTKAN_REPR_SPLINE_COMPONENT) return fail(LUTKAN_EINVAL, "lutkan_compile: bad value_repr %d", desc->value_repr);
  if (desc->param_dtype != LUTKAN_PARAM_FP32 && desc->param_dtype != LUTKAN_PARAM_FP16) return fail(LUTKAN_EINVAL, "lutkan_compile: bad param_dtype %d", desc->param_dtype);
  if (desc->knot_span != LUTKAN_SPAN_DOMAIN && desc->knot_span != LUTKAN_SPAN_EXTENDED) return fail(LUTKAN_EINVAL, "lutkan_compile: bad knot_span %d", desc->knot_span);
  if (desc->knots_per_input != 0 && desc->knots_per_input != 1) return fail(LUTKAN_EINVAL, "lutkan_compile: bad knots_per_input %d", desc->knots_per_input);
  const bool extended = (desc->knot_span == LUTKAN_SPAN_EXTENDED);
  const bool per_input = (desc->knots_per_input == 1);
  const bool half_params = (desc->param_dtype == LUTKAN_PARAM_FP16);
  const bool with_base = (desc->value_repr == LUTKAN_REPR_SPLINE_COMPONENT);
  if (with_base && (!desc->edge_base_scale || !desc->edge_spline_scale || !desc->edge_out_scale))
    return fail(LUTKAN_EINVAL, "lutkan_compile: spline_component needs edge_base_scale, edge_spline_scale and edge_out_scale");
  const int R = G + P, n_knots = G + 2 * P + 1;
  const int first_knot = extended ? 0 : P;             // LUT knot k is extended knot first_knot + k
  const int K = extended ? G + 2 * P : G;
  if (K > LUTKAN_MAX_K) return fail(LUTKAN_EUNSUPPORTED, "lutkan_compile: K=%d exceeds LUTKAN_MAX_K=%d", K, LUTKAN_MAX_K);
  if ((int64_t)K * L > LUTKAN_MAX_ROWS) return fail(LUTKAN_EUNSUPPORTED, "lutkan_compile: K*L=%lld exceeds %d", (long long)K * L, LUTKAN_MAX_ROWS);
  const int n_vectors = per_input ? d : 1;             // distinct knot vectors
  for (int h = 0; h < n_vectors; ++h) {
    const float *tau_h = desc->ext_knots + (size_t)h * n_knots;
    for (int r = 0; r < n_knots; ++r)
      if (!std::isfinite(tau_h[r])) return fail(LUTKAN_EINVAL, "lutkan_compile: knot %d of vector %d is not finite", r, h);
    for (int r = 0; r + 1 < n_knots; ++r)
      if (!(tau_h[r] < tau_h[r + 1])) return fail(LUTKAN_EINVAL, "lutkan_compile: knots of vector %d not strictly increasing at %d", h, r);
  }
  const size_t E = (size_t)d * m;
  for (size_t n = 0; n < E * R; ++n)
    if (!std::isfinite(desc->coef[n])) return fail(LUTKAN_EINVAL, "lutkan_compile: coefficient %zu is not finite", n);
  if (with_base)
    for (size_t e = 0; e < E; ++e)
      if (!std::isfinite(desc->edge_base_scale[e]) || !std::isfinite(desc->edge_spline_scale[e]) || !std::isfinite(desc->edge_out_scale[e]))
        return fail(LUTKAN_EINVAL, "lutkan_compile: edge scale %zu is not finite", e);

  lutkan_artifact *a = new (std::nothrow) lutkan_artifact();
  if (!a) return fail(LUTKAN_ENOMEM, "lutkan_compile: out of host memory");
  const int scheme = desc->scheme;
  const int repr = desc->value_repr;
  const int jt = choose_jt(m, K, L, scheme, repr, desc->param_dtype);
  const int n_tiles = (m + jt - 1) / jt;
  const BlobLayout lay = blob_layout(K, L, jt, scheme, repr, desc->param_dtype);
  const int coef_rows = coef_slice_rows(R, repr);
  const int cjt = choose_coef_jt(m);
  const int coef_tiles = (m + cjt - 1) / cjt;
  const int coef_blob = coef_rows * cjt * 4;
  try {
    a->ext_knots.assign(desc->ext_knots, desc->ext_knots + (size_t)n_vectors * n_knots);
    a->knots.resize((size_t)n_vectors * (K + 1));
    for (int h = 0; h < n_vectors; ++h)
      for (int k = 0; k <= K; ++k) a->knots[(size_t)h * (K + 1) + k] = desc->ext_knots[(size_t)h * n_knots + first_knot + k];
    a->q.resize(E * K * L);
    a->scale.resize(E * K);
    a->ymin.resize(E * K);
    a->table.assign((size_t)n_tiles * d * lay.bytes, 0);
    a->coef_table.assign((size_t)coef_tiles * d * coef_rows * cjt, 0.0f);
    if (with_base) {
      a->edge_base.assign(desc->edge_base_scale, desc->edge_base_scale + E);
      a->edge_spline.assign(desc->edge_spline_scale, desc->edge_spline_scale + E);
      a->edge_out.assign(desc->edge_out_scale, desc->edge_out_scale + E);
    }
  } catch (const std::bad_alloc &) {
    delete a;
    return fail(LUTKAN_ENOMEM, "lutkan_compile: out of host memory for %zu edges", E);
  }

  // Basis values at the K*L sampling positions x_{k,l} = t_k + l*(t_{k+1}-t_k)/L (Eq. 7).  A knot vector is
  // shared by all edges on it (the whole layer, or the edges leaving one input), so this small table is built once
  // per vector: basis[(k*L+l)*4 + a] multiplies coefficient c_{mu-3+a} of span mu = first_knot + k (on the domain
  // grid mu-3 = k; outside it some of the four functions do not exist and their entry is 0).
  auto basis_table = [&](int h, std::vector<double> &basis) {
    const std::vector<double> tau(a->ext_knots.begin() + (size_t)h * n_knots, a->ext_knots.begin() + (size_t)(h + 1) * n_knots);
    const float *T = a->knots.data() + (size_t)h * (K + 1);
    basis.resize((size_t)K * L * 4);
    for (int k = 0; k < K; ++k) {
      const double left = (double)T[k];
      const double step = ((double)T[k + 1] - left) / (double)L;
      for (int l = 0; l < L; ++l) {
        double *out = &basis[((size_t)k * L + l) * 4];
        if (extended) cubic_basis_on_any_span(tau, R, first_knot + k, left + (double)l * step, out);
        else nonzero_cubic_basis(tau.data(), k + P, left + (double)l * step, out);
      }
    }
  };
  std::vector<double> shared_basis;
  if (!per_input) basis_table(0, shared_basis);

  int nt = n_threads > 0 ? n_threads : (int)std::thread::hardware_concurrency();
  nt = std::max(1, std::min(nt, 64));
  nt = (int)std::min<size_t>((size_t)nt, (size_t)d);
  std::atomic<long> unrepresentable{0};       // float16 parameters that overflowed
  const SlicePacker packer{lay, jt, L, scheme, device_params_are_half(repr, half_params ? LUTKAN_PARAM_FP16 : LUTKAN_PARAM_FP32, jt)};
  auto work = [&](int tid) {
    std::vector<float> v((size_t)L);
    std::vector<double> own_basis;
    for (int i = tid; i < d; i += nt) {
      if (per_input) basis_table(i, own_basis);
      const std::vector<double> &basis = per_input ? own_basis : shared_basis;
      for (int j = 0; j < m; ++j) {
        const size_t e = (size_t)i * m + j;
        const float *c = desc->coef + e * R;
        const int t = j / jt, jj = j % jt;
        uint8_t *slice = a->table.data() + ((size_t)t * d + i) * lay.bytes;
        const int cj = j % cjt;
        float *cslice = a->coef_table.data() + ((size_t)(j / cjt) * d + i) * coef_rows * cjt;
        // spline_component (Eq. 2): the device tables carry s_out*s_base per edge as an extra row and fold
        // s_out*s_spline into the edge's dequantisation parameters / B-spline coefficients.
        float spline_gain = 1.0f;
        if (with_base) {
          const float base_gain = desc->edge_out_scale[e] * desc->edge_base_scale[e];
          spline_gain = desc->edge_out_scale[e] * desc->edge_spline_scale[e];
          packer.put_base(slice, jj, base_gain);
          cslice[cj] = base_gain;
          cslice += cjt;
        }
        for (int r = 0; r < R; ++r) cslice[(size_t)r * cjt + cj] = with_base ? spline_gain * c[r] : c[r];
        for (int k = 0; k < K; ++k) {
          const int r0 = first_knot + k - P;               // coefficient of the span's first basis function
          auto coefficient = [&](int r) { return (r >= 0 && r < R) ? (double)c[r] : 0.0; };
          const double c0 = coefficient(r0), c1 = coefficient(r0 + 1), c2 = coefficient(r0 + 2), c3 = coefficient(r0 + 3);
          for (int l = 0; l < L; ++l) {
            const double *N = &basis[((size_t)k * L + l) * 4];
            double s = 0.0;
            s += c0 * N[0];
            s += c1 * N[1];
            s += c2 * N[2];
            s += c3 * N[3];
            v[l] = (float)s;
          }
          uint8_t *qc = a->q.data() + (e * K + k) * L;
          const SegmentCodes sc = (scheme == LUTKAN_SYM_INT8)
                                      ? quantise_symmetric(v.data(), L, reinterpret_cast<int8_t *>(qc))
                                      : quantise_asymmetric(v.data(), L, qc);
          float alpha = sc.alpha, ymin = sc.ymin;
          if (half_params) {
            alpha = to_binary16(sc.alpha).value;
            ymin = to_binary16(sc.ymin).value;
            if (std::isinf(alpha) || std::isinf(ymin)) unrepresentable.fetch_add(1);
          }
          a->scale[e * K + k] = alpha;
          a->ymin[e * K + k] = ymin;
          packer.put_segment(slice, jj, k, alpha, ymin, with_base, spline_gain, qc);
        }
      }
    }
  };
  if (nt == 1) {
    work(0);
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < nt; ++t) pool.emplace_back(work, t);
    for (auto &th : pool) th.join();
  }

  if (unrepresentable.load() != 0) {
    const long n = unrepresentable.load();
    delete a;
    return fail(LUTKAN_EUNSUPPORTED, "lutkan_compile: %ld segments have an alpha or y_min too large for float16", n);
  }

  fill_info(a, d, m, K, L, G, scheme, desc->boundary, desc->oob, repr, desc->param_dtype, desc->knots_per_input, jt, n_tiles, lay, cjt, coef_blob);
  a->info.knot_span = desc->knot_span;
  *out = a;
  return LUTKAN_OK;
}

extern "C" int lutkan_artifact_from_arrays(const lutkan_artifact_arrays *in, lutkan_artifact **out) {
  const char *who = "lutkan_artifact_from_arrays";
  if (!in || !out) return fail(LUTKAN_EINVAL, "%s: null argument", who);
  if (!in->knots || !in->q_table || !in->scale || !in->y_min) return fail(LUTKAN_EINVAL, "%s: null knots / q_table / scale / y_min", who);
  const int d = in->d, m = in->m, K = in->K, L = in->L, scheme = in->scheme, repr = in->value_repr;
  if (d < 1 || m < 1 || K < 1) return fail(LUTKAN_EINVAL, "%s: d, m, K must be >= 1", who);
  if (L < 2) return fail(LUTKAN_EINVAL, "%s: L must be >= 2 (got %d)", who, L);
  if (scheme != LUTKAN_SYM_INT8 && scheme != LUTKAN_ASYM_UINT8) return fail(LUTKAN_EINVAL, "%s: bad scheme %d", who, scheme);
  if (in->boundary != LUTKAN_HALF_OPEN && in->boundary != LUTKAN_CLOSED) return fail(LUTKAN_EINVAL, "%s: bad boundary_mode %d", who, in->boundary);
  if (in->oob != LUTKAN_CLIP_X && in->oob != LUTKAN_ZERO_SPLINE) return fail(LUTKAN_EINVAL, "%s: bad oob_policy %d", who, in->oob);
  if (repr != LUTKAN_REPR_PHI && repr != LUTKAN_REPR_SPLINE_COMPONENT) return fail(LUTKAN_EINVAL, "%s: bad value_repr %d", who, repr);
  if (in->param_dtype != LUTKAN_PARAM_FP32 && in->param_dtype != LUTKAN_PARAM_FP16) return fail(LUTKAN_EINVAL, "%s: bad param_dtype %d", who, in->param_dtype);
  if (in->knots_per_input != 0 && in->knots_per_input != 1) return fail(LUTKAN_EINVAL, "%s: bad knots_per_input %d", who, in->knots_per_input);
  const int n_vectors = in->knots_per_input ? d : 1;
  const bool with_base = (repr == LUTKAN_REPR_SPLINE_COMPONENT);
  const bool half_params = (in->param_dtype == LUTKAN_PARAM_FP16);
  if (with_base && (!in->edge_base_scale || !in->edge_spline_scale || !in->edge_out_scale))
    return fail(LUTKAN_EINVAL, "%s: spline_component needs edge_base_scale, edge_spline_scale and edge_out_scale", who);
  if (K > LUTKAN_MAX_K) return fail(LUTKAN_EUNSUPPORTED, "%s: K=%d exceeds LUTKAN_MAX_K=%d", who, K, LUTKAN_MAX_K);
  if ((int64_t)K * L > LUTKAN_MAX_ROWS) return fail(LUTKAN_EUNSUPPORTED, "%s: K*L=%lld exceeds %d", who, (long long)K * L, LUTKAN_MAX_ROWS);
  for (int h = 0; h < n_vectors; ++h) {
    const float *T = in->knots + (size_t)h * (K + 1);
    for (int k = 0; k <= K; ++k)
      if (!std::isfinite(T[k])) return fail(LUTKAN_EINVAL, "%s: knot %d of vector %d is not finite", who, k, h);
    for (int k = 0; k < K; ++k)
      if (!(T[k] < T[k + 1])) return fail(LUTKAN_EINVAL, "%s: knots of vector %d not strictly increasing at %d", who, h, k);
  }
  const size_t E = (size_t)d * m;
  for (size_t n = 0; n < E * K; ++n) {
    if (!std::isfinite(in->scale[n]) || !std::isfinite(in->y_min[n])) return fail(LUTKAN_EINVAL, "%s: scale / y_min entry %zu is not finite", who, n);
    // Eq. 11 fixes y_min = 0 for the symmetric scheme; its device table carries no y_min plane, so any other value
    // would silently drop out of Eq. 10
    if (scheme == LUTKAN_SYM_INT8 && in->y_min[n] != 0.0f)
      return fail(LUTKAN_EINVAL, "%s: y_min entry %zu is %g, but the symmetric int8 scheme has y_min = 0 (Eq. 11)", who, n, (double)in->y_min[n]);
    if (half_params && (to_binary16(in->scale[n]).value != in->scale[n] || to_binary16(in->y_min[n]).value != in->y_min[n]))
      return fail(LUTKAN_EINVAL, "%s: scale / y_min entry %zu is not a float16 value", who, n);
  }
  if (with_base)
    for (size_t e = 0; e < E; ++e)
      if (!std::isfinite(in->edge_base_scale[e]) || !std::isfinite(in->edge_spline_scale[e]) || !std::isfinite(in->edge_out_scale[e]))
        return fail(LUTKAN_EINVAL, "%s: edge scale %zu is not finite", who, e);

  lutkan_artifact *a = new (std::nothrow) lutkan_artifact();
  if (!a) return fail(LUTKAN_ENOMEM, "%s: out of host memory", who);
  const int jt = choose_jt(m, K, L, scheme, repr, in->param_dtype);
  const int n_tiles = (m + jt - 1) / jt;
  const BlobLayout lay = blob_layout(K, L, jt, scheme, repr, in->param_dtype);
  try {
    a->knots.assign(in->knots, in->knots + (size_t)n_vectors * (K + 1));
    a->q.assign(static_cast<const uint8_t *>(in->q_table), static_cast<const uint8_t *>(in->q_table) + E * K * L);
    a->scale.assign(in->scale, in->scale + E * K);
    a->ymin.assign(in->y_min, in->y_min + E * K);
    a->table.assign((size_t)n_tiles * d * lay.bytes, 0);
    if (with_base) {
      a->edge_base.assign(in->edge_base_scale, in->edge_base_scale + E);
      a->edge_spline.assign(in->edge_spline_scale, in->edge_spline_scale + E);
      a->edge_out.assign(in->edge_out_scale, in->edge_out_scale + E);
    }
  } catch (const std::bad_alloc &) {
    delete a;
    return fail(LUTKAN_ENOMEM, "%s: out of host memory for %zu edges", who, E);
  }
  const SlicePacker packer{lay, jt, L, scheme, device_params_are_half(repr, half_params ? LUTKAN_PARAM_FP16 : LUTKAN_PARAM_FP32, jt)};
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < m; ++j) {
      const size_t e = (size_t)i * m + j;
      uint8_t *slice = a->table.data() + ((size_t)(j / jt) * d + i) * lay.bytes;
      float spline_gain = 1.0f;
      if (with_base) {
        spline_gain = a->edge_out[e] * a->edge_spline[e];
        packer.put_base(slice, j % jt, a->edge_out[e] * a->edge_base[e]);
      }
      for (int k = 0; k < K; ++k)
        packer.put_segment(slice, j % jt, k, a->scale[e * K + k], a->ymin[e * K + k], with_base, spline_gain, a->q.data() + (e * K + k) * L);
    }
  // a LUT artifact holds no spline coefficients: G = 0 and an empty B-spline table say so
  fill_info(a, d, m, K, L, 0, scheme, in->boundary, in->oob, repr, in->param_dtype, in->knots_per_input, jt, n_tiles, lay, 0, 0);
  *out = a;
  return LUTKAN_OK;
}

extern "C" void lutkan_artifact_free(lutkan_artifact *a) { delete a; }

extern "C" int lutkan_artifact_info(const lutkan_artifact *a, lutkan_info *out) {
  if (!a || !out) return fail(LUTKAN_EINVAL, "lutkan_artifact_info: null argument");
  *out = a->info;
  return LUTKAN_OK;
}

extern "C" const void *lutkan_artifact_q(const lutkan_artifact *a) { return a ? a->q.data() : nullptr; }
extern "C" const float *lutkan_artifact_scale(const lutkan_artifact *a) { return a ? a->scale.data() : nullptr; }
extern "C" const float *lutkan_artifact_ymin(const lutkan_artifact *a) { return a ? a->ymin.data() : nullptr; }
extern "C" const float *lutkan_artifact_knots(const lutkan_artifact *a) { return a ? a->knots.data() : nullptr; }
extern "C" const float *lutkan_artifact_ext_knots(const lutkan_artifact *a) { return (a && !a->ext_knots.empty()) ? a->ext_knots.data() : nullptr; }
extern "C" const float *lutkan_artifact_edge_base_scale(const lutkan_artifact *a) { return (a && !a->edge_base.empty()) ? a->edge_base.data() : nullptr; }
extern "C" const float *lutkan_artifact_edge_spline_scale(const lutkan_artifact *a) { return (a && !a->edge_spline.empty()) ? a->edge_spline.data() : nullptr; }
extern "C" const float *lutkan_artifact_edge_out_scale(const lutkan_artifact *a) { return (a && !a->edge_out.empty()) ? a->edge_out.data() : nullptr; }
extern "C" const void *lutkan_artifact_table(const lutkan_artifact *a) { return a ? a->table.data() : nullptr; }
extern "C" const void *lutkan_artifact_coef_table(const lutkan_artifact *a) { return (a && !a->coef_table.empty()) ? a->coef_table.data() : nullptr; }

extern "C" int lutkan_dev_layer_init(const lutkan_artifact *a, lutkan_dev_layer *out) {
  if (!a || !out) return fail(LUTKAN_EINVAL, "lutkan_dev_layer_init: null argument");
  std::memset(out, 0, sizeof(*out));
  const lutkan_info &I = a->info;
  out->d = I.d; out->m = I.m; out->K = I.K; out->L = I.L;
  out->scheme = I.scheme; out->boundary = I.boundary; out->oob = I.oob; out->value_repr = I.value_repr;
  out->param_dtype = I.param_dtype;
  out->jt = I.jt; out->n_tiles = I.n_tiles; out->blob_bytes = I.blob_bytes;
  out->algo = LUTKAN_ALGO_AUTO;
  for (int k = 0; k <= I.K; ++k) out->knots[k] = a->knots[k];
  out->table = nullptr;
  out->knots_per_input = I.knots_per_input;
  out->input_knots = nullptr;
  return LUTKAN_OK;
}

extern "C" int bspline_dev_layer_init(const lutkan_artifact *a, bspline_dev_layer *out) {
  if (!a || !out) return fail(LUTKAN_EINVAL, "bspline_dev_layer_init: null argument");
  if (a->coef_table.empty()) return fail(LUTKAN_EUNSUPPORTED, "bspline_dev_layer_init: the artifact was built from LUT arrays and holds no spline coefficients");
  std::memset(out, 0, sizeof(*out));
  const lutkan_info &I = a->info;
  out->d = I.d; out->m = I.m; out->G = I.G; out->degree = I.degree;
  out->boundary = I.boundary; out->oob = I.oob; out->value_repr = I.value_repr; out->knot_span = I.knot_span;
  out->jt = I.coef_jt; out->n_tiles = I.coef_n_tiles; out->coef_blob_bytes = I.coef_blob_bytes;
  out->algo = LUTKAN_ALGO_AUTO;
  for (int r = 0; r < I.G + 2 * P + 1; ++r) out->ext_knots[r] = a->ext_knots[r];
  out->coef_table = nullptr;
  out->knots_per_input = I.knots_per_input;
  out->input_ext_knots = nullptr;
  return LUTKAN_OK;
}

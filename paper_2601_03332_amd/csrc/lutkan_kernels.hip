// gfx950 kernels and launchers of liblutkan: the LUT-KAN layer forward (the B-spline baseline layer is in
// bspline_kernels.hip, what the two share in lutkan_device.h).
//
// Work split (Sec. 4.5, Sec. 5):
//   1. locate kernel   per (row, input): domain test on the raw x (Sec. 5.2), safe clip (Eq. 13), segment
//                      (Eq. 14), local coordinate (Eq. 15), (l0, w) (Eq. 16), all in IEEE fp32 with one
//                      rounding per operation, written as an 8-byte "record" [input][row] so that it is
//                      computed once and reused by all m outputs.
//   2. edge kernel     per (row, output): for every input gather the two adjacent codes, dequantise (Eq. 10),
//                      interpolate (Eq. 17), apply the oob_policy (Sec. 5.4) and accumulate (Eq. 1).
//                      "tiled" variant: a work-group owns (row tile) x (column tile), walks the inputs, and
//                      stages each input's table slice in LDS;  "gather" variant: codes straight from global
//                      memory (used for table slices too large for LDS and for the code trace).
//   3. chain kernel    both steps for every layer of a narrow network in one launch, activations in LDS (small
//                      batches, where the launches of 1. and 2. per layer cost more than the arithmetic).
// The file is compiled with -ffp-contract=off; every fused multiply-add below is written out as fmaf().
#include "lutkan_device.h"
#include "lutkan_pieces.h"

namespace {

// ------------------------------------------------------------------------------------------------
// Locate kernel (steps 1-4 of Sec. 4.5 + Sec. 5.2).
// ------------------------------------------------------------------------------------------------
struct LocateArgs {
  const float *x;        // [B][d]
  void *rec;             // [d][Bp] records of 8 bytes, or 16 with the base branch
  int64_t B, Bp;
  int32_t d, K, L;
  int32_t closed, zero_spline;
  float tKs;             // safe upper clip value
  float knots[LUTKAN_MAX_K + 1];
  const float *input_knots;    // [d][K+1]: one knot vector per input (then knots and tKs are not used)
  int32_t *k_out, *l0_out;     // nullable trace outputs, [B][d]
  uint8_t *in_out;
  float *w_out;
  uint16_t *silu_pieces;       // nullable, [3][Bp][d]: SiLU(x) cut into three bf16 pieces (rows B .. Bp-1 zero), the first
                               // operand of the base branch when it runs as a matrix product of its own
};

struct Located {
  int k, l0;
  float w;
  bool inside, is_nan;
};


// s_knots: the K+1 knots of this element's input in LDS.  With one vector per layer (PERIN false) the comparisons
// run against the copy in the kernel arguments (scalar registers) and LDS serves the two lookups by the lane's own
// segment index; with one vector per input every lane reads its own input's row.
template <bool PERIN, typename Args>
__device__ __forceinline__ Located locate_one(const Args &a, const float *s_knots, float x) {
  Located o;
  const float t0 = PERIN ? s_knots[0] : a.knots[0];
  const float tK = PERIN ? s_knots[a.K] : a.knots[a.K];
  const float tKs = PERIN ? (a.closed ? tK : next_float_below(tK)) : a.tKs;
  o.is_nan = (x != x);
  o.inside = a.closed ? (x >= t0 && x <= tK) : (x >= t0 && x < tK);
  float xc = o.is_nan ? t0 : x;
  xc = (xc < t0) ? t0 : xc;
  xc = (xc > tKs) ? tKs : xc;
  // k = #{kappa in 1..K-1 : T[kappa] <= x'}; T[0] <= x' always holds and T[K] is clipped away (Eq. 14).
  int k = 0;
  for (int kappa = 1; kappa < a.K; ++kappa) k += ((PERIN ? s_knots[kappa] : a.knots[kappa]) <= xc) ? 1 : 0;
  const float tk = s_knots[k], tk1 = s_knots[k + 1];
  const float num = __fsub_rn(xc, tk);
  const float den = __fsub_rn(tk1, tk);
  const float u = __fdiv_rn(num, den);                       // Eq. 15, correctly rounded
  const float z = __fmul_rn(u, (float)(a.L - 1));            // Eq. 16
  int l0 = (int)floorf(z);
  l0 = min(max(l0, 0), a.L - 1);
  o.k = k;
  o.l0 = l0;
  o.w = __fsub_rn(z, (float)l0);
  return o;
}

constexpr int kLocTile = 2048;  // (row, input) pairs per block of the LUT locate kernel: 256 threads x 8

// One block locates a tile of ROWS rows x COLS inputs (ROWS * COLS = 2048; COLS = 64, 32 or 16 so that narrow layers
// do not idle most lanes): x is read along inputs (coalesced), every thread locates eight elements, the records are
// transposed through LDS and written along rows (coalesced): records are stored [input][row].
// blockIdx.x = row tile, blockIdx.y = input tile, so small batches still fill the GPU.
// BASE: value_repr = spline_component, the record also carries SiLU(x).
// PERIN: one knot vector per input; the block keeps the vectors of its COLS inputs in LDS (odd row stride, so lanes
// that read the same knot index of different inputs hit different banks).
template <bool BASE, int COLS, bool PERIN>
__global__ __launch_bounds__(256) void lutkan_locate_kernel(const LocateArgs a) {
  typedef typename std::conditional<BASE, u32x4, u32x2>::type rec_t;
  constexpr int ROWS = kLocTile / COLS;
  constexpr int ROW_GROUPS = 256 / COLS;                 // rows handled side by side in phase 1
  constexpr int KSTRIDE = LUTKAN_MAX_K + 1;
  static_assert(KSTRIDE % 2 == 1, "odd stride between the knot rows");
  __shared__ rec_t s_rec[COLS][ROWS + 1];
  __shared__ float s_knots[(PERIN ? COLS : 1) * KSTRIDE];
  rec_t *const rec_out = static_cast<rec_t *>(a.rec);
  const int tid = threadIdx.x;
  const int64_t b0 = (int64_t)blockIdx.x * ROWS;
  const int i0 = blockIdx.y * COLS;
  if constexpr (PERIN) {
    for (int q = tid; q < COLS * (a.K + 1); q += 256) {
      const int c = q / (a.K + 1), kappa = q - c * (a.K + 1);
      s_knots[c * KSTRIDE + kappa] = (i0 + c < a.d) ? a.input_knots[(int64_t)(i0 + c) * (a.K + 1) + kappa] : 0.0f;
    }
  } else {
    if (tid <= a.K) s_knots[tid] = a.knots[tid];
  }
  const unsigned masked_index = (unsigned)(a.K * a.L) | ((unsigned)a.K << 16);
  const int il = tid % COLS;
  const int i = i0 + il;
  float xv[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {                          // all eight loads in flight before the first is used
    const int64_t b = b0 + p * ROW_GROUPS + tid / COLS;
    xv[p] = (b < a.B && i < a.d) ? a.x[b * a.d + i] : 0.0f;
  }
  __syncthreads();                                       // s_knots is filled
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int bl = p * ROW_GROUPS + tid / COLS;
    const int64_t b = b0 + bl;
    rec_t rec = {};
    rec.x = masked_index;
    if (b < a.B && i < a.d) {
      const float x = xv[p];
      const Located o = locate_one<PERIN>(a, s_knots + (PERIN ? il * KSTRIDE : 0), x);
      const bool masked = a.zero_spline && !o.inside && !o.is_nan;
      if (!masked) {
        rec.x = (unsigned)(o.k * a.L + o.l0) | ((unsigned)o.k << 16);
        rec.y = __float_as_uint(o.is_nan ? __builtin_nanf("") : o.w);
      }
      // base branch b(x) = SiLU(x) = x / (1 + exp(-x)) at the RAW input (Eq. 2); it is never masked (Sec. 5.4)
      if constexpr (BASE) rec.z = __float_as_uint(__fdiv_rn(x, 1.0f + expf(-x)));
      else if (a.silu_pieces) {
        unsigned h, m, lo;
        lutkan_cut3(__fdiv_rn(x, 1.0f + expf(-x)), h, m, lo);
        uint16_t *dst = a.silu_pieces + b * a.d + i;
        dst[0] = (uint16_t)h;
        dst[a.Bp * a.d] = (uint16_t)m;
        dst[2 * a.Bp * a.d] = (uint16_t)lo;
      }
      if (a.k_out) {
        a.k_out[b * a.d + i] = o.k;
        a.l0_out[b * a.d + i] = o.l0;
        a.in_out[b * a.d + i] = o.inside ? 1 : 0;
        a.w_out[b * a.d + i] = o.w;
      }
    }
    else if (!BASE && a.silu_pieces && i < a.d) {          // a padding row: zero pieces, so that the product needs no row checks
      uint16_t *dst = a.silu_pieces + b * a.d + i;
      dst[0] = 0;
      dst[a.Bp * a.d] = 0;
      dst[2 * a.Bp * a.d] = 0;
    }
    s_rec[il][bl] = rec;
  }
  __syncthreads();
  const int bl2 = tid % ROWS;
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int il2 = p * (256 / ROWS) + tid / ROWS;
    const int i2 = i0 + il2;
    if (i2 < a.d && b0 + bl2 < a.Bp) rec_out[(int64_t)i2 * a.Bp + b0 + bl2] = s_rec[il2][bl2];
  }
}

// OOB counters of Sec. 5.5-5.6 (optional): inputs (b,i) with In(x) = 0 and rows with at least one such input.
// One wave per row at a time; one atomic per work-group and counter.
constexpr int kOobRowsPerWave = 8;

// input_knots (nullable): [d][K+1], every input has its own domain [row[0], row[K]] instead of [t0, tK].
__global__ __launch_bounds__(256) void oob_count_kernel(const float *x, int64_t B, int d, float t0, float tK, int closed,
                                                        const float *input_knots, int K, unsigned long long *stats) {
  __shared__ unsigned s_inputs[4], s_rows[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned inputs = 0, rows = 0;
  for (int r = 0; r < kOobRowsPerWave; ++r) {
    const int64_t b = ((int64_t)blockIdx.x * kOobRowsPerWave + r) * 4 + wave;
    if (b >= B) break;                                   // wave-uniform
    unsigned outside = 0;
    for (int i = lane; i < d; i += 64) {
      const float v = x[b * d + i];
      const float lo = input_knots ? input_knots[(int64_t)i * (K + 1)] : t0;
      const float hi = input_knots ? input_knots[(int64_t)i * (K + 1) + K] : tK;
      const bool in = closed ? (v >= lo && v <= hi) : (v >= lo && v < hi);
      outside += in ? 0u : 1u;
    }
    for (int off = 32; off > 0; off >>= 1) outside += __shfl_down(outside, off, kWave);
    outside = __shfl(outside, 0, kWave);
    inputs += outside;
    rows += outside ? 1u : 0u;
  }
  if (lane == 0) { s_inputs[wave] = inputs; s_rows[wave] = rows; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned ti = s_inputs[0] + s_inputs[1] + s_inputs[2] + s_inputs[3];
    const unsigned tr = s_rows[0] + s_rows[1] + s_rows[2] + s_rows[3];
    if (ti) atomicAdd(&stats[0], (unsigned long long)ti);
    if (tr) atomicAdd(&stats[1], (unsigned long long)tr);
  }
}

// ------------------------------------------------------------------------------------------------
// Edge kernels.
// ------------------------------------------------------------------------------------------------
struct EdgeArgs {
  const unsigned char *table;
  const void *rec;       // lookup records written by the locate kernel, [d][Bp], 8 bytes each (16 with_base)
  float *y;
  int16_t *q01_out;      // nullable, [B][d][m][2]
  int64_t B, Bp;
  int32_t d, m, K, L;
  int32_t jt, n_tiles, blob_bytes;
  int32_t codes_off, params_off, param_row_bytes;
  int32_t with_base;       // value_repr = spline_component: slices start with a row of s_out*s_base, records carry SiLU(x)
  int32_t param_fp16;      // the table's dequantisation parameters are binary16 values (phi layers with float16 parameters), else fp32
  const int32_t *k_out, *l0_out;   // code trace only: the located (k, l0) of every (row, input), [B][d]
  int32_t chunk;           // tiled kernels: inputs per work-group (blockIdx.y selects the chunk of inputs)
  int64_t split_stride;    // tiled kernels: floats between the partial outputs of consecutive chunks (0 if one chunk)
  int32_t accumulate;      // tiled kernel writing y itself (one chunk): add to what y holds (the base branch) instead of overwriting
  int32_t wide;            // tiled kernel: 2 or 4 when table, blob_bytes and the offsets describe a wide form (bytes per code), else 0
  int32_t deep;            // tiled kernel: the launch waits for the table to stream from HBM; keep two slices in flight
  int32_t asym;            // the layer's scheme is asymmetric uint8 (a second parameter plane)
};

// Device-table byte -> code value.  Symmetric int8 codes are stored excess-128 (byte = q + 128).
template <int SCHEME>
__device__ __forceinline__ float code_to_float(unsigned byte) {
  if (SCHEME == LUTKAN_SYM_INT8) return (float)((int)(byte & 0xffu) - 128);
  return (float)(byte & 0xffu);
}

__device__ __forceinline__ f16x2 bits_to_f16x2(unsigned v) {
  union { unsigned u; f16x2 h; } c;
  c.u = v;
  return c.h;
}

// Gather variant: one thread per (row, output column); consecutive threads take consecutive columns so the
// two code rows and the parameter row are read as contiguous runs.  Inputs are taken four at a time: the four
// records are independent loads, then the eight codes and four parameters, so the dependent-load latency is
// paid once per four inputs.  Masked records point at the slice's zero rows (no branch).  With TRACE the two
// gathered codes of every edge are also written out, addressed by the traced (k, l0) so that masked edges
// report the codes they would have used.
// blockIdx.z selects a chunk of a.chunk inputs; with more than one chunk the kernel writes partial sums (chunk
// after chunk, a.split_stride floats apart) that sum_partials_kernel adds in chunk order.  That is how a batch of a
// few rows still fills the GPU: the walk over the inputs, a chain of dependent reads, is cut into many short ones.
template <int SCHEME, bool TRACE>
__global__ __launch_bounds__(256) void lutkan_gather_kernel(const EdgeArgs a, const int jx_log2) {
  constexpr int U = 4;
  const int jx = 1 << jx_log2;
  const int tx = threadIdx.x & (jx - 1);
  const int ty = threadIdx.x >> jx_log2;
  const int j = blockIdx.y * jx + tx;
  const int64_t b = (int64_t)blockIdx.x * (256 >> jx_log2) + ty;
  if (j >= a.m || b >= a.B) return;
  const int t = j / a.jt, jj = j - t * a.jt;
  const unsigned char *tile = a.table + (size_t)t * a.d * a.blob_bytes;
  const int rec_words = a.with_base ? 4 : 2;
  const unsigned *recs = static_cast<const unsigned *>(a.rec);
  const int i_begin = blockIdx.z * a.chunk;
  const int i_end = min(a.d, i_begin + a.chunk);
  float acc = 0.0f;
  for (int i0 = i_begin; i0 < i_end; i0 += U) {
    u32x2 rec[U];
    float silu_x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned *r = recs + ((int64_t)min(i0 + u, i_end - 1) * a.Bp + b) * rec_words;
      rec[u] = *reinterpret_cast<const u32x2 *>(r);
      silu_x[u] = a.with_base ? __uint_as_float(r[2]) : 0.0f;
    }
    unsigned c0[U], c1[U];
    float al[U], ym[U], bg[U];             // alpha, y_min, s_out*s_base
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned char *slice = tile + (size_t)min(i0 + u, i_end - 1) * a.blob_bytes;
      const unsigned code_off = (unsigned)a.codes_off + (rec[u].x & 0xffffu) * (unsigned)a.jt;
      const unsigned param_off = (unsigned)a.params_off + (rec[u].x >> 16) * (unsigned)a.param_row_bytes;
      c0[u] = slice[code_off + jj];
      c1[u] = slice[code_off + a.jt + jj];
      // a parameter row is the alpha of every column, then (asymmetric) the y_min of every column
      if (a.param_fp16) {
        const _Float16 *prm = reinterpret_cast<const _Float16 *>(slice + param_off);
        al[u] = (float)prm[jj];
        ym[u] = (SCHEME == LUTKAN_ASYM_UINT8) ? (float)prm[a.jt + jj] : 0.0f;
      } else {
        const float *prm = reinterpret_cast<const float *>(slice + param_off);
        al[u] = prm[jj];
        ym[u] = (SCHEME == LUTKAN_ASYM_UINT8) ? prm[a.jt + jj] : 0.0f;
      }
      bg[u] = a.with_base ? reinterpret_cast<const float *>(slice)[jj] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (i0 + u < i_end) {
        const float w = __uint_as_float(rec[u].y);
        const float f0 = code_to_float<SCHEME>(c0[u]), f1 = code_to_float<SCHEME>(c1[u]);
        const float tq = fmaf(w, f1 - f0, f0);                             // interpolate the codes ...
        acc = fmaf(al[u], tq, acc);                                        // ... then one scale per edge
        if (SCHEME == LUTKAN_ASYM_UINT8) acc += ym[u];
        if (a.with_base) acc = fmaf(bg[u], silu_x[u], acc);                  // + s_out*s_base * SiLU(x)
        if (TRACE && a.q01_out) {
          const int l0 = a.l0_out[b * a.d + i0 + u];
          const int row = a.k_out[b * a.d + i0 + u] * a.L + l0;
          const int row1 = (l0 + 1 < a.L) ? row + 1 : row;                 // l1 = min(l0+1, L-1)
          const unsigned char *codes = tile + (size_t)(i0 + u) * a.blob_bytes + a.codes_off;
          int16_t *o = a.q01_out + ((b * a.d + i0 + u) * a.m + j) * 2;
          o[0] = (int16_t)code_to_float<SCHEME>(codes[(size_t)row * a.jt + jj]);
          o[1] = (int16_t)code_to_float<SCHEME>(codes[(size_t)row1 * a.jt + jj]);
        }
      }
    }
  }
  a.y[(int64_t)blockIdx.z * a.split_stride + b * a.m + j] = acc;
}


// Gather variant for the plain launch (no code trace): the lane layout of the tiled kernel without its staging.  A lane
// owns 4 adjacent columns of one row, jt/4 lanes share a row, so per input a lane issues four vector-memory reads for
// its 4 edges -- the row's record (the same address for the lanes of a row), one dword of code row l0, one of row
// l0+1, 16 bytes of alpha (plus 16 of y_min for the asymmetric scheme) -- where the kernel above issues five per
// edge.  Only the table rows a batch touches are read, each as whole 4..64-byte runs of its column tile, which is what
// makes this the kernel for batches that touch less than the whole table: the tiled kernel streams every slice
// whatever the batch.  Inputs four at a time (all records, then all codes and parameters: two dependent round trips
// per four inputs); blockIdx.z selects the chunk of inputs, partial sums as above.  Arithmetic per edge as above.
template <int SCHEME, bool BASE, bool PH, int U>
__global__ __launch_bounds__(256) void lutkan_gather4_kernel(const EdgeArgs a, const int lpr_log2) {
  typedef typename std::conditional<BASE, u32x4, u32x2>::type rec_t;
  const int sub = threadIdx.x & ((1 << lpr_log2) - 1);                  // which 4-column group of the tile
  const int64_t b = (int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);    // < Bp: padding rows carry masked records
  const int t = blockIdx.y;
  const unsigned char *tile = a.table + (size_t)t * a.d * a.blob_bytes;
  const rec_t *recs = static_cast<const rec_t *>(a.rec) + b;
  const unsigned col_codes = (unsigned)a.codes_off + sub * 4;
  const unsigned col_params = (unsigned)a.params_off + sub * (PH ? 8 : 16);
  const unsigned plane = (unsigned)a.jt * (PH ? 2 : 4);
  const int i_begin = blockIdx.z * a.chunk;
  const int i_end = min(a.d, i_begin + a.chunk);
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  rec_t rec[U];
#pragma unroll
  for (int u = 0; u < U; ++u) rec[u] = recs[(int64_t)min(i_begin + u, i_end - 1) * a.Bp];
  for (int i0 = i_begin; i0 < i_end; i0 += U) {
    unsigned c0[U], c1[U];
    f32x4 al[U], ym[U], bg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned char *slice = tile + (size_t)min(i0 + u, i_end - 1) * a.blob_bytes;
      const unsigned char *cp = slice + col_codes + (rec[u].x & 0xffffu) * (unsigned)a.jt;
      const unsigned char *pp = slice + col_params + (rec[u].x >> 16) * (unsigned)a.param_row_bytes;
      c0[u] = *reinterpret_cast<const unsigned *>(cp);
      c1[u] = *reinterpret_cast<const unsigned *>(cp + a.jt);
      ym[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      if constexpr (PH) {
        const u32x2 ha = *reinterpret_cast<const u32x2 *>(pp);
        const f16x2 a01 = bits_to_f16x2(ha.x), a23 = bits_to_f16x2(ha.y);
        al[u] = f32x4{(float)a01.x, (float)a01.y, (float)a23.x, (float)a23.y};
        if (SCHEME == LUTKAN_ASYM_UINT8) {
          const u32x2 hy = *reinterpret_cast<const u32x2 *>(pp + plane);
          const f16x2 y01 = bits_to_f16x2(hy.x), y23 = bits_to_f16x2(hy.y);
          ym[u] = f32x4{(float)y01.x, (float)y01.y, (float)y23.x, (float)y23.y};
        }
      } else {
        al[u] = *reinterpret_cast<const f32x4 *>(pp);
        if (SCHEME == LUTKAN_ASYM_UINT8) ym[u] = *reinterpret_cast<const f32x4 *>(pp + plane);
      }
      bg[u] = BASE ? *reinterpret_cast<const f32x4 *>(slice + sub * 16) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // the records of the next U inputs travel while this round's codes and parameters do: one exposed round trip per round
    rec_t rec_next[U];
#pragma unroll
    for (int u = 0; u < U; ++u) rec_next[u] = recs[(int64_t)min(i0 + U + u, i_end - 1) * a.Bp];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (i0 + u < i_end) {
        const float w = __uint_as_float(rec[u].y);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float f0 = code_to_float<SCHEME>(c0[u] >> (8 * c)), f1 = code_to_float<SCHEME>(c1[u] >> (8 * c));
          const float tq = fmaf(w, f1 - f0, f0);                              // interpolate the codes ...
          acc[c] = fmaf(al[u][c], tq, acc[c]);                               // ... then one scale per edge
          if (SCHEME == LUTKAN_ASYM_UINT8) acc[c] += ym[u][c];
          if constexpr (BASE) acc[c] = fmaf(bg[u][c], __uint_as_float(rec[u].z), acc[c]);    // + s_out*s_base * SiLU(x)
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) rec[u] = rec_next[u];
  }
  if (b >= a.B) return;
  const int j = t * a.jt + sub * 4;
  float *yout = a.y + (int64_t)blockIdx.z * a.split_stride + b * a.m + j;
  if (j + 3 < a.m && (a.m & 3) == 0) {
    *reinterpret_cast<f32x4 *>(yout) = f32x4{acc[0], acc[1], acc[2], acc[3]};
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (j + c < a.m) yout[c] = acc[c];
  }
}


constexpr int kGather4Inputs = 8;

constexpr double kBaseProductMinEdges = 5e8;      // batch * d * m from which the base branch runs as a matrix product

// Tiled variant.  A work-group of NW waves owns NW*RW rows and one column tile of JT = 4*LPR outputs.
// A wave works on RPS = 64/LPR rows at a time: LPR lanes share a row and each lane owns 4 adjacent columns,
// so one dword holds a lane's four codes of a table row and one 16-byte read its four scales.  Each wave owns
// RW = RPS*NP rows and keeps 4*NP running sums per lane in registers for the whole walk over the d inputs.
//
// LDS holds two slice buffers and, per wave, two record buffers.  While input i is processed out of one
// buffer, the (tile, i+1) table slice and the wave's RW records for input i+1 stream from global memory
// straight into the other one (no registers, no LDS store instructions); one barrier per input separates
// the two roles.  Per row a lane reads its row's record (an LDS broadcast), turns the table row and the segment
// in it into two LDS addresses (one 16-bit multiply-add each), and reads code row l0, code row l0+1 and the scales.
// Arithmetic per edge (Eq. 10 + Eq. 17 folded): acc += alpha * (q0 + w * (q1 - q0)) [+ y_min].  A byte code c,
// zero-extended to 16 bits, IS the fp16 denormal c * 2^-24, so the four codes of a dword become two packed-fp16
// registers with two byte permutes; the difference q1 - q0 (and the removal of the excess-128 bias of symmetric
// codes) is then exact packed-fp16 arithmetic on denormals, and q0 + w*(q1-q0) one mixed-precision FMA with a
// single fp32 rounding.  The running sums therefore carry a factor 2^-24, removed exactly at the end.
// There is no branch per row: a masked record (oob_policy zero_spline, or a padding row) points to the
// all-zero code row K*L and the all-zero parameter row K that every slice carries, which makes its
// contribution exactly zero.  l0+1 is read even when l0 = L-1: then w = 0 exactly and the neighbour (the
// next segment's first row, or a zero row) does not change the result.
// With BASE (value_repr = spline_component) every slice starts with a row of s_out*s_base; a lane loads its four
// values once per input and adds base * SiLU(x) per row, SiLU(x) being the third word of the row's record.
// With PH the dequantisation parameters are binary16 values: half the LDS bytes per edge; they enter the same FMAs
// through the mixed-precision form (fp16 factor, fp32 product and sum), so the arithmetic is that of the fp32 path
// on the stored values.
//
// PIPE: how the copies, the barrier and the LDS reads of consecutive inputs overlap.
//   2  two buffers.  Every input ends in "wait for my copies of the next slice, barrier", and every wave then refills
//      its read pipeline (record -> addresses -> codes and scales, two LDS round trips) at the same moment, with
//      nothing else on the SIMD to cover it.
//   3  three buffers, reads carried across inputs (no BASE, NP >= 2; where three buffers fit the LDS).  The slice of
//      input i+2 is copied while input i is processed; the one barrier per input (before input i: "everyone has
//      finished input i-1", so its buffer may be overwritten, and "everyone's share of slice i+1 has landed", waited
//      for one whole input after the copies were issued) no longer guards the data the wave is about to read, so the
//      read pipeline runs on from the last row steps of input i into the first of input i+1 without a refill.
//   4  three buffers, two slices in flight (no BASE), for launches that wait for the table to stream from HBM: a
//      work-group with one 44 KiB slice in flight draws about 21 GB/s, 256 of them 5.4 TB/s.  Before input i a wave
//      waits only until its copies of slice i have landed -- those of slice i+1, issued one input ago, stay in flight
//      -- and after the barrier it issues the copies of slice i+2; the read pipeline is refilled per input as with 2.
//      (vmcnt counts a wave's copies in issue order: with n0 = the fewest copies any wave issues per input, "at
//      most n0 outstanding" implies that everything older than the newest input's copies has landed.)
//
// CB: bytes per code of the slices.  1: the table as compiled.  2: the wide form whose codes are binary16 values
// already (q * 2^-24, signed): a lane reads its four codes of a row as two packed pairs, and the permutes and the
// bias removal fall away; the arithmetic after them is the same.  4: the wide form that holds the dequantised values
// of Eq. 10 as fp32: a lane reads its four values of both rows, nothing of the parameters, and interpolates them
// (Sec. 4.5 step 5) with a subtraction, a multiply-add and the addition to the sum.
template <int SCHEME, int LPR, int NP, int NW, bool BASE, bool PH, int PIPE, int CB>
__global__ __launch_bounds__(NW * 64) void lutkan_tiled_kernel(const EdgeArgs a) {
  static_assert(!(BASE && PH), "with the base branch the device table holds fp32 products, never binary16 parameters");
  static_assert(CB == 1 || CB == 2 || CB == 4, "bytes per code");
  constexpr bool WIDE = (CB == 2), VALUES = (CB == 4);
  static_assert(!(BASE && CB == 2), "the form with 16-bit codes is used with 8-byte records only");
  static_assert(!(VALUES && (PH || SCHEME != 0)), "the fp32 values are the same for both schemes and any parameter type: one instance");
  static_assert(PIPE == 2 || (PIPE == 3 && !BASE && NP >= 2) || (PIPE == 4 && !BASE), "carried reads need two row steps of the same input; three buffers go with 8-byte records");
  constexpr int NBUF = (PIPE == 2) ? 2 : 3;
  constexpr bool CARRY = (PIPE == 3), DEEP = (PIPE == 4);
  // Row steps between the issue of a step's code and parameter reads and their use.  One step of the byte form (18
  // vector instructions on each of a SIMD's four waves) covers the LDS latency; one of the wide forms (12 or 13) does
  // not: the waves of the binary16 form spent 13 % of their cycles waiting for LDS reads, so they read two steps ahead.
  constexpr int AHEAD = (CB > 1) ? 2 : 1;
  static_assert(!CARRY || NP > AHEAD, "carried reads: the pipeline must fit into one input's row steps");
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int JT = 4 * LPR;
  constexpr int RPS = 64 / LPR;
  constexpr int RW = RPS * NP;

  constexpr int PSZ = PH ? 8 : 16;         // bytes of a lane's four alphas (and of its four y_min, one plane further)
  constexpr int PLANE = JT * (PH ? 2 : 4); // a parameter row is the alpha plane, then (asymmetric) the y_min plane
  constexpr int RB = BASE ? 16 : 8;                              // bytes per record
  static_assert(RW <= 64, "a wave's records for one input must fit one 1 KiB copy step");
  constexpr int REC_LANES = RW * RB / 16;                        // lanes that copy 16 bytes of the wave's records
  static_assert((RW * RB) % 16 == 0, "a wave's records are whole 16-byte vectors");
  typedef const __attribute__((address_space(3))) unsigned char *lds_bytes;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sub = lane & (LPR - 1);        // which 4-column group of the tile
  const int hrow = lane / LPR;             // which of the RPS rows of a step
  const int t = blockIdx.x % a.n_tiles;
  const int64_t rt = blockIdx.x / a.n_tiles;
  const int64_t b0 = rt * (NW * RW) + (int64_t)wave * RW;
  const int nvec = a.blob_bytes >> 4;

  float acc[NP][4];
#pragma unroll
  for (int p = 0; p < NP; ++p)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[p][c] = 0.0f;

  const unsigned char *src = a.table + (size_t)t * a.d * a.blob_bytes;                   // slice (t, 0); wave-uniform
  const unsigned char *rec_src = static_cast<const unsigned char *>(a.rec) + b0 * RB;     // this wave's records of input 0; wave-uniform
  const unsigned lane_off = lane * 16;
  unsigned char *rec_area = lds + NBUF * a.blob_bytes + wave * (NBUF * RW * RB);

  // this work-group walks the inputs [i_begin, i_end) and writes one set of (partial) sums
  const int i_begin = blockIdx.y * a.chunk;
  const int i_end = min(a.d, i_begin + a.chunk);
  float *yout = a.y + (int64_t)blockIdx.y * a.split_stride;

  // copies slice (t, i) and this wave's records of input i into buffer `buf`
  auto stage_input = [&](int i, int buf) {
    stage_slice<NW>(src + (size_t)i * a.blob_bytes, lds + buf * a.blob_bytes, nvec, wave, lane, lane_off);
    if (lane < REC_LANES) copy16_global_to_lds_at(rec_src + (int64_t)i * a.Bp * RB, lane_off, rec_area + buf * (RW * RB));
  };
  stage_input(i_begin, 0);
  if (NBUF == 3 && i_begin + 1 < i_end) stage_input(i_begin + 1, 1);
  if (!DEEP) {                                         // (DEEP waits at the top of every input)
    wait_all_vector_loads();
    __syncthreads();
  }
  const int fewest_copies = (nvec >> 6) / NW + 1;      // per wave and input: its whole 1 KiB chunks of the slice, its records

  // Software pipeline over the row steps.  The reads of step p+1 (codes, parameters) and the record of
  // step p+2 are issued before the arithmetic of step p, and they are issued right AFTER the one point per
  // step where the wave waits for its outstanding LDS reads (the first touch of step p's data): what the
  // wave waits for was issued a whole step earlier, what it issues now has a whole step to arrive.
  typedef typename std::conditional<BASE, u32x3, u32x2>::type rec_t;        // 12-byte or 8-byte LDS read
  // parameters of the lane's 4 columns as loaded: pa = the four alphas, pb = the four y_min (asymmetric);
  // binary16 parameters are packed two per word in .x and .y.  With fp32 values: pa = the row's four values, pb =
  // the next row's.
  struct Fetched { unsigned c0, c1, c0b, c1b; f32x4 pa, pb; };                // c0b, c1b: columns 2 and 3 of a wide row
  // col_codes / col_params: LDS byte addresses of this lane's columns in code row 0 and parameter row 0 of a slice
  auto fetch = [&](const rec_t &rc, unsigned col_codes, unsigned col_params) {
    Fetched f;
    // address = column address + (16-bit half of the record word) * (bytes per row): D = S0.u16 * S1.u16 + S2
    unsigned code_addr, param_addr;
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[0,0,0,0]" : "=v"(code_addr) : "v"(rc.x), "s"(JT * CB), "v"(col_codes));
    lds_bytes cp = (lds_bytes)(uintptr_t)code_addr;
    typedef const __attribute__((address_space(3))) unsigned *lds_u32;
    typedef const __attribute__((address_space(3))) f32x4 *lds_f32x4;
    if constexpr (VALUES) {
      f.c0 = 0; f.c1 = 0; f.c0b = 0; f.c1b = 0;
      f.pa = *(lds_f32x4)cp;
      f.pb = *(lds_f32x4)(cp + JT * CB);
      return f;
    }
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(param_addr) : "v"(rc.x), "s"(a.param_row_bytes), "v"(col_params));
    lds_bytes pp = (lds_bytes)(uintptr_t)param_addr;
    if constexpr (WIDE) {
      typedef const __attribute__((address_space(3))) u32x2 *lds_u32x2;
      const u32x2 r0 = *(lds_u32x2)cp, r1 = *(lds_u32x2)(cp + JT * CB);
      f.c0 = r0.x; f.c0b = r0.y; f.c1 = r1.x; f.c1b = r1.y;
    } else {
      f.c0 = *(lds_u32)cp;
      f.c1 = *(lds_u32)(cp + JT);
      f.c0b = 0; f.c1b = 0;
    }
    f.pb = f32x4{0.f, 0.f, 0.f, 0.f};
    if constexpr (PH) {
      typedef const __attribute__((address_space(3))) f32x2 *lds_f32x2;
      const f32x2 ha = *(lds_f32x2)pp;
      f.pa = f32x4{ha.x, ha.y, 0.f, 0.f};
      if (SCHEME == LUTKAN_ASYM_UINT8) {
        const f32x2 hy = *(lds_f32x2)(pp + PLANE);
        f.pb = f32x4{hy.x, hy.y, 0.f, 0.f};
      }
    } else {
      f.pa = *(lds_f32x4)pp;
      if (SCHEME == LUTKAN_ASYM_UINT8) f.pb = *(lds_f32x4)(pp + PLANE);
    }
    return f;
  };
  auto columns_of = [&](int buf, unsigned &col_codes, unsigned &col_params) {
    const unsigned slice_addr = (unsigned)(uintptr_t)(lds_bytes)(lds + buf * a.blob_bytes);
    col_codes = slice_addr + (unsigned)a.codes_off + sub * (4 * CB);
    col_params = slice_addr + (unsigned)a.params_off + sub * PSZ;
  };

  // The read pipeline: rcq[k] is the record of row step p+k, fq[k] the codes and parameters of row step p+k, for the
  // current step p.  Carried from one input to the next (PIPE 3), else refilled at the top of every input.
  rec_t rcq[AHEAD + 1];
  Fetched fq[AHEAD];
  auto fill_read_pipeline = [&](const unsigned char *rec_buf, unsigned col_codes, unsigned col_params) {
#pragma unroll
    for (int k = 0; k <= AHEAD; ++k) rcq[k] = *reinterpret_cast<const rec_t *>(rec_buf + (k < NP ? k : NP - 1) * (RPS * RB));
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) fq[k] = fetch(rcq[k], col_codes, col_params);
  };
  int cur = 0;                                         // buffer of input i
  if (CARRY) {
    unsigned cc, cp;
    columns_of(0, cc, cp);
    fill_read_pipeline(rec_area + hrow * RB, cc, cp);
  }

  for (int i = i_begin; i < i_end; ++i) {
    // two buffers: the other one; three: the next of the ring, and the one after it for the copies
    const int nxt = (NBUF == 2) ? (cur ^ 1) : (cur == 2 ? 0 : cur + 1);
    if (PIPE == 2) {
      if (i + 1 < i_end) stage_input(i + 1, nxt);                  // stream the next input's slice and records
    } else if (CARRY) {
      // My share of slice i+1, copied during input i-1, has landed; after the barrier everyone's has, and everyone has
      // finished input i-1, whose buffer now takes the slice of input i+2.  The reads this wave has in flight (the
      // first row steps of input i) stay in flight: the barrier is the bare instruction, without the wait for LDS
      // traffic that a fence would add.
      wait_all_vector_loads();
      asm volatile("s_barrier" ::: "memory");
      if (i + 2 < i_end) stage_input(i + 2, nxt == 2 ? 0 : nxt + 1);
    } else {
      // My copies of slice i have landed (those of slice i+1 may still be in flight); after the barrier everyone's
      // have, and everyone has finished input i-1, whose buffer now takes the slice of input i+2.
      if (i + 1 < i_end) wait_until_vector_loads_outstanding(fewest_copies); else wait_all_vector_loads();
      lds_barrier();
      if (i + 2 < i_end) stage_input(i + 2, nxt == 2 ? 0 : nxt + 1);
    }
    const unsigned char *slice = lds + cur * a.blob_bytes;
    const unsigned char *rec_buf = rec_area + cur * (RW * RB) + hrow * RB;
    unsigned col_codes, col_params;
    columns_of(cur, col_codes, col_params);
    // carried reads: where the reads for the next input's first row steps go.  After the last input they re-read this
    // input's buffers (valid records and rows, results unused).
    const int ahead = (CARRY && i + 1 < i_end) ? nxt : cur;
    const unsigned char *rec_ahead = rec_area + ahead * (RW * RB) + hrow * RB;
    unsigned ahead_codes = col_codes, ahead_params = col_params;
    if (CARRY) columns_of(ahead, ahead_codes, ahead_params);
    f32x4 base_gain = {0.f, 0.f, 0.f, 0.f};
    if (BASE) base_gain = *reinterpret_cast<const f32x4 *>(slice + sub * 16) * (VALUES ? 1.0f : kTwoToMinus24);   // (the sums on fp32 values are not scaled)
    if (!CARRY) fill_read_pipeline(rec_buf, col_codes, col_params);
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const Fetched f_cur = fq[0];
      const rec_t rc_cur = rcq[0];
      Fetched f_new = fq[AHEAD - 1];
      rec_t rc_new = rcq[AHEAD];
      // first touch of step p's data, and of the record whose addresses are computed next (everything older has
      // arrived then: LDS reads return in order)
      if (SCHEME == LUTKAN_ASYM_UINT8 || VALUES) asm volatile("" ::"v"(f_cur.pb.x));
      if (VALUES) asm volatile("" ::"v"(f_cur.pa.x), "v"(rcq[AHEAD].y));
      else asm volatile("" ::"v"(f_cur.pa.x), "v"(f_cur.c1), "v"(rcq[AHEAD].y));
      __builtin_amdgcn_sched_barrier(0);
      if (p + AHEAD + 1 < NP) rc_new = *reinterpret_cast<const rec_t *>(rec_buf + (p + AHEAD + 1) * (RPS * RB));
      else if (CARRY) rc_new = *reinterpret_cast<const rec_t *>(rec_ahead + (p + AHEAD + 1 - NP) * (RPS * RB));
      if (p + AHEAD < NP) f_new = fetch(rcq[AHEAD], col_codes, col_params);
      else if (CARRY) f_new = fetch(rcq[AHEAD], ahead_codes, ahead_params);
      __builtin_amdgcn_sched_barrier(0);
      const float w = __uint_as_float(rc_cur.y);
      if constexpr (VALUES) {
        // v0 + w * (v1 - v0) of the two dequantised values: three roundings, then the one of the sum.  The multiply-add
        // is written in its two-operand encoding, which issues faster than the three-operand one the compiler
        // picks here (v0 is dead afterwards, so it may be overwritten).
        float v[4] = {f_cur.pa.x, f_cur.pa.y, f_cur.pa.z, f_cur.pa.w};
        const float dv[4] = {f_cur.pb.x - f_cur.pa.x, f_cur.pb.y - f_cur.pa.y, f_cur.pb.z - f_cur.pa.z, f_cur.pb.w - f_cur.pa.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          asm("v_fmac_f32 %0, %1, %2" : "+v"(v[c]) : "v"(w), "v"(dv[c]));
          acc[p][c] += v[c];
        }
        if constexpr (BASE) {
          const float silu_x = __uint_as_float(rc_cur.z);
          acc[p][0] = fmaf(base_gain.x, silu_x, acc[p][0]);
          acc[p][1] = fmaf(base_gain.y, silu_x, acc[p][1]);
          acc[p][2] = fmaf(base_gain.z, silu_x, acc[p][2]);
          acc[p][3] = fmaf(base_gain.w, silu_x, acc[p][3]);
        }
      } else {
        float al[4], ym[4];
        if constexpr (PH) {
          const f16x2 a01 = bits_to_f16x2(__float_as_uint(f_cur.pa.x)), a23 = bits_to_f16x2(__float_as_uint(f_cur.pa.y));
          const f16x2 y01 = bits_to_f16x2(__float_as_uint(f_cur.pb.x)), y23 = bits_to_f16x2(__float_as_uint(f_cur.pb.y));
          al[0] = (float)a01.x; al[1] = (float)a01.y; al[2] = (float)a23.x; al[3] = (float)a23.y;
          ym[0] = (float)y01.x; ym[1] = (float)y01.y; ym[2] = (float)y23.x; ym[3] = (float)y23.y;
        } else {
          al[0] = f_cur.pa.x; al[1] = f_cur.pa.y; al[2] = f_cur.pa.z; al[3] = f_cur.pa.w;
          ym[0] = f_cur.pb.x; ym[1] = f_cur.pb.y; ym[2] = f_cur.pb.z; ym[3] = f_cur.pb.w;
        }
        f16x2 q0lo, q0hi, q1lo, q1hi;
        if constexpr (WIDE) {                                                    // the table holds q * 2^-24 as it is needed
          q0lo = bits_to_f16x2(f_cur.c0); q0hi = bits_to_f16x2(f_cur.c0b);
          q1lo = bits_to_f16x2(f_cur.c1); q1hi = bits_to_f16x2(f_cur.c1b);
        } else {
          // bytes {b3,b2,b1,b0} -> packed fp16 denormals {b1,b0} and {b3,b2}, each worth byte * 2^-24
          q0lo = bits_to_f16x2(__builtin_amdgcn_perm(f_cur.c0, f_cur.c0, 0x0c010c00u));
          q0hi = bits_to_f16x2(__builtin_amdgcn_perm(f_cur.c0, f_cur.c0, 0x0c030c02u));
          q1lo = bits_to_f16x2(__builtin_amdgcn_perm(f_cur.c1, f_cur.c1, 0x0c010c00u));
          q1hi = bits_to_f16x2(__builtin_amdgcn_perm(f_cur.c1, f_cur.c1, 0x0c030c02u));
        }
        const f16x2 dlo = q1lo - q0lo, dhi = q1hi - q0hi;                        // (q1 - q0) * 2^-24, exact
        if (SCHEME == LUTKAN_SYM_INT8 && !WIDE) {                                // remove the excess-128 bias, exact
          const f16x2 bias = bits_to_f16x2(0x00800080u);
          q0lo = q0lo - bias;
          q0hi = q0hi - bias;
        }
        const float t0 = fmaf(w, (float)dlo.x, (float)q0lo.x);                   // one rounding each
        const float t1 = fmaf(w, (float)dlo.y, (float)q0lo.y);
        const float t2 = fmaf(w, (float)dhi.x, (float)q0hi.x);
        const float t3 = fmaf(w, (float)dhi.y, (float)q0hi.y);
        acc[p][0] = fmaf(al[0], t0, acc[p][0]);
        acc[p][1] = fmaf(al[1], t1, acc[p][1]);
        acc[p][2] = fmaf(al[2], t2, acc[p][2]);
        acc[p][3] = fmaf(al[3], t3, acc[p][3]);
        if (SCHEME == LUTKAN_ASYM_UINT8) {
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[p][c] = fmaf(ym[c], kTwoToMinus24, acc[p][c]);
        }
        if constexpr (BASE) {
          const float silu_x = __uint_as_float(rc_cur.z);
          acc[p][0] = fmaf(base_gain.x, silu_x, acc[p][0]);
          acc[p][1] = fmaf(base_gain.y, silu_x, acc[p][1]);
          acc[p][2] = fmaf(base_gain.z, silu_x, acc[p][2]);
          acc[p][3] = fmaf(base_gain.w, silu_x, acc[p][3]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k = 0; k < AHEAD; ++k) rcq[k] = rcq[k + 1];
      rcq[AHEAD] = rc_new;
#pragma unroll
      for (int k = 0; k + 1 < AHEAD; ++k) fq[k] = fq[k + 1];
      fq[AHEAD - 1] = f_new;
    }
    if (PIPE == 2) {
      wait_all_vector_loads();                         // my share of the next slice has landed ...
      lds_barrier();                                   // ... everyone's has, and everyone is done with this one
    }
    cur = nxt;
  }

  const int j = t * JT + sub * 4;
#pragma unroll
  for (int p = 0; p < NP; ++p) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (!VALUES) acc[p][c] *= kTwoTo24;                                      // exact: undo the 2^-24 of the codes
    const int64_t b = b0 + p * RPS + hrow;
    if (b < a.B) {
      if (j + 3 < a.m && (a.m & 3) == 0) {
        f32x4 out = f32x4{acc[p][0], acc[p][1], acc[p][2], acc[p][3]};
        if (a.accumulate) out = *reinterpret_cast<const f32x4 *>(yout + b * a.m + j) + out;
        *reinterpret_cast<f32x4 *>(yout + b * a.m + j) = out;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (j + c < a.m) yout[b * a.m + j + c] = a.accumulate ? yout[b * a.m + j + c] + acc[p][c] : acc[p][c];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Fused chain for narrow networks and small batches (Sec. 5.1 chaining; the batch-256 latency setting of Sec. 8).
// ------------------------------------------------------------------------------------------------
// WPR waves (4 or 1) carry one row through every layer; nothing but the input row, the optional hidden activations
// and the output row touches global memory besides the tables, and the whole network is one launch.  Per layer:
//   locate   the row's WPR*64 lanes take the layer's inputs (from global memory for the first layer, from the row's
//            activation buffer in LDS afterwards), run steps 1-4 of Sec. 4.5 with the same code as the locate
//            kernel and leave one record per input in the row's LDS record buffer
//   edges    a wave is S = 64/jt groups of jt columns, the row's waves WPR*S groups; group g walks the inputs g,
//            g + WPR*S, ... (four at a time, so their table reads are in flight together), a lane accumulates its
//            column over them with the arithmetic of the gather kernel; a fixed butterfly adds the groups of a wave,
//            and with WPR = 4 the four waves' sums are added in wave order through LDS
//   the m sums become the next layer's inputs (LDS), and, if asked for, a row of the hidden-activation trace.
// A work-group is four waves: one row (WPR = 4) or four rows (WPR = 1).  Splitting a row's inputs over four waves
// shortens the chain of dependent table reads per layer, which is what a small batch waits for; one wave per row
// moves a quarter of the work-groups through the GPU and wins from a few thousand rows on.  Every barrier is reached
// by every thread: all loops over layers are uniform, rows past B are computed on row B-1 and not stored.
constexpr int kChainWaves = 4;          // the sum over the waves below is written out for four
constexpr int kChainMaxLayers = 8;
constexpr int kChainMaxInputs = 1024;     // widest layer input: its records must fit the LDS record buffer
constexpr int kChainMaxColumns = 64;      // widest layer output: one lane per column

struct ChainLayer {
  const unsigned char *table;
  const float *input_knots;        // nullable: [d][K+1], one knot vector per input (read from global memory)
  int32_t d, m, K, L, jt_log2, blob_bytes;
  int32_t codes_off, params_off, param_row_bytes;
  int32_t sym, with_base, param_fp16, closed, zero_spline;
  float tKs;
  float knots[LUTKAN_MAX_K + 1];
};

struct ChainArgs {
  const float *x;
  float *y;
  float *hidden;                   // nullable: the activations between the layers, layer after layer, each [B][m_l]
  unsigned long long *stats;       // nullable: two counters per layer
  int64_t B;
  int32_t n_layers, rec_stride;    // rec_stride: record slots (the widest layer input)
  ChainLayer layer[kChainMaxLayers];
};

template <int WPR>
__global__ __launch_bounds__(kChainWaves * 64) void lutkan_chain_kernel(const ChainArgs a) {
  static_assert(WPR == 1 || WPR == kChainWaves, "a row is carried by one wave or by the whole work-group");
  constexpr int ROWS = kChainWaves / WPR;                // rows per work-group
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int rrow = wave / WPR;                           // which of the work-group's rows
  const int wr = wave % WPR;                             // which of the row's waves
  const int rtid = wr * 64 + lane;                       // thread index inside the row's waves
  // LDS: records [ROWS][rec_stride] of 16 bytes, activations [ROWS][64], per-wave sums [waves][64], outside
  // counts [waves], knots [n_layers][MAX_K+1]
  u32x4 *s_rec = reinterpret_cast<u32x4 *>(lds) + (size_t)rrow * a.rec_stride;
  float *s_act_all = reinterpret_cast<float *>(lds + (size_t)ROWS * a.rec_stride * 16);
  float *s_act = s_act_all + rrow * kChainMaxColumns;
  float *s_part = s_act_all + ROWS * kChainMaxColumns;
  unsigned *s_outside = reinterpret_cast<unsigned *>(s_part + kChainWaves * kChainMaxColumns);
  float *s_knots = reinterpret_cast<float *>(s_outside + kChainWaves);
  for (int q = tid; q < a.n_layers * (LUTKAN_MAX_K + 1); q += kChainWaves * 64) {
    const int l = q / (LUTKAN_MAX_K + 1), kappa = q - l * (LUTKAN_MAX_K + 1);
    s_knots[q] = (kappa <= a.layer[l].K) ? a.layer[l].knots[kappa] : 0.0f;
  }
  __syncthreads();
  const int64_t row = (int64_t)blockIdx.x * ROWS + rrow;
  const bool live = row < a.B;
  const int64_t b = live ? row : a.B - 1;
  int64_t hidden_off = 0;

  for (int l = 0; l < a.n_layers; ++l) {
    const ChainLayer &Y = a.layer[l];
    const float *T = s_knots + l * (LUTKAN_MAX_K + 1);
    // ---- locate: one record per input of this row
    const unsigned masked_index = (unsigned)(Y.K * Y.L) | ((unsigned)Y.K << 16);
    unsigned outside = 0;
    for (int i = rtid; i < Y.d; i += WPR * 64) {
      const float x = (l == 0) ? a.x[b * Y.d + i] : s_act[i];
      const Located o = Y.input_knots ? locate_one<true>(Y, Y.input_knots + (int64_t)i * (Y.K + 1), x) : locate_one<false>(Y, T, x);
      u32x4 rec = {masked_index, 0u, 0u, 0u};
      const bool masked = Y.zero_spline && !o.inside && !o.is_nan;
      if (!masked) {
        rec.x = (unsigned)(o.k * Y.L + o.l0) | ((unsigned)o.k << 16);
        rec.y = __float_as_uint(o.is_nan ? __builtin_nanf("") : o.w);
      }
      if (Y.with_base) rec.z = __float_as_uint(__fdiv_rn(x, 1.0f + expf(-x)));          // SiLU at the raw input, never masked
      s_rec[i] = rec;
      outside += o.inside ? 0u : 1u;
    }
    if (a.stats) {                                       // Sec. 5.5 counters of this layer
      for (int off = 32; off > 0; off >>= 1) outside += __shfl_down(outside, off, kWave);
      if (lane == 0) s_outside[wave] = outside;
    }
    __syncthreads();                                     // records written (and the activations they came from read)
    if (a.stats && rtid == 0 && live) {
      unsigned total = 0;
      for (int v = 0; v < WPR; ++v) total += s_outside[rrow * WPR + v];
      if (total) {
        atomicAdd(&a.stats[2 * l], (unsigned long long)total);
        atomicAdd(&a.stats[2 * l + 1], 1ull);
      }
    }

    // ---- edges: lane = (group s of its wave, column jj); group g = wave * S + s takes the inputs g, g + 4S, ...
    const int jt = 1 << Y.jt_log2;
    const int jj = lane & (jt - 1);
    const int S = 64 >> Y.jt_log2;
    const int g = wr * S + (lane >> Y.jt_log2);
    const int stride = WPR * S;
    constexpr int U = 4;
    float acc = 0.0f;
    for (int i0 = g; i0 < Y.d; i0 += U * stride) {
      u32x4 rec[U];
      unsigned c0[U], c1[U];
      float al[U], ym[U], bg[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = min(i0 + u * stride, Y.d - 1);
        rec[u] = s_rec[i];
        const unsigned char *slice = Y.table + (size_t)i * Y.blob_bytes;
        const unsigned code_off = (unsigned)Y.codes_off + (rec[u].x & 0xffffu) * (unsigned)jt;
        const unsigned param_off = (unsigned)Y.params_off + (rec[u].x >> 16) * (unsigned)Y.param_row_bytes;
        c0[u] = slice[code_off + jj];
        c1[u] = slice[code_off + jt + jj];
        if (Y.param_fp16) {
          const _Float16 *prm = reinterpret_cast<const _Float16 *>(slice + param_off);
          al[u] = (float)prm[jj];
          ym[u] = Y.sym ? 0.0f : (float)prm[jt + jj];
        } else {
          const float *prm = reinterpret_cast<const float *>(slice + param_off);
          al[u] = prm[jj];
          ym[u] = Y.sym ? 0.0f : prm[jt + jj];
        }
        bg[u] = Y.with_base ? reinterpret_cast<const float *>(slice)[jj] : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i0 + u * stride < Y.d) {
          const float w = __uint_as_float(rec[u].y);
          const float bias = Y.sym ? 128.0f : 0.0f;                           // int8 codes are stored excess-128
          const float f0 = (float)c0[u] - bias, f1 = (float)c1[u] - bias;
          const float tq = fmaf(w, f1 - f0, f0);                               // Eq. 17 on the codes ...
          acc = fmaf(al[u], tq, acc);                                          // ... Eq. 10 once per edge
          if (!Y.sym) acc += ym[u];
          if (Y.with_base) acc = fmaf(bg[u], __uint_as_float(rec[u].z), acc);  // + s_out*s_base * SiLU(x)
        }
      }
    }
    for (int off = jt; off < 64; off <<= 1) acc += __shfl_xor(acc, off, kWave);          // fixed order over a wave's groups
    if (lane < jt) s_part[wave * kChainMaxColumns + lane] = acc;
    __syncthreads();                                     // the waves' sums are in place; everyone is done with the records
    const bool last = (l + 1 == a.n_layers);
    if (rtid < Y.m) {
      const float *part = s_part + rrow * WPR * kChainMaxColumns + rtid;
      float total = part[0];
      for (int v = 1; v < WPR; ++v) total += part[v * kChainMaxColumns];     // wave order
      if (last) {
        if (live) a.y[b * Y.m + rtid] = total;
      } else {
        s_act[rtid] = total;
        if (a.hidden && live) a.hidden[hidden_off + b * Y.m + rtid] = total;
      }
    }
    hidden_off += a.B * Y.m;
    __syncthreads();                                     // the next layer's inputs are in place, its records may be overwritten
  }
}

int validate_layer(const lutkan_dev_layer *l, const char *who) {
  if (!l) return fail(LUTKAN_EINVAL, "%s: null layer", who);
  if (!l->table) return fail(LUTKAN_EINVAL, "%s: layer.table is null", who);
  if (l->d < 1 || l->m < 1 || l->K < 1 || l->L < 2) return fail(LUTKAN_EINVAL, "%s: bad d/m/K/L (%d,%d,%d,%d)", who, l->d, l->m, l->K, l->L);
  if (l->K > LUTKAN_MAX_K || (int64_t)l->K * l->L > LUTKAN_MAX_ROWS) return fail(LUTKAN_EUNSUPPORTED, "%s: K or K*L too large", who);
  if (l->scheme != LUTKAN_SYM_INT8 && l->scheme != LUTKAN_ASYM_UINT8) return fail(LUTKAN_EINVAL, "%s: bad scheme %d", who, l->scheme);
  if (l->boundary != LUTKAN_HALF_OPEN && l->boundary != LUTKAN_CLOSED) return fail(LUTKAN_EINVAL, "%s: bad boundary_mode %d", who, l->boundary);
  if (l->oob != LUTKAN_CLIP_X && l->oob != LUTKAN_ZERO_SPLINE) return fail(LUTKAN_EINVAL, "%s: bad oob_policy %d", who, l->oob);
  if (l->algo < LUTKAN_ALGO_AUTO || l->algo > LUTKAN_ALGO_TILED_WIDE) return fail(LUTKAN_EINVAL, "%s: bad algo %d", who, l->algo);
  if (l->value_repr != LUTKAN_REPR_PHI && l->value_repr != LUTKAN_REPR_SPLINE_COMPONENT) return fail(LUTKAN_EINVAL, "%s: bad value_repr %d", who, l->value_repr);
  if (l->param_dtype != LUTKAN_PARAM_FP32 && l->param_dtype != LUTKAN_PARAM_FP16) return fail(LUTKAN_EINVAL, "%s: bad param_dtype %d", who, l->param_dtype);
  for (int k = 0; k < l->K; ++k)
    if (!(l->knots[k] < l->knots[k + 1])) return fail(LUTKAN_EINVAL, "%s: knots not strictly increasing at %d", who, k);
  if (l->jt < 4 || l->jt > 64 || (l->jt & (l->jt - 1))) return fail(LUTKAN_EINVAL, "%s: jt=%d is not a power of two in [4,64]", who, l->jt);
  if (l->n_tiles != (l->m + l->jt - 1) / l->jt) return fail(LUTKAN_ESHAPE, "%s: n_tiles does not match m and jt", who);
  if (l->blob_bytes != lutkan::blob_layout(l->K, l->L, l->jt, l->scheme, l->value_repr, l->param_dtype).bytes) return fail(LUTKAN_ESHAPE, "%s: blob_bytes does not match K, L, jt, scheme, param_dtype", who);
  if ((reinterpret_cast<uintptr_t>(l->table) & 15) != 0) return fail(LUTKAN_EINVAL, "%s: table must be 16-byte aligned", who);
  if (l->wide_table) {
    const int cb = l->wide_code_bytes;
    if (!lutkan::has_wide_form(l->jt, l->K, l->L, l->scheme, l->value_repr, l->param_dtype, cb)) return fail(LUTKAN_EINVAL, "%s: wide_table set on a layer that has no wide form with wide_code_bytes = %d", who, cb);
    if (l->wide_blob_bytes != lutkan::wide_blob_layout(l->K, l->L, l->jt, l->scheme, l->value_repr, l->param_dtype, cb).bytes) return fail(LUTKAN_ESHAPE, "%s: wide_blob_bytes does not match K, L, jt, scheme, param_dtype, wide_code_bytes", who);
    if ((reinterpret_cast<uintptr_t>(l->wide_table) & 15) != 0) return fail(LUTKAN_EINVAL, "%s: wide_table must be 16-byte aligned", who);
  }
  if (l->knots_per_input != 0 && l->knots_per_input != 1) return fail(LUTKAN_EINVAL, "%s: bad knots_per_input %d", who, l->knots_per_input);
  if (l->knots_per_input && (!l->input_knots || (reinterpret_cast<uintptr_t>(l->input_knots) & 3) != 0))
    return fail(LUTKAN_EINVAL, "%s: knots_per_input needs layer.input_knots (device, 4-byte aligned)", who);
  return LUTKAN_OK;
}

// True when a batch is so small that gathering only the table rows it touches (gather kernel, inputs split over the
// GPU) beats the tiled kernel, which streams the whole table once whatever the batch.  A table that the caches hold
// (up to 128 MiB): when the bytes the lanes request (per row, input and column tile two code rows and one parameter
// row) stay below the table's (measured: 256x256 near 128 rows).  A larger table streams from HBM on every tiled
// launch, and scattered reads of it pay off for longer: the gather kernel is priced at 8 us plus the requested bytes
// at 9.4 TB/s, the tiled launch at the estimate of its launch planning (measured: 1024x1024 between 128 and 256 rows).
bool prefer_gather_for_small_batch(const lutkan_dev_layer *l, int64_t B, double tiled_cost_us) {
  const lutkan::BlobLayout lay = lutkan::blob_layout(l->K, l->L, l->jt, l->scheme, l->value_repr, l->param_dtype);
  const double touched = (double)B * l->d * l->n_tiles * (2.0 * l->jt + (double)lay.param_row_bytes);
  const double table = (double)l->n_tiles * l->d * l->blob_bytes;
  if (table <= 128.0 * 1024 * 1024) return touched <= table;
  return 8.0 + touched / 9.4e6 <= tiled_cost_us;
}

// Which pipeline mode of the tiled kernel a launch runs in (its PIPE parameter): three slice and record buffers where
// they fit and the kernel has that form -- the barrier leaves the critical path (3), or, for a launch that waits for
// the table to stream from HBM, two slices are in flight (4) -- else two buffers (2).
int tiled_pipe(const EdgeArgs &ea, int np) {
  const int rows_per_wave = 64 / (ea.jt / 4) * np;
  const size_t lds3 = 3 * (size_t)ea.blob_bytes + (size_t)kTileWaves * 3 * rows_per_wave * 8;
  if (ea.with_base || lds3 > (size_t)kMaxTiledLds) return 2;
  if (ea.deep && !ea.wide) return 4;
  if (ea.wide == 2 && ea.asym && np == 16) return 2;    // (what that variant carries across inputs no longer fits 128 registers)
  return np >= (ea.wide ? 4 : 2) ? 3 : 2;             // carried reads: more row steps per input than the kernel reads ahead
}

template <int SCHEME, int LPR, int NP>
int launch_tiled_np(const EdgeArgs &ea, hipStream_t s) {
  constexpr int NW = kTileWaves;
  constexpr int RW = (64 / LPR) * NP;
  const int64_t row_tiles = (ea.B + NW * RW - 1) / (NW * RW);
  if (row_tiles * ea.n_tiles > 0x7fffffffLL) return fail(LUTKAN_EUNSUPPORTED, "lutkan_tiled_kernel: B * m too large for one launch");
  const dim3 grid((unsigned)(row_tiles * ea.n_tiles), (unsigned)((ea.d + ea.chunk - 1) / ea.chunk));
  const int pipe = tiled_pipe(ea, NP);
  const size_t lds = (pipe == 2) ? 2 * (size_t)ea.blob_bytes + (size_t)NW * 2 * RW * (ea.with_base ? 16 : 8)
                                 : 3 * (size_t)ea.blob_bytes + (size_t)NW * 3 * RW * 8;
#define LUTKAN_LAUNCH_TILED(SCH, BASE, PH, PIPE, CB)                                                                             \
  do {                                                                                                                           \
    static LdsCap raised;                                                                                                        \
    return launch_with_lds(lutkan_tiled_kernel<SCH, LPR, NP, NW, BASE, PH, PIPE, CB>, &raised, grid, lds, s, ea, "lutkan_tiled_kernel"); \
  } while (0)
  // binary16 parameter rows exist on tiles of at most 32 columns only (device_params_are_half), the wide forms of the
  // table on 64-column tiles only: neither kernel variant is built for the other tile widths
  constexpr bool kHalfParams = (LPR <= 8), kWideForms = (LPR == 16);
  if (ea.param_fp16 && !kHalfParams) return fail(LUTKAN_EINVAL, "lutkan_tiled_kernel: binary16 parameter rows go with tiles of at most 32 columns");
  if (ea.wide && !kWideForms) return fail(LUTKAN_EINVAL, "lutkan_tiled_kernel: the wide table goes with 64-column tiles");
  if (ea.with_base) {
    if (ea.wide == 2) return fail(LUTKAN_EINVAL, "lutkan_tiled_kernel: the table with 16-bit codes goes with 8-byte records");
    if constexpr (kWideForms) { if (ea.wide == 4) LUTKAN_LAUNCH_TILED(0, true, false, 2, 4); }
    LUTKAN_LAUNCH_TILED(SCHEME, true, false, 2, 1);
  }
  if constexpr (kHalfParams) {
    if (ea.param_fp16) {
      if (pipe == 4) LUTKAN_LAUNCH_TILED(SCHEME, false, true, 4, 1);
      if constexpr (NP >= 2) { if (pipe == 3) LUTKAN_LAUNCH_TILED(SCHEME, false, true, 3, 1); }
      LUTKAN_LAUNCH_TILED(SCHEME, false, true, 2, 1);
    }
  }
  if constexpr (kWideForms) {
    if constexpr (NP >= 4) {
      if (pipe == 3 && ea.wide == 4) LUTKAN_LAUNCH_TILED(0, false, false, 3, 4);
      if constexpr (!(SCHEME == LUTKAN_ASYM_UINT8 && NP == 16)) {          // (tiled_pipe never asks for that one: it does not fit the registers)
        if (pipe == 3 && ea.wide == 2) LUTKAN_LAUNCH_TILED(SCHEME, false, false, 3, 2);
      }
    }
    if (ea.wide == 4) LUTKAN_LAUNCH_TILED(0, false, false, 2, 4);
    if (ea.wide == 2) LUTKAN_LAUNCH_TILED(SCHEME, false, false, 2, 2);
  }
  if (pipe == 4) LUTKAN_LAUNCH_TILED(SCHEME, false, false, 4, 1);
  if constexpr (NP >= 2) { if (pipe == 3) LUTKAN_LAUNCH_TILED(SCHEME, false, false, 3, 1); }
  LUTKAN_LAUNCH_TILED(SCHEME, false, false, 2, 1);
#undef LUTKAN_LAUNCH_TILED
}

template <int SCHEME, int LPR>
int launch_tiled(const EdgeArgs &ea, int np, hipStream_t s) {
  constexpr int kMaxNp = (64 / (64 / LPR) < 16) ? 64 / (64 / LPR) : 16;      // at most 64 rows per wave
  if constexpr (kMaxNp >= 16) { if (np >= 16) return launch_tiled_np<SCHEME, LPR, 16>(ea, s); }
  if constexpr (kMaxNp >= 8) { if (np >= 8) return launch_tiled_np<SCHEME, LPR, 8>(ea, s); }
  if constexpr (kMaxNp >= 4) { if (np >= 4) return launch_tiled_np<SCHEME, LPR, 4>(ea, s); }
  if constexpr (kMaxNp >= 2) { if (np >= 2) return launch_tiled_np<SCHEME, LPR, 2>(ea, s); }
  return launch_tiled_np<SCHEME, LPR, 1>(ea, s);
}

template <int SCHEME>
int launch_tiled_jt(const EdgeArgs &ea, int np, hipStream_t s) {
  switch (ea.jt) {
    case 64: return launch_tiled<SCHEME, 16>(ea, np, s);
    case 32: return launch_tiled<SCHEME, 8>(ea, np, s);
    case 16: return launch_tiled<SCHEME, 4>(ea, np, s);
    case 8: return launch_tiled<SCHEME, 2>(ea, np, s);
    default: return launch_tiled<SCHEME, 1>(ea, np, s);
  }
}

bool tiled_supported(int jt, int blob_bytes, int value_repr) {
  return jt >= 4 && blob_bytes <= lutkan::lds_slice_budget(value_repr);
}


template <bool BASE, bool PERIN>
void launch_locate(int cols, dim3 grid, hipStream_t s, const LocateArgs &la) {
  if (cols == 64) hipLaunchKernelGGL((lutkan_locate_kernel<BASE, 64, PERIN>), grid, dim3(256), 0, s, la);
  else if (cols == 32) hipLaunchKernelGGL((lutkan_locate_kernel<BASE, 32, PERIN>), grid, dim3(256), 0, s, la);
  else hipLaunchKernelGGL((lutkan_locate_kernel<BASE, 16, PERIN>), grid, dim3(256), 0, s, la);
}

// The fused chain: validation, kernel arguments and launch (the body of lutkan_chain_forward; lutkan_forward also
// comes here with a single small layer).
int chain_impl(const lutkan_dev_layer *layers, int32_t n_layers, const float *x, int64_t B, float *y,
               float *hidden, lutkan_oob_stats *stats, void *hip_stream, const char *who) {
  if (!layers || n_layers < 1) return fail(LUTKAN_EINVAL, "%s: need at least one layer", who);
  if (n_layers > kChainMaxLayers) return fail(LUTKAN_EUNSUPPORTED, "%s: at most %d layers (got %d)", who, kChainMaxLayers, n_layers);
  ChainArgs ca = {};
  int widest = 0;
  for (int l = 0; l < n_layers; ++l) {
    const lutkan_dev_layer *L = &layers[l];
    if (int rc = validate_layer(L, who)) return rc;
    if (l + 1 < n_layers && L->m != layers[l + 1].d) return fail(LUTKAN_ESHAPE, "%s: layer %d has m=%d but layer %d has d=%d", who, l, L->m, l + 1, layers[l + 1].d);
    if (L->n_tiles != 1 || L->jt > kChainMaxColumns) return fail(LUTKAN_EUNSUPPORTED, "%s: layer %d has %d outputs in %d column tiles, the fused chain takes one tile of at most %d columns", who, l, L->m, L->n_tiles, kChainMaxColumns);
    if (L->d > kChainMaxInputs) return fail(LUTKAN_EUNSUPPORTED, "%s: layer %d has %d inputs, the fused chain takes at most %d", who, l, L->d, kChainMaxInputs);
    const lutkan::BlobLayout lay = lutkan::blob_layout(L->K, L->L, L->jt, L->scheme, L->value_repr, L->param_dtype);
    ChainLayer &c = ca.layer[l];
    c.table = static_cast<const unsigned char *>(L->table);
    c.input_knots = L->knots_per_input ? L->input_knots : nullptr;
    c.d = L->d; c.m = L->m; c.K = L->K; c.L = L->L; c.blob_bytes = L->blob_bytes;
    c.jt_log2 = 0;
    while ((1 << c.jt_log2) < L->jt) ++c.jt_log2;
    c.codes_off = lay.codes_off; c.params_off = lay.params_off; c.param_row_bytes = lay.param_row_bytes;
    c.sym = (L->scheme == LUTKAN_SYM_INT8);
    c.with_base = (L->value_repr == LUTKAN_REPR_SPLINE_COMPONENT);
    c.param_fp16 = lutkan::device_params_are_half(L->value_repr, L->param_dtype, L->jt);
    c.closed = (L->boundary == LUTKAN_CLOSED);
    c.zero_spline = (L->oob == LUTKAN_ZERO_SPLINE);
    c.tKs = c.closed ? L->knots[L->K] : std::nextafterf(L->knots[L->K], -INFINITY);
    for (int k = 0; k <= L->K; ++k) c.knots[k] = L->knots[k];
    widest = std::max(widest, L->d);
  }
  if (B < 0) return fail(LUTKAN_EINVAL, "%s: B < 0", who);
  if (B == 0) return LUTKAN_OK;
  if (!x || !y || x == y) return fail(LUTKAN_EINVAL, "%s: null or aliased x / y", who);
  // up to 1024 rows a whole work-group carries a row (the shortest path through a layer); beyond, one wave does
  const int wpr = (B <= 1024) ? kChainWaves : 1;
  const int rows_per_group = kChainWaves / wpr;
  const int64_t groups = (B + rows_per_group - 1) / rows_per_group;
  if (groups > 0x7fffffff) return fail(LUTKAN_EUNSUPPORTED, "%s: B too large", who);
  ca.x = x; ca.y = y; ca.hidden = hidden;
  ca.stats = reinterpret_cast<unsigned long long *>(stats);
  ca.B = B; ca.n_layers = n_layers; ca.rec_stride = widest;
  const size_t lds = (size_t)rows_per_group * widest * 16 + (size_t)(rows_per_group + kChainWaves) * kChainMaxColumns * 4 +
                     kChainWaves * 4 + (size_t)n_layers * (LUTKAN_MAX_K + 1) * 4;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (wpr == 1) {
    static LdsCap raised;         // four rows of the widest layer need more than the default 64 KiB
    if (int rc = raise_lds_cap(lutkan_chain_kernel<1>, &raised, who)) return rc;
    hipLaunchKernelGGL(lutkan_chain_kernel<1>, dim3((unsigned)groups), dim3(kChainWaves * 64), lds, s, ca);
  } else {
    hipLaunchKernelGGL(lutkan_chain_kernel<kChainWaves>, dim3((unsigned)groups), dim3(kChainWaves * 64), lds, s, ca);
  }
  lutkan::plan_note("chain layers=%d wpr=%d; ", n_layers, wpr);
  return check_launch("lutkan_chain_kernel");
}

// The layers that AUTO runs as a launch of the chain kernel (see forward_impl): one column tile, d * jt <= 4096, and
// few enough rows.  Measured on 16x2 ... 256x16 layers between 8192 and 131072 rows: the chain kernel takes about
// 4 us + (0.35 + 0.00088 d jt) us per 1000 rows, locate + tiled kernel + summing pass about 17 us + (0.05 + 0.00035 d jt)
// us per 1000 rows; the chain kernel wins below their crossing, taken a little low (16x2: up to 30000 rows, 78x16:
// 10000, 64x32: 7000, 256x16: 4000).
bool small_layer_runs_as_chain(const lutkan_dev_layer *l, int64_t B) {
  if (l->algo != LUTKAN_ALGO_AUTO || l->n_tiles != 1 || l->jt > kChainMaxColumns || l->d * l->jt > 4096) return false;
  return (double)B * (0.30 + 0.00053 * l->d * l->jt) <= 10000.0;
}

int forward_impl(const lutkan_dev_layer *l, const float *x, int64_t B, float *y, lutkan_oob_stats *stats,
                 int32_t *k_out, int32_t *l0_out, uint8_t *in_out, float *w_out, int16_t *q01_out, bool trace,
                 void *workspace, size_t workspace_bytes, void *hip_stream, const char *who, int phases = kLocate | kEdges) {
  if (int rc = validate_layer(l, who)) return rc;
  if (B < 0) return fail(LUTKAN_EINVAL, "%s: B < 0", who);
  if (B == 0) return LUTKAN_OK;
  if (((phases & kLocate) && !x) || ((phases & kEdges) && !y)) return fail(LUTKAN_EINVAL, "%s: null x or y", who);
  if (x == y) return fail(LUTKAN_EINVAL, "%s: x and y alias", who);
  if (trace && (!k_out || !l0_out || !in_out || !w_out)) return fail(LUTKAN_EINVAL, "%s: null trace output", who);
  const size_t need = lutkan_forward_workspace_bytes(l, B);
  if (!workspace || workspace_bytes < need) return fail(LUTKAN_ESHAPE, "%s: workspace of %zu bytes, need %zu", who, workspace_bytes, need);
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return fail(LUTKAN_EINVAL, "%s: workspace must be 256-byte aligned", who);
  // A small narrow layer at a moderate batch: the one-launch chain kernel with a single layer beats locate + edge
  // kernel (+ partial sums) by 1.4-2x (78x16, 128x8, 64x32 up to 8192 rows); with more inputs per output column the
  // per-row walk over the inputs gets too long for it (256x64, 1024x64: slower).
  if (phases == (kLocate | kEdges) && !trace && !q01_out && small_layer_runs_as_chain(l, B))
    return chain_impl(l, 1, x, B, y, nullptr, stats, hip_stream, who);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t Bp = padded_rows(B);
  const lutkan::BlobLayout lay = lutkan::blob_layout(l->K, l->L, l->jt, l->scheme, l->value_repr, l->param_dtype);

  // Which edge kernel runs, and how the base branch of a spline_component layer is evaluated, follow from the layer
  // and B alone, so that the two phases agree when they are called separately.
  const bool with_base = (l->value_repr == LUTKAN_REPR_SPLINE_COMPONENT);
  bool tiled = tiled_supported(l->jt, l->blob_bytes, l->value_repr) && !q01_out;
  if (l->algo == LUTKAN_ALGO_GATHER) tiled = false;
  const TilePlan tp = tiled ? plan_tiles(B, l->d, l->m, l->n_tiles, 64 / (l->jt / 4), l->blob_bytes) : TilePlan{1, 1, l->d, 0.0, false};
  if (l->algo == LUTKAN_ALGO_AUTO && tiled && prefer_gather_for_small_batch(l, B, tp.cost)) tiled = false;
  const bool tiled_asked_for = (l->algo == LUTKAN_ALGO_TILED || l->algo == LUTKAN_ALGO_TILED_WIDE);
  if (tiled_asked_for && !tiled) return fail(LUTKAN_EUNSUPPORTED, "%s: tiled kernel needs a table slice <= 72 KiB (64 KiB with the base branch)%s", who, q01_out ? " and writes no code trace" : "");
  // Base branch as a matrix product of its own (SiLU(X) times the s_out*s_base of the table's base rows, into y) with
  // the edge kernel of a phi layer adding the spline branch on top.  Measured against the base FMAs inside the edge
  // kernel (four per four edges, 16-byte records): 1024x1024 at 32768 rows 5.87 -> 5.47 ms (uint8 codes 6.67 -> 5.97),
  // at 2048 rows 0.55 -> 0.52; 128x128 at 131072 rows 0.59 -> 0.55; 256x256 at 16384 rows 0.260 -> 0.248, but at
  // 2048 rows 0.056 -> 0.071 (three more launches): hence the floor on the work of the layer.
  const bool base_by_product = with_base && tiled && (double)B * l->d * l->m >= kBaseProductMinEdges && lutkan::base_product_fits(l->d, l->m, B);
  const int rec_bytes = (with_base && !base_by_product) ? 16 : 8;
  // A wide form of the table (16-bit codes or fp32 values: fewer vector instructions per edge, two or four times the
  // table bytes), where the layer has one and the launch planning prices it lower.
  // With 16-byte records (the base branch inside the edge kernel) only the fp32 values can be used, and their slice
  // must leave room for the larger record buffers.
  const int wide_cb = l->wide_code_bytes;
  const bool can_wide = tiled && l->wide_table != nullptr &&
                        (rec_bytes == 8 || (wide_cb == 4 && l->wide_blob_bytes <= lutkan::lds_slice_budget(LUTKAN_REPR_SPLINE_COMPONENT)));
  const TilePlan tpw = can_wide ? plan_tiles(B, l->d, l->m, l->n_tiles, 64 / (l->jt / 4), l->wide_blob_bytes, wide_cb) : tp;
  // (with y_min the row step on 16-bit codes reads 56 bytes per lane from LDS and measured within 3 % of the byte form
  // either way on 256x256 and 128x128 layers: left to the byte form unless asked for)
  const bool wide = can_wide && ((tpw.cost < tp.cost && (wide_cb == 4 || l->scheme == LUTKAN_SYM_INT8)) || l->algo == LUTKAN_ALGO_TILED_WIDE);
  if (l->algo == LUTKAN_ALGO_TILED_WIDE && !wide)
    return fail(LUTKAN_EUNSUPPORTED, "%s: algo TILED_WIDE on a layer %s", who, l->wide_table ? "whose base branch runs inside the edge kernel (16-byte records: fp32 values of at most 64 KiB per slice only)" : "without a wide table");
  // workspace: [records: room for 16 bytes each with the base branch; 8-byte records leave room for the 6 bytes per
  // (row, input) of the SiLU pieces behind them] [pieces of s_out*s_base, spline_component only] [partial sums]
  char *const ws_bytes = static_cast<char *>(workspace);
  uint16_t *silu_pieces = reinterpret_cast<uint16_t *>(ws_bytes + record_bytes(l->d, Bp, 8));
  const size_t records_end = record_bytes(l->d, Bp, lut_record_bytes(l->value_repr));
  uint16_t *w_pieces = reinterpret_cast<uint16_t *>(ws_bytes + records_end);
  float *const partials = reinterpret_cast<float *>(ws_bytes + records_end + (with_base ? lutkan::base_product_workspace_bytes(l->d, l->m) : 0));

  LocateArgs la;
  la.x = x;
  la.rec = workspace;
  la.silu_pieces = base_by_product ? silu_pieces : nullptr;
  la.B = B; la.Bp = Bp; la.d = l->d; la.K = l->K; la.L = l->L;
  la.closed = (l->boundary == LUTKAN_CLOSED);
  la.zero_spline = (l->oob == LUTKAN_ZERO_SPLINE);
  la.tKs = la.closed ? l->knots[l->K] : std::nextafterf(l->knots[l->K], -INFINITY);
  for (int k = 0; k <= l->K; ++k) la.knots[k] = l->knots[k];
  la.input_knots = l->knots_per_input ? l->input_knots : nullptr;
  la.k_out = trace ? k_out : nullptr; la.l0_out = l0_out; la.in_out = in_out; la.w_out = w_out;
  if (phases & kLocate) {
    // inputs per block: the width in {64, 32, 16} that pads d least (the widest on ties: longer runs of x)
    int cols = 64;
    for (int c = 32; c >= 16; c >>= 1)
      if ((l->d + c - 1) / c * c < (l->d + cols - 1) / cols * cols) cols = c;
    const dim3 lgrid((unsigned)(Bp / (kLocTile / cols)), (unsigned)((l->d + cols - 1) / cols));
    if (lgrid.y > 65535u) return fail(LUTKAN_EUNSUPPORTED, "%s: d too large", who);
    if (l->knots_per_input) {
      if (rec_bytes == 16) launch_locate<true, true>(cols, lgrid, s, la);
      else launch_locate<false, true>(cols, lgrid, s, la);
    } else {
      if (rec_bytes == 16) launch_locate<true, false>(cols, lgrid, s, la);
      else launch_locate<false, false>(cols, lgrid, s, la);
    }
    if (int rc = check_launch("lutkan_locate_kernel")) return rc;
    lutkan::plan_note("locate; ");
    if (stats) {
      const int64_t rows_per_group = 4 * kOobRowsPerWave;
      hipLaunchKernelGGL(oob_count_kernel, dim3((unsigned)((B + rows_per_group - 1) / rows_per_group)), dim3(256), 0, s, x, B, l->d,
                         l->knots[0], l->knots[l->K], la.closed, la.input_knots, l->K, reinterpret_cast<unsigned long long *>(stats));
      if (int rc = check_launch("oob_count_kernel")) return rc;
      lutkan::plan_note("oob; ");
    }
  }
  if (!(phases & kEdges)) return LUTKAN_OK;

  EdgeArgs ea;
  ea.table = static_cast<const unsigned char *>(l->table);
  ea.rec = la.rec; ea.y = y; ea.q01_out = q01_out;
  ea.B = B; ea.Bp = Bp; ea.d = l->d; ea.m = l->m; ea.K = l->K; ea.L = l->L;
  ea.jt = l->jt; ea.n_tiles = l->n_tiles; ea.blob_bytes = l->blob_bytes;
  ea.codes_off = lay.codes_off; ea.params_off = lay.params_off; ea.param_row_bytes = lay.param_row_bytes;
  ea.with_base = (rec_bytes == 16); ea.k_out = k_out; ea.l0_out = l0_out;
  ea.param_fp16 = lutkan::device_params_are_half(l->value_repr, l->param_dtype, l->jt);
  ea.accumulate = 0;
  ea.wide = 0;
  ea.deep = 0;
  ea.asym = (l->scheme == LUTKAN_ASYM_UINT8);
  ea.chunk = l->d;
  ea.split_stride = 0;
  if (base_by_product) {
    if (int rc = lutkan::launch_base_product(silu_pieces, Bp, l->table, w_pieces, l->d, l->m, l->jt, l->blob_bytes, B, y, hip_stream, who)) return rc;
    lutkan::plan_note("base_product; ");
  }
  if (tiled) {
    const TilePlan &plan = wide ? tpw : tp;
    if (wide) {
      ea.table = static_cast<const unsigned char *>(l->wide_table);       // same tiles, longer code rows
      ea.blob_bytes = l->wide_blob_bytes;
      ea.wide = wide_cb;
      if (wide_cb == 4) {                                                   // no parameter rows: the value rows follow the base row
        ea.codes_off = lay.params_off; ea.params_off = lay.params_off; ea.param_row_bytes = 0;
        ea.param_fp16 = 0;
      }
    }
    ea.chunk = plan.chunk;
    ea.deep = plan.hbm_bound ? 1 : 0;
    if (plan.n_split > 1) { ea.y = partials; ea.split_stride = B * l->m; }
    ea.accumulate = (base_by_product && plan.n_split == 1) ? 1 : 0;     // with chunks, the summing pass adds to y instead
    const int rc = (l->scheme == LUTKAN_SYM_INT8) ? launch_tiled_jt<LUTKAN_SYM_INT8>(ea, plan.np, s) : launch_tiled_jt<LUTKAN_ASYM_UINT8>(ea, plan.np, s);
    if (rc) return rc;
    lutkan::plan_note("tiled%s np=%d split=%d pipe=%d; ", !wide ? "" : wide_cb == 4 ? " wide32" : " wide", plan.np, plan.n_split, tiled_pipe(ea, plan.np));
    if (plan.n_split == 1) return rc;
    const int64_t n = B * l->m;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, partials, y, n, plan.n_split, base_by_product ? 1 : 0);
    lutkan::plan_note("sum; ");
    return check_launch("sum_partials_kernel");
  }
  if (!q01_out) {
    // the plain launch: four columns per lane
    int lpr_log2 = 0;
    while ((4 << lpr_log2) < l->jt) ++lpr_log2;
    const GatherPlan gp = plan_gather(B, l->d, (l->n_tiles * l->jt) / 4);
    ea.chunk = gp.chunk;
    if (gp.n_split > 1) { ea.y = partials; ea.split_stride = B * l->m; }
    const int rows_per_group = 256 >> lpr_log2;
    const dim3 grid((unsigned)((B + rows_per_group - 1) / rows_per_group), (unsigned)l->n_tiles, (unsigned)gp.n_split);
    if (grid.y > 65535u) return fail(LUTKAN_EUNSUPPORTED, "%s: m too large for the gather kernel", who);
    const bool sym = (l->scheme == LUTKAN_SYM_INT8);
#define LUTKAN_LAUNCH_GATHER4(S, BASE, PH) hipLaunchKernelGGL((lutkan_gather4_kernel<S, BASE, PH, kGather4Inputs>), grid, dim3(256), 0, s, ea, lpr_log2)
    if (with_base) { if (sym) LUTKAN_LAUNCH_GATHER4(LUTKAN_SYM_INT8, true, false); else LUTKAN_LAUNCH_GATHER4(LUTKAN_ASYM_UINT8, true, false); }
    else if (ea.param_fp16) { if (sym) LUTKAN_LAUNCH_GATHER4(LUTKAN_SYM_INT8, false, true); else LUTKAN_LAUNCH_GATHER4(LUTKAN_ASYM_UINT8, false, true); }
    else { if (sym) LUTKAN_LAUNCH_GATHER4(LUTKAN_SYM_INT8, false, false); else LUTKAN_LAUNCH_GATHER4(LUTKAN_ASYM_UINT8, false, false); }
#undef LUTKAN_LAUNCH_GATHER4
    if (int rc = check_launch("lutkan_gather4_kernel")) return rc;
    lutkan::plan_note("gather split=%d; ", gp.n_split);
    if (gp.n_split == 1) return LUTKAN_OK;
    const int64_t n = B * l->m;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, partials, y, n, gp.n_split, 0);
    lutkan::plan_note("sum; ");
    return check_launch("sum_partials_kernel");
  }
  // the code trace: one column per lane, so that every edge's two codes can be written out
  const int lg = gather_jx_log2(l->m);
  const GatherPlan gp = plan_gather(B, l->d, l->m);
  ea.chunk = gp.chunk;
  if (gp.n_split > 1) { ea.y = partials; ea.split_stride = B * l->m; }
  const dim3 grid((unsigned)((B + (256 >> lg) - 1) / (256 >> lg)), (unsigned)((l->m + (1 << lg) - 1) >> lg), (unsigned)gp.n_split);
  if (grid.y > 65535u) return fail(LUTKAN_EUNSUPPORTED, "%s: m too large for the gather kernel", who);
  if (l->scheme == LUTKAN_SYM_INT8) {
    if (q01_out) hipLaunchKernelGGL((lutkan_gather_kernel<LUTKAN_SYM_INT8, true>), grid, dim3(256), 0, s, ea, lg);
    else hipLaunchKernelGGL((lutkan_gather_kernel<LUTKAN_SYM_INT8, false>), grid, dim3(256), 0, s, ea, lg);
  } else {
    if (q01_out) hipLaunchKernelGGL((lutkan_gather_kernel<LUTKAN_ASYM_UINT8, true>), grid, dim3(256), 0, s, ea, lg);
    else hipLaunchKernelGGL((lutkan_gather_kernel<LUTKAN_ASYM_UINT8, false>), grid, dim3(256), 0, s, ea, lg);
  }
  if (int rc = check_launch("lutkan_gather_kernel")) return rc;
  lutkan::plan_note("gather split=%d; ", gp.n_split);
  if (gp.n_split == 1) return LUTKAN_OK;
  const int64_t n = B * l->m;
  hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s, partials, y, n, gp.n_split, 0);
  lutkan::plan_note("sum; ");
  return check_launch("sum_partials_kernel");
}

}  // namespace

extern "C" size_t lutkan_forward_workspace_bytes(const lutkan_dev_layer *layer, int64_t B) {
  // 0 for anything validate_layer would refuse on these fields (a tile width that is not a power of two in 4 .. 64
  // would divide by zero in the launch planning)
  if (!layer || B <= 0 || layer->d < 1 || layer->m < 1 || layer->n_tiles < 1 || layer->blob_bytes < 1) return 0;
  if (layer->jt < 4 || layer->jt > 64 || (layer->jt & (layer->jt - 1))) return 0;
  size_t bytes = tiled_workspace_bytes(layer->d, layer->m, layer->jt, layer->n_tiles, B, lut_record_bytes(layer->value_repr), layer->blob_bytes);
  if (layer->wide_table && layer->wide_blob_bytes >= 1)
    bytes = std::max(bytes, tiled_workspace_bytes(layer->d, layer->m, layer->jt, layer->n_tiles, B, lut_record_bytes(layer->value_repr), layer->wide_blob_bytes, layer->wide_code_bytes));
  return bytes + (layer->value_repr == LUTKAN_REPR_SPLINE_COMPONENT ? lutkan::base_product_workspace_bytes(layer->d, layer->m) : 0);
}

// ------------------------------------------------------------------------------------------------
// The wide form of the table.
// ------------------------------------------------------------------------------------------------
namespace {

struct WidenArgs {
  const unsigned char *src;          // byte table, slices [t][i]
  unsigned char *dst;                // wide table, slices [t][i]
  int32_t jt, src_blob, dst_blob, codes_off, n_code_rows;
  int32_t sym;
  // fp32 values only
  int32_t params_off, param_row_bytes, L, K;
};

// One work-group per slice (t, i).  Base row and parameter rows are copied as they are (16 bytes per thread and
// step: codes_off is a multiple of 16); a code byte becomes the binary16 bit pattern of q * 2^-24: sign bit and, as
// the subnormal's significand, the magnitude of q.
__global__ __launch_bounds__(256) void lutkan_widen_kernel(const WidenArgs a) {
  const unsigned char *src = a.src + (size_t)blockIdx.x * a.src_blob;
  unsigned char *dst = a.dst + (size_t)blockIdx.x * a.dst_blob;
  for (int e = threadIdx.x * 16; e < a.codes_off; e += 256 * 16) *reinterpret_cast<u32x4 *>(dst + e) = *reinterpret_cast<const u32x4 *>(src + e);
  const int n_codes = a.n_code_rows * a.jt;
  uint16_t *dc = reinterpret_cast<uint16_t *>(dst + a.codes_off);
  for (int e = threadIdx.x; e < n_codes; e += 256) {
    const int byte = src[a.codes_off + e];
    const int q = a.sym ? byte - 128 : byte;
    dc[e] = (uint16_t)(q < 0 ? (0x8000 | -q) : q);
  }
  for (int e = a.codes_off + n_codes * 2 + threadIdx.x; e < a.dst_blob; e += 256) dst[e] = 0;      // padding to 16 bytes
}

// One work-group per slice (t, i).  The base row is copied; every code becomes the value of Eq. 10 in fp32 arithmetic,
// fl(y_min + fl(alpha * q)) with the parameters of its segment (row / L; the rows past K*L take the all-zero
// parameter row K and come out zero).  The value rows start where the parameter rows of the byte table do.
__global__ __launch_bounds__(256) void lutkan_dequantise_kernel(const WidenArgs a) {
  const unsigned char *src = a.src + (size_t)blockIdx.x * a.src_blob;
  unsigned char *dst = a.dst + (size_t)blockIdx.x * a.dst_blob;
  for (int e = threadIdx.x * 16; e < a.params_off; e += 256 * 16) *reinterpret_cast<u32x4 *>(dst + e) = *reinterpret_cast<const u32x4 *>(src + e);
  const int n_codes = a.n_code_rows * a.jt;
  float *dv = reinterpret_cast<float *>(dst + a.params_off);
  for (int e = threadIdx.x; e < n_codes; e += 256) {
    const int row = e / a.jt, col = e - row * a.jt;
    const int byte = src[a.codes_off + e];
    const int q = a.sym ? byte - 128 : byte;
    const unsigned char *prow = src + a.params_off + (size_t)min(row / a.L, a.K) * a.param_row_bytes;
    const float alpha = reinterpret_cast<const float *>(prow)[col];                   // (64-column tiles hold fp32 parameters)
    const float y_min = a.sym ? 0.0f : reinterpret_cast<const float *>(prow)[a.jt + col];
    dv[e] = __fadd_rn(y_min, __fmul_rn(alpha, (float)q));
  }
  for (int e = a.params_off + n_codes * 4 + threadIdx.x; e < a.dst_blob; e += 256) dst[e] = 0;     // padding to 16 bytes
}

}  // namespace

extern "C" size_t lutkan_wide_table_bytes(const lutkan_dev_layer *layer, int32_t code_bytes) {
  if (!layer || layer->d < 1 || layer->m < 1 || layer->n_tiles < 1 || layer->K < 1 || layer->L < 2 || layer->K > LUTKAN_MAX_K) return 0;
  if (!lutkan::has_wide_form(layer->jt, layer->K, layer->L, layer->scheme, layer->value_repr, layer->param_dtype, code_bytes)) return 0;
  return (size_t)layer->n_tiles * layer->d * lutkan::wide_blob_layout(layer->K, layer->L, layer->jt, layer->scheme, layer->value_repr, layer->param_dtype, code_bytes).bytes;
}

extern "C" int lutkan_wide_table_build(lutkan_dev_layer *layer, int32_t code_bytes, void *wide_table, size_t bytes, void *hip_stream) {
  const char *who = "lutkan_wide_table_build";
  if (layer) { layer->wide_table = nullptr; layer->wide_blob_bytes = 0; layer->wide_code_bytes = 0; }
  if (int rc = validate_layer(layer, who)) return rc;
  if (code_bytes != 2 && code_bytes != 4) return fail(LUTKAN_EINVAL, "%s: code_bytes %d (2: binary16 codes, 4: fp32 values)", who, code_bytes);
  const size_t need = lutkan_wide_table_bytes(layer, code_bytes);
  if (!need) return fail(LUTKAN_EUNSUPPORTED, "%s: the layer has no wide form of %d bytes per code (64-column tiles whose wide slice fits the LDS twice; jt = %d, K*L = %d)", who, code_bytes, layer->jt, layer->K * layer->L);
  if (!wide_table || (reinterpret_cast<uintptr_t>(wide_table) & 15) != 0) return fail(LUTKAN_EINVAL, "%s: wide_table must be a 16-byte aligned device pointer", who);
  if (bytes < need) return fail(LUTKAN_ESHAPE, "%s: %zu bytes, need %zu", who, bytes, need);
  if ((int64_t)layer->n_tiles * layer->d > 0x7fffffffLL) return fail(LUTKAN_EUNSUPPORTED, "%s: too many slices", who);
  const lutkan::BlobLayout lay = lutkan::blob_layout(layer->K, layer->L, layer->jt, layer->scheme, layer->value_repr, layer->param_dtype);
  WidenArgs a;
  a.src = static_cast<const unsigned char *>(layer->table);
  a.dst = static_cast<unsigned char *>(wide_table);
  a.jt = layer->jt;
  a.src_blob = layer->blob_bytes;
  a.dst_blob = lutkan::wide_blob_layout(layer->K, layer->L, layer->jt, layer->scheme, layer->value_repr, layer->param_dtype, code_bytes).bytes;
  a.codes_off = lay.codes_off;
  a.n_code_rows = layer->K * layer->L + 2;
  a.sym = (layer->scheme == LUTKAN_SYM_INT8);
  a.params_off = lay.params_off; a.param_row_bytes = lay.param_row_bytes; a.L = layer->L; a.K = layer->K;
  if (lutkan::device_params_are_half(layer->value_repr, layer->param_dtype, layer->jt)) return fail(LUTKAN_EUNSUPPORTED, "%s: binary16 parameter rows", who);   // (not on 64-column tiles)
  const dim3 grid((unsigned)((int64_t)layer->n_tiles * layer->d));
  if (code_bytes == 2) hipLaunchKernelGGL(lutkan_widen_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(hip_stream), a);
  else hipLaunchKernelGGL(lutkan_dequantise_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(hip_stream), a);
  if (int rc = check_launch(code_bytes == 2 ? "lutkan_widen_kernel" : "lutkan_dequantise_kernel")) return rc;
  layer->wide_table = wide_table;
  layer->wide_blob_bytes = a.dst_blob;
  layer->wide_code_bytes = code_bytes;
  return LUTKAN_OK;
}

extern "C" int lutkan_forward(const lutkan_dev_layer *layer, const float *x, int64_t B, float *y,
                              lutkan_oob_stats *stats, void *workspace, size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return forward_impl(layer, x, B, y, stats, nullptr, nullptr, nullptr, nullptr, nullptr, false, workspace,
                      workspace_bytes, hip_stream, "lutkan_forward");
}

// Device memory for lutkan_forward_static_scratch: one array per GPU that loads this library, held until the process
// ends.  In host code the name is only a handle for hipGetSymbolAddress; what kernels and copies get is the address
// that call returns on the current device.
static __device__ __align__(256) unsigned char scratch[LUTKAN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];     // per device ordinal: the device address of that GPU's copy of `scratch`

// The current device's copy of the scratch array (looked up once per device, with that device current).
int static_scratch(void **out, const char *who) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: hipGetDevice: %s", who, hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(LUTKAN_EUNSUPPORTED, "%s: device ordinal %d", who, dev);
  void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(LUTKAN_EHIP, "%s: hipGetSymbolAddress(scratch): %s", who, hipGetErrorString(e));
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return LUTKAN_OK;
}
}  // namespace

extern "C" int lutkan_forward_static_scratch(const lutkan_dev_layer *layer, const float *x, int64_t B, float *y,
                                             lutkan_oob_stats *stats, void *hip_stream) {
  const char *who = "lutkan_forward_static_scratch";
  lutkan::plan_clear();
  if (int rc = validate_layer(layer, who)) return rc;
  if (B < 0) return fail(LUTKAN_EINVAL, "%s: B < 0", who);
  if (B == 0) return LUTKAN_OK;
  const size_t need = lutkan_forward_workspace_bytes(layer, B);
  if (need > (size_t)LUTKAN_STATIC_SCRATCH_BYTES)
    return fail(LUTKAN_ESHAPE, "%s: %lld rows of this %d -> %d layer need %zu bytes of scratch, the built-in array holds %zu; "
                "use lutkan_forward with a workspace of the caller's", who, (long long)B, layer->d, layer->m, need,
                (size_t)LUTKAN_STATIC_SCRATCH_BYTES);
  void *ptr = nullptr;
  if (int rc = static_scratch(&ptr, who)) return rc;
  // Nothing in the scratch has to start at zero: the locate kernel writes every record of every padded row, and the
  // edge kernels write every partial sum that the summing pass reads.
  return forward_impl(layer, x, B, y, stats, nullptr, nullptr, nullptr, nullptr, nullptr, false, ptr,
                      (size_t)LUTKAN_STATIC_SCRATCH_BYTES, hip_stream, who);
}

extern "C" int lutkan_forward_locate(const lutkan_dev_layer *layer, const float *x, int64_t B, lutkan_oob_stats *stats,
                                     void *workspace, size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return forward_impl(layer, x, B, nullptr, stats, nullptr, nullptr, nullptr, nullptr, nullptr, false, workspace,
                      workspace_bytes, hip_stream, "lutkan_forward_locate", kLocate);
}

extern "C" int lutkan_forward_edges(const lutkan_dev_layer *layer, int64_t B, float *y, void *workspace,
                                    size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return forward_impl(layer, nullptr, B, y, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, false, workspace,
                      workspace_bytes, hip_stream, "lutkan_forward_edges", kEdges);
}

extern "C" int lutkan_forward_trace(const lutkan_dev_layer *layer, const float *x, int64_t B, float *y,
                                    int32_t *k_out, int32_t *l0_out, uint8_t *in_out, float *w_out, int16_t *q01_out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream) {
  lutkan::plan_clear();
  return forward_impl(layer, x, B, y, nullptr, k_out, l0_out, in_out, w_out, q01_out, true, workspace,
                      workspace_bytes, hip_stream, "lutkan_forward_trace");
}

extern "C" size_t lutkan_model_workspace_bytes(const lutkan_dev_layer *layers, int32_t n_layers, int64_t B) {
  if (!layers || n_layers < 1 || B <= 0) return 0;
  size_t act = 0, scratch = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (l + 1 < n_layers) act = std::max(act, (size_t)round_up((int64_t)layers[l].m * B * 4, 256));
    scratch = std::max(scratch, lutkan_forward_workspace_bytes(&layers[l], B));
  }
  return 2 * act + scratch;
}

extern "C" int lutkan_chain_forward(const lutkan_dev_layer *layers, int32_t n_layers, const float *x, int64_t B, float *y,
                                    float *hidden, lutkan_oob_stats *stats, void *hip_stream) {
  lutkan::plan_clear();
  return chain_impl(layers, n_layers, x, B, y, hidden, stats, hip_stream, "lutkan_chain_forward");
}

extern "C" int lutkan_model_forward(const lutkan_dev_layer *layers, int32_t n_layers, const float *x, int64_t B, float *y,
                                    lutkan_oob_stats *stats, void *workspace, size_t workspace_bytes, void *hip_stream) {
  const char *who = "lutkan_model_forward";
  lutkan::plan_clear();
  if (!layers || n_layers < 1 || n_layers > LUTKAN_MAX_LAYERS) return fail(LUTKAN_EINVAL, "%s: need 1..%d layers", who, LUTKAN_MAX_LAYERS);
  for (int l = 0; l < n_layers; ++l)                       // before anything is computed from a layer's fields
    if (int rc = validate_layer(&layers[l], who)) return rc;
  for (int l = 0; l + 1 < n_layers; ++l)
    if (layers[l].m != layers[l + 1].d) return fail(LUTKAN_ESHAPE, "%s: layer %d has m=%d but layer %d has d=%d", who, l, layers[l].m, l + 1, layers[l + 1].d);
  if (B < 0) return fail(LUTKAN_EINVAL, "%s: B < 0", who);
  if (B == 0) return LUTKAN_OK;
  const size_t need = lutkan_model_workspace_bytes(layers, n_layers, B);
  if (!workspace || workspace_bytes < need) return fail(LUTKAN_ESHAPE, "%s: workspace of %zu bytes, need %zu", who, workspace_bytes, need);
  if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return fail(LUTKAN_EINVAL, "%s: workspace must be 256-byte aligned", who);
  size_t act = 0, scratch = 0;
  for (int l = 0; l < n_layers; ++l) {
    if (l + 1 < n_layers) act = std::max(act, (size_t)round_up((int64_t)layers[l].m * B * 4, 256));
    scratch = std::max(scratch, lutkan_forward_workspace_bytes(&layers[l], B));
  }
  // Every layer would run as its own launch of the chain kernel: run them as one launch of it instead.  The
  // arithmetic per layer is the same, so the result is bit-identical to the layer-by-layer calls.
  bool all_small = (n_layers <= kChainMaxLayers);
  for (int l = 0; l < n_layers && all_small; ++l) all_small = small_layer_runs_as_chain(&layers[l], B);
  if (all_small && n_layers > 1) return chain_impl(layers, n_layers, x, B, y, nullptr, stats, hip_stream, who);
  char *base = static_cast<char *>(workspace);
  float *ping[2] = {reinterpret_cast<float *>(base), reinterpret_cast<float *>(base + act)};
  void *rec = base + 2 * act;
  const float *in = x;
  for (int l = 0; l < n_layers; ++l) {
    float *out = (l + 1 == n_layers) ? y : ping[l & 1];
    int rc = forward_impl(&layers[l], in, B, out, stats ? stats + l : nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, false, rec,
                          scratch, hip_stream, who);
    if (rc) return rc;
    in = out;
  }
  return LUTKAN_OK;
}

// The base branch of value_repr = spline_component (Eq. 2) for a whole layer as one dense contraction on the matrix
// cores:  Y0[b][j] = sum_i SiLU(x[b][i]) * (s_out * s_base)[i][j].  It is the one piece of the layer forward without
// a gather: a [B, d] x [d, m] product.  The LUT edge kernel then adds the spline branch on top of Y0.
//
// fp32 accuracy from bf16 matrix instructions: every fp32 operand is cut, exactly, into three bf16 pieces of eight
// significand bits each (a = a_h + a_m + a_l by truncation, nothing is lost), and the product is accumulated in fp32
// from the six piece products that are not below 2^-24 of it (h*h, h*m, m*h, m*m, h*l, l*h).  bf16 has the exponent
// range of fp32, so no scaling is needed.  A non-finite SiLU(x) keeps its class in the high piece; its row comes out
// non-finite (NaN where an edge-by-edge evaluation may give +-inf).
//
// Both operands arrive already cut: SiLU(x) by the locate kernel (lutkan_cut3 below, three planes [piece][row][input]),
// s_out*s_base by lutkan_base_pieces_kernel from the base rows of the LUT device table (three planes
// [piece][column][input]); in both the inputs are contiguous, which is the operand order of the matrix instruction
// (a lane holds 8 consecutive k of one row resp. column).  One work-group of 256 threads computes a 128 x 128 tile of
// Y0, its four waves 64 x 64 each as 2 x 2 tiles of v_mfma_f32_32x32x16_bf16; the inputs are walked 32 at a time: 48 KiB
// of pieces go global -> registers -> LDS (the loads of the next step are in flight while this step multiplies), each
// wave then reads its operands with 16-byte LDS reads.  Two work-groups fit a compute unit.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lutkan_internal.h"
#include "lutkan_pieces.h"

using lutkan::fail;

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128, kBN = 128, kBK = 32;
constexpr int kLdk = kBK + 8;            // bf16 elements per LDS row: 80 bytes, so that the 16 rows of a 16-byte read group fall into different banks
constexpr int kVecPerStep = 3 * kBM * kBK * 2 / 16;      // 16-byte vectors of one operand per k step: 1536, six per thread

struct BasePiecesArgs {
  const unsigned char *table;        // LUT device table: slice (t, i) starts with the jt floats s_out*s_base of its columns
  uint16_t *w_pieces;                // [3][m_pad][d] bf16 bit patterns, rows m .. m_pad-1 zero
  int32_t d, m, m_pad, jt_log2, blob_bytes;
};

// One thread per (column, group of 8 inputs): adjacent threads take adjacent columns, so the eight 4-byte reads of a
// wave are contiguous runs of the base rows; each thread writes three 16-byte vectors.
__global__ __launch_bounds__(256) void lutkan_base_pieces_kernel(const BasePiecesArgs a) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int j = (int)(g % a.m_pad);
  const int k = (int)(g / a.m_pad) * 8;
  if (k >= a.d) return;
  unsigned h[8], m[8], l[8];
  const unsigned char *w = a.table + ((size_t)(j >> a.jt_log2) * a.d + k) * a.blob_bytes + (size_t)(j & ((1 << a.jt_log2) - 1)) * 4;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float v = (j < a.m) ? *reinterpret_cast<const float *>(w + (size_t)e * a.blob_bytes) : 0.0f;   // d is a multiple of 32
    lutkan_cut3(v, h[e], m[e], l[e]);
  }
  const size_t plane = (size_t)a.m_pad * a.d;
  uint16_t *dst = a.w_pieces + (size_t)j * a.d + k;
  *reinterpret_cast<u32x4 *>(dst) = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
  *reinterpret_cast<u32x4 *>(dst + plane) = u32x4{m[0] | (m[1] << 16), m[2] | (m[3] << 16), m[4] | (m[5] << 16), m[6] | (m[7] << 16)};
  *reinterpret_cast<u32x4 *>(dst + 2 * plane) = u32x4{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
}

struct BaseGemmArgs {
  const uint16_t *a_pieces;          // [3][Bp][d]: SiLU(x) cut into pieces, rows B .. Bp-1 zero (Bp a multiple of 128)
  const uint16_t *w_pieces;          // [3][m_pad][d]
  float *y;                          // [B][m]
  int64_t B, Bp;
  int32_t d, m, m_pad;
};

__global__ __launch_bounds__(256) void lutkan_base_gemm_kernel(const BaseGemmArgs a) {
  static_assert(kBM == kBN, "both operand tiles share one LDS shape");
  __shared__ __align__(16) uint16_t sA[3][kBM][kLdk];
  __shared__ __align__(16) uint16_t sW[3][kBN][kLdk];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;               // this wave's 64 x 64 quarter of the tile
  const int64_t row0 = (int64_t)blockIdx.y * kBM;
  const int col0 = blockIdx.x * kBN;

  f32x16 acc[2][2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rt][ct][v] = 0.0f;

  // this thread's six vectors of each operand tile: vector v = tid + 256 q is piece v / 512, row (v % 512) / 4,
  // inputs 8 * (v % 4) .. + 7 of the step (four adjacent threads read the 64 contiguous bytes of one row)
  const uint16_t *ga[6], *gw[6];
  uint16_t *la[6], *lw[6];
#pragma unroll
  for (int q = 0; q < 6; ++q) {
    const int v = tid + 256 * q;
    const int piece = v >> 9, r = (v & 511) >> 2, k8 = (v & 3) * 8;
    ga[q] = a.a_pieces + ((size_t)piece * a.Bp + row0 + r) * a.d + k8;
    gw[q] = a.w_pieces + ((size_t)piece * a.m_pad + col0 + r) * a.d + k8;
    la[q] = &sA[piece][r][k8];
    lw[q] = &sW[piece][r][k8];
  }
  static_assert(kVecPerStep == 6 * 256, "six vectors per thread and operand");
  u32x4 ra[6], rw[6];
#pragma unroll
  for (int q = 0; q < 6; ++q) { ra[q] = *reinterpret_cast<const u32x4 *>(ga[q]); rw[q] = *reinterpret_cast<const u32x4 *>(gw[q]); }

  for (int k0 = 0; k0 < a.d; k0 += kBK) {
#pragma unroll
    for (int q = 0; q < 6; ++q) { *reinterpret_cast<u32x4 *>(la[q]) = ra[q]; *reinterpret_cast<u32x4 *>(lw[q]) = rw[q]; }
    __syncthreads();
    if (k0 + kBK < a.d) {                                // the next step's pieces travel while this step multiplies
#pragma unroll
      for (int q = 0; q < 6; ++q) {
        ra[q] = *reinterpret_cast<const u32x4 *>(ga[q] + k0 + kBK);
        rw[q] = *reinterpret_cast<const u32x4 *>(gw[q] + k0 + kBK);
      }
    }
    // ---- 2 k sub-steps of 16: a lane holds 8 consecutive k of row resp. column lane % 32, k offset 8 * (lane / 32)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int kk = ks * 16 + (lane >> 5) * 8;
      bf16x8 af[2][3], wf[2][3];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int p = 0; p < 3; ++p) {
          af[t][p] = *reinterpret_cast<const bf16x8 *>(&sA[p][wr * 64 + t * 32 + (lane & 31)][kk]);
          wf[t][p] = *reinterpret_cast<const bf16x8 *>(&sW[p][wc * 64 + t * 32 + (lane & 31)][kk]);
        }
      // the six piece products, the small ones first; the four accumulators take turns, so that no matrix instruction
      // waits for the one before it
      constexpr int kPieceOfA[6] = {2, 0, 1, 1, 0, 0}, kPieceOfW[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
      for (int p = 0; p < 6; ++p)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rt][kPieceOfA[p]], wf[ct][kPieceOfW[p]], acc[rt][ct], 0, 0, 0);
    }
    __syncthreads();                                     // everyone is done with this step's operands
  }

  // ---- the accumulator of a 32 x 32 tile: element v of a lane is row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const int j = col0 + wc * 64 + ct * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t b = row0 + wr * 64 + rt * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (b < a.B && j < a.m) a.y[b * a.m + j] = acc[rt][ct][v];
      }
    }
}

inline int32_t padded_columns(int32_t m) { return (m + kBN - 1) / kBN * kBN; }

}  // namespace

namespace lutkan {

bool base_product_fits(int32_t d, int32_t m, int64_t B) { return d % kBK == 0 && m >= 64 && (B + kBM - 1) / kBM <= 65535; }

size_t base_product_workspace_bytes(int32_t d, int32_t m) {
  return base_product_fits(d, m, 1) ? ((size_t)6 * padded_columns(m) * d + 255) / 256 * 256 : 0;
}

int launch_base_product(const uint16_t *silu_pieces, int64_t Bp, const void *table, uint16_t *w_pieces, int32_t d, int32_t m, int32_t jt,
                        int32_t blob_bytes, int64_t B, float *y, void *hip_stream, const char *who) {
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  BasePiecesArgs p;
  p.table = static_cast<const unsigned char *>(table);
  p.w_pieces = w_pieces;
  p.d = d; p.m = m; p.m_pad = padded_columns(m); p.blob_bytes = blob_bytes;
  p.jt_log2 = 0;
  while ((1 << p.jt_log2) < jt) ++p.jt_log2;
  const int64_t groups = ((int64_t)p.m_pad * (d / 8) + 255) / 256;
  hipLaunchKernelGGL(lutkan_base_pieces_kernel, dim3((unsigned)groups), dim3(256), 0, s, p);
  BaseGemmArgs a;
  a.a_pieces = silu_pieces; a.w_pieces = w_pieces; a.y = y;
  a.B = B; a.Bp = Bp; a.d = d; a.m = m; a.m_pad = p.m_pad;
  hipLaunchKernelGGL(lutkan_base_gemm_kernel, dim3((unsigned)(p.m_pad / kBN), (unsigned)((B + kBM - 1) / kBM)), dim3(256), 0, s, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LUTKAN_EHIP, "%s: base-branch product: %s", who, hipGetErrorString(e));
  return LUTKAN_OK;
}

}  // namespace lutkan

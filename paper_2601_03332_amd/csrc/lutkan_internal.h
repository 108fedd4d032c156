// Internal declarations shared by the host compiler and the HIP launchers of liblutkan.
// Nothing here is part of the C ABI (see include/lutkan.h).
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "lutkan.h"

namespace lutkan {

// Thread-local error text behind lutkan_last_error().
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
// Thread-local text behind lutkan_last_plan(): which kernels the last forward call launched, one clause per launch.
void plan_clear();
void plan_note(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

// Byte offsets inside one (tile, input) slice of the LUT device table:
//   [base jt f32 (spline_component only)][params (K+1) rows of jt entries][codes (K*L+2) rows of jt bytes][pad to 16 B]
// A parameter row is alpha[jt], then for the asymmetric scheme y_min[jt]; fp32 values, or binary16 values (see
// device_params_are_half).
// Parameter row K and code rows K*L, K*L+1 are all zero: the kernels send masked inputs there.
struct BlobLayout {
  int32_t params_off, param_row_bytes, codes_off, bytes;
};

// True when the device table holds the parameters as binary16 values: float16 parameters of a phi layer on tiles
// of at most 32 columns, where the shorter rows were measured 0-5 % faster; on the widest layer (64-column tiles) they
// were a repeatable 3 % slower, so on wider tiles the (rounded) values are held as fp32.  With spline_component the table holds the fp32 products
// s_out*s_spline*alpha of the rounded alpha: a product cannot be stored in 16 bits without a second rounding.
inline bool device_params_are_half(int value_repr, int param_dtype, int jt) {
  return param_dtype == LUTKAN_PARAM_FP16 && value_repr != LUTKAN_REPR_SPLINE_COMPONENT && jt <= 32;
}

inline BlobLayout blob_layout(int K, int L, int jt, int scheme, int value_repr, int param_dtype) {
  BlobLayout b;
  b.params_off = (value_repr == LUTKAN_REPR_SPLINE_COMPONENT) ? jt * 4 : 0;
  b.param_row_bytes = jt * ((scheme == LUTKAN_ASYM_UINT8) ? 2 : 1) * (device_params_are_half(value_repr, param_dtype, jt) ? 2 : 4);
  b.codes_off = b.params_off + (K + 1) * b.param_row_bytes;
  int raw = b.codes_off + (K * L + 2) * jt;
  b.bytes = (raw + 15) & ~15;
  return b;
}

// Rows of one (tile, input) slice of the B-spline device table: [base row (spline_component only)][R coefficient rows].
inline int coef_slice_rows(int R, int value_repr) { return R + (value_repr == LUTKAN_REPR_SPLINE_COMPONENT ? 1 : 0); }

// LDS that one work-group of the tiled kernels may use: all 160 KiB of a gfx950 compute unit.
constexpr int kLdsPerWorkGroup = 160 * 1024;

// Largest table slice of the LUT tiled kernel: two slice buffers plus the per-wave record buffers (16 waves x 2 buffers
// x at most 64 rows of 8-byte records, 16-byte with the base branch) must fit: 72 KiB, 64 KiB with the base branch.
inline int lds_slice_budget(int value_repr) {
  const int record_bytes = (value_repr == LUTKAN_REPR_SPLINE_COMPONENT) ? 16 : 8;
  return (kLdsPerWorkGroup - 16 * 2 * 64 * record_bytes) / 2;
}

// The wide forms of the LUT table (see lutkan_wide_table_build).  code_bytes = 2: the same slice layout with code
// rows of jt binary16 values.  code_bytes = 4: [base jt f32 (spline_component only)][(K*L+2) rows of jt fp32 values
// y_min + alpha * q, the last two rows zero]; there are no parameter rows (params_off = codes_off, param_row_bytes 0).
inline BlobLayout wide_blob_layout(int K, int L, int jt, int scheme, int value_repr, int param_dtype, int code_bytes) {
  BlobLayout b = blob_layout(K, L, jt, scheme, value_repr, param_dtype);
  if (code_bytes == 4) {
    b.param_row_bytes = 0;
    b.codes_off = b.params_off;
  }
  b.bytes = (b.codes_off + (K * L + 2) * jt * code_bytes + 15) & ~15;
  return b;
}
// A layer has a wide form when its table is on 64-column tiles and the wide slice fits twice into the LDS beside the
// record buffers of the 8-byte records it is used with.  (On 32-column tiles the kernel's LDS reads come in eight
// short runs per wave and bound it: measured 12 % slower than the byte form on the 1024x1024 layer, whose wide
// slices only fit at that width.)
inline bool has_wide_form(int jt, int K, int L, int scheme, int value_repr, int param_dtype, int code_bytes) {
  if (code_bytes != 2 && code_bytes != 4) return false;
  return jt == 64 && wide_blob_layout(K, L, jt, scheme, value_repr, param_dtype, code_bytes).bytes <= lds_slice_budget(LUTKAN_REPR_PHI);
}

// Column-tile width of a layer's LUT table: the widest power of two in 4 .. 64 (not wider than the next power of two
// >= m) whose slice fits the LDS budget; a table of 4096 rows still runs on the tiled kernel, 8 columns at a time,
// twice as fast as on the gather kernel.  If not even 4 columns fit: 32 (or the layer's width), for the gather kernel.
// 128-column tiles, where they fit, measured 1-6 % slower than 64 from 4096 rows on.
int choose_jt(int m, int K, int L, int scheme, int value_repr, int param_dtype);
// Column-tile width of the B-spline coefficient table: a power of two in 4 .. 128 (its slices always fit; that layer
// measured 1.5-4 % faster on 128 columns than on 64 at the largest batches).
int choose_coef_jt(int m);

// The base branch of a spline_component layer as one product on the matrix cores (lutkan_base_gemm.hip):
// y[B][m] = SiLU(x)[B][d] x (s_out*s_base)[d][m], both operands as three bf16 pieces per fp32 value.
//   silu_pieces  [3][Bp][d] bf16 bit patterns written by the locate kernel, rows B .. Bp-1 zero, Bp a multiple of 128
//   w_pieces     scratch of base_product_workspace_bytes(d, m) bytes, filled from the base rows of `table` by the call
// base_product_fits: the shapes the product exists for (d a multiple of 32, at least 64 columns); for other shapes the
// scratch size is 0.
size_t base_product_workspace_bytes(int32_t d, int32_t m);
bool base_product_fits(int32_t d, int32_t m, int64_t B);
int launch_base_product(const uint16_t *silu_pieces, int64_t Bp, const void *table, uint16_t *w_pieces, int32_t d, int32_t m, int32_t jt,
                        int32_t blob_bytes, int64_t B, float *y, void *hip_stream, const char *who);

}  // namespace lutkan

struct lutkan_artifact {
  lutkan_info info;
  std::vector<float> ext_knots;   // [G+2p+1]
  std::vector<float> knots;       // [K+1]
  std::vector<uint8_t> q;         // canonical [E][K][L]
  std::vector<float> scale;       // [E][K]
  std::vector<float> ymin;        // [E][K]
  std::vector<float> edge_base, edge_spline, edge_out;   // [E] each, empty for value_repr = phi
  std::vector<uint8_t> table;     // device LUT table, [t][i] slices
  std::vector<float> coef_table;  // device B-spline table, [t][i][R][jt]
};

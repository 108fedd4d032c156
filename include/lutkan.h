/*
 * lutkan.h -- C ABI of the MI355X (gfx950) LUT-KAN layer-forward library.
 *
 * The library computes the forward pass of a dense Kolmogorov-Arnold layer
 *     y_j = sum_i phi_ij(x_i)                                            (Sec. 3.1, Eq. 1)
 * in which every edge function is a segment-wise int8/uint8 lookup table (Sec. 4), together
 * with a same-backend cubic B-spline layer (Sec. 3.2-3.3) that serves as the honest baseline.
 *
 * Conventions
 *   - Every function returns 0 (LUTKAN_OK) or a negative lutkan_status.  No exception crosses the
 *     ABI.  lutkan_last_error() gives a thread-local, human readable reason for the last failure.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory that the
 *     CALLER owns (allocated by any allocator, e.g. a torch tensor).  The library never allocates
 *     or frees device memory and never synchronises: forward calls only enqueue kernels on the
 *     stream handed in (a hipStream_t passed as void*; NULL = the default stream).
 *   - Host artifacts returned by lutkan_compile are owned by the library until lutkan_artifact_free.
 *   - Row-major everywhere.  x is [B][d] fp32, y is [B][m] fp32; x and y must not alias.
 *   - B == 0 is a no-op that returns LUTKAN_OK.
 */
#ifndef LUTKAN_H
#define LUTKAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LUTKAN_OK = 0,
  LUTKAN_EINVAL = -1,        /* null pointer, bad enum, L < 2, knots not strictly increasing, non-finite coef */
  LUTKAN_ESHAPE = -2,        /* sizes that do not fit together (workspace too small, d/m mismatch in a chain) */
  LUTKAN_ENOMEM = -3,        /* host allocation failed */
  LUTKAN_EHIP = -4,          /* a HIP runtime call failed */
  LUTKAN_EUNSUPPORTED = -5   /* degree != 3, K > LUTKAN_MAX_K, K*L > LUTKAN_MAX_ROWS, fp16 parameters out of range */
} lutkan_status;

typedef enum { LUTKAN_SYM_INT8 = 0, LUTKAN_ASYM_UINT8 = 1 } lutkan_scheme;        /* Sec. 4.4, Eq. 11-12 */
typedef enum { LUTKAN_HALF_OPEN = 0, LUTKAN_CLOSED = 1 } lutkan_boundary;          /* Sec. 5.2 */
typedef enum { LUTKAN_CLIP_X = 0, LUTKAN_ZERO_SPLINE = 1 } lutkan_oob;             /* Sec. 5.4 */
/* Which edge kernel runs.  TILED stages each (tile, input) table slice in LDS; GATHER reads the touched table rows
 * from global memory and splits the inputs over the GPU.  AUTO: tiled when a slice fits LDS, except for batches of so
 * few rows that they touch less than the whole table (then gather), and except for a small narrow layer (one column
 * tile, d * jt <= 4096) at up to 10000 / (0.30 + 0.00053 d jt) rows (30000 for a 16x2 layer, 4000 for 256x16), which
 * lutkan_forward runs as a one-layer launch of the fused chain kernel;
 * results agree to rounding, not bit for bit.  TILED (and AUTO) take the table's wide form, where the layer holds one
 * (lutkan_wide_table_build), when the launch planning prices it lower; TILED_WIDE takes it whatever the price and is
 * an error for a layer without one or a call it does not serve (16-bit codes with 16-byte records).  LUT layers only. */
typedef enum { LUTKAN_ALGO_AUTO = 0, LUTKAN_ALGO_GATHER = 1, LUTKAN_ALGO_TILED = 2, LUTKAN_ALGO_TILED_WIDE = 3 } lutkan_algo;
typedef enum { LUTKAN_REPR_PHI = 0, LUTKAN_REPR_SPLINE_COMPONENT = 1 } lutkan_value_repr;  /* Sec. 4.3 A / B */
typedef enum { LUTKAN_PARAM_FP32 = 0, LUTKAN_PARAM_FP16 = 1 } lutkan_param_dtype;   /* Sec. 4.6: dtype of scale, y_min */
/* Which knots are the LUT's "knot grid" (Sec. 4.2): the G+1 breakpoints of the domain [ext_knots[p], ext_knots[p+G]]
 * (K = G), or every knot of the extended vector (K = G + 2p, domain [ext_knots[0], ext_knots[G+2p]]) -- the reading
 * under which the per-layer byte counts of Table 9 come out exactly. */
typedef enum { LUTKAN_SPAN_DOMAIN = 0, LUTKAN_SPAN_EXTENDED = 1 } lutkan_knot_span;

#define LUTKAN_MAX_K 64            /* segments per layer (the knot vector travels in the kernel arguments) */
#define LUTKAN_MAX_ROWS 65535      /* K * L, table rows per input (a row index travels in 16 bits) */
#define LUTKAN_MAX_LAYERS 16

const char *lutkan_last_error(void);
const char *lutkan_version(void);
/* What the last forward call of this thread launched, for logs and tests: one clause per kernel launch, e.g.
 * "locate; tiled np=16 split=2 pipe=3; sum; " (row steps per wave, chunks of inputs, pipeline mode: 2 = two slice
 * buffers, 3 = three with the reads carried across inputs, 4 = three with two slices in flight; "tiled wide" on the
 * table's form with 16-bit codes, "tiled wide32" on the one with fp32 values) or "chain layers=2 wpr=4; " or "locate; gather split=16; sum; " or, for a large
 * spline_component layer, "locate; base_product; tiled np=16 split=1 pipe=3; " (model_forward: the clauses of all its
 * layers).  Thread-local, overwritten by the next forward call, never null. */
const char *lutkan_last_plan(void);

/* ------------------------------------------------------------------------------------------------
 * Host side: compile a B-spline KAN layer into a LUT artifact (Sec. 4.2-4.6, Sec. 6.3).
 * ---------------------------------------------------------------------------------------------- */

/* One dense layer.  All pointers are host.
 * value_repr = LUTKAN_REPR_PHI: pure-spline edges, phi_ij = s_ij (Sec. 4.3 A with no base branch); the three
 *   edge_* pointers are ignored.
 * value_repr = LUTKAN_REPR_SPLINE_COMPONENT (Sec. 4.3 B, Eq. 2): the table still holds the spline branch s_ij and
 *   the edge output is  s_out * (s_base * SiLU(x) + s_spline * m(x) * s^(x'))  with the base branch evaluated at
 *   the raw input and the oob mask m(x) applied to the spline branch only (Sec. 5.4); the three arrays are [d][m]. */
typedef struct {
  int32_t d, m;              /* inputs, outputs */
  int32_t G;                 /* grid intervals; the LUT has K = G segments on the domain grid (Sec. 4.2) */
  int32_t degree;            /* spline degree p; must be 3 */
  const float *ext_knots;    /* [G + 2*degree + 1] strictly increasing; domain = [ext_knots[p], ext_knots[p+G]];
                                [d][G + 2*degree + 1] with knots_per_input */
  const float *coef;         /* [d][m][G + degree] B-spline coefficients c_r of Eq. 3 */
  int32_t L;                 /* samples per segment, >= 2 (Eq. 7) */
  int32_t scheme;            /* lutkan_scheme */
  int32_t boundary;          /* lutkan_boundary */
  int32_t oob;               /* lutkan_oob */
  int32_t value_repr;        /* lutkan_value_repr */
  const float *edge_base_scale;    /* s_base   [d][m], spline_component only */
  const float *edge_spline_scale;  /* s_spline [d][m] */
  const float *edge_out_scale;     /* s_out    [d][m] */
  int32_t param_dtype;       /* lutkan_param_dtype.  FP16: the codes are computed from the fp32 alpha and y_min of
                                Eq. 11-12, then both are stored rounded to the nearest binary16 value and inference
                                dequantises with the stored values (Eq. 10).  EUNSUPPORTED if a parameter is too
                                large for binary16. */
  int32_t knot_span;         /* lutkan_knot_span.  EXTENDED: the spline is still the sum of Eq. 3 over the G+p
                                coefficients; on the outer p intervals of each side fewer than p+1 basis functions
                                exist, and at the last knot itself all of them are 0 (half-open indicator of Eq. 4).
                                The B-spline layer of the artifact uses the same domain.  Needs G + 2p <= LUTKAN_MAX_K. */
  int32_t knots_per_input;   /* 0: one knot vector for the layer (Sec. 4.6).  1: one per input dimension (the grid
                                "shared per input dimension" of Sec. 6.2, e.g. after a per-feature grid update): all
                                edges leaving input i are sampled, located and masked on row i of ext_knots. */
} lutkan_layer_desc;

typedef struct lutkan_artifact lutkan_artifact;     /* opaque, host memory */

typedef struct {
  int32_t d, m, K, L, G, degree, scheme, boundary, oob, value_repr, param_dtype, knot_span, knots_per_input;
  int32_t jt;                /* column-tile width of the LUT device table: a power of two in 4 .. 64 */
  int32_t n_tiles;           /* ceil(m / jt) */
  int32_t blob_bytes;        /* bytes of one (tile, input) slice of the LUT device table */
  int32_t coef_jt;           /* column-tile width of the B-spline device table: a power of two in 4 .. 128 (0 if none) */
  int32_t coef_n_tiles;      /* ceil(m / coef_jt) */
  int32_t coef_blob_bytes;   /* bytes of one (tile, input) slice of the B-spline device table */
  float t0, tK, tK_star;     /* domain ends and the safe upper clip value of Eq. 13 (of input 0 with knots_per_input) */
  size_t q_canonical_bytes;  /* d*m*K*L */
  size_t params_canonical_bytes; /* d*m*K*4 (d*m*K*2 with fp16 parameters), for scale and for y_min each */
  size_t table_bytes;        /* whole LUT device table = n_tiles*d*blob_bytes */
  size_t coef_table_bytes;   /* whole B-spline device table = coef_n_tiles*d*coef_blob_bytes */
  size_t artifact_bytes;     /* Sec. 4.6 arrays: q + scale + y_min + knots (what Sec. 6.6 "LUT artifact bytes" counts;
                                knots are 4*(K+1) bytes, times d with knots_per_input) */
} lutkan_info;

/* Samples every edge on every segment in fp64 (Eq. 3-5, Eq. 7), quantises in fp32 (Eq. 11-12) and lays the
 * result out twice: the canonical arrays of Sec. 4.6 and the device tables described below.
 * n_threads <= 0 picks the number of host cores.  *out is set only on success. */
int lutkan_compile(const lutkan_layer_desc *desc, int32_t n_threads, lutkan_artifact **out);
void lutkan_artifact_free(lutkan_artifact *a);
int lutkan_artifact_info(const lutkan_artifact *a, lutkan_info *out);

/* The stored arrays of one layer artifact (Sec. 4.6 "Stored Arrays and Shapes" and the manifest fields of its
 * "Serialization Format"), all host pointers, edge e = i*m + j:
 *   knots fp32 [K+1] strictly increasing ([d][K+1], every row increasing, with knots_per_input); q_table int8 /
 *   uint8 [E][K][L]; scale, y_min fp32 [E][K] (with
 *   param_dtype = FP16 every value must already be a binary16 value); the three edge_* arrays fp32 [E] with
 *   value_repr = spline_component, else ignored. */
typedef struct {
  int32_t d, m, K, L;
  int32_t scheme, boundary, oob, value_repr, param_dtype, knots_per_input;
  const float *knots;
  const void *q_table;
  const float *scale, *y_min;
  const float *edge_base_scale, *edge_spline_scale, *edge_out_scale;
} lutkan_artifact_arrays;

/* Rebuilds an artifact (canonical arrays + LUT device table) from stored arrays, e.g. after reading them back from
 * disk: the inverse of the lutkan_artifact_* accessors.  The arrays are copied.  Such an artifact carries no spline
 * coefficients: info.G = 0, the ext_knots / coef_table accessors return NULL and bspline_dev_layer_init refuses it.
 * Errors as lutkan_compile; EINVAL also for non-finite parameters or fp16 parameters that are not binary16 values. */
int lutkan_artifact_from_arrays(const lutkan_artifact_arrays *arrays, lutkan_artifact **out);

/* Read-only host views, valid until lutkan_artifact_free.  Canonical arrays (Sec. 4.6), edge e = i*m + j: */
const void *lutkan_artifact_q(const lutkan_artifact *a);          /* int8 or uint8 [E][K][L] */
const float *lutkan_artifact_scale(const lutkan_artifact *a);     /* alpha  [E][K] (fp16 parameters: the rounded values, as floats) */
const float *lutkan_artifact_ymin(const lutkan_artifact *a);      /* y_min  [E][K] (zeros for symmetric) */
const float *lutkan_artifact_knots(const lutkan_artifact *a);     /* [K+1], or [d][K+1] with knots_per_input */
const float *lutkan_artifact_ext_knots(const lutkan_artifact *a); /* [G+2p+1], or [d][G+2p+1] */
const float *lutkan_artifact_edge_base_scale(const lutkan_artifact *a);   /* [E], NULL for value_repr = phi (Sec. 4.6) */
const float *lutkan_artifact_edge_spline_scale(const lutkan_artifact *a); /* [E] */
const float *lutkan_artifact_edge_out_scale(const lutkan_artifact *a);    /* [E] */

/* Device tables (host copies to upload verbatim).  Columns are cut into n_tiles tiles of jt outputs; the
 * last tile is zero padded.  LUT table: for tile t and input i one contiguous slice of blob_bytes bytes
 *     float   base  [jt]                       (spline_component only: s_out * s_base of the edge (i, column))
 *     param   p     [K+1] rows                 (a row is alpha[jt], followed for the asymmetric scheme by y_min[jt] --
 *                                               y_min is elided when it is identically 0, Sec. 7.5; row K is all zero;
 *                                               values are fp32, or binary16 for a phi layer with fp16 parameters
 *                                               on tiles of at most 32 columns)
 *     code    q     [K*L+2][jt]                (one byte per code, row k*L+l, i.e. the [i][segment][sample][j]
 *                                               order per tile: uint8 codes as they are, int8 codes excess-128,
 *                                               byte = q + 128; the two trailing rows are all-zero bytes)
 *     zero padding up to a multiple of 16 bytes
 * The zero rows are where the kernels redirect inputs whose contribution is exactly 0 (oob_policy zero_spline).
 * With spline_component the product s_out * s_spline of the edge is folded into its alpha and y_min, held as fp32
 * (with fp16 parameters: the products of the rounded values; the canonical arrays keep the rounded values
 * themselves), and into the coefficients of the B-spline table, whose slices then start with the same base[jt] row.
 * slices ordered [t][i].  B-spline table: slices of float c[R = G+p][jt], ordered [t][i]. */
const void *lutkan_artifact_table(const lutkan_artifact *a);
const void *lutkan_artifact_coef_table(const lutkan_artifact *a);

/* ------------------------------------------------------------------------------------------------
 * Device side.  The structs are plain host structs; the pointers inside are DEVICE pointers.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t d, m, K, L, scheme, boundary, oob, value_repr, param_dtype;
  int32_t jt, n_tiles, blob_bytes;
  int32_t algo;                       /* lutkan_algo; AUTO picks by shape */
  float knots[LUTKAN_MAX_K + 1];      /* host copy of T, entries 0..K used (not used with knots_per_input) */
  const void *table;                  /* device, lutkan_info.table_bytes bytes, 16-byte aligned */
  int32_t knots_per_input;            /* 1: every input is located on its own row of input_knots */
  const float *input_knots;           /* device fp32 [d][K+1], a verbatim copy of lutkan_artifact_knots; NULL if shared */
  /* Optional second copy of the LUT table with 16-bit codes (see lutkan_wide_table_build); NULL / 0: none. */
  const void *wide_table;             /* device, lutkan_wide_table_bytes() bytes, 16-byte aligned */
  int32_t wide_blob_bytes;            /* bytes of one (tile, input) slice of the wide table */
  int32_t wide_code_bytes;            /* 2: binary16 codes; 4: dequantised fp32 values */
} lutkan_dev_layer;

typedef struct {
  int32_t d, m, G, degree, boundary, oob, value_repr, knot_span;
  int32_t jt, n_tiles, coef_blob_bytes;
  int32_t algo;
  float ext_knots[LUTKAN_MAX_K + 7];  /* host copy, entries 0..G+6 used */
  const float *coef_table;            /* device, lutkan_info.coef_table_bytes bytes, 16-byte aligned */
  int32_t knots_per_input;
  const float *input_ext_knots;       /* device fp32 [d][G+2p+1], a copy of lutkan_artifact_ext_knots; NULL if shared */
} bspline_dev_layer;

/* Fills every field of the device structs from an artifact except the device pointers (set to NULL). */
int lutkan_dev_layer_init(const lutkan_artifact *a, lutkan_dev_layer *out);
int bspline_dev_layer_init(const lutkan_artifact *a, bspline_dev_layer *out);

/* A wide form of the LUT device table: the same tiles and slice order ([t][i]) with more than a byte per code, so that
 * the tiled kernel spends fewer vector instructions per edge.  The codes stay 8-bit values and the artifact is what it
 * was; a wide form is a second, larger copy on the device (the byte table stays: the other kernels keep using it).
 *   code_bytes = 2  every code as the binary16 value q * 2^-24 (sign and magnitude; a subnormal whose bit pattern is
 *                   the magnitude of the code); the slice is otherwise the byte form's ([base][parameter rows][code
 *                   rows]).  A lane reads its codes as packed binary16 pairs and spends nothing on unpacking bytes or on
 *                   the excess-128 bias: 12 vector instructions per four edges instead of 18 (16 instead of 20 with
 *                   y_min), on the same arithmetic, bit for bit (Eq. 10 + Eq. 17).
 *   code_bytes = 4  every code dequantised: the fp32 value y_min + alpha * q of Eq. 10 (one rounding per operation; with
 *                   spline_component the folded parameters), slices [base][value rows], no parameter rows.  Per edge
 *                   the kernel then does Eq. 17 on the stored values, v0 + w * (v1 - v0): three plain fp32 instructions,
 *                   no scale or y_min to read, the same for both schemes.
 * Both cost device memory and LDS traffic per edge, and exist only for layers on 64-column tiles whose wide slice still
 * fits the LDS twice (K*L up to about 540 rows with 2 bytes per code, 285 with 4): on narrower tiles the LDS reads, not
 * the instructions, bound the kernel.  A forward call uses the form a layer holds on the tiled kernel when its launch
 * planning prices it below the byte form (large batches; the 2-byte form only for symmetric codes -- with y_min it
 * measured on par with the byte form); algo = TILED_WIDE takes it whatever the price.  A spline_component layer whose
 * base branch runs inside the edge kernel (16-byte records: calls below 5e8 edges) can use only the fp32 values, and
 * only if a slice of them is at most 64 KiB.
 * lutkan_wide_table_bytes: size of that form of the layer's table, 0 if the layer has none.
 * lutkan_wide_table_build: fills `wide_table` (device, 16-byte aligned, at least that many bytes) from layer->table on
 * `hip_stream` and sets layer->wide_table, wide_blob_bytes and wide_code_bytes; the layer may be used on that stream
 * right away, on others after the stream has been synchronised.  The memory stays the caller's.  Errors: EINVAL (null /
 * misaligned pointers, bad layer, code_bytes not 2 or 4), ESHAPE (bytes too small), EUNSUPPORTED (no such form), EHIP. */
size_t lutkan_wide_table_bytes(const lutkan_dev_layer *layer, int32_t code_bytes);
int lutkan_wide_table_build(lutkan_dev_layer *layer, int32_t code_bytes, void *wide_table, size_t bytes, void *hip_stream);

/* Sec. 5.5 / 5.6 counters: inputs (b,i) with In(x) = 0, and rows with at least one such input. */
typedef struct { unsigned long long oob_count, oob_any_rows; } lutkan_oob_stats;

/* Scratch needed by one forward call for B rows (per-(row,input) lookup records); 256-byte aligned use. */
size_t lutkan_forward_workspace_bytes(const lutkan_dev_layer *layer, int64_t B);
size_t bspline_forward_workspace_bytes(const bspline_dev_layer *layer, int64_t B);

/* LUT layer forward (Sec. 4.5 steps 1-5, Sec. 5.2-5.4, Eq. 1).  Per (row, input): the domain test on the raw
 * x, the safe clip x', the segment k, the local coordinate u and (l0, w) are computed once in IEEE fp32 and
 * reused for all m outputs; per edge two adjacent codes are gathered, dequantised with the segment's
 * (alpha, y_min), interpolated and summed over i in fp32.
 *   x          device [B][d] fp32          y   device [B][m] fp32 (overwritten)
 *   stats      device, nullable; the two counters are ADDED to (the caller zeroes them)
 *   workspace  device, >= lutkan_forward_workspace_bytes(layer, B), 256-byte aligned, contents undefined after
 * value_repr = spline_component (Eq. 2): the base branch s_out * s_base * SiLU(x), summed over the inputs, is evaluated
 * inside the edge kernel or, from 5e8 edge evaluations per call (d a multiple of 32, m >= 64, tiled kernel), as one
 * [B, d] x [d, m] product on the matrix cores with every fp32 operand cut exactly into three bf16 pieces (relative error
 * per term <= 2^-23), on top of which the edge kernel adds the spline branch; the two ways agree to rounding.  With
 * the product a row that contains an infinite input comes out NaN (edge by edge it may be +-inf).
 * Errors: EINVAL for null/ill-formed arguments, ESHAPE for a short workspace, EHIP if a launch fails. */
int lutkan_forward(const lutkan_dev_layer *layer, const float *x, int64_t B, float *y,
                   lutkan_oob_stats *stats, void *workspace, size_t workspace_bytes, void *hip_stream);

/* lutkan_forward for callers that cannot hand over a workspace because they cannot allocate one: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The lookup records and partial sums go to an array
 * of LUTKAN_STATIC_SCRATCH_BYTES bytes that is part of the library's device code: every GPU the library runs on holds
 * one copy from the first call on it until the process ends.  The call allocates and frees nothing and launches the
 * same kernels as lutkan_forward, so y and stats are bit-identical to lutkan_forward's.
 *   ESHAPE when lutkan_forward_workspace_bytes(layer, B) exceeds LUTKAN_STATIC_SCRATCH_BYTES (the message says by how
 *   much); other errors as lutkan_forward.
 * All calls on one GPU share that GPU's array: two calls may be in flight together only on the same stream (or
 * otherwise ordered one after the other); calls that overlap on one GPU race on the records.  Contents are undefined
 * between calls and nothing in the array needs clearing. */
#define LUTKAN_STATIC_SCRATCH_BYTES (64u << 20)
int lutkan_forward_static_scratch(const lutkan_dev_layer *layer, const float *x, int64_t B, float *y,
                                  lutkan_oob_stats *stats, void *hip_stream);

/* The two phases of lutkan_forward as separate calls, for callers that time or overlap them:
 *   lutkan_forward_locate   steps 1-4 of Sec. 4.5 and the domain test of Sec. 5.2 for every (row, input);
 *                           fills the workspace with the lookup records (and adds to stats, nullable)
 *   lutkan_forward_edges    step 5 (Eq. 10, 17), Sec. 5.4 and the sum of Eq. 1 from the records in the workspace
 * Calling locate then edges on one stream with the same layer, B and workspace equals lutkan_forward. */
int lutkan_forward_locate(const lutkan_dev_layer *layer, const float *x, int64_t B, lutkan_oob_stats *stats,
                          void *workspace, size_t workspace_bytes, void *hip_stream);
int lutkan_forward_edges(const lutkan_dev_layer *layer, int64_t B, float *y,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Same computation, additionally writing what the paper's contract fixes bit-exactly, for parity checks:
 *   k_out, l0_out  device int32 [B][d]  segment index (Eq. 14) and lower LUT index (Eq. 16)
 *   in_out         device uint8 [B][d]  In(x) of Sec. 5.2
 *   w_out          device fp32  [B][d]  interpolation weight (Eq. 16)
 *   q01_out        device int16 [B][d][m][2], nullable: the two gathered codes per edge (small layers only) */
int lutkan_forward_trace(const lutkan_dev_layer *layer, const float *x, int64_t B, float *y,
                         int32_t *k_out, int32_t *l0_out, uint8_t *in_out, float *w_out, int16_t *q01_out,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* B-spline layer forward (Eq. 1 over Eq. 3-5): per (row, input) the span and the four non-zero cubic basis
 * values are computed once by the Cox-de Boor recursion in fp32; per edge four coefficient FMAs; the same
 * boundary_mode / oob_policy as the LUT layer is applied to x first. */
int bspline_kan_forward(const bspline_dev_layer *layer, const float *x, int64_t B, float *y,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/* The two phases of bspline_kan_forward (span + basis values per (row, input); coefficient FMAs + sum). */
int bspline_forward_locate(const bspline_dev_layer *layer, const float *x, int64_t B,
                           void *workspace, size_t workspace_bytes, void *hip_stream);
int bspline_forward_edges(const bspline_dev_layer *layer, int64_t B, float *y,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Per-layer chaining (Sec. 5.1: intermediate activations feed the next layer and may leave its domain):
 * y of layer l is x of layer l+1.  The workspace holds two ping-pong activation buffers plus the largest
 * per-layer scratch.  layers[l].m must equal layers[l+1].d.  stats (nullable) points to n_layers entries.
 * The result is bit-identical to calling lutkan_forward layer by layer; when every layer is one that lutkan_forward
 * runs as a launch of the chain kernel (see lutkan_algo), the whole network runs as ONE launch of it. */
size_t lutkan_model_workspace_bytes(const lutkan_dev_layer *layers, int32_t n_layers, int64_t B);
int lutkan_model_forward(const lutkan_dev_layer *layers, int32_t n_layers, const float *x, int64_t B, float *y,
                         lutkan_oob_stats *stats, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same chain as lutkan_model_forward in ONE launch, for narrow networks at small batches (the batch-256 latency
 * setting of Sec. 8, where the per-layer launches cost more than the arithmetic): a work-group (up to 1024 rows) or a
 * wave (beyond) carries one row through all layers, activations stay in LDS, no workspace.  Per (row, input) and per edge the arithmetic is that of
 * lutkan_forward; only the order of the sum over the inputs differs (interleaved groups of inputs, then a fixed
 * butterfly), so results agree with lutkan_model_forward to rounding, not bit for bit.
 *   hidden   device, nullable: receives the activations between the layers, layer after layer, each [B][m_l]
 *            (sum over l < n_layers-1 of B*m_l floats)
 *   stats    device, nullable, n_layers entries, ADDED to
 * EUNSUPPORTED: more than 8 layers, a layer with more than one column tile (more than 64 outputs) or more than 1024
 * inputs.  Other errors as lutkan_model_forward. */
int lutkan_chain_forward(const lutkan_dev_layer *layers, int32_t n_layers, const float *x, int64_t B, float *y,
                         float *hidden, lutkan_oob_stats *stats, void *hip_stream);

/* Error statistics of the OOB evaluation protocol (Sec. 5.6 and the accuracy metrics of Sec. 6.5), in one pass on the
 * device: |y - y_ref| over the outputs of the in-range samples (rows whose d inputs all satisfy the domain predicate
 * In(x) of Sec. 5.2 under `boundary` on [t0, tK]) and of the OOB-only samples (rows with at least one input outside;
 * NaN counts as outside).  input_domain (device fp32 [d][2], nullable) gives every input its own {t0, tK} instead,
 * for layers with one knot vector per input.
 *   y, y_ref   device [B][m] fp32 (e.g. the LUT layer and the B-spline layer on the same x)
 *   x          device [B][d] fp32, the layer input that decides the subset of each row
 *   out        device, 8-byte aligned, overwritten
 *   workspace  device, >= lutkan_error_stats_workspace_bytes(B), 16-byte aligned
 * Differences are taken and summed in fp64; partial sums are combined in a fixed order (the result is reproducible).
 * An output whose difference is NaN is counted in its subset's nan_* and left out of that subset's sum, maximum and
 * mean:  mae = sum_abs / (rows * m - nan)  per subset, i.e. the mean of the differences that exist (NaN when the
 * subset has none);  oob_any_frac = rows_oob / B  (Sec. 5.6). */
typedef struct {
  unsigned long long rows_in, rows_oob;
  unsigned long long nan_in, nan_oob;
  double sum_abs_in, sum_abs_oob;
  double max_abs_in, max_abs_oob;
  double mae_in, mae_oob;
  double oob_any_frac;
} lutkan_error_summary;
size_t lutkan_error_stats_workspace_bytes(int64_t B);
int lutkan_error_stats(const float *y, const float *y_ref, int64_t B, int32_t m, const float *x, int32_t d,
                       float t0, float tK, const float *input_domain, int32_t boundary, lutkan_error_summary *out,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Measurement aid, not part of the method: launches one kernel of known work that exercises a single resource, so
 * that a caller who times it (events on hip_stream) learns the rate this machine sustains and can put the layer
 * kernels' roofline terms beside measured peaks as well as published ones.
 *   kind          LUTKAN_PROBE_VALU_FMA  non-packed fp32 FMAs, 16 independent chains per lane   work = flop
 *                                        (three-operand encoding with a scalar operand: the 4-cycle issue rate that the
 *                                        layer kernels' instructions share)
 *                 LUTKAN_PROBE_VALU_FMAC the same count in the two-operand encoding on registers, which gfx950 issues
 *                                        faster than once per 4 cycles                          work = flop
 *                 LUTKAN_PROBE_LDS_READ  conflict-free 16-byte LDS reads                        work = bytes
 *                 LUTKAN_PROBE_L2_READ   every work-group re-reads the same 2 MiB               work = bytes
 *                 LUTKAN_PROBE_HBM_READ  the whole buffer once per pass (buffer >= 1 GiB)       work = bytes
 *                 LUTKAN_PROBE_VALU_MIX  the instruction mix of the tiled LUT kernel (per row step 2 16-bit
 *                                        multiply-adds, 4 byte permutes, 4 packed-fp16 adds, 4 mixed-precision FMAs,
 *                                        4 fp32 FMAs), one 16-wave work-group per compute unit  work = lane-instructions
 *   buffer        device, 16-byte aligned; the first 16 bytes are a sink, the rest is read (contents irrelevant, but
 *                 finite floats for the LDS probe); needs 16 B / 16 KiB+16 / 2 MiB+16 / >= 1 GiB by kind
 *   iters         repetitions inside the kernel, 1 .. 2^20
 *   work_out      host: the flop or bytes one launch performs
 * Errors: EINVAL (null, misaligned, unknown kind, iters), ESHAPE (buffer too small), EHIP. */
typedef enum { LUTKAN_PROBE_VALU_FMA = 0, LUTKAN_PROBE_LDS_READ = 1, LUTKAN_PROBE_L2_READ = 2, LUTKAN_PROBE_HBM_READ = 3,
               LUTKAN_PROBE_VALU_MIX = 4, LUTKAN_PROBE_VALU_FMAC = 5 } lutkan_probe_kind;
int lutkan_probe_launch(int32_t kind, void *buffer, size_t buffer_bytes, int32_t iters, double *work_out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LUTKAN_H */

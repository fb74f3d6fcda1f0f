/* libaaac — MI355X (gfx950) kernels for the per-layer activation-weighted
 * k-means of AAAC (Activation-Aware Adaptive Codebooks, 4-bit LLM weight
 * quantisation): two learned 16-entry scalar codebooks T0, T1 per linear layer,
 * one of them selected per weight group, the choice stored in the sign bit of the
 * group's positive scale.
 *
 * C ABI.  Conventions common to every entry point:
 *   - "dev" pointers are HIP device pointers on the current device; "HOST"
 *     pointers are ordinary host memory, read before the call returns.
 *   - The caller owns every buffer.  The library allocates nothing, keeps no state
 *     between calls (aaac_act_stats_static excepted, see there) and never
 *     synchronises: all work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream); outputs are
 *     valid once the caller has synchronised that stream.  Two calls may run
 *     concurrently if they use different workspaces and outputs.
 *   - bf16 tensors are arrays of 16-bit patterns (upper half of an IEEE fp32).
 *   - Matrices are row-major with a leading dimension in elements; weight groups
 *     of `group_size` run along the input dimension K of W [N x K].
 *   - Return value: AAAC_OK or a negative aaac_status_t.  Arguments are validated
 *     on the host before any HIP call, and the workspace queries make none, so
 *     argument errors and workspace sizes are reported without a GPU; a failed
 *     launch gives AAAC_ERR_HIP.  Not checked: that W, X and the importances are
 *     finite and the importances non-negative.
 *   - The launch paths ask the runtime for the current device's compute-unit
 *     count at every call; nothing is cached between calls or across devices.
 *   - Matrix pointers may be NULL when N == 0 (nothing is read or written).
 *   - Shapes: K % group_size == 0, group_size in {16, 32, 64, 128}, leading
 *     dimensions >= K and multiples of 8, device matrices and the importance
 *     vector 16-byte aligned.
 */
#ifndef AAAC_H_
#define AAAC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Scale format of a group (paper section 3.1, base quantiser; Alg. 1 step 1; the
 * constants are those of the two benchmark settings):
 *   NVFP4: stored scale = OCP FP8 E4M3 (nearest-even, saturating) of absmax/6, 1 byte
 *   INT4 : stored scale = bf16 (nearest-even) of absmax/7, 2 bytes
 * A scale that would be 0 (or, for bf16, subnormal) is replaced by the smallest
 * positive value (E4M3 0x01 = 2^-9, bf16 0x0080 = 2^-126), so a stored scale is
 * always > 0 and its top bit is free to carry the selection bit. */
typedef enum { AAAC_FMT_NVFP4 = 0, AAAC_FMT_INT4 = 1 } aaac_format_t;

typedef enum {
  AAAC_OK = 0,
  AAAC_ERR_NULL = -1,      /* a required pointer is NULL */
  AAAC_ERR_SHAPE = -2,     /* sizes, leading dimensions, group size or alignment */
  AAAC_ERR_ARG = -3,       /* format, iteration count or initial grid (unsorted / not finite) */
  AAAC_ERR_WORKSPACE = -4, /* workspace NULL, misaligned (256 B) or too small */
  AAAC_ERR_HIP = -5        /* a HIP call failed */
} aaac_status_t;

const char* aaac_status_string(int status);

/* ---- Activation importance (paper Eq. "importance": I_k = sum_t X[t,k]^2;
 * Alg. 1 step 3).  X: dev bf16 [tokens x ldx].  importance: dev fp32 [K],
 * overwritten; each entry is the sum taken in fp64 and rounded once to fp32.
 * tokens == 0 gives zeros.  ws: dev scratch of at least
 * aaac_act_stats_workspace(tokens, K) bytes, 256-byte aligned. */
size_t aaac_act_stats_workspace(int64_t tokens, int64_t K);
int aaac_act_stats(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                   void* ws, size_t ws_bytes, void* hip_stream);

/* ---- aaac_act_stats for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels, the same result bit for bit, with the partial sums kept in an 8 MiB array
 * that is part of the library's device code, so no workspace is passed and neither
 * this call nor anything it calls allocates or frees memory.
 *   - Limit: K <= 1,048,576 columns (what 8 MiB of partial sums hold); a larger K is
 *     AAAC_ERR_WORKSPACE.  Other arguments and errors as aaac_act_stats.
 *   - Each GPU the library runs on holds its own copy of the array until the process
 *     ends.  The first call on a device looks up that copy's address (one runtime
 *     query, kept per device); make that first call outside graph capture.
 *   - All calls on one GPU share the array: calls that overlap on one GPU (different
 *     streams, or threads) race and give wrong sums; calls on one stream are ordered.
 *     Nothing has to be cleared between calls: every partial sum a call reads, it has
 *     written before. */
int aaac_act_stats_static(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                          void* hip_stream);

/* ---- Codebook learning (paper Alg. 1 from "compute scales" to the end of the
 * outer loop, with n_inner = 1 and caller-supplied initial tables; Eq.
 * "selection" for the assignment step, Eq. "kmeans_update" for the table update).
 * One iteration = one assignment step over every group (nearest entry of each
 * normalised weight w~ = w * fl32(1/s) in T0 and in T1 by the midpoint rule: index
 * = number of midpoints fl32(0.5*(T[i]+T[i+1])) strictly below w~; per-group errors
 * sum_k I_k (w~ - T[idx])^2 in fp32, summed as a balanced tree of adjacent pairs;
 * sigma = 1 iff e1 < e0) followed by one weighted-centroid update of all 32
 * entries (sums in fp64; an entry whose cell has zero total importance keeps its
 * value), after which each table is sorted ascending.
 *   W            dev bf16 [N x ldw]
 *   importance   dev fp32 [K], >= 0
 *   init_grid    HOST fp32 [32]: T0[0..15] then T1[0..15], each non-decreasing, finite
 *   iterations   >= 0 (0 returns the initial grid)
 *   tables_f32   dev fp32 [32] or NULL: tables after the last update (not rounded);
 *                feeding them back as init_grid continues the iteration exactly
 *   tables_bf16  dev u16 [32]: the same rounded to bf16 (nearest-even) — the
 *                64-byte per-layer artefact (paper section 3.2 "Storage")
 *   objective_trace dev fp64 [iterations] or NULL: sum over groups of min(e0, e1)
 *                as seen by each assignment step
 *   ws           dev scratch, >= aaac_fit_workspace(N, K, group_size, fmt) bytes
 * N == 0 is allowed (tables stay at init_grid).
 * How the passes are launched does not change what is computed: a single small layer
 * (at most 512 rows of 512-column strips) runs all its passes in one launch whose blocks
 * exchange partial sums and add them in a fixed order; larger layers and batches take
 * one launch per pass, with fp64 sums added in arrival order (results may differ between
 * runs in the last bits of an fp64 sum).  The environment variable AAAC_FIT_PATH, read at
 * every call, overrides the choice for measurements and tests: "launches" never takes
 * the one-launch path, "persistent" takes it for every single layer it can hold (2048
 * rows of strips).  If the blocks of a one-launch fit cannot exchange their sums within
 * about four seconds (a device kept busy by other work), the tables come back as NaN. */
size_t aaac_fit_workspace(int64_t N, int64_t K, int group_size, aaac_format_t fmt);
int aaac_fit(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, aaac_format_t fmt,
             const float* importance, const float* init_grid, int iterations, float* tables_f32,
             uint16_t* tables_bf16, double* objective_trace, void* ws, size_t ws_bytes,
             void* hip_stream);

/* Several layers that share group size, format, initial grid and iteration count
 * (e.g. the seven linears of a decoder block) in one call; per-layer semantics are
 * exactly those of aaac_fit.  `layers` is a HOST array. */
typedef struct {
  const void* W;           /* dev bf16 [N x ldw] */
  int64_t N, K, ldw;
  const float* importance; /* dev fp32 [K] */
  float* tables_f32;       /* dev [32] or NULL */
  uint16_t* tables_bf16;   /* dev [32] */
  double* objective_trace; /* dev [iterations] or NULL */
} aaac_layer_t;
size_t aaac_fit_batch_workspace(const aaac_layer_t* layers, int n_layers, int group_size,
                                aaac_format_t fmt);
int aaac_fit_batch(const aaac_layer_t* layers, int n_layers, int group_size, aaac_format_t fmt,
                   const float* init_grid, int iterations, void* ws, size_t ws_bytes,
                   void* hip_stream);

/* ---- Codebook learning as the paper's Alg. 1 states it in full: both loops and both
 * granularity parameters ("Granularity parameters": every group_size weights share a
 * scale, every sel_size weights share a table choice; sel_size is 16, 32, 64 or 128
 * and divides group_size).  n_outer assignment steps (Eq. "selection", one choice per
 * sel_size weights), each followed by n_inner k-means steps (Eq. "kmeans_update") that
 * keep the choices fixed: every weight of a selection group that chose table r goes to
 * the cell of its nearest entry of the current T_r, entries move to the weighted
 * centroids (empty cell: keep), and the tables are sorted after each step.
 * n_inner = 1 with sel_size = group_size is aaac_fit_batch with iterations = n_outer.
 * objective_trace of a layer holds n_outer values (the objective seen by each
 * assignment step).  n_outer >= 0, n_inner >= 1.
 * init_grid (HOST, 32 floats) as in aaac_fit, or NULL: the tables then start from the
 * quantiles of each layer's normalised weights, as Alg. 1 steps 4-5 state (see
 * aaac_quantile_init); a layer without weights is then AAAC_ERR_SHAPE.
 * Errors as aaac_fit; a sel_size that is not allowed is AAAC_ERR_SHAPE. */
size_t aaac_fit_nested_workspace(const aaac_layer_t* layers, int n_layers, int group_size,
                                 int sel_size, aaac_format_t fmt);
int aaac_fit_nested(const aaac_layer_t* layers, int n_layers, int group_size, int sel_size,
                    aaac_format_t fmt, const float* init_grid, int n_outer, int n_inner, void* ws,
                    size_t ws_bytes, void* hip_stream);

/* ---- Quantile initialisation of the two tables (paper Eq. "init_t0", Eq. "init_t1";
 * Alg. 1 steps 4-5), 16 entries each:
 *   T0[i] = Quantile_{i/15},  T1[i] = Quantile_{1/30 + (29/30) i/15},  i = 0..15,
 * of all N*K normalised weights w~ of the layer.  The quantile of level q = num/den
 * is taken by linear interpolation between order statistics x_(0) <= ... <= x_(n-1):
 * with lo = num*(n-1) div den and rem = num*(n-1) mod den (exact integers),
 * value = fl32( x_(lo) + (rem/den) * (x_(lo+1) - x_(lo)) ) evaluated in fp64; a zero is
 * stored as +0.  The order statistics are exact (radix select, no sampling; three passes
 * over the weights and one over the keys that can still matter, kept in ws).
 *   grid   dev fp32 [32], overwritten: T0[0..15] then T1[0..15], each ascending
 *   ws     dev scratch of aaac_quantile_init_workspace(...) bytes, 256-byte aligned
 * N = 0 or K = 0 is AAAC_ERR_SHAPE (no weights to take quantiles of); other errors as
 * aaac_fit. */
size_t aaac_quantile_init_workspace(int64_t N, int64_t K, int group_size, aaac_format_t fmt);
int aaac_quantile_init(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size,
                       aaac_format_t fmt, float* grid, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- Final encode (paper Alg. 1, last four steps; Eq. "aaac_code").  With the
 * bf16 tables (each non-decreasing), recompute sigma per group, write each
 * weight's nearest-entry index into the selected table as a 4-bit code, and the
 * group's scale with sigma in its top bit.
 *   tables_bf16  dev u16 [32]
 *   codes        dev u8 [N x K/2], dense: column k even -> low nibble, odd -> high
 *   scales       dev [N x K/group_size] of u8 (NVFP4) or u16 (INT4); top bit = sigma */
int aaac_encode(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, aaac_format_t fmt,
                const float* importance, const uint16_t* tables_bf16, uint8_t* codes, void* scales,
                void* hip_stream);

/* ---- Dequantisation (paper Eq. "aaac_dequant"): W_hat[n,k] = bf16( T_sigma[code]
 * * s ), sigma = top bit of the stored scale, s = the scale with that bit cleared.
 *   W_hat        dev bf16 [N x ldo] */
int aaac_dequant(const uint8_t* codes, const void* scales, const uint16_t* tables_bf16, int64_t N,
                 int64_t K, int group_size, aaac_format_t fmt, void* W_hat, int64_t ldo,
                 void* hip_stream);

/* ---- Encode and dequantisation with selection groups smaller than scale groups
 * (paper "Granularity parameters"; Alg. 1 last step: the choices are stored in the
 * sign bits of the scales if sel_size == group_size, separately otherwise, at
 * 1/sel_size bits per weight).
 * sel_size == group_size: exactly aaac_encode / aaac_dequant; sel_bits is ignored and
 * may be NULL.  sel_size < group_size: the stored scales are unsigned (top bit 0) and
 *   sel_bits   dev u8 [N x sel_stride]: the choice of selection group j of row n
 *              (columns j*sel_size .. (j+1)*sel_size - 1) is bit (j % 8), counted from
 *              the least significant, of byte n*sel_stride + j/8; the unused bits of a
 *              row's last used byte are written as 0; bytes beyond ceil(K/sel_size/8)
 *              in a row are not touched.
 *   sel_stride bytes per row, >= ceil(K / sel_size / 8).
 * Errors as aaac_encode / aaac_dequant; sel_bits NULL when needed is AAAC_ERR_NULL, a
 * bad sel_size or sel_stride AAAC_ERR_SHAPE. */
int aaac_encode_sel(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, int sel_size,
                    aaac_format_t fmt, const float* importance, const uint16_t* tables_bf16,
                    uint8_t* codes, void* scales, uint8_t* sel_bits, int64_t sel_stride,
                    void* hip_stream);
int aaac_dequant_sel(const uint8_t* codes, const void* scales, const uint8_t* sel_bits,
                     int64_t sel_stride, const uint16_t* tables_bf16, int64_t N, int64_t K,
                     int group_size, int sel_size, aaac_format_t fmt, void* W_hat, int64_t ldo,
                     void* hip_stream);

/* ---- The quantised layer applied to activations, W4A16 (paper Eq. "pipeline": the
 * dequantised values w^ = T[c] * s are the weights used at inference; Eq. "aaac_dequant"
 * with the two tables):
 *   y[m, n] = sum_k x[m, k] * T_sigma[code[n, k]] * s[n, k / group_size]
 * computed from the codes, scales (and selection bits) as aaac_encode / aaac_encode_sel
 * write them; the dequantised weights are never stored and w^ is the real product (no
 * bf16 rounding of it).  Arithmetic: fp32 accumulation of exact bf16 products, every term
 * exact; only the order of the additions differs from exact evaluation: at most
 * 22 + 4 * ceil(K / 2048) roundings lie on the path of a term, so
 * |error| <= (22 + 4 * ceil(K / 2048)) * 2^-24 * sum_k |x w^| to first order.  The additions
 * across column slabs are LDS atomics whose order is not fixed: results may differ between
 * runs in the last bits.
 * Meant for a few rows of x (decode); x is taken eight rows at a time, so larger M
 * re-reads the codes M/8 times.
 *   x        dev bf16 [M x ldx], ldx >= K, ldx % 8 == 0, 16-byte aligned
 *   codes    dev u8 [N x K/2] dense, 16-byte aligned; K % 32 == 0
 *   scales, sel_bits, sel_stride, tables_bf16, group_size, sel_size, fmt: as aaac_dequant_sel
 *            (scales 4-byte aligned)
 *   y        dev fp32 [M x ldy], ldy >= N, overwritten
 * Errors as aaac_dequant_sel; K % 32 != 0 is AAAC_ERR_SHAPE. */
int aaac_gemv_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                    const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16, int64_t N,
                    int64_t K, int group_size, int sel_size, aaac_format_t fmt, float* y, int64_t ldy,
                    void* hip_stream);

/* ---- The same product for a batch of activation rows on the matrix cores: the
 * dequantised weights are rounded to bf16, w^ = bf16(T_sigma[code] * s), exactly the
 * values aaac_dequant / aaac_dequant_sel store (a matrix-core operand is bf16), products
 * are accumulated in fp32:
 *   y[m, n] = sum_k x[m, k] * w^[n, k]
 * so the result is the fp32-accumulated product of x with the dequantised layer, without
 * that layer ever being written.  Small batches go 32 rows of x at a time, which stay in
 * registers while the codes are read once; large batches use 128 x 128 / 128 x 256 tiles
 * whose weights are dequantised once per tile.  Where the layer's rows (small batches) or
 * the tiles (large batches) are fewer than the compute units, K is split over blocks that
 * add their parts into y with atomics whose order is not fixed: results may then differ
 * between runs in the last bits.
 * Arguments and errors as aaac_gemv_w4a16, except K % 64 == 0, scales 8-byte aligned, and
 *   ws       dev scratch of aaac_gemm_w4a16_workspace(M, K) bytes, 256-byte aligned (x
 *            is first copied into the matrix instruction's operand order); too small or
 *            misaligned is AAAC_ERR_WORKSPACE. */
size_t aaac_gemm_w4a16_workspace(int64_t M, int64_t K);
int aaac_gemm_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                    const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16, int64_t N,
                    int64_t K, int group_size, int sel_size, aaac_format_t fmt, float* y, int64_t ldy,
                    void* ws, size_t ws_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AAAC_H_ */

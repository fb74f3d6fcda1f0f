// C ABI of libaaac (declared in include/aaac.h): argument validation on the
// host, workspace carving, then kernel launches on the caller's stream.
#include "aaac.h"

#include <cmath>

#include "aaac_internal.h"

namespace {

bool valid_group(int g) { return g == 16 || g == 32 || g == 64 || g == 128; }
bool valid_fmt(int f) { return f == AAAC_FMT_NVFP4 || f == AAAC_FMT_INT4; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Shape rules shared by every entry point that takes a [N x K] matrix.
int check_matrix(const void* p, int64_t N, int64_t K, int64_t ld, int group_size) {
  if (N < 0 || K < 0) return AAAC_ERR_SHAPE;
  if (!valid_group(group_size)) return AAAC_ERR_SHAPE;
  if (K % group_size != 0) return AAAC_ERR_SHAPE;
  if (ld < K || ld % 8 != 0) return AAAC_ERR_SHAPE;
  if (N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31) return AAAC_ERR_SHAPE;
  if (!aligned(p, 16)) return AAAC_ERR_SHAPE;
  return AAAC_OK;
}

// sel_size: 16..128 and a divisor of the scale group size.
bool valid_sel(int sel_size, int group_size) {
  return valid_group(sel_size) && sel_size <= group_size && group_size % sel_size == 0;
}

int check_grid(const float* g) {
  for (int i = 0; i < 32; ++i)
    if (!std::isfinite(g[i])) return AAAC_ERR_ARG;
  for (int t = 0; t < 2; ++t)
    for (int i = 1; i < 16; ++i)
      if (g[16 * t + i] < g[16 * t + i - 1]) return AAAC_ERR_ARG;
  return AAAC_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return AAAC_OK;
  if (ws == nullptr || !aligned(ws, 256) || have < need) return AAAC_ERR_WORKSPACE;
  return AAAC_OK;
}

int from_hip(hipError_t e) { return e == hipSuccess ? AAAC_OK : AAAC_ERR_HIP; }

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int check_layer(const aaac_layer_t& l, int group_size) {
  if ((l.W == nullptr && l.N > 0) || l.importance == nullptr || l.tables_bf16 == nullptr) return AAAC_ERR_NULL;
  if (!aligned(l.importance, 16)) return AAAC_ERR_SHAPE;
  return check_matrix(l.W, l.N, l.K, l.ldw, group_size);
}

// Shared body of the two W4A16 products: vector ALUs (a few rows of x, weights unrounded) or matrix
// cores (weights rounded to bf16).
int w4a16_entry(bool matrix_cores, const void* x, int64_t M, int64_t ldx, const uint8_t* codes,
                const void* scales, const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                int64_t N, int64_t K, int group_size, int sel_size, aaac_format_t fmt, float* y, int64_t ldy,
                void* ws, size_t ws_bytes, void* hip_stream) {
  if (tables_bf16 == nullptr) return AAAC_ERR_NULL;
  if (M > 0 && N > 0 && (y == nullptr || (K > 0 && (x == nullptr || codes == nullptr || scales == nullptr))))
    return AAAC_ERR_NULL;
  if (M < 0 || N < 0 || K < 0 || M >= (int64_t)1 << 31 || N >= (int64_t)1 << 31 || K >= (int64_t)1 << 31)
    return AAAC_ERR_SHAPE;
  if (!valid_group(group_size) || !valid_sel(sel_size, group_size)) return AAAC_ERR_SHAPE;
  if (K % group_size != 0 || K % (matrix_cores ? 64 : 32) != 0) return AAAC_ERR_SHAPE;
  if (ldx < K || ldx % 8 != 0 || ldy < N) return AAAC_ERR_SHAPE;
  if (sel_size < group_size) {
    if (M > 0 && N > 0 && K > 0 && sel_bits == nullptr) return AAAC_ERR_NULL;
    if (sel_stride < (K / sel_size + 7) / 8) return AAAC_ERR_SHAPE;
  }
  if (!valid_fmt(fmt)) return AAAC_ERR_ARG;
  if (!aligned(x, 16) || !aligned(codes, 16) || !aligned(scales, matrix_cores ? 8 : 4) || !aligned(y, 4))
    return AAAC_ERR_SHAPE;
  if (matrix_cores && M > 0 && N > 0 && K > 0) {
    const int rc = check_ws(ws, ws_bytes, aaac::gemm_w4a16_workspace(M, K));
    if (rc) return rc;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  return from_hip(matrix_cores ? aaac::launch_gemm_w4a16(x, M, ldx, codes, scales, sel_bits, sel_stride, tables_bf16,
                                                         N, K, group_size, sel_size, fmt, y, ldy, ws, stream)
                               : aaac::launch_gemv_w4a16(x, M, ldx, codes, scales, sel_bits, sel_stride, tables_bf16,
                                                         N, K, group_size, sel_size, fmt, y, ldy, stream));
}

}  // namespace

extern "C" {

const char* aaac_status_string(int status) {
  switch (status) {
    case AAAC_OK: return "ok";
    case AAAC_ERR_NULL: return "a required pointer is NULL";
    case AAAC_ERR_SHAPE: return "bad shape, leading dimension, group size or alignment";
    case AAAC_ERR_ARG: return "bad format, iteration count or initial grid";
    case AAAC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case AAAC_ERR_HIP: return "a HIP call failed";
    default: return "unknown status";
  }
}

size_t aaac_act_stats_workspace(int64_t tokens, int64_t K) {
  if (tokens < 0 || K <= 0) return 0;
  return aaac::make_stats_plan(tokens, K).bytes;
}

int aaac_act_stats(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance, void* ws,
                   size_t ws_bytes, void* hip_stream) {
  if (importance == nullptr || (X == nullptr && tokens > 0)) return AAAC_ERR_NULL;
  if (tokens < 0 || K <= 0 || K % 8 != 0 || ldx < K || ldx % 8 != 0) return AAAC_ERR_SHAPE;
  if (tokens > (int64_t)1 << 40 || K > (int64_t)1 << 31) return AAAC_ERR_SHAPE;
  if (!aligned(X, 16)) return AAAC_ERR_SHAPE;
  aaac::StatsPlan plan = aaac::make_stats_plan(tokens, K);
  if (tokens > 0) {
    int rc = check_ws(ws, ws_bytes, plan.bytes);
    if (rc) return rc;
  }
  return from_hip(aaac::launch_act_stats(X, tokens, K, ldx, importance, ws, plan,
                                         static_cast<hipStream_t>(hip_stream)));
}

int aaac_act_stats_static(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                          void* hip_stream) {
  if (importance == nullptr || (X == nullptr && tokens > 0)) return AAAC_ERR_NULL;
  if (tokens < 0 || K <= 0 || K % 8 != 0 || ldx < K || ldx % 8 != 0) return AAAC_ERR_SHAPE;
  if (tokens > (int64_t)1 << 40 || K > (int64_t)1 << 31) return AAAC_ERR_SHAPE;
  if (!aligned(X, 16)) return AAAC_ERR_SHAPE;
  aaac::StatsPlan plan = aaac::make_stats_plan(tokens, K);
  if (plan.bytes > aaac::kStaticScratchBytes) return AAAC_ERR_WORKSPACE;  // K beyond what the array holds
  return from_hip(aaac::launch_act_stats_static(X, tokens, K, ldx, importance, plan,
                                                static_cast<hipStream_t>(hip_stream)));
}

size_t aaac_fit_workspace(int64_t N, int64_t K, int group_size, aaac_format_t fmt) {
  if (N < 0 || K < 0 || !valid_group(group_size) || !valid_fmt(fmt) || K % group_size != 0) return 0;
  return aaac::fit_layout(N, K, group_size, group_size).bytes;
}

size_t aaac_quantile_init_workspace(int64_t N, int64_t K, int group_size, aaac_format_t fmt) {
  return aaac_fit_workspace(N, K, group_size, fmt);
}

int aaac_quantile_init(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, aaac_format_t fmt,
                       float* grid, void* ws, size_t ws_bytes, void* hip_stream) {
  if (W == nullptr || grid == nullptr) return AAAC_ERR_NULL;
  int rc = check_matrix(W, N, K, ldw, group_size);
  if (rc) return rc;
  if (N == 0 || K == 0) return AAAC_ERR_SHAPE;
  if (!valid_fmt(fmt)) return AAAC_ERR_ARG;
  const aaac::FitLayout p = aaac::fit_layout(N, K, group_size, group_size);
  rc = check_ws(ws, ws_bytes, p.bytes);
  if (rc) return rc;
  char* base = static_cast<char*>(ws);
  float* rinv = reinterpret_cast<float*>(base + p.off_rinv);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (aaac::launch_group_rinv(W, N, K, ldw, group_size, fmt, rinv, stream) != hipSuccess) return AAAC_ERR_HIP;
  return from_hip(aaac::launch_quantile_init(W, N, K, ldw, group_size, rinv, base + p.off_quant,
                                             reinterpret_cast<uint32_t*>(base + p.off_cand),
                                             aaac::quant_candidates(N, K), grid, stream));
}

int aaac_fit(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, aaac_format_t fmt,
             const float* importance, const float* init_grid, int iterations, float* tables_f32,
             uint16_t* tables_bf16, double* objective_trace, void* ws, size_t ws_bytes,
             void* hip_stream) {
  if (init_grid == nullptr) return AAAC_ERR_NULL;
  aaac_layer_t layer = {W, N, K, ldw, importance, tables_f32, tables_bf16, objective_trace};
  return aaac_fit_batch(&layer, 1, group_size, fmt, init_grid, iterations, ws, ws_bytes, hip_stream);
}

size_t aaac_fit_batch_workspace(const aaac_layer_t* layers, int n_layers, int group_size,
                                aaac_format_t fmt) {
  return aaac_fit_nested_workspace(layers, n_layers, group_size, group_size, fmt);
}

int aaac_fit_batch(const aaac_layer_t* layers, int n_layers, int group_size, aaac_format_t fmt,
                   const float* init_grid, int iterations, void* ws, size_t ws_bytes,
                   void* hip_stream) {
  if (init_grid == nullptr) return AAAC_ERR_NULL;
  return aaac_fit_nested(layers, n_layers, group_size, group_size, fmt, init_grid, iterations, 1, ws, ws_bytes,
                         hip_stream);
}

size_t aaac_fit_nested_workspace(const aaac_layer_t* layers, int n_layers, int group_size,
                                 int sel_size, aaac_format_t fmt) {
  if (layers == nullptr || n_layers < 0) return 0;
  if (!valid_group(group_size) || !valid_sel(sel_size, group_size) || !valid_fmt(fmt)) return 0;
  size_t total = 0;
  for (int i = 0; i < n_layers; ++i) {
    const int64_t N = layers[i].N, K = layers[i].K;
    if (N < 0 || K < 0 || K % group_size != 0) return 0;
    total += align256(aaac::fit_layout(N, K, group_size, sel_size).bytes);
  }
  return total;
}

int aaac_fit_nested(const aaac_layer_t* layers, int n_layers, int group_size, int sel_size,
                    aaac_format_t fmt, const float* init_grid, int n_outer, int n_inner, void* ws,
                    size_t ws_bytes, void* hip_stream) {
  if (layers == nullptr) return AAAC_ERR_NULL;
  if (n_layers < 0) return AAAC_ERR_SHAPE;
  if (!valid_fmt(fmt) || n_outer < 0 || n_inner < 1) return AAAC_ERR_ARG;
  if ((int64_t)n_outer * n_inner > (int64_t)1 << 30) return AAAC_ERR_ARG;
  if (!valid_group(group_size) || !valid_sel(sel_size, group_size)) return AAAC_ERR_SHAPE;
  for (int i = 0; i < n_layers; ++i) {
    int rc = check_layer(layers[i], group_size);
    if (rc) return rc;
  }
  int rc = AAAC_OK;
  if (init_grid != nullptr) {
    rc = check_grid(init_grid);
    if (rc) return rc;
  } else {  // quantile initialisation needs weights to take quantiles of
    for (int i = 0; i < n_layers; ++i)
      if (layers[i].N == 0 || layers[i].K == 0) return AAAC_ERR_SHAPE;
  }
  rc = check_ws(ws, ws_bytes, aaac_fit_nested_workspace(layers, n_layers, group_size, sel_size, fmt));
  if (rc) return rc;

  aaac::Grid32 grid = {};
  if (init_grid != nullptr)
    for (int i = 0; i < 32; ++i) grid.t[i] = init_grid[i];
  char* base = static_cast<char*>(ws);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // the layers are fitted in groups whose passes share one launch each
  for (int first = 0; first < n_layers; first += aaac::kMaxFusedLayers) {
    aaac::FitTask tasks[aaac::kMaxFusedLayers];
    int n = 0;
    for (int i = first; i < n_layers && n < aaac::kMaxFusedLayers; ++i, ++n) {
      const aaac_layer_t& l = layers[i];
      tasks[n] = {l.W, l.N, l.K, l.ldw, l.importance, l.tables_f32, l.tables_bf16, l.objective_trace, base};
      base += align256(aaac::fit_layout(l.N, l.K, group_size, sel_size).bytes);
    }
    if (aaac::launch_fit_group(tasks, n, group_size, sel_size, fmt, init_grid ? &grid : nullptr, n_outer, n_inner,
                               stream) != hipSuccess)
      return AAAC_ERR_HIP;
  }
  return AAAC_OK;
}

int aaac_encode(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, aaac_format_t fmt,
                const float* importance, const uint16_t* tables_bf16, uint8_t* codes, void* scales,
                void* hip_stream) {
  return aaac_encode_sel(W, N, K, ldw, group_size, group_size, fmt, importance, tables_bf16, codes, scales,
                         nullptr, 0, hip_stream);
}

int aaac_dequant(const uint8_t* codes, const void* scales, const uint16_t* tables_bf16, int64_t N,
                 int64_t K, int group_size, aaac_format_t fmt, void* W_hat, int64_t ldo,
                 void* hip_stream) {
  return aaac_dequant_sel(codes, scales, nullptr, 0, tables_bf16, N, K, group_size, group_size, fmt, W_hat, ldo,
                          hip_stream);
}

int aaac_encode_sel(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, int sel_size,
                    aaac_format_t fmt, const float* importance, const uint16_t* tables_bf16,
                    uint8_t* codes, void* scales, uint8_t* sel_bits, int64_t sel_stride,
                    void* hip_stream) {
  if (importance == nullptr || tables_bf16 == nullptr) return AAAC_ERR_NULL;
  if (N > 0 && (W == nullptr || codes == nullptr || scales == nullptr)) return AAAC_ERR_NULL;
  int rc = check_matrix(W, N, K, ldw, group_size);
  if (rc) return rc;
  if (!valid_sel(sel_size, group_size)) return AAAC_ERR_SHAPE;
  if (sel_size < group_size) {
    if (N > 0 && sel_bits == nullptr) return AAAC_ERR_NULL;
    if (sel_stride < (K / sel_size + 7) / 8) return AAAC_ERR_SHAPE;
  }
  if (!valid_fmt(fmt)) return AAAC_ERR_ARG;
  if (!aligned(codes, 4) || !aligned(scales, 2) || !aligned(importance, 16)) return AAAC_ERR_SHAPE;
  return from_hip(aaac::launch_encode(W, N, K, ldw, group_size, sel_size, fmt, importance, tables_bf16, codes,
                                      scales, sel_bits, sel_stride, static_cast<hipStream_t>(hip_stream)));
}

int aaac_dequant_sel(const uint8_t* codes, const void* scales, const uint8_t* sel_bits,
                     int64_t sel_stride, const uint16_t* tables_bf16, int64_t N, int64_t K,
                     int group_size, int sel_size, aaac_format_t fmt, void* W_hat, int64_t ldo,
                     void* hip_stream) {
  if (tables_bf16 == nullptr) return AAAC_ERR_NULL;
  if (N > 0 && (codes == nullptr || scales == nullptr || W_hat == nullptr)) return AAAC_ERR_NULL;
  int rc = check_matrix(W_hat, N, K, ldo, group_size);
  if (rc) return rc;
  if (!valid_sel(sel_size, group_size)) return AAAC_ERR_SHAPE;
  if (sel_size < group_size) {
    if (N > 0 && sel_bits == nullptr) return AAAC_ERR_NULL;
    if (sel_stride < (K / sel_size + 7) / 8) return AAAC_ERR_SHAPE;
  }
  if (!valid_fmt(fmt)) return AAAC_ERR_ARG;
  if (!aligned(codes, 4) || !aligned(scales, 2)) return AAAC_ERR_SHAPE;
  return from_hip(aaac::launch_dequant(codes, scales, sel_bits, sel_stride, tables_bf16, N, K, group_size,
                                       sel_size, fmt, W_hat, ldo, static_cast<hipStream_t>(hip_stream)));
}

int aaac_gemv_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                    const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16, int64_t N,
                    int64_t K, int group_size, int sel_size, aaac_format_t fmt, float* y, int64_t ldy,
                    void* hip_stream) {
  return w4a16_entry(false, x, M, ldx, codes, scales, sel_bits, sel_stride, tables_bf16, N, K, group_size, sel_size,
                     fmt, y, ldy, nullptr, 0, hip_stream);
}

size_t aaac_gemm_w4a16_workspace(int64_t M, int64_t K) { return aaac::gemm_w4a16_workspace(M, K); }

int aaac_gemm_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                    const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16, int64_t N,
                    int64_t K, int group_size, int sel_size, aaac_format_t fmt, float* y, int64_t ldy, void* ws,
                    size_t ws_bytes, void* hip_stream) {
  return w4a16_entry(true, x, M, ldx, codes, scales, sel_bits, sel_stride, tables_bf16, N, K, group_size, sel_size,
                     fmt, y, ldy, ws, ws_bytes, hip_stream);
}

}  // extern "C"

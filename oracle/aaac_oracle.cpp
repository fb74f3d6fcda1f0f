// CPU oracle for the AAAC per-layer activation-weighted k-means.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
// single-threaded C++ restatement of the paper's Algorithm 1 (with
// caller-supplied initial tables; one or both loops; selection groups equal to
// or smaller than the scale groups) and of the equations it cites, written so that a reader can check each function against the paper
// by eye.  It shares no code, header, table or helper with the HIP library and
// must only ever be called from tests, from the smoke check and from the
// benchmark's cpu_baseline leg.
//
// Arithmetic contract (the reading of every point the paper leaves open):
//   * weights and activations arrive as bf16 bit patterns and are widened to
//     fp32 exactly;
//   * every fp32 operation below is a single IEEE-754 round-to-nearest-even
//     operation, no fused multiply-add, denormals kept (build with
//     -ffp-contract=off and without fast-math);
//   * long sums (importance, the 32 bin sums, the objective) are Neumaier-
//     compensated in long double and rounded once.
//
// Parity pins: every function here is pinned by tests/test_oracle_*.py
// (closed forms, brute force, exact rational centroids, hand-derived vectors,
// library bf16/fp8 conversions, textbook 1-D Lloyd; for the quantile
// initialisation a library quantile routine and exact rational interpolation;
// for the selection bit array a hand-worked vector and brute-force errors of the
// small groups; for the W4A16 products a matmul of weights rebuilt with library
// conversions, unit vectors and a hand-worked product).  The method as a whole has
// no printed intermediate values in the paper to compare with: whole-method
// results against the paper's tables are "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

enum { FMT_NVFP4 = 0, FMT_INT4 = 1 };

// ----------------------------------------------------------------- formats

float bf16_to_f32(uint16_t h) {
  uint32_t u = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// Round an fp32 value to the nearest bf16 (ties to even), by comparing the two
// neighbouring bf16 values explicitly.
uint16_t f32_to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if (std::isnan(f)) return static_cast<uint16_t>((u >> 16) | 0x0040u);
  uint16_t lo = static_cast<uint16_t>(u >> 16);  // truncation toward zero
  if ((u & 0xFFFFu) == 0) return lo;             // already representable
  uint16_t hi = static_cast<uint16_t>(lo + 1);   // next bf16 away from zero
  double x = std::fabs(static_cast<double>(f));
  double a = std::fabs(static_cast<double>(bf16_to_f32(lo)));
  double b = ((hi & 0x7FFFu) == 0x7F80u) ? std::ldexp(1.0, 128)  // past the largest finite
                                         : std::fabs(static_cast<double>(bf16_to_f32(hi)));
  double da = x - a, db = b - x;
  if (da < db) return lo;
  if (db < da) return hi;
  return (lo & 1u) ? hi : lo;
}

// Value of a non-negative OCP FP8 E4M3 code (1 sign, 4 exponent bits with
// bias 7, 3 mantissa bits; no infinities; 0x7F is NaN; largest finite 448).
float e4m3_to_f32(uint8_t code) {
  int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
  float v;
  if (e == 15 && m == 7)
    v = NAN;
  else if (e == 0)
    v = std::ldexp(static_cast<float>(m), -9);
  else
    v = std::ldexp(1.0f + static_cast<float>(m) / 8.0f, e - 7);
  return sign ? -v : v;
}

// Nearest finite E4M3 code of |q|, ties to the even code, saturating at 448;
// the sign of q is carried over.  Done by searching the 127 finite magnitudes.
uint8_t f32_to_e4m3(float q) {
  uint8_t sign = std::signbit(q) ? 0x80 : 0x00;
  double x = std::fabs(static_cast<double>(q));
  if (std::isnan(q)) return sign | 0x7F;
  int best = 0x7E;  // 448: anything at or beyond the top saturates
  for (int c = 0; c < 0x7E; ++c) {
    double lo = e4m3_to_f32(static_cast<uint8_t>(c));
    double hi = e4m3_to_f32(static_cast<uint8_t>(c + 1));
    if (x >= lo && x < hi) {
      double dl = x - lo, dh = hi - x;
      if (dl < dh) best = c;
      else if (dh < dl) best = c + 1;
      else best = (c & 1) ? c + 1 : c;
      break;
    }
  }
  return sign | static_cast<uint8_t>(best);
}

// ------------------------------------------------------ compensated summing

struct Sum {  // Neumaier's compensated sum in long double
  long double s = 0.0L, c = 0.0L;
  void add(long double x) {
    long double t = s + x;
    if (std::fabs(s) >= std::fabs(x)) c += (s - t) + x;
    else c += (x - t) + s;
    s = t;
  }
  long double value() const { return s + c; }
};

// ------------------------------------------------------------ method steps

// Importance of column k: I_k = sum_t X[t,k]^2  (paper Eq. "importance").
void act_stats(const uint16_t* X, int64_t tokens, int64_t K, int64_t ldx, float* I) {
  for (int64_t k = 0; k < K; ++k) {
    Sum acc;
    for (int64_t t = 0; t < tokens; ++t) {
      float x = bf16_to_f32(X[t * ldx + k]);
      acc.add(static_cast<long double>(x) * static_cast<long double>(x));
    }
    I[k] = static_cast<float>(static_cast<double>(acc.value()));
  }
}

// Scale of one group (Alg. 1 step "compute scales"; constants from the two
// benchmark settings): NVFP4 stores E4M3(absmax/6), INT4 stores bf16(absmax/7);
// a scale that would be zero is replaced by the smallest positive value so that
// the scale stays strictly positive and its sign bit stays free.
// Returns the unsigned stored code; *s receives its fp32 value.
uint16_t group_scale(const uint16_t* w, int g, int fmt, float* s) {
  float a = 0.0f;
  for (int p = 0; p < g; ++p) a = std::max(a, std::fabs(bf16_to_f32(w[p])));
  if (fmt == FMT_NVFP4) {
    float q = a / 6.0f;
    uint8_t c = f32_to_e4m3(q);
    if (c == 0) c = 0x01;
    *s = e4m3_to_f32(c);
    return c;
  }
  float q = a / 7.0f;
  uint16_t c = f32_to_bf16(q);
  if (c < 0x0080) c = 0x0080;  // below the smallest normal (2^-126): clamp
  *s = bf16_to_f32(c);
  return c;
}

// Normalised weight w~ = w / s, taken as one multiplication by the group's
// reciprocal r = fl32(1/s) (Alg. 1 step "normalise").
float normalise(uint16_t w, float r) { return bf16_to_f32(w) * r; }

// Index of the nearest entry of an ascending 16-entry table
// (Eq. "nearest_recon"): the number of midpoints m_i = (T[i]+T[i+1])/2 that the
// value strictly exceeds, so an exact tie goes to the lower entry.
int nearest_index(float x, const float* T) {
  int idx = 0;
  for (int i = 0; i < 15; ++i) {
    float m = 0.5f * (T[i] + T[i + 1]);
    if (x > m) ++idx;
  }
  return idx;
}

// Sum of u[0..n) as a balanced tree of adjacent pairs in fp32 (n a power of 2).
float pair_tree_sum(float* u, int n) {
  for (int width = n; width > 1; width /= 2)
    for (int i = 0; i < width / 2; ++i) u[i] = u[2 * i] + u[2 * i + 1];
  return u[0];
}

// Activation-weighted error of one group under one table (the summand of
// Eq. "selection"); idx[p] receives each weight's nearest-entry index.
float group_error(const float* wn, const float* I, int g, const float* T, int* idx) {
  float u[128];
  for (int p = 0; p < g; ++p) {
    idx[p] = nearest_index(wn[p], T);
    float d = wn[p] - T[idx[p]];
    float q = d * d;
    u[p] = I[p] * q;
  }
  return pair_tree_sum(u, g);
}

bool valid_shape(int64_t N, int64_t K, int64_t ld, int g) {
  if (N < 0 || K < 0 || ld < K) return false;
  if (g != 16 && g != 32 && g != 64 && g != 128) return false;
  return K % g == 0;
}

void sort_table(float* T) { std::stable_sort(T, T + 16); }

}  // namespace

extern "C" {

float oracle_bf16_to_f32(uint16_t h) { return bf16_to_f32(h); }
uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16(f); }
float oracle_e4m3_to_f32(uint8_t c) { return e4m3_to_f32(c); }
uint8_t oracle_f32_to_e4m3(float f) { return f32_to_e4m3(f); }
int oracle_nearest_index(float x, const float* table16) { return nearest_index(x, table16); }

void oracle_act_stats(const uint16_t* X, int64_t tokens, int64_t K, int64_t ldx, float* importance) {
  act_stats(X, tokens, K, ldx, importance);
}

// Unsigned scale codes (u8 for NVFP4, u16 for INT4), their fp32 values and the
// normalised weights of a whole layer; any output pointer may be null.
int oracle_normalise(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int fmt,
                     void* scale_codes, float* scale_values, float* wn) {
  if (!valid_shape(N, K, ldw, g) || (fmt != FMT_NVFP4 && fmt != FMT_INT4)) return -1;
  int64_t G = K / g;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t j = 0; j < G; ++j) {
      float s;
      uint16_t c = group_scale(W + n * ldw + j * g, g, fmt, &s);
      if (scale_codes) {
        if (fmt == FMT_NVFP4) static_cast<uint8_t*>(scale_codes)[n * G + j] = static_cast<uint8_t>(c);
        else static_cast<uint16_t*>(scale_codes)[n * G + j] = c;
      }
      if (scale_values) scale_values[n * G + j] = s;
      if (wn) {
        float r = 1.0f / s;
        for (int p = 0; p < g; ++p) wn[n * K + j * g + p] = normalise(W[n * ldw + j * g + p], r);
      }
    }
  return 0;
}

// One assignment step over normalised weights wn [N x K] (Eq. "selection"):
// per group e0, e1 and sigma = 1 iff e1 < e0; per weight the index under each
// table.  Output pointers may be null.  Returns the objective
// sum_groups min(e0, e1) through *objective.
int oracle_assign(const float* wn, int64_t N, int64_t K, int g, const float* importance,
                  const float* tables /*32*/, float* e0_out, float* e1_out, uint8_t* sigma_out,
                  uint8_t* idx0_out, uint8_t* idx1_out, double* objective) {
  if (!valid_shape(N, K, K, g)) return -1;
  int64_t G = K / g;
  Sum J;
  int i0[128], i1[128];
  for (int64_t n = 0; n < N; ++n)
    for (int64_t j = 0; j < G; ++j) {
      const float* x = wn + n * K + j * g;
      const float* I = importance + j * g;
      float e0 = group_error(x, I, g, tables, i0);
      float e1 = group_error(x, I, g, tables + 16, i1);
      uint8_t sigma = (e1 < e0) ? 1 : 0;
      if (e0_out) e0_out[n * G + j] = e0;
      if (e1_out) e1_out[n * G + j] = e1;
      if (sigma_out) sigma_out[n * G + j] = sigma;
      for (int p = 0; p < g; ++p) {
        if (idx0_out) idx0_out[n * K + j * g + p] = static_cast<uint8_t>(i0[p]);
        if (idx1_out) idx1_out[n * K + j * g + p] = static_cast<uint8_t>(i1[p]);
      }
      J.add(sigma ? e1 : e0);
    }
  if (objective) *objective = static_cast<double>(J.value());
  return 0;
}

// One Lloyd iteration (assignment step, then one weighted-centroid update of
// every table entry, Eq. "kmeans_update"; Alg. 1 loop body with n_inner = 1).
// tables[32] is updated in place.  sums_out (optional, 64 doubles) receives
// Swx[32] then Sw[32].
int oracle_lloyd_iteration(const float* wn, int64_t N, int64_t K, int g, const float* importance,
                           float* tables, double* sums_out, double* objective) {
  if (!valid_shape(N, K, K, g)) return -1;
  int64_t G = K / g;
  Sum Swx[32], Sw[32], J;
  int i0[128], i1[128];
  for (int64_t n = 0; n < N; ++n)
    for (int64_t j = 0; j < G; ++j) {
      const float* x = wn + n * K + j * g;
      const float* I = importance + j * g;
      float e0 = group_error(x, I, g, tables, i0);
      float e1 = group_error(x, I, g, tables + 16, i1);
      int sigma = (e1 < e0) ? 1 : 0;
      J.add(sigma ? e1 : e0);
      const int* idx = sigma ? i1 : i0;
      for (int p = 0; p < g; ++p) {
        int b = 16 * sigma + idx[p];
        Swx[b].add(static_cast<long double>(I[p]) * static_cast<long double>(x[p]));
        Sw[b].add(static_cast<long double>(I[p]));
      }
    }
  for (int b = 0; b < 32; ++b) {
    double num = static_cast<double>(Swx[b].value());
    double den = static_cast<double>(Sw[b].value());
    if (sums_out) { sums_out[b] = num; sums_out[32 + b] = den; }
    if (den > 0.0) tables[b] = static_cast<float>(num / den);  // empty cell: keep
  }
  sort_table(tables);
  sort_table(tables + 16);
  if (objective) *objective = static_cast<double>(J.value());
  return 0;
}

// Algorithm 1 from the scale step to the end of the outer loop, with caller-
// supplied initial tables (init_grid: T0[16] then T1[16], each ascending).
// tables_trace (optional) receives the 32 entries after every iteration.
int oracle_fit(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int fmt,
               const float* importance, const float* init_grid, int iterations,
               float* tables_f32, uint16_t* tables_bf16, double* objective_trace,
               float* tables_trace) {
  if (!valid_shape(N, K, ldw, g) || iterations < 0) return -1;
  std::vector<float> wn(static_cast<size_t>(N) * K);
  int rc = oracle_normalise(W, N, K, ldw, g, fmt, nullptr, nullptr, wn.data());
  if (rc) return rc;
  float T[32];
  std::memcpy(T, init_grid, sizeof(T));
  for (int t = 0; t < iterations; ++t) {
    double J;
    oracle_lloyd_iteration(wn.data(), N, K, g, importance, T, nullptr, &J);
    if (objective_trace) objective_trace[t] = J;
    if (tables_trace) std::memcpy(tables_trace + 32 * t, T, sizeof(T));
  }
  if (tables_f32) std::memcpy(tables_f32, T, sizeof(T));
  if (tables_bf16)
    for (int b = 0; b < 32; ++b) tables_bf16[b] = f32_to_bf16(T[b]);
  return 0;
}

// One step of the inner k-means of Alg. 1 with the table choice frozen: every
// weight of a group with sigma = r goes to the Voronoi cell of its nearest entry
// of T_r, and each entry moves to the importance-weighted centroid of its cell
// (empty cell: keep).  The tables are sorted afterwards; cells are ordered
// intervals, so this only matters among equal entries.  sigma: [N x K/g].
int oracle_kmeans_step(const float* wn, int64_t N, int64_t K, int g, const float* importance,
                       const uint8_t* sigma, float* tables) {
  if (!valid_shape(N, K, K, g)) return -1;
  int64_t G = K / g;
  Sum Swx[32], Sw[32];
  for (int64_t n = 0; n < N; ++n)
    for (int64_t j = 0; j < G; ++j) {
      int r = sigma[n * G + j] ? 1 : 0;
      for (int p = 0; p < g; ++p) {
        float x = wn[n * K + j * g + p];
        float I = importance[j * g + p];
        int b = 16 * r + nearest_index(x, tables + 16 * r);
        Swx[b].add(static_cast<long double>(I) * static_cast<long double>(x));
        Sw[b].add(static_cast<long double>(I));
      }
    }
  for (int b = 0; b < 32; ++b) {
    double num = static_cast<double>(Swx[b].value());
    double den = static_cast<double>(Sw[b].value());
    if (den > 0.0) tables[b] = static_cast<float>(num / den);
  }
  sort_table(tables);
  sort_table(tables + 16);
  return 0;
}

// Algorithm 1 with both loops: n_outer assignment steps, each followed by
// n_inner k-means steps on the groups it assigned to each table.
// objective_trace: [n_outer], the objective seen by each assignment step.
// tables_trace (optional): the 32 entries after every k-means step,
// [n_outer * n_inner][32].
int oracle_fit_nested(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int fmt,
                      const float* importance, const float* init_grid, int n_outer, int n_inner,
                      float* tables_f32, uint16_t* tables_bf16, double* objective_trace,
                      float* tables_trace) {
  if (!valid_shape(N, K, ldw, g) || n_outer < 0 || n_inner < 1) return -1;
  std::vector<float> wn(static_cast<size_t>(N) * K);
  int rc = oracle_normalise(W, N, K, ldw, g, fmt, nullptr, nullptr, wn.data());
  if (rc) return rc;
  std::vector<uint8_t> sigma(static_cast<size_t>(N) * (K / g));
  float T[32];
  std::memcpy(T, init_grid, sizeof(T));
  for (int t = 0; t < n_outer; ++t) {
    double J;
    oracle_assign(wn.data(), N, K, g, importance, T, nullptr, nullptr, sigma.data(), nullptr, nullptr, &J);
    if (objective_trace) objective_trace[t] = J;
    for (int l = 0; l < n_inner; ++l) {
      oracle_kmeans_step(wn.data(), N, K, g, importance, sigma.data(), T);
      if (tables_trace) std::memcpy(tables_trace + 32 * (t * n_inner + l), T, sizeof(T));
    }
  }
  if (tables_f32) std::memcpy(tables_f32, T, sizeof(T));
  if (tables_bf16)
    for (int b = 0; b < 32; ++b) tables_bf16[b] = f32_to_bf16(T[b]);
  return 0;
}

// Final steps of Alg. 1: with the bf16 tables (each still ascending, because
// rounding is monotone; it can only create ties), recompute sigma per group,
// write 4-bit nearest-entry indices into the selected table (even k in the low
// nibble) and put sigma into the sign bit of the stored scale.
int oracle_encode(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int fmt,
                  const float* importance, const uint16_t* tables_bf16, uint8_t* codes,
                  void* scales) {
  if (!valid_shape(N, K, ldw, g)) return -1;
  float T[32];
  for (int b = 0; b < 32; ++b) T[b] = bf16_to_f32(tables_bf16[b]);
  int64_t G = K / g;
  float x[128];
  int i0[128], i1[128];
  for (int64_t n = 0; n < N; ++n)
    for (int64_t j = 0; j < G; ++j) {
      const uint16_t* w = W + n * ldw + j * g;
      float s;
      uint16_t sc = group_scale(w, g, fmt, &s);
      float r = 1.0f / s;
      for (int p = 0; p < g; ++p) x[p] = normalise(w[p], r);
      float e0 = group_error(x, importance + j * g, g, T, i0);
      float e1 = group_error(x, importance + j * g, g, T + 16, i1);
      int sigma = (e1 < e0) ? 1 : 0;
      const int* idx = sigma ? i1 : i0;
      for (int p = 0; p < g; p += 2)
        codes[(n * K + j * g + p) / 2] = static_cast<uint8_t>(idx[p] | (idx[p + 1] << 4));
      if (fmt == FMT_NVFP4)
        static_cast<uint8_t*>(scales)[n * G + j] = static_cast<uint8_t>(sc | (sigma << 7));
      else
        static_cast<uint16_t*>(scales)[n * G + j] = static_cast<uint16_t>(sc | (sigma << 15));
    }
  return 0;
}

// Dequantisation (Eq. "aaac_dequant"): w^ = T_sigma[code] * s, rounded to bf16.
int oracle_dequant(const uint8_t* codes, const void* scales, const uint16_t* tables_bf16,
                   int64_t N, int64_t K, int g, int fmt, uint16_t* W_hat, int64_t ldo) {
  if (!valid_shape(N, K, ldo, g)) return -1;
  int64_t G = K / g;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) {
      int64_t j = k / g;
      int sigma;
      float s;
      if (fmt == FMT_NVFP4) {
        uint8_t c = static_cast<const uint8_t*>(scales)[n * G + j];
        sigma = c >> 7;
        s = e4m3_to_f32(c & 0x7F);
      } else {
        uint16_t c = static_cast<const uint16_t*>(scales)[n * G + j];
        sigma = c >> 15;
        s = bf16_to_f32(c & 0x7FFF);
      }
      uint8_t byte = codes[(n * K + k) / 2];
      int code = (k & 1) ? (byte >> 4) : (byte & 15);
      float t = bf16_to_f32(tables_bf16[16 * sigma + code]);
      W_hat[n * ldo + k] = f32_to_bf16(t * s);
    }
  return 0;
}

// ---------------------------------------------------------------------------
// Selection groups smaller than scale groups (S < g): every g weights share a
// scale, every S weights share a table choice (S divides g).  The assignment and
// k-means steps above act on normalised weights and only know the selection
// group, so the learning loop is the same with S in place of g after normalising
// with g.  With S == g this is oracle_fit_nested.
int oracle_fit_sel(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int S, int fmt,
                   const float* importance, const float* init_grid, int n_outer, int n_inner,
                   float* tables_f32, uint16_t* tables_bf16, double* objective_trace,
                   float* tables_trace) {
  if (!valid_shape(N, K, ldw, g) || !valid_shape(N, K, ldw, S) || S > g) return -1;
  if (n_outer < 0 || n_inner < 1) return -1;
  std::vector<float> wn(static_cast<size_t>(N) * K);
  int rc = oracle_normalise(W, N, K, ldw, g, fmt, nullptr, nullptr, wn.data());
  if (rc) return rc;
  std::vector<uint8_t> sigma(static_cast<size_t>(N) * (K / S));
  float T[32];
  std::memcpy(T, init_grid, sizeof(T));
  for (int t = 0; t < n_outer; ++t) {
    double J;
    oracle_assign(wn.data(), N, K, S, importance, T, nullptr, nullptr, sigma.data(), nullptr, nullptr, &J);
    if (objective_trace) objective_trace[t] = J;
    for (int l = 0; l < n_inner; ++l) {
      oracle_kmeans_step(wn.data(), N, K, S, importance, sigma.data(), T);
      if (tables_trace) std::memcpy(tables_trace + 32 * (t * n_inner + l), T, sizeof(T));
    }
  }
  if (tables_f32) std::memcpy(tables_f32, T, sizeof(T));
  if (tables_bf16)
    for (int b = 0; b < 32; ++b) tables_bf16[b] = f32_to_bf16(T[b]);
  return 0;
}

// Final steps of Alg. 1 for S <= g.  With S == g sigma goes into the sign bit of
// the stored scale and sel_bits is not touched.  With S < g the scales stay
// unsigned and sigma is stored separately, one bit per selection group: group j
// of row n is bit (j mod 8) of byte n * sel_stride + j / 8, where
// sel_stride >= ceil(K / S / 8); padding bits of a row's last byte are zero.
int oracle_encode_sel(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int S, int fmt,
                      const float* importance, const uint16_t* tables_bf16, uint8_t* codes,
                      void* scales, uint8_t* sel_bits, int64_t sel_stride) {
  if (!valid_shape(N, K, ldw, g) || !valid_shape(N, K, ldw, S) || S > g) return -1;
  if (S < g && (!sel_bits || sel_stride < (K / S + 7) / 8)) return -1;
  float T[32];
  for (int b = 0; b < 32; ++b) T[b] = bf16_to_f32(tables_bf16[b]);
  int64_t G = K / g;
  float x[128];
  int i0[128], i1[128];
  for (int64_t n = 0; n < N; ++n) {
    if (S < g) std::memset(sel_bits + n * sel_stride, 0, static_cast<size_t>((K / S + 7) / 8));
    for (int64_t j = 0; j < G; ++j) {
      const uint16_t* w = W + n * ldw + j * g;
      float s;
      uint16_t sc = group_scale(w, g, fmt, &s);
      float r = 1.0f / s;
      for (int p = 0; p < g; ++p) x[p] = normalise(w[p], r);
      int first_sigma = 0;
      for (int q = 0; q < g / S; ++q) {  // the selection groups inside this scale group
        float e0 = group_error(x + q * S, importance + j * g + q * S, S, T, i0);
        float e1 = group_error(x + q * S, importance + j * g + q * S, S, T + 16, i1);
        int sigma = (e1 < e0) ? 1 : 0;
        if (q == 0) first_sigma = sigma;
        const int* idx = sigma ? i1 : i0;
        for (int p = 0; p < S; p += 2)
          codes[(n * K + j * g + q * S + p) / 2] = static_cast<uint8_t>(idx[p] | (idx[p + 1] << 4));
        if (S < g) {
          int64_t sel = (j * g + q * S) / S;
          sel_bits[n * sel_stride + sel / 8] |= static_cast<uint8_t>(sigma << (sel % 8));
        }
      }
      int sign = (S == g) ? first_sigma : 0;
      if (fmt == FMT_NVFP4)
        static_cast<uint8_t*>(scales)[n * G + j] = static_cast<uint8_t>(sc | (sign << 7));
      else
        static_cast<uint16_t*>(scales)[n * G + j] = static_cast<uint16_t>(sc | (sign << 15));
    }
  }
  return 0;
}

// Dequantisation for S <= g: sigma from the scale's sign bit (S == g) or from the
// separate bits (S < g, layout as in oracle_encode_sel).
int oracle_dequant_sel(const uint8_t* codes, const void* scales, const uint8_t* sel_bits,
                       int64_t sel_stride, const uint16_t* tables_bf16, int64_t N, int64_t K, int g,
                       int S, int fmt, uint16_t* W_hat, int64_t ldo) {
  if (!valid_shape(N, K, ldo, g) || !valid_shape(N, K, ldo, S) || S > g) return -1;
  if (S < g && !sel_bits) return -1;
  int64_t G = K / g;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) {
      int64_t j = k / g;
      int sign;
      float s;
      if (fmt == FMT_NVFP4) {
        uint8_t c = static_cast<const uint8_t*>(scales)[n * G + j];
        sign = c >> 7;
        s = e4m3_to_f32(c & 0x7F);
      } else {
        uint16_t c = static_cast<const uint16_t*>(scales)[n * G + j];
        sign = c >> 15;
        s = bf16_to_f32(c & 0x7FFF);
      }
      int sigma = sign;
      if (S < g) {
        int64_t sel = k / S;
        sigma = (sel_bits[n * sel_stride + sel / 8] >> (sel % 8)) & 1;
      }
      uint8_t byte = codes[(n * K + k) / 2];
      int code = (k & 1) ? (byte >> 4) : (byte & 15);
      float t = bf16_to_f32(tables_bf16[16 * sigma + code]);
      W_hat[n * ldo + k] = f32_to_bf16(t * s);
    }
  return 0;
}

// ---------------------------------------------------------------------------
// Quantile initialisation (Eq. "init_t0", Eq. "init_t1"; Alg. 1 steps 4-5) with
// M = 16 entries per table: T0[i] = Quantile_{i/15}, T1[i] = Quantile_{d + (1-d) i/15},
// d = 1/30, of all N*K normalised weights of the layer.
//
// Quantile convention (the paper names none): linear interpolation between order
// statistics, position q * (n - 1) counted from 0 in the ascending sequence
// x_(0) <= ... <= x_(n-1).  The quantile levels are rationals, q = num/den with
// (num, den) = (i, 15) for T0 and (15 + 29 i, 450) for T1, so the position is
// split exactly in integers: lo = num*(n-1) div den, rem = num*(n-1) mod den, and
//   value = fl32( x_(lo) + (rem/den) * (x_(lo+1) - x_(lo)) )  evaluated in fp64
// (x_(lo+1) is not read when rem == 0).  A zero result is stored as +0 whatever
// the sign of the zero weight it came from (the order of -0 and +0 in the sorted
// sequence is not defined by their values).
int oracle_quantile_init(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int g, int fmt,
                         float* grid32) {
  if (!valid_shape(N, K, ldw, g) || N == 0 || K == 0) return -1;
  std::vector<float> x(static_cast<size_t>(N) * K);
  int rc = oracle_normalise(W, N, K, ldw, g, fmt, nullptr, nullptr, x.data());
  if (rc) return rc;
  std::sort(x.begin(), x.end());
  const unsigned __int128 last = static_cast<unsigned __int128>(x.size() - 1);
  for (int t = 0; t < 2; ++t)
    for (int i = 0; i < 16; ++i) {
      unsigned __int128 num = (t == 0) ? i : 15 + 29 * i;
      unsigned __int128 den = (t == 0) ? 15 : 450;
      unsigned __int128 pos = num * last;
      size_t lo = static_cast<size_t>(pos / den);
      double rem = static_cast<double>(static_cast<uint64_t>(pos % den));
      double v = static_cast<double>(x[lo]);
      if (rem != 0.0) {
        double frac = rem / static_cast<double>(static_cast<uint64_t>(den));
        v = v + frac * (static_cast<double>(x[lo + 1]) - v);
      }
      grid32[16 * t + i] = static_cast<float>(v) + 0.0f;  // -0 becomes +0
    }
  return 0;
}

// ---------------------------------------------------------------------------
// The quantised layer applied to activations (W4A16: 4-bit weights, 16-bit
// activations): y[m, n] = sum_k x[m, k] * w^[n, k] with the dequantised weight
// of Eq. "aaac_dequant", w^ = T_sigma[code] * s, taken as the real product (a
// fused kernel never stores w^, so there is no bf16 rounding of it).  x, the
// table entries and the scale carry 8 significant bits each, so every term is
// exact in fp64; the sum is compensated and rounded once to fp32.
// abs_sum (optional, [M x N]) receives sum_k |x * w^|, the quantity a
// floating-point summation error bound is stated against.
// sel_bits / S as in oracle_dequant_sel.
static int w4a16_product(bool round_weights, const uint16_t* x, int64_t M, int64_t ldx, const uint8_t* codes,
                         const void* scales, const uint8_t* sel_bits, int64_t sel_stride,
                         const uint16_t* tables_bf16, int64_t N, int64_t K, int g, int S, int fmt, float* y,
                         double* abs_sum) {
  if (!valid_shape(N, K, K, g) || !valid_shape(N, K, K, S) || S > g || M < 0 || ldx < K) return -1;
  if (S < g && !sel_bits) return -1;
  int64_t G = K / g;
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      Sum acc, mag;
      for (int64_t k = 0; k < K; ++k) {
        int64_t j = k / g;
        int sigma;
        float s;
        if (fmt == FMT_NVFP4) {
          uint8_t c = static_cast<const uint8_t*>(scales)[n * G + j];
          sigma = c >> 7;
          s = e4m3_to_f32(c & 0x7F);
        } else {
          uint16_t c = static_cast<const uint16_t*>(scales)[n * G + j];
          sigma = c >> 15;
          s = bf16_to_f32(c & 0x7FFF);
        }
        if (S < g) {
          int64_t sel = k / S;
          sigma = (sel_bits[n * sel_stride + sel / 8] >> (sel % 8)) & 1;
        }
        uint8_t byte = codes[(n * K + k) / 2];
        int code = (k & 1) ? (byte >> 4) : (byte & 15);
        float w = bf16_to_f32(tables_bf16[16 * sigma + code]) * s;  // exact: 8 x 8 significant bits
        if (round_weights) w = bf16_to_f32(f32_to_bf16(w));
        long double t = static_cast<long double>(w) * static_cast<long double>(bf16_to_f32(x[m * ldx + k]));
        acc.add(t);
        mag.add(std::fabs(t));
      }
      y[m * N + n] = static_cast<float>(static_cast<double>(acc.value()));
      if (abs_sum) abs_sum[m * N + n] = static_cast<double>(mag.value());
    }
  return 0;
}

int oracle_gemv_w4a16(const uint16_t* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                      const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                      int64_t N, int64_t K, int g, int S, int fmt, float* y, double* abs_sum) {
  return w4a16_product(false, x, M, ldx, codes, scales, sel_bits, sel_stride, tables_bf16, N, K, g, S, fmt, y,
                       abs_sum);
}

// The same product with the dequantised weights rounded to bf16 first, w^ =
// bf16(T_sigma[code] * s), i.e. exactly the weights oracle_dequant_sel returns:
// what a matrix-core kernel with bf16 operands computes.
int oracle_gemm_w4a16(const uint16_t* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                      const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                      int64_t N, int64_t K, int g, int S, int fmt, float* y, double* abs_sum) {
  return w4a16_product(true, x, M, ldx, codes, scales, sel_bits, sel_stride, tables_bf16, N, K, g, S, fmt, y,
                       abs_sum);
}

}  // extern "C"

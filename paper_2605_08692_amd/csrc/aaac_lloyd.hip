// The fused Lloyd iteration (assignment step + accumulation of the table
// update) for gfx950, and the launcher of a whole fit.
//
// Work mapping: a wavefront owns a strip of 512 columns (64 lanes x 8 bf16) and
// a range of rows; a lane keeps the importances of its 8 columns in registers.
// A group of g weights is held by g/8 adjacent lanes.
//
// Nearest-entry search.  The index of a normalised weight x in an ascending
// table is the number of midpoints strictly below x.  Instead of 15 compares
// per table, the block builds (once per launch, in LDS) a bucket table over the
// range of the midpoints: bucket(x) is a monotone function of x computed with
// one fused multiply-add and a clamp, and for every bucket and table it stores
// i = number of midpoints whose bucket is lower.  If at most one midpoint falls
// into the bucket itself, that midpoint is m[i], and index = i + (x > m[i]) with
// reconstruction T[i] or T[i+1]: one compare.  A bucket holding two or more
// midpoints of a table points at a poisoned row (NaN entries); the NaN reaches
// the lane's error sum, the wavefront notices and redoes that row with the
// plain 15-compare count.  Results are identical either way.
//
// The bucket table is replicated 32 times (one copy per LDS bank column) so
// that data-dependent look-ups never conflict; the 16-entry midpoint and entry
// arrays need no replication because their entries already sit in distinct
// banks.
//
// Table update.  sum I*x and sum I of the 32 bins go through fp64 LDS atomics
// into a block-wide histogram with 32 slots per bin (slot = lane mod 32) and are
// reduced per block into a record in global memory.  There is no grid-wide
// synchronisation inside a launch: the kernel of iteration t+1 starts by
// reducing the records of iteration t (every block does so, in the same fixed
// order, so all blocks hold bit-identical tables), divides, keeps entries whose
// cell was empty and sorts.  Records and tables are double-buffered by iteration
// parity, so a block that is still reading the previous records never races with
// one that already writes new ones.
#include "aaac_device.h"
#include "aaac_internal.h"

namespace aaac {

namespace {

constexpr int kLloydBlock = 1024;
constexpr int kLloydWaves = kLloydBlock / kWave;
constexpr int kBuckets = 256;
constexpr int kReplicas = 32;
constexpr int kSlots = 32;
constexpr int kPoison = 16;  // row of the stage-2 arrays that holds NaN entries

struct LloydLds {
  uint32_t lut[kBuckets * kReplicas];  // (4*i0) | (4*i1) << 16, replicated
  double hist[2][32][kSlots];          // [0] = sum I*x, [1] = sum I
  float thr[2][20];                    // midpoints m[0..14], +inf at 15 and at the poison row
  float tab[2][20];                    // entries T[0..15], NaN at 16 and 17
  float lutpar[4];                     // inv, off for bucket()
  uint32_t entry[kBuckets];            // unreplicated bucket entries while building
  double red[kLloydWaves][72];
  double sums[72];
  float newtab[32];
};

// Monotone map from a normalised weight to the byte offset of its bucket row
// (bucket * 128): integer part of fma(x, inv, off) read from the mantissa of a
// float in [2^23, 2^24), clamped.
__device__ __forceinline__ uint32_t bucket_row(float x, float inv, float off) {
  float t = __builtin_fmaf(x, inv, off);
  t = __builtin_amdgcn_fmed3f(t, 8388608.0f, 8388608.0f + 32767.0f);
  return __float_as_uint(t) & 0x7F80u;
}

__device__ __forceinline__ float lds_f32(const void* base, uint32_t byte_off) {
  return *reinterpret_cast<const float*>(static_cast<const char*>(base) + byte_off);
}

__device__ __forceinline__ int count_above15(float x, const float* m) {
  int idx = 0;
#pragma unroll
  for (int i = 0; i < 15; ++i) idx += (x > m[i]) ? 1 : 0;
  return idx;
}

__device__ __forceinline__ float tree8(const float (&u)[8]) {
  return ((u[0] + u[1]) + (u[2] + u[3])) + ((u[4] + u[5]) + (u[6] + u[7]));
}

// Per-lane result of the assignment of 8 weights: byte offset (4*index) of the
// chosen entry in each table, and the lane's partial error sums.
struct Lane8 {
  float wn[8];
  uint32_t k0[8], k1[8];  // 4 * index under T0 / T1
  float p0, p1;
};

__device__ __forceinline__ void assign_fast(const W8& x, float r, const float (&Iv)[8], const LloydLds& sm,
                                            float inv, float off, uint32_t rep4, Lane8& a) {
  float u0[8], u1[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = x.w[p] * r;
    a.wn[p] = wn;
    const uint32_t e = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(sm.lut) +
                                                          (bucket_row(wn, inv, off) | rep4));
    const uint32_t a0 = e & 0xFFFFu, a1 = e >> 16;
    const bool c0 = wn > lds_f32(sm.thr[0], a0);
    const bool c1 = wn > lds_f32(sm.thr[1], a1);
    const float lo0 = lds_f32(sm.tab[0], a0), hi0 = lds_f32(sm.tab[0], a0 + 4);
    const float lo1 = lds_f32(sm.tab[1], a1), hi1 = lds_f32(sm.tab[1], a1 + 4);
    const float d0 = wn - (c0 ? hi0 : lo0);
    const float d1 = wn - (c1 ? hi1 : lo1);
    a.k0[p] = a0 + (c0 ? 4u : 0u);
    a.k1[p] = a1 + (c1 ? 4u : 0u);
    const float q0 = d0 * d0;
    const float q1 = d1 * d1;
    u0[p] = Iv[p] * q0;
    u1[p] = Iv[p] * q1;
  }
  a.p0 = tree8(u0);
  a.p1 = tree8(u1);
}

// Same result by counting all 15 midpoints (used for rows that met a poisoned bucket).
__device__ __forceinline__ void assign_slow(const float (&Iv)[8], const LloydLds& sm, Lane8& a) {
  float u0[8], u1[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = a.wn[p];
    const int i0 = count_above15(wn, sm.thr[0]);
    const int i1 = count_above15(wn, sm.thr[1]);
    a.k0[p] = 4u * i0;
    a.k1[p] = 4u * i1;
    const float d0 = wn - sm.tab[0][i0];
    const float d1 = wn - sm.tab[1][i1];
    const float q0 = d0 * d0;
    const float q1 = d1 * d1;
    u0[p] = Iv[p] * q0;
    u1[p] = Iv[p] * q1;
  }
  a.p0 = tree8(u0);
  a.p1 = tree8(u1);
}

// Fills thr/tab/lut from the current tables (sm.newtab).  All threads of the block call it.
__device__ void build_search_tables(LloydLds& sm) {
  const int tid = threadIdx.x;
  if (tid < 40) {
    const int r = tid / 20, i = tid % 20;
    const float* T = sm.newtab + 16 * r;
    sm.tab[r][i] = i < 16 ? T[i] : __builtin_nanf("");
    sm.thr[r][i] = i < 15 ? 0.5f * (T[i] + T[i + 1]) : __builtin_inff();
  }
  __syncthreads();
  if (tid == 0) {
    const float lo = fminf(sm.thr[0][0], sm.thr[1][0]);
    const float hi = fmaxf(sm.thr[0][14], sm.thr[1][14]);
    const float range = fmaxf(hi - lo, 1e-20f);
    const float inv = (128.0f * (kBuckets - 2)) / range;  // buckets 1..254 span [lo, hi]
    sm.lutpar[0] = inv;
    sm.lutpar[1] = (128.0f - lo * inv) + 8388608.0f;
  }
  __syncthreads();
  const float inv = sm.lutpar[0], off = sm.lutpar[1];
  if (tid < kBuckets) {
    uint32_t e = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      int below = 0, inside = 0;
      for (int j = 0; j < 15; ++j) {
        const int bj = (int)(bucket_row(sm.thr[r][j], inv, off) >> 7);
        below += bj < tid ? 1 : 0;
        inside += bj == tid ? 1 : 0;
      }
      const uint32_t row = inside <= 1 ? (uint32_t)below : (uint32_t)kPoison;
      e |= (4u * row) << (16 * r);
    }
    sm.entry[tid] = e;
  }
  __syncthreads();
  // replicate: thread -> (replica = tid % 32, buckets tid/32 + 16*k)
  for (int b = tid / kReplicas; b < kBuckets; b += kLloydBlock / kReplicas)
    sm.lut[b * kReplicas + (tid % kReplicas)] = sm.entry[b];
  for (int i = tid; i < 2 * 32 * kSlots; i += kLloydBlock) (&sm.hist[0][0][0])[i] = 0.0;
  __syncthreads();
}

// Table update from the records of one iteration: reduce them in a fixed order,
// divide, keep entries whose cell was empty, sort each table (stable).  The
// result is left in sm.newtab and the objective in sm.sums[64].  All threads of
// the block call it; every block computes the same bits.
__device__ void update_tables(LloydLds& sm, const double* __restrict__ records, int n_records,
                              const float* __restrict__ old_tables) {
  const int tid = threadIdx.x, b = tid & 63, part = tid >> 6;
  double s = 0.0, o = 0.0;
  for (int i = part; i < n_records; i += kLloydWaves) {
    s += records[(int64_t)i * kPartialStride + b];
    if (b == 0) o += records[(int64_t)i * kPartialStride + 64];
  }
  sm.red[part][b] = s;
  if (b == 0) sm.red[part][64] = o;
  __syncthreads();
  if (tid <= 64) {
    double t = 0.0;
#pragma unroll
    for (int p = 0; p < kLloydWaves; ++p) t += sm.red[p][tid];
    sm.sums[tid] = t;
  }
  __syncthreads();
  float* cand = &sm.tab[0][0];  // scratch: 32 candidate entries
  if (tid < 32) {
    const double den = sm.sums[32 + tid];
    cand[tid] = den > 0.0 ? (float)(sm.sums[tid] / den) : old_tables[tid];
  }
  __syncthreads();
  if (tid < 32) {  // stable rank sort inside each table
    const int base = tid & 16, i = tid & 15;
    const float v = cand[tid];
    int rank = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float u = cand[base + j];
      rank += (u < v || (u == v && j < i)) ? 1 : 0;
    }
    sm.newtab[base + rank] = v;
  }
  __syncthreads();
}

template <int LANES>
__global__ __launch_bounds__(kLloydBlock) void lloyd_iter_kernel(
    const uint16_t* __restrict__ W, int64_t N, int64_t K, int64_t ldw, const float* __restrict__ rinv,
    const float* __restrict__ importance, FitState* __restrict__ state, double* __restrict__ records,
    int prev_records, double* __restrict__ objective_trace, int iteration, int strips, int rows_per_unit,
    int64_t units) {
  __shared__ LloydLds sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // tables of this iteration: the initial grid, or the update of the previous ones
  if (iteration == 0) {
    if (tid < 32) sm.newtab[tid] = state->tables[0][tid];
    __syncthreads();
  } else {
    const int prev = (iteration - 1) & 1;
    update_tables(sm, records + (int64_t)prev * prev_records * kPartialStride, prev_records,
                  state->tables[prev]);
    if (blockIdx.x == 0) {
      if (tid < 32) state->tables[iteration & 1][tid] = sm.newtab[tid];
      if (tid == 32 && objective_trace) objective_trace[iteration - 1] = sm.sums[64];
    }
  }
  build_search_tables(sm);
  const float inv = sm.lutpar[0], off = sm.lutpar[1];
  const uint32_t rep4 = (uint32_t)(lane & (kReplicas - 1)) * 4u;
  double* partials = records + (int64_t)(iteration & 1) * gridDim.x * kPartialStride;

  double obj = 0.0;
  const int64_t unit = (int64_t)blockIdx.x * kLloydWaves + wave;
  if (unit < units) {
    const int strip = (int)(unit % strips);
    const int64_t r0 = (unit / strips) * rows_per_unit;
    const int64_t r1 = r0 + rows_per_unit < N ? r0 + rows_per_unit : N;
    const int64_t col = (int64_t)strip * kStripCols + lane * 8;
    const bool active = col < K;
    const int64_t G = K / (8 * LANES);
    const int64_t gidx = col / (8 * LANES);
    float Iv[8];
    double Id[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      Iv[p] = active ? importance[col + p] : 0.0f;
      Id[p] = (double)Iv[p];
    }
    const uint32_t slot8 = (uint32_t)(lane & (kSlots - 1)) * 8u;
    const uint16_t* wp = W + r0 * ldw + (active ? col : 0);
    const float* rp = rinv + r0 * G + (active ? gidx : 0);
    char* hist = reinterpret_cast<char*>(&sm.hist[0][0][0]);
    for (int64_t row = r0; row < r1; ++row, wp += ldw, rp += G) {
      uint4 v = make_uint4(0, 0, 0, 0);
      float r = 0.0f;
      if (active) {
        v = *reinterpret_cast<const uint4*>(wp);
        r = *rp;
      }
      Lane8 a;
      assign_fast(unpack8(v), r, Iv, sm, inv, off, rep4, a);
      if (__any((a.p0 != a.p0) || (a.p1 != a.p1))) assign_slow(Iv, sm, a);
      const float e0 = group_sum<LANES>(a.p0);
      const float e1 = group_sum<LANES>(a.p1);
      const bool sigma = e1 < e0;
      if (active) {
        const uint32_t base = slot8 + (sigma ? 16u * kSlots * 8u : 0u);
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const uint32_t k = sigma ? a.k1[p] : a.k0[p];
          char* h = hist + (k * (kSlots * 2u) + base);  // bin (k/4) * 32 slots * 8 bytes
          atomicAdd(reinterpret_cast<double*>(h), Id[p] * (double)a.wn[p]);
          atomicAdd(reinterpret_cast<double*>(h + sizeof(sm.hist[0])), Id[p]);
        }
        if ((lane % LANES) == 0) obj += (double)(sigma ? e1 : e0);
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) obj += __shfl_down(obj, o);
  if (lane == 0) sm.red[wave][64] = obj;
  __syncthreads();
  double* out = partials + (int64_t)blockIdx.x * kPartialStride;
  if (tid < 64) {
    const double* h = &sm.hist[0][0][0] + tid * kSlots;
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < kSlots; ++k) s += h[k];
    out[tid] = s;
  } else if (tid == 64) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kLloydWaves; ++w) s += sm.red[w][64];
    out[64] = s;
  }
}

__global__ void init_state_kernel(Grid32 grid, FitState* state) {
  if (threadIdx.x < 32) state->tables[0][threadIdx.x] = grid.t[threadIdx.x];
}

// After the last iteration: update the tables from its records and write the outputs.
__global__ __launch_bounds__(kLloydBlock) void final_tables_kernel(
    FitState* __restrict__ state, const double* __restrict__ records, int n_records, int iterations,
    float* __restrict__ tables_f32, uint16_t* __restrict__ tables_bf16, double* __restrict__ objective_trace) {
  __shared__ LloydLds sm;
  const int tid = threadIdx.x;
  if (iterations == 0) {
    if (tid < 32) sm.newtab[tid] = state->tables[0][tid];
  } else {
    const int prev = (iterations - 1) & 1;
    update_tables(sm, records + (int64_t)prev * n_records * kPartialStride, n_records, state->tables[prev]);
    if (tid == 32 && objective_trace) objective_trace[iterations - 1] = sm.sums[64];
  }
  __syncthreads();
  if (tid < 32) {
    const float t = sm.newtab[tid];
    if (tables_f32) tables_f32[tid] = t;
    tables_bf16[tid] = (uint16_t)bf16_rne(t);
  }
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <int LANES>
hipError_t launch_iterations(const uint16_t* W, const FitPlan& p, const float* importance, int iterations,
                             FitState* state, const float* rinv, double* records,
                             double* objective_trace, hipStream_t stream) {
  for (int it = 0; it < iterations; ++it) {
    lloyd_iter_kernel<LANES><<<p.blocks, kLloydBlock, 0, stream>>>(W, p.N, p.K, p.ldw, rinv, importance, state,
                                                                  records, p.blocks, objective_trace, it,
                                                                  p.strips, p.rows_per_unit, p.units);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

FitPlan make_fit_plan(int64_t N, int64_t K, int64_t ldw, int group_size) {
  FitPlan p;
  p.N = N; p.K = K; p.ldw = ldw; p.group_size = group_size;
  p.strips = (int)ceil_div(K > 0 ? K : 1, kStripCols);
  const int64_t rows = N > 0 ? N : 1;
  // about 4096 wavefront units = 256 blocks of 16 wavefronts = one block per CU
  p.rows_per_unit = (int)ceil_div(rows * p.strips, 4096);
  if (p.rows_per_unit < 1) p.rows_per_unit = 1;
  p.units = p.strips * ceil_div(rows, p.rows_per_unit);
  p.blocks = (int)ceil_div(p.units, kLloydWaves);
  auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
  p.off_state = 0;
  p.off_rinv = align(sizeof(FitState));
  p.off_partials = p.off_rinv + align((size_t)(N > 0 ? N : 0) * (K / group_size) * sizeof(float));
  p.bytes = p.off_partials + align((size_t)2 * p.blocks * kPartialStride * sizeof(double));
  return p;
}

hipError_t launch_fit(const void* W, const FitPlan& p, int fmt, const float* importance,
                      const Grid32& grid, int iterations, float* tables_f32, uint16_t* tables_bf16,
                      double* objective_trace, void* ws, hipStream_t stream) {
  char* base = static_cast<char*>(ws);
  FitState* state = reinterpret_cast<FitState*>(base + p.off_state);
  float* rinv = reinterpret_cast<float*>(base + p.off_rinv);
  double* partials = reinterpret_cast<double*>(base + p.off_partials);
  init_state_kernel<<<1, 64, 0, stream>>>(grid, state);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  int done = 0;
  if (p.N > 0 && p.K > 0 && iterations > 0) {
    const uint16_t* Wp = static_cast<const uint16_t*>(W);
    e = launch_group_rinv(W, p.N, p.K, p.ldw, p.group_size, fmt, rinv, stream);
    if (e != hipSuccess) return e;
    switch (p.group_size / 8) {
      case 2: e = launch_iterations<2>(Wp, p, importance, iterations, state, rinv, partials, objective_trace, stream); break;
      case 4: e = launch_iterations<4>(Wp, p, importance, iterations, state, rinv, partials, objective_trace, stream); break;
      case 8: e = launch_iterations<8>(Wp, p, importance, iterations, state, rinv, partials, objective_trace, stream); break;
      default: e = launch_iterations<16>(Wp, p, importance, iterations, state, rinv, partials, objective_trace, stream); break;
    }
    if (e != hipSuccess) return e;
    done = iterations;
  } else if (objective_trace && iterations > 0) {
    e = launch_fill_zero(objective_trace, sizeof(double) * iterations, stream);
    if (e != hipSuccess) return e;
  }
  final_tables_kernel<<<1, kLloydBlock, 0, stream>>>(state, partials, p.blocks, done, tables_f32, tables_bf16,
                                                    objective_trace);
  return hipGetLastError();
}

}  // namespace aaac

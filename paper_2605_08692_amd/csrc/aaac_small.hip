// Codebook learning of a small layer in ONE launch (all passes of Alg. 1's two loops).
//
// A layer of a few hundred thousand weights is two or three weights per lane of the chip: with a
// launch per pass its fit is all launch gaps, prologues and tails.  Here a handful of blocks (at
// most 32, eight wavefronts each, all resident at once) keep their weights and reciprocal scales in
// LDS for the whole fit (a private region per wavefront, so no barrier guards it); per pass a block accumulates its 64 sums and its share of the objective as
// the large-layer kernel does (same search, same fp32 error tree, same fp64 LDS histogram) and the
// blocks then exchange their partial sums through global memory, each block reading every block's
// sums and adding them in block order, so every block derives the same tables, bit for bit, and the
// result does not depend on timing.
//
// Exchange.  A partial sum travels as two 64-bit words, each {pass number + 1 : payload half}; a
// word is written and read with one relaxed device-scope atomic, so a reader either sees the old
// word (wrong tag: it asks again) or the new one, and no fence or flag is needed.  The slots are
// double-buffered by pass parity: a block writes pass p + 2 only after it has read every block's
// pass p + 1, which those blocks wrote after reading all of pass p.  The init kernel zeroes the
// tags before the launch.  Waiting is bounded: a block that does not get its words within about
// four seconds gives up, every block then gives up within the same bound, and the tables come back
// as NaN; the kernel always ends.
#include "aaac_device.h"
#include "aaac_internal.h"
#include "aaac_search.h"

namespace aaac {

namespace {

constexpr int kSmallBlock = 512;
constexpr int kSmallWaves = kSmallBlock / kWave;
constexpr int kSmallRepl = 4;      // copies of the bucket table: few rows per launch, so a small table
constexpr unsigned kSpinLimit = 1u << 22;

struct alignas(16) SmallLds {
  SearchTables st;
  double hist[2][32][kSlots];  // [0] = sum I*x, [1] = sum I
  double sums[72];             // this block's sums, then the totals over all blocks
  double red[kSmallWaves];
  double objs[kSmallMaxBlocks];  // every block's share of the objective
  SearchLutT<kSmallRepl> sl;
  int failed;
  uint4 wraw[kSmallWaves][kSmallRows][kWave];   // the wavefront's rows: 8 bf16 weights per lane
  float rinv[kSmallWaves][kSmallRows][kWave];   // and the reciprocal scale of the lane's group
};

struct SmallArgs {
  const uint16_t* W;
  const float* importance;
  const float* grid;             // initial tables in device memory (written by the init kernel or the quantile step)
  unsigned long long* words;     // [2][kSmallMaxBlocks][kSmallWords]
  double* objective_trace;
  float* tables_f32;
  uint16_t* tables_bf16;
  int64_t ldw;
  int N, K, strips, waves_per_strip, rows_per_wave, scale_lanes, n_outer, n_inner;
};

// LANES: lanes per selection group; FMT: scale format.
template <int LANES, int FMT>
__global__ __launch_bounds__(kSmallBlock) void small_fit_kernel(const SmallArgs a) {
  __shared__ SmallLds sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int B = (int)gridDim.x, b = (int)blockIdx.x;
  const int gw = b * kSmallWaves + wave;  // wavefront gw works on strip gw % strips, rows rank, rank + waves_per_strip, ...
  const int strip = gw % a.strips, rank = gw / a.strips;
  const int col = strip * kStripCols + lane * 8;
  const bool active = rank < a.waves_per_strip && col < a.K;

  float Iv[8];
  {
    float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
    if (active) {
      lo = *reinterpret_cast<const float4*>(a.importance + col);
      hi = *reinterpret_cast<const float4*>(a.importance + col + 4);
    }
    Iv[0] = lo.x; Iv[1] = lo.y; Iv[2] = lo.z; Iv[3] = lo.w;
    Iv[4] = hi.x; Iv[5] = hi.y; Iv[6] = hi.z; Iv[7] = hi.w;
  }
  // the wavefront's rows and their reciprocal scales, loaded once
  for (int j = 0; j < a.rows_per_wave; ++j) {
    const int row = rank + j * a.waves_per_strip;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (active && row < a.N) v = *reinterpret_cast<const uint4*>(a.W + (int64_t)row * a.ldw + col);
    float s;
    scale_code<FMT>(group_max_lanes(absmax8(unpack8(v)), a.scale_lanes), &s);
    sm.wraw[wave][j][lane] = v;
    sm.rinv[wave][j][lane] = div_rn(1.0f, s);
  }
  double Id[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) Id[p] = (double)Iv[p];
  const uint32_t rep4 = (uint32_t)(lane & (kSmallRepl - 1)) * 4u;
  const uint32_t slot8 = (uint32_t)(lane & (kSlots - 1)) * 8u;
  const uint32_t slot_up = slot8 + kSlots * 8u;  // same slot, one bin further
  char* hist = reinterpret_cast<char*>(&sm.hist[0][0][0]);
  uint32_t sigbits = 0;  // bit j: the choice of this lane's selection group in row j
  if (tid == 0) sm.failed = 0;

  const int passes = a.n_outer * a.n_inner;
  for (int pass = 0; pass <= passes; ++pass) {
    // the tables of this pass (after the last pass: the final tables), by wavefront 0
    if (wave == 0) {
      float entry = 0.0f;
      if (lane < 32) {
        if (pass == 0) {
          entry = a.grid[lane];
        } else {
          const double num = sm.sums[lane], den = sm.sums[32 + lane];
          entry = sm.st.newtab[lane];
          if (den > 0.0) entry = (float)(num / den);
        }
      }
      wave_sort_tables(sm.st, entry);
    }
    if (pass == passes) break;
    for (int i = tid; i < 2 * 32 * kSlots; i += kSmallBlock) (&sm.hist[0][0][0])[i] = 0.0;
    __syncthreads();
    build_bucket_table<kSmallRepl, kSmallBlock>(sm.st, sm.sl);
    const float inv = sm.st.lutpar[0], off = sm.st.lutpar[1];
    const bool assign = pass % a.n_inner == 0;
    double obj = 0.0;
    if (assign) sigbits = 0;
    for (int j = 0; j < a.rows_per_wave; ++j) {
      const bool ok = active && rank + j * a.waves_per_strip < a.N;
      const W8 x = unpack8(sm.wraw[wave][j][lane]);
      const float r = sm.rinv[wave][j][lane];
      if (assign) {
        Lane8 r8;
        assign_fast_batched(x, r, Iv, sm.st, sm.sl, inv, off, rep4, r8);
        if (__any((r8.p0 != r8.p0) || (r8.p1 != r8.p1))) assign_slow(Iv, sm.st, r8);
        const float e0 = group_sum<LANES>(r8.p0);
        const float e1 = group_sum<LANES>(r8.p1);
        const bool sigma = e1 < e0;
        const uint64_t sigma_mask = __builtin_amdgcn_ballot_w64(sigma);
        sigbits |= sigma ? 1u << j : 0u;
        if (ok) {
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            const uint32_t k = sigma ? r8.k1[p] : r8.k0[p];
            const bool up = __builtin_amdgcn_inverse_ballot_w64((r8.m0[p] & ~sigma_mask) | (r8.m1[p] & sigma_mask));
            char* h = hist + (k + (up ? slot_up : slot8));
            atomicAdd(reinterpret_cast<double*>(h), Id[p] * (double)r8.wn[p]);
            atomicAdd(reinterpret_cast<double*>(h + sizeof(sm.hist[0])), Id[p]);
          }
          if ((lane % LANES) == 0) obj += (double)(sigma ? e1 : e0);
        }
      } else {
        Lane8One r1;
        const bool sigma = (sigbits >> j) & 1u;
        assign_one_fast(x, r, sm.st, sm.sl, inv, off, rep4 + (sigma ? (uint32_t)sizeof(sm.sl.lut[0]) : 0u), r1);
        if (__any(r1.check != r1.check)) assign_one_slow(sm.st, sigma ? 1 : 0, r1);
        if (ok) {
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            const bool up = __builtin_amdgcn_inverse_ballot_w64(r1.m[p]);
            char* h = hist + (r1.k[p] + (up ? slot_up : slot8));
            atomicAdd(reinterpret_cast<double*>(h), Id[p] * (double)r1.wn[p]);
            atomicAdd(reinterpret_cast<double*>(h + sizeof(sm.hist[0])), Id[p]);
          }
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) obj += __shfl_down(obj, o);
    if (lane == 0) sm.red[wave] = obj;
    __syncthreads();
    // Thread (bin = tid / 8, part = tid % 8): the block's sum of `bin` from the kSlots copies (4 neighbouring
    // slots per thread, then across the 8 threads), published by the thread with part 0 as two tagged
    // words; the thread with part 1 of bin 0 publishes the block's share of the objective.
    static_assert(kSmallBlock == 64 * 8 && kSlots == 32 && kSmallMaxBlocks == 32, "8 threads per sum, 4 blocks per thread");
    const int bin = tid >> 3, part = tid & 7;
    const uint32_t tag = (uint32_t)pass + 1u;
    unsigned long long* slots = a.words + (size_t)(pass & 1) * kSmallMaxBlocks * kSmallWords;
    {
      const double* h = &sm.hist[0][0][0] + bin * kSlots + part * 4;
      double s = (h[0] + h[1]) + (h[2] + h[3]);
#pragma unroll
      for (int o = 1; o < 8; o <<= 1) s += __shfl_xor(s, o);
      int word = 2 * bin;
      if (tid == 1) {
        s = 0.0;
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) s += sm.red[w];
        word = 128;
      }
      if (part == 0 || tid == 1) {
        const unsigned long long bits = (unsigned long long)__double_as_longlong(s);
        unsigned long long* dst = slots + (size_t)b * kSmallWords + word;
        __hip_atomic_store(dst, ((unsigned long long)tag << 32) | (uint32_t)bits, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(dst + 1, ((unsigned long long)tag << 32) | (uint32_t)(bits >> 32), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // Collect: the same thread waits for the two words of `bin` from blocks part, part + 8, part + 16,
    // part + 24 (its own block's included) and, if tid < B, for the objective words of block tid.
    double total = 0.0;
    {
      constexpr int kItems = 10;
      const unsigned long long* src[kItems];
      uint32_t got = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = part + 8 * q;
        src[2 * q] = slots + (size_t)(k < B ? k : 0) * kSmallWords + 2 * bin;
        src[2 * q + 1] = src[2 * q] + 1;
        if (k >= B) got |= 3u << (2 * q);
      }
      src[8] = slots + (size_t)(tid < B ? tid : 0) * kSmallWords + 128;
      src[9] = src[8] + 1;
      if (tid >= B) got |= 3u << 8;
      uint32_t half[kItems];
#pragma unroll
      for (int i = 0; i < kItems; ++i) half[i] = 0;
      unsigned spins = 0;
      while (got != (1u << kItems) - 1u) {
        unsigned long long v[kItems];
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
          v[i] = 0;
          if (!((got >> i) & 1u)) v[i] = __hip_atomic_load(src[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int i = 0; i < kItems; ++i)
          if (!((got >> i) & 1u) && (uint32_t)(v[i] >> 32) == tag) {
            half[i] = (uint32_t)v[i];
            got |= 1u << i;
          }
        if (++spins > kSpinLimit) {
          sm.failed = 1;
          break;
        }
      }
      // totals in a fixed order: blocks part, part + 8, ... in this thread, then across the 8 threads
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (part + 8 * q < B)
          total += __longlong_as_double((long long)(((unsigned long long)half[2 * q + 1] << 32) | half[2 * q]));
#pragma unroll
      for (int o = 1; o < 8; o <<= 1) total += __shfl_xor(total, o);
      if (part == 0) sm.sums[bin] = total;
      if (tid < B) sm.objs[tid] = __longlong_as_double((long long)(((unsigned long long)half[9] << 32) | half[8]));
    }
    __syncthreads();
    if (sm.failed) break;
    if (tid == 64 && b == 0 && assign && a.objective_trace) {  // off the path to the next tables
      double s = 0.0;
      for (int k = 0; k < B; ++k) s += sm.objs[k];
      a.objective_trace[pass / a.n_inner] = s;
    }
  }
  if (b == 0 && wave == 0 && lane < 32) {
    const bool failed = sm.failed != 0;
    const float t = failed ? __builtin_nanf("") : sm.st.newtab[lane];
    if (a.tables_f32) a.tables_f32[lane] = t;
    a.tables_bf16[lane] = failed ? (uint16_t)0x7FC0 : (uint16_t)bf16_rne(t);
  }
}

// Zeroes the tags of the exchange words and puts the caller's grid where the kernel reads it.
__global__ void small_init_kernel(unsigned long long* words, float* grid_dst, const Grid32 grid, int copy_grid) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 2 * kSmallMaxBlocks * kSmallWords) words[i] = 0ull;
  if (copy_grid && i < 32) grid_dst[i] = grid.t[i];
}

int64_t ceil_div(int64_t x, int64_t y) { return (x + y - 1) / y; }

}  // namespace

SmallPlan make_small_plan(int64_t N, int64_t K) {
  SmallPlan best = {};
  if (N <= 0 || K <= 0) return best;
  const int64_t strips = ceil_div(K, kStripCols);
  if (N * strips > (int64_t)kSmallMaxBlocks * kSmallWaves * kSmallRows) return best;
  // Cost model (microseconds per pass, fitted to measurements): a wavefront needs about 1.3 us per row it
  // holds (its eight weights per lane are some 300 vector instructions, four cycles each), the exchange
  // grows slowly with the number of blocks; tables, bucket table, reduction and exchange are ~4 us whatever
  // the split.
  double best_cost = 1e30;
  for (int blocks = 1; blocks <= kSmallMaxBlocks; ++blocks) {
    const int64_t waves = (int64_t)blocks * kSmallWaves;
    if (waves < strips) continue;
    const int64_t wps = waves / strips;
    const int64_t rows = ceil_div(N, wps);
    if (rows > kSmallRows) continue;
    const double cost = 4.0 + 0.02 * blocks + 1.3 * (double)rows;
    if (cost < best_cost) {
      best_cost = cost;
      best.blocks = blocks;
      best.strips = (int)strips;
      best.waves_per_strip = (int)wps;
      best.rows_per_wave = (int)rows;
    }
  }
  return best;
}

hipError_t launch_fit_small(const FitTask& t, const SmallPlan& plan, int group_size, int sel_size, int fmt,
                            const Grid32* grid, float* grid_dev, unsigned long long* words, int n_outer,
                            int n_inner, hipStream_t stream) {
  SmallArgs a = {};
  a.W = static_cast<const uint16_t*>(t.W);
  a.importance = t.importance;
  a.grid = grid_dev;
  a.words = words;
  a.objective_trace = t.objective_trace;
  a.tables_f32 = t.tables_f32;
  a.tables_bf16 = t.tables_bf16;
  a.ldw = t.ldw;
  a.N = (int)t.N;
  a.K = (int)t.K;
  a.strips = plan.strips;
  a.waves_per_strip = plan.waves_per_strip;
  a.rows_per_wave = plan.rows_per_wave;
  a.scale_lanes = group_size / 8;
  a.n_outer = n_outer;
  a.n_inner = n_inner;
  const int n_words = 2 * kSmallMaxBlocks * kSmallWords;
  small_init_kernel<<<(n_words + 255) / 256, 256, 0, stream>>>(words, grid_dev, grid ? *grid : Grid32{}, grid ? 1 : 0);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
#define AAAC_SMALL(L, F) small_fit_kernel<L, F><<<plan.blocks, kSmallBlock, 0, stream>>>(a)
  switch (sel_size / 8) {
    case 2: if (fmt == 0) AAAC_SMALL(2, 0); else AAAC_SMALL(2, 1); break;
    case 4: if (fmt == 0) AAAC_SMALL(4, 0); else AAAC_SMALL(4, 1); break;
    case 8: if (fmt == 0) AAAC_SMALL(8, 0); else AAAC_SMALL(8, 1); break;
    default: if (fmt == 0) AAAC_SMALL(16, 0); else AAAC_SMALL(16, 1); break;
  }
#undef AAAC_SMALL
  return hipGetLastError();
}

}  // namespace aaac

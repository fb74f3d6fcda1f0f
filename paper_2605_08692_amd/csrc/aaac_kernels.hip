// gfx950 kernels of the AAAC hot path and their launchers.
//
// Work mapping used throughout: one lane owns 8 consecutive bf16 weights of a row
// (one 16-byte load), so a weight group of g = 16..128 is held by g/8 = 2..16
// adjacent lanes and group reductions are DPP exchanges inside a wavefront.
// All fp32 arithmetic that decides a code or a selection bit is written as single
// IEEE operations (the file is compiled with -ffp-contract=off).  This file holds
// the importance, scale, encode and dequant kernels; the Lloyd iteration is in
// aaac_lloyd.hip, the nearest-entry search shared with it in aaac_search.h.
#include <atomic>

#include "aaac_device.h"
#include "aaac_internal.h"
#include "aaac_search.h"

namespace aaac {

namespace {

constexpr int kBlock = 256;

// ------------------------------------------------------------ importance

// Partial column sums of squares over one chunk of tokens.  A wavefront reads
// whole rows of up to 4096 columns (eight 16-byte loads per lane, 8 KB
// contiguous), two rows in flight, so that HBM is read in long sequential runs;
// the 8 wavefronts of a block take every 8th row of the block's token chunk.  X
// is read once, so the loads are non-temporal.  The wavefronts' fp64 partials
// are added in wavefront order through LDS.
constexpr int kStatsBlock = 512;
constexpr int kStatsWaves = kStatsBlock / kWave;
constexpr int kStatsStrips = 8;                          // strips of 512 columns per wavefront
constexpr int kStatsCols = kStatsStrips * kStripCols;    // 4096
__global__ __launch_bounds__(kStatsBlock) void act_stats_partial_kernel(
    const uint16_t* __restrict__ X, int64_t tokens, int64_t K, int64_t ldx, int64_t tokens_per_chunk,
    double* __restrict__ partials, int64_t Kpad) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  __shared__ double buf[kStatsCols];  // [(strip * 8 + p) * 64 + lane]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t col0 = (int64_t)blockIdx.x * kStatsCols + lane * 8;
  const int64_t t0 = (int64_t)blockIdx.y * tokens_per_chunk;
  const int64_t t1 = t0 + tokens_per_chunk < tokens ? t0 + tokens_per_chunk : tokens;
  double acc[kStatsStrips][8];
#pragma unroll
  for (int s = 0; s < kStatsStrips; ++s)
#pragma unroll
    for (int p = 0; p < 8; ++p) acc[s][p] = 0.0;
  // Two rows are in flight per wavefront, and the one that has just been added is asked for again
  // (its successor) before the other is added, so loads and additions overlap.  The loads are
  // unconditional (a load under a branch would make every wait a wait for all loads): a row beyond
  // the chunk reads the chunk's last row and is not added, a column beyond K reads column 0 of its
  // strip position and lands in an accumulator that is never stored.
  const uint16_t* base = X + (col0 < K ? col0 : 0);
  bool col_ok[kStatsStrips];
#pragma unroll
  for (int s = 0; s < kStatsStrips; ++s) col_ok[s] = col0 + s * kStripCols < K;
  auto load_row = [&](u32x4 (&v)[kStatsStrips], int64_t t) {
    const uint16_t* row = base + (t < t1 ? t : t1 - 1) * ldx;
#pragma unroll
    for (int s = 0; s < kStatsStrips; ++s)
      v[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + (col_ok[s] ? s * kStripCols : 0)));
  };
  auto add_row = [&](const u32x4 (&v)[kStatsStrips]) {
#pragma unroll
    for (int s = 0; s < kStatsStrips; ++s) {
      const W8 x = unpack8(make_uint4(v[s].x, v[s].y, v[s].z, v[s].w));
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const double d = (double)x.w[p];
        acc[s][p] = fma(d, d, acc[s][p]);
      }
    }
  };
  if (t0 + wave < t1) {
    u32x4 va[kStatsStrips], vb[kStatsStrips];
    int64_t t = t0 + wave;
    load_row(va, t);
    load_row(vb, t + kStatsWaves);
    for (; t < t1; t += 2 * kStatsWaves) {
      add_row(va);
      asm volatile("" ::: "memory");
      load_row(va, t + 2 * kStatsWaves);
      asm volatile("" ::: "memory");
      if (t + kStatsWaves < t1) add_row(vb);
      asm volatile("" ::: "memory");
      load_row(vb, t + 3 * kStatsWaves);
      asm volatile("" ::: "memory");
    }
  }
  for (int w = 0; w < kStatsWaves; ++w) {
    if (wave == w) {
#pragma unroll
      for (int s = 0; s < kStatsStrips; ++s)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const int i = (s * 8 + p) * 64 + lane;
          buf[i] = w == 0 ? acc[s][p] : buf[i] + acc[s][p];
        }
    }
    __syncthreads();
  }
  double* out = partials + (int64_t)blockIdx.y * Kpad + (int64_t)blockIdx.x * kStatsCols;
  for (int c = threadIdx.x; c < kStatsCols; c += kStatsBlock) {
    const int s = c / kStripCols, l = (c % kStripCols) / 8, p = c % 8;
    out[c] = buf[(s * 8 + p) * 64 + l];
  }
}

// Sum of the chunk partials of each column, in a fixed order: block = 16
// columns x 16 parts, part q adds chunks q, q+16, ..., then the parts are added.
__global__ __launch_bounds__(kBlock) void act_stats_reduce_kernel(const double* __restrict__ partials,
                                                                  int chunks, int64_t K, int64_t Kpad,
                                                                  float* __restrict__ importance) {
  __shared__ double sred[16][16];
  const int c16 = threadIdx.x & 15, part = threadIdx.x >> 4;
  const int64_t col = (int64_t)blockIdx.x * 16 + c16;
  double s = 0.0;
  if (col < K) {
    for (int c0 = part; c0 < chunks; c0 += 16 * 8) {
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = c0 + 16 * u;
        v[u] = c < chunks ? partials[(int64_t)c * Kpad + col] : 0.0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
  }
  sred[part][c16] = s;
  __syncthreads();
  if (threadIdx.x < 16 && col < K) {
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < 16; ++q) t += sred[q][threadIdx.x];
    importance[col] = (float)t;
  }
}

// ---------------------------------------------------- scales (reciprocals)

// Chunks of 8 weights are numbered row by row; thread t takes chunks t, t + T, t + 2T, ... (T = threads of
// the grid), four at a time with their loads in flight together.  Row and column advance by additions
// (one division per thread, none per chunk).
constexpr int kStreamUnroll = 4;
struct ChunkWalk {
  int64_t row, cc;   // row and chunk within the row
  int64_t dr, dc;    // T / cpr, T % cpr
  int64_t cpr;
  __device__ __forceinline__ void step() {
    row += dr;
    cc += dc;
    if (cc >= cpr) { cc -= cpr; ++row; }
  }
};
__device__ __forceinline__ ChunkWalk chunk_walk(int64_t cpr) {
  const int64_t T = (int64_t)gridDim.x * kBlock, c = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  return ChunkWalk{c / cpr, c % cpr, T / cpr, T % cpr, cpr};
}

// One chunk of 8 weights per thread.  The grid is (blocks of 256 chunks along a row) x (rows, at most
// 65535: further rows in a loop), so that no thread divides to find its row.  Measured 104 us for 235 M
// weights (4.5 TB/s), the same with four rows per thread and their loads in flight together, and 15 %
// slower as a grid-stride loop of fewer, longer-lived blocks.
template <int LANES, int FMT>
__global__ __launch_bounds__(kBlock) void group_rinv_kernel(const uint16_t* __restrict__ W, int64_t N,
                                                            int64_t K, int64_t ldw,
                                                            float* __restrict__ rinv) {
  const int cpr = (int)(K / 8);  // chunks per row
  const int cc = (int)blockIdx.x * kBlock + (int)threadIdx.x;
  const bool active = cc < cpr;
  const int col = active ? cc * 8 : 0;  // an idle lane reads the row's first chunk
  const int groups = cpr / LANES;
  for (int64_t row = blockIdx.y; row < N; row += gridDim.y) {
    const uint4 v = *reinterpret_cast<const uint4*>(W + row * ldw + col);
    const float a = group_max<LANES>(absmax8(unpack8(v)));
    float s;
    scale_code<FMT>(a, &s);
    if (active && (threadIdx.x % LANES) == 0) rinv[row * groups + cc / LANES] = div_rn(1.0f, s);
  }
}

// ----------------------------------------------------------------- encode

struct alignas(16) EncodeLds {
  SearchTables st;
  SearchLut sl;
};

// Same block / wavefront / row mapping and the same bucket-table search as the
// Lloyd iteration; per row a lane recomputes its scale group's scale, takes both
// errors of its selection group, and writes 8 codes as one 32-bit store.  The
// first lane of a scale group stores the scale; the table choice goes into the
// scale's top bit when both groups coincide (sel_bits null), otherwise into the
// separate bit array: selection group j of a row is bit j % 8 of byte j / 8.
// LANES: lanes per selection group; scale_lanes: lanes per scale group; SAME: the two groups
// coincide (scale_lanes == LANES, no separate bits).
template <int LANES, int FMT, bool SAME>
__global__ __launch_bounds__(kSearchBlock) void encode_kernel(
    const uint16_t* __restrict__ W, int N, int K, int64_t ldw, const float* __restrict__ importance,
    const uint16_t* __restrict__ tables_bf16, uint8_t* __restrict__ codes, void* __restrict__ scales,
    uint8_t* __restrict__ sel_bits, int64_t sel_stride, int scale_lanes,
    int strips, int strips_per_block, int strip_groups, int rows_per_block) {
  __shared__ EncodeLds sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (wave == 0) {
    if (lane < 32) sm.st.newtab[lane] = __uint_as_float((uint32_t)tables_bf16[lane] << 16);
    wave_make_rows(sm.st);
  }
  const int queue = wave % strips_per_block;
  const int strip = (blockIdx.x % strip_groups) * strips_per_block + queue;
  const int block_r0 = (blockIdx.x / strip_groups) * rows_per_block;
  const int block_r1 = block_r0 + rows_per_block < N ? block_r0 + rows_per_block : N;
  const int waves_per_queue = kSearchWaves / strips_per_block;
  const int col = strip * kStripCols + lane * 8;
  const bool has_strip = strip < strips;
  const bool active = has_strip && col < K;
  const int Gs = K / (8 * scale_lanes);  // scale groups per row
  // selection bits: a wavefront's strip holds 64 / LANES groups = 8 / LANES bytes; lane b builds byte b
  constexpr int kSelBytes = LANES <= 8 ? 8 / LANES : 1;
  const int sel_lane = lane & (kSelBytes - 1);
  const int sel_byte = strip * kSelBytes + sel_lane;             // byte index inside the row
  const bool sel_writer = !SAME && sel_bits != nullptr && has_strip && lane < kSelBytes &&
                          (int64_t)sel_byte * 64 * LANES < K;   // the byte's first group starts inside the row
  const uint16_t* wbase = W + (active ? col : 0);
  int row = has_strip ? block_r0 + wave / strips_per_block : block_r1;
  if (tid < strips_per_block) sm.st.next_row[tid] = block_r0 + waves_per_queue;
  uint4 v_next = make_uint4(0, 0, 0, 0);
  if (active && row < block_r1) v_next = *reinterpret_cast<const uint4*>(wbase + (int64_t)row * ldw);
  float Iv[8];
  {
    float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
    if (active) {
      lo = *reinterpret_cast<const float4*>(importance + col);
      hi = *reinterpret_cast<const float4*>(importance + col + 4);
    }
    Iv[0] = lo.x; Iv[1] = lo.y; Iv[2] = lo.z; Iv[3] = lo.w;
    Iv[4] = hi.x; Iv[5] = hi.y; Iv[6] = hi.z; Iv[7] = hi.w;
  }
  __syncthreads();
  build_bucket_table(sm.st, sm.sl);
  const float inv = sm.st.lutpar[0], off = sm.st.lutpar[1];
  const uint32_t rep4 = (uint32_t)(lane & (kReplicas - 1)) * 4u;
  // (everything loaded so far is waited for here, so that no wait is left at the top of the loop,
  // where it would also wait for the stores of the round before; see the end of the loop)
  asm volatile("" ::"v"(v_next.x), "v"(v_next.y), "v"(v_next.z), "v"(v_next.w), "v"(Iv[0]), "v"(Iv[1]), "v"(Iv[2]),
               "v"(Iv[3]), "v"(Iv[4]), "v"(Iv[5]), "v"(Iv[6]), "v"(Iv[7]));
  while (row < block_r1) {
    const uint4 v = v_next;
    const int cur = row;
    int next = 0;
    if (lane == 0) next = atomicAdd(&sm.st.next_row[queue], 1);
    next = __builtin_amdgcn_readfirstlane(next);
    if (active && next < block_r1) v_next = *reinterpret_cast<const uint4*>(wbase + (int64_t)next * ldw);
    row = next;
    const W8 x = unpack8(v);
    float s;
    const uint32_t sc = scale_code<FMT>(SAME ? group_max<LANES>(absmax8(x)) : group_max_lanes(absmax8(x), scale_lanes), &s);
    const float r = div_rn(1.0f, s);
    Lane8 a;
    assign_fast(x, r, Iv, sm.st, sm.sl, inv, off, rep4, a);
    if (__any((a.p0 != a.p0) || (a.p1 != a.p1))) assign_slow(Iv, sm.st, a);
    const float e0 = group_sum<LANES>(a.p0);
    const float e1 = group_sum<LANES>(a.p1);
    const bool sigma = active && e1 < e0;
    const uint64_t sigma_mask = __builtin_amdgcn_ballot_w64(sigma);
    uint32_t packed = 0;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const uint32_t k = sigma ? a.k1[p] : a.k0[p];  // (16 * table + index) * kSlots * 8
      const bool up = __builtin_amdgcn_inverse_ballot_w64((a.m0[p] & ~sigma_mask) | (a.m1[p] & sigma_mask));
      const uint32_t idx = ((k / (kSlots * 8u)) & 15u) + (up ? 1u : 0u);
      packed |= idx << (4 * p);
    }
    // The next row's weights are waited for here, before this row's stores go out: loads and stores
    // complete in order, so a wait placed after the stores (at the top of the next round) would also
    // wait for the stores just issued; here only the load, asked for a whole round ago, is outstanding.
    asm volatile("" ::"v"(v_next.x), "v"(v_next.y), "v"(v_next.z), "v"(v_next.w));
    if (active) {
      *reinterpret_cast<uint32_t*>(codes + ((int64_t)cur * K + col) / 2) = packed;
      if ((lane % (SAME ? LANES : scale_lanes)) == 0) {
        const int64_t g = (int64_t)cur * Gs + col / (8 * (SAME ? LANES : scale_lanes));
        const bool sign = (SAME || sel_bits == nullptr) && sigma;
        if (FMT == 0) static_cast<uint8_t*>(scales)[g] = (uint8_t)(sc | (sign ? 0x80u : 0u));
        else static_cast<uint16_t*>(scales)[g] = (uint16_t)(sc | (sign ? 0x8000u : 0u));
      }
    }
    if (sel_writer) {  // bit i of this lane's byte: the choice of the group led by lane (8 * sel_lane + i) * LANES
      uint32_t byte = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        byte |= (uint32_t)((sigma_mask >> (((8 * sel_lane + i) * LANES) & 63)) & 1u) << i;
      sel_bits[(int64_t)cur * sel_stride + sel_byte] = (uint8_t)byte;
    }
  }
}

// ---------------------------------------------------------------- dequant

// sel_bits null: the table choice is the top bit of the scale; otherwise bit j % 8 of byte
// j / 8 of the row's sel_stride bytes, j = column / sel_size.
template <int FMT, bool BITS>
__global__ __launch_bounds__(kBlock) void dequant_kernel(
    const uint8_t* __restrict__ codes, const void* __restrict__ scales,
    const uint8_t* __restrict__ sel_bits, int64_t sel_stride, int sshift,
    const uint16_t* __restrict__ tables_bf16, int64_t N, int64_t K, int gshift,
    uint16_t* __restrict__ W_hat, int64_t ldo) {
  __shared__ float sT[32];
  if (threadIdx.x < 32) sT[threadIdx.x] = __uint_as_float((uint32_t)tables_bf16[threadIdx.x] << 16);
  __syncthreads();
  ChunkWalk w = chunk_walk(K / 8);
  const int64_t Gs = K >> gshift;
  while (w.row < N) {
    // the loads of four chunks go out together (unconditional: past the end the last row is read again)
    uint32_t packed[kStreamUnroll], sc[kStreamUnroll], sb[kStreamUnroll];
    int64_t row[kStreamUnroll], col[kStreamUnroll];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      row[u] = w.row;
      col[u] = w.cc * 8;
      const int64_t r = w.row < N ? w.row : N - 1;
      const int64_t g = r * Gs + (col[u] >> gshift);
      sc[u] = FMT == 0 ? (uint32_t) static_cast<const uint8_t*>(scales)[g] : (uint32_t) static_cast<const uint16_t*>(scales)[g];
      sb[u] = 0;
      if (BITS) sb[u] = sel_bits[r * sel_stride + ((col[u] >> sshift) >> 3)];
      packed[u] = *reinterpret_cast<const uint32_t*>(codes + (r * K + col[u]) / 2);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      uint32_t sigma;
      float s;
      if (FMT == 0) {
        sigma = sc[u] >> 7;
        s = e4m3_value(sc[u] & 0x7Fu);
      } else {
        sigma = sc[u] >> 15;
        s = __uint_as_float((sc[u] & 0x7FFFu) << 16);
      }
      if (BITS) sigma = (sb[u] >> ((col[u] >> sshift) & 7)) & 1u;
      const float* T = sT + 16 * sigma;
      uint32_t h[8];
#pragma unroll
      for (int p = 0; p < 8; ++p) h[p] = bf16_rne(T[(packed[u] >> (4 * p)) & 15u] * s);
      if (row[u] < N)
        *reinterpret_cast<uint4*>(W_hat + row[u] * ldo + col[u]) =
            make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
  }
}

// Plain fill, used instead of a memset node so that callers may capture the
// stream into a graph.
__global__ void fill_zero_kernel(uint32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = 0u;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

hipError_t fill_zero(void* p, size_t bytes, hipStream_t stream) {  // bytes % 4 == 0
  const int64_t n = (int64_t)(bytes / 4);
  if (n == 0) return hipSuccess;
  fill_zero_kernel<<<(unsigned)ceil_div(n, kBlock), kBlock, 0, stream>>>(static_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

}  // namespace

// ---------------------------------------------------------------- plans

StatsPlan make_stats_plan(int64_t tokens, int64_t K) {
  StatsPlan p;
  p.strips = (int)ceil_div(K, kStatsCols);  // column groups of 4096
  const int64_t tok = tokens > 0 ? tokens : 1;
  // One block of 8 wavefronts per compute unit and never more blocks than the 256 compute units: a
  // compute unit holds one block, so a 257th block would run alone after all the others (7 column
  // groups x 37 token chunks = 259 blocks ran at 4.8 TB/s, 7 x 36 run at 6.5).
  int64_t chunks = 256 / p.strips;
  const int64_t most = ceil_div(tok, 4 * kStatsWaves);  // at least 4 rows per wavefront
  if (chunks > most) chunks = most;
  if (chunks < 1) chunks = 1;
  if (chunks > 65535) chunks = 65535;
  p.tokens_per_chunk = ceil_div(ceil_div(tok, chunks), kStatsWaves) * kStatsWaves;
  p.token_chunks = (int)ceil_div(tok, p.tokens_per_chunk);
  p.bytes = (size_t)p.token_chunks * p.strips * kStatsCols * sizeof(double);
  return p;
}

// -------------------------------------------------------------- launchers

// Blocks for the kernels that walk chunks of 8 weights with a grid-sized stride: enough for every thread
// to take about kStreamUnroll chunks, at most 8 blocks per compute unit (256 of them).
unsigned stream_blocks(int64_t chunks) {
  const int64_t want = ceil_div(chunks, (int64_t)kBlock * kStreamUnroll);
  return (unsigned)(want < 1 ? 1 : want > 2048 ? 2048 : want);
}

#define AAAC_LAUNCH_CHECK()                     \
  do {                                          \
    hipError_t e_ = hipGetLastError();          \
    if (e_ != hipSuccess) return e_;            \
  } while (0)

hipError_t launch_act_stats(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                            void* ws, const StatsPlan& plan, hipStream_t stream) {
  const int64_t Kpad = (int64_t)plan.strips * kStatsCols;
  double* partials = static_cast<double*>(ws);
  if (tokens == 0) {
    return fill_zero(importance, (size_t)K * sizeof(float), stream);
  }
  act_stats_partial_kernel<<<dim3(plan.strips, plan.token_chunks), kStatsBlock, 0, stream>>>(
      static_cast<const uint16_t*>(X), tokens, K, ldx, plan.tokens_per_chunk, partials, Kpad);
  AAAC_LAUNCH_CHECK();
  act_stats_reduce_kernel<<<(unsigned)ceil_div(K, 16), kBlock, 0, stream>>>(partials, plan.token_chunks,
                                                                                 K, Kpad, importance);
  AAAC_LAUNCH_CHECK();
  return hipSuccess;
}

// ---- partial sums of the importance without a caller's workspace
//
// The array lives in the library's device code; every GPU that loads the library holds its own
// copy at its own address.  In host code the array's name is only a handle for the runtime: the
// address a kernel can use comes from hipGetSymbolAddress, asked once per device with that device
// current and kept in scratch_ptr[]; kernels get that pointer as an argument, exactly as they get
// the caller's workspace in launch_act_stats.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> scratch_ptr[kMaxDevices];

static hipError_t static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    scratch_ptr[dev].store(p, std::memory_order_release);  // two first calls at once store the same address
  }
  *out = p;
  return hipSuccess;
}

hipError_t launch_act_stats_static(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                                   const StatsPlan& plan, hipStream_t stream) {
  if (plan.bytes > kStaticScratchBytes) return hipErrorInvalidValue;
  void* ws = nullptr;
  if (tokens > 0) {
    hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return e;
  }
  return launch_act_stats(X, tokens, K, ldx, importance, ws, plan, stream);
}

template <int LANES>
static hipError_t launch_rinv_lanes(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, int fmt, float* rinv,
                                    hipStream_t stream) {
  const dim3 grid((unsigned)ceil_div(K / 8, kBlock), (unsigned)(N < 65535 ? N : 65535));
  if (fmt == 0)
    group_rinv_kernel<LANES, 0><<<grid, kBlock, 0, stream>>>(W, N, K, ldw, rinv);
  else
    group_rinv_kernel<LANES, 1><<<grid, kBlock, 0, stream>>>(W, N, K, ldw, rinv);
  AAAC_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_group_rinv(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, int fmt,
                             float* rinv, hipStream_t stream) {
  if (N == 0 || K == 0) return hipSuccess;
  const uint16_t* Wp = static_cast<const uint16_t*>(W);
  switch (group_size / 8) {
    case 2: return launch_rinv_lanes<2>(Wp, N, K, ldw, fmt, rinv, stream);
    case 4: return launch_rinv_lanes<4>(Wp, N, K, ldw, fmt, rinv, stream);
    case 8: return launch_rinv_lanes<8>(Wp, N, K, ldw, fmt, rinv, stream);
    default: return launch_rinv_lanes<16>(Wp, N, K, ldw, fmt, rinv, stream);
  }
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream) { return fill_zero(p, bytes, stream); }

struct EncodeCall {
  const uint16_t* W;
  int64_t N, K, ldw;
  int group_size, fmt;
  const float* importance;
  const uint16_t* tables_bf16;
  uint8_t* codes;
  void* scales;
  uint8_t* sel_bits;
  int64_t sel_stride;
};

template <int LANES>
static hipError_t launch_encode_lanes(const EncodeCall& c, hipStream_t stream) {
  const FitPlan p = make_fit_plan(c.N, c.K, c.ldw, c.group_size, 8 * LANES, device_compute_units());
#define AAAC_ENCODE(FMT, SAME)                                                                              \
  encode_kernel<LANES, FMT, SAME><<<p.blocks, kSearchBlock, 0, stream>>>(                                    \
      c.W, (int)c.N, (int)c.K, c.ldw, c.importance, c.tables_bf16, c.codes, c.scales, c.sel_bits, c.sel_stride, \
      c.group_size / 8, p.strips, p.strips_per_block, p.strip_groups, p.rows_per_block)
  const bool same = c.group_size == 8 * LANES;
  if (c.fmt == 0) {
    if (same) AAAC_ENCODE(0, true); else AAAC_ENCODE(0, false);
  } else {
    if (same) AAAC_ENCODE(1, true); else AAAC_ENCODE(1, false);
  }
#undef AAAC_ENCODE
  AAAC_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t launch_encode(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, int sel_size,
                         int fmt, const float* importance, const uint16_t* tables_bf16, uint8_t* codes,
                         void* scales, uint8_t* sel_bits, int64_t sel_stride, hipStream_t stream) {
  if (N == 0 || K == 0) return hipSuccess;
  const EncodeCall c = {static_cast<const uint16_t*>(W), N, K, ldw, group_size, fmt, importance, tables_bf16,
                        codes, scales, sel_size < group_size ? sel_bits : nullptr, sel_stride};
  switch (sel_size / 8) {
    case 2: return launch_encode_lanes<2>(c, stream);
    case 4: return launch_encode_lanes<4>(c, stream);
    case 8: return launch_encode_lanes<8>(c, stream);
    default: return launch_encode_lanes<16>(c, stream);
  }
}

hipError_t launch_dequant(const uint8_t* codes, const void* scales, const uint8_t* sel_bits,
                          int64_t sel_stride, const uint16_t* tables_bf16, int64_t N, int64_t K,
                          int group_size, int sel_size, int fmt, void* W_hat, int64_t ldo,
                          hipStream_t stream) {
  if (N == 0 || K == 0) return hipSuccess;
  const unsigned gblocks = stream_blocks(N * (K / 8));
  uint16_t* out = static_cast<uint16_t*>(W_hat);
  int gshift = 0, sshift = 0;
  for (int g = group_size; g > 1; g >>= 1) ++gshift;
  for (int g = sel_size; g > 1; g >>= 1) ++sshift;
  const uint8_t* bits = sel_size < group_size ? sel_bits : nullptr;
#define AAAC_DEQUANT(FMT, BITS)                                                                              \
  dequant_kernel<FMT, BITS><<<gblocks, kBlock, 0, stream>>>(codes, scales, bits, sel_stride, sshift, tables_bf16, \
                                                            N, K, gshift, out, ldo)
  if (fmt == 0) {
    if (bits) AAAC_DEQUANT(0, true); else AAAC_DEQUANT(0, false);
  } else {
    if (bits) AAAC_DEQUANT(1, true); else AAAC_DEQUANT(1, false);
  }
#undef AAAC_DEQUANT
  AAAC_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace aaac

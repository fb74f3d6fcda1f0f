// The quantised layer applied to a batch of activation rows on the matrix cores
// (W4A16): y[m, n] = sum_k x[m, k] * w^[n, k] with w^ = bf16(T_sigma[code] * s), the
// weights of paper Eq. "aaac_dequant" rounded to bf16 as aaac_dequant stores them,
// fp32 accumulation (v_mfma_f32_16x16x32_bf16).  The codes are dequantised in
// registers straight into the MFMA's A operand; the dequantised weights never go
// to memory.
//
// Mapping.  D[n][m] = sum_k A[n][k] B[k][m] with A = w^ (16 rows of the layer) and
// B = x^T (16 rows of x).  In a 16x16x32 MFMA lane (r, q), r = lane % 16, q = lane / 16,
// supplies A[r][8q..8q+7] and B[8q..8q+7][r] and receives D[4q..4q+3][r].  The sum
// over k may run in any order as long as A and B agree, so per 256-column chunk a lane
// takes the 64 consecutive columns 64q..64q+63 of its row (two 16-byte code loads: the
// four lanes of a row read one 128-byte line) and feeds them in eight steps of 8;
// the lane that holds x row r takes the same columns of x (a small kernel first copies x
// into that order, so that an operand load is one contiguous kilobyte).
//
// Two codes are dequantised with one LDS read (code byte -> fp32 pair of table
// values), multiplied by the scale (exact: 8 x 8 significant bits) and rounded to
// bf16 pairs by the hardware conversion.
//
// Two kernels: gemm_w4a16_rows_kernel (up to 32 rows of x at a time, which stay in registers
// while a wavefront walks down the layer rows; the mapping above) and gemm_w4a16_tiled_kernel
// (large batches: weights dequantised once per 128 x 64 tile into LDS).
#include <cmath>

#include "aaac_device.h"
#include "aaac_internal.h"

namespace aaac {

namespace {

constexpr int kGemmBlock = 512;
constexpr int kGemmWaves = kGemmBlock / 64;
constexpr int kChunkCols = 256;      // columns per wavefront step: 4 lane quarters x 64
constexpr int kGemmReplicas = 8;     // copies of the pair table

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int FMT>
__device__ __forceinline__ float gemm_scale_value(uint32_t code, uint32_t* sign) {
  if (FMT == 0) {
    *sign = code >> 7;
    return __uint_as_float((code & 0x7Fu) << 20) * 0x1p120f;  // E4M3 -> fp32, subnormals included
  }
  *sign = code >> 15;
  return __uint_as_float((code & 0x7FFFu) << 16);
}

// two fp32 -> packed bf16 pair, round to nearest even
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  uint32_t u;
  __builtin_memcpy(&u, &b, 4);
  return u;
}

// x in the order the matrix instruction wants it: element ((c * 8 + st) * MT + j) * 64 + lane of
// the packed array is the 16-byte B operand of lane (r, q) for chunk c, step st, x tile j, i.e.
// x[16 j + r][256 c + 64 q + 8 st .. + 7] (zero outside the matrix), so that a wavefront's operand
// load is one contiguous kilobyte.
// With clear_n > 0 the kernel also clears y[0 .. M)[0 .. clear_n) (for a product that adds its parts into y).
template <int MT>
__global__ void pack_x_kernel(const uint16_t* __restrict__ x, int64_t ldx, int M, int K, int chunks,
                              uint4* __restrict__ xpack, float* __restrict__ y = nullptr, int64_t ldy = 0,
                              int clear_n = 0) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int64_t e = i; e < (int64_t)M * clear_n; e += (int64_t)gridDim.x * blockDim.x)
    y[(e / clear_n) * ldy + e % clear_n] = 0.0f;
  if (i >= (int64_t)chunks * 8 * MT * 64) return;
  const int lane = (int)(i & 63), r = lane & 15, q = lane >> 4;
  const int64_t rest = i >> 6;
  const int j = (int)(rest % MT), st = (int)((rest / MT) & 7), c = (int)(rest / (MT * 8));
  const int m = 16 * j + r, k = c * kChunkCols + 64 * q + 8 * st;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (m < M && k < K) v = *reinterpret_cast<const uint4*>(x + (int64_t)m * ldx + k);
  xpack[i] = v;
}

// ---------------------------------------------------------------------------------
// Up to 32 rows of x (batched decoding): x stays in registers.  A block owns 64 layer rows; a
// wavefront owns one 256-column chunk at a time (lane (r, q): columns 64q .. 64q + 63 of it), loads
// the B operands of that chunk once, from the packed copy of x, and walks down the block's four
// tiles of 16 layer rows: two 16-byte code loads per lane and tile, dequantised into the A operand,
// and 8 MT matrix instructions into accumulators that stay in registers over all the wavefront's
// chunks.  At the end every wavefront writes its 64 x 16 MT partial sums to a slab of its own in
// LDS (over the pair table, which is no longer needed) and the block adds the 8 slabs while
// storing y.  x is read once per 64 layer rows and the codes once per 32 rows of x.
constexpr int kRowsTile = 64;  // layer rows of a block, at most
constexpr int kSlabPad = 4;  // a slab row is 16 MT + 4 floats: lanes (r, q) of one store fall into 64 banks

template <int MT>
struct alignas(16) RowsLds {
  union {
    float2 pair[2][256][kGemmReplicas];
    float part[kGemmWaves][kRowsTile][MT * 16 + kSlabPad];
  };
  float T[32];
};

struct TileRegs {  // what a lane loads per tile of 16 layer rows: 32 code bytes, raw scale bytes, selection byte
  uint4 c0, c1;
  uint2 sc;
  uint32_t selbyte;
};

template <int FMT, int MT, int GS, bool SEL, int RT>
__global__ __launch_bounds__(kGemmBlock) void gemm_w4a16_rows_kernel(
    const uint4* __restrict__ xpack, int M, const uint8_t* __restrict__ codes,
    const void* __restrict__ scales, const uint8_t* __restrict__ sel_bits, int64_t sel_stride,
    const uint16_t* __restrict__ tables_bf16, int N, int K, int gshift, int sshift, float* __restrict__ y,
    int64_t ldy) {
  __shared__ RowsLds<MT> sm;
  constexpr int kRowsTile = 16 * RT, kRowsTiles = RT;  // the block's layer rows: 64, or 32 / 16 on small layers
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 32) sm.T[tid] = __uint_as_float((uint32_t)tables_bf16[tid] << 16);
  __syncthreads();

  const int r = lane & 15, q = lane >> 4;
  const int r0 = blockIdx.x * kRowsTile;
  const int r1 = r0 + kRowsTile < N ? r0 + kRowsTile : N;
  const int chunks = (K + kChunkCols - 1) / kChunkCols;
  const int Gs = K >> gshift;
  const int rep = lane & (kGemmReplicas - 1);
  const int64_t row_bytes = K / 2;

  // this lane's columns of chunk c: all 64 or none (K % 64 == 0); a lane beyond K reads the row's
  // first columns and multiplies them with the zeros that the packed x holds there
  auto lane_cols = [&](int c) { return c * kChunkCols + 64 * q; };
  // loads are unconditional, from clamped addresses (a row beyond the block's last reads the last
  // row; its sums are not stored)
  auto fetch = [&](TileRegs& tr, int c, int t) {
    const int k0 = lane_cols(c), kc = k0 < K ? k0 : 0;
    const int n0 = r0 + 16 * t + r;
    const int n = n0 < r1 ? n0 : r1 - 1;
    const uint8_t* cp = codes + (int64_t)n * row_bytes + kc / 2;
    tr.c0 = *reinterpret_cast<const uint4*>(cp);
    tr.c1 = *reinterpret_cast<const uint4*>(cp + 16);
    const int64_t g0 = (int64_t)n * Gs + (kc >> gshift);
    tr.sc = make_uint2(0, 0);
    if (FMT == 0) {
      const uint8_t* sp = static_cast<const uint8_t*>(scales) + g0;
      if (GS == 4) tr.sc.x = *reinterpret_cast<const uint32_t*>(sp);
      else if (GS == 5) tr.sc.x = *reinterpret_cast<const uint16_t*>(sp);
      else tr.sc.x = *sp;
    } else {
      const uint16_t* sp = static_cast<const uint16_t*>(scales) + g0;
      if (GS == 4) tr.sc = *reinterpret_cast<const uint2*>(sp);
      else if (GS == 5) tr.sc.x = *reinterpret_cast<const uint32_t*>(sp);
      else tr.sc.x = *sp;
    }
    tr.selbyte = 0;
    if (SEL) tr.selbyte = sel_bits[(int64_t)n * sel_stride + ((kc >> sshift) >> 3)];
  };

  f32x4 acc[kRowsTiles][MT];
#pragma unroll
  for (int t = 0; t < kRowsTiles; ++t)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[t][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // blockIdx.y: which part of the chunk sequence this block sums (the parts are added in y)
  const int c_begin = (int)((int64_t)chunks * blockIdx.y / gridDim.y);
  const int c_end = (int)((int64_t)chunks * (blockIdx.y + 1) / gridDim.y);
  // the first tile's codes travel while the pair table is built (a barrier waits for loads in flight,
  // so they are asked for after the first one)
  TileRegs cur, nxt;
  fetch(cur, c_begin + wave < c_end ? c_begin + wave : c_end - 1, 0);
  for (int i = tid; i < 2 * 256 * kGemmReplicas / 2; i += kGemmBlock) {  // 16-byte stores of two copies each
    const int b = (i / (kGemmReplicas / 2)) & 255, t = i / (256 * (kGemmReplicas / 2));
    const float lo = sm.T[16 * t + (b & 15)], hi = sm.T[16 * t + (b >> 4)];
    reinterpret_cast<float4*>(&sm.pair[0][0][0])[i] = make_float4(lo, hi, lo, hi);
  }
  __syncthreads();
  if (c_begin + wave < c_end) {
    for (int c = c_begin + wave; c < c_end; c += kGemmWaves) {
      const int k0 = lane_cols(c);
      const bool active = k0 < K;
      const int kc = active ? k0 : 0;
      // the chunk's B operands, one contiguous kilobyte per step and x tile (zero beyond M and K)
      uint4 xv[8][MT];
#pragma unroll
      for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int st = 0; st < 8; ++st) xv[st][j] = xpack[((int64_t)(c * 8 + st) * MT + j) * 64 + lane];
      const int c_next = c + kGemmWaves < c_end ? c + kGemmWaves : c;
#pragma unroll
      for (int t = 0; t < kRowsTiles; ++t) {
        // the next tile's codes are on their way while this one is worked on
        asm volatile("" ::: "memory");
        if (t + 1 < kRowsTiles) fetch(nxt, c, t + 1);
        else fetch(nxt, c_next, 0);
        asm volatile("" ::: "memory");
        float s_val[4];
        uint32_t sigma[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {  // block b: columns k0 + 16 b .. + 15, scale number e of the lane's
          constexpr int kW = FMT == 0 ? 8 : 16;
          const int e = (16 * b) >> GS;
          const uint32_t word = FMT == 1 && e >= 2 ? cur.sc.y : cur.sc.x;
          const uint32_t code = (word >> (kW * (FMT == 1 ? e & 1 : e))) & (FMT == 0 ? 0xFFu : 0xFFFFu);
          s_val[b] = gemm_scale_value<FMT>(code, &sigma[b]);
          if (SEL) sigma[b] = (cur.selbyte >> (((kc + 16 * b) >> sshift) & 7)) & 1u;
        }
        // columns k0 + 8 st .. + 7 are four code bytes; their table entries are read one step ahead of
        // the multiplications, so that LDS latency is not waited for byte by byte
        auto lookup = [&](float2 (&p)[4], int st) {
          const uint32_t cw = st < 4 ? (st == 0 ? cur.c0.x : st == 1 ? cur.c0.y : st == 2 ? cur.c0.z : cur.c0.w)
                                     : (st == 4 ? cur.c1.x : st == 5 ? cur.c1.y : st == 6 ? cur.c1.z : cur.c1.w);
          const float2* tab = &sm.pair[sigma[st / 2]][0][rep];
#pragma unroll
          for (int i = 0; i < 4; ++i) p[i] = tab[((cw >> (8 * i)) & 0xFFu) * kGemmReplicas];
        };
        float2 pa[4], pb[4];
        lookup(pa, 0);
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          float2(&p)[4] = (st & 1) ? pb : pa;
          float2(&pn)[4] = (st & 1) ? pa : pb;
          if (st + 1 < 8) lookup(pn, st + 1);
          const float sv = s_val[st / 2];
          uint32_t a32[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) a32[i] = pack_bf16(p[i].x * sv, p[i].y * sv);
          bf16x8 a;
          __builtin_memcpy(&a, a32, 16);
#pragma unroll
          for (int j = 0; j < MT; ++j) {
            bf16x8 bv;
            __builtin_memcpy(&bv, &xv[st][j], 16);
            acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bv, acc[t][j], 0, 0, 0);
          }
        }
        cur = nxt;
      }
    }
  }
  __syncthreads();  // every wavefront is done with the pair table
  // this lane holds D[4q + e][r] of each tile: layer rows 16 t + 4q + e of the block, x row 16 j + r
#pragma unroll
  for (int t = 0; t < kRowsTiles; ++t)
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) sm.part[wave][16 * t + 4 * q + e][16 * j + r] = acc[t][j][e];
  __syncthreads();
  const int rows = r1 - r0;
  for (int i = tid; i < rows * MT * 16; i += kGemmBlock) {
    const int row = i % rows, m = i / rows;
    if (m < M) {
      float sum = 0.0f;
#pragma unroll
      for (int w = 0; w < kGemmWaves; ++w) sum += sm.part[w][row][m];
      float* out = y + (int64_t)m * ldy + r0 + row;
      if (gridDim.y == 1) *out = sum;
      else atomicAdd(out, sum);  // y was cleared by the kernel that packed x
    }
  }
}

// ---------------------------------------------------------------------------------
// Large batches of activation rows (prefill-sized M): a tiled matrix product.  A block of 4
// wavefronts owns 128 layer rows x 128 x rows and walks K in stages of 64 columns.  Per stage
// every thread dequantises 32 weights of one layer row into a bf16 tile in LDS and copies 32
// activations of one x row into a second tile, so the dequantisation is paid once per 128 rows
// of x; then each wavefront multiplies its 64 x 64 quarter (4 x 4 tiles of 16 x 16, two
// k-steps of 32) with operands read from LDS.  A tile row is 64 bf16 = eight 16-byte units;
// unit u of row r is stored at unit u ^ (r & 7), so that the 8 lanes served per clock, which
// read the same unit of 8 consecutive rows, fall into different banks.
constexpr int kTileN = 128, kTileK = 64;  // the tile's x rows (128 or 256) are a template parameter
constexpr int kTiledBlock = 256;
// Copies of the pair table.  Four keep the block's LDS at 64 KB (256 rows of x) or 48 KB (128 rows), so that
// two or three blocks share a compute unit and one block's dequantisation overlaps another's matrix
// instructions; with eight, one 256-row block filled the compute unit alone and ran a third slower.
constexpr int kTiledReplicas = 4;

template <int BM>
struct alignas(16) TiledLds {
  float2 pair[2][256][kTiledReplicas];
  uint4 a[kTileN][8];   // dequantised weights, bf16, swizzled units
  uint4 b[BM][8];       // activations, bf16, swizzled units
  float T[32];
};

// GS: log2 of the scale group size, 5 standing for 32 and more (one scale per 32 columns); SEL:
// selection bits come from the bit array.  Both are template parameters so that every load of a stage
// is unconditional: a load under a branch makes the compiler wait for all loads wherever it waits for one.
template <int FMT, int BM, int GS, bool SEL>
__global__ __launch_bounds__(kTiledBlock) __attribute__((amdgpu_waves_per_eu(BM == 256 ? 2 : 3, BM == 256 ? 2 : 3)))
void gemm_w4a16_tiled_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int M, const uint8_t* __restrict__ codes,
    const void* __restrict__ scales, const uint8_t* __restrict__ sel_bits, int64_t sel_stride,
    const uint16_t* __restrict__ tables_bf16, int N, int K, int gshift, int sshift, float* __restrict__ y,
    int64_t ldy) {
  __shared__ TiledLds<BM> sm;
  constexpr int kXRows = BM / 128;  // x rows a thread copies per stage
  constexpr int kMJ = BM / 32;      // 16-row x tiles per wavefront
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 32) sm.T[tid] = __uint_as_float((uint32_t)tables_bf16[tid] << 16);
  __syncthreads();
  for (int i = tid; i < 2 * 256 * kTiledReplicas / 2; i += kTiledBlock) {  // 16-byte stores of two copies each
    const int b = (i / (kTiledReplicas / 2)) & 255, t = i / (256 * (kTiledReplicas / 2));
    const float lo = sm.T[16 * t + (b & 15)], hi = sm.T[16 * t + (b >> 4)];
    reinterpret_cast<float4*>(&sm.pair[0][0][0])[i] = make_float4(lo, hi, lo, hi);
  }
  __syncthreads();

  const int n_base = blockIdx.x * kTileN, m_base = blockIdx.y * BM;
  // loader role: row of both tiles and which half (32 columns) of the stage
  const int lrow = tid >> 1, half = tid & 1;
  const int n = n_base + lrow;
  const bool has_n = n < N;
  const int Gs = K >> gshift;
  const int rep = lane & (kTiledReplicas - 1);
  // multiplier role: quarter of the block tile
  const int r = lane & 15, q = lane >> 4;
  const int wn = (wave >> 1) * 64, wm = (wave & 1) * (BM / 2);

  f32x4 acc[4][kMJ];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < kMJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // What a thread loads per stage: 16 code bytes, the raw scale codes (taken apart where they are used) and
  // selection byte, four or eight units of 8 activations.  The loads are unconditional, from clamped
  // addresses: a layer row beyond N reads row N - 1 and an x row beyond M reads row M - 1 (their outputs
  // are not stored), the stage after the last reads the last stage again (never used).
  struct StageRegs {
    uint4 cw4;
    uint32_t sc, selbyte;
    u32x4 xv[kXRows * 4];
  };
  const int n_load = has_n ? n : N - 1;
  const uint8_t* crow_load = codes + (int64_t)n_load * (K / 2);
  // x: load j of a thread is unit tid & 7 (8 columns) of row 32 j + tid / 8 of the block's x tile, so that
  // 8 consecutive lanes read one 128-byte line of x (with the weights' mapping, two lanes per row, a load
  // touched 32 lines for 32 bytes each: 2-9 % slower)
  constexpr int kXLoads = kXRows * 4;
  const int xunit = tid & 7, xr0 = tid >> 3;
  const uint16_t* xrow[kXLoads];
#pragma unroll
  for (int j = 0; j < kXLoads; ++j) {
    const int m = m_base + 32 * j + xr0;
    xrow[j] = x + (int64_t)(m < M ? m : M - 1) * ldx + 8 * xunit;
  }
  auto fetch = [&](StageRegs& sr, int k_stage) {
    const int k0 = (k_stage < K ? k_stage : K - kTileK) + 32 * half;
    sr.cw4 = *reinterpret_cast<const uint4*>(crow_load + k0 / 2);
    const int64_t g0 = (int64_t)n_load * Gs + (k0 >> gshift);
    if (GS == 4)
      sr.sc = FMT == 0 ? (uint32_t) * reinterpret_cast<const uint16_t*>(static_cast<const uint8_t*>(scales) + g0)
                       : *reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(scales) + g0);
    else
      sr.sc = FMT == 0 ? (uint32_t) static_cast<const uint8_t*>(scales)[g0]
                       : (uint32_t) static_cast<const uint16_t*>(scales)[g0];
    sr.selbyte = 0;
    if (SEL) sr.selbyte = sel_bits[(int64_t)n_load * sel_stride + ((k0 >> sshift) >> 3)];
  };
  auto fetch_x = [&](StageRegs& sr, int k_stage) {
    const int kx = k_stage < K ? k_stage : K - kTileK;
#pragma unroll
    for (int j = 0; j < kXLoads; ++j) sr.xv[j] = *reinterpret_cast<const u32x4*>(xrow[j] + kx);
  };
  // blockIdx.z: which part of K this block sums (stages of 64 columns; with more than one part the
  // parts are added into y, which the host has cleared)
  const int stages = K / kTileK;
  const int k_begin = (int)((int64_t)stages * blockIdx.z / gridDim.z) * kTileK;
  const int k_end = (int)((int64_t)stages * (blockIdx.z + 1) / gridDim.z) * kTileK;
  StageRegs sr;
  fetch(sr, k_begin);
  fetch_x(sr, k_begin);
  __builtin_assume(K >= kTileK);  // checked by the host
  for (int k_stage = k_begin; k_stage < k_end; k_stage += kTileK) {
    const int k0 = k_stage + 32 * half;
    // the activations go to LDS first and their registers are asked for again at once, so the next
    // stage's x (most of a stage's loads) has this stage's dequantisation and matrix instructions to arrive in
#pragma unroll
    for (int j = 0; j < kXLoads; ++j)  // rows 32 apart have the same row & 7
      *reinterpret_cast<u32x4*>(&sm.b[32 * j + xr0][xunit ^ (xr0 & 7)]) = sr.xv[j];
    asm volatile("" ::: "memory");
    fetch_x(sr, k_stage + kTileK);
    asm volatile("" ::: "memory");
    // dequantise the 32 weights: two 16-column blocks with their scale and selection
    const uint32_t cw[4] = {sr.cw4.x, sr.cw4.y, sr.cw4.z, sr.cw4.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // unit u: columns k0 + 8u .. k0 + 8u + 7
      const int blk = u / 2;
      constexpr uint32_t kScaleMask = FMT == 0 ? 0xFFu : 0xFFFFu;
      const uint32_t sc = GS == 4 ? (sr.sc >> (blk * (FMT == 0 ? 8 : 16))) & kScaleMask : sr.sc;
      uint32_t sigma;
      const float s_val = gemm_scale_value<FMT>(sc, &sigma);
      if (SEL) sigma = (sr.selbyte >> (((k0 + 16 * blk) >> sshift) & 7)) & 1u;
      const float2* tab = &sm.pair[sigma][0][rep];
      uint32_t a32[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t byte = (cw[u] >> (8 * i)) & 0xFFu;
        const float2 p = tab[byte * kTiledReplicas];
        a32[i] = pack_bf16(p.x * s_val, p.y * s_val);
      }
      const int unit = (4 * half + u) ^ (lrow & 7);
      sm.a[lrow][unit] = make_uint4(a32[0], a32[1], a32[2], a32[3]);
    }
    __syncthreads();
    // the next stage's codes and scales are in flight during the matrix instructions (the empty statements keep the
    // compiler from moving them below)
    asm volatile("" ::: "memory");
    fetch(sr, k_stage + kTileK);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      // the four A operands stay in registers; the B operands come one x tile at a time, the next one
      // read from LDS while the current one's four matrix instructions run
      bf16x8 af[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = wn + 16 * i + r;
        const uint4 v = sm.a[row][(4 * ks + q) ^ (row & 7)];
        __builtin_memcpy(&af[i], &v, 16);
      }
      auto b_operand = [&](int j) {
        const int row = wm + 16 * j + r;
        return sm.b[row][(4 * ks + q) ^ (row & 7)];
      };
      uint4 b_cur = b_operand(0);
#pragma unroll
      for (int j = 0; j < kMJ; ++j) {
        uint4 b_next = b_cur;
        if (j + 1 < kMJ) b_next = b_operand(j + 1);
        bf16x8 bv;
        __builtin_memcpy(&bv, &b_cur, 16);
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bv, acc[i][j], 0, 0, 0);
        b_cur = b_next;
      }
    }
    __syncthreads();
  }
  // Lane (r, q) holds D[4q + e][r] of each 16 x 16 tile: layer rows n_base + wn + 16 i + 4q + e, x row
  // m_base + wm + 16 j + r.  Rows of y run along the layer rows, so a wavefront turns each strip of
  // 64 layer rows x 16 x rows through LDS (its own region, over the tiles that are no longer needed; LDS
  // accesses of one wavefront complete in order) and writes, or adds, 64 consecutive floats per x row.
  constexpr int kStageStride = 65;
  static_assert(4 * 16 * kStageStride * sizeof(float) <= sizeof(sm.a) + sizeof(sm.b), "staging fits the tiles");
  float* stage = reinterpret_cast<float*>(&sm.a[0][0]) + wave * (16 * kStageStride);
  const int nn = n_base + wn + lane;
#pragma unroll
  for (int j = 0; j < kMJ; ++j) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) stage[r * kStageStride + 16 * i + 4 * q + e] = acc[i][j][e];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int mr = 0; mr < 16; ++mr) {
      const int mm = m_base + wm + 16 * j + mr;
      const float v = stage[mr * kStageStride + lane];
      if (mm < M && nn < N) {
        if (gridDim.z == 1) y[(int64_t)mm * ldy + nn] = v;
        else atomicAdd(&y[(int64_t)mm * ldy + nn], v);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// y[0 .. M)[0 .. N) = 0, for products whose blocks add their parts into y
__global__ void clear_y_kernel(float* __restrict__ y, int64_t ldy, int M, int N) {
  const int64_t total = (int64_t)M * N;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x)
    y[(e / N) * ldy + e % N] = 0.0f;
}

int log2i(int v) {
  int s = 0;
  while (v > 1) { v >>= 1; ++s; }
  return s;
}

// the few-row kernel (M <= 32): x in registers, one pass over the codes
hipError_t launch_rows(int fmt, int gsh, bool sel, hipStream_t stream, const uint16_t* xp, int64_t ldx, int M,
                       const uint8_t* codes, const void* scales, const uint8_t* bits, int64_t sel_stride,
                       const uint16_t* tables_bf16, int N, int K, int ssh, float* y, int64_t ldy, uint4* xpk,
                       int cus) {
  const int chunks = (K + kChunkCols - 1) / kChunkCols;
  // With few row tiles the chunk sequence is split over blockIdx.y and the parts are added into y,
  // which the packing kernel clears: two blocks per compute unit if every wavefront still gets two
  // chunks, else one (a block pays about 3 us for its table and the final sum), at least one chunk
  // per wavefront.  If blocks of 64 layer rows still leave a quarter of the compute units without a
  // block, the blocks take 32 rows, then 16 (4096 x 4096 at 16 rows: 9.3 us against 10.7; 1024 x 4096:
  // 7.2 against 9.4; with 224 blocks of 64 rows on 256 compute units, 14336 x 4096, smaller blocks
  // were 2 us slower).
  int rt = 4, row_tiles = 0, ksplit = 1;
  for (;; rt /= 2) {
    row_tiles = (N + 16 * rt - 1) / (16 * rt);
    ksplit = (2 * cus + row_tiles / 2) / row_tiles;
    if (ksplit < 1 || chunks / (kGemmWaves * ksplit) < 2) {
      ksplit = (cus + row_tiles / 2) / row_tiles;
      if (ksplit > chunks / kGemmWaves) ksplit = chunks / kGemmWaves;
      if (ksplit < 1) ksplit = 1;
    }
    if (rt == 1 || 4 * row_tiles * ksplit >= 3 * cus) break;
  }
  const int mt = M <= 16 ? 1 : 2;
  const int64_t items = (int64_t)chunks * 8 * mt * 64;
  const unsigned pack_grid = (unsigned)((items + 255) / 256);
  const int clear_n = ksplit > 1 ? N : 0;
  if (mt == 1) pack_x_kernel<1><<<pack_grid, 256, 0, stream>>>(xp, ldx, M, K, chunks, xpk, y, ldy, clear_n);
  else pack_x_kernel<2><<<pack_grid, 256, 0, stream>>>(xp, ldx, M, K, chunks, xpk, y, ldy, clear_n);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)row_tiles, (unsigned)ksplit);
#define AAAC_ROWS_RT(FMT, MT, GS, SEL, RT)                                                                            \
  gemm_w4a16_rows_kernel<FMT, MT, GS, SEL, RT><<<grid, kGemmBlock, 0, stream>>>(xpk, M, codes, scales, bits,           \
                                                                                sel_stride, tables_bf16, N, K, gsh, ssh, \
                                                                                y, ldy)
#define AAAC_ROWS(FMT, MT, GS, SEL)                   \
  do {                                                \
    if (rt == 4) AAAC_ROWS_RT(FMT, MT, GS, SEL, 4);   \
    else if (rt == 2) AAAC_ROWS_RT(FMT, MT, GS, SEL, 2); \
    else AAAC_ROWS_RT(FMT, MT, GS, SEL, 1);           \
  } while (0)
#define AAAC_ROWS_GS(FMT, MT, SEL)                    \
  do {                                                \
    if (gsh == 4) AAAC_ROWS(FMT, MT, 4, SEL);         \
    else if (gsh == 5) AAAC_ROWS(FMT, MT, 5, SEL);    \
    else AAAC_ROWS(FMT, MT, 6, SEL);                  \
  } while (0)
#define AAAC_ROWS_MT(FMT, SEL)                        \
  do {                                                \
    if (mt == 1) AAAC_ROWS_GS(FMT, 1, SEL);           \
    else AAAC_ROWS_GS(FMT, 2, SEL);                   \
  } while (0)
  if (fmt == 0) {
    if (sel) AAAC_ROWS_MT(0, true); else AAAC_ROWS_MT(0, false);
  } else {
    if (sel) AAAC_ROWS_MT(1, true); else AAAC_ROWS_MT(1, false);
  }
#undef AAAC_ROWS_MT
#undef AAAC_ROWS_GS
#undef AAAC_ROWS
#undef AAAC_ROWS_RT
  return hipGetLastError();
}

}  // namespace

size_t gemm_w4a16_workspace(int64_t M, int64_t K) {
  if (M <= 0 || K <= 0) return 0;
  const int64_t chunks = (K + kChunkCols - 1) / kChunkCols;
  const int64_t mt = M <= 16 ? 1 : M <= 32 ? 2 : 4;
  return (size_t)(chunks * 8 * mt * 64 * 16);
}

hipError_t launch_gemm_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                             const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                             int64_t N, int64_t K, int group_size, int sel_size, int fmt, float* y, int64_t ldy,
                             void* ws, hipStream_t stream) {
  if (M == 0 || N == 0) return hipSuccess;
  if (K == 0) {
    for (int64_t m = 0; m < M; ++m) {
      hipError_t e = launch_fill_zero(y + m * ldy, (size_t)N * sizeof(float), stream);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  const int cus = device_compute_units();
  const uint8_t* bits = sel_size < group_size ? sel_bits : nullptr;
  const uint16_t* xp = static_cast<const uint16_t*>(x);
  // Large batches take the tiled kernel, which pays the dequantisation once per 128 or 256 rows of x
  // but walks all of K inside one block; small ones take the few-row kernel, 32 rows of x per pass
  // over the codes.  The choice compares cost models fitted to measurements on MI355X.
  // Tiled: a stage of 64 columns takes a block 1.33 us when it has the compute unit to itself and
  // 1.95 / 2.6 us when two / three blocks share it (128 rows of x; three fit), 2.0 / 3.0 us for one /
  // two blocks of 256 rows; the blocks run in rounds of (compute units x blocks that fit).
  // Few rows: per pass 9 us + 0.2 ps per weight.
  const double work = (double)N * (double)K;
  const int64_t n_tiles = (N + kTileN - 1) / kTileN;
  // With fewer tiles than compute units a block would walk all of K alone at the one-block stage time;
  // K is then split over blockIdx.z (parts added into y with atomics, y cleared first: about 3 us more)
  // until the blocks fill the compute units once, each part keeping at least 8 stages.
  const auto k_parts = [&](int bm) {
    const int64_t tiles = n_tiles * ((M + bm - 1) / bm);
    int64_t parts = cus / tiles;
    if (parts > K / kTileK / 8) parts = K / kTileK / 8;
    return (int)(parts < 1 ? 1 : parts);
  };
  const auto tiled_us = [&](int bm, const double* per_stage, int fit) {
    const int parts = k_parts(bm);
    const int64_t blocks = n_tiles * ((M + bm - 1) / bm) * parts, per_round = (int64_t)cus * fit;
    const int64_t full = blocks / per_round, rem = blocks % per_round;
    double t = (double)full * per_stage[fit - 1];
    if (rem > 0) t += per_stage[(rem + cus - 1) / cus - 1];
    return t * (double)(K / kTileK) / parts + (parts > 1 ? 3.0 : 0.0);
  };
  static const double kNarrowStage[3] = {1.33, 1.95, 2.6}, kWideStage[2] = {2.0, 3.0};
  const double narrow_us = tiled_us(128, kNarrowStage, 3), wide_us = tiled_us(256, kWideStage, 2);
  const double rows_us = (double)((M + 31) / 32) * (9.0 + 0.2e-6 * work);
  if (M > 64 && (narrow_us < rows_us || wide_us < rows_us)) {
    const bool wide = wide_us < narrow_us;
    const int bm = wide ? 256 : 128;
    const int parts = k_parts(bm);
    if (parts > 1) {
      const int64_t want = ((int64_t)M * N + 1023) / 1024;
      clear_y_kernel<<<(unsigned)(want < 2048 ? want : 2048), 256, 0, stream>>>(y, ldy, (int)M, (int)N);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)n_tiles, (unsigned)((M + bm - 1) / bm), (unsigned)parts);
#define AAAC_TILED(FMT, BM, GS, SEL)                                                                              \
  gemm_w4a16_tiled_kernel<FMT, BM, GS, SEL><<<grid, kTiledBlock, 0, stream>>>(                                     \
      xp, ldx, (int)M, codes, scales, bits, sel_stride, tables_bf16, (int)N, (int)K, log2i(group_size),          \
      log2i(sel_size), y, ldy)
#define AAAC_TILED_SEL(FMT, BM, GS)                                   \
  do {                                                                \
    if (bits != nullptr) AAAC_TILED(FMT, BM, GS, true);               \
    else AAAC_TILED(FMT, BM, GS, false);                              \
  } while (0)
#define AAAC_TILED_GS(FMT, BM)                                        \
  do {                                                                \
    if (group_size == 16) AAAC_TILED_SEL(FMT, BM, 4);                 \
    else AAAC_TILED_SEL(FMT, BM, 5);                                  \
  } while (0)
    if (fmt == 0) {
      if (wide) AAAC_TILED_GS(0, 256); else AAAC_TILED_GS(0, 128);
    } else {
      if (wide) AAAC_TILED_GS(1, 256); else AAAC_TILED_GS(1, 128);
    }
#undef AAAC_TILED_GS
#undef AAAC_TILED_SEL
#undef AAAC_TILED
    return hipGetLastError();
  }
  uint4* xpack = static_cast<uint4*>(ws);
  const int gsh = log2i(group_size), ssh = log2i(sel_size);
  for (int64_t m0 = 0; m0 < M; m0 += 32) {  // 32 rows of x at a time (the packed copy is reused)
    const int rows = (int)(M - m0 < 32 ? M - m0 : 32);
    const hipError_t e = launch_rows(fmt, gsh, bits != nullptr, stream, xp + m0 * ldx, ldx, rows, codes, scales, bits,
                                     sel_stride, tables_bf16, (int)N, (int)K, ssh, y + m0 * ldy, ldy, xpack, cus);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace aaac

// The quantised layer applied to a few activation rows (W4A16 decode):
// y[m, n] = sum_k x[m, k] * T_sigma[code[n, k]] * s[n, k / g]  (paper Eq. "pipeline",
// Eq. "aaac_dequant"), reading the 4-bit codes, the scales with the selection bit
// (or the separate selection bits) and the two 16-entry tables; the dequantised
// weights are never written.
//
// Mapping.  A lane owns 32 consecutive columns of a row (16 code bytes, one
// 16-byte load), a wavefront a slab of 2048 columns; it keeps its slice of x in
// registers as fp32 and walks down the rows of its block.  The 8 wavefronts of a
// block take different slabs of the same rows (and different rows when the
// matrix has fewer than 8 slabs).  Two codes are dequantised with one LDS read:
// a 256-entry table per selection value maps a code byte to the pair
// (T[low nibble], T[high nibble]) in fp32, replicated 16 times so that the 16
// lanes served per clock never share a bank.  Within 16 columns the scale is
// constant, so it multiplies the 16-term partial sum once.  Lane sums are reduced
// over 16 lanes with DPP and added to the block's row sums in LDS; one fp32
// store per output.  All arithmetic is fp32 (explicit FMAs); every term
// x * T * s is exact in fp32, so only the order of the additions differs from an
// exact evaluation.
#include "aaac_device.h"
#include "aaac_internal.h"

namespace aaac {

namespace {

constexpr int kGemvBlock = 512;
constexpr int kGemvWaves = kGemvBlock / 64;
constexpr int kSlabCols = 2048;     // columns of a wavefront: 64 lanes x 32 weights
constexpr int kPairReplicas = 16;

struct alignas(16) GemvLds {
  float2 pair[2][256][kPairReplicas];  // [sigma][code byte][replica] = (T[b & 15], T[b >> 4])
  float y[kGemvMaxRows][4];            // row sums of the block
  float T[32];
};

// Unsigned scale value and the selection bit stored in its top bit.
template <int FMT>
__device__ __forceinline__ float scale_value(uint32_t code, uint32_t* sign) {
  if (FMT == 0) {
    *sign = code >> 7;
    return e4m3_value(code & 0x7Fu);
  }
  *sign = code >> 15;
  return __uint_as_float((code & 0x7FFFu) << 16);
}

// FMT: 0 = E4M3 scales (u8), 1 = bf16 scales (u16); G16: scale groups of 16 (a lane's 32
// columns span two groups) or of 32 and more (one group); MB: rows of x held at once.
template <int FMT, bool G16, int MB>
__global__ __launch_bounds__(kGemvBlock) void gemv_w4a16_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int M, const uint8_t* __restrict__ codes,
    const void* __restrict__ scales, const uint8_t* __restrict__ sel_bits, int64_t sel_stride,
    const uint16_t* __restrict__ tables_bf16, int N, int K, int gshift, int sshift, float* __restrict__ y,
    int64_t ldy, int rows_per_block) {
  __shared__ GemvLds sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 32) sm.T[tid] = __uint_as_float((uint32_t)tables_bf16[tid] << 16);
  for (int i = tid; i < kGemvMaxRows * 4; i += kGemvBlock) (&sm.y[0][0])[i] = 0.0f;
  __syncthreads();
  for (int i = tid; i < 2 * 256 * kPairReplicas; i += kGemvBlock) {
    const int b = (i / kPairReplicas) & 255, t = i / (256 * kPairReplicas);
    (&sm.pair[0][0][0])[i] = make_float2(sm.T[16 * t + (b & 15)], sm.T[16 * t + (b >> 4)]);
  }
  __syncthreads();

  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = r0 + rows_per_block < N ? r0 + rows_per_block : N;
  const int slabs = (K + kSlabCols - 1) / kSlabCols;
  const int slabs_at_once = slabs < kGemvWaves ? slabs : kGemvWaves;
  const int row_step = kGemvWaves / slabs_at_once;  // wavefronts that share a slab take rows in turn
  const int row_first = wave / slabs_at_once;
  const int Gs = K >> gshift;
  const int rep = lane & (kPairReplicas - 1);
  const int64_t row_bytes = K / 2;

  if (row_first < row_step) {
    for (int slab = wave % slabs_at_once; slab < slabs; slab += slabs_at_once) {
      const int k0 = slab * kSlabCols + lane * 32;
      const bool active = k0 < K;
      // this lane's slice of x, rows beyond M are zero
      float xr[MB][32];
#pragma unroll
      for (int m = 0; m < MB; ++m) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint4 v = make_uint4(0, 0, 0, 0);
          if (active && m < M) v = *reinterpret_cast<const uint4*>(x + (int64_t)m * ldx + k0 + 8 * q);
          const W8 w = unpack8(v);
#pragma unroll
          for (int p = 0; p < 8; ++p) xr[m][8 * q + p] = w.w[p];
        }
      }
      const uint8_t* cbase = codes + (active ? k0 / 2 : 0);
      const int sidx = active ? k0 >> gshift : 0;   // first scale group of the lane
      const int jsel = active ? k0 >> sshift : 0;   // selection group of the lane's first column
      const int jsel_hi = active ? (k0 + 16) >> sshift : 0;

      uint4 c_next = make_uint4(0, 0, 0, 0);
      uint32_t s_next = 0, b_next = 0;
      auto fetch = [&](int row) {
        c_next = *reinterpret_cast<const uint4*>(cbase + (int64_t)row * row_bytes);
        const int64_t g = (int64_t)row * Gs + sidx;
        if (FMT == 0) {
          if (G16) s_next = *reinterpret_cast<const uint16_t*>(static_cast<const uint8_t*>(scales) + g);
          else s_next = static_cast<const uint8_t*>(scales)[g];
        } else {
          if (G16) s_next = *reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(scales) + g);
          else s_next = static_cast<const uint16_t*>(scales)[g];
        }
        if (sel_bits != nullptr) {
          const uint8_t* sb = sel_bits + (int64_t)row * sel_stride;
          b_next = ((uint32_t)(sb[jsel >> 3] >> (jsel & 7)) & 1u) | (((uint32_t)(sb[jsel_hi >> 3] >> (jsel_hi & 7)) & 1u) << 1);
        }
      };
      int row = r0 + row_first;
      if (active && row < r1) fetch(row);
      for (; row < r1; row += row_step) {
        const uint4 c = c_next;
        const uint32_t sc = s_next, bits = b_next;
        if (active && row + row_step < r1) fetch(row + row_step);
        // the two 16-column halves of the lane: scale value and selection
        float s_val[2];
        uint32_t sigma[2];
        if (G16) {
          const uint32_t width = FMT == 0 ? 8u : 16u, mask = FMT == 0 ? 0xFFu : 0xFFFFu;
          s_val[0] = scale_value<FMT>(sc & mask, &sigma[0]);
          s_val[1] = scale_value<FMT>((sc >> width) & mask, &sigma[1]);
        } else {
          s_val[0] = s_val[1] = scale_value<FMT>(sc, &sigma[0]);
          sigma[1] = sigma[0];
        }
        if (sel_bits != nullptr) { sigma[0] = bits & 1u; sigma[1] = bits >> 1; }
        if (!active) s_val[0] = s_val[1] = 0.0f;
        const uint32_t cw[4] = {c.x, c.y, c.z, c.w};
        float total[MB];
#pragma unroll
        for (int m = 0; m < MB; ++m) total[m] = 0.0f;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const float2* tab = &sm.pair[sigma[h]][0][rep];
          float part[MB];
#pragma unroll
          for (int m = 0; m < MB; ++m) part[m] = 0.0f;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const uint32_t byte = (cw[2 * h + i / 4] >> (8 * (i % 4))) & 0xFFu;
            const float2 t = tab[byte * kPairReplicas];
#pragma unroll
            for (int m = 0; m < MB; ++m) {
              part[m] = __builtin_fmaf(xr[m][16 * h + 2 * i], t.x, part[m]);
              part[m] = __builtin_fmaf(xr[m][16 * h + 2 * i + 1], t.y, part[m]);
            }
          }
#pragma unroll
          for (int m = 0; m < MB; ++m) total[m] = __builtin_fmaf(part[m], s_val[h], total[m]);
        }
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          const float v = group_sum<16>(total[m]);
          if ((lane & 15) == 0) atomicAdd(&sm.y[row - r0][m], v);
        }
      }
    }
  }
  __syncthreads();
  const int rows = r1 - r0;
  for (int i = tid; i < rows * M; i += kGemvBlock) {
    const int m = i / rows, r = i % rows;
    y[(int64_t)m * ldy + r0 + r] = sm.y[r][m];
  }
}

template <int FMT, bool G16>
hipError_t launch_mb(int mb, dim3 grid, hipStream_t stream, const uint16_t* x, int64_t ldx, int M,
                     const uint8_t* codes, const void* scales, const uint8_t* sel_bits, int64_t sel_stride,
                     const uint16_t* tables_bf16, int N, int K, int gshift, int sshift, float* y, int64_t ldy,
                     int rows_per_block) {
  if (mb == 1)
    gemv_w4a16_kernel<FMT, G16, 1><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
                                                                   tables_bf16, N, K, gshift, sshift, y, ldy,
                                                                   rows_per_block);
  else if (mb == 2)
    gemv_w4a16_kernel<FMT, G16, 2><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
                                                                   tables_bf16, N, K, gshift, sshift, y, ldy,
                                                                   rows_per_block);
  else
    gemv_w4a16_kernel<FMT, G16, 4><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
                                                                   tables_bf16, N, K, gshift, sshift, y, ldy,
                                                                   rows_per_block);
  return hipGetLastError();
}

int log2i(int v) {
  int s = 0;
  while (v > 1) { v >>= 1; ++s; }
  return s;
}

}  // namespace

hipError_t launch_gemv_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                             const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                             int64_t N, int64_t K, int group_size, int sel_size, int fmt, float* y, int64_t ldy,
                             hipStream_t stream) {
  if (M == 0 || N == 0) return hipSuccess;
  if (K == 0) {
    for (int64_t m = 0; m < M; ++m) {
      hipError_t e = launch_fill_zero(y + m * ldy, (size_t)N * sizeof(float), stream);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  int cus = 256, dev = 0;
  if (hipGetDevice(&dev) == hipSuccess) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
  }
  // two blocks fit a compute unit; rows per block bounded by the row-sum buffer
  int64_t rpb = (N + 2 * cus - 1) / (2 * cus);
  if (rpb < 8) rpb = 8;
  if (rpb > kGemvMaxRows) rpb = kGemvMaxRows;
  const dim3 grid((unsigned)((N + rpb - 1) / rpb));
  const uint8_t* bits = sel_size < group_size ? sel_bits : nullptr;
  const uint16_t* xp = static_cast<const uint16_t*>(x);
  for (int64_t m0 = 0; m0 < M; m0 += 4) {  // four rows of x at a time
    const int rows = (int)(M - m0 < 4 ? M - m0 : 4);
    const int mb = rows == 1 ? 1 : rows == 2 ? 2 : 4;
    hipError_t e;
#define AAAC_GEMV(FMT, G16)                                                                                  \
  e = launch_mb<FMT, G16>(mb, grid, stream, xp + m0 * ldx, ldx, rows, codes, scales, bits, sel_stride,       \
                          tables_bf16, (int)N, (int)K, log2i(group_size), log2i(sel_size), y + m0 * ldy, ldy, \
                          (int)rpb)
    if (fmt == 0) {
      if (group_size == 16) AAAC_GEMV(0, true); else AAAC_GEMV(0, false);
    } else {
      if (group_size == 16) AAAC_GEMV(1, true); else AAAC_GEMV(1, false);
    }
#undef AAAC_GEMV
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace aaac

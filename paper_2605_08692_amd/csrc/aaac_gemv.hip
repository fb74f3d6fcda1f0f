// The quantised layer applied to a few activation rows (W4A16 decode):
// y[m, n] = sum_k x[m, k] * T_sigma[code[n, k]] * s[n, k / g]  (paper Eq. "pipeline",
// Eq. "aaac_dequant"), reading the 4-bit codes, the scales with the selection bit
// (or the separate selection bits) and the two 16-entry tables; the dequantised
// weights are never written.
//
// Mapping.  A lane owns 32 consecutive columns of a row (16 code bytes, one
// 16-byte load), a wavefront a slab of 2048 columns; it keeps its slice of x in
// registers as packed bf16 pairs, exactly as loaded, and walks down the rows of
// its block, four rows at a time (their loads go out together).  The 8 wavefronts of a block take different
// slabs of the same rows (and different rows when the matrix has fewer than 8
// slabs).  Two codes are dequantised with one LDS read: a 256-entry table per
// selection value maps a code byte to the bf16 pair (T[low nibble], T[high
// nibble]), replicated 32 times so that the 32 lanes served per clock never
// share a bank, and one v_dot2c_f32_bf16 multiplies the pair with the two
// activations and adds to the fp32 partial sum (bf16 products are exact in
// fp32).  Within 16 columns the scale is constant, so it multiplies the partial
// sum of those 16 columns once.  The lane sums of the four rows are reduced over 16 lanes
// together (a transposing DPP reduction) and added to the block's row sums in LDS; one fp32
// store per output.  Every term
// x * T * s is exact in fp32, so only the order and number of the roundings in
// the additions differ from an exact evaluation.
#include <type_traits>
#include "aaac_device.h"
#include "aaac_internal.h"
#include "aaac_stream.h"

namespace aaac {

namespace {

constexpr int kGemvBlock = 512;
constexpr int kGemvWaves = kGemvBlock / 64;
constexpr int kSlabCols = 2048;     // columns of a wavefront: 64 lanes x 32 weights
constexpr int kPairReplicas = 32;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct alignas(16) GemvLds {
  uint32_t pair[2][256][kPairReplicas];  // [sigma][code byte][replica] = bf16 T[b & 15] | bf16 T[b >> 4] << 16
  float y[kGemvMaxRows][8];              // row sums of the block
  uint32_t T[32];                        // the tables' bf16 bit patterns
};

struct RowRegs {  // what a lane loads for one row: 16 code bytes, its scale code(s), selection bytes
  uint4 c;
  uint32_t sc, b0, b1;
};

// acc + a.lo * b.lo + a.hi * b.hi, a and b packed bf16 pairs
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  bf16x2 va, vb;
  __builtin_memcpy(&va, &a, 4);
  __builtin_memcpy(&vb, &b, 4);
  return __builtin_amdgcn_fdot2_f32_bf16(va, vb, acc, false);
}

// Unsigned value of scale number `pos` (0 or 1) among the raw bytes a lane loaded, and the selection
// bit stored in its top bit.  E4M3: the hardware conversion of byte `pos` (exact; this chip's FP8 is the
// OCP E4M3 of the scales: bias 7, subnormals, no infinities; 0x7F, its NaN, is never stored), sign
// dropped.  bf16: the 16 bits moved to the top of an fp32, sign dropped.
template <int FMT, int POS>
__device__ __forceinline__ float scale_value(uint32_t raw, uint32_t* sign) {
  if (FMT == 0) {
    *sign = (raw >> (8 * POS + 7)) & 1u;
    return __builtin_fabsf(__builtin_amdgcn_cvt_f32_fp8((int)raw, POS));
  }
  *sign = (raw >> (16 * POS + 15)) & 1u;
  return __builtin_fabsf(__uint_as_float(POS == 0 ? raw << 16 : raw & 0xFFFF0000u));
}

constexpr int kDppRor4 = 0x124, kDppRor8 = 0x128;  // rotate right by 4 / 8 inside each row of 16 lanes
// Four values per lane, summed over each 16-lane row at once: first the lanes of a pair, then the pairs
// of a quad, exchange the halves they do not keep, so that after two steps lane j of a quad holds the
// quad's sum of one value (j = 0, 1, 2, 3 holds value 0, 2, 1, 3); two rotations add the four quads.
// 11 operations instead of 4 x 4.
__device__ __forceinline__ float sum4_over16(float v0, float v1, float v2, float v3, int lane) {
  const bool odd = lane & 1, hi = lane & 2;
  const float keep0 = odd ? v2 : v0, give0 = odd ? v0 : v2;
  const float keep1 = odd ? v3 : v1, give1 = odd ? v1 : v3;
  const float a0 = keep0 + dpp<kDppXor1>(give0);
  const float a1 = keep1 + dpp<kDppXor1>(give1);
  const float keep = hi ? a1 : a0, give = hi ? a0 : a1;
  float b = keep + dpp<kDppXor2>(give);
  b += dpp<kDppRor8>(b);
  b += dpp<kDppRor4>(b);
  return b;
}

// FMT: 0 = E4M3 scales (u8), 1 = bf16 scales (u16); G16: scale groups of 16 (a lane's 32
// columns span two groups) or of 32 and more (one group); MB: rows of x held at once.
template <int FMT, bool G16, int MB, bool SEL>
__global__ __launch_bounds__(kGemvBlock) __attribute__((amdgpu_waves_per_eu(MB >= 8 ? 2 : 4))) void gemv_w4a16_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int M, const uint8_t* __restrict__ codes,
    const void* __restrict__ scales, const uint8_t* __restrict__ sel_bits, int64_t sel_stride,
    const uint16_t* __restrict__ tables_bf16, int N, int K, int gshift, int sshift, float* __restrict__ y,
    int64_t ldy, int rows_per_block) {
  // rows whose loads go out together; fewer when x takes many registers, to keep two blocks per compute unit
  constexpr int kRowsInFlight = MB >= 4 ? 2 : 4;
  __shared__ GemvLds sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 32) sm.T[tid] = tables_bf16[tid];
  for (int i = tid; i < kGemvMaxRows * 8; i += kGemvBlock) (&sm.y[0][0])[i] = 0.0f;
  __syncthreads();
  // 16-byte stores of four copies each (neighbouring threads write neighbouring 16 bytes): the table
  // is 64 KB per block, and the block's loads start only after it
  for (int i = tid; i < 2 * 256 * kPairReplicas / 4; i += kGemvBlock) {
    const int b = (i / (kPairReplicas / 4)) & 255, t = i / (256 * (kPairReplicas / 4));
    const uint32_t v = sm.T[16 * t + (b & 15)] | (sm.T[16 * t + (b >> 4)] << 16);
    reinterpret_cast<uint4*>(&sm.pair[0][0][0])[i] = make_uint4(v, v, v, v);
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
      // this lane's slice of x as 16 bf16 pairs per row; rows beyond M are zero, and so is the slice of
      // a lane past the last column (its codes and scales read as zero too: it adds 0 * 0)
      uint32_t xp[MB][16];
#pragma unroll
      for (int m = 0; m < MB; ++m) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint4 v = make_uint4(0, 0, 0, 0);
          if (active && m < M) v = *reinterpret_cast<const uint4*>(x + (int64_t)m * ldx + k0 + 8 * q);
          xp[m][4 * q] = v.x; xp[m][4 * q + 1] = v.y; xp[m][4 * q + 2] = v.z; xp[m][4 * q + 3] = v.w;
        }
      }
      const uint8_t* cbase = codes + (active ? k0 / 2 : 0);
      const int sidx = active ? k0 >> gshift : 0;   // first scale group of the lane
      const int jsel = active ? k0 >> sshift : 0;   // selection group of the lane's first column
      const int jsel_hi = active ? (k0 + 16) >> sshift : 0;

      // Rows are taken four at a time: their loads go out together, then they are worked on in
      // order.  (Keeping a second set of four in flight did not pay: the kernel is bound by its
      // vector instructions, and the extra registers cost occupancy.)
      // (loads are unconditional, from clamped addresses: a load under a branch makes the number of loads
      // in flight unknown to the compiler, which then waits for all of them wherever it waits for one; a
      // row past the block's last reads the last row and is not worked on, a lane past the last column
      // reads the row's first bytes and multiplies them with x = 0)
      auto fetch = [&](RowRegs (&rr)[kRowsInFlight], int base) {
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
          const int row0 = base + u * row_step;
          const int row = row0 < r1 ? row0 : r1 - 1;
          rr[u].c = load_once_16(cbase + (int64_t)row * row_bytes);
          const int64_t g = (int64_t)row * Gs + sidx;
          if (FMT == 0) {
            if (G16) rr[u].sc = *reinterpret_cast<const uint16_t*>(static_cast<const uint8_t*>(scales) + g);
            else rr[u].sc = static_cast<const uint8_t*>(scales)[g];
          } else {
            if (G16) rr[u].sc = *reinterpret_cast<const uint32_t*>(static_cast<const uint16_t*>(scales) + g);
            else rr[u].sc = static_cast<const uint16_t*>(scales)[g];
          }
          rr[u].b0 = 0;
          rr[u].b1 = 0;
          if (SEL) {  // the bytes only; the bits are picked out when the row is worked on
            const uint8_t* sb = sel_bits + (int64_t)row * sel_stride;
            rr[u].b0 = sb[jsel >> 3];
            rr[u].b1 = sb[jsel_hi >> 3];
          }
        }
      };
      auto work = [&](const RowRegs (&rr)[kRowsInFlight], int base, auto full) {
        constexpr bool kFull = decltype(full)::value;
        float total[kRowsInFlight][MB];
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
#pragma unroll
          for (int m = 0; m < MB; ++m) total[u][m] = 0.0f;
          if (kFull || base + u * row_step < r1) {
            // the two 16-column halves of the lane: scale value and selection
            float s_val[2];
            uint32_t sigma[2];
            s_val[0] = scale_value<FMT, 0>(rr[u].sc, &sigma[0]);
            if (G16) {
              s_val[1] = scale_value<FMT, 1>(rr[u].sc, &sigma[1]);
            } else {
              s_val[1] = s_val[0];
              sigma[1] = sigma[0];
            }
            if (SEL) {
              sigma[0] = (rr[u].b0 >> (jsel & 7)) & 1u;
              sigma[1] = (rr[u].b1 >> (jsel_hi & 7)) & 1u;
            }
            const uint32_t cw[4] = {rr[u].c.x, rr[u].c.y, rr[u].c.z, rr[u].c.w};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const uint32_t* tab = &sm.pair[sigma[h]][0][rep];
              float part[MB];
#pragma unroll
              for (int m = 0; m < MB; ++m) part[m] = 0.0f;
#pragma unroll
              for (int i = 0; i < 8; ++i) {
                const uint32_t byte = (cw[2 * h + i / 4] >> (8 * (i % 4))) & 0xFFu;
                const uint32_t t = tab[byte * kPairReplicas];
#pragma unroll
                for (int m = 0; m < MB; ++m) part[m] = dot2_bf16(xp[m][8 * h + i], t, part[m]);
              }
#pragma unroll
              for (int m = 0; m < MB; ++m) total[u][m] = __builtin_fmaf(part[m], s_val[h], total[u][m]);
            }
          }
        }
        // lane sums over each 16 lanes, four values at a time; lane j < 4 of the 16 adds value {0, 2, 1, 3}[j]
        const int j = lane & 3, pick = j == 1 ? 2 : j == 2 ? 1 : j;
        const bool adder = (lane & 12) == 0;
        if (kRowsInFlight == 4) {
#pragma unroll
          for (int m = 0; m < MB; ++m) {
            const float v = sum4_over16(total[0][m], total[1 % kRowsInFlight][m], total[2 % kRowsInFlight][m],
                                        total[3 % kRowsInFlight][m], lane);
            const int row = base + pick * row_step;
            if (adder && (kFull || row < r1)) atomicAdd(&sm.y[row - r0][m], v);
          }
        } else {
#pragma unroll
          for (int u = 0; u < kRowsInFlight; ++u) {
            const int row = base + u * row_step;
#pragma unroll
            for (int m4 = 0; m4 < MB / 4; ++m4) {
              const float v = sum4_over16(total[u][(4 * m4) % MB], total[u][(4 * m4 + 1) % MB], total[u][(4 * m4 + 2) % MB],
                                          total[u][(4 * m4 + 3) % MB], lane);
              if (adder && (kFull || row < r1)) atomicAdd(&sm.y[row - r0][4 * m4 + pick], v);
            }
          }
        }
      };
      RowRegs rr[kRowsInFlight];
      int base = r0 + row_first;
      for (; base + (kRowsInFlight - 1) * row_step < r1; base += kRowsInFlight * row_step) {
        fetch(rr, base);
        work(rr, base, std::true_type{});
      }
      if (base < r1) {  // the last, incomplete set of rows
        fetch(rr, base);
        work(rr, base, std::false_type{});
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

template <int FMT, bool G16, bool SEL>
hipError_t launch_mb(int mb, dim3 grid, hipStream_t stream, const uint16_t* x, int64_t ldx, int M,
                     const uint8_t* codes, const void* scales, const uint8_t* sel_bits, int64_t sel_stride,
                     const uint16_t* tables_bf16, int N, int K, int gshift, int sshift, float* y, int64_t ldy,
                     int rows_per_block) {
  if (mb == 8)
    gemv_w4a16_kernel<FMT, G16, 8, SEL><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
                                                                   tables_bf16, N, K, gshift, sshift, y, ldy,
                                                                   rows_per_block);
  else if (mb == 1)
    gemv_w4a16_kernel<FMT, G16, 1, SEL><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
                                                                   tables_bf16, N, K, gshift, sshift, y, ldy,
                                                                   rows_per_block);
  else if (mb == 2)
    gemv_w4a16_kernel<FMT, G16, 2, SEL><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
                                                                   tables_bf16, N, K, gshift, sshift, y, ldy,
                                                                   rows_per_block);
  else
    gemv_w4a16_kernel<FMT, G16, 4, SEL><<<grid, kGemvBlock, 0, stream>>>(x, ldx, M, codes, scales, sel_bits, sel_stride,
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
  const int cus = device_compute_units();
  // two blocks fit a compute unit; rows per block bounded by the row-sum buffer
  int64_t rpb = (N + 2 * cus - 1) / (2 * cus);
  if (rpb < 8) rpb = 8;
  if (rpb > kGemvMaxRows) rpb = kGemvMaxRows;
  const dim3 grid((unsigned)((N + rpb - 1) / rpb));
  const uint8_t* bits = sel_size < group_size ? sel_bits : nullptr;
  const uint16_t* xp = static_cast<const uint16_t*>(x);
  for (int64_t m0 = 0; m0 < M; m0 += 8) {  // eight rows of x at a time
    const int rows = (int)(M - m0 < 8 ? M - m0 : 8);
    const int mb = rows == 1 ? 1 : rows == 2 ? 2 : rows <= 4 ? 4 : 8;
    hipError_t e;
#define AAAC_GEMV(FMT, G16)                                                                                  \
  e = bits != nullptr                                                                                         \
          ? launch_mb<FMT, G16, true>(mb, grid, stream, xp + m0 * ldx, ldx, rows, codes, scales, bits,        \
                                      sel_stride, tables_bf16, (int)N, (int)K, log2i(group_size),            \
                                      log2i(sel_size), y + m0 * ldy, ldy, (int)rpb)                          \
          : launch_mb<FMT, G16, false>(mb, grid, stream, xp + m0 * ldx, ldx, rows, codes, scales, bits, sel_stride, \
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

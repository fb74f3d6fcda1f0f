// Host-side launch interface between the C ABI (aaac_api.hip) and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace aaac {

constexpr int kStripCols = 512;      // columns covered by one wavefront: 64 lanes x 8 bf16
constexpr int kAccStride = 72;       // doubles per accumulator: 32 sum I*x, 32 sum I, objective, pad
constexpr int kAccCopies = 16;       // copies of an accumulator; block b adds to copy b % 16

struct Grid32 {  // initial tables, passed to a kernel by value
  float t[32];
};

// Device-resident state of one layer's fit (lives at the start of its workspace).
struct FitState {
  float tables[2][32];        // T0[16], T1[16] of iteration t at [t & 1], ascending
  double acc[3][kAccCopies][kAccStride];  // sums of iteration t at [t % 3], spread over copies
};

// State of the quantile initialisation (radix select over the keys of the
// normalised weights); lives in the layer's workspace.
constexpr int kQuantSlots = 64;  // distinct key prefixes followed at once = wanted ranks at most
struct QuantState {
  unsigned long long hist1[4096];              // pass 1: counts per top 12 key bits
  unsigned long long hist[kQuantSlots][256];   // passes 2-4: counts per slot and next key bits
  uint32_t cand_count[256];                    // keys that block b of pass 3 put on its part of the candidate list
  uint32_t cand_overflow;                      // non-zero: some key did not fit, pass 4 reads the weights again
  uint32_t cand_pad;
  uint8_t map1[4096];                          // top 12 bits -> slot of pass 2 (0xFF: not followed)
  uint8_t map2[kQuantSlots][256];              // slot of pass 2, next 8 bits -> slot of pass 3
  uint8_t map3[kQuantSlots][256];              // slot of pass 3, next 8 bits -> slot of pass 4
  unsigned long long rank[kQuantSlots];        // rank of each target among the keys that share its prefix
  uint32_t prefix[kQuantSlots];                // key bits found so far
  uint8_t slot[kQuantSlots];
  float grid[32];                              // the resulting tables when they feed a fit directly
};
struct QuantLevel {   // one quantile: value = x[lo] + rem/den * (x[hi] - x[lo]), lo/hi index the target list
  uint32_t rem, den;
  uint8_t lo, hi;
};
struct QuantTargets {  // passed to kernels by value
  int count;                                   // wanted order statistics, <= 64
  unsigned long long rank[kQuantSlots];        // ascending, distinct, counted from 0
  QuantLevel level[32];                        // T0[0..15] then T1[0..15]
};
QuantTargets make_quant_targets(int64_t N, int64_t K);
// rinv: the reciprocal scales of the layer (launch_group_rinv) must be enqueued before.
// cand: room for cand_cap 32-bit keys (the keys that still matter after three passes; see quant_candidates).
hipError_t launch_quantile_init(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size,
                                const float* rinv, void* quant_state, uint32_t* cand, int64_t cand_cap,
                                float* grid_out, hipStream_t stream);
// Keys the candidate list of a layer has room for: one in 32 weights, at least 16384.
inline int64_t quant_candidates(int64_t N, int64_t K) {
  const int64_t n = (N > 0 ? N : 0) * (K > 0 ? K : 0) / 32;
  return n < 16384 ? 16384 : n;
}

// How a layer is cut into blocks for the Lloyd iteration: a block owns a
// rectangle of `strips_per_block` 512-column strips x `rows_per_block` rows.
struct FitPlan {
  int64_t N, K, ldw;
  int group_size;        // weights that share a scale
  int sel_size;          // weights that share a table choice (divides group_size)
  int strips;            // ceil(K / 512)
  int strips_per_block;  // 1, 2, 4, 8 or 16 (wavefront w works on strip w % strips_per_block)
  int strip_groups;      // ceil(strips / strips_per_block)
  int rows_per_block;
  int blocks;            // strip_groups * ceil(N / rows_per_block)
};
// cus: compute units this layer may fill (at least 1).
FitPlan make_fit_plan(int64_t N, int64_t K, int64_t ldw, int group_size, int sel_size, int cus);

// Byte offsets of the parts of a layer's fit workspace; depends on the shape only (no device query).
struct FitLayout {
  size_t off_state, off_rinv, off_sigma, off_quant, off_cand, off_small, bytes;
};
FitLayout fit_layout(int64_t N, int64_t K, int group_size, int sel_size);

// Compute units of the current device, asked from the runtime at every call (256 on MI355X, also the
// value returned when no device can be asked).  Launch paths only: argument checks and workspace
// queries never call it.
int device_compute_units();

struct StatsPlan {
  int strips;             // column groups of 4096
  int token_chunks;       // blocks along the token axis
  int64_t tokens_per_chunk;
  size_t bytes;
};
StatsPlan make_stats_plan(int64_t tokens, int64_t K);

hipError_t launch_act_stats(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                            void* ws, const StatsPlan& plan, hipStream_t stream);
// The same with the partial sums in the library's own device array (no workspace from the caller);
// plan.bytes must not exceed kStaticScratchBytes.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
hipError_t launch_act_stats_static(const void* X, int64_t tokens, int64_t K, int64_t ldx, float* importance,
                                   const StatsPlan& plan, hipStream_t stream);
// One layer of a fit as the launcher sees it (host side).
struct FitTask {
  const void* W;
  int64_t N, K, ldw;
  const float* importance;
  float* tables_f32;
  uint16_t* tables_bf16;
  double* objective_trace;
  void* ws;  // this layer's workspace (fit_layout(...).bytes)
};
constexpr int kMaxFusedLayers = 8;  // layers whose iterations share one launch
// grid == nullptr: the initial tables are the quantiles of each layer's normalised weights.
// Fits n <= kMaxFusedLayers layers together: every pass over the weights is one launch that
// covers all of them.  n_outer assignment passes, each followed by n_inner - 1 passes that
// only refine the tables with the choice frozen.
hipError_t launch_fit_group(const FitTask* tasks, int n, int group_size, int sel_size, int fmt,
                            const Grid32* grid, int n_outer, int n_inner, hipStream_t stream);
hipError_t launch_group_rinv(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, int fmt,
                             float* rinv, hipStream_t stream);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);
// sel_bits: the separate selection bits (row stride sel_stride bytes) when sel_size < group_size,
// null when the choice lives in the sign bit of the scale (sel_size == group_size).
hipError_t launch_encode(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size, int sel_size,
                         int fmt, const float* importance, const uint16_t* tables_bf16, uint8_t* codes,
                         void* scales, uint8_t* sel_bits, int64_t sel_stride, hipStream_t stream);
hipError_t launch_dequant(const uint8_t* codes, const void* scales, const uint8_t* sel_bits,
                          int64_t sel_stride, const uint16_t* tables_bf16, int64_t N, int64_t K,
                          int group_size, int sel_size, int fmt, void* W_hat, int64_t ldo,
                          hipStream_t stream);

// ---- a small layer fitted by one launch (aaac_small.hip)
constexpr int kSmallMaxBlocks = 32;  // blocks that exchange their partial sums
constexpr int kSmallRows = 8;        // rows of a strip that one wavefront keeps in registers
constexpr int kSmallWords = 130;     // 64-bit words per block and pass: 65 sums, two tagged halves each
constexpr size_t kSmallStateBytes = (size_t)2 * kSmallMaxBlocks * kSmallWords * sizeof(unsigned long long);
struct SmallPlan {
  int blocks;  // 0: the layer is too large for this path
  int strips, waves_per_strip, rows_per_wave;
};
SmallPlan make_small_plan(int64_t N, int64_t K);
// grid: the caller's initial tables, or null when grid_dev already holds them (quantile initialisation,
// enqueued before).  grid_dev: 32 floats of device memory; words: kSmallStateBytes of device memory.
hipError_t launch_fit_small(const FitTask& t, const SmallPlan& plan, int group_size, int sel_size, int fmt,
                            const Grid32* grid, float* grid_dev, unsigned long long* words, int n_outer,
                            int n_inner, hipStream_t stream);

constexpr int kGemvMaxRows = 128;  // output rows one block of the W4A16 product accumulates
// y[M x ldy] fp32 = x[M x ldx] bf16 times the quantised layer (codes, scales, tables), K % 32 == 0.
hipError_t launch_gemv_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                             const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                             int64_t N, int64_t K, int group_size, int sel_size, int fmt, float* y, int64_t ldy,
                             hipStream_t stream);

// The same product on the matrix cores, dequantised weights rounded to bf16; K % 64 == 0.
// ws: gemm_w4a16_workspace(M, K) bytes for the copy of x in operand order.
size_t gemm_w4a16_workspace(int64_t M, int64_t K);
hipError_t launch_gemm_w4a16(const void* x, int64_t M, int64_t ldx, const uint8_t* codes, const void* scales,
                             const uint8_t* sel_bits, int64_t sel_stride, const uint16_t* tables_bf16,
                             int64_t N, int64_t K, int group_size, int sel_size, int fmt, float* y, int64_t ldy,
                             void* ws, hipStream_t stream);

}  // namespace aaac

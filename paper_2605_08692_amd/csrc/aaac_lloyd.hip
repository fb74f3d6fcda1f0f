// The fused Lloyd iteration (assignment step + accumulation of the table
// update) for gfx950, and the launcher of a whole fit.
//
// Work mapping: a block of 16 wavefronts (one per compute unit) owns a
// rectangle of 1..16 strips of 512 columns x a range of rows.  A wavefront is
// bound to one strip (64 lanes x 8 bf16; a lane keeps the importances of its 8
// columns in registers) and takes rows of that strip one at a time from a
// counter in LDS, so all wavefronts of a block finish together whatever order
// the hardware favours them in.  A selection group of S weights (the weights
// that share a table choice) is held by S/8 adjacent lanes; the scale group
// (g >= S weights) only decides which reciprocal scale a lane reads.  Up to
// eight layers are fitted by the same launches: the grid is split among them in
// proportion to their sizes and a block first looks up the layer it belongs to.
//
// Nearest entry: the bucket-table search of aaac_search.h.
//
// Passes.  A fit is a sequence of passes over the weights, one launch each: an
// assignment pass (choose the table per group, accumulate the update of both
// tables) followed by n_inner - 1 refinement passes that keep the choice (stored
// as one byte per group by the assignment pass) and only search the chosen table.
//
// Table update.  sum I*x and sum I of the 32 bins go through fp64 LDS atomics
// into a block-wide histogram with 32 slots per bin (slot = lane mod 32); each
// block then adds its 64 sums (and its share of the objective) to a small
// accumulator in global memory with fp64 atomics.  There is no grid-wide
// synchronisation inside a launch: the kernel of iteration t+1 starts by
// reading the accumulator of iteration t, divides, keeps entries whose cell was
// empty and sorts, so every block holds the same tables.  Three accumulators
// rotate (read t-1, add to t, clear t+1), and the tables are double-buffered, so
// a slow block never races with a fast one.  The order of the cross-block adds
// is not fixed: sums can differ between runs in the last bits of an fp64.
#include <cstdlib>
#include <cstring>

#include "aaac_device.h"
#include "aaac_internal.h"
#include "aaac_search.h"

namespace aaac {

namespace {

constexpr int kLloydBlock = kSearchBlock;
constexpr int kLloydWaves = kSearchWaves;

// The small arrays come first so that their LDS offsets fit the 16-bit offset
// field of the DS instructions; the bucket tables go last.
struct alignas(16) LloydLds {
  SearchTables st;
  double hist[2][32][kSlots];             // [0] = sum I*x, [1] = sum I
  double sums[72];
  double red[kLloydWaves];
  double copies[kAccCopies][kAccStride];  // the accumulator copies, staged by 16 wavefronts
  SearchLut sl;
};

// One layer as a block sees it.  Passed to the kernels by value.
struct LayerArgs {
  const uint16_t* W;
  const float* rinv;
  const float* importance;
  FitState* state;
  uint8_t* sigma;         // table choice per group, written by assignment passes (may be null)
  const float* grid_dev;  // initial tables in device memory (null: the grid passed by value)
  double* objective_trace;
  float* tables_f32;      // outputs of the final kernel
  uint16_t* tables_bf16;
  int64_t ldw;
  int N, K;
  int strips, strips_per_block, strip_groups, rows_per_block;
  int block_begin;  // first block of this layer in the grid
  int pad;
};
struct BatchArgs {
  int n;
  int gshift;  // log2 of the scale group size
  LayerArgs layer[kMaxFusedLayers];
};

// fp64 add to global memory, performed by the memory system, visible device-wide.
__device__ __forceinline__ void device_add(double* p, double v) {
  __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Tables of an iteration, computed by ONE wavefront (all 64 lanes call it, no
// block barrier inside): from the accumulated sums of the previous iteration,
// staged in sm.copies (per copy: [0..31] = sum I*x, [32..63] = sum I, [64] =
// objective), divide, keep entries whose cell was empty, sort each table
// (stable); without sums the old tables (lane b passes entry b) are taken as
// they are.  Leaves the tables in sm.st.newtab, the
// objective in sm.sums[64], and fills the search rows, the bucket map parameters
// and the bucket of every midpoint.  Lanes of one wavefront run in lockstep and
// LDS accesses of a wavefront complete in order, so its stores are visible to
// its own later loads; wave_barrier() only keeps the compiler from reordering.
__device__ void wave_make_tables(LloydLds& sm, bool have_sums, float old_entry) {
  const int lane = threadIdx.x & 63;
  float entry = old_entry;  // lane b < 32 holds entry b of the previous tables
  if (have_sums) {
    // Lane l adds element l of the copies: lanes 0..31 the numerators, lanes 32..63 the denominators of
    // the same entries, 16 loads in flight and a fixed tree of additions; lane 0 also adds the objective.
    double v[kAccCopies];
#pragma unroll
    for (int c = 0; c < kAccCopies; ++c) v[c] = sm.copies[c][lane];
    static_assert(kAccCopies == 16, "tree of 16");
#pragma unroll
    for (int w = 1; w < kAccCopies; w *= 2)
#pragma unroll
      for (int c = 0; c < kAccCopies; c += 2 * w) v[c] += v[c + w];
    const double den = __shfl_down(v[0], 32);
    if (lane == 0) {
      double obj = 0.0;
#pragma unroll
      for (int c = 0; c < kAccCopies; ++c) obj += sm.copies[c][64];
      sm.sums[64] = obj;
    }
    if (lane < 32 && den > 0.0) entry = (float)(v[0] / den);
  }
  wave_sort_tables(sm.st, entry);
}


// pass: index of this pass (selects the accumulator and table buffers);
// prev_trace: where the objective found in the previous pass's sums goes (-1: nowhere);
// LANES: lanes per selection group (S / 8);
// ASSIGN: assignment pass (true) or refinement pass with the stored choice (false).
template <int LANES, bool ASSIGN>
__global__ __launch_bounds__(kLloydBlock) void lloyd_iter_kernel(const BatchArgs batch, const int pass,
                                                                 const int prev_trace) {
  const int iteration = pass;
  __shared__ LloydLds sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int li = 0;
  for (int i = 1; i < batch.n; ++i) li = (int)blockIdx.x >= batch.layer[i].block_begin ? i : li;
  const LayerArgs& L = batch.layer[li];
  const uint16_t* __restrict__ W = L.W;
  const float* __restrict__ rinv = L.rinv;
  const float* __restrict__ importance = L.importance;
  FitState* __restrict__ state = L.state;
  uint8_t* __restrict__ sigma_arr = L.sigma;
  double* __restrict__ objective_trace = L.objective_trace;
  const int64_t ldw = L.ldw;
  const int N = L.N, K = L.K, strips = L.strips, strips_per_block = L.strips_per_block,
            strip_groups = L.strip_groups, rows_per_block = L.rows_per_block;
  const int bid = (int)blockIdx.x - L.block_begin;  // block index inside the layer

  // Each wavefront fetches one copy of last iteration's sums (these loads go out
  // first, nothing queues ahead of them) and the histogram is cleared.
  const bool first = iteration == 0;
  float old_entry = 0.0f;
  if (tid < 32) old_entry = state->tables[first ? 0 : (iteration - 1) & 1][tid];
  double acc_val = 0.0, acc_obj = 0.0;
  if (!first && wave < kAccCopies) {
    const double* src = state->acc[(iteration - 1) % 3][wave];
    acc_val = src[lane];
    if (lane == 0) acc_obj = src[64];
  }
  for (int i = tid; i < 2 * 32 * kSlots; i += kLloydBlock) (&sm.hist[0][0][0])[i] = 0.0;

  // this block's rectangle and this wavefront's strip; the first rows are handed out
  // statically (wavefront w takes row w / strips_per_block)
  const int queue = wave % strips_per_block;
  const int strip = (bid % strip_groups) * strips_per_block + queue;
  const int block_r0 = (bid / strip_groups) * rows_per_block;
  const int block_r1 = block_r0 + rows_per_block < N ? block_r0 + rows_per_block : N;
  const int waves_per_queue = kLloydWaves / strips_per_block;
  const int col = strip * kStripCols + lane * 8;
  const bool has_strip = strip < strips;
  const bool active = has_strip && col < K;
  const int G = K / (8 * LANES);       // selection groups per row
  const int Gs = K >> batch.gshift;    // scale groups per row
  const uint16_t* wbase = W + (active ? col : 0);
  const float* rbase = rinv + (active ? col >> batch.gshift : 0);
  int row = has_strip ? block_r0 + wave / strips_per_block : block_r1;
  if (tid < strips_per_block) sm.st.next_row[tid] = block_r0 + waves_per_queue;
  uint8_t* sbase = sigma_arr ? sigma_arr + (active ? col / (8 * LANES) : 0) : nullptr;
  if (!first && wave < kAccCopies) {
    sm.copies[wave][lane] = acc_val;
    if (lane == 0) sm.copies[wave][64] = acc_obj;
  }
  __syncthreads();
  // The first row's weights and the importances are asked for only now: a wait for the sums above
  // would also wait for every load asked for before it, and these come from HBM; they are in flight
  // while the tables and the bucket table are built.
  uint4 v_next = make_uint4(0, 0, 0, 0);
  float r_next = 0.0f;
  uint32_t s_next = 0;  // the stored choice of the next row's group (refinement passes)
  if (active && row < block_r1) {
    v_next = *reinterpret_cast<const uint4*>(wbase + (int64_t)row * ldw);
    r_next = rbase[(int64_t)row * Gs];
    if (!ASSIGN) s_next = sbase[(int64_t)row * G];
  }
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
  // wavefront 0 turns the sums into this iteration's tables
  if (wave == 0) {
    wave_make_tables(sm, !first, old_entry);
    if (bid == 0) {
      if (lane < 32 && !first) state->tables[iteration & 1][lane] = sm.st.newtab[lane];
      if (lane == 32 && prev_trace >= 0 && objective_trace) objective_trace[prev_trace] = sm.sums[64];
      for (int i = lane; i < kAccCopies * kAccStride; i += 64) (&state->acc[(iteration + 1) % 3][0][0])[i] = 0.0;
    }
  }
  __syncthreads();
  build_bucket_table(sm.st, sm.sl);
  const float inv = sm.st.lutpar[0], off = sm.st.lutpar[1];
  const uint32_t rep4 = (uint32_t)(lane & (kReplicas - 1)) * 4u;

  double obj = 0.0;
  double Id[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) Id[p] = (double)Iv[p];
  const uint32_t slot8 = (uint32_t)(lane & (kSlots - 1)) * 8u;
  char* hist = reinterpret_cast<char*>(&sm.hist[0][0][0]);
  while (row < block_r1) {
    const uint4 v = v_next;
    const float r = r_next;
    const uint32_t s_cur = s_next;
    const int cur = row;
    // take the next row of this strip and start its loads before working on this one
    int next = 0;
    if (lane == 0) next = atomicAdd(&sm.st.next_row[queue], 1);
    next = __builtin_amdgcn_readfirstlane(next);
    if (active && next < block_r1) {
      v_next = *reinterpret_cast<const uint4*>(wbase + (int64_t)next * ldw);
      r_next = rbase[(int64_t)next * Gs];
      if (!ASSIGN) s_next = sbase[(int64_t)next * G];
    }
    row = next;
    const uint32_t slot_up = slot8 + kSlots * 8u;  // same slot, one bin further
    if (ASSIGN) {
      Lane8 a;
      assign_fast(unpack8(v), r, Iv, sm.st, sm.sl, inv, off, rep4, a);
      if (__any((a.p0 != a.p0) || (a.p1 != a.p1))) assign_slow(Iv, sm.st, a);
      const float e0 = group_sum<LANES>(a.p0);
      const float e1 = group_sum<LANES>(a.p1);
      const bool sigma = e1 < e0;
      const uint64_t sigma_mask = __builtin_amdgcn_ballot_w64(sigma);
      if (active) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const uint32_t k = sigma ? a.k1[p] : a.k0[p];
          const bool up = __builtin_amdgcn_inverse_ballot_w64((a.m0[p] & ~sigma_mask) | (a.m1[p] & sigma_mask));
          char* h = hist + (k + (up ? slot_up : slot8));
          atomicAdd(reinterpret_cast<double*>(h), Id[p] * (double)a.wn[p]);
          atomicAdd(reinterpret_cast<double*>(h + sizeof(sm.hist[0])), Id[p]);
        }
        if ((lane % LANES) == 0) {
          obj += (double)(sigma ? e1 : e0);
          if (sbase) sbase[(int64_t)cur * G] = sigma ? 1 : 0;
        }
      }
    } else {
      Lane8One a;
      const bool sigma = s_cur != 0;
      assign_one_fast(unpack8(v), r, sm.st, sm.sl, inv, off, rep4 + (sigma ? (uint32_t)sizeof(sm.sl.lut[0]) : 0u), a);
      if (__any(a.check != a.check)) assign_one_slow(sm.st, sigma ? 1 : 0, a);
      if (active) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          const bool up = __builtin_amdgcn_inverse_ballot_w64(a.m[p]);
          char* h = hist + (a.k[p] + (up ? slot_up : slot8));
          atomicAdd(reinterpret_cast<double*>(h), Id[p] * (double)a.wn[p]);
          atomicAdd(reinterpret_cast<double*>(h + sizeof(sm.hist[0])), Id[p]);
        }
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) obj += __shfl_down(obj, o);
  if (lane == 0) sm.red[wave] = obj;
  __syncthreads();
  double* acc = state->acc[iteration % 3][bid % kAccCopies];
  // The kSlots copies of each of the 64 sums: 16 threads per sum, each adds kSlots / 16 neighbouring
  // slots (consecutive lanes read consecutive addresses; one thread per sum walking its slots would
  // put all 64 lanes on the same bank), then the 16 partial sums are added across the lanes.
  {
    static_assert(kLloydBlock == 64 * 16 && kSlots % 16 == 0, "16 threads per sum");
    const int bin = tid >> 4, part = tid & 15;
    const double* h = &sm.hist[0][0][0] + bin * kSlots + part * (kSlots / 16);
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < kSlots / 16; ++k) s += h[k];
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o);
    if (part == 0) device_add(acc + bin, s);
  }
  if (tid == 64) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kLloydWaves; ++w) s += sm.red[w];
    device_add(acc + 64, s);
  }
}

// One block per layer: initial tables, cleared accumulators.
__global__ void init_state_kernel(const BatchArgs batch, const Grid32 grid) {
  FitState* state = batch.layer[blockIdx.x].state;
  const int tid = threadIdx.x;
  const float* dev = batch.layer[blockIdx.x].grid_dev;
  if (tid < 32) state->tables[0][tid] = dev ? dev[tid] : grid.t[tid];
  for (int i = tid; i < 3 * kAccCopies * kAccStride; i += blockDim.x) (&state->acc[0][0][0])[i] = 0.0;
}

// After the last iteration, one block per layer: update the tables from its sums
// and write the outputs.
// passes: number of passes that ran; prev_trace as in lloyd_iter_kernel.
__global__ __launch_bounds__(kLloydBlock) void final_tables_kernel(const BatchArgs batch, const int passes,
                                                                   const int prev_trace) {
  const int iterations = passes;
  __shared__ LloydLds sm;
  const LayerArgs& L = batch.layer[blockIdx.x];
  FitState* __restrict__ state = L.state;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool none = iterations == 0;
  float old_entry = 0.0f;
  if (threadIdx.x < 32) old_entry = state->tables[none ? 0 : (iterations - 1) & 1][threadIdx.x];
  if (!none && wave < kAccCopies) {
    const double* src = state->acc[(iterations - 1) % 3][wave];
    sm.copies[wave][lane] = src[lane];
    if (lane == 0) sm.copies[wave][64] = src[64];
  }
  __syncthreads();
  if (wave != 0) return;
  wave_make_tables(sm, !none, old_entry);
  __builtin_amdgcn_wave_barrier();
  if (lane == 32 && prev_trace >= 0 && L.objective_trace) L.objective_trace[prev_trace] = sm.sums[64];
  if (lane < 32) {
    const float t = sm.st.newtab[lane];
    if (L.tables_f32) L.tables_f32[lane] = t;
    L.tables_bf16[lane] = (uint16_t)bf16_rne(t);
  }
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Layers up to this many (row, strip) pairs take the one-launch path by default.
constexpr int64_t kSmallAutoUnits = 512;

// Index in the objective trace that the sums of pass p carry (-1: none).
int trace_index(int p, int n_inner) { return p >= 0 && p % n_inner == 0 ? p / n_inner : -1; }

template <int LANES>
hipError_t launch_passes(const BatchArgs& batch, int blocks, int n_outer, int n_inner, hipStream_t stream) {
  const int passes = n_outer * n_inner;
  for (int p = 0; p < passes; ++p) {
    const int prev_trace = trace_index(p - 1, n_inner);
    if (p % n_inner == 0)
      lloyd_iter_kernel<LANES, true><<<blocks, kLloydBlock, 0, stream>>>(batch, p, prev_trace);
    else
      lloyd_iter_kernel<LANES, false><<<blocks, kLloydBlock, 0, stream>>>(batch, p, prev_trace);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

int device_compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
    return n;
  return 256;
}

FitLayout fit_layout(int64_t N, int64_t K, int group_size, int sel_size) {
  auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
  FitLayout p;
  p.off_state = 0;
  p.off_rinv = align(sizeof(FitState));
  const size_t groups = (size_t)(N > 0 ? N : 0) * (K / group_size);
  p.off_sigma = p.off_rinv + align(groups * sizeof(float));
  p.off_quant = p.off_sigma + align((size_t)(N > 0 ? N : 0) * (K / sel_size));  // one byte per selection group
  p.off_cand = p.off_quant + align(sizeof(QuantState));
  p.off_small = p.off_cand + align((size_t)quant_candidates(N, K) * sizeof(uint32_t));
  p.bytes = p.off_small + align(kSmallStateBytes);
  return p;
}

FitPlan make_fit_plan(int64_t N, int64_t K, int64_t ldw, int group_size, int sel_size, int cus) {
  FitPlan p;
  p.N = N; p.K = K; p.ldw = ldw; p.group_size = group_size; p.sel_size = sel_size;
  p.strips = (int)ceil_div(K > 0 ? K : 1, kStripCols);
  const int64_t rows = N > 0 ? N : 1;
  // One block of 16 wavefronts per compute unit.  Among 1, 2, 4, 8, 16 strips per
  // block take the choice that keeps the most wavefronts busy: as many blocks as
  // possible without exceeding the compute units (all blocks resident at once, no
  // second round), few wavefronts bound to strips past the last one, and at least
  // one row per wavefront.
  if (cus < 1) cus = 1;
  double best = -1.0;
  for (int spb = 1; spb <= kLloydWaves; spb *= 2) {
    const int64_t groups = ceil_div(p.strips, spb);
    int64_t chunks = cus / groups;  // row chunks per strip group
    if (chunks < 1) chunks = 1;
    const int64_t min_rows = kLloydWaves / spb;
    const int64_t most = rows / min_rows > 0 ? rows / min_rows : 1;
    if (chunks > most) chunks = most;
    const int64_t rpb = ceil_div(rows, chunks);
    const int64_t blocks = groups * ceil_div(rows, rpb);
    const double used = (double)p.strips / (double)(groups * spb);  // wavefronts that have a strip
    const double fill = blocks <= cus ? (double)blocks : (double)cus * cus / (double)blocks;
    const double score = used * fill;
    if (score > best * 1.0000001) {
      best = score;
      p.strips_per_block = spb;
      p.strip_groups = (int)groups;
      p.rows_per_block = (int)rpb;
      p.blocks = (int)blocks;
    }
  }
  return p;
}

hipError_t launch_fit_group(const FitTask* tasks, int n, int group_size, int sel_size, int fmt,
                            const Grid32* grid, int n_outer, int n_inner, hipStream_t stream) {
  const int iterations = n_outer;
  if (n <= 0) return hipSuccess;
  // A single small layer: all passes in one launch (AAAC_FIT_PATH=launches keeps it on the
  // launch-per-pass path, =persistent sends every layer that fits; default: up to kSmallAutoUnits rows of strips).
  if (n == 1 && tasks[0].N > 0 && tasks[0].K > 0) {
    const FitTask& t = tasks[0];
    const SmallPlan sp = make_small_plan(t.N, t.K);
    const char* path = std::getenv("AAAC_FIT_PATH");
    const bool never = path != nullptr && std::strcmp(path, "launches") == 0;
    const bool always = path != nullptr && std::strcmp(path, "persistent") == 0;
    const int64_t units = t.N * (int64_t)sp.strips;
    if (sp.blocks > 0 && !never && (always || units <= kSmallAutoUnits)) {
      const FitLayout lay = fit_layout(t.N, t.K, group_size, sel_size);
      char* base = static_cast<char*>(t.ws);
      QuantState* qs = reinterpret_cast<QuantState*>(base + lay.off_quant);
      if (!grid) {
        float* rinv = reinterpret_cast<float*>(base + lay.off_rinv);
        hipError_t e = launch_group_rinv(t.W, t.N, t.K, t.ldw, group_size, fmt, rinv, stream);
        if (e != hipSuccess) return e;
        e = launch_quantile_init(t.W, t.N, t.K, t.ldw, group_size, rinv, qs,
                                 reinterpret_cast<uint32_t*>(base + lay.off_cand), quant_candidates(t.N, t.K),
                                 qs->grid, stream);
        if (e != hipSuccess) return e;
      }
      return launch_fit_small(t, sp, group_size, sel_size, fmt, grid, qs->grid,
                              reinterpret_cast<unsigned long long*>(base + lay.off_small), n_outer, n_inner, stream);
    }
  }
  // every layer gets its state initialised and its outputs written; only layers
  // that hold weights take part in the iterations
  BatchArgs all = {}, work = {};
  QuantState* quant[kMaxFusedLayers] = {};  // of the layers in `work`
  uint32_t* cand[kMaxFusedLayers] = {};     // their candidate lists
  for (int g = group_size; g > 1; g >>= 1) ++work.gshift;
  double total = 0.0;
  for (int i = 0; i < n; ++i) total += (double)tasks[i].N * (double)tasks[i].K;
  const int cus = device_compute_units();
  // Compute units per layer.  All layers' blocks run side by side in one launch, one block per compute
  // unit, so a pass takes as long as the layer with the most weights per block: start from each layer's
  // share rounded down, then hand the compute units that are left, one step at a time, to the layer whose
  // blocks are the largest (a layer's block count moves in steps: strips x row chunks).
  FitPlan plans[kMaxFusedLayers];
  {
    int budget[kMaxFusedLayers];
    bool stuck[kMaxFusedLayers];
    int used = 0;
    for (int i = 0; i < n; ++i) {
      const FitTask& t = tasks[i];
      const double share = total > 0.0 ? (double)t.N * (double)t.K / total : 0.0;
      budget[i] = n == 1 ? cus : (int)(share * cus);
      if (budget[i] < 1) budget[i] = 1;
      plans[i] = make_fit_plan(t.N, t.K, t.ldw, group_size, sel_size, budget[i]);
      stuck[i] = !(t.N > 0 && t.K > 0);
      used += stuck[i] ? 0 : plans[i].blocks;
    }
    for (int round = 0; round < 64 && used < cus; ++round) {
      int j = -1;
      double worst = 0.0;
      for (int i = 0; i < n; ++i) {
        const double load = (double)tasks[i].N * (double)tasks[i].K / (double)plans[i].blocks;
        if (!stuck[i] && load > worst) { worst = load; j = i; }
      }
      if (j < 0) break;
      bool grown = false;
      for (int extra = 1; extra <= 16 && !grown; ++extra) {
        const FitTask& t = tasks[j];
        const FitPlan q = make_fit_plan(t.N, t.K, t.ldw, group_size, sel_size, budget[j] + extra);
        if (q.blocks > plans[j].blocks && used - plans[j].blocks + q.blocks <= cus) {
          used += q.blocks - plans[j].blocks;
          budget[j] += extra;
          plans[j] = q;
          grown = true;
        }
      }
      if (!grown) stuck[j] = true;
    }
  }
  int blocks = 0;
  for (int i = 0; i < n; ++i) {
    const FitTask& t = tasks[i];
    const FitPlan& p = plans[i];
    const FitLayout lay = fit_layout(t.N, t.K, group_size, sel_size);
    char* base = static_cast<char*>(t.ws);
    LayerArgs a = {};
    a.W = static_cast<const uint16_t*>(t.W);
    a.rinv = reinterpret_cast<const float*>(base + lay.off_rinv);
    a.importance = t.importance;
    a.state = reinterpret_cast<FitState*>(base + lay.off_state);
    a.sigma = n_inner > 1 ? reinterpret_cast<uint8_t*>(base + lay.off_sigma) : nullptr;
    QuantState* qs = reinterpret_cast<QuantState*>(base + lay.off_quant);
    a.grid_dev = grid ? nullptr : qs->grid;
    a.objective_trace = t.objective_trace;
    a.tables_f32 = t.tables_f32;
    a.tables_bf16 = t.tables_bf16;
    a.ldw = t.ldw;
    a.N = (int)t.N;
    a.K = (int)t.K;
    a.strips = p.strips;
    a.strips_per_block = p.strips_per_block;
    a.strip_groups = p.strip_groups;
    a.rows_per_block = p.rows_per_block;
    all.layer[all.n++] = a;
    if (t.N > 0 && t.K > 0) {
      a.block_begin = blocks;
      blocks += p.blocks;
      quant[work.n] = qs;
      cand[work.n] = reinterpret_cast<uint32_t*>(base + lay.off_cand);
      work.layer[work.n++] = a;
    }
  }
  hipError_t e = hipSuccess;
  // reciprocal scales, then (without a caller's grid) the quantile tables, which need them
  if (iterations > 0 || !grid)
    for (int i = 0; i < work.n; ++i) {
      const LayerArgs& a = work.layer[i];
      e = launch_group_rinv(a.W, a.N, a.K, a.ldw, group_size, fmt, const_cast<float*>(a.rinv), stream);
      if (e != hipSuccess) return e;
      if (!grid) {
        e = launch_quantile_init(a.W, a.N, a.K, a.ldw, group_size, a.rinv, quant[i], cand[i],
                                 quant_candidates(a.N, a.K), quant[i]->grid, stream);
        if (e != hipSuccess) return e;
      }
    }
  init_state_kernel<<<all.n, 256, 0, stream>>>(all, grid ? *grid : Grid32{});
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  int done = 0;
  if (work.n > 0 && iterations > 0) {
    switch (sel_size / 8) {
      case 2: e = launch_passes<2>(work, blocks, n_outer, n_inner, stream); break;
      case 4: e = launch_passes<4>(work, blocks, n_outer, n_inner, stream); break;
      case 8: e = launch_passes<8>(work, blocks, n_outer, n_inner, stream); break;
      default: e = launch_passes<16>(work, blocks, n_outer, n_inner, stream); break;
    }
    if (e != hipSuccess) return e;
    done = n_outer * n_inner;
  }
  // layers without weights: the objective is zero and the tables stay the initial grid
  for (int i = 0; i < n; ++i) {
    const FitTask& t = tasks[i];
    if (!(t.N > 0 && t.K > 0) && t.objective_trace && iterations > 0) {
      e = launch_fill_zero(t.objective_trace, sizeof(double) * iterations, stream);
      if (e != hipSuccess) return e;
    }
  }
  if (work.n > 0) {
    final_tables_kernel<<<work.n, kLloydBlock, 0, stream>>>(work, done, trace_index(done - 1, n_inner));
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  BatchArgs empty = {};
  for (int i = 0; i < all.n; ++i)
    if (!(all.layer[i].N > 0 && all.layer[i].K > 0)) empty.layer[empty.n++] = all.layer[i];
  if (empty.n > 0) {
    final_tables_kernel<<<empty.n, kLloydBlock, 0, stream>>>(empty, 0, -1);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace aaac

// Quantile initialisation of the two tables (paper Eq. "init_t0", Eq. "init_t1";
// Alg. 1 steps 4-5) for gfx950: T0[i] and T1[i] are quantiles of all N*K
// normalised weights of a layer, linear interpolation between order statistics.
//
// The order statistics are found exactly, without sorting, by a radix select over
// the order-preserving 32-bit key of w~ = w * (1/s): four passes (12 + 8 + 8 + 4
// key bits), the first three over the weights and the last over the short list of
// keys that the third found still to matter, each a histogram in LDS (merged into
// global memory with 64-bit atomics), each followed by a one-block kernel that
// walks the histogram for all wanted ranks at once.  At most 64 ranks are wanted (32
// quantiles, two neighbouring order statistics each); after a pass, the ranks
// that still share a key prefix share a "slot", and the next pass only counts
// keys whose prefix has a slot, looked up through small tables in LDS.
// Everything here is integer work except the final interpolation, which is a
// fixed sequence of fp64 operations.
#include <type_traits>
#include "aaac_device.h"
#include "aaac_internal.h"

namespace aaac {

namespace {

constexpr int kQBlock = 1024;

// float bits -> unsigned key with the same order as the float values (-0 < +0)
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t b = __float_as_uint(x);
  return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
  return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// Key bits consumed before pass P and the bits it looks at.
template <int PASS> struct PassBits;
template <> struct PassBits<1> { static constexpr int shift = 20, bins = 4096; };
template <> struct PassBits<2> { static constexpr int shift = 12, bins = 256; };
template <> struct PassBits<3> { static constexpr int shift = 4, bins = 256; };
template <> struct PassBits<4> { static constexpr int shift = 0, bins = 16; };

constexpr int kWaveQueue = 512;   // keys a wavefront can hold before it moves them to the candidate list
constexpr int kQueueMove = 256;   // it moves them when it holds this many (looked at once per 32 weights of a lane)

constexpr uint32_t kDeadSlot = kQuantSlots;  // in the LDS copies of the maps: "no wanted rank follows this prefix"

struct QuantLds {
  // the slot maps, 0xFF ("not followed") turned into kDeadSlot; row kDeadSlot of map2 / map3 is all
  // kDeadSlot, so a dead key walks through the maps without a test and is told apart at the end.
  // They come first: their offsets then fit the 16-bit offset field of the LDS instructions.
  uint8_t map1[4096];
  uint8_t map2[kQuantSlots + 1][256];
  uint8_t map3[kQuantSlots + 1][256];
  uint32_t hist[kQuantSlots * 256];  // pass 1 uses the first 4096 counters
  uint32_t queue[kQBlock / 64][kWaveQueue];  // pass 3: the keys each wavefront has found and not yet moved
  uint32_t queued[kQBlock / 64];             // how many
  uint32_t listed;                           // keys the block has moved to its part of the list
};

// four map bytes at once: 0xFF -> kDeadSlot (0x40), slots (< 0x40) unchanged
__device__ __forceinline__ uint32_t dead_slots(uint32_t w) { return w ^ (((w & 0x80808080u) >> 7) * 0xBFu); }

// One histogram pass.  The matrix is cut into 16-byte chunks (8 weights); block b
// owns chunks [b * per_block, (b + 1) * per_block), a thread takes every 1024th.
//
// Pass 3 also writes every key it counts (a key whose first 20 bits some wanted rank still follows:
// one weight in sixty or fewer) to the candidate list, and pass 4 then reads that list instead of
// the weights.  Block b owns part b of the list (no global atomics: thousands of them on one counter
// cost more than the pass); a wavefront collects its keys in an LDS queue of its own (position from an
// LDS atomic, which only the few lanes with such a key execute; positions from a ballot over the
// lanes, with the fill count in a scalar register, measured 5 % slower) and moves them to the block's
// part when it holds 256.  Keys that find the wavefront's queue or the block's part full (many equal
// weights) are dropped and cand_overflow is set: pass 4 then reads the weights like the other passes.
//
// The passes are bound by their vector instructions and by the latency of the dependent LDS reads, so
// the loop over the weights is kept lean: whole batches of four chunks per lane run without any test
// of validity, addresses advance by pointer increments, and the maps need no "not followed" test
// between levels.  CONTIG: the rows follow each other without padding (ldw == K), chunk e is then
// at W + 8 e and its group is numbered like its weights.
template <int PASS, bool CONTIG>
__global__ __launch_bounds__(kQBlock) void quant_hist_kernel(const uint16_t* __restrict__ W,
                                                             const float* __restrict__ rinv, int64_t N, int K,
                                                             int64_t ldw, int gshift, int64_t per_block,
                                                             QuantState* __restrict__ qs, uint32_t* __restrict__ cand,
                                                             const unsigned long long cand_cap) {
  __shared__ QuantLds sm;
  constexpr int kCounters = PASS == 1 ? 4096 : kQuantSlots * PassBits<PASS>::bins;
  constexpr uint32_t kBins = PassBits<PASS>::bins;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < kCounters; i += kQBlock) sm.hist[i] = 0u;
  if (tid < kQBlock / 64) sm.queued[tid] = 0u;
  if (tid == 0) sm.listed = 0u;
  const uint32_t part_cap = (uint32_t)(cand_cap / gridDim.x < 0xFFFFFFFFull ? cand_cap / gridDim.x : 0xFFFFFFFFull);
  uint32_t* const part = cand + (size_t)blockIdx.x * part_cap;
  if (PASS >= 2)
    for (int i = tid; i < 4096 / 4; i += kQBlock)
      reinterpret_cast<uint32_t*>(sm.map1)[i] = dead_slots(reinterpret_cast<const uint32_t*>(qs->map1)[i]);
  if (PASS >= 3) {
    for (int i = tid; i < kQuantSlots * 256 / 4; i += kQBlock)
      reinterpret_cast<uint32_t*>(&sm.map2[0][0])[i] = dead_slots(reinterpret_cast<const uint32_t*>(&qs->map2[0][0])[i]);
    if (tid < 64) reinterpret_cast<uint32_t*>(&sm.map2[kQuantSlots][0])[tid] = kDeadSlot * 0x01010101u;
  }
  if (PASS >= 4) {
    for (int i = tid; i < kQuantSlots * 256 / 4; i += kQBlock)
      reinterpret_cast<uint32_t*>(&sm.map3[0][0])[i] = dead_slots(reinterpret_cast<const uint32_t*>(&qs->map3[0][0])[i]);
    if (tid < 64) reinterpret_cast<uint32_t*>(&sm.map3[kQuantSlots][0])[tid] = kDeadSlot * 0x01010101u;
  }
  __syncthreads();

  // The wavefront's queue (pass 3); move_queue() moves its keys to the block's part of the list when it
  // holds `least` or more.  All 64 lanes call it together.
  uint32_t* const queue = sm.queue[wave];
  bool dropped = false;
  auto move_queue = [&](const uint32_t least) {
    __builtin_amdgcn_wave_barrier();
    uint32_t n = sm.queued[wave];  // one address: the same value in every lane
    if (n < least || n == 0u) return;
    if (n > (uint32_t)kWaveQueue) n = kWaveQueue;
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&sm.listed, n);
    base = __builtin_amdgcn_readfirstlane(base);
    for (uint32_t i = lane; i < n; i += 64)
      if (base + i < part_cap) part[base + i] = queue[i];
    if (base + n > part_cap) dropped = true;
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) sm.queued[wave] = 0u;
    __builtin_amdgcn_wave_barrier();
  };
  // Counts the 8 keys of a lane; all_valid: every key counts, else bit p of valid says whether key p
  // does.  The look-ups of the 8 keys go out together.
  auto count_keys = [&](const uint32_t (&key)[8], auto all_valid, const uint32_t valid) {
    constexpr bool kAll = decltype(all_valid)::value;
    if (PASS == 1) {
#pragma unroll
      for (int p = 0; p < 8; ++p)
        if (kAll || ((valid >> p) & 1u)) atomicAdd(&sm.hist[key[p] >> 20], 1u);
      return;
    }
    uint32_t slot[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) slot[p] = sm.map1[key[p] >> 20];
    if (PASS >= 3) {
#pragma unroll
      for (int p = 0; p < 8; ++p) slot[p] = sm.map2[slot[p]][(key[p] >> 12) & 0xFFu];
    }
    if (PASS >= 4) {
#pragma unroll
      for (int p = 0; p < 8; ++p) slot[p] = sm.map3[slot[p]][(key[p] >> 4) & 0xFFu];
    }
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      if ((kAll || ((valid >> p) & 1u)) && slot[p] != kDeadSlot) {
        atomicAdd(&sm.hist[slot[p] * kBins + ((key[p] >> PassBits<PASS>::shift) & (kBins - 1u))], 1u);
        if (PASS == 3) {
          const uint32_t at = atomicAdd(&sm.queued[wave], 1u);
          if (at < (uint32_t)kWaveQueue) queue[at] = key[p];
          else dropped = true;
        }
      }
    }
  };

  if (PASS == 4 && qs->cand_overflow == 0u) {
    // the candidate list holds every key that can still matter (this block reads the part that the
    // block of the same number wrote: both passes run the same grid); a thread takes 8 keys at a time
    const uint32_t n = qs->cand_count[blockIdx.x];  // <= part_cap
    for (uint32_t i = (uint32_t)tid * 8u; i < n; i += kQBlock * 8u) {
      uint32_t key[8];
#pragma unroll
      for (int p = 0; p < 8; ++p) key[p] = part[i + p < n ? i + p : i];
      const uint32_t left = n - i;  // a key past the end repeats key i and is not counted
      count_keys(key, std::false_type{}, left >= 8u ? 0xFFu : (1u << left) - 1u);
    }
  } else {
    const int cpr = K / 8;  // chunks per row
    const int Gs = K >> gshift;
    const int64_t total = N * (int64_t)cpr;
    const int64_t begin = (int64_t)blockIdx.x * per_block;
    int64_t end = begin + per_block;
    if (end > total) end = total;
    // this lane's chunk: (row, c), the address of its weights; +1024 chunks per step, by increments
    int64_t e = begin + tid;
    int row = (int)(e / cpr);
    int c = (int)(e - (int64_t)row * cpr);
    const uint16_t* wp = W + (int64_t)row * ldw + c * 8;
    const int step_rows = kQBlock / cpr, step_c = kQBlock % cpr;
    const int64_t wstep = (int64_t)step_rows * ldw + step_c * 8, wwrap = ldw - (int64_t)cpr * 8;
    auto advance = [&]() {
      if (CONTIG) {
        wp += (int64_t)kQBlock * 8;
        return;
      }
      row += step_rows;
      c += step_c;
      wp += wstep;
      if (c >= cpr) { c -= cpr; ++row; wp += wwrap; }
    };
    auto scale_index = [&]() -> int64_t {  // of the chunk's reciprocal scale
      if (CONTIG) return ((int64_t)(wp - W)) >> gshift;
      return (int64_t)row * Gs + ((c * 8) >> gshift);
    };
    auto keys_of = [&](const uint4 v, const float r, uint32_t (&key)[8]) {
      const W8 w = unpack8(v);
#pragma unroll
      for (int p = 0; p < 8; ++p) key[p] = order_key(w.w[p] * r);
    };
    // Whole batches: four chunks per lane asked for together (a thread has few chunks, and waiting for
    // each before asking for the next left the pass bound by memory latency), all of them inside the
    // block's range for every lane of the wavefront, so nothing is tested.  The loop runs the same
    // number of times in every lane of a wavefront (in pass 3 the lanes move their keys together).
    constexpr int kBatch = 4;
    int64_t we = begin + (tid & ~63);  // lane 0's chunk
    for (; we + (kBatch - 1) * kQBlock + 63 < end; we += kBatch * kQBlock, e += kBatch * kQBlock) {
      uint4 v[kBatch];
      float r[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        v[u] = *reinterpret_cast<const uint4*>(wp);
        r[u] = rinv[scale_index()];
        advance();
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        uint32_t key[8];
        keys_of(v[u], r[u], key);
        count_keys(key, std::true_type{}, 0xFFu);
      }
      if (PASS == 3) move_queue(kQueueMove);
    }
    // The rest, a chunk at a time; a lane past the end reads the block's first chunk and counts nothing.
    const uint16_t* const wp_first = W + (begin / cpr) * ldw + (begin % cpr) * 8;
    const int64_t r_first = (begin / cpr) * Gs + (((begin % cpr) * 8) >> gshift);
    for (; we < end; we += kQBlock, e += kQBlock) {
      const bool ok = e < end;
      const uint4 v = *reinterpret_cast<const uint4*>(ok ? wp : wp_first);
      const float r = rinv[ok ? scale_index() : r_first];
      advance();
      uint32_t key[8];
      keys_of(v, r, key);
      count_keys(key, std::false_type{}, ok ? 0xFFu : 0u);
      if (PASS == 3) move_queue(kQueueMove);
    }
    if (PASS == 3) {
      move_queue(1u);
      if (dropped) qs->cand_overflow = 1u;
    }
  }
  __syncthreads();
  if (PASS == 3 && tid == 0) qs->cand_count[blockIdx.x] = sm.listed < part_cap ? sm.listed : part_cap;
  unsigned long long* out = PASS == 1 ? qs->hist1 : &qs->hist[0][0];
  for (int i = tid; i < kCounters; i += kQBlock) {
    const uint32_t n = sm.hist[i];
    if (n != 0u) {
      // pass 4 has 16 bins per slot; they are stored at the start of the slot's 256 counters
      const int dst = PASS == 4 ? (i / 16) * 256 + (i % 16) : i;
      atomicAdd(out + dst, (unsigned long long)n);
    }
  }
}

struct SelectLds {
  // pass 1: 4096 prefix sums; later: the staged histograms, bin b of slot s at s * 272 + b + b / 16
  // (runs of 16 bins start in different banks)
  unsigned long long cum[kQuantSlots * 272];
  unsigned long long lane_total[64];
  unsigned long long part[kQuantSlots][16];
  unsigned long long rank[kQuantSlots];
  uint32_t prefix[kQuantSlots];
  uint32_t bin[kQuantSlots];
  uint8_t slot[kQuantSlots];
};

// After histogram pass PASS: for every wanted rank find its bin, narrow the rank,
// hand out the slots of the next pass and clear the counters.  One block.
// After the last pass the keys are complete and the 32 table entries are written.
template <int PASS>
__global__ __launch_bounds__(kQBlock) void quant_select_kernel(QuantState* __restrict__ qs, const QuantTargets tg,
                                                               float* __restrict__ grid_out) {
  __shared__ SelectLds sm;
  const int tid = threadIdx.x, lane = tid & 63;
  const int U = tg.count;
  if (PASS == 1) {
    // exclusive prefix sums of the 4096 counters: 64 lanes x 64 consecutive bins; counter i sits at
    // i + i / 64, so that the lanes' runs start in different banks
    auto pad = [](int i) { return i + (i >> 6); };
    {  // four counters per thread, loaded together
      unsigned long long v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = qs->hist1[tid + k * kQBlock];
#pragma unroll
      for (int k = 0; k < 4; ++k) sm.cum[pad(tid + k * kQBlock)] = v[k];
    }
    __syncthreads();
    if (tid < 64) {  // 16 counters at a time go to registers first, so that the LDS reads overlap
      unsigned long long s = 0;
#pragma unroll
      for (int j0 = 0; j0 < 64; j0 += 16) {
        unsigned long long n[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) n[j] = sm.cum[lane * 65 + j0 + j];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          sm.cum[lane * 65 + j0 + j] = s;
          s += n[j];
        }
      }
      sm.lane_total[lane] = s;
    }
    __syncthreads();
    if (tid < 64) {  // exclusive scan of the 64 lane totals across the first wavefront
      const unsigned long long mine = sm.lane_total[lane];
      unsigned long long incl = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
      }
      sm.lane_total[lane] = incl - mine;
    }
    __syncthreads();
    for (int i = tid; i < 4096; i += kQBlock) sm.cum[pad(i)] += sm.lane_total[i / 64];
    __syncthreads();
    if (tid < U) {  // the last bin whose prefix sum does not exceed the rank
      const unsigned long long rank = tg.rank[tid];
      int lo = 0, hi = 4095;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (sm.cum[pad(mid)] <= rank) lo = mid; else hi = mid - 1;
      }
      sm.bin[tid] = (uint32_t)lo;
      sm.prefix[tid] = (uint32_t)lo;
      sm.rank[tid] = rank - sm.cum[pad(lo)];
    }
    for (int i = tid; i < 4096; i += kQBlock) qs->hist1[i] = 0;
    for (int i = tid; i < 4096 / 4; i += kQBlock) reinterpret_cast<uint32_t*>(qs->map1)[i] = 0xFFFFFFFFu;
  } else {
    constexpr int kBins = PassBits<PASS>::bins;
    // slots are handed out in ascending order, so the last target holds the highest one in use
    const int used = (int)qs->slot[U - 1] + 1;
    {  // the counters of the slots in use, every thread's loads issued together
      constexpr int kPerThread = kQuantSlots * kBins / kQBlock;  // 16 (256 bins) or 1 (16 bins)
      unsigned long long v[kPerThread];
      int at[kPerThread];
#pragma unroll
      for (int k = 0; k < kPerThread; ++k) {
        const int i = tid + k * kQBlock;
        at[k] = (i / kBins) * 256 + (i % kBins);
        v[k] = i < used * kBins ? (&qs->hist[0][0])[at[k]] : 0ull;
      }
#pragma unroll
      for (int k = 0; k < kPerThread; ++k) {
        const int b = at[k] & 255;
        sm.cum[(at[k] >> 8) * 272 + b + (b >> 4)] = v[k];
        if (tid + k * kQBlock < used * kBins) (&qs->hist[0][0])[at[k]] = 0;
      }
    }
    if (tid < U) {
      sm.rank[tid] = qs->rank[tid];
      sm.prefix[tid] = qs->prefix[tid];
      sm.slot[tid] = qs->slot[tid];
    }
    __syncthreads();
    // 16 threads per target: thread j adds up bins [j * kBins/16, (j + 1) * kBins/16) of the
    // target's slot, then the group's first thread walks the 16 partial sums and the one
    // segment that holds the rank
    {
      constexpr int kSeg = kBins / 16;
      const int u = tid >> 4, j = tid & 15;
      const bool live = u < U;
      const unsigned long long* h = sm.cum + (live ? (int)sm.slot[u] : 0) * 272;  // bin b at h[b + b / 16]
      unsigned long long part = 0;
#pragma unroll
      for (int b = 0; b < kSeg; ++b) part += h[j * kSeg + b + ((j * kSeg + b) >> 4)];
      sm.part[u][j] = part;
      __syncthreads();
      if (live && j == 0) {
        const unsigned long long rank = sm.rank[u];
        unsigned long long below = 0, taken = 0;
        int seg = 0;
        for (int k = 0; k < 16; ++k) {  // the last segment whose prefix sum does not exceed the rank
          if (below <= rank) { seg = k; taken = below; }
          below += sm.part[u][k];
        }
        below = taken;
        int bin = seg * kSeg;
        for (int b = 0; b < kSeg; ++b) {  // and the last such bin inside it
          if (below <= rank) { bin = seg * kSeg + b; taken = below; }
          below += h[seg * kSeg + b + ((seg * kSeg + b) >> 4)];
        }
        sm.bin[u] = (uint32_t)bin;
        sm.prefix[u] = (sm.prefix[u] << (kBins == 16 ? 4 : 8)) | (uint32_t)bin;
        sm.rank[u] = rank - taken;
      }
    }
    for (int i = tid; i < kQuantSlots * 256 / 4; i += kQBlock) {
      if (PASS == 2) reinterpret_cast<uint32_t*>(&qs->map2[0][0])[i] = 0xFFFFFFFFu;
      if (PASS == 3) reinterpret_cast<uint32_t*>(&qs->map3[0][0])[i] = 0xFFFFFFFFu;
    }
  }
  __syncthreads();
  if (PASS < 4) {
    // ranks are ascending, so prefixes are too: a new slot starts where the prefix changes.
    // The targets are the lanes of the first wavefront; targets that share a prefix write
    // the same slot to the same map entry.
    if (tid < 64) {
      const bool live = tid < U;
      const bool opens = live && (tid == 0 || sm.prefix[tid] != sm.prefix[tid - 1]);
      const uint64_t opened = __builtin_amdgcn_ballot_w64(opens);
      if (live) {
        const uint8_t s = (uint8_t)(__builtin_popcountll(opened & (~0ull >> (63 - tid))) - 1);
        if (PASS == 1) qs->map1[sm.bin[tid]] = s;
        if (PASS == 2) qs->map2[sm.slot[tid]][sm.bin[tid]] = s;
        if (PASS == 3) qs->map3[sm.slot[tid]][sm.bin[tid]] = s;
        qs->slot[tid] = s;
        qs->rank[tid] = sm.rank[tid];
        qs->prefix[tid] = sm.prefix[tid];
      }
    }
  } else if (tid < 32) {
    // the prefixes are the full keys now: interpolate the 32 quantiles
    const QuantLevel q = tg.level[tid];
    double v = (double)key_value(sm.prefix[q.lo]);
    if (q.rem != 0u) {
      const double frac = (double)q.rem / (double)q.den;
      v = v + frac * ((double)key_value(sm.prefix[q.hi]) - v);
    }
    grid_out[tid] = (float)v + 0.0f;  // a zero is stored as +0
  }
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

QuantTargets make_quant_targets(int64_t N, int64_t K) {
  QuantTargets tg = {};
  const unsigned __int128 last = (unsigned __int128)N * (unsigned __int128)K - 1;
  unsigned long long lo[32], rem[32];
  for (int t = 0; t < 2; ++t)
    for (int i = 0; i < 16; ++i) {
      const unsigned __int128 num = t == 0 ? i : 15 + 29 * i, den = t == 0 ? 15 : 450;
      const unsigned __int128 pos = num * last;
      lo[16 * t + i] = (unsigned long long)(pos / den);
      rem[16 * t + i] = (unsigned long long)(pos % den);
      tg.level[16 * t + i].rem = (uint32_t)rem[16 * t + i];
      tg.level[16 * t + i].den = (uint32_t)den;
    }
  // the wanted ranks, ascending and without repeats (levels ascend inside a table, the two tables interleave)
  unsigned long long all[64];
  int n = 0;
  for (int q = 0; q < 32; ++q) {
    all[n++] = lo[q];
    if (rem[q] != 0) all[n++] = lo[q] + 1;
  }
  for (int i = 1; i < n; ++i) {  // insertion sort
    const unsigned long long v = all[i];
    int j = i - 1;
    while (j >= 0 && all[j] > v) { all[j + 1] = all[j]; --j; }
    all[j + 1] = v;
  }
  int U = 0;
  for (int i = 0; i < n; ++i)
    if (U == 0 || tg.rank[U - 1] != all[i]) tg.rank[U++] = all[i];
  tg.count = U;
  auto find = [&](unsigned long long r) {
    for (int u = 0; u < U; ++u)
      if (tg.rank[u] == r) return u;
    return 0;
  };
  for (int q = 0; q < 32; ++q) {
    tg.level[q].lo = (uint8_t)find(lo[q]);
    tg.level[q].hi = (uint8_t)(rem[q] != 0 ? find(lo[q] + 1) : tg.level[q].lo);
  }
  return tg;
}

hipError_t launch_quantile_init(const void* W, int64_t N, int64_t K, int64_t ldw, int group_size,
                                const float* rinv, void* quant_state, uint32_t* cand, int64_t cand_cap,
                                float* grid_out, hipStream_t stream) {
  QuantState* qs = static_cast<QuantState*>(quant_state);
  const uint16_t* Wp = static_cast<const uint16_t*>(W);
  int gshift = 0;
  for (int g = group_size; g > 1; g >>= 1) ++gshift;
  const QuantTargets tg = make_quant_targets(N, K);
  // counters start at zero (the select kernels clear them again after each pass)
  hipError_t e = launch_fill_zero(qs, offsetof(QuantState, map1), stream);
  if (e != hipSuccess) return e;
  const int64_t chunks = N * (K / 8);
  int64_t blocks = ceil_div(chunks, 4 * kQBlock);  // at least four chunks per thread
  if (blocks > 256) blocks = 256;  // one block per compute unit: every block merges its counters with global atomics
  const int64_t per_block = ceil_div(ceil_div(chunks, blocks), kQBlock) * kQBlock;
  blocks = ceil_div(chunks, per_block);
#define AAAC_QPASS(P)                                                                                          \
  if (ldw == K)                                                                                                \
    quant_hist_kernel<P, true><<<(unsigned)blocks, kQBlock, 0, stream>>>(Wp, rinv, N, (int)K, ldw, gshift, per_block, \
                                                                         qs, cand, (unsigned long long)cand_cap); \
  else                                                                                                         \
    quant_hist_kernel<P, false><<<(unsigned)blocks, kQBlock, 0, stream>>>(Wp, rinv, N, (int)K, ldw, gshift, per_block, \
                                                                          qs, cand, (unsigned long long)cand_cap); \
  if ((e = hipGetLastError()) != hipSuccess) return e;                                                         \
  quant_select_kernel<P><<<1, kQBlock, 0, stream>>>(qs, tg, grid_out);                                         \
  if ((e = hipGetLastError()) != hipSuccess) return e;
  AAAC_QPASS(1)
  AAAC_QPASS(2)
  AAAC_QPASS(3)
  AAAC_QPASS(4)
#undef AAAC_QPASS
  return hipSuccess;
}

}  // namespace aaac

// Nearest-entry search shared by the Lloyd iteration and the encode kernel.
//
// The index of a normalised weight x in an ascending 16-entry table is the number
// of midpoints strictly below x.  Instead of 15 compares per table, a block
// builds (once per launch, in LDS) a bucket table over the range of the
// midpoints: bucket(x) is a monotone function of x computed with one fused
// multiply-add and a clamp, and for every bucket and table it stores i = number
// of midpoints whose bucket is lower.  If at most one midpoint falls into the
// bucket itself, that midpoint is m[i], and index = i + (x > m[i]) with
// reconstruction T[i] or T[i+1]: one 16-byte LDS read {m[i], T[i], T[i+1], bin}
// and one compare.  A bucket holding two or more midpoints of a table points at a
// poisoned row (NaN entries); the NaN reaches the lane's error sum, the wavefront
// notices and redoes that row with the plain 15-compare count.  Results are
// identical either way.
//
// The bucket table is replicated 32 times (one copy per LDS bank column) so
// that data-dependent look-ups do not conflict; the 16 rows of {m, T, T, bin}
// of a table need no replication because distinct rows already sit in distinct
// banks.  A pass that searches one table per weight (the table its group chose
// earlier) and needs no reconstruction value reads 8-byte rows {m, bin}
// instead: half the LDS cycles, and the two tables' rows then lie in different
// halves of the banks, so lanes that search different tables do not collide
// (with the 16-byte rows, which fill all banks once per table, they did: 9 % of
// that pass's LDS cycles).
#pragma once
#include <cstddef>
#include "aaac_device.h"

namespace aaac {

constexpr int kSearchBlock = 1024;  // threads per block of the kernels that use the search
constexpr int kSearchWaves = kSearchBlock / kWave;
constexpr int kBuckets = 256;
constexpr int kReplicas = 32;
constexpr int kSlots = 32;          // histogram slots per bin; a bin is kSlots * 8 bytes

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct alignas(16) SearchRow {  // 16 bytes: one LDS read serves a compare, a select and the bin address
  float thr;        // midpoint m[i] (+inf for i >= 15)
  float lo, hi;     // T[i], T[i+1]
  uint32_t bin;     // (16 * table + i) * kSlots * 8: byte offset of the bin in a histogram
};

struct alignas(8) SearchRow8 {  // the same row for a search that needs the index only
  float thr;        // midpoint m[i] (+inf for i = 15, NaN in the poisoned row)
  uint32_t bin;
};

// Small search state; keep it at the start of the block's LDS so that its
// offsets fit the 16-bit offset field of the DS instructions.
// A bucket entry is the byte offset of its row from row[0][0]: 16 i for T0, 256 + 16 i for T1,
// 512 / 528 for the two poisoned rows; half of it is the offset of the 8-byte row from row8[0][0].
struct alignas(16) SearchTables {
  SearchRow row[2][16];         // rows 0..15 of T0, then of T1
  SearchRow poison[2];          // NaN entries; must follow row[][]
  SearchRow8 row8[2][16];
  SearchRow8 poison8[2];        // must follow row8[][]
  float lutpar[4];              // inv, off of bucket_row()
  int mid_bucket[2][16];        // bucket of each midpoint
  float newtab[32];             // the tables T0[16], T1[16], ascending
  int next_row[kSearchWaves];   // per strip of the block: next row to hand out
  uint32_t entry[2][kBuckets];  // unreplicated bucket entries while building
};

// REPL: copies of every bucket entry (a power of two up to 32).  32 copies make the data-dependent
// look-ups of a wavefront conflict-free; kernels that see only a few rows per launch take fewer
// copies, because building the table then costs more than the conflicts.
template <int REPL>
struct alignas(16) SearchLutT {
  // per table: byte offset of the candidate row from row[0][0] (16 * row, plus
  // sizeof(row[0]) for table 1), replicated
  uint32_t lut[2][kBuckets * REPL];
};
using SearchLut = SearchLutT<kReplicas>;

// Monotone map from a normalised weight to the byte offset of its bucket's
// replica block (bucket * 128): integer part of fma(x, inv, off), read from the
// mantissa of a float in [2^23, 2^24), clamped.
__device__ __forceinline__ uint32_t bucket_row(float x, float inv, float off) {
  float t = __builtin_fmaf(x, inv, off);
  t = __builtin_amdgcn_fmed3f(t, 8388608.0f, 8388608.0f + 32767.0f);
  return __float_as_uint(t) & 0x7F80u;
}
// The same as the byte offset of the bucket's first copy in a table of REPL copies (bucket * 4 * REPL).
template <int REPL>
__device__ __forceinline__ uint32_t bucket_offset(float x, float inv, float off) {
  static_assert(REPL == 1 || REPL == 2 || REPL == 4 || REPL == 8 || REPL == 16 || REPL == 32, "copies per bucket");
  const uint32_t b = bucket_row(x, inv, off);
  return REPL == 32 ? b : b / (32u / REPL);
}

__device__ __forceinline__ float tree8(const float (&u)[8]) {
  return ((u[0] + u[1]) + (u[2] + u[3])) + ((u[4] + u[5]) + (u[6] + u[7]));
}

// Per-lane result of the assignment of 8 weights.
struct Lane8 {
  float wn[8];
  uint32_t k0[8], k1[8];  // bin field of the candidate row under T0 / T1
  uint64_t m0[8], m1[8];  // lane masks: weight lies above that row's midpoint, index is one higher
  float p0, p1;           // the lane's partial error sums
};

template <int REPL>
__device__ __forceinline__ void assign_fast(const W8& x, float r, const float (&Iv)[8], const SearchTables& st,
                                            const SearchLutT<REPL>& sl, float inv, float off, uint32_t rep4, Lane8& a) {
  float u0[8], u1[8];
  const char* lut = reinterpret_cast<const char*>(sl.lut);
  const char* rows = reinterpret_cast<const char*>(st.row[0]);
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = x.w[p] * r;
    a.wn[p] = wn;
    const char* e = lut + (bucket_offset<REPL>(wn, inv, off) | rep4);
    const uint32_t a0 = *reinterpret_cast<const uint32_t*>(e);
    const uint32_t a1 = *reinterpret_cast<const uint32_t*>(e + sizeof(sl.lut[0]));
    // each row is one 16-byte DS read; all four fields are used, so it is not narrowed
    // (12-byte or split reads of these rows are several times slower)
    const f32x4 s0 = *reinterpret_cast<const f32x4*>(rows + a0);
    const f32x4 s1 = *reinterpret_cast<const f32x4*>(rows + a1);
    const bool c0 = wn > s0.x;
    const bool c1 = wn > s1.x;
    const float d0 = wn - (c0 ? s0.z : s0.y);
    const float d1 = wn - (c1 ? s1.z : s1.y);
    a.k0[p] = __float_as_uint(s0.w);
    a.k1[p] = __float_as_uint(s1.w);
    a.m0[p] = __builtin_amdgcn_ballot_w64(c0);
    a.m1[p] = __builtin_amdgcn_ballot_w64(c1);
    const float q0 = d0 * d0;
    const float q1 = d1 * d1;
    u0[p] = Iv[p] * q0;
    u1[p] = Iv[p] * q1;
  }
  a.p0 = tree8(u0);
  a.p1 = tree8(u1);
}

// The same as assign_fast with the look-ups of the 8 weights issued together (all bucket reads, then all
// row reads, then the arithmetic): more registers, but a wavefront that has the SIMD almost to itself
// does not wait for one LDS read after the other.
template <int REPL>
__device__ __forceinline__ void assign_fast_batched(const W8& x, float r, const float (&Iv)[8], const SearchTables& st,
                                                    const SearchLutT<REPL>& sl, float inv, float off, uint32_t rep4,
                                                    Lane8& a) {
  float u0[8], u1[8];
  const char* lut = reinterpret_cast<const char*>(sl.lut);
  const char* rows = reinterpret_cast<const char*>(st.row[0]);
  uint32_t a0[8], a1[8];
  f32x4 s0[8], s1[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    a.wn[p] = x.w[p] * r;
    const char* e = lut + (bucket_offset<REPL>(a.wn[p], inv, off) | rep4);
    a0[p] = *reinterpret_cast<const uint32_t*>(e);
    a1[p] = *reinterpret_cast<const uint32_t*>(e + sizeof(sl.lut[0]));
  }
  asm volatile("" ::: "memory");
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    s0[p] = *reinterpret_cast<const f32x4*>(rows + a0[p]);
    s1[p] = *reinterpret_cast<const f32x4*>(rows + a1[p]);
  }
  asm volatile("" ::: "memory");
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = a.wn[p];
    const bool c0 = wn > s0[p].x;
    const bool c1 = wn > s1[p].x;
    const float d0 = wn - (c0 ? s0[p].z : s0[p].y);
    const float d1 = wn - (c1 ? s1[p].z : s1[p].y);
    a.k0[p] = __float_as_uint(s0[p].w);
    a.k1[p] = __float_as_uint(s1[p].w);
    a.m0[p] = __builtin_amdgcn_ballot_w64(c0);
    a.m1[p] = __builtin_amdgcn_ballot_w64(c1);
    const float q0 = d0 * d0;
    const float q1 = d1 * d1;
    u0[p] = Iv[p] * q0;
    u1[p] = Iv[p] * q1;
  }
  a.p0 = tree8(u0);
  a.p1 = tree8(u1);
}

// Same result by counting all 15 midpoints (rows that met a poisoned bucket).
__device__ __forceinline__ void assign_slow(const float (&Iv)[8], const SearchTables& st, Lane8& a) {
  float u0[8], u1[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = a.wn[p];
    int i0 = 0, i1 = 0;
    for (int j = 0; j < 15; ++j) {
      i0 += wn > st.row[0][j].thr ? 1 : 0;
      i1 += wn > st.row[1][j].thr ? 1 : 0;
    }
    a.k0[p] = st.row[0][i0].bin;
    a.k1[p] = st.row[1][i1].bin;
    a.m0[p] = 0;
    a.m1[p] = 0;
    const float d0 = wn - st.row[0][i0].lo;
    const float d1 = wn - st.row[1][i1].lo;
    const float q0 = d0 * d0;
    const float q1 = d1 * d1;
    u0[p] = Iv[p] * q0;
    u1[p] = Iv[p] * q1;
  }
  a.p0 = tree8(u0);
  a.p1 = tree8(u1);
}

// One table only (r_off = 0 for T0, sizeof(lut[0]) for T1, per lane): bin field of the
// candidate row, the lane mask of "one higher", and a value that is NaN iff some
// weight met a poisoned bucket.
struct Lane8One {
  float wn[8];
  uint32_t k[8];
  uint64_t m[8];
  float check;
};

template <int REPL>
__device__ __forceinline__ void assign_one_fast(const W8& x, float r, const SearchTables& st, const SearchLutT<REPL>& sl,
                                                float inv, float off, uint32_t rep4_table, Lane8One& a) {
  const char* lut = reinterpret_cast<const char*>(sl.lut);
  const char* rows = reinterpret_cast<const char*>(st.row8[0]);
  // a row's midpoint is finite or +inf, the poisoned row's NaN: the sum is NaN iff some weight met it
  float check = 0.0f;
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = x.w[p] * r;
    a.wn[p] = wn;
    const uint32_t e = *reinterpret_cast<const uint32_t*>(lut + (bucket_offset<REPL>(wn, inv, off) | rep4_table));
    uint2 s = *reinterpret_cast<const uint2*>(rows + (e >> 1));  // {m[i], bin}
    // (both halves are wanted here: left alone the compiler reads them apart, the bin later, under the
    // branch that uses it, and two 4-byte reads cost the LDS what the 16-byte row did)
    asm volatile("" : "+v"(s.x), "+v"(s.y));
    const float thr = __uint_as_float(s.x);
    a.k[p] = s.y;
    a.m[p] = __builtin_amdgcn_ballot_w64(wn > thr);
    check += thr;
  }
  a.check = check;
}

__device__ __forceinline__ void assign_one_slow(const SearchTables& st, int table, Lane8One& a) {
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const float wn = a.wn[p];
    int i = 0;
    for (int j = 0; j < 15; ++j) i += wn > st.row[table][j].thr ? 1 : 0;
    a.k[p] = st.row[table][i].bin;
    a.m[p] = 0;
  }
  a.check = 0.0f;
}

// Search rows, bucket map parameters and the bucket of every midpoint from the
// tables in st.newtab.  Called by ONE wavefront (all 64 lanes), no block barrier
// inside: lanes of a wavefront run in lockstep and its LDS accesses complete in
// order, so its stores are visible to its own later loads; wave_barrier() only
// keeps the compiler from reordering.
__device__ __forceinline__ void wave_make_rows(SearchTables& st) {
  const int lane = threadIdx.x & 63;
  __builtin_amdgcn_wave_barrier();
  static_assert(offsetof(SearchTables, poison) == 512 && offsetof(SearchTables, poison8) - offsetof(SearchTables, row8) == 256,
                "bucket entries address the rows by these offsets");
  if (lane < 32) {
    const int r = lane >> 4, i = lane & 15;
    const float* T = st.newtab + 16 * r;
    SearchRow s;
    s.thr = i < 15 ? 0.5f * (T[i] + T[i + 1]) : __builtin_inff();
    s.lo = T[i];
    s.hi = i < 15 ? T[i + 1] : __builtin_nanf("");
    s.bin = (uint32_t)(16 * r + i) * (kSlots * 8u);
    st.row[r][i] = s;
    st.row8[r][i] = SearchRow8{s.thr, s.bin};
  } else if (lane < 34) {
    const int r = lane - 32;
    const uint32_t bin = (uint32_t)(16 * r) * (kSlots * 8u);
    st.poison[r] = SearchRow{__builtin_inff(), __builtin_nanf(""), __builtin_nanf(""), bin};
    st.poison8[r] = SearchRow8{__builtin_nanf(""), bin};
  }
  __builtin_amdgcn_wave_barrier();
  if (lane < 32) {
    const float lo = fminf(st.row[0][0].thr, st.row[1][0].thr);
    const float hi = fmaxf(st.row[0][14].thr, st.row[1][14].thr);
    const float range = fmaxf(hi - lo, 1e-20f);
    const float inv = (128.0f * (kBuckets - 2)) / range;  // buckets 1..254 span [lo, hi]
    const float off = (128.0f - lo * inv) + 8388608.0f;
    if (lane == 0) {
      st.lutpar[0] = inv;
      st.lutpar[1] = off;
    }
    const int r = lane >> 4, j = lane & 15;
    st.mid_bucket[r][j] = j < 15 ? (int)(bucket_row(st.row[r][j].thr, inv, off) >> 7) : kBuckets;
  }
}

// Bucket table from the midpoint buckets, replicated; all BLOCK threads of the block
// (at least 2 * kBuckets) call it after wave_make_rows() and a barrier.  Ends with a barrier.
template <int REPL, int BLOCK = kSearchBlock>
__device__ __forceinline__ void build_bucket_table(SearchTables& st, SearchLutT<REPL>& sl) {
  static_assert(BLOCK >= 2 * kBuckets && BLOCK % REPL == 0, "one thread per bucket and table");
  const int tid = threadIdx.x;
  if (tid < 2 * kBuckets) {  // one thread per bucket and table
    const int r = tid / kBuckets, b = tid % kBuckets;
    int below = 0, inside = 0;
#pragma unroll
    for (int j = 0; j < 15; ++j) {
      const int bj = st.mid_bucket[r][j];
      below += bj < b ? 1 : 0;
      inside += bj == b ? 1 : 0;
    }
    const uint32_t e = inside <= 1 ? 16u * (uint32_t)below + (uint32_t)(r * sizeof(st.row[0]))
                                   : (uint32_t)(sizeof(st.row) + r * sizeof(SearchRow));
    if constexpr (REPL == 4) {  // the four copies are one 16-byte store: no staging, one barrier less
      *reinterpret_cast<uint4*>(&sl.lut[r][b * REPL]) = make_uint4(e, e, e, e);
    } else {
      st.entry[r][b] = e;
    }
  }
  __syncthreads();
  if constexpr (REPL == 4) return;
  // replicate with 16-byte stores: unit u of 4 copies -> table u / (kBuckets * REPL / 4), bucket
  // (u / (REPL / 4)) % kBuckets; consecutive threads write consecutive units
  if constexpr (REPL >= 4) {
    constexpr int kUnitsPerBucket = REPL / 4, kUnits = 2 * kBuckets * kUnitsPerBucket;
    uint4* dst = reinterpret_cast<uint4*>(&sl.lut[0][0]);
    for (int u = tid; u < kUnits; u += BLOCK) {
      const uint32_t e = (&st.entry[0][0])[u / kUnitsPerBucket];
      dst[u] = make_uint4(e, e, e, e);
    }
  } else {
    for (int b = tid / REPL; b < kBuckets; b += BLOCK / REPL) {
      sl.lut[0][b * REPL + (tid % REPL)] = st.entry[0][b];
      sl.lut[1][b * REPL + (tid % REPL)] = st.entry[1][b];
    }
  }
  __syncthreads();
}

// One step of the rank count of wave_sort_tables: the entry K lanes away in the row of 16 (value and
// index, both rotated the same way) against this lane's; equal values rank by index.
template <int K>
__device__ __forceinline__ void rank_step(float v, int i, int& rank) {
  constexpr int kRor = 0x120 + K;  // row_ror:K
  const float u = dpp<kRor>(v);
  const int j = __builtin_amdgcn_update_dpp(0, i, kRor, 0xF, 0xF, false);
  rank += (u < v || (u == v && j < i)) ? 1 : 0;
}

// Called by ONE wavefront (all 64 lanes): lane b < 32 passes entry b of the two tables (T0 in lanes
// 0..15, T1 in 16..31).  Sorts each table (stable rank sort: a table is one row of 16 lanes, the other
// 15 entries come by lane rotation together with their indices), leaves them in st.newtab and
// builds the search rows (wave_make_rows).
__device__ __forceinline__ void wave_sort_tables(SearchTables& st, float entry) {
  const int lane = threadIdx.x & 63;
  const int base = lane & 16, i = lane & 15;
  const float v = lane < 32 ? entry : 0.0f;
  int rank = 0;
  rank_step<1>(v, i, rank);
  rank_step<2>(v, i, rank);
  rank_step<3>(v, i, rank);
  rank_step<4>(v, i, rank);
  rank_step<5>(v, i, rank);
  rank_step<6>(v, i, rank);
  rank_step<7>(v, i, rank);
  rank_step<8>(v, i, rank);
  rank_step<9>(v, i, rank);
  rank_step<10>(v, i, rank);
  rank_step<11>(v, i, rank);
  rank_step<12>(v, i, rank);
  rank_step<13>(v, i, rank);
  rank_step<14>(v, i, rank);
  rank_step<15>(v, i, rank);
  if (lane < 32) st.newtab[base + rank] = v;
  wave_make_rows(st);
}

}  // namespace aaac

// Host-side checks of the library's launch plans and workspace layouts (no GPU needed): for a sweep of
// shapes and compute-unit counts every plan must cover the layer exactly once within its limits.
// Linked against the library's objects by tests/test_host_plans.py.
#include <cstdio>
#include <cstdlib>

#include "aaac_internal.h"

using namespace aaac;

#define CHECK(cond)                                                                                   \
  do {                                                                                                \
    if (!(cond)) {                                                                                    \
      std::printf("FAILED %s (line %d) N=%lld K=%lld cus=%d g=%d\n", #cond, __LINE__, (long long)N, (long long)K, cus, g); \
      return 1;                                                                                       \
    }                                                                                                 \
  } while (0)

static int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

int main() {
  const int64_t Ns[] = {1, 2, 7, 15, 16, 17, 33, 128, 255, 256, 1000, 1024, 4096, 8192, 14336, 28672, 40001, 1000000};
  const int64_t Ks[] = {16, 128, 256, 512, 528, 1024, 1040, 4096, 8192, 11008, 14336, 28672, 65536, 200064};
  const int cu_counts[] = {1, 2, 5, 19, 68, 69, 104, 256, 304};
  const int gs[] = {16, 32, 64, 128};
  long checked = 0;
  for (int64_t N : Ns)
    for (int64_t K : Ks)
      for (int g : gs) {
        if (K % g) continue;
        int cus = 0;
        for (int s = 16; s <= g; s *= 2) {  // workspace layout: aligned, ordered, large enough
          const FitLayout lay = fit_layout(N, K, g, s);
          CHECK(lay.off_state == 0 && lay.off_rinv >= sizeof(FitState));
          CHECK(lay.off_rinv % 256 == 0 && lay.off_sigma % 256 == 0 && lay.off_quant % 256 == 0 && lay.off_small % 256 == 0);
          CHECK(lay.off_sigma - lay.off_rinv >= (size_t)N * (K / g) * sizeof(float));
          CHECK(lay.off_quant - lay.off_sigma >= (size_t)N * (K / s));
          CHECK(lay.off_cand % 256 == 0 && lay.off_cand - lay.off_quant >= sizeof(QuantState));
          CHECK(quant_candidates(N, K) >= 16384 && quant_candidates(N, K) >= N * K / 32);
          CHECK(lay.off_small - lay.off_cand >= (size_t)quant_candidates(N, K) * sizeof(uint32_t));
          CHECK(lay.bytes - lay.off_small >= kSmallStateBytes && lay.bytes % 256 == 0);
        }
        for (int c : cu_counts) {
          cus = c;
          const FitPlan p = make_fit_plan(N, K, K, g, g, cus);
          const int spb = p.strips_per_block;
          CHECK(p.strips == cdiv(K, kStripCols));
          CHECK(spb == 1 || spb == 2 || spb == 4 || spb == 8 || spb == 16);
          CHECK((int64_t)p.strip_groups * spb >= p.strips && (int64_t)(p.strip_groups - 1) * spb < p.strips);
          CHECK(p.rows_per_block >= 1 && p.blocks >= 1);
          CHECK((int64_t)p.blocks == (int64_t)p.strip_groups * cdiv(N, p.rows_per_block));
          CHECK(cdiv(N, p.rows_per_block) * p.rows_per_block >= N);
          // never more blocks than compute units unless the strips alone need more
          CHECK(p.blocks <= cus || cdiv(N, p.rows_per_block) == 1);
          ++checked;
        }
        const SmallPlan sp = make_small_plan(N, K);
        const int64_t strips = cdiv(K, kStripCols);
        if (sp.blocks > 0) {
          CHECK(sp.blocks <= kSmallMaxBlocks && sp.strips == strips);
          CHECK((int64_t)sp.blocks * 8 >= strips);
          CHECK(sp.waves_per_strip == sp.blocks * 8 / sp.strips && sp.waves_per_strip >= 1);
          CHECK(sp.rows_per_wave >= 1 && sp.rows_per_wave <= kSmallRows);
          CHECK((int64_t)sp.rows_per_wave * sp.waves_per_strip >= N);
        } else {
          CHECK(N * strips > (int64_t)kSmallMaxBlocks * 8 * kSmallRows || strips > kSmallMaxBlocks * 8 ||
                cdiv(N, (int64_t)kSmallMaxBlocks * 8 / strips) > kSmallRows);
        }
        {  // quantile targets: at most 64 distinct ascending ranks inside the layer; levels point at them
          const QuantTargets tg = make_quant_targets(N, K);
          CHECK(tg.count >= 1 && tg.count <= kQuantSlots);
          const unsigned long long total = (unsigned long long)N * (unsigned long long)K;
          for (int u = 0; u < tg.count; ++u) {
            CHECK(tg.rank[u] < total);
            CHECK(u == 0 || tg.rank[u] > tg.rank[u - 1]);
          }
          CHECK(tg.rank[0] == 0 && tg.rank[tg.count - 1] == total - 1);  // levels 0 and 1 of T0
          for (int q = 0; q < 32; ++q) {
            const QuantLevel& l = tg.level[q];
            CHECK(l.lo < tg.count && l.hi < tg.count && l.rem < l.den);
            CHECK(l.rem == 0 ? l.hi == l.lo : tg.rank[l.hi] == tg.rank[l.lo] + 1);
          }
        }
      }
  for (int64_t tokens : {(int64_t)0, (int64_t)1, (int64_t)31, (int64_t)256, (int64_t)5000, (int64_t)65536, (int64_t)131072, (int64_t)3000001})
    for (int64_t K : {(int64_t)8, (int64_t)512, (int64_t)4096, (int64_t)4104, (int64_t)11008, (int64_t)28672, (int64_t)1048576, (int64_t)1052672}) {
      const int64_t N = tokens;
      const int cus = 256, g = 0;
      const StatsPlan p = make_stats_plan(tokens, K);
      CHECK((int64_t)p.strips * 4096 >= K && (int64_t)(p.strips - 1) * 4096 < K);
      CHECK(p.token_chunks >= 1 && p.tokens_per_chunk >= 1);
      CHECK((int64_t)p.token_chunks * p.tokens_per_chunk >= tokens);
      CHECK((int64_t)(p.token_chunks - 1) * p.tokens_per_chunk < (tokens > 0 ? tokens : 1));
      CHECK((int64_t)p.strips * p.token_chunks <= 256 || p.token_chunks == 1);
      CHECK(p.bytes == (size_t)p.token_chunks * p.strips * 4096 * sizeof(double));
      CHECK((K <= 1048576) == (p.bytes <= kStaticScratchBytes));
      ++checked;
    }
  std::printf("host_plan_check ok: %ld plans\n", checked);
  return 0;
}

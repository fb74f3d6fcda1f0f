// Sanitizer run of the CPU oracle: every entry point of aaac_oracle.cpp on small random inputs (ragged
// widths, padded rows, every group and selection size, both scale formats, degenerate values), meant to
// be compiled with -fsanitize=address,undefined.  It checks nothing about the values (the pins in
// tests/ do that); it exists so that an out-of-bounds index or an undefined shift in the oracle's
// fixed-size buffers and index arithmetic is reported.  Test infrastructure, like the oracle itself.
#include <cstdio>
#include <vector>

#include "aaac_oracle.cpp"

namespace {

uint32_t state = 0x9E3779B9u;
uint32_t rnd() {
  state ^= state << 13;
  state ^= state >> 17;
  state ^= state << 5;
  return state;
}
// a finite bf16 pattern: mostly moderate magnitudes, some zeros, tiny and huge values
uint16_t rand_bf16() {
  const uint32_t r = rnd();
  const uint32_t kind = r % 16;
  if (kind == 0) return (uint16_t)((r >> 8) & 0x8000u);                           // +-0
  if (kind == 1) return (uint16_t)(((r >> 8) & 0x807Fu) | 0x0080u);               // smallest normals
  if (kind == 2) return (uint16_t)(((r >> 8) & 0x807Fu) | 0x7E80u);               // very large
  const uint32_t exp = 118u + (r >> 20) % 10u;                                    // around 2^-9 .. 1
  return (uint16_t)(((r >> 4) & 0x8000u) | (exp << 7) | ((r >> 9) & 0x7Fu));
}

int run() {
  const int shapes[][2] = {{1, 16}, {3, 128}, {5, 1040}, {7, 640}, {2, 2048}, {9, 256}};
  const int groups[] = {16, 32, 64, 128};
  int calls = 0;
  for (const auto& sh : shapes)
    for (int g : groups)
      for (int fmt = 0; fmt < 2; ++fmt) {
        const int64_t N = sh[0], K = sh[1];
        if (K % g) continue;
        const int64_t ldw = K + 8 * (int64_t)(rnd() % 3);
        std::vector<uint16_t> W(N * ldw), X(11 * K);
        for (auto& w : W) w = rand_bf16();
        for (auto& x : X) x = rand_bf16() & 0xBFFFu;  // keep the squares finite
        std::vector<float> I(K), grid(32), tf(32), wn(N * K), sv(N * (K / g));
        std::vector<uint16_t> tb(32);
        oracle_act_stats(X.data(), 11, K, K, I.data());
        for (int t = 0; t < 2; ++t)
          for (int i = 0; i < 16; ++i) grid[16 * t + i] = (float)(i - 8 + t) * 0.75f;
        std::vector<uint8_t> sc8(N * (K / g) * 2);
        if (oracle_normalise(W.data(), N, K, ldw, g, fmt, sc8.data(), sv.data(), wn.data())) return 1;
        std::vector<float> e0(N * (K / g)), e1(N * (K / g));
        std::vector<uint8_t> sigma(N * (K / g)), i0(N * K), i1(N * K);
        double J = 0;
        if (oracle_assign(wn.data(), N, K, g, I.data(), grid.data(), e0.data(), e1.data(), sigma.data(), i0.data(),
                          i1.data(), &J)) return 2;
        std::vector<float> T(grid);
        std::vector<double> sums(64);
        if (oracle_lloyd_iteration(wn.data(), N, K, g, I.data(), T.data(), sums.data(), &J)) return 3;
        if (oracle_kmeans_step(wn.data(), N, K, g, I.data(), sigma.data(), T.data())) return 4;
        std::vector<double> obj(3);
        std::vector<float> trace(3 * 2 * 32);
        if (oracle_fit(W.data(), N, K, ldw, g, fmt, I.data(), grid.data(), 3, tf.data(), tb.data(), obj.data(),
                       trace.data())) return 5;
        if (oracle_fit_nested(W.data(), N, K, ldw, g, fmt, I.data(), grid.data(), 3, 2, tf.data(), tb.data(),
                              obj.data(), trace.data())) return 6;
        std::vector<float> q(32);
        if (oracle_quantile_init(W.data(), N, K, ldw, g, fmt, q.data())) return 7;
        std::vector<uint8_t> codes(N * K / 2), scales(N * (K / g) * 2);
        if (oracle_encode(W.data(), N, K, ldw, g, fmt, I.data(), tb.data(), codes.data(), scales.data())) return 8;
        std::vector<uint16_t> What(N * ldw);
        if (oracle_dequant(codes.data(), scales.data(), tb.data(), N, K, g, fmt, What.data(), ldw)) return 9;
        calls += 10;
        for (int S : groups) {
          if (S > g) continue;
          const int64_t stride = (K / S + 7) / 8 + (int64_t)(rnd() % 2);
          std::vector<uint8_t> bits(N * stride, 0xFF);
          if (oracle_fit_sel(W.data(), N, K, ldw, g, S, fmt, I.data(), q.data(), 2, 2, tf.data(), tb.data(), obj.data(),
                             trace.data())) return 10;
          if (oracle_encode_sel(W.data(), N, K, ldw, g, S, fmt, I.data(), tb.data(), codes.data(), scales.data(),
                                S < g ? bits.data() : nullptr, stride)) return 11;
          if (oracle_dequant_sel(codes.data(), scales.data(), S < g ? bits.data() : nullptr, stride, tb.data(), N, K, g, S,
                                 fmt, What.data(), ldw)) return 12;
          const int64_t M = 1 + (int64_t)(rnd() % 3);
          std::vector<uint16_t> x(M * K);
          for (auto& v : x) v = rand_bf16() & 0xBFFFu;
          std::vector<float> y(M * N);
          std::vector<double> mag(M * N);
          if (K % 32 == 0 &&
              oracle_gemv_w4a16(x.data(), M, K, codes.data(), scales.data(), S < g ? bits.data() : nullptr, stride,
                                tb.data(), N, K, g, S, fmt, y.data(), mag.data())) return 13;
          if (K % 64 == 0 &&
              oracle_gemm_w4a16(x.data(), M, K, codes.data(), scales.data(), S < g ? bits.data() : nullptr, stride,
                                tb.data(), N, K, g, S, fmt, y.data(), mag.data())) return 14;
          calls += 5;
        }
      }
  // the scalar conversions over their whole domains
  for (uint32_t c = 0; c < 256; ++c) oracle_f32_to_e4m3(oracle_e4m3_to_f32((uint8_t)(c & 0x7F)));
  for (uint32_t h = 0; h < 0x7F80u; h += 7) oracle_f32_to_bf16(oracle_bf16_to_f32((uint16_t)h) * 1.0009765625f);
  std::printf("sanitize_check ok: %d calls\n", calls);
  return 0;
}

}  // namespace

int main() { return run(); }

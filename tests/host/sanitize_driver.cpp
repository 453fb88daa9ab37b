// Host-side walk through the library's CPU code for a build with
// -fsanitize=address,undefined: the codebook solver, the rotation builder, the
// split composer, and the argument checks of every GPU entry point (each call
// here must be answered with a status code before any device is touched).
// Prints one line per group and exits non-zero on the first wrong answer; the
// sanitizers abort on their own findings.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../include/turboquant.h"

#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                             \
    }                                                                       \
  } while (0)

int main() {
  // tq_build_codebook: every width, small and large d, exact-size output buffers
  for (int d : {3, 4, 8, 128, 200, 1536, 3072}) {
    for (int bits = 0; bits <= 5; ++bits) {
      std::vector<float> c((size_t)1 << bits), t(((size_t)1 << bits) - 1 + (bits == 0 ? 1 : 0));
      double cost = -1.0;
      EXPECT(tq_build_codebook(d, bits, c.data(), bits ? t.data() : nullptr, &cost) == TQ_OK);
      for (size_t k = 0; k + 1 < c.size(); ++k) EXPECT(c[k] < c[k + 1]);
      for (size_t k = 0; k < c.size(); ++k) EXPECT(c[k] == -c[c.size() - 1 - k]);
      EXPECT(cost >= 0.0 && cost <= 1.0 / d + 1e-12);
    }
  }
  float one[2];
  EXPECT(tq_build_codebook(2, 1, one, one, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_build_codebook(128, 9, one, one, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_build_codebook(128, 1, nullptr, one, nullptr) == TQ_ERR_INVALID_ARG);
  std::puts("codebook ok");

  // tq_build_rotation: orthogonal, and R = Pi^T G upper triangular with a positive diagonal
  std::mt19937_64 rng(7);
  std::normal_distribution<double> gauss(0.0, 1.0);
  for (int d : {1, 2, 5, 64, 193}) {
    std::vector<double> g((size_t)d * d);
    for (auto& v : g) v = gauss(rng);
    std::vector<float> pi((size_t)d * d);
    EXPECT(tq_build_rotation(d, g.data(), pi.data()) == TQ_OK);
    for (int i = 0; i < d; ++i)
      for (int j = 0; j < d; ++j) {
        double dot = 0.0, r = 0.0;
        for (int k = 0; k < d; ++k) {
          dot += (double)pi[(size_t)k * d + i] * pi[(size_t)k * d + j];
          r += (double)pi[(size_t)k * d + i] * g[(size_t)k * d + j];
        }
        EXPECT(std::fabs(dot - (i == j ? 1.0 : 0.0)) < 1e-5);
        if (i == j) EXPECT(r > 0.0);
        if (i > j) EXPECT(std::fabs(r) < 1e-4);
      }
  }
  EXPECT(tq_build_rotation(0, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_build_rotation(4, nullptr, one) == TQ_ERR_INVALID_ARG);
  std::puts("rotation ok");

  // tq_compose_split
  {
    const int d = 8, d_hi = 3;
    const int32_t hi[3] = {1, 4, 6};
    std::vector<float> a(9), b(25), out(64, -1.f);
    for (int i = 0; i < 9; ++i) a[i] = 1.f + i;
    for (int i = 0; i < 25; ++i) b[i] = 100.f + i;
    EXPECT(tq_compose_split(d, d_hi, hi, a.data(), b.data(), out.data()) == TQ_OK);
    const int order[8] = {1, 4, 6, 0, 2, 3, 5, 7};
    for (int r = 0; r < 8; ++r)
      for (int c = 0; c < 8; ++c) {
        float want = 0.f;
        if (r < 3 && c < 3) want = a[r * 3 + c];
        if (r >= 3 && c >= 3) want = b[(r - 3) * 5 + (c - 3)];
        EXPECT(out[r * 8 + order[c]] == want);
      }
    const int32_t bad[3] = {4, 1, 6};
    EXPECT(tq_compose_split(d, d_hi, bad, a.data(), b.data(), out.data()) == TQ_ERR_INVALID_ARG);
    const int32_t far[3] = {1, 4, 8};
    EXPECT(tq_compose_split(d, d_hi, far, a.data(), b.data(), out.data()) == TQ_ERR_INVALID_ARG);
    EXPECT(tq_compose_split(d, 8, hi, a.data(), b.data(), out.data()) == TQ_ERR_INVALID_ARG);
  }
  std::puts("compose ok");

  // entropy codec: bucket masses, code construction, a round trip, a truncated stream
  {
    float c16[16], t15[15];
    EXPECT(tq_build_codebook(128, 4, c16, t15, nullptr) == TQ_OK);
    double p[16], sum = 0.0, mean = 0.0;
    EXPECT(tq_bucket_masses(128, 4, c16, p) == TQ_OK);
    for (double v : p) sum += v;
    EXPECT(std::fabs(sum - 1.0) < 1e-12);
    uint8_t len[16];
    uint32_t cw[16];
    EXPECT(tq_prefix_code_build(16, p, len, cw, &mean) == TQ_OK);
    EXPECT(mean > 3.7 && mean < 3.9);
    const int d = 96, n = 37, words = d / 32 * 4;
    std::vector<uint32_t> idx((size_t)n * words), back((size_t)n * words, 0xffffffffu);
    for (auto& w : idx) w = (uint32_t)rng();
    std::vector<uint8_t> stream((size_t)n * d * 4);
    std::vector<uint64_t> offs((size_t)n + 1);
    size_t used = 0;
    EXPECT(tq_entropy_encode(d, 4, len, cw, idx.data(), n, stream.data(), stream.size(), &used, offs.data()) == TQ_OK);
    EXPECT(used == (offs[(size_t)n] + 7) / 8);
    std::vector<uint8_t> exact(stream.begin(), stream.begin() + (long)used);  // no slack behind the stream
    EXPECT(tq_entropy_decode(d, 4, len, exact.data(), exact.size(), 0, n, back.data()) == TQ_OK);
    EXPECT(back == idx);
    EXPECT(tq_entropy_decode(d, 4, len, exact.data(), exact.size(), offs[20], 1, back.data()) == TQ_OK);
    for (int w = 0; w < words; ++w) EXPECT(back[(size_t)w] == idx[(size_t)20 * words + w]);
    EXPECT(tq_entropy_decode(d, 4, len, exact.data(), exact.size() - 3, 0, n, back.data()) == TQ_ERR_INVALID_ARG);
    EXPECT(tq_entropy_encode(d, 4, len, cw, idx.data(), n, stream.data(), 10, &used, nullptr) == TQ_ERR_WORKSPACE);
  }
  std::puts("entropy codec ok");

  // argument checks of the GPU entry points: all answered on the host
  float c4[4] = {-1.5f, -0.5f, 0.5f, 1.5f}, t3[3] = {-1.f, 0.f, 1.f};
  tq_params p{};
  p.d = 100;
  p.bits_mse = 2;
  p.centroids = c4;
  p.bounds = t3;
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 4, 100, nullptr, nullptr, nullptr) == TQ_ERR_UNSUPPORTED);
  p.d = 128;
  EXPECT(tq_quantize_mse(nullptr, nullptr, TQ_F32, 4, 128, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 4, 128, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, -1, 128, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_quantize_mse(&p, nullptr, 7, 4, 128, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 0, 128, nullptr, nullptr, nullptr) == TQ_OK);
  // row strides beyond what the kernels' 32-bit row offsets cover
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 4, (int64_t(1) << 22) + 4, nullptr, nullptr, nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_dequantize(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, (int64_t(1) << 22) + 4, nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_score(&p, nullptr, (int64_t(1) << 22) + 4, 1, 1, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 0, nullptr, nullptr,
                  nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_quantize_prod(&p, nullptr, TQ_BF16, 4, 64, nullptr, nullptr, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_append(&p, nullptr, TQ_F32, 4, 128, nullptr, nullptr, nullptr, nullptr, -1, 1, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_append(&p, nullptr, TQ_F32, 1 << 20, 128, nullptr, nullptr, nullptr, nullptr, 0, 1, nullptr) == TQ_ERR_UNSUPPORTED);
  p.bits_mse = 5;
  EXPECT(tq_dequantize(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, 128, nullptr) == TQ_ERR_UNSUPPORTED);
  p.bits_mse = 2;
  EXPECT(tq_dequantize(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, 128, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_dequantize(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, 64, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_score(&p, nullptr, 128, 1, 1, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 0, nullptr, nullptr, nullptr) ==
         TQ_ERR_INVALID_ARG);
  EXPECT(tq_score(&p, nullptr, 128, 1, 1, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 65, nullptr, nullptr, nullptr) ==
         TQ_ERR_UNSUPPORTED);
  EXPECT(tq_score(&p, nullptr, 128, 0, 4, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 0, nullptr, nullptr, nullptr) == TQ_OK);
  EXPECT(tq_score_static(nullptr, nullptr, 128, 1, 1, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 0, nullptr, nullptr,
                         nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_score_static(&p, nullptr, 128, 1, 100000, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 0, nullptr, nullptr,
                         nullptr) == TQ_ERR_WORKSPACE);
  EXPECT(tq_score_static_scratch_bytes() == (size_t)16 << 20);
  EXPECT(tq_attend(&p, &p, nullptr, 128, 1, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, -1, 1.f,
                   nullptr, 128, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_stage_pack(&p, nullptr, 4, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_stage_pack(&p, nullptr, 0, nullptr, nullptr) == TQ_OK);
  EXPECT(tq_stage_unpack(&p, nullptr, 3, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_stage_sign_pack(100, nullptr, 1, nullptr, nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_stage_sign_pack(128, nullptr, 1, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_derive_params(128, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  EXPECT(tq_workspace_bytes(&p, 1000, 10, 0) >= (size_t)1000 * 128 * 4);
  EXPECT(tq_workspace_bytes(nullptr, 1000, 10, 0) == 0);
  EXPECT(tq_attend_workspace_bytes(&p, &p, 8, 4, 1000) > 0);
  // two instances
  float c8[8] = {-4, -3, -2, -1, 1, 2, 3, 4}, t7[7] = {-3.5f, -2.5f, -1.5f, 0, 1.5f, 2.5f, 3.5f};
  p.d_hi = 48;
  p.bits_mse_hi = 3;
  p.centroids_hi = c8;
  p.bounds_hi = t7;
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 4, 128, nullptr, nullptr, nullptr) == TQ_ERR_INVALID_ARG);
  p.d_hi = 64;
  p.bits_mse_hi = 2;
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 4, 128, nullptr, nullptr, nullptr) == TQ_ERR_UNSUPPORTED);
  p.bits_mse_hi = 3;
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 0, 128, nullptr, nullptr, nullptr) == TQ_OK);
  // row strides beyond what the kernels' 32-bit row offsets cover
  EXPECT(tq_quantize_mse(&p, nullptr, TQ_F32, 4, (int64_t(1) << 22) + 4, nullptr, nullptr, nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_dequantize(&p, nullptr, nullptr, nullptr, nullptr, 1, nullptr, (int64_t(1) << 22) + 4, nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_score(&p, nullptr, (int64_t(1) << 22) + 4, 1, 1, nullptr, nullptr, nullptr, nullptr, 10, nullptr, 10, 0, nullptr, nullptr,
                  nullptr) == TQ_ERR_UNSUPPORTED);
  EXPECT(tq_stage_pack(&p, nullptr, 4, nullptr, nullptr) == TQ_ERR_UNSUPPORTED);
  for (int s = 0; s <= 5; ++s) EXPECT(tq_status_string((tq_status)s) != nullptr);
  std::puts("argument checks ok");
  return 0;
}

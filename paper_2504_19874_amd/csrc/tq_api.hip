// C ABI entry points: argument validation, workspace carving, kernel launches.
// No allocation, no synchronisation; everything is enqueued on the caller's
// stream.
#include <cmath>
#include <cstring>
#include <mutex>

#include "tq_attend.h"
#include "tq_score_i8.h"

using namespace tq;

namespace tq {
int device_cu_count() {
  static std::mutex m;
  static int count[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  std::lock_guard<std::mutex> lock(m);
  if (count[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    count[dev] = v;
  }
  return count[dev];
}
}  // namespace tq

namespace {

constexpr int64_t kChunkRows = 65536;  // rows per pass when a residual workspace is needed
// Row strides of vectors (x, q) and of dequantised output: the kernels address a tile's rows with 32-bit byte
// offsets from a 64-bit tile base (up to 256 rows of ld * 4 bytes)
constexpr int64_t kMaxRowStride = int64_t(1) << 22;
constexpr int64_t kRowsQuantMax = 64;  // at most this many long vectors take the matrix-vector route of the quantiser
// That route reads every matrix once per block of four vectors, the tiled contraction once per 128: it wins while
// blocks x d^2 x matrices stays below about 4e7 elements (measured: d = 1536, Alg. 1: 14 / 18 / 52 us for 1 / 8 / 64
// vectors against 78; d = 3072, Alg. 2: 47 / 112 us for 1 / 8 against 223, but 722 us for 64).
// (The dequantiser's route reads both matrices in one kernel and has no second stage: d = 1536, Alg. 1: 10 / 12 / 50
// us for 1 / 8 / 64 vectors against 108; d = 3072, Alg. 2: 17 us for one against 153; its bound is twice as wide.)
bool rows_route_serves(int64_t n, int d, int matrices, int64_t limit = 150) {
  return n <= kRowsQuantMax && d >= 512 && d <= 4096 && ((n + 3) / 4) * (int64_t)d * d * matrices <= limit * 512 * 512;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

tq_status check_params(const tq_params* p, bool need_codebook) {
  if (p == nullptr) return TQ_ERR_INVALID_ARG;
  if (p->d <= 0 || p->bits_mse < 0) return TQ_ERR_INVALID_ARG;
  if (p->d % 32 != 0 || p->bits_mse > 4 || p->d > 16384) return TQ_ERR_UNSUPPORTED;
  if (need_codebook) {
    if (p->centroids == nullptr) return TQ_ERR_INVALID_ARG;
    if (p->bits_mse > 0 && p->bounds == nullptr) return TQ_ERR_INVALID_ARG;
  }
  if (p->d_hi != 0) {
    // two instances over a split of the rotated coordinates (Sec. 4.3)
    if (p->d_hi < 0 || p->d_hi >= p->d || p->d_hi % 32 != 0 || p->bits_mse_hi < 0) return TQ_ERR_INVALID_ARG;
    if (need_codebook && (p->centroids_hi == nullptr || (p->bits_mse_hi > 0 && p->bounds_hi == nullptr)))
      return TQ_ERR_INVALID_ARG;
    // what the kernels cover: head dimension 128, one more bit for the outlier instance
    if (p->d != 128 || p->bits_mse_hi != p->bits_mse + 1 || p->bits_mse_hi > 4) return TQ_ERR_UNSUPPORTED;
  }
  return TQ_OK;
}

Codebook make_codebook_hi(const tq_params* p) {
  Codebook cb;
  std::memset(&cb, 0, sizeof(cb));
  if (p->d_hi == 0) return cb;
  cb.bits = p->bits_mse_hi;
  const int K = 1 << p->bits_mse_hi;
  for (int k = 0; k < K; ++k) cb.c[k] = p->centroids_hi[k];
  for (int k = 0; k + 1 < K; ++k) cb.t[k] = p->bounds_hi[k];
  return cb;
}

Codebook make_codebook(const tq_params* p) {
  Codebook cb;
  std::memset(&cb, 0, sizeof(cb));
  cb.bits = p->bits_mse;
  const int K = 1 << p->bits_mse;
  for (int k = 0; k < K; ++k) cb.c[k] = p->centroids[k];
  for (int k = 0; k + 1 < K; ++k) cb.t[k] = p->bounds[k];
  return cb;
}

float kappa_of(int d) { return (float)(std::sqrt(1.5707963267948966) / (double)d); }

// TQ_FLAG_FP32_MFMA keeps every contraction of the call on the fp32 matrix instructions
bool fp32_mfma_only(const tq_params* p) { return (p->flags & TQ_FLAG_FP32_MFMA) != 0; }

// tq_params.images: [image of the d = 128 quantisation kernel][image of the d = 128 dequantisation kernel]
const void* quant_image(const tq_params* p) { return p->d == 128 ? p->images : nullptr; }
const void* dequant_image(const tq_params* p) {
  return p->d == 128 && p->images != nullptr ? static_cast<const char*>(p->images) + quant128_bf3_image_bytes() : nullptr;
}

tq_status from_hip(hipError_t e) { return e == hipSuccess ? TQ_OK : TQ_ERR_HIP; }

// Quant_prod of fp32 vectors on the bf16 matrix cores keeps the two leading pieces of x: the rotated vector is off
// by up to 2^-17 |x| in norm (2^-18.6 in the root mean square).  The indices do not notice, but the residual norm
// gamma and the sketch signs of Alg. 2 are judged relative to gamma, which shrinks with the bit-width of the MSE
// stage (sqrt(D_mse) of Theorem 1: 1, 0.60, 0.34, 0.18, 0.097 for 0..4 bits); the error's component along the
// residual is about 2^-18.6 / sqrt(d).  Where that exceeds about 1e-6 gamma the rotation stays on fp32 MFMA
// (d = 128: the 4-bit MSE stage; 3 bits below d = 128; 2 bits at d = 32).
bool two_piece_x_serves_prod(int d, int bits_mse) {
  static const float gamma_typ[5] = {1.f, 0.60f, 0.342f, 0.183f, 0.097f};
  return gamma_typ[bits_mse] * std::sqrt((float)d) >= 2.f;
}

struct Workspace {
  char* base;
  size_t size;
  size_t used;
  void* take(size_t bytes) {
    const size_t off = round_up(used, 256);
    if (base == nullptr || off + bytes > size) return nullptr;
    used = off + bytes;
    return base + off;
  }
};

tq_status quantize_common(const tq_params* p, const void* x, int32_t dtype, int64_t n, int64_t ldx,
                          uint32_t* idx, uint32_t* qjl, float* gamma, float* norm, bool prod,
                          hipStream_t stream, int64_t out_first = 0, int64_t out_step = 1, bool scattered = false) {
  tq_status st = check_params(p, true);
  if (st != TQ_OK) return st;
  if (n < 0 || ldx < p->d) return TQ_ERR_INVALID_ARG;
  if (ldx > kMaxRowStride) return TQ_ERR_UNSUPPORTED;
  if (dtype != TQ_F32 && dtype != TQ_BF16) return TQ_ERR_INVALID_ARG;
  if (n == 0) return TQ_OK;
  if (x == nullptr || p->Pi == nullptr) return TQ_ERR_INVALID_ARG;
  if (p->bits_mse > 0 && idx == nullptr) return TQ_ERR_INVALID_ARG;
  if (prod && (qjl == nullptr || gamma == nullptr || p->SPiT == nullptr)) return TQ_ERR_INVALID_ARG;
  if (ldx % 4 != 0 || !aligned16(p->Pi) || (prod && !aligned16(p->SPiT))) return TQ_ERR_UNSUPPORTED;
  if (dtype == TQ_F32 ? !aligned16(x) : (reinterpret_cast<uintptr_t>(x) & 7u) != 0)
    return TQ_ERR_UNSUPPORTED;

  const int d = p->d;
  const size_t esz = dtype == TQ_F32 ? 4 : 2;
  const int words_per_row = (d / 32) * p->bits_mse;

  if (scattered) {
    // rows scattered into a larger store (tq_append): the short-chain d = 128 kernel only
    if (d != 128 || n > kSmallQuantRows || !aligned16(x) || (ldx * esz) % 16 != 0) return TQ_ERR_UNSUPPORTED;
    if (p->d_hi != 0 && norm == nullptr) return TQ_ERR_INVALID_ARG;
    return from_hip(launch_quant128_small(p->bits_mse, prod, dtype == TQ_BF16, x, ldx, n, p->Pi,
                                          prod ? p->SPiT : nullptr, idx, qjl, gamma, norm, make_codebook(p),
                                          p->d_hi / 32, p->d_hi != 0 ? make_codebook_hi(p) : make_codebook(p), stream,
                                          out_first, out_step));
  }

  if (p->d_hi != 0) {
    // two instances: the d = 128 kernels; both norms are always stored
    if (norm == nullptr) return TQ_ERR_INVALID_ARG;
    if (!aligned16(x) || (ldx * esz) % 16 != 0) return TQ_ERR_UNSUPPORTED;
    const Codebook cb_hi = make_codebook_hi(p);
    if (dtype == TQ_BF16 && n >= kBf3QuantRows && !fp32_mfma_only(p) && (!prod || aligned16(qjl)) &&
        quant128_bf3_applicable(p->bits_mse, prod, false, x, ldx, make_codebook(p), &cb_hi))
      return from_hip(launch_quant128_bf3(p->bits_mse, prod, false, x, ldx, n, p->Pi, prod ? p->SPiT : nullptr, idx, qjl, gamma,
                                          norm, make_codebook(p), p->d_hi / 32, make_codebook_hi(p), quant_image(p), stream));
    return from_hip(launch_quant128(p->bits_mse, prod, dtype == TQ_BF16, x, ldx, n, p->Pi,
                                    prod ? p->SPiT : nullptr, idx, qjl, gamma, norm, make_codebook(p),
                                    p->d_hi / 32, make_codebook_hi(p), stream));
  }

  // head dimension 128, a large batch of bf16 or fp32 vectors: the contractions on the bf16 matrix cores
  if (d == 128 && n >= kBf3QuantRows && !fp32_mfma_only(p) && !(prod && dtype == TQ_F32 && !two_piece_x_serves_prod(d, p->bits_mse)) &&
      quant128_bf3_applicable(p->bits_mse, prod, dtype == TQ_F32, x, ldx, make_codebook(p), nullptr) &&
      (p->bits_mse == 0 || aligned16(idx)) && (!prod || aligned16(qjl)))
    return from_hip(launch_quant128_bf3(p->bits_mse, prod, dtype == TQ_F32, x, ldx, n, p->Pi, prod ? p->SPiT : nullptr, idx, qjl, gamma,
                                        norm, make_codebook(p), 0, make_codebook(p), quant_image(p), stream));

  // head dimension 128: one fused kernel, parameters resident in LDS
  if (d == 128 && aligned16(x) && (ldx * esz) % 16 == 0) {
    return from_hip(launch_quant128(p->bits_mse, prod, dtype == TQ_BF16, x, ldx, n, p->Pi,
                                    prod ? p->SPiT : nullptr, idx, qjl, gamma, norm, make_codebook(p), 0,
                                    make_codebook(p), stream));
  }

  GemmArgs a;
  std::memset(&a, 0, sizeof(a));
  a.W1 = p->Pi;
  a.ldw = d;
  a.M = d;
  a.d = d;
  a.segs = 1;
  a.ldx = ldx;
  a.normalise = norm != nullptr;
  a.kappa = kappa_of(d);
  a.cb = make_codebook(p);
  const bool pieces = !fp32_mfma_only(p);
  a.pieces = pieces && !(prod && dtype == TQ_F32 && !two_piece_x_serves_prod(d, p->bits_mse));
  // (d = 128 arrives here with bf16 rows that are only 8-byte aligned; params.images then holds the images of the
  // d = 128 kernels, which are not this kernel's)
  const char* const gemm_images = d != 128 ? static_cast<const char*>(p->images) : nullptr;
  a.W1_image = a.pieces ? gemm_images : nullptr;
  const NKind nk = dtype == TQ_F32 ? N_F32 : N_BF16;

  if (!prod) {
    // a handful of long vectors: a matrix-vector product per vector instead of the tiled contraction's serial k-loop,
    // when the workspace holds the rotated vectors
    if (rows_route_serves(n, d, 1) && !fp32_mfma_only(p)) {
      Workspace ws{static_cast<char*>(p->workspace), p->workspace_bytes, 0};
      if (float* const yw = static_cast<float*>(ws.take((size_t)n * d * sizeof(float))); yw != nullptr)
        return from_hip(launch_quant_rows(p->bits_mse, dtype == TQ_BF16, x, ldx, n, d, p->Pi, make_codebook(p), yw, idx, norm, stream));
    }
    a.X = x;
    a.n = n;
    a.rownorm_out = norm;
    a.words_out = idx;
    return from_hip(launch_gemm(nk, E_QUANT, p->bits_mse, a, 1, stream));
  }

  // a handful of long vectors: the matrix-vector route (see above), the sketch included
  if (rows_route_serves(n, d, 2) && !fp32_mfma_only(p)) {
    Workspace ws2{static_cast<char*>(p->workspace), p->workspace_bytes, 0};
    float* const yw = static_cast<float*>(ws2.take((size_t)n * d * sizeof(float)));
    float* const ew = static_cast<float*>(ws2.take((size_t)n * d * sizeof(float)));
    if (yw != nullptr && ew != nullptr)
      return from_hip(launch_quant_rows(p->bits_mse, dtype == TQ_BF16, x, ldx, n, d, p->Pi, make_codebook(p), yw, idx, norm, stream,
                                        p->SPiT, ew, qjl, gamma));
  }

  // prod: pass 1 writes idx and the rotated-basis residual e = y - c[idx];
  // pass 2 streams e (its row norms are gamma) against S Pi^T and packs signs.
  Workspace ws{static_cast<char*>(p->workspace), p->workspace_bytes, 0};
  int64_t chunk = n < kChunkRows ? n : kChunkRows;
  float* resid = nullptr;
  while (true) {
    resid = static_cast<float*>(ws.take((size_t)chunk * d * sizeof(float)));
    if (resid != nullptr || chunk <= 128) break;
    ws.used = 0;
    chunk = (chunk / 2 + 127) / 128 * 128;
  }
  if (resid == nullptr) return TQ_ERR_WORKSPACE;

  for (int64_t r0 = 0; r0 < n; r0 += chunk) {
    const int64_t rows = (n - r0 < chunk) ? n - r0 : chunk;
    GemmArgs a1 = a;
    a1.X = static_cast<const char*>(x) + (size_t)r0 * ldx * esz;
    a1.n = rows;
    a1.rownorm_out = norm ? norm + r0 : nullptr;
    a1.words_out = idx ? idx + r0 * words_per_row : nullptr;
    a1.resid_out = resid;
    hipError_t e = launch_gemm(nk, E_QUANT, p->bits_mse, a1, 1, stream);
    if (e != hipSuccess) return TQ_ERR_HIP;

    GemmArgs a2;
    std::memset(&a2, 0, sizeof(a2));
    a2.W1 = p->SPiT;
    a2.ldw = d;
    a2.M = d;
    a2.d = d;
    a2.segs = 1;
    a2.X = resid;
    a2.ldx = d;
    a2.n = rows;
    a2.rownorm_out = gamma + r0;
    a2.words_out = qjl + r0 * (d / 32);
    a2.pieces = pieces;  // the residual's own two pieces leave out 2^-17 of the residual: relative to gamma as it must be
    a2.W1_image = pieces && gemm_images != nullptr ? gemm_images + gemm_image_bytes(d, d, 3) : nullptr;
    e = launch_gemm(N_F32, E_SIGN, 0, a2, 1, stream);
    if (e != hipSuccess) return TQ_ERR_HIP;
  }
  return TQ_OK;
}

}  // namespace

extern "C" {

const char* tq_status_string(tq_status s) {
  switch (s) {
    case TQ_OK: return "TQ_OK";
    case TQ_ERR_INVALID_ARG: return "TQ_ERR_INVALID_ARG";
    case TQ_ERR_UNSUPPORTED: return "TQ_ERR_UNSUPPORTED";
    case TQ_ERR_HIP: return "TQ_ERR_HIP";
    case TQ_ERR_WORKSPACE: return "TQ_ERR_WORKSPACE";
    default: return "TQ_ERR_UNKNOWN";
  }
}

size_t tq_images_bytes(int32_t d) {
  if (d == 128) return quant128_bf3_image_bytes() + dequant128_bf3_image_bytes();
  if (d <= 0 || d % 32 != 0 || d > 16384) return 0;
  return gemm_image_bytes(d, d, 3) + gemm_image_bytes(d, d, 2);  // Pi in three pieces, S Pi^T in two
}

tq_status tq_build_images(const tq_params* p, void* images, void* stream) {
  if (p == nullptr || p->d <= 0) return TQ_ERR_INVALID_ARG;
  if (tq_images_bytes(p->d) == 0) return TQ_OK;  // no kernel at this d takes one
  if (images == nullptr || p->Pi == nullptr) return TQ_ERR_INVALID_ARG;
  if (p->d != 128) {
    // the generic quantiser: Pi, and S Pi^T when there is a sketch
    if ((p->S == nullptr) != (p->SPiT == nullptr)) return TQ_ERR_INVALID_ARG;
    if (!aligned16(images) || !aligned16(p->Pi) || (p->SPiT != nullptr && !aligned16(p->SPiT))) return TQ_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (launch_gemm_image(p->Pi, p->d, p->d, p->d, 3, images, s) != hipSuccess) return TQ_ERR_HIP;
    if (p->SPiT != nullptr &&
        launch_gemm_image(p->SPiT, p->d, p->d, p->d, 2, static_cast<char*>(images) + gemm_image_bytes(p->d, p->d, 3), s) != hipSuccess)
      return TQ_ERR_HIP;
    return TQ_OK;
  }
  if (p->PiT == nullptr) return TQ_ERR_INVALID_ARG;
  if ((p->S == nullptr) != (p->ST == nullptr) || (p->S == nullptr) != (p->SPiT == nullptr)) return TQ_ERR_INVALID_ARG;
  if (!aligned16(images) || !aligned16(p->Pi) || !aligned16(p->PiT) || (p->S != nullptr && (!aligned16(p->ST) || !aligned16(p->SPiT))))
    return TQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (launch_quant128_bf3_image(p->Pi, p->SPiT, images, s) != hipSuccess) return TQ_ERR_HIP;
  if (launch_dequant128_bf3_image(p->PiT, p->ST, static_cast<char*>(images) + quant128_bf3_image_bytes(), s) != hipSuccess)
    return TQ_ERR_HIP;
  return TQ_OK;
}

tq_status tq_derive_params(int32_t d, const float* Pi, const float* S, float* PiT, float* ST,
                           float* SPiT, void* stream) {
  if (d <= 0 || Pi == nullptr) return TQ_ERR_INVALID_ARG;
  if (d % 32 != 0 || d > 16384) return TQ_ERR_UNSUPPORTED;
  if ((ST != nullptr || SPiT != nullptr) && S == nullptr) return TQ_ERR_INVALID_ARG;
  if (!aligned16(Pi) || (S && !aligned16(S)) || (SPiT && !aligned16(SPiT))) return TQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (PiT != nullptr && launch_transpose(d, Pi, PiT, s) != hipSuccess) return TQ_ERR_HIP;
  if (ST != nullptr && launch_transpose(d, S, ST, s) != hipSuccess) return TQ_ERR_HIP;
  if (SPiT != nullptr) {
    // row m of S Pi^T is Pi applied to row m of S: the rotate contraction with
    // the rows of S as the vectors, stored plainly
    GemmArgs a;
    std::memset(&a, 0, sizeof(a));
    a.W1 = Pi;
    a.ldw = d;
    a.M = d;
    a.d = d;
    a.segs = 1;
    a.X = S;
    a.ldx = d;
    a.n = d;
    a.out = SPiT;
    a.ldo = d;
    if (launch_gemm(N_F32, E_STORE_T, 0, a, 1, s) != hipSuccess) return TQ_ERR_HIP;
  }
  return TQ_OK;
}

size_t tq_workspace_bytes(const tq_params* p, int64_t n, int64_t nq, int32_t topk) {
  if (p == nullptr || p->d <= 0 || n < 0 || nq < 0) return 0;
  const size_t d = (size_t)p->d;
  const size_t rows = (size_t)(n < kChunkRows ? n : kChunkRows);
  size_t bytes = round_up(rows * d * sizeof(float), 256);          // residual of quantize_prod
  // a handful of long vectors: their rotated coordinates beside the residual (the matrix-vector route)
  bytes += round_up((size_t)(n < kRowsQuantMax ? n : kRowsQuantMax) * d * sizeof(float), 256);
  bytes += 2 * round_up((size_t)nq * d * sizeof(float), 256);      // rotated / sketched queries
  bytes += round_up(score_i8_workspace_bytes(p->d, nq), 256);      // or their int8 digit images
  if (topk > 0) bytes += round_up((size_t)nq * (size_t)(n + 3) * sizeof(float), 256);  // scores when not returned
  // partial top-k lists of a few long rows: at most 4096 (score, index) pairs for each of at most 128 rows
  if (topk > 0) bytes += 2 * round_up((size_t)(nq < 128 ? nq : 128) * 4096 * sizeof(float), 256);
  return bytes + 256;
}

tq_status tq_quantize_mse(const tq_params* p, const void* x, int32_t dtype, int64_t n, int64_t ldx,
                          uint32_t* idx, float* norm, void* stream) {
  return quantize_common(p, x, dtype, n, ldx, idx, nullptr, nullptr, norm, false,
                         static_cast<hipStream_t>(stream));
}

tq_status tq_quantize_prod(const tq_params* p, const void* x, int32_t dtype, int64_t n, int64_t ldx,
                           uint32_t* idx, uint32_t* qjl, float* gamma, float* norm, void* stream) {
  return quantize_common(p, x, dtype, n, ldx, idx, qjl, gamma, norm, true,
                         static_cast<hipStream_t>(stream));
}

tq_status tq_append(const tq_params* p, const void* x, int32_t dtype, int64_t n, int64_t ldx, uint32_t* idx,
                    uint32_t* qjl, float* gamma, float* norm, int64_t first_row, int64_t row_step, void* stream) {
  if (first_row < 0 || row_step < 1) return TQ_ERR_INVALID_ARG;
  if (p != nullptr && p->d != 128) return TQ_ERR_UNSUPPORTED;
  if (n > kSmallQuantRows) return TQ_ERR_UNSUPPORTED;
  return quantize_common(p, x, dtype, n, ldx, idx, qjl, gamma, norm, qjl != nullptr, static_cast<hipStream_t>(stream),
                         first_row, row_step, true);
}

tq_status tq_dequantize(const tq_params* p, const uint32_t* idx, const uint32_t* qjl,
                        const float* gamma, const float* norm, int64_t n, float* x_out, int64_t ldo,
                        void* stream) {
  tq_status st = check_params(p, true);
  if (st != TQ_OK) return st;
  if (n < 0 || ldo < p->d) return TQ_ERR_INVALID_ARG;
  if (ldo > kMaxRowStride) return TQ_ERR_UNSUPPORTED;
  if (n == 0) return TQ_OK;
  const bool prod = qjl != nullptr;
  if (x_out == nullptr || p->PiT == nullptr || (p->bits_mse > 0 && idx == nullptr)) return TQ_ERR_INVALID_ARG;
  if (prod && (gamma == nullptr || p->ST == nullptr)) return TQ_ERR_INVALID_ARG;
  if (ldo % 4 != 0 || !aligned16(x_out) || !aligned16(p->PiT) || (prod && !aligned16(p->ST)))
    return TQ_ERR_UNSUPPORTED;
  if (p->d_hi != 0) {
    // two instances: d = 128 kernel only; idx rows are not 16-byte multiples there
    if (norm == nullptr || idx == nullptr || p->Pi == nullptr || (prod && p->S == nullptr)) return TQ_ERR_INVALID_ARG;
    if (!aligned16(p->Pi) || (prod && (!aligned16(p->S) || !aligned16(qjl)))) return TQ_ERR_UNSUPPORTED;
    if (n > kBf3DequantRows && !fp32_mfma_only(p) && p->PiT != nullptr && (!prod || p->ST != nullptr))
      return from_hip(launch_dequant128_bf3(p->bits_mse, prod, idx, qjl, gamma, norm, p->PiT, p->ST, x_out, ldo, n,
                                            kappa_of(p->d - p->d_hi), make_codebook(p), p->d_hi / 32, kappa_of(p->d_hi),
                                            make_codebook_hi(p), dequant_image(p), static_cast<hipStream_t>(stream)));
    return from_hip(launch_dequant128(p->bits_mse, prod, idx, qjl, gamma, norm, p->Pi, p->S, x_out, ldo, n,
                                      kappa_of(p->d - p->d_hi), make_codebook(p), p->d_hi / 32,
                                      kappa_of(p->d_hi), make_codebook_hi(p), static_cast<hipStream_t>(stream)));
  }
  // large batches at d = 128: decoded codes straight into bf16 MFMA operands, pieces of Pi^T / S^T in LDS
  if (p->d == 128 && n > kBf3DequantRows && !fp32_mfma_only(p) && dequant128_bf3_applicable(p->bits_mse, prod, make_codebook(p), x_out, ldo))
    return from_hip(launch_dequant128_bf3(p->bits_mse, prod, idx, qjl, gamma, norm, p->PiT, p->ST, x_out, ldo, n,
                                          kappa_of(128), make_codebook(p), 0, 0.f, make_codebook(p), dequant_image(p),
                                          static_cast<hipStream_t>(stream)));
  if (p->d == 128 && p->Pi != nullptr && aligned16(p->Pi) && (!prod || (p->S != nullptr && aligned16(p->S))) &&
      aligned16(idx) && (!prod || aligned16(qjl))) {
    return from_hip(launch_dequant128(p->bits_mse, prod, idx, qjl, gamma, norm, p->Pi, p->S, x_out, ldo, n,
                                      kappa_of(p->d), make_codebook(p), 0, 0.f, make_codebook(p),
                                      static_cast<hipStream_t>(stream)));
  }
  // a handful of long vectors: matrix-vector products (the matrices are read once per block of 4 vectors, 2 with a
  // sketch; the same bound as for the quantiser's route)
  if (p->d < 4096 && !fp32_mfma_only(p) && rows_route_serves(prod ? 2 * n : n, p->d, prod ? 2 : 1, 300))
    return from_hip(launch_dequant_rows(p->bits_mse, prod, p->d, n, idx, qjl, gamma, norm, p->PiT, p->ST, make_codebook(p),
                                        kappa_of(p->d), x_out, ldo, static_cast<hipStream_t>(stream)));
  // x~_i[k] = <e_k, DeQuant(code i)>: the scoring contraction with the rows of Pi^T (and S^T) as the queries,
  // stored one row per code; on the bf16 matrix cores where that kernel takes the codes
  if (!fp32_mfma_only(p) && score_bf3_applicable(p->bits_mse, prod, p->d, n, 1, p->d, make_codebook(p)))
    return from_hip(launch_score_bf3(p->bits_mse, prod, p->PiT, p->ST, p->d, p->d, idx, qjl, gamma, norm, n, 1, x_out, ldo,
                                     true, kappa_of(p->d), make_codebook(p), static_cast<hipStream_t>(stream)));
  GemmArgs a;
  std::memset(&a, 0, sizeof(a));
  a.W1 = p->PiT;  // x~[k] = sum_j Pi[j][k] y~[j]: rows of Pi^T against the decoded code
  a.W2 = p->ST;
  a.ldw = p->d;
  a.M = p->d;
  a.d = p->d;
  a.segs = prod ? 2 : 1;
  a.n = n;
  a.idx = idx;
  a.qjl = qjl;
  a.gamma = gamma;
  a.scale_in = norm;
  a.out = x_out;
  a.ldo = ldo;
  a.kappa = kappa_of(p->d);
  a.cb = make_codebook(p);
  return from_hip(launch_gemm(N_CODE, E_STORE_T, p->bits_mse, a, 1, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

namespace {

// How one tq_score call is carried out and what scratch memory it takes.  tq_score follows it and
// tq_score_workspace_bytes reports it, so the two cannot drift apart.
struct ScorePlan {
  enum Route { R_SPLIT_I8, R_I8, R_SMALL, R_BF3, R_GEMM } route;
  size_t img_bytes;     // int8 digit images of the rotated queries (R_SPLIT_I8, R_I8)
  size_t q_bytes;       // one [nq][d] fp32 matrix of rotated queries (other routes; a second one for prod)
  int64_t ld_scores;    // row stride of a score matrix in scratch memory
  size_t scores_bytes;  // that matrix: only when scores == NULL and top-k is not taken inside the scoring kernel
  int ranges;           // > 0: top-k inside the scoring kernel, this many partial lists per query
  int topk_chunks;      // > 0: top-k over a score matrix of few long rows, this many chunks (partial lists) per row
  size_t part_bytes;    // one array [nq][ranges or topk_chunks][topk] (values; indices take the same again)
  bool prod;
  size_t total() const {
    const size_t a = 256;
    size_t t = round_up(img_bytes, a) + (q_bytes ? round_up(q_bytes, a) * (prod ? 2 : 1) : 0) + round_up(scores_bytes, a) +
               2 * round_up(part_bytes, a);
    return t + a;
  }
};

ScorePlan plan_route(const tq_params* p, bool prod, int n_groups, int q_per_group, int64_t n_per_group, bool scores_given,
                     int topk, bool codes_aligned);

ScorePlan plan_score(const tq_params* p, bool prod, int n_groups, int q_per_group, int64_t n_per_group, bool scores_given,
                     int topk, bool codes_aligned) {
  ScorePlan pl = plan_route(p, prod, n_groups, q_per_group, n_per_group, scores_given, topk, codes_aligned);
  // top-k over a score matrix: a few long rows are cut into chunks so that the selection fills the chip
  if (topk > 0 && pl.ranges == 0) {
    const int64_t nq = (int64_t)n_groups * q_per_group;
    pl.topk_chunks = topk_chunks(nq, n_per_group, topk);
    if (pl.topk_chunks > 0) pl.part_bytes = (size_t)nq * pl.topk_chunks * topk * sizeof(float);
  }
  return pl;
}

ScorePlan plan_route(const tq_params* p, bool prod, int n_groups, int q_per_group, int64_t n_per_group, bool scores_given,
                     int topk, bool codes_aligned) {
  ScorePlan pl;
  std::memset(&pl, 0, sizeof(pl));
  pl.prod = prod;
  const int d = p->d;
  const int64_t nq = (int64_t)n_groups * q_per_group;
  pl.ld_scores = (n_per_group + 3) / 4 * 4;
  const size_t scratch_scores = scores_given ? 0 : (size_t)nq * pl.ld_scores * sizeof(float);
  if (p->d_hi != 0) {
    pl.route = ScorePlan::R_SPLIT_I8;
    pl.img_bytes = score_i8_workspace_bytes(d, nq);
    pl.scores_bytes = scratch_scores;
    return pl;
  }
  // few queries per code; with a short code list also a few more (every block of 4 queries re-reads the
  // codes, which costs less than the launches of the contraction path while the list is short)
  // (beyond 512 coordinates that kernel takes one launch per 512 and a matrix-vector kernel rotates the queries:
  // up to 16 queries per group, where the dense contraction would run on tiles that are mostly padding; up to 32
  // at d <= 1024, where the alternative is the lane-per-key kernel: measured at d = 1024 and 10^6 codes, 17-32
  // queries take 2.1-3.2 ms there and 1.1-1.7 ms here)
  if ((d <= 512 ? (q_per_group <= 32 || (q_per_group <= 64 && n_per_group <= 16384))
                : ((q_per_group <= 16 || (q_per_group <= 32 && d <= 1024)) && nq <= 64)) &&
      score_i8_applicable(p->bits_mse, d, make_codebook(p))) {
    pl.route = ScorePlan::R_I8;
    pl.img_bytes = score_i8_workspace_bytes(d, nq);
    pl.scores_bytes = scratch_scores;
    return pl;
  }
  pl.q_bytes = (size_t)nq * d * sizeof(float);
  if (q_per_group <= 32 && d % 128 == 0 && d <= 1024 && codes_aligned) {
    pl.route = ScorePlan::R_SMALL;
    pl.scores_bytes = scratch_scores;
    return pl;
  }
  if (n_per_group > 0 && !fp32_mfma_only(p) &&
      score_bf3_applicable(p->bits_mse, prod, d, n_per_group, n_groups, q_per_group, make_codebook(p))) {
    pl.route = ScorePlan::R_BF3;
    pl.ranges = topk > 0 ? score_bf3_topk_ranges(p->bits_mse, prod, n_per_group, n_groups, q_per_group, topk) : 0;
    if (pl.ranges > 0)
      pl.part_bytes = (size_t)nq * pl.ranges * topk * sizeof(float);
    else
      pl.scores_bytes = scratch_scores;
    return pl;
  }
  pl.route = ScorePlan::R_GEMM;
  pl.scores_bytes = scratch_scores;
  return pl;
}

// tq_score with the scratch memory given explicitly (the caller's workspace, or this library's static array)
tq_status score_impl(const tq_params* p, Workspace ws, const float* q, int64_t ldq, int32_t n_groups,
                     int32_t q_per_group, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                     const float* norm, int64_t n_per_group, float* scores, int64_t lds, int32_t topk,
                     int32_t* topk_idx, float* topk_val, void* stream) {
  tq_status st = check_params(p, true);
  if (st != TQ_OK) return st;
  if (n_groups < 0 || q_per_group < 0 || n_per_group < 0 || ldq < p->d || topk < 0) return TQ_ERR_INVALID_ARG;
  // groups and blocks of four queries are grid dimensions of the few-query kernels
  if (topk > 64 || n_per_group > 0x7fffffff || n_groups > 65535 || q_per_group > 4 * 65535 || ldq > kMaxRowStride)
    return TQ_ERR_UNSUPPORTED;
  const int64_t nq = (int64_t)n_groups * q_per_group;
  if (nq == 0) return TQ_OK;
  const bool prod = qjl != nullptr;
  if (q == nullptr || p->Pi == nullptr) return TQ_ERR_INVALID_ARG;
  if (n_per_group > 0 && p->bits_mse > 0 && idx == nullptr) return TQ_ERR_INVALID_ARG;
  if (prod && (gamma == nullptr || p->S == nullptr)) return TQ_ERR_INVALID_ARG;
  if (scores == nullptr && topk == 0) return TQ_ERR_INVALID_ARG;
  if (scores != nullptr && lds < n_per_group) return TQ_ERR_INVALID_ARG;
  if (topk > 0 && topk_idx == nullptr) return TQ_ERR_INVALID_ARG;
  if (ldq % 4 != 0 || !aligned16(q) || !aligned16(p->Pi) || (prod && !aligned16(p->S))) return TQ_ERR_UNSUPPORTED;
  if (p->d_hi != 0) {
    // two instances over a split of the coordinates: d = 128, the kernel written for few queries per code (every
    // block of four queries streams the group's codes once more, so many queries are served, not served fast)
    if (norm == nullptr) return TQ_ERR_INVALID_ARG;
    if (q_per_group > 4096 || !score_i8_split_applicable(p->bits_mse, make_codebook(p), make_codebook_hi(p)))
      return TQ_ERR_UNSUPPORTED;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int d = p->d;
  const ScorePlan pl = plan_score(p, prod, n_groups, q_per_group, n_per_group, scores != nullptr, topk,
                                  aligned16(idx) && (!prod || aligned16(qjl)));

  // all scratch memory is taken before the first launch
  void* img = pl.img_bytes ? ws.take(pl.img_bytes) : nullptr;
  float* qr = pl.q_bytes ? static_cast<float*>(ws.take(pl.q_bytes)) : nullptr;
  float* qs = pl.q_bytes && prod ? static_cast<float*>(ws.take(pl.q_bytes)) : nullptr;
  int64_t ld_scores = lds;
  if (scores == nullptr && pl.scores_bytes) {
    ld_scores = pl.ld_scores;
    scores = static_cast<float*>(ws.take(pl.scores_bytes));
    if (scores == nullptr) return TQ_ERR_WORKSPACE;
  }
  float* part_val = pl.part_bytes ? static_cast<float*>(ws.take(pl.part_bytes)) : nullptr;
  int32_t* part_idx = pl.part_bytes ? static_cast<int32_t*>(ws.take(pl.part_bytes)) : nullptr;
  // the chunks of a top-k over a score matrix are an optimisation: without room for their lists, one workgroup per row
  const int topk_chunks = (part_val != nullptr && part_idx != nullptr) ? pl.topk_chunks : 0;
  if ((pl.img_bytes && img == nullptr) || (pl.q_bytes && (qr == nullptr || (prod && qs == nullptr))) ||
      (pl.ranges > 0 && (part_val == nullptr || part_idx == nullptr)))
    return TQ_ERR_WORKSPACE;

  if (pl.route == ScorePlan::R_SPLIT_I8) {
    if (launch_score_i8_split(p->bits_mse, prod, p->Pi, p->S, p->PiT, p->ST, q, ldq, img, idx, qjl, gamma, norm, scores, ld_scores,
                              n_per_group, n_groups, q_per_group, p->d_hi / 32, kappa_of(d - p->d_hi),
                              kappa_of(p->d_hi), make_codebook(p), make_codebook_hi(p), s) != hipSuccess)
      return TQ_ERR_HIP;
  } else if (pl.route == ScorePlan::R_I8) {
    // masked sums of fixed-point query digits on the int8 matrix cores (at d = 128 one kernel; otherwise a
    // preparation kernel rotates the queries and writes their digits)
    if (launch_score_i8(p->bits_mse, prod, p->Pi, p->S, p->PiT, p->ST, q, ldq, img, idx, qjl, gamma, norm, scores, ld_scores,
                        n_per_group, d, n_groups, q_per_group, kappa_of(d), make_codebook(p), s) != hipSuccess)
      return TQ_ERR_HIP;
  } else {
    // queries into the rotated basis and the sketch basis: Pi q and S q
    if (nq <= 64 && d <= 4096) {
      if (launch_matvec_small(d, (int)nq, p->Pi, prod ? p->S : nullptr, q, ldq, qr, qs, s) != hipSuccess)
        return TQ_ERR_HIP;
    } else {
      GemmArgs a;
      std::memset(&a, 0, sizeof(a));
      a.W1 = p->Pi;
      a.ldw = d;
      a.M = d;
      a.d = d;
      a.segs = 1;
      a.X = q;
      a.ldx = ldq;
      a.n = nq;
      a.out = qr;
      a.ldo = d;
      if (launch_gemm(N_F32, E_STORE_T, 0, a, 1, s) != hipSuccess) return TQ_ERR_HIP;
      if (prod) {
        a.W1 = p->S;
        a.out = qs;
        if (launch_gemm(N_F32, E_STORE_T, 0, a, 1, s) != hipSuccess) return TQ_ERR_HIP;
      }
    }
    if (n_per_group > 0 && pl.route == ScorePlan::R_SMALL) {
      // few queries per code: stream the codes once, lane = key
      if (launch_score_small(p->bits_mse, prod, qr, qs, idx, qjl, gamma, norm, scores, ld_scores, n_per_group,
                             d, n_groups, q_per_group, kappa_of(d), make_codebook(p), s) != hipSuccess)
        return TQ_ERR_HIP;
    } else if (pl.route == ScorePlan::R_BF3) {
      // many queries per code: dense contraction on the bf16 matrix cores, every fp32 factor as two bf16 pieces;
      // with top-k wanted the kernel keeps the k best pairs of every query itself and a small kernel joins them
      if (launch_score_bf3(p->bits_mse, prod, qr, qs, q_per_group, d, idx, qjl, gamma, norm, n_per_group, n_groups, scores,
                           ld_scores, false, kappa_of(d), make_codebook(p), s, pl.ranges > 0 ? topk : 0, part_val,
                           part_idx) != hipSuccess)
        return TQ_ERR_HIP;
      if (pl.ranges > 0)
        return from_hip(launch_topk_merge(part_val, part_idx, nq, pl.ranges, topk, topk_idx, topk_val, s));
    } else if (n_per_group > 0) {
      GemmArgs a;
      std::memset(&a, 0, sizeof(a));
      a.W1 = qr;
      a.W2 = qs;
      a.ldw = d;
      a.w_group_stride = (int64_t)q_per_group * d;
      a.M = q_per_group;
      a.d = d;
      a.segs = prod ? 2 : 1;
      a.n = n_per_group;
      a.idx = idx;
      a.qjl = qjl;
      a.gamma = gamma;
      a.scale_in = norm;
      a.out = scores;
      a.ldo = ld_scores;
      a.out_group_stride = (int64_t)q_per_group * ld_scores;
      a.kappa = kappa_of(d);
      a.cb = make_codebook(p);
      if (launch_gemm(N_CODE, E_STORE_N, p->bits_mse, a, n_groups, s) != hipSuccess) return TQ_ERR_HIP;
    }
  }
  if (topk > 0 && topk_chunks > 0) {
    if (launch_topk(scores, nq, n_per_group, ld_scores, topk, nullptr, nullptr, s, topk_chunks, part_val, part_idx) != hipSuccess)
      return TQ_ERR_HIP;
    return from_hip(launch_topk_merge(part_val, part_idx, nq, topk_chunks, topk, topk_idx, topk_val, s));
  }
  if (topk > 0) return from_hip(launch_topk(scores, nq, n_per_group, ld_scores, topk, topk_idx, topk_val, s));
  return TQ_OK;
}

// Scratch memory of tq_score_static: one copy per GPU the library runs on, held until the process ends.
constexpr size_t kStaticScratchBytes = size_t(16) << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once asked for

// The array's name is only a host-side handle: its address in the current device's memory has to be asked for.
tq_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return TQ_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return TQ_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return TQ_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return TQ_OK;
}

}  // namespace

extern "C" {

tq_status tq_score(const tq_params* p, const float* q, int64_t ldq, int32_t n_groups,
                   int32_t q_per_group, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                   const float* norm, int64_t n_per_group, float* scores, int64_t lds, int32_t topk,
                   int32_t* topk_idx, float* topk_val, void* stream) {
  if (p == nullptr) return TQ_ERR_INVALID_ARG;
  return score_impl(p, Workspace{static_cast<char*>(p->workspace), p->workspace_bytes, 0}, q, ldq, n_groups, q_per_group,
                    idx, qjl, gamma, norm, n_per_group, scores, lds, topk, topk_idx, topk_val, stream);
}

size_t tq_score_workspace_bytes(const tq_params* p, int32_t n_groups, int32_t q_per_group, int64_t n_per_group,
                                int32_t prod, int32_t scores_given, int32_t topk) {
  if (p == nullptr || p->d <= 0 || p->bits_mse < 0 || p->bits_mse > 4 || n_groups < 0 || q_per_group < 0 || n_per_group < 0 ||
      topk < 0 || topk > 64 || p->centroids == nullptr || (p->bits_mse > 0 && p->bounds == nullptr))
    return 0;
  // codes that are not 16-byte aligned can take a route with the smaller need; report the larger
  const size_t a = plan_score(p, prod != 0, n_groups, q_per_group, n_per_group, scores_given != 0, topk, true).total();
  const size_t b = plan_score(p, prod != 0, n_groups, q_per_group, n_per_group, scores_given != 0, topk, false).total();
  return a > b ? a : b;
}

size_t tq_score_static_scratch_bytes(void) { return kStaticScratchBytes; }

tq_status tq_score_static(const tq_params* p, const float* q, int64_t ldq, int32_t n_groups,
                          int32_t q_per_group, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                          const float* norm, int64_t n_per_group, float* scores, int64_t lds, int32_t topk,
                          int32_t* topk_idx, float* topk_val, void* stream) {
  if (p == nullptr || n_groups < 0 || q_per_group < 0 || n_per_group < 0) return TQ_ERR_INVALID_ARG;
  // the whole need of the call must fit the static array
  const size_t need = tq_score_workspace_bytes(p, n_groups, q_per_group, n_per_group, qjl != nullptr, scores != nullptr, topk);
  if (need == 0) return TQ_ERR_INVALID_ARG;
  if (need > kStaticScratchBytes) return TQ_ERR_WORKSPACE;
  void* base = nullptr;
  const tq_status st = static_scratch(&base);
  if (st != TQ_OK) return st;
  return score_impl(p, Workspace{static_cast<char*>(base), kStaticScratchBytes, 0}, q, ldq, n_groups, q_per_group, idx, qjl,
                    gamma, norm, n_per_group, scores, lds, topk, topk_idx, topk_val, stream);
}

}  // extern "C"

namespace {
struct AttendPlan {
  bool fast;  // the d = 128 kernel on the integer matrix cores takes the value codes
  int nchunks;
  int64_t ld_scores;
  size_t scores_bytes, part_bytes, score_ws_bytes;
};
AttendPlan attend_plan(const tq_params* pk, const tq_params* pv, bool v_prod, int64_t nq, int64_t n_per_group) {
  AttendPlan pl;
  const Codebook v_hi = make_codebook_hi(pv);
  pl.fast = pv->centroids != nullptr && (pv->d_hi == 0 || pv->centroids_hi != nullptr) &&
            attend128_applicable(pv->d, v_prod, make_codebook(pv), pv->d_hi != 0 ? &v_hi : nullptr);
  pl.nchunks = pl.fast ? attend128_chunks(n_per_group) : attend_simple_chunks(n_per_group);
  pl.ld_scores = (n_per_group + 3) / 4 * 4;
  pl.scores_bytes = round_up((size_t)nq * pl.ld_scores * sizeof(float), 256);
  pl.part_bytes = round_up((size_t)nq * pl.nchunks * attend_part_stride(pv->d) * sizeof(float), 256);
  pl.score_ws_bytes = tq_workspace_bytes(pk, 0, nq, 0);
  return pl;
}
}  // namespace

extern "C" {

size_t tq_attend_workspace_bytes(const tq_params* pk, const tq_params* pv, int32_t n_groups, int32_t q_per_group,
                                 int64_t n_per_group) {
  if (pk == nullptr || pv == nullptr || pk->d <= 0 || pv->d <= 0 || n_groups < 0 || q_per_group < 0 || n_per_group < 0)
    return 0;
  // whichever kind of value code the call then brings
  const AttendPlan pl = attend_plan(pk, pv, true, (int64_t)n_groups * q_per_group, n_per_group);
  const AttendPlan pm = attend_plan(pk, pv, false, (int64_t)n_groups * q_per_group, n_per_group);
  return pl.scores_bytes + (pl.part_bytes > pm.part_bytes ? pl.part_bytes : pm.part_bytes) + pl.score_ws_bytes + 512;
}

tq_status tq_attend(const tq_params* pk, const tq_params* pv, const float* q, int64_t ldq, int32_t n_groups,
                    int32_t q_per_group, const uint32_t* k_idx, const uint32_t* k_qjl, const float* k_gamma,
                    const float* k_norm, const uint32_t* v_idx, const uint32_t* v_qjl, const float* v_gamma,
                    const float* v_norm, int64_t n_per_group, float scale, float* out, int64_t ldo, void* stream) {
  return tq_attend_cache(pk, pv, q, ldq, n_groups, q_per_group, k_idx, k_qjl, k_gamma, k_norm, v_idx, v_qjl, v_gamma, v_norm,
                         n_per_group, n_per_group, scale, out, ldo, stream);
}

tq_status tq_attend_cache(const tq_params* pk, const tq_params* pv, const float* q, int64_t ldq, int32_t n_groups,
                          int32_t q_per_group, const uint32_t* k_idx, const uint32_t* k_qjl, const float* k_gamma,
                          const float* k_norm, const uint32_t* v_idx, const uint32_t* v_qjl, const float* v_gamma,
                          const float* v_norm, int64_t n_per_group, int64_t group_stride, float scale, float* out,
                          int64_t ldo, void* stream) {
  tq_status st = check_params(pk, true);
  if (st != TQ_OK) return st;
  st = check_params(pv, true);
  if (st != TQ_OK) return st;
  if (n_groups < 0 || q_per_group < 0 || n_per_group < 0 || ldo < pv->d || group_stride < n_per_group) return TQ_ERR_INVALID_ARG;
  const int64_t nq = (int64_t)n_groups * q_per_group;
  if (nq == 0) return TQ_OK;
  const bool v_prod = v_qjl != nullptr;
  if (out == nullptr || pv->Pi == nullptr || (v_prod && (v_gamma == nullptr || pv->S == nullptr)))
    return TQ_ERR_INVALID_ARG;
  if (n_per_group > 0 && (v_norm == nullptr || (pv->bits_mse > 0 && v_idx == nullptr))) return TQ_ERR_INVALID_ARG;
  if (pv->d > 4096 || n_groups > 65535 || q_per_group > 4 * 65535 || ldq > kMaxRowStride || ldo > kMaxRowStride)
    return TQ_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);

  const AttendPlan pl = attend_plan(pk, pv, v_prod, nq, n_per_group);
  // value codes of two instances: the d = 128 kernel or nothing
  if (pv->d_hi != 0 && !pl.fast) return TQ_ERR_UNSUPPORTED;
  if (pl.nchunks > 4096) return TQ_ERR_UNSUPPORTED;  // the joining kernel keeps one factor per chunk in LDS
  Workspace ws{static_cast<char*>(pk->workspace), pk->workspace_bytes, 0};
  float* scores = static_cast<float*>(ws.take(pl.scores_bytes));
  float* part = static_cast<float*>(ws.take(pl.part_bytes));
  char* rest = static_cast<char*>(ws.take(pl.score_ws_bytes));
  if (scores == nullptr || part == nullptr || rest == nullptr) return TQ_ERR_WORKSPACE;
  if (n_per_group > 0) {
    AttendArgs a;
    a.scores = scores; a.lds = pl.ld_scores;
    a.idx = v_idx; a.qjl = v_qjl; a.gamma = v_gamma; a.norm = v_norm;
    a.part = part; a.nchunks = pl.nchunks; a.n = n_per_group; a.group_stride = group_stride; a.d = pv->d; a.q_per_group = q_per_group;
    a.scale = scale; a.cb = make_codebook(pv); a.gs_hi = pv->d_hi / 32; a.cb_hi = make_codebook_hi(pv);
    // keys the single-kernel d = 128 scoring path takes are scored inside the read-out kernel
    const bool k_prod = k_qjl != nullptr;
    ScoreI8Args ka;
    const bool fused = pl.fast && pk->d == 128 && pk->d_hi == 0 && q != nullptr && ldq >= 128 &&
                       score128_args(pk->bits_mse, k_prod, pk->PiT, pk->ST, q, ldq, k_idx, k_qjl, k_gamma, k_norm,
                                     n_per_group, n_groups, q_per_group, kappa_of(128), make_codebook(pk), group_stride, &ka);
    if (fused) {
      if (launch_attend128(pk->bits_mse, k_prod, &ka, v_prod, a, n_groups, s) != hipSuccess) return TQ_ERR_HIP;
    } else {
      // tq_score knows densely stored groups only
      if (group_stride != n_per_group) return TQ_ERR_UNSUPPORTED;
      tq_params pk_inner = *pk;  // the scoring call carves its own needs from what is left
      pk_inner.workspace = rest;
      pk_inner.workspace_bytes = pl.score_ws_bytes;
      st = tq_score(&pk_inner, q, ldq, n_groups, q_per_group, k_idx, k_qjl, k_gamma, k_norm, n_per_group, scores,
                    pl.ld_scores, 0, nullptr, nullptr, stream);
      if (st != TQ_OK) return st;
      if ((pl.fast ? launch_attend128(0, false, nullptr, v_prod, a, n_groups, s) : launch_attend_values(v_prod, a, n_groups, s)) !=
          hipSuccess)
        return TQ_ERR_HIP;
    }
  }
  return from_hip(launch_attend_combine(part, pl.nchunks, pv->d, nq, pv->Pi, v_prod ? pv->S : nullptr,
                                        kappa_of(pv->d), out, ldo, s));
}

tq_status tq_stage_pack(const tq_params* p, const float* y, int64_t n, uint32_t* idx, void* stream) {
  tq_status st = check_params(p, true);
  if (st != TQ_OK) return st;
  if (p->d_hi != 0) return TQ_ERR_UNSUPPORTED;  // the stand-alone stages know one instance only
  if (n < 0) return TQ_ERR_INVALID_ARG;
  if (n == 0 || p->bits_mse == 0) return TQ_OK;
  if (y == nullptr || idx == nullptr) return TQ_ERR_INVALID_ARG;
  return from_hip(launch_stage_pack(make_codebook(p), p->d, y, n, idx, static_cast<hipStream_t>(stream)));
}

tq_status tq_stage_sign_pack(int32_t d, const float* u, int64_t n, uint32_t* qjl, void* stream) {
  if (d <= 0 || n < 0) return TQ_ERR_INVALID_ARG;
  if (d % 32 != 0) return TQ_ERR_UNSUPPORTED;
  if (n == 0) return TQ_OK;
  if (u == nullptr || qjl == nullptr) return TQ_ERR_INVALID_ARG;
  return from_hip(launch_stage_sign_pack(d, u, n, qjl, static_cast<hipStream_t>(stream)));
}

tq_status tq_stage_unpack(const tq_params* p, const uint32_t* idx, int64_t n, float* y_tilde,
                          void* stream) {
  tq_status st = check_params(p, true);
  if (st != TQ_OK) return st;
  if (p->d_hi != 0) return TQ_ERR_UNSUPPORTED;  // the stand-alone stages know one instance only
  if (n < 0) return TQ_ERR_INVALID_ARG;
  if (n == 0) return TQ_OK;
  if (y_tilde == nullptr || (p->bits_mse > 0 && idx == nullptr)) return TQ_ERR_INVALID_ARG;
  return from_hip(launch_stage_unpack(make_codebook(p), p->d, idx, n, y_tilde, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

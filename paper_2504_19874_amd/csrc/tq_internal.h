// Internal declarations shared by the HIP translation units of the library.
// Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/turboquant.h"

namespace tq {

constexpr int kMaxDevices = 64;

// Compute units of the current device (asked once per device; 256 when the query fails).
int device_cu_count();

// A kernel that needs more dynamic LDS than the default limit has the limit raised once per
// device and instantiation; concurrent first calls from several host threads are serialised.
struct LdsLimit {
  std::once_flag once[kMaxDevices];
  hipError_t err[kMaxDevices];
};
inline hipError_t raise_lds_limit(LdsLimit& st, const void* kernel, int bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::call_once(st.once[dev], [&] {
    st.err[dev] = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  });
  return st.err[dev];
}

// Codebook of Alg. 1 passed to kernels by value (lives in scalar registers).
struct Codebook {
  float c[16];  // centroids, ascending
  float t[15];  // cell boundaries: midpoints of consecutive centroids
  int bits;
};

// ---------------------------------------------------------------------------
// The one contraction kernel.  It computes, for a block of "vectors" i (the
// N side) and a block of "rows" m (the M side),
//     D[m][i] = sum_k W[m][k] * V[i][k],        k over one or two segments,
// with both operands contiguous along k, using v_mfma_f32_32x32x2_f32.
// What V is and what happens to D are template choices:
//   V:  fp32 rows / bf16 rows (optionally unit-normalised on the fly) or
//       packed codes decoded on the fly (centroid values, then +-kappa*gamma)
//   D:  stored transposed (out[i][m]) or plain (out[m][i]), or turned into
//       packed indices (nearest centroid + bit planes) or packed signs.
// ---------------------------------------------------------------------------
enum NKind { N_F32 = 0, N_BF16 = 1, N_CODE = 2 };
enum EKind { E_STORE_T = 0, E_STORE_N = 1, E_QUANT = 2, E_SIGN = 3 };

struct GemmArgs {
  // M side: W1 (segment 1) and W2 (segment 2), row stride ldw, M rows per group
  const float* W1;
  const float* W2;
  int64_t ldw;
  int64_t w_group_stride;  // elements between the W rows of consecutive groups
  int M;
  // K: d per segment
  int d;
  int segs;
  // N side
  const void* X;  // fp32 or bf16 rows
  int64_t ldx;
  int64_t n;                // vectors per group
  const uint32_t* idx;      // codes: n_groups*n rows
  const uint32_t* qjl;
  const float* gamma;
  const float* scale_in;    // per-vector factor applied to stored D (norm), nullable
  int normalise;            // fp32/bf16 rows: divide by the row's L2 norm
  float* rownorm_out;       // sqrt(sum of squares of the streamed row), nullable
  // outputs
  float* out;
  int64_t ldo;
  int64_t out_group_stride;
  uint32_t* words_out;
  float* resid_out;  // E_QUANT: y - c[idx], n rows of d floats, nullable
  float kappa;       // sqrt(pi/2)/d
  int pieces;        // E_QUANT / E_SIGN: multiply bf16 pieces of the fp32 factors instead of the fp32 values
  // pieces, nullable: W1 already split, [row][k / 32][piece][32 k] bf16 with 3 (E_QUANT) or 2 (E_SIGN) pieces, as
  // launch_gemm_image writes it; the kernel then copies its W tiles instead of splitting them in every workgroup
  const void* W1_image;
  Codebook cb;
};

size_t gemm_image_bytes(int M, int d, int np);
hipError_t launch_gemm_image(const float* W, int64_t ldw, int M, int d, int np, void* image, hipStream_t stream);

hipError_t launch_gemm(NKind nk, EKind ek, int bits, const GemmArgs& a, int n_groups,
                       hipStream_t stream);

// d = 128 fused kernels (tq_d128.hip)
hipError_t launch_quant128(int bits, bool prod, bool bf16, const void* X, int64_t ldx, int64_t n,
                           const float* Pi, const float* SPiT, uint32_t* idx, uint32_t* qjl, float* gamma,
                           float* norm, const Codebook& cb, int gs_hi, const Codebook& cb_hi, hipStream_t s);
// d = 128, few vectors: one workgroup per block of 32 (tq_d128_small.hip)
constexpr int64_t kSmallQuantRows = 24576;
hipError_t launch_quant128_small(int bits, bool prod, bool bf16, const void* X, int64_t ldx, int64_t n,
                                 const float* Pi, const float* SPiT, uint32_t* idx, uint32_t* qjl,
                                 float* gamma, float* norm, const Codebook& cb, int gs_hi,
                                 const Codebook& cb_hi, hipStream_t s, int64_t out_first = 0, int64_t out_step = 1);
hipError_t launch_dequant128_small(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl,
                                   const float* gamma, const float* norm, const float* Pi, const float* S,
                                   float* out, int64_t ldo, int64_t n, float kappa, const Codebook& cb,
                                   int gs_hi, float kappa_hi, const Codebook& cb_hi, hipStream_t s);
constexpr int64_t kSmallDequantRows = 24576;  // crossover of the two fp32 kernels
constexpr int64_t kBf3DequantRows = 8192;     // above this the bf16-piece kernel wins (12 us at 32768 against 37)
hipError_t launch_dequant128(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl,
                             const float* gamma, const float* norm, const float* Pi, const float* S,
                             float* out, int64_t ldo, int64_t n, float kappa, const Codebook& cb,
                             int gs_hi, float kappa_hi, const Codebook& cb_hi, hipStream_t s);

// d = 128, large batches, bf16 matrix cores at fp32 accuracy (tq_d128_bf3.hip)
bool dequant128_bf3_applicable(int bits, bool prod, const Codebook& cb, const float* out, int64_t ldo);
constexpr int64_t kBf3QuantRows = 8193;   // bf16 input: from here on the bf16-piece kernel wins (17 us flat up to 65536 rows against 20 / 29 / 37)
bool quant128_bf3_applicable(int bits, bool prod, bool f32, const void* X, int64_t ldx, const Codebook& cb, const Codebook* cb_hi);
hipError_t launch_quant128_bf3(int bits, bool prod, bool f32, const void* X, int64_t ldx, int64_t n, const float* Pi,
                               const float* SPiT, uint32_t* idx, uint32_t* qjl, float* gamma, float* norm,
                               const Codebook& cb, int gs_hi, const Codebook& cb_hi, const void* image, hipStream_t s);
// the matrices of those two kernels as they sit in LDS, made once (tq_build_images); null pointers above mean
// "split the fp32 matrices in the kernel's prologue"
size_t quant128_bf3_image_bytes();
size_t dequant128_bf3_image_bytes();
hipError_t launch_quant128_bf3_image(const float* Pi, const float* SPiT, void* image, hipStream_t s);
hipError_t launch_dequant128_bf3_image(const float* PiT, const float* ST, void* image, hipStream_t s);
hipError_t launch_dequant128_bf3(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                                 const float* norm, const float* PiT, const float* ST, float* out, int64_t ldo, int64_t n,
                                 float kappa, const Codebook& cb, int gs_hi, float kappa_hi, const Codebook& cb_hi,
                                 const void* image, hipStream_t s);

// few queries per code (tq_score_small.hip)
// Quant_mse / Quant_prod for a handful of long vectors: y = Pi x by a matrix-vector kernel into yw [n][d], then norm,
// decision and packing per vector (tq_score_small.hip); with ew != NULL also the residual e = y - c[idx] into ew
// [n][d], gamma = |e|, u = (S Pi^T) e by the same matrix-vector kernel and its signs into qjl.  d a multiple of 32 up
// to 4096.
hipError_t launch_quant_rows(int bits, bool bf16, const void* x, int64_t ldx, int64_t n, int d, const float* Pi,
                             const Codebook& cb, float* yw, uint32_t* idx, float* norm, hipStream_t stream,
                             const float* SPiT = nullptr, float* ew = nullptr, uint32_t* qjl = nullptr, float* gamma = nullptr);
// DeQuant for a handful of long vectors by matrix-vector products (tq_score_small.hip); d a multiple of 32 up to 4096
hipError_t launch_dequant_rows(int bits, bool prod, int d, int64_t n, const uint32_t* idx, const uint32_t* qjl,
                               const float* gamma, const float* norm, const float* PiT, const float* ST, const Codebook& cb,
                               float kappa, float* out, int64_t ldo, hipStream_t s);
hipError_t launch_matvec_small(int d, int nq, const float* W0, const float* W1, const float* x,
                               int64_t ldx, float* out0, float* out1, hipStream_t stream);
hipError_t launch_score_small(int bits, bool prod, const float* qr, const float* qs, const uint32_t* idx,
                              const uint32_t* qjl, const float* gamma, const float* norm, float* scores,
                              int64_t lds, int64_t n, int d, int n_groups, int q_per_group, float kappa,
                              const Codebook& cb, hipStream_t stream);

// few queries per code on the integer matrix cores (tq_score_i8.hip)
size_t score_i8_workspace_bytes(int d, int64_t nq);
bool score_i8_applicable(int bits, int d, const Codebook& cb);
// d = 128 split into two instances (tq_score_i8_split.hip)
bool score_i8_split_applicable(int bits_lo, const Codebook& cb_lo, const Codebook& cb_hi);
hipError_t launch_score_i8_split(int bits_lo, bool prod, const float* Pi, const float* S, const float* PiT,
                                 const float* ST, const float* q, int64_t ldq,
                                 void* workspace, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                                 const float* norm, float* scores, int64_t lds, int64_t n, int n_groups,
                                 int q_per_group, int gs_hi, float kappa_lo, float kappa_hi, const Codebook& cb_lo,
                                 const Codebook& cb_hi, hipStream_t stream);  // d % 128 == 0, d <= 512, symmetric table
hipError_t launch_score_i8(int bits, bool prod, const float* Pi, const float* S, const float* PiT, const float* ST,
                           const float* q, int64_t ldq,
                           void* workspace, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                           const float* norm, float* scores, int64_t lds, int64_t n, int d, int n_groups,
                           int q_per_group, float kappa, const Codebook& cb, hipStream_t stream);

// many queries per code on the bf16 matrix cores, fp32 factors as two bf16 pieces (tq_score_bf3.hip)
bool score_bf3_applicable(int bits, bool prod, int d, int64_t n, int n_groups, int q_per_group, const Codebook& cb);
hipError_t launch_score_bf3(int bits, bool prod, const float* qr, const float* qs, int q_per_group, int d,
                            const uint32_t* idx, const uint32_t* qjl, const float* gamma, const float* norm, int64_t n,
                            int n_groups, float* out, int64_t ldo, bool transposed, float kappa, const Codebook& cb,
                            hipStream_t s, int topk = 0, float* part_val = nullptr, int32_t* part_idx = nullptr);
// transposed: out[code][query] (queries = rows of Pi^T: dequantisation).  topk in 1..16 (not transposed): the
// kernel also keeps the topk best (score, index) pairs of every query per range of code tiles and writes them
// to part_val / part_idx [n_groups * q_per_group][ranges][topk], ranges = score_bf3_topk_ranges(...); out may
// then be NULL.  launch_topk_merge joins the ranges (descending, equal scores by lower index, -1 past n).
int score_bf3_topk_ranges(int bits, bool prod, int64_t n, int n_groups, int q_per_group, int topk);
hipError_t launch_topk_merge(const float* part_val, const int32_t* part_idx, int64_t rows, int ranges, int k,
                             int32_t* out_idx, float* out_val, hipStream_t s);

// codec stages
hipError_t launch_stage_pack(const Codebook& cb, int d, const float* y, int64_t n, uint32_t* idx,
                             hipStream_t stream);
hipError_t launch_stage_sign_pack(int d, const float* u, int64_t n, uint32_t* qjl,
                                  hipStream_t stream);
hipError_t launch_stage_unpack(const Codebook& cb, int d, const uint32_t* idx, int64_t n,
                               float* y_tilde, hipStream_t stream);

// out[c][r] = in[r][c] for a d x d matrix
hipError_t launch_transpose(int d, const float* in, float* out, hipStream_t stream);

// per-row top-k of scores[rows][ld] over the first n columns.  A few long rows are cut into chunks (topk_chunks > 0):
// the call then writes the k best pairs of every chunk to part_val / part_idx [rows][chunks][k] and
// launch_topk_merge(part_val, part_idx, rows, chunks, k, ...) joins them.
int topk_chunks(int64_t rows, int64_t n, int k);
hipError_t launch_topk(const float* scores, int64_t rows, int64_t n, int64_t ld, int k,
                       int32_t* out_idx, float* out_val, hipStream_t stream, int chunks = 0, float* part_val = nullptr,
                       int32_t* part_idx = nullptr);

}  // namespace tq

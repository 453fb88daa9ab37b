// Shared by the two few-query scoring kernels on the integer matrix cores
// (tq_score_i8.hip: any d that is a multiple of 128 up to 4096, queries prepared by a
// kernel of their own, 512 coordinates per launch; tq_score_i8_128.hip: d = 128 with everything in one kernel).
#pragma once
#include "tq_internal.h"

namespace tq {

typedef int v4i __attribute__((ext_vector_type(4)));

// coordinate block of (k-step s, k-chunk kq): 16 coordinates starting here
__host__ __device__ constexpr int i8_coord0(int s, int kq) { return 32 * (kq + 4 * (s >> 1)) + 16 * (s & 1); }

// Image of one query's A operand, written by prep_i8_kernel: for matrix m (0: Pi q, 1: S q),
// k-step s, digit row dg, k-chunk kq the 16 bytes of coordinates i8_coord0(s, kq) .. + 15.
//   bytes:   img[((q * 2 + m) * ks + s) * 16 + dg * 4 + kq]      (16-byte units)
//   scalars: scal[(q * 2 + m) * 4 + {0: 1/scale, 1: sum of the rounded coordinates, 2 and 3: the same sum over
//            the first d_hi coordinates and over the others (split into two instances)}]
struct ScoreI8Args {
  const uint4* img;
  const float* scal;
  const float* PiT;  // fused variant only: transposed matrices and the raw queries
  const float* ST;
  const float* x;
  int64_t ldx;
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;
  float* scores;
  int64_t lds;
  int64_t n;
  int64_t total_rows;  // rows in the code arrays (all groups)
  int64_t group_stride;  // single-kernel d = 128 path: code rows between the first keys of consecutive groups (>= n)
  int d;
  int q_per_group;
  float kappa;
  float coef[16];  // coef[0]: factor of sum_j qr_j; coef[S]: factor of M_S (odd |S| only)
  // tq_score_i8.hip only: one launch covers k-steps [k0, k0 + ks_slice) of the d / 64; a launch with `accumulate`
  // adds its masked sums to the scores an earlier launch left (the terms that do not depend on the code are
  // added by the launch without it)
  int k0;
  int ks_slice;
  int accumulate;
};

constexpr int I8_MAX_KS = 8;     // k-steps of one launch: 512 coordinates (the A operands of a launch sit in registers)
constexpr int I8_MAX_D = 4096;   // longer vectors take several launches, each adding its 512 coordinates
// the terms the kernel evaluates: plane subsets of odd size (symmetric codebook)
__host__ __device__ constexpr bool i8_term(int m) { return __builtin_popcount((unsigned)m) & 1; }
// tiles of 16 keys per wavefront: as many as the register file holds code words for
__host__ __device__ constexpr int i8_tiles(int bits, int ksm) { return (bits >= 4 ? 16 : 32) / ksm; }
constexpr int I8_COPIES = 32;
constexpr int I8_TABLE_BYTES = 256 * I8_COPIES * 8;


hipError_t launch_score_i8_128(int bits, bool prod, const ScoreI8Args& a, int n_groups, hipStream_t stream);
bool score128_args(int bits, bool prod, const float* PiT, const float* ST, const float* q, int64_t ldq,
                   const uint32_t* idx, const uint32_t* qjl, const float* gamma, const float* norm, int64_t n,
                   int n_groups, int q_per_group, float kappa, const Codebook& cb, int64_t group_stride, ScoreI8Args* a);
bool i8_coefficients(int bits, const Codebook& cb, float* coef);  // factors of the masked sums (tq_score_i8.hip)
void i8_walsh(int bits, const Codebook& cb, double* w);  // Walsh coefficients of a centroid table (tq_score_i8.hip)
hipError_t launch_prep_i8_128(int d_hi, const float* Pi, const float* S, const float* q, int64_t ldq, int64_t nq,
                              bool prod, uint4* img, float* scal, hipStream_t stream);

}  // namespace tq

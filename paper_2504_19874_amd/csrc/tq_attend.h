// Shared by the attention read-out kernels (tq_attend.hip, tq_attend_128.hip).
#pragma once
#include "tq_internal.h"

namespace tq {

// Partial result of one (query, chunk of keys):  [0] m = largest logit of the chunk,
// [1] l = sum exp(logit - m), [4, 4 + d) sum exp(logit - m) nu c[idx] (rotated basis),
// [4 + d, 4 + 2 d) sum exp(logit - m) nu gamma z (sketch basis; zero for an MSE value cache).
__host__ __device__ constexpr int attend_part_stride(int d) { return 4 + 2 * d; }

struct AttendArgs {
  const float* scores;  // [n_groups * q_per_group][lds]: key scores, not yet multiplied by scale
  int64_t lds;
  const uint32_t* idx;  // value codes, n_groups * n rows
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;
  float* part;          // [n_groups * q_per_group][nchunks][attend_part_stride(d)]
  int nchunks;
  int64_t n;            // keys per group
  int64_t group_stride; // value code rows between the first tokens of consecutive groups (>= n)
  int d;
  int q_per_group;
  float scale;
  Codebook cb;          // of the value codes (two instances: of instance lo)
  int gs_hi;            // two instances: coordinate groups of instance hi (0: one instance); norm is [n][2] then
  Codebook cb_hi;
};

// d = 128 on the integer matrix cores (tq_attend_128.hip)
int attend128_chunks(int64_t n);
bool attend128_applicable(int d, bool prod, const Codebook& cb, const Codebook* cb_hi);
struct ScoreI8Args;
hipError_t launch_attend128(int kb, bool kprod, const ScoreI8Args* ka, bool vprod, const AttendArgs& a, int n_groups,
                            hipStream_t s);

int attend_simple_chunks(int64_t n);
hipError_t launch_attend_values(bool prod, const AttendArgs& a, int n_groups, hipStream_t s);
hipError_t launch_attend_combine(const float* part, int nchunks, int d, int64_t nq, const float* Pi, const float* S,
                                 float kappa, float* out, int64_t ldo, hipStream_t s);

}  // namespace tq

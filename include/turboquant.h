/*
 * turboquant.h - C ABI of the MI355X (gfx950) TurboQuant library.
 *
 * TurboQuant (arxiv 2504.19874) quantises d-dimensional vectors to b bits per
 * coordinate: rotate by a random orthogonal matrix, replace every rotated
 * coordinate by the index of the nearest centroid of a Lloyd-Max codebook,
 * and (inner-product variant) add a 1-bit sketch of the residual.
 *
 * Conventions for every call
 *  - "device" pointers are HIP device memory of the current device; "host"
 *    pointers are ordinary host memory.  All pointers are borrowed: the
 *    caller allocates, and keeps device buffers alive until the stream work
 *    has finished.  The library allocates nothing and never synchronises;
 *    device work is enqueued on `stream` (a hipStream_t passed as void*; NULL
 *    is the default stream).
 *  - Matrices are row-major fp32.  Vectors are rows.  d must be a multiple of
 *    32 (GPU entry points), bits_mse in [0, 4].  Row strides of vectors,
 *    queries and dequantised / attention output (ldx, ldq, ldo) are at most
 *    2^22 elements, else TQ_ERR_UNSUPPORTED; the row stride of a score matrix
 *    (lds) is not limited.
 *  - Every failure is a return code; nothing is launched when arguments are
 *    rejected.
 *
 * Packed code layout (the b*d-bit string of Sec. 1.1; the paper fixes only its
 * size): coordinates are taken in groups of 32 and stored as bit planes.
 *    idx word [i][g*bits_mse + p], bit l  =  bit p of idx_{32g+l} of vector i
 *    qjl word [i][g],              bit l  =  1 iff sign(S r)_{32g+l} = +1
 * so one vector owns bits_mse*d/32 idx words and d/32 qjl words, contiguous.
 * Per-vector scalars are separate fp32 arrays: gamma[i] = ||r||_2 (Alg. 2) and
 * norm[i] = ||x||_2 (Sec. 1.3, norms kept in floating point).
 *
 * Two instances over a split of the channels (Sec. 4.3: outlier channels get
 * more bits, which gives the non-integer bit-widths 2.5 and 3.5).  With
 * params.d_hi > 0 the first d_hi ROTATED coordinates belong to an instance
 * "hi" of dimension d_hi with bits_mse_hi bits and its own codebook, the
 * remaining d - d_hi to an instance "lo" with bits_mse bits.  The caller
 * makes Pi (and S) block diagonal up to the channel permutation that brings
 * the outlier channels to the front: Pi = blockdiag(Pi_hi, Pi_lo) * P, so x
 * stays in its original channel order and each block only ever sees its own
 * channels.  Each instance normalises, quantises and sketches its own part:
 *    idx words of vector i: group g < d_hi/32 has bits_mse_hi planes, the
 *        others bits_mse, groups stored back to back in order;
 *        words per vector = (d_hi/32)*bits_mse_hi + ((d-d_hi)/32)*bits_mse
 *    norm[2i], norm[2i+1]   = L2 norms of the hi and lo channels of x_i
 *    gamma[2i], gamma[2i+1] = residual norms of the two instances
 * and the sketch scale of Def. 1 is sqrt(pi/2)/d_hi resp. sqrt(pi/2)/(d-d_hi).
 * Covered for d = 128 with d_hi in {32, 64, 96}: tq_quantize_*, tq_dequantize,
 * tq_score (up to 4096 queries per group, through the kernel written for a few
 * queries per code), and tq_attend (keys: any width; values: MSE codes with
 * 1 + 2 or 2 + 3 index bits).
 *
 * Arithmetic.  Every contraction has fp32 operands and an fp32 (or int32)
 * accumulator; the bucket decision is an fp32 comparison.  Where it is faster
 * the fp32 factors are fed to the bf16 or int8 matrix cores as exact pieces
 * (bf16 pieces of 8 significant bits each, or base-128 digits of a fixed-point
 * value with 2^-19 relative spacing):
 *   quantise, bf16 batches above 8192 vectors at d = 128 and every d other
 *     than 128: the rotation from three pieces of Pi and the two leading
 *     pieces of an fp32 x (a bf16 x is one exact piece); what is dropped of x is
 *     below 2^-17 |x_k| per element, so a rotated coordinate moves by at most
 *     2^-17 |Pi_j| |x| = 7.6e-6 of the unit norm and the rotated vector by that in
 *     L2 norm: an index can differ from the fp32 evaluation only inside the
 *     1e-5 band around a cell boundary that every path is allowed.  The sketch,
 *     of which only signs are kept, from two pieces of the residual and two of
 *     S Pi^T (a sign can differ from the exact one only where
 *     |<S_j, r>| < 1e-6 |S_j| |r|).  tq_quantize_prod of fp32 vectors keeps the
 *     rotation on the fp32 instructions where the residual is so small that the
 *     part of x left out would show in gamma (4-bit MSE stage up to d = 416,
 *     3 bits up to d = 96, 2 bits at d = 32);
 *     Up to 64 vectors at d >= 512 with params.workspace large enough for
 *     their rotated coordinates (tq_workspace_bytes counts them) are rotated by
 *     plain fp32 multiply-adds, one matrix-vector product per vector, and so
 *     are a handful of long vectors in tq_dequantize;
 *   dequantise, large batches: two pieces of each factor (error
 *     below 4e-5 of a coordinate's typical size), at every d;
 *   scoring: two bf16 pieces of each factor (many queries; scores within
 *     3e-6 |q| norm of the exact ones) or int8 digits (few queries: up to 32
 *     per group at d <= 1024, up to 16 per group at d <= 4096 (64 in all
 *     beyond d = 512),
 *     d a multiple of 128, codebook symmetric about zero).
 * At d = 128, fp32 inputs and smaller batches run on the fp32 matrix
 * instructions.  All paths meet the same tolerances (indices equal to an fp32
 * evaluation except within 1e-5 of a cell boundary; values and scores within
 * 1e-4 relative).  With TQ_FLAG_FP32_MFMA in params.flags every contraction of
 * tq_quantize_*, tq_dequantize and many-query tq_score stays on the fp32 matrix
 * instructions.
 */
#ifndef TURBOQUANT_H
#define TURBOQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TQ_OK = 0,
  TQ_ERR_INVALID_ARG = 1, /* NULL where a pointer is required, bad size, bad enum */
  TQ_ERR_UNSUPPORTED = 2, /* valid request outside what the kernels cover        */
  TQ_ERR_HIP = 3,         /* a HIP runtime call or launch reported an error      */
  TQ_ERR_WORKSPACE = 4    /* params.workspace is NULL or too small for the call  */
} tq_status;

/* Element type of input vectors; passed as int32_t so that any value a caller
 * sends is rejected by a check instead of being undefined. */
typedef enum { TQ_F32 = 0, TQ_BF16 = 1 } tq_dtype;

/* Human-readable name of a status (static storage). */
const char* tq_status_string(tq_status s);

/*
 * Lloyd-Max codebook for one coordinate of a uniformly random unit vector in
 * R^d: the minimiser of the continuous 1-D k-means problem of eq. (4) for the
 * density f_X of Lemma 1, with 2^bits centroids.  Host only, fp64 inside.
 *   d >= 3, bits in [0, 8].
 *   centroids      host out, 2^bits floats, ascending, antisymmetric.
 *   bounds         host out, 2^bits - 1 floats: midpoints of consecutive
 *                  centroids (the Voronoi cell boundaries), computed in fp64
 *                  and rounded once.  May be NULL when bits == 0.
 *   cost_per_coord host out, nullable: C(f_X, bits); d times it is D_mse.
 */
tq_status tq_build_codebook(int32_t d, int32_t bits, float* centroids, float* bounds,
                            double* cost_per_coord);

/*
 * Probability of every codebook index (Sec. 3.1, entropy-coding paragraph):
 * p[l] = mass of the coordinate law f_X of Lemma 1 in the Voronoi cell of
 * centroid l.  Host only.  centroids: host, 2^bits ascending floats;
 * p: host out, 2^bits doubles summing to 1.
 */
tq_status tq_bucket_masses(int32_t d, int32_t bits, const float* centroids, double* p);

/*
 * Entropy coding of stored indices (Sec. 3.1, entropy-coding paragraph: an
 * optimal prefix code for {p_l} lowers the average bit-width towards the
 * entropy of the index distribution, by about 5 % at b = 4; the paper leaves it
 * out of the method, and so do the GPU kernels: this is an optional host-side
 * codec for codes at rest).  All pointers are host memory.
 *
 * tq_prefix_code_build: Huffman code lengths for probabilities p[0..K), K <=
 *   256, and the canonical codewords for them (symbols ordered by (length,
 *   symbol) take consecutive binary numbers).  lengths: out, K bytes;
 *   codewords: out, K words (right-aligned); mean_bits: out, nullable, sum p*len.
 *   TQ_ERR_UNSUPPORTED when a codeword would exceed 32 bits.
 * tq_entropy_encode: the codewords of coordinates 0..d-1 of each of n vectors,
 *   most significant bit first, vectors back to back, the last byte padded with
 *   zero bits.  idx: n * (bits*d/32) words in the packed layout above.
 *   out_capacity bytes are available at out (n*d*4 is always enough for codes
 *   made by tq_prefix_code_build with bits <= 4); TQ_ERR_WORKSPACE when they do
 *   not suffice.  out_bytes: out, bytes written.  row_bit_offsets: out,
 *   nullable, n + 1 values: the bit at which each vector starts, and the end.
 * tq_entropy_decode: n vectors starting at bit first_bit of the stream back
 *   into the packed layout.  TQ_ERR_INVALID_ARG when the stream ends early or
 *   holds a bit pattern that is no codeword.
 */
tq_status tq_prefix_code_build(int32_t K, const double* p, uint8_t* lengths, uint32_t* codewords,
                               double* mean_bits);
tq_status tq_entropy_encode(int32_t d, int32_t bits, const uint8_t* lengths, const uint32_t* codewords,
                            const uint32_t* idx, int64_t n, uint8_t* out, size_t out_capacity,
                            size_t* out_bytes, uint64_t* row_bit_offsets);
tq_status tq_entropy_decode(int32_t d, int32_t bits, const uint8_t* lengths, const uint8_t* in,
                            size_t in_bytes, uint64_t first_bit, int64_t n, uint32_t* idx);

/*
 * The random rotation of Sec. 3.1: the orthogonal factor Q of a QR
 * decomposition of a d x d matrix with i.i.d. N(0,1) entries, made unique (and
 * Haar distributed) by negating column j of Q where R[j][j] < 0, so that R has
 * a positive diagonal.  Host only: Householder reflections in fp64 on up to 16
 * threads, result rounded to fp32 once.
 *   gaussian  host, d*d doubles, row-major (the caller draws them).
 *   Pi        host out, d*d floats, row-major; y = Pi x rotates a vector.
 *   d in [1, 16384].
 */
tq_status tq_build_rotation(int32_t d, const double* gaussian, float* Pi);

/*
 * Parameter matrix of two instances over a channel split (Sec. 4.3: outlier
 * channels form an instance of their own): out = blockdiag(block_hi, block_lo)
 * * P, where P lists the d_hi channels in hi_channels first and the others
 * after them, both in ascending order.  Used for Pi (blocks = the two
 * rotations) and for S (blocks = the two sketch matrices); rotated coordinates
 * [0, d_hi) then belong to instance hi while x keeps its channel order.  Host
 * only, pure data movement.
 *   hi_channels host, d_hi ascending distinct channel numbers in [0, d).
 *   block_hi    host, d_hi*d_hi floats;  block_lo host, (d-d_hi)^2 floats.
 *   out         host out, d*d floats, row-major.
 */
tq_status tq_compose_split(int32_t d, int32_t d_hi, const int32_t* hi_channels, const float* block_hi,
                           const float* block_lo, float* out);

/*
 * Global parameters of Alg. 1 / Alg. 2 for one (d, bits_mse).
 * TurboQuant_prod with total bit-width b uses bits_mse = b - 1.
 */
typedef struct tq_params {
  int32_t d;
  int32_t bits_mse;
  const float* Pi;        /* device d*d: rotation, y = Pi x                         */
  const float* PiT;       /* device d*d: transpose of Pi   (tq_dequantize)          */
  const float* S;         /* device d*d: sketch matrix, N(0,1) entries; NULL = mse  */
  const float* ST;        /* device d*d: transpose of S    (tq_dequantize, prod)    */
  const float* SPiT;      /* device d*d: S * Pi^T          (tq_quantize_prod)       */
  const float* centroids; /* host, 2^bits_mse floats (tq_build_codebook)            */
  const float* bounds;    /* host, 2^bits_mse - 1 floats                            */
  void* workspace;        /* device scratch, see tq_workspace_bytes                 */
  size_t workspace_bytes;
  /* split into two instances (see the head of this file); all zero / NULL = one instance */
  int32_t d_hi;               /* 0, or a multiple of 32 below d                         */
  int32_t bits_mse_hi;        /* bits of the MSE stage of instance hi, in [0, 4]        */
  const float* centroids_hi;  /* host, 2^bits_mse_hi floats: codebook of dimension d_hi */
  const float* bounds_hi;     /* host, 2^bits_mse_hi - 1 floats; `centroids`/`bounds`   */
                              /* are then the codebook of dimension d - d_hi            */
  uint32_t flags;             /* TQ_FLAG_* bits, 0 = the library's own choice           */
  const void* images;         /* device, nullable: tq_images_bytes(d) bytes filled by
                                 tq_build_images from THESE matrices (see there)        */
} tq_params;

/* Keep every contraction of tq_quantize_*, tq_dequantize and many-query
 * tq_score on the fp32 matrix instructions (v_mfma_f32_32x32x2_f32) instead
 * of feeding them to the bf16 matrix cores as pieces (see "Arithmetic" at the
 * head of this file).  Same results within the stated tolerances, about half
 * the speed; meant for measurements against the fp32 peak and for callers who
 * want the plain fp32 evaluation. */
#define TQ_FLAG_FP32_MFMA 1u

/*
 * Fill the derived matrices from Pi and S on the device: PiT = Pi^T,
 * ST = S^T, SPiT = S Pi^T.  S, ST, SPiT may all be NULL (mse only).
 * S Pi^T lets the sketch of Alg. 2 (sign(S r), r = x - Pi^T y~) be taken in
 * the rotated basis, S r = (S Pi^T)(y - y~), an exact identity for orthogonal
 * Pi.
 */
tq_status tq_derive_params(int32_t d, const float* Pi, const float* S, float* PiT, float* ST,
                           float* SPiT, void* stream);

/* Optional, once per parameter set: the matrices already split into the bf16 pieces the quantisation and
 * dequantisation kernels multiply (see "Arithmetic" above), in the kernels' own order, so that no launch splits them
 * again (Alg. 1 / Alg. 2 fix the matrices "at setup"; this is that setup carried one step further).  d = 128: Pi,
 * S Pi^T, Pi^T and S^T as the large-batch kernels keep them in on-chip memory (their prologue becomes a copy);
 * every other d: Pi and S Pi^T as the tiles the quantiser's workgroups stage (10 d^2 bytes).
 * tq_images_bytes: size of the buffer for dimension d (0: none is taken at this d, tq_build_images then does
 * nothing).  tq_build_images reads p->Pi and, when p->S is set, p->SPiT (at d = 128 also p->PiT and p->ST), device
 * memory as tq_derive_params left it, and writes `images` (device, 16-byte aligned, owned by the caller) on
 * `stream`; the caller then stores the pointer in params.images.  A null params.images is always valid and gives
 * identical results.  The image must be rebuilt whenever one of the matrices changes: the kernels that take it do
 * not look at the fp32 matrices again.  Errors: TQ_ERR_INVALID_ARG (null pointers, S given without its derived
 * matrices), TQ_ERR_UNSUPPORTED (misaligned), TQ_ERR_HIP. */
size_t tq_images_bytes(int32_t d);
tq_status tq_build_images(const tq_params* p, void* images, void* stream);

/* Device scratch large enough for any call with up to n vectors (per call),
 * nq queries and this topk under these params: an upper bound that counts a
 * score matrix [nq][n] whenever topk > 0.  tq_score_workspace_bytes gives the
 * (often far smaller) exact need of one tq_score call. */
size_t tq_workspace_bytes(const tq_params* p, int64_t n, int64_t nq, int32_t topk);

/*
 * Quant_mse of Alg. 1 for n vectors.
 *   x     device, n rows of d values (dtype TQ_F32: fp32, TQ_BF16: bf16 bit
 *         patterns), row stride ldx elements.
 *   idx   device out, n * (bits_mse*d/32) words.
 *   norm  device out, n floats, or NULL.  Non-NULL: each row is divided by its
 *         L2 norm before rotation and the norm is stored (a zero row stays
 *         zero with norm 0).  NULL: rows are taken as unit-norm as given.
 * A coordinate exactly on a cell boundary goes to the upper cell.
 */
tq_status tq_quantize_mse(const tq_params* p, const void* x, int32_t dtype, int64_t n,
                          int64_t ldx, uint32_t* idx, float* norm, void* stream);

/*
 * Quant_prod of Alg. 2: idx from the MSE stage at bits_mse bits, then
 * qjl = sign(S r) and gamma = ||r||_2 for the residual r of the
 * (unit-normalised) vector.  sign(0) is +1.  Needs p->SPiT and, unless the
 * fused d = 128 kernel applies, workspace.
 *   qjl   device out, n * (d/32) words.   gamma device out, n floats.
 */
tq_status tq_quantize_prod(const tq_params* p, const void* x, int32_t dtype, int64_t n,
                           int64_t ldx, uint32_t* idx, uint32_t* qjl, float* gamma, float* norm,
                           void* stream);

/*
 * DeQuant_mse (Alg. 1) when qjl == NULL, DeQuant_prod (Alg. 2) otherwise:
 *   x_out[i] = norm[i] * ( Pi^T c[idx_i]  +  sqrt(pi/2)/d * gamma[i] * S^T z_i ).
 * norm may be NULL (= 1).  x_out: device, n rows of d floats, row stride ldo.
 */
tq_status tq_dequantize(const tq_params* p, const uint32_t* idx, const uint32_t* qjl,
                        const float* gamma, const float* norm, int64_t n, float* x_out,
                        int64_t ldo, void* stream);

/*
 * Inner-product estimates of Sec. 3.2 for every (query, code) pair inside a
 * group: query row g*q_per_group + j is scored against the n_per_group codes
 * of group g (code row g*n_per_group + i):
 *   s = norm * ( <Pi q, c[idx]>  +  sqrt(pi/2)/d * gamma * <S q, z> ),
 * the second term only when qjl != NULL.  Equal to <q, tq_dequantize(code)>.
 *   q        device, n_groups*q_per_group rows of d floats, row stride ldq.
 *   scores   device out [n_groups*q_per_group][lds], first n_per_group columns
 *            written; may be NULL when only top-k is wanted.
 *   topk     0, or 1..64: also return, per query, the indices (within the
 *            group, int32) and values of the topk largest scores, descending,
 *            equal scores ordered by lower index.  topk_idx/topk_val: device
 *            out [n_groups*q_per_group][topk]; topk_val nullable.  Where
 *            topk > n_per_group the surplus entries are index -1, value -inf.
 *            NaN scores are never returned.
 * Workspace (tq_score_workspace_bytes gives the exact need of a call): the
 * rotated queries or their int8 digit images, and for top-k without a score
 * buffer either nothing more than topk candidates per query and per range of
 * codes (many queries per code, topk <= 16: the selection runs inside the
 * scoring kernel and no score matrix exists anywhere) or a score matrix
 * [nq][n_per_group] (other cases).
 * n_groups <= 65535 and q_per_group <= 262140, else TQ_ERR_UNSUPPORTED.
 */
size_t tq_score_workspace_bytes(const tq_params* p, int32_t n_groups, int32_t q_per_group,
                                int64_t n_per_group, int32_t prod /* qjl will be given */,
                                int32_t scores_given /* scores != NULL */, int32_t topk);
tq_status tq_score(const tq_params* p, const float* q, int64_t ldq, int32_t n_groups,
                   int32_t q_per_group, const uint32_t* idx, const uint32_t* qjl,
                   const float* gamma, const float* norm, int64_t n_per_group, float* scores,
                   int64_t lds, int32_t topk, int32_t* topk_idx, float* topk_val, void* stream);

/*
 * tq_score for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and error codes as tq_score,
 * but p->workspace is ignored: the scratch memory (rotated queries or their
 * int8 digit images, and the score matrix when scores == NULL) is a static
 * device array inside the library, tq_score_static_scratch_bytes() bytes
 * (16 MiB) on every GPU the library has run on, held until the process ends.
 * The call allocates and frees nothing and calls no allocating routine.
 *   TQ_ERR_WORKSPACE  the call needs more than the array holds:
 *                     tq_score_workspace_bytes() of the same arguments must
 *                     not exceed tq_score_static_scratch_bytes().
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (two streams, two threads) race on it; serialise them.  Nothing in
 * the array has to survive between calls and nothing is read before the call
 * itself has written it.
 */
size_t tq_score_static_scratch_bytes(void);
tq_status tq_score_static(const tq_params* p, const float* q, int64_t ldq, int32_t n_groups,
                          int32_t q_per_group, const uint32_t* idx, const uint32_t* qjl,
                          const float* gamma, const float* norm, int64_t n_per_group, float* scores,
                          int64_t lds, int32_t topk, int32_t* topk_idx, float* topk_val,
                          void* stream);

/*
 * Attention read-out of a few queries over a quantised key/value cache
 * (Sec. 4.3: keys and values of past tokens are kept as codes; the paper gives
 * the value side nothing beyond DeQuant, so this is the usual read-out on the
 * dequantised cache).  For query row g*q_per_group + j and the n_per_group
 * cached tokens of group g:
 *   logit_i = scale * tq_score(pk; q, key code i)      (estimator of Sec. 3.2)
 *   out     = sum_i softmax(logit)_i * tq_dequantize(pv; value code i).
 * DeQuant is linear in the decoded code, so the sum is taken over the codes in
 * the rotated basis and rotated back once per query; no dequantised value is
 * ever written.
 *   pk, pv    parameters of the key and of the value codes (they may be the
 *             same object).  Key codes: anything tq_score accepts, including
 *             the two-instance split.  Value codes: one instance with
 *             bits_mse >= 0 (v_qjl/v_gamma NULL for an MSE value cache), or two
 *             instances of the MSE quantiser at d = 128 with 1 + 2 or 2 + 3 index
 *             bits (v_norm then holds two floats per token, as tq_quantize_mse
 *             writes them).
 *   k_*, v_*  device, codes of n_groups*n_per_group tokens, layouts as above.
 *   out       device out [n_groups*q_per_group][ldo], pv->d floats per row;
 *             zero rows when n_per_group == 0.
 * Uses pk->workspace only: tq_attend_workspace_bytes() bytes.  pk->d and pv->d
 * may differ (q has pk->d columns).
 */
size_t tq_attend_workspace_bytes(const tq_params* pk, const tq_params* pv, int32_t n_groups,
                                 int32_t q_per_group, int64_t n_per_group);
tq_status tq_attend(const tq_params* pk, const tq_params* pv, const float* q, int64_t ldq,
                    int32_t n_groups, int32_t q_per_group, const uint32_t* k_idx,
                    const uint32_t* k_qjl, const float* k_gamma, const float* k_norm,
                    const uint32_t* v_idx, const uint32_t* v_qjl, const float* v_gamma,
                    const float* v_norm, int64_t n_per_group, float scale, float* out, int64_t ldo,
                    void* stream);

/*
 * The same read-out over a cache that is still growing: every group owns
 * group_stride token slots (its capacity) of which the first n_per_group are
 * filled, so code row g*group_stride + i holds token i of group g.  With
 * group_stride == n_per_group this is tq_attend.  Otherwise TQ_ERR_UNSUPPORTED
 * unless pk->d == pv->d == 128, the key codes are of one instance with at most
 * 32 queries per group, pk->PiT (and pk->ST for prod keys) are set, the
 * codebooks are symmetric about zero (what tq_build_codebook produces), and the
 * value codes are among: MSE with 1..4 bits, prod with 0..2, or the two-instance
 * MSE codes above.  Workspace: tq_attend_workspace_bytes() as for tq_attend.
 */
tq_status tq_attend_cache(const tq_params* pk, const tq_params* pv, const float* q, int64_t ldq,
                          int32_t n_groups, int32_t q_per_group, const uint32_t* k_idx,
                          const uint32_t* k_qjl, const float* k_gamma, const float* k_norm,
                          const uint32_t* v_idx, const uint32_t* v_qjl, const float* v_gamma,
                          const float* v_norm, int64_t n_per_group, int64_t group_stride,
                          float scale, float* out, int64_t ldo, void* stream);

/*
 * Quantise n new vectors straight into such a cache (Sec. 4.3: tokens are
 * quantised as they are generated): tq_quantize_mse (qjl == NULL) or
 * tq_quantize_prod of row i of x, written to code row first_row + i*row_step of
 * idx / qjl / gamma / norm.  One new token for each of H heads of a cache laid
 * out [head][capacity] is n = H, first_row = tokens so far, row_step = capacity.
 * first_row >= 0, row_step >= 1; the caller guarantees the target rows exist.
 * d = 128 (one or two instances) and n <= 24576, else TQ_ERR_UNSUPPORTED; x
 * 16-byte aligned with row stride a multiple of 16 bytes.  No workspace.
 */
tq_status tq_append(const tq_params* p, const void* x, int32_t dtype, int64_t n, int64_t ldx,
                    uint32_t* idx, uint32_t* qjl, float* gamma, float* norm, int64_t first_row,
                    int64_t row_step, void* stream);

/*
 * Codec stages on their own (HBM-bound; they are also what the bit-exactness
 * tests drive): the decision idx_j = argmin_k |y_j - c_k| of Alg. 1 plus
 * packing for given rotated coordinates y[n][d]; the sign packing of Alg. 2
 * for given u = S r; and the table lookup y~_j = c[idx_j] of DeQuant_mse.
 */
tq_status tq_stage_pack(const tq_params* p, const float* y, int64_t n, uint32_t* idx, void* stream);
tq_status tq_stage_sign_pack(int32_t d, const float* u, int64_t n, uint32_t* qjl, void* stream);
tq_status tq_stage_unpack(const tq_params* p, const uint32_t* idx, int64_t n, float* y_tilde,
                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TURBOQUANT_H */

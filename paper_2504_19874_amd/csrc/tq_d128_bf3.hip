// DeQuant (Alg. 1 / Alg. 2) at d = 128 for large batches, on the bf16 matrix cores (bf16 pieces of the fp32
// factors, see tq_bf3.h; fp32 accumulation):
//     x~_i[k] = nu_i ( sum_j c[idx_ij] Pi[j][k]  +  kappa gamma_i sum_j z_ij S[j][k] ).
// The VECTOR is the row of the MFMA and the output coordinate the column, so
//   * the A operand (lane = vector, 8 consecutive j) is exactly what decoding 8 coordinates of one code
//     yields: a lane decodes its code's bit planes straight into the operand registers, no staging;
//   * the B operand is a piece of Pi^T / S^T (row k, 8 consecutive j), resident in LDS for the life of the
//     workgroup;
//   * D[vector][k]: output tile t holds the columns k = 4 l + t of lane l, so a lane owns 16 contiguous bytes
//     of its vector's row and a half-wave stores one whole row per instruction.
// Pieces: a centroid and an entry of Pi^T are taken as their two leading bf16 pieces and the three products
// of combined weight >= 2^-9 are summed (what is left out is 2^-17.8 of a term in the root mean square, 2^-15 at
// worst: about 5e-6 of a coordinate's typical size, against the 1e-4 the output has to meet).  The sign part is folded into the same
// accumulator: its operand is +-(kappa gamma_i), the two leading pieces of kappa gamma_i with the sign bit of
// z_ij, against two pieces of S^T, again three products.  A 1-bit table is +-c_1: the pieces of c_1 with a sign.
// Workgroup = 8 wavefronts, two per SIMD; a wavefront takes 32 vectors per block, workgroups stride over the
// blocks of 256 vectors.  (Four wavefronts of 64 vectors halve the LDS reads per MFMA but leave every SIMD idle
// while its one wavefront pushes out the block's stores: 13-20 % slower.)
#include "tq_bf3.h"

namespace tq {

namespace {

constexpr int MAT_ELEMS = 128 * 128;  // one piece of one matrix
constexpr int RING = 4;               // B operands in flight

// element offset of column j (a multiple of 4) of row k inside a piece: the 16-byte chunks of a row are
// rotated by k / 4, so the rows 4 l + t that the lanes l of one read touch fall into different banks
__device__ __forceinline__ int lds_at(int k, int j) { return k * 128 + ((((j >> 3) ^ (k >> 2)) & 15) << 3) + (j & 7); }

struct Dq128Args {
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;  // nullable
  const float* PiT;
  const float* ST;
  const u32x4* image;  // nullable: Pi^T and S^T as the kernel's LDS image, made ahead of time by dq128_image_kernel
  float* out;
  int64_t ldo;
  int64_t n;
  float kappa;
  Codebook cb;
  // two instances over a split of the rotated coordinates (MIXED, Sec. 4.3): coordinate groups [0, gs_hi) belong to
  // instance hi with BITS + 1 planes, codebook cb_hi and sketch scale kappa_hi; idx rows hold 4 BITS + gs_hi words,
  // gamma and norm two floats per vector (hi, lo)
  int gs_hi;
  float kappa_hi;
  Codebook cb_hi;
};

// One 128 x 128 fp32 matrix as its two leading pieces at dst ([piece][k][128], chunk rotation of lds_at), by 256
// threads.  dst is LDS in the dequantisation kernel and device memory in dq128_image_kernel.
__device__ __forceinline__ void dq128_split_matrix(const float* W, unsigned short* dst, int tid) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    f32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const f32x4*>(W + half * 8192 + (i * 256 + tid) * 4);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = half * 8192 + (i * 256 + tid) * 4;
      const int k = e >> 7, j = e & 127;
      uint32_t lo[2], hi[2];
      split2_pair(f32x2{v[i][0], v[i][1]}, lo[0], lo[1]);
      split2_pair(f32x2{v[i][2], v[i][3]}, hi[0], hi[1]);
#pragma unroll
      for (int pc = 0; pc < 2; ++pc)
        *reinterpret_cast<uint2*>(dst + pc * MAT_ELEMS + lds_at(k, j)) = make_uint2(lo[pc], hi[pc]);
    }
  }
}

// workgroup 0: Pi^T, workgroup 1: S^T, each 2 * MAT_ELEMS * 2 bytes of the image
__global__ __launch_bounds__(256) void dq128_image_kernel(const float* PiT, const float* ST, unsigned short* image) {
  const float* W = blockIdx.x == 0 ? PiT : ST;
  if (W != nullptr) dq128_split_matrix(W, image + blockIdx.x * 2 * MAT_ELEMS, threadIdx.x);
}

// VT = vector tiles (of 32) per wavefront.  VT = 2: four wavefronts of 64 vectors, each LDS read of a matrix
// operand feeds both tiles.  VT = 1: eight wavefronts of 32 vectors, two per SIMD, so that one can issue MFMAs
// while the other sits in the burst of stores that ends its block; every variant stays within the 256 registers
// that leaves a wavefront.  VT = 1 is what is launched.
template <int BITS, bool PROD, bool MIXED, int VT>
__global__ __launch_bounds__(512 / VT) void dequant128_bf3_kernel(const Dq128Args a) {
  constexpr int NT = 512 / VT;  // threads
  constexpr bool TABLE = BITS >= 2 || MIXED;  // centroid pieces looked up in LDS (1 bit: the pieces of c_1 with a sign)
  constexpr int NB = (BITS > 0 ? BITS : 1) + (MIXED ? 1 : 0);  // plane words per coordinate group, at most
  constexpr int MATS = (BITS > 0 || MIXED ? 1 : 0) + (PROD ? 1 : 0);
  constexpr bool PI = BITS > 0 || MIXED;  // there is a centroid part
  constexpr int READS = 4 * 2 * MATS;  // B operands per step: 4 tiles x 2 pieces x matrices
  extern __shared__ __attribute__((aligned(16))) unsigned short lds_s[];  // [matrix][piece][k][128], then the table
  uint32_t* const table_s = reinterpret_cast<uint32_t*>(lds_s + MATS * 2 * MAT_ELEMS);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- Pi^T (and S^T), two leading pieces each -----------------------------------------------------
  {
    int m = 0;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if (s == 0 ? !PI : !PROD) continue;
      if (a.image != nullptr) {
        // a straight copy of the matrix's 64 KB, 16 bytes per thread and step
        const u32x4* const src = a.image + s * (2 * MAT_ELEMS * 2 / 16);
        u32x4* const dst = reinterpret_cast<u32x4*>(lds_s + m * 2 * MAT_ELEMS);
        u32x4 v[4096 / NT];
#pragma unroll
        for (int i = 0; i < 4096 / NT; ++i) v[i] = src[i * NT + tid];
#pragma unroll
        for (int i = 0; i < 4096 / NT; ++i) dst[i * NT + tid] = v[i];
      } else {
        if (tid < 256) dq128_split_matrix(s == 0 ? a.PiT : a.ST, lds_s + m * 2 * MAT_ELEMS, tid);
      }
      ++m;
    }
    if (TABLE && tid < (MIXED ? 32 : 16)) {  // MIXED: entries 16.. are instance hi's
      uint32_t p1, p2, p3;
      split3(tid < 16 ? a.cb.c[tid] : a.cb_hi.c[tid - 16], p1, p2, p3);
      table_s[tid] = p1 | (p2 << 16);
    }
  }
  __syncthreads();

  const int vi = lane & 31, jg = lane >> 5;  // A: vector within the tile, which 8 of the 16 values of j
  uint32_t c1p[2] = {0u, 0u};  // 1 bit: the two pieces of c_1, each twice in a word
  if (BITS == 1) {
    uint32_t p1, p2, p3;
    split3(a.cb.c[1], p1, p2, p3);
    c1p[0] = p1 * 0x00010001u;
    c1p[1] = p2 * 0x00010001u;
  }
  const int64_t blocks = (a.n + 255) / 256;
  const int gs = MIXED ? a.gs_hi : 0;
  // MIXED: which of this lane's four output columns belong to instance hi.  The matrices are block diagonal up to a
  // permutation of the channels, so column k belongs to hi exactly when row k of the transposed matrix has an
  // entry among the first 32 gs_hi.
  uint32_t hi_cols = 0u;
  if (MIXED) {
    // thread t scans one half of the range for row t / 2; the flags go through LDS (behind the table)
    uint32_t* const flag_s = table_s + 32;
    if (tid < 256) {
      const float* row = (PROD ? a.ST : a.PiT) + (tid >> 1) * 128;
      bool any = false;
      for (int j = 16 * gs * (tid & 1); j < 16 * gs * ((tid & 1) + 1); j += 4) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(row + j);
        any = any || v[0] != 0.f || v[1] != 0.f || v[2] != 0.f || v[3] != 0.f;
      }
      flag_s[tid] = any ? 1u : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) hi_cols |= (flag_s[2 * (4 * vi + ct)] | flag_s[2 * (4 * vi + ct) + 1]) << ct;
  }

  // MIXED: nu / kg are instance lo's, nuh / kgh instance hi's
  uint32_t w[VT][4][NB], z[VT][4], wn[VT][4][NB], zn[VT][4];
  float nu[VT], kg[VT], nun[VT], kgn[VT], nuh[VT] = {}, kgh[VT] = {}, nuhn[VT] = {}, kghn[VT] = {};
  auto load_code = [&](int64_t blk) {  // into the "next" registers
#pragma unroll
    for (int mt = 0; mt < VT; ++mt) {
      const int64_t v = blk * 256 + wave * (32 * VT) + 32 * mt + vi;
      const int64_t row = v < a.n ? v : a.n - 1;  // clamped: such rows are not stored
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (MIXED) {  // group g: BITS (+ 1 below gs) planes, the groups back to back
          const uint32_t* src = a.idx + row * (4 * BITS + gs) + g * BITS + (g < gs ? g : gs);
#pragma unroll
          for (int pl = 0; pl < BITS + 1; ++pl) wn[mt][g][pl] = (pl < BITS || g < gs) ? src[pl < BITS || g < gs ? pl : 0] : 0u;
        } else {
#pragma unroll
          for (int pl = 0; pl < BITS; ++pl) wn[mt][g][pl] = a.idx[row * (4 * BITS) + g * BITS + pl];
        }
        zn[mt][g] = PROD ? a.qjl[row * 4 + g] : 0u;
      }
      if (MIXED) {
        nuhn[mt] = a.norm[2 * row];
        nun[mt] = a.norm[2 * row + 1];
        kghn[mt] = PROD ? a.kappa_hi * a.gamma[2 * row] : 0.f;
        kgn[mt] = PROD ? a.kappa * a.gamma[2 * row + 1] : 0.f;
      } else {
        nun[mt] = a.norm != nullptr ? a.norm[row] : 1.f;
        kgn[mt] = PROD ? a.kappa * a.gamma[row] : 0.f;
      }
    }
  };

  // B operand r of a step: tile r % 4 (columns k = 4 l + tile), then piece 1 before piece 0 of Pi^T, then of S^T
  auto b_piece = [&](int s, int r) {
    const int ct = r & 3, q = r >> 2;  // q: (matrix, piece) in the order (0, 1), (0, 0), (1, 1), (1, 0)
    const int m = q >> 1, pc = 1 - (q & 1);
    return *reinterpret_cast<const bf16x8*>(lds_s + (m * 2 + pc) * MAT_ELEMS + lds_at(4 * vi + ct, 16 * s + 8 * jg));
  };

  load_code(blockIdx.x);
  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
#pragma unroll
    for (int mt = 0; mt < VT; ++mt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int pl = 0; pl < (MIXED ? BITS + 1 : BITS); ++pl) w[mt][g][pl] = wn[mt][g][pl];
        z[mt][g] = zn[mt][g];
      }
      nu[mt] = nun[mt];
      kg[mt] = kgn[mt];
      nuh[mt] = nuhn[mt];
      kgh[mt] = kghn[mt];
    }
    load_code(blk + gridDim.x);  // the next block's codes travel during this block (clamped past the end)
    floatx16 acc[VT][4];  // [vector tile][column tile]
#pragma unroll
    for (int mt = 0; mt < VT; ++mt)
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][ct][r] = 0.f;
    uint32_t kgp[VT][2], kghp[VT][2];  // the two pieces of kappa gamma of this lane's vectors, each twice in a word
#pragma unroll
    for (int mt = 0; mt < VT; ++mt) {
      uint32_t p1, p2, p3;
      split3(kg[mt], p1, p2, p3);
      kgp[mt][0] = p1 * 0x00010001u;
      kgp[mt][1] = p2 * 0x00010001u;
      split3(kgh[mt], p1, p2, p3);
      kghp[mt][0] = p1 * 0x00010001u;
      kghp[mt][1] = p2 * 0x00010001u;
    }
    bf16x8 ring[RING];
#pragma unroll
    for (int r = 0; r < RING; ++r) ring[r] = b_piece(0, r);
    // table entries of the coordinates of one step, looked up one step ahead: they travel during the MFMAs
    uint32_t te[VT][8];
    auto look_up = [&](int s) {
      const int g = s >> 1, off = (s & 1) * 16 + 8 * jg;
#pragma unroll
      for (int mt = 0; mt < VT; ++mt) {
        uint32_t lv[2] = {0u, 0u};  // bucket numbers of 4 coordinates, one per byte
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int pl = 0; pl < (MIXED ? BITS + 1 : BITS); ++pl)  // a missing plane was loaded as zero
            lv[h] |= ((((w[mt][g][pl] >> (off + 4 * h)) & 0xFu) * 0x00204081u) & 0x01010101u) << pl;
        const uint32_t* const tab = table_s + (MIXED && g < gs ? 16 : 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) te[mt][u] = tab[(lv[u >> 2] >> (8 * (u & 3))) & 0xFFu];
      }
    };
    if (TABLE) look_up(0);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int g = s >> 1, off = (s & 1) * 16 + 8 * jg;  // word of the code, first bit
      // ---- A operands: this lane's 8 coordinates of two vectors decoded into pieces ----------------------
      bf16x8 ca[VT][2], za[VT][2];
#pragma unroll
      for (int mt = 0; mt < VT; ++mt) {
        if (BITS == 1 && !MIXED) {
          u32x4 v1, v2;
#pragma unroll
          for (int e = 0; e < 4; ++e) {  // bit 1 = +c_1: the sign bit is set where the code bit is 0
            const uint32_t sg = ((((w[mt][g][0] >> (off + 2 * e)) & 1u) << 15) | (((w[mt][g][0] >> (off + 2 * e + 1)) & 1u) << 31)) ^ 0x80008000u;
            v1[e] = c1p[0] ^ sg;
            v2[e] = c1p[1] ^ sg;
          }
          ca[mt][0] = *reinterpret_cast<const bf16x8*>(&v1);
          ca[mt][1] = *reinterpret_cast<const bf16x8*>(&v2);
        } else if (TABLE) {
          u32x4 v1, v2;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            v1[u] = __builtin_amdgcn_perm(te[mt][2 * u + 1], te[mt][2 * u], 0x05040100u);
            v2[u] = __builtin_amdgcn_perm(te[mt][2 * u + 1], te[mt][2 * u], 0x07060302u);
          }
          ca[mt][0] = *reinterpret_cast<const bf16x8*>(&v1);
          ca[mt][1] = *reinterpret_cast<const bf16x8*>(&v2);
        }
        if (PROD) {
          u32x4 v1, v2;
#pragma unroll
          for (int e = 0; e < 4; ++e) {  // bit 1 = +1
            const uint32_t sg = ((((z[mt][g] >> (off + 2 * e)) & 1u) << 15) | (((z[mt][g] >> (off + 2 * e + 1)) & 1u) << 31)) ^ 0x80008000u;
            v1[e] = (MIXED && g < gs ? kghp[mt][0] : kgp[mt][0]) ^ sg;
            v2[e] = (MIXED && g < gs ? kghp[mt][1] : kgp[mt][1]) ^ sg;
          }
          za[mt][0] = *reinterpret_cast<const bf16x8*>(&v1);
          za[mt][1] = *reinterpret_cast<const bf16x8*>(&v2);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (TABLE && s + 1 < 8) look_up(s + 1);
      __builtin_amdgcn_sched_barrier(0);
      // ---- B operands through the ring, MFMAs ----------------------------------------------------------
#pragma unroll
      for (int r = 0; r < READS; ++r) {
        const int ct = r & 3, q = r >> 2;
        const bool sign_part = !PI || q >= 2;  // which matrix this operand belongs to
        const int pc = 1 - (q & 1);
        const bf16x8 b = ring[(s * READS + r) % RING];
        // piece pc of the matrix meets the pieces a of the decoded operand with a + pc <= 1; the two MFMAs on
        // one accumulator are kept apart by the other vector tile's
        if (pc == 0) {
#pragma unroll
          for (int mt = 0; mt < VT; ++mt)
            acc[mt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sign_part ? za[mt][1] : ca[mt][1], b, acc[mt][ct], 0, 0, 0);
        }
#pragma unroll
        for (int mt = 0; mt < VT; ++mt)
          acc[mt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sign_part ? za[mt][0] : ca[mt][0], b, acc[mt][ct], 0, 0, 0);
        const int nxt = s * READS + r + RING;  // the read that takes this slot
        if (nxt < 8 * READS) ring[nxt % RING] = b_piece(nxt / READS, nxt % READS);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // ---- epilogue: D[vector][k]; the factors of a row's vector sit in the lane with that number --------
    // Addresses: a base that is uniform over the wavefront (scalar registers) plus a 32-bit byte offset per lane
    // that advances by a scalar from row to row: one vector add per store.  (Written as out + v * ldo per lane,
    // every one of the 32 stores carried its own 64-bit multiply.)
    const int64_t v0 = blk * 256 + wave * (32 * VT);
    const bool full = v0 + 32 * VT <= a.n;  // uniform: no vector of this wavefront is past the end
    char* const wbase = reinterpret_cast<char*>(a.out + v0 * a.ldo);
    const int rows_left = full ? 32 * VT : (int)(a.n - v0 > 0 ? a.n - v0 : 0);
    const uint32_t row_bytes = (uint32_t)a.ldo * 4u;
    const uint32_t lane_off = 4u * (uint32_t)(lane >> 5) * row_bytes + 16u * (uint32_t)vi;
#pragma unroll
    for (int mt = 0; mt < VT; ++mt) {
      // every row's norm first (one LDS round trip for all of them), then the arithmetic and the stores
      float rnu[16], rnuh[MIXED ? 16 : 1];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        rnu[r] = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (8 * (r >> 2) + (r & 3) + 4 * (lane >> 5)), __float_as_int(nu[mt])));
        if (MIXED)
          rnuh[r] = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (8 * (r >> 2) + (r & 3) + 4 * (lane >> 5)), __float_as_int(nuh[mt])));
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * mt + 8 * (r >> 2) + (r & 3);  // of lanes 0..31; lanes 32..63 hold row + 4
        f32x4 o;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) o[ct] = (MIXED && ((hi_cols >> ct) & 1u) ? rnuh[MIXED ? r : 0] : rnu[r]) * acc[mt][ct][r];
        if (full || row + 4 * (lane >> 5) < rows_left)
          __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(wbase + (lane_off + (uint32_t)row * row_bytes)));
      }
    }
  }
}

template <int BITS, bool PROD, bool MIXED, int VT>
hipError_t launch_vt(const Dq128Args& a, hipStream_t s) {
  constexpr int MATS = (BITS > 0 || MIXED ? 1 : 0) + (PROD ? 1 : 0);
  constexpr int lds = MATS * 2 * MAT_ELEMS * 2 + (32 + 256) * 4;  // matrices, centroid tables, column flags
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&dequant128_bf3_kernel<BITS, PROD, MIXED, VT>), lds); e != hipSuccess) return e;
  const int64_t blocks = (a.n + 255) / 256, cus = device_cu_count();  // one workgroup per compute unit
  hipLaunchKernelGGL((dequant128_bf3_kernel<BITS, PROD, MIXED, VT>), dim3((unsigned)(blocks < cus ? blocks : cus)), dim3(512 / VT), lds, s, a);
  return hipGetLastError();
}

// eight wavefronts of 32 vectors: measured against four of 64 (VT = 2) on the same box, 524288 vectors: 110 against
// 127 us (two-instance codes and 4-bit codes alike), 131072 vectors: 30 against 38 us
template <int BITS, bool PROD, bool MIXED>
hipError_t launch_one(const Dq128Args& a, hipStream_t s) {
  return launch_vt<BITS, PROD, MIXED, 1>(a, s);
}

}  // namespace

// d = 128; a 1-bit table of one instance must be +-c; rows of the output 16-byte aligned
bool dequant128_bf3_applicable(int bits, bool prod, const Codebook& cb, const float* out, int64_t ldo) {
  if (bits < 0 || bits > 4 || (bits == 0 && !prod)) return false;
  if ((reinterpret_cast<uintptr_t>(out) & 15u) != 0 || ldo % 4 != 0) return false;
  if (ldo < 128 || ldo > (1 << 22)) return false;  // 64 rows of a wavefront are addressed with 32-bit byte offsets
  return bits != 1 || cb.c[0] == -cb.c[1];
}

// gs_hi > 0: two instances (cb_hi with bits + 1 bits and kappa_hi for the first gs_hi coordinate groups; norm and
// gamma hold two floats per vector)
hipError_t launch_dequant128_bf3(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                                 const float* norm, const float* PiT, const float* ST, float* out, int64_t ldo, int64_t n,
                                 float kappa, const Codebook& cb, int gs_hi, float kappa_hi, const Codebook& cb_hi,
                                 const void* image, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (gs_hi < 0 || gs_hi > 3 || (gs_hi > 0 && (bits > 3 || cb_hi.bits != bits + 1 || norm == nullptr))) return hipErrorInvalidValue;
  Dq128Args a;
  a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm; a.PiT = PiT; a.ST = ST; a.out = out; a.ldo = ldo; a.n = n;
  a.image = static_cast<const u32x4*>(image);

  a.kappa = kappa; a.cb = cb; a.gs_hi = gs_hi; a.kappa_hi = kappa_hi; a.cb_hi = cb_hi;
  if (gs_hi > 0) {
    switch (bits * 2 + (prod ? 1 : 0)) {
      case 0: return launch_one<0, false, true>(a, s);
      case 1: return launch_one<0, true, true>(a, s);
      case 2: return launch_one<1, false, true>(a, s);
      case 3: return launch_one<1, true, true>(a, s);
      case 4: return launch_one<2, false, true>(a, s);
      case 5: return launch_one<2, true, true>(a, s);
      case 6: return launch_one<3, false, true>(a, s);
      case 7: return launch_one<3, true, true>(a, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (bits * 2 + (prod ? 1 : 0)) {
    case 1: return launch_one<0, true, false>(a, s);
    case 2: return launch_one<1, false, false>(a, s);
    case 3: return launch_one<1, true, false>(a, s);
    case 4: return launch_one<2, false, false>(a, s);
    case 5: return launch_one<2, true, false>(a, s);
    case 6: return launch_one<3, false, false>(a, s);
    case 7: return launch_one<3, true, false>(a, s);
    case 8: return launch_one<4, false, false>(a, s);
    case 9: return launch_one<4, true, false>(a, s);
    default: return hipErrorInvalidValue;
  }
}

size_t dequant128_bf3_image_bytes() { return (size_t)4 * MAT_ELEMS * 2; }

// ST may be null (no sketch): the second half of the image is left alone then
hipError_t launch_dequant128_bf3_image(const float* PiT, const float* ST, void* image, hipStream_t s) {
  hipLaunchKernelGGL(dq128_image_kernel, dim3(2), dim3(256), 0, s, PiT, ST, static_cast<unsigned short*>(image));
  return hipGetLastError();
}

}  // namespace tq

// HIP kernels (gfx950) and device entry points of the LUT mpGEMM library.
//
//   precompute_kernel  Algorithm 1 "Precompute": one 16-entry table per 4 activations, plus
//                      the per-quantisation-group activation sums needed by the bias term of
//                      Section 4 ("Bit-serial linear transformation").
//   mpgemm_lds_kernel  Algorithm 1 main loop: the tables of a K-slice live in LDS (Section 3.2
//                      "Put lookup table on on-chip memory"); every lane streams its packed
//                      4-bit indices from HBM with wide coalesced loads, looks each one up,
//                      accumulates the bit planes with weight 2^i (Eq. 1), applies scale and
//                      zero once per quantisation group and reduces over the K-slices.
//
// Lane mapping of the lookup kernel: a wavefront owns one tile of 16 rows; lane = 16*phi + r
// handles row r and the LUT groups kg = 4j + phi of every 128-wide chunk.  The four tables a
// wavefront touches in one step are 4 x 32 contiguous bytes, i.e. all 32 LDS banks exactly once,
// and lanes reading the same entry are served by broadcast, so the lookups are conflict-free.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <tuple>
#include <utility>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

template <typename Tuple, size_t... I>
static void fill_ptrs(Tuple& t, void** ptrs, std::index_sequence<I...>) {
  ((ptrs[I] = static_cast<void*>(&std::get<I>(t))), ...);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) int16_t lds_i16;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef __attribute__((address_space(3))) __half lds_f16;

// ------------------------------------------------------------------------------------------
// LUT buffer geometry
// ------------------------------------------------------------------------------------------
// (LutGeom / lut_geom live in tmac_internal.h)

// ------------------------------------------------------------------------------------------
// Table precompute
// ------------------------------------------------------------------------------------------
// One wavefront per (n, quantisation group): the group sum S[n][gq] = sum of its activations,
// four elements per lane and step (the row base, lda and the group size are multiples of 4),
// then a butterfly.
template <bool IS_INT>
__device__ __forceinline__ void group_sums_wave(const void* __restrict__ A_, int N, int64_t lda,
                                                void* __restrict__ S_, int Geff, int nq, int wave) {
  const int lane = threadIdx.x & 63;
  if (wave >= N * nq) return;
  const int n = wave / nq, gq = wave % nq;
  const int64_t base = n * lda + (int64_t)gq * Geff;
  if constexpr (IS_INT) {
    const uint32_t* a = reinterpret_cast<const uint32_t*>(static_cast<const int8_t*>(A_) + base);
    int s = 0;
    for (int k4 = lane; 4 * k4 < Geff; k4 += 64) s = __builtin_amdgcn_sdot4((int)a[k4], 0x01010101, s, false);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) static_cast<int*>(S_)[wave] = s;
  } else {
    const uint2* a = reinterpret_cast<const uint2*>(static_cast<const __half*>(A_) + base);
    float s = 0.f;
    for (int k4 = lane; 4 * k4 < Geff; k4 += 64) {
      const uint2 v = a[k4];
      const float a0 = __half2float(__ushort_as_half((uint16_t)(v.x & 0xffffu)));
      const float a1 = __half2float(__ushort_as_half((uint16_t)(v.x >> 16)));
      const float a2 = __half2float(__ushort_as_half((uint16_t)(v.y & 0xffffu)));
      const float a3 = __half2float(__ushort_as_half((uint16_t)(v.y >> 16)));
      s += (a0 + a1) + (a2 + a3);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) static_cast<float*>(S_)[wave] = s;
  }
}

template <bool IS_INT>
__global__ __launch_bounds__(256) void precompute_kernel(const void* __restrict__ A_, int N, int K,
                                                         int64_t lda, int KG,
                                                         uint4* __restrict__ tables,
                                                         void* __restrict__ S_, void* __restrict__ S16_,
                                                         void* __restrict__ S128_,
                                                         uint4* __restrict__ HT, int U, int Geff, int nq,
                                                         int n_tab_blocks) {
  if ((int)blockIdx.x < n_tab_blocks) {
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tid >= (int64_t)N * KG) return;
    const int n = (int)(tid / KG), kg = (int)(tid % KG);
    uint32_t packed[8];
    float sum4f = 0.f;  // sum of this table's four activations (for the per-16 unit sums)
    int sum4i = 0;
    if (4 * kg >= K) {
#pragma unroll
      for (int i = 0; i < 8; ++i) packed[i] = 0;  // k padding: all-zero table
    } else if constexpr (IS_INT) {
      const int8_t* a = static_cast<const int8_t*>(A_) + n * lda + 4 * kg;
      const int a0 = a[0], a1 = a[1], a2 = a[2], a3 = a[3];
      sum4i = a0 + a1 + a2 + a3;
      int e[16];
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        e[p] = ((p & 1) ? a0 : -a0) + ((p & 2) ? a1 : -a1) + ((p & 4) ? a2 : -a2) - a3;
      }
#pragma unroll
      for (int p = 0; p < 8; ++p) e[15 - p] = -e[p];  // mirror half
#pragma unroll
      for (int i = 0; i < 8; ++i)
        packed[i] = ((uint32_t)e[2 * i] & 0xffffu) | ((uint32_t)e[2 * i + 1] << 16);
    } else {
      const __half* a = static_cast<const __half*>(A_) + n * lda + 4 * kg;
      const float a0 = __half2float(a[0]), a1 = __half2float(a[1]);
      const float a2 = __half2float(a[2]), a3 = __half2float(a[3]);
      sum4f = ((a0 + a1) + a2) + a3;
      uint16_t e[16];
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const float v = (((p & 1) ? a0 : -a0) + ((p & 2) ? a1 : -a1)) + (((p & 4) ? a2 : -a2) - a3);
        const __half h = __float2half_rn(v);
        e[p] = __half_as_ushort(h);
        e[15 - p] = e[p] ^ 0x8000u;  // mirror half: exact negation
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) packed[i] = (uint32_t)e[2 * i] | ((uint32_t)e[2 * i + 1] << 16);
    }
    uint4* dst = tables + tid * 2;
    dst[0] = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    dst[1] = make_uint4(packed[4], packed[5], packed[6], packed[7]);
    // Mirror-consolidated copy for the register-table kernel: entries 0..7 as fp16 (int16 entries
    // are at most 508 in magnitude, exact in fp16).  Units are grouped in nB blocks; inside a block
    // of nu units, table tb of the unit in slot s sits at 16-byte slot tb*nu + s, so that the
    // lanes loading "their" table tb read one contiguous run.
    {
      uint4 half;
      if constexpr (IS_INT) {
        uint32_t h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int lo = (int)(short)(packed[i] & 0xffffu), hi = (int)(short)(packed[i] >> 16);
          h[i] = (uint32_t)__half_as_ushort(__int2half_rn(lo)) | ((uint32_t)__half_as_ushort(__int2half_rn(hi)) << 16);
        }
        half = make_uint4(h[0], h[1], h[2], h[3]);
      } else {
        half = make_uint4(packed[0], packed[1], packed[2], packed[3]);
      }
      // split into the two 8-byte byte-permute sources (Section 4: an fp16 table as two 8-bit
      // tables): low bytes of entries 0..3, 4..7, then high bytes of entries 0..3, 4..7
      const uint4 split = make_uint4(__builtin_amdgcn_perm(half.y, half.x, 0x06040200u),
                                     __builtin_amdgcn_perm(half.w, half.z, 0x06040200u),
                                     __builtin_amdgcn_perm(half.y, half.x, 0x07050301u),
                                     __builtin_amdgcn_perm(half.w, half.z, 0x07050301u));
      const int u = kg >> 2, tb = kg & 3;
      const BlockSplit bs = block_split(U);
      const int blk = block_of(bs, u >> 3);
      const int c0 = block_start(bs, blk), ng = block_start(bs, blk + 1) - c0;
      HT[((size_t)n * U + 8 * c0) * 4 + (size_t)tb * (8 * ng) + block_slot(u, c0, ng)] = split;
      if (tid == 0) HT[(size_t)N * U * 4] = make_uint4(0, 0, 0, 0);  // the all-zero slot
    }
    // unit sums S16[n][kg / 4] and chunk sums S128[n][kg / 32]: the tables of a unit sit in four
    // adjacent lanes, those of a 128-k chunk in 32 adjacent lanes (KG is a multiple of 32 and the
    // workgroup size a multiple of 64, so a chunk never straddles a wavefront); fixed tree order
    if constexpr (IS_INT) {
      sum4i += __shfl_xor(sum4i, 1);
      sum4i += __shfl_xor(sum4i, 2);
      if ((kg & 3) == 0) static_cast<int*>(S16_)[tid >> 2] = sum4i;
      sum4i += __shfl_xor(sum4i, 4);
      sum4i += __shfl_xor(sum4i, 8);
      sum4i += __shfl_xor(sum4i, 16);
      if ((kg & 31) == 0) static_cast<int*>(S128_)[tid >> 5] = sum4i;
    } else {
      sum4f += __shfl_xor(sum4f, 1);
      sum4f += __shfl_xor(sum4f, 2);
      if ((kg & 3) == 0) static_cast<float*>(S16_)[tid >> 2] = sum4f;
      sum4f += __shfl_xor(sum4f, 4);
      sum4f += __shfl_xor(sum4f, 8);
      sum4f += __shfl_xor(sum4f, 16);
      if ((kg & 31) == 0) static_cast<float*>(S128_)[tid >> 5] = sum4f;
    }
  } else {
    group_sums_wave<IS_INT>(A_, N, lda, S_, Geff, nq, ((int)blockIdx.x - n_tab_blocks) * 4 + (threadIdx.x >> 6));
  }
}

// Table quantisation (Section 3.3): one thread per unit of 16 activations builds the mirror halves
// of its four tables in fp32 (same sums as above), takes the unit's largest magnitude
// amax = max_t sum_j |a_j| (attained by the entry whose signs match), and stores
// rint(T * 127 / amax) as int8 together with the scale amax / 127.  Per unit: two 16-byte pieces
// (tables 0,1 and 2,3; eight entries of one byte each), laid out like the fp16 half tables.
__global__ __launch_bounds__(256) void precompute_q8_kernel(const __half* __restrict__ A, int N, int K, int64_t lda,
                                                            int U, float* __restrict__ S, float* __restrict__ S16,
                                                            float* __restrict__ S128, float* __restrict__ usc,
                                                            uint4* __restrict__ HTQ, int Geff, int nq,
                                                            int n_unit_blocks) {
  if ((int)blockIdx.x >= n_unit_blocks) {
    group_sums_wave<false>(A, N, lda, S, Geff, nq, ((int)blockIdx.x - n_unit_blocks) * 4 + (threadIdx.x >> 6));
    return;
  }
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (tid >= (int64_t)N * U) return;  // N*U is a multiple of 8: chunks never straddle the cut
  const int n = (int)(tid / U), u = (int)(tid % U);
  float a[16];
  if (16 * u < K) {  // K is a multiple of 4: a unit may end early
    const __half* ap = A + n * lda + 16 * u;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (16 * u + 4 * t < K) {
        const uint2 v = *reinterpret_cast<const uint2*>(ap + 4 * t);
        a[4 * t + 0] = __half2float(__ushort_as_half((uint16_t)(v.x & 0xffffu)));
        a[4 * t + 1] = __half2float(__ushort_as_half((uint16_t)(v.x >> 16)));
        a[4 * t + 2] = __half2float(__ushort_as_half((uint16_t)(v.y & 0xffffu)));
        a[4 * t + 3] = __half2float(__ushort_as_half((uint16_t)(v.y >> 16)));
      } else {
        a[4 * t] = a[4 * t + 1] = a[4 * t + 2] = a[4 * t + 3] = 0.f;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = 0.f;
  }
  float e[4][8], t4[4], amax = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const float x0 = a[4 * t], x1 = a[4 * t + 1], x2 = a[4 * t + 2], x3 = a[4 * t + 3];
    const float sp = x0 + x1, dp = x0 - x1, tq = x2 + x3, wq = x2 - x3;
    e[t][0] = -sp - tq; e[t][1] = dp - tq; e[t][2] = -dp - tq; e[t][3] = sp - tq;
    e[t][4] = wq - sp;  e[t][5] = dp + wq; e[t][6] = wq - dp;  e[t][7] = sp + wq;
    t4[t] = ((x0 + x1) + x2) + x3;
    amax = fmaxf(amax, (fabsf(x0) + fabsf(x1)) + (fabsf(x2) + fabsf(x3)));
  }
  const float inv = amax > 0.f ? 127.0f / amax : 0.f;
  uint32_t w[8];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t word = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int v = (int)rintf(e[t][4 * h + q] * inv);
        v = v > 127 ? 127 : (v < -127 ? -127 : v);
        word |= ((uint32_t)v & 0xffu) << (8 * q);
      }
      w[2 * t + h] = word;
    }
  }
  const BlockSplit bs = block_split(U);
  const int blk = block_of(bs, u >> 3);
  const int c0 = block_start(bs, blk), ng = block_start(bs, blk + 1) - c0;
  uint4* dst = HTQ + ((size_t)n * U + 8 * c0) * 2 + block_slot(u, c0, ng);
  dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
  dst[8 * ng] = make_uint4(w[4], w[5], w[6], w[7]);
  if (tid == 0) HTQ[(size_t)N * U * 2] = make_uint4(0, 0, 0, 0);  // the all-zero slot
  usc[tid] = amax / 127.0f;
  float s16 = (t4[0] + t4[1]) + (t4[2] + t4[3]);
  S16[tid] = s16;
  s16 += __shfl_xor(s16, 1);  // the eight units of a 128-k chunk sit in eight adjacent lanes
  s16 += __shfl_xor(s16, 2);
  s16 += __shfl_xor(s16, 4);
  if ((u & 7) == 0) S128[tid >> 3] = s16;
}

// ------------------------------------------------------------------------------------------
// Lookup + accumulate
// ------------------------------------------------------------------------------------------
struct MpParams {
  const uint32_t* idx;
  const uint32_t* sz;      // {fp16 scale, fp16 zero} per (tile, group, row)
  const uint16_t* tables;  // [N][KG][16]
  const void* S;           // [N][nq] fp32 or int32
  float* ws_part;          // [nslices][N][Mp] partial sums (fp32, or int32 bit patterns)
  int* ws_ctr;             // arrival counters, one per (row block, n tile)
  void* out;
  const float* act_scale;
  int64_t ldo;
  int M, Mp, N, KG, n_tiles, n_chunks, nq;
  int gmode;       // 0: one group per row or tensor (partials are unscaled), 1: group scales
  int gpc_shift;   // gmode 1: log2(groups per 128-chunk) = 0, 1, 2
  int G;           // gmode 1: elements per quantisation group
  int per_tensor;  // gmode 0: scale/zero from wscale/zero_point instead of the blob
  int int_exact;   // integer path with an integer zero point: exact (L + icoef*S)/2
  int icoef;       // 2^b - 1 - 2z
  float wscale, zero_point, mid;
  int out_t;
  int cpg;         // gmode 1 with whole-chunk groups: 128-chunks per quantisation group
};

template <bool IS_INT, int NT>
__device__ __forceinline__ void finalize_store(const MpParams& p, int n, int m, float vf, int vi) {
  // vf: fp accumulator (grouped: finished sum; single group fp: raw L); vi: raw integer L
  float res;
  int ires = 0;
  const float as = p.act_scale ? p.act_scale[n] : 1.0f;
  if (p.gmode == 1) {
    res = vf * as;
  } else {
    float s, z;
    if (p.per_tensor) {
      s = p.wscale;
      z = p.zero_point;
    } else {
      const uint32_t szv = p.sz[(size_t)(m >> 4) * 16 + (m & 15)];
      s = __half2float(__ushort_as_half((uint16_t)(szv & 0xffff)));
      z = __half2float(__ushort_as_half((uint16_t)(szv >> 16)));
    }
    if constexpr (IS_INT) {
      const int St = static_cast<const int*>(p.S)[n];
      if (p.int_exact) {
        ires = (vi + p.icoef * St) >> 1;  // numerator is always even
        res = ((float)ires * as) * s;     // two roundings, left to right
      } else {
        res = ((0.5f * (float)vi + (p.mid - z) * (float)St) * as) * s;
      }
    } else {
      const float St = static_cast<const float*>(p.S)[n];
      res = (s * (0.5f * vf + (p.mid - z) * St)) * as;
    }
  }
  const size_t o = (size_t)n * p.ldo + m;
  if (p.out_t == TMAC_OUT_F32) static_cast<float*>(p.out)[o] = res;
  else if (p.out_t == TMAC_OUT_F16) static_cast<__half*>(p.out)[o] = __float2half_rn(res);
  else static_cast<int*>(p.out)[o] = ires;
}

template <bool IS_INT, int BITS, int NT, int KS>
__global__ __launch_bounds__(512) void mpgemm_lds_kernel(const MpParams p) {
  using AccT = typename std::conditional<IS_INT, int, float>::type;
  __shared__ __attribute__((aligned(16))) uint16_t tab[KS * 32 * 16 * NT];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int phi = lane >> 4, r = lane & 15;
  const int tile = blockIdx.x * 8 + wave;
  const int c0 = blockIdx.y * KS;
  const int n0 = blockIdx.z * NT;
  const bool tile_ok = tile < p.n_tiles;

  // 1. issue the weight-index loads first: they do not depend on the tables
  uint32_t w[KS][BITS];
#pragma unroll
  for (int i = 0; i < KS; ++i) {
    const int c = c0 + i;
    if (tile_ok && c < p.n_chunks) {
      const uint32_t* src = p.idx + (((size_t)tile * p.n_chunks + c) * 64 + lane) * BITS;
      if constexpr (BITS == 4) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
        w[i][0] = v.x; w[i][1] = v.y; w[i][2] = v.z; w[i][3] = v.w;
      } else if constexpr (BITS == 2) {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
        w[i][0] = v.x; w[i][1] = v.y;
      } else {
#pragma unroll
        for (int b = 0; b < BITS; ++b) w[i][b] = __builtin_nontemporal_load(src + b);
      }
    } else {
#pragma unroll
      for (int b = 0; b < BITS; ++b) w[i][b] = 0;
    }
  }

  // 2. stage the tables of this K-slice (and NT activation rows) into LDS
  {
    constexpr int ITEMS = NT * KS * 64;  // 16-byte pieces: (n, table, half)
    for (int it = threadIdx.x; it < ITEMS; it += 512) {
      const int nl = it / (KS * 64), rem = it % (KS * 64);
      const int kl = rem >> 1, h = rem & 1;
      const int n = n0 + nl, kg = c0 * 32 + kl;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (n < p.N && kg < p.KG)
        v = *reinterpret_cast<const uint4*>(p.tables + ((size_t)n * p.KG + kg) * 16 + 8 * h);
      if constexpr (NT == 1) {
        *reinterpret_cast<uint4*>(&tab[kl * 16 + 8 * h]) = v;
      } else {
        const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint16_t x = (uint16_t)(vv[e >> 1] >> (16 * (e & 1)));
          tab[(kl * 16 + 8 * h + e) * NT + nl] = x;
        }
      }
    }
  }
  __syncthreads();

  // 3. look up, accumulate bit planes, apply scale and zero per quantisation group
  float acc[NT];
  AccT Lone[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) { acc[t] = 0.f; Lone[t] = 0; }
  const uint32_t phi_rep = (uint32_t)phi * 0x20202020u;
  const char* tab_bytes = reinterpret_cast<const char*>(tab);

#pragma unroll
  for (int i = 0; i < KS; ++i) {
    const int c = c0 + i;
    if (c >= p.n_chunks) break;
    AccT L[4][NT];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t) L[u][t] = 0;
#pragma unroll
    for (int b = 0; b < BITS; ++b) {
      const uint32_t x = w[i][b];
      // byte jj of zz[h] = 32*phi + 2*index: byte offset of the entry inside the 128-byte
      // run of four tables (weight interleaving makes both words come out in order)
      const uint32_t zz[2] = {((x << 1) & 0x1E1E1E1Eu) | phi_rep, ((x >> 3) & 0x1E1E1E1Eu) | phi_rep};
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int j = 4 * h + jj;
          const int u = j >> 1;
          const uint32_t v = (zz[h] >> (8 * jj)) & 0xffu;
          const char* ent = tab_bytes + (size_t)((i * 32 + 4 * j) * 32 * NT) + v * NT;
          if constexpr (NT == 1) {
            if constexpr (IS_INT) {
              const int e = *reinterpret_cast<const int16_t*>(ent);
              L[u][0] += e << b;
            } else {
              const __half e = *reinterpret_cast<const __half*>(ent);
              L[u][0] = fmaf(__half2float(e), (float)(1 << b), L[u][0]);
            }
          } else {
            static_assert(NT == 1 || NT == 4, "NT");
            const uint2 ev = *reinterpret_cast<const uint2*>(ent);
            const uint32_t evv[2] = {ev.x, ev.y};
#pragma unroll
            for (int t = 0; t < NT; ++t) {
              const uint16_t raw = (uint16_t)(evv[t >> 1] >> (16 * (t & 1)));
              if constexpr (IS_INT) L[u][t] += ((int)(int16_t)raw) << b;
              else L[u][t] = fmaf(__half2float(__ushort_as_half(raw)), (float)(1 << b), L[u][t]);
            }
          }
        }
      }
    }
    if (p.gmode == 0) {
#pragma unroll
      for (int t = 0; t < NT; ++t) Lone[t] += (L[0][t] + L[1][t]) + (L[2][t] + L[3][t]);
    } else {
      const int gpc = 1 << p.gpc_shift;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (u >= gpc) break;
        const int gq = (gpc == 1) ? (c * 128) / p.G : c * gpc + u;
        if (gq >= p.nq || !tile_ok) continue;
        const uint32_t szv = p.sz[((size_t)tile * p.nq + gq) * 16 + r];
        const float s = __half2float(__ushort_as_half((uint16_t)(szv & 0xffff)));
        const float z = __half2float(__ushort_as_half((uint16_t)(szv >> 16)));
        // bias term once per (row, quantisation group): first chunk of the group, lane phi 0
        const bool first_chunk = (gpc != 1) || ((c * 128) % p.G == 0);
        const float bz = (phi == 0 && first_chunk) ? (p.mid - z) : 0.f;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          AccT Lg;
          if (gpc == 1) Lg = (L[0][t] + L[1][t]) + (L[2][t] + L[3][t]);
          else if (gpc == 2) Lg = L[2 * u][t] + L[2 * u + 1][t];
          else Lg = L[u][t];
          const int n = n0 + t;
          float Sv = 0.f;
          if (n < p.N) {
            if constexpr (IS_INT) Sv = (float)static_cast<const int*>(p.S)[(size_t)n * p.nq + gq];
            else Sv = static_cast<const float*>(p.S)[(size_t)n * p.nq + gq];
          }
          acc[t] += s * (0.5f * (float)Lg + bz * Sv);
        }
      }
    }
  }

  // 4. reduce over the four phi lanes of a row; lanes 0..15 hold the row results
  float vf[NT];
  int vi[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (p.gmode == 0 && IS_INT) {
      int v = (int)Lone[t];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      vi[t] = v; vf[t] = 0.f;
    } else {
      float v = (p.gmode == 0) ? (float)Lone[t] : acc[t];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      vf[t] = v; vi[t] = 0;
    }
  }

  const int nslices = gridDim.y;
  const int m = tile * 16 + r;
  if (nslices == 1) {
    if (tile_ok && phi == 0 && m < p.M) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
        if (n0 + t < p.N) finalize_store<IS_INT, NT>(p, n0 + t, m, vf[t], vi[t]);
    }
    return;
  }

  // 5. split-K: publish the partial sums; the last workgroup to arrive for this block of rows
  // adds the slices in slice order (fixed order => reproducible) and writes the result.
  //
  // Visibility across the chip's XCDs (one L2 each) without a full L2 write-back: partials are
  // written with agent-scope atomic stores (write-through past the L2), every wave waits for
  // its stores to complete (workgroup-scope release = s_waitcnt vmcnt(0)), the barrier orders
  // all waves before thread 0's agent-scope counter increment, and the reader uses agent-scope
  // atomic loads, which do not hit stale lines of its own L2.
  const bool raw_int = (p.gmode == 0 && IS_INT);
  if (tile_ok && phi == 0) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int n = n0 + t;
      if (n < p.N) {
        const size_t o = ((size_t)blockIdx.y * p.N + n) * p.Mp + m;
        const float v = raw_int ? __int_as_float(vi[t]) : vf[t];
        __hip_atomic_store(p.ws_part + o, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) {
    int* ctr = p.ws_ctr + (size_t)blockIdx.z * gridDim.x + blockIdx.x;
    const int ticket = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (ticket == nslices - 1);
    if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = last;
  }
  __syncthreads();
  if (!s_last) return;
  for (int it = threadIdx.x; it < 128 * NT; it += 512) {
    const int t = it >> 7, rr = it & 127;
    const int mm = blockIdx.x * 128 + rr, n = n0 + t;
    if (mm >= p.M || n >= p.N) continue;
    float sf = 0.f;
    int si = 0;
    for (int sl = 0; sl < nslices; ++sl) {
      const size_t o = ((size_t)sl * p.N + n) * p.Mp + mm;
      const float v = __hip_atomic_load(p.ws_part + o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (raw_int) si += __float_as_int(v);
      else sf += v;
    }
    finalize_store<IS_INT, NT>(p, n, mm, sf, si);
  }
}

// ------------------------------------------------------------------------------------------
// Decode GEMV (N = 1..3): one workgroup = one 16-row tile over the whole K
// ------------------------------------------------------------------------------------------
// All K/4 tables of one activation row sit in LDS (32 bytes each; 32 KB at K = 4096), the
// eight waves of the workgroup take the 128-wide chunks round-robin, and the per-wave partial
// sums are combined through LDS in wave order.  No cross-workgroup reduction, no workspace,
// fixed summation order.  Index loads for the next batch of chunks are issued before the
// lookups of the current one (software pipelining), and the first batch is issued before
// the tables are staged.
template <bool IS_INT, int BITS, int GM>
__global__ __launch_bounds__(512) void mpgemv_fullk_kernel(const MpParams p) {
  using AccT = typename std::conditional<IS_INT, int, float>::type;
  constexpr int NW = 8, UN = 4;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int phi = lane >> 4, r = lane & 15;
  const int tile = blockIdx.x, n = blockIdx.y;
  const int n_its = (p.n_chunks + NW - 1) / NW;
  const uint32_t* idx_tile = p.idx + (size_t)tile * p.n_chunks * 64 * BITS + lane * BITS;
  const uint32_t* sz_tile = p.sz + (size_t)tile * p.nq * 16 + r;

  struct Batch {
    uint32_t w[UN][BITS];
    uint32_t sz[UN];
    float S[UN];
  };
  auto load_batch = [&](int it0, Batch& bt) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int c = (it0 + u) * NW + wave;
      if (c < p.n_chunks) {
        const uint32_t* src = idx_tile + (size_t)c * 64 * BITS;
        if constexpr (BITS == 4) {
          const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
          bt.w[u][0] = v.x; bt.w[u][1] = v.y; bt.w[u][2] = v.z; bt.w[u][3] = v.w;
        } else if constexpr (BITS == 2) {
          const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
          bt.w[u][0] = v.x; bt.w[u][1] = v.y;
        } else {
#pragma unroll
          for (int b = 0; b < BITS; ++b) bt.w[u][b] = __builtin_nontemporal_load(src + b);
        }
        if constexpr (GM == 1) {
          const int gq = (p.cpg == 1) ? c : c / p.cpg;
          bt.sz[u] = sz_tile[(size_t)gq * 16];
          if constexpr (IS_INT) bt.S[u] = (float)static_cast<const int*>(p.S)[(size_t)n * p.nq + gq];
          else bt.S[u] = static_cast<const float*>(p.S)[(size_t)n * p.nq + gq];
          // the bias term is added once per quantisation group: only with its first chunk
          if (p.cpg != 1 && gq * p.cpg != c) bt.S[u] = 0.f;
        }
      } else {
#pragma unroll
        for (int b = 0; b < BITS; ++b) bt.w[u][b] = 0;
        bt.sz[u] = 0;
        bt.S[u] = 0.f;
      }
    }
  };

  Batch b0, b1;
  load_batch(0, b0);

  // stage all tables of activation row n: four 16-byte pieces in flight per thread
  {
    const uint4* src = reinterpret_cast<const uint4*>(p.tables + (size_t)n * p.KG * 16);
    uint4* dst = reinterpret_cast<uint4*>(smem);
    const int items = p.KG * 2;
    for (int base = threadIdx.x; base < items; base += 512 * 4) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = src[min(base + u * 512, items - 1)];  // clamped: always in range
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (base + u * 512 < items) dst[base + u * 512] = v[u];
    }
    // all-zero chunk (32 tables) right after the real ones, used by chunk slots past the end of K
    if (threadIdx.x < 64) dst[items + threadIdx.x] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();

  float acc = 0.f;
  AccT Lone = 0;
  const uint32_t phi_rep = (uint32_t)phi * 0x20202020u;
  const float bz_on = (phi == 0) ? 1.f : 0.f;
  // LDS byte address of the tables (0: this kernel has no static LDS; the byte-permute below
  // needs it to be a multiple of 256, which any LDS base is not guaranteed to be in general)
  const uint32_t lds_base = (uint32_t)(uintptr_t)((lds_char*)smem);

  // Lookups of one index dword (one bit plane, eight LUT groups): eight LDS reads in flight.
  using RawT = typename std::conditional<IS_INT, int, uint32_t>::type;
  auto issue = [&](uint32_t x, uint32_t base, RawT (&e)[8]) {
    const uint32_t zz[2] = {((x << 1) & 0x1E1E1E1Eu) | phi_rep, ((x >> 3) & 0x1E1E1E1Eu) | phi_rep};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int j = 4 * h + jj;
        // address = {0, base byte 2, base byte 1, byte jj of zz}: one byte-permute
        const uint32_t a = __builtin_amdgcn_perm(zz[h], base, 0x0C020100u + 4u + (uint32_t)jj);
        const uint32_t ea = a + j * 128;  // constant part folds into the ds_read offset field
        if constexpr (IS_INT) e[j] = *reinterpret_cast<const lds_i16*>(ea);
        else e[j] = *reinterpret_cast<const lds_u16*>(ea);
      }
    }
  };
  auto consume = [&](const RawT (&e)[8], int b, AccT (&L)[4]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if constexpr (IS_INT) L[j >> 1] += e[j] << b;
      else L[j >> 1] = fmaf(__half2float(__ushort_as_half((uint16_t)e[j])), (float)(1 << b), L[j >> 1]);
    }
  };

  // One batch = UN chunks x BITS index dwords, walked as one flat, fully unrolled sequence: the
  // reads of dword d+1 are issued before the values of dword d are accumulated.  Chunks past the
  // end of K use the all-zero chunk appended after the real tables (and carry zero scales), so
  // the sequence has no branches.
  auto compute_batch = [&](int it0, const Batch& bt) {
    constexpr int ND = UN * BITS;
    uint32_t base[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int c = (it0 + u) * NW + wave;
      base[u] = lds_base + (uint32_t)min(c, p.n_chunks) * 1024u;
    }
    RawT e[2][8];
    AccT L[4] = {0, 0, 0, 0};
    issue(bt.w[0][0], base[0], e[0]);
#pragma unroll
    for (int d = 0; d < ND; ++d) {
      const int u = d / BITS, b = d % BITS;
      if (d + 1 < ND) issue(bt.w[(d + 1) / BITS][(d + 1) % BITS], base[(d + 1) / BITS], e[(d + 1) & 1]);
      consume(e[d & 1], b, L);
      // keep about 16 reads in flight instead of hoisting the reads of the whole batch
      // (the empty asm pins both the reads issued above and the accumulation of this step)
      asm volatile("" : "+v"(L[0]), "+v"(L[1]), "+v"(L[2]), "+v"(L[3]) : : "memory");
      __builtin_amdgcn_sched_barrier(0);
      if (b == BITS - 1) {
        const AccT Lc = (L[0] + L[1]) + (L[2] + L[3]);
        L[0] = L[1] = L[2] = L[3] = 0;
        if constexpr (GM == 0) {
          Lone += Lc;
        } else {
          const float s = __half2float(__ushort_as_half((uint16_t)(bt.sz[u] & 0xffff)));
          const float z = __half2float(__ushort_as_half((uint16_t)(bt.sz[u] >> 16)));
          acc += s * (0.5f * (float)Lc + (bz_on * (p.mid - z)) * bt.S[u]);
        }
      }
    }
  };

  for (int it0 = 0; it0 < n_its; it0 += 2 * UN) {
    if (it0 + UN < n_its) load_batch(it0 + UN, b1);
    compute_batch(it0, b0);
    if (it0 + 2 * UN < n_its) load_batch(it0 + 2 * UN, b0);
    if (it0 + UN < n_its) compute_batch(it0 + UN, b1);
  }

  // reduce: four phi lanes per row, then the eight waves through LDS in wave order
  float* red = reinterpret_cast<float*>(smem + (size_t)p.KG * 32 + 1024);
  constexpr bool RAW_INT = (GM == 0 && IS_INT);
  if constexpr (RAW_INT) {
    int v = (int)Lone;
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    if (phi == 0) red[wave * 16 + r] = __int_as_float(v);
  } else {
    float v = (GM == 0) ? (float)Lone : acc;
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    if (phi == 0) red[wave * 16 + r] = v;
  }
  __syncthreads();
  if (threadIdx.x < 16) {
    const int m = tile * 16 + threadIdx.x;
    float sf = 0.f;
    int si = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float v = red[w * 16 + threadIdx.x];
      if constexpr (RAW_INT) si += __float_as_int(v);
      else sf += v;
    }
    if (m < p.M) finalize_store<IS_INT, 1>(p, n, m, sf, si);
  }
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Last HIP error seen by this thread while enqueuing (diagnostics only).
static thread_local hipError_t g_last_hip_error = hipSuccess;
void note_hip_error(int hip_error) { g_last_hip_error = static_cast<hipError_t>(hip_error); }

// Launch through hipLaunchKernel so that the status is this launch's own and not a stale
// error left behind by some other user of the runtime in the same process.
template <typename... KArgs, typename... Args>
static hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st,
                         Args... args) {
  std::tuple<KArgs...> store(args...);
  void* ptrs[sizeof...(KArgs)];
  fill_ptrs(store, ptrs, std::index_sequence_for<KArgs...>{});
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, st);
  if (e != hipSuccess) g_last_hip_error = e;
  return e;
}

struct LaunchShape {
  int ks, nt, nslices, row_blocks, n_tiles_z;
};

static LaunchShape launch_shape(const tmac_wdesc* d, int N, const tmac_tuning* tun) {
  const Geometry ge = geometry(d);
  LaunchShape ls;
  ls.nt = (tun && tun->n_tile) ? tun->n_tile : (N >= 4 ? 4 : 1);
  ls.ks = (tun && tun->chunks_per_wave) ? tun->chunks_per_wave : (ls.nt == 1 ? (d->bits <= 2 ? 8 : 4) : 4);
  ls.nslices = (ge.n_chunks + ls.ks - 1) / ls.ks;
  ls.row_blocks = (ge.n_tiles + 7) / 8;
  ls.n_tiles_z = (N + ls.nt - 1) / ls.nt;
  return ls;
}

static const int KS_MAX_SLICES_CHUNKS = 2;  // smallest chunks_per_wave: bounds the workspace

template <bool IS_INT, int BITS, int NT>
static hipError_t launch_ks(const MpParams& p, const LaunchShape& ls, hipStream_t st) {
  const dim3 grid(ls.row_blocks, ls.nslices, ls.n_tiles_z), block(512);
  switch (ls.ks) {
    case 2: return launch(mpgemm_lds_kernel<IS_INT, BITS, NT, 2>, grid, block, 0, st, p);
    case 4: return launch(mpgemm_lds_kernel<IS_INT, BITS, NT, 4>, grid, block, 0, st, p);
    case 8: return launch(mpgemm_lds_kernel<IS_INT, BITS, NT, 8>, grid, block, 0, st, p);
  }
  return hipErrorInvalidValue;
}

template <bool IS_INT, int BITS>
static hipError_t launch_nt(const MpParams& p, const LaunchShape& ls, hipStream_t st) {
  if (ls.nt == 1) return launch_ks<IS_INT, BITS, 1>(p, ls, st);
  if (ls.nt == 4) return launch_ks<IS_INT, BITS, 4>(p, ls, st);
  return hipErrorInvalidValue;
}

template <bool IS_INT>
static hipError_t launch_bits(int bits, const MpParams& p, const LaunchShape& ls, hipStream_t st) {
  switch (bits) {
    case 1: return launch_nt<IS_INT, 1>(p, ls, st);
    case 2: return launch_nt<IS_INT, 2>(p, ls, st);
    case 3: return launch_nt<IS_INT, 3>(p, ls, st);
    case 4: return launch_nt<IS_INT, 4>(p, ls, st);
  }
  return hipErrorInvalidValue;
}

// ---- full-K GEMV dispatch ----
constexpr size_t LDS_LIMIT = 160 * 1024;

// tables, one all-zero chunk, per-wave partial sums
static size_t fullk_lds_bytes(int KG) { return (size_t)KG * 32 + 1024 + 8 * 16 * 4; }

template <bool IS_INT, int BITS, int GM>
static hipError_t launch_fullk_one(const MpParams& p, hipStream_t st) {
  const size_t lds = fullk_lds_bytes(p.KG);
  auto kernel = mpgemv_fullk_kernel<IS_INT, BITS, GM>;
  if (lds > 64 * 1024) {
    // opt in to more than 64 KB of dynamic LDS, once per kernel instantiation
    static bool raised = false;
    if (!raised) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_LIMIT);
      if (e != hipSuccess) { g_last_hip_error = e; return e; }
      raised = true;
    }
  }
  return launch(kernel, dim3(p.n_tiles, p.N), dim3(512), lds, st, p);
}

template <bool IS_INT, int BITS>
static hipError_t launch_fullk_gm(const MpParams& p, hipStream_t st) {
  return p.gmode == 0 ? launch_fullk_one<IS_INT, BITS, 0>(p, st) : launch_fullk_one<IS_INT, BITS, 1>(p, st);
}

template <bool IS_INT>
static hipError_t launch_fullk(int bits, const MpParams& p, hipStream_t st) {
  switch (bits) {
    case 1: return launch_fullk_gm<IS_INT, 1>(p, st);
    case 2: return launch_fullk_gm<IS_INT, 2>(p, st);
    case 3: return launch_fullk_gm<IS_INT, 3>(p, st);
    case 4: return launch_fullk_gm<IS_INT, 4>(p, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace tmac

using namespace tmac;

extern "C" size_t tmac_lut_bytes(int32_t N, int32_t K, int32_t g, int32_t group, tmac_lut_t lut) {
  LutGeom lg;
  if (lut != TMAC_LUT_F16 && lut != TMAC_LUT_I16 && lut != TMAC_LUT_I8Q) return 0;
  if (!lut_geom(N, K, g, group, (int)lut, &lg)) return 0;
  return lg.total;
}

extern "C" tmac_status tmac_precompute_lut(const void* A_dev, tmac_act_t act, int32_t N, int32_t K,
                                           int64_t lda, int32_t g, int32_t group, tmac_lut_t lut,
                                           void* lut_dev, size_t lut_bytes, void* stream) {
  if (!A_dev || !lut_dev) return TMAC_EINVAL;
  if (!((act == TMAC_ACT_F16 && (lut == TMAC_LUT_F16 || lut == TMAC_LUT_I8Q)) ||
        (act == TMAC_ACT_I8 && lut == TMAC_LUT_I16)))
    return TMAC_EINVAL;
  LutGeom lg;
  if (!lut_geom(N, K, g, group, (int)lut, &lg)) return TMAC_EINVAL;
  if (lda < K) return TMAC_EINVAL;
  if (!aligned16(lut_dev)) return TMAC_EINVAL;
  const uintptr_t a_align = (act == TMAC_ACT_F16) ? 7u : 3u;  // one group of 4 activations per load
  if ((reinterpret_cast<uintptr_t>(A_dev) & a_align) != 0 || (lda % 4) != 0) return TMAC_EINVAL;
  if (lut_bytes < lg.total) return TMAC_ESIZE;

  const int n_sum_blocks = (N * lg.nq + 3) / 4;
  if (lut == TMAC_LUT_I8Q) {
    char* base = static_cast<char*>(lut_dev);
    const int n_unit_blocks = (int)(((int64_t)N * lg.U + 255) / 256);
    const hipError_t eq = launch(precompute_q8_kernel, dim3(n_unit_blocks + n_sum_blocks), dim3(256), 0,
                                 static_cast<hipStream_t>(stream), static_cast<const __half*>(A_dev), N, K, lda, lg.U,
                                 reinterpret_cast<float*>(base + lg.s_off), reinterpret_cast<float*>(base + lg.s16_off),
                                 reinterpret_cast<float*>(base + lg.s128_off), reinterpret_cast<float*>(base + lg.usc_off),
                                 reinterpret_cast<uint4*>(base + lg.ht_off), lg.Geff, lg.nq, n_unit_blocks);
    return eq == hipSuccess ? TMAC_OK : TMAC_EHIP;
  }
  const int64_t n_items = (int64_t)N * lg.KG;
  const int n_tab_blocks = (int)((n_items + 255) / 256);
  uint4* tables = static_cast<uint4*>(lut_dev);
  void* S = static_cast<char*>(lut_dev) + lg.s_off;
  void* S16 = static_cast<char*>(lut_dev) + lg.s16_off;
  void* S128 = static_cast<char*>(lut_dev) + lg.s128_off;
  uint4* HT = reinterpret_cast<uint4*>(static_cast<char*>(lut_dev) + lg.ht_off);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid(n_tab_blocks + n_sum_blocks), block(256);
  const hipError_t e =
      (act == TMAC_ACT_F16)
          ? launch(precompute_kernel<false>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S, S16, S128, HT,
                   lg.U, lg.Geff, lg.nq, n_tab_blocks)
          : launch(precompute_kernel<true>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S, S16, S128, HT,
                   lg.U, lg.Geff, lg.nq, n_tab_blocks);
  return e == hipSuccess ? TMAC_OK : TMAC_EHIP;
}

extern "C" size_t tmac_workspace_bytes(const tmac_wdesc* desc, int32_t N) {
  if (!desc_valid(desc) || N <= 0) return 0;
  if (desc->layout == TMAC_LAYOUT_R8U16) return 256;  // the register-table kernel uses none
  if (desc->layout == TMAC_LAYOUT_R64K32) {
    const RowsPlan pl = rows_plan(desc, N);
    return pl.part_bytes + pl.ctr_bytes + 256;
  }
  const Geometry ge = geometry(desc);
  const size_t max_slices = (ge.n_chunks + KS_MAX_SLICES_CHUNKS - 1) / KS_MAX_SLICES_CHUNKS;
  const size_t part = (max_slices * (size_t)N * ge.Mp * 4 + 255) / 256 * 256;
  const size_t row_blocks = (ge.n_tiles + 7) / 8;
  const size_t ctr = (row_blocks * (size_t)N * 4 + 255) / 256 * 256;  // n tiles <= N
  return part + ctr;
}

extern "C" tmac_status tmac_mpgemm_ex(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                                      tmac_lut_t lut, int32_t N, const float* act_scale_dev,
                                      float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                      void* workspace_dev, size_t workspace_bytes, void* stream,
                                      const tmac_tuning* tuning) {
  if (!desc_valid(desc) || !packed_dev || !lut_dev || !out_dev || N <= 0) return TMAC_EINVAL;
  if (lut != TMAC_LUT_F16 && lut != TMAC_LUT_I16 && lut != TMAC_LUT_I8Q) return TMAC_EINVAL;
  if (out != TMAC_OUT_F32 && out != TMAC_OUT_F16 && out != TMAC_OUT_I32) return TMAC_EINVAL;
  if (!aligned16(packed_dev) || !aligned16(lut_dev) || !aligned16(workspace_dev)) return TMAC_EINVAL;
  if (lut == TMAC_LUT_I8Q && desc->layout != TMAC_LAYOUT_R8U16) return TMAC_EUNSUPPORTED;
  if (ldo < desc->M) return TMAC_EINVAL;
  if (!group_supported(desc)) return TMAC_EUNSUPPORTED;
  if (tuning) {
    const int ks = tuning->chunks_per_wave, nt = tuning->n_tile;
    if (!(ks == 0 || ks == 2 || ks == 4 || ks == 8) || !(nt == 0 || nt == 1 || nt == 4)) return TMAC_EINVAL;
    if (tuning->kernel < 0 || tuning->kernel > 2) return TMAC_EINVAL;
  }
  const Geometry ge = geometry(desc);
  LutGeom lg;
  if (!lut_geom(N, desc->K, desc->g, desc->group, (int)lut, &lg)) return TMAC_EINVAL;
  const bool is_int = (lut == TMAC_LUT_I16);
  const bool one_group = (desc->group == 0 || desc->group == desc->K);
  if (desc->layout == TMAC_LAYOUT_R8U16) {
    // register-table decode kernel; it needs no workspace and takes none of the LDS kernels' knobs
    if (tuning && (tuning->kernel != 0 || tuning->chunks_per_wave != 0 || tuning->n_tile != 0))
      return TMAC_EUNSUPPORTED;
    const int rpg = tuning ? tuning->rows_per_group : 0;
    if (rpg != 0 && rpg != 8 && rpg != 16) return TMAC_EINVAL;
    return static_cast<tmac_status>(launch_perm_gemv(desc, packed_dev, lut_dev, nullptr, 0, (int)lut, N,
                                                      act_scale_dev, weight_scale, out_dev, (int)out, ldo,
                                                      stream, rpg));
  }
  if (desc->layout == TMAC_LAYOUT_R64K32) {
    // batched lookup kernel (lane = weight row); no workspace, no launch-shape knobs
    if (tuning && (tuning->kernel != 0 || tuning->chunks_per_wave != 0 || tuning->n_tile != 0 ||
                   tuning->rows_per_group != 0))
      return TMAC_EUNSUPPORTED;
    return static_cast<tmac_status>(launch_rows_gemm(desc, packed_dev, lut_dev, (int)lut, N, act_scale_dev,
                                                      weight_scale, out_dev, (int)out, ldo, workspace_dev,
                                                      workspace_bytes, stream));
  }
  // int32 accumulators: |L| <= 508 * (2^b - 1) * K/4 must stay below 2^31
  if (is_int && (double)508.0 * ((1 << desc->bits) - 1) * (desc->K / 4) >= 2147483647.0) return TMAC_EUNSUPPORTED;

  MpParams p;
  const char* blob = static_cast<const char*>(packed_dev);
  p.idx = reinterpret_cast<const uint32_t*>(blob + ge.idx_off);
  p.sz = reinterpret_cast<const uint32_t*>(blob + ge.sz_off);
  p.tables = static_cast<const uint16_t*>(lut_dev);
  p.S = static_cast<const char*>(lut_dev) + lg.s_off;
  p.out = out_dev;
  p.act_scale = act_scale_dev;
  p.ldo = ldo;
  p.M = desc->M; p.Mp = ge.Mp; p.N = N; p.KG = lg.KG;
  p.n_tiles = ge.n_tiles; p.n_chunks = ge.n_chunks; p.nq = lg.nq;
  p.gmode = one_group ? 0 : 1;
  p.G = lg.Geff;
  p.gpc_shift = (!one_group && desc->group == 32) ? 2 : (!one_group && desc->group == 64) ? 1 : 0;
  p.per_tensor = (desc->group == 0);
  p.wscale = weight_scale;
  p.mid = 0.5f * (float)((1 << desc->bits) - 1);
  p.zero_point = 0.f;
  p.int_exact = 0;
  p.icoef = 0;
  p.out_t = (int)out;
  if (p.per_tensor) {
    p.zero_point = desc->zero_point;
    const float z = desc->zero_point;
    if (is_int && z == rintf(z) && fabsf(z) < 64.f) {
      p.int_exact = 1;
      p.icoef = ((1 << desc->bits) - 1) - 2 * (int)z;
    }
  }
  if (out == TMAC_OUT_I32 && !p.int_exact) return TMAC_EINVAL;
  const bool whole_chunk_groups = !one_group && (desc->group % 128 == 0);
  p.cpg = whole_chunk_groups ? desc->group / 128 : 1;
  hipStream_t st = static_cast<hipStream_t>(stream);

  // Decode GEMV: few activation rows, all tables of a row fit in LDS
  const int want = tuning ? tuning->kernel : 0;
  const bool fullk_ok = (one_group || whole_chunk_groups) && fullk_lds_bytes(lg.KG) <= LDS_LIMIT &&
                        ge.n_tiles <= 0x7fffffff && N <= 65535;
  if (want == 2 && !fullk_ok) return TMAC_EUNSUPPORTED;
  const bool sliced_knobs = tuning && (tuning->chunks_per_wave != 0 || tuning->n_tile != 0);
  if (want == 2 || (want == 0 && fullk_ok && N <= 3 && !sliced_knobs)) {
    const hipError_t e = is_int ? launch_fullk<true>(desc->bits, p, st) : launch_fullk<false>(desc->bits, p, st);
    return e == hipSuccess ? TMAC_OK : TMAC_EHIP;
  }

  const LaunchShape ls = launch_shape(desc, N, tuning);
  const size_t max_slices = (ge.n_chunks + KS_MAX_SLICES_CHUNKS - 1) / KS_MAX_SLICES_CHUNKS;
  const size_t part_bytes = (max_slices * (size_t)N * ge.Mp * 4 + 255) / 256 * 256;
  if (ls.nslices > 1) {
    if (!workspace_dev) return TMAC_EINVAL;
    if (workspace_bytes < tmac_workspace_bytes(desc, N)) return TMAC_ESIZE;
  }
  p.ws_part = static_cast<float*>(workspace_dev);
  p.ws_ctr = workspace_dev ? reinterpret_cast<int*>(static_cast<char*>(workspace_dev) + part_bytes) : nullptr;
  if (ls.row_blocks > 65535 * 32 || ls.nslices > 65535 || ls.n_tiles_z > 65535) return TMAC_EUNSUPPORTED;

  const hipError_t e = is_int ? launch_bits<true>(desc->bits, p, ls, st) : launch_bits<false>(desc->bits, p, ls, st);
  return e == hipSuccess ? TMAC_OK : TMAC_EHIP;
}

extern "C" tmac_status tmac_mpgemv_fused_ex(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                                            tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                                            float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                            void* stream, const tmac_tuning* tuning) {
  if (!desc_valid(desc) || !packed_dev || !A_dev || !out_dev || N <= 0) return TMAC_EINVAL;
  if (act != TMAC_ACT_F16 && act != TMAC_ACT_I8) return TMAC_EINVAL;
  if (out != TMAC_OUT_F32 && out != TMAC_OUT_F16 && out != TMAC_OUT_I32) return TMAC_EINVAL;
  if (!aligned16(packed_dev) || !aligned16(A_dev)) return TMAC_EINVAL;
  if (ldo < desc->M || lda < desc->K) return TMAC_EINVAL;
  // every lane reads the 16 activations of its unit with 16-byte loads
  const int64_t row_elems_16B = (act == TMAC_ACT_F16) ? 8 : 16;
  if (lda % row_elems_16B != 0) return TMAC_EINVAL;
  if (desc->layout != TMAC_LAYOUT_R8U16 || desc->K % 16 != 0) return TMAC_EUNSUPPORTED;
  if (!group_supported(desc)) return TMAC_EUNSUPPORTED;
  int rpg = 0;
  if (tuning) {
    if (tuning->kernel != 0 || tuning->chunks_per_wave != 0 || tuning->n_tile != 0) return TMAC_EUNSUPPORTED;
    rpg = tuning->rows_per_group;
    if (rpg != 0 && rpg != 8 && rpg != 16) return TMAC_EINVAL;
  }
  return static_cast<tmac_status>(launch_perm_gemv(desc, packed_dev, nullptr, A_dev, lda,
                                                    act == TMAC_ACT_I8 ? (int)TMAC_LUT_I16 : (int)TMAC_LUT_F16,
                                                    N, act_scale_dev, weight_scale, out_dev, (int)out, ldo,
                                                    stream, rpg));
}

extern "C" tmac_status tmac_mpgemv_fused(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                                         tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                                         float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                         void* stream) {
  return tmac_mpgemv_fused_ex(desc, packed_dev, A_dev, act, N, lda, act_scale_dev, weight_scale, out_dev, out, ldo,
                              stream, nullptr);
}

extern "C" tmac_status tmac_mpgemm(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                                   tmac_lut_t lut, int32_t N, const float* act_scale_dev, float weight_scale,
                                   void* out_dev, tmac_out_t out, int64_t ldo, void* workspace_dev,
                                   size_t workspace_bytes, void* stream) {
  return tmac_mpgemm_ex(desc, packed_dev, lut_dev, lut, N, act_scale_dev, weight_scale, out_dev, out, ldo,
                        workspace_dev, workspace_bytes, stream, nullptr);
}

extern "C" const char* tmac_last_error_detail(void) {
  return g_last_hip_error == hipSuccess ? "" : hipGetErrorString(g_last_hip_error);
}

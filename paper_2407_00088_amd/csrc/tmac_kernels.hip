// Table precompute kernels (gfx950) and the device entry points of the LUT mpGEMM library.
//
//   precompute_kernel     Algorithm 1 "Precompute": one 16-entry table per 4 activations, plus
//                         the activation sums (per quantisation group, per 16 and per 128
//                         activations) needed by the bias term of Section 4 ("Bit-serial linear
//                         transformation"), plus the mirror-consolidated, byte-split half tables
//                         of the decode kernel (Section 3.3, Section 4).
//   precompute_q8_kernel  the same with table quantisation (Section 3.3): int8 entries and one
//                         scale per 16 activations.
//   precompute_g_kernel   tables for the LUT group sizes 2 and 8.
//
// The lookup kernels live in tmac_perm.hip (decode, packed layout 2) and tmac_rows.hip (many
// activation rows, packed layout 3).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <tuple>
#include <utility>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

template <typename Tuple, size_t... I>
static void fill_ptrs(Tuple& t, void** ptrs, std::index_sequence<I...>) {
  ((ptrs[I] = static_cast<void*>(&std::get<I>(t))), ...);
}


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

// The tables as the batched kernels keep them in LDS: [n tile][KG][2^G][NT] 16-bit entries, NT
// activation rows side by side per entry, so that staging a K slice is a plain copy.  Thread `id`
// builds the two consecutive entries 2 id, 2 id + 1 (counted over [n tile][KG][2^G]) for the NT
// rows of its tile: T[p] = sum_j (bit j of p ? +a_j : -a_j), added pairwise in fp16 (the tree of
// half_table_f16, one level less at g = 2, one more at g = 8; exact int16 for int8 activations);
// rows past N and tables past K are zero.
template <bool IS_INT, int G, int NT>
__device__ __forceinline__ void staged_tables(const void* __restrict__ A_, int N, int K, int64_t lda, int KG,
                                              uint4* __restrict__ tables, int64_t id) {
  constexpr int ENT = 1 << G;
  const int64_t per_tile = (int64_t)KG * ENT / 2;
  const int tile = (int)(id / per_tile);
  const int64_t f = (id % per_tile) * 2;            // first of the two entries in [KG][ENT]
  const int kg = (int)(f >> G), e0 = (int)(f & (ENT - 1));
  const int k0 = kg * G;
  uint32_t w[2][NT / 2];                            // [entry][pair of rows]
#pragma unroll
  for (int r = 0; r < NT; ++r) {
    const int n = tile * NT + r;
    uint16_t e[2] = {0, 0};
    if (n < N && k0 < K) {                          // K is a multiple of 4 and of G: all or nothing
      if constexpr (IS_INT) {
        // (row bases and lda are multiples of 4 bytes: G elements come with 2- or 4-byte loads)
        const int8_t* ap = static_cast<const int8_t*>(A_) + n * lda + k0;
        int a[G];
        if constexpr (G == 2) {
          const uint16_t v = *reinterpret_cast<const uint16_t*>(ap);
          a[0] = (int8_t)(v & 0xff); a[1] = (int8_t)(v >> 8);
        } else {
#pragma unroll
          for (int q = 0; q < G / 4; ++q) {
            const uint32_t v = reinterpret_cast<const uint32_t*>(ap)[q];
#pragma unroll
            for (int j = 0; j < 4; ++j) a[4 * q + j] = (int8_t)((v >> (8 * j)) & 0xff);
          }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          int v = 0;
#pragma unroll
          for (int j = 0; j < G; ++j) v += (((e0 + u) >> j) & 1) ? a[j] : -a[j];
          e[u] = (uint16_t)(int16_t)v;
        }
      } else {
        // (row bases and lda are multiples of 8 bytes: G elements come with 4- or 8-byte loads)
        const __half* ap = static_cast<const __half*>(A_) + n * lda + k0;
        _Float16 x[G];
        if constexpr (G == 2) {
          const tmac_h2 v = *reinterpret_cast<const tmac_h2*>(ap);
          x[0] = v.x; x[1] = v.y;
        } else {
#pragma unroll
          for (int q = 0; q < G / 4; ++q) {
            const uint2 v = reinterpret_cast<const uint2*>(ap)[q];
            const tmac_h2 v0 = __builtin_bit_cast(tmac_h2, v.x), v1 = __builtin_bit_cast(tmac_h2, v.y);
            x[4 * q + 0] = v0.x; x[4 * q + 1] = v0.y; x[4 * q + 2] = v1.x; x[4 * q + 3] = v1.y;
          }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          _Float16 y[G];
#pragma unroll
          for (int j = 0; j < G; ++j) y[j] = (((e0 + u) >> j) & 1) ? x[j] : -x[j];
#pragma unroll
          for (int st = 1; st < G; st *= 2) {       // pairwise, every add in fp16: ((y0+y1)+(y2+y3))+...
#pragma unroll
            for (int j = 0; j + st < G; j += 2 * st) y[j] = y[j] + y[j + st];
          }
          e[u] = __builtin_bit_cast(uint16_t, y[0]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (r & 1) w[u][r >> 1] |= (uint32_t)e[u] << 16;
      else w[u][r >> 1] = e[u];
    }
  }
  if constexpr (NT == 8) {
    tables[id * 2] = make_uint4(w[0][0], w[0][1], w[0][2], w[0][3]);
    tables[id * 2 + 1] = make_uint4(w[1][0], w[1][1], w[1][2], w[1][3]);
  } else {
    tables[id] = make_uint4(w[0][0], w[0][1], w[1][0], w[1][1]);
  }
}

template <bool IS_INT>
__global__ __launch_bounds__(256) void precompute_kernel(const void* __restrict__ A_, int N, int K,
                                                         int64_t lda, int KG,
                                                         uint4* __restrict__ tables,
                                                         void* __restrict__ S_, void* __restrict__ S16_,
                                                         void* __restrict__ S128_,
                                                         uint4* __restrict__ HT, int U, int Geff, int nq,
                                                         int n_tab_blocks, int n_stage_blocks, int NT) {
  if ((int)blockIdx.x >= n_tab_blocks && (int)blockIdx.x < n_tab_blocks + n_stage_blocks) {
    // the tables of the batched kernels, one thread per two entries of an n tile
    const int64_t id = (int64_t)((int)blockIdx.x - n_tab_blocks) * 256 + threadIdx.x;
    const int64_t n_ids = (int64_t)((N + NT - 1) / NT) * KG * 8;
    if (id >= n_ids) return;
    if (NT == 8) staged_tables<IS_INT, 4, 8>(A_, N, K, lda, KG, tables, id);
    else staged_tables<IS_INT, 4, 4>(A_, N, K, lda, KG, tables, id);
    return;
  }
  if ((int)blockIdx.x < n_tab_blocks) {
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tid >= (int64_t)N * KG) return;
    const int n = (int)(tid / KG), kg = (int)(tid % KG);
    uint32_t packed[4];  // entries 0..7 (the mirror half), two per dword
    float sum4f = 0.f;  // sum of this table's four activations (for the per-16 unit sums)
    int sum4i = 0;
    if (4 * kg >= K) {
#pragma unroll
      for (int i = 0; i < 4; ++i) packed[i] = 0;  // k padding: all-zero table
    } else if constexpr (IS_INT) {
      const int8_t* a = static_cast<const int8_t*>(A_) + n * lda + 4 * kg;
      const int a0 = a[0], a1 = a[1], a2 = a[2], a3 = a[3];
      sum4i = a0 + a1 + a2 + a3;
      int e[8];
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        e[p] = ((p & 1) ? a0 : -a0) + ((p & 2) ? a1 : -a1) + ((p & 4) ? a2 : -a2) - a3;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        packed[i] = ((uint32_t)e[2 * i] & 0xffffu) | ((uint32_t)e[2 * i + 1] << 16);
    } else {
      // (row bases and lda are multiples of 8 bytes)
      const uint2 v = *reinterpret_cast<const uint2*>(static_cast<const __half*>(A_) + n * lda + 4 * kg);
      sum4f = sum4_f16(v.x, v.y);
      half_table_f16(v.x, v.y, packed);
    }
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
    group_sums_wave<IS_INT>(A_, N, lda, S_, Geff, nq,
                            ((int)blockIdx.x - n_tab_blocks - n_stage_blocks) * 4 + (threadIdx.x >> 6));
  }
}

// Tables for LUT group sizes other than 4 (Section 4 discusses the choice of g), in the layout
// of the batched kernels, and the group sums.
template <bool IS_INT, int G, int NT>
__global__ __launch_bounds__(256) void precompute_g_kernel(const void* __restrict__ A_, int N, int K, int64_t lda,
                                                           int KG, uint4* __restrict__ tables,
                                                           void* __restrict__ S_, int Geff, int nq,
                                                           int n_tab_blocks) {
  static_assert(G == 2 || G == 8, "g = 4 has its own kernel");
  if ((int)blockIdx.x >= n_tab_blocks) {
    group_sums_wave<IS_INT>(A_, N, lda, S_, Geff, nq, ((int)blockIdx.x - n_tab_blocks) * 4 + (threadIdx.x >> 6));
    return;
  }
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= (int64_t)((N + NT - 1) / NT) * KG * ((1 << G) / 2)) return;
  staged_tables<IS_INT, G, NT>(A_, N, K, lda, KG, tables, id);
}

// Table quantisation (Section 3.3): one thread per unit of 16 activations builds the mirror halves
// of its four tables in fp32 (they are rounded once, to int8), takes the unit's largest magnitude
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
// Host side
// ------------------------------------------------------------------------------------------
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launch-shape knobs: NULL or all zero = defaults.
static bool tuning_valid(const tmac_tuning* t) {
  if (!t) return true;
  if (t->rows_per_group != 0 && t->rows_per_group != 8 && t->rows_per_group != 16) return false;
  if (t->group_waves < 0 || t->group_waves > 16 || t->workgroup_waves < 0 || t->workgroup_waves > 16) return false;
  if (t->workgroups_per_cu != 0 && (t->workgroups_per_cu < 2 || t->workgroups_per_cu > 8)) return false;
  for (int r : t->reserved)
    if (r != 0) return false;
  return true;
}
static bool tuning_default(const tmac_tuning* t) {
  return !t || (t->rows_per_group == 0 && t->group_waves == 0 && t->workgroup_waves == 0 && t->workgroups_per_cu == 0);
}

// Last HIP error seen by this thread while enqueuing (diagnostics only).
static thread_local hipError_t g_last_hip_error = hipSuccess;
static thread_local const char* g_last_detail = nullptr;  // a refusal's explanation (a string literal), newer than the error
void note_hip_error(int hip_error) {
  g_last_hip_error = static_cast<hipError_t>(hip_error);
  g_last_detail = nullptr;
}
void note_detail(const char* text) { g_last_detail = text; }

// Launch through hipLaunchKernel so that the status is this launch's own and not a stale
// error left behind by some other user of the runtime in the same process.
template <typename... KArgs, typename... Args>
static hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st,
                         Args... args) {
  std::tuple<KArgs...> store(args...);
  void* ptrs[sizeof...(KArgs)];
  fill_ptrs(store, ptrs, std::index_sequence_for<KArgs...>{});
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, st);
  if (e != hipSuccess) note_hip_error((int)e);
  return e;
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

  const int64_t n_sum_blocks64 = ((int64_t)N * lg.nq + 3) / 4;
  const int64_t n_stage_ids = (int64_t)((N + lg.NT - 1) / lg.NT) * lg.KG * ((1 << g) / 2);
  const int64_t n_items = (int64_t)N * lg.KG;  // tables (g = 4: one lane each in the half-table part)
  // every part of the grid, and their sum, must fit the 32-bit block index
  if (n_sum_blocks64 + (n_stage_ids + 255) / 256 + (n_items + 255) / 256 > 0x7fffffff) return TMAC_EUNSUPPORTED;
  const int n_sum_blocks = (int)n_sum_blocks64;
  const int n_stage_blocks = (int)((n_stage_ids + 255) / 256);
  if (g != 4) {
    uint4* tables = static_cast<uint4*>(lut_dev);
    void* S = static_cast<char*>(lut_dev) + lg.s_off;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(n_stage_blocks + n_sum_blocks), block(256);
    const bool is_int = (act == TMAC_ACT_I8);
    hipError_t e;
    if (g == 2 && lg.NT == 8) {
      e = is_int ? launch(precompute_g_kernel<true, 2, 8>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S,
                          lg.Geff, lg.nq, n_stage_blocks)
                 : launch(precompute_g_kernel<false, 2, 8>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S,
                          lg.Geff, lg.nq, n_stage_blocks);
    } else if (g == 2) {
      e = is_int ? launch(precompute_g_kernel<true, 2, 4>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S,
                          lg.Geff, lg.nq, n_stage_blocks)
                 : launch(precompute_g_kernel<false, 2, 4>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S,
                          lg.Geff, lg.nq, n_stage_blocks);
    } else {
      e = is_int ? launch(precompute_g_kernel<true, 8, 4>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S,
                          lg.Geff, lg.nq, n_stage_blocks)
                 : launch(precompute_g_kernel<false, 8, 4>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S,
                          lg.Geff, lg.nq, n_stage_blocks);
    }
    return e == hipSuccess ? TMAC_OK : TMAC_EHIP;
  }
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
  const int n_tab_blocks = lg.decode_parts ? (int)((n_items + 255) / 256) : 0;
  uint4* tables = static_cast<uint4*>(lut_dev);
  void* S = static_cast<char*>(lut_dev) + lg.s_off;
  void* S16 = static_cast<char*>(lut_dev) + lg.s16_off;
  void* S128 = static_cast<char*>(lut_dev) + lg.s128_off;
  uint4* HT = reinterpret_cast<uint4*>(static_cast<char*>(lut_dev) + lg.ht_off);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid(n_tab_blocks + n_stage_blocks + n_sum_blocks), block(256);
  const hipError_t e =
      (act == TMAC_ACT_F16)
          ? launch(precompute_kernel<false>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S, S16, S128, HT,
                   lg.U, lg.Geff, lg.nq, n_tab_blocks, n_stage_blocks, lg.NT)
          : launch(precompute_kernel<true>, grid, block, 0, st, A_dev, N, K, lda, lg.KG, tables, S, S16, S128, HT,
                   lg.U, lg.Geff, lg.nq, n_tab_blocks, n_stage_blocks, lg.NT);
  return e == hipSuccess ? TMAC_OK : TMAC_EHIP;
}

extern "C" size_t tmac_workspace_bytes(const tmac_wdesc* desc, int32_t N) {
  if (!desc_valid(desc) || N <= 0) return 0;
  if (desc->layout == TMAC_LAYOUT_R8U16) return 256;  // the register-table kernel uses none
  const RowsPlan pl = rows_plan(desc, N);
  return pl.part_bytes + pl.ctr_bytes + pl.srow_bytes + 256;
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
  if (ldo < desc->M) return TMAC_EINVAL;
  if (!group_supported(desc)) return TMAC_EUNSUPPORTED;
  if (!tuning_valid(tuning)) return TMAC_EINVAL;
  if (desc->layout == TMAC_LAYOUT_R8U16) {
    // register-table decode kernel; it needs no workspace
    return static_cast<tmac_status>(launch_perm_gemv(desc, packed_dev, lut_dev, nullptr, 0, (int)lut, N,
                                                      act_scale_dev, weight_scale, out_dev, (int)out, ldo,
                                                      stream, tuning));
  }
  // batched lookup kernel (lane = weight row); no launch-shape knobs
  if (!tuning_default(tuning)) return TMAC_EUNSUPPORTED;
  return static_cast<tmac_status>(launch_rows_gemm(desc, packed_dev, lut_dev, nullptr, 0, (int)lut, N, act_scale_dev,
                                                    weight_scale, out_dev, (int)out, ldo, workspace_dev,
                                                    workspace_bytes, stream));
}

extern "C" tmac_status tmac_mpgemv_fused_ex(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                                            tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                                            float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                            void* stream, const tmac_tuning* tuning) {
  if (!desc_valid(desc) || !packed_dev || !A_dev || !out_dev || N <= 0) return TMAC_EINVAL;
  if (act != TMAC_ACT_F16 && act != TMAC_ACT_I8 && act != TMAC_ACT_F16_TQ) return TMAC_EINVAL;
  if (out != TMAC_OUT_F32 && out != TMAC_OUT_F16 && out != TMAC_OUT_I32) return TMAC_EINVAL;
  if (!aligned16(packed_dev) || !aligned16(A_dev)) return TMAC_EINVAL;
  if (ldo < desc->M || lda < desc->K) return TMAC_EINVAL;
  // every lane reads the 16 activations of its unit with 16-byte loads
  const int64_t row_elems_16B = (act == TMAC_ACT_I8) ? 16 : 8;
  if (lda % row_elems_16B != 0) return TMAC_EINVAL;
  if (desc->layout != TMAC_LAYOUT_R8U16 || desc->K % 16 != 0) return TMAC_EUNSUPPORTED;
  if (!group_supported(desc)) return TMAC_EUNSUPPORTED;
  if (!tuning_valid(tuning)) return TMAC_EINVAL;
  return static_cast<tmac_status>(launch_perm_gemv(desc, packed_dev, nullptr, A_dev, lda,
                                                    act == TMAC_ACT_I8       ? (int)TMAC_LUT_I16
                                                    : act == TMAC_ACT_F16_TQ ? (int)TMAC_LUT_I8Q
                                                                             : (int)TMAC_LUT_F16,
                                                    N, act_scale_dev, weight_scale, out_dev, (int)out, ldo,
                                                    stream, tuning));
}

extern "C" tmac_status tmac_mpgemv_fused_multi(const tmac_gemv_item* items, int32_t count, tmac_act_t act, int32_t N,
                                               tmac_out_t out, void* stream, const tmac_tuning* tuning) {
  if (!items || N <= 0) return TMAC_EINVAL;
  if (count < 1 || count > TMAC_MULTI_MAX) return TMAC_EUNSUPPORTED;
  if (act != TMAC_ACT_F16 && act != TMAC_ACT_I8 && act != TMAC_ACT_F16_TQ) return TMAC_EINVAL;
  if (out != TMAC_OUT_F32 && out != TMAC_OUT_F16 && out != TMAC_OUT_I32) return TMAC_EINVAL;
  if (!tuning_valid(tuning)) return TMAC_EINVAL;
  const int64_t row_elems_16B = (act == TMAC_ACT_I8) ? 16 : 8;
  for (int i = 0; i < count; ++i) {
    const tmac_gemv_item& it = items[i];
    if (!desc_valid(it.desc) || !it.packed_dev || !it.A_dev || !it.out_dev) return TMAC_EINVAL;
    if (!aligned16(it.packed_dev) || !aligned16(it.A_dev)) return TMAC_EINVAL;
    if (it.ldo < it.desc->M || it.lda < it.desc->K || it.lda % row_elems_16B != 0) return TMAC_EINVAL;
    if (it.desc->layout != TMAC_LAYOUT_R8U16 || it.desc->K % 16 != 0) return TMAC_EUNSUPPORTED;
    if (!group_supported(it.desc)) return TMAC_EUNSUPPORTED;
  }
  return static_cast<tmac_status>(launch_perm_gemv_multi(items, count, (int)act, N, (int)out, stream, tuning));
}

extern "C" tmac_status tmac_blob_check(const tmac_wdesc* desc, const void* header_host) {
  if (!desc_valid(desc) || !header_host) return TMAC_EINVAL;
  tmac_blob_header h;
  memcpy(&h, header_host, sizeof(h));
  const Geometry ge = geometry(desc);
  const float zp = desc->group == 0 ? desc->zero_point : 0.0f;
  const bool same = h.magic == TMAC_MAGIC && h.layout == (uint32_t)desc->layout && h.M == desc->M && h.K == desc->K &&
                    h.bits == desc->bits && h.g == desc->g && h.group == desc->group && h.Mp == ge.Mp &&
                    h.Kp == ge.Kp && h.n_tiles == ge.n_tiles && h.n_chunks == ge.n_chunks &&
                    h.n_qgroups == ge.n_qgroups && h.zero_point == zp && h.idx_off == ge.idx_off &&
                    h.idx_bytes == ge.idx_bytes && h.sz_off == ge.sz_off && h.sz_bytes == ge.sz_bytes &&
                    h.total_bytes == ge.total_bytes;
  return same ? TMAC_OK : TMAC_EINVAL;
}

extern "C" size_t tmac_lut_bytes_max(int32_t N_max, int32_t K, int32_t g, int32_t group, tmac_lut_t lut) {
  // every region grows with N (the padded row count of the table region is N rounded up to 4 or
  // 8, never less than for N - 1), but the register-table kernel's regions exist only up to
  // TMAC_DECODE_MAX_ROWS rows: the largest size is at N_max or at that row count
  if (N_max <= 0) return 0;
  size_t best = 0;
  const int cand[] = {N_max, TMAC_DECODE_MAX_ROWS};
  for (int n : cand) {
    if (n > N_max) continue;
    const size_t b = tmac_lut_bytes(n, K, g, group, lut);
    if (b > best) best = b;
  }
  return best;
}

extern "C" size_t tmac_workspace_bytes_max(const tmac_wdesc* desc, int32_t N_max) {
  if (!desc_valid(desc) || N_max <= 0) return 0;
  size_t best = 0;
  for (int n = 1; n <= N_max; ++n) {  // host arithmetic only; the split of a call changes with N in steps
    const size_t b = tmac_workspace_bytes(desc, n);
    if (b > best) best = b;
  }
  return best;
}

extern "C" size_t tmac_fused_workspace_bytes_max(const tmac_wdesc* desc, int32_t N_max, tmac_act_t act) {
  if (!desc_valid(desc) || N_max <= 0) return 0;
  size_t best = 0;
  for (int n = 1; n <= N_max; ++n) {
    const size_t b = tmac_fused_workspace_bytes(desc, n, act);
    if (b == 0) return 0;
    if (b > best) best = b;
  }
  return best;
}

extern "C" tmac_status tmac_mpgemv_fused(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                                         tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                                         float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                         void* stream) {
  return tmac_mpgemv_fused_ex(desc, packed_dev, A_dev, act, N, lda, act_scale_dev, weight_scale, out_dev, out, ldo,
                              stream, nullptr);
}

// Bytes of the two regions of the workspace of tmac_mpgemm_fused: the split-K workspace of
// tmac_mpgemm, then (only where the tables are not built inside the lookup kernel) a LUT buffer.
static bool fused_regions(const tmac_wdesc* desc, int N, tmac_act_t act, size_t* ws, size_t* lut) {
  if (!desc_valid(desc) || N <= 0 || (act != TMAC_ACT_F16 && act != TMAC_ACT_I8 && act != TMAC_ACT_F16_TQ)) return false;
  const tmac_lut_t lt = (act == TMAC_ACT_I8) ? TMAC_LUT_I16 : TMAC_LUT_F16;
  *ws = (tmac_workspace_bytes(desc, N) + 255) / 256 * 256;
  const bool in_kernel = (desc->layout == TMAC_LAYOUT_R8U16) ? (desc->K % 16 == 0 && group_supported(desc))
                                                             : (group_supported(desc) && rows_builds_tables(desc, N));
  // (int8 tables are quantised inside the register-table kernel only)
  if (act == TMAC_ACT_F16_TQ && !(in_kernel && desc->layout == TMAC_LAYOUT_R8U16)) return false;
  // (the register-table kernel reads its tables from a LUT buffer for at most TMAC_DECODE_MAX_ROWS rows)
  if (!in_kernel && desc->layout == TMAC_LAYOUT_R8U16 && N > TMAC_DECODE_MAX_ROWS) return false;
  *lut = in_kernel ? 0 : tmac_lut_bytes(N, desc->K, desc->g, desc->group, lt);
  return true;
}

extern "C" size_t tmac_fused_workspace_bytes(const tmac_wdesc* desc, int32_t N, tmac_act_t act) {
  size_t ws, lut;
  if (!fused_regions(desc, N, act, &ws, &lut)) return 0;
  return ws + lut;
}

extern "C" tmac_status tmac_mpgemm_fused(const tmac_wdesc* desc, const void* packed_dev, const void* A_dev,
                                         tmac_act_t act, int32_t N, int64_t lda, const float* act_scale_dev,
                                         float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                         void* workspace_dev, size_t workspace_bytes, void* stream) {
  size_t ws, lutb;
  if (!desc_valid(desc) || N <= 0 || (act != TMAC_ACT_F16 && act != TMAC_ACT_I8 && act != TMAC_ACT_F16_TQ))
    return TMAC_EINVAL;
  if (!fused_regions(desc, N, act, &ws, &lutb)) return TMAC_EUNSUPPORTED;
  if (!packed_dev || !A_dev || !out_dev || !workspace_dev) return TMAC_EINVAL;
  if (out != TMAC_OUT_F32 && out != TMAC_OUT_F16 && out != TMAC_OUT_I32) return TMAC_EINVAL;
  if (!aligned16(packed_dev) || !aligned16(A_dev) || !aligned16(workspace_dev)) return TMAC_EINVAL;
  if (ldo < desc->M || lda < desc->K) return TMAC_EINVAL;
  if (lutb == 0 && lda % 8 != 0) return TMAC_EINVAL;  // the kernels read eight activations per load
  if (!group_supported(desc)) return TMAC_EUNSUPPORTED;
  if (workspace_bytes < ws + lutb) return TMAC_ESIZE;
  const tmac_lut_t lt = (act == TMAC_ACT_I8) ? TMAC_LUT_I16 : TMAC_LUT_F16;
  if (lutb == 0) {
    if (desc->layout == TMAC_LAYOUT_R8U16)
      return tmac_mpgemv_fused(desc, packed_dev, A_dev, act, N, lda, act_scale_dev, weight_scale, out_dev, out, ldo,
                               stream);
    return static_cast<tmac_status>(launch_rows_gemm(desc, packed_dev, nullptr, A_dev, lda, (int)lt, N, act_scale_dev,
                                                      weight_scale, out_dev, (int)out, ldo, workspace_dev, ws, stream));
  }
  void* lut_dev = static_cast<char*>(workspace_dev) + ws;
  const tmac_status st = tmac_precompute_lut(A_dev, act, N, desc->K, lda, desc->g, desc->group, lt, lut_dev, lutb, stream);
  if (st != TMAC_OK) return st;
  return tmac_mpgemm(desc, packed_dev, lut_dev, lt, N, act_scale_dev, weight_scale, out_dev, out, ldo, workspace_dev,
                     ws, stream);
}

extern "C" tmac_status tmac_mpgemm(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                                   tmac_lut_t lut, int32_t N, const float* act_scale_dev, float weight_scale,
                                   void* out_dev, tmac_out_t out, int64_t ldo, void* workspace_dev,
                                   size_t workspace_bytes, void* stream) {
  return tmac_mpgemm_ex(desc, packed_dev, lut_dev, lut, N, act_scale_dev, weight_scale, out_dev, out, ldo,
                        workspace_dev, workspace_bytes, stream, nullptr);
}

extern "C" const char* tmac_last_error_detail(void) {
  if (g_last_detail) return g_last_detail;
  return g_last_hip_error == hipSuccess ? "" : hipGetErrorString(g_last_hip_error);
}

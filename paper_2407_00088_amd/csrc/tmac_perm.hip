// Register-table decode kernel (gfx950) for packed layout 2.
//
// The GPU analogue of the paper's in-register TBL/PSHUFB lookup (Section 4 "Efficient table
// look-up"; Section 3.2 "Put lookup table on on-chip memory"): every lane keeps the tables of
// its own 16 activations (four tables) in VGPRs and looks indices up with v_perm_b32, a byte
// permute that selects 4 bytes out of an 8-byte source per instruction.
//
//   * Mirror consolidation (Section 3.3): only entries 0..7 of a table are kept, 8 fp16 values =
//     16 bytes.  A stored 4-bit code is {negate, 3-bit entry}; negation is an XOR of the fp16
//     sign bit, which the packer has placed so that one shift-and-mask aligns it.
//   * fp16 entries as two 8-bit tables (Section 4: "split float16 into two 8-bit LUTs"): the low
//     bytes and the high bytes of the 8 entries form two 8-byte sources; two permutes fetch both
//     halves of 4 entries, two more permutes re-interleave them into fp16 pairs.
//   * Bit-plane shift-accumulate (Eq. 1): v_dot2_f32_f16 multiplies a looked-up pair by the plane
//     weights (2^i, 2^(i+1)) and adds into an fp32 accumulator: two lookups per instruction.
//   * Scale, zero and bias once per (row, lane): the four tables of a lane lie in one
//     quantisation group, so acc starts at (mid - z) * S16 (bias term of Section 4's linear
//     transform, S16 = sum of the lane's 16 activations), collects the half-weighted lookups and
//     is multiplied by the scale once.
//   * The integer path reuses the same code: int16 table entries (|T| <= 508) are exact in fp16,
//     all partial sums are integers below 2^24 and therefore exact in fp32; sums across waves
//     are taken in int32.
//
// Work split: one workgroup = one 8-row tile over the whole K; wave w owns a contiguous run of
// 16-k units (one per lane), so each wave streams one contiguous piece of the tile's packed
// indices with 16-byte loads, all issued before the first lookup.  Cross-lane reduction of the 8
// row sums is a transposing butterfly (v_permlane32_swap, v_permlane16_swap, DPP), cross-wave
// reduction goes through LDS in wave order: the summation order is fixed.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

typedef uint32_t pu32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

struct PermParams {
  const uint32_t* idx;     // [n_tiles][U][4][bits]
  const uint32_t* sz;      // [n_tiles][nq][8] {fp16 scale, fp16 zero}
  const pu32x4* ht;        // fp16 half tables, [N][U][4] 16-byte slots, piece-major per block
  const void* S;           // [N][nq] fp32 / int32 group sums
  const void* S16;         // [N][U]  fp32 / int32 unit sums
  void* out;
  const float* act_scale;
  int64_t ldo;
  int M, N, KG, U, n_tiles, nq;
  int G;           // elements per quantisation group (group-scale mode)
  int nB;          // number of 64-unit blocks the units are split into
  int per_tensor, int_exact, icoef;
  float wscale, zero_point, mid;
  int out_t;
};

__device__ __forceinline__ uint32_t bperm(uint32_t hi, uint32_t lo, uint32_t sel) {
  return __builtin_amdgcn_perm(hi, lo, sel);  // bytes 0..3 of the source = lo, 4..7 = hi
}

__device__ __forceinline__ float dot2(uint32_t pair, uint32_t w, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, pair), __builtin_bit_cast(h2, w), acc, false);
}

template <int CTRL>
__device__ __forceinline__ float dpp_add_t(float v) {
  return v + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), CTRL, 0xf, 0xf, false));
}

// fp16 bit patterns of the plane weights
constexpr uint32_t h2pack(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }
constexpr uint16_t H_0 = 0x0000, H_05 = 0x3800, H_1 = 0x3C00, H_2 = 0x4000, H_4 = 0x4400, H_8 = 0x4800;

template <bool IS_INT, int BITS, int GM>
__global__ __launch_bounds__(1024) void mpgemv_perm_kernel(const PermParams p) {
  __shared__ float red[16 * 8];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int NW = blockDim.x >> 6;
  const int tile = blockIdx.x, n = blockIdx.y;

  // plane weights: halved in group-scale mode, where acc = bias + 1/2 * sum_i 2^i L_i
  constexpr uint32_t W01 = GM ? h2pack(H_05, H_1) : h2pack(H_1, H_2);
  constexpr uint32_t W23 = GM ? h2pack(H_2, H_4) : h2pack(H_4, H_8);
  constexpr uint16_t WS0 = GM ? H_05 : H_1;  // single plane 0
  constexpr uint16_t WS2 = GM ? H_2 : H_4;   // single plane 2

  float tot[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) tot[r] = 0.f;

  for (int blk = wave; blk < p.nB; blk += NW) {
    const int u0 = (int)(((int64_t)blk * p.U) / p.nB), u1 = (int)(((int64_t)(blk + 1) * p.U) / p.nB);
    const int u = u0 + lane;
    const bool valid = u < u1;
    const int uc = valid ? u : u0;  // lanes past the end of the block re-read unit u0 with zero tables

    // 1. packed indices of this lane: 16*BITS bytes, issued first
    uint32_t w[4 * BITS];
    {
      // the block's records are stored piece-major: 16-byte piece i of lane l sits at slot
      // i*nu + l, so every load instruction of the wavefront reads one contiguous run
      const int nu = u1 - u0;
      const pu32x4* src = reinterpret_cast<const pu32x4*>(p.idx + ((size_t)tile * p.U + u0) * (4 * BITS)) +
                          (uc - u0);
#pragma unroll
      for (int i = 0; i < BITS; ++i) {
        const pu32x4 v = __builtin_nontemporal_load(src + (size_t)i * nu);
        w[4 * i + 0] = v.x; w[4 * i + 1] = v.y; w[4 * i + 2] = v.z; w[4 * i + 3] = v.w;
      }
    }

    // 2. scale and zero of the lane's quantisation group for the 8 rows
    uint32_t szr[8];
    if constexpr (GM == 1) {
      int gq = (16 * uc) / p.G;
      gq = gq < p.nq ? gq : p.nq - 1;  // units in the K padding: tables and S16 are zero there
      const pu32x4* szp = reinterpret_cast<const pu32x4*>(p.sz + ((size_t)tile * p.nq + gq) * 8);
      const pu32x4 a = szp[0], b = szp[1];
      szr[0] = a.x; szr[1] = a.y; szr[2] = a.z; szr[3] = a.w;
      szr[4] = b.x; szr[5] = b.y; szr[6] = b.z; szr[7] = b.w;
    }

    // 3. the lane's four tables: stored half (entries 0..7), split into low-byte and high-byte sources
    uint32_t lo0[4], lo1[4], hi0[4], hi1[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      // fp16 half table tb of the block's l-th unit: 16-byte slot tb*nu + l (contiguous over lanes)
      pu32x4 d = p.ht[((size_t)n * p.U + u0) * 4 + (size_t)t * (u1 - u0) + (uc - u0)];
      if (!valid) d = pu32x4{0, 0, 0, 0};
      const uint32_t e[4] = {d.x, d.y, d.z, d.w};
      lo0[t] = bperm(e[1], e[0], 0x06040200u);
      hi0[t] = bperm(e[1], e[0], 0x07050301u);
      lo1[t] = bperm(e[3], e[2], 0x06040200u);
      hi1[t] = bperm(e[3], e[2], 0x07050301u);
    }
    float Sl = 0.f;
    if (valid) {
      if constexpr (IS_INT) Sl = (float)static_cast<const int*>(p.S16)[(size_t)n * p.U + u];
      else Sl = static_cast<const float*>(p.S16)[(size_t)n * p.U + u];
    }

    // 4. accumulators start at the bias term (group-scale mode)
    float acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      if constexpr (GM == 1) {
        const float z = __half2float(__ushort_as_half((uint16_t)(szr[r] >> 16)));
        acc[r] = fmaf(-z, Sl, p.mid * Sl);
      } else {
        acc[r] = 0.f;
      }
    }

    // 5. lookups
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      // four lookups of table t: selector bytes `sel` (0..7 each), sign bits `sgn` at bit 7 of each byte
      auto look = [&](uint32_t sel, uint32_t sgn, uint32_t& p01, uint32_t& p23) {
        const uint32_t lo = bperm(lo1[t], lo0[t], sel);
        const uint32_t hi = bperm(hi1[t], hi0[t], sel) ^ sgn;
        p01 = bperm(hi, lo, 0x05010400u);  // fp16 pair of bytes 0 and 1
        p23 = bperm(hi, lo, 0x07030602u);  // fp16 pair of bytes 2 and 3
      };
      auto quad = [&](uint32_t x, int r_lo, int r_hi) {  // 4 planes of row r_lo (low nibbles), r_hi (high)
        uint32_t a, b;
        look(x & 0x07070707u, (x << 4) & 0x80808080u, a, b);
        acc[r_lo] = dot2(a, W01, acc[r_lo]);
        acc[r_lo] = dot2(b, W23, acc[r_lo]);
        look((x >> 4) & 0x07070707u, x & 0x80808080u, a, b);
        acc[r_hi] = dot2(a, W01, acc[r_hi]);
        acc[r_hi] = dot2(b, W23, acc[r_hi]);
      };
      auto pair = [&](uint32_t x, int r0) {  // planes 0,1 of rows r0, r0+1 (low) and r0+2, r0+3 (high)
        uint32_t a, b;
        look(x & 0x07070707u, (x << 4) & 0x80808080u, a, b);
        acc[r0] = dot2(a, W01, acc[r0]);
        acc[r0 + 1] = dot2(b, W01, acc[r0 + 1]);
        look((x >> 4) & 0x07070707u, x & 0x80808080u, a, b);
        acc[r0 + 2] = dot2(a, W01, acc[r0 + 2]);
        acc[r0 + 3] = dot2(b, W01, acc[r0 + 3]);
      };
      auto single = [&](uint32_t x, uint16_t wgt) {  // one plane of rows 0..3 (low) and 4..7 (high)
        const uint32_t wl = h2pack(wgt, H_0), wh = h2pack(H_0, wgt);
        uint32_t a, b;
        look(x & 0x07070707u, (x << 4) & 0x80808080u, a, b);
        acc[0] = dot2(a, wl, acc[0]);
        acc[1] = dot2(a, wh, acc[1]);
        acc[2] = dot2(b, wl, acc[2]);
        acc[3] = dot2(b, wh, acc[3]);
        look((x >> 4) & 0x07070707u, x & 0x80808080u, a, b);
        acc[4] = dot2(a, wl, acc[4]);
        acc[5] = dot2(a, wh, acc[5]);
        acc[6] = dot2(b, wl, acc[6]);
        acc[7] = dot2(b, wh, acc[7]);
      };
      const uint32_t* wt = &w[t * BITS];
      if constexpr (BITS == 4) {
#pragma unroll
        for (int d = 0; d < 4; ++d) quad(wt[d], 2 * d, 2 * d + 1);
      } else if constexpr (BITS == 2) {
        pair(wt[0], 0);
        pair(wt[1], 4);
      } else if constexpr (BITS == 1) {
        single(wt[0], WS0);
      } else {
        pair(wt[0], 0);
        pair(wt[1], 4);
        single(wt[2], WS2);
      }
    }

    // 6. scale once per (row, lane)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      if constexpr (GM == 1) {
        const float s = __half2float(__ushort_as_half((uint16_t)(szr[r] & 0xffffu)));
        tot[r] = fmaf(s, acc[r], tot[r]);
      } else {
        tot[r] += acc[r];
      }
    }
  }

  // 7. transposing butterfly over the 64 lanes: 8 values per lane -> 1 value per lane, the row it
  // belongs to is tracked by running the same exchanges on the row numbers
  float v4[4], v2[2];
  uint32_t g4[4], g2[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const auto rv = __builtin_amdgcn_permlane32_swap(__float_as_uint(tot[i]), __float_as_uint(tot[i + 4]), false, false);
    v4[i] = __uint_as_float(rv[0]) + __uint_as_float(rv[1]);
    const auto rg = __builtin_amdgcn_permlane32_swap((uint32_t)i, (uint32_t)(i + 4), false, false);
    g4[i] = rg[0];
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const auto rv = __builtin_amdgcn_permlane16_swap(__float_as_uint(v4[i]), __float_as_uint(v4[i + 2]), false, false);
    v2[i] = __uint_as_float(rv[0]) + __uint_as_float(rv[1]);
    const auto rg = __builtin_amdgcn_permlane16_swap(g4[i], g4[i + 2], false, false);
    g2[i] = rg[0];
  }
  const bool up = (lane & 8) != 0;
  const float keep = up ? v2[1] : v2[0], send = up ? v2[0] : v2[1];
  const uint32_t row = up ? g2[1] : g2[0];
  float v = keep + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(send), 0x128, 0xf, 0xf, false));  // row_ror:8
  v = dpp_add_t<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add_t<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add_t<0x141>(v);  // row_half_mirror
  constexpr bool RAW_INT = (GM == 0 && IS_INT);
  if ((lane & 7) == 0) {
    if constexpr (RAW_INT) red[wave * 8 + row] = __int_as_float((int)v);  // exact: integer < 2^24
    else red[wave * 8 + row] = v;
  }
  __syncthreads();

  // 8. sum the waves in wave order, finish and store
  if (threadIdx.x < 8) {
    const int r = threadIdx.x, m = tile * 8 + r;
    float sf = 0.f;
    int si = 0;
    for (int wv = 0; wv < NW; ++wv) {
      const float x = red[wv * 8 + r];
      if constexpr (RAW_INT) si += __float_as_int(x);
      else sf += x;
    }
    if (m < p.M) {
      const float as = p.act_scale ? p.act_scale[n] : 1.0f;
      float res;
      int ires = 0;
      if constexpr (GM == 1) {
        res = sf * as;
      } else {
        float s, z;
        if (p.per_tensor) {
          s = p.wscale;
          z = p.zero_point;
        } else {
          const uint32_t szv = p.sz[(size_t)tile * 8 + r];
          s = __half2float(__ushort_as_half((uint16_t)(szv & 0xffffu)));
          z = __half2float(__ushort_as_half((uint16_t)(szv >> 16)));
        }
        if constexpr (IS_INT) {
          const int St = static_cast<const int*>(p.S)[n];
          if (p.int_exact) {
            ires = (si + p.icoef * St) >> 1;  // numerator is always even
            res = ((float)ires * as) * s;     // two roundings, left to right
          } else {
            res = ((0.5f * (float)si + (p.mid - z) * (float)St) * as) * s;
          }
        } else {
          const float St = static_cast<const float*>(p.S)[n];
          res = (s * (0.5f * sf + (p.mid - z) * St)) * as;
        }
      }
      const size_t o = (size_t)n * p.ldo + m;
      if (p.out_t == TMAC_OUT_F32) static_cast<float*>(p.out)[o] = res;
      else if (p.out_t == TMAC_OUT_F16) static_cast<__half*>(p.out)[o] = __float2half_rn(res);
      else static_cast<int*>(p.out)[o] = ires;
    }
  }
}

template <bool IS_INT, int BITS, int GM>
static hipError_t launch_one(const PermParams& p, int NW, hipStream_t st) {
  PermParams local = p;
  void* args[] = {&local};
  return hipLaunchKernel(reinterpret_cast<const void*>(mpgemv_perm_kernel<IS_INT, BITS, GM>),
                         dim3(p.n_tiles, p.N), dim3(NW * 64), args, 0, st);
}

template <bool IS_INT, int BITS>
static hipError_t launch_gm(const PermParams& p, int gm, int NW, hipStream_t st) {
  return gm ? launch_one<IS_INT, BITS, 1>(p, NW, st) : launch_one<IS_INT, BITS, 0>(p, NW, st);
}

template <bool IS_INT>
static hipError_t launch_bits(const PermParams& p, int bits, int gm, int NW, hipStream_t st) {
  switch (bits) {
    case 1: return launch_gm<IS_INT, 1>(p, gm, NW, st);
    case 2: return launch_gm<IS_INT, 2>(p, gm, NW, st);
    case 3: return launch_gm<IS_INT, 3>(p, gm, NW, st);
    case 4: return launch_gm<IS_INT, 4>(p, gm, NW, st);
  }
  return hipErrorInvalidValue;
}

int launch_perm_gemv(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, int lut_is_int,
                     int N, const float* act_scale_dev, float weight_scale, void* out_dev, int out_t,
                     int64_t ldo, void* stream) {
  const Geometry ge = geometry(desc);
  LutGeom lg;
  if (!lut_geom(N, desc->K, desc->g, desc->group, &lg)) return TMAC_EINVAL;
  if (N > 65535) return TMAC_EUNSUPPORTED;
  const bool one_group = (desc->group == 0 || desc->group == desc->K);

  PermParams p;
  const char* blob = static_cast<const char*>(packed_dev);
  p.idx = reinterpret_cast<const uint32_t*>(blob + ge.idx_off);
  p.sz = reinterpret_cast<const uint32_t*>(blob + ge.sz_off);
  p.ht = reinterpret_cast<const pu32x4*>(static_cast<const char*>(lut_dev) + lg.ht_off);
  p.S = static_cast<const char*>(lut_dev) + lg.s_off;
  p.S16 = static_cast<const char*>(lut_dev) + lg.s16_off;
  p.out = out_dev;
  p.act_scale = act_scale_dev;
  p.ldo = ldo;
  p.M = desc->M; p.N = N; p.KG = lg.KG; p.U = lg.U; p.n_tiles = ge.n_tiles; p.nq = lg.nq;
  p.G = lg.Geff;
  p.nB = (lg.U + 63) / 64;
  p.per_tensor = (desc->group == 0);
  p.wscale = weight_scale;
  p.mid = 0.5f * (float)((1 << desc->bits) - 1);
  p.zero_point = p.per_tensor ? desc->zero_point : 0.f;
  p.int_exact = 0;
  p.icoef = 0;
  p.out_t = out_t;
  if (p.per_tensor && lut_is_int) {
    const float z = desc->zero_point;
    if (z == rintf(z) && fabsf(z) < 64.f) {
      p.int_exact = 1;
      p.icoef = ((1 << desc->bits) - 1) - 2 * (int)z;
    }
  }
  if (out_t == TMAC_OUT_I32 && !p.int_exact) return TMAC_EINVAL;
  const int NW = p.nB < 16 ? p.nB : 16;
  if (lut_is_int) {
    // integer sums are carried in fp32 inside a wave: a wave's total must stay below 2^24
    const int passes = (p.nB + NW - 1) / NW;
    if ((double)508.0 * ((1 << desc->bits) - 1) * 256.0 * passes >= 16777216.0) return TMAC_EUNSUPPORTED;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int gm = one_group ? 0 : 1;
  const hipError_t e = lut_is_int ? launch_bits<true>(p, desc->bits, gm, NW, st)
                                  : launch_bits<false>(p, desc->bits, gm, NW, st);
  if (e != hipSuccess) {
    note_hip_error((int)e);
    return TMAC_EHIP;
  }
  return TMAC_OK;
}

}  // namespace tmac

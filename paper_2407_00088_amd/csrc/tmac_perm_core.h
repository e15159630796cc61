// Device helpers of the register-table decode kernels (gfx950): byte-permute lookups, the table
// build inside a lane, and the wavefront reductions.  Shared by the one-block-per-wave kernel
// (tmac_perm.hip) and the streaming kernel (tmac_stream.hip) so that both take exactly the same
// arithmetic in the same order.
#ifndef TMAC_PERM_CORE_H_
#define TMAC_PERM_CORE_H_

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

typedef uint32_t pu32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bperm(uint32_t hi, uint32_t lo, uint32_t sel) {
  return __builtin_amdgcn_perm(hi, lo, sel);  // bytes 0..3 of the source = lo, 4..7 = hi
}

__device__ __forceinline__ float dot2(uint32_t pair, uint32_t w, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, pair), __builtin_bit_cast(h2, w), acc, false);
}

// The same dot product for a sum that starts at zero: the three-operand form with the constant 0 as
// addend (the compiler only picks the accumulate-in-place form, which needs a zeroed register first).
// The plane weights come in a scalar register: this encoding takes no literal.
// The result may only be used as the addend of another dot product: the compiler cannot see inside
// an assembly statement, so it does not keep the three wait states this chip wants between a dot
// product and an instruction of another kind that reads its result (a dot product that takes the
// result as its addend may follow at once).
__device__ __forceinline__ float dot2_from_zero(uint32_t pair, uint32_t w_sgpr) {
  float r;
  asm("v_dot2_f32_f16 %0, %1, %2, 0" : "=v"(r) : "v"(pair), "s"(w_sgpr));
  return r;
}

template <int CTRL>
__device__ __forceinline__ float dpp_add_t(float v) {
  return v + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), CTRL, 0xf, 0xf, false));
}

// Sum 8 per-lane values over lane bits 5, 4, 3 with a transposing butterfly; afterwards every
// lane holds row (lane >> 3), summed over the eight lanes with the same (lane & 7).
//   v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of the second,
//   v_permlane16_swap does the same for the odd/even 16-lane rows; after each exchange the two
//   operands hold, in every lane, two partial sums of the same row.
__device__ __forceinline__ float reduce_hi3(const float* t, int lane) {
  float v4[4], v2[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const auto rv = __builtin_amdgcn_permlane32_swap(__float_as_uint(t[i]), __float_as_uint(t[i + 4]), false, false);
    v4[i] = __uint_as_float(rv[0]) + __uint_as_float(rv[1]);  // row i (lanes < 32) or i + 4
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const auto rv = __builtin_amdgcn_permlane16_swap(__float_as_uint(v4[i]), __float_as_uint(v4[i + 2]), false, false);
    v2[i] = __uint_as_float(rv[0]) + __uint_as_float(rv[1]);  // row i + 2 * bit4(lane) + 4 * bit5(lane)
  }
  const bool up = (lane & 8) != 0;
  const float keep = up ? v2[1] : v2[0], send = up ? v2[0] : v2[1];
  return keep + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(send), 0x128, 0xf, 0xf, false));  // row_ror:8
}

// Sum over lane bits 0, 1, 2 (all lanes of a group of 8 end with the total).
__device__ __forceinline__ float reduce_lo3(float v) {
  v = dpp_add_t<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add_t<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add_t<0x141>(v);  // row_half_mirror
  return v;
}

// fp16 bit patterns of the plane weights
constexpr uint32_t h2pack(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }
constexpr uint16_t H_0 = 0x0000, H_05 = 0x3800, H_1 = 0x3C00, H_2 = 0x4000, H_4 = 0x4400, H_8 = 0x4800;

// One weight matrix of a launch.  A launch serves up to PERM_MAX_MATS matrices (one each for the
// single-matrix entry points): the workgroups of matrix i are blockIdx.x in [wg_end of matrix i - 1,
// wg_end of matrix i).
struct PermMat {
  const pu32x4* idx;       // packed indices, 16-byte slots (see layout 2 in tmac.h)
  const pu32x4* sz;        // [n_tiles][nq] x 32 bytes: {fp16 scale, fp16 zero} of the 8 rows
  const pu32x4* ht;        // split fp16 half tables, [N][U][4] 16-byte slots, piece-major per block
  const void* S;           // [N][nq] fp32 / int32 group sums
  const void* S16;         // [N][U]  fp32 / int32 unit sums
  const void* S128;        // [N][U/8] fp32 / int32 sums of every 128 consecutive activations
  const float* usc;        // int8 tables: [N][U] scale of the lane's four tables
  const void* A;           // fused mode: activations [N][lda], fp16 or int8 (no LUT buffer is read)
  int64_t lda;
  void* out;
  const float* act_scale;
  int64_t ldo;
  int M, K, U, n_tiles, nq;
  uint32_t q_magic;  // ceil(2^32 / d), d = units (mode 1) or chunks (mode 2) per quantisation group; 0 if d = 1
  BlockSplit bs;     // split of the U/8 chunks into blocks of at most 8
  uint32_t ht_zero;  // slot index of the all-zero table
  int per_tensor, int_exact, icoef;
  float wscale, zero_point;
  int gsz;           // wavefronts that share one group of row tiles: min(blocks, 16); they split K
  int gpw;           // groups of row tiles per workgroup: (waves per workgroup) / gsz
  uint32_t ginv;     // ceil(256 / gsz): wave / gsz == (wave * ginv) >> 8 for wave < 16
};
constexpr int PERM_MAX_MATS = TMAC_MULTI_MAX;
constexpr int PERM_GROUP_WAVES = 8;    // default cap on the waves that split the K of one group of row tiles
                                       // (workgroups of eight waves finish closer together than larger ones)
constexpr int PERM_WG_WAVES_MAX = 16;  // most waves per workgroup

// NM = 1: the single-matrix entry points; NM = PERM_MAX_MATS: several matrices in one launch.
template <int NM>
struct PermParamsT {
  int wg_end[NM];    // first workgroup after matrix i's; INT_MAX for unused slots
  int N;
  float mid;
  int out_t;
  int pad;
  PermMat m[NM];
};
using PermParams = PermParamsT<PERM_MAX_MATS>;  // what the host code fills

// Fills the description of one matrix (everything but gpw, which the launch shape decides) and checks
// what the kernels assume; defined in tmac_perm.hip.  group_waves: most waves that split the K of one
// group of row tiles (0 = default).  lut_t, out_t: tmac_lut_t / tmac_out_t values; *gm_out: how the
// scales are grouped (the GM template parameter of the kernels).  Returns a tmac_status value.
int perm_fill(PermMat& p, const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
              int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale, void* out_dev,
              int out_t, int64_t ldo, int group_waves, int* gm_out);

// The four tables of a lane's 16-k unit as byte-permute sources (Section 3.3 mirror half, Section 4
// "fp16 as two 8-bit tables"): for table t, lo0/lo1 hold the low bytes of entries 0..3 / 4..7 and
// hi0/hi1 the high bytes.
struct LaneTables {
  uint32_t lo0[4], lo1[4], hi0[4], hi1[4];
};

// Where lane `lane` of a wavefront works inside block `blk` of a row (see BlockSplit): the eight
// lanes with equal (lane & 7) cover one 128-k chunk.
struct LaneBlock {
  uint32_t u0, nu;   // first unit and number of units of the block
  uint32_t l;        // slot of the lane's unit inside the block (0 for lanes without a unit)
  uint32_t c, u;     // 128-k chunk and 16-k unit of the lane
  bool valid;        // the lane owns a unit
};
__device__ __forceinline__ LaneBlock lane_block(const BlockSplit& bs, int blk, int lane) {
  const uint32_t jl = (uint32_t)lane & 7u, pos = (uint32_t)lane >> 3;
  const uint32_t c0 = (uint32_t)block_start(bs, blk);
  const uint32_t ng = (uint32_t)(blk < bs.r ? bs.q + 1 : bs.q);
  LaneBlock b;
  b.u0 = 8u * c0;
  b.nu = 8u * ng;
  b.valid = jl < ng;
  b.l = b.valid ? pos * ng + jl : 0u;
  b.c = b.valid ? c0 + jl : c0;
  b.u = 8u * b.c + pos;
  return b;
}

// A wave-uniform global pointer pinned whole in scalar registers, so that a load from it plus a
// lane's 32-bit byte offset takes the base from scalar registers (no 64-bit address arithmetic in
// the vector ALU; left alone the compiler folds the lane's offset into the pointer first).
typedef const __attribute__((address_space(1))) char* gbase_t;
__device__ __forceinline__ gbase_t scalar_base(const void* uniform_ptr) {
  gbase_t b = (gbase_t)uniform_ptr;
  asm("" : "+s"(b));
  return b;
}
template <typename T>
__device__ __forceinline__ T load_at(gbase_t base, uint32_t byte_off) {
  return *reinterpret_cast<const __attribute__((address_space(1))) T*>(base + byte_off);
}

// The lane's 16 activations, raw (zero past the end of K and for lanes without a unit): fp16 two per
// dword in araw[0..7]; int8 four per dword (one table each) in araw[0..3].
template <bool IS_INT>
__device__ __forceinline__ void lane_load_act(const void* A, int64_t lda, int n, int K, const LaneBlock& b,
                                              uint32_t (&araw)[8]) {
  const bool have = b.valid && 16u * b.u < (uint32_t)K;
  pu32x4 v0 = {0u, 0u, 0u, 0u}, v1 = {0u, 0u, 0u, 0u};
  if constexpr (IS_INT) {
    const gbase_t row = scalar_base(static_cast<const int8_t*>(A) + (size_t)n * lda);
    if (have) v0 = load_at<pu32x4>(row, 16u * b.u);
  } else {
    const gbase_t row = scalar_base(static_cast<const __half*>(A) + (size_t)n * lda);
    if (have) {
      v0 = load_at<pu32x4>(row, 32u * b.u);
      v1 = load_at<pu32x4>(row, 32u * b.u + 16u);
    }
  }
  araw[0] = v0.x; araw[1] = v0.y; araw[2] = v0.z; araw[3] = v0.w;
  araw[4] = v1.x; araw[5] = v1.y; araw[6] = v1.z; araw[7] = v1.w;
}

// Sum of the lane's 16 activations, in the order of the precompute kernel's tree (exact for ints:
// |sum| <= 16 * 128).
template <bool IS_INT>
__device__ __forceinline__ float lane_act_sum(const uint32_t (&araw)[8]) {
  if constexpr (IS_INT) {
    int s16 = 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) s16 = __builtin_amdgcn_sdot4((int)araw[t], 0x01010101, s16, false);
    return (float)s16;
  } else {
    float t4[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) t4[t] = sum4_f16(araw[2 * t], araw[2 * t + 1]);
    return (t4[0] + t4[1]) + (t4[2] + t4[3]);
  }
}

// Sum over the eight lanes of a 128-k chunk (lane bits 3, 4, 5), pairing units as the precompute kernel does.
__device__ __forceinline__ float chunk_sum(float Sl) {
  Sl += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(Sl), 0x128, 0xf, 0xf, false));  // row_ror:8
  Sl += __shfl_xor(Sl, 16);
  Sl += __shfl_xor(Sl, 32);
  return Sl;
}

// Algorithm 1 Precompute inside a lane: the four tables of its unit (mirror half: entries 0..7, the
// fourth activation subtracted), as low-byte and high-byte permute sources.
template <bool IS_INT>
__device__ __forceinline__ void lane_build_tables(const uint32_t (&araw)[8], LaneTables& T) {
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    uint32_t pk[4];
    if constexpr (IS_INT) {
      // int8 activations are exact in fp16 and so is every sum of four of them (|T| <= 508): the
      // fp16 additions of the fp16 path give the integer table
      // (conversion: byte b + 128 under the high byte 0x64 is the fp16 number 1024 + 128 + b)
      const uint32_t biased = araw[t] ^ 0x80808080u;
      const h2 off = {(_Float16)1152.0f, (_Float16)1152.0f};
      const h2 x01 = __builtin_bit_cast(h2, bperm(0x64646464u, biased, 0x04010400u)) - off;
      const h2 x23 = __builtin_bit_cast(h2, bperm(0x64646464u, biased, 0x04030402u)) - off;
      half_table_f16(__builtin_bit_cast(uint32_t, x01), __builtin_bit_cast(uint32_t, x23), pk);
    } else {
      half_table_f16(araw[2 * t], araw[2 * t + 1], pk);  // fp16 additions, as every table builder
    }
    T.lo0[t] = bperm(pk[1], pk[0], 0x06040200u);
    T.lo1[t] = bperm(pk[3], pk[2], 0x06040200u);
    T.hi0[t] = bperm(pk[1], pk[0], 0x07050301u);
    T.hi1[t] = bperm(pk[3], pk[2], 0x07050301u);
  }
}

// Table quantisation inside a lane (Section 3.3): the four tables of the unit as int8 entries
// rint(T * 127 / amax) with amax = the largest |entry| of the unit (the sum of its |activations| per
// table, maximised over the four tables), and the scale amax / 127.  Entries are formed in fp32 from
// the fp16 activations (dot products with +-1), so they equal the exact sums whenever those fit
// fp32.  lo0[t] / lo1[t]: entries 0..3 / 4..7 of table t, one byte each.
//
// The dot products are written as assembly in the three-operand form (the accumulate-in-place form
// the compiler picks would copy the addend first).  The compiler does not know what an assembly
// statement holds, so it cannot keep the distance this chip wants between a dot product and an
// instruction of another kind that reads its result (three wait states; a dot product that takes it
// as its addend may follow at once): every statement below ends with s_nop 2.
__device__ __forceinline__ void lane_build_tables_q8(const uint32_t (&araw)[8], LaneTables& T, float& uscale) {
  constexpr uint16_t H_M1 = 0xBC00;
  constexpr uint32_t PP = h2pack(H_1, H_1), PM = h2pack(H_1, H_M1), MP = h2pack(H_M1, H_1), MM = h2pack(H_M1, H_M1);
  // the largest |entry| of a table is the sum of its |activations| (one table at a time: few
  // registers are live next to the index registers, whose loads are already in flight)
  float amax = 0.f;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    float sa;
    asm("v_dot2_f32_f16 %0, %1, %3, 0\n\t"
        "v_dot2_f32_f16 %0, %2, %3, %0\n\t"
        "s_nop 2"
        : "=&v"(sa)
        : "v"(araw[2 * t] & 0x7fff7fffu), "v"(araw[2 * t + 1] & 0x7fff7fffu), "s"(PP));
    amax = fmaxf(amax, sa);
  }
  // 127 / amax: the hardware reciprocal refined by one Newton step (the quotient then is within an
  // ulp of the exact one: an entry changes only if its exact quotient is that close to a half-integer)
  float inv = 0.f;
  if (amax > 0.f) {
    const float r0 = __builtin_amdgcn_rcpf(amax);
    const float r1 = fmaf(fmaf(-amax, r0, 1.0f), r0, r0);
    inv = 127.0f * r1;
  }
  uscale = amax * (1.0f / 127.0f);
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      // entry p = +-a0 +-a1 +-a2 - a3 (bit j of p set = +a_j); h = bit 2: first -a2 - a3 (h = 0) or
      // a2 - a3 (h = 1), then the four sign pairs of a0, a1 on top of it
      float e0, e1, e2, e3, base;
      asm("v_dot2_f32_f16 %4, %6, %7, 0\n\t"
          "v_dot2_f32_f16 %0, %5, %8, %4\n\t"
          "v_dot2_f32_f16 %1, %5, %9, %4\n\t"
          "v_dot2_f32_f16 %2, %5, %10, %4\n\t"
          "v_dot2_f32_f16 %3, %5, %11, %4\n\t"
          "s_nop 2"
          : "=&v"(e0), "=&v"(e1), "=&v"(e2), "=&v"(e3), "=&v"(base)
          : "v"(araw[2 * t]), "v"(araw[2 * t + 1]), "s"(h ? PM : MM), "s"(MM), "s"(PM), "s"(MP), "s"(PP));
      // adding 1.5 * 2^23 rounds e * inv to the nearest integer (ties to even) and leaves it, in two's
      // complement, in the low mantissa bits: byte 0 of the sum is the int8 entry (|e * inv| <= 127
      // up to an ulp: the entries are bounded by amax)
      const uint32_t r0 = __float_as_uint(fmaf(e0, inv, 12582912.0f)), r1 = __float_as_uint(fmaf(e1, inv, 12582912.0f));
      const uint32_t r2 = __float_as_uint(fmaf(e2, inv, 12582912.0f)), r3 = __float_as_uint(fmaf(e3, inv, 12582912.0f));
      const uint32_t word = bperm(bperm(r3, r2, 0x0c0c0400u), bperm(r1, r0, 0x0c0c0400u), 0x05040100u);
      if (h == 0) T.lo0[t] = word;
      else T.lo1[t] = word;
    }
  }
}

// The lookups of one row tile and one unit: w = the lane's 4 * BITS index dwords (table t in dwords
// t * BITS ..), acc[r] += sum over the unit's tables and planes of 2^plane (halved when HALF) times the
// looked-up entry, for the eight rows r of the tile (Eq. 1).
// ZERO: the sums start at zero (what acc holds on entry is ignored).  FENCE: see the end of the body.
template <int BITS, bool HALF, bool ZERO = false, bool FENCE = false>
__device__ __forceinline__ void lane_lookups(uint32_t* w, const LaneTables& T, float (&acc)[8]) {
  // plane weights: halved in the group-scale modes, where acc = bias + 1/2 * sum_i 2^i L_i
  constexpr uint32_t W01 = HALF ? h2pack(H_05, H_1) : h2pack(H_1, H_2);
  constexpr uint32_t W23 = HALF ? h2pack(H_2, H_4) : h2pack(H_4, H_8);
  constexpr uint16_t WS0 = HALF ? H_05 : H_1;  // single plane 0
  constexpr uint16_t WS2 = HALF ? H_2 : H_4;   // single plane 2
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    // four lookups of table t: selector bytes `sel` (0..7 each), sign bits `sgn` at bit 7 of each byte
    auto look = [&](uint32_t sel, uint32_t sgn, uint32_t& p01, uint32_t& p23) {
      const uint32_t lo = bperm(T.lo1[t], T.lo0[t], sel);
      const uint32_t hi = bperm(T.hi1[t], T.hi0[t], sel) ^ sgn;
      p01 = bperm(hi, lo, 0x05010400u);  // fp16 pair of bytes 0 and 1
      p23 = bperm(hi, lo, 0x07030602u);  // fp16 pair of bytes 2 and 3
    };
    // the "high" rows of a dword: rotated by four bits their entries sit in bits 0..2 and their
    // negate bits (stored in bit 3 of the following byte) in bit 7 of each byte
    auto hi_set = [](uint32_t x) { return __builtin_amdgcn_alignbit(x, x, 4); };
    auto quad = [&](uint32_t x, float& a_lo, float& a_hi) {  // 4 planes of one row (low nibbles), one (high)
      uint32_t a, b;
      look(x & 0x07070707u, x & 0x80808080u, a, b);
      a_lo = (ZERO && t == 0) ? dot2_from_zero(a, W01) : dot2(a, W01, a_lo);
      a_lo = dot2(b, W23, a_lo);
      look(hi_set(x) & 0x07070707u, hi_set(x) & 0x80808080u, a, b);
      a_hi = (ZERO && t == 0) ? dot2_from_zero(a, W01) : dot2(a, W01, a_hi);
      a_hi = dot2(b, W23, a_hi);
    };
    // first: these sums start here (the first table of a call whose sums start at zero)
    auto acc2 = [&](uint32_t pr, uint32_t wgt, float c, bool first) {
      return first ? dot2_from_zero(pr, wgt) : dot2(pr, wgt, c);
    };
    auto pair = [&](uint32_t x, float* a4) {  // planes 0,1 of rows 0,1 (low) and 2,3 (high) of a4
      constexpr bool F = ZERO;
      const bool first = F && t == 0;
      uint32_t a, b;
      look(x & 0x07070707u, x & 0x80808080u, a, b);
      a4[0] = acc2(a, W01, a4[0], first);
      a4[1] = acc2(b, W01, a4[1], first);
      look(hi_set(x) & 0x07070707u, hi_set(x) & 0x80808080u, a, b);
      a4[2] = acc2(a, W01, a4[2], first);
      a4[3] = acc2(b, W01, a4[3], first);
    };
    auto single = [&](uint32_t x, uint16_t wgt, float* a8, bool may_be_first) {  // one plane of rows 0..3 (low), 4..7 (high)
      const uint32_t wl = h2pack(wgt, H_0), wh = h2pack(H_0, wgt);
      const bool first = ZERO && may_be_first && t == 0;
      uint32_t a, b;
      look(x & 0x07070707u, x & 0x80808080u, a, b);
      a8[0] = acc2(a, wl, a8[0], first);
      a8[1] = acc2(a, wh, a8[1], first);
      a8[2] = acc2(b, wl, a8[2], first);
      a8[3] = acc2(b, wh, a8[3], first);
      look(hi_set(x) & 0x07070707u, hi_set(x) & 0x80808080u, a, b);
      a8[4] = acc2(a, wl, a8[4], first);
      a8[5] = acc2(a, wh, a8[5], first);
      a8[6] = acc2(b, wl, a8[6], first);
      a8[7] = acc2(b, wh, a8[7], first);
    };
    const uint32_t* wt = &w[t * BITS];
    if constexpr (BITS == 4) {
#pragma unroll
      for (int d = 0; d < 4; ++d) quad(wt[d], acc[2 * d], acc[2 * d + 1]);
    } else if constexpr (BITS == 2) {
      pair(wt[0], acc);
      pair(wt[1], acc + 4);
    } else if constexpr (BITS == 1) {
      single(wt[0], WS0, acc, true);
    } else {
      pair(wt[0], acc);
      pair(wt[1], acc + 4);
      single(wt[2], WS2, acc, false);
    }
    // Table by table, in the order the index pieces were requested: the lookups of table t run while
    // the pieces of the later tables are still in flight, and few registers are live at a time.
    // FENCE: a scheduling barrier between the tables.  With two row tiles per wave it takes the
    // kernel from 77 to 69 vector registers and 1.5 % off the three-matrix step; with one row tile
    // the same barrier costs 4.6 %, and the order is made a data dependency instead: an empty asm
    // statement that "rewrites" the sums of table t together with the index dwords of table t + 1.
    if constexpr (FENCE) {
      if (t < 3) __builtin_amdgcn_sched_barrier(0);
    } else if (t < 3) {
      uint32_t* wn = &w[(t + 1) * BITS];
      if constexpr (BITS == 4)
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),
                          "+v"(acc[6]), "+v"(acc[7]), "+v"(wn[0]), "+v"(wn[1]), "+v"(wn[2]), "+v"(wn[3]));
      else if constexpr (BITS == 3)
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),
                          "+v"(acc[6]), "+v"(acc[7]), "+v"(wn[0]), "+v"(wn[1]), "+v"(wn[2]));
      else if constexpr (BITS == 2)
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),
                          "+v"(acc[6]), "+v"(acc[7]), "+v"(wn[0]), "+v"(wn[1]));
      else
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),
                          "+v"(acc[6]), "+v"(acc[7]), "+v"(wn[0]));
    }
  }
}

}  // namespace tmac
#endif  // TMAC_PERM_CORE_H_

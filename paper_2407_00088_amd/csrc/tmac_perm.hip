// Register-table decode kernel (gfx950) for packed layout 2.
//
// The GPU analogue of the paper's in-register TBL/PSHUFB lookup (Section 4 "Efficient table
// look-up"; Section 3.2 "Put lookup table on on-chip memory"): every lane keeps the tables of
// its own 16 activations (four tables) in VGPRs and looks indices up with v_perm_b32, a byte
// permute that selects 4 bytes out of an 8-byte source per instruction.
//
//   * Mirror consolidation (Section 3.3): only entries 0..7 of a table are kept, 8 fp16 values =
//     16 bytes.  A stored 4-bit code is {negate, 3-bit entry}; negation is an XOR of the fp16
//     sign bit, which the packer has placed at bit 7 of a byte: of the code's own byte for the
//     "low" rows, and of the byte that the code's entry reaches when the dword is rotated by
//     four bits for the "high" rows, so that neither needs a shift of its own.
//   * fp16 entries as two 8-bit tables (Section 4: "split float16 into two 8-bit LUTs"): the low
//     bytes and the high bytes of the 8 entries form two 8-byte sources (the precompute kernel
//     stores them already split); two permutes fetch both halves of 4 entries, two more permutes
//     re-interleave them into fp16 pairs.
//   * Bit-plane shift-accumulate (Eq. 1): v_dot2_f32_f16 multiplies a looked-up pair by the plane
//     weights (2^i, 2^(i+1)) and adds into an fp32 accumulator: two lookups per instruction.
//   * Scale, zero and bias once per (row, lane): the four tables of a lane lie in one
//     quantisation group, so acc starts at (mid - z) * S16 (bias term of Section 4's linear
//     transform, S16 = sum of the lane's 16 activations), collects the half-weighted lookups and
//     is multiplied by the scale once.
//   * Table quantisation (Section 3.3, TMAC_LUT_I8Q): one-byte entries need one permute per four
//     lookups; the negate bits select signed plane weights (+-2^i, again by a byte permute) and
//     v_dot4_i32_i8 does the shift-accumulate of four planes in integers; the four tables of a
//     lane share one scale, applied once per (row, lane).
//   * The integer path reuses the same code: int16 table entries (|T| <= 508) are exact in fp16,
//     all partial sums are integers below 2^24 and therefore exact in fp32; sums across waves
//     are taken in int32.
//
// Work split: one workgroup = RT tiles of 8 rows over the whole K; wave w owns one block of at
// most 8 chunks of 128 k (one 16-k unit per lane), so each wave streams contiguous pieces of the
// tiles' packed indices with 16-byte loads.  The eight lanes with equal (lane & 7) cover one
// 128-k chunk.  When the quantisation group is a multiple of 128 the 8 row sums of a lane are
// first reduced over those eight lanes with a transposing butterfly (v_permlane32_swap,
// v_permlane16_swap, DPP), which leaves one (row, chunk) sum per lane; scale, zero and bias are
// then applied once per (row, chunk) with a 4-byte scale/zero load per lane, and the chunks are
// summed with three DPP steps.  Other group sizes (multiples of 16) scale per (row, lane) before
// the same butterfly.  Cross-wave reduction goes through LDS and is finished by one wave with a
// fixed summation tree: results do not depend on timing.
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
  int M, N, K, U, n_tiles, nq;
  int G;           // elements per quantisation group
  uint32_t q_magic;  // ceil(2^32 / d), d = units (mode 1) or chunks (mode 2) per quantisation group; 0 if d = 1
  BlockSplit bs;   // split of the U/8 chunks into blocks of at most 8
  uint32_t ht_zero;  // slot index of the all-zero table
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

// GM: 0 = one scale per row or per tensor (raw sums, finished at the end), 1 = group scales applied
// per (row, lane) (any group size that is a multiple of 16), 2 = group scales applied per
// (row, 128-k chunk) after the in-chunk reduction (group sizes that are multiples of 128).
// FUSED: the lane builds the four tables of its unit from the activations itself (Algorithm 1
// Precompute inside the lookup kernel), with the arithmetic of the stand-alone precompute kernel.
// Q8: int8 tables with one scale per lane-unit (not with IS_INT or FUSED).
template <bool IS_INT, int BITS, int GM, int RT, bool FUSED, bool Q8>
__global__ __launch_bounds__(1024) void mpgemv_perm_kernel(const PermParams p) {
  static_assert(!(Q8 && (IS_INT || FUSED)), "int8 tables: fp16 activations, tables from the LUT buffer");
  constexpr int NR = 8 * RT;
  __shared__ float red[16 * NR];
  __shared__ float redS[16];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int NW = blockDim.x >> 6;
  const int n = blockIdx.y;
  const uint32_t jl = (uint32_t)lane & 7u, pos = (uint32_t)lane >> 3;  // chunk in block, unit in chunk
  uint32_t tile[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const uint32_t t = blockIdx.x * RT + rt;
    tile[rt] = t < (uint32_t)p.n_tiles ? t : (uint32_t)p.n_tiles - 1;  // clamped; stores are masked
  }

  // values the last stage needs, requested now so that their latency is hidden behind the main loop
  const float as = p.act_scale ? p.act_scale[n] : 1.0f;
  float fin_s = p.wscale, fin_z = p.zero_point, fin_Sf = 0.f;
  int fin_Si = 0;
  if constexpr (GM == 0) {
    if constexpr (!FUSED) {
      if constexpr (IS_INT) fin_Si = static_cast<const int*>(p.S)[n];
      else fin_Sf = static_cast<const float*>(p.S)[n];
    }
  }
  uint32_t fin_sz[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    fin_sz[rt] = 0;
    if constexpr (GM == 0)
      if (!p.per_tensor) fin_sz[rt] = reinterpret_cast<const uint32_t*>(p.sz)[(size_t)tile[rt] * 8 + jl];
  }

  // plane weights: halved in the group-scale modes, where acc = bias + 1/2 * sum_i 2^i L_i
  constexpr uint32_t W01 = GM ? h2pack(H_05, H_1) : h2pack(H_1, H_2);
  constexpr uint32_t W23 = GM ? h2pack(H_2, H_4) : h2pack(H_4, H_8);
  constexpr uint16_t WS0 = GM ? H_05 : H_1;  // single plane 0
  constexpr uint16_t WS2 = GM ? H_2 : H_4;   // single plane 2

  // GM 0: raw sums, GM 1: scaled sums per (row, lane); GM 2: one scaled (row, chunk) sum per tile
  float tot[GM == 2 ? RT : NR];
#pragma unroll
  for (int r = 0; r < (GM == 2 ? RT : NR); ++r) tot[r] = 0.f;

  float Stot = 0.f;  // fused mode, GM 0: this lane's share of the sum of all activations
  for (int blk = wave; blk < p.bs.nB; blk += NW) {
    const uint32_t c0 = (uint32_t)block_start(p.bs, blk);
    const uint32_t ng = (uint32_t)(blk < p.bs.r ? p.bs.q + 1 : p.bs.q);
    const uint32_t u0 = 8u * c0, nu = 8u * ng;
    const bool valid = jl < ng;
    const uint32_t l = valid ? pos * ng + jl : 0u;  // lanes without a unit re-read slot 0, with zero tables
    const uint32_t c = valid ? c0 + jl : c0;        // 128-k chunk of this lane
    const uint32_t u = 8u * c + pos;                // 16-k unit of this lane

    // 1. scale and zero, and (from the LUT buffer) the activation sum the bias term needs
    uint32_t szr[GM == 1 ? NR : RT];
    float Sl = 0.f;
    if constexpr (GM == 1) {
      uint32_t gq = p.q_magic ? __umulhi(u, p.q_magic) : u;  // u / (units per group), exact for u < 2^16
      gq = gq < (uint32_t)p.nq ? gq : (uint32_t)p.nq - 1;  // units in the K padding: tables and S16 are zero
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const pu32x4* szp = p.sz + (tile[rt] * (uint32_t)p.nq + gq) * 2;
        const pu32x4 a = szp[0], b = szp[1];
        szr[8 * rt + 0] = a.x; szr[8 * rt + 1] = a.y; szr[8 * rt + 2] = a.z; szr[8 * rt + 3] = a.w;
        szr[8 * rt + 4] = b.x; szr[8 * rt + 5] = b.y; szr[8 * rt + 6] = b.z; szr[8 * rt + 7] = b.w;
      }
      if constexpr (!FUSED) {
        if constexpr (IS_INT) Sl = (float)static_cast<const int*>(p.S16)[(uint32_t)n * (uint32_t)p.U + u];
        else Sl = static_cast<const float*>(p.S16)[(uint32_t)n * (uint32_t)p.U + u];
        Sl = valid ? Sl : 0.f;
      }
    } else if constexpr (GM == 2) {
      // one {scale, zero} per lane: row pos of the tile, quantisation group of chunk c
      const uint32_t gq = p.q_magic ? __umulhi(c, p.q_magic) : c;  // c / (chunks per group), exact for c < 2^16
      const uint32_t* szw = reinterpret_cast<const uint32_t*>(p.sz);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) szr[rt] = szw[(tile[rt] * (uint32_t)p.nq + gq) * 8 + pos];
      if constexpr (!FUSED) {
        if constexpr (IS_INT) Sl = (float)static_cast<const int*>(p.S128)[(uint32_t)n * ((uint32_t)p.U >> 3) + c];
        else Sl = static_cast<const float*>(p.S128)[(uint32_t)n * ((uint32_t)p.U >> 3) + c];
        Sl = valid ? Sl : 0.f;
      }
    }

    // 1b. in fused mode: the lane's 16 activations (zero past the end of K and for idle lanes), raw;
    // they are unpacked only after the index loads have been requested
    uint32_t araw[8];  // fp16: two per dword; int8: four per dword (one table each) in araw[0..3]
    if constexpr (FUSED) {
      const bool have = valid && 16u * u < (uint32_t)p.K;
      pu32x4 v0 = {0u, 0u, 0u, 0u}, v1 = {0u, 0u, 0u, 0u};
      if constexpr (IS_INT) {
        if (have) v0 = *reinterpret_cast<const pu32x4*>(static_cast<const int8_t*>(p.A) + (size_t)n * p.lda + 16u * u);
      } else {
        if (have) {
          const pu32x4* ap = reinterpret_cast<const pu32x4*>(static_cast<const __half*>(p.A) + (size_t)n * p.lda + 16u * u);
          v0 = ap[0];
          v1 = ap[1];
        }
      }
      araw[0] = v0.x; araw[1] = v0.y; araw[2] = v0.z; araw[3] = v0.w;
      araw[4] = v1.x; araw[5] = v1.y; araw[6] = v1.z; araw[7] = v1.w;
    }

    // 2. tables from the LUT buffer (requested before the indices: they are needed first)
    uint32_t lo0[4], lo1[4], hi0[4], hi1[4];
    float uscale = 0.f;
    if constexpr (Q8) {
      // two 16-byte pieces: tables 0,1 and 2,3, eight one-byte entries each (lo0 = entries 0..3,
      // lo1 = entries 4..7); plus the unit's scale
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t slot = valid ? ((uint32_t)n * (uint32_t)p.U + u0) * 2 + (uint32_t)h * nu + l : p.ht_zero;
        const pu32x4 d = p.ht[slot];
        lo0[2 * h] = d.x; lo1[2 * h] = d.y; lo0[2 * h + 1] = d.z; lo1[2 * h + 1] = d.w;
      }
      uscale = p.usc[(uint32_t)n * (uint32_t)p.U + u];  // idle lanes: an in-range unit; their sums are zero
    } else if constexpr (!FUSED) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t slot = valid ? ((uint32_t)n * (uint32_t)p.U + u0) * 4 + (uint32_t)t * nu + l : p.ht_zero;
        const pu32x4 d = p.ht[slot];
        lo0[t] = d.x; lo1[t] = d.y; hi0[t] = d.z; hi1[t] = d.w;
      }
    }

    // 3. packed indices of this lane: 16*BITS bytes per tile.  The block's records are stored
    // piece-major: 16-byte piece i of slot l sits at i*nu + l, so every load instruction of the
    // wavefront reads one contiguous run.
    uint32_t w[RT][4 * BITS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const pu32x4* src = p.idx + (tile[rt] * (uint32_t)p.U + u0) * BITS + l;
#pragma unroll
      for (int i = 0; i < BITS; ++i) {
        const pu32x4 v = __builtin_nontemporal_load(src + i * nu);
        w[rt][4 * i + 0] = v.x; w[rt][4 * i + 1] = v.y; w[rt][4 * i + 2] = v.z; w[rt][4 * i + 3] = v.w;
      }
    }

    // every load of this block is requested above this line; keep the scheduler from sinking index
    // loads below the first lookups (or, in fused mode, the first use of the activations)
    __builtin_amdgcn_sched_barrier(0);

    // 4. fused mode: the activation sum the bias term needs
    if constexpr (FUSED) {
      // sum of the lane's 16 activations, in the order of the precompute kernel's tree
      if constexpr (IS_INT) {
        int s16 = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) s16 = __builtin_amdgcn_sdot4((int)araw[t], 0x01010101, s16, false);
        Sl = (float)s16;  // |s16| <= 16 * 128
      } else {
        float t4[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) t4[t] = sum4_f16(araw[2 * t], araw[2 * t + 1]);
        Sl = (t4[0] + t4[1]) + (t4[2] + t4[3]);
      }
      if constexpr (GM == 0) Stot += Sl;
      if constexpr (GM == 2) {
        // sum over the chunk's eight lanes (lane bits 3, 4, 5), pairing units as the precompute kernel does
        Sl += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(Sl), 0x128, 0xf, 0xf, false));  // row_ror:8
        Sl += __shfl_xor(Sl, 16);
        Sl += __shfl_xor(Sl, 32);
      }
    }
    // 4b. fused mode: build the four tables while the indices are in flight (mirror half: entries
    // 0..7, i.e. the fourth activation subtracted), as low-byte and high-byte permute sources
    if constexpr (FUSED) {
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
        lo0[t] = bperm(pk[1], pk[0], 0x06040200u);
        lo1[t] = bperm(pk[3], pk[2], 0x06040200u);
        hi0[t] = bperm(pk[1], pk[0], 0x07050301u);
        hi1[t] = bperm(pk[3], pk[2], 0x07050301u);
      }
    }

#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      // 5. accumulators: GM 1 starts at the bias term, GM 0 continues the raw sums
      float acc[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        if constexpr (GM == 1) {
          const float z = __half2float(__ushort_as_half((uint16_t)(szr[8 * rt + r] >> 16)));
          acc[r] = fmaf(-z, Sl, p.mid * Sl);
        } else if constexpr (GM == 0) {
          acc[r] = tot[8 * rt + r];
        } else {
          acc[r] = 0.f;
        }
      }

      // 6. lookups
      if constexpr (Q8) {
        // signed plane weights as permute sources: bytes (+1, -1, +2, -2 | +4, -4, +8, -8); the
        // selector of a byte is 2 * plane + negate
        constexpr uint32_t WLO = 0xFE02FF01u, WHI = 0xF808FC04u;
        int ia[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) ia[r] = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          auto lookq = [&](uint32_t sel) { return bperm(lo1[t], lo0[t], sel); };
          // x: a dword of the record; planes: selector base (2 * plane of each byte)
          auto both = [&](uint32_t x, uint32_t planes, uint32_t& vA, uint32_t& wA, uint32_t& vB, uint32_t& wB) {
            // the selector base sits in a vector register so that (bits & mask) | base is one
            // v_and_or_b32 (a VOP3 instruction takes a single literal or scalar operand)
            uint32_t pv;
            asm("v_mov_b32 %0, %1" : "=v"(pv) : "s"(planes));
            const uint32_t xh = __builtin_amdgcn_alignbit(x, x, 4);  // the "high" rows: entries in bits 0..2, negate in bit 7
            vA = lookq(x & 0x07070707u);
            wA = bperm(WHI, WLO, ((x >> 7) & 0x01010101u) | pv);
            vB = lookq(xh & 0x07070707u);
            wB = bperm(WHI, WLO, ((xh >> 7) & 0x01010101u) | pv);
          };
          auto dot4 = [&](uint32_t v, uint32_t w, int a) { return __builtin_amdgcn_sdot4((int)v, (int)w, a, false); };
          auto quadq = [&](uint32_t x, int& a_lo, int& a_hi) {  // 4 planes of one row (low nibbles), one (high)
            uint32_t vA, wA, vB, wB;
            both(x, 0x06040200u, vA, wA, vB, wB);
            a_lo = dot4(vA, wA, a_lo);
            a_hi = dot4(vB, wB, a_hi);
          };
          auto pairq = [&](uint32_t x, int* a4) {  // planes 0,1 of rows 0,1 (low) and 2,3 (high) of a4
            uint32_t vA, wA, vB, wB;
            both(x, 0x02000200u, vA, wA, vB, wB);
            a4[0] = dot4(vA, wA & 0x0000FFFFu, a4[0]);
            a4[1] = dot4(vA, wA & 0xFFFF0000u, a4[1]);
            a4[2] = dot4(vB, wB & 0x0000FFFFu, a4[2]);
            a4[3] = dot4(vB, wB & 0xFFFF0000u, a4[3]);
          };
          auto singleq = [&](uint32_t x, uint32_t planes, int* a8) {  // one plane of rows 0..3 (low), 4..7 (high)
            uint32_t vA, wA, vB, wB;
            both(x, planes, vA, wA, vB, wB);
#pragma unroll
            for (int y = 0; y < 4; ++y) {
              a8[y] = dot4(vA, wA & (0xFFu << (8 * y)), a8[y]);
              a8[4 + y] = dot4(vB, wB & (0xFFu << (8 * y)), a8[4 + y]);
            }
          };
          const uint32_t* wt = &w[rt][t * BITS];
          if constexpr (BITS == 4) {
#pragma unroll
            for (int d = 0; d < 4; ++d) quadq(wt[d], ia[2 * d], ia[2 * d + 1]);
          } else if constexpr (BITS == 2) {
            pairq(wt[0], ia);
            pairq(wt[1], ia + 4);
          } else if constexpr (BITS == 1) {
            singleq(wt[0], 0x00000000u, ia);
          } else {
            pairq(wt[0], ia);
            pairq(wt[1], ia + 4);
            singleq(wt[2], 0x04040404u, ia);
          }
        }
        // integer sum of the unit's four tables, converted once and scaled (the scale is halved
        // together with the plane weights in the group-scale modes)
        const float us = GM != 0 ? 0.5f * uscale : uscale;
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = fmaf((float)ia[r], us, acc[r]);
      } else {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        // four lookups of table t: selector bytes `sel` (0..7 each), sign bits `sgn` at bit 7 of each byte
        auto look = [&](uint32_t sel, uint32_t sgn, uint32_t& p01, uint32_t& p23) {
          const uint32_t lo = bperm(lo1[t], lo0[t], sel);
          const uint32_t hi = bperm(hi1[t], hi0[t], sel) ^ sgn;
          p01 = bperm(hi, lo, 0x05010400u);  // fp16 pair of bytes 0 and 1
          p23 = bperm(hi, lo, 0x07030602u);  // fp16 pair of bytes 2 and 3
        };
        // the "high" rows of a dword: rotated by four bits their entries sit in bits 0..2 and their
        // negate bits (stored in bit 3 of the following byte) in bit 7 of each byte
        auto hi_set = [](uint32_t x) { return __builtin_amdgcn_alignbit(x, x, 4); };
        auto quad = [&](uint32_t x, float& a_lo, float& a_hi) {  // 4 planes of one row (low nibbles), one (high)
          uint32_t a, b;
          look(x & 0x07070707u, x & 0x80808080u, a, b);
          a_lo = dot2(a, W01, a_lo);
          a_lo = dot2(b, W23, a_lo);
          look(hi_set(x) & 0x07070707u, hi_set(x) & 0x80808080u, a, b);
          a_hi = dot2(a, W01, a_hi);
          a_hi = dot2(b, W23, a_hi);
        };
        auto pair = [&](uint32_t x, float* a4) {  // planes 0,1 of rows 0,1 (low) and 2,3 (high) of a4
          uint32_t a, b;
          look(x & 0x07070707u, x & 0x80808080u, a, b);
          a4[0] = dot2(a, W01, a4[0]);
          a4[1] = dot2(b, W01, a4[1]);
          look(hi_set(x) & 0x07070707u, hi_set(x) & 0x80808080u, a, b);
          a4[2] = dot2(a, W01, a4[2]);
          a4[3] = dot2(b, W01, a4[3]);
        };
        auto single = [&](uint32_t x, uint16_t wgt, float* a8) {  // one plane of rows 0..3 (low), 4..7 (high)
          const uint32_t wl = h2pack(wgt, H_0), wh = h2pack(H_0, wgt);
          uint32_t a, b;
          look(x & 0x07070707u, x & 0x80808080u, a, b);
          a8[0] = dot2(a, wl, a8[0]);
          a8[1] = dot2(a, wh, a8[1]);
          a8[2] = dot2(b, wl, a8[2]);
          a8[3] = dot2(b, wh, a8[3]);
          look(hi_set(x) & 0x07070707u, hi_set(x) & 0x80808080u, a, b);
          a8[4] = dot2(a, wl, a8[4]);
          a8[5] = dot2(a, wh, a8[5]);
          a8[6] = dot2(b, wl, a8[6]);
          a8[7] = dot2(b, wh, a8[7]);
        };
        const uint32_t* wt = &w[rt][t * BITS];
        if constexpr (BITS == 4) {
#pragma unroll
          for (int d = 0; d < 4; ++d) quad(wt[d], acc[2 * d], acc[2 * d + 1]);
        } else if constexpr (BITS == 2) {
          pair(wt[0], acc);
          pair(wt[1], acc + 4);
        } else if constexpr (BITS == 1) {
          single(wt[0], WS0, acc);
        } else {
          pair(wt[0], acc);
          pair(wt[1], acc + 4);
          single(wt[2], WS2, acc);
        }
      }
      }

      // 7. scale: once per (row, lane) in GM 1, once per (row, chunk) in GM 2
      if constexpr (GM == 1) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const float s = __half2float(__ushort_as_half((uint16_t)(szr[8 * rt + r] & 0xffffu)));
          tot[8 * rt + r] = fmaf(s, acc[r], tot[8 * rt + r]);
        }
      } else if constexpr (GM == 0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) tot[8 * rt + r] = acc[r];
      } else {
        const float v = reduce_hi3(acc, lane);  // row pos, summed over the chunk (sums of this size are exact for ints)
        const float s = __half2float(__ushort_as_half((uint16_t)(szr[rt] & 0xffffu)));
        const float z = __half2float(__ushort_as_half((uint16_t)(szr[rt] >> 16)));
        tot[rt] = fmaf(s, fmaf(p.mid - z, Sl, v), tot[rt]);
      }
    }
  }

  // 8. cross-lane sums: lane 8*r publishes row r of each tile
  constexpr bool RAW_INT = (GM == 0 && IS_INT);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    float v;
    if constexpr (GM == 2) v = tot[rt];
    else v = reduce_hi3(&tot[8 * rt], lane);
    v = reduce_lo3(v);
    if (jl == 0) {
      const int row = 8 * rt + (int)pos;
      if constexpr (RAW_INT) red[wave * NR + row] = __int_as_float((int)v);  // exact: integer < 2^24
      else red[wave * NR + row] = v;
    }
  }
  if constexpr (FUSED && GM == 0) {
    // the wave's sum of activations (exact for ints: below 2^24)
    const float t8[8] = {Stot, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float sw = reduce_lo3(reduce_hi3(t8, lane));  // lanes 0..7 hold the total
    if (lane == 0) redS[wave] = sw;
  }
  __syncthreads();

  // 9. wave 0 sums the waves with a fixed tree (lane = 8*slot + row: waves slot and slot + 8, then
  // the slots), finishes and stores
  if (wave != 0) return;
  if constexpr (FUSED && GM == 0) {
    float st = 0.f;
    for (int wv = 0; wv < NW; ++wv) st += redS[wv];  // wave order
    fin_Sf = st;
    fin_Si = (int)st;
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int r = 8 * rt + (int)jl;   // row of this lane
    const int ws = (int)pos;          // wave slot
    float sf = 0.f;
    int si = 0;
    if constexpr (RAW_INT) {
      si = ws < NW ? __float_as_int(red[ws * NR + r]) : 0;
      if (ws + 8 < NW) si += __float_as_int(red[(ws + 8) * NR + r]);
      si += __builtin_amdgcn_update_dpp(0, si, 0x128, 0xf, 0xf, false);  // row_ror:8
      si += __shfl_xor(si, 16);
      si += __shfl_xor(si, 32);
    } else {
      sf = ws < NW ? red[ws * NR + r] : 0.f;
      if (ws + 8 < NW) sf += red[(ws + 8) * NR + r];
      sf += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(sf), 0x128, 0xf, 0xf, false));
      sf += __shfl_xor(sf, 16);
      sf += __shfl_xor(sf, 32);
    }
    const uint32_t t = blockIdx.x * RT + rt;
    const int m = (int)t * 8 + (int)jl;
    if (lane < 8 && t < (uint32_t)p.n_tiles && m < p.M) {
      float res;
      int ires = 0;
      if constexpr (GM != 0) {
        res = sf * as;
      } else {
        float s = fin_s, z = fin_z;
        if (!p.per_tensor) {
          s = __half2float(__ushort_as_half((uint16_t)(fin_sz[rt] & 0xffffu)));
          z = __half2float(__ushort_as_half((uint16_t)(fin_sz[rt] >> 16)));
        }
        if constexpr (IS_INT) {
          const int St = fin_Si;
          if (p.int_exact) {
            ires = (si + p.icoef * St) >> 1;  // numerator is always even
            res = ((float)ires * as) * s;     // two roundings, left to right
          } else {
            res = (fmaf(p.mid - z, (float)St, 0.5f * (float)si) * as) * s;  // explicit fma: same rounding in every instantiation
          }
        } else {
          const float St = fin_Sf;
          res = (s * fmaf(p.mid - z, St, 0.5f * sf)) * as;  // explicit fma: same rounding in every instantiation
        }
      }
      const size_t o = (size_t)n * p.ldo + m;
      if (p.out_t == TMAC_OUT_F32) static_cast<float*>(p.out)[o] = res;
      else if (p.out_t == TMAC_OUT_F16) static_cast<__half*>(p.out)[o] = __float2half_rn(res);
      else static_cast<int*>(p.out)[o] = ires;
    }
  }
}

template <bool IS_INT, int BITS, int GM, int RT, bool FUSED, bool Q8 = false>
static hipError_t launch_one(const PermParams& p, int NW, hipStream_t st) {
  PermParams local = p;
  void* args[] = {&local};
  return hipLaunchKernel(reinterpret_cast<const void*>(mpgemv_perm_kernel<IS_INT, BITS, GM, RT, FUSED, Q8>),
                         dim3((p.n_tiles + RT - 1) / RT, p.N), dim3(NW * 64), args, 0, st);
}

// rt: row tiles per workgroup (1 or 2)
template <bool IS_INT, int BITS, int GM>
static hipError_t launch_rt(const PermParams& p, int rt, bool fused, int NW, hipStream_t st) {
  if (fused)
    return rt == 2 ? launch_one<IS_INT, BITS, GM, 2, true>(p, NW, st) : launch_one<IS_INT, BITS, GM, 1, true>(p, NW, st);
  return rt == 2 ? launch_one<IS_INT, BITS, GM, 2, false>(p, NW, st) : launch_one<IS_INT, BITS, GM, 1, false>(p, NW, st);
}

// int8 tables: one row tile per workgroup, tables from the LUT buffer
template <int BITS>
static hipError_t launch_q8(const PermParams& p, int gm, int NW, hipStream_t st) {
  switch (gm) {
    case 0: return launch_one<false, BITS, 0, 1, false, true>(p, NW, st);
    case 1: return launch_one<false, BITS, 1, 1, false, true>(p, NW, st);
    default: return launch_one<false, BITS, 2, 1, false, true>(p, NW, st);
  }
}

static hipError_t launch_q8_bits(const PermParams& p, int bits, int gm, int NW, hipStream_t st) {
  switch (bits) {
    case 1: return launch_q8<1>(p, gm, NW, st);
    case 2: return launch_q8<2>(p, gm, NW, st);
    case 3: return launch_q8<3>(p, gm, NW, st);
    case 4: return launch_q8<4>(p, gm, NW, st);
  }
  return hipErrorInvalidValue;
}

template <bool IS_INT, int BITS>
static hipError_t launch_gm(const PermParams& p, int gm, int rt, bool fused, int NW, hipStream_t st) {
  switch (gm) {
    case 0: return launch_rt<IS_INT, BITS, 0>(p, rt, fused, NW, st);
    case 1: return launch_rt<IS_INT, BITS, 1>(p, rt, fused, NW, st);
    default: return launch_rt<IS_INT, BITS, 2>(p, rt, fused, NW, st);
  }
}

template <bool IS_INT>
static hipError_t launch_bits(const PermParams& p, int bits, int gm, int rt, bool fused, int NW, hipStream_t st) {
  switch (bits) {
    case 1: return launch_gm<IS_INT, 1>(p, gm, rt, fused, NW, st);
    case 2: return launch_gm<IS_INT, 2>(p, gm, rt, fused, NW, st);
    case 3: return launch_gm<IS_INT, 3>(p, gm, rt, fused, NW, st);
    case 4: return launch_gm<IS_INT, 4>(p, gm, rt, fused, NW, st);
  }
  return hipErrorInvalidValue;
}

int launch_perm_gemv(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
                     int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale,
                     void* out_dev, int out_t, int64_t ldo, void* stream, int rows_per_group) {
  const bool fused = (lut_dev == nullptr);
  const bool q8 = (lut_t == TMAC_LUT_I8Q);
  const int lut_is_int = (lut_t == TMAC_LUT_I16);
  if (q8 && (fused || rows_per_group == 16)) return TMAC_EUNSUPPORTED;
  const Geometry ge = geometry(desc);
  LutGeom lg;
  if (!lut_geom(N, desc->K, desc->g, desc->group, lut_t, &lg)) return TMAC_EINVAL;
  if (N > 65535) return TMAC_EUNSUPPORTED;
  if (!fused && !lg.decode_parts) return TMAC_EUNSUPPORTED;  // a LUT buffer for this many rows has no half tables
  // 32-bit slot arithmetic inside the kernel
  if ((double)ge.n_tiles * lg.U * desc->bits >= 4294967296.0 || (double)N * lg.U * 4 >= 4294967296.0)
    return TMAC_EUNSUPPORTED;
  const bool one_group = (desc->group == 0 || desc->group == desc->K);

  PermParams p;
  const char* blob = static_cast<const char*>(packed_dev);
  p.idx = reinterpret_cast<const pu32x4*>(blob + ge.idx_off);
  p.sz = reinterpret_cast<const pu32x4*>(blob + ge.sz_off);
  const char* lut = static_cast<const char*>(lut_dev);
  p.ht = fused ? nullptr : reinterpret_cast<const pu32x4*>(lut + lg.ht_off);
  p.ht_zero = (uint32_t)((size_t)N * lg.U * lg.ht_slots);
  p.usc = (fused || !q8) ? nullptr : reinterpret_cast<const float*>(lut + lg.usc_off);
  p.S = fused ? nullptr : lut + lg.s_off;
  p.S16 = fused ? nullptr : lut + lg.s16_off;
  p.S128 = fused ? nullptr : lut + lg.s128_off;
  p.A = A_dev;
  p.lda = lda;
  p.K = desc->K;
  p.out = out_dev;
  p.act_scale = act_scale_dev;
  p.ldo = ldo;
  p.M = desc->M; p.N = N; p.U = lg.U; p.n_tiles = ge.n_tiles; p.nq = lg.nq;
  p.G = lg.Geff;
  p.bs = block_split(lg.U);
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
  const int NW = p.bs.nB < 16 ? p.bs.nB : 16;
  if (lut_is_int) {
    // integer sums are carried in fp32 inside a wave: a wave's total must stay below 2^24
    const int passes = (p.bs.nB + NW - 1) / NW;
    if ((double)508.0 * ((1 << desc->bits) - 1) * 256.0 * passes >= 16777216.0) return TMAC_EUNSUPPORTED;
  }
  // Two row tiles per workgroup share one set of tables (built or loaded once for 16 rows) but
  // halve the number of wavefronts.  Measured: worth 3-6 % once a call has more than about 8000
  // wavefronts, eight per SIMD (22016 x 4096, 8192 x 8192, 28672 x 8192), a loss of 2-5 % below
  // (4096 x 4096 up to 12288 x 4096); with several activation rows (one GEMV each in one launch)
  // the same count decides (4096 x 4096: from four rows on).  The default follows it.
  int rt = rows_per_group == 16 ? 2 : 1;
  if (rows_per_group == 0 && !q8 && (int64_t)ge.n_tiles * NW * N >= 8192) rt = 2;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int gm = one_group ? 0 : (desc->group % 128 == 0 ? 2 : 1);
  {
    // divisor of the lane's unit (mode 1) or chunk (mode 2) index that gives its quantisation group
    const uint32_t d = gm == 2 ? (uint32_t)desc->group / 128u : gm == 1 ? (uint32_t)desc->group / 16u : 1u;
    if (d >= 65536u || lg.U >= 65536) return TMAC_EUNSUPPORTED;
    p.q_magic = d == 1 ? 0u : (uint32_t)((4294967296ull + d - 1) / d);
  }
  const hipError_t e = q8 ? launch_q8_bits(p, desc->bits, gm, NW, st)
                          : lut_is_int ? launch_bits<true>(p, desc->bits, gm, rt, fused, NW, st)
                                       : launch_bits<false>(p, desc->bits, gm, rt, fused, NW, st);
  if (e != hipSuccess) {
    note_hip_error((int)e);
    return TMAC_EHIP;
  }
  return TMAC_OK;
}

}  // namespace tmac

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
#include <cstring>

#include "tmac.h"
#include "tmac_internal.h"
#include "tmac_perm_core.h"

namespace tmac {

// GM: 0 = one scale per row or per tensor (raw sums, finished at the end), 1 = group scales applied
// per (row, lane) (any group size that is a multiple of 16), 2 = group scales applied per
// (row, 128-k chunk) after the in-chunk reduction (group sizes that are multiples of 128).
// FUSED: the lane builds the four tables of its unit from the activations itself (Algorithm 1
// Precompute inside the lookup kernel), with the arithmetic of the stand-alone precompute kernel.
// Q8: int8 tables with one scale per lane-unit (not with IS_INT or FUSED).
template <bool IS_INT, int BITS, int GM, int RT, bool FUSED, bool Q8, int NM>
__global__ __launch_bounds__(1024) void mpgemv_perm_kernel(int e0, int e1, int e2, int e3, int e4, int e5, int e6,
                                                           const PermParamsT<NM> pp) {
  static_assert(!(Q8 && IS_INT), "int8 tables: fp16 activations");
  constexpr int NR = 8 * RT;
  __shared__ float red[16 * NR];
  __shared__ float redS[16];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = blockIdx.y;
  const uint32_t jl = (uint32_t)lane & 7u, pos = (uint32_t)lane >> 3;  // chunk in block, unit in chunk
  // the matrix this workgroup serves (all wave-uniform).  Its description is copied out of the
  // kernel arguments in one go: every scalar load is requested before the first wait.
  int mi = 0, wg0 = 0;
  if constexpr (NM > 1) {
    // (the first seven entries of wg_end travel as arguments of their own, ahead of the struct: the
    // first dwords of the kernel arguments can be handed to a wave in registers at its start, so the
    // matrix is known without a trip to memory)
    const int ends[7] = {e0, e1, e2, e3, e4, e5, e6};
#pragma unroll
    for (int i = 0; i < NM - 1; ++i) {  // wg_end is non-decreasing, INT_MAX past the last matrix
      // (sign bit of end - 1 - id as an integer: keeps the count in scalar registers)
      const int past = (int)((uint32_t)(ends[i] - 1 - (int)blockIdx.x) >> 31);
      mi += past;
      wg0 = past ? ends[i] : wg0;
    }
  }
  const PermMat p = pp.m[mi];
  // The waves of a workgroup form gpw groups of gsz waves; a group serves RT row tiles over the whole
  // K, wave wig of it taking the blocks wig, wig + gsz, ...  Waves left over (blockDim is shared by
  // the matrices of a launch) have no group: they skip the work and join the barrier.
  const int NW = p.gsz;
  const int grp = (int)(((uint32_t)wave * p.ginv) >> 8);
  const int wig = wave - grp * NW;
  const bool active = grp < p.gpw;
  const uint32_t tg = (uint32_t)(((int)blockIdx.x - wg0) * p.gpw + (active ? grp : 0));  // group of row tiles
  uint32_t tile[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const uint32_t t = tg * RT + rt;
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

  // GM 0: raw sums, GM 1: scaled sums per (row, lane); GM 2: one scaled (row, chunk) sum per tile
  float tot[GM == 2 ? RT : NR];
#pragma unroll
  for (int r = 0; r < (GM == 2 ? RT : NR); ++r) tot[r] = 0.f;

  float Stot = 0.f;  // fused mode, GM 0: this lane's share of the sum of all activations
  for (int blk = active ? wig : p.bs.nB; blk < p.bs.nB; blk += NW) {
    const LaneBlock lb = lane_block(p.bs, blk, lane);
    const uint32_t u0 = lb.u0, nu = lb.nu;
    const bool valid = lb.valid;
    const uint32_t l = lb.l;  // lanes without a unit re-read slot 0, with zero tables
    const uint32_t c = lb.c;  // 128-k chunk of this lane
    const uint32_t u = lb.u;  // 16-k unit of this lane

    // 1. in fused mode: the lane's 16 activations (zero past the end of K and for idle lanes), raw;
    // they are unpacked only after the index loads have been requested.  Requested first: the tables
    // are built from them while the indices are in flight (ahead of the scale loads it is 1.3 % off a
    // single-matrix launch)
    uint32_t araw[8];
    if constexpr (FUSED) lane_load_act<IS_INT>(p.A, p.lda, n, p.K, lb, araw);

    // 1b. scale and zero, and (from the LUT buffer) the activation sum the bias term needs
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
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        szr[rt] = load_at<uint32_t>(scalar_base(reinterpret_cast<const char*>(p.sz) + (size_t)(tile[rt] * (uint32_t)p.nq) * 32),
                                    (gq * 8 + pos) * 4);
      if constexpr (!FUSED) {
        if constexpr (IS_INT) Sl = (float)static_cast<const int*>(p.S128)[(uint32_t)n * ((uint32_t)p.U >> 3) + c];
        else Sl = static_cast<const float*>(p.S128)[(uint32_t)n * ((uint32_t)p.U >> 3) + c];
        Sl = valid ? Sl : 0.f;
      }
    }

    // 2. tables from the LUT buffer (requested before the indices: they are needed first)
    LaneTables T;
    uint32_t (&lo0)[4] = T.lo0, (&lo1)[4] = T.lo1, (&hi0)[4] = T.hi0, (&hi1)[4] = T.hi1;
    float uscale = 0.f;
    if constexpr (Q8 && !FUSED) {
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
      // wave-uniform 64-bit base (scalar registers) plus the lane's 32-bit byte offset: the loads
      // take the base from scalar registers and need no address arithmetic in the vector ALU
      const char* base = reinterpret_cast<const char*>(p.idx) + (size_t)((tile[rt] * (uint32_t)p.U + u0) * BITS) * 16;
      const uint32_t voff = l * 16u;
#pragma unroll
      for (int i = 0; i < BITS; ++i) {
        const gbase_t bi = scalar_base(base + (size_t)(i * nu) * 16);
        const pu32x4 v = __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) pu32x4*>(bi + voff));
        w[rt][4 * i + 0] = v.x; w[rt][4 * i + 1] = v.y; w[rt][4 * i + 2] = v.z; w[rt][4 * i + 3] = v.w;
      }
    }

    // every load of this block is requested above this line; keep the scheduler from sinking index
    // loads below the first lookups (or, in fused mode, the first use of the activations)
    __builtin_amdgcn_sched_barrier(0);

    // 4. fused mode: the activation sum the bias term needs, and the four tables, built while the
    // indices are in flight
    if constexpr (FUSED) {
      Sl = lane_act_sum<IS_INT>(araw);
      if constexpr (GM == 0) Stot += Sl;
      if constexpr (GM == 2) Sl = chunk_sum(Sl);
      if constexpr (Q8) lane_build_tables_q8(araw, T, uscale);
      else lane_build_tables<IS_INT>(araw, T);
    }

#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      // 5. accumulators: GM 1 starts at the bias term, GM 0 continues the raw sums
      float acc[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        if constexpr (GM == 1) {
          const float z = __half2float(__ushort_as_half((uint16_t)(szr[8 * rt + r] >> 16)));
          acc[r] = fmaf(-z, Sl, pp.mid * Sl);
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
          // (the sums of the first table start at zero: the three-operand form with the constant 0
          // as addend instead of a zeroed register; the result feeds the addend of the next table's
          // dot product, see dot2_from_zero)
          auto dot4 = [&](uint32_t v, uint32_t w, int a, bool first = true) {
            if (t == 0 && first) {
              int r;
              asm("v_dot4_i32_i8 %0, %1, %2, 0" : "=v"(r) : "v"(v), "v"(w));
              return r;
            }
            return __builtin_amdgcn_sdot4((int)v, (int)w, a, false);
          };
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
          // first: these are the first terms of the sums (false for the third plane at three bits)
          auto singleq = [&](uint32_t x, uint32_t planes, int* a8, bool first) {  // one plane of rows 0..3 (low), 4..7 (high)
            uint32_t vA, wA, vB, wB;
            both(x, planes, vA, wA, vB, wB);
#pragma unroll
            for (int y = 0; y < 4; ++y) {
              a8[y] = dot4(vA, wA & (0xFFu << (8 * y)), a8[y], first);
              a8[4 + y] = dot4(vB, wB & (0xFFu << (8 * y)), a8[4 + y], first);
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
            singleq(wt[0], 0x00000000u, ia, true);
          } else {
            pairq(wt[0], ia);
            pairq(wt[1], ia + 4);
            singleq(wt[2], 0x04040404u, ia, false);
          }
          __builtin_amdgcn_sched_barrier(0);  // table by table: few registers live at a time
        }
        // integer sum of the unit's four tables, converted once and scaled (the scale is halved
        // together with the plane weights in the group-scale modes)
        const float us = GM != 0 ? 0.5f * uscale : uscale;
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = fmaf((float)ia[r], us, acc[r]);
      } else {
        lane_lookups<BITS, GM != 0, GM == 2, RT == 2>(w[rt], T, acc);
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
        tot[rt] = fmaf(s, fmaf(pp.mid - z, Sl, v), tot[rt]);
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

  // 9. the first wave of every group sums the group's waves with a fixed tree (lane = 8*slot + row:
  // waves slot and slot + 8, then the slots), finishes and stores
  if (wig != 0 || !active) return;
  const int w0 = grp * NW;  // first wave of the group
  if constexpr (FUSED && GM == 0) {
    float st = 0.f;
    for (int wv = 0; wv < NW; ++wv) st += redS[w0 + wv];  // wave order
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
      si = ws < NW ? __float_as_int(red[(w0 + ws) * NR + r]) : 0;
      if (ws + 8 < NW) si += __float_as_int(red[(w0 + ws + 8) * NR + r]);
      si += __builtin_amdgcn_update_dpp(0, si, 0x128, 0xf, 0xf, false);  // row_ror:8
      si += __shfl_xor(si, 16);
      si += __shfl_xor(si, 32);
    } else {
      sf = ws < NW ? red[(w0 + ws) * NR + r] : 0.f;
      if (ws + 8 < NW) sf += red[(w0 + ws + 8) * NR + r];
      sf += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(sf), 0x128, 0xf, 0xf, false));
      sf += __shfl_xor(sf, 16);
      sf += __shfl_xor(sf, 32);
    }
    const uint32_t t = tg * RT + rt;
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
            res = (fmaf(pp.mid - z, (float)St, 0.5f * (float)si) * as) * s;  // explicit fma: same rounding in every instantiation
          }
        } else {
          const float St = fin_Sf;
          res = (s * fmaf(pp.mid - z, St, 0.5f * sf)) * as;  // explicit fma: same rounding in every instantiation
        }
      }
      const size_t o = (size_t)n * p.ldo + m;
      if (pp.out_t == TMAC_OUT_F32) static_cast<float*>(p.out)[o] = res;
      else if (pp.out_t == TMAC_OUT_F16) static_cast<__half*>(p.out)[o] = __float2half_rn(res);
      else static_cast<int*>(p.out)[o] = ires;
    }
  }
}

// count == 1 launches the single-matrix instantiation (its arguments hold one matrix); only the
// kernels that build their tables themselves have an instantiation for several matrices.
template <bool IS_INT, int BITS, int GM, int RT, bool FUSED, bool Q8 = false>
static hipError_t launch_one(const PermParams& p, int count, int NW, hipStream_t st) {
  const dim3 grid(p.wg_end[count - 1], p.N), block(NW * 64);
  const size_t lds = (size_t)p.pad;  // dynamic LDS nobody uses: caps the workgroups per CU (0: no cap)
  if (count == 1) {
    PermParamsT<1> one;
    one.wg_end[0] = p.wg_end[0];
    one.N = p.N; one.mid = p.mid; one.out_t = p.out_t; one.pad = 0;
    one.m[0] = p.m[0];
    int e[7] = {0, 0, 0, 0, 0, 0, 0};
    void* args[] = {&e[0], &e[1], &e[2], &e[3], &e[4], &e[5], &e[6], &one};
    return hipLaunchKernel(reinterpret_cast<const void*>(mpgemv_perm_kernel<IS_INT, BITS, GM, RT, FUSED, Q8, 1>), grid,
                           block, args, lds, st);
  }
  if constexpr (FUSED) {
    PermParams local = p;
    static_assert(PERM_MAX_MATS == 8, "seven workgroup bounds travel as arguments of their own");
    int e[7];
    for (int i = 0; i < 7; ++i) e[i] = p.wg_end[i];
    void* args[] = {&e[0], &e[1], &e[2], &e[3], &e[4], &e[5], &e[6], &local};
    return hipLaunchKernel(
        reinterpret_cast<const void*>(mpgemv_perm_kernel<IS_INT, BITS, GM, RT, FUSED, Q8, PERM_MAX_MATS>), grid, block,
        args, lds, st);
  }
  return hipErrorInvalidValue;
}

// rt: row tiles per workgroup (1 or 2)
template <bool IS_INT, int BITS, int GM>
static hipError_t launch_rt(const PermParams& p, int count, int rt, bool fused, int NW, hipStream_t st) {
  if (fused)
    return rt == 2 ? launch_one<IS_INT, BITS, GM, 2, true>(p, count, NW, st) : launch_one<IS_INT, BITS, GM, 1, true>(p, count, NW, st);
  return rt == 2 ? launch_one<IS_INT, BITS, GM, 2, false>(p, count, NW, st) : launch_one<IS_INT, BITS, GM, 1, false>(p, count, NW, st);
}

// int8 tables: from the LUT buffer (one row tile per group of waves) or quantised inside the kernel
// (one or two row tiles, one or several matrices).  The int8 lookups save 4 of 17 instructions per
// index dword and the table build costs 50 more per unit than fp16 tables: with two row tiles the
// instruction counts are level (719 against 734 at 4 bit), with one the fp16 tables are ahead.
template <int BITS, int GM>
static hipError_t launch_q8_gm(const PermParams& p, int count, int rt, bool fused, int NW, hipStream_t st) {
  if (fused)
    return rt == 2 ? launch_one<false, BITS, GM, 2, true, true>(p, count, NW, st)
                   : launch_one<false, BITS, GM, 1, true, true>(p, count, NW, st);
  return launch_one<false, BITS, GM, 1, false, true>(p, 1, NW, st);
}

template <int BITS>
static hipError_t launch_q8(const PermParams& p, int count, int gm, int rt, bool fused, int NW, hipStream_t st) {
  switch (gm) {
    case 0: return launch_q8_gm<BITS, 0>(p, count, rt, fused, NW, st);
    case 1: return launch_q8_gm<BITS, 1>(p, count, rt, fused, NW, st);
    default: return launch_q8_gm<BITS, 2>(p, count, rt, fused, NW, st);
  }
}

static hipError_t launch_q8_bits(const PermParams& p, int count, int bits, int gm, int rt, bool fused, int NW,
                                 hipStream_t st) {
  switch (bits) {
    case 1: return launch_q8<1>(p, count, gm, rt, fused, NW, st);
    case 2: return launch_q8<2>(p, count, gm, rt, fused, NW, st);
    case 3: return launch_q8<3>(p, count, gm, rt, fused, NW, st);
    case 4: return launch_q8<4>(p, count, gm, rt, fused, NW, st);
  }
  return hipErrorInvalidValue;
}

template <bool IS_INT, int BITS>
static hipError_t launch_gm(const PermParams& p, int count, int gm, int rt, bool fused, int NW, hipStream_t st) {
  switch (gm) {
    case 0: return launch_rt<IS_INT, BITS, 0>(p, count, rt, fused, NW, st);
    case 1: return launch_rt<IS_INT, BITS, 1>(p, count, rt, fused, NW, st);
    default: return launch_rt<IS_INT, BITS, 2>(p, count, rt, fused, NW, st);
  }
}

template <bool IS_INT>
static hipError_t launch_bits(const PermParams& p, int count, int bits, int gm, int rt, bool fused, int NW, hipStream_t st) {
  switch (bits) {
    case 1: return launch_gm<IS_INT, 1>(p, count, gm, rt, fused, NW, st);
    case 2: return launch_gm<IS_INT, 2>(p, count, gm, rt, fused, NW, st);
    case 3: return launch_gm<IS_INT, 3>(p, count, gm, rt, fused, NW, st);
    case 4: return launch_gm<IS_INT, 4>(p, count, gm, rt, fused, NW, st);
  }
  return hipErrorInvalidValue;
}

int perm_fill(PermMat& p, const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
              int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale, void* out_dev,
              int out_t, int64_t ldo, int group_waves, int* gm_out) {
  const bool fused = (lut_dev == nullptr);
  const bool q8 = (lut_t == TMAC_LUT_I8Q);
  const int lut_is_int = (lut_t == TMAC_LUT_I16);
  const Geometry ge = geometry(desc);
  LutGeom lg;
  // (tables quantised inside the kernel need no LUT buffer: the geometry of the fp16 type gives K's padding
  // and the groups without the buffer's limit on N)
  if (!lut_geom(N, desc->K, desc->g, desc->group, fused && q8 ? (int)TMAC_LUT_F16 : lut_t, &lg)) return TMAC_EINVAL;
  if (N > 65535) return TMAC_EUNSUPPORTED;
  if (!fused && !lg.decode_parts) return TMAC_EUNSUPPORTED;  // a LUT buffer for this many rows has no half tables
  // 32-bit slot arithmetic inside the kernel
  if ((double)ge.n_tiles * lg.U * desc->bits >= 4294967296.0 || (double)N * lg.U * 4 >= 4294967296.0)
    return TMAC_EUNSUPPORTED;
  const bool one_group = (desc->group == 0 || desc->group == desc->K);

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
  p.M = desc->M; p.U = lg.U; p.n_tiles = ge.n_tiles; p.nq = lg.nq;
  p.bs = block_split(lg.U);
  p.per_tensor = (desc->group == 0);
  p.wscale = weight_scale;
  p.zero_point = p.per_tensor ? desc->zero_point : 0.f;
  p.int_exact = 0;
  p.icoef = 0;
  if (p.per_tensor && lut_is_int) {
    const float z = desc->zero_point;
    if (z == rintf(z) && fabsf(z) < 64.f) {
      p.int_exact = 1;
      p.icoef = ((1 << desc->bits) - 1) - 2 * (int)z;
    }
  }
  if (out_t == TMAC_OUT_I32 && !p.int_exact) return TMAC_EINVAL;
  const int gcap = group_waves > 0 ? group_waves : PERM_GROUP_WAVES;
  p.gsz = p.bs.nB < gcap ? p.bs.nB : gcap;
  p.ginv = (256u + (uint32_t)p.gsz - 1u) / (uint32_t)p.gsz;
  if (lut_is_int) {
    // integer sums are carried in fp32 inside a wave: a wave's total must stay below 2^24
    const int passes = (p.bs.nB + p.gsz - 1) / p.gsz;
    if ((double)508.0 * ((1 << desc->bits) - 1) * 256.0 * passes >= 16777216.0) return TMAC_EUNSUPPORTED;
    // fused call with one scale per row or tensor: the sum of an activation row (|sum| <= 128 K)
    // is carried in fp32 across lanes and waves as well
    if (fused && one_group && (double)128.0 * desc->K >= 16777216.0) return TMAC_EUNSUPPORTED;
  }
  const int gm = one_group ? 0 : (desc->group % 128 == 0 ? 2 : 1);
  {
    // divisor of the lane's unit (mode 1) or chunk (mode 2) index that gives its quantisation group
    const uint32_t d = gm == 2 ? (uint32_t)desc->group / 128u : gm == 1 ? (uint32_t)desc->group / 16u : 1u;
    if (d >= 65536u || lg.U >= 65536) return TMAC_EUNSUPPORTED;
    p.q_magic = d == 1 ? 0u : (uint32_t)((4294967296ull + d - 1) / d);
  }
  *gm_out = gm;
  return TMAC_OK;
}

// Bytes of unused dynamic LDS that let at most `wgs_per_cu` workgroups share a CU's 160 KB (0: no cap).
// Fewer resident waves finish in a more staggered way, which evens out the end of a launch.
static int perm_lds_cap(int wgs_per_cu) {
  if (wgs_per_cu <= 0) return 0;
  const int total = 160 * 1024, n = wgs_per_cu < 2 ? 2 : wgs_per_cu;  // (one per CU would exceed the 64 KB a workgroup may ask for)
  return total / (n + 1) + 1024;  // n + 1 of these do not fit
}

// Launch shape of matrix i for W waves per workgroup and rt row tiles per group of waves; returns the
// number of workgroups.
static int64_t perm_shape(PermMat& p, int W, int rt) {
  p.gpw = W / p.gsz;
  const int64_t groups = ((int64_t)p.n_tiles + rt - 1) / rt;
  return (groups + p.gpw - 1) / p.gpw;
}

int launch_perm_gemv(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
                     int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale,
                     void* out_dev, int out_t, int64_t ldo, void* stream, const tmac_tuning* tuning) {
  const int rows_per_group = tuning ? tuning->rows_per_group : 0;
  const int group_waves = tuning ? tuning->group_waves : 0;
  const int wg_waves = tuning ? tuning->workgroup_waves : 0;
  const bool fused = (lut_dev == nullptr);
  const bool q8 = (lut_t == TMAC_LUT_I8Q);
  const int lut_is_int = (lut_t == TMAC_LUT_I16);
  if (q8 && !fused && rows_per_group == 16) return TMAC_EUNSUPPORTED;
  PermParams pp;
  memset(&pp, 0, sizeof(pp));
  PermMat& p = pp.m[0];
  int gm = 0;
  const int stt = perm_fill(p, desc, packed_dev, lut_dev, A_dev, lda, lut_t, N, act_scale_dev, weight_scale, out_dev,
                            out_t, ldo, group_waves, &gm);
  if (stt != TMAC_OK) return stt;
  pp.N = N;
  pp.mid = 0.5f * (float)((1 << desc->bits) - 1);
  pp.out_t = out_t;
  // waves per workgroup: one group of waves unless asked otherwise (then whole groups)
  const int NW = wg_waves > 0 ? (wg_waves / p.gsz > 0 ? wg_waves / p.gsz * p.gsz : p.gsz) : p.gsz;
  // Two row tiles per group of waves share one set of tables (built or loaded once for 16 rows) but
  // halve the number of wavefronts.  Measured: worth 3-6 % once a call has more than about 8000
  // wavefronts, eight per SIMD (22016 x 4096, 8192 x 8192, 28672 x 8192), a loss of 2-5 % below
  // (4096 x 4096 up to 12288 x 4096); with several activation rows (one GEMV each in one launch)
  // the same count decides (4096 x 4096: from four rows on).  The default follows it.
  int rt = rows_per_group == 16 ? 2 : 1;
  if (rows_per_group == 0 && (fused || !q8) && (int64_t)p.n_tiles * p.gsz * N >= 8192) rt = 2;
  const int64_t wgs = perm_shape(p, NW, rt);
  if (wgs > 0x7fffffff) return TMAC_EUNSUPPORTED;
  pp.wg_end[0] = (int)wgs;
  pp.pad = perm_lds_cap(tuning ? tuning->workgroups_per_cu : 0);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const hipError_t e = q8 ? launch_q8_bits(pp, 1, desc->bits, gm, rt, fused, NW, st)
                          : lut_is_int ? launch_bits<true>(pp, 1, desc->bits, gm, rt, fused, NW, st)
                                       : launch_bits<false>(pp, 1, desc->bits, gm, rt, fused, NW, st);
  if (e != hipSuccess) {
    note_hip_error((int)e);
    return TMAC_EHIP;
  }
  return TMAC_OK;
}

// Several matrices, one launch: the workgroups of the grid are dealt out over the matrices' groups of
// row tiles.  All matrices share the code path (bit-width, how scales are grouped, activation type);
// K, M and every pointer are per matrix.  The waves per workgroup W are common to the launch: each
// matrix puts floor(W / gsz) groups of gsz waves into a workgroup, and W is chosen so that the fewest
// wave slots stay idle.  The summation order of a matrix depends on its gsz alone, so results equal
// those of the single-matrix call bit for bit.
int launch_perm_gemv_multi(const tmac_gemv_item* items, int count, int act_t, int N, int out_t, void* stream,
                           const tmac_tuning* tuning) {
  const int rows_per_group = tuning ? tuning->rows_per_group : 0;
  const int group_waves = tuning ? tuning->group_waves : 0;
  const int wg_waves = tuning ? tuning->workgroup_waves : 0;
  if (count < 1 || count > PERM_MAX_MATS) return TMAC_EUNSUPPORTED;
  const int lut_t = act_t == TMAC_ACT_I8 ? (int)TMAC_LUT_I16 : act_t == TMAC_ACT_F16_TQ ? (int)TMAC_LUT_I8Q : (int)TMAC_LUT_F16;
  PermParams pp;
  memset(&pp, 0, sizeof(pp));
  int gm0 = 0, max_gsz = 1;
  int64_t waves = 0;
  for (int i = 0; i < count; ++i) {
    const tmac_gemv_item& it = items[i];
    int gm = 0;
    const int stt = perm_fill(pp.m[i], it.desc, it.packed_dev, nullptr, it.A_dev, it.lda, lut_t, N, it.act_scale_dev,
                              it.weight_scale, it.out_dev, out_t, it.ldo, group_waves, &gm);
    if (stt != TMAC_OK) return stt;
    if (i == 0) gm0 = gm;
    if (gm != gm0 || it.desc->bits != items[0].desc->bits) return TMAC_EUNSUPPORTED;
    if (pp.m[i].gsz > max_gsz) max_gsz = pp.m[i].gsz;
    waves += (int64_t)pp.m[i].n_tiles * pp.m[i].gsz;
  }
  pp.N = N;
  pp.mid = 0.5f * (float)((1 << items[0].desc->bits) - 1);
  pp.out_t = out_t;
  const bool q8 = (lut_t == TMAC_LUT_I8Q);
  int rt = rows_per_group == 16 ? 2 : 1;
  if (rows_per_group == 0 && waves * N >= 8192) rt = 2;
  // waves per workgroup: the W in [largest gsz, 8] (up to 16 when asked) that leaves the fewest wave
  // slots idle; measured on the three Llama-2-7B shapes in one launch: 14.2 us with workgroups of
  // eight waves, 17-19 us with sixteen
  int W = max_gsz;
  int64_t best = -1;
  const int w_cap = max_gsz > PERM_GROUP_WAVES ? max_gsz : PERM_GROUP_WAVES;
  const int w_lo = wg_waves >= max_gsz ? wg_waves : max_gsz, w_hi = wg_waves >= max_gsz ? wg_waves : w_cap;
  for (int w = w_lo; w <= w_hi; ++w) {
    int64_t slots = 0;
    for (int i = 0; i < count; ++i) slots += perm_shape(pp.m[i], w, rt) * w;
    if (best < 0 || slots < best) { best = slots; W = w; }
  }
  int64_t end = 0;
  for (int i = 0; i < count; ++i) {
    end += perm_shape(pp.m[i], W, rt);
    if (end > 0x7fffffff) return TMAC_EUNSUPPORTED;
    pp.wg_end[i] = (int)end;
  }
  for (int i = count; i < PERM_MAX_MATS; ++i) pp.wg_end[i] = 0x7fffffff;
  pp.pad = perm_lds_cap(tuning ? tuning->workgroups_per_cu : 0);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int bits = items[0].desc->bits;
  const hipError_t e = q8                        ? launch_q8_bits(pp, count, bits, gm0, rt, true, W, st)
                       : (lut_t == TMAC_LUT_I16) ? launch_bits<true>(pp, count, bits, gm0, rt, true, W, st)
                                                 : launch_bits<false>(pp, count, bits, gm0, rt, true, W, st);
  if (e != hipSuccess) {
    note_hip_error((int)e);
    return TMAC_EHIP;
  }
  return TMAC_OK;
}

}  // namespace tmac

// Batched lookup kernels (gfx950) for packed layout 3: several to many activation rows (batched
// decode, prefill mpGEMM).
//
// Section 3.2 of the paper argues that the tables must sit in fast on-chip memory and that a large
// tile over M lets many weight rows reuse one table.  Here the tables of a K-slice and of NT = 4 or
// 8 activation rows live in LDS, laid out [table][entry][n] (NT fp16 values = 8 or 16 bytes per
// entry), and every LANE owns one weight row: a wavefront looks one table up for 64 rows at a
// time.  All lanes of a read address the same table, whose 16 entries cover the LDS banks evenly,
// so lanes that want the same entry are served by broadcast and lanes that want different entries
// hit different banks: the lookups are free of bank conflicts, and one lookup feeds NT
// activation rows.
//
//   * Weight permutation / interleaving (Section 3.2): a lane reads the `bits` index dwords of its
//     row and of one 32-k chunk with one load (16 bytes at 4 bit); the eight nibbles of a dword are
//     the indices of eight consecutive tables, and two mask-and-shift operations turn them into
//     the byte offsets of the entries (even and odd tables) four at a time.
//   * Aggregation: the eight entries of a chunk and plane are added as packed 16-bit pairs, two
//     activation rows per instruction, then widened.  Exact for integer tables.  For fp16 tables
//     this is this library's own choice and it is lossy (three fp16 roundings per chunk sum: about
//     1.5e-4 -> 3.4e-4 relative error, still a sixth of the 2e-3 bar); it is not the paper's "fast
//     8-bit aggregation" (Section 4), an integer averaging trick that is not built here.
//   * Bit-plane shift-accumulate (Eq. 1): the widening v_fma_mix_f32 takes the fp16 chunk sum and
//     multiplies by 2^i.
//   * Scale, zero and bias once per quantisation group (Section 4, bit-serial linear transform).
//     In the many-row kernel with fp16 tables the group's scale rides on the plane weights
//     (s/2 * 2^i, four multiplies when a group starts) and the bias term s * (mid - z) * S is
//     added at the same moment, so a group costs 12 instructions instead of 32 and the finished
//     group sums need no registers of their own; integer tables keep exact integer group sums
//     and convert once per group.
//   * Axis order (Section 3.2 "axis reordering"): K is walked slice by slice inside the
//     workgroup, so only a 32 KB slice of the tables is live in LDS; the sums of a row stay
//     in the lane's registers: fixed order.
//   * Few activation rows (batched decode) leave too few (row block, n tile) pairs to fill the
//     chip: K is then also split over gridDim.z workgroups, whose partial sums meet in the
//     workspace; rows_sum_kernel, the next kernel on the stream, adds them in slice order (fixed
//     order again) and writes the result.  When the slices are as short as eight chunks (a handful
//     of activation rows), mpgemm_rows8_kernel further down takes the call instead.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

typedef uint32_t ru32x4v __attribute__((ext_vector_type(4)));
typedef uint32_t ru32x2v __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) char rows_lds_char;
typedef __attribute__((address_space(3))) const ru32x2v rows_lds_u32x2;
typedef __attribute__((address_space(3))) const ru32x4v rows_lds_u32x4;

#ifndef TMAC_ROWS_WAVES
#define TMAC_ROWS_WAVES 4
#endif
#ifndef TMAC_ROWS_TARGET_WGS
#define TMAC_ROWS_TARGET_WGS 4096
#endif
constexpr int ROWS_WAVES = TMAC_ROWS_WAVES;  // 64-row tiles per workgroup
constexpr int ROWS_TARGET_WGS = TMAC_ROWS_TARGET_WGS;  // K is split until a call has about this many workgroups
constexpr int ROWS_LDS = 32768;     // bytes of tables per LDS slice: 1024 k for 4 activation rows, 512 k for 8
constexpr int ROWS_NT_WIDE = 8;     // activation rows per workgroup when there are enough of them
constexpr int ROWS_NT_NARROW = 4;   // ... and otherwise

typedef _Float16 rh2v __attribute__((ext_vector_type(2)));
typedef short rs2v __attribute__((ext_vector_type(2)));

struct RowsParams {
  const uint32_t* idx;     // [n_tiles][n_chunks][64][bits] dwords
  const uint32_t* sz;      // [n_tiles][nq][64] {fp16 scale, fp16 zero}
  const uint16_t* tables;  // [n tile][KG][2^g][NT] fp16 or int16: the LDS layout, n tile by n tile
  const void* S;           // [N][nq] fp32 / int32 group sums
  void* out;
  const float* act_scale;
  int64_t ldo;
  int M, N, KG, n_tiles, n_chunks, nq;
  int cpg;                 // 32-k chunks per quantisation group (grouped mode)
  int cpg_log2;            // its logarithm when it is a power of two (the eight-chunk kernel needs one)
  int cps;                 // 32-k chunks per workgroup along K (a multiple of cpg); gridDim.z slices
  int Mp;                  // M rounded up to 64
  float* ws_part;          // split K: [slices][N][Mp] partial sums (fp32, or int32 bit patterns)
  float* ws_srow;          // fused table build, one scale per row or tensor: [slices][N] sums of the
                           // activations of a K slice (fp32, or int32 bit patterns)
  int grouped;             // 1: group scales, 0: one scale per row or per tensor
  int per_tensor, int_exact, icoef;
  float wscale, zero_point, mid;
  const void* A;           // fused table build: activations [N][lda], fp16 or int8 (else unused)
  int64_t lda;
  int K;
  float pw[4];             // plane weights 1, 2, 4, 8: kernel arguments, so that plane 0 also takes the
                           // fused convert-multiply-add (a literal 1.0 would be folded into cvt + add)
  int out_t;
};

// 32-k chunks of tables one LDS slice holds, for LUT group size g and nt activation rows
constexpr int rows_lds_chunks(int g, int nt) { return ROWS_LDS / ((32 / g) * (1 << g) * 2 * nt); }

// a[0] = sum of a[0..N), added pairwise: ((a0 + a1) + (a2 + a3)) + ...
template <typename T, int N>
__device__ __forceinline__ void tree_sum(T (&a)[N]) {
#pragma unroll
  for (int s = 1; s < N; s *= 2) {
#pragma unroll
    for (int i = 0; i + s < N; i += 2 * s) a[i] += a[i + s];
  }
}


template <int NT, int G>
struct RowsShape {
  static constexpr int ENT = 1 << G;          // entries per table
  static constexpr int ES = 2 * NT;           // bytes per entry: NT 16-bit values
  static constexpr int TB = ENT * ES;         // bytes per table
  static constexpr int TPC = 32 / G;          // tables, i.e. lookups per plane, of a 32-k chunk
  static constexpr int CB = TPC * TB;         // bytes per chunk
  static constexpr int HD = NT / 2;           // dwords per entry
};


// Algorithm 1 Precompute for one (activation row, LUT group of four) inside a lookup kernel: the
// eight entries 8h..8h+7 of the table, as four dwords of two 16-bit entries, with the arithmetic
// of the stand-alone precompute kernel ((+-a0 +- a1) + (+-a2 - a3), every addition in fp16;
// entries 8..15 are the negated entries 7..0: mirror consolidation, Section 3.3).
template <bool IS_INT>
__device__ __forceinline__ ru32x4v rows_build_half_table(const void* A, int64_t lda, int n, int kg, int h, bool live) {
  uint32_t low[4];  // entries 0..7
  if constexpr (IS_INT) {
    int a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if (live) {
      const uint32_t v = *reinterpret_cast<const uint32_t*>(static_cast<const int8_t*>(A) + n * lda + 4 * kg);
      a0 = (int8_t)(v & 0xff); a1 = (int8_t)((v >> 8) & 0xff); a2 = (int8_t)((v >> 16) & 0xff); a3 = (int8_t)(v >> 24);
    }
    int e[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) e[q] = ((q & 1) ? a0 : -a0) + ((q & 2) ? a1 : -a1) + ((q & 4) ? a2 : -a2) - a3;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int x = h ? -e[7 - 2 * d] : e[2 * d], y = h ? -e[6 - 2 * d] : e[2 * d + 1];
      low[d] = ((uint32_t)x & 0xffffu) | ((uint32_t)y << 16);
    }
    return ru32x4v{low[0], low[1], low[2], low[3]};
  } else {
    ru32x2v v = {0u, 0u};
    if (live) v = *reinterpret_cast<const ru32x2v*>(static_cast<const __half*>(A) + n * lda + 4 * kg);
    half_table_f16(v.x, v.y, low);
    if (!h) return ru32x4v{low[0], low[1], low[2], low[3]};
    // entries 8 + q = -(entry 7 - q): halves swapped, order reversed, sign bits flipped
    ru32x4v r;
#pragma unroll
    for (int d = 0; d < 4; ++d) r[d] = __builtin_amdgcn_alignbit(low[3 - d], low[3 - d], 16) ^ 0x80008000u;
    return r;
  }
}

// Stage a K slice of tables into LDS: the LUT buffer holds them in the LDS layout, so this is a copy,
// `per` 16-byte pieces per thread, all loads requested before the first store; consecutive lanes
// write consecutive 16 bytes (no bank conflicts).  Tables from kg_end on are written as zeros.
template <int NT, int G, int BYTES>
__device__ __forceinline__ void rows_stage_copy(const RowsParams& p, char* tab, int ntile, int kg0, int kg_end) {
  using Sh = RowsShape<NT, G>;
  constexpr int THREADS = 64 * ROWS_WAVES, PER = BYTES / 16 / THREADS;
  static_assert(PER >= 1 && BYTES % (16 * THREADS) == 0, "whole pieces per thread");
  const char* src = reinterpret_cast<const char*>(p.tables) + ((size_t)ntile * p.KG + (size_t)kg0) * Sh::TB;
  // (pieces of tables from kg_end on read the slice's first piece instead and are zeroed afterwards:
  // no branches between the loads)
  const int live_bytes = max(kg_end - kg0, 0) * Sh::TB;
  ru32x4v v[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int off = (i * THREADS + (int)threadIdx.x) * 16;
    v[i] = *reinterpret_cast<const ru32x4v*>(src + (off < live_bytes ? off : 0));
  }
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int off = (i * THREADS + (int)threadIdx.x) * 16;
    const ru32x4v z = {0u, 0u, 0u, 0u};
    *reinterpret_cast<ru32x4v*>(tab + off) = off < live_bytes ? v[i] : z;
  }
}

// Build and stage tables in one go (tables from the activations, g = 4): item `it` is eight
// consecutive entries (half a table) counted from table kg0, built for the NT activation rows n0..
// and written entry-major [table][entry][n].  Tables from kg_end on are written as zeros.
template <int NT, int G, bool IS_INT>
__device__ __forceinline__ void rows_stage_item(const RowsParams& p, char* tab, int it, int n0, int kg0, int kg_end) {
  using Sh = RowsShape<NT, G>;
  static_assert(G == 4, "tables are built in the kernel for g = 4 only");
  const int flat = it * 8;
  const int kg = kg0 + (flat >> G);
  ru32x4v v[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const bool live = n0 + t < p.N && kg < kg_end && 4 * kg < p.K;
    v[t] = rows_build_half_table<IS_INT>(p.A, p.lda, min(n0 + t, p.N - 1), kg, it & 1, live);
  }
  ru32x4v* dst = reinterpret_cast<ru32x4v*>(tab + flat * Sh::ES);
#pragma unroll
  for (int d = 0; d < 4; ++d) {  // dword d of every row holds entries 2d, 2d+1 of the item
    uint32_t lo[Sh::HD], hi[Sh::HD];
#pragma unroll
    for (int u = 0; u < Sh::HD; ++u) {
      lo[u] = __builtin_amdgcn_perm(v[2 * u + 1][d], v[2 * u][d], 0x05040100u);  // entry 2d: rows 2u, 2u+1
      hi[u] = __builtin_amdgcn_perm(v[2 * u + 1][d], v[2 * u][d], 0x07060302u);  // entry 2d+1
    }
    if constexpr (NT == 4) {
      dst[d] = ru32x4v{lo[0], lo[1], hi[0], hi[1]};
    } else {
      dst[2 * d] = ru32x4v{lo[0], lo[1], lo[2], lo[3]};
      dst[2 * d + 1] = ru32x4v{hi[0], hi[1], hi[2], hi[3]};
    }
  }
}

// The lookups of one 32-k chunk: x = the lane's `BITS` index dwords, cbase = LDS byte address of
// the chunk's first table (low byte zero); L += sum over planes of 2^plane * (sum of the looked-up
// entries), per activation row.
// With OCT = 2 the workgroup serves two sets of NT activation rows whose tables sit OSTRIDE bytes
// apart in LDS: one address (one permute) then feeds two reads, and L holds 2 NT sums.
template <bool IS_INT, int BITS, int NT, int G, typename AccT, int OCT = 1, int OSTRIDE = 0>
__device__ __forceinline__ void rows_chunk(const uint32_t (&x)[BITS], uint32_t cbase, AccT (&L)[NT * OCT],
                                           const float (&pw)[4]) {
  using Sh = RowsShape<NT, G>;
  constexpr int TPC = Sh::TPC, HD = Sh::HD, TB = Sh::TB;
  static_assert(OCT == 1 || (OCT == 2 && NT == 8 && TPC * OCT <= 16), "two row sets: eight rows each, g = 4");
  // rounds of 16 LDS reads (one, two or four planes at g = 2, 4, 8): the hardware counts at
  // most 15 outstanding LDS operations exactly, so a round's reads can be consumed as they return
  constexpr int PL = 16 / (TPC * OCT);
#pragma unroll
  for (int b0 = 0; b0 < BITS; b0 += PL) {
    uint32_t e[PL][TPC][OCT * HD];
#pragma unroll
    for (int bb = 0; bb < PL; ++bb) {
      const int b = b0 + bb;
      if (b >= BITS) break;
      // byte offsets of the entries inside their tables (entry * ES), four tables per dword
      uint32_t off[4];
      if constexpr (G == 4) {
        off[0] = (NT == 4) ? (x[b] << 3) & 0x78787878u : (x[b] << 4) & 0xF0F0F0F0u;  // even tables
        off[1] = (NT == 4) ? (x[b] >> 1) & 0x78787878u : x[b] & 0xF0F0F0F0u;         // odd tables
      } else if constexpr (G == 2) {
        // field r of byte i is table 4 i + r
        if constexpr (NT == 4) {
          off[0] = (x[b] << 3) & 0x18181818u; off[1] = (x[b] << 1) & 0x18181818u;
          off[2] = (x[b] >> 1) & 0x18181818u; off[3] = (x[b] >> 3) & 0x18181818u;
        } else {
          off[0] = (x[b] << 4) & 0x30303030u; off[1] = (x[b] << 2) & 0x30303030u;
          off[2] = x[b] & 0x30303030u;        off[3] = (x[b] >> 2) & 0x30303030u;
        }
      }
#pragma unroll
      for (int j = 0; j < TPC; ++j) {
        uint32_t a;
        if constexpr (G == 8) {
          a = cbase + ((x[b] >> (8 * j)) & 0xffu) * (uint32_t)Sh::ES;
        } else {
          // address = {0, cbase byte 2, cbase byte 1, one byte of the offsets}: one byte permute;
          // the table's own TB * j goes into the instruction's offset field
          constexpr int FPB = 8 / G;  // index fields per byte
          a = __builtin_amdgcn_perm(off[j % FPB], cbase, 0x0C020100u + 4u + (uint32_t)(j / FPB));
        }
        if constexpr (NT == 4) {
          const ru32x2v r = *reinterpret_cast<rows_lds_u32x2*>(a + j * TB);
          e[bb][j][0] = r.x; e[bb][j][1] = r.y;
        } else {
#pragma unroll
          for (int o = 0; o < OCT; ++o) {
            const ru32x4v r = *reinterpret_cast<rows_lds_u32x4*>(a + j * TB + o * OSTRIDE);
            e[bb][j][4 * o + 0] = r.x; e[bb][j][4 * o + 1] = r.y; e[bb][j][4 * o + 2] = r.z; e[bb][j][4 * o + 3] = r.w;
          }
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the reads above the accumulation
    // The entries of a plane (one per table of the chunk) are added pairwise as packed 16-bit
    // values, two activation rows per instruction: exact for the integer tables (|sum| <= 4096),
    // log2(32/g) roundings to fp16 for the fp16 tables (lossy, this library's choice: the widening
    // happens once per chunk and plane); the chunk sum then enters the 32-bit sum of the
    // quantisation group times 2^plane.
#pragma unroll
    for (int bb = 0; bb < PL; ++bb) {
      const int b = b0 + bb;
      if (b >= BITS) break;
#pragma unroll
      for (int u = 0; u < OCT * HD; ++u) {
        if constexpr (IS_INT) {
          rs2v q[TPC];
#pragma unroll
          for (int j = 0; j < TPC; ++j) q[j] = __builtin_bit_cast(rs2v, e[bb][j][u]);
          tree_sum(q);
          L[2 * u] += (int)q[0].x << b;
          L[2 * u + 1] += (int)q[0].y << b;
        } else {
          rh2v q[TPC];
#pragma unroll
          for (int j = 0; j < TPC; ++j) q[j] = __builtin_bit_cast(rh2v, e[bb][j][u]);
          tree_sum(q);
          const float w = pw[b];
          L[2 * u] = fmaf((float)q[0].x, w, L[2 * u]);
          L[2 * u + 1] = fmaf((float)q[0].y, w, L[2 * u + 1]);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Scale of activation row n (int8 activations quantised per token), 1 where there is none.
__device__ __forceinline__ float rows_act_scale(const RowsParams& p, int n) { return p.act_scale ? p.act_scale[n] : 1.0f; }

// Sum of activation row n from the LUT buffer (one scale per row or per tensor: nq = 1).
template <bool IS_INT>
__device__ __forceinline__ void rows_row_sum(const RowsParams& p, int n, float& Sf, int& Si) {
  Sf = 0.f;
  Si = 0;
  if (p.grouped) return;
  if constexpr (IS_INT) Si = static_cast<const int*>(p.S)[n];
  else Sf = static_cast<const float*>(p.S)[n];
}

// Last step for output (n, m): vf = finished group sums (group scales) or the raw look-up sum (fp
// tables), vi = the raw integer look-up sum; s, z = scale and zero of row m when there is one
// scale per row or per tensor; Sf / Si = the sum of activation row n in that case.
template <bool IS_INT>
__device__ __forceinline__ void rows_finish(const RowsParams& p, int n, int m, float vf, int vi, float s, float z,
                                            float Sf, int Si, float as) {
  float res;
  int ires = 0;
  if (p.grouped) {
    res = vf * as;
  } else if constexpr (IS_INT) {
    const int St = Si;
    if (p.int_exact) {
      ires = (vi + p.icoef * St) >> 1;  // numerator is always even
      res = ((float)ires * as) * s;     // two roundings, left to right
    } else {
      res = (fmaf(p.mid - z, (float)St, 0.5f * (float)vi) * as) * s;
    }
  } else {
    const float St = Sf;
    res = (s * fmaf(p.mid - z, St, 0.5f * vf)) * as;
  }
  const size_t o = (size_t)n * p.ldo + m;
  if (p.out_t == TMAC_OUT_F32) static_cast<float*>(p.out)[o] = res;
  else if (p.out_t == TMAC_OUT_F16) static_cast<__half*>(p.out)[o] = __float2half_rn(res);
  else static_cast<int*>(p.out)[o] = ires;
}


// OCT = 2: the workgroup serves two n tiles of NT = 8 activation rows (their tables side by side in
// the two halves of the LDS slice), so that one address permute feeds two reads; the LUT buffer's
// n tiles stay eight rows wide.
template <bool IS_INT, int BITS, int NT, int G, int OCT>
__global__ __launch_bounds__(64 * ROWS_WAVES) void mpgemm_rows_kernel(const RowsParams p) {
  using Sh = RowsShape<NT, G>;
  constexpr int TPC = Sh::TPC, CB = Sh::CB;
  constexpr int CPS = rows_lds_chunks(G, NT) / OCT;  // 32-k chunks per slice
  constexpr int NTT = NT * OCT;                      // activation rows of the workgroup
  constexpr int OSTRIDE = ROWS_LDS / OCT;            // bytes between the two row sets' tables
  static_assert(CPS >= 1 && CB % 256 == 0, "chunk bases must keep a zero low byte");
  __shared__ __attribute__((aligned(2048))) char tab[ROWS_LDS];  // byte-permuted addresses need the alignment
  using AccT = typename std::conditional<IS_INT, int, float>::type;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n0 = blockIdx.x * NTT;                      // activation rows of this workgroup
  const int tile_raw = blockIdx.y * ROWS_WAVES + wave;  // 64-row tile of this wave
  const bool tile_ok = tile_raw < p.n_tiles;
  const int tile = tile_ok ? tile_raw : p.n_tiles - 1;  // clamped: loads stay in range, stores are masked
  const uint32_t* my_idx = p.idx + ((size_t)tile * p.n_chunks * 64 + lane) * BITS;
  const uint32_t* my_sz = p.sz + (size_t)tile * p.nq * 64 + lane;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((rows_lds_char*)tab);  // a multiple of 1024

  // fp tables: L is the running result, the plane weights w carry half the current group's scale and
  // the group's bias term is added when the group starts; integer tables (and one scale per row or
  // tensor): L is the raw look-up sum of the group (row), finished in acc at the group's end
  float acc[NTT];
  AccT L[NTT];
#pragma unroll
  for (int t = 0; t < NTT; ++t) { acc[t] = 0.f; L[t] = 0; }
  float w[4] = {p.pw[0], p.pw[1], p.pw[2], p.pw[3]};

  auto load_idx = [&](int c, uint32_t (&x)[BITS]) {
    const uint32_t* src = my_idx + (size_t)c * 64 * BITS;
    if constexpr (BITS == 4) {
      const ru32x4v v = *reinterpret_cast<const ru32x4v*>(src);
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else if constexpr (BITS == 2) {
      const ru32x2v v = *reinterpret_cast<const ru32x2v*>(src);
      x[0] = v.x; x[1] = v.y;
    } else {
#pragma unroll
      for (int b = 0; b < BITS; ++b) x[b] = src[b];
    }
  };

  // this workgroup's share of K: chunks [cz0, cz1)
  const int cz0 = blockIdx.z * p.cps, cz1 = min(cz0 + p.cps, p.n_chunks);
  const int kg_end = min(cz1 * TPC, p.KG);  // tables beyond it are read as zero
  int gq = p.grouped ? cz0 / p.cpg : 0, cg = 0;  // current quantisation group, chunks done in it (wave-uniform)
  // {scale, zero} of the lane's row and the activation sums of a group, requested one group ahead
  uint32_t szv = 0, szv_next = 0;
  float Sg[NTT], Sg_next[NTT];
  auto load_group = [&](int g) {
    const int gc = min(g, p.nq - 1);
    szv_next = my_sz[(size_t)gc * 64];
#pragma unroll
    for (int t = 0; t < NTT; ++t) {
      const int n = min(n0 + t, p.N - 1);
      if constexpr (IS_INT) Sg_next[t] = (float)static_cast<const int*>(p.S)[(size_t)n * p.nq + gc];
      else Sg_next[t] = static_cast<const float*>(p.S)[(size_t)n * p.nq + gc];
    }
  };
#pragma unroll
  for (int t = 0; t < NTT; ++t) Sg[t] = Sg_next[t] = 0.f;
  if (p.grouped) load_group(gq);
  uint32_t xn[BITS];
  load_idx(cz0, xn);

  for (int c0 = cz0; c0 < cz1; c0 += CPS) {
    // stage the tables of this K-slice for the NT activation rows: item = (table, half) reads the
    // 8 entries of the four rows and writes them entry-major
    __syncthreads();
    {
      const int last8 = (p.N + NT - 1) / NT - 1;  // last n tile of the LUT buffer (a second row set past it repeats it)
#pragma unroll
      for (int o = 0; o < OCT; ++o)
        rows_stage_copy<NT, G, OSTRIDE>(p, tab + o * OSTRIDE, min((int)blockIdx.x * OCT + o, last8), c0 * TPC, kg_end);
    }
    __syncthreads();

    const int c_end = min(c0 + CPS, cz1);
    // Per chunk and pair of bit planes: 16 LDS reads are issued first, then accumulated in issue
    // order, so that the reads overlap each other and the accumulation of the earlier ones; the
    // other waves of the SIMD cover the start of every round.
    for (int c = c0; c < c_end; ++c) {
      uint32_t x[BITS];
#pragma unroll
      for (int b = 0; b < BITS; ++b) x[b] = xn[b];
      if (c + 1 < cz1) load_idx(c + 1, xn);  // next chunk's indices, one chunk ahead
      if (p.grouped && cg == 0 && gq < p.nq) {  // (chunks in the K padding belong to no group)
        // a group starts: its scale/zero and activation sums have been requested a group ago
        szv = szv_next;
#pragma unroll
        for (int t = 0; t < NTT; ++t) Sg[t] = Sg_next[t];
        if constexpr (!IS_INT) {
          const float s = __half2float(__ushort_as_half((uint16_t)(szv & 0xffffu)));
          const float z = __half2float(__ushort_as_half((uint16_t)(szv >> 16)));
          const float hs = 0.5f * s, bz = s * (p.mid - z);
#pragma unroll
          for (int b = 0; b < 4; ++b) w[b] = hs * p.pw[b];
#pragma unroll
          for (int t = 0; t < NTT; ++t) L[t] = fmaf(bz, Sg[t], L[t]);  // bias term of Section 4's linear transform
        }
        // (the requests for the next group come after the last use of this group's values, so that they
        // can land in the same registers and nobody has to wait for them before the next group starts)
        __builtin_amdgcn_sched_barrier(0);
        load_group(gq + 1);
      }
      rows_chunk<IS_INT, BITS, NT, G, AccT, OCT, OSTRIDE>(x, lds0 + (uint32_t)(c - c0) * (uint32_t)CB, L, w);
      if (p.grouped && gq < p.nq && ++cg == p.cpg) {
        if constexpr (IS_INT) {
          const float s = __half2float(__ushort_as_half((uint16_t)(szv & 0xffffu)));
          const float z = __half2float(__ushort_as_half((uint16_t)(szv >> 16)));
#pragma unroll
          for (int t = 0; t < NTT; ++t) {
            acc[t] = fmaf(s, fmaf(p.mid - z, Sg[t], 0.5f * (float)L[t]), acc[t]);
            L[t] = 0;
          }
        }
        cg = 0;
        ++gq;
      }
    }
  }

  // finish and store: lanes of a wave write 64 consecutive outputs of one activation row
  const int m = tile_raw * 64 + lane;
  const bool row_ok = tile_ok && m < p.M;
  float s = p.wscale, z = p.zero_point;
  if (!p.grouped && !p.per_tensor) {
    const uint32_t v = my_sz[0];
    s = __half2float(__ushort_as_half((uint16_t)(v & 0xffffu)));
    z = __half2float(__ushort_as_half((uint16_t)(v >> 16)));
  }
  auto finish = [&](int n, float vf, int vi) {
    float Sf;
    int Si;
    rows_row_sum<IS_INT>(p, n, Sf, Si);
    rows_finish<IS_INT>(p, n, m, vf, vi, s, z, Sf, Si, rows_act_scale(p, n));
  };
  constexpr bool RAW_INT = IS_INT;  // ungrouped integer tables: partial sums are exact integers
  const int nz = gridDim.z;
  if (nz == 1) {
    if (!row_ok) return;
#pragma unroll
    for (int t = 0; t < NTT; ++t) {
      if (n0 + t >= p.N) break;
      finish(n0 + t, (IS_INT && p.grouped) ? acc[t] : (float)L[t], IS_INT ? (int)L[t] : 0);
    }
    return;
  }

  // Split K: publish the partial sums with plain stores; rows_sum_kernel, launched behind this
  // kernel on the same stream, adds the slices in slice order and finishes.  The kernel boundary
  // orders the stores before the loads on every XCD (one L2 each); handing over inside the kernel
  // instead (release fence, arrival counter, acquire fence in the last workgroup) makes every
  // workgroup write back its L2, which cost more than the second launch at every size tried.
  const bool raw_int = RAW_INT && !p.grouped;
  if (tile_ok) {
#pragma unroll
    for (int t = 0; t < NTT; ++t) {
      const int n = n0 + t;
      if (n < p.N) {
        const size_t o = ((size_t)blockIdx.z * p.N + n) * p.Mp + (size_t)tile_raw * 64 + lane;
        p.ws_part[o] = (IS_INT && p.grouped) ? acc[t] : (raw_int ? __int_as_float((int)L[t]) : (float)L[t]);
      }
    }
  }
}

template <bool IS_INT>
__global__ void rows_sum_kernel(const RowsParams p, int nz);

template <bool IS_INT, int BITS, int NT, int G, int OCT>
static hipError_t launch_rows_one(const RowsParams& p, hipStream_t st) {
  RowsParams local = p;
  void* args[] = {&local};
  const dim3 grid((p.N + NT * OCT - 1) / (NT * OCT), (p.n_tiles + ROWS_WAVES - 1) / ROWS_WAVES,
                  (p.n_chunks + p.cps - 1) / p.cps);
  hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(mpgemm_rows_kernel<IS_INT, BITS, NT, G, OCT>), grid,
                                 dim3(64 * ROWS_WAVES), args, 0, st);
  int nz = (int)grid.z;
  if (e != hipSuccess || nz == 1) return e;
  void* args2[] = {&local, &nz};
  return hipLaunchKernel(reinterpret_cast<const void*>(rows_sum_kernel<IS_INT>), dim3((p.M + 63) / 64, p.N),
                         dim3(64), args2, 0, st);
}

template <bool IS_INT, int NT, int G, int OCT = 1>
static hipError_t launch_rows_bits(const RowsParams& p, int bits, hipStream_t st) {
  switch (bits) {
    case 1: return launch_rows_one<IS_INT, 1, NT, G, OCT>(p, st);
    case 2: return launch_rows_one<IS_INT, 2, NT, G, OCT>(p, st);
    case 3: return launch_rows_one<IS_INT, 3, NT, G, OCT>(p, st);
    case 4: return launch_rows_one<IS_INT, 4, NT, G, OCT>(p, st);
  }
  return hipErrorInvalidValue;
}

// oct: n tiles per workgroup (2 only with g = 4 and eight-row n tiles)
template <bool IS_INT>
static hipError_t launch_rows_nt(const RowsParams& p, int g, int nt, int oct, int bits, hipStream_t st) {
  if (g == 8) return launch_rows_bits<IS_INT, ROWS_NT_NARROW, 8>(p, bits, st);  // (rows_nt: always narrow)
  if (g == 2)
    return nt == ROWS_NT_WIDE ? launch_rows_bits<IS_INT, ROWS_NT_WIDE, 2>(p, bits, st)
                              : launch_rows_bits<IS_INT, ROWS_NT_NARROW, 2>(p, bits, st);
  if (oct == 2) return launch_rows_bits<IS_INT, ROWS_NT_WIDE, 4, 2>(p, bits, st);
  return nt == ROWS_NT_WIDE ? launch_rows_bits<IS_INT, ROWS_NT_WIDE, 4>(p, bits, st)
                            : launch_rows_bits<IS_INT, ROWS_NT_NARROW, 4>(p, bits, st);
}


// ------------------------------------------------------------------------------------------
// Few activation rows: one slice of eight chunks per workgroup, sums finished by a second kernel
// ------------------------------------------------------------------------------------------
// With few activation rows a call is a chain of latencies, not a stream: the general kernel above
// asks for a chunk's indices one chunk ahead.  Here the share of a workgroup is fixed at eight
// chunks (256 k, g = 4), so that every global load it will ever need (indices of all eight chunks,
// scales and zeros, tables, group sums) is requested in one go at the start, the chunk loop is
// straight-line code, and the partial sums are written with plain stores; rows_sum_kernel, the
// next kernel on the stream, adds the slices in slice order and finishes.
constexpr int R8_CH = 8;

// Which (n tile, row block, K slice) a workgroup serves.  The hardware hands workgroups to the
// chip's eight XCDs (one L2 each) round-robin by linear id; with the plain blockIdx mapping the
// n tiles that share a block of packed indices would sit on eight different L2s and each would
// fetch the block from memory.  Here the (row block, K slice) groups go round-robin over the XCDs
// and the n tiles of a group follow each other on one XCD, so a block of indices is fetched once
// (measured: 74 -> 26 MB fetched at 64 activation rows of a 4096 x 4096 4-bit matrix, same time;
// the general kernel keeps the plain order, where the same remapping trades index re-reads for
// table re-reads and changes neither bytes nor time).
struct RowsUnit {
  int nt, rb, kz;
};
__device__ __forceinline__ RowsUnit rows_unit() {
  const uint32_t gx = gridDim.x, gy = gridDim.y, groups = gy * gridDim.z;
  const uint32_t lin = (blockIdx.z * gy + blockIdx.y) * gx + blockIdx.x;
  const uint32_t whole = (groups & ~7u) * gx;  // ids of the groups that fill all eight XCDs evenly
  uint32_t grp = lin / gx, nt = lin % gx;      // the few groups left over keep the plain order
  if (lin < whole) {
    const uint32_t xcd = lin & 7u, slot = lin >> 3;
    grp = xcd + 8u * (slot / gx);
    nt = slot % gx;
  }
  RowsUnit r;
  r.nt = (int)nt;
  r.rb = (int)(grp % gy);
  r.kz = (int)(grp / gy);
  return r;
}


template <bool IS_INT, int BITS, int NT, bool FUSED>
__global__ __launch_bounds__(64 * ROWS_WAVES) void mpgemm_rows8_kernel(const RowsParams p) {
  static_assert(ROWS_WAVES * 64 >= 32 * NT, "one thread per eight activations of the slice");
  constexpr int G = 4;
  using Sh = RowsShape<NT, G>;
  __shared__ __attribute__((aligned(2048))) char tab[R8_CH * Sh::CB];
  __shared__ float sS[R8_CH][NT];  // per chunk: the sum of activations of its quantisation group
  using AccT = typename std::conditional<IS_INT, int, float>::type;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const RowsUnit un = rows_unit();
  const int n0 = un.nt * NT;
  const int tile_raw = un.rb * ROWS_WAVES + wave;
  const bool tile_ok = tile_raw < p.n_tiles;
  const int tile = tile_ok ? tile_raw : p.n_tiles - 1;  // clamped: loads stay in range, stores are masked
  const uint32_t* my_idx = p.idx + ((size_t)tile * p.n_chunks * 64 + lane) * BITS;
  const uint32_t* my_sz = p.sz + (size_t)tile * p.nq * 64 + lane;
  const uint32_t lds0 = (uint32_t)(uintptr_t)((rows_lds_char*)tab);
  const int cz0 = un.kz * R8_CH;
  const int nc = min(R8_CH, p.n_chunks - cz0);  // chunks of this workgroup (at least one)

  // 1. all global loads, unconditional (clamped addresses): indices, {scale, zero} of every chunk's group
  uint32_t x[R8_CH][BITS];
#pragma unroll
  for (int c = 0; c < R8_CH; ++c) {
    const uint32_t* src = my_idx + (size_t)min(cz0 + c, p.n_chunks - 1) * 64 * BITS;
    if constexpr (BITS == 4) {
      const ru32x4v v = *reinterpret_cast<const ru32x4v*>(src);
      x[c][0] = v.x; x[c][1] = v.y; x[c][2] = v.z; x[c][3] = v.w;
    } else if constexpr (BITS == 2) {
      const ru32x2v v = *reinterpret_cast<const ru32x2v*>(src);
      x[c][0] = v.x; x[c][1] = v.y;
    } else {
#pragma unroll
      for (int b = 0; b < BITS; ++b) x[c][b] = src[b];
    }
  }
  uint32_t szv[R8_CH];
#pragma unroll
  for (int c = 0; c < R8_CH; ++c) {
    const int gq = p.grouped ? min((cz0 + c) >> p.cpg_log2, p.nq - 1) : 0;
    szv[c] = (p.grouped || !p.per_tensor) ? my_sz[(size_t)gq * 64] : 0u;
  }

  // 2. tables of the eight chunks, and the group sums, into LDS
  const int kg_end = min((cz0 + nc) * Sh::TPC, p.KG);
  if constexpr (FUSED) {
    // sums of the quantisation groups of the slice, from the activations: thread
    // i takes eight activations of row i / 32, the 4 cpg threads of a group add up by butterfly
    // (they sit in one half of a wavefront), and one thread per chunk publishes the group's sum
    const int t = threadIdx.x >> 5, seg = threadIdx.x & 31;
    float ssum = 0.f;
    const int n = n0 + t, k0 = (cz0 << 5) + 8 * seg;
    if (t < NT && n < p.N && k0 < p.K) {
      if constexpr (IS_INT) {
        const ru32x2v v = *reinterpret_cast<const ru32x2v*>(static_cast<const int8_t*>(p.A) + n * p.lda + k0);
        int si = __builtin_amdgcn_sdot4((int)v.x, 0x01010101, 0, false);
        si = __builtin_amdgcn_sdot4((int)v.y, 0x01010101, si, false);
        ssum = (float)si;  // sums of a group stay below 2^24: exact
      } else {
        const ru32x4v v = *reinterpret_cast<const ru32x4v*>(static_cast<const __half*>(p.A) + n * p.lda + k0);
        float f[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = __half2float(__ushort_as_half((uint16_t)(v[i >> 1] >> (16 * (i & 1)))));
        ssum = ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
      }
    }
    // (one scale per row or per tensor: the whole slice's sum per row, for rows_sum_kernel)
    const int span = p.grouped ? (4 << p.cpg_log2) : 32;
    for (int o = 1; o < span; o <<= 1) ssum += __shfl_xor(ssum, o);
    if (p.grouped) {
      if (t < NT && (seg & 3) == 0) sS[seg >> 2][t] = ssum;
    } else if (un.rb == 0 && t < NT && n < p.N && seg == 0) {
      p.ws_srow[(size_t)un.kz * p.N + n] = IS_INT ? __int_as_float((int)ssum) : ssum;
    }
    for (int it = threadIdx.x; it < R8_CH * Sh::CB / (8 * Sh::ES); it += 64 * ROWS_WAVES)
      rows_stage_item<NT, G, IS_INT>(p, tab, it, n0, cz0 * Sh::TPC, kg_end);
  } else {
  rows_stage_copy<NT, G, R8_CH * Sh::CB>(p, tab, un.nt, cz0 * Sh::TPC, kg_end);
  if (p.grouped && threadIdx.x < R8_CH * NT) {
    const int c = threadIdx.x / NT, t = threadIdx.x % NT;
    const int gq = min((cz0 + c) >> p.cpg_log2, p.nq - 1);
    const int n = min(n0 + t, p.N - 1);
    if constexpr (IS_INT) sS[c][t] = (float)static_cast<const int*>(p.S)[(size_t)n * p.nq + gq];
    else sS[c][t] = static_cast<const float*>(p.S)[(size_t)n * p.nq + gq];
  }
  }
  __syncthreads();

  // 3. the chunks, straight-line
  float acc[NT];
  AccT L[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) { acc[t] = 0.f; L[t] = 0; }
  const int cmask = (1 << p.cpg_log2) - 1;
#pragma unroll
  for (int c = 0; c < R8_CH; ++c) {
    if (c < nc) {
      rows_chunk<IS_INT, BITS, NT, G>(x[c], lds0 + (uint32_t)c * (uint32_t)Sh::CB, L, p.pw);
      // a quantisation group ends with this chunk (chunks in the K padding belong to no group)
      if (p.grouped && ((cz0 + c + 1) & cmask) == 0 && ((cz0 + c) >> p.cpg_log2) < p.nq) {
        const float s = __half2float(__ushort_as_half((uint16_t)(szv[c] & 0xffffu)));
        const float z = __half2float(__ushort_as_half((uint16_t)(szv[c] >> 16)));
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          acc[t] = fmaf(s, fmaf(p.mid - z, sS[c][t], 0.5f * (float)L[t]), acc[t]);
          L[t] = 0;
        }
      }
    }
  }

  // 4. one slice: finish here; several: publish the partial sums for rows_sum_kernel
  const int m = tile_raw * 64 + lane;
  if (gridDim.z == 1) {
    if (!tile_ok || m >= p.M) return;
    float s = p.wscale, z = p.zero_point;
    if (!p.grouped && !p.per_tensor) {
      s = __half2float(__ushort_as_half((uint16_t)(szv[0] & 0xffffu)));
      z = __half2float(__ushort_as_half((uint16_t)(szv[0] >> 16)));
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (n0 + t >= p.N) break;
      float Sf;
      int Si;
      rows_row_sum<IS_INT>(p, n0 + t, Sf, Si);
      rows_finish<IS_INT>(p, n0 + t, m, p.grouped ? acc[t] : (float)L[t], IS_INT ? (int)L[t] : 0, s, z, Sf, Si,
                          rows_act_scale(p, n0 + t));
    }
    return;
  }
  if (!tile_ok) return;
  const bool raw_int = IS_INT && !p.grouped;  // ungrouped integer tables: partial sums are exact integers
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = n0 + t;
    if (n < p.N) {
      const size_t o = ((size_t)un.kz * p.N + n) * p.Mp + (size_t)m;
      p.ws_part[o] = p.grouped ? acc[t] : (raw_int ? __int_as_float((int)L[t]) : (float)L[t]);
    }
  }
}

// Adds the partial sums [nz][N][Mp] of the K slices in slice order and finishes: one thread per
// output.  Everything the thread needs is requested before the first wait (scale and zero, the
// activation scale, the row sum or its per-slice parts, sixteen partial sums per round), so that a
// call pays one round trip to memory, not one per operand.
template <bool IS_INT>
__global__ __launch_bounds__(64) void rows_sum_kernel(const RowsParams p, int nz) {
  const int m = blockIdx.x * 64 + threadIdx.x, n = blockIdx.y;
  if (m >= p.M) return;
  const bool raw_int = IS_INT && !p.grouped;
  const float* src = p.ws_part + (size_t)n * p.Mp + m;
  const size_t stride = (size_t)p.N * p.Mp;
  const bool own_sz = !p.grouped && !p.per_tensor;
  const uint32_t szv = own_sz ? p.sz[(size_t)(m >> 6) * p.nq * 64 + (m & 63)] : 0u;
  const float as = rows_act_scale(p, n);
  // fused table build: the row sum is the sum of the slices' sums, taken in slice order below
  const bool slice_sums = !p.grouped && p.ws_srow != nullptr;
  float Sf = 0.f;
  int Si = 0;
  if (!p.grouped && !slice_sums) rows_row_sum<IS_INT>(p, n, Sf, Si);
  float sf = 0.f;
  int si = 0;
  for (int sl0 = 0; sl0 < nz; sl0 += 16) {
    float v[16], r[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int sl = min(sl0 + u, nz - 1);
      v[u] = src[(size_t)sl * stride];
      r[u] = slice_sums ? p.ws_srow[(size_t)sl * p.N + n] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if (sl0 + u < nz) {
        if (raw_int) si += __float_as_int(v[u]);
        else sf += v[u];
        if constexpr (IS_INT) Si += slice_sums ? __float_as_int(r[u]) : 0;
        else Sf += r[u];
      }
    }
  }
  float s = p.wscale, z = p.zero_point;
  if (own_sz) {
    s = __half2float(__ushort_as_half((uint16_t)(szv & 0xffffu)));
    z = __half2float(__ushort_as_half((uint16_t)(szv >> 16)));
  }
  rows_finish<IS_INT>(p, n, m, sf, si, s, z, Sf, Si, as);
}

template <bool IS_INT, int BITS, int NT, bool FUSED>
static hipError_t launch_rows8_one(const RowsParams& p, hipStream_t st) {
  RowsParams local = p;
  int nz = (p.n_chunks + R8_CH - 1) / R8_CH;
  void* args[] = {&local};
  const dim3 grid((p.N + NT - 1) / NT, (p.n_tiles + ROWS_WAVES - 1) / ROWS_WAVES, nz);
  hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(mpgemm_rows8_kernel<IS_INT, BITS, NT, FUSED>), grid,
                                 dim3(64 * ROWS_WAVES), args, 0, st);
  if (e != hipSuccess || nz == 1) return e;
  void* args2[] = {&local, &nz};
  return hipLaunchKernel(reinterpret_cast<const void*>(rows_sum_kernel<IS_INT>), dim3((p.M + 63) / 64, p.N),
                         dim3(64), args2, 0, st);
}

template <bool IS_INT, int NT, bool FUSED>
static hipError_t launch_rows8_bits(const RowsParams& p, int bits, hipStream_t st) {
  switch (bits) {
    case 1: return launch_rows8_one<IS_INT, 1, NT, FUSED>(p, st);
    case 2: return launch_rows8_one<IS_INT, 2, NT, FUSED>(p, st);
    case 3: return launch_rows8_one<IS_INT, 3, NT, FUSED>(p, st);
    case 4: return launch_rows8_one<IS_INT, 4, NT, FUSED>(p, st);
  }
  return hipErrorInvalidValue;
}

template <bool IS_INT, bool FUSED = false>
static hipError_t launch_rows8_nt(const RowsParams& p, int nt, int bits, hipStream_t st) {
  return nt == ROWS_NT_WIDE ? launch_rows8_bits<IS_INT, ROWS_NT_WIDE, FUSED>(p, bits, st)
                            : launch_rows8_bits<IS_INT, ROWS_NT_NARROW, FUSED>(p, bits, st);
}

// How a call is split: workgroups along N and M, and the number of K slices (1 when the (row block,
// n tile) pairs alone fill the chip; otherwise enough slices of at least 256 k, whole quantisation
// groups each, to give about two workgroups per CU).
// The plan with `oct` n tiles per workgroup.
static RowsPlan rows_plan_oct(const tmac_wdesc* desc, int N, int oct) {
  const Geometry ge = geometry(desc);
  RowsPlan pl;
  pl.row_blocks = (ge.n_tiles + ROWS_WAVES - 1) / ROWS_WAVES;
  pl.nt = rows_nt(N, desc->g);
  pl.oct = oct;
  pl.n_tiles_n = (N + pl.nt * pl.oct - 1) / (pl.nt * pl.oct);
  const bool one_group = (desc->group == 0 || desc->group == desc->K);
  const int cpg = (one_group || desc->group < 32) ? 1 : desc->group / 32;  // (sizes below 32 are rejected at launch)
  const int min_cps = (8 + cpg - 1) / cpg * cpg;  // at least 256 k, whole groups
  const int64_t pairs = (int64_t)pl.n_tiles_n * pl.row_blocks;
  int64_t want = pairs >= ROWS_TARGET_WGS ? 1 : (ROWS_TARGET_WGS + pairs - 1) / pairs;
  const int max_slices = (ge.n_chunks + min_cps - 1) / min_cps;
  if (want > max_slices) want = max_slices;
  int cps = (int)((ge.n_chunks + want - 1) / want);
  // whole LDS slices where a workgroup gets at least one (nothing staged in vain), whole groups always
  const int lds_chunks = rows_lds_chunks(desc->g, pl.nt) / pl.oct;
  int unit = cpg;
  if (want > 1 && cps >= lds_chunks) {
    unit = lds_chunks;
    while (unit % cpg) unit += lds_chunks;
  }
  cps = (cps + unit - 1) / unit * unit;
  if (cps < min_cps) cps = min_cps;
  pl.cps = cps;
  // eight-chunk slices, several of them, g = 4, a group size that divides 256 (or no groups):
  // the kernel pair for few activation rows
  pl.eight = pl.oct == 1 && desc->g == 4 && cps == R8_CH && ge.n_chunks > R8_CH && (one_group || R8_CH % cpg == 0);
  pl.slices = (ge.n_chunks + cps - 1) / cps;
  pl.part_bytes = pl.slices > 1 ? ((size_t)pl.slices * N * ge.Mp * 4 + 255) / 256 * 256 : 0;
  pl.ctr_bytes = 0;  // (no arrival counters: the slices meet in rows_sum_kernel)
  pl.srow_bytes = pl.eight ? ((size_t)pl.slices * N * 4 + 255) / 256 * 256 : 0;
  return pl;
}

// Many activation rows at g = 4: a workgroup takes two n tiles (16 rows), one address permute per two
// reads.  Measured against one n tile per workgroup (precompute + lookup, 4 bit): 13824 x 5120 even
// at 48 rows, 7 % ahead at 64, 9 % at 96, 6 % at 128 and beyond; 4096 x 4096, where the eight-chunk
// kernel pair serves up to 192 rows, behind below 96 rows, even at 96, 4 % ahead at 128.
RowsPlan rows_plan(const tmac_wdesc* desc, int N) {
  const RowsPlan one = rows_plan_oct(desc, N, 1);
  const bool can = desc->g == 4 && one.nt == ROWS_NT_WIDE;
  if (can && (N >= 128 || (N >= 64 && !one.eight))) return rows_plan_oct(desc, N, 2);
  return one;
}

// Whether a call builds its tables inside the lookup kernel when it is given activations instead
// of a LUT buffer: the eight-chunk kernel, up to 32 activation rows (every
// block of 256 weight rows builds the tables again: from 64 rows on that costs more than the
// launch of the precompute kernel it saves).
bool rows_builds_tables(const tmac_wdesc* desc, int N) {
  return N <= 32 && desc->K % 8 == 0 && rows_plan(desc, N).eight;  // (activations are summed eight at a time)
}

// lut_dev: buffer of tmac_precompute_lut, or NULL with A_dev / lda given (only where
// rows_builds_tables says so).
int launch_rows_gemm(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
                     int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale, void* out_dev,
                     int out_t, int64_t ldo, void* workspace_dev, size_t workspace_bytes, void* stream) {
  if (lut_t != TMAC_LUT_F16 && lut_t != TMAC_LUT_I16) return TMAC_EUNSUPPORTED;
  const bool fused = (lut_dev == nullptr);
  if (fused && (!A_dev || !rows_builds_tables(desc, N))) return TMAC_EUNSUPPORTED;
  const Geometry ge = geometry(desc);
  LutGeom lg;
  if (!lut_geom(N, desc->K, desc->g, desc->group, lut_t, &lg)) return TMAC_EINVAL;
  const bool is_int = (lut_t == TMAC_LUT_I16);
  const bool one_group = (desc->group == 0 || desc->group == desc->K);
  const RowsPlan pl = rows_plan(desc, N);
  if (pl.n_tiles_n > 0x7fffffff || pl.row_blocks > 65535 || pl.slices > 65535) return TMAC_EUNSUPPORTED;
  if (pl.slices > 1) {
    if (!workspace_dev) return TMAC_EINVAL;
    if (workspace_bytes < pl.part_bytes + pl.ctr_bytes + pl.srow_bytes) return TMAC_ESIZE;
  }
  // int32 accumulators: |L| <= 128 * (2^b - 1) * K must stay below 2^31
  if (is_int && (double)128.0 * ((1 << desc->bits) - 1) * desc->K >= 2147483647.0) return TMAC_EUNSUPPORTED;

  RowsParams p;
  const char* blob = static_cast<const char*>(packed_dev);
  p.idx = reinterpret_cast<const uint32_t*>(blob + ge.idx_off);
  p.sz = reinterpret_cast<const uint32_t*>(blob + ge.sz_off);
  p.tables = static_cast<const uint16_t*>(lut_dev);
  p.S = fused ? nullptr : static_cast<const char*>(lut_dev) + lg.s_off;
  p.A = A_dev;
  p.lda = lda;
  p.K = desc->K;
  p.out = out_dev;
  p.act_scale = act_scale_dev;
  p.ldo = ldo;
  p.M = desc->M; p.N = N; p.KG = lg.KG; p.n_tiles = ge.n_tiles; p.n_chunks = ge.n_chunks; p.nq = lg.nq;
  p.grouped = one_group ? 0 : 1;
  p.cpg = one_group ? 1 : desc->group / 32;
  p.cpg_log2 = 0;
  while ((2 << p.cpg_log2) <= p.cpg) ++p.cpg_log2;
  p.cps = pl.cps;
  p.Mp = ge.Mp;
  p.ws_part = static_cast<float*>(workspace_dev);
  p.ws_srow = (fused && one_group) ? reinterpret_cast<float*>(static_cast<char*>(workspace_dev) + pl.part_bytes + pl.ctr_bytes)
                                   : nullptr;
  p.per_tensor = (desc->group == 0);
  p.wscale = weight_scale;
  p.mid = 0.5f * (float)((1 << desc->bits) - 1);
  p.zero_point = p.per_tensor ? desc->zero_point : 0.f;
  p.int_exact = 0;
  p.icoef = 0;
  p.out_t = out_t;
  p.pw[0] = 1.f; p.pw[1] = 2.f; p.pw[2] = 4.f; p.pw[3] = 8.f;
  if (p.per_tensor && is_int) {
    const float z = desc->zero_point;
    if (z == rintf(z) && fabsf(z) < 64.f) {
      p.int_exact = 1;
      p.icoef = ((1 << desc->bits) - 1) - 2 * (int)z;
    }
  }
  if (out_t == TMAC_OUT_I32 && !p.int_exact) return TMAC_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (fused) e = is_int ? launch_rows8_nt<true, true>(p, pl.nt, desc->bits, st) : launch_rows8_nt<false, true>(p, pl.nt, desc->bits, st);
  else if (pl.eight) e = is_int ? launch_rows8_nt<true>(p, pl.nt, desc->bits, st) : launch_rows8_nt<false>(p, pl.nt, desc->bits, st);
  else e = is_int ? launch_rows_nt<true>(p, desc->g, pl.nt, pl.oct, desc->bits, st) : launch_rows_nt<false>(p, desc->g, pl.nt, pl.oct, desc->bits, st);
  if (e != hipSuccess) {
    note_hip_error((int)e);
    return TMAC_EHIP;
  }
  return TMAC_OK;
}

}  // namespace tmac

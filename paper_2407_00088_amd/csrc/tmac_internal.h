// Shared host-side helpers of the library (not part of the public ABI).
#ifndef TMAC_INTERNAL_H_
#define TMAC_INTERNAL_H_

#include <cstddef>
#include <cstdint>

#include "tmac.h"

namespace tmac {

constexpr uint32_t TMAC_MAGIC = 0x43414D54u;  // "TMAC"

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Geometry of a packed weight blob (both layouts).
//   layout 2: row tiles of 8, lane-units of 16 k;  layout 3: row tiles of 64, k chunks of 32.
struct Geometry {
  int Mp, Kp;          // padded M and K
  int n_tiles;         // row tiles (8 rows in layout 2, 64 in layout 3)
  int n_chunks;        // layout 2: 16-k lane-units; layout 3: 32-k chunks
  int n_qgroups;       // scale groups per row stored in the blob (0 when per-tensor)
  int tile_rows;       // 8 or 64
  uint64_t idx_off, idx_bytes, sz_off, sz_bytes, total_bytes;
};

bool desc_valid(const tmac_wdesc* d);
bool group_supported(const tmac_wdesc* d);
Geometry geometry(const tmac_wdesc* d);

// Geometry of the LUT buffer written by tmac_precompute_lut.
constexpr int TMAC_DECODE_MAX_ROWS = 64;  // activation rows the register-table kernel takes from a LUT buffer

struct LutGeom {
  int Kp, KG, nq;       // K padded to 128, tables per row, quantisation groups per row (>= 1)
  int Geff;             // elements per quantisation group (K when one group per row/tensor)
  int U;                // 16-k units per row (Kp / 16)
  int ht_slots;         // 16-byte slots per unit in the half-table region: 4 (fp16) or 2 (int8)
  size_t s_off;         // byte offset of the group sums S[N][nq]
  size_t s16_off;       // byte offset of the unit sums S16[N][U]
  size_t s128_off;      // byte offset of the 128-k chunk sums S128[N][U/8]
  size_t usc_off;       // int8 tables only: byte offset of the unit scales [N][U] (fp32)
  size_t ht_off;        // byte offset of the half tables, piece-major per block
  size_t total;
  int NT;  // activation rows per n tile of the table region
  bool decode_parts;  // per-16 and per-128 sums and half tables present
};

// Activation rows the batched kernels serve per workgroup ("n tile") for a call with N rows: eight
// once that wastes at most a fifth of the lookups on padding rows; 256-entry tables (g = 8) take
// four always (eight rows of them would leave an LDS slice two chunks long).  The precompute
// kernel lays the tables out per n tile, so both sides derive the tile from N and g alone.
inline int rows_nt(int N, int g) {
  if (g == 8) return 4;
  return (N >= 40 || N % 8 == 0 || N % 8 >= 5) && N > 4 ? 8 : 4;
}

// lut_t: a tmac_lut_t value.  The 2^g-entry tables at offset 0 (read by the batched kernels; laid
// out [n tile][KG][2^g][NT], i.e. as the kernels keep them in LDS) exist for the 16-bit table
// types only; the per-16 and per-128 sums and the half tables of the register-table kernel exist
// for g = 4 only.
inline bool lut_geom(int N, int K, int g, int group, int lut_t, LutGeom* lg) {
  if (N <= 0 || K <= 0 || (g != 2 && g != 4 && g != 8) || K % 4 != 0 || K % g != 0 || group < 0) return false;
  if (group > 0 && (K % group != 0 || group % 4 != 0 || group % g != 0)) return false;
  const bool q8 = (lut_t == TMAC_LUT_I8Q);
  if (q8 && g != 4) return false;
  lg->Kp = round_up(K, 128);
  lg->KG = lg->Kp / g;
  lg->U = lg->Kp / 16;
  lg->Geff = (group == 0) ? K : group;
  lg->nq = K / lg->Geff;
  lg->ht_slots = q8 ? 2 : 4;
  lg->NT = rows_nt(N, g);
  const size_t n_pad = (size_t)(N + lg->NT - 1) / lg->NT * lg->NT;  // whole n tiles
  const size_t tab = q8 ? 0 : n_pad * lg->KG * (2u << g);
  lg->s_off = (tab + 255) / 256 * 256;
  lg->s16_off = (lg->s_off + (size_t)N * lg->nq * 4 + 255) / 256 * 256;
  // the regions of the register-table kernel exist for g = 4 and at most TMAC_DECODE_MAX_ROWS
  // activation rows (that kernel serves a handful of rows; a prefill-sized buffer goes without them)
  lg->decode_parts = (g == 4 && N <= TMAC_DECODE_MAX_ROWS);
  if (!lg->decode_parts) {
    if (q8) return false;
    lg->s128_off = lg->usc_off = lg->ht_off = lg->s16_off;
    lg->total = lg->s16_off + 256;
    return true;
  }
  lg->s128_off = (lg->s16_off + (size_t)N * lg->U * 4 + 255) / 256 * 256;
  lg->usc_off = (lg->s128_off + (size_t)N * (lg->U / 8) * 4 + 255) / 256 * 256;
  lg->ht_off = q8 ? (lg->usc_off + (size_t)N * lg->U * 4 + 255) / 256 * 256 : lg->usc_off;
  // one extra all-zero 16-byte slot (in a 256-byte tail) for lanes that own no unit
  lg->total = (lg->ht_off + (size_t)N * lg->U * 16 * lg->ht_slots + 256 + 255) / 256 * 256;
  return true;
}

// Split of a row's C = U/8 chunks (128 k = 8 units of 16 k each) into nB = ceil(C/8) blocks of at
// most 8 chunks, one block per wavefront pass of the register-table kernel: the first r blocks
// have q+1 chunks, the others q.  Inside a block of ng chunks starting at chunk c0, lane l of the
// wavefront owns unit 8*(c0 + (l & 7)) + (l >> 3), i.e. the eight lanes with equal l & 7 cover
// one 128-k chunk; lanes with (l & 7) >= ng own nothing.  The lane's data sits at slot
// (l >> 3) * ng + (l & 7) of the block.  Shared by the packer, the precompute kernel and the
// lookup kernel.
#if defined(__HIPCC__)
#define TMAC_HD __host__ __device__
#else
#define TMAC_HD
#endif
struct BlockSplit {
  int nB, q, r;
};
TMAC_HD inline BlockSplit block_split(int U) {
  const int C = U / 8;
  BlockSplit b;
  b.nB = (C + 7) / 8;
  b.q = C / b.nB;
  b.r = C % b.nB;
  return b;
}
// first chunk of block blk
TMAC_HD inline int block_start(const BlockSplit& b, int blk) { return blk * b.q + (blk < b.r ? blk : b.r); }
// block that holds chunk c
TMAC_HD inline int block_of(const BlockSplit& b, int c) {
  const int big = b.r * (b.q + 1);
  return c < big ? c / (b.q + 1) : b.r + (c - big) / b.q;
}
// slot of unit u inside its block (c0 = first chunk, ng = chunks of the block)
TMAC_HD inline int block_slot(int u, int c0, int ng) { return (u & 7) * ng + ((u >> 3) - c0); }

#if defined(__HIPCC__)
// Algorithm 1 Precompute for one LUT group of four fp16 activations, in the activations' own
// precision: x01 = {a0, a1}, x23 = {a2, a3} as packed pairs; T[p] = (+-a0 +- a1) + (+-a2 +- a3),
// the pair sums first, then their sum, every addition in fp16 (round to nearest even).  out[d] =
// {T[2d], T[2d+1]} for the mirror half p = 0..7 (a3 subtracted); entries 8..15 are the negated
// entries 7..0 (Section 3.3), exactly, because negation commutes with rounding.  Six packed
// additions; every table builder of the library goes through here so that they agree bit for bit.
typedef _Float16 tmac_h2 __attribute__((ext_vector_type(2)));
__device__ inline __attribute__((always_inline)) void half_table_f16(uint32_t x01, uint32_t x23, uint32_t (&out)[4]) {
  const tmac_h2 a = __builtin_bit_cast(tmac_h2, x01), b = __builtin_bit_cast(tmac_h2, x23);
  const tmac_h2 sd = tmac_h2{a.x, a.x} + tmac_h2{a.y, -a.y};  // {a0 + a1, a0 - a1}
  const tmac_h2 tw = tmac_h2{b.x, b.x} + tmac_h2{b.y, -b.y};  // {a2 + a3, a2 - a3}
  const tmac_h2 m0 = tmac_h2{-sd.x, sd.y}, m1 = tmac_h2{-sd.y, sd.x};  // signs of a0, a1: --, +-  and  -+, ++
  out[0] = __builtin_bit_cast(uint32_t, m0 - tmac_h2{tw.x, tw.x});
  out[1] = __builtin_bit_cast(uint32_t, m1 - tmac_h2{tw.x, tw.x});
  out[2] = __builtin_bit_cast(uint32_t, m0 + tmac_h2{tw.y, tw.y});
  out[3] = __builtin_bit_cast(uint32_t, m1 + tmac_h2{tw.y, tw.y});
}
// Sum of four fp16 activations given as two packed pairs, in fp32 (two dot products with ones).
__device__ inline __attribute__((always_inline)) float sum4_f16(uint32_t x01, uint32_t x23) {
  const tmac_h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
  // (the first product in the three-operand form with the constant 0 as addend: the compiler would
  // zero a register and accumulate in place; its result feeds only the addend of the second dot
  // product, which may follow at once -- an instruction of another kind would need three wait states
  // that the compiler does not keep after an assembly statement)
  float s;
  asm("v_dot2_f32_f16 %0, %1, %2, 0" : "=v"(s) : "v"(x01), "s"(0x3C003C00u));
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(tmac_h2, x23), ones, s, false);
}
#endif

// Register-table decode kernel (layout 2); defined in tmac_perm.hip.  Arguments are those of
// tmac_mpgemm after validation; with lut_dev == nullptr the kernel builds its tables itself from
// the activations A_dev (leading dimension lda).  lut_t is a tmac_lut_t value.  Returns a
// tmac_status value.
int launch_perm_gemv(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
                     int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale,
                     void* out_dev, int out_t, int64_t ldo, void* stream, const tmac_tuning* tuning);

// Several matrices in one launch of the register-table kernel, tables built in the kernel (items
// validated by the caller as for launch_perm_gemv with lut_dev == nullptr).
int launch_perm_gemv_multi(const tmac_gemv_item* items, int count, int act_t, int N, int out_t, void* stream,
                           const tmac_tuning* tuning);

// Batched lookup kernel (layout 3); defined in tmac_rows.hip.
struct RowsPlan {
  int nt;                     // activation rows per n tile of the LUT buffer (4 or 8)
  int oct;                    // n tiles per workgroup (2 for many rows at g = 4, else 1)
  int n_tiles_n, row_blocks;  // workgroups along N (nt * oct activation rows each) and M (256 weight rows each)
  int cps, slices;            // 32-k chunks per K slice, number of K slices (gridDim.z)
  bool eight;                 // slices of eight chunks: the kernel pair for few activation rows serves the call
  size_t part_bytes, ctr_bytes;  // workspace: partial sums (0 when slices == 1); ctr_bytes is always 0
  size_t srow_bytes;             // ... and the slices' sums of every activation row (eight-chunk plans)
};
RowsPlan rows_plan(const tmac_wdesc* desc, int N);
bool rows_builds_tables(const tmac_wdesc* desc, int N);
// Returns a tmac_status value.  lut_dev NULL: tables built in the kernel from A_dev (where
// rows_builds_tables(desc, N) holds).
int launch_rows_gemm(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev, const void* A_dev,
                     int64_t lda, int lut_t, int N, const float* act_scale_dev, float weight_scale, void* out_dev,
                     int out_t, int64_t ldo, void* workspace_dev, size_t workspace_bytes, void* stream);

// Records the last HIP error of this thread (diagnostics for TMAC_EHIP).
void note_hip_error(int hip_error);
// Explanation of a refusal (a string literal) for tmac_last_error_detail.
void note_detail(const char* text);

}  // namespace tmac
#endif

// Offline weight preparation for the LUT mpGEMM library (host code only).
//
// Algorithm 1 "PreprocessWeights": the b-bit codes are split into b one-bit planes and every
// g = 4 consecutive bits of a plane along K are packed into one 4-bit index, bit (k % g)
// belonging to element k.  Section 3.2 "Weight permutation": the indices are stored tile by
// tile in exactly the order the lookup kernel walks them, so that one wavefront reads one
// contiguous run per step.  Section 3.2 "Weight interleaving": inside a dword the indices
// are placed so that the kernel's mask-and-shift unpacking leaves them in processing order.  Section 3.3 "Mirror consolidation" (layout 2 only): an index p >= 8 is stored as a
// sign bit plus the 3-bit selector of its mirror entry 15 - p, because T[p] = -T[15 - p].
#include <cstring>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

bool desc_valid(const tmac_wdesc* d) {
  if (!d) return false;
  if (d->M <= 0 || d->K <= 0) return false;
  if (d->bits < 1 || d->bits > 4) return false;
  if (d->layout != TMAC_LAYOUT_R8U16 && d->layout != TMAC_LAYOUT_R64K32) return false;
  if (d->g != 4 && !(d->layout == TMAC_LAYOUT_R64K32 && (d->g == 2 || d->g == 8))) return false;
  if (d->K % 4 != 0 || d->K % d->g != 0) return false;
  if (d->group < 0 || d->reserved != 0) return false;
  if (!(d->zero_point == d->zero_point)) return false;  // NaN
  if (d->group > 0) {
    if (d->K % d->group != 0 || d->group % d->g != 0) return false;
  }
  return true;
}

// Group sizes the lookup kernels can apply scales for.
//   layout 2: any multiple of 16 (a lane's four tables must share one group), one group per
//             row, or one per tensor.
//   layout 3: any multiple of 32 (a chunk of eight tables must share one group), one group per
//             row, or one per tensor.
bool group_supported(const tmac_wdesc* d) {
  const int G = d->group;
  if (G == 0 || G == d->K) return true;
  if (d->layout == TMAC_LAYOUT_R8U16) return G % 16 == 0;
  return G % 32 == 0;
}

Geometry geometry(const tmac_wdesc* d) {
  Geometry ge;
  ge.Kp = round_up(d->K, 128);
  ge.n_qgroups = d->group == 0 ? 0 : d->K / d->group;
  ge.idx_off = sizeof(tmac_blob_header);
  if (d->layout == TMAC_LAYOUT_R8U16) {
    ge.tile_rows = 8;
    ge.Mp = round_up(d->M, 8);
    ge.n_tiles = ge.Mp / 8;
    ge.n_chunks = ge.Kp / 16;
    ge.idx_bytes = (uint64_t)ge.n_tiles * ge.n_chunks * 16 * d->bits;
  } else {
    ge.tile_rows = 64;
    ge.Mp = round_up(d->M, 64);
    ge.n_tiles = ge.Mp / 64;
    ge.n_chunks = ge.Kp / 32;
    ge.idx_bytes = (uint64_t)ge.n_tiles * ge.n_chunks * 64 * d->bits * 4;
  }
  ge.sz_off = (ge.idx_off + ge.idx_bytes + 255) / 256 * 256;
  ge.sz_bytes = (uint64_t)ge.n_tiles * ge.n_qgroups * ge.tile_rows * 4;
  ge.total_bytes = (ge.sz_off + ge.sz_bytes + 255) / 256 * 256;
  return ge;
}

// 4-bit index of bit plane `plane` of row `row` (length K) for LUT group kg; 0 past the end of K.
static inline uint32_t index_of(const uint8_t* row, int K, int kg, int plane) {
  const int k0 = 4 * kg;
  if (k0 >= K) return 0;
  uint32_t nib = 0;
  for (int e = 0; e < 4; ++e) nib |= (uint32_t)((row[k0 + e] >> plane) & 1) << e;
  return nib;
}

// Mirror-consolidated form of an index: sign bit 3, selector of the stored half in bits 0..2.
static inline uint32_t mirror_fold(uint32_t p) { return p < 8 ? p : (8u | (15u - p)); }

// Layout 3: lane = row of a 64-row tile; per (tile, 32-k chunk, row) `bits` dwords, dword i holding the
// eight indices of plane i for the chunk's eight tables, table j in nibble j.
static void pack_indices_layout3(const tmac_wdesc* d, const Geometry& ge, const uint8_t* q, uint32_t* idx) {
  const int M = d->M, K = d->K, b = d->bits;
  for (int t = 0; t < ge.n_tiles; ++t)
    for (int c = 0; c < ge.n_chunks; ++c)
      for (int r = 0; r < 64; ++r) {
        const int m = 64 * t + r;
        if (m >= M) continue;
        uint32_t* dst = idx + (((size_t)t * ge.n_chunks + c) * 64 + r) * b;
        const uint8_t* row = q + (size_t)m * K;
        for (int i = 0; i < b; ++i) {
          uint32_t word = 0;
          for (int j = 0; j < 8; ++j) word |= index_of(row, K, 8 * c + j, i) << (4 * j);
          dst[i] = word;
        }
      }
}

// Bit order of a layout-2 dword of eight folded codes.  In: byte y = {code of the "high" row in the
// high nibble, code of the "low" row in the low nibble}, a code being {negate, 3-bit entry}.  Out:
// byte y = {negate_low(y), entry_high(y), negate_high(y - 1 mod 4), entry_low(y)}: the low rows' negate
// bits sit at bit 7 of their own byte, and after a rotation of the dword by four bits (which brings
// the high rows' entries to bits 0..2) so do the high rows'.  The lookup kernel then needs no shift
// of its own for either sign.
static inline uint32_t place_negate_bits(uint32_t w) {
  uint32_t out = 0;
  for (int y = 0; y < 4; ++y) {
    const uint32_t byte = (w >> (8 * y)) & 0xffu;
    const uint32_t e_lo = byte & 7u, n_lo = (byte >> 3) & 1u, e_hi = (byte >> 4) & 7u, n_hi = byte >> 7;
    out |= (e_lo | (e_hi << 4) | (n_lo << 7)) << (8 * y);
    out |= (n_hi << 3) << (8 * ((y + 1) & 3));
  }
  return out;
}

// Layout 2: per (8-row tile, 16-k unit) four tables, each with `bits` dwords.  Byte y of a dword
// carries two indices of the same table: the low nibble belongs to the "low" row set and the
// high nibble to the "high" row set; which (row, plane) a byte stands for depends on how many
// planes share the dword (see tmac.h).
static void pack_indices_layout2(const tmac_wdesc* d, const Geometry& ge, const uint8_t* q, uint32_t* idx) {
  const int M = d->M, K = d->K, b = d->bits;
  auto nib = [&](int m, int kg, int plane) -> uint32_t {
    if (m >= M) return 0;
    return mirror_fold(index_of(q + (size_t)m * K, K, kg, plane));
  };
  const int U = ge.n_chunks;
  const BlockSplit bs = block_split(U);
  for (int t = 0; t < ge.n_tiles; ++t)
    for (int blk = 0; blk < bs.nB; ++blk) {
     const int c0 = block_start(bs, blk), ng = block_start(bs, blk + 1) - c0;
     const int u0 = 8 * c0, u1 = u0 + 8 * ng, nu = 8 * ng;
     for (int u = u0; u < u1; ++u) {
      uint32_t rec[16];  // the unit's record: [table][dword]
      for (int tb = 0; tb < 4; ++tb) {
        const int kg = 4 * u + tb, m0 = 8 * t;
        uint32_t* dst = rec + tb * b;
        int nd = 0;
        auto quad = [&](int dw) {  // four planes of rows 2dw (low) and 2dw+1 (high)
          uint32_t w = 0;
          for (int y = 0; y < 4; ++y)
            w |= (nib(m0 + 2 * dw, kg, y) | (nib(m0 + 2 * dw + 1, kg, y) << 4)) << (8 * y);
          return w;
        };
        auto pair = [&](int dw, int p0) {  // planes p0, p0+1 of rows 4dw, 4dw+1 (low), 4dw+2, 4dw+3 (high)
          uint32_t w = 0;
          for (int y = 0; y < 4; ++y)
            w |= (nib(m0 + 4 * dw + y / 2, kg, p0 + y % 2) | (nib(m0 + 4 * dw + 2 + y / 2, kg, p0 + y % 2) << 4))
                 << (8 * y);
          return w;
        };
        auto single = [&](int p0) {  // plane p0 of rows 0..3 (low) and 4..7 (high)
          uint32_t w = 0;
          for (int y = 0; y < 4; ++y) w |= (nib(m0 + y, kg, p0) | (nib(m0 + 4 + y, kg, p0) << 4)) << (8 * y);
          return w;
        };
        if (b == 4) { for (int dw = 0; dw < 4; ++dw) dst[nd++] = quad(dw); }
        else if (b == 2) { dst[nd++] = pair(0, 0); dst[nd++] = pair(1, 0); }
        else if (b == 1) { dst[nd++] = single(0); }
        else { dst[nd++] = pair(0, 0); dst[nd++] = pair(1, 0); dst[nd++] = single(2); }
        for (int i = 0; i < nd; ++i) dst[i] = place_negate_bits(dst[i]);
      }
      // 16-byte piece i of the record goes to (piece i, slot of the unit's lane) of the block, so
      // that the lanes of a wavefront read one contiguous run per load instruction
      uint32_t* blk_base = idx + ((size_t)t * U + u0) * (4 * b);
      const int slot = block_slot(u, c0, ng);
      for (int i = 0; i < b; ++i)
        for (int e = 0; e < 4; ++e) blk_base[((size_t)i * nu + slot) * 4 + e] = rec[4 * i + e];
     }
    }
}

}  // namespace tmac

using namespace tmac;

extern "C" size_t tmac_packed_bytes(const tmac_wdesc* desc) {
  if (!desc_valid(desc)) return 0;
  return (size_t)geometry(desc).total_bytes;
}

extern "C" tmac_status tmac_pack_weights(const tmac_wdesc* desc, const uint8_t* q,
                                         const uint16_t* scales, const uint16_t* zeros,
                                         void* packed, size_t packed_bytes) {
  if (!desc_valid(desc) || !q || !packed) return TMAC_EINVAL;
  if (desc->group > 0 && !scales) return TMAC_EINVAL;
  const Geometry ge = geometry(desc);
  if (packed_bytes < ge.total_bytes) return TMAC_ESIZE;
  const int M = desc->M, K = desc->K, b = desc->bits, G = desc->group;
  const int code_lim = 1 << b;
  for (int64_t i = 0; i < (int64_t)M * K; ++i)
    if (q[i] >= code_lim) return TMAC_EINVAL;

  uint8_t* out = static_cast<uint8_t*>(packed);
  std::memset(out, 0, ge.total_bytes);
  tmac_blob_header h;
  std::memset(&h, 0, sizeof(h));
  h.magic = TMAC_MAGIC;
  h.layout = (uint32_t)desc->layout;
  h.M = M; h.K = K; h.bits = b; h.g = desc->g; h.group = G;
  h.Mp = ge.Mp; h.Kp = ge.Kp;
  h.n_tiles = ge.n_tiles; h.n_chunks = ge.n_chunks; h.n_qgroups = ge.n_qgroups;
  h.zero_point = (G == 0) ? desc->zero_point : 0.0f;
  h.idx_off = ge.idx_off; h.idx_bytes = ge.idx_bytes;
  h.sz_off = ge.sz_off; h.sz_bytes = ge.sz_bytes; h.total_bytes = ge.total_bytes;
  std::memcpy(out, &h, sizeof(h));

  uint32_t* idx = reinterpret_cast<uint32_t*>(out + ge.idx_off);
  if (desc->layout == TMAC_LAYOUT_R8U16) pack_indices_layout2(desc, ge, q, idx);
  else pack_indices_layout3(desc, ge, q, idx);

  // scales and zeros, {s, z} per (row tile, quantisation group, row in tile)
  if (G > 0) {
    uint16_t* sz = reinterpret_cast<uint16_t*>(out + ge.sz_off);
    const int nq = ge.n_qgroups, R = ge.tile_rows;
    // fp16 bits of (2^b-1)/2: 0.5, 1.5, 3.5, 7.5
    static const uint16_t mid_bits[5] = {0, 0x3800, 0x3E00, 0x4300, 0x4780};
    for (int t = 0; t < ge.n_tiles; ++t)
      for (int gq = 0; gq < nq; ++gq)
        for (int r = 0; r < R; ++r) {
          const int m = R * t + r;
          uint16_t* dst = sz + (((size_t)t * nq + gq) * R + r) * 2;
          if (m >= M) { dst[0] = 0; dst[1] = 0; continue; }
          dst[0] = scales[(size_t)m * nq + gq];
          dst[1] = zeros ? zeros[(size_t)m * nq + gq] : mid_bits[b];
        }
  }
  return TMAC_OK;
}

extern "C" const char* tmac_status_str(tmac_status s) {
  switch (s) {
    case TMAC_OK: return "ok";
    case TMAC_EINVAL: return "invalid argument";
    case TMAC_EUNSUPPORTED: return "unsupported configuration";
    case TMAC_ESIZE: return "buffer too small";
    case TMAC_EHIP: return "HIP runtime error";
  }
  return "unknown status";
}

extern "C" int32_t tmac_version(void) { return 1000 * 0 + 7; }

// Offline weight preparation for the LUT mpGEMM library (host code only).
//
// Algorithm 1 "PreprocessWeights": the b-bit codes are split into b one-bit planes and every
// g = 4 consecutive bits of a plane along K are packed into one 4-bit index, bit (k % g)
// belonging to element k.  Section 3.2 "Weight permutation": the indices are stored tile by
// tile in exactly the order the lookup kernel walks them, so that one wavefront reads one
// contiguous run per step.  Section 3.2 "Weight interleaving": inside a dword the eight
// indices are placed so that two mask-and-shift operations leave byte-aligned table offsets
// in processing order.
#include <cmath>
#include <cstring>
#include <vector>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

bool desc_valid(const tmac_wdesc* d) {
  if (!d) return false;
  if (d->M <= 0 || d->K <= 0) return false;
  if (d->bits < 1 || d->bits > 4) return false;
  if (d->g != 4) return false;
  if (d->layout != TMAC_LAYOUT_T16K128) return false;
  if (d->K % d->g != 0) return false;
  if (d->group < 0 || d->reserved != 0) return false;
  if (!(d->zero_point == d->zero_point)) return false;  // NaN
  if (d->group > 0) {
    if (d->K % d->group != 0 || d->group % d->g != 0) return false;
  }
  return true;
}

// Group sizes the lookup kernels can apply scales for: whole chunks (multiples of 128),
// the two sub-chunk sizes 32 and 64, one group per row, or one per tensor.
bool group_supported(const tmac_wdesc* d) {
  const int G = d->group;
  return G == 0 || G == d->K || G == 32 || G == 64 || (G % 128 == 0);
}

Geometry geometry(const tmac_wdesc* d) {
  Geometry ge;
  ge.Mp = (d->M + 15) / 16 * 16;
  ge.Kp = (d->K + 127) / 128 * 128;
  ge.n_tiles = ge.Mp / 16;
  ge.n_chunks = ge.Kp / 128;
  ge.n_qgroups = d->group == 0 ? 0 : d->K / d->group;
  ge.idx_off = sizeof(tmac_blob_header);
  ge.idx_bytes = (uint64_t)ge.n_tiles * ge.n_chunks * 64 * d->bits * 4;
  ge.sz_off = (ge.idx_off + ge.idx_bytes + 255) / 256 * 256;
  ge.sz_bytes = (uint64_t)ge.n_tiles * ge.n_qgroups * 16 * 4;
  ge.total_bytes = (ge.sz_off + ge.sz_bytes + 255) / 256 * 256;
  return ge;
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

  // indices
  uint32_t* idx = reinterpret_cast<uint32_t*>(out + ge.idx_off);
  for (int t = 0; t < ge.n_tiles; ++t) {
    for (int c = 0; c < ge.n_chunks; ++c) {
      for (int lane = 0; lane < 64; ++lane) {
        const int r = lane & 15, phi = lane >> 4;
        const int m = 16 * t + r;
        uint32_t* dst = idx + (((size_t)t * ge.n_chunks + c) * 64 + lane) * b;
        if (m >= M) continue;
        const uint8_t* row = q + (size_t)m * K;
        for (int i = 0; i < b; ++i) {
          uint32_t word = 0;
          for (int j = 0; j < 8; ++j) {
            const int kg = 32 * c + 4 * j + phi;   // LUT group
            const int k0 = 4 * kg;
            if (k0 >= K) continue;
            uint32_t nib = 0;
            for (int e = 0; e < 4; ++e) nib |= (uint32_t)((row[k0 + e] >> i) & 1) << e;
            const int pos = (j < 4) ? 2 * j : 2 * (j - 4) + 1;
            word |= nib << (4 * pos);
          }
          dst[i] = word;
        }
      }
    }
  }

  // scales and zeros, {s, z} per (tile, quantisation group, row)
  if (G > 0) {
    uint16_t* sz = reinterpret_cast<uint16_t*>(out + ge.sz_off);
    const int nq = ge.n_qgroups;
    // fp16 bits of (2^b-1)/2: 0.5, 1.5, 3.5, 7.5
    static const uint16_t mid_bits[5] = {0, 0x3800, 0x3E00, 0x4300, 0x4780};
    for (int t = 0; t < ge.n_tiles; ++t)
      for (int gq = 0; gq < nq; ++gq)
        for (int r = 0; r < 16; ++r) {
          const int m = 16 * t + r;
          uint16_t* dst = sz + (((size_t)t * nq + gq) * 16 + r) * 2;
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

extern "C" int32_t tmac_version(void) { return 1000 * 0 + 1; }

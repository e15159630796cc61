// Shared host-side helpers of the library (not part of the public ABI).
#ifndef TMAC_INTERNAL_H_
#define TMAC_INTERNAL_H_

#include <cstdint>

#include "tmac.h"

namespace tmac {

constexpr uint32_t TMAC_MAGIC = 0x43414D54u;  // "TMAC"

struct Geometry {
  int Mp, Kp, n_tiles, n_chunks, n_qgroups;
  uint64_t idx_off, idx_bytes, sz_off, sz_bytes, total_bytes;
};

bool desc_valid(const tmac_wdesc* d);
bool group_supported(const tmac_wdesc* d);
Geometry geometry(const tmac_wdesc* d);

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

}  // namespace tmac
#endif

// Longest-processing-time-first packing of transfers into windows (paper Sec. 4.2; Graham's list-scheduling rule the
// paper cites).  Host code only.
#include <algorithm>
#include <stdio.h>

#include "transfers.hpp"

namespace rp {

std::vector<rp_piece> plan_transfers(const size_t* item_bytes, int n_items, int n_windows, size_t max_piece) {
  std::vector<rp_piece> pieces;
  for (int i = 0; i < n_items; ++i) {
    const size_t b = item_bytes[i];
    if (b == 0) continue;
    const size_t n = (b + max_piece - 1) / max_piece;
    size_t sz = (b + n - 1) / n;
    sz = (sz + 255) / 256 * 256;
    for (size_t off = 0; off < b; off += sz) {
      rp_piece p;
      p.item = i; p.window = 0; p.offset = off; p.bytes = std::min(sz, b - off);
      pieces.push_back(p);
    }
  }
  std::stable_sort(pieces.begin(), pieces.end(), [](const rp_piece& a, const rp_piece& b) {
    if (a.bytes != b.bytes) return a.bytes > b.bytes;
    if (a.item != b.item) return a.item < b.item;
    return a.offset < b.offset;
  });
  std::vector<size_t> load((size_t)n_windows, 0);
  for (rp_piece& p : pieces) {
    int best = 0;
    for (int w = 1; w < n_windows; ++w)
      if (load[w] < load[best]) best = w;
    p.window = best;
    load[best] += p.bytes;
  }
  return pieces;
}

}  // namespace rp

extern "C" rp_status rp_plan_transfers(const size_t* item_bytes, int n_items, int n_windows, size_t max_piece_bytes,
                                       rp_piece* pieces, int capacity, int* n_pieces) {
  if (n_items < 0 || (n_items > 0 && !item_bytes) || n_windows <= 0 || max_piece_bytes == 0 || !n_pieces || capacity < 0 ||
      (capacity > 0 && !pieces))
    return RP_EINVAL;
  if (max_piece_bytes % 256) return RP_EINVAL;
  const std::vector<rp_piece> v = rp::plan_transfers(item_bytes, n_items, n_windows, max_piece_bytes);
  *n_pieces = (int)v.size();
  if ((int)v.size() > capacity) return RP_ENOMEM;
  for (size_t i = 0; i < v.size(); ++i) pieces[i] = v[i];
  return RP_OK;
}

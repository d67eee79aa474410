// Packing of parameter / gradient transfers into the data-transfer windows of a round (paper Sec. 4.2, "Scheduling
// parameter transfers").  Pure host code.
#pragma once
#include <stddef.h>
#include <vector>
#include "../../include/rp.h"

namespace rp {

// Splits every item larger than max_piece into equal pieces (multiples of 256 bytes, the last one shorter), takes the
// pieces in descending size (ties: lower item, lower offset) and gives each to the window that holds the fewest bytes so
// far (ties: lower window).  Returns the pieces in the order they were assigned.
std::vector<rp_piece> plan_transfers(const size_t* item_bytes, int n_items, int n_windows, size_t max_piece);

}  // namespace rp

// Host-only helpers shared by the host runtime (gv_api.cpp) and the host producers (gv_augment.cpp).
#pragma once

#include <stdint.h>

#include <vector>

namespace gv {

// Alias table over weights q (Vose's method, the construction both sides of the parity tests follow: sum left
// to right in fp64, p_i = q_i * size / sum, two index-ordered stacks, leftovers keep themselves, thresholds
// floor(p * 2^32) saturated).  alias[i] is an index into q.  *sum_out (may be null) receives the sum of the
// weights.  False when the weights sum to zero (or q is empty); may throw std::bad_alloc.
bool vose_table(const double *q, uint64_t size, uint32_t *thresh, uint32_t *alias, double *sum_out);

}  // namespace gv

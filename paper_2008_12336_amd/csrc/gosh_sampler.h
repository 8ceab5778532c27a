// Host side of the part-pair rotation (Alg. 5 of the paper): the positive samples.
#pragma once

#include <cstdint>

#include "gosh.h"

namespace gosh {

// Positives of the sources of part [lo, lo + cnt) against the partner range [olo, ohi) of a
// HOST graph (Sec. 3.3: the large graph stays on the host and positives are drawn there):
// pool[local * B + r] = for round r a uniform member of the source's neighbours inside the
// partner range, -1 if it has none there.  Neighbour lists are ascending, so the candidates
// are one contiguous run found by two binary searches.  The draw of (source, round) is
// Philox4x32-10 with counter (source, side * B * per_round + r * per_round, rotation, word3)
// and key (key0, key1), scaled by multiply-high -- the same values the device functions
// philox_draw / scale_draw give.
void fill_pool(const gosh_csr &g, int32_t lo, int32_t cnt, int32_t olo, int32_t ohi, int side,
               int32_t B, int32_t per_round, uint32_t key0, uint32_t key1, uint32_t rotation,
               uint32_t word3, int threads, int32_t *pool);

}  // namespace gosh

// Host sampler of the part-pair rotation.  The draws dominate its cost (ten Philox rounds
// per positive), so sources are handled eight at a time with the generator written as
// eight-lane loops that the compiler turns into vector multiplies; an AVX2 build of the
// same loops is chosen at run time where the CPU has it.
#include "gosh_sampler.h"

#include <omp.h>

#include <algorithm>

namespace {

constexpr int kLanes = 8;
constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;

// Philox4x32-10 (Salmon et al., SC'11) for kLanes counters that differ in word 0 only;
// w0/w1 receive output words 0 and 1 of every lane.
__attribute__((always_inline)) inline void philox_lanes(const uint32_t *c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1, uint32_t *w0,
                                                        uint32_t *w1) {
  uint32_t a0[kLanes], a1[kLanes], a2[kLanes], a3[kLanes];
  for (int l = 0; l < kLanes; ++l) {
    a0[l] = c0[l];
    a1[l] = c1;
    a2[l] = c2;
    a3[l] = c3;
  }
  for (int round = 0; round < 10; ++round) {
    for (int l = 0; l < kLanes; ++l) {
      const uint64_t pa = static_cast<uint64_t>(kMulA) * a0[l];
      const uint64_t pb = static_cast<uint64_t>(kMulB) * a2[l];
      const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ a1[l] ^ k0;
      const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ a3[l] ^ k1;
      a1[l] = static_cast<uint32_t>(pb);
      a3[l] = static_cast<uint32_t>(pa);
      a0[l] = n0;
      a2[l] = n2;
    }
    k0 += kWeylA;
    k1 += kWeylB;
  }
  for (int l = 0; l < kLanes; ++l) {
    w0[l] = a0[l];
    w1[l] = a1[l];
  }
}

void philox_lanes_base(const uint32_t *c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                       uint32_t *w0, uint32_t *w1) {
  philox_lanes(c0, c1, c2, c3, k0, k1, w0, w1);
}

// (all sources of the library go through the HIP compiler; its device pass must not see
// x86 attributes or builtins)
#if !defined(__HIP_DEVICE_COMPILE__)
__attribute__((target("avx2")))
#endif
void philox_lanes_avx2(const uint32_t *c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                       uint32_t k0, uint32_t k1, uint32_t *w0, uint32_t *w1) {
  philox_lanes(c0, c1, c2, c3, k0, k1, w0, w1);
}

using PhiloxLanes = void (*)(const uint32_t *, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t *,
                             uint32_t *);

PhiloxLanes pick_philox() {
#if !defined(__HIP_DEVICE_COMPILE__)
  __builtin_cpu_init();
  if (__builtin_cpu_supports("avx2")) return philox_lanes_avx2;
#endif
  return philox_lanes_base;
}

// floor(draw * bound / 2^64) for bound < 2^32, draw = w0 | w1 << 32.
inline uint32_t scale_draw(uint32_t w0, uint32_t w1, uint32_t bound) {
  const uint64_t t = static_cast<uint64_t>(w1) * bound + ((static_cast<uint64_t>(w0) * bound) >> 32);
  return static_cast<uint32_t>(t >> 32);
}

inline int64_t row_begin(const gosh_csr &g, int64_t v) {
  return g.xadj_is64 ? static_cast<const int64_t *>(g.xadj)[v] : static_cast<const int32_t *>(g.xadj)[v];
}

}  // namespace

namespace gosh {

void fill_pool(const gosh_csr &g, int32_t lo, int32_t cnt, int32_t olo, int32_t ohi, int side, int32_t B,
               int32_t per_round, uint32_t key0, uint32_t key1, uint32_t rotation, uint32_t word3, int threads,
               int32_t *pool) {
  static const PhiloxLanes philox = pick_philox();
  const int32_t *adj = g.adj;
  const int32_t blocks = (cnt + kLanes - 1) / kLanes;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 128)
  for (int32_t blk = 0; blk < blocks; ++blk) {
    const int32_t local0 = blk * kLanes;
    const int lanes = std::min<int32_t>(kLanes, cnt - local0);
    const int32_t *first[kLanes];
    uint32_t candidates[kLanes], src[kLanes];
    for (int l = 0; l < kLanes; ++l) {
      // lanes beyond the part repeat its last source; their draws are discarded
      const int64_t v = static_cast<int64_t>(lo) + local0 + std::min(l, lanes - 1);
      int64_t row_lo = row_begin(g, v), row_hi = row_begin(g, v + 1);
      if (row_lo < 0 || row_lo > row_hi || row_hi > g.nnz) row_lo = row_hi = 0;  // offsets that leave adj
      const int32_t *begin = adj + row_lo, *end = adj + row_hi;
      first[l] = std::lower_bound(begin, end, olo);
      candidates[l] = static_cast<uint32_t>(std::lower_bound(first[l], end, ohi) - first[l]);
      src[l] = static_cast<uint32_t>(v);
    }
    for (int32_t r = 0; r < B; ++r) {
      uint32_t w0[kLanes], w1[kLanes];
      philox(src, static_cast<uint32_t>(side * B * per_round + r * per_round), rotation, word3, key0, key1, w0, w1);
      for (int l = 0; l < lanes; ++l)
        pool[static_cast<int64_t>(local0 + l) * B + r] =
            candidates[l] > 0 ? first[l][scale_draw(w0[l], w1[l], candidates[l])] : -1;
    }
  }
}

}  // namespace gosh

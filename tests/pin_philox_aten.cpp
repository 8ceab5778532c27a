// Pin helper: prints Philox4x32-10 outputs computed by ATen's header-only engine
// (an implementation independent of the oracle's) for a list of inputs read from
// stdin: lines "seed subsequence offset" (decimal u64).  For each line it prints the
// four 32-bit outputs of the block with key = (seed_lo, seed_hi) and
// counter = (offset_lo, offset_hi, subsequence_lo, subsequence_hi).
#include <ATen/core/PhiloxRNGEngine.h>

#include <cinttypes>
#include <cstdio>

int main() {
  unsigned long long seed, subseq, offset;
  while (std::scanf("%llu %llu %llu", &seed, &subseq, &offset) == 3) {
    at::Philox4_32 eng(seed, subseq, 0);
    eng.set_offset(offset);
    uint32_t w0 = eng(), w1 = eng(), w2 = eng(), w3 = eng();
    std::printf("%" PRIu32 " %" PRIu32 " %" PRIu32 " %" PRIu32 "\n", w0, w1, w2, w3);
  }
  return 0;
}

// libgosh from C++ without Python: embeds a small synthetic graph (two communities joined
// by a few edges) through the C ABI alone and reports how well the embedding separates
// neighbours from non-neighbours.
//
//   hipcc -O2 -I include embed_example.cpp -L paper_2008_12336_amd -lgosh -o embed_example
//   ./embed_example              coarsen on the device, run Alg. 2, print the result
//   ./embed_example --host-only  only the host entry points (needs no GPU)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <set>
#include <utility>
#include <vector>

#include "gosh.h"

#define CHECK_GOSH(call)                                                   \
  do {                                                                     \
    if ((call) != GOSH_OK) {                                               \
      std::fprintf(stderr, "%s failed: %s\n", #call, gosh_last_error());   \
      return 1;                                                            \
    }                                                                      \
  } while (0)
#define CHECK_HIP(call)                                                            \
  do {                                                                             \
    hipError_t e_ = (call);                                                        \
    if (e_ != hipSuccess) {                                                        \
      std::fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));       \
      return 1;                                                                    \
    }                                                                              \
  } while (0)

namespace {

// A small deterministic generator for the example's edges (not the library's Philox).
struct Lcg {
  uint64_t state;
  uint32_t next(uint32_t bound) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return static_cast<uint32_t>((state >> 33) % bound);
  }
};

}  // namespace

int main(int argc, char **argv) {
  const bool host_only = argc > 1 && std::strcmp(argv[1], "--host-only") == 0;
  const int64_t n = 4000;
  const int32_t d = 32, k_neg = 3;

  // two communities of n/2 vertices, 8 random edges per vertex inside, 20 edges across
  std::vector<std::set<int32_t>> nbrs(static_cast<size_t>(n));
  Lcg rng{12345};
  auto add = [&](int32_t u, int32_t v) {
    if (u == v) return;
    nbrs[static_cast<size_t>(u)].insert(v);
    nbrs[static_cast<size_t>(v)].insert(u);
  };
  const int32_t half = static_cast<int32_t>(n / 2);
  for (int32_t u = 0; u < n; ++u)
    for (int e = 0; e < 8; ++e) add(u, (u < half ? 0 : half) + static_cast<int32_t>(rng.next(half)));
  for (int e = 0; e < 20; ++e) add(static_cast<int32_t>(rng.next(half)), half + static_cast<int32_t>(rng.next(half)));
  std::vector<int64_t> xadj(static_cast<size_t>(n) + 1, 0);
  std::vector<int32_t> adj;
  for (int64_t v = 0; v < n; ++v) {
    adj.insert(adj.end(), nbrs[static_cast<size_t>(v)].begin(), nbrs[static_cast<size_t>(v)].end());  // ascending
    xadj[static_cast<size_t>(v) + 1] = static_cast<int64_t>(adj.size());
  }
  const gosh_csr g{n, static_cast<int64_t>(adj.size()), xadj.data(), adj.data(), 1};
  CHECK_GOSH(gosh_csr_validate(&g));

  gosh_hierarchy *h = nullptr;
  if (host_only) CHECK_GOSH(gosh_coarsen(&g, 100, 0.8, 64, 0, &h));
  else CHECK_GOSH(gosh_coarsen_device(&g, 100, 0.8, 64, 0, &h));
  const int D = gosh_hierarchy_levels(h);
  std::printf("hierarchy: %d levels:", D);
  for (int i = 0; i < D; ++i) {
    int64_t ni = 0, nnzi = 0;
    CHECK_GOSH(gosh_hierarchy_shape(h, i, &ni, &nnzi));
    std::printf(" %lld/%lld", (long long)ni, (long long)nnzi);
  }
  std::printf("\n");
  const int64_t epochs = 600;
  std::vector<int64_t> e_i(static_cast<size_t>(D));
  CHECK_GOSH(gosh_epoch_split(epochs, 0.3, D, e_i.data()));
  std::printf("epochs per level (level 0 first):");
  for (int64_t e : e_i) std::printf(" %lld", (long long)e);
  std::printf("\n");
  if (host_only) {
    gosh_hierarchy_free(h);
    return 0;
  }

  float *M_dev = nullptr;
  CHECK_HIP(hipMalloc(&M_dev, static_cast<size_t>(n) * d * sizeof(float)));
  std::vector<gosh_level_stats> stats(static_cast<size_t>(D));
  CHECK_GOSH(gosh_embed(h, d, k_neg, epochs, 0.3, 0.035f, /*seed=*/1, /*flags=*/0, /*device_budget_bytes=*/0, M_dev,
                        stats.data(), /*hip_stream=*/nullptr));
  std::vector<float> M(static_cast<size_t>(n) * d);
  CHECK_HIP(hipMemcpy(M.data(), M_dev, M.size() * sizeof(float), hipMemcpyDeviceToHost));
  CHECK_HIP(hipFree(M_dev));
  gosh_hierarchy_free(h);

  // mean sigmoid-free score: dot product over edges against dot product over random pairs
  auto dot = [&](int64_t u, int64_t v) {
    double s = 0;
    for (int c = 0; c < d; ++c) s += static_cast<double>(M[u * d + c]) * M[v * d + c];
    return s;
  };
  double on_edges = 0, on_pairs = 0;
  for (int64_t u = 0; u < n; ++u)
    for (int64_t j = xadj[u]; j < xadj[u + 1]; ++j) on_edges += dot(u, adj[j]);
  on_edges /= static_cast<double>(adj.size());
  const int pairs = 100000;
  for (int i = 0; i < pairs; ++i) on_pairs += dot(rng.next(static_cast<uint32_t>(n)), rng.next(static_cast<uint32_t>(n)));
  on_pairs /= pairs;
  double ms = 0;
  for (const gosh_level_stats &s : stats) ms += s.train_ms;
  std::printf("trained %lld epochs in %.2f ms; mean dot over edges %.3f, over random pairs %.3f\n", (long long)epochs,
              ms, on_edges, on_pairs);
  // neighbours must score clearly above pairs drawn at random
  return (on_edges > 0.05 && on_edges > 5 * (on_pairs < 0 ? -on_pairs : on_pairs)) ? 0 : 2;
}

// Which parts of a large device allocation answer random row traffic independently of each
// other?  Random 512-byte row read-modify-writes are spread over two 4 GiB blocks of one big
// buffer; two blocks in the same class of memory give one rate, two blocks in different classes
// a higher one.  On an MI355X the blocks fall into three classes (the three ranks of its
// twelve-high HBM stacks).  Diagnostic only: no part of the library uses it.
//
//   hipcc -O2 hbm_rank_probe.cpp -o hbm_rank_probe && ./hbm_rank_probe [GiB, default 240]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK_HIP(call)                                                        \
  do {                                                                         \
    hipError_t e_ = (call);                                                    \
    if (e_ != hipSuccess) {                                                    \
      std::printf("%s failed: %s\n", #call, hipGetErrorString(e_));            \
      return 1;                                                                \
    }                                                                          \
  } while (0)

__device__ inline uint64_t mix(uint64_t x) {
  x ^= x >> 33; x *= 0xff51afd7ed558ccdULL; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL; x ^= x >> 33;
  return x;
}

// One wavefront per access: a random row of block A or of block B (64 lanes x 8 bytes).
__global__ __launch_bounds__(256) void probe(float2 *a, float2 *b, uint64_t rows, uint64_t accesses, uint64_t salt) {
  const uint64_t wave = (blockIdx.x * 256ull + threadIdx.x) >> 6, waves = (gridDim.x * 256ull) >> 6;
  const int lane = threadIdx.x & 63;
  for (uint64_t i = wave; i < accesses; i += waves) {
    const uint64_t h = mix(i ^ salt);
    float2 *p = ((h & 1) ? b : a) + ((h >> 1) % rows) * 64 + lane;
    float2 v = *p;
    v.x += 1.f;
    *p = v;
  }
}

int main(int argc, char **argv) {
  const size_t GiB = size_t{1} << 30, block = 4 * GiB;
  const size_t total = static_cast<size_t>(argc > 1 ? std::atoll(argv[1]) : 240) * GiB;
  if (total < 2 * block) { std::printf("need at least 8 GiB\n"); return 1; }
  char *buf = nullptr;
  CHECK_HIP(hipMalloc(reinterpret_cast<void **>(&buf), total));
  CHECK_HIP(hipMemset(buf, 0, total));
  CHECK_HIP(hipDeviceSynchronize());
  const uint64_t rows = block / 512, accesses = rows * 8;
  hipEvent_t t0, t1;
  CHECK_HIP(hipEventCreate(&t0));
  CHECK_HIP(hipEventCreate(&t1));
  auto rate = [&](size_t a, size_t b, double *tb_per_s) -> int {
    float best = 1e30f;
    for (int it = 0; it < 2; ++it) {
      CHECK_HIP(hipEventRecord(t0, nullptr));
      hipLaunchKernelGGL(probe, dim3(2048), dim3(256), 0, nullptr, reinterpret_cast<float2 *>(buf + a * block),
                         reinterpret_cast<float2 *>(buf + b * block), rows, accesses, static_cast<uint64_t>(it) + 3);
      CHECK_HIP(hipGetLastError());
      CHECK_HIP(hipEventRecord(t1, nullptr));
      CHECK_HIP(hipEventSynchronize(t1));
      float ms = 0.f;
      CHECK_HIP(hipEventElapsedTime(&ms, t0, t1));
      if (ms < best) best = ms;
    }
    *tb_per_s = accesses * 1024.0 / best / 1e9;
    return 0;
  };
  const size_t blocks = total / block;
  // class of a block = the first earlier representative it shares a rate with
  std::vector<int> cls(blocks, -1);
  std::vector<size_t> reps;
  double same = 0, other = 0;
  if (rate(0, 0, &same)) return 1;  // both halves in one block: the "same class" rate
  for (size_t b = 0; b < blocks; ++b) {
    for (size_t r = 0; r < reps.size() && cls[b] < 0; ++r) {
      double x = 0;
      if (rate(reps[r], b, &x)) return 1;
      if (x < same * 1.06) cls[b] = static_cast<int>(r);
      else if (x > other) other = x;
    }
    if (cls[b] < 0) {
      cls[b] = static_cast<int>(reps.size());
      reps.push_back(b);
    }
  }
  std::printf("blocks of 4 GiB, class per block (offset in the allocation grows to the right):\n");
  for (size_t b = 0; b < blocks; ++b) std::printf("%c", 'A' + cls[b]);
  std::printf("\n%zu classes; two blocks of one class %.2f TB/s, of two classes up to %.2f TB/s\n", reps.size(), same, other);
  CHECK_HIP(hipFree(buf));
  return 0;
}

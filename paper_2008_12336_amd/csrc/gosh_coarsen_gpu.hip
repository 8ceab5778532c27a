// Rebuilding the CSR of a coarse graph on the device ("Coarsen" in Alg. 4 of the paper).
//
// Every fine entry (x, y) becomes the 64-bit key map[x] * n_coarse + map[y] (entries
// inside one cluster get a sentinel key above all others); a radix sort of the keys with
// their multiplicities followed by a reduction of equal keys leaves exactly the distinct
// coarse entries, in row-major ascending order, with the merged multiplicities -- the
// same arrays the host implementation produces, since sorted distinct keys are unique.
// Sort and reduce-by-key are rocPRIM device primitives; the surrounding kernels are here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>

#include <rocprim/rocprim.hpp>

#include "gosh_coarsen_internal.h"
#include "gosh_common.h"

namespace {

// One wavefront per fine row: lanes stride over the row's entries (coalesced reads).
template <typename OffT>
__global__ __launch_bounds__(256) void make_keys_kernel(const OffT *__restrict__ xadj,
                                                        const int32_t *__restrict__ adj,
                                                        const int64_t *__restrict__ mult_in,
                                                        const int32_t *__restrict__ map, int64_t n,
                                                        uint64_t n_coarse, uint64_t sentinel,
                                                        uint64_t *__restrict__ keys,
                                                        int64_t *__restrict__ vals) {
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = (blockIdx.x * 256LL + threadIdx.x) >> 6;
  const int64_t nwaves = (gridDim.x * 256LL) >> 6;
  for (int64_t x = wave0; x < n; x += nwaves) {
    const uint64_t a = static_cast<uint64_t>(map[x]);
    const int64_t begin = static_cast<int64_t>(xadj[x]), end = static_cast<int64_t>(xadj[x + 1]);
    for (int64_t e = begin + lane; e < end; e += 64) {
      const uint64_t b = static_cast<uint64_t>(map[adj[e]]);
      keys[e] = a != b ? a * n_coarse + b : sentinel;
      vals[e] = mult_in ? mult_in[e] : 1;
    }
  }
}

// xadj_out[a] = number of distinct keys below a * n_coarse (binary search per coarse row);
// adj_out[i] = column of distinct key i.
__global__ __launch_bounds__(256) void offsets_kernel(const uint64_t *__restrict__ unique_keys,
                                                      int64_t n_unique, uint64_t n_coarse,
                                                      int64_t *__restrict__ xadj_out) {
  for (uint64_t a = blockIdx.x * 256ull + threadIdx.x; a <= n_coarse; a += gridDim.x * 256ull) {
    const uint64_t target = a * n_coarse;
    int64_t lo = 0, hi = n_unique;
    while (lo < hi) {
      const int64_t mid = lo + (hi - lo) / 2;
      if (unique_keys[mid] < target) lo = mid + 1;
      else hi = mid;
    }
    xadj_out[a] = lo;
  }
}

__global__ __launch_bounds__(256) void columns_kernel(const uint64_t *__restrict__ unique_keys,
                                                      int64_t n_unique, uint64_t n_coarse,
                                                      int32_t *__restrict__ adj_out) {
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < n_unique; i += gridDim.x * 256LL)
    adj_out[i] = static_cast<int32_t>(unique_keys[i] % n_coarse);
}

// Device blocks recycled over the levels of one run: hipMalloc and hipFree of gigabyte
// blocks cost more than the kernels of a small level.  Levels only shrink, so the blocks
// of the first level serve all later ones (best fit).
struct Pool {
  struct Block {
    void *p;
    size_t bytes;
    bool busy;
  };
  std::vector<Block> blocks;
  ~Pool() {
    for (Block &b : blocks) (void)hipFree(b.p);
  }
  void *take(size_t bytes) {
    Block *best = nullptr;
    for (Block &b : blocks)
      if (!b.busy && b.bytes >= bytes && (best == nullptr || b.bytes < best->bytes)) best = &b;
    if (best != nullptr) {
      best->busy = true;
      return best->p;
    }
    void *p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    blocks.push_back(Block{p, bytes, true});
    return p;
  }
  void give(void *p) {
    for (Block &b : blocks)
      if (b.p == p) b.busy = false;
  }
};

// The blocks one call holds; whatever is not handed on goes back to the pool on return.
struct Buffers {
  Pool &pool;
  std::vector<void *> ptrs;
  explicit Buffers(Pool &pl) : pool(pl) {}
  ~Buffers() {
    for (void *p : ptrs)
      if (p) pool.give(p);
  }
  template <typename T>
  int alloc(T **out, size_t count, const char *what) {
    const size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
    void *p = pool.take(bytes);
    if (p == nullptr) return gosh::fail(GOSH_ENOMEM, "cannot allocate %zu device bytes for %s", bytes, what);
    ptrs.push_back(p);
    *out = static_cast<T *>(p);
    return GOSH_OK;
  }
  void forget(void *p) {
    for (void *&q : ptrs)
      if (q == p) q = nullptr;
  }
  void release(void *p) {
    for (void *&q : ptrs)
      if (q == p) {
        pool.give(q);
        q = nullptr;
      }
  }
};

#define COARSE_HIP(call, what)                                                         \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) return gosh::fail(GOSH_EHIP, "%s: %s", what, hipGetErrorString(e_)); \
  } while (0)

int blocks_for(int64_t items, int per_block) {
  int64_t b = (items + per_block - 1) / per_block;
  return static_cast<int>(std::min<int64_t>(std::max<int64_t>(b, 1), 1 << 20));
}

}  // namespace

namespace gosh {

struct DeviceCarry {
  Pool pool;  // destroyed last: every block below lives in it
  int64_t n = -1, nnz = -1;
  int64_t *xadj = nullptr;
  int32_t *adj = nullptr;
  int64_t *mult = nullptr;
  // two pinned staging slots for large downloads, made on first use
  static constexpr size_t kSlotBytes = size_t(64) << 20;
  char *slot[2] = {nullptr, nullptr};
  hipStream_t stream = nullptr;
  hipEvent_t landed[2] = {nullptr, nullptr};
  ~DeviceCarry() {
    drop();
    for (int i = 0; i < 2; ++i) {
      if (slot[i]) (void)hipHostFree(slot[i]);
      if (landed[i]) (void)hipEventDestroy(landed[i]);
    }
    if (stream) (void)hipStreamDestroy(stream);
  }
  void drop() {
    if (xadj) pool.give(xadj);
    if (adj) pool.give(adj);
    if (mult) pool.give(mult);
    xadj = nullptr, adj = nullptr, mult = nullptr, n = -1, nnz = -1;
  }
};

DeviceCarry *device_carry_new() { return new DeviceCarry(); }

void device_carry_free(DeviceCarry *c) { delete c; }

namespace {

// Device -> pageable host copy.  Large copies go through two pinned slots: while one slot
// receives the next piece by DMA, all threads copy the previous one to its place (which
// also spreads the page faults of a fresh destination over the threads).
int download(void *dst, const void *src_d, size_t bytes, int threads, DeviceCarry *carry) {
  if (bytes == 0) return GOSH_OK;
  if (bytes < 4 * DeviceCarry::kSlotBytes) {
    COARSE_HIP(hipMemcpy(dst, src_d, bytes, hipMemcpyDeviceToHost), "download");
    return GOSH_OK;
  }
  if (carry->stream == nullptr) {
    COARSE_HIP(hipStreamCreate(&carry->stream), "create copy stream");
    for (int i = 0; i < 2; ++i) {
      COARSE_HIP(hipEventCreateWithFlags(&carry->landed[i], hipEventDisableTiming), "create copy event");
      void *p = nullptr;
      COARSE_HIP(hipHostMalloc(&p, DeviceCarry::kSlotBytes, hipHostMallocDefault), "allocate pinned staging");
      carry->slot[i] = static_cast<char *>(p);
    }
  }
  const size_t slot_bytes = DeviceCarry::kSlotBytes;
  const size_t pieces = (bytes + slot_bytes - 1) / slot_bytes;
  auto piece_bytes = [&](size_t c) { return std::min(slot_bytes, bytes - c * slot_bytes); };
  auto start = [&](size_t c) -> hipError_t {
    hipError_t e = hipMemcpyAsync(carry->slot[c & 1], static_cast<const char *>(src_d) + c * slot_bytes,
                                  piece_bytes(c), hipMemcpyDeviceToHost, carry->stream);
    return e != hipSuccess ? e : hipEventRecord(carry->landed[c & 1], carry->stream);
  };
  COARSE_HIP(start(0), "start download");
  for (size_t c = 0; c < pieces; ++c) {
    if (c + 1 < pieces) COARSE_HIP(start(c + 1), "start download");
    COARSE_HIP(hipEventSynchronize(carry->landed[c & 1]), "wait for download");
    char *to = static_cast<char *>(dst) + c * slot_bytes;
    const char *from = carry->slot[c & 1];
    const int64_t len = static_cast<int64_t>(piece_bytes(c));
    const int64_t grain = int64_t(1) << 20;
    const int64_t grains = (len + grain - 1) / grain;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t g = 0; g < grains; ++g)
      memcpy(to + g * grain, from + g * grain, static_cast<size_t>(std::min(grain, len - g * grain)));
  }
  return GOSH_OK;
}

}  // namespace

int build_coarse_on_device(const gosh_csr &fine, const int64_t *mult_in, const int32_t *map,
                           int64_t n_coarse, int threads, DeviceCarry *carry,
                           RawVector<int64_t> &xadj_out, RawVector<int32_t> &adj_out,
                           RawVector<int64_t> &mult_out) {
  const int64_t n = fine.n, nnz = fine.nnz;
  xadj_out.assign(static_cast<size_t>(n_coarse) + 1, 0);
  adj_out.clear();
  mult_out.clear();
  if (carry == nullptr) return gosh::fail(GOSH_EINVAL, "device state is null");
  if (nnz == 0) {
    carry->drop();
    return GOSH_OK;
  }
  const uint64_t nc = static_cast<uint64_t>(n_coarse);
  const uint64_t sentinel = nc * nc;  // above every real key
  unsigned end_bit = 1;
  while (end_bit < 64 && (sentinel >> end_bit) != 0) ++end_bit;

  Buffers buf(carry->pool);
  int32_t *map_d = nullptr;
  if (int rc = buf.alloc(&map_d, static_cast<size_t>(n), "map")) return rc;
  COARSE_HIP(hipMemcpy(map_d, map, static_cast<size_t>(n) * 4, hipMemcpyHostToDevice), "copy map");
  uint64_t *keys = nullptr, *keys_sorted = nullptr;
  int64_t *vals = nullptr, *vals_sorted = nullptr;
  if (int rc = buf.alloc(&keys, static_cast<size_t>(nnz), "keys")) return rc;
  if (int rc = buf.alloc(&vals, static_cast<size_t>(nnz), "values")) return rc;
  const int key_blocks = blocks_for(n, 4);  // four wavefronts (rows) per block
  const bool carried = carry->n == n && carry->nnz == nnz && fine.xadj_is64 && mult_in != nullptr;
  if (carried) {
    hipLaunchKernelGGL(make_keys_kernel<int64_t>, dim3(key_blocks), dim3(256), 0, nullptr, carry->xadj,
                       carry->adj, carry->mult, map_d, n, nc, sentinel, keys, vals);
    if (int rc = gosh::check_launch("make_keys_kernel")) return rc;
    COARSE_HIP(hipDeviceSynchronize(), "make keys");
  } else {
    void *xadj_d = nullptr;
    int32_t *adj_d = nullptr;
    int64_t *mult_d = nullptr;
    const size_t off_bytes = static_cast<size_t>(n + 1) * (fine.xadj_is64 ? 8 : 4);
    {
      char *p = nullptr;
      if (int rc = buf.alloc(&p, off_bytes, "offsets")) return rc;
      xadj_d = p;
    }
    if (int rc = buf.alloc(&adj_d, static_cast<size_t>(nnz), "adjacency")) return rc;
    COARSE_HIP(hipMemcpy(xadj_d, fine.xadj, off_bytes, hipMemcpyHostToDevice), "copy offsets");
    COARSE_HIP(hipMemcpy(adj_d, fine.adj, static_cast<size_t>(nnz) * 4, hipMemcpyHostToDevice), "copy adjacency");
    if (mult_in) {
      if (int rc = buf.alloc(&mult_d, static_cast<size_t>(nnz), "multiplicities")) return rc;
      COARSE_HIP(hipMemcpy(mult_d, mult_in, static_cast<size_t>(nnz) * 8, hipMemcpyHostToDevice),
                 "copy multiplicities");
    }
    if (fine.xadj_is64)
      hipLaunchKernelGGL(make_keys_kernel<int64_t>, dim3(key_blocks), dim3(256), 0, nullptr,
                         static_cast<const int64_t *>(xadj_d), adj_d, mult_d, map_d, n, nc, sentinel, keys, vals);
    else
      hipLaunchKernelGGL(make_keys_kernel<int32_t>, dim3(key_blocks), dim3(256), 0, nullptr,
                         static_cast<const int32_t *>(xadj_d), adj_d, mult_d, map_d, n, nc, sentinel, keys, vals);
    if (int rc = gosh::check_launch("make_keys_kernel")) return rc;
    COARSE_HIP(hipDeviceSynchronize(), "make keys");
    buf.release(xadj_d);
    buf.release(adj_d);
    if (mult_d) buf.release(mult_d);
  }
  // the fine graph is no longer needed on the device
  carry->drop();
  buf.release(map_d);

  if (int rc = buf.alloc(&keys_sorted, static_cast<size_t>(nnz), "sorted keys")) return rc;
  if (int rc = buf.alloc(&vals_sorted, static_cast<size_t>(nnz), "sorted values")) return rc;
  size_t temp_bytes = 0;
  COARSE_HIP(rocprim::radix_sort_pairs(nullptr, temp_bytes, keys, keys_sorted, vals, vals_sorted,
                                       static_cast<size_t>(nnz), 0u, end_bit, nullptr),
             "radix sort (size query)");
  {
    char *temp = nullptr;
    if (int rc = buf.alloc(&temp, temp_bytes, "sort workspace")) return rc;
    COARSE_HIP(rocprim::radix_sort_pairs(temp, temp_bytes, keys, keys_sorted, vals, vals_sorted,
                                         static_cast<size_t>(nnz), 0u, end_bit, nullptr),
               "radix sort");
    COARSE_HIP(hipDeviceSynchronize(), "radix sort");
    buf.release(temp);
  }
  buf.release(keys);
  buf.release(vals);
  // distinct keys and their summed multiplicities
  unsigned long long *count_d = nullptr;
  if (int rc = buf.alloc(&count_d, 1, "distinct count")) return rc;
  // at most one distinct key per fine entry; usually far fewer, but the count is only
  // known afterwards
  uint64_t *unique_keys = nullptr;
  int64_t *sums = nullptr;
  if (int rc = buf.alloc(&unique_keys, static_cast<size_t>(nnz), "distinct keys")) return rc;
  if (int rc = buf.alloc(&sums, static_cast<size_t>(nnz), "merged multiplicities")) return rc;
  temp_bytes = 0;
  COARSE_HIP(rocprim::reduce_by_key(nullptr, temp_bytes, keys_sorted, vals_sorted, static_cast<size_t>(nnz),
                                    unique_keys, sums, count_d, rocprim::plus<int64_t>(),
                                    rocprim::equal_to<uint64_t>(), nullptr),
             "reduce by key (size query)");
  unsigned long long n_unique = 0;
  {
    char *temp = nullptr;
    if (int rc = buf.alloc(&temp, temp_bytes, "reduce workspace")) return rc;
    COARSE_HIP(rocprim::reduce_by_key(temp, temp_bytes, keys_sorted, vals_sorted, static_cast<size_t>(nnz),
                                      unique_keys, sums, count_d, rocprim::plus<int64_t>(),
                                      rocprim::equal_to<uint64_t>(), nullptr),
               "reduce by key");
    COARSE_HIP(hipMemcpy(&n_unique, count_d, sizeof(n_unique), hipMemcpyDeviceToHost), "copy distinct count");
    buf.release(temp);
  }
  buf.release(keys_sorted);
  buf.release(vals_sorted);
  // entries inside clusters collapse into one sentinel key, the largest: drop it
  if (n_unique > 0) {
    uint64_t last = 0;
    COARSE_HIP(hipMemcpy(&last, unique_keys + (n_unique - 1), 8, hipMemcpyDeviceToHost), "copy last key");
    if (last == sentinel) --n_unique;
  }
  const int64_t nnz_coarse = static_cast<int64_t>(n_unique);

  adj_out.resize(static_cast<size_t>(nnz_coarse));
  mult_out.resize(static_cast<size_t>(nnz_coarse));

  int64_t *xadj_out_d = nullptr;
  int32_t *adj_out_d = nullptr;
  if (int rc = buf.alloc(&xadj_out_d, static_cast<size_t>(n_coarse) + 1, "coarse offsets")) return rc;
  if (int rc = buf.alloc(&adj_out_d, static_cast<size_t>(nnz_coarse), "coarse adjacency")) return rc;
  hipLaunchKernelGGL(offsets_kernel, dim3(blocks_for(n_coarse + 1, 256)), dim3(256), 0, nullptr, unique_keys,
                     nnz_coarse, nc, xadj_out_d);
  if (int rc = gosh::check_launch("offsets_kernel")) return rc;
  if (nnz_coarse > 0) {
    hipLaunchKernelGGL(columns_kernel, dim3(blocks_for(nnz_coarse, 256)), dim3(256), 0, nullptr, unique_keys,
                       nnz_coarse, nc, adj_out_d);
    if (int rc = gosh::check_launch("columns_kernel")) return rc;
  }
  COARSE_HIP(hipDeviceSynchronize(), "coarse CSR");
  if (int rc = download(xadj_out.data(), xadj_out_d, (static_cast<size_t>(n_coarse) + 1) * 8, threads, carry)) return rc;
  if (int rc = download(adj_out.data(), adj_out_d, static_cast<size_t>(nnz_coarse) * 4, threads, carry)) return rc;
  if (int rc = download(mult_out.data(), sums, static_cast<size_t>(nnz_coarse) * 8, threads, carry)) return rc;
  buf.release(unique_keys);
  if (nnz_coarse > 0) {
    // hand the coarse graph to the next level: these three buffers now belong to carry
    carry->n = n_coarse;
    carry->nnz = nnz_coarse;
    carry->xadj = xadj_out_d;
    carry->adj = adj_out_d;
    carry->mult = sums;
    buf.forget(xadj_out_d);
    buf.forget(adj_out_d);
    buf.forget(sums);
  }
  return GOSH_OK;
}

}  // namespace gosh

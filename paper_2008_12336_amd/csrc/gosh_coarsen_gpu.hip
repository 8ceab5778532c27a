// MultiEdgeCollapse (Alg. 4 of the paper) on the device: the degree order, the marking
// sweep and the rebuild of the coarse CSR, with the results of the sequential algorithm.
//
// Order: a stable radix sort of the vertex ids by descending degree.
//
// Marking: in the sequential sweep a vertex becomes a hub iff none of the neighbours that
// precede it in the order and may take it (one of the two degrees is at most the mean
// degree) is itself a hub.  That recurrence is resolved out of order: a vertex above the
// mean degree is always a hub, a low-degree vertex with such a neighbour never is, and
// the remaining low-degree vertices are decided in rounds (hub once every preceding
// neighbour is decided and none is a hub, taken as soon as one is).  A decision is final
// and equals the sequential one, so stale reads can only delay it.  Hubs are numbered by
// a scan over the order; every other vertex joins its first hub in the order.
//
// Rebuild: every fine entry (x, y) becomes the 64-bit key map[x] * n' + map[y] (entries
// inside one cluster get a sentinel key above all others); a radix sort of the keys with
// their multiplicities followed by a reduction of equal keys leaves exactly the distinct
// coarse entries, in row-major ascending order, with the merged multiplicities -- the
// same arrays the host implementation produces, since sorted distinct keys are unique.
// The keys are made one thread per entry (the row of an entry is found by a search that a
// block narrows to the few rows it spans), so hub rows are no long tail.
//
// Sort, scan and reduce-by-key are rocPRIM device primitives; the kernels around them
// are here.  Everything runs on the null stream and the calls block.
#include <hip/hip_runtime.h>
#include <omp.h>

#include <algorithm>
#include <chrono>
#include <cstring>

#include <rocprim/rocprim.hpp>

#include "gosh_coarsen_internal.h"
#include "gosh_common.h"

namespace {

constexpr uint32_t kHighBit = 0x80000000u;   // set in rk[v] when deg(v) is above the mean
constexpr uint32_t kRankMask = 0x7FFFFFFFu;  // rk[v] & kRankMask = position of v in the order
enum : int32_t { kUndecided = 0, kHub = 1, kTaken = 2 };

__device__ inline int64_t first_wave() { return (blockIdx.x * 256LL + threadIdx.x) >> 6; }
__device__ inline int64_t wave_count() { return (gridDim.x * 256LL) >> 6; }

__device__ inline int32_t load_status(const int32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store_status(int32_t *p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// key = 2^31 - 1 - degree: ascending keys are descending degrees; stable => ties by id.
template <typename OffT>
__global__ __launch_bounds__(256) void degree_keys_kernel(const OffT *__restrict__ xadj, int64_t n,
                                                          uint32_t *__restrict__ keys,
                                                          int32_t *__restrict__ ids) {
  for (int64_t v = blockIdx.x * 256LL + threadIdx.x; v < n; v += gridDim.x * 256LL) {
    keys[v] = kRankMask - static_cast<uint32_t>(xadj[v + 1] - xadj[v]);
    ids[v] = static_cast<int32_t>(v);
  }
}

// rk[order[t]] = t, with the high bit set when the degree exceeds the mean degree
// (deg * n > nnz, exact in 64-bit integers).
__global__ __launch_bounds__(256) void rank_kernel(const uint32_t *__restrict__ sorted_keys,
                                                   const int32_t *__restrict__ order, int64_t n,
                                                   int64_t nnz, uint32_t *__restrict__ rk) {
  for (int64_t t = blockIdx.x * 256LL + threadIdx.x; t < n; t += gridDim.x * 256LL) {
    const int64_t deg = static_cast<int64_t>(kRankMask - sorted_keys[t]);
    rk[order[t]] = static_cast<uint32_t>(t) | (deg * n > nnz ? kHighBit : 0u);
  }
}

// First classification, one wavefront per vertex: needs no knowledge of other decisions.
template <typename OffT>
__global__ __launch_bounds__(256) void classify_kernel(const OffT *__restrict__ xadj,
                                                       const int32_t *__restrict__ adj,
                                                       const uint32_t *__restrict__ rk, int64_t n,
                                                       int32_t *__restrict__ status,
                                                       int32_t *__restrict__ pending,
                                                       unsigned long long *__restrict__ pending_count) {
  const int lane = threadIdx.x & 63;
  for (int64_t v = first_wave(); v < n; v += wave_count()) {
    const uint32_t r = rk[v];
    int32_t st = kHub;
    if (!(r & kHighBit)) {
      bool high_neighbour = false, predecessor = false;
      const int64_t begin = static_cast<int64_t>(xadj[v]), end = static_cast<int64_t>(xadj[v + 1]);
      for (int64_t e = begin + lane; e < end; e += 64) {
        const uint32_t ru = rk[adj[e]];
        high_neighbour |= (ru & kHighBit) != 0;
        predecessor |= (ru & kRankMask) < r;
      }
      if (__ballot(high_neighbour) != 0) st = kTaken;
      else if (__ballot(predecessor) != 0) st = kUndecided;
    }
    if (lane == 0) {
      status[v] = st;
      if (st == kUndecided) pending[atomicAdd(pending_count, 1ull)] = static_cast<int32_t>(v);
    }
  }
}

// One round over the undecided vertices, one wavefront per vertex.
template <typename OffT>
__global__ __launch_bounds__(256) void round_kernel(const OffT *__restrict__ xadj,
                                                    const int32_t *__restrict__ adj,
                                                    const uint32_t *__restrict__ rk,
                                                    int32_t *status,  // shared with other waves
                                                    const int32_t *__restrict__ pending, int64_t count,
                                                    int32_t *__restrict__ still,
                                                    unsigned long long *__restrict__ still_count) {
  const int lane = threadIdx.x & 63;
  for (int64_t i = first_wave(); i < count; i += wave_count()) {
    const int32_t v = pending[i];
    const uint32_t r = rk[v];  // low degree: no high bit
    bool taken = false, blocked = false;
    const int64_t begin = static_cast<int64_t>(xadj[v]), end = static_cast<int64_t>(xadj[v + 1]);
    for (int64_t e = begin + lane; e < end; e += 64) {
      const int32_t u = adj[e];
      if ((rk[u] & kRankMask) < r) {
        const int32_t su = load_status(status + u);
        taken |= su == kHub;
        blocked |= su == kUndecided;
      }
    }
    const bool any_taken = __ballot(taken) != 0, any_blocked = __ballot(blocked) != 0;
    if (lane == 0) {
      if (any_taken) store_status(status + v, kTaken);
      else if (!any_blocked) store_status(status + v, kHub);
      else still[atomicAdd(still_count, 1ull)] = v;
    }
  }
}

__global__ __launch_bounds__(256) void hub_flags_kernel(const int32_t *__restrict__ status,
                                                        const int32_t *__restrict__ order, int64_t n,
                                                        int32_t *__restrict__ flags) {
  for (int64_t t = blockIdx.x * 256LL + threadIdx.x; t < n; t += gridDim.x * 256LL)
    flags[t] = status[order[t]] == kHub ? 1 : 0;
}

// Cluster ids are the hubs' positions among the hubs in the order.
__global__ __launch_bounds__(256) void number_hubs_kernel(const int32_t *__restrict__ flags,
                                                          const int32_t *__restrict__ index,
                                                          const int32_t *__restrict__ order, int64_t n,
                                                          int32_t *__restrict__ map) {
  for (int64_t t = blockIdx.x * 256LL + threadIdx.x; t < n; t += gridDim.x * 256LL)
    if (flags[t]) map[order[t]] = index[t];
}

// Every taken vertex joins its first hub in the order, one wavefront per vertex.  The
// hubs' own entries of map (read here) were written by the launch before this one; this
// launch writes only entries of taken vertices.
template <typename OffT>
__global__ __launch_bounds__(256) void join_kernel(const OffT *__restrict__ xadj,
                                                   const int32_t *__restrict__ adj,
                                                   const uint32_t *__restrict__ rk,
                                                   const int32_t *__restrict__ status,
                                                   const int32_t *__restrict__ order, int64_t n,
                                                   int32_t *map) {
  const int lane = threadIdx.x & 63;
  for (int64_t v = first_wave(); v < n; v += wave_count()) {
    if (status[v] != kTaken) continue;
    const uint32_t r = rk[v];
    uint32_t best = kRankMask;
    const int64_t begin = static_cast<int64_t>(xadj[v]), end = static_cast<int64_t>(xadj[v + 1]);
    for (int64_t e = begin + lane; e < end; e += 64) {
      const int32_t u = adj[e];
      const uint32_t ru = rk[u] & kRankMask;
      if (ru < r && ru < best && status[u] == kHub) best = ru;
    }
    for (int offset = 32; offset > 0; offset >>= 1) best = min(best, __shfl_xor(best, offset, 64));
    // a taken vertex has a hub before it, so best is a valid position; the guard keeps a
    // broken invariant from turning into a wild read
    if (lane == 0 && best < static_cast<uint32_t>(n)) map[v] = map[order[best]];
  }
}

// Shape checks before any kernel follows the offsets or the neighbour ids: *bad becomes
// nonzero if the offsets do not run from 0 to nnz without decreasing, or (second kernel)
// if a neighbour id is outside [0, n).
template <typename OffT>
__global__ __launch_bounds__(256) void check_offsets_kernel(const OffT *__restrict__ xadj, int64_t n,
                                                            int64_t nnz, int32_t *__restrict__ bad) {
  for (int64_t v = blockIdx.x * 256LL + threadIdx.x; v < n; v += gridDim.x * 256LL) {
    const int64_t lo = static_cast<int64_t>(xadj[v]), hi = static_cast<int64_t>(xadj[v + 1]);
    if (lo > hi || lo < 0 || hi > nnz || (v == 0 && lo != 0) || (v == n - 1 && hi != nnz)) *bad = 1;
  }
}

__global__ __launch_bounds__(256) void check_neighbours_kernel(const int32_t *__restrict__ adj, int64_t nnz,
                                                               int64_t n, int32_t *__restrict__ bad) {
  for (int64_t e = blockIdx.x * 256LL + threadIdx.x; e < nnz; e += gridDim.x * 256LL)
    if (adj[e] < 0 || adj[e] >= n) *bad = 1;
}

// Largest row r in [lo, hi] with xadj[r] <= e, i.e. the row that holds entry e (empty rows
// share their offset with the next row and are skipped).
template <typename OffT>
__device__ inline int64_t row_of_entry(const OffT *__restrict__ xadj, int64_t lo, int64_t hi, int64_t e) {
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo + 1) / 2;
    if (static_cast<int64_t>(xadj[mid]) <= e) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

// One thread per fine entry, kKeysPerBlock consecutive entries per block: the block first
// finds the rows of its first and last entry, then every thread searches only between
// them (a handful of rows; none at all inside a hub's row), so hubs and short rows cost
// the same per entry and all accesses to adj, keys and vals are coalesced.
constexpr int kKeysPerBlock = 4096;
template <typename OffT>
__global__ __launch_bounds__(256) void make_keys_kernel(const OffT *__restrict__ xadj,
                                                        const int32_t *__restrict__ adj,
                                                        const int64_t *__restrict__ mult_in,
                                                        const int32_t *__restrict__ map, int64_t n,
                                                        int64_t nnz, uint64_t n_coarse, uint64_t sentinel,
                                                        uint64_t *__restrict__ keys,
                                                        int64_t *__restrict__ vals) {
  __shared__ int64_t span[2];
  for (int64_t e0 = static_cast<int64_t>(blockIdx.x) * kKeysPerBlock; e0 < nnz;
       e0 += static_cast<int64_t>(gridDim.x) * kKeysPerBlock) {
    const int64_t e_last = min(e0 + kKeysPerBlock, nnz) - 1;
    if (threadIdx.x < 2) span[threadIdx.x] = row_of_entry(xadj, 0, n - 1, threadIdx.x == 0 ? e0 : e_last);
    __syncthreads();
    const int64_t row_lo = span[0], row_hi = span[1];
    for (int64_t e = e0 + threadIdx.x; e <= e_last; e += 256) {
      const int64_t x = row_of_entry(xadj, row_lo, row_hi, e);
      const uint64_t a = static_cast<uint64_t>(map[x]);
      const uint64_t b = static_cast<uint64_t>(map[adj[e]]);
      keys[e] = a != b ? a * n_coarse + b : sentinel;
      if (mult_in) vals[e] = mult_in[e];  // without multiplicities every entry counts once
    }
    __syncthreads();  // span is rewritten in the next round
  }
}

// xadj_out[a] = number of distinct keys below a * n_coarse (binary search per coarse row).
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

// adj_out[i] = column of distinct key i; mult_out[i] = its merged multiplicity.
__global__ __launch_bounds__(256) void columns_kernel(const uint64_t *__restrict__ unique_keys,
                                                      const int64_t *__restrict__ sums, int64_t n_unique,
                                                      uint64_t n_coarse, int32_t *__restrict__ adj_out,
                                                      int64_t *__restrict__ mult_out) {
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < n_unique; i += gridDim.x * 256LL) {
    adj_out[i] = static_cast<int32_t>(unique_keys[i] % n_coarse);
    mult_out[i] = sums[i];
  }
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
  ~Pool() { trim(); }
  void trim() {
    for (Block &b : blocks) (void)hipFree(b.p);
    blocks.clear();
  }
  void *take(size_t bytes) {
    // best fit, but a small request never occupies a block that a large one will want
    const size_t too_big = std::max<size_t>(bytes * 8, size_t(64) << 20);
    Block *best = nullptr;
    for (Block &b : blocks)
      if (!b.busy && b.bytes >= bytes && b.bytes <= too_big && (best == nullptr || b.bytes < best->bytes))
        best = &b;
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

// The blocks one call holds; they go back to the pool on return.
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
  void release(void *p) {
    for (void *&q : ptrs)
      if (q == p) {
        pool.give(q);
        q = nullptr;
      }
  }
};

int blocks_for(int64_t items, int per_block) {
  int64_t b = (items + per_block - 1) / per_block;
  return static_cast<int>(std::min<int64_t>(std::max<int64_t>(b, 1), 1 << 16));
}

// Exact-sized block that outlives the run (a level's array).
template <typename T>
int persistent(T **out, size_t count, const char *what) {
  void *p = nullptr;
  const size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
  if (hipMalloc(&p, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return gosh::fail(GOSH_ENOMEM, "cannot allocate %zu device bytes for %s", bytes, what);
  }
  *out = static_cast<T *>(p);
  return GOSH_OK;
}

double ms_since(std::chrono::steady_clock::time_point t0) {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

}  // namespace

namespace gosh {

struct DeviceCoarsener {
  Pool pool;
  int threads = 1;
  // Two pinned staging slots for large downloads, made on first use and kept.  The copy
  // stream is NOT kept: a process has few hardware queues, and an idle stream of ours
  // would make the streams of a later training call share one.
  static constexpr size_t kSlotBytes = size_t(64) << 20;
  char *slot[2] = {nullptr, nullptr};
  ~DeviceCoarsener() {
    for (int i = 0; i < 2; ++i)
      if (slot[i]) (void)hipHostFree(slot[i]);
  }
};

DeviceCoarsener *device_coarsener_new(int threads) {
  DeviceCoarsener *dc = new DeviceCoarsener();
  dc->threads = std::max(threads, 1);
  return dc;
}

void device_coarsener_free(DeviceCoarsener *dc) { delete dc; }

void device_coarsener_trim(DeviceCoarsener *dc) {
  if (dc) dc->pool.trim();
}

void device_level_free(DeviceLevel &level) {
  if (level.xadj && !level.borrowed_graph) (void)hipFree(level.xadj);
  if (level.adj && !level.borrowed_graph) (void)hipFree(level.adj);
  if (level.mult) (void)hipFree(level.mult);
  if (level.map) (void)hipFree(level.map);
  level = DeviceLevel();
}

void device_level_drop_map(DeviceLevel &level) {
  if (level.map) (void)hipFree(level.map);
  level.map = nullptr;
}

int device_level_upload(DeviceCoarsener *dc, const gosh_csr &host, DeviceLevel &out) {
  device_level_free(out);
  GOSH_TRY_HIP(hipGetDevice(&out.device), "hipGetDevice");
  out.n = host.n;
  out.nnz = host.nnz;
  out.xadj_is64 = host.xadj_is64 ? 1 : 0;
  const size_t off_bytes = static_cast<size_t>(host.n + 1) * (host.xadj_is64 ? 8 : 4);
  char *offsets = nullptr;
  if (int rc = persistent(&offsets, off_bytes, "offsets")) return rc;
  out.xadj = offsets;
  if (int rc = persistent(&out.adj, static_cast<size_t>(host.nnz), "adjacency")) return rc;
  if (int rc = device_upload(dc, out.xadj, host.xadj, off_bytes)) return rc;
  if (int rc = device_upload(dc, out.adj, host.adj, static_cast<size_t>(host.nnz) * 4)) return rc;
  return device_level_check(out);
}

int device_level_borrow(const gosh_csr &on_device, DeviceLevel &out) {
  device_level_free(out);
  GOSH_TRY_HIP(hipGetDevice(&out.device), "hipGetDevice");
  out.n = on_device.n;
  out.nnz = on_device.nnz;
  out.xadj_is64 = on_device.xadj_is64 ? 1 : 0;
  out.xadj = const_cast<void *>(on_device.xadj);
  out.adj = const_cast<int32_t *>(on_device.adj);
  out.borrowed_graph = true;
  return device_level_check(out);
}

bool is_device_pointer(const void *p) {
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
    (void)hipGetLastError();  // plain pageable memory is unknown to the runtime
    return false;
  }
  return attr.type == hipMemoryTypeDevice;
}

// The kernels follow offsets and neighbour ids without further checks: verify them once.
int device_level_check(const DeviceLevel &out) {
  const gosh_csr host{out.n, out.nnz, out.xadj, out.adj, out.xadj_is64};
  int32_t *bad_dev = nullptr;
  if (int rc = persistent(&bad_dev, 1, "check flag")) return rc;
  struct FlagGuard {
    int32_t *p;
    ~FlagGuard() { (void)hipFree(p); }
  } guard{bad_dev};
  int32_t bad = 0;
  GOSH_TRY_HIP(hipMemset(bad_dev, 0, 4), "clear check flag");
  const int off_blocks = blocks_for(host.n, 256);
  if (host.xadj_is64)
    hipLaunchKernelGGL(check_offsets_kernel<int64_t>, dim3(off_blocks), dim3(256), 0, nullptr,
                       static_cast<const int64_t *>(out.xadj), out.n, out.nnz, bad_dev);
  else
    hipLaunchKernelGGL(check_offsets_kernel<int32_t>, dim3(off_blocks), dim3(256), 0, nullptr,
                       static_cast<const int32_t *>(out.xadj), out.n, out.nnz, bad_dev);
  if (int rc = gosh::check_launch("check_offsets_kernel")) return rc;
  GOSH_TRY_HIP(hipMemcpy(&bad, bad_dev, 4, hipMemcpyDeviceToHost), "read check flag");
  if (bad) return gosh::fail(GOSH_EINVAL, "xadj does not run from 0 to nnz without decreasing");
  if (host.nnz > 0) {
    hipLaunchKernelGGL(check_neighbours_kernel, dim3(blocks_for(host.nnz, 256)), dim3(256), 0, nullptr, out.adj,
                       out.nnz, out.n, bad_dev);
    if (int rc = gosh::check_launch("check_neighbours_kernel")) return rc;
    GOSH_TRY_HIP(hipMemcpy(&bad, bad_dev, 4, hipMemcpyDeviceToHost), "read check flag");
    if (bad) return gosh::fail(GOSH_EINVAL, "a neighbour id is outside [0, n)");
  }
  return GOSH_OK;
}

int device_level_set_map(DeviceLevel &level, const int32_t *map_host) {
  if (level.map == nullptr)
    if (int rc = persistent(&level.map, static_cast<size_t>(level.n), "map")) return rc;
  GOSH_TRY_HIP(hipMemcpy(level.map, map_host, static_cast<size_t>(level.n) * 4, hipMemcpyHostToDevice), "copy map");
  return GOSH_OK;
}

namespace {

// Copies between pageable host memory and the device through two pinned slots, so that the
// DMA of one piece overlaps the host-side copy of the next, which all threads share (on a
// download that also spreads the page faults of a fresh destination over the threads).
// The copy stream lives only for the call.
struct StagedCopy {
  DeviceCoarsener *dc;
  hipStream_t stream = nullptr;
  hipEvent_t done[2] = {nullptr, nullptr};  // the DMA that last used slot i
  explicit StagedCopy(DeviceCoarsener *d) : dc(d) {}
  ~StagedCopy() {
    for (int i = 0; i < 2; ++i)
      if (done[i]) (void)hipEventDestroy(done[i]);
    if (stream) (void)hipStreamDestroy(stream);
  }
  int open() {
    for (int i = 0; i < 2; ++i)
      if (dc->slot[i] == nullptr) {
        void *p = nullptr;
        GOSH_TRY_HIP(hipHostMalloc(&p, DeviceCoarsener::kSlotBytes, hipHostMallocDefault), "allocate pinned staging");
        dc->slot[i] = static_cast<char *>(p);
      }
    GOSH_TRY_HIP(hipStreamCreate(&stream), "create copy stream");
    for (int i = 0; i < 2; ++i)
      GOSH_TRY_HIP(hipEventCreateWithFlags(&done[i], hipEventDisableTiming), "create copy event");
    return GOSH_OK;
  }
  void host_copy(char *to, const char *from, size_t bytes) const {
    const int64_t len = static_cast<int64_t>(bytes);
    const int64_t grain = int64_t(1) << 20;
    const int64_t grains = (len + grain - 1) / grain;
#pragma omp parallel for num_threads(dc->threads) schedule(static)
    for (int64_t g = 0; g < grains; ++g)
      memcpy(to + g * grain, from + g * grain, static_cast<size_t>(std::min(grain, len - g * grain)));
  }
};

bool is_pinned_host(const void *p) {
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
    (void)hipGetLastError();  // plain pageable memory is unknown to the runtime
    return false;
  }
  return attr.type == hipMemoryTypeHost;
}

}  // namespace

int device_download(DeviceCoarsener *dc, void *dst, const void *src_dev, size_t bytes) {
  if (bytes == 0) return GOSH_OK;
  if (dc == nullptr || bytes < 4 * DeviceCoarsener::kSlotBytes) {
    GOSH_TRY_HIP(hipMemcpy(dst, src_dev, bytes, hipMemcpyDeviceToHost), "download");
    return GOSH_OK;
  }
  StagedCopy q(dc);
  if (int rc = q.open()) return rc;
  const size_t slot_bytes = DeviceCoarsener::kSlotBytes;
  const size_t pieces = (bytes + slot_bytes - 1) / slot_bytes;
  auto piece_bytes = [&](size_t c) { return std::min(slot_bytes, bytes - c * slot_bytes); };
  auto start = [&](size_t c) -> hipError_t {
    hipError_t e = hipMemcpyAsync(dc->slot[c & 1], static_cast<const char *>(src_dev) + c * slot_bytes,
                                  piece_bytes(c), hipMemcpyDeviceToHost, q.stream);
    return e != hipSuccess ? e : hipEventRecord(q.done[c & 1], q.stream);
  };
  GOSH_TRY_HIP(start(0), "start download");
  for (size_t c = 0; c < pieces; ++c) {
    // slot (c + 1) & 1 was emptied in the previous iteration
    if (c + 1 < pieces) GOSH_TRY_HIP(start(c + 1), "start download");
    GOSH_TRY_HIP(hipEventSynchronize(q.done[c & 1]), "wait for download");
    q.host_copy(static_cast<char *>(dst) + c * slot_bytes, dc->slot[c & 1], piece_bytes(c));
  }
  return GOSH_OK;
}

int device_upload(DeviceCoarsener *dc, void *dst_dev, const void *src, size_t bytes) {
  if (bytes == 0) return GOSH_OK;
  if (dc == nullptr || bytes < 4 * DeviceCoarsener::kSlotBytes || is_pinned_host(src)) {
    GOSH_TRY_HIP(hipMemcpy(dst_dev, src, bytes, hipMemcpyHostToDevice), "upload");
    return GOSH_OK;
  }
  StagedCopy q(dc);
  if (int rc = q.open()) return rc;
  const size_t slot_bytes = DeviceCoarsener::kSlotBytes;
  const size_t pieces = (bytes + slot_bytes - 1) / slot_bytes;
  for (size_t c = 0; c < pieces; ++c) {
    const size_t len = std::min(slot_bytes, bytes - c * slot_bytes);
    // the DMA of piece c - 2 must have drained this slot
    if (c >= 2) GOSH_TRY_HIP(hipEventSynchronize(q.done[c & 1]), "wait for upload");
    q.host_copy(dc->slot[c & 1], static_cast<const char *>(src) + c * slot_bytes, len);
    GOSH_TRY_HIP(hipMemcpyAsync(static_cast<char *>(dst_dev) + c * slot_bytes, dc->slot[c & 1], len,
                              hipMemcpyHostToDevice, q.stream), "upload piece");
    GOSH_TRY_HIP(hipEventRecord(q.done[c & 1], q.stream), "record upload");
  }
  GOSH_TRY_HIP(hipStreamSynchronize(q.stream), "finish upload");
  return GOSH_OK;
}

namespace {

template <typename OffT>
int mark_impl(DeviceCoarsener *dc, DeviceLevel &fine, int64_t *n_coarse, bool *done, double *order_ms) {
  const int64_t n = fine.n, nnz = fine.nnz;
  const OffT *xadj = static_cast<const OffT *>(fine.xadj);
  const int32_t *adj = fine.adj;
  *done = false;
  Buffers buf(dc->pool);
  const auto t_order = std::chrono::steady_clock::now();

  // degree order
  uint32_t *keys = nullptr, *keys_sorted = nullptr, *rk = nullptr;
  int32_t *ids = nullptr, *order = nullptr;
  if (int rc = buf.alloc(&keys, static_cast<size_t>(n), "degree keys")) return rc;
  if (int rc = buf.alloc(&keys_sorted, static_cast<size_t>(n), "sorted degree keys")) return rc;
  if (int rc = buf.alloc(&ids, static_cast<size_t>(n), "vertex ids")) return rc;
  if (int rc = buf.alloc(&order, static_cast<size_t>(n), "order")) return rc;
  if (int rc = buf.alloc(&rk, static_cast<size_t>(n), "ranks")) return rc;
  const int flat_blocks = blocks_for(n, 256);
  hipLaunchKernelGGL(degree_keys_kernel<OffT>, dim3(flat_blocks), dim3(256), 0, nullptr, xadj, n, keys, ids);
  if (int rc = gosh::check_launch("degree_keys_kernel")) return rc;
  {
    size_t temp_bytes = 0;
    GOSH_TRY_HIP(rocprim::radix_sort_pairs(nullptr, temp_bytes, keys, keys_sorted, ids, order,
                                         static_cast<size_t>(n), 0u, 31u, nullptr),
               "degree sort (size query)");
    char *temp = nullptr;
    if (int rc = buf.alloc(&temp, temp_bytes, "sort workspace")) return rc;
    GOSH_TRY_HIP(rocprim::radix_sort_pairs(temp, temp_bytes, keys, keys_sorted, ids, order,
                                         static_cast<size_t>(n), 0u, 31u, nullptr),
               "degree sort");
    GOSH_TRY_HIP(hipDeviceSynchronize(), "degree sort");
    buf.release(temp);
  }
  hipLaunchKernelGGL(rank_kernel, dim3(flat_blocks), dim3(256), 0, nullptr, keys_sorted, order, n, nnz, rk);
  if (int rc = gosh::check_launch("rank_kernel")) return rc;
  GOSH_TRY_HIP(hipDeviceSynchronize(), "ranks");
  buf.release(keys);
  buf.release(keys_sorted);
  buf.release(ids);
  *order_ms = ms_since(t_order);

  // first classification
  int32_t *status = nullptr, *pending = nullptr, *still = nullptr;
  unsigned long long *counters = nullptr;  // sizes of the two pending lists
  if (int rc = buf.alloc(&status, static_cast<size_t>(n), "status")) return rc;
  if (int rc = buf.alloc(&pending, static_cast<size_t>(n), "pending list")) return rc;
  if (int rc = buf.alloc(&still, static_cast<size_t>(n), "pending list")) return rc;
  if (int rc = buf.alloc(&counters, 2, "pending counters")) return rc;
  GOSH_TRY_HIP(hipMemset(counters, 0, 16), "clear counters");
  const int wave_blocks = blocks_for(n, 4);  // four wavefronts (vertices) per block
  hipLaunchKernelGGL(classify_kernel<OffT>, dim3(wave_blocks), dim3(256), 0, nullptr, xadj, adj, rk, n, status,
                     pending, counters);
  if (int rc = gosh::check_launch("classify_kernel")) return rc;
  unsigned long long count = 0;
  GOSH_TRY_HIP(hipMemcpy(&count, counters, 8, hipMemcpyDeviceToHost), "read pending count");

  // rounds: each decides at least the first pending vertex of the order, usually most
  const int kMaxRounds = 256;
  int which = 0;  // counters[which] is the size of `pending`
  for (int round = 0; count > 0; ++round) {
    if (round == kMaxRounds) return GOSH_OK;  // *done stays false
    GOSH_TRY_HIP(hipMemset(counters + (which ^ 1), 0, 8), "clear counter");
    hipLaunchKernelGGL(round_kernel<OffT>, dim3(blocks_for(static_cast<int64_t>(count), 4)), dim3(256), 0, nullptr,
                       xadj, adj, rk, status, pending, static_cast<int64_t>(count), still, counters + (which ^ 1));
    if (int rc = gosh::check_launch("round_kernel")) return rc;
    unsigned long long left = 0;
    GOSH_TRY_HIP(hipMemcpy(&left, counters + (which ^ 1), 8, hipMemcpyDeviceToHost), "read pending count");
    // a long chain: a few vertices per round would take forever
    if (round >= 16 && left > 4096 && left * 100 > count * 99) return GOSH_OK;
    std::swap(pending, still);
    which ^= 1;
    count = left;
  }
  buf.release(pending);
  buf.release(still);

  // number the hubs in the order
  int32_t *flags = nullptr, *index = nullptr;
  if (int rc = buf.alloc(&flags, static_cast<size_t>(n), "hub flags")) return rc;
  if (int rc = buf.alloc(&index, static_cast<size_t>(n), "hub numbers")) return rc;
  hipLaunchKernelGGL(hub_flags_kernel, dim3(flat_blocks), dim3(256), 0, nullptr, status, order, n, flags);
  if (int rc = gosh::check_launch("hub_flags_kernel")) return rc;
  {
    size_t temp_bytes = 0;
    GOSH_TRY_HIP(rocprim::exclusive_scan(nullptr, temp_bytes, flags, index, int32_t(0), static_cast<size_t>(n),
                                       rocprim::plus<int32_t>(), nullptr),
               "hub scan (size query)");
    char *temp = nullptr;
    if (int rc = buf.alloc(&temp, temp_bytes, "scan workspace")) return rc;
    GOSH_TRY_HIP(rocprim::exclusive_scan(temp, temp_bytes, flags, index, int32_t(0), static_cast<size_t>(n),
                                       rocprim::plus<int32_t>(), nullptr),
               "hub scan");
    GOSH_TRY_HIP(hipDeviceSynchronize(), "hub scan");
    buf.release(temp);
  }
  int32_t last_flag = 0, last_index = 0;
  GOSH_TRY_HIP(hipMemcpy(&last_flag, flags + (n - 1), 4, hipMemcpyDeviceToHost), "read hub count");
  GOSH_TRY_HIP(hipMemcpy(&last_index, index + (n - 1), 4, hipMemcpyDeviceToHost), "read hub count");
  if (fine.map == nullptr)
    if (int rc = persistent(&fine.map, static_cast<size_t>(n), "map")) return rc;
  hipLaunchKernelGGL(number_hubs_kernel, dim3(flat_blocks), dim3(256), 0, nullptr, flags, index, order, n, fine.map);
  if (int rc = gosh::check_launch("number_hubs_kernel")) return rc;
  hipLaunchKernelGGL(join_kernel<OffT>, dim3(wave_blocks), dim3(256), 0, nullptr, xadj, adj, rk, status, order, n,
                     fine.map);
  if (int rc = gosh::check_launch("join_kernel")) return rc;
  GOSH_TRY_HIP(hipDeviceSynchronize(), "marking");
  *n_coarse = static_cast<int64_t>(last_flag) + last_index;
  *done = true;
  return GOSH_OK;
}

}  // namespace

int device_mark(DeviceCoarsener *dc, DeviceLevel &fine, int64_t *n_coarse, bool *done, double *order_ms) {
  if (dc == nullptr || !fine.present() || fine.n < 1) return gosh::fail(GOSH_EINVAL, "device level is missing");
  return fine.xadj_is64 ? mark_impl<int64_t>(dc, fine, n_coarse, done, order_ms)
                        : mark_impl<int32_t>(dc, fine, n_coarse, done, order_ms);
}

int device_rebuild(DeviceCoarsener *dc, const DeviceLevel &fine, int64_t n_coarse, DeviceLevel &coarse) {
  if (dc == nullptr || !fine.present() || fine.map == nullptr)
    return gosh::fail(GOSH_EINVAL, "device level or its map is missing");
  device_level_free(coarse);
  const int64_t n = fine.n, nnz = fine.nnz;
  const uint64_t nc = static_cast<uint64_t>(n_coarse);
  const uint64_t sentinel = nc * nc;  // above every real key
  unsigned end_bit = 1;
  while (end_bit < 64 && (sentinel >> end_bit) != 0) ++end_bit;
  coarse.device = fine.device;
  coarse.n = n_coarse;
  coarse.xadj_is64 = 1;
  int64_t *xadj_out = nullptr;
  if (int rc = persistent(&xadj_out, static_cast<size_t>(n_coarse) + 1, "coarse offsets")) return rc;
  coarse.xadj = xadj_out;
  if (nnz == 0) {
    coarse.nnz = 0;
    GOSH_TRY_HIP(hipMemset(xadj_out, 0, (static_cast<size_t>(n_coarse) + 1) * 8), "clear coarse offsets");
    if (int rc = persistent(&coarse.adj, 0, "coarse adjacency")) return rc;
    if (int rc = persistent(&coarse.mult, 0, "coarse multiplicities")) return rc;
    return GOSH_OK;
  }

  Buffers buf(dc->pool);
  // G_0 carries no multiplicities (every entry counts once): its keys are sorted alone and
  // the reduction adds a constant 1 per key, which halves the bytes the sort moves.
  const bool weighted = fine.mult != nullptr;
  uint64_t *keys = nullptr, *keys_sorted = nullptr;
  int64_t *vals = nullptr, *vals_sorted = nullptr;
  if (int rc = buf.alloc(&keys, static_cast<size_t>(nnz), "keys")) return rc;
  if (weighted)
    if (int rc = buf.alloc(&vals, static_cast<size_t>(nnz), "values")) return rc;
  const int key_blocks = blocks_for(nnz, kKeysPerBlock);
  if (fine.xadj_is64)
    hipLaunchKernelGGL(make_keys_kernel<int64_t>, dim3(key_blocks), dim3(256), 0, nullptr,
                       static_cast<const int64_t *>(fine.xadj), fine.adj, fine.mult, fine.map, n, nnz, nc,
                       sentinel, keys, vals);
  else
    hipLaunchKernelGGL(make_keys_kernel<int32_t>, dim3(key_blocks), dim3(256), 0, nullptr,
                       static_cast<const int32_t *>(fine.xadj), fine.adj, fine.mult, fine.map, n, nnz, nc,
                       sentinel, keys, vals);
  if (int rc = gosh::check_launch("make_keys_kernel")) return rc;

  if (int rc = buf.alloc(&keys_sorted, static_cast<size_t>(nnz), "sorted keys")) return rc;
  if (weighted)
    if (int rc = buf.alloc(&vals_sorted, static_cast<size_t>(nnz), "sorted values")) return rc;
  size_t temp_bytes = 0;
  if (weighted)
    GOSH_TRY_HIP(rocprim::radix_sort_pairs(nullptr, temp_bytes, keys, keys_sorted, vals, vals_sorted,
                                         static_cast<size_t>(nnz), 0u, end_bit, nullptr),
               "radix sort (size query)");
  else
    GOSH_TRY_HIP(rocprim::radix_sort_keys(nullptr, temp_bytes, keys, keys_sorted, static_cast<size_t>(nnz), 0u,
                                        end_bit, nullptr),
               "radix sort (size query)");
  {
    char *temp = nullptr;
    if (int rc = buf.alloc(&temp, temp_bytes, "sort workspace")) return rc;
    if (weighted)
      GOSH_TRY_HIP(rocprim::radix_sort_pairs(temp, temp_bytes, keys, keys_sorted, vals, vals_sorted,
                                           static_cast<size_t>(nnz), 0u, end_bit, nullptr),
                 "radix sort");
    else
      GOSH_TRY_HIP(rocprim::radix_sort_keys(temp, temp_bytes, keys, keys_sorted, static_cast<size_t>(nnz), 0u,
                                          end_bit, nullptr),
                 "radix sort");
    GOSH_TRY_HIP(hipDeviceSynchronize(), "radix sort");
    buf.release(temp);
  }
  // distinct keys go where the unsorted ones were (at most one distinct key per fine entry;
  // the count is only known afterwards), their summed multiplicities beside them
  uint64_t *unique_keys = keys;
  int64_t *sums = vals;
  if (!weighted)
    if (int rc = buf.alloc(&sums, static_cast<size_t>(nnz), "merged multiplicities")) return rc;
  unsigned long long *count_dev = nullptr;
  if (int rc = buf.alloc(&count_dev, 1, "distinct count")) return rc;
  unsigned long long n_unique = 0;
  auto reduce = [&](auto values_in) -> int {
    size_t bytes = 0;
    GOSH_TRY_HIP(rocprim::reduce_by_key(nullptr, bytes, keys_sorted, values_in, static_cast<size_t>(nnz),
                                      unique_keys, sums, count_dev, rocprim::plus<int64_t>(),
                                      rocprim::equal_to<uint64_t>(), nullptr),
               "reduce by key (size query)");
    char *temp = nullptr;
    if (int rc = buf.alloc(&temp, bytes, "reduce workspace")) return rc;
    GOSH_TRY_HIP(rocprim::reduce_by_key(temp, bytes, keys_sorted, values_in, static_cast<size_t>(nnz),
                                      unique_keys, sums, count_dev, rocprim::plus<int64_t>(),
                                      rocprim::equal_to<uint64_t>(), nullptr),
               "reduce by key");
    GOSH_TRY_HIP(hipMemcpy(&n_unique, count_dev, sizeof(n_unique), hipMemcpyDeviceToHost), "copy distinct count");
    buf.release(temp);
    return GOSH_OK;
  };
  if (weighted) {
    if (int rc = reduce(static_cast<const int64_t *>(vals_sorted))) return rc;
  } else {
    if (int rc = reduce(rocprim::constant_iterator<int64_t>(1))) return rc;
  }
  buf.release(keys_sorted);
  if (vals_sorted) buf.release(vals_sorted);
  // entries inside clusters collapse into one sentinel key, the largest: drop it
  if (n_unique > 0) {
    uint64_t last = 0;
    GOSH_TRY_HIP(hipMemcpy(&last, unique_keys + (n_unique - 1), 8, hipMemcpyDeviceToHost), "copy last key");
    if (last == sentinel) --n_unique;
  }
  const int64_t nnz_coarse = static_cast<int64_t>(n_unique);
  coarse.nnz = nnz_coarse;
  if (int rc = persistent(&coarse.adj, static_cast<size_t>(nnz_coarse), "coarse adjacency")) return rc;
  if (int rc = persistent(&coarse.mult, static_cast<size_t>(nnz_coarse), "coarse multiplicities")) return rc;
  hipLaunchKernelGGL(offsets_kernel, dim3(blocks_for(n_coarse + 1, 256)), dim3(256), 0, nullptr, unique_keys,
                     nnz_coarse, nc, xadj_out);
  if (int rc = gosh::check_launch("offsets_kernel")) return rc;
  if (nnz_coarse > 0) {
    hipLaunchKernelGGL(columns_kernel, dim3(blocks_for(nnz_coarse, 256)), dim3(256), 0, nullptr, unique_keys, sums,
                       nnz_coarse, nc, coarse.adj, coarse.mult);
    if (int rc = gosh::check_launch("columns_kernel")) return rc;
  }
  GOSH_TRY_HIP(hipDeviceSynchronize(), "coarse CSR");
  return GOSH_OK;
}

}  // namespace gosh

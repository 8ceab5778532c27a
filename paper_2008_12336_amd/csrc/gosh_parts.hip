// Training of a graph whose embedding matrix does not fit a device budget
// ("LargeGraphGPU", Alg. 5 and Sec. 3.3 of the paper): the matrix stays on the host,
// split into K parts of consecutive vertices; pairs of parts are brought into a few
// device slots, trained against each other by the pair kernel, and written back.
//
// Roles (the paper runs them as three host threads; here the device-side ordering is
// carried by HIP streams and events, and one extra host thread draws the positives):
//   * sampler thread: fills pools of positive samples on the host, a bounded number of
//     pairs ahead (an OpenMP team fills one pool);
//   * copy-in stream: part upload / pool upload, and copy-out stream: part write-back
//     (the two directions of the host link run at the same time), overlapped with
//   * compute stream: one pair kernel per visited pair, in the fixed inside-out order.
#include <hip/hip_runtime.h>
#include <omp.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

#include "gosh_coarsen_internal.h"
#include "gosh_common.h"
#include "gosh_sampler.h"
#include "gosh_device.h"

namespace {

using gosh::philox_draw;
using gosh::scale_draw;

// Fourth counter word of the parts mode: level in the low 8 bits, visited-pair index + 1
// above it, so no draw of this mode coincides with one of the epoch kernel.
__host__ __device__ inline uint32_t level_word(uint32_t level, uint32_t pair_index) {
  return (level & 0xFFu) | ((pair_index + 1u) << 8);
}

// Work description of one visit of a pair of parts (a, b).  Sources are the vertices of
// part a (side 0) followed, unless a == b, by those of part b (side 1).  A source runs B
// rounds of 1 + k_neg samples: the positive of round r comes from its pool entry, the
// negatives are uniform over the partner part.
struct PairWork {
  int32_t a_lo, a_n, b_lo, b_n;  // vertex id ranges of the two parts
  float *a_rows, *b_rows;        // device slots holding their rows
  const int32_t *pool_a;         // a_n * B positives for the sources of a
  const int32_t *pool_b;         // b_n * B positives for the sources of b (unused if a == b)
  int32_t B, per_round, d, diagonal;
  uint32_t key0, key1, rotation, word3;

  __host__ __device__ __forceinline__ int64_t count() const {
    return diagonal ? a_n : static_cast<int64_t>(a_n) + b_n;
  }
  __device__ __forceinline__ int32_t source_id(int64_t i) const {
    return i < a_n ? a_lo + static_cast<int32_t>(i) : b_lo + static_cast<int32_t>(i - a_n);
  }
  __device__ __forceinline__ float *source_row(int64_t i) const {
    return i < a_n ? a_rows + i * d : b_rows + (i - a_n) * d;
  }
  // Nothing of a pair's sampling depends on memory that the source index alone names.
  struct Pre {};
  __device__ __forceinline__ Pre stage1(int64_t, bool) const { return Pre{}; }
  // Branch-free around the pool read: a lane that does not want a positive reads entry 0.
  __device__ __forceinline__ uint64_t draw(int64_t i, int32_t src, int32_t t) const {
    const int side = i >= a_n;
    return philox_draw(static_cast<uint32_t>(src), static_cast<uint32_t>(side * B * per_round + t), rotation,
                       word3, key0, key1);
  }
  __device__ __forceinline__ int32_t stage2(int64_t i, int32_t, int32_t t, bool want, bool positive, const Pre &,
                                            uint64_t r) const {
    const int side = i >= a_n;
    const int64_t local = side ? i - a_n : i;
    const int32_t *pool = side ? pool_b : pool_a;
    const int32_t other_lo = side ? a_lo : b_lo, other_n = side ? a_n : b_n;
    // a pool entry outside the partner part (the rows of a malformed graph can yield one)
    // is no sample: the kernel never leaves the two slots
    int32_t from_pool = pool[(want && positive) ? local * B + t / per_round : 0];
    if (static_cast<uint32_t>(from_pool - other_lo) >= static_cast<uint32_t>(other_n)) from_pool = -1;
    // an empty partner part (possible for the last parts of a split) offers no negative
    const int32_t uniform =
        other_n > 0 ? other_lo + static_cast<int32_t>(scale_draw(r, static_cast<uint32_t>(other_n))) : -1;
    return want ? (positive ? from_pool : uniform) : -1;
  }
  __device__ __forceinline__ float *sample_row(int64_t i, int32_t v) const {
    return i >= a_n ? a_rows + static_cast<int64_t>(v - a_lo) * d
                    : b_rows + static_cast<int64_t>(v - b_lo) * d;
  }
};

// Debug: the ids the pair kernel would use, source by source, sample by sample.
__global__ __launch_bounds__(256) void pair_stream_kernel(PairWork w, int32_t samples,
                                                          int32_t *__restrict__ out) {
  const int64_t total = w.count() * samples;
  for (int64_t x = blockIdx.x * 256LL + threadIdx.x; x < total; x += gridDim.x * 256LL) {
    const int64_t i = x / samples;
    const int32_t t = static_cast<int32_t>(x % samples);
    const int32_t src = w.source_id(i);
    out[x] = w.stage2(i, src, t, true, t % w.per_round == 0, w.stage1(i, true), w.draw(i, src, t));
  }
}

// The positives of one side of a pair, drawn on the device from a graph that lives there:
// the same runs (two binary searches in the ascending row) and the same draws as the host
// sampler, one thread per source.
template <typename OffT>
__global__ __launch_bounds__(256) void fill_pool_kernel(const OffT *__restrict__ xadj,
                                                        const int32_t *__restrict__ adj, int64_t nnz,
                                                        int32_t lo, int32_t cnt, int32_t olo, int32_t ohi,
                                                        int32_t side, int32_t B,
                                                        int32_t per_round, uint32_t key0, uint32_t key1,
                                                        uint32_t rotation, uint32_t word3,
                                                        int32_t *__restrict__ pool) {
  for (int64_t local = blockIdx.x * 256LL + threadIdx.x; local < cnt; local += gridDim.x * 256LL) {
    const int64_t src = static_cast<int64_t>(lo) + local;
    int64_t first = static_cast<int64_t>(xadj[src]), end = static_cast<int64_t>(xadj[src + 1]);
    if (first < 0 || first > end || end > nnz) first = end = 0;  // offsets that leave adj: an empty row
    int64_t hi = end;
    while (first < hi) {  // first entry >= olo
      const int64_t mid = first + (hi - first) / 2;
      if (adj[mid] < olo) first = mid + 1;
      else hi = mid;
    }
    int64_t last = first;
    hi = end;
    while (last < hi) {  // first entry >= ohi
      const int64_t mid = last + (hi - last) / 2;
      if (adj[mid] < ohi) last = mid + 1;
      else hi = mid;
    }
    const uint32_t candidates = static_cast<uint32_t>(last - first);
    for (int32_t r = 0; r < B; ++r) {
      int32_t pick = -1;
      if (candidates > 0) {
        const uint64_t draw = philox_draw(static_cast<uint32_t>(src),
                                          static_cast<uint32_t>(side * B * per_round + r * per_round), rotation,
                                          word3, key0, key1);
        pick = adj[first + scale_draw(draw, candidates)];
      }
      pool[local * B + r] = pick;
    }
  }
}

// Bit v of the hot-row bitmap: deg(v) >= min_degree (one thread per 64 vertices).
template <typename OffT>
__global__ __launch_bounds__(256) void degree_bitmap_kernel(const OffT *__restrict__ xadj, int64_t n,
                                                            int64_t min_degree, uint64_t *__restrict__ bits) {
  const int64_t words = (n + 63) / 64;
  for (int64_t w = blockIdx.x * 256LL + threadIdx.x; w < words; w += gridDim.x * 256LL) {
    uint64_t word = 0;
    for (int bit = 0; bit < 64; ++bit) {
      const int64_t v = w * 64 + bit;
      if (v < n && static_cast<int64_t>(xadj[v + 1]) - static_cast<int64_t>(xadj[v]) >= min_degree)
        word |= uint64_t{1} << bit;
    }
    bits[w] = word;
  }
}

struct HostCsr {
  const gosh_csr *g;
  int64_t begin(int64_t v) const {
    return g->xadj_is64 ? static_cast<const int64_t *>(g->xadj)[v] : static_cast<const int32_t *>(g->xadj)[v];
  }
};

struct Layout {
  int64_t n;
  int32_t K;
  int64_t part_rows;  // ceil(n / K)
  int32_t lo(int32_t p) const { return static_cast<int32_t>(std::min<int64_t>(n, p * part_rows)); }
  int32_t size(int32_t p) const { return static_cast<int32_t>(std::min<int64_t>(n, (p + 1) * part_rows) - lo(p)); }
};

// The order in which part pairs are visited in one rotation (Sec. 3.3.1, "inside-out"):
// (0,0), (1,0), (1,1), (2,0), ...
void pair_order(int32_t K, std::vector<int32_t> &a, std::vector<int32_t> &b) {
  a.clear();
  b.clear();
  for (int32_t m = 0; m < K; ++m)
    for (int32_t s = 0; s <= m; ++s) {
      a.push_back(m);
      b.push_back(s);
    }
}

// A visiting order for hardware whose host link, not its kernels, bounds the rotation (it
// is not the paper's): the parts are cut into blocks of R consecutive parts; for every
// block in turn, first the pairs inside the block in the order above, then for each later
// part c the pairs (c, r) for every r of the block.  With the block resident and the later
// parts streamed through, a loaded part meets R partners instead of one.  Every pair
// (a, b), a >= b, still occurs exactly once; R >= K gives the order above.
void pair_order_blocked(int32_t K, int32_t R, std::vector<int32_t> &a, std::vector<int32_t> &b) {
  a.clear();
  b.clear();
  for (int32_t first = 0; first < K; first += R) {
    const int32_t end = std::min(first + R, K);
    for (int32_t m = first; m < end; ++m)
      for (int32_t s = first; s <= m; ++s) {
        a.push_back(m);
        b.push_back(s);
      }
    for (int32_t c = end; c < K; ++c)
      for (int32_t r = first; r < end; ++r) {
        a.push_back(c);
        b.push_back(r);
      }
  }
}

#define PARTS_HIP(call, what)                                                          \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) {                                                            \
      rc = gosh::hip_fail(e_, what);                                                   \
      goto done;                                                                       \
    }                                                                                  \
  } while (0)

uint64_t device_bytes_for(int64_t n, int32_t K, int32_t d, int32_t P, int32_t S, int32_t B) {
  const int64_t ps = (n + K - 1) / K;
  return static_cast<uint64_t>(P) * ps * d * 4 + static_cast<uint64_t>(S) * 2 * ps * B * 4 +
         static_cast<uint64_t>((n + 63) / 64) * 8;
}

int check_parts_args(const gosh_csr *g, const float *M, int32_t d, int32_t k_neg, int32_t P,
                     int32_t S, int32_t B, uint32_t flags) {
  if (int rc = gosh::check_csr(g)) return rc;
  if (int rc = gosh::check_matrix(M, d, "M")) return rc;
  if (k_neg < 0 || k_neg > GOSH_MAX_NEG)
    return gosh::fail(GOSH_EINVAL, "k_neg = %d: must be in [0, %d]", k_neg, GOSH_MAX_NEG);
  if (P < 2 || P > 64) return gosh::fail(GOSH_EINVAL, "P_gpu = %d: must be in [2, 64]", P);
  if (S < 1 || S > 64) return gosh::fail(GOSH_EINVAL, "S_gpu = %d: must be in [1, 64]", S);
  if (B < 1 || B > 64) return gosh::fail(GOSH_EINVAL, "B = %d: must be in [1, 64]", B);
  if (flags & ~(GOSH_FLAG_SEQUENTIAL | GOSH_FLAG_PLAIN_STORES | GOSH_FLAG_ATOMIC_ADDS | GOSH_FLAG_BLOCKED_ORDER |
                GOSH_FLAG_CONCURRENT_LAYOUT))
    return gosh::fail(GOSH_EINVAL, "unknown flags 0x%x", flags);
  if ((flags & GOSH_FLAG_PLAIN_STORES) && (flags & GOSH_FLAG_ATOMIC_ADDS))
    return gosh::fail(GOSH_EINVAL, "flags ask for plain stores and atomic adds at once");
  return GOSH_OK;
}

constexpr int32_t kMaxParts = 4096;
// Parts of a matrix that is trained in device memory, unless the caller names a count: with
// 16 the pair kernels ran fastest on a 2^24-vertex graph (11.3 ms per epoch's worth of
// samples; 13.2 ms with 2 parts, 11.9 with 32, 22.7 with 64).
constexpr int32_t kResidentParts = 16;

// What a call of gosh_train_parts is asked to do, after planning.
struct RotationPlan {
  const gosh_csr *g;  // host or device arrays
  float *M_host;      // the matrix: on the host, or (matrix_on_device) in device memory
  bool matrix_on_device;
  int32_t d, k_neg, B;
  float lr0;
  uint64_t seed;
  uint32_t level, flags;
  int32_t K, P, S;    // parts, slots (K when the matrix is on the device), pools
  int32_t order_P;    // the slot count the blocked pair order is laid out for
  int64_t rotations;
};

// One call of gosh_train_parts: owns the device slots and pools, the three streams, the
// events that order them and the sampler thread; the destructor waits for everything that
// is queued, stops the thread and frees it all, on every path.
// With the matrix in device memory every part is its own slot, in place (P = K): nothing is
// copied, and what remains of Alg. 5 is its visiting order and its sampling rule.
class Rotation {
 public:
  explicit Rotation(const RotationPlan &plan)
      : pl(plan), L{plan.g->n, plan.K, (plan.g->n + plan.K - 1) / plan.K}, P(plan.P), S(plan.S), NS(plan.S + 1),
        per_round(plan.k_neg + 1), samples(plan.B * (plan.k_neg + 1)),
        seq((plan.flags & GOSH_FLAG_SEQUENTIAL) != 0),
        concurrent_paths(!seq || (plan.flags & GOSH_FLAG_CONCURRENT_LAYOUT) != 0), tune(gosh::tuning()), key0(static_cast<uint32_t>(plan.seed)),
        key1(static_cast<uint32_t>(plan.seed >> 32)), host_threads(std::max(1, omp_get_max_threads())),
        graph_on_device(gosh::is_device_pointer(plan.g->xadj)),
        pool_ints(static_cast<size_t>(2) * L.part_rows * plan.B) {
    // the blocked order keeps all slots but two for a block; the two take turns receiving
    // the streamed parts
    if (pl.flags & GOSH_FLAG_BLOCKED_ORDER) pair_order_blocked(pl.K, std::max(1, pl.order_P - 2), pa, pb);
    else pair_order(pl.K, pa, pb);
    npairs = static_cast<int64_t>(pa.size());
    visits = pl.rotations * npairs;
    st.K = pl.K;
    st.rotations = pl.rotations;
    st.pair_visits = visits;
  }
  Rotation(const Rotation &) = delete;
  Rotation &operator=(const Rotation &) = delete;

  // Stops the sampler thread and waits for everything that is queued; the statistics are
  // complete after this.
  void finish() {
    {
      std::lock_guard<std::mutex> lock(mu);
      stop = true;
    }
    cv.notify_all();
    if (sampler.joinable()) sampler.join();
    st.sampler_ms = sampler_busy_ms;
    for (hipStream_t s : {compute, copy, copy_out})
      if (s) (void)hipStreamSynchronize(s);
  }

  ~Rotation() {
    finish();
    for (auto *events : {&chunk_flushed, &k_begin, &k_end, &slot_ready, &slot_used, &pool_ready, &pool_used,
                         &staging_done})
      for (hipEvent_t e : *events)
        if (e) (void)hipEventDestroy(e);
    if (arrived) (void)hipEventDestroy(arrived);
    if (!pl.matrix_on_device)
      for (auto p : slot) if (p) (void)hipFree(p);
    for (auto p : dpool) if (p) (void)hipFree(p);
    for (auto p : staging) if (p) (void)hipHostFree(p);
    if (hot_bits_dev) (void)hipFree(hot_bits_dev);
    if (check) (void)hipFree(check);
    for (hipStream_t s : {compute, copy, copy_out})
      if (s) (void)hipStreamDestroy(s);
  }

  // Streams, slots, pools, events, the hot-row set, the sampler thread.
  int prepare() {
    if (graph_on_device)
      if (int rc = gosh::check_device_csr(pl.g)) return rc;
    slot.assign(P, nullptr);
    dpool.assign(S, nullptr);
    staging.assign(NS, nullptr);
    slot_part.assign(P, -1);
    const int moving = pl.matrix_on_device ? 0 : P;  // slots whose content changes
    chunk_flushed.assign(static_cast<size_t>(moving) * kSwapChunks, nullptr);
    slot_ready.assign(moving, nullptr);
    slot_used.assign(moving, nullptr);
    pool_ready.assign(S, nullptr);
    pool_used.assign(S, nullptr);
    staging_done.assign(NS, nullptr);
    k_begin.assign(kTimers, nullptr);
    k_end.assign(kTimers, nullptr);
    k_pending.assign(kTimers, 0);
    GOSH_TRY_HIP(hipStreamCreateWithFlags(&compute, hipStreamNonBlocking), "hipStreamCreate");
    GOSH_TRY_HIP(hipStreamCreateWithFlags(&copy, hipStreamNonBlocking), "hipStreamCreate");
    GOSH_TRY_HIP(hipStreamCreateWithFlags(&copy_out, hipStreamNonBlocking), "hipStreamCreate");
    for (int s = 0; s < P; ++s) {
      if (pl.matrix_on_device) {
        slot[s] = pl.M_host + static_cast<int64_t>(L.lo(s)) * pl.d;
        slot_part[s] = s;
      } else {
        GOSH_TRY_HIP(hipMalloc(&slot[s], static_cast<size_t>(L.part_rows) * pl.d * 4), "hipMalloc part slot");
      }
    }
    for (int s = 0; s < S; ++s) GOSH_TRY_HIP(hipMalloc(&dpool[s], pool_ints * 4), "hipMalloc pool");
    for (int s = 0; s < NS && !graph_on_device; ++s)
      GOSH_TRY_HIP(hipHostMalloc(reinterpret_cast<void **>(&staging[s]), pool_ints * 4, hipHostMallocDefault),
              "hipHostMalloc staging");
    for (auto *events : {&chunk_flushed, &slot_ready, &slot_used, &pool_ready, &pool_used, &staging_done})
      for (hipEvent_t &e : *events) GOSH_TRY_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming), "hipEventCreate");
    GOSH_TRY_HIP(hipEventCreateWithFlags(&arrived, hipEventDisableTiming), "hipEventCreate");
    for (int t = 0; t < kTimers; ++t) {
      GOSH_TRY_HIP(hipEventCreate(&k_begin[t]), "hipEventCreate");
      GOSH_TRY_HIP(hipEventCreate(&k_end[t]), "hipEventCreate");
    }
    GOSH_TRY_HIP(hipMalloc(reinterpret_cast<void **>(&check), sizeof(gosh::CheckResult)), "hipMalloc check result");
    if (int rc = gosh::matrix_check_clear(check, copy_out)) return rc;
    if (int rc = build_hot_set()) return rc;
    if (!graph_on_device) sampler = std::thread([this] { sampler_loop(); });
    return GOSH_OK;
  }

  // Every visit of every rotation, then the write-back of what is still resident.
  int run() {
    std::vector<int32_t> keep;
    const int64_t max_ahead = (pl.flags & GOSH_FLAG_BLOCKED_ORDER) ? P : 1;
    for (int64_t vi = 0; vi < visits; ++vi) {
      const Visit v = visit(vi);
      // 1. the two parts of this visit (nothing is running that they could disturb: the
      //    copy stream waits for the last kernel of any slot it overwrites)
      keep.clear();
      if (!pl.matrix_on_device && ensure_parts(vi, keep) == kError) return error;
      const int sa = slot_of(v.a), sb = slot_of(v.b);
      if (sa < 0 || sb < 0) return gosh::fail(GOSH_EHIP, "internal: part not resident");
      // 2. the pool of this visit
      if (int rc = graph_on_device ? pool_from_device(vi, v) : pool_from_sampler(vi, v)) return rc;
      // 3. the pair kernel
      if (int rc = launch_pair(vi, v, sa, sb)) return rc;
      // 4. while that kernel runs: bring in what the next visit needs.  In the blocked order
      //    the part after the one being streamed is known to be worth its slot, so there
      //    the fetch runs as far ahead as slots that none of the visits in between uses can
      //    be found; in the paper's order fetching further ahead evicts parts the next row
      //    would have reused (measured: 376 GB instead of 309 GB per rotation at 5 slots).
      if (!pl.matrix_on_device) {
        keep.assign({v.a, v.b});
        int got = kPlaced;
        for (int64_t ahead = 1; ahead <= max_ahead && got == kPlaced; ++ahead) got = ensure_parts(vi + ahead, keep);
        if (got == kError) return error;
      }
      // 5. keep the host from running ahead
      if (graph_on_device) {
        // it continues once the parts of this visit have arrived, as it does with a host
        // sampler (with several swaps queued at once the copies of a swap took four times
        // as long)
        GOSH_TRY_HIP(hipEventSynchronize(arrived), "hipEventSynchronize");
      } else {
        // hand the staging buffer back to the sampler once its upload is done
        GOSH_TRY_HIP(hipEventSynchronize(staging_done[vi % NS]), "hipEventSynchronize");
        {
          std::lock_guard<std::mutex> lock(mu);
          released = vi + 1;
        }
        cv.notify_all();
      }
    }
    return write_back_all();
  }

  gosh_parts_stats st{};

 private:
  struct Visit {
    int32_t a, b;      // the two parts
    uint32_t rot, q;   // rotation, index of the pair inside the rotation
  };
  enum { kPlaced = 0, kNoSlot = 1, kError = -2 };
  // A part swap runs in kSwapChunks pieces: piece c of the new part goes up as soon as piece
  // c of the old one is down, so both directions of the host link are busy at once.
  static constexpr int kSwapChunks = 8;
  // Kernel timing: a ring of event pairs, read when a pair is used again and at the end.
  // The host is normally a few visits ahead of the kernels, so that read does not wait;
  // when nothing else paces it (every part resident, graph on the device) the ring does,
  // at kTimers visits.
  static constexpr int kTimers = 64;

  const RotationPlan pl;
  const Layout L;
  const int32_t P, S, NS;  // slots, device pools, host staging buffers for pools
  const int32_t per_round, samples;
  const bool seq;
  const bool concurrent_paths;  // the concurrent kernel's layout and write paths are in use
  const gosh_tuning tune;
  const uint32_t key0, key1;
  const int host_threads;
  const bool graph_on_device;  // then it is sampled there: no sampler thread, no pool uploads
  const size_t pool_ints;      // side 0 then side 1
  std::vector<int32_t> pa, pb;
  int64_t npairs = 0, visits = 0;

  std::vector<float *> slot;
  std::vector<int32_t *> dpool, staging;
  std::vector<int32_t> slot_part;
  uint32_t *hot_bits_dev = nullptr;
  gosh::HotSet hot{nullptr, gosh::kHotNone};
  gosh::CheckResult *check = nullptr;  // divergence check, accumulated on the outbound stream
  hipStream_t compute = nullptr, copy = nullptr, copy_out = nullptr;
  std::vector<hipEvent_t> chunk_flushed, slot_ready, slot_used, pool_ready, pool_used, staging_done, k_begin, k_end;
  std::vector<char> k_pending;
  hipEvent_t arrived = nullptr;  // device-sampled path: the parts of the current visit are in

  // sampler thread state
  std::mutex mu;
  std::condition_variable cv;
  int64_t filled = 0;    // pools produced so far (visit indices [0, filled))
  int64_t released = 0;  // staging buffers given back (visit indices [0, released))
  int error = GOSH_OK;  // status behind a kError
  bool stop = false;
  double sampler_busy_ms = 0;  // written by the sampler thread only, read after it has joined
  std::thread sampler;

  Visit visit(int64_t vi) const {
    const uint32_t q = static_cast<uint32_t>(vi % npairs);
    return Visit{pa[q], pb[q], static_cast<uint32_t>(vi / npairs), q};
  }

  // Hot rows: the degree rule evaluated once, where the graph lives.
  int build_hot_set() {
    const int64_t n = pl.g->n;
    if (concurrent_paths) {
      const int gpw = gosh::SgdLauncher<PairWork>::groups_per_wave(pl.d);
      const int64_t pair_sources = 2 * L.part_rows;
      const int64_t waves = std::min<int64_t>((pair_sources + gpw - 1) / gpw, tune.max_waves);
      const int64_t in_flight = std::min<int64_t>(waves, gosh::resident_waves()) * gpw;
      // per visit a row takes about B*k_neg uniform hits plus its own turn
      int mode = (tune.hot_min_degree == 0 &&
                  (static_cast<int64_t>(pl.B) * pl.k_neg + 1) * in_flight * tune.hot_all_inv_eps > pair_sources)
                     ? gosh::kHotAll
                     : gosh::kHotBitmap;
      if (pl.flags & GOSH_FLAG_PLAIN_STORES) mode = gosh::kHotNone;
      if (pl.flags & GOSH_FLAG_ATOMIC_ADDS) mode = gosh::kHotAll;
      if (mode == gosh::kHotBitmap) {
        const int64_t min_degree = tune.hot_min_degree > 0
                                       ? tune.hot_min_degree
                                       : pl.g->nnz / (tune.hot_inv_eps * in_flight * pl.B) + 1;
        const int64_t words = (n + 63) / 64;
        GOSH_TRY_HIP(hipMalloc(&hot_bits_dev, static_cast<size_t>(words) * 8), "hipMalloc hot bitmap");
        if (graph_on_device) {
          const int blocks = static_cast<int>(std::min<int64_t>((words + 255) / 256, 65536));
          if (pl.g->xadj_is64)
            hipLaunchKernelGGL(degree_bitmap_kernel<int64_t>, dim3(blocks), dim3(256), 0, nullptr,
                               static_cast<const int64_t *>(pl.g->xadj), n, min_degree,
                               reinterpret_cast<uint64_t *>(hot_bits_dev));
          else
            hipLaunchKernelGGL(degree_bitmap_kernel<int32_t>, dim3(blocks), dim3(256), 0, nullptr,
                               static_cast<const int32_t *>(pl.g->xadj), n, min_degree,
                               reinterpret_cast<uint64_t *>(hot_bits_dev));
          if (int rc = gosh::check_launch("degree_bitmap_kernel")) return rc;
          GOSH_TRY_HIP(hipDeviceSynchronize(), "hot bitmap");
        } else {
          const HostCsr csr{pl.g};
          std::vector<uint64_t> bits(static_cast<size_t>(words), 0);
#pragma omp parallel for num_threads(host_threads) schedule(static)
          for (int64_t w64 = 0; w64 < words; ++w64) {
            uint64_t word = 0;
            for (int bit = 0; bit < 64; ++bit) {
              const int64_t v = w64 * 64 + bit;
              if (v < n && csr.begin(v + 1) - csr.begin(v) >= min_degree) word |= uint64_t{1} << bit;
            }
            bits[static_cast<size_t>(w64)] = word;
          }
          GOSH_TRY_HIP(hipMemcpy(hot_bits_dev, bits.data(), bits.size() * 8, hipMemcpyHostToDevice), "copy bitmap");
        }
        hot.bits = hot_bits_dev;
      }
      hot.mode = mode;
    }
    if (hot.bits == nullptr) {
      // the kernel reads word 0 of the bitmap unconditionally
      GOSH_TRY_HIP(hipMalloc(&hot_bits_dev, 64), "hipMalloc hot bitmap");
      GOSH_TRY_HIP(hipMemset(hot_bits_dev, 0, 64), "hipMemset hot bitmap");
      hot.bits = hot_bits_dev;
    }
    return GOSH_OK;
  }

  // Sampler thread (host graph only): pools of positives, at most NS visits ahead of their
  // release.
  void sampler_loop() {
    for (int64_t vi = 0; vi < visits; ++vi) {
      {
        std::unique_lock<std::mutex> lock(mu);
        cv.wait(lock, [&] { return stop || vi - released < NS; });
        if (stop) return;
      }
      const Visit v = visit(vi);
      int32_t *buf = staging[vi % NS];
      const uint32_t w3 = level_word(pl.level, v.q);
      const auto t_fill = std::chrono::steady_clock::now();
      gosh::fill_pool(*pl.g, L.lo(v.a), L.size(v.a), L.lo(v.b), L.lo(v.b) + L.size(v.b), 0, pl.B, per_round, key0,
                      key1, v.rot, w3, host_threads, buf);
      if (v.a != v.b)
        gosh::fill_pool(*pl.g, L.lo(v.b), L.size(v.b), L.lo(v.a), L.lo(v.a) + L.size(v.a), 1, pl.B, per_round, key0,
                        key1, v.rot, w3, host_threads, buf + static_cast<size_t>(L.part_rows) * pl.B);
      const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_fill).count();
      sampler_busy_ms += ms;
      {
        std::lock_guard<std::mutex> lock(mu);
        filled = vi + 1;
      }
      cv.notify_all();
    }
  }

  // Next visit (>= from) that uses part p, or a large number.
  int64_t next_use(int32_t p, int64_t from) const {
    for (int64_t vi = from; vi < std::min(visits, from + 4 * npairs + 4); ++vi) {
      const int64_t q = vi % npairs;
      if (pa[q] == p || pb[q] == p) return vi;
    }
    return visits + npairs;
  }
  int slot_of(int32_t p) const {
    if (pl.matrix_on_device) return p;
    for (int s = 0; s < P; ++s)
      if (slot_part[s] == p) return s;
    return -1;
  }

  // Brings part p into a slot whose part is not in `keep` (SwitchSubMatrices): among the
  // other slots an empty one is taken, else the part whose next use is farthest is
  // written back and replaced.  Everything is queued on the copy streams behind the last
  // kernel that used the slot.  kNoSlot if every slot is kept, kError after a failed call.
  int load_part(int32_t p, const std::vector<int32_t> &keep, int64_t now) {
    int victim = -1;
    int64_t farthest = -1;
    for (int s = 0; s < P; ++s) {
      const int32_t sp = slot_part[s];
      if (sp == -1) { victim = s; break; }
      if (std::find(keep.begin(), keep.end(), sp) != keep.end()) continue;
      const int64_t nu = next_use(sp, now);
      if (nu > farthest) { farthest = nu; victim = s; }
    }
    if (victim < 0) return kNoSlot;
    if ((error = swap_in(p, victim)) != GOSH_OK) return kError;
    slot_part[victim] = p;
    return kPlaced;
  }

  int swap_in(int32_t p, int victim) {
    const int32_t d = pl.d;
    const size_t new_bytes = static_cast<size_t>(L.size(p)) * d * 4;
    float *new_host = pl.M_host + static_cast<int64_t>(L.lo(p)) * d;
    if (slot_part[victim] >= 0) {
      // Write the old part back on the outbound stream and bring the new one in on the
      // inbound stream, piece by piece: the upload of a piece waits only for the
      // write-back of the same bytes of the slot.  A later upload of the old part must
      // see its host bytes; it is queued on the inbound stream after these waits, the
      // last of which covers the whole write-back.
      const int32_t old = slot_part[victim];
      const size_t old_bytes = static_cast<size_t>(L.size(old)) * d * 4;
      float *old_host = pl.M_host + static_cast<int64_t>(L.lo(old)) * d;
      const size_t longest = std::max(old_bytes, new_bytes);
      size_t piece = (longest + kSwapChunks - 1) / kSwapChunks;
      piece = std::max<size_t>((piece + 255) / 256 * 256, size_t(8) << 20);
      // after the last kernel that used the slot, and after the upload that filled it (a
      // part brought in ahead of time may leave again before any kernel has used it)
      GOSH_TRY_HIP(hipStreamWaitEvent(copy_out, slot_used[victim], 0), "hipStreamWaitEvent");
      GOSH_TRY_HIP(hipStreamWaitEvent(copy_out, slot_ready[victim], 0), "hipStreamWaitEvent");
      // the part as training leaves it, checked where it still is (read-only, ahead of the copies)
      if (int rc = gosh::matrix_check_add(slot[victim], static_cast<int64_t>(L.size(old)) * d, check, copy_out)) return rc;
      char *slot_bytes = reinterpret_cast<char *>(slot[victim]);
      int c = 0;
      for (size_t off = 0; off < longest; off += piece, ++c) {
        hipEvent_t flushed = chunk_flushed[static_cast<size_t>(victim) * kSwapChunks + c];
        if (off < old_bytes) {
          GOSH_TRY_HIP(hipMemcpyAsync(reinterpret_cast<char *>(old_host) + off, slot_bytes + off,
                                 std::min(piece, old_bytes - off), hipMemcpyDeviceToHost, copy_out),
                  "part write-back");
          GOSH_TRY_HIP(hipEventRecord(flushed, copy_out), "hipEventRecord");
          GOSH_TRY_HIP(hipStreamWaitEvent(copy, flushed, 0), "hipStreamWaitEvent");
        }
        if (off < new_bytes)
          GOSH_TRY_HIP(hipMemcpyAsync(slot_bytes + off, reinterpret_cast<const char *>(new_host) + off,
                                 std::min(piece, new_bytes - off), hipMemcpyHostToDevice, copy),
                  "part upload");
      }
      st.bytes_d2h += old_bytes;
    } else {
      GOSH_TRY_HIP(hipStreamWaitEvent(copy, slot_used[victim], 0), "hipStreamWaitEvent");
      GOSH_TRY_HIP(hipMemcpyAsync(slot[victim], new_host, new_bytes, hipMemcpyHostToDevice, copy), "part upload");
    }
    st.bytes_h2d += new_bytes;
    GOSH_TRY_HIP(hipEventRecord(slot_ready[victim], copy), "hipEventRecord");
    return GOSH_OK;
  }

  // Makes the parts of visit vi resident as far as slots allow, never evicting a part in
  // `keep` (the parts of the running visit and of the visits before vi).  kNoSlot if a
  // needed part could not be placed (or vi is past the end), kError after a failed call,
  // else kPlaced; the parts of vi join `keep`.
  int ensure_parts(int64_t vi, std::vector<int32_t> &keep) {
    if (vi >= visits) return kNoSlot;
    const Visit v = visit(vi);
    keep.push_back(v.a);
    keep.push_back(v.b);
    const int32_t need[2] = {v.a, v.b};
    for (int t = 0; t < 2; ++t) {
      if (t == 1 && need[1] == need[0]) break;
      if (slot_of(need[t]) >= 0) continue;
      const int got = load_part(need[t], keep, vi);
      if (got != kPlaced) return got;
    }
    return kPlaced;
  }

  // The pool of a visit drawn on the device right before the kernel that reads it (same
  // stream: the pool's previous reader is done, its next reader waits).
  int pool_from_device(int64_t vi, const Visit &v) {
    const int ps = static_cast<int>(vi % S);
    const uint32_t w3 = level_word(pl.level, v.q);
    auto fill = [&](int32_t lo, int32_t cnt, int32_t olo, int32_t ohi, int32_t side, int32_t *pool) {
      if (cnt <= 0) return;
      const int blocks = static_cast<int>(std::min<int64_t>((static_cast<int64_t>(cnt) + 255) / 256, 65536));
      if (pl.g->xadj_is64)
        hipLaunchKernelGGL(fill_pool_kernel<int64_t>, dim3(blocks), dim3(256), 0, compute,
                           static_cast<const int64_t *>(pl.g->xadj), pl.g->adj, pl.g->nnz, lo, cnt, olo, ohi, side,
                           pl.B, per_round, key0, key1, v.rot, w3, pool);
      else
        hipLaunchKernelGGL(fill_pool_kernel<int32_t>, dim3(blocks), dim3(256), 0, compute,
                           static_cast<const int32_t *>(pl.g->xadj), pl.g->adj, pl.g->nnz, lo, cnt, olo, ohi, side,
                           pl.B, per_round, key0, key1, v.rot, w3, pool);
    };
    fill(L.lo(v.a), L.size(v.a), L.lo(v.b), L.lo(v.b) + L.size(v.b), 0, dpool[ps]);
    if (v.a != v.b)
      fill(L.lo(v.b), L.size(v.b), L.lo(v.a), L.lo(v.a) + L.size(v.a), 1,
           dpool[ps] + static_cast<size_t>(L.part_rows) * pl.B);
    if (int rc = gosh::check_launch("fill_pool_kernel")) return rc;
    GOSH_TRY_HIP(hipEventRecord(pool_ready[ps], compute), "hipEventRecord");
    // marks, on the inbound stream, the point up to which this visit's parts are in
    GOSH_TRY_HIP(hipEventRecord(arrived, copy), "hipEventRecord");
    return GOSH_OK;
  }

  // The pool of a visit from the sampler thread: wait for it, upload on the copy stream.
  int pool_from_sampler(int64_t vi, const Visit &v) {
    const int ps = static_cast<int>(vi % S), hs = static_cast<int>(vi % NS);
    {
      const auto t_wait = std::chrono::steady_clock::now();
      std::unique_lock<std::mutex> lock(mu);
      cv.wait(lock, [&] { return filled > vi; });
      st.sampler_wait_ms +=
          std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_wait).count();
    }
    GOSH_TRY_HIP(hipStreamWaitEvent(copy, pool_used[ps], 0), "hipStreamWaitEvent");
    const size_t side0 = static_cast<size_t>(L.size(v.a)) * pl.B * 4;
    GOSH_TRY_HIP(hipMemcpyAsync(dpool[ps], staging[hs], side0, hipMemcpyHostToDevice, copy), "pool upload");
    st.bytes_h2d += side0;
    if (v.a != v.b) {
      const size_t side1 = static_cast<size_t>(L.size(v.b)) * pl.B * 4;
      GOSH_TRY_HIP(hipMemcpyAsync(dpool[ps] + static_cast<size_t>(L.part_rows) * pl.B,
                             staging[hs] + static_cast<size_t>(L.part_rows) * pl.B, side1, hipMemcpyHostToDevice,
                             copy),
              "pool upload");
      st.bytes_h2d += side1;
    }
    GOSH_TRY_HIP(hipEventRecord(pool_ready[ps], copy), "hipEventRecord");
    GOSH_TRY_HIP(hipEventRecord(staging_done[hs], copy), "hipEventRecord");
    return GOSH_OK;
  }

  int launch_pair(int64_t vi, const Visit &v, int sa, int sb) {
    const int ps = static_cast<int>(vi % S);
    if (!pl.matrix_on_device) {
      GOSH_TRY_HIP(hipStreamWaitEvent(compute, slot_ready[sa], 0), "hipStreamWaitEvent");
      GOSH_TRY_HIP(hipStreamWaitEvent(compute, slot_ready[sb], 0), "hipStreamWaitEvent");
    }
    GOSH_TRY_HIP(hipStreamWaitEvent(compute, pool_ready[ps], 0), "hipStreamWaitEvent");
    PairWork w{};
    w.a_lo = L.lo(v.a); w.a_n = L.size(v.a); w.b_lo = L.lo(v.b); w.b_n = L.size(v.b);
    w.a_rows = slot[sa]; w.b_rows = slot[sb];
    w.pool_a = dpool[ps];
    w.pool_b = dpool[ps] + static_cast<size_t>(L.part_rows) * pl.B;
    w.B = pl.B; w.per_round = per_round; w.d = pl.d; w.diagonal = v.a == v.b;
    w.key0 = key0; w.key1 = key1; w.rotation = v.rot; w.word3 = level_word(pl.level, v.q);
    gosh::SgdArgs args{};
    args.hot = hot;
    args.d = pl.d;
    args.k_neg = pl.k_neg;
    args.samples = samples;
    args.lr = gosh_lr(pl.lr0, v.rot, pl.rotations);
    const int timer = static_cast<int>(vi % kTimers);
    if (k_pending[timer]) {
      float ms = 0.f;
      GOSH_TRY_HIP(hipEventSynchronize(k_end[timer]), "hipEventSynchronize");
      GOSH_TRY_HIP(hipEventElapsedTime(&ms, k_begin[timer], k_end[timer]), "hipEventElapsedTime");
      st.kernel_ms += ms;
      k_pending[timer] = 0;
    }
    GOSH_TRY_HIP(hipEventRecord(k_begin[timer], compute), "hipEventRecord");
    gosh::SgdLauncher<PairWork>::launch(w, args, w.count(), seq, tune.plain_rows != 0 || !concurrent_paths,
                                        tune.max_waves, compute);
    if (int rc = gosh::check_launch("sgd_kernel (pair)")) return rc;
    GOSH_TRY_HIP(hipEventRecord(k_end[timer], compute), "hipEventRecord");
    k_pending[timer] = 1;
    st.updates += w.count() * samples;
    if (!pl.matrix_on_device) {
      GOSH_TRY_HIP(hipEventRecord(slot_used[sa], compute), "hipEventRecord");
      GOSH_TRY_HIP(hipEventRecord(slot_used[sb], compute), "hipEventRecord");
    }
    GOSH_TRY_HIP(hipEventRecord(pool_used[ps], compute), "hipEventRecord");
    return GOSH_OK;
  }

  // Writes every resident part back and waits for all three streams.
  int write_back_all() {
    for (int s = 0; s < P && !pl.matrix_on_device; ++s) {
      if (slot_part[s] < 0) continue;
      const int32_t old = slot_part[s];
      const size_t bytes = static_cast<size_t>(L.size(old)) * pl.d * 4;
      GOSH_TRY_HIP(hipStreamWaitEvent(copy_out, slot_used[s], 0), "hipStreamWaitEvent");
      if (int rc = gosh::matrix_check_add(slot[s], static_cast<int64_t>(L.size(old)) * pl.d, check, copy_out)) return rc;
      GOSH_TRY_HIP(hipMemcpyAsync(pl.M_host + static_cast<int64_t>(L.lo(old)) * pl.d, slot[s], bytes,
                             hipMemcpyDeviceToHost, copy_out),
              "part write-back");
      st.bytes_d2h += bytes;
    }
    GOSH_TRY_HIP(hipStreamSynchronize(compute), "hipStreamSynchronize");
    GOSH_TRY_HIP(hipStreamSynchronize(copy), "hipStreamSynchronize");
    if (pl.matrix_on_device)  // every kernel is done: one pass over the matrix where it lives
      if (int rc = gosh::matrix_check_add(pl.M_host, pl.g->n * pl.d, check, copy_out)) return rc;
    if (int rc = gosh::matrix_check_read(check, &st.max_abs, &st.nonfinite, copy_out)) return rc;
    for (int t = 0; t < kTimers; ++t) {
      float ms = 0.f;
      if (k_pending[t] && hipEventElapsedTime(&ms, k_begin[t], k_end[t]) == hipSuccess) st.kernel_ms += ms;
      k_pending[t] = 0;
    }
    return GOSH_OK;
  }
};

}  // namespace

extern "C" {

int gosh_pair_order(int32_t K, int32_t *a, int32_t *b) {
  if (K < 1 || K > kMaxParts) return gosh::fail(GOSH_EINVAL, "K = %d: must be in [1, %d]", K, kMaxParts);
  if (a == nullptr || b == nullptr) return gosh::fail(GOSH_EINVAL, "output array is null");
  std::vector<int32_t> va, vb;
  pair_order(K, va, vb);
  std::copy(va.begin(), va.end(), a);
  std::copy(vb.begin(), vb.end(), b);
  return GOSH_OK;
}

int gosh_pair_order_blocked(int32_t K, int32_t R, int32_t *a, int32_t *b) {
  if (K < 1 || K > kMaxParts) return gosh::fail(GOSH_EINVAL, "K = %d: must be in [1, %d]", K, kMaxParts);
  if (R < 1) return gosh::fail(GOSH_EINVAL, "R = %d: must be >= 1", R);
  if (a == nullptr || b == nullptr) return gosh::fail(GOSH_EINVAL, "output array is null");
  std::vector<int32_t> va, vb;
  pair_order_blocked(K, R, va, vb);
  std::copy(va.begin(), va.end(), a);
  std::copy(vb.begin(), vb.end(), b);
  return GOSH_OK;
}

int gosh_parts_plan(int64_t n, int32_t d, int64_t epochs, uint64_t device_budget_bytes, int32_t P_gpu,
                    int32_t S_gpu, int32_t B, int32_t *K_out, int64_t *rotations_out,
                    uint64_t *device_bytes_out) {
  if (n < 1 || n >= 2147483647LL) return gosh::fail(GOSH_EINVAL, "n = %lld out of range", (long long)n);
  if (int rc = gosh::check_dim(d)) return rc;
  if (P_gpu < 2 || S_gpu < 1 || B < 1 || epochs < 1)
    return gosh::fail(GOSH_EINVAL, "need P_gpu >= 2, S_gpu >= 1, B >= 1, epochs >= 1");
  int32_t K = 1;
  const int32_t K_max = static_cast<int32_t>(std::min<int64_t>(n, kMaxParts));
  // With K parts only min(P_gpu, K) slots are needed.
  while (K <= K_max &&
         device_bytes_for(n, K, d, std::min(P_gpu, K), S_gpu, B) > device_budget_bytes)
    ++K;
  if (K > K_max)
    return gosh::fail(GOSH_EBUDGET, "a budget of %llu bytes cannot hold %d parts of a %d-part split",
                      (unsigned long long)device_budget_bytes, P_gpu, K_max);
  if (K_out) *K_out = K;
  if (rotations_out) {
    const int64_t per = static_cast<int64_t>(B) * K;
    *rotations_out = std::max<int64_t>(1, (epochs + per - 1) / per);
  }
  if (device_bytes_out) *device_bytes_out = device_bytes_for(n, K, d, std::min(P_gpu, K), S_gpu, B);
  return GOSH_OK;
}

int gosh_parts_sample_pair(const gosh_csr *g_host, int32_t K, int32_t pa, int32_t pb, int32_t B,
                           int32_t k_neg, uint64_t seed, uint32_t rotation, uint32_t level,
                           uint32_t pair_index, int32_t *out_host) {
  if (int rc = gosh::check_csr(g_host)) return rc;
  if (gosh::is_device_pointer(g_host->xadj) || gosh::is_device_pointer(g_host->adj))
    return gosh::fail(GOSH_EINVAL, "gosh_parts_sample_pair takes a host graph");
  if (K < 1 || K > kMaxParts || pa < 0 || pb < 0 || pa >= K || pb >= K || pb > pa)
    return gosh::fail(GOSH_EINVAL, "need 0 <= pb <= pa < K <= %d", kMaxParts);
  if (B < 1 || B > 64 || k_neg < 0 || k_neg > GOSH_MAX_NEG || out_host == nullptr)
    return gosh::fail(GOSH_EINVAL, "bad B, k_neg or output pointer");
  const Layout L{g_host->n, K, (g_host->n + K - 1) / K};
  const int32_t per_round = k_neg + 1, samples = B * per_round;
  PairWork w{};
  w.a_lo = L.lo(pa); w.a_n = L.size(pa); w.b_lo = L.lo(pb); w.b_n = L.size(pb);
  w.B = B; w.per_round = per_round; w.d = 4; w.diagonal = pa == pb;
  w.key0 = static_cast<uint32_t>(seed); w.key1 = static_cast<uint32_t>(seed >> 32);
  w.rotation = rotation; w.word3 = level_word(level, pair_index);
  std::vector<int32_t> pool_a(static_cast<size_t>(w.a_n) * B + 1), pool_b(static_cast<size_t>(w.b_n) * B + 1);
  const int threads = omp_get_max_threads();
  gosh::fill_pool(*g_host, w.a_lo, w.a_n, w.b_lo, w.b_lo + w.b_n, 0, B, per_round, w.key0, w.key1, rotation,
            w.word3, threads, pool_a.data());
  if (!w.diagonal)
    gosh::fill_pool(*g_host, w.b_lo, w.b_n, w.a_lo, w.a_lo + w.a_n, 1, B, per_round, w.key0, w.key1, rotation,
              w.word3, threads, pool_b.data());
  const int64_t total = w.count() * samples;
  int rc = GOSH_OK;
  int32_t *d_pa = nullptr, *d_pb = nullptr, *d_out = nullptr;
  PARTS_HIP(hipMalloc(&d_pa, pool_a.size() * 4), "hipMalloc");
  PARTS_HIP(hipMalloc(&d_pb, pool_b.size() * 4), "hipMalloc");
  PARTS_HIP(hipMalloc(&d_out, static_cast<size_t>(std::max<int64_t>(total, 1)) * 4), "hipMalloc");
  PARTS_HIP(hipMemcpy(d_pa, pool_a.data(), pool_a.size() * 4, hipMemcpyHostToDevice), "copy pool");
  PARTS_HIP(hipMemcpy(d_pb, pool_b.data(), pool_b.size() * 4, hipMemcpyHostToDevice), "copy pool");
  w.pool_a = d_pa;
  w.pool_b = d_pb;
  if (total > 0) {
    const int blocks = static_cast<int>(std::min<int64_t>((total + 255) / 256, 1 << 16));
    hipLaunchKernelGGL(pair_stream_kernel, dim3(blocks), dim3(256), 0, nullptr, w, samples, d_out);
    if ((rc = gosh::check_launch("pair_stream_kernel"))) goto done;
    PARTS_HIP(hipMemcpy(out_host, d_out, static_cast<size_t>(total) * 4, hipMemcpyDeviceToHost), "copy stream");
  }
done:
  if (d_pa) (void)hipFree(d_pa);
  if (d_pb) (void)hipFree(d_pb);
  if (d_out) (void)hipFree(d_out);
  return rc;
}

int gosh_train_parts(const gosh_csr *g_host, float *M_host, int32_t d, int32_t k_neg, int64_t epochs,
                     float lr0, uint64_t seed, uint32_t level, uint64_t device_budget_bytes,
                     int32_t P_gpu, int32_t S_gpu, int32_t B, int32_t force_K, uint32_t flags,
                     gosh_parts_stats *stats_out) {
  if (int rc = check_parts_args(g_host, M_host, d, k_neg, P_gpu, S_gpu, B, flags)) return rc;
  if (epochs < 1) return gosh::fail(GOSH_EINVAL, "epochs = %lld: must be >= 1", (long long)epochs);
  const int64_t n = g_host->n;
  int32_t K = 0;
  int64_t rotations = 0;
  uint64_t planned_bytes = 0;
  // A matrix in device memory is trained where it is: every part its own slot, no copies.
  const bool matrix_on_device = gosh::is_device_pointer(M_host);
  if (matrix_on_device) {
    if (int rc = gosh::check_device_span(M_host, static_cast<size_t>(n) * d * 4, "M")) return rc;
    if (force_K > kMaxParts || force_K > n) return gosh::fail(GOSH_EINVAL, "force_K = %d too large", force_K);
    K = force_K > 0 ? force_K : static_cast<int32_t>(std::min<int64_t>(n, kResidentParts));
    planned_bytes = device_bytes_for(n, K, d, 0, S_gpu, B);
    if (device_budget_bytes != 0 && planned_bytes > device_budget_bytes)
      return gosh::fail(GOSH_EBUDGET, "the pools of K = %d parts need %llu device bytes, budget is %llu", K,
                        (unsigned long long)planned_bytes, (unsigned long long)device_budget_bytes);
  } else if (force_K > 0) {
    if (force_K > kMaxParts || force_K > n) return gosh::fail(GOSH_EINVAL, "force_K = %d too large", force_K);
    K = force_K;
    planned_bytes = device_bytes_for(n, K, d, std::min(P_gpu, K), S_gpu, B);
    if (device_budget_bytes != 0 && planned_bytes > device_budget_bytes)
      return gosh::fail(GOSH_EBUDGET, "K = %d needs %llu device bytes, budget is %llu", K,
                        (unsigned long long)planned_bytes, (unsigned long long)device_budget_bytes);
  } else if (int rc = gosh_parts_plan(n, d, epochs, device_budget_bytes, P_gpu, S_gpu, B, &K, nullptr,
                                      &planned_bytes)) {
    return rc;
  }
  rotations = std::max<int64_t>(1, (epochs + static_cast<int64_t>(B) * K - 1) / (static_cast<int64_t>(B) * K));
  const auto wall0 = std::chrono::steady_clock::now();
  const RotationPlan plan{g_host, M_host, matrix_on_device, d,     k_neg, B, lr0, seed, level, flags, K,
                          matrix_on_device ? K : std::min(P_gpu, K), S_gpu, std::min(P_gpu, K), rotations};
  gosh_parts_stats st{};
  int rc = GOSH_OK;
  {
    Rotation rotation(plan);
    rc = rotation.prepare();
    if (rc == GOSH_OK) rc = rotation.run();
    rotation.finish();
    st = rotation.st;
  }
  st.device_bytes = planned_bytes;
  st.wall_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - wall0).count();
  if (stats_out) *stats_out = st;
  if (rc == GOSH_OK && st.nonfinite > 0)
    return gosh::fail(GOSH_EDIVERGED, "training diverged: %lld non-finite entries met in the trained parts",
                      (long long)st.nonfinite);
  return rc;
}

}  // extern "C"

// Device side of libgosh: sampler, epoch kernel (Alg. 3 with the update of Alg. 1),
// initialisation and projection.  gfx950 only: 64-lane wavefronts, 128-bit row
// accesses, cross-lane reductions with DPP.
//
// Work layout of the epoch kernel.  A row of d floats is d/4 float4 vectors.  A
// "lane group" of LPG lanes (a power of two, LPG*VPL >= d/4) owns one source vertex;
// lane g of the group holds vectors g, g+LPG, ... of every row it touches, so a row
// access is one fully coalesced 128-bit load or store per lane.  A wavefront carries
// 64/LPG groups (two sources at d = 128).  The source row stays in registers for its
// 1 + k_neg updates and is written back once; sample rows are fetched four at a time
// before the first dot product so that their HBM latencies overlap.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

#include "gosh_common.h"

namespace {

// ---------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  Returns the first two output words as one
// 64-bit draw.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t philox_draw(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1, uint32_t *w2 = nullptr,
                                                uint32_t *w3 = nullptr) {
  constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
  constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hiA = __umulhi(kMulA, c0), loA = kMulA * c0;
    const uint32_t hiB = __umulhi(kMulB, c2), loB = kMulB * c2;
    c0 = hiB ^ c1 ^ k0;
    c1 = loB;
    c2 = hiA ^ c3 ^ k1;
    c3 = loA;
    k0 += kWeylA;
    k1 += kWeylB;
  }
  if (w2) *w2 = c2;
  if (w3) *w3 = c3;
  return static_cast<uint64_t>(c0) | (static_cast<uint64_t>(c1) << 32);
}

// floor(r * bound / 2^64) for bound < 2^32.
__device__ __forceinline__ uint32_t scale_draw(uint64_t r, uint32_t bound) {
  const uint32_t lo = static_cast<uint32_t>(r), hi = static_cast<uint32_t>(r >> 32);
  const uint64_t t = static_cast<uint64_t>(hi) * bound + __umulhi(lo, bound);
  return static_cast<uint32_t>(t >> 32);
}

struct SamplerArgs {
  const void *xadj;
  const int32_t *adj;
  uint32_t n;
  uint32_t key0, key1;
  uint32_t epoch, level;
};

// Sample j of source src: j = 0 positive (uniform neighbour, -1 if none), j >= 1
// negative (uniform vertex).
template <typename OffT>
__device__ __forceinline__ int32_t draw_sample(const SamplerArgs &a, uint32_t src, uint32_t j) {
  const uint64_t r = philox_draw(src, j, a.epoch, a.level, a.key0, a.key1);
  if (j != 0) return static_cast<int32_t>(scale_draw(r, a.n));
  const OffT *xadj = static_cast<const OffT *>(a.xadj);
  const OffT begin = xadj[src];
  const uint32_t deg = static_cast<uint32_t>(xadj[src + 1] - begin);
  if (deg == 0) return -1;
  return a.adj[begin + static_cast<OffT>(scale_draw(r, deg))];
}

template <typename OffT>
__global__ __launch_bounds__(256) void sample_epoch_kernel(SamplerArgs a, int32_t k_neg,
                                                           int32_t *__restrict__ out) {
  const int64_t total = static_cast<int64_t>(a.n) * (k_neg + 1);
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < total; i += gridDim.x * 256LL) {
    const uint32_t src = static_cast<uint32_t>(i / (k_neg + 1));
    const uint32_t j = static_cast<uint32_t>(i % (k_neg + 1));
    out[i] = draw_sample<OffT>(a, src, j);
  }
}

// ---------------------------------------------------------------------------------
// Sum over the LPG lanes of a group; every lane of the group gets the total.
// Steps inside a 16-lane row use DPP (no LDS traffic); 32 and 64 lanes finish with
// swizzle / bpermute.
// ---------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

template <int LPG>
__device__ __forceinline__ float group_sum(float x) {
  if (LPG >= 2) x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
  if (LPG >= 4) x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
  if (LPG >= 8) x += dpp_move<0x141>(x);  // row_half_mirror (quads already uniform)
  if (LPG >= 16) x += dpp_move<0x140>(x); // row_mirror (halves already uniform)
  if (LPG >= 32) x += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x401F));  // lane ^ 16
  if (LPG >= 64) x += __shfl_xor(x, 32, 64);
  return x;
}

// ---------------------------------------------------------------------------------
// Row access policies.  A row is moved in "units" of F floats per lane.
//
// The chip's eight XCDs each have their own L2, and plain stores sit in the writer's
// L2 until they are evicted or the kernel ends: with plain accesses a row updated on
// one XCD is read stale on the others and the last write-back wins.  Lock-free SGD
// needs the rows to be coherent across the whole device, so the concurrent kernel
// moves rows with agent-scope (device-scope) accesses, which are served behind the
// per-XCD L2s.  Every sample row is touched once per turn, so no L2 reuse is lost.
//   RowAgent32: 32-bit relaxed atomic loads and stores at agent scope, lanes interleaved
//     over the row (lane g owns floats g, g+LPG, ...) so that every access instruction
//     of a group covers one whole 128-byte line.  Measured on the 2^24-vertex graph this
//     is as fast as wider per-lane accesses, and it makes the atomic adds used for hot
//     rows (below) dense: one line per instruction instead of half-filled lines, which
//     the memory-side atomic units process at half the rate.
//   RowPlain128: ordinary 128-bit accesses (coherent only inside one XCD); used by the
//     sequential-order mode, which runs on a single wavefront.
// ---------------------------------------------------------------------------------
template <int F>
struct Unit {
  float v[F];
};

__device__ __forceinline__ void atomic_step(float *p, float x) {
  // Built with -munsafe-fp-atomics: the matrix is ordinary coarse-grained device
  // memory, where the hardware fp32 add is available.
  __hip_atomic_fetch_add(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct RowPlain128 {
  static constexpr int F = 4;
  static __device__ __forceinline__ Unit<4> load(const float *p) {
    const float4 x = *reinterpret_cast<const float4 *>(p);
    return Unit<4>{{x.x, x.y, x.z, x.w}};
  }
  static __device__ __forceinline__ void store(float *p, const Unit<4> &u) {
    *reinterpret_cast<float4 *>(p) = float4{u.v[0], u.v[1], u.v[2], u.v[3]};
  }
};

struct RowAgent32 {
  static constexpr int F = 1;
  static __device__ __forceinline__ Unit<1> load(const float *p) {
    return Unit<1>{{__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)}};
  }
  static __device__ __forceinline__ void store(float *p, const Unit<1> &u) {
    __hip_atomic_store(p, u.v[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
};

// ---------------------------------------------------------------------------------
// Hot rows.  A lock-free update is a read-modify-write of a row; when two wavefronts
// hold the same row at once, one of the two writes is lost (Sec. 3.1 of the paper
// accepts such races, and reports that too many of them hurt the embedding).  With
// C sources in flight out of n, a row that is touched h times per epoch has about
// h*C/n concurrent holders.  Rows for which that is not small -- every row of a
// small graph, the high-degree vertices of a large one, which are drawn as positive
// samples in proportion to their degree -- are "hot": their updates are applied as
// atomic adds of the step (M[v] += g*M[src], and M[src] += its accumulated change),
// which cannot be lost.  Cold rows are written back with plain stores, which cost
// half as much on this memory system.
// ---------------------------------------------------------------------------------
enum HotMode : int32_t { kHotNone = 0, kHotBitmap = 1, kHotAll = 2 };

template <typename OffT>
__global__ __launch_bounds__(256) void mark_hot_kernel(const OffT *__restrict__ xadj, int64_t n,
                                                       int64_t min_degree,
                                                       unsigned long long *__restrict__ bits) {
  // one vertex per lane, one 64-bit word of the bitmap per wavefront
  const int64_t words = (n + 63) / 64;
  const int64_t wave0 = (blockIdx.x * 256LL + threadIdx.x) >> 6;
  const int64_t nwaves = (gridDim.x * 256LL) >> 6;
  const int lane = threadIdx.x & 63;
  for (int64_t w = wave0; w < words; w += nwaves) {
    const int64_t v = w * 64 + lane;
    bool hot = false;
    if (v < n) hot = static_cast<int64_t>(xadj[v + 1] - xadj[v]) >= min_degree;
    const unsigned long long mask = __ballot(hot);
    if (lane == 0) bits[w] = mask;
  }
}

struct TrainArgs {
  SamplerArgs s;
  float *M;
  const uint32_t *hot_bits;  // n bits, used when hot_mode == kHotBitmap
  int32_t hot_mode;
  int32_t d;
  int32_t k_neg;
  float lr;
  int64_t active_waves;  // wavefronts that take part; the rest of the grid exits at once
};

constexpr int kChunk = 4;  // sample rows in flight per source

__device__ __forceinline__ bool is_hot(const TrainArgs &a, int32_t v) {
  if (a.hot_mode == kHotBitmap) return (a.hot_bits[v >> 5] >> (v & 31)) & 1u;
  return a.hot_mode == kHotAll;
}

// One epoch.  P: row access policy; LPG lanes per source, UPL units per lane
// (LPG * UPL * P::F >= d).  SEQ: a single lane group walks all sources in ascending
// order (the sequential-order result); otherwise groups stride over the sources.
template <class P, int LPG, int UPL, typename OffT, bool SEQ>
__global__ __launch_bounds__(256) void train_epoch_kernel(TrainArgs a) {
  constexpr int kGroupsPerWave = 64 / LPG;
  constexpr int F = P::F;
  using U = Unit<F>;
  const int lane = threadIdx.x & 63;
  const int gl = lane & (LPG - 1);
  if (SEQ && (lane >= LPG || threadIdx.x >= 64 || blockIdx.x != 0)) return;

  const int64_t wave = blockIdx.x * static_cast<int64_t>(blockDim.x / 64) + (threadIdx.x >> 6);
  if (!SEQ && wave >= a.active_waves) return;
  const int64_t n = a.s.n;
  const int64_t stride = SEQ ? 1 : a.active_waves * kGroupsPerWave;
  const int64_t first = SEQ ? 0 : wave * kGroupsPerWave + lane / LPG;
  const int32_t d = a.d;
  float *const M = a.M;

  // Lane gl owns floats [(gl + i*LPG)*F, +F) of a row, i < UPL: consecutive lanes touch
  // consecutive addresses, so each access instruction covers whole cache lines.
  int32_t col[UPL];
  bool col_ok[UPL];
#pragma unroll
  for (int i = 0; i < UPL; ++i) {
    col[i] = (gl + i * LPG) * F;
    col_ok[i] = col[i] < d;
  }
  const U zero{};

  // The loop bound is uniform over the wave; groups past the end idle inside.
  const int64_t first_of_wave = SEQ ? 0 : wave * kGroupsPerWave;
  for (int64_t base = first_of_wave; base < n; base += stride) {
    const int64_t src = first + (base - first_of_wave);
    if (src >= n) continue;
    float *const src_row = M + src * d;
    U s[UPL];
#pragma unroll
    for (int i = 0; i < UPL; ++i) s[i] = col_ok[i] ? P::load(src_row + col[i]) : zero;
    const bool src_hot = !SEQ && is_hot(a, static_cast<int32_t>(src));
    U s_before[UPL];
#pragma unroll
    for (int i = 0; i < UPL; ++i) s_before[i] = s[i];

    for (int32_t j0 = 0; j0 <= a.k_neg; j0 += kChunk) {
      // Sample ids of this chunk: lane q of the group evaluates draw j0+q, then the
      // ids are broadcast inside the group.
      int32_t v[kChunk];
#pragma unroll
      for (int p = 0; p < kChunk; p += LPG) {
        const int32_t j = j0 + p + gl;
        int32_t mine = -1;
        if (p + gl < kChunk && j <= a.k_neg)
          mine = draw_sample<OffT>(a.s, static_cast<uint32_t>(src), static_cast<uint32_t>(j));
#pragma unroll
        for (int q = 0; q < LPG && p + q < kChunk; ++q) v[p + q] = __shfl(mine, q, LPG);
      }
      // A negative that hits the source itself applies no update.
#pragma unroll
      for (int q = 0; q < kChunk; ++q)
        if (v[q] == static_cast<int32_t>(src)) v[q] = -1;

      // Fetch all rows of the chunk before using any of them.
      U t[kChunk][UPL];
      bool hot[kChunk];
#pragma unroll
      for (int q = 0; q < kChunk; ++q) {
        const float *row = M + static_cast<int64_t>(v[q] < 0 ? 0 : v[q]) * d;
#pragma unroll
        for (int i = 0; i < UPL; ++i) t[q][i] = (v[q] >= 0 && col_ok[i]) ? P::load(row + col[i]) : zero;
        hot[q] = !SEQ && v[q] >= 0 && is_hot(a, v[q]);
      }

#pragma unroll
      for (int q = 0; q < kChunk; ++q) {
        if (v[q] < 0) continue;  // uniform over the group
        float partial = 0.f;
#pragma unroll
        for (int i = 0; i < UPL; ++i)
#pragma unroll
          for (int c = 0; c < F; ++c) partial = fmaf(s[i].v[c], t[q][i].v[c], partial);
        const float x = group_sum<LPG>(partial);
        const float label = (j0 + q == 0) ? 1.f : 0.f;
        const float g = a.lr * (label - 1.f / (1.f + expf(-x)));
        float *row = M + static_cast<int64_t>(v[q]) * d;
#pragma unroll
        for (int i = 0; i < UPL; ++i)
#pragma unroll
          for (int c = 0; c < F; ++c) {
            s[i].v[c] = fmaf(g, t[q][i].v[c], s[i].v[c]);
            t[q][i].v[c] = fmaf(g, s[i].v[c], t[q][i].v[c]);
          }
        if (hot[q]) {  // uniform over the group
#pragma unroll
          for (int i = 0; i < UPL; ++i)
#pragma unroll
            for (int c = 0; c < F; ++c)
              if (col_ok[i]) atomic_step(row + col[i] + c, g * s[i].v[c]);
        } else {
#pragma unroll
          for (int i = 0; i < UPL; ++i)
            if (col_ok[i]) P::store(row + col[i], t[q][i]);
        }
        // A later sample of the same chunk that names the same vertex must see this
        // update: forward the registers instead of the stale prefetched copy.
#pragma unroll
        for (int r = q + 1; r < kChunk; ++r)
          if (v[r] == v[q]) {
#pragma unroll
            for (int i = 0; i < UPL; ++i) t[r][i] = t[q][i];
          }
      }
    }
    if (src_hot) {
#pragma unroll
      for (int i = 0; i < UPL; ++i)
#pragma unroll
        for (int c = 0; c < F; ++c)
          if (col_ok[i]) atomic_step(src_row + col[i] + c, s[i].v[c] - s_before[i].v[c]);
    } else {
#pragma unroll
      for (int i = 0; i < UPL; ++i)
        if (col_ok[i]) P::store(src_row + col[i], s[i]);
    }
  }
}

// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void init_embedding_kernel(float4 *__restrict__ M, int64_t total4,
                                                             int32_t d4, uint32_t key0,
                                                             uint32_t key1, uint32_t level) {
  const double d = 4.0 * d4;
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < total4; i += gridDim.x * 256LL) {
    const uint32_t v = static_cast<uint32_t>(i / d4), c4 = static_cast<uint32_t>(i % d4);
    uint32_t w2, w3;
    const uint64_t w01 = philox_draw(v, c4, 0xFFFFFFFFu, level, key0, key1, &w2, &w3);
    const uint32_t w[4] = {static_cast<uint32_t>(w01), static_cast<uint32_t>(w01 >> 32), w2, w3};
    float o[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      // 24 random bits -> [0,1) exactly; centre, divide by d in fp64, round once.
      const double u = static_cast<double>(w[c] >> 8) * (1.0 / 16777216.0) - 0.5;
      o[c] = static_cast<float>(u / d);
    }
    M[i] = float4{o[0], o[1], o[2], o[3]};
  }
}

__global__ __launch_bounds__(256) void project_kernel(const float4 *__restrict__ coarse,
                                                      const int32_t *__restrict__ map,
                                                      float4 *__restrict__ fine, int64_t total4,
                                                      int32_t d4) {
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < total4; i += gridDim.x * 256LL) {
    const int64_t v = i / d4;
    const int32_t c4 = static_cast<int32_t>(i % d4);
    fine[i] = coarse[static_cast<int64_t>(map[v]) * d4 + c4];
  }
}

int grid_for(int64_t items, int per_block, int max_blocks) {
  int64_t b = (items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > max_blocks) b = max_blocks;
  return static_cast<int>(b);
}

SamplerArgs sampler_args(const gosh_csr *g, uint64_t seed, uint32_t epoch, uint32_t level) {
  SamplerArgs s;
  s.xadj = g->xadj;
  s.adj = g->adj;
  s.n = static_cast<uint32_t>(g->n);
  s.key0 = static_cast<uint32_t>(seed);
  s.key1 = static_cast<uint32_t>(seed >> 32);
  s.epoch = epoch;
  s.level = level;
  return s;
}

long env_long(const char *name, long fallback) {
  const char *e = getenv(name);
  return e ? atol(e) : fallback;
}

// Tuning / experiment overrides (read once).  GOSH_ROW_POLICY: 0 = plain 128-bit row
// accesses also in the concurrent kernel (coherent inside one XCD only).
// GOSH_MAX_WAVES: cap on participating wavefronts.  GOSH_HOT_INV_EPS: 1/eps of the
// hot-row rule.
struct Tuning {
  int row_policy = static_cast<int>(env_long("GOSH_ROW_POLICY", 1));
  int64_t max_waves = env_long("GOSH_MAX_WAVES", 1L << 22);
  int64_t hot_inv_eps = env_long("GOSH_HOT_INV_EPS", 64);
  int64_t hot_all_inv_eps = env_long("GOSH_HOT_ALL_INV_EPS", 4);
};
const Tuning &tuning() {
  static const Tuning t;
  return t;
}

// Per-device scratch for the hot-row bitmap (n bits), grown on demand and kept until
// the process ends.  Calls on one device must not overlap on different streams.
struct HotScratch {
  void *ptr = nullptr;
  size_t bytes = 0;
};
constexpr int kMaxDevices = 64;
HotScratch g_hot_scratch[kMaxDevices];

int hot_scratch(size_t bytes, void **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return gosh::fail(GOSH_EHIP, "cannot identify the current device");
  HotScratch &h = g_hot_scratch[dev];
  if (h.bytes < bytes) {
    if (h.ptr) (void)hipFree(h.ptr);
    h.ptr = nullptr;
    h.bytes = 0;
    const size_t want = bytes + bytes / 4 + 4096;
    if (hipMalloc(&h.ptr, want) != hipSuccess) {
      (void)hipGetLastError();
      return gosh::fail(GOSH_ENOMEM, "cannot allocate %zu bytes for the hot-row bitmap", want);
    }
    h.bytes = want;
  }
  *out = h.ptr;
  return GOSH_OK;
}

int resident_waves() {
  static const int value = [] {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
      int v = 0;
      if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        cus = v;
    }
    return cus * 32;  // 8 wavefronts on each of the 4 SIMDs of a CU
  }();
  return value;
}

template <class P, int LPG, int UPL>
int launch_train_p(TrainArgs a, const gosh_csr *g, uint32_t flags, hipStream_t st) {
  const bool seq = (flags & GOSH_FLAG_SEQUENTIAL) != 0;
  constexpr int kWavesPerBlock = 4;
  constexpr int kGroupsPerWave = 64 / LPG;
  const bool is64 = g->xadj_is64 != 0;
  const int64_t n = g->n;
  int64_t waves = (n + kGroupsPerWave - 1) / kGroupsPerWave;
  if (waves > tuning().max_waves) waves = tuning().max_waves;
  if (waves < 1) waves = 1;
  a.active_waves = waves;
  a.hot_mode = kHotNone;
  a.hot_bits = nullptr;
  if (!seq) {
    // Sources in flight C, and the hot-row rule.  A vertex is hot if its expected
    // positive hits per epoch, deg/avg_deg, give more than eps = 1/64 concurrent holders:
    // deg * C / nnz > eps.  On graphs so small that even the k+1 uniform touches of
    // every row overlap ((k+1)*C/n > 1/4, i.e. fewer than 16 rounds at k = 3) all rows
    // are hot.  Both constants come from link-prediction AUCROC against the sequential
    // reference on R-MAT graphs of 2^12..2^18 vertices: with them the concurrent kernel
    // stays within 0.001..0.005 of the reference, without them it drops by up to 0.4.
    const int64_t in_flight = (waves < resident_waves() ? waves : resident_waves()) * kGroupsPerWave;
    const int64_t inv_eps = tuning().hot_inv_eps;
    int mode = ((a.k_neg + 1) * in_flight * tuning().hot_all_inv_eps > n) ? kHotAll : kHotBitmap;
    if (flags & GOSH_FLAG_PLAIN_STORES) mode = kHotNone;
    if (flags & GOSH_FLAG_ATOMIC_ADDS) mode = kHotAll;
    if (mode == kHotBitmap) {
      int64_t min_degree = g->nnz / (inv_eps * in_flight) + 1;
      void *bits = nullptr;
      const size_t bytes = static_cast<size_t>((n + 63) / 64) * 8;
      if (int rc = hot_scratch(bytes, &bits)) return rc;
      const int blocks = static_cast<int>(std::min<int64_t>(((n + 63) / 64 + 3) / 4, 1 << 16));
      if (is64)
        hipLaunchKernelGGL(mark_hot_kernel<int64_t>, dim3(blocks), dim3(256), 0, st,
                           static_cast<const int64_t *>(g->xadj), n, min_degree,
                           static_cast<unsigned long long *>(bits));
      else
        hipLaunchKernelGGL(mark_hot_kernel<int32_t>, dim3(blocks), dim3(256), 0, st,
                           static_cast<const int32_t *>(g->xadj), n, min_degree,
                           static_cast<unsigned long long *>(bits));
      if (int rc = gosh::check_launch("mark_hot_kernel")) return rc;
      a.hot_bits = static_cast<const uint32_t *>(bits);
    }
    a.hot_mode = mode;
  }
  const int blocks = static_cast<int>((a.active_waves + kWavesPerBlock - 1) / kWavesPerBlock);
  if (seq) {
    if (is64) hipLaunchKernelGGL((train_epoch_kernel<P, LPG, UPL, int64_t, true>), dim3(1), dim3(64), 0, st, a);
    else hipLaunchKernelGGL((train_epoch_kernel<P, LPG, UPL, int32_t, true>), dim3(1), dim3(64), 0, st, a);
  } else {
    if (is64) hipLaunchKernelGGL((train_epoch_kernel<P, LPG, UPL, int64_t, false>), dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((train_epoch_kernel<P, LPG, UPL, int32_t, false>), dim3(blocks), dim3(256), 0, st, a);
  }
  return gosh::check_launch("train_epoch_kernel");
}

// LPG lanes per source, V128 = 128-bit vectors per lane.
template <int LPG, int V128>
int launch_train(const TrainArgs &a, const gosh_csr *g, uint32_t flags, hipStream_t st) {
  if ((flags & GOSH_FLAG_SEQUENTIAL) || tuning().row_policy == 0)
    return launch_train_p<RowPlain128, LPG, V128>(a, g, flags, st);
  return launch_train_p<RowAgent32, LPG, 4 * V128>(a, g, flags, st);
}

}  // namespace

extern "C" {

int gosh_init_embedding(float *M_dev, int64_t n, int32_t d, uint64_t seed, uint32_t level,
                        void *hip_stream) {
  if (int rc = gosh::check_matrix(M_dev, d, "M")) return rc;
  if (n < 1 || n >= 2147483647LL) return gosh::fail(GOSH_EINVAL, "n = %lld out of range", (long long)n);
  const int64_t total4 = n * (d / 4);
  hipLaunchKernelGGL(init_embedding_kernel, dim3(grid_for(total4, 256, 1 << 16)), dim3(256), 0,
                     gosh::as_stream(hip_stream), reinterpret_cast<float4 *>(M_dev), total4, d / 4,
                     static_cast<uint32_t>(seed),
                     static_cast<uint32_t>(seed >> 32), level);
  return gosh::check_launch("init_embedding_kernel");
}

int gosh_sample_epoch(const gosh_csr *g_dev, int32_t k_neg, uint64_t seed, uint32_t epoch,
                      uint32_t level, int32_t *out_dev, void *hip_stream) {
  if (int rc = gosh::check_csr(g_dev)) return rc;
  if (k_neg < 0 || k_neg > GOSH_MAX_NEG)
    return gosh::fail(GOSH_EINVAL, "k_neg = %d: must be in [0, %d]", k_neg, GOSH_MAX_NEG);
  if (out_dev == nullptr) return gosh::fail(GOSH_EINVAL, "out is null");
  const SamplerArgs s = sampler_args(g_dev, seed, epoch, level);
  const int blocks = grid_for(g_dev->n * (k_neg + 1), 256, 1 << 16);
  if (g_dev->xadj_is64)
    hipLaunchKernelGGL(sample_epoch_kernel<int64_t>, dim3(blocks), dim3(256), 0,
                       gosh::as_stream(hip_stream), s, k_neg, out_dev);
  else
    hipLaunchKernelGGL(sample_epoch_kernel<int32_t>, dim3(blocks), dim3(256), 0,
                       gosh::as_stream(hip_stream), s, k_neg, out_dev);
  return gosh::check_launch("sample_epoch_kernel");
}

int gosh_train_epoch(const gosh_csr *g_dev, float *M_dev, int32_t d, int32_t k_neg, float lr_epoch,
                     uint64_t seed, uint32_t epoch, uint32_t level, uint32_t flags,
                     void *hip_stream) {
  if (int rc = gosh::check_csr(g_dev)) return rc;
  if (int rc = gosh::check_matrix(M_dev, d, "M")) return rc;
  if (k_neg < 0 || k_neg > GOSH_MAX_NEG)
    return gosh::fail(GOSH_EINVAL, "k_neg = %d: must be in [0, %d]", k_neg, GOSH_MAX_NEG);
  if (flags & ~(GOSH_FLAG_SEQUENTIAL | GOSH_FLAG_PLAIN_STORES | GOSH_FLAG_ATOMIC_ADDS))
    return gosh::fail(GOSH_EINVAL, "unknown flags 0x%x", flags);
  if ((flags & GOSH_FLAG_PLAIN_STORES) && (flags & GOSH_FLAG_ATOMIC_ADDS))
    return gosh::fail(GOSH_EINVAL, "flags ask for plain stores and atomic adds at once");
  if (!(lr_epoch == lr_epoch)) return gosh::fail(GOSH_EINVAL, "lr is NaN");

  TrainArgs a;
  a.s = sampler_args(g_dev, seed, epoch, level);
  a.M = M_dev;
  a.d = d;
  a.k_neg = k_neg;
  a.lr = lr_epoch;
  hipStream_t st = gosh::as_stream(hip_stream);

  // Smallest power-of-two lane group that covers d/4 vectors (two vectors per lane
  // above 64 vectors).
  const int d4 = d / 4;
  int lpg = 1;
  while (lpg < d4 && lpg < 64) lpg *= 2;
  if (d4 > 64) return launch_train<64, 2>(a, g_dev, flags, st);
  switch (lpg) {
    case 64: return launch_train<64, 1>(a, g_dev, flags, st);
    case 32: return launch_train<32, 1>(a, g_dev, flags, st);
    case 16: return launch_train<16, 1>(a, g_dev, flags, st);
    case 8: return launch_train<8, 1>(a, g_dev, flags, st);
    case 4: return launch_train<4, 1>(a, g_dev, flags, st);
    case 2: return launch_train<2, 1>(a, g_dev, flags, st);
    default: return launch_train<1, 1>(a, g_dev, flags, st);
  }
}

int gosh_project(const float *M_coarse_dev, int64_t n_coarse, const int32_t *map_dev, int64_t n_fine,
                 int32_t d, float *M_fine_dev, void *hip_stream) {
  if (int rc = gosh::check_matrix(M_coarse_dev, d, "M_coarse")) return rc;
  if (int rc = gosh::check_matrix(M_fine_dev, d, "M_fine")) return rc;
  if (map_dev == nullptr) return gosh::fail(GOSH_EINVAL, "map is null");
  if (n_coarse < 1 || n_fine < 1 || n_coarse > n_fine)
    return gosh::fail(GOSH_EINVAL, "need 1 <= n_coarse (%lld) <= n_fine (%lld)", (long long)n_coarse,
                      (long long)n_fine);
  const int64_t total4 = n_fine * (d / 4);
  hipLaunchKernelGGL(project_kernel, dim3(grid_for(total4, 256, 1 << 16)), dim3(256), 0,
                     gosh::as_stream(hip_stream), reinterpret_cast<const float4 *>(M_coarse_dev),
                     map_dev, reinterpret_cast<float4 *>(M_fine_dev), total4, d / 4);
  return gosh::check_launch("project_kernel");
}

}  // extern "C"

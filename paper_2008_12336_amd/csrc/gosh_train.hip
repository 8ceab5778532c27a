// Device side of libgosh for graphs that fit the device: sampler, epoch kernel
// (Alg. 3 with the update of Alg. 1), initialisation and projection.  gfx950 only:
// 64-lane wavefronts, coalesced row accesses, cross-lane reductions with DPP.
//
// Work layout of the epoch kernel (the generic kernel lives in gosh_device.h).  A
// "lane group" of LPG lanes (a power of two covering d/4) owns one source vertex, so a
// wavefront carries 64/LPG sources (two at d = 128, eight at d = 32).  The source row
// stays in registers for its 1 + k_neg updates and is written back once; sample rows
// are fetched four at a time before the first dot product so that their HBM latencies
// overlap.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <mutex>

#include "gosh_common.h"
#include "gosh_device.h"

namespace {

using gosh::philox_draw;
using gosh::scale_draw;

struct SamplerArgs {
  const void *xadj;
  const int32_t *adj;
  int64_t nnz;
  uint32_t n;
  uint32_t key0, key1;
  uint32_t epoch, level;
};

// Number of entries of the row [begin, end) that may be read.  The kernels stay inside
// their operands whatever the graph arrays hold: a row that the offsets place outside adj
// counts as empty, and an entry that names no vertex is no sample.
template <typename OffT>
__device__ __forceinline__ uint32_t row_entries(OffT begin, OffT end, int64_t nnz) {
  const bool inside = begin >= 0 && begin <= end && static_cast<int64_t>(end) <= nnz;
  return inside ? static_cast<uint32_t>(end - begin) : 0u;
}

// Sample j of source src: j = 0 positive (uniform neighbour, -1 if none), j >= 1
// negative (uniform vertex).
template <typename OffT>
__device__ __forceinline__ int32_t draw_sample(const SamplerArgs &a, uint32_t src, uint32_t j) {
  const uint64_t r = philox_draw(src, j, a.epoch, a.level, a.key0, a.key1);
  if (j != 0) return static_cast<int32_t>(scale_draw(r, a.n));
  const OffT *xadj = static_cast<const OffT *>(a.xadj);
  const OffT begin = xadj[src];
  const uint32_t deg = row_entries(begin, xadj[src + 1], a.nnz);
  if (deg == 0) return -1;
  const int32_t neighbour = a.adj[begin + static_cast<OffT>(scale_draw(r, deg))];
  return static_cast<uint32_t>(neighbour) < a.n ? neighbour : -1;
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

// Work description of one epoch of Alg. 3 for the generic kernel: every vertex is a
// source, sample t is draw t of that source, rows live in one matrix.
template <typename OffT>
struct EpochWork {
  SamplerArgs s;
  float *M;
  int32_t d;
  __device__ __forceinline__ int64_t count() const { return s.n; }
  __device__ __forceinline__ int32_t source_id(int64_t i) const { return static_cast<int32_t>(i); }
  __device__ __forceinline__ float *source_row(int64_t i) const { return M + i * d; }
  // What sampling needs from memory knowing the source alone: where its neighbour list is.
  struct Pre {
    OffT begin;
    uint32_t deg;
  };
  __device__ __forceinline__ Pre stage1(int64_t i, bool) const {  // i is a valid source also when unwanted
    const OffT *xadj = static_cast<const OffT *>(s.xadj);
    const OffT begin = xadj[i];
    return Pre{begin, row_entries(begin, xadj[i + 1], s.nnz)};
  }
  // Sample t of a source is draw t; the positive reads the neighbour list.  Written
  // without branches around the read: lanes that do not want a positive read the
  // first offset again instead of a neighbour entry.
  // The draw itself is arithmetic only; the kernel skips it where no group of the wavefront wants it.
  __device__ __forceinline__ uint64_t draw(int64_t, int32_t src, int32_t t) const {
    return philox_draw(static_cast<uint32_t>(src), static_cast<uint32_t>(t), s.epoch, s.level, s.key0, s.key1);
  }
  __device__ __forceinline__ int32_t stage2(int64_t, int32_t, int32_t, bool want, bool positive, const Pre &pre,
                                            uint64_t r) const {
    const bool read_adj = want && positive && pre.deg != 0;
    const int32_t *entry = read_adj ? s.adj + (pre.begin + static_cast<OffT>(scale_draw(r, pre.deg)))
                                    : reinterpret_cast<const int32_t *>(s.xadj);
    const int32_t neighbour = *entry;
    const int32_t uniform = static_cast<int32_t>(scale_draw(r, s.n));
    const bool is_vertex = static_cast<uint32_t>(neighbour) < s.n;
    const int32_t id = positive ? (read_adj && is_vertex ? neighbour : -1) : uniform;
    return want ? id : -1;
  }
  __device__ __forceinline__ float *sample_row(int64_t, int32_t v) const {
    return M + static_cast<int64_t>(v) * d;
  }
};

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
    if (v < n) hot = static_cast<int64_t>(xadj[v + 1]) - static_cast<int64_t>(xadj[v]) >= min_degree;
    const unsigned long long mask = __ballot(hot);
    if (lane == 0) bits[w] = mask;
  }
}

// ---------------------------------------------------------------------------------
// M points at row `first_row` of the matrix being initialised.
__global__ __launch_bounds__(256) void init_embedding_kernel(float4 *__restrict__ M, int64_t total4,
                                                             int64_t first_row, int32_t d4,
                                                             uint32_t key0, uint32_t key1,
                                                             uint32_t level) {
  const double d = 4.0 * d4;
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < total4; i += gridDim.x * 256LL) {
    const uint32_t v = static_cast<uint32_t>(first_row + i / d4), c4 = static_cast<uint32_t>(i % d4);
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

// A map entry that names no coarse vertex gives a row of zeros.
__global__ __launch_bounds__(256) void project_kernel(const float4 *__restrict__ coarse,
                                                      const int32_t *__restrict__ map,
                                                      float4 *__restrict__ fine, int64_t total4,
                                                      int32_t d4, uint32_t n_coarse) {
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < total4; i += gridDim.x * 256LL) {
    const int64_t v = i / d4;
    const int32_t c4 = static_cast<int32_t>(i % d4);
    const uint32_t c = static_cast<uint32_t>(map[v]);
    fine[i] = c < n_coarse ? coarse[static_cast<int64_t>(c) * d4 + c4] : float4{0.f, 0.f, 0.f, 0.f};
  }
}

// Row probe: the row traffic of the training kernels without their arithmetic.  A lane group
// of `lpg` lanes (a power of two covering d/4, at most 64) moves one row with 128-bit
// accesses, so a wavefront carries 64/lpg rows at a time, like the training kernels.
//   kProbeReadWrite  a random row is read and written back with `nothing` (zero) added
//   kProbeRead       a random row is read (a store that never happens keeps the loads alive)
//   kProbeWrite      a random row is overwritten with `nothing`
//   kProbeEpochMix   what one source of an epoch with three negatives moves: row i (sources
//                    are consecutive) and four random rows are read, all five requested
//                    before the first is used, then written back with `nothing` added
// Draw q of access i is Philox(counter = (i_lo, i_hi, 0xFFFFFFFE, q), key = seed).
enum ProbeMode : int32_t { kProbeReadWrite = 0, kProbeRead = 1, kProbeWrite = 2, kProbeEpochMix = 3 };

template <int MODE>
__global__ __launch_bounds__(256) void row_probe_kernel(float4 *__restrict__ M, uint64_t n, int32_t d4,
                                                        int32_t lpg, uint64_t accesses, uint32_t key0,
                                                        uint32_t key1, float nothing) {
  constexpr int kRows = MODE == kProbeEpochMix ? 5 : 1;
  const int lane = threadIdx.x & 63, gl = lane & (lpg - 1), gpw = 64 / lpg;
  const uint64_t wave = (blockIdx.x * 256ull + threadIdx.x) >> 6, waves = (gridDim.x * 256ull) >> 6;
  float sink = 0.f;
  for (uint64_t base = wave * gpw; base < accesses; base += waves * gpw) {
    const uint64_t i = base + lane / lpg;
    if (i >= accesses) continue;
    uint64_t row[kRows];
#pragma unroll
    for (int q = 0; q < kRows; ++q) {
      const uint64_t draw = philox_draw(static_cast<uint32_t>(i), static_cast<uint32_t>(i >> 32), 0xFFFFFFFEu,
                                        static_cast<uint32_t>(q), key0, key1);
      row[q] = (MODE == kProbeEpochMix && q == 0) ? i % n : scale_draw(draw, static_cast<uint32_t>(n));
    }
    float4 v[kRows][2];
#pragma unroll
    for (int q = 0; q < kRows; ++q)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = gl + u * lpg;
        v[q][u] = float4{0.f, 0.f, 0.f, 0.f};
        if (MODE != kProbeWrite && c < d4) v[q][u] = M[row[q] * d4 + c];
      }
#pragma unroll
    for (int q = 0; q < kRows; ++q)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = gl + u * lpg;
        if (MODE == kProbeRead) {
          sink += v[q][u].x;
        } else if (c < d4) {
          float4 x = v[q][u];
          x.x += nothing;
          M[row[q] * d4 + c] = x;
        }
      }
  }
  if (MODE == kProbeRead && sink == 1.2345e-30f) M[0].x = sink;  // practically never: keeps the loads
}

// Largest finite |x| and the number of non-finite entries of `total4` float4s, accumulated
// into *out (which the caller has cleared).  The bits of a non-negative finite float order
// like the float, so the maximum is taken on them.
__global__ __launch_bounds__(256) void matrix_check_kernel(const float4 *__restrict__ M, int64_t total4,
                                                           gosh::CheckResult *__restrict__ out) {
  uint32_t top = 0, bad = 0;
  for (int64_t i = blockIdx.x * 256LL + threadIdx.x; i < total4; i += gridDim.x * 256LL) {
    const float4 x = M[i];
    const float e[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t mag = __float_as_uint(e[c]) & 0x7FFFFFFFu;
      const bool finite = mag < 0x7F800000u;
      top = finite ? max(top, mag) : top;
      bad += finite ? 0u : 1u;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    top = max(top, static_cast<uint32_t>(__shfl_xor(static_cast<int>(top), off, 64)));
    bad += static_cast<uint32_t>(__shfl_xor(static_cast<int>(bad), off, 64));
  }
  if ((threadIdx.x & 63) == 0) {
    if (top) atomicMax(&out->max_bits, top);
    if (bad) atomicAdd(&out->nonfinite, static_cast<unsigned long long>(bad));
  }
}

__global__ void clear_check_kernel(gosh::CheckResult *out) {
  out->max_bits = 0;
  out->pad = 0;
  out->nonfinite = 0;
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
  s.nnz = g->nnz;
  s.n = static_cast<uint32_t>(g->n);
  s.key0 = static_cast<uint32_t>(seed);
  s.key1 = static_cast<uint32_t>(seed >> 32);
  s.epoch = epoch;
  s.level = level;
  return s;
}

// bits_override: the hot-row bitmap to use instead of the library's grown-on-demand scratch
// (at least (n + 63) / 64 * 8 bytes), or null.
template <typename OffT>
int launch_epoch(const gosh_csr *g, float *M, int32_t d, int32_t k_neg, float lr, uint64_t seed,
                 uint32_t epoch, uint32_t level, uint32_t flags, void *bits_override, hipStream_t st) {
  const bool seq = (flags & GOSH_FLAG_SEQUENTIAL) != 0;
  // the write paths of the concurrent kernel: in concurrent mode, and in the sequential walk
  // that is asked to use them
  const bool concurrent_paths = !seq || (flags & GOSH_FLAG_CONCURRENT_LAYOUT) != 0;
  const gosh_tuning tune = gosh::tuning();
  const int64_t n = g->n;
  EpochWork<OffT> w;
  w.s = sampler_args(g, seed, epoch, level);
  w.M = M;
  w.d = d;
  gosh::SgdArgs a{};
  a.d = d;
  a.k_neg = k_neg;
  a.samples = k_neg + 1;
  a.lr = lr;
  a.hot = gosh::HotSet{nullptr, gosh::kHotNone};
  const int64_t max_waves = tune.max_waves;
  if (concurrent_paths) {
    // Sources in flight C, and the hot-row rule.  A vertex is hot if its expected
    // positive hits per epoch, deg/avg_deg, give more than eps = 1/64 concurrent holders:
    // deg * C / nnz > eps.  On graphs so small that even the k+1 uniform touches of
    // every row overlap ((k+1)*C/n > 1/4, i.e. fewer than 16 rounds at k = 3) all rows
    // are hot.  Both constants come from link-prediction AUCROC against the sequential
    // reference on R-MAT graphs of 2^12..2^20 vertices: with them the concurrent kernel
    // stays within 0.001..0.005 of the reference, without them it drops by up to 0.4.
    const int gpw = gosh::SgdLauncher<EpochWork<OffT>>::groups_per_wave(d);
    int64_t waves = std::min<int64_t>((n + gpw - 1) / gpw, max_waves);
    const int64_t in_flight = std::min<int64_t>(waves, gosh::resident_waves()) * gpw;
    int mode = gosh::kHotBitmap;
    if (tune.hot_min_degree == 0 && (k_neg + 1) * in_flight * tune.hot_all_inv_eps > n) mode = gosh::kHotAll;
    if (flags & GOSH_FLAG_PLAIN_STORES) mode = gosh::kHotNone;
    if (flags & GOSH_FLAG_ATOMIC_ADDS) mode = gosh::kHotAll;
    if (mode == gosh::kHotBitmap) {
      const int64_t min_degree =
          tune.hot_min_degree > 0 ? tune.hot_min_degree : g->nnz / (tune.hot_inv_eps * in_flight) + 1;
      void *bits = bits_override;
      if (bits == nullptr)
        if (int rc = gosh::hot_scratch(static_cast<size_t>((n + 63) / 64) * 8, &bits)) return rc;
      const int blocks = static_cast<int>(std::min<int64_t>(((n + 63) / 64 + 3) / 4, 1 << 16));
      hipLaunchKernelGGL(mark_hot_kernel<OffT>, dim3(blocks), dim3(256), 0, st,
                         static_cast<const OffT *>(g->xadj), n, min_degree,
                         static_cast<unsigned long long *>(bits));
      if (int rc = gosh::check_launch("mark_hot_kernel")) return rc;
      a.hot.bits = static_cast<const uint32_t *>(bits);
    }
    a.hot.mode = mode;
  }
  if (a.hot.bits == nullptr) {
    // the kernel reads word 0 of the bitmap unconditionally
    void *bits = bits_override;
    if (bits == nullptr)
      if (int rc = gosh::hot_scratch(8, &bits)) return rc;
    a.hot.bits = static_cast<const uint32_t *>(bits);
  }
  const bool plain_rows = tune.plain_rows != 0 || (seq && !concurrent_paths);
  gosh::SgdLauncher<EpochWork<OffT>>::launch(w, a, n, seq, plain_rows, max_waves, st);
  return gosh::check_launch("sgd_kernel (epoch)");
}

// Hot-row bitmap of gosh_train_epoch_static: one bit per vertex, in the code object itself.
// Host code must not use this name as an address (on the host it is a stand-in, not device
// memory): static_bitmap() asks the runtime for the array's address on the current device.
static __device__ __align__(256) unsigned long long scratch[GOSH_STATIC_MAX_N / 64];

int static_bitmap(void **out) {
  constexpr int kMaxDevices = 64;
  static void *address[kMaxDevices] = {};  // every device holds its own copy of the array
  static std::mutex mutex;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return gosh::fail(GOSH_EHIP, "cannot identify the current device");
  std::lock_guard<std::mutex> lock(mutex);
  if (address[dev] == nullptr) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return gosh::fail(GOSH_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    }
    address[dev] = p;
  }
  *out = address[dev];
  return GOSH_OK;
}

int check_epoch_args(const gosh_csr *g_dev, float *M_dev, int32_t d, int32_t k_neg, float lr_epoch,
                     uint32_t flags) {
  if (int rc = gosh::check_csr(g_dev)) return rc;
  if (int rc = gosh::check_matrix(M_dev, d, "M")) return rc;
  if (k_neg < 0 || k_neg > GOSH_MAX_NEG)
    return gosh::fail(GOSH_EINVAL, "k_neg = %d: must be in [0, %d]", k_neg, GOSH_MAX_NEG);
  if (flags & ~(GOSH_FLAG_SEQUENTIAL | GOSH_FLAG_PLAIN_STORES | GOSH_FLAG_ATOMIC_ADDS | GOSH_FLAG_CONCURRENT_LAYOUT))
    return gosh::fail(GOSH_EINVAL, "unknown flags 0x%x", flags);
  if ((flags & GOSH_FLAG_PLAIN_STORES) && (flags & GOSH_FLAG_ATOMIC_ADDS))
    return gosh::fail(GOSH_EINVAL, "flags ask for plain stores and atomic adds at once");
  if (!(lr_epoch == lr_epoch)) return gosh::fail(GOSH_EINVAL, "lr is NaN");
  if (int rc = gosh::check_device_csr(g_dev)) return rc;
  return gosh::check_device_span(M_dev, static_cast<size_t>(g_dev->n) * d * 4, "M");
}

}  // namespace

namespace gosh {

int matrix_check_clear(CheckResult *result_dev, hipStream_t st) {
  hipLaunchKernelGGL(clear_check_kernel, dim3(1), dim3(1), 0, st, result_dev);
  return check_launch("clear_check_kernel");
}

int matrix_check_add(const float *rows_dev, int64_t floats, CheckResult *result_dev, hipStream_t st) {
  const int64_t total4 = floats / 4;
  if (total4 <= 0) return GOSH_OK;
  hipLaunchKernelGGL(matrix_check_kernel, dim3(grid_for(total4, 1024, 1 << 13)), dim3(256), 0, st,
                     reinterpret_cast<const float4 *>(rows_dev), total4, result_dev);
  return check_launch("matrix_check_kernel");
}

int matrix_check_read(const CheckResult *result_dev, float *max_abs, int64_t *nonfinite, hipStream_t st) {
  CheckResult host{};
  GOSH_TRY_HIP(hipMemcpyAsync(&host, result_dev, sizeof(host), hipMemcpyDeviceToHost, st), "read matrix check");
  GOSH_TRY_HIP(hipStreamSynchronize(st), "matrix check");
  if (max_abs) {
    float f;
    static_assert(sizeof(f) == sizeof(host.max_bits), "fp32");
    __builtin_memcpy(&f, &host.max_bits, 4);
    *max_abs = f;
  }
  if (nonfinite) *nonfinite = static_cast<int64_t>(host.nonfinite);
  return GOSH_OK;
}

int row_probe(float *M_dev, int64_t n, int32_t d, int64_t accesses, uint64_t seed, int32_t mode, hipStream_t st) {
  if (accesses <= 0) return GOSH_OK;
  const int32_t d4 = d / 4;
  int32_t lpg = 1;
  while (lpg < d4 && lpg < 64) lpg *= 2;
  const int64_t per_block = 4 * (64 / lpg);  // four wavefronts per block
  const int blocks = grid_for(accesses, static_cast<int>(per_block), 1 << 18);
  float4 *M4 = reinterpret_cast<float4 *>(M_dev);
  const uint64_t un = static_cast<uint64_t>(n), ua = static_cast<uint64_t>(accesses);
  const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
  switch (mode) {
    case kProbeReadWrite:
      hipLaunchKernelGGL(row_probe_kernel<kProbeReadWrite>, dim3(blocks), dim3(256), 0, st, M4, un, d4, lpg, ua, k0, k1, 0.0f);
      break;
    case kProbeRead:
      hipLaunchKernelGGL(row_probe_kernel<kProbeRead>, dim3(blocks), dim3(256), 0, st, M4, un, d4, lpg, ua, k0, k1, 0.0f);
      break;
    case kProbeWrite:
      hipLaunchKernelGGL(row_probe_kernel<kProbeWrite>, dim3(blocks), dim3(256), 0, st, M4, un, d4, lpg, ua, k0, k1, 0.0f);
      break;
    case kProbeEpochMix:
      hipLaunchKernelGGL(row_probe_kernel<kProbeEpochMix>, dim3(blocks), dim3(256), 0, st, M4, un, d4, lpg, ua, k0, k1, 0.0f);
      break;
    default:
      return fail(GOSH_EINVAL, "probe mode %d: must be 0 (read-write), 1 (read), 2 (write) or 3 (epoch mix)", mode);
  }
  return check_launch("row_probe_kernel");
}

int init_rows(float *rows_dev, int64_t first_row, int64_t count, int32_t d, uint64_t seed,
              uint32_t level, hipStream_t st) {
  const int64_t total4 = count * (d / 4);
  hipLaunchKernelGGL(init_embedding_kernel, dim3(grid_for(total4, 256, 1 << 16)), dim3(256), 0, st,
                     reinterpret_cast<float4 *>(rows_dev), total4, first_row, d / 4,
                     static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32), level);
  return check_launch("init_embedding_kernel");
}

}  // namespace gosh

extern "C" {

int gosh_init_embedding(float *M_dev, int64_t n, int32_t d, uint64_t seed, uint32_t level,
                        void *hip_stream) {
  if (int rc = gosh::check_matrix(M_dev, d, "M")) return rc;
  if (n < 1 || n >= 2147483647LL) return gosh::fail(GOSH_EINVAL, "n = %lld out of range", (long long)n);
  if (int rc = gosh::check_device_span(M_dev, static_cast<size_t>(n) * d * 4, "M")) return rc;
  return gosh::init_rows(M_dev, 0, n, d, seed, level, gosh::as_stream(hip_stream));
}

int gosh_sample_epoch(const gosh_csr *g_dev, int32_t k_neg, uint64_t seed, uint32_t epoch,
                      uint32_t level, int32_t *out_dev, void *hip_stream) {
  if (int rc = gosh::check_csr(g_dev)) return rc;
  if (k_neg < 0 || k_neg > GOSH_MAX_NEG)
    return gosh::fail(GOSH_EINVAL, "k_neg = %d: must be in [0, %d]", k_neg, GOSH_MAX_NEG);
  if (out_dev == nullptr) return gosh::fail(GOSH_EINVAL, "out is null");
  if (int rc = gosh::check_device_csr(g_dev)) return rc;
  if (int rc = gosh::check_device_span(out_dev, static_cast<size_t>(g_dev->n) * (k_neg + 1) * 4, "out")) return rc;
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
  if (int rc = check_epoch_args(g_dev, M_dev, d, k_neg, lr_epoch, flags)) return rc;
  hipStream_t st = gosh::as_stream(hip_stream);
  if (g_dev->xadj_is64)
    return launch_epoch<int64_t>(g_dev, M_dev, d, k_neg, lr_epoch, seed, epoch, level, flags, nullptr, st);
  return launch_epoch<int32_t>(g_dev, M_dev, d, k_neg, lr_epoch, seed, epoch, level, flags, nullptr, st);
}

int gosh_train_epoch_static(const gosh_csr *g_dev, float *M_dev, int32_t d, int32_t k_neg, float lr_epoch,
                            uint64_t seed, uint32_t epoch, uint32_t level, uint32_t flags,
                            void *hip_stream) {
  if (g_dev != nullptr && g_dev->n > GOSH_STATIC_MAX_N)
    return gosh::fail(GOSH_EINVAL, "n = %lld: gosh_train_epoch_static takes at most %lld vertices (use gosh_train_epoch)",
                      (long long)g_dev->n, (long long)GOSH_STATIC_MAX_N);
  if (int rc = check_epoch_args(g_dev, M_dev, d, k_neg, lr_epoch, flags)) return rc;
  void *bits = nullptr;
  if (int rc = static_bitmap(&bits)) return rc;
  hipStream_t st = gosh::as_stream(hip_stream);
  if (g_dev->xadj_is64)
    return launch_epoch<int64_t>(g_dev, M_dev, d, k_neg, lr_epoch, seed, epoch, level, flags, bits, st);
  return launch_epoch<int32_t>(g_dev, M_dev, d, k_neg, lr_epoch, seed, epoch, level, flags, bits, st);
}

int gosh_matrix_check(const float *M_dev, int64_t n, int32_t d, float *max_abs, int64_t *nonfinite,
                      void *hip_stream) {
  if (int rc = gosh::check_matrix(M_dev, d, "M")) return rc;
  if (n < 1 || n >= 2147483647LL) return gosh::fail(GOSH_EINVAL, "n = %lld out of range", (long long)n);
  if (int rc = gosh::check_device_span(M_dev, static_cast<size_t>(n) * d * 4, "M")) return rc;
  hipStream_t st = gosh::as_stream(hip_stream);
  gosh::CheckResult *result = nullptr;
  if (int rc = gosh::check_scratch(&result)) return rc;
  if (int rc = gosh::matrix_check_clear(result, st)) return rc;
  if (int rc = gosh::matrix_check_add(M_dev, n * d, result, st)) return rc;
  return gosh::matrix_check_read(result, max_abs, nonfinite, st);
}

int gosh_row_probe(float *M_dev, int64_t n, int32_t d, int64_t accesses, uint64_t seed, int32_t mode,
                   void *hip_stream) {
  if (int rc = gosh::check_matrix(M_dev, d, "M")) return rc;
  if (n < 1 || n >= 2147483647LL) return gosh::fail(GOSH_EINVAL, "n = %lld out of range", (long long)n);
  if (accesses < 0) return gosh::fail(GOSH_EINVAL, "accesses = %lld is negative", (long long)accesses);
  if (mode < 0 || mode > 3)
    return gosh::fail(GOSH_EINVAL, "probe mode %d: must be 0 (read-write), 1 (read), 2 (write) or 3 (epoch mix)", mode);
  if (int rc = gosh::check_device_span(M_dev, static_cast<size_t>(n) * d * 4, "M")) return rc;
  return gosh::row_probe(M_dev, n, d, accesses, seed, mode, gosh::as_stream(hip_stream));
}

int gosh_project(const float *M_coarse_dev, int64_t n_coarse, const int32_t *map_dev, int64_t n_fine,
                 int32_t d, float *M_fine_dev, void *hip_stream) {
  if (int rc = gosh::check_matrix(M_coarse_dev, d, "M_coarse")) return rc;
  if (int rc = gosh::check_matrix(M_fine_dev, d, "M_fine")) return rc;
  if (map_dev == nullptr) return gosh::fail(GOSH_EINVAL, "map is null");
  if (n_coarse < 1 || n_fine < 1)
    return gosh::fail(GOSH_EINVAL, "need n_coarse (%lld) >= 1 and n_fine (%lld) >= 1",
                      (long long)n_coarse, (long long)n_fine);
  if (int rc = gosh::check_device_span(M_coarse_dev, static_cast<size_t>(n_coarse) * d * 4, "M_coarse")) return rc;
  if (int rc = gosh::check_device_span(M_fine_dev, static_cast<size_t>(n_fine) * d * 4, "M_fine")) return rc;
  if (int rc = gosh::check_device_span(map_dev, static_cast<size_t>(n_fine) * 4, "map")) return rc;
  const int64_t total4 = n_fine * (d / 4);
  hipLaunchKernelGGL(project_kernel, dim3(grid_for(total4, 256, 1 << 16)), dim3(256), 0,
                     gosh::as_stream(hip_stream), reinterpret_cast<const float4 *>(M_coarse_dev),
                     map_dev, reinterpret_cast<float4 *>(M_fine_dev), total4, d / 4,
                     static_cast<uint32_t>(std::min<int64_t>(n_coarse, 2147483647LL)));
  return gosh::check_launch("project_kernel");
}

}  // extern "C"

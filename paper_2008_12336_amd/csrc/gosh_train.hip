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

__device__ __forceinline__ float dot4(const float4 &a, const float4 &b) {
  return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w;
}
__device__ __forceinline__ void axpy4(float4 &y, float g, const float4 &x) {
  y.x = fmaf(g, x.x, y.x);
  y.y = fmaf(g, x.y, y.y);
  y.z = fmaf(g, x.z, y.z);
  y.w = fmaf(g, x.w, y.w);
}

struct TrainArgs {
  SamplerArgs s;
  float *M;
  int32_t d4;  // d / 4
  int32_t k_neg;
  float lr;
};

constexpr int kChunk = 4;  // sample rows in flight per source

// One epoch.  SEQ: a single lane group walks all sources in ascending order (the
// sequential-order result); otherwise groups stride over the sources.
template <int LPG, int VPL, typename OffT, bool SEQ>
__global__ __launch_bounds__(256) void train_epoch_kernel(TrainArgs a) {
  constexpr int kGroupsPerWave = 64 / LPG;
  const int lane = threadIdx.x & 63;
  const int gl = lane & (LPG - 1);
  if (SEQ && (lane >= LPG || threadIdx.x >= 64 || blockIdx.x != 0)) return;

  const int64_t wave = blockIdx.x * static_cast<int64_t>(blockDim.x / 64) + (threadIdx.x >> 6);
  const int64_t n = a.s.n;
  const int64_t stride = SEQ ? 1 : static_cast<int64_t>(gridDim.x) * (blockDim.x / 64) * kGroupsPerWave;
  const int64_t first = SEQ ? 0 : wave * kGroupsPerWave + lane / LPG;
  const int32_t d4 = a.d4;
  float4 *const Mv = reinterpret_cast<float4 *>(a.M);

  bool col_ok[VPL];
#pragma unroll
  for (int i = 0; i < VPL; ++i) col_ok[i] = gl + i * LPG < d4;

  // The loop bound is uniform over the wave; groups past the end idle inside.
  const int64_t first_of_wave = SEQ ? 0 : wave * kGroupsPerWave;
  for (int64_t base = first_of_wave; base < n; base += stride) {
    const int64_t src = first + (base - first_of_wave);
    if (src >= n) continue;
    float4 *const src_row = Mv + src * d4;
    float4 s[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) s[i] = col_ok[i] ? src_row[gl + i * LPG] : float4{0.f, 0.f, 0.f, 0.f};

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
      float4 t[kChunk][VPL];
#pragma unroll
      for (int q = 0; q < kChunk; ++q) {
        const float4 *row = Mv + static_cast<int64_t>(v[q] < 0 ? 0 : v[q]) * d4;
#pragma unroll
        for (int i = 0; i < VPL; ++i)
          t[q][i] = (v[q] >= 0 && col_ok[i]) ? row[gl + i * LPG] : float4{0.f, 0.f, 0.f, 0.f};
      }

#pragma unroll
      for (int q = 0; q < kChunk; ++q) {
        if (v[q] < 0) continue;  // uniform over the group
        float partial = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) partial += dot4(s[i], t[q][i]);
        const float x = group_sum<LPG>(partial);
        const float label = (j0 + q == 0) ? 1.f : 0.f;
        const float g = a.lr * (label - 1.f / (1.f + expf(-x)));
        float4 *row = Mv + static_cast<int64_t>(v[q]) * d4;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
          axpy4(s[i], g, t[q][i]);
          axpy4(t[q][i], g, s[i]);
          if (col_ok[i]) row[gl + i * LPG] = t[q][i];
        }
        // A later sample of the same chunk that names the same vertex must see this
        // update: forward the registers instead of the stale prefetched copy.
#pragma unroll
        for (int r = q + 1; r < kChunk; ++r)
          if (v[r] == v[q]) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) t[r][i] = t[q][i];
          }
      }
    }
#pragma unroll
    for (int i = 0; i < VPL; ++i)
      if (col_ok[i]) src_row[gl + i * LPG] = s[i];
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

template <int LPG, int VPL>
void launch_train(const TrainArgs &a, bool is64, bool seq, int blocks, hipStream_t st) {
  if (seq) {
    if (is64) hipLaunchKernelGGL((train_epoch_kernel<LPG, VPL, int64_t, true>), dim3(1), dim3(64), 0, st, a);
    else hipLaunchKernelGGL((train_epoch_kernel<LPG, VPL, int32_t, true>), dim3(1), dim3(64), 0, st, a);
  } else {
    if (is64) hipLaunchKernelGGL((train_epoch_kernel<LPG, VPL, int64_t, false>), dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((train_epoch_kernel<LPG, VPL, int32_t, false>), dim3(blocks), dim3(256), 0, st, a);
  }
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
  if (flags & ~GOSH_FLAG_SEQUENTIAL) return gosh::fail(GOSH_EINVAL, "unknown flags 0x%x", flags);
  if (!(lr_epoch == lr_epoch)) return gosh::fail(GOSH_EINVAL, "lr is NaN");

  TrainArgs a;
  a.s = sampler_args(g_dev, seed, epoch, level);
  a.M = M_dev;
  a.d4 = d / 4;
  a.k_neg = k_neg;
  a.lr = lr_epoch;
  const bool seq = (flags & GOSH_FLAG_SEQUENTIAL) != 0;
  const bool is64 = g_dev->xadj_is64 != 0;
  hipStream_t st = gosh::as_stream(hip_stream);

  // Smallest power-of-two lane group that covers d/4 vectors (two vectors per lane
  // above 64 vectors).
  int lpg = 1;
  while (lpg < a.d4 && lpg < 64) lpg *= 2;
  const int64_t groups_per_block = 256 / lpg;
  const int blocks = grid_for(g_dev->n, static_cast<int>(groups_per_block), 1 << 20);
  if (a.d4 > 64) launch_train<64, 2>(a, is64, seq, blocks, st);
  else switch (lpg) {
    case 64: launch_train<64, 1>(a, is64, seq, blocks, st); break;
    case 32: launch_train<32, 1>(a, is64, seq, blocks, st); break;
    case 16: launch_train<16, 1>(a, is64, seq, blocks, st); break;
    case 8: launch_train<8, 1>(a, is64, seq, blocks, st); break;
    case 4: launch_train<4, 1>(a, is64, seq, blocks, st); break;
    case 2: launch_train<2, 1>(a, is64, seq, blocks, st); break;
    default: launch_train<1, 1>(a, is64, seq, blocks, st); break;
  }
  return gosh::check_launch("train_epoch_kernel");
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

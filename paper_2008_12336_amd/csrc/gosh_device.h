// Device-side building blocks of libgosh shared by the epoch kernel (Alg. 3) and the
// part-pair kernel (Alg. 5): the counter-based generator, the cross-lane reduction,
// the row access policies and the generic lock-free SGD kernel.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

namespace gosh {

// ---------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  Returns the first two output words as one
// 64-bit draw; w2/w3 optionally receive the other two.  Usable on host and device.
// ---------------------------------------------------------------------------------
__host__ __device__ __forceinline__ uint32_t mul_hi32(uint32_t a, uint32_t b) {
  return static_cast<uint32_t>((static_cast<uint64_t>(a) * b) >> 32);
}

__host__ __device__ __forceinline__ uint64_t philox_draw(uint32_t c0, uint32_t c1, uint32_t c2,
                                                         uint32_t c3, uint32_t k0, uint32_t k1,
                                                         uint32_t *w2 = nullptr,
                                                         uint32_t *w3 = nullptr) {
  constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
  constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hiA = mul_hi32(kMulA, c0), loA = kMulA * c0;
    const uint32_t hiB = mul_hi32(kMulB, c2), loB = kMulB * c2;
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
__host__ __device__ __forceinline__ uint32_t scale_draw(uint64_t r, uint32_t bound) {
  const uint32_t lo = static_cast<uint32_t>(r), hi = static_cast<uint32_t>(r >> 32);
  const uint64_t t = static_cast<uint64_t>(hi) * bound + mul_hi32(lo, bound);
  return static_cast<uint32_t>(t >> 32);
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
  if (LPG >= 2) x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
  if (LPG >= 4) x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
  if (LPG >= 8) x += dpp_move<0x141>(x);   // row_half_mirror (quads already uniform)
  if (LPG >= 16) x += dpp_move<0x140>(x);  // row_mirror (halves already uniform)
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
// needs the rows to be coherent across the whole device, so the concurrent kernels
// move rows with agent-scope (device-scope) accesses, which are served behind the
// per-XCD L2s.  Every sample row is touched once per turn, so no L2 reuse is lost.
//   RowAgent32: 32-bit relaxed atomic loads and stores at agent scope, lanes interleaved
//     over the row (lane g owns floats g, g+LPG, ...) so that every access instruction
//     of a group covers one whole 128-byte line.  Measured on a 2^24-vertex graph this
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
// Four floats live in one 128-bit register tuple: an explicit 128-bit load (RowAgent128)
// then delivers straight into the unit, with no instruction in between that could touch
// registers whose data has not arrived yet.
typedef float Float4 __attribute__((ext_vector_type(4)));
template <>
struct Unit<4> {
  Float4 v;
};

__device__ __forceinline__ void atomic_step(float *p, float x) {
  // Built with -munsafe-fp-atomics: the matrix is ordinary coarse-grained device
  // memory, where the hardware fp32 add is available.
  __hip_atomic_fetch_add(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Policies whose loads the compiler issues itself need no explicit wait.
struct TrackedLoads {
  static constexpr bool kWaveAtomics = false;  // a hot row is added to by the lanes that own it
  static __device__ __forceinline__ void wait_all() {}
  template <int F>
  static __device__ __forceinline__ void settle(Unit<F> &) {}
};

struct RowPlain128 : TrackedLoads {
  static constexpr int F = 4;
  static __device__ __forceinline__ Unit<4> load(const float *p) {
    return Unit<4>{*reinterpret_cast<const Float4 *>(p)};
  }
  static __device__ __forceinline__ void store(float *p, const Unit<4> &u) {
    *reinterpret_cast<Float4 *>(p) = u.v;
  }
};

// RowAgent128: 128-bit accesses at agent scope, four consecutive floats per lane, for
// d <= 64, where a row is at most two lines: rows that short move 12-23 % faster in 128-bit
// pieces on d/4 lanes than in 64-bit pieces on d/2 lanes (5.9 against 4.8 TB/s at d = 32),
// plain or device-scope alike.  The compiler offers device-scope accesses only as atomics of
// at most 64 bits, so the two instructions are written out (global_load_dwordx4 / global_store_dwordx4 with the sc1
// bit, which is what an agent-scope access is on this chip).  The compiler does not count
// these loads in its waits: settle() waits for all outstanding memory operations and ties
// every loaded unit to that wait, and must be called for a unit before its first use.
struct RowAgent128 {
  static constexpr int F = 4;
  static constexpr bool kWaveAtomics = true;  // a hot row is added to by the whole wavefront, see add_rows_as_a_wave
  static __device__ __forceinline__ Unit<4> load(const float *p) {
    Unit<4> u;
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(u.v) : "v"(p) : "memory");
    return u;
  }
  static __device__ __forceinline__ void store(float *p, const Unit<4> &u) {
    // A store of more than 64 bits still reads its data registers for two wait states after
    // it issues; the compiler pads its own stores and cannot see into this one.
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(u.v) : "memory");
  }
  static __device__ __forceinline__ void wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
  static __device__ __forceinline__ void settle(Unit<4> &u) { asm volatile("" : "+v"(u.v)); }
};

struct RowAgent32 : TrackedLoads {
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

struct HotSet {
  const uint32_t *bits;  // one bit per vertex when mode == kHotBitmap; in the other modes
                         // still a readable device word (the kernel reads word 0 blindly)
  int32_t mode;
};

struct SgdArgs {
  HotSet hot;
  int32_t d;
  int32_t k_neg;    // sample t of a source is a positive iff t % (k_neg + 1) == 0
  int32_t samples;  // samples per source: k_neg + 1 per round
  float lr;
  int64_t sources_per_block;  // consecutive sources that one workgroup walks (a multiple of
                              // the sources that its wavefronts take per turn)
};

constexpr int kChunk = 4;  // sample rows in flight per source

// Atomic adds of whole rows with 128-bit units, one row at a time by the whole wavefront.
// A memory-side fp32 atomic costs one operation per instruction and line it touches, full or
// sparse.  A lane group of d/4 lanes that adds its own four floats per lane needs four
// instructions per row, each touching every line of the row; here the rows to be added (one
// per lane group that asks, `mine`) are taken in turn, lane l of the wavefront fetches float l
// of the row's step from the lane that holds it and adds it at row + l: one instruction per
// row, each line touched once.  Needs d <= 64 and every lane of the wavefront present (no
// divergent branch around the call); `mine` and `row` are uniform inside a lane group.
template <int LPG>
__device__ __forceinline__ void add_rows_as_a_wave(bool mine, float *row, const Unit<4> &step, int32_t d, int lane) {
  unsigned long long todo = __ballot(mine && (lane & (LPG - 1)) == 0);
  const uint64_t address = reinterpret_cast<uint64_t>(row);
  const int piece = lane & 3;
  while (todo != 0) {
    const int leader = __builtin_amdgcn_readfirstlane(__builtin_ctzll(todo));
    todo &= todo - 1;
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(address), leader);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(address >> 32), leader);
    float *const target = reinterpret_cast<float *>((static_cast<uint64_t>(hi) << 32) | lo);
    const int owner = leader + (lane >> 2);  // lanes past the row wrap around and are masked below
    const float x0 = __shfl(step.v[0], owner, 64), x1 = __shfl(step.v[1], owner, 64);
    const float x2 = __shfl(step.v[2], owner, 64), x3 = __shfl(step.v[3], owner, 64);
    const float x = piece == 0 ? x0 : piece == 1 ? x1 : piece == 2 ? x2 : x3;
    if (lane < d) atomic_step(target + lane, x);
  }
}

// Position of a chunk of kChunk samples in the work of one lane group: source index, first
// sample of the chunk, and the index of the next positive sample at or after it.  All lane
// groups of a wavefront are at the same (t0, np); only idx differs.
struct ChunkPos {
  int64_t idx;
  int32_t t0, np;
  // The chunk that follows: the next kChunk samples of the same source, or the first chunk of
  // the group's next source.
  __device__ __forceinline__ ChunkPos next(int32_t samples, int32_t per_round, int64_t stride) const {
    const int32_t end = t0 + kChunk;
    int32_t p = np;
#pragma unroll
    for (int q = 0; q < kChunk; ++q) p = p < end ? p + per_round : p;
    const bool wrap = end >= samples;
    return ChunkPos{wrap ? idx + stride : idx, wrap ? 0 : end, wrap ? 0 : p};
  }
  // Which of the chunk's samples are positives.
  __device__ __forceinline__ void positives(int32_t per_round, bool (&is_pos)[kChunk]) const {
    int32_t p = np;
#pragma unroll
    for (int q = 0; q < kChunk; ++q) {
      is_pos[q] = (t0 + q == p);
      p = is_pos[q] ? p + per_round : p;
    }
  }
};

// The lock-free SGD kernel.  Every source applies `samples` updates of Alg. 1 in order:
//   g = lr * (b - sigmoid(M[src] . M[v]));  M[src] += g*M[v];  M[v] += g*M[src]
// with the source row held in registers for its whole turn.
//   W (work description, passed by value) provides
//     int64_t count()                         number of sources
//     int32_t source_id(int64_t i)            vertex id of source i (random counter, self test)
//     float  *source_row(int64_t i)
//     Pre     stage1(int64_t i, bool want)    what sampling for source i needs from memory and
//                                             can be asked for knowing i alone (row offsets)
//     uint64_t draw(int64_t i, int32_t id, int32_t t)
//                                             the random draw of sample t: arithmetic only
//     int32_t stage2(int64_t i, int32_t id, int32_t t, bool want, bool positive, Pre, uint64_t r)
//                                             vertex id of sample t from its draw r (-1 = none,
//                                             or !want)
//     float  *sample_row(int64_t i, int32_t v)
//     Both stages must be free of branches around their memory reads (read a safe address
//     when !want).
//   Sample t of a source is a positive iff t % (k_neg + 1) == 0.
//   P: row access policy; LPG lanes per source, UPL units per lane (LPG*UPL*P::F >= d).
//   SEQ: a single lane group walks all sources in ascending index (the sequential-order
//   result), with whatever policy, geometry and hot-row mode it is instantiated and called
//   with: all accesses to the matrix then come from one wavefront in program order, and the
//   memory system keeps the accesses of a wavefront to one address in that order, so stores
//   and atomic adds alike take effect in the order of Alg. 3.  Otherwise every workgroup
//   walks a block of consecutive sources, its lane groups working side by side.
//
// Sampling is independent of the matrix (the draws are counter-based), so it runs ahead of
// the updates as a three-stage pipeline over chunks of kChunk samples: while the rows of
// chunk c are in flight, the neighbour-list entry (or pool entry) of chunk c+1 is requested
// with offsets that were requested one chunk earlier, and the offsets of chunk c+2 are
// requested.  A lane group thus waits for one memory round trip per chunk -- its rows --
// instead of three in a row (offsets, then neighbour, then rows); for rows of a few hundred
// bytes or less that chain, not bandwidth, is what bounds the kernel.
//
// The body is written without branches around memory reads: a sample that does not
// exist, or a column beyond d, reads a harmless valid address and is masked afterwards
// (its step is forced to zero, its store is skipped).  All reads of a chunk are therefore
// issued back to back and waited for once, which is what keeps their latencies overlapped;
// with predicated reads the compiler splits the code into blocks and waits in each.
template <class P, int LPG, int UPL, class W, bool SEQ>
__global__ __launch_bounds__(256) void sgd_kernel(W w, SgdArgs a) {
  constexpr int kGroupsPerWave = 64 / LPG;
  constexpr int kPasses = (kChunk + LPG - 1) / LPG;  // sampler passes per chunk (lane q takes sample q)
  constexpr int F = P::F;
  using U = Unit<F>;
  using Pre = typename W::Pre;
  const int lane = threadIdx.x & 63;
  const int gl = lane & (LPG - 1);
  // The sequential walk is done by the first lane group of the first wavefront; the other
  // groups of that wavefront tag along without a source (the wavefront-wide atomic adds want
  // all 64 lanes present).
  if (SEQ && (threadIdx.x >= 64 || blockIdx.x != 0)) return;
  const bool group_on = !SEQ || lane < LPG;

  // A workgroup walks a block of consecutive sources: in each turn its wavefronts take one load
  // of kGroupsPerWave sources each, next to each other.  Workgroups start in the order of their
  // index, so the sources of an epoch are taken up in ascending order in time however many of
  // them one wavefront walks, and neighbouring sources (whose neighbour lists share cache
  // lines) are handled on one compute unit at one time.  `n` is the end of the block.
  const int64_t waves_per_block = SEQ ? 1 : blockDim.x / 64;
  const int64_t block_lo = SEQ ? 0 : blockIdx.x * a.sources_per_block;
  const int64_t first_of_wave = block_lo + (SEQ ? 0 : (threadIdx.x >> 6) * kGroupsPerWave);
  const int64_t n = SEQ ? w.count() : std::min<int64_t>(w.count(), block_lo + a.sources_per_block);
  const int64_t stride = SEQ ? 1 : waves_per_block * kGroupsPerWave;
  const int64_t first = first_of_wave + (SEQ ? 0 : lane / LPG);
  const int32_t d = a.d;
  const int32_t per_round = a.k_neg + 1;
  const bool use_bitmap = a.hot.mode == kHotBitmap;
  const bool all_hot = a.hot.mode == kHotAll;
  const uint32_t *const bits = a.hot.bits;  // always a readable word, also without a bitmap

  // Lane gl owns floats [(gl + i*LPG)*F, +F) of a row, i < UPL: consecutive lanes touch
  // consecutive addresses, so each access instruction covers whole cache lines.  Columns
  // beyond d are read from the last unit of the row instead and masked.
  int32_t col[UPL], col_read[UPL];
  bool col_ok[UPL];
#pragma unroll
  for (int i = 0; i < UPL; ++i) {
    col[i] = (gl + i * LPG) * F;
    col_ok[i] = col[i] < d;
    col_read[i] = col_ok[i] ? col[i] : d - F;
  }

  // Stage 2 for the chunk at `pos`: lane q of the group evaluates sample pos.t0 + q (in
  // several passes if the group has fewer than kChunk lanes).
  auto draw_ids = [&](const ChunkPos &pos, const Pre &pre, int32_t (&mine)[kPasses]) {
    const bool live = group_on && pos.idx < n;
    const bool any_live = __ballot(live) != 0;  // the same for the whole wavefront: a jump, not a mask
    const int64_t i = live ? pos.idx : 0;
    const int32_t id = w.source_id(i);
    bool is_pos[kChunk];
    pos.positives(per_round, is_pos);
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int32_t t = pos.t0 + p * LPG + gl;
      const bool want = live && p * LPG + gl < kChunk && t < a.samples;
      bool mine_pos = false;
#pragma unroll
      for (int q = 0; q < LPG && p * LPG + q < kChunk; ++q) mine_pos = (gl == q) ? is_pos[p * LPG + q] : mine_pos;
      // Past a wavefront's last chunk nobody wants the draw: only the arithmetic is skipped,
      // the reads of stage 2 stay unconditional.
      uint64_t r = 0;
      if (any_live) r = w.draw(i, id, want ? t : 0);
      mine[p] = w.stage2(i, id, want ? t : 0, want, mine_pos, pre, r);
    }
  };
  auto offsets_for = [&](const ChunkPos &pos) {
    const bool live = group_on && pos.idx < n;
    return w.stage1(live ? pos.idx : 0, live);
  };

  // Pipeline prologue: the ids of the group's first chunk and the offsets of its second.
  int32_t mine[kPasses];
  Pre pre_next;
  {
    const ChunkPos c0{first, 0, 0};
    draw_ids(c0, offsets_for(c0), mine);
    pre_next = offsets_for(c0.next(a.samples, per_round, stride));
  }

  // The loop bound is uniform over the wave.  A group without a source (past the end, or
  // tagging along in the sequential walk) goes through the motions on source 0 -- it reads,
  // computes and writes nothing -- so that no lane ever leaves the wavefront's control flow.
  for (int64_t base = first_of_wave; base < n; base += stride) {
    const int64_t idx_raw = first + (base - first_of_wave);
    const bool live = group_on && idx_raw < n;
    const int64_t idx = live ? idx_raw : 0;
    const int32_t src = w.source_id(idx);
    float *const src_row = w.source_row(idx);
    // The source row is requested here and first touched after the rows of the first chunk
    // have been requested too (`fresh`): nothing may read a unit before P::settle.
    U s[UPL], s_before[UPL];
#pragma unroll
    for (int i = 0; i < UPL; ++i) s[i] = P::load(src_row + col_read[i]);
    const uint32_t src_word = bits[use_bitmap ? (src >> 5) : 0];
    bool fresh = true;

    ChunkPos cur{idx_raw, 0, 0};
    for (int32_t t0 = 0; t0 < a.samples; t0 += kChunk) {
      bool is_pos[kChunk];
      cur.positives(per_round, is_pos);
      // The ids of this chunk were drawn one chunk ago; spread them over the group.
      int32_t v[kChunk];
#pragma unroll
      for (int p = 0; p < kPasses; ++p)
#pragma unroll
        for (int q = 0; q < LPG && p * LPG + q < kChunk; ++q) v[p * LPG + q] = __shfl(mine[p], q, LPG);

      // Request every row of the chunk (a missing sample reads the source row instead).
      U r[kChunk][UPL];
      uint32_t word[kChunk];
      bool valid[kChunk];
#pragma unroll
      for (int q = 0; q < kChunk; ++q) {
        valid[q] = live && v[q] >= 0 && v[q] != src;  // a sample that hits the source applies no update
        const float *row = valid[q] ? w.sample_row(idx, v[q]) : src_row;
#pragma unroll
        for (int i = 0; i < UPL; ++i) r[q][i] = P::load(row + col_read[i]);
        word[q] = bits[(use_bitmap && valid[q]) ? (v[q] >> 5) : 0];
      }
      // While they are in flight: the ids of the next chunk (its offsets arrived a chunk
      // ago) and the offsets of the chunk after it.
      const ChunkPos ahead1 = cur.next(a.samples, per_round, stride);
      draw_ids(ahead1, pre_next, mine);
      pre_next = offsets_for(ahead1.next(a.samples, per_round, stride));
      cur = ahead1;  // (its idx is this source's again unless this was the last chunk)

      // Everything this chunk needs has been asked for: from here on the rows may be used.
      P::wait_all();
#pragma unroll
      for (int i = 0; i < UPL; ++i) {
        P::settle(s[i]);
#pragma unroll
        for (int c = 0; c < F; ++c) {
          s[i].v[c] = col_ok[i] ? s[i].v[c] : 0.f;
          s_before[i].v[c] = fresh ? s[i].v[c] : s_before[i].v[c];
        }
      }
      fresh = false;
#pragma unroll
      for (int q = 0; q < kChunk; ++q)
#pragma unroll
        for (int i = 0; i < UPL; ++i) {
          P::settle(r[q][i]);
#pragma unroll
          for (int c = 0; c < F; ++c) r[q][i].v[c] = col_ok[i] ? r[q][i].v[c] : 0.f;
        }

#pragma unroll
      for (int q = 0; q < kChunk; ++q) {
        float partial = 0.f;
#pragma unroll
        for (int i = 0; i < UPL; ++i)
#pragma unroll
          for (int c = 0; c < F; ++c) partial = fmaf(s[i].v[c], r[q][i].v[c], partial);
        const float x = group_sum<LPG>(partial);
        const float label = is_pos[q] ? 1.f : 0.f;
        // a missing sample takes a zero step: both rows stay exactly as they are
        const float g = valid[q] ? a.lr * (label - 1.f / (1.f + expf(-x))) : 0.f;
#pragma unroll
        for (int i = 0; i < UPL; ++i)
#pragma unroll
          for (int c = 0; c < F; ++c) {
            s[i].v[c] = fmaf(g, r[q][i].v[c], s[i].v[c]);
            r[q][i].v[c] = fmaf(g, s[i].v[c], r[q][i].v[c]);
          }
        {
          float *const row = valid[q] ? w.sample_row(idx, v[q]) : src_row;
          const bool hot = valid[q] && (all_hot || ((word[q] >> (v[q] & 31)) & 1u));
          if (valid[q] && !hot) {  // uniform over the group; only writes inside
#pragma unroll
            for (int i = 0; i < UPL; ++i)
              if (col_ok[i]) P::store(row + col[i], r[q][i]);
          }
          if constexpr (P::kWaveAtomics) {
            static_assert(!P::kWaveAtomics || (UPL == 1 && F == 4), "one 128-bit unit per lane");
            U step;
#pragma unroll
            for (int c = 0; c < F; ++c) step.v[c] = g * s[0].v[c];
            add_rows_as_a_wave<LPG>(hot, row, step, d, lane);
          } else if (hot) {
#pragma unroll
            for (int i = 0; i < UPL; ++i)
#pragma unroll
              for (int c = 0; c < F; ++c)
                if (col_ok[i]) atomic_step(row + col[i] + c, g * s[i].v[c]);
          }
        }
        // A later sample of the same chunk that names the same vertex must see this
        // update: forward the registers instead of the stale prefetched copy.
#pragma unroll
        for (int z = q + 1; z < kChunk; ++z) {
          const bool same = valid[q] && v[z] == v[q];
#pragma unroll
          for (int i = 0; i < UPL; ++i)
#pragma unroll
            for (int c = 0; c < F; ++c) r[z][i].v[c] = same ? r[q][i].v[c] : r[z][i].v[c];
        }
      }
    }
    const bool src_hot = live && (all_hot || ((src_word >> (src & 31)) & 1u));
    if (live && !src_hot) {
#pragma unroll
      for (int i = 0; i < UPL; ++i)
        if (col_ok[i]) P::store(src_row + col[i], s[i]);
    }
    if constexpr (P::kWaveAtomics) {
      U step;
#pragma unroll
      for (int c = 0; c < F; ++c) step.v[c] = s[0].v[c] - s_before[0].v[c];
      add_rows_as_a_wave<LPG>(src_hot, src_row, step, d, lane);
    } else if (src_hot) {
#pragma unroll
      for (int i = 0; i < UPL; ++i)
#pragma unroll
        for (int c = 0; c < F; ++c)
          if (col_ok[i]) atomic_step(src_row + col[i] + c, s[i].v[c] - s_before[i].v[c]);
    }
  }
}

// Launches sgd_kernel for a given dimension.  Geometry:
//   plain_rows             plain 128-bit units, LPG = pow2ceil(d/4) lanes (<= 64): the layout
//                          of the sequential-order debug mode
//   otherwise, d <= 64     128-bit agent-scope units, LPG = pow2ceil(d/4) lanes, one unit per
//                          lane (4..64 sources per wavefront); hot rows are added to by the
//                          whole wavefront, one row at a time
//   otherwise, d  > 64     32-bit agent-scope units interleaved over LPG = pow2ceil(d/4)
//                          lanes (<= 64), four or eight units per lane
// Each of them runs concurrently (seq = false) or as one lane group (seq = true).
// `a.sources_per_block` is filled in here from `count`.
template <class W>
struct SgdLauncher {
  template <class P, int LPG, int UPL>
  static void run(const W &w, SgdArgs a, int64_t count, bool seq, int64_t max_waves, hipStream_t st) {
    constexpr int kWavesPerBlock = 4;
    constexpr int kGroupsPerWave = 64 / LPG;
    constexpr int64_t kPerTurn = kWavesPerBlock * kGroupsPerWave;  // sources a workgroup takes per turn
    const int64_t turns = std::max<int64_t>((count + kPerTurn - 1) / kPerTurn, 1);
    const int64_t max_blocks = std::max<int64_t>(max_waves / kWavesPerBlock, 1);
    const int64_t per_block = (turns + max_blocks - 1) / max_blocks;  // turns of one workgroup
    const int64_t blocks64 = (turns + per_block - 1) / per_block;
    a.sources_per_block = per_block * kPerTurn;
    if (seq) {
      hipLaunchKernelGGL((sgd_kernel<P, LPG, UPL, W, true>), dim3(1), dim3(64), 0, st, w, a);
    } else {
      const int blocks = static_cast<int>(blocks64);
      hipLaunchKernelGGL((sgd_kernel<P, LPG, UPL, W, false>), dim3(blocks), dim3(256), 0, st, w, a);
    }
  }

  static int pow2_lanes(int units) {
    int lanes = 1;
    while (lanes < units && lanes < 64) lanes *= 2;
    return lanes;
  }

  // Lane groups per wavefront in concurrent mode (to size the launch and the hot-row rule).
  static int groups_per_wave(int32_t d) { return 64 / pow2_lanes(d / 4); }

  static void launch(const W &w, const SgdArgs &a, int64_t count, bool seq, bool plain_rows,
                     int64_t max_waves, hipStream_t st) {
    const int d = a.d;
    if (plain_rows) {
      if (d > 256) return run<RowPlain128, 64, 2>(w, a, count, seq, max_waves, st);
      switch (pow2_lanes(d / 4)) {
        case 64: return run<RowPlain128, 64, 1>(w, a, count, seq, max_waves, st);
        case 32: return run<RowPlain128, 32, 1>(w, a, count, seq, max_waves, st);
        case 16: return run<RowPlain128, 16, 1>(w, a, count, seq, max_waves, st);
        case 8: return run<RowPlain128, 8, 1>(w, a, count, seq, max_waves, st);
        case 4: return run<RowPlain128, 4, 1>(w, a, count, seq, max_waves, st);
        case 2: return run<RowPlain128, 2, 1>(w, a, count, seq, max_waves, st);
        default: return run<RowPlain128, 1, 1>(w, a, count, seq, max_waves, st);
      }
    }
    if (d <= 64) {
      switch (pow2_lanes(d / 4)) {
        case 16: return run<RowAgent128, 16, 1>(w, a, count, seq, max_waves, st);
        case 8: return run<RowAgent128, 8, 1>(w, a, count, seq, max_waves, st);
        case 4: return run<RowAgent128, 4, 1>(w, a, count, seq, max_waves, st);
        case 2: return run<RowAgent128, 2, 1>(w, a, count, seq, max_waves, st);
        default: return run<RowAgent128, 1, 1>(w, a, count, seq, max_waves, st);
      }
    }
    if (d > 256) return run<RowAgent32, 64, 8>(w, a, count, seq, max_waves, st);
    if (d > 128) return run<RowAgent32, 64, 4>(w, a, count, seq, max_waves, st);
    return run<RowAgent32, 32, 4>(w, a, count, seq, max_waves, st);
  }
};

}  // namespace gosh

// GOSH oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
//
// A plain, slow, single-threaded CPU statement of what the GOSH training path
// computes, written from the paper (Akyildiz, Aljundi, Kaya: "GOSH: Embedding Big
// Graphs on Small Hardware", ICPP'20).  Only the tests, the smoke check and the
// benchmark's CPU-baseline leg may load this library.  It shares no code, header,
// table or helper with the HIP library; the counter-based generator below is
// implemented a second time there, independently.
//
// Conventions (readings of places where the paper is silent are marked READING):
//   * graph: CSR, xadj = n+1 int64 offsets, adj = int32 neighbour ids (Sec. 3.2.1,
//     "Complexity analysis" paragraph).
//   * embedding matrix M: n x d, row-major fp32 storage.  All arithmetic of one
//     update is done in fp64 on the fp32-stored rows and rounded once on store.
//   * random draws: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) keyed by the
//     seed, counter (src, j, epoch, level); READING -- the paper only says that
//     samples are drawn on the device (Sec. 3.1).
//
// Pin status (tests/test_oracle_*.py):
//   philox            pinned against an independent implementation (ATen's engine)
//   bounded index     pinned (brute force 128-bit product, edge values)
//   update            pinned (hand-worked values, finite-difference gradient)
//   sampling          pinned (membership, chi-square uniformity, degenerate cases)
//   epoch / schedule  pinned (closed form; an epoch and the e_i-epoch loop replayed as
//                     single updates over the recorded streams, with hand-typed rates)
//   initial matrix    pinned (entries worked out from an independent Philox's words)
//   coarsening        pinned (worked examples, invariants, dense brute force)
//   projection/split  pinned (closed form)
//   pair order/parts  pinned (closed form, coverage invariants; a pair visit and the
//                     rotation loop replayed from draws, candidate lists and single
//                     updates; chi-square of the in-part positive); the host/device
//                     overlap of the parts driver has no numeric oracle:
//                     "parity unpinned" for scheduling, pinned for results.
//   level loop        (gosh_oracle.py: embed, embed_budget, parts_split) pinned (a
//                     three-level toy composed by hand, budgets worked out by hand)
//   hogwild slice     the one multi-threaded function (orc_train_sources_hogwild): the
//                     sequential loop under a parallel-for, for timing the paper's
//                     multi-core CPU baseline; no expected value is ever taken from it
//                     (pinned only at threads = 1, where it is the sequential slice).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <map>
#include <utility>
#include <vector>

extern "C" {

// ---------------------------------------------------------------------------
// Philox4x32-10.  One round maps (c0,c1,c2,c3) with round key (k0,k1) to
//   (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
// and the key is advanced by the Weyl constants between rounds.
// ---------------------------------------------------------------------------
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t mul0 = 0xD2511F53u, mul1 = 0xCD9E8D57u;
  const uint32_t weyl0 = 0x9E3779B9u, weyl1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += weyl0;
      k1 += weyl1;
    }
    uint64_t p0 = mul0 * (uint64_t)c0;
    uint64_t p1 = mul1 * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// READING (RNG keying): draw j of source src in a given epoch and level is the low
// 64 bits of Philox(counter = (src, j, epoch, level), key = (seed_lo, seed_hi)).
uint64_t orc_draw(uint64_t seed, uint32_t src, uint32_t j, uint32_t epoch, uint32_t level) {
  uint32_t ctr[4] = {src, j, epoch, level};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t out[4];
  orc_philox4x32_10(ctr, key, out);
  return (uint64_t)out[0] | ((uint64_t)out[1] << 32);
}

// READING (index mapping): a 64-bit draw r becomes an index in [0, bound) as
// floor(r * bound / 2^64) -- multiply-high, no rejection.
uint64_t orc_bounded(uint64_t r, uint64_t bound) {
  return (uint64_t)(((unsigned __int128)r * (unsigned __int128)bound) >> 64);
}

// ---------------------------------------------------------------------------
// Samples of one source (Alg. 3 "TrainInGPU": one positive, then n_s negatives).
//   out[0]    = positive: uniform member of Gamma(src) (adjacency similarity,
//               Sec. 2 / Sec. 3.1); -1 if src has no neighbour (READING).
//   out[1..k] = negatives: uniform over V_i, no rejection (Sec. 3.1).
// ---------------------------------------------------------------------------
void orc_sample_source(int64_t n, const int64_t *xadj, const int32_t *adj, int32_t k,
                       uint64_t seed, uint32_t epoch, uint32_t level, int64_t src,
                       int32_t *out) {
  int64_t begin = xadj[src], deg = xadj[src + 1] - begin;
  uint64_t r0 = orc_draw(seed, (uint32_t)src, 0, epoch, level);
  out[0] = deg > 0 ? adj[begin + (int64_t)orc_bounded(r0, (uint64_t)deg)] : -1;
  for (int32_t j = 1; j <= k; ++j) {
    uint64_t r = orc_draw(seed, (uint32_t)src, (uint32_t)j, epoch, level);
    out[j] = (int32_t)orc_bounded(r, (uint64_t)n);
  }
}

void orc_sample_epoch(int64_t n, const int64_t *xadj, const int32_t *adj, int32_t k,
                      uint64_t seed, uint32_t epoch, uint32_t level, int32_t *out) {
  for (int64_t src = 0; src < n; ++src)
    orc_sample_source(n, xadj, adj, k, seed, epoch, level, src, out + src * (k + 1));
}

// ---------------------------------------------------------------------------
// Alg. 1 "UpdateEmbedding".  READING: the garbled first line is
//   score = (b - sigmoid(M[v] . M[sample])) * lr
// (the prose of Sec. 2 calls lr the learning rate of the classifier), and the
// three lines run in the printed order, so the sample row is updated with the
// already-updated source row.  b = 1 for a positive, 0 for a negative (Alg. 3).
// ---------------------------------------------------------------------------
void orc_update(float *m_v, float *m_sample, int32_t d, int32_t b, float lr) {
  double dot = 0.0;
  for (int32_t c = 0; c < d; ++c) dot += (double)m_v[c] * (double)m_sample[c];
  double sigma = 1.0 / (1.0 + std::exp(-dot));
  double score = ((double)b - sigma) * (double)lr;
  for (int32_t c = 0; c < d; ++c)
    m_v[c] = (float)((double)m_v[c] + (double)m_sample[c] * score);
  for (int32_t c = 0; c < d; ++c)
    m_sample[c] = (float)((double)m_sample[c] + (double)m_v[c] * score);
}

// Learning rate of epoch j out of e_i at one level (Sec. 3, Alg. 3 first line of the
// loop): lr * max(1 - j/e_i, 1e-4), evaluated in fp64 and rounded once to fp32.
float orc_lr(float lr0, int64_t j, int64_t e_i) {
  double f = 1.0 - (double)j / (double)e_i;
  if (f < 1e-4) f = 1e-4;
  return (float)((double)lr0 * f);
}

// ---------------------------------------------------------------------------
// One epoch of Alg. 3 in sequential order: sources in ascending id; for each, the
// positive update and then the n_s negative updates, applied directly to M.
// READING (degenerate samples): no positive update for an isolated source; a
// negative equal to the source itself is drawn but applies no update; negatives
// that happen to be neighbours, or repeat, are applied like any other.
// ---------------------------------------------------------------------------
// Sources first .. first+count-1 of one epoch (a contiguous slice of the sequential
// order; the whole epoch is the slice [0, n)).
void orc_train_sources(int64_t n, const int64_t *xadj, const int32_t *adj, float *M,
                       int32_t d, int32_t k, float lr_epoch, uint64_t seed, uint32_t epoch,
                       uint32_t level, int64_t first, int64_t count) {
  std::vector<int32_t> smp((size_t)k + 1);
  for (int64_t src = first; src < first + count && src < n; ++src) {
    orc_sample_source(n, xadj, adj, k, seed, epoch, level, src, smp.data());
    for (int32_t j = 0; j <= k; ++j) {
      int64_t v = smp[j];
      if (v < 0 || v == src) continue;
      orc_update(M + src * d, M + v * d, d, j == 0 ? 1 : 0, lr_epoch);
    }
  }
}

// The same slice with the sources spread over `threads` OpenMP threads, lock-free
// (Hogwild), as the paper's multi-core CPU baseline does (Sec. 4.8, the 16-thread CPU
// runs).  Rows are updated concurrently without synchronisation, so the result depends on
// the interleaving: this function is for TIMING a CPU baseline and for quality checks,
// never an expected value.  With threads = 1 it is orc_train_sources.
void orc_train_sources_hogwild(int64_t n, const int64_t *xadj, const int32_t *adj, float *M,
                               int32_t d, int32_t k, float lr_epoch, uint64_t seed,
                               uint32_t epoch, uint32_t level, int64_t first, int64_t count,
                               int32_t threads) {
  const int64_t last = first + count < n ? first + count : n;
#pragma omp parallel num_threads(threads)
  {
    std::vector<int32_t> smp((size_t)k + 1);
#pragma omp for schedule(static)
    for (int64_t src = first; src < last; ++src) {
      orc_sample_source(n, xadj, adj, k, seed, epoch, level, src, smp.data());
      for (int32_t j = 0; j <= k; ++j) {
        int64_t v = smp[j];
        if (v < 0 || v == src) continue;
        orc_update(M + src * d, M + v * d, d, j == 0 ? 1 : 0, lr_epoch);
      }
    }
  }
}

void orc_train_epoch(int64_t n, const int64_t *xadj, const int32_t *adj, float *M,
                     int32_t d, int32_t k, float lr_epoch, uint64_t seed, uint32_t epoch,
                     uint32_t level) {
  orc_train_sources(n, xadj, adj, M, d, k, lr_epoch, seed, epoch, level, 0, n);
}

// e_i epochs at one level with the decaying learning rate (Alg. 3 outer loop).
void orc_train_level(int64_t n, const int64_t *xadj, const int32_t *adj, float *M,
                     int32_t d, int32_t k, float lr0, int64_t e_i, uint64_t seed,
                     uint32_t level) {
  for (int64_t j = 0; j < e_i; ++j)
    orc_train_epoch(n, xadj, adj, M, d, k, orc_lr(lr0, j, e_i), seed, (uint32_t)j, level);
}

// READING (initialisation; Alg. 2 only says "randomly initialize"): entries are
// uniform in [-0.5/d, 0.5/d).  Entry (v, c) uses word c%4 of
// Philox(counter = (v, c/4, 0xFFFFFFFF, level)); word w maps to
// ((w >> 8) * 2^-24 - 0.5) / d evaluated in fp64 and rounded to fp32.
// Rows first .. first+count-1 of the initial matrix, written to out (count x d).
void orc_init_rows(float *out, int64_t first, int64_t count, int32_t d, uint64_t seed,
                   uint32_t level) {
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  for (int64_t r = 0; r < count; ++r)
    for (int32_t c = 0; c < d; ++c) {
      uint32_t ctr[4] = {(uint32_t)(first + r), (uint32_t)(c / 4), 0xFFFFFFFFu, level};
      uint32_t out4[4];
      orc_philox4x32_10(ctr, key, out4);
      double u = (double)(out4[c % 4] >> 8) * (1.0 / 16777216.0);
      out[r * d + c] = (float)((u - 0.5) / (double)d);
    }
}

void orc_init_embedding(float *M, int64_t n, int32_t d, uint64_t seed, uint32_t level) {
  orc_init_rows(M, 0, n, d, seed, level);
}

// ---------------------------------------------------------------------------
// Projection between levels (Sec. 3: the row of a vertex of G_{i-1} is the row of
// its super vertex in G_i): M_fine[v] = M_coarse[map[v]].
// ---------------------------------------------------------------------------
void orc_project(const float *M_coarse, const int32_t *map, int64_t n_fine, int32_t d,
                 float *M_fine) {
  for (int64_t v = 0; v < n_fine; ++v)
    for (int32_t c = 0; c < d; ++c) M_fine[v * d + c] = M_coarse[(int64_t)map[v] * d + c];
}

// Epoch budget per level (Sec. 3): a share p of e spread evenly over the D levels,
// the rest geometrically, each level getting half of the next coarser one.
// READING: exact_i = p*e/D + (1-p)*e*2^i/(2^D-1); levels i >= 1 get
// max(1, floor(exact_i)) and level 0 gets what is left, so the sum is exactly e.
// Returns 0, or -1 if e cannot give every level at least one epoch.
int orc_epoch_split(int64_t e, double p, int32_t D, int64_t *e_i) {
  if (D < 1 || D > 62 || e < D || p < 0.0 || p > 1.0) return -1;
  double geo_total = (double)(((uint64_t)1 << D) - 1);
  int64_t used = 0;
  for (int32_t i = D - 1; i >= 1; --i) {
    double exact = p * (double)e / (double)D +
                   (1.0 - p) * (double)e * (double)((uint64_t)1 << i) / geo_total;
    int64_t v = (int64_t)std::floor(exact);
    if (v < 1) v = 1;
    e_i[i] = v;
    used += v;
  }
  e_i[0] = e - used;
  return e_i[0] >= 1 ? 0 : -1;
}

// ---------------------------------------------------------------------------
// Alg. 4 "MultiEdgeCollapse", one level, sequential, as printed.
//   order : vertices by degree, larger first (Sec. 3.2); READING: ties by
//           ascending id.
//   delta : |E_i|/|V_i|; READING: |E_i| is the number of CSR entries, so delta is
//           the mean degree; the test deg <= delta is done as deg*n <= nnz.
// Returns the number of clusters = |V_{i+1}|.
// ---------------------------------------------------------------------------
int64_t orc_coarsen_map(int64_t n, const int64_t *xadj, const int32_t *adj, int32_t *map) {
  int64_t nnz = xadj[n];
  std::vector<int64_t> order((size_t)n);
  for (int64_t v = 0; v < n; ++v) order[(size_t)v] = v;
  std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) {
    return (xadj[a + 1] - xadj[a]) > (xadj[b + 1] - xadj[b]);
  });
  for (int64_t v = 0; v < n; ++v) map[v] = -1;
  auto small = [&](int64_t v) { return (xadj[v + 1] - xadj[v]) * n <= nnz; };
  int32_t cluster = 0;
  for (int64_t t = 0; t < n; ++t) {
    int64_t v = order[(size_t)t];
    if (map[v] != -1) continue;
    map[v] = cluster++;
    for (int64_t p = xadj[v]; p < xadj[v + 1]; ++p) {
      int64_t u = adj[p];
      if ((small(v) || small(u)) && map[u] == -1) map[u] = map[v];
    }
  }
  return cluster;
}

// "Coarsen(G_i, map_i)".  READING (the paper gives only its complexity): G_{i+1} has
// the entry (a, b) iff some entry (x, y) of G_i has map[x] = a, map[y] = b, a != b;
// self loops vanish, parallel entries merge, rows come out ascending.  mult_out
// carries how many fine entries (weighted by mult_in, or 1 each when mult_in is
// null) merged into each coarse entry.  Call with adj_out == nullptr to get the
// size first.  Returns nnz of G_{i+1}.
int64_t orc_coarsen_graph(int64_t n, const int64_t *xadj, const int32_t *adj,
                          const int64_t *mult_in, const int32_t *map, int64_t n_coarse,
                          int64_t *xadj_out, int32_t *adj_out, int64_t *mult_out) {
  std::map<std::pair<int32_t, int32_t>, int64_t> entries;
  for (int64_t x = 0; x < n; ++x)
    for (int64_t p = xadj[x]; p < xadj[x + 1]; ++p) {
      int32_t a = map[x], b = map[adj[p]];
      if (a != b) entries[{a, b}] += mult_in ? mult_in[p] : 1;
    }
  if (adj_out) {
    for (int64_t a = 0; a <= n_coarse; ++a) xadj_out[a] = 0;
    int64_t pos = 0;
    for (auto &kv : entries) {
      xadj_out[kv.first.first + 1] += 1;
      adj_out[pos] = kv.first.second;
      if (mult_out) mult_out[pos] = kv.second;
      ++pos;
    }
    for (int64_t a = 0; a < n_coarse; ++a) xadj_out[a + 1] += xadj_out[a];
  }
  return (int64_t)entries.size();
}

// ---------------------------------------------------------------------------
// Large-graph rotation (Sec. 3.3, Alg. 5).
// ---------------------------------------------------------------------------

// The order in which part pairs are visited in one rotation ("inside-out"):
// (0,0), (1,0), (1,1), (2,0), ... ; K(K+1)/2 pairs.  Returns the pair count.
int64_t orc_pair_order(int32_t K, int32_t *a, int32_t *b) {
  int64_t cnt = 0;
  int32_t ca = 0, cb = 0;
  while (ca < K) {
    a[cnt] = ca;
    b[cnt] = cb;
    ++cnt;
    if (ca > cb) {
      cb += 1;
    } else {
      ca += 1;
      cb = 0;
    }
  }
  return cnt;
}

// A second visiting order, NOT the paper's: "blocked".  The parts are cut into blocks of R
// consecutive parts; for every block in turn, first the pairs inside the block in the
// order above, then for each later part c the pairs (c, r) for every r of the block.  A
// device that keeps one block resident and streams the later parts through meets R pairs
// per part it loads, where the order above meets one.  Every pair (a, b), a >= b, still
// occurs exactly once per rotation, and with R >= K the order is the one above.
int64_t orc_pair_order_blocked(int32_t K, int32_t R, int32_t *a, int32_t *b) {
  int64_t cnt = 0;
  for (int32_t first = 0; first < K; first += R) {
    int32_t end = first + R < K ? first + R : K;
    for (int32_t m = first; m < end; ++m)
      for (int32_t s = first; s <= m; ++s) {
        a[cnt] = m;
        b[cnt] = s;
        ++cnt;
      }
    for (int32_t c = end; c < K; ++c)
      for (int32_t r = first; r < end; ++r) {
        a[cnt] = c;
        b[cnt] = r;
        ++cnt;
      }
  }
  return cnt;
}

// READING (partition): parts are contiguous id ranges of ceil(n/K) vertices.
static inline int64_t part_size(int64_t n, int32_t K) { return (n + K - 1) / K; }

// Draw counter for the parts mode.  READING: the fourth counter word carries the
// level in its low 8 bits and (pair index + 1) above it; the third word is the
// rotation; the second is side * B*(1+n_s) + round * (1+n_s) + j where side tells
// which part of the pair owns the source.
static inline uint64_t parts_draw(uint64_t seed, uint32_t src, uint32_t slot, uint32_t rotation,
                                  uint32_t level, uint32_t pair) {
  return orc_draw(seed, src, slot, rotation, (level & 0xFFu) | ((pair + 1u) << 8));
}

// Positive sample of v restricted to the partner part [lo, hi): uniform member of
// Gamma(v) inside the range, -1 if none (Sec. 3.3: such a vertex gets no positive
// update for this pair).
static int32_t positive_in_range(const int64_t *xadj, const int32_t *adj, int64_t v,
                                 int64_t lo, int64_t hi, uint64_t r) {
  std::vector<int32_t> cand;
  for (int64_t p = xadj[v]; p < xadj[v + 1]; ++p)
    if (adj[p] >= lo && adj[p] < hi) cand.push_back(adj[p]);
  if (cand.empty()) return -1;
  return cand[(size_t)orc_bounded(r, (uint64_t)cand.size())];
}

// One visit of the pair (pa, pb): every vertex of part pa takes B rounds of one
// positive from Gamma(v) in part pb plus n_s negatives uniform in part pb; then, if
// pa != pb, the same with the roles swapped (Sec. 3.3).  Sequential order: side 0
// sources ascending, then side 1 sources ascending; per source rounds in order.
// If stream_out is given it receives, per source of each side, B*(1+n_s) sample ids
// (side 0 block first, then side 1 block).
void orc_train_pair(int64_t n, const int64_t *xadj, const int32_t *adj, float *M, int32_t d,
                    int32_t k, int32_t B, int32_t K, int32_t pa, int32_t pb, float lr,
                    uint64_t seed, uint32_t rotation, uint32_t level, uint32_t pair_index,
                    int32_t *stream_out) {
  int64_t ps = part_size(n, K);
  int32_t per_src = B * (k + 1);
  int64_t written = 0;
  for (int side = 0; side < (pa == pb ? 1 : 2); ++side) {
    int32_t own = side == 0 ? pa : pb, other = side == 0 ? pb : pa;
    int64_t lo = std::min<int64_t>(n, own * ps), hi = std::min<int64_t>(n, lo + ps);
    int64_t olo = std::min<int64_t>(n, other * ps), ohi = std::min<int64_t>(n, olo + ps);
    for (int64_t src = lo; src < hi; ++src)
      for (int32_t round = 0; round < B; ++round)
        for (int32_t j = 0; j <= k; ++j) {
          uint32_t slot = (uint32_t)(side * per_src + round * (k + 1) + j);
          uint64_t r = parts_draw(seed, (uint32_t)src, slot, rotation, level, pair_index);
          int64_t v;
          if (j == 0)
            v = positive_in_range(xadj, adj, src, olo, ohi, r);
          else
            v = ohi > olo ? olo + (int64_t)orc_bounded(r, (uint64_t)(ohi - olo)) : -1;
          if (stream_out) stream_out[written++] = (int32_t)v;
          if (v < 0 || v == src) continue;
          orc_update(M + src * d, M + v * d, d, j == 0 ? 1 : 0, lr);
        }
  }
}

// Number of rotations equivalent to e_i epochs (Alg. 5 first line):
// READING: ceil(e_i / (B*K)), at least 1.
int64_t orc_rotations(int64_t e_i, int32_t B, int32_t K) {
  int64_t per = (int64_t)B * K;
  int64_t r = (e_i + per - 1) / per;
  return r < 1 ? 1 : r;
}

// Alg. 5 executed sequentially on host memory with no device budget.
// READING: the learning rate decays per rotation with the epoch formula.
// block = 0: the paper's order; block = R > 0: the blocked order with blocks of R parts.
void orc_train_parts(int64_t n, const int64_t *xadj, const int32_t *adj, float *M, int32_t d,
                     int32_t k, int64_t e_i, float lr0, uint64_t seed, uint32_t level, int32_t K,
                     int32_t B, int32_t block) {
  int64_t rotations = orc_rotations(e_i, B, K);
  int64_t npairs = (int64_t)K * (K + 1) / 2;
  std::vector<int32_t> a((size_t)npairs), b((size_t)npairs);
  if (block > 0) orc_pair_order_blocked(K, block, a.data(), b.data());
  else orc_pair_order(K, a.data(), b.data());
  for (int64_t r = 0; r < rotations; ++r) {
    float lr = orc_lr(lr0, r, rotations);
    for (int64_t q = 0; q < npairs; ++q)
      orc_train_pair(n, xadj, adj, M, d, k, B, K, a[(size_t)q], b[(size_t)q], lr, seed,
                     (uint32_t)r, level, (uint32_t)q, nullptr);
  }
}

}  // extern "C"

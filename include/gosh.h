/* libgosh -- MI355X (gfx950) implementation of the GOSH graph-embedding training
 * path (Akyildiz, Aljundi, Kaya, "GOSH: Embedding Big Graphs on Small Hardware",
 * ICPP'20).  Plain C ABI: raw pointers and sizes only.
 *
 * Conventions
 *   - "device" pointers are HIP device memory of the current device; "host" pointers
 *     are ordinary host memory.  The library never frees or keeps caller arrays.
 *   - Graphs are CSR (Sec. 3.2.1 of the paper): adj holds the neighbour lists back to
 *     back, xadj holds n+1 offsets into it, xadj[n] == nnz.  Rows must be sorted
 *     ascending, without duplicates or self loops (gosh_csr_validate checks a host
 *     copy).  The training entry points do not verify this, but no array content can
 *     take their kernels outside the operands: a row whose offsets leave adj counts
 *     as empty, an entry that names no vertex (or, in the part-pair rotation, no vertex
 *     of the partner part) is no sample.  What such a graph trains is unspecified.
 *   - The embedding matrix M is n x d, row-major fp32, 16-byte aligned, d a multiple
 *     of 4 with 4 <= d <= 512.
 *   - Every function returns GOSH_OK (0) or a negative gosh_status; the message of the
 *     last failure on the calling thread is returned by gosh_last_error().  No
 *     exception crosses this boundary.
 *   - Device entry points are asynchronous: they enqueue work on the given HIP
 *     stream (a hipStream_t passed as void*, NULL = the default stream) and return.
 *     Faults inside a kernel surface at the caller's next synchronisation.
 */
#ifndef GOSH_H
#define GOSH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GOSH_OK = 0,
  GOSH_EINVAL = -1,  /* an argument violates a documented precondition */
  GOSH_ENOMEM = -2,  /* host or device allocation failed */
  GOSH_EHIP = -3,    /* a HIP runtime call failed */
  GOSH_EBUDGET = -4, /* device budget too small for the requested part layout */
  GOSH_EDIVERGED = -5 /* training finished, but the matrix it leaves holds non-finite values
                         (nothing in Alg. 1 bounds a row; a learning rate too large for the
                         graph's hubs makes rows grow until fp32 overflows) */
} gosh_status;

/* Borrowed view of a CSR graph.  All three arrays live on the same side (host or
 * device) as the entry point documents. */
typedef struct {
  int64_t n;          /* |V| : 1 <= n < 2^31 - 1 */
  int64_t nnz;        /* length of adj (= 2|E| for a symmetrised graph) */
  const void *xadj;   /* n+1 offsets; int32_t* if xadj_is64 == 0, else int64_t* */
  const int32_t *adj; /* neighbour ids */
  int32_t xadj_is64;
} gosh_csr;

#define GOSH_MAX_DIM 512
#define GOSH_MAX_NEG 15

/* gosh_train_epoch flags */
#define GOSH_FLAG_SEQUENTIAL 1u   /* debug: one wavefront walks the sources in ascending
                                     id, giving the sequential-order result */
#define GOSH_FLAG_PLAIN_STORES 2u /* concurrent mode: write every updated row back with
                                     plain stores (the paper's lock-free scheme as it
                                     stands: concurrent updates of one row can be lost) */
#define GOSH_FLAG_ATOMIC_ADDS 4u  /* concurrent mode: apply every update as atomic adds of
                                     the step (no update is ever lost; about 2x the cost) */

#define GOSH_FLAG_CONCURRENT_LAYOUT 64u /* debug, with GOSH_FLAG_SEQUENTIAL: the one lane group
                                     that walks the sources runs the concurrent kernel as it
                                     is shipped -- its lane-to-column layout, its device-scope
                                     row accesses, its hot-row rule with the atomic-add and the
                                     plain-store write paths -- instead of the plain 128-bit
                                     layout, so that exactly that code can be compared with a
                                     sequential reference.  No effect without
                                     GOSH_FLAG_SEQUENTIAL */

/* gosh_embed / gosh_embed_host only */
#define GOSH_FLAG_EDGE_EPOCHS 8u  /* an epoch is |E_i| sampled sources, the definition of the
                                     paper's experiments (Sec. 4.3), not the |V_i| of Alg. 3:
                                     level i runs e_i * ceil(|E_i| / |V_i|) passes of Alg. 3,
                                     |E_i| = nnz_i / 2, and the learning rate decays over all
                                     of them */

#define GOSH_FLAG_PAIR_LEVELS 32u /* a level that fits the device is trained in place with the
                                     pair scheme of Alg. 5 instead of Alg. 3 -- gosh_train_parts
                                     on the device matrix, B = 5 -- on the largest K of 16, 8,
                                     4, 2, 1 whose parts keep 2^22 vertices (pair_level_min_n of
                                     gosh_set_tuning) and whose whole
                                     rotations overshoot the level's epochs by at most an
                                     eighth; a level for which no K does keeps Alg. 3.  Not the
                                     paper's choice: see gosh_train_parts for what it buys */

/* gosh_train_parts / gosh_embed_host only */
#define GOSH_FLAG_BLOCKED_ORDER 16u /* visit the part pairs in the blocked order of
                                       gosh_pair_order_blocked (block = P_gpu - 2 parts, at
                                       least 1) instead of the paper's: the same pairs once
                                       per rotation, fewer parts over the host link */

const char *gosh_last_error(void);

/* ---- tuning record ------------------------------------------------------------------ */

/* Constants of this implementation that the paper does not have (Sec. 3.1 accepts lost
 * updates and only notes that too many of them hurt): how the training kernels are launched
 * and which rows count as "hot" (updated with atomic adds instead of plain stores, see
 * gosh_train_epoch).  One record per process, read at the start of every training call;
 * the library never reads the environment.  Meant for experiments and tests. */
typedef struct {
  int32_t plain_rows;        /* non-zero: plain 128-bit row accesses also in the concurrent
                                kernels (coherent inside one XCD only).  Default 0 */
  int64_t max_waves;         /* cap on the wavefronts that share the sources of one launch
                                (each then walks several sources, sampling ahead).
                                Default 2^18 */
  int64_t hot_inv_eps;       /* a vertex is hot if deg * C / nnz > 1 / hot_inv_eps, C = sources
                                in flight.  Default 64 */
  int64_t hot_all_inv_eps;   /* every row is hot if (k_neg + 1) * C / n > 1 / hot_all_inv_eps;
                                0 switches that rule off.  Default 4 */
  int64_t hot_min_degree;    /* > 0: skip both rules; a vertex is hot iff its degree is at
                                least this.  Default 0 */
  int64_t pair_level_min_n;  /* GOSH_FLAG_PAIR_LEVELS: smallest part, in vertices.
                                Default 2^22 */
} gosh_tuning;

void gosh_tuning_defaults(gosh_tuning *t);
/* NULL restores the defaults.  GOSH_EINVAL for a value outside its range (max_waves,
 * hot_inv_eps, pair_level_min_n >= 1; the others >= 0); the record is unchanged then. */
int gosh_set_tuning(const gosh_tuning *t);
int gosh_get_tuning(gosh_tuning *t);

/* ---- schedule helpers (host, pure) ------------------------------------------------ */

/* Learning rate of epoch j (0-based) out of e_i at one level: lr0 * max(1 - j/e_i, 1e-4)
 * (Sec. 3, last paragraph before Alg. 2; Alg. 3 first line of the epoch loop).
 * Evaluated in double, rounded once.  Returns 0 if e_i <= 0. */
float gosh_lr(float lr0, int64_t j, int64_t e_i);

/* Epoch budget per level ("calculateEpochs", Sec. 3 paragraph on the smoothing ratio
 * p): a share p of e evenly over the D levels, the rest geometrically with each level
 * getting half of the next coarser one.  exact_i = p*e/D + (1-p)*e*2^i/(2^D-1); levels
 * i >= 1 get max(1, floor(exact_i)), level 0 the remainder, so sum(e_i) == e.
 * e_i: host array of D entries (written).  GOSH_EINVAL if D < 1, D > 62, p outside
 * [0,1] or e cannot give every level one epoch. */
int gosh_epoch_split(int64_t e, double p, int32_t D, int64_t *e_i);

/* The rule of GOSH_FLAG_PAIR_LEVELS (host, pure; not the paper's): parts for training a
 * resident level of n vertices for `epochs` epochs with the pair scheme in place -- the
 * largest K of 16, 8, 4, 2, 1 with K * min_n <= n whose whole rotations of B rounds overshoot
 * the epochs by at most an eighth (ceil(epochs / (B*K)) * B*K - epochs <= epochs / 8); 0 =
 * "train the level with Alg. 3". */
int32_t gosh_pair_level_parts(int64_t epochs, int64_t n, int64_t min_n, int32_t B);

/* ---- coarsening (host) -------------------------------------------------------------- */

/* Checks a host CSR graph against the conventions above (offsets start at 0, end at
 * nnz and never decrease; neighbour ids in range; rows strictly ascending; no self
 * loops).  GOSH_OK or GOSH_EINVAL with the first violation in gosh_last_error(). */
int gosh_csr_validate(const gosh_csr *g_host);

/* The set of coarsened graphs and the maps between them ("MultiEdgeCollapse", Alg. 4,
 * Sec. 3.2).  Opaque; owned by the library, released with gosh_hierarchy_free. */
typedef struct gosh_hierarchy gosh_hierarchy;

/* Alg. 4, sequential semantics.  Per level: vertices are visited by degree, largest
 * first (ties: smaller id first); an unmarked vertex v opens cluster number
 * (clusters so far) and takes every unmarked neighbour u, in neighbour-list order,
 * for which deg(v) <= delta or deg(u) <= delta, delta = nnz/n (tested as deg*n <= nnz).
 * G_{i+1} has the entry (a, b), a != b, iff some entry (x, y) of G_i has map[x] = a,
 * map[y] = b; rows ascending, parallel entries merged.
 * Levels are built while |V_i| > threshold (the paper's default is 100); building stops
 * after a level with |V_{i+1}| > min_shrink*|V_i| (that level is kept), at a level that
 * merged nothing (|V_{i+1}| == |V_i|: it would repeat G_i and is dropped), or when
 * max_levels graphs exist.  min_shrink in (0, 1]; 1.0 keeps only the no-progress guard.
 * n_threads <= 0 uses every available core (the result does not depend on the thread
 * count).
 * g0_host: host CSR, borrowed for the lifetime of the hierarchy (level 0 is a view of
 * it, not a copy).  *out receives the hierarchy; on failure it is NULL. */
int gosh_coarsen(const gosh_csr *g0_host, int64_t threshold, double min_shrink,
                 int32_t max_levels, int32_t n_threads, gosh_hierarchy **out);

/* MultiEdgeCollapse on the current HIP device: the same hierarchy, bit for bit (Alg. 4 has
 * one result), with the degree order a device radix sort, the marking sweep resolved in
 * parallel rounds, and "Coarsen" (the rebuild of the CSR of G_{i+1}, Sec. 3.2.1) a sort
 * and a reduction of (cluster, cluster) keys.  g0 may be a host graph, which is uploaded
 * once, or a graph already in the current device's memory (detected from the pointers),
 * which is used where it is: in both cases it is borrowed for the lifetime of the
 * hierarchy, and its offsets and neighbour ids are range-checked on the device
 * (GOSH_EINVAL).  Every level then STAYS on
 * that device, where gosh_embed / gosh_embed_host read it without another upload, and the
 * host arrays behind gosh_hierarchy_graph / _map / _mult are downloaded on first request.
 * A graph whose marking does not resolve in a bounded number of rounds (long chains of
 * equal degrees) is marked on the host instead.  Device memory: about 36 bytes per entry
 * of G_0 while running; afterwards 12 bytes per entry of all levels, and the run's scratch
 * blocks (about 32 bytes per entry of G_0), which stay allocated until
 * gosh_hierarchy_trim_scratch, gosh_hierarchy_release_device or gosh_hierarchy_free
 * (called with the same device current) because freeing them at once would slow the host
 * link down for whatever follows (the driver clears freed memory in the background).
 * GOSH_ENOMEM / GOSH_EHIP if the device cannot.  Blocking; null stream. */
int gosh_coarsen_device(const gosh_csr *g0, int64_t threshold, double min_shrink,
                        int32_t max_levels, int32_t n_threads, gosh_hierarchy **out);

/* Returns the scratch blocks a device-built hierarchy still holds from its construction
 * (no-op otherwise).  The levels stay where they are. */
int gosh_hierarchy_trim_scratch(gosh_hierarchy *h);

/* Brings every array of a device-built hierarchy to the host and frees its device copies
 * (no-op for a host-built one).  Accessors and training keep working, from the host
 * copies.  Blocking. */
int gosh_hierarchy_release_device(gosh_hierarchy *h);

/* Accessors.  The arrays they hand out are host memory owned by the hierarchy (level 0:
 * by the caller) and stay valid until gosh_hierarchy_free.  For a device-built hierarchy
 * the first request for an array downloads it (blocking; the building device must be
 * current; GOSH_EHIP / GOSH_ENOMEM possible), so a hierarchy must not be used from two
 * threads at once. */

/* D, the number of graphs G_0..G_{D-1} (0 for NULL). */
int gosh_hierarchy_levels(const gosh_hierarchy *h);
/* |V_i| and the length of G_i's adj; either pointer may be NULL.  Never downloads. */
int gosh_hierarchy_shape(const gosh_hierarchy *h, int32_t i, int64_t *n, int64_t *nnz);
/* Borrowed host view of G_i (coarse levels have 64-bit offsets). */
int gosh_hierarchy_graph(const gosh_hierarchy *h, int32_t i, gosh_csr *view);
/* map_i: one entry per vertex of G_i, its super vertex in G_{i+1}; 0 <= i < D-1. */
int gosh_hierarchy_map(const gosh_hierarchy *h, int32_t i, const int32_t **map, int64_t *len);
/* Per entry of G_i's adj, how many entries of G_0 were merged into it (NULL and 0 for
 * level 0, where every entry counts once).  Not used by training; it makes edge-weight
 * conservation checkable: sum(mult_{i+1}) + (weight of entries inside clusters) =
 * sum(mult_i). */
int gosh_hierarchy_mult(const gosh_hierarchy *h, int32_t i, const int64_t **mult, int64_t *len);
/* Wall-clock milliseconds the three stages of Alg. 4 took when level i was coarsened
 * (0 <= i < D-1): ms3[0] degree sort, ms3[1] marking sweep, ms3[2] rebuilding the CSR of
 * G_{i+1} (Sec. 3.2.1 names these three stages). */
int gosh_hierarchy_times(const gosh_hierarchy *h, int32_t i, double *ms3);
void gosh_hierarchy_free(gosh_hierarchy *h);

/* ---- device entry points ---------------------------------------------------------- */
/* Every array these take must be memory a kernel can reach -- a device allocation, or
 * pinned host memory -- and must hold the documented number of elements inside the
 * allocation it starts in; both are checked before anything is launched (GOSH_EINVAL), so
 * that a wrong pointer or size becomes an error and not a memory fault on the device. */

/* "Randomly initialize M" (Alg. 2, second line).  Fills the device matrix M (n x d)
 * with values uniform in [-0.5/d, 0.5/d): entry (v, c) is word c%4 of
 * Philox4x32-10(counter = (v, c/4, 0xFFFFFFFF, level), key = seed), mapped as
 * ((w >> 8) * 2^-24 - 0.5) / d. */
int gosh_init_embedding(float *M_dev, int64_t n, int32_t d, uint64_t seed, uint32_t level,
                        void *hip_stream);

/* The sampler of Alg. 3 on its own (parity/debug): for every source src writes
 * out[src*(k_neg+1) + j], j = 0..k_neg.  j = 0 is the positive sample, a uniform member
 * of the neighbour list of src (Sec. 3.1; -1 if the list is empty); j >= 1 are the
 * negative samples, uniform over all n vertices.  Draw j of src is the low 64 bits of
 * Philox4x32-10(counter = (src, j, epoch, level), key = seed), reduced to an index
 * by multiply-high with the bound.  g_dev: CSR arrays on the device (the struct
 * itself on the host).  out_dev: device int32[n*(k_neg+1)]. */
int gosh_sample_epoch(const gosh_csr *g_dev, int32_t k_neg, uint64_t seed, uint32_t epoch,
                      uint32_t level, int32_t *out_dev, void *hip_stream);

/* One epoch of Alg. 3 ("TrainInGPU"): every vertex is the source of one positive and
 * k_neg negative updates of Alg. 1 ("UpdateEmbedding"), applied in that order:
 *   g = lr_epoch * (b - sigmoid(M[src] . M[v]));  M[src] += g*M[v];  M[v] += g*M[src]
 * (the second axpy uses the already updated source row; b = 1 for the positive, 0 for
 * negatives).  No positive update for a vertex without neighbours; a negative equal
 * to the source applies no update.  Sources run concurrently without locks (Sec. 3.1);
 * the launch is the epoch barrier.  With GOSH_FLAG_SEQUENTIAL the sources are taken one
 * by one in ascending id, which is deterministic.  In concurrent mode the sources are
 * handed out in ascending id too (workgroups start in the order of their index and each walks
 * a block of consecutive sources), so an epoch sweeps the graph in the order of the sequential
 * one, a window of concurrently running sources wide.  The default write path is a
 * mix: rows likely to be held by several wavefronts at once (every row of a small
 * graph, high-degree vertices of a large one) receive atomic adds of the step, the
 * others plain stores; GOSH_FLAG_PLAIN_STORES / GOSH_FLAG_ATOMIC_ADDS force one kind.
 * The mix uses a per-device scratch bitmap owned by the library (n bits, allocated on
 * first use), so concurrent-mode calls on one device must not overlap on different
 * streams.
 * g_dev: CSR arrays on the device.  M_dev: device matrix, updated in place.
 * (Where M_dev lies matters on this device: random row traffic inside one of the three HBM
 * ranks runs at about 5.2 TB/s, across two at about 6.2 TB/s; gosh_matrix_place allocates a
 * matrix that lies across two.)
 * lr_epoch: the already decayed learning rate (gosh_lr).  0 <= k_neg <= GOSH_MAX_NEG. */
int gosh_train_epoch(const gosh_csr *g_dev, float *M_dev, int32_t d, int32_t k_neg,
                     float lr_epoch, uint64_t seed, uint32_t epoch, uint32_t level,
                     uint32_t flags, void *hip_stream);

/* gosh_train_epoch for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same epoch with the
 * same arguments, results and error behaviour, except that the hot-row bitmap -- the one
 * buffer gosh_train_epoch allocates (on first use, and again when a larger graph comes) --
 * lives in a fixed array inside the library's code object: GOSH_STATIC_MAX_N bits = 8 MiB of
 * device memory on every GPU the library is loaded on, held until the process ends.  The
 * call allocates and frees nothing, on the device or the host, and takes graphs of at most
 * GOSH_STATIC_MAX_N vertices (GOSH_EINVAL beyond).  The bitmap is rewritten by every call
 * that uses it (nothing of a previous call is relied on), and all calls on one GPU share it:
 * calls that overlap on one GPU -- different streams, or threads -- race on it. */
#define GOSH_STATIC_MAX_N 67108864 /* 2^26 vertices */
int gosh_train_epoch_static(const gosh_csr *g_dev, float *M_dev, int32_t d, int32_t k_neg,
                            float lr_epoch, uint64_t seed, uint32_t epoch, uint32_t level,
                            uint32_t flags, void *hip_stream);

/* Divergence check (no passage of the paper: nothing in Alg. 1 bounds a row, and a learning
 * rate too large for a graph's hubs makes rows grow until fp32 overflows; the training calls
 * themselves are asynchronous and cannot tell).  Reads the n x d device matrix once and
 * returns the largest finite |entry| in *max_abs and the number of non-finite entries in
 * *nonfinite (either may be NULL).  Blocking: waits for the stream.  Uses a 16-byte
 * per-device result buffer owned by the library, so calls on one device must not overlap. */
int gosh_matrix_check(const float *M_dev, int64_t n, int32_t d, float *max_abs, int64_t *nonfinite,
                      void *hip_stream);

/* Row probe (no passage of the paper: the memory of the device, not the method): the row
 * traffic of the training kernels without their arithmetic, to be timed by the caller (HIP
 * events on the stream) -- to compare candidate locations for a matrix (on this device
 * random row traffic inside one of the three HBM ranks is slower than traffic that spans
 * two, see gosh_train_epoch), and to measure what the memory system allows a kernel that
 * moves rows of 4*d bytes at random.  A lane group of pow2ceil(d/4) lanes moves one row with
 * 128-bit accesses.  `accesses` units of work, drawn with Philox from `seed`:
 *   GOSH_PROBE_READ_WRITE  a uniformly random row is read and written back unchanged
 *   GOSH_PROBE_READ        a uniformly random row is read
 *   GOSH_PROBE_WRITE       a uniformly random row is overwritten with zeros
 *   GOSH_PROBE_EPOCH_MIX   the traffic of one source of Alg. 3 with three negatives: row
 *                          (i mod n) and four random rows are read, then all five written
 *                          back unchanged (5 + 5 row transfers per access)
 * Except in GOSH_PROBE_WRITE mode the matrix keeps its values, provided nothing else writes
 * it meanwhile.  Asynchronous on the stream. */
#define GOSH_PROBE_READ_WRITE 0
#define GOSH_PROBE_READ 1
#define GOSH_PROBE_WRITE 2
#define GOSH_PROBE_EPOCH_MIX 3
int gosh_row_probe(float *M_dev, int64_t n, int32_t d, int64_t accesses, uint64_t seed, int32_t mode,
                   void *hip_stream);

/* What gosh_matrix_place found (all sizes in bytes). */
typedef struct {
  uint64_t arena_bytes;          /* physical memory mapped for the search */
  uint64_t window_offset_bytes;  /* where in the arena the matrix starts */
  uint64_t kept_bytes;           /* what stays allocated: the 1 GiB pieces under the matrix */
  int32_t probes;                /* windows timed */
  float probe_ms_best, probe_ms_median;
  double search_ms;
} gosh_placement_info;

/* Allocates an n x d device matrix where random row traffic is fastest (no passage of the
 * paper: the memory of the device).  Maps an arena of arena_bytes (0: 120 GiB; never more
 * than what is free less 8 GiB; at least three times the matrix, else GOSH_ENOMEM) out of
 * 1 GiB pieces with the virtual-memory API, times gosh_row_probe on windows of it, returns
 * the fastest window in *M_dev -- in practice one that lies across two of the three HBM
 * ranks -- and gives the pieces outside it back before returning.  The matrix is
 * uninitialised.  Blocking; uses the null stream.  Free it with gosh_matrix_release (not
 * hipFree), after the work that uses it is done.  info may be NULL. */
int gosh_matrix_place(int64_t n, int32_t d, uint64_t arena_bytes, float **M_dev,
                      gosh_placement_info *info);
int gosh_matrix_release(float *M_dev);

/* "ExpandEmbedding" (Alg. 2; Sec. 3: the row of a vertex of G_{i-1} is the row of its
 * super vertex in G_i): M_fine[v,:] = M_coarse[map[v],:] for v < n_fine.  All pointers
 * are device memory; map holds n_fine ids in [0, n_coarse); an entry outside that range
 * gives a row of zeros.  M_fine and M_coarse must not overlap.  A slice of the fine level
 * can be projected by passing the matching slice of map and of M_fine. */
int gosh_project(const float *M_coarse_dev, int64_t n_coarse, const int32_t *map_dev,
                 int64_t n_fine, int32_t d, float *M_fine_dev, void *hip_stream);

/* ---- multilevel driver ---------------------------------------------------------------- */

typedef struct {
  int32_t level;     /* i */
  int64_t n, nnz;    /* size of G_i */
  int64_t epochs;    /* passes of Alg. 3 run on G_i: e_i, times ceil(|E_i|/|V_i|) with
                        GOSH_FLAG_EDGE_EPOCHS */
  double upload_ms;  /* host -> device copy of G_i (wall clock) */
  double train_ms;   /* the e_i epoch launches (HIP events on the stream) */
  double project_ms; /* map upload + projection to level i-1 (wall clock; 0 at level 0) */
  int32_t parts_K;   /* 0: trained with the epoch kernel; K > 0: trained with the part-pair
                        rotation on K parts (train_ms is then the wall time of that call) */
  float max_abs;     /* largest finite |entry| of M_i after training (levels trained by the
                        rotation on a host matrix: as met when parts were written back) */
  int64_t nonfinite; /* non-finite entries of M_i after training; 0 unless training diverged */
} gosh_level_stats;

/* Alg. 2 ("GOSH") for levels that fit the device: with D = levels of h and
 * e_i = gosh_epoch_split(epochs, p, D), for i = D-1 down to 0: copy G_i to the device,
 * (i = D-1: initialise M_{D-1} with gosh_init_embedding(seed, level D-1)), run e_i epochs
 * of gosh_train_epoch with lr = gosh_lr(lr0, j, e_i), epoch j and level i in the random
 * counter, then (i > 0) project to level i-1 with map_{i-1}.  The paper prints the loop
 * as "D-1 to 1"; the text trains until M_0 is obtained, which is what is done here.
 * h: hierarchy (host).  M0_dev: device matrix n_0 x d, receives the embedding of G_0.
 * flags: as for gosh_train_epoch, plus GOSH_FLAG_EDGE_EPOCHS and GOSH_FLAG_PAIR_LEVELS.  device_budget_bytes: if non-zero and the graph plus
 * matrix of level 0 exceed it, the call is refused with GOSH_EBUDGET (use gosh_embed_host,
 * which keeps such levels on the host).  stats: NULL or host array of D entries, filled per level.
 * Blocking: returns after the last level finished; intermediate device buffers are
 * allocated and freed inside the call.  Every level is checked after its training
 * (gosh_matrix_check: one more read of the matrix): if any level ends with non-finite
 * entries the run is still completed, stats are filled, and GOSH_EDIVERGED is returned. */
int gosh_embed(const gosh_hierarchy *h, int32_t d, int32_t k_neg, int64_t epochs, double p,
               float lr0, uint64_t seed, uint32_t flags, uint64_t device_budget_bytes,
               float *M0_dev, gosh_level_stats *stats, void *hip_stream);

/* Alg. 2 including its "fits into GPU" branch, with the result on the host.  Levels whose
 * graph and matrix fit device_budget_bytes (0 = what the current device has free when the
 * call starts, less a sixteenth; graphs the hierarchy already keeps there are outside
 * that figure) are trained as in
 * gosh_embed; the others are trained with gosh_train_parts(level i, e_i epochs, the same
 * budget, P_gpu, S_gpu, B) on a host-resident matrix.  Projection runs on the device
 * (slice by slice when the finer level lives on the host); only when both levels live
 * on the host are the rows gathered there.  The initial matrix of a coarsest level that
 * does not fit is produced on the device slice by slice (same values as
 * gosh_init_embedding).  M0_host: host matrix n_0 x d (pinned memory recommended). */
int gosh_embed_host(const gosh_hierarchy *h, int32_t d, int32_t k_neg, int64_t epochs, double p,
                    float lr0, uint64_t seed, uint32_t flags, uint64_t device_budget_bytes,
                    int32_t P_gpu, int32_t S_gpu, int32_t B, float *M0_host,
                    gosh_level_stats *stats, void *hip_stream);

/* ---- graphs larger than a device budget (Sec. 3.3, Alg. 5 "LargeGraphGPU") -------------- */

typedef struct {
  int32_t K;             /* number of parts (contiguous ranges of ceil(n/K) vertices) */
  int64_t rotations;     /* ceil(epochs / (B*K)), at least 1 */
  int64_t pair_visits;   /* rotations * K(K+1)/2 pair kernels */
  int64_t updates;       /* updates of Alg. 1 attempted (sources * B * (k_neg+1) per visit) */
  uint64_t device_bytes; /* part slots + sample pools + hot-row bitmap */
  uint64_t bytes_h2d;    /* parts and pools copied to the device */
  uint64_t bytes_d2h;    /* parts copied back */
  double kernel_ms;      /* sum of the pair kernels' durations (HIP events) */
  double wall_ms;        /* whole call, host wall clock */
  double sampler_ms;     /* time the host sampler spent drawing positives (its own clock) */
  double sampler_wait_ms; /* time the driving thread waited for a pool of positives */
  float max_abs;         /* largest finite |entry| met when parts were written back (device
                            matrix: of the matrix after the last rotation) */
  int64_t nonfinite;     /* non-finite entries met there (a part that leaves the device several
                            times is counted each time); 0 unless training diverged */
} gosh_parts_stats;

/* Visiting order of the part pairs in one rotation (Sec. 3.3.1): (0,0), (1,0), (1,1),
 * (2,0), ... -- K(K+1)/2 pairs written to a[] and b[] (host arrays), a[j] >= b[j]. */
int gosh_pair_order(int32_t K, int32_t *a, int32_t *b);

/* A visiting order that is not the paper's, for hardware whose host link bounds the
 * rotation: the parts are cut into blocks of R consecutive parts; for every block in turn,
 * first the pairs inside the block in the order of gosh_pair_order, then for each later
 * part c the pairs (c, r) for every r of the block.  A device that keeps the block resident
 * and streams the later parts through meets R pairs per part it loads.  Every pair (a, b),
 * a >= b, occurs exactly once; R >= K gives gosh_pair_order.  GOSH_EINVAL if R < 1. */
int gosh_pair_order_blocked(int32_t K, int32_t R, int32_t *a, int32_t *b);

/* The part layout gosh_train_parts would use: the smallest K for which min(P_gpu, K) part
 * slots of ceil(n/K) rows, S_gpu sample pools of 2*ceil(n/K)*B ids and the hot-row bitmap
 * fit device_budget_bytes; rotations = ceil(epochs/(B*K)) (Alg. 5, first line).  Any of
 * the output pointers may be NULL.  GOSH_EBUDGET if no K up to min(n, 4096) fits. */
int gosh_parts_plan(int64_t n, int32_t d, int64_t epochs, uint64_t device_budget_bytes,
                    int32_t P_gpu, int32_t S_gpu, int32_t B, int32_t *K_out,
                    int64_t *rotations_out, uint64_t *device_bytes_out);

/* Parity/debug: the sample ids of one visit of the pair (pa, pb), pb <= pa, in the order
 * the sequential reference applies them: for every vertex of part pa, B rounds of
 * (positive, k_neg negatives), then -- if pa != pb -- the same for every vertex of part pb.
 * Positive of a vertex: uniform member of its neighbours inside the partner part, -1 if
 * none; negatives: uniform over the partner part.  Draw t of a source uses
 * Philox4x32-10(counter = (src, side*B*(k_neg+1) + t, rotation,
 * (level & 255) | (pair_index+1) << 8), key = seed).  Positives are drawn on the host,
 * negatives on the device, exactly as in training.  g_host: host CSR; out_host: host
 * int32[(size(pa) + size(pb))*B*(k_neg+1)] (only size(pa) sources if pa == pb). */
int gosh_parts_sample_pair(const gosh_csr *g_host, int32_t K, int32_t pa, int32_t pb, int32_t B,
                           int32_t k_neg, uint64_t seed, uint32_t rotation, uint32_t level,
                           uint32_t pair_index, int32_t *out_host);

/* Alg. 5 for one level: the matrix stays on the host, K parts rotate through P_gpu device
 * slots, every pair of parts is trained against each other once per rotation (in the
 * order of gosh_pair_order) for `rotations` rotations, with lr = gosh_lr(lr0, r, rotations)
 * in rotation r.  In a visit of (a, b) every vertex of a runs B rounds of one positive
 * update (a neighbour inside b, drawn on the host into a pool that is shipped to the
 * device) and k_neg negative updates (drawn on the device, uniform over b), and vice versa;
 * a vertex without a neighbour in the partner part gets no positive update there.
 * g_host: host CSR, or a CSR in the current device's memory (detected from the pointers;
 * what gosh_embed_host passes for a level of a device-built hierarchy): the pools of
 * positives are then filled by a kernel on the device, with the same values, and no host
 * sampler runs -- on this hardware the graph usually fits the device where the matrix
 * does not (one pool is enough then: S_gpu = 1 leaves more of the budget to the parts).
 * The graph is outside device_budget_bytes either way.
 * M_host: host matrix n x d, updated in place; pinned memory makes the
 * transfers asynchronous.  A matrix in the current device's memory (detected from the
 * pointer) is trained where it is: every part is its own slot, nothing is copied, P_gpu
 * only shapes the blocked pair order, the part count is force_K or else 16, and the budget
 * covers the pools and the bitmap alone.  What is left of Alg. 5 then is its visiting
 * order and its sampling rule, which on this hardware make an epoch's worth of samples
 * 1.2-1.4x cheaper than an epoch of Alg. 3 (a source row is loaded once per B rounds, and
 * the negatives of a visit fall into one part).
 * device_budget_bytes: cap for slots + pools + bitmap (0 only together with force_K > 0,
 * or with a device matrix).  P_gpu >= 2 (paper: 3), S_gpu >= 1 (paper: 4), B >= 1
 * (paper: 5).  force_K > 0 overrides the part count.  flags as for gosh_train_epoch
 * (GOSH_FLAG_SEQUENTIAL: every pair kernel runs on one wavefront, sources in order), plus
 * GOSH_FLAG_BLOCKED_ORDER.
 * The library owns its streams, device buffers and sampler thread for the duration of
 * the call, which blocks until the matrix is back on the host.  stats_out may be NULL.
 * Every part is checked for non-finite entries on the device before it is written back (the
 * whole matrix at the end, if it lives on the device): GOSH_EDIVERGED, with the matrix as
 * training left it, if there were any. */
int gosh_train_parts(const gosh_csr *g_host, float *M_host, int32_t d, int32_t k_neg,
                     int64_t epochs, float lr0, uint64_t seed, uint32_t level,
                     uint64_t device_budget_bytes, int32_t P_gpu, int32_t S_gpu, int32_t B,
                     int32_t force_K, uint32_t flags, gosh_parts_stats *stats_out);

#ifdef __cplusplus
}
#endif
#endif /* GOSH_H */

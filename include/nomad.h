/*
 * libnomad -- the per-epoch optimisation of a 2-D embedding under the NOMAD Projection loss
 * (arxiv 2505.15511), on one AMD MI355X (gfx950).  C ABI, plain pointers and sizes.
 *
 * One epoch (nomad_epoch) is one full-batch SGD step on the sampled NOMAD loss:
 *   1. cluster (cell) means mu_r of the embedding                        -- Section 3.3, mu_r below Eq. 6
 *   2. mean-field sums over the cells approximated for each head         -- Eq. 5
 *   3. per directed kNN edge ij: Cauchy-kernel attraction (Eq. 1, numerator of Eq. 4),
 *      s sampled negatives m (uniform noise over tails, Section 3.3) and their repulsion
 *      (denominator of Eq. 2 / Eq. 4, sampled part Eq. 6)
 *   4. gradient scatter to heads, tails and negatives
 *   5. theta <- theta - eta_t g, eta_t = lr0 (1 - t/T)                   -- Section 3.4
 *
 * Conventions
 *   - Every function returns NOMAD_OK (0) or a negative NOMAD_E_* code; nothing throws or aborts
 *     across this boundary.  nomad_last_error() returns text for the last failure of a context.
 *   - `mem` says where a caller buffer lives: NOMAD_HOST (pageable or pinned host memory) or
 *     NOMAD_DEVICE (memory of the context's HIP device).
 *   - Ownership: the caller owns every buffer it passes.  set_* calls copy their inputs (the
 *     caller may free them afterwards); get_* calls copy into caller memory.  The library owns
 *     all of its device state.
 *   - All point indices and edge positions, in arguments and in results, are the caller's:
 *     points 0..n-1 and CSR positions 0..E-1 as passed to nomad_set_graph.
 *   - One context = one device + one stream.  A context is not thread-safe; different contexts
 *     are independent.  nomad_epoch only enqueues work on the stream; get_* and nomad_loss wait
 *     for it.
 */
#ifndef NOMAD_H
#define NOMAD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NOMAD_HOST 0
#define NOMAD_DEVICE 1

#define NOMAD_OK 0
#define NOMAD_E_INVALID_ARG (-1) /* null pointer, value out of range, struct_size mismatch          */
#define NOMAD_E_BAD_GRAPH (-2)   /* CSR / weights / cluster ids violate a stated requirement        */
#define NOMAD_E_ORDER (-3)       /* call made before the state it needs exists                      */
#define NOMAD_E_TOO_LARGE (-4)   /* n or E does not fit 31-bit indices                              */
#define NOMAD_E_OOM (-5)         /* device or host allocation failed                                */
#define NOMAD_E_HIP (-6)         /* a HIP runtime call failed; see nomad_last_error                 */

#define NOMAD_SCATTER_DETERMINISTIC 0
#define NOMAD_SCATTER_ATOMIC 1

#define NOMAD_MAX_NEG 16
#define NOMAD_MAX_BATCHES 4096

typedef struct nomad_ctx nomad_ctx; /* opaque, library-owned */

typedef struct {
    uint32_t struct_size;      /* = sizeof(nomad_config); checked by nomad_create                     */
    int64_t n_points;          /* n >= 1                                                              */
    int32_t n_clusters;        /* |R| >= 1: number of cells of the partition                          */
    int32_t n_neg;             /* s: sampled negatives per directed edge, 0..NOMAD_MAX_NEG            */
    float noise_count;         /* |M| of Eq. 2 / Eq. 4-6; <= 0 means "= n_neg"                        */
    int32_t n_epochs;          /* T >= 1 of the linear schedule                                       */
    float lr0;                 /* eta_0, applied to g = grad(n * L): per-point units                  */
    uint64_t seed;             /* key of the counter-based negative sampler                           */
    int32_t scatter_mode;      /* NOMAD_SCATTER_DETERMINISTIC or NOMAD_SCATTER_ATOMIC                 */
    int32_t batches_per_epoch; /* B, 1..NOMAD_MAX_BATCHES: sequential sub-steps of an epoch (see nomad_epoch) */
    int32_t device;            /* HIP device ordinal                                                  */
    void* stream;              /* hipStream_t borrowed from the caller; NULL = the null stream        */
    int32_t pool_size;         /* 0: the paper's i.i.d. negatives per edge.  1..NOMAD_MAX_POOL: opt-in */
                               /* pooled sampler, points per pool (see below)                         */
    int32_t pool_block;        /* pooled sampler: consecutive CSR positions sharing one pool, >= 1;    */
                               /* must be 0 exactly when pool_size is 0                               */
    int32_t far_field;         /* NOMAD_FAR_FIELD_EXACT (Eq. 5 summed over the approximated cells) or    */
                               /* NOMAD_FAR_FIELD_SAMPLED (opt-in estimate of it, see below)            */
    int32_t mean_gradient;     /* 0: the cell means are constants of an epoch (no gradient flows through */
                               /* them); 1: opt-in, see below                                            */
    int32_t pool_mode;         /* pooled sampler: NOMAD_POOL_PICKS16 (0), NOMAD_POOL_DISTINCT (1) or NOMAD_POOL_STRATIFIED (2), see below; */
                               /* 0 when pool_size is 0                                                  */
    int32_t pool_line;         /* NOMAD_POOL_DISTINCT / _STRATIFIED: consecutive points per pool line, a power of two, at most n_points */
                               /* (1 = every pool entry drawn on its own); 0 is read as 1                 */
    int32_t pool_segment;      /* NOMAD_POOL_DISTINCT / _STRATIFIED: consecutive CSR positions dealt to a block together, a */
                               /* power of two >= 64 that divides pool_block; 0 is read as 64; not used by */
                               /* NOMAD_POOL_PICKS16                                                      */
    int32_t edge_weights;      /* NOMAD_WEIGHTS_GIVEN (0): p(j|i) from nomad_set_graph's weights;          */
                               /* NOMAD_WEIGHTS_INVERSE_RANK (1): from the position of j in i's row, Eq. 7 */
} nomad_config;

/*
 * Edge weights from ranks (edge_weights = NOMAD_WEIGHTS_INVERSE_RANK; nomad_set_graph's `weights` must then be
 * NULL).  Eq. 7 models p(j|i) by the rank of j among i's nearest neighbours.  With the row of head i listing its
 * k_i neighbours in ascending distance (which is what nomad_knn_in_clusters returns), the edge at position rho =
 * 1..k_i of the row gets p(j|i) = exp(1/rho) / sum_{rho' = 1..k_i} exp(1/rho'): ranks counted from 1 and the
 * normaliser taken over the row's own k_i terms, so that every row is a distribution (as printed, Eq. 7 has a
 * 1/0 at rank 0 and k + 1 terms in the normaliser).  Computed on the device in float64, stored as float32.
 */
#define NOMAD_WEIGHTS_GIVEN 0
#define NOMAD_WEIGHTS_INVERSE_RANK 1

/*
 * Gradient through the means (opt-in; needs far_field = NOMAD_FAR_FIELD_EXACT and batches_per_epoch = 1; has no
 * effect without cluster_group).  mu_r below Eq. 6 is the mean of the cell's members, mu_r = (1/n_r) sum_{l in r}
 * theta_l.  With mean_gradient = 1 the gradient of Eq. 4 also flows through it: every member l of a cell r receives
 * (1/n_r) d(n L)/d mu_r, where d(n L)/d mu_r = |M| p_r sum_{i: r approximated for i} c_i q(theta_i, mu_r)^2
 * (theta_i - mu_r) and c_i = sum_{e in row i} 2 p_e / S_e.  The gradient is then the derivative of the sampled loss
 * as a function of the embedding alone (forces cancel, no net torque).  Costs a second pass over all (head, cell)
 * pairs per epoch.
 */

/*
 * Sampled far field (opt-in variant; needs pool_size = 0).  Eq. 5 replaces the points of the approximated cells
 * by their means and sums over those cells for every head: n |R| kernel evaluations per epoch.  With
 * NOMAD_FAR_FIELD_SAMPLED that sum is estimated by the s samples instead: the negatives of every edge are drawn
 * uniformly from ALL n points (same Philox words, multiply-high onto 0..n-1); a negative whose cell belongs to
 * another group than the head's stands for its cell, enters S_e as q(theta_i, mu_cell) and receives no force (the
 * means are constants of the epoch); a negative of the head's own group enters as itself.  Every sample weighs
 * |M| / s.  The sample sum then has the expectation |M| sum_{r approximated} p_r q(theta_i, mu_r) +
 * (|M| / n) sum_{m in own group} q(theta_i, theta_m), i.e. Eq. 5 plus the expectation of Eq. 6's sampled term, at
 * the cost of one extra index lookup per negative.  Without cluster_group it is the plain sampler.
 * nomad_get_mean_field returns zeros in this mode.
 */
#define NOMAD_FAR_FIELD_EXACT 0
#define NOMAD_FAR_FIELD_SAMPLED 1

/*
 * Pooled sampler (opt-in variant; NOT the i.i.d. noise samples of Section 3.1/3.3).  The CSR positions
 * are cut into blocks of pool_block consecutive positions.  Block beta draws, per epoch t, a pool of
 * pool_size points, entry u = point picked by word (u & 3) of Philox(counter (beta, 0xFFFFFFFF, t, u >> 2),
 * key seed).  Slot k of edge e takes pool entry (x16 * pool_size) >> 16, x16 = 16-bit half (k & 1) of word
 * ((k >> 1) & 3) of the per-edge Philox(counter (lo32 e, hi32 e, t, k >> 3)): one Philox call serves eight
 * slots.  Every negative is still uniform over the points, so the sampled loss
 * stays an unbiased estimate of Eq. 2; negatives of one block are no longer independent.  The pool lives
 * in LDS, which replaces s random 128-byte line fetches and s scattered force records per edge by
 * pool_size of each per block.  Needs cluster_group = NULL (one sampling population).  The fast kernel
 * applies when pool_block is a multiple of 1024; other values run the general kernels.
 */
#define NOMAD_MAX_POOL 4096
#define NOMAD_POOL_PICKS16 0
#define NOMAD_POOL_DISTINCT 1
#define NOMAD_POOL_STRATIFIED 2

/*
 * Pooled sampler with distinct picks (pool_mode = NOMAD_POOL_DISTINCT; opt-in like the variant above, same
 * restrictions, plus batches_per_epoch = 1).  Section 3.1 defines the noise samples of ONE edge as i.i.d. draws from
 * the noise distribution; this variant keeps exactly that and gives up only independence between different edges:
 *   - blocks: the CSR positions are cut into segments of g = pool_segment positions; with Q = pool_block / g segments
 *     per block and NS segments there are NB = ceil(NS / Q) blocks; segment sigma belongs to block beta = sigma mod NB
 *     and position e has rank g (sigma div NB) + (e mod g) in its block.  A block is thus Q segments spread evenly
 *     over the edge list (g = pool_block: blocks of consecutive positions);
 *   - pool of block beta in epoch t: L = pool_size / pool_line lines of pool_line cyclically consecutive points
 *     (after point n-1 comes point 0); line gamma starts at floor(x n / 2^32), x = word (gamma & 3) of
 *     Philox(counter (beta, 0xFFFFFFFF, t, gamma >> 2), key seed); entry u is point number (u div L) of line (u mod L);
 *   - picks: an edge takes one word W = word ((rank >> 10) & 3) of Philox(counter (beta, 0xFFFFFFFE, t,
 *     (rank & 1023) + 1024 (rank >> 12))); with lg = log2(pool_size): u_0 = the top lg bits of W, c = 2 (bits
 *     1..lg-1 of W) + 1, and slot k takes entry (u_0 + k c) mod pool_size.
 * pool_size is a power of two (2..NOMAD_MAX_POOL), pool_line <= n and s <= L: the odd stride c then puts the s picks of an edge into s
 * different lines, whose starts are independent uniform draws, so the s negatives are independent and uniform over
 * the points.  Negatives of different edges of a block share lines and are dependent; spreading a block over the
 * edge list (small g) makes the edges that share a pool come from unrelated neighbourhoods.  The fast kernel
 * applies when pool_block is 1024, 2048, 4096 or 8192 and its tables fit LDS; other shapes run the general kernels.
 *
 * Stratified pools (pool_mode = NOMAD_POOL_STRATIFIED): as NOMAD_POOL_DISTINCT, except for where the lines of a pool start.
 * With independent draws the number of pools a point belongs to in one epoch is Poisson-distributed, and what a point
 * receives as a negative comes in bursts: on data with real neighbourhood structure that costs quality.  Here the
 * lines of an epoch's pools are dealt from a keyed permutation pi_t of the NL = ceil(n / pool_line) lines of
 * consecutive points: line gamma of block beta starts at (pool_line pi_t((beta L + gamma) mod NL) + r_t) mod n, so every
 * line of points serves the same number of pools (to within one).  Keys per epoch from two Philox calls, counters
 * (0, 0xFFFFFFFD, t, 0) -> (w0..w3) and (1, 0xFFFFFFFD, t, 0) -> (w4..w7): multipliers A = (w0|1, w2|1, w4|1), increments
 * C = (w1, w3, w5), shift r_t = floor(w6 n / 2^32).  pi_t works on b = max(1, ceil(log2 NL)) bits: three rounds of
 * x <- (A_k x + C_k) mod 2^b, x <- x xor (x >> max(1, b / 2)), repeated until x < NL.  Every negative is still uniform
 * over the points (r_t is uniform); the lines of one pool are distinct, i.e. the negatives of one edge are drawn
 * without replacement at the granularity of lines instead of independently (a difference of order s^2 pool_line / n).
 */

/* Create a context.  Allocates nothing on the device yet.  *out is set only on success. */
int nomad_create(const nomad_config* cfg, nomad_ctx** out);

/* Free the context and everything it owns.  NULL is allowed. */
void nomad_destroy(nomad_ctx* ctx);

/*
 * The input kNN digraph (Section 3.1: a distribution P over directed edges ij, head i, tail j),
 * the partition R into cells (Section 3.3) and, optionally, which cells each head approximates.
 *
 *   row_ptr  [n+1] int32  CSR offsets, row_ptr[0] = 0, non-decreasing, E = row_ptr[n] < 2^31
 *   col_idx  [E]   int32  tails, 0 <= col < n, no self loops
 *   weights  [E]   fp32   edge weights >= 0 with a positive sum on every non-empty row, or NULL
 *                         for unit weights.  p(j|i) of Eq. 4 is the row-normalised weight.
 *   cluster_of    [n]   int32  cell of each point, 0 <= id < |R|
 *   cluster_group [|R|] int32  group label of each cell, 0 <= label < |R|, or NULL for a single
 *                         group.  For a head i the cells of *other* groups are replaced by their
 *                         means (they form R-tilde of Eq. 5); negatives are sampled from the points
 *                         of i's own group and weighted |M| (n_group/n) / s (Eq. 6).  NULL means
 *                         nothing is approximated and Eq. 4 is the InfoNC-t-SNE loss, Eq. 2.
 *
 * The graph need not be symmetric.  Violations of the requirements above give NOMAD_E_BAD_GRAPH
 * and leave the context without a graph.  Replaces any earlier graph and embedding.
 */
int nomad_set_graph(nomad_ctx* ctx, const int32_t* row_ptr, const int32_t* col_idx, const float* weights,
                    const int32_t* cluster_of, const int32_t* cluster_group, int mem);

/* theta [n*2] fp32 row-major (Section 3.1: the matrix of low-dimensional positions). */
int nomad_set_embedding(nomad_ctx* ctx, const float* theta, int mem);

/*
 * One epoch with epoch index t, 0 <= t < T: fresh negatives keyed on (seed, t, edge, slot), the
 * gradient of the sampled loss (Eq. 4 with Eq. 5-6) and the SGD step with eta_t = lr0 (1 - t/T)
 * (Section 3.4).  With batches_per_epoch = B > 1 (a reading of "approximates the expectation over heads via
 * random sampling", Section 3.3) the epoch is B sequential sub-steps: sub-step b takes the heads
 * floor(n b / B) .. floor(n (b+1) / B) - 1, evaluates the gradient of their edges at the current embedding with
 * the cell means of the start of the epoch, and applies it with eta_t.  Enqueued on the context's stream;
 * returns without waiting.
 */
int nomad_epoch(nomad_ctx* ctx, int32_t t);

/*
 * The sampled loss of Eq. 4 at the current embedding, with the negatives of epoch index
 * t_sample >= 0 and cell means of the current embedding.  Waits for the stream.  *out_host is a
 * host double.  Does not change the embedding or the stored gradient.
 */
int nomad_loss(nomad_ctx* ctx, int32_t t_sample, double* out_host);

/* Current embedding, [n*2] fp32.  Waits for the stream. */
int nomad_get_embedding(nomad_ctx* ctx, float* out, int mem);

/* ---- test hooks (same conventions; all wait for the stream) ---- */

/* g = grad(n * L_t) of the most recent nomad_epoch (of its last sub-step), as it was applied.  [n*2] fp32. */
int nomad_get_gradient(nomad_ctx* ctx, float* out, int mem);

/* Negative indices of CSR edges e_begin..e_end-1 for epoch index t: [(e_end-e_begin)*s] int32. */
int nomad_get_negatives(nomad_ctx* ctx, int32_t t, int64_t e_begin, int64_t e_end, int32_t* out, int mem);

/* Cell means of the current embedding, mu [|R|*2] fp32, and cell sizes, counts [|R|] int64. */
int nomad_get_means(nomad_ctx* ctx, float* mu, int64_t* counts, int mem);

/* Mean-field sums of the current embedding: A [n] = sum_{r in R-tilde_i} p_r q(theta_i, mu_r) and
 * B [n*2] = sum p_r q^2 (theta_i - mu_r) (Eq. 5 without |M|, and the factor of its derivative).
 * All zero when no cell is approximated. */
int nomad_get_mean_field(nomad_ctx* ctx, float* A, float* B, int mem);

/* Number of directed edges E of the current graph (0 before nomad_set_graph). */
int64_t nomad_num_edges(const nomad_ctx* ctx);

/*
 * Which gradient-scatter path nomad_set_graph chose for this context (0 before it):
 *   NOMAD_PATH_ATOMIC_FP32   scatter_mode = NOMAD_SCATTER_ATOMIC: fp32 global atomics, order not reproducible
 *   NOMAD_PATH_BINNED        deterministic: forces binned by destination tile in the edge pass, summed per tile in LDS
 *   NOMAD_PATH_BINNED_POOLED deterministic, pooled sampler: the same with the pool's rows and force sums in LDS
 *   NOMAD_PATH_FIXED_ATOMICS deterministic fallback: 64-bit fixed-point global atomics (several times slower); taken
 *                            when the per-tile tables do not fit LDS (s > 8, more than 67 M points) or the record pool
 *                            could not be allocated -- nomad_set_graph then still returns NOMAD_OK and
 *                            nomad_last_error says why
 * Results of the three deterministic paths agree to rounding (each is reproducible run to run).
 */
#define NOMAD_PATH_ATOMIC_FP32 1
#define NOMAD_PATH_BINNED 2
#define NOMAD_PATH_BINNED_POOLED 3
#define NOMAD_PATH_FIXED_ATOMICS 4
int nomad_scatter_path(const nomad_ctx* ctx);

/* Device memory the context holds, in bytes (graph, embedding, work space; 0 before nomad_set_graph). */
int64_t nomad_device_bytes(const nomad_ctx* ctx);

/*
 * Launch-shape knobs for experiments and tests; results do not depend on them beyond rounding order (every setting
 * is reproducible run to run).  Call between nomad_create and nomad_set_graph (NOMAD_E_ORDER afterwards).
 *   NOMAD_TUNE_EDGE_BLOCK      lanes per workgroup of the binned edge pass: 1024 (default) or 512
 *   NOMAD_TUNE_WORKGROUPS_PER_CU persistent workgroups per compute unit, 1..8 (default 1; 2 with 512 lanes)
 *   NOMAD_TUNE_SCATTER_PATH    0 (default: the fastest path that fits) or NOMAD_PATH_FIXED_ATOMICS to force the fallback
 *   NOMAD_TUNE_POOL_KERNEL     1 (default) or 0: run the pooled samplers on the general kernels
 *   NOMAD_TUNE_RECORD_PHASES   0 (default: chosen from the record volume) or 1..64: the edge pass of an epoch runs in
 *                              this many phases over ranges of CSR positions, each followed by the accumulation of its
 *                              records, so that the record pool holds one phase at a time
 *   NOMAD_TUNE_RECORD_SORT     0 (default: sorted unless there are more tiles than a round has records), 1: a round's
 *                              records are counting-sorted by tile in LDS and written by consecutive lanes, 2: every
 *                              lane writes its own records
 *   NOMAD_TUNE_FLUSH_ROUNDS    0 (default: 2), 1 or 2: rounds of 1024 positions the unsorted form takes between two
 *                              flushes of its records (1024-lane workgroups only)
 */
#define NOMAD_TUNE_EDGE_BLOCK 1
#define NOMAD_TUNE_WORKGROUPS_PER_CU 2
#define NOMAD_TUNE_SCATTER_PATH 3
#define NOMAD_TUNE_POOL_KERNEL 4
#define NOMAD_TUNE_RECORD_PHASES 5
#define NOMAD_TUNE_RECORD_SORT 6
#define NOMAD_TUNE_FLUSH_ROUNDS 7
int nomad_tune(nomad_ctx* ctx, int knob, int value);

/* ---- kernel timing (HIP events on the context's stream, around each launch) ---- */

#define NOMAD_K_MEANS 0      /* cell means                         */
#define NOMAD_K_MEANFIELD 1  /* mean-field sums                    */
#define NOMAD_K_EDGES 2      /* attraction + sampling + repulsion  */
#define NOMAD_K_SCATTER 3    /* fallback: combine of fixed-point sums */
#define NOMAD_K_UPDATE 4     /* SGD step                           */
#define NOMAD_K_LOSS 5       /* loss terms + reduction             */
#define NOMAD_K_ZERO 6       /* clearing of accumulators           */
#define NOMAD_K_TILES 7      /* per-tile accumulation of the binned forces */
#define NOMAD_K_MEANGRAD 8   /* gradient through the means: head coefficients, sum over heads per cell */
#define NOMAD_K_COUNT 9

/* Switch per-launch timing on (1) or off (0); switching on clears earlier samples. */
int nomad_profile(nomad_ctx* ctx, int enable);

/* Waits for the stream; total milliseconds and number of launches of one kernel kind since
 * timing was switched on. */
int nomad_profile_read(nomad_ctx* ctx, int kind, double* total_ms, int64_t* launches);

/*
 * Bandwidth probe: enqueue one streaming device-to-device copy of `bytes` bytes (a multiple of 16,
 * both pointers 16-byte aligned, device memory of the current device) on `stream`.  Reads `bytes`
 * and writes `bytes`: the kernel of known traffic used to calibrate profiler byte counters and to
 * measure the practical HBM ceiling next to the epoch kernels.  Returns without waiting.
 */
int nomad_copy_probe(void* dst, const void* src, uint64_t bytes, void* stream);

/*
 * Gather probe: enqueue one kernel in which every lane loads 8-byte slots at uniformly random positions of `table`
 * (device memory, 8-byte aligned, table_bytes >= 8 and < 32 GiB), eight requests in flight per lane, about
 * n_requests in all (rounded up to a whole number of rounds of 2^24 requests, at most 4096 rounds; *issued_out
 * receives the exact count).  What it measures: the rate at which the memory system serves independent small
 * gathers from a table of that size -- the pattern of the negatives' embedding rows in the epoch kernel.  `sink`
 * points to 4 bytes of device memory (written only if the loaded values add up to one particular number, which
 * keeps the loads alive).  Follows no passage of the paper; returns without waiting.
 */
int nomad_gather_probe(const void* table, uint64_t table_bytes, uint64_t n_requests, uint64_t* issued_out, void* sink, void* stream);

/*
 * Scatter probes, same conventions: kind NOMAD_PROBE_ATOMIC_F32X2 (two fp32 atomic adds to a random 8-byte slot per
 * request), NOMAD_PROBE_ATOMIC_U64 (one 64-bit integer atomic add per request), NOMAD_PROBE_APPEND12 (256 persistent
 * workgroups of 1,024 lanes, each lane appending 12-byte records to a random one of its workgroup's `chains` private
 * regions of the table: one partial-line write per lane) and NOMAD_PROBE_APPEND12_GROUPED (the same with eight
 * adjacent lanes writing 96 contiguous bytes).  The append kinds need table_bytes >= about 1.25 x 12 x n_requests
 * plus 768 bytes per (workgroup, chain) (NOMAD_E_INVALID_ARG otherwise); `chains` (1..16384) is ignored by the
 * atomic kinds.  The table's contents are overwritten.
 */
#define NOMAD_PROBE_ATOMIC_F32X2 1
#define NOMAD_PROBE_ATOMIC_U64 2
#define NOMAD_PROBE_APPEND12 3
#define NOMAD_PROBE_APPEND12_GROUPED 4
int nomad_scatter_probe(int kind, void* table, uint64_t table_bytes, uint64_t n_requests, uint32_t chains, uint64_t* issued_out,
                        void* stream);

/*
 * ---- the upstream index: exact nearest neighbours inside clusters (Section 3.2) ----
 *
 * The paper builds its kNN graph from a K-Means partition: the candidates for a point's neighbours are the points of
 * its own cluster, and among those the nearest neighbours are computed exactly.  This call is that second half; the
 * partition is an input.
 *
 *   X          [n*d] fp32 row-major, the high-dimensional vectors; 1 <= d <= NOMAD_KNN_MAX_DIM
 *   cluster_of [n]   int32, 0 <= id < n_clusters
 *   out_nbrs   [n*k] int32: for every point its k nearest other points of the same cluster in ascending distance,
 *                    ties to the lower point index; -1 in the slots a cluster with fewer than k+1 points cannot fill
 *   mem        where X, cluster_of and out_nbrs live (NOMAD_HOST or NOMAD_DEVICE of `device`)
 *   stats      NULL, or [2] host int64: queries that needed the exact fallback, point pairs the filter evaluated
 *
 * Distance: sum over t = 0..d-1, in that order, of (x_t - y_t)^2 with every operation in float64.  The result is that
 * definition exactly: a float32 pass on the matrix cores only selects k + 8 candidates per point, their distances are
 * recomputed in float64, and a point whose candidates cannot be proven complete (the float32 error bound against
 * the first key left out) is redone against its whole cluster.  Inputs must be finite.  Stand-alone: needs no context;
 * allocates its work space on `device` and frees it before it returns; waits for `stream`.
 * Errors: NOMAD_E_INVALID_ARG, NOMAD_E_TOO_LARGE (n >= 2^31 - 256), NOMAD_E_BAD_GRAPH (cluster id out of range), NOMAD_E_OOM,
 * NOMAD_E_HIP.
 */
#define NOMAD_KNN_MAX_K 32
#define NOMAD_KNN_MAX_DIM 768
int nomad_knn_in_clusters(const float* X, int64_t n, int32_t d, const int32_t* cluster_of, int32_t n_clusters, int32_t k,
                          int32_t* out_nbrs, int mem, int32_t device, void* stream, int64_t* stats);

/*
 * Lloyd's iterations of the K-Means clustering behind the index (Section 3.2: "expectation maximization until
 * convergence"; the initial centroids are the caller's: the paper's locality-sensitive-hash start is not specified).
 *
 *   X          [n*d] fp32 row-major
 *   centroids  [K*d] fp32, in: the initial centroids, out: the final ones; 1 <= K <= n
 *   labels     [n]   int32 out: the cluster of every point
 *   max_iters  >= 1: E steps at most
 *   iters_out  host int32, may be NULL: E steps run;  inertia_out  host double, may be NULL: sum over the points of
 *              the distance to their centroid at the last E step
 *
 * One iteration: E step, label_i = argmin_j D(x_i, c_j) with the float64 distance of nomad_knn_in_clusters, ties to
 * the lower j, computed with the same matrix-core filter, float64 refinement and exact fallback (so the labels are
 * that definition exactly); M step, c_j = float32(sum of the rows of cluster j in float64, in ascending point order,
 * / n_j), an empty cluster keeps its centroid.  Stops when an E step changes no label.  Deterministic.
 * Same conventions, limits and errors as nomad_knn_in_clusters.
 */
int nomad_kmeans_lloyd(const float* X, int64_t n, int32_t d, int32_t K, float* centroids, int32_t max_iters, int32_t* labels,
                       int32_t* iters_out, double* inertia_out, int mem, int32_t device, void* stream);

/*
 * Initial centroids for nomad_kmeans_lloyd from a locality-sensitive hash (Section 3.2 names such a start without
 * detail; this is random-hyperplane hashing with the random draws made by the caller).
 *
 *   X            [n*d] fp32 row-major
 *   planes       [n_planes*d] fp32: the normals h_j;  anchors [n_planes] int32: plane j passes through the data point
 *                x_{anchors[j]};  1 <= n_planes <= 30 and 2^n_planes >= K.  anchors == NULL: the library takes, for every
 *                plane, the median along h_j of the sample of min(1024, n) points floor(s n / m) (projection sum_t h_{j,t} x_t
 *                in sequential float64, rank floor(m / 2) in ascending (projection, point)): every plane then halves the data
 *   centroids_out [K*d] fp32 out;  buckets_out NULL or [n] int32 out: the bucket of every point
 *
 * bit j of a point = [ sum_t h_{j,t} (x_t - x_{anchors[j],t}) > 0 ], the sum over t = 0..d-1 in order with difference,
 * product and running sum each rounded once in float64; code = sum_j bit_j 2^j; bucket = floor(code K / 2^n_planes);
 * centroid j = float32 mean of bucket j (rows added in ascending point order in float64, as in the M step); an empty
 * bucket takes the data point floor(j n / K).  Deterministic and exactly reproducible.  All arrays live in `mem`.
 * Same conventions, limits and errors as nomad_knn_in_clusters (an anchor outside 0..n-1: NOMAD_E_INVALID_ARG).
 */
int nomad_kmeans_lsh_init(const float* X, int64_t n, int32_t d, int32_t K, const float* planes, const int32_t* anchors,
                          int32_t n_planes, float* centroids_out, int32_t* buckets_out, int mem, int32_t device, void* stream);

/*
 * Neighbourhood preservation at k (Section 4: the average overlap between the k-neighbourhoods of a point in the
 * data space and in the projection).
 *
 *   X          [n*d] fp32 row-major: the data;  Y [n*d_low] fp32 row-major: the projection; n >= 2
 *   k          1..NOMAD_KNN_MAX_K; d, d_low <= NOMAD_KNN_MAX_DIM
 *   queries    NULL (every point; then n_queries is 0 or n), or [n_queries] int32 point indices: the points whose
 *              neighbourhoods are compared (a sample at large n; repeats count as often as they are listed)
 *   hits_out   host int64: common members of the two neighbourhoods, summed over the queries; the measure is
 *              hits / (k * queries)
 *
 * A neighbourhood is the k nearest other points among all n under the float64 distance of nomad_knn_in_clusters,
 * ties to the lower index, exactly (same filter, refinement and fallback).  Cost: queries * n distance
 * evaluations per space.  X, Y and queries live in `mem`; same conventions and errors as nomad_knn_in_clusters
 * (a query outside 0..n-1: NOMAD_E_INVALID_ARG).
 */
int nomad_neighbourhood_preservation(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low, int32_t k,
                                     const int32_t* queries, int64_t n_queries, int64_t* hits_out, int mem, int32_t device,
                                     void* stream);

/*
 * Random triplet accuracy (Section 4: the probability that a random triplet of points has the same ordering of its
 * pairwise distances in the data space and in the projection).
 *
 *   X, Y       as above; n >= 3; any d, d_low >= 1
 *   n_triplets triplets drawn, 0 .. 2^40
 *   agree_out  host int64: triplets that agree; the measure is agree / n_triplets
 *
 * Triplet t = anchor i and two other points j, k, all distinct and uniform: with (o0, o1, o2, .) =
 * Philox4x32-10(counter = (lo32 t, hi32 t, 0x54524950, 0), key = (lo32 seed, hi32 seed)), i = floor(o0 n / 2^32),
 * j = floor(o1 (n-1) / 2^32) moved up by one if >= i, k = floor(o2 (n-2) / 2^32) moved up by one if >= min(i,j) and by
 * one more if >= max(i,j).  It agrees when [D_X(i,j) < D_X(i,k)] == [D_Y(i,j) < D_Y(i,k)], D the float64 distance of
 * nomad_knn_in_clusters: the count is exact and reproducible.  Same conventions and errors.
 */
int nomad_random_triplet_accuracy(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low, int64_t n_triplets,
                                  uint64_t seed, int64_t* agree_out, int mem, int32_t device, void* stream);

/*
 * nomad_random_triplet_accuracy for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same definition and result; differences:
 *   - X and Y must already be device memory of `device` (there is no `mem` argument: staging host data would need an
 *     allocation); agree_out is a host int64;
 *   - the agreement counter lives in a 256-byte work space that is part of the library's code object (one copy per
 *     device, held until the process ends) instead of a buffer allocated for the call.  The call performs no
 *     hipMalloc / hipFree; it clears the counter with a kernel, counts, copies the result out and waits for `stream`;
 *   - limits: n < 2^31 - 256 and n_triplets <= 2^40 (NOMAD_E_TOO_LARGE beyond), device ordinal < 64
 *     (NOMAD_E_INVALID_ARG beyond);
 *   - all calls on one device share that device's work space: calls that overlap in time on one device (two host
 *     threads, two streams) race on the counter and must be serialised by the caller.
 */
int nomad_random_triplet_accuracy_noalloc(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low, int64_t n_triplets,
                                          uint64_t seed, int64_t* agree_out, int32_t device, void* stream);

/*
 * PCA initialisation of the projection (Section 3.5: the optimisation starts from a PCA of the data).
 *
 *   X          [n*d] fp32 row-major, n >= 2, 2 <= d <= NOMAD_KNN_MAX_DIM
 *   std0       > 0: both coordinates are multiplied by std0 / sqrt(lambda_1), so the first has standard deviation std0;
 *              <= 0: the scores as they are
 *   theta_out  [n*2] fp32 out (in `mem`): theta_i = ((x_i - mean) . v_1, (x_i - mean) . v_2), v_1, v_2 the eigenvectors of
 *              the covariance (1/n) sum (x_i - mean)(x_i - mean)^T with the largest eigenvalues lambda_1 >= lambda_2,
 *              each oriented so that its entry of largest magnitude is positive; computed in float64, rounded once
 *   stats      NULL, or [4] host double: lambda_1, lambda_2, the residual max_m |C v_m - lambda_m v_m| / lambda_1 reached,
 *              iterations of the eigenvector solver
 *
 * Mean and covariance are exact sums in float64 (the covariance on the float64 matrix cores); the eigenvectors come
 * from subspace iteration with Rayleigh-Ritz steps until the residual is below 1e-12 or 2,000 steps have run
 * (eigenvalues that nearly coincide with their successors converge slowly and leave the axes ill-defined anyway:
 * stats[2] says what was reached).  Deterministic.  Same conventions and errors as nomad_knn_in_clusters;
 * NOMAD_E_INVALID_ARG also when std0 > 0 and the data has no variance.
 */
int nomad_pca_init(const float* X, int64_t n, int32_t d, float std0, float* theta_out, double* stats, int mem, int32_t device,
                   void* stream);

/* Text of the last error of this context ("" if none), or, after a successful nomad_set_graph that had to take a
 * slower path, the reason (see nomad_scatter_path).  Valid until the next call on it. */
const char* nomad_last_error(const nomad_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* NOMAD_H */

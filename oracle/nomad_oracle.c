/*
 * CPU oracle for one NOMAD Projection epoch -- TEST INFRASTRUCTURE, NOT PRODUCT.
 *
 * Plain C loops in double precision, OpenMP over heads with one private gradient buffer
 * per thread.  Same definitions as oracle/nomad_oracle.py (which is the readable
 * statement of them) for graphs too large for Python loops, and the program timed as the
 * CPU baseline.  It shares no code with the HIP library and nothing in the product path
 * may link or call it.
 *
 * Definitions followed (arxiv 2505.15511):
 *   Eq. 1   Cauchy kernel q(a,b) = 1/(1+|a-b|^2)
 *   Eq. 4   per-edge term  -log q(ij) + log( q(ij) + Mtilde_i + Mcal_ij ), weighted by p(j|i),
 *           averaged over heads (uniform head marginal, Section 3.3)
 *   Eq. 5   Mtilde_i = |M| sum_{r in Rtilde_i} p(m in r) q(theta_i, mu_r), mu_r the cell mean
 *   Eq. 6   Mcal_ij estimated from s sampled negatives of the exact cells
 *   Section 3.4  SGD, learning rate annealed linearly to zero
 * The readings taken where the paper is silent are listed in nomad_oracle.py's header.
 *
 * parity status: pinned through tests/test_oracle_*.py, which run the same closed forms,
 * finite differences, brute-force comparisons and Philox known answers on this library as
 * on the Python oracle.  The two entry points that only large runs use are pinned there too:
 * the row-by-row mode of oracle_loss_grad (target_slot) against the rows of the full gradient
 * (test_single_gradient_rows_equal_the_rows_of_the_full_gradient), and oracle_train against
 * the Python oracle's epoch applied T times, bit for bit
 * (test_training_run_is_the_epoch_applied_T_times); oracle_mean_field_at against the Python
 * oracle's mean_field (test_mean_field_sums_of_single_heads).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t n;                    /* points                                           */
    const int32_t* row_ptr;       /* [n+1]                                            */
    const int32_t* col_idx;       /* [E]                                              */
    const float* weights;         /* [E] or NULL (unit)                               */
    const int32_t* cluster_of;    /* [n]                                              */
    int32_t n_clusters;           /* |R|                                              */
    const int32_t* cluster_group; /* [|R|] or NULL (one group: nothing approximated)  */
    int32_t n_neg;                /* s                                                */
    double noise_count;           /* |M|                                              */
    uint64_t seed;
    int32_t pool_size;            /* pooled sampler: points per pool (0 = i.i.d. per-edge sampler) */
    int32_t pool_block;           /* pooled sampler: consecutive CSR positions that share a pool   */
    int32_t batches_per_epoch;    /* B >= 1 (0 is read as 1): sequential sub-steps of an epoch, see oracle_epoch */
    int64_t head_begin, head_end; /* loss / gradient restricted to the edges of heads head_begin..head_end-1;   */
                                  /* head_end < 0 = all heads                                                   */
    int32_t sampled_far_field;    /* opt-in variant of Eq. 5: negatives are drawn from all points; one whose cell is  */
                                  /* approximated for the head enters through the cell mean and receives no force     */
    int32_t mean_gradient;        /* opt-in: the gradient also flows through mu_r = (1/n_r) sum_{l in r} theta_l: every */
                                  /* member of cell r receives (1/n_r) d(n L)/d mu_r (full mode, exact far field only)  */
    int32_t pool_mode;            /* pooled sampler: 0 = 16-bit picks from the pool of a block of consecutive positions; */
                                  /* 1 = distinct picks from the pool of an interleaved block (see edge_negatives);      */
                                  /* 2 = the same with the pools' lines dealt from a permutation (stratified_line_start) */
    int32_t pool_line;            /* pool_mode 1: consecutive points per pool line, a power of two                       */
    int32_t pool_segment;         /* pool_mode 1: consecutive positions dealt to a block together: a power of two >= 64   */
                                  /* that divides pool_block                                                             */
} oracle_problem;

/* ---- Philox4x32-10 (published algorithm: Salmon, Moraes, Dror, Shaw, SC'11) ---- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ---- derived, per-problem tables ---- */
typedef struct {
    int64_t* gstart;  /* [max group label + 2] offsets into members */
    int32_t* members; /* points ordered by (group, index)           */
    int64_t* counts;  /* [|R|] cluster sizes                        */
    int32_t max_label;
} oracle_tables;

static int build_tables(const oracle_problem* P, oracle_tables* T) {
    memset(T, 0, sizeof(*T));
    int32_t R = P->n_clusters;
    T->counts = (int64_t*)calloc((size_t)R, sizeof(int64_t));
    for (int64_t i = 0; i < P->n; ++i) {
        int32_t r = P->cluster_of[i];
        if (r < 0 || r >= R) return -1;
        T->counts[r]++;
    }
    int32_t maxl = 0;
    if (P->cluster_group)
        for (int32_t r = 0; r < R; ++r) {
            if (P->cluster_group[r] < 0) return -1;
            if (P->cluster_group[r] > maxl) maxl = P->cluster_group[r];
        }
    T->max_label = maxl;
    T->gstart = (int64_t*)calloc((size_t)maxl + 2, sizeof(int64_t));
    T->members = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P->n > 0 ? P->n : 1));
    for (int64_t i = 0; i < P->n; ++i) {
        int32_t g = P->cluster_group ? P->cluster_group[P->cluster_of[i]] : 0;
        T->gstart[g + 1]++;
    }
    for (int32_t g = 0; g <= maxl; ++g) T->gstart[g + 1] += T->gstart[g];
    int64_t* cur = (int64_t*)malloc(sizeof(int64_t) * ((size_t)maxl + 1));
    memcpy(cur, T->gstart, sizeof(int64_t) * ((size_t)maxl + 1));
    for (int64_t i = 0; i < P->n; ++i) { /* ascending i => each group's list is ascending */
        int32_t g = P->cluster_group ? P->cluster_group[P->cluster_of[i]] : 0;
        T->members[cur[g]++] = (int32_t)i;
    }
    free(cur);
    return 0;
}

static void free_tables(oracle_tables* T) {
    free(T->counts); free(T->gstart); free(T->members);
}

static inline int32_t group_of_point(const oracle_problem* P, int64_t i) {
    return P->cluster_group ? P->cluster_group[P->cluster_of[i]] : 0;
}

/* negatives of edge e with head i: m[slot], slot < s.
 * i.i.d. sampler: word (slot & 3) of Philox(counter (lo32 e, hi32 e, t, slot >> 2)) picks a point of the
 * head's population.
 * pooled sampler (opt-in variant, not the paper's i.i.d. noise samples; needs a single population): the
 * pool_block consecutive CSR positions of block beta = e / pool_block share a pool of pool_size points,
 * pool[u] = point picked by word (u & 3) of Philox(counter (beta, 0xFFFFFFFF, t, u >> 2)).  Slot k of
 * edge e picks the pool entry u = (x16 * pool_size) >> 16, x16 = 16-bit half (k & 1) of word
 * ((k >> 1) & 3) of Philox(counter (lo32 e, hi32 e, t, k >> 3)): eight slots per Philox call.  Every
 * negative is still uniform over the points; negatives of different edges of a block are no longer
 * independent.
 * pooled sampler with distinct picks (pool_mode 1; single population): the positions are cut into segments of
 * g = pool_segment; there are NB = ceil(NS / Q) blocks for NS segments and Q = pool_block / g segments per block;
 * segment sigma belongs to block beta = sigma mod NB and position e has rank g (sigma div NB) + (e mod g) in its
 * block, so a block is Q segments spread evenly over the edge list (g = pool_block: consecutive blocks).  The pool of a block is L = pool_size / pool_line lines
 * of pool_line cyclically consecutive points; line gamma starts at the point picked by word (gamma & 3) of
 * Philox(counter (beta, 0xFFFFFFFF, t, gamma >> 2)); entry u is point (u div L) of line (u mod L).  An edge takes
 * one word W = word ((rank >> 10) & 3) of Philox(counter (beta, 0xFFFFFFFE, t, (rank & 1023) + 1024 (rank >> 12)));
 * with lg = log2(pool_size), u_0 = top lg bits of W and the odd stride c = 2 (bits 1..lg-1 of W) + 1, slot k takes
 * entry (u_0 + k c) mod pool_size.  The s <= L picks lie in s different lines, whose starts are independent
 * uniform draws: the negatives of one edge are i.i.d. uniform over the points, as Section 3.1 defines them;
 * negatives of different edges of a block are dependent.
 * sampled far field: the i.i.d. sampler with every head's population = all n points. */
/* Stratified pools (pool_mode 2): the lines of an epoch's pools are dealt from a keyed permutation of the NL = ceil(n / l)
 * lines of l = pool_line consecutive points, so that every line serves the same number of pools (to within one).
 * Keys per epoch from Philox(counter (0, 0xFFFFFFFD, t, 0)) = (w0, w1, w2, w3) and (counter (1, ...)) = (w4, .., w7):
 * multipliers A = (w0|1, w2|1, w4|1), increments C = (w1, w3, w5), cyclic shift r = floor(w6 n / 2^32).  The permutation
 * works on b = max(1, ceil(log2 NL)) bits: three rounds of x <- (A_k x + C_k) mod 2^b; x <- x xor (x >> max(1, b / 2)),
 * repeated until x < NL.  Line gamma of block beta starts at (l pi((beta L + gamma) mod NL) + r) mod n. */
static uint64_t stratified_line_start(const oracle_problem* P, uint64_t n, uint64_t beta, int32_t t, uint32_t gamma, uint32_t L) {
    uint32_t key[2] = {(uint32_t)P->seed, (uint32_t)(P->seed >> 32)};
    uint32_t c0[4] = {0u, 0xFFFFFFFDu, (uint32_t)t, 0u}, c1[4] = {1u, 0xFFFFFFFDu, (uint32_t)t, 0u}, w[8];
    oracle_philox4x32_10(c0, key, w);
    oracle_philox4x32_10(c1, key, w + 4);
    const uint64_t A[3] = {w[0] | 1u, w[2] | 1u, w[4] | 1u}, C[3] = {w[1], w[3], w[5]};
    const uint64_t r = ((uint64_t)w[6] * n) >> 32;
    const uint64_t line = (uint64_t)P->pool_line, NL = (n + line - 1) / line;
    int b = 1;
    while (((uint64_t)1 << b) < NL) ++b;
    const uint64_t mask = ((uint64_t)1 << b) - 1;
    const int sh = b / 2 > 1 ? b / 2 : 1;
    uint64_t x = (beta * L + gamma) % NL;
    do {
        for (int k = 0; k < 3; ++k) {
            x = (A[k] * x + C[k]) & mask;
            x ^= x >> sh;
        }
    } while (x >= NL);
    return (line * x + r) % n;
}

static void edge_negatives(const oracle_problem* P, const oracle_tables* T, int64_t e, int64_t i, int32_t t, int32_t* m) {
    int32_t g = group_of_point(P, i);
    int64_t base = T->gstart[g];
    uint64_t nloc = (uint64_t)(T->gstart[g + 1] - base);
    uint32_t key[2] = {(uint32_t)P->seed, (uint32_t)(P->seed >> 32)};
    if (P->pool_size > 0 && (P->pool_mode == 1 || P->pool_mode == 2)) {
        const int64_t E = P->row_ptr[P->n];
        const int64_t seg = P->pool_segment;
        const int64_t NS = (E + seg - 1) / seg, Q = P->pool_block / seg;
        int64_t NB = (NS + Q - 1) / Q;
        if (NB < 1) NB = 1;
        const int64_t sigma = e / seg;
        const uint64_t beta = (uint64_t)(sigma % NB);
        const uint64_t rank = (uint64_t)(seg * (sigma / NB) + (e % seg));
        uint32_t ctr[4] = {(uint32_t)beta, 0xFFFFFFFEu, (uint32_t)t, (uint32_t)((rank & 1023) + 1024 * (rank >> 12))};
        uint32_t w[4];
        oracle_philox4x32_10(ctr, key, w);
        const uint32_t W = w[(rank >> 10) & 3];
        int lg = 0;
        while ((1 << (lg + 1)) <= P->pool_size) ++lg;
        const uint32_t PS = (uint32_t)P->pool_size, L = PS / (uint32_t)P->pool_line;
        const uint32_t u0 = W >> (32 - lg), c = 2u * ((W >> 1) & (PS / 2 - 1)) + 1u;
        for (int32_t k = 0; k < P->n_neg; ++k) {
            const uint32_t u = (u0 + (uint32_t)k * c) % PS;
            const uint32_t gamma = u % L, o = u / L;
            uint64_t start;
            if (P->pool_mode == 2) {
                start = stratified_line_start(P, nloc, beta, t, gamma, L);
            } else {
                uint32_t pctr[4] = {(uint32_t)beta, 0xFFFFFFFFu, (uint32_t)t, gamma >> 2};
                uint32_t pw[4];
                oracle_philox4x32_10(pctr, key, pw);
                start = ((uint64_t)pw[gamma & 3] * nloc) >> 32;
            }
            m[k] = T->members[base + (int64_t)((start + o) % nloc)];
        }
        return;
    }
    if (P->pool_size > 0) {
        uint64_t beta = (uint64_t)e / (uint64_t)P->pool_block;
        for (int32_t k = 0; k < P->n_neg; ++k) {
            uint32_t ctr[4] = {(uint32_t)(uint64_t)e, (uint32_t)((uint64_t)e >> 32), (uint32_t)t, (uint32_t)(k >> 3)};
            uint32_t w[4], pw[4];
            oracle_philox4x32_10(ctr, key, w);
            uint32_t x16 = (w[(k >> 1) & 3] >> (16 * (k & 1))) & 0xFFFFu;
            uint32_t u = (x16 * (uint32_t)P->pool_size) >> 16;
            uint32_t pctr[4] = {(uint32_t)beta, 0xFFFFFFFFu, (uint32_t)t, u >> 2};
            oracle_philox4x32_10(pctr, key, pw);
            uint64_t pt = ((uint64_t)pw[u & 3] * nloc) >> 32;
            m[k] = T->members[base + (int64_t)pt];
        }
        return;
    }
    for (int32_t blk = 0; 4 * blk < P->n_neg; ++blk) {
        uint32_t ctr[4] = {(uint32_t)(uint64_t)e, (uint32_t)((uint64_t)e >> 32), (uint32_t)t, (uint32_t)blk};
        uint32_t w[4];
        oracle_philox4x32_10(ctr, key, w);
        for (int32_t lane = 0; lane < 4 && 4 * blk + lane < P->n_neg; ++lane) {
            if (P->sampled_far_field) {
                m[4 * blk + lane] = (int32_t)(((uint64_t)w[lane] * (uint64_t)P->n) >> 32);
                continue;
            }
            uint64_t u = ((uint64_t)w[lane] * nloc) >> 32;
            m[4 * blk + lane] = T->members[base + (int64_t)u];
        }
    }
}

int oracle_negatives(const oracle_problem* P, int32_t t, int64_t e_begin, int64_t e_end, int32_t* out) {
    oracle_tables T;
    if (build_tables(P, &T)) return -1;
    int64_t s = P->n_neg;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < P->n; ++i) {
        int64_t a = P->row_ptr[i], b = P->row_ptr[i + 1];
        if (b <= e_begin || a >= e_end) continue;
        for (int64_t e = (a > e_begin ? a : e_begin); e < b && e < e_end; ++e)
            edge_negatives(P, &T, e, i, t, out + (e - e_begin) * s);
    }
    free_tables(&T);
    return 0;
}

/* cell sizes and means */
int oracle_cluster_stats(const oracle_problem* P, const float* theta, int64_t* counts, double* mu) {
    int32_t R = P->n_clusters;
    memset(counts, 0, sizeof(int64_t) * (size_t)R);
    memset(mu, 0, sizeof(double) * 2 * (size_t)R);
    for (int64_t i = 0; i < P->n; ++i) {
        int32_t r = P->cluster_of[i];
        if (r < 0 || r >= R) return -1;
        counts[r]++;
        mu[2 * r] += (double)theta[2 * i];
        mu[2 * r + 1] += (double)theta[2 * i + 1];
    }
    for (int32_t r = 0; r < R; ++r)
        if (counts[r]) { mu[2 * r] /= (double)counts[r]; mu[2 * r + 1] /= (double)counts[r]; }
    return 0;
}

static inline double cauchy(double ax, double ay, double bx, double by) {
    double dx = ax - bx, dy = ay - by;
    return 1.0 / (1.0 + dx * dx + dy * dy);
}

/* A_i = sum_{r in Rtilde_i} p_r q(theta_i, mu_r) and B_i = sum p_r q^2 (theta_i - mu_r): Eq. 5 without
   its |M| factor, and the factor of its derivative.  Rtilde_i = cells whose group differs from gi. */
static void mean_field_sums(const oracle_problem* P, const int64_t* counts, const double* mu, double xi, double yi,
                            int32_t gi, double* Ai, double* Bx, double* By) {
    *Ai = 0.0; *Bx = 0.0; *By = 0.0;
    if (!P->cluster_group || P->sampled_far_field) return;
    for (int32_t r = 0; r < P->n_clusters; ++r) {
        if (P->cluster_group[r] == gi || counts[r] == 0) continue;
        const double pr = (double)counts[r] / (double)P->n;
        const double q = cauchy(xi, yi, mu[2 * r], mu[2 * r + 1]);
        *Ai += pr * q;
        *Bx += pr * q * q * (xi - mu[2 * r]);
        *By += pr * q * q * (yi - mu[2 * r + 1]);
    }
}

/*
 * Sampled loss L_t(theta) and g = grad(n * L_t) with the negatives of epoch index t.
 *   loss   : out, may be NULL
 *   grad   : out [n*2] (or [n_targets*2] when target_slot is given), may be NULL
 *   target_slot : NULL, or int32 [n] with the output slot of each wanted point and -1
 *                 elsewhere.  Then only edges that touch a wanted point (as head, tail or
 *                 sampled negative) are evaluated and `loss` is not meaningful; this is how
 *                 single outputs are computed one by one at sizes where the full pass (and
 *                 above all the full mean-field sum) is out of reach.
 *   A_out, B_out: NULL or out [n], [n*2]: the mean-field sums (full mode only).
 *   mu_fixed: NULL, or [|R|*2] cell means to use instead of the means of theta (the gradient
 *             holds the means constant; a finite-difference check has to do the same).
 */
int oracle_loss_grad(const oracle_problem* P, const float* theta, int32_t t, double* loss, double* grad,
                     const int32_t* target_slot, int64_t n_targets, double* A_out, double* B_out,
                     const double* mu_fixed) {
    oracle_tables T;
    if (build_tables(P, &T)) return -1;
    const int64_t n = P->n;
    const int32_t R = P->n_clusters, s = P->n_neg;
    const double Mn = P->noise_count;
    int64_t* counts = (int64_t*)malloc(sizeof(int64_t) * (size_t)R);
    double* mu = (double*)malloc(sizeof(double) * 2 * (size_t)R);
    oracle_cluster_stats(P, theta, counts, mu);
    if (mu_fixed) memcpy(mu, mu_fixed, sizeof(double) * 2 * (size_t)R);
    const int64_t gn = target_slot ? n_targets : n;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    double* gbuf = NULL;
    if (grad) gbuf = (double*)calloc((size_t)nthreads * (size_t)gn * 2, sizeof(double));
    const int through_means = P->mean_gradient && P->cluster_group && grad;
    if (through_means && (target_slot || P->sampled_far_field)) { free(counts); free(mu); free(gbuf); free_tables(&T); return -3; }
    double* mbuf = through_means ? (double*)calloc((size_t)nthreads * (size_t)R * 2, sizeof(double)) : NULL; /* d(nL)/d mu_r */
    double total = 0.0;
    int bad = 0;

#pragma omp parallel reduction(+ : total)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double* g = gbuf ? gbuf + (size_t)tid * (size_t)gn * 2 : NULL;
        double* gm = mbuf ? mbuf + (size_t)tid * (size_t)R * 2 : NULL;
        int32_t* m = (int32_t*)malloc(sizeof(int32_t) * (size_t)(s > 0 ? s : 1));
        double* qim = (double*)malloc(sizeof(double) * (size_t)(s > 0 ? s : 1));
        double* nx = (double*)malloc(sizeof(double) * (size_t)(s > 0 ? s : 1));   /* where each negative sits */
        double* ny = (double*)malloc(sizeof(double) * (size_t)(s > 0 ? s : 1));
        int* moved = (int*)malloc(sizeof(int) * (size_t)(s > 0 ? s : 1));          /* does it receive its force? */
        const int64_t h0 = P->head_end >= 0 ? P->head_begin : 0;
        const int64_t h1 = P->head_end >= 0 ? P->head_end : n;
#pragma omp for schedule(dynamic, 256)
        for (int64_t i = h0; i < h1; ++i) {
            const int64_t ea = P->row_ptr[i], eb = P->row_ptr[i + 1];
            const double xi = theta[2 * i], yi = theta[2 * i + 1];
            const int32_t gi = group_of_point(P, i);
            const double nloc = (double)(T.gstart[gi + 1] - T.gstart[gi]);
            const double om = s > 0 ? Mn * (P->sampled_far_field ? 1.0 : nloc / (double)n) / (double)s : 0.0;
            double wsum = 0.0;
            if (P->weights)
                for (int64_t e = ea; e < eb; ++e) wsum += (double)P->weights[e];
            int have_mf = 0;
            double Ai = 0.0, Bx = 0.0, By = 0.0;
            if (!target_slot) { /* full mode: the sums of every head, edges or not */
                have_mf = 1;
                mean_field_sums(P, counts, mu, xi, yi, gi, &Ai, &Bx, &By);
                if (A_out) { A_out[i] = Ai; B_out[2 * i] = Bx; B_out[2 * i + 1] = By; }
            }
            const int head_wanted = !target_slot || target_slot[i] >= 0;
            double c_head = 0.0; /* sum over the row of 2 p_e / S_e */
            for (int64_t e = ea; e < eb; ++e) {
                const int64_t j = P->col_idx[e];
                if (j < 0 || j >= n) {
#pragma omp atomic write
                    bad = 1;
                    continue;
                }
                edge_negatives(P, &T, e, i, t, m);
                if (target_slot) {
                    int touch = head_wanted || target_slot[j] >= 0;
                    for (int32_t k = 0; k < s && !touch; ++k) touch = target_slot[m[k]] >= 0;
                    if (!touch) continue;
                }
                if (!have_mf) { /* target mode: only heads with a touched edge pay for the sums */
                    have_mf = 1;
                    mean_field_sums(P, counts, mu, xi, yi, gi, &Ai, &Bx, &By);
                }
                const double pe = P->weights ? (double)P->weights[e] / wsum : 1.0 / (double)(eb - ea);
                const double dx = xi - (double)theta[2 * j], dy = yi - (double)theta[2 * j + 1];
                const double qij = 1.0 / (1.0 + dx * dx + dy * dy);
                double qs = 0.0;
                for (int32_t k = 0; k < s; ++k) {
                    /* sampled far field: a negative of another group stands for its cell and enters through the mean */
                    const int32_t rk = P->cluster_of[m[k]];
                    const int far = P->sampled_far_field && P->cluster_group && P->cluster_group[rk] != gi;
                    nx[k] = far ? mu[2 * rk] : (double)theta[2 * (int64_t)m[k]];
                    ny[k] = far ? mu[2 * rk + 1] : (double)theta[2 * (int64_t)m[k] + 1];
                    moved[k] = !far;
                    qim[k] = cauchy(xi, yi, nx[k], ny[k]);
                    qs += qim[k];
                }
                const double S = qij + Mn * Ai + om * qs;
                total += pe * (-log(qij) + log(S));
                if (!g) continue;
                const int64_t si = target_slot ? target_slot[i] : i;
                const int64_t sj = target_slot ? target_slot[j] : j;
                const double a = 2.0 * pe * qij * (1.0 - qij / S);
                if (si >= 0) { g[2 * si] += a * dx; g[2 * si + 1] += a * dy; }
                if (sj >= 0) { g[2 * sj] -= a * dx; g[2 * sj + 1] -= a * dy; }
                for (int32_t k = 0; k < s; ++k) {
                    const int64_t mk = m[k];
                    const int64_t sm = target_slot ? target_slot[mk] : mk;
                    const double ex = xi - nx[k], ey = yi - ny[k];
                    const double b = 2.0 * pe * om * qim[k] * qim[k] / S;
                    if (si >= 0) { g[2 * si] -= b * ex; g[2 * si + 1] -= b * ey; }
                    if (sm >= 0 && moved[k]) { g[2 * sm] += b * ex; g[2 * sm + 1] += b * ey; }
                }
                if (si >= 0) {
                    const double c = 2.0 * pe * Mn / S;
                    g[2 * si] -= c * Bx;
                    g[2 * si + 1] -= c * By;
                }
                c_head += 2.0 * pe / S;
            }
            if (gm && c_head != 0.0) /* d S_e / d mu_r = |M| p_r 2 q^2 (theta_i - mu_r) for every approximated cell r */
                for (int32_t r = 0; r < R; ++r) {
                    if (P->cluster_group[r] == gi || counts[r] == 0) continue;
                    const double pr = (double)counts[r] / (double)n;
                    const double q = cauchy(xi, yi, mu[2 * r], mu[2 * r + 1]);
                    gm[2 * r] += c_head * Mn * pr * q * q * (xi - mu[2 * r]);
                    gm[2 * r + 1] += c_head * Mn * pr * q * q * (yi - mu[2 * r + 1]);
                }
        }
        free(m);
        free(qim);
        free(nx); free(ny); free(moved);
    }
    if (grad) {
#pragma omp parallel for schedule(static)
        for (int64_t x = 0; x < gn * 2; ++x) {
            double acc = 0.0;
            for (int th = 0; th < nthreads; ++th) acc += gbuf[(size_t)th * (size_t)gn * 2 + (size_t)x];
            grad[x] = acc;
        }
        free(gbuf);
        if (mbuf) {
            for (int32_t r = 0; r < R; ++r)
                for (int th = 1; th < nthreads; ++th) {
                    mbuf[2 * r] += mbuf[(size_t)th * (size_t)R * 2 + 2 * r];
                    mbuf[2 * r + 1] += mbuf[(size_t)th * (size_t)R * 2 + 2 * r + 1];
                }
            for (int64_t l = 0; l < n; ++l) { /* mu_r is the mean of its members: each takes 1/n_r of its gradient */
                const int32_t r = P->cluster_of[l];
                grad[2 * l] += mbuf[2 * r] / (double)counts[r];
                grad[2 * l + 1] += mbuf[2 * r + 1] / (double)counts[r];
            }
            free(mbuf);
        }
    }
    if (loss) *loss = total / (double)n;
    free(counts); free(mu);
    free_tables(&T);
    return bad ? -2 : 0;
}

/* Mean-field sums of single heads: A [n_heads], B [n_heads*2] for the listed points, each from the plain loop over
 * all cells (Eq. 5 without |M|, and the factor of its derivative), with the cell means of theta.  The way to check
 * these sums at sizes where the sums of every head are out of reach. */
int oracle_mean_field_at(const oracle_problem* P, const float* theta, const int64_t* heads, int64_t n_heads, double* A,
                         double* B) {
    const int32_t R = P->n_clusters;
    int64_t* counts = (int64_t*)malloc(sizeof(int64_t) * (size_t)R);
    double* mu = (double*)malloc(sizeof(double) * 2 * (size_t)R);
    int rc = oracle_cluster_stats(P, theta, counts, mu);
    for (int64_t h = 0; h < n_heads && rc == 0; ++h) {
        const int64_t i = heads[h];
        if (i < 0 || i >= P->n) { rc = -1; break; }
        mean_field_sums(P, counts, mu, (double)theta[2 * i], (double)theta[2 * i + 1], group_of_point(P, i), &A[h], &B[2 * h],
                        &B[2 * h + 1]);
    }
    free(counts); free(mu);
    return rc;
}

/* One epoch in place.  B = batches_per_epoch sequential sub-steps: sub-step b takes the heads
 * floor(n b / B) .. floor(n (b+1) / B) - 1, evaluates the gradient of their edges at the current theta with the
 * cell means of the start of the epoch, and applies theta <- fp32(theta - lr0 (1 - t/T) g_b).  B = 1 is the
 * full-batch step.  grad_out (may be NULL) receives the gradient of the last sub-step; loss_out (may be NULL)
 * the sum of the sub-steps' loss terms, each at the theta it was evaluated at (B = 1: the loss at theta). */
int oracle_epoch(const oracle_problem* P, float* theta, int32_t t, int32_t T_epochs, double lr0, double* grad_out,
                 double* loss_out) {
    const int64_t n = P->n;
    const int32_t B = P->batches_per_epoch > 1 ? P->batches_per_epoch : 1;
    const int32_t R = P->n_clusters;
    double* g = grad_out ? grad_out : (double*)malloc(sizeof(double) * 2 * (size_t)n);
    int64_t* counts = (int64_t*)malloc(sizeof(int64_t) * (size_t)R);
    double* mu0 = (double*)malloc(sizeof(double) * 2 * (size_t)R);
    oracle_cluster_stats(P, theta, counts, mu0);
    const double eta = lr0 * (1.0 - (double)t / (double)T_epochs);
    double total = 0.0;
    int rc = 0;
    for (int32_t b = 0; b < B && rc == 0; ++b) {
        oracle_problem Pb = *P;
        Pb.head_begin = n * (int64_t)b / B;
        Pb.head_end = n * (int64_t)(b + 1) / B;
        double part = 0.0;
        rc = oracle_loss_grad(&Pb, theta, t, &part, g, NULL, 0, NULL, NULL, mu0);
        total += part;
        if (rc == 0)
            for (int64_t x = 0; x < 2 * n; ++x) theta[x] = (float)((double)theta[x] - eta * g[x]);
    }
    if (loss_out) *loss_out = total;
    free(counts); free(mu0);
    if (!grad_out) free(g);
    return rc;
}

/* epochs t_begin .. t_end-1 in place; loss_curve (may be NULL) gets L at the start of each. */
int oracle_train(const oracle_problem* P, float* theta, int32_t t_begin, int32_t t_end, int32_t T_epochs, double lr0,
                 double* loss_curve) {
    double* g = (double*)malloc(sizeof(double) * 2 * (size_t)P->n);
    int rc = 0;
    for (int32_t t = t_begin; t < t_end && rc == 0; ++t)
        rc = oracle_epoch(P, theta, t, T_epochs, lr0, g, loss_curve ? loss_curve + (t - t_begin) : NULL);
    free(g);
    return rc;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

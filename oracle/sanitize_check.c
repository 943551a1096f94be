/*
 * Driver for a sanitizer build of the C oracle -- TEST INFRASTRUCTURE, NOT PRODUCT.
 *
 * tests/test_oracle_sanitized.py compiles nomad_oracle.c together with this file under
 * -fsanitize=address,undefined and runs it on problems it writes to a directory; every entry
 * point of the oracle is called once, and a few sums of the results are printed so that the
 * test can hold them against the ordinary build.  Holds no arithmetic of the method.
 *
 * usage: sanitize_check DIR n E R s noise pool_size pool_block pool_mode pool_line pool_segment batches sampled mean_gradient
 * files in DIR: row_ptr.i32 col.i32 cluster.i32 theta.f32, optional weights.f32 group.i32
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int64_t n;
    const int32_t* row_ptr;
    const int32_t* col_idx;
    const float* weights;
    const int32_t* cluster_of;
    int32_t n_clusters;
    const int32_t* cluster_group;
    int32_t n_neg;
    double noise_count;
    uint64_t seed;
    int32_t pool_size, pool_block, batches_per_epoch;
    int64_t head_begin, head_end;
    int32_t sampled_far_field, mean_gradient, pool_mode, pool_line, pool_segment;
} oracle_problem;   /* the layout nomad_oracle.c declares */

int oracle_negatives(const oracle_problem*, int32_t, int64_t, int64_t, int32_t*);
int oracle_cluster_stats(const oracle_problem*, const float*, int64_t*, double*);
int oracle_loss_grad(const oracle_problem*, const float*, int32_t, double*, double*, const int32_t*, int64_t, double*, double*,
                     const double*);
int oracle_mean_field_at(const oracle_problem*, const float*, const int64_t*, int64_t, double*, double*);
int oracle_epoch(const oracle_problem*, float*, int32_t, int32_t, double, double*, double*);
int oracle_train(const oracle_problem*, float*, int32_t, int32_t, int32_t, double, double*);

static void* slurp(const char* dir, const char* name, size_t bytes, int optional) {
    char path[1024];
    snprintf(path, sizeof(path), "%s/%s", dir, name);
    FILE* f = fopen(path, "rb");
    if (!f) {
        if (optional) return NULL;
        fprintf(stderr, "missing %s\n", path);
        exit(2);
    }
    void* p = malloc(bytes ? bytes : 1);
    if (fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short read of %s\n", path); exit(2); }
    fclose(f);
    return p;
}

static double weighted_sum(const double* v, int64_t count) {
    double s = 0.0;
    for (int64_t x = 0; x < count; ++x) s += v[x] * (double)(x % 97 + 1);
    return s;
}

int main(int argc, char** argv) {
    if (argc != 15) return 2;
    const char* dir = argv[1];
    oracle_problem P;
    memset(&P, 0, sizeof(P));
    P.n = atoll(argv[2]);
    const int64_t E = atoll(argv[3]);
    P.n_clusters = atoi(argv[4]);
    P.n_neg = atoi(argv[5]);
    P.noise_count = atof(argv[6]);
    P.pool_size = atoi(argv[7]); P.pool_block = atoi(argv[8]); P.pool_mode = atoi(argv[9]); P.pool_line = atoi(argv[10]);
    P.pool_segment = atoi(argv[11]); P.batches_per_epoch = atoi(argv[12]); P.sampled_far_field = atoi(argv[13]);
    P.mean_gradient = atoi(argv[14]);
    P.seed = 0x1234567890ull;
    P.head_begin = 0; P.head_end = -1;
    P.row_ptr = (const int32_t*)slurp(dir, "row_ptr.i32", 4 * (size_t)(P.n + 1), 0);
    P.col_idx = (const int32_t*)slurp(dir, "col.i32", 4 * (size_t)E, 0);
    P.cluster_of = (const int32_t*)slurp(dir, "cluster.i32", 4 * (size_t)P.n, 0);
    P.weights = (const float*)slurp(dir, "weights.f32", 4 * (size_t)E, 1);
    P.cluster_group = (const int32_t*)slurp(dir, "group.i32", 4 * (size_t)P.n_clusters, 1);
    float* theta = (float*)slurp(dir, "theta.f32", 8 * (size_t)P.n, 0);
    const int64_t n = P.n;
    const int32_t s = P.n_neg;

    int32_t* neg = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E * s + 1));
    if (oracle_negatives(&P, 3, 0, E, neg)) return 3;
    long long nsum = 0;
    for (int64_t x = 0; x < E * s; ++x) nsum += (long long)neg[x] * (x % 31 + 1);
    printf("negatives %lld\n", nsum);

    double loss = 0.0;
    double* g = (double*)malloc(sizeof(double) * 2 * (size_t)n);
    double* A = (double*)malloc(sizeof(double) * (size_t)n);
    double* B = (double*)malloc(sizeof(double) * 2 * (size_t)n);
    if (oracle_loss_grad(&P, theta, 3, &loss, g, NULL, 0, A, B, NULL)) return 4;
    printf("loss %.17g\ngrad %.17g\nA %.17g\nB %.17g\n", loss, weighted_sum(g, 2 * n), weighted_sum(A, n), weighted_sum(B, 2 * n));

    if (!P.mean_gradient) {   /* single rows: the last point, the first, one in the middle */
        int32_t* slot = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
        for (int64_t i = 0; i < n; ++i) slot[i] = -1;
        slot[n - 1] = 0; slot[0] = 1; slot[n / 2] = 2;
        double rows[6];
        if (oracle_loss_grad(&P, theta, 3, NULL, rows, slot, 3, NULL, NULL, NULL)) return 5;
        printf("rows %.17g %.17g %.17g %.17g %.17g %.17g\n", rows[0], rows[1], rows[2], rows[3], rows[4], rows[5]);
        free(slot);
    }
    int64_t heads[3] = {n - 1, 0, n / 2};
    double hA[3], hB[6];
    if (oracle_mean_field_at(&P, theta, heads, 3, hA, hB)) return 6;
    printf("mean_field_at %.17g %.17g\n", hA[0] + 2 * hA[1] + 3 * hA[2], weighted_sum(hB, 6));

    float* th = (float*)malloc(8 * (size_t)n);
    memcpy(th, theta, 8 * (size_t)n);
    double eloss = 0.0;
    if (oracle_epoch(&P, th, 1, 4, 0.3, g, &eloss)) return 7;
    double tsum = 0.0;
    for (int64_t x = 0; x < 2 * n; ++x) tsum += (double)th[x] * (double)(x % 97 + 1);
    printf("epoch %.17g %.17g\n", eloss, tsum);
    double curve[3];
    if (oracle_train(&P, th, 1, 4, 4, 0.3, curve)) return 8;
    tsum = 0.0;
    for (int64_t x = 0; x < 2 * n; ++x) tsum += (double)th[x] * (double)(x % 97 + 1);
    printf("train %.17g %.17g\n", curve[2], tsum);

    free(neg); free(g); free(A); free(B); free(th); free(theta);
    free((void*)P.row_ptr); free((void*)P.col_idx); free((void*)P.cluster_of); free((void*)P.weights); free((void*)P.cluster_group);
    return 0;
}

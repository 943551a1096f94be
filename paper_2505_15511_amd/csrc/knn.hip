// libnomad: the upstream index (K-Means, in-cluster exact nearest neighbours) and the quality measures behind the C ABI of
// include/nomad.h (host side).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <vector>

#include "host_util.h"
#include "knn_kernels.h"
#include "metrics_kernels.h"
#include "nomad.h"

using namespace nomad_knn;
using namespace nomad_metrics;

namespace {


template <int D4, int L>
hipError_t launch_filter_dl(hipStream_t st, uint32_t n_blocks, const KnnSets& P, const KnnBlock* blocks, int32_t list_len, int32_t* cand,
                            float* tau) {
    const size_t lds = knn_filter_lds_bytes(D4, L);
    hipError_t e = hipFuncSetAttribute((const void*)k_knn_filter<D4, L>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_knn_filter<D4, L>), dim3(n_blocks), dim3(64 * knn_filter_waves(D4)), lds, st, P, blocks, list_len, cand, tau);
    return hipGetLastError();
}

template <int D4>
hipError_t launch_filter_d(hipStream_t st, uint32_t n_blocks, const KnnSets& P, const KnnBlock* blocks, int32_t list_len, int32_t* cand,
                           float* tau) {
    switch (knn_filter_list_class(list_len)) {
        case 2: return launch_filter_dl<D4, 2>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 8: return launch_filter_dl<D4, 8>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 12: return launch_filter_dl<D4, 12>(st, n_blocks, P, blocks, list_len, cand, tau);
        default: return launch_filter_dl<D4, 20>(st, n_blocks, P, blocks, list_len, cand, tau);
    }
}

// width class of the filter kernel for rows of d values
inline int width_class(int32_t d) {
    const int d4 = (d + 3) / 4;
    return d4 <= 8 ? 8 : d4 <= 16 ? 16 : d4 <= 32 ? 32 : d4 <= 64 ? 64 : d4 <= 96 ? 96 : d4 <= 128 ? 128 : 192;
}

hipError_t launch_filter(hipStream_t st, uint32_t n_blocks, const KnnSets& P, const KnnBlock* blocks, int32_t list_len, int32_t* cand,
                         float* tau) {
    switch (width_class(P.d)) {
        case 8: return launch_filter_d<8>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 16: return launch_filter_d<16>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 32: return launch_filter_d<32>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 64: return launch_filter_d<64>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 96: return launch_filter_d<96>(st, n_blocks, P, blocks, list_len, cand, tau);
        case 128: return launch_filter_d<128>(st, n_blocks, P, blocks, list_len, cand, tau);
        default: return launch_filter_d<192>(st, n_blocks, P, blocks, list_len, cand, tau);
    }
}

// The k nearest candidates of every query inside its group (filter, refinement, exact fallback).  `cand` [n_q * (k + kPad)],
// `tau` [n_q], `flagged` [n_q], `n_flagged` [1] are work space; blocks: the filter's work list (n_blocks entries).
int nearest_in_groups(hipStream_t st, const KnnSets& P, const KnnBlock* blocks, uint32_t n_blocks, int32_t k, int32_t* cand, float* tau,
                      int32_t* flagged, uint32_t* n_flagged, int32_t* out, uint32_t* flagged_count) {
    const int32_t list_len = k + kPad;
    KTRY(hipMemsetAsync(cand, 0xFF, sizeof(int32_t) * (size_t)P.n_q * list_len, st));   // every slot "no candidate" until the filter fills it
    KTRY(hipMemsetAsync(n_flagged, 0, sizeof(uint32_t), st));
    KTRY(launch_filter(st, n_blocks, P, blocks, list_len, cand, tau));
    if (list_len <= 16)
        hipLaunchKernelGGL(k_knn_refine<16>, dim3(blocks_of(P.n_q, 16)), dim3(256), 0, st, P, cand, tau, k, list_len, out, flagged, n_flagged);
    else if (list_len <= 32)
        hipLaunchKernelGGL(k_knn_refine<32>, dim3(blocks_of(P.n_q, 8)), dim3(256), 0, st, P, cand, tau, k, list_len, out, flagged, n_flagged);
    else
        hipLaunchKernelGGL(k_knn_refine<64>, dim3(blocks_of(P.n_q, 4)), dim3(256), 0, st, P, cand, tau, k, list_len, out, flagged, n_flagged);
    uint32_t hflag = 0;
    KTRY(hipMemcpyAsync(&hflag, n_flagged, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (hflag && k <= 16) hipLaunchKernelGGL(k_knn_exact<16>, dim3(hflag), dim3(256), 0, st, P, flagged, k, out);
    else if (hflag) hipLaunchKernelGGL(k_knn_exact<kMaxK>, dim3(hflag), dim3(256), 0, st, P, flagged, k, out);
    KTRY(hipGetLastError());
    *flagged_count = hflag;
    return NOMAD_OK;
}

// The M step of Lloyd's iteration: the points sorted by label with a stable radix sort (ascending point order inside a
// cluster), then float64 sums in that order per (centroid, column); a label without points leaves its centroid as it is.
struct MeanStep {
    int64_t n = 0;
    int32_t K = 0;
    int passes = 1;                 // radix passes of 8 bits that cover the labels 0..K-1
    uint32_t n_blocks = 0;          // workgroups of a sort pass
    uint32_t *counts = nullptr, *lstart = nullptr, *hist = nullptr, *tile_total = nullptr;
    uint32_t n_tiles = 0;           // tiles of the scan over the 256 n_blocks digit counters
    int32_t *keys[2] = {nullptr, nullptr}, *ids[2] = {nullptr, nullptr};   // a pass reads one pair of arrays and writes the other
    int* bad = nullptr;
    std::vector<uint32_t> hcounts, hstart;

    int init(Buffers& buf, hipStream_t, int64_t n_, int32_t K_) {
        n = n_; K = K_;
        hcounts.assign((size_t)K, 0u);
        hstart.assign((size_t)K + 1, 0u);
        int bits = 1;
        while (((int64_t)1 << bits) < K) ++bits;
        passes = (bits + 7) / 8;
        n_blocks = blocks_of(n, kSortSpan);
        KTRY(buf.alloc(&counts, (size_t)K)); KTRY(buf.alloc(&lstart, (size_t)K + 1)); KTRY(buf.alloc(&bad, 1));
        n_tiles = (uint32_t)(((size_t)256 * n_blocks + kScanTile - 1) / kScanTile);
        KTRY(buf.alloc(&hist, (size_t)256 * n_blocks));
        KTRY(buf.alloc(&tile_total, (size_t)n_tiles));
        for (int x = 0; x < (passes > 1 ? 2 : 1); ++x) { KTRY(buf.alloc(&keys[x], (size_t)n)); KTRY(buf.alloc(&ids[x], (size_t)n)); }
        return NOMAD_OK;
    }
    // labels [n] in 0..K-1 (on the device); dC [K * d] in and out
    int run(hipStream_t st, const float* dX, int32_t d, const int32_t* labels, float* dC) {
        KTRY(hipMemsetAsync(counts, 0, sizeof(uint32_t) * (size_t)K, st));
        KTRY(hipMemsetAsync(bad, 0, sizeof(int), st));
        hipLaunchKernelGGL(k_knn_count, dim3(blocks_of(n, kCountSpan)), dim3(256), 0, st, labels, n, K, counts, bad);
        KTRY(hipMemcpyAsync(hcounts.data(), counts, sizeof(uint32_t) * (size_t)K, hipMemcpyDeviceToHost, st));
        KTRY(hipStreamSynchronize(st));
        for (int32_t j = 0; j < K; ++j) hstart[j + 1] = hstart[j] + hcounts[j];
        KTRY(hipMemcpyAsync(lstart, hstart.data(), sizeof(uint32_t) * ((size_t)K + 1), hipMemcpyHostToDevice, st));
        const int32_t* kin = labels;
        const int32_t* vin = nullptr;   // first pass: the point at position i is i
        int out = 0;
        for (int p = 0; p < passes; ++p) {
            hipLaunchKernelGGL(k_sort_count, dim3(n_blocks), dim3(256), 0, st, kin, n, 8 * p, n_blocks, hist);
            hipLaunchKernelGGL(k_sort_scan_tiles, dim3(n_tiles), dim3(256), 0, st, hist, (uint64_t)256 * n_blocks, tile_total);
            hipLaunchKernelGGL(k_sort_scan, dim3(1), dim3(1024), 0, st, tile_total, (uint64_t)n_tiles);
            hipLaunchKernelGGL(k_sort_scatter, dim3(n_blocks), dim3(256), 0, st, kin, vin, n, 8 * p, n_blocks, (const uint32_t*)hist,
                               (const uint32_t*)tile_total, keys[out], ids[out]);
            kin = keys[out]; vin = ids[out];
            out ^= 1;
        }
        hipLaunchKernelGGL(k_kmeans_update, dim3(blocks_of((int64_t)K * d, 256)), dim3(256), 0, st, dX, d, vin, (const uint32_t*)lstart, K, dC);
        KTRY(hipGetLastError());
        return NOMAD_OK;
    }
};

}  // namespace

#pragma GCC visibility push(default)
extern "C" int nomad_knn_in_clusters(const float* X, int64_t n, int32_t d, const int32_t* cluster_of, int32_t n_clusters, int32_t k,
                                     int32_t* out_nbrs, int mem, int32_t device, void* stream, int64_t* stats) {
    if (!X || !cluster_of || !out_nbrs || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return NOMAD_E_INVALID_ARG;
    if (n < 1 || d < 1 || d > NOMAD_KNN_MAX_DIM || n_clusters < 1 || k < 1 || k > NOMAD_KNN_MAX_K || device < 0) return NOMAD_E_INVALID_ARG;
    if (n >= ((int64_t)1 << 31) - 256) return NOMAD_E_TOO_LARGE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    Buffers buf;
    const int32_t R = n_clusters;
    const int32_t list_len = k + kPad;

    // inputs on the device
    const float* dX = X;
    const int32_t* dC = cluster_of;
    int32_t* dOut = out_nbrs;
    if (mem == NOMAD_HOST) {
        float* x = nullptr;
        int32_t *c = nullptr, *o = nullptr;
        KTRY(buf.alloc(&x, (size_t)n * d));
        KTRY(buf.alloc(&c, (size_t)n));
        KTRY(buf.alloc(&o, (size_t)n * k));
        KTRY(hipMemcpyAsync(x, X, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice, st));
        KTRY(hipMemcpyAsync(c, cluster_of, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice, st));
        dX = x; dC = c; dOut = o;
    }

    // members grouped by cluster
    uint32_t *counts = nullptr, *start = nullptr, *cursor = nullptr, *max_norm = nullptr, *n_flagged = nullptr;
    int32_t *members = nullptr, *cand = nullptr, *flagged = nullptr;
    float *norm = nullptr, *tau = nullptr, *centre = nullptr;
    int* bad = nullptr;
    KTRY(buf.alloc(&counts, (size_t)R));
    KTRY(buf.alloc(&start, (size_t)R + 1));
    KTRY(buf.alloc(&cursor, (size_t)R));
    KTRY(buf.alloc(&max_norm, (size_t)R));
    KTRY(buf.alloc(&n_flagged, 1));
    KTRY(buf.alloc(&bad, 1));
    KTRY(buf.alloc(&members, (size_t)n));
    KTRY(buf.alloc(&norm, (size_t)n));
    KTRY(buf.alloc(&tau, (size_t)n));
    KTRY(buf.alloc(&centre, (size_t)R * d));
    KTRY(hipMemsetAsync(centre, 0, sizeof(float) * (size_t)R * d, st));
    KTRY(buf.alloc(&cand, (size_t)n * list_len));
    KTRY(buf.alloc(&flagged, (size_t)n));
    KTRY(hipMemsetAsync(counts, 0, sizeof(uint32_t) * (size_t)R, st));
    KTRY(hipMemsetAsync(cursor, 0, sizeof(uint32_t) * (size_t)R, st));
    KTRY(hipMemsetAsync(max_norm, 0, sizeof(uint32_t) * (size_t)R, st));
    KTRY(hipMemsetAsync(bad, 0, sizeof(int), st));
    hipLaunchKernelGGL(k_knn_count, dim3(blocks_of(n, kCountSpan)), dim3(256), 0, st, dC, n, R, counts, bad);
    std::vector<uint32_t> hcounts(R), hstart((size_t)R + 1, 0);
    int hbad = 0;
    KTRY(hipMemcpyAsync(hcounts.data(), counts, sizeof(uint32_t) * (size_t)R, hipMemcpyDeviceToHost, st));
    KTRY(hipMemcpyAsync(&hbad, bad, sizeof(int), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (hbad) return NOMAD_E_BAD_GRAPH;   // a cluster id outside 0..n_clusters-1
    // the width class of the filter kernel decides how many queries a workgroup takes
    const uint32_t block_queries = (uint32_t)knn_filter_block_queries(width_class(d));
    std::vector<KnnBlock> hblocks, hslabs;
    for (int32_t r = 0; r < R; ++r) {
        hstart[r + 1] = hstart[r] + hcounts[r];
        for (uint32_t q0 = 0; q0 < hcounts[r]; q0 += block_queries) hblocks.push_back(KnnBlock{r, (int32_t)q0});
        for (uint32_t q0 = 0; q0 < hcounts[r]; q0 += kCentroidRows) hslabs.push_back(KnnBlock{r, (int32_t)q0});
    }
    KnnBlock *blocks = nullptr, *slabs = nullptr;
    KTRY(buf.alloc(&blocks, hblocks.size()));
    KTRY(buf.alloc(&slabs, hslabs.size()));
    KTRY(hipMemcpyAsync(slabs, hslabs.data(), sizeof(KnnBlock) * hslabs.size(), hipMemcpyHostToDevice, st));
    KTRY(hipMemcpyAsync(start, hstart.data(), sizeof(uint32_t) * ((size_t)R + 1), hipMemcpyHostToDevice, st));
    KTRY(hipMemcpyAsync(blocks, hblocks.data(), sizeof(KnnBlock) * hblocks.size(), hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(k_knn_group, dim3(blocks_of(n, kGroupSpan)), dim3(256), 0, st, dC, n, R, start, cursor, members);
    hipLaunchKernelGGL(k_knn_centroid_sums, dim3((uint32_t)hslabs.size()), dim3(256), 0, st, dX, d, members, start, slabs, centre);
    hipLaunchKernelGGL(k_knn_centroid_finish, dim3(blocks_of((int64_t)R * d, 256)), dim3(256), 0, st, centre, start, R, d);
    hipLaunchKernelGGL(k_knn_norms, dim3(blocks_of(n, kNormRows)), dim3(256), 0, st, dX, n, d, dC, centre, norm, max_norm);

    // filter on the matrix cores, float64 refinement, exact fallback
    KnnSets P{};
    P.XQ = dX; P.XC = dX; P.qmembers = members; P.cmembers = members; P.qstart = start; P.cstart = start;
    P.cnorm = norm; P.centre = centre; P.group_of_q = dC; P.max_norm_bits = max_norm; P.n_q = n; P.n_c = n; P.d = d; P.same_set = 1;
    uint32_t hflag = 0;
    int rc = nearest_in_groups(st, P, blocks, (uint32_t)hblocks.size(), k, cand, tau, flagged, n_flagged, dOut, &hflag);
    if (rc) return rc;
    if (mem == NOMAD_HOST) KTRY(hipMemcpyAsync(out_nbrs, dOut, sizeof(int32_t) * (size_t)n * k, hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (stats) {
        stats[0] = (int64_t)hflag;
        int64_t pairs = 0;
        for (int32_t r = 0; r < R; ++r) pairs += (int64_t)hcounts[r] * (int64_t)hcounts[r];
        stats[1] = pairs;
    }
    return NOMAD_OK;
}

extern "C" int nomad_kmeans_lloyd(const float* X, int64_t n, int32_t d, int32_t K, float* centroids, int32_t max_iters, int32_t* labels,
                                  int32_t* iters_out, double* inertia_out, int mem, int32_t device, void* stream) {
    if (!X || !centroids || !labels || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return NOMAD_E_INVALID_ARG;
    if (n < 1 || d < 1 || d > NOMAD_KNN_MAX_DIM || K < 1 || K > n || max_iters < 1 || device < 0) return NOMAD_E_INVALID_ARG;
    if (n >= ((int64_t)1 << 31) - 256) return NOMAD_E_TOO_LARGE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    Buffers buf;
    const int32_t k = 1, list_len = k + kPad;

    const float* dX = X;
    float* dC = centroids;
    int32_t* dLab = labels;
    if (mem == NOMAD_HOST) {
        float *x = nullptr, *c = nullptr;
        int32_t* l = nullptr;
        KTRY(buf.alloc(&x, (size_t)n * d));
        KTRY(buf.alloc(&c, (size_t)K * d));
        KTRY(buf.alloc(&l, (size_t)n));
        KTRY(hipMemcpyAsync(x, X, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice, st));
        KTRY(hipMemcpyAsync(c, centroids, sizeof(float) * (size_t)K * d, hipMemcpyHostToDevice, st));
        dX = x; dC = c; dLab = l;
    }
    // work space
    uint32_t *qstart = nullptr, *cstart = nullptr, *max_pts = nullptr, *max_norm = nullptr, *n_flagged = nullptr;
    int32_t *new_lab = nullptr, *cand = nullptr, *flagged = nullptr;
    float *cnorm = nullptr, *tau = nullptr, *centre = nullptr, *c_used = nullptr;
    unsigned long long* changed = nullptr;
    double* inertia = nullptr;
    KnnBlock *blocks = nullptr, *slabs = nullptr;
    KTRY(buf.alloc(&qstart, 2)); KTRY(buf.alloc(&cstart, 2));
    KTRY(buf.alloc(&max_pts, 1)); KTRY(buf.alloc(&max_norm, 1)); KTRY(buf.alloc(&n_flagged, 1));
    KTRY(buf.alloc(&new_lab, (size_t)n)); KTRY(buf.alloc(&cand, (size_t)n * list_len)); KTRY(buf.alloc(&flagged, (size_t)n));
    KTRY(buf.alloc(&cnorm, (size_t)K)); KTRY(buf.alloc(&tau, (size_t)n)); KTRY(buf.alloc(&centre, (size_t)d)); KTRY(buf.alloc(&c_used, (size_t)K * d));
    KTRY(buf.alloc(&changed, 1)); KTRY(buf.alloc(&inertia, 1));
    const uint32_t hq[2] = {0u, (uint32_t)n}, hc[2] = {0u, (uint32_t)K};
    KTRY(hipMemcpyAsync(qstart, hq, sizeof(hq), hipMemcpyHostToDevice, st));
    KTRY(hipMemcpyAsync(cstart, hc, sizeof(hc), hipMemcpyHostToDevice, st));
    const uint32_t block_queries = (uint32_t)knn_filter_block_queries(width_class(d));
    std::vector<KnnBlock> hblocks, hslabs;
    for (int64_t q0 = 0; q0 < n; q0 += block_queries) hblocks.push_back(KnnBlock{0, (int32_t)q0});
    for (int64_t q0 = 0; q0 < n; q0 += kCentroidRows) hslabs.push_back(KnnBlock{0, (int32_t)q0});
    KTRY(buf.alloc(&blocks, hblocks.size()));
    KTRY(buf.alloc(&slabs, hslabs.size()));
    KTRY(hipMemcpyAsync(blocks, hblocks.data(), sizeof(KnnBlock) * hblocks.size(), hipMemcpyHostToDevice, st));
    KTRY(hipMemcpyAsync(slabs, hslabs.data(), sizeof(KnnBlock) * hslabs.size(), hipMemcpyHostToDevice, st));
    // both sides are centred on the mean of the points; the largest centred |x|^2 of the points, once
    KTRY(hipMemsetAsync(centre, 0, sizeof(float) * (size_t)d, st));
    KTRY(hipMemsetAsync(max_pts, 0, sizeof(uint32_t), st));
    hipLaunchKernelGGL(k_knn_centroid_sums, dim3((uint32_t)hslabs.size()), dim3(256), 0, st, dX, d, (const int32_t*)nullptr, qstart, slabs, centre);
    hipLaunchKernelGGL(k_knn_centroid_finish, dim3(blocks_of(d, 256)), dim3(256), 0, st, centre, qstart, 1, d);
    hipLaunchKernelGGL(k_knn_norms, dim3(blocks_of(n, kNormRows)), dim3(256), 0, st, dX, n, d, (const int32_t*)nullptr, centre, (float*)nullptr, max_pts);
    MeanStep m_step;
    {
        int rc = m_step.init(buf, st, n, K);
        if (rc) return rc;
    }

    KnnSets P{};
    P.XQ = dX; P.XC = dC; P.qmembers = nullptr; P.cmembers = nullptr; P.qstart = qstart; P.cstart = cstart;
    P.cnorm = cnorm; P.centre = centre; P.group_of_q = nullptr; P.max_norm_bits = max_norm; P.n_q = n; P.n_c = K; P.d = d; P.same_set = 0;
    float* key2 = nullptr;   // the two smallest filter keys of every point: a clear winner skips the float64 refinement
    KTRY(buf.alloc(&key2, (size_t)2 * n));
    P.key2 = key2;
    int32_t it = 0;
    bool have_labels = false;
    while (it < max_iters) {
        // E step: the nearest centroid of every point, exactly
        KTRY(hipMemcpyAsync(max_norm, max_pts, sizeof(uint32_t), hipMemcpyDeviceToDevice, st));
        hipLaunchKernelGGL(k_knn_norms, dim3(blocks_of(K, kNormRows)), dim3(256), 0, st, (const float*)dC, (int64_t)K, d, (const int32_t*)nullptr, centre, cnorm,
                           max_norm);
        uint32_t hflag = 0;
        int rc = nearest_in_groups(st, P, blocks, (uint32_t)hblocks.size(), k, cand, tau, flagged, n_flagged, new_lab, &hflag);
        if (rc) return rc;
        ++it;
        KTRY(hipMemcpyAsync(c_used, dC, sizeof(float) * (size_t)K * d, hipMemcpyDeviceToDevice, st));
        unsigned long long hchanged = 1;
        if (have_labels) {
            KTRY(hipMemsetAsync(changed, 0, sizeof(unsigned long long), st));
            hipLaunchKernelGGL(k_kmeans_changed, dim3(blocks_of(n, 256)), dim3(256), 0, st, (const int32_t*)new_lab, (const int32_t*)dLab, n, changed);
            KTRY(hipMemcpyAsync(&hchanged, changed, sizeof(hchanged), hipMemcpyDeviceToHost, st));
            KTRY(hipStreamSynchronize(st));
        }
        if (have_labels && hchanged == 0) break;   // nothing moved: the centroids are the means of these labels already
        KTRY(hipMemcpyAsync(dLab, new_lab, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToDevice, st));
        have_labels = true;
        // M step
        {
            int rc = m_step.run(st, dX, d, (const int32_t*)dLab, dC);
            if (rc) return rc;
        }
    }
    // inertia of the labels against the centroids they were computed from
    double hinertia = 0.0;
    KTRY(hipMemsetAsync(inertia, 0, sizeof(double), st));
    hipLaunchKernelGGL(k_kmeans_inertia, dim3(blocks_of(n, 256)), dim3(256), 0, st, dX, (const float*)c_used, d, (const int32_t*)dLab, n, inertia);
    KTRY(hipMemcpyAsync(&hinertia, inertia, sizeof(double), hipMemcpyDeviceToHost, st));
    KTRY(hipGetLastError());
    if (mem == NOMAD_HOST) {
        KTRY(hipMemcpyAsync(centroids, dC, sizeof(float) * (size_t)K * d, hipMemcpyDeviceToHost, st));
        KTRY(hipMemcpyAsync(labels, dLab, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
    }
    KTRY(hipStreamSynchronize(st));
    if (iters_out) *iters_out = it;
    if (inertia_out) *inertia_out = hinertia;
    return NOMAD_OK;
}
extern "C" int nomad_kmeans_lsh_init(const float* X, int64_t n, int32_t d, int32_t K, const float* planes, const int32_t* anchors,
                                     int32_t n_planes, float* centroids_out, int32_t* buckets_out, int mem, int32_t device, void* stream) {
    if (!X || !planes || !centroids_out || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return NOMAD_E_INVALID_ARG;
    if (n < 1 || d < 1 || d > NOMAD_KNN_MAX_DIM || K < 1 || K > n || n_planes < 1 || n_planes > kMaxPlanes || device < 0) return NOMAD_E_INVALID_ARG;
    if (((int64_t)1 << n_planes) < K) return NOMAD_E_INVALID_ARG;
    if (n >= ((int64_t)1 << 31) - 256) return NOMAD_E_TOO_LARGE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    Buffers buf;
    const float *dX = X, *dP = planes;
    const int32_t* dA = anchors;
    float* dC = centroids_out;
    int32_t* dB = buckets_out;
    std::vector<int32_t> hanchors((size_t)n_planes, 0);
    if (mem == NOMAD_HOST) {
        float *x = nullptr, *pl = nullptr, *c = nullptr;
        KTRY(buf.alloc(&x, (size_t)n * d));
        KTRY(buf.alloc(&pl, (size_t)n_planes * d));
        KTRY(buf.alloc(&c, (size_t)K * d));
        KTRY(hipMemcpyAsync(x, X, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice, st));
        KTRY(hipMemcpyAsync(pl, planes, sizeof(float) * (size_t)n_planes * d, hipMemcpyHostToDevice, st));
        dX = x; dP = pl; dC = c;
        if (anchors) {
            int32_t* a = nullptr;
            KTRY(buf.alloc(&a, (size_t)n_planes));
            KTRY(hipMemcpyAsync(a, anchors, sizeof(int32_t) * (size_t)n_planes, hipMemcpyHostToDevice, st));
            for (int32_t j = 0; j < n_planes; ++j) hanchors[j] = anchors[j];
            dA = a;
        }
    } else if (anchors) {
        KTRY(hipMemcpyAsync(hanchors.data(), anchors, sizeof(int32_t) * (size_t)n_planes, hipMemcpyDeviceToHost, st));
        KTRY(hipStreamSynchronize(st));
    }
    for (int32_t j = 0; j < n_planes; ++j)
        if (hanchors[j] < 0 || hanchors[j] >= n) return NOMAD_E_INVALID_ARG;   // an anchor that is no data point
    if (!anchors) {   // every plane through the median of a sample along its normal
        int32_t* a = nullptr;
        KTRY(buf.alloc(&a, (size_t)n_planes));
        hipLaunchKernelGGL(k_lsh_median_anchors, dim3((uint32_t)n_planes), dim3(256), 0, st, dX, n, d, dP, a);
        dA = a;
    }
    if (!dB || mem == NOMAD_HOST) {
        int32_t* bk = nullptr;
        KTRY(buf.alloc(&bk, (size_t)n));
        dB = bk;
    }
    MeanStep m_step;
    {
        int rc = m_step.init(buf, st, n, K);
        if (rc) return rc;
    }
    hipLaunchKernelGGL(k_lsh_buckets, dim3(blocks_of(n, 256)), dim3(256), 0, st, dX, n, d, dP, dA, n_planes, K, dB);
    hipLaunchKernelGGL(k_lsh_fallback, dim3(blocks_of((int64_t)K * d, 256)), dim3(256), 0, st, dX, n, d, K, dC);
    // bucket means: the M step of Lloyd's iteration on the buckets
    {
        int rc = m_step.run(st, dX, d, (const int32_t*)dB, dC);
        if (rc) return rc;
    }
    KTRY(hipGetLastError());
    if (mem == NOMAD_HOST) {
        KTRY(hipMemcpyAsync(centroids_out, dC, sizeof(float) * (size_t)K * d, hipMemcpyDeviceToHost, st));
        if (buckets_out) KTRY(hipMemcpyAsync(buckets_out, dB, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
    }
    KTRY(hipStreamSynchronize(st));
    return NOMAD_OK;
}

namespace {

// Exact k nearest other points, among all n rows of A, of the rows listed in dQ (m of them; nullptr: every row).
// out [m * k] on the device.  A workgroup of the filter scans every candidate of its group, so few queries would leave
// most of the chip idle: the candidates are then cut into slices, every slice is a group of its own with a copy of the
// queries, and the per-slice answers are merged by exact distance.
int neighbours_of_queries(hipStream_t st, Buffers& buf, const float* A, int64_t n, int32_t d, const int32_t* dQ, int64_t m, int32_t k,
                          int32_t* out) {
    const int32_t list_len = k + kPad;
    const uint32_t block_queries = (uint32_t)knn_filter_block_queries(width_class(d));
    const int64_t base_blocks = (m + block_queries - 1) / block_queries;
    int64_t G = std::max<int64_t>(1, 1024 / base_blocks);
    G = std::min<int64_t>(G, 256 / k);                       // the merge ranks slices * k candidates in one workgroup
    G = std::min<int64_t>(G, std::max<int64_t>(1, n / 4096));   // slices of at least 4,096 candidates
    const int64_t slice = (n + G - 1) / G, mq = m * G;
    if (mq >= ((int64_t)1 << 31) - 256) return NOMAD_E_TOO_LARGE;
    uint32_t *qstart = nullptr, *cstart = nullptr, *max_norm = nullptr, *n_flagged = nullptr;
    int32_t *cand = nullptr, *flagged = nullptr, *self = nullptr, *group_of_q = nullptr, *slice_of = nullptr, *part = nullptr;
    float *cnorm = nullptr, *tau = nullptr, *centre = nullptr, *AQ = nullptr;
    int* bad = nullptr;
    KnnBlock *blocks = nullptr, *slabs = nullptr;
    KTRY(buf.alloc(&qstart, (size_t)G + 1)); KTRY(buf.alloc(&cstart, (size_t)G + 1)); KTRY(buf.alloc(&max_norm, (size_t)G));
    KTRY(buf.alloc(&n_flagged, 1)); KTRY(buf.alloc(&bad, 1));
    KTRY(buf.alloc(&cand, (size_t)mq * list_len)); KTRY(buf.alloc(&flagged, (size_t)mq)); KTRY(buf.alloc(&tau, (size_t)mq));
    KTRY(buf.alloc(&cnorm, (size_t)n)); KTRY(buf.alloc(&centre, (size_t)G * d)); KTRY(buf.alloc(&AQ, (size_t)mq * d));
    KTRY(buf.alloc(&self, (size_t)mq));
    std::vector<uint32_t> hq((size_t)G + 1), hc((size_t)G + 1);
    std::vector<KnnBlock> hblocks, hslabs;
    for (int64_t g = 0; g <= G; ++g) {
        hq[g] = (uint32_t)(g * m);
        hc[g] = (uint32_t)std::min<int64_t>(n, g * slice);
    }
    for (int64_t g = 0; g < G; ++g) {
        for (int64_t q0 = 0; q0 < m; q0 += block_queries) hblocks.push_back(KnnBlock{(int32_t)g, (int32_t)q0});
        for (int64_t q0 = 0; q0 < (int64_t)(hc[g + 1] - hc[g]); q0 += kCentroidRows) hslabs.push_back(KnnBlock{(int32_t)g, (int32_t)q0});
    }
    KTRY(hipMemcpyAsync(qstart, hq.data(), sizeof(uint32_t) * hq.size(), hipMemcpyHostToDevice, st));
    KTRY(hipMemcpyAsync(cstart, hc.data(), sizeof(uint32_t) * hc.size(), hipMemcpyHostToDevice, st));
    KTRY(buf.alloc(&blocks, hblocks.size()));
    KTRY(buf.alloc(&slabs, hslabs.size()));
    KTRY(hipMemcpyAsync(blocks, hblocks.data(), sizeof(KnnBlock) * hblocks.size(), hipMemcpyHostToDevice, st));
    KTRY(hipMemcpyAsync(slabs, hslabs.data(), sizeof(KnnBlock) * hslabs.size(), hipMemcpyHostToDevice, st));
    KTRY(hipMemsetAsync(centre, 0, sizeof(float) * (size_t)G * d, st));
    KTRY(hipMemsetAsync(max_norm, 0, sizeof(uint32_t) * (size_t)G, st));
    KTRY(hipMemsetAsync(bad, 0, sizeof(int), st));
    if (G > 1) {
        KTRY(buf.alloc(&group_of_q, (size_t)mq));
        KTRY(buf.alloc(&slice_of, (size_t)n));
        KTRY(buf.alloc(&part, (size_t)mq * k));
        hipLaunchKernelGGL(k_periodic_ids, dim3(blocks_of(n, 256)), dim3(256), 0, st, (const int32_t*)nullptr, slice, n, slice_of, (int32_t*)nullptr);
    }
    // every slice centred on its own mean; the largest centred norm of a group covers its candidates and its queries
    hipLaunchKernelGGL(k_periodic_ids, dim3(blocks_of(mq, 256)), dim3(256), 0, st, dQ, m, mq, group_of_q, self);
    hipLaunchKernelGGL(k_gather_rows, dim3(blocks_of(mq * d, 256)), dim3(256), 0, st, A, n, d, dQ, m, mq, AQ, bad);
    int hbad = 0;
    KTRY(hipMemcpyAsync(&hbad, bad, sizeof(int), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (hbad) return NOMAD_E_INVALID_ARG;   // a query outside 0..n-1
    hipLaunchKernelGGL(k_knn_centroid_sums, dim3((uint32_t)hslabs.size()), dim3(256), 0, st, A, d, (const int32_t*)nullptr, cstart, slabs, centre);
    hipLaunchKernelGGL(k_knn_centroid_finish, dim3(blocks_of(G * d, 256)), dim3(256), 0, st, centre, cstart, (int32_t)G, d);
    hipLaunchKernelGGL(k_knn_norms, dim3(blocks_of(n, kNormRows)), dim3(256), 0, st, A, n, d, (const int32_t*)slice_of, centre, cnorm, max_norm);
    hipLaunchKernelGGL(k_knn_norms, dim3(blocks_of(mq, kNormRows)), dim3(256), 0, st, (const float*)AQ, mq, d, (const int32_t*)group_of_q, centre,
                       (float*)nullptr, max_norm);
    KnnSets P{};
    P.XQ = AQ; P.XC = A; P.qmembers = nullptr; P.cmembers = nullptr; P.qstart = qstart; P.cstart = cstart;
    P.cnorm = cnorm; P.centre = centre; P.group_of_q = group_of_q; P.max_norm_bits = max_norm; P.n_q = mq; P.n_c = n; P.d = d; P.same_set = 0;
    P.self_row = self;
    uint32_t hflag = 0;
    int rc = nearest_in_groups(st, P, blocks, (uint32_t)hblocks.size(), k, cand, tau, flagged, n_flagged, G > 1 ? part : out, &hflag);
    if (rc) return rc;
    if (G > 1) {
        hipLaunchKernelGGL(k_merge_slices, dim3((uint32_t)m), dim3(256), 0, st, (const float*)AQ, A, d, (const int32_t*)part, (int32_t)G, m, k, out);
        KTRY(hipGetLastError());
    }
    return NOMAD_OK;
}

}  // namespace

extern "C" int nomad_neighbourhood_preservation(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low, int32_t k,
                                                const int32_t* queries, int64_t n_queries, int64_t* hits_out, int mem, int32_t device,
                                                void* stream) {
    if (!X || !Y || !hits_out || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return NOMAD_E_INVALID_ARG;
    if (n < 2 || d < 1 || d > NOMAD_KNN_MAX_DIM || d_low < 1 || d_low > NOMAD_KNN_MAX_DIM || k < 1 || k > NOMAD_KNN_MAX_K || device < 0)
        return NOMAD_E_INVALID_ARG;
    if (queries ? n_queries < 1 : (n_queries != 0 && n_queries != n)) return NOMAD_E_INVALID_ARG;
    if (n >= ((int64_t)1 << 31) - 256 || n_queries >= ((int64_t)1 << 31) - 256) return NOMAD_E_TOO_LARGE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    const int64_t m = queries ? n_queries : n;
    const float *dX = X, *dY = Y;
    const int32_t* dQ = queries;
    Buffers io;
    if (mem == NOMAD_HOST) {
        float *x = nullptr, *y = nullptr;
        KTRY(io.alloc(&x, (size_t)n * d));
        KTRY(io.alloc(&y, (size_t)n * d_low));
        KTRY(hipMemcpyAsync(x, X, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice, st));
        KTRY(hipMemcpyAsync(y, Y, sizeof(float) * (size_t)n * d_low, hipMemcpyHostToDevice, st));
        dX = x; dY = y;
        if (queries) {
            int32_t* q = nullptr;
            KTRY(io.alloc(&q, (size_t)m));
            KTRY(hipMemcpyAsync(q, queries, sizeof(int32_t) * (size_t)m, hipMemcpyHostToDevice, st));
            dQ = q;
        }
    }
    int32_t *high = nullptr, *low = nullptr;
    unsigned long long* hits = nullptr;
    KTRY(io.alloc(&high, (size_t)m * k));
    KTRY(io.alloc(&low, (size_t)m * k));
    KTRY(io.alloc(&hits, 1));
    {
        Buffers work;   // released before the second space takes its own
        int rc = neighbours_of_queries(st, work, dX, n, d, dQ, m, k, high);
        if (rc) return rc;
        KTRY(hipStreamSynchronize(st));
    }
    {
        Buffers work;
        int rc = neighbours_of_queries(st, work, dY, n, d_low, dQ, m, k, low);
        if (rc) return rc;
        KTRY(hipStreamSynchronize(st));
    }
    unsigned long long hhits = 0;
    KTRY(hipMemsetAsync(hits, 0, sizeof(unsigned long long), st));
    hipLaunchKernelGGL(k_overlap, dim3(blocks_of(m, 256)), dim3(256), 0, st, (const int32_t*)high, (const int32_t*)low, k, m, hits);
    KTRY(hipMemcpyAsync(&hhits, hits, sizeof(hhits), hipMemcpyDeviceToHost, st));
    KTRY(hipGetLastError());
    KTRY(hipStreamSynchronize(st));
    *hits_out = (int64_t)hhits;
    return NOMAD_OK;
}

namespace {

// One launch covers at most kTripletsPerLaunch triplets (65,536 workgroups), so that any count up to the documented
// 2^40 stays inside the grid limits; the launches add into the same counter.
constexpr int64_t kTripletsPerLaunch = (int64_t)1 << 24;

int check_triplet_arguments(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low, int64_t n_triplets,
                            const int64_t* agree_out, int32_t device) {
    if (!X || !Y || !agree_out) return NOMAD_E_INVALID_ARG;
    if (n < 3 || d < 1 || d_low < 1 || n_triplets < 0 || device < 0) return NOMAD_E_INVALID_ARG;
    if (n >= ((int64_t)1 << 31) - 256 || n_triplets > ((int64_t)1 << 40)) return NOMAD_E_TOO_LARGE;
    return NOMAD_OK;
}

// enqueue the count of the triplets 0 .. n_triplets-1 into *agree (device memory, cleared first by a kernel)
int enqueue_triplets(hipStream_t st, const float* dX, int32_t d, const float* dY, int32_t d_low, int64_t n, int64_t n_triplets,
                     uint64_t seed, unsigned long long* agree) {
    hipLaunchKernelGGL(k_store_u64, dim3(1), dim3(64), 0, st, agree, 0ull);
    for (int64_t t0 = 0; t0 < n_triplets; t0 += kTripletsPerLaunch) {
        const int64_t t1 = std::min(n_triplets, t0 + kTripletsPerLaunch);
        hipLaunchKernelGGL(k_triplets, dim3(blocks_of(t1 - t0, 256)), dim3(256), 0, st, dX, d, dY, d_low, (uint32_t)n, t0, t1,
                           (uint32_t)seed, (uint32_t)(seed >> 32), agree);
    }
    KTRY(hipGetLastError());
    return NOMAD_OK;
}

// ---- work space of nomad_random_triplet_accuracy_noalloc: lives in the code object, one copy per device
constexpr int kScratchWords = 32;   // 256 bytes; word 0 is the agreement counter
static __device__ __align__(256) unsigned long long scratch[kScratchWords];

constexpr int kMaxScratchDevices = 64;
unsigned long long* scratch_address[kMaxScratchDevices];   // device address of `scratch` on every device, once asked for
std::mutex scratch_mutex;

// Device address of this device's copy of `scratch` (the device must be current).  The array's name is only a
// host-side handle: kernels and copies take the address hipGetSymbolAddress returns.
int scratch_on_device(int32_t device, unsigned long long** out) {
    if (device >= kMaxScratchDevices) return NOMAD_E_INVALID_ARG;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_address[device]) {
        void* p = nullptr;
        KTRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return NOMAD_E_HIP;
        scratch_address[device] = (unsigned long long*)p;
    }
    *out = scratch_address[device];
    return NOMAD_OK;
}

}  // namespace

extern "C" int nomad_random_triplet_accuracy(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low, int64_t n_triplets,
                                             uint64_t seed, int64_t* agree_out, int mem, int32_t device, void* stream) {
    if (mem != NOMAD_HOST && mem != NOMAD_DEVICE) return NOMAD_E_INVALID_ARG;
    if (int rc = check_triplet_arguments(X, n, d, Y, d_low, n_triplets, agree_out, device)) return rc;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    const float *dX = X, *dY = Y;
    Buffers buf;
    if (mem == NOMAD_HOST) {
        float *x = nullptr, *y = nullptr;
        KTRY(buf.alloc(&x, (size_t)n * d));
        KTRY(buf.alloc(&y, (size_t)n * d_low));
        KTRY(hipMemcpyAsync(x, X, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice, st));
        KTRY(hipMemcpyAsync(y, Y, sizeof(float) * (size_t)n * d_low, hipMemcpyHostToDevice, st));
        dX = x; dY = y;
    }
    unsigned long long* agree = nullptr;
    unsigned long long hagree = 0;
    KTRY(buf.alloc(&agree, 1));
    if (int rc = enqueue_triplets(st, dX, d, dY, d_low, n, n_triplets, seed, agree)) return rc;
    KTRY(hipMemcpyAsync(&hagree, agree, sizeof(hagree), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    *agree_out = (int64_t)hagree;
    return NOMAD_OK;
}

extern "C" int nomad_random_triplet_accuracy_noalloc(const float* X, int64_t n, int32_t d, const float* Y, int32_t d_low,
                                                     int64_t n_triplets, uint64_t seed, int64_t* agree_out, int32_t device,
                                                     void* stream) {
    if (int rc = check_triplet_arguments(X, n, d, Y, d_low, n_triplets, agree_out, device)) return rc;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    unsigned long long* counter = nullptr;
    if (int rc = scratch_on_device(device, &counter)) return rc;
    unsigned long long hagree = 0;
    if (int rc = enqueue_triplets(st, X, d, Y, d_low, n, n_triplets, seed, counter)) return rc;
    KTRY(hipMemcpyAsync(&hagree, counter, sizeof(hagree), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    *agree_out = (int64_t)hagree;
    return NOMAD_OK;
}
#pragma GCC visibility pop

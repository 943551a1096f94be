// libnomad: the in-cluster exact nearest-neighbour index behind the C ABI of include/nomad.h (host side).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <vector>

#include "knn_kernels.h"
#include "nomad.h"

using namespace nomad_knn;

namespace {

struct Buffers {   // device allocations of one call, released on every path
    std::vector<void*> ptrs;
    ~Buffers() { for (void* p : ptrs) (void)hipFree(p); }
    template <typename T>
    hipError_t alloc(T** p, size_t count) {
        *p = nullptr;
        hipError_t e = hipMalloc((void**)p, std::max<size_t>(count, 1) * sizeof(T));
        if (e == hipSuccess) ptrs.push_back(*p);
        return e;
    }
};

#define KTRY(call)                                                          \
    do {                                                                    \
        hipError_t e_ = (call);                                             \
        if (e_ != hipSuccess) return e_ == hipErrorOutOfMemory ? NOMAD_E_OOM : NOMAD_E_HIP; \
    } while (0)

inline uint32_t blocks_of(int64_t items, int per) { return (uint32_t)((items + per - 1) / per); }

template <int D4, int L>
hipError_t launch_filter_dl(hipStream_t st, uint32_t n_blocks, const float* X, int32_t d, const float* norm, const int32_t* members,
                            const uint32_t* start, const KnnBlock* blocks, const float* centre, int32_t list_len, int32_t* cand, float* tau) {
    const size_t lds = knn_filter_lds_bytes(D4, L);
    hipError_t e = hipFuncSetAttribute((const void*)k_knn_filter<D4, L>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_knn_filter<D4, L>), dim3(n_blocks), dim3(64 * knn_filter_waves(D4)), lds, st, X, d, norm, members, start, blocks,
                       centre, list_len, cand, tau);
    return hipGetLastError();
}

template <int D4>
hipError_t launch_filter(hipStream_t st, uint32_t n_blocks, const float* X, int32_t d, const float* norm, const int32_t* members,
                         const uint32_t* start, const KnnBlock* blocks, const float* centre, int32_t list_len, int32_t* cand, float* tau) {
    switch (knn_filter_list_class(list_len)) {
        case 8: return launch_filter_dl<D4, 8>(st, n_blocks, X, d, norm, members, start, blocks, centre, list_len, cand, tau);
        case 12: return launch_filter_dl<D4, 12>(st, n_blocks, X, d, norm, members, start, blocks, centre, list_len, cand, tau);
        default: return launch_filter_dl<D4, 20>(st, n_blocks, X, d, norm, members, start, blocks, centre, list_len, cand, tau);
    }
}

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
    KTRY(hipMemsetAsync(n_flagged, 0, sizeof(uint32_t), st));
    KTRY(hipMemsetAsync(bad, 0, sizeof(int), st));
    KTRY(hipMemsetAsync(cand, 0xFF, sizeof(int32_t) * (size_t)n * list_len, st));   // every slot "no candidate" until the filter fills it
    hipLaunchKernelGGL(k_knn_count, dim3(blocks_of(n, 256)), dim3(256), 0, st, dC, n, R, counts, bad);
    std::vector<uint32_t> hcounts(R), hstart((size_t)R + 1, 0);
    int hbad = 0;
    KTRY(hipMemcpyAsync(hcounts.data(), counts, sizeof(uint32_t) * (size_t)R, hipMemcpyDeviceToHost, st));
    KTRY(hipMemcpyAsync(&hbad, bad, sizeof(int), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (hbad) return NOMAD_E_BAD_GRAPH;   // a cluster id outside 0..n_clusters-1
    // the width class of the filter kernel decides how many queries a workgroup takes
    const int d4 = (d + 3) / 4;
    const int d4_class = d4 <= 8 ? 8 : d4 <= 16 ? 16 : d4 <= 32 ? 32 : d4 <= 64 ? 64 : d4 <= 128 ? 128 : 192;
    const uint32_t block_queries = (uint32_t)(kWaveQueries * knn_filter_waves(d4_class));
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
    hipLaunchKernelGGL(k_knn_group, dim3(blocks_of(n, 256)), dim3(256), 0, st, dC, n, start, cursor, members);
    hipLaunchKernelGGL(k_knn_centroid_sums, dim3((uint32_t)hslabs.size()), dim3(256), 0, st, dX, d, members, start, slabs, centre);
    hipLaunchKernelGGL(k_knn_centroid_finish, dim3(blocks_of((int64_t)R * d, 256)), dim3(256), 0, st, centre, start, R, d);
    hipLaunchKernelGGL(k_knn_norms, dim3(blocks_of(n, 256)), dim3(256), 0, st, dX, n, d, dC, centre, norm, max_norm);

    // stage 1: float32 filter on the matrix cores
    hipError_t e = hipErrorInvalidValue;
    const uint32_t nb = (uint32_t)hblocks.size();
#define NOMAD_KNN_CASE(D4)                                                                                             \
    e = launch_filter<D4>(st, nb, dX, d, norm, members, start, blocks, centre, list_len, cand, tau)
    if (d4_class == 8) NOMAD_KNN_CASE(8);
    else if (d4_class == 16) NOMAD_KNN_CASE(16);
    else if (d4_class == 32) NOMAD_KNN_CASE(32);
    else if (d4_class == 64) NOMAD_KNN_CASE(64);
    else if (d4_class == 128) NOMAD_KNN_CASE(128);
    else NOMAD_KNN_CASE(192);
#undef NOMAD_KNN_CASE
    KTRY(e);

    // stage 2: exact distances of the candidates, certification
    hipLaunchKernelGGL(k_knn_refine, dim3(blocks_of(n, 4)), dim3(256), 0, st, dX, d, members, dC, max_norm, centre, cand, tau, n, k, list_len,
                       dOut, flagged, n_flagged);
    uint32_t hflag = 0;
    KTRY(hipMemcpyAsync(&hflag, n_flagged, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));

    // stage 3: what could not be certified, exactly
    if (hflag) hipLaunchKernelGGL(k_knn_exact, dim3(hflag), dim3(256), 0, st, dX, d, members, start, dC, flagged, k, dOut);
    KTRY(hipGetLastError());
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
#pragma GCC visibility pop

// Device code of the two quality measures of Section 4: neighbourhood preservation (the overlap of exact
// k-neighbourhoods in the data space and in the projection; the neighbourhoods come from the nearest-neighbour kernels
// of knn_kernels.h) and random triplet accuracy (the fraction of random triplets whose two distances from the anchor
// are ordered alike in both spaces).  Distances are the float64 definition of knn_kernels.h (t = 0..d-1 in order), so
// every decision, and with it every count, is exact.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "knn_kernels.h"
#include "philox.h"

namespace nomad_metrics {

constexpr uint32_t kTripletStream = 0x54524950u;   // third counter word of the triplet generator

// out[p] = X[rows[p % period]] (rows == nullptr: row p % period) for p < m: the listed rows, repeated every `period`;
// bad is set where a row lies outside [0, n)
__global__ void __launch_bounds__(256) k_gather_rows(const float* __restrict__ X, int64_t n, int32_t d, const int32_t* __restrict__ rows,
                                                     int64_t period, int64_t m, float* __restrict__ out, int* __restrict__ bad) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= m * d) return;
    const int64_t p = x / d;
    const int32_t t = (int32_t)(x % d);
    const int64_t r = rows ? rows[p % period] : p % period;
    if (r < 0 || r >= n) { *bad = 1; out[x] = 0.f; return; }
    out[x] = X[r * d + t];
}

// block[p] = p / period (may be nullptr); tiled[p] = rows[p % period] (rows == nullptr: p % period) (may be nullptr)
__global__ void __launch_bounds__(256) k_periodic_ids(const int32_t* __restrict__ rows, int64_t period, int64_t m, int32_t* __restrict__ block,
                                                      int32_t* __restrict__ tiled) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= m) return;
    if (block) block[p] = (int32_t)(p / period);
    if (tiled) tiled[p] = rows ? rows[p % period] : (int32_t)(p % period);
}

// The candidate set was cut into `slices` parts and query r has the k nearest of each part in
// part_nbrs[(g * m + r) * k ..]: the k nearest overall are the k smallest (distance, index) among those slices * k <= 256
// candidates.  One workgroup per query, one thread per candidate, rank by counting.
__global__ void __launch_bounds__(256) k_merge_slices(const float* __restrict__ AQ, const float* __restrict__ A, int32_t d,
                                                      const int32_t* __restrict__ part_nbrs, int32_t slices, int64_t m, int32_t k,
                                                      int32_t* __restrict__ out) {
    __shared__ double sD[256];
    __shared__ int32_t sC[256];
    const int64_t r = blockIdx.x;
    const int t = threadIdx.x, total = slices * k;
    int32_t c = -1;
    double D = __builtin_inf();
    if (t < total) {
        c = part_nbrs[((int64_t)(t / k) * m + r) * k + t % k];
        if (c >= 0) D = nomad_knn::exact_distance(AQ + r * d, A + (int64_t)c * d, d);
    }
    sD[t] = D;
    sC[t] = c;
    __syncthreads();
    int rank = 0, found = 0;
    for (int o = 0; o < total; ++o) {
        const int32_t co = sC[o];
        if (co < 0) continue;
        ++found;
        const double Do = sD[o];
        if (Do < D || (Do == D && co < c)) ++rank;
    }
    if (c >= 0 && rank < k) out[r * k + rank] = c;
    if (t >= found && t < k) out[r * k + t] = -1;   // fewer than k candidates in all
}

// common members of the two neighbour lists of every query (-1 = empty slot), summed
__global__ void __launch_bounds__(256) k_overlap(const int32_t* __restrict__ a, const int32_t* __restrict__ b, int32_t k, int64_t m,
                                                 unsigned long long* __restrict__ hits) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int found = 0;
    if (p < m) {
        for (int x = 0; x < k; ++x) {
            const int32_t v = a[p * k + x];
            if (v < 0) continue;
            for (int y = 0; y < k; ++y) found += b[p * k + y] == v;
        }
    }
    for (int w = 32; w > 0; w >>= 1) found += __shfl_xor(found, w, 64);
    if ((threadIdx.x & 63) == 0 && found) atomicAdd(hits, (unsigned long long)found);
}

// squared distances from row a to rows b and c: difference, product and running sum each rounded once in float64,
// t = 0..d-1 in order (two independent chains)
__device__ __forceinline__ void anchor_distances(const float* __restrict__ a, const float* __restrict__ b, const float* __restrict__ c,
                                                 int32_t d, double& Dab, double& Dac) {
    double s1 = 0.0, s2 = 0.0;
    int t = 0;
    if ((d & 3) == 0) {
        for (; t + 8 <= d; t += 8) {   // six loads in flight
            const float4 a0 = *(const float4*)(a + t), a1 = *(const float4*)(a + t + 4);
            const float4 b0 = *(const float4*)(b + t), b1 = *(const float4*)(b + t + 4);
            const float4 c0 = *(const float4*)(c + t), c1 = *(const float4*)(c + t + 4);
            const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const float bv[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
            const float cv[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const double e1 = (double)av[u] - (double)bv[u], e2 = (double)av[u] - (double)cv[u];
                s1 = __dadd_rn(s1, __dmul_rn(e1, e1));
                s2 = __dadd_rn(s2, __dmul_rn(e2, e2));
            }
        }
    }
    for (; t < d; ++t) {
        const double e1 = (double)a[t] - (double)b[t], e2 = (double)a[t] - (double)c[t];
        s1 = __dadd_rn(s1, __dmul_rn(e1, e1));
        s2 = __dadd_rn(s2, __dmul_rn(e2, e2));
    }
    Dab = s1;
    Dac = s2;
}

// Triplet number t (one per thread): anchor i and two other points j, k, all distinct and uniform, from the words of
// Philox(counter = (lo32 t, hi32 t, stream, 0), key = seed) by multiply-high range reduction over n, n - 1 and n - 2
// values, stepping over the points already taken.  It agrees when [D_X(i,j) < D_X(i,k)] == [D_Y(i,j) < D_Y(i,k)].
// A launch covers the triplets t_begin .. t_end-1 and adds its count to *agree.
__global__ void __launch_bounds__(256) k_triplets(const float* __restrict__ X, int32_t d, const float* __restrict__ Y, int32_t d_low,
                                                  uint32_t n, int64_t t_begin, int64_t t_end, uint32_t key0, uint32_t key1,
                                                  unsigned long long* __restrict__ agree) {
    const int64_t t = t_begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool same = false;
    if (t < t_end) {
        uint32_t w[4];
        philox4x32_10((uint32_t)t, (uint32_t)((uint64_t)t >> 32), kTripletStream, 0u, key0, key1, w);
        const uint32_t i = __umulhi(w[0], n);
        uint32_t j = __umulhi(w[1], n - 1u);
        j += j >= i;
        uint32_t k = __umulhi(w[2], n - 2u);
        const uint32_t lo = min(i, j), hi = max(i, j);
        k += k >= lo;
        k += k >= hi;
        double hij, hik, lij, lik;
        anchor_distances(X + (int64_t)i * d, X + (int64_t)j * d, X + (int64_t)k * d, d, hij, hik);
        anchor_distances(Y + (int64_t)i * d_low, Y + (int64_t)j * d_low, Y + (int64_t)k * d_low, d_low, lij, lik);
        same = (hij < hik) == (lij < lik);
    }
    const unsigned long long m = __ballot(same);
    if ((threadIdx.x & 63) == 0 && m) atomicAdd(agree, (unsigned long long)__popcll(m));
}

// *p = v (one lane): clears a counter without a memset node, so that a caller may record the call into a HIP graph
__global__ void k_store_u64(unsigned long long* __restrict__ p, unsigned long long v) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *p = v;
}

}  // namespace nomad_metrics

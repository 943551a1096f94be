// Device kernels of the in-cluster exact nearest-neighbour index for gfx950 (Section 3.2 of arxiv 2505.15511: the
// candidates for a point's neighbours are the points of its own cluster; among those the neighbours are exact).
//
// A dense contraction: all pairwise dot products inside a cluster.  Three stages:
//   k_knn_filter   float32 matrix cores (v_mfma_f32_16x16x4f32): for every query the K' = k + pad candidates with the
//                  smallest key |c|^2 - 2 q.c, and tau = the K'-th smallest key (every point left out has key >= tau);
//   k_knn_refine   the exact distances of those candidates, sum_t (x_t - y_t)^2 in float64 in the order t = 0..d-1,
//                  sorted by (distance, index); the first k are the answer if the k-th exact key lies below
//                  tau by more than the float32 error bound of the filter -- otherwise the query is flagged;
//   k_knn_exact    flagged queries (near-ties beyond the pad, duplicates in bulk): exact distances to the whole cluster.
// The result therefore does not depend on float32 rounding: it is the float64 definition, tie-broken by index.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nomad_knn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kMaxK = 32;          // neighbours per point
constexpr int kPad = 8;            // extra candidates the filter keeps
constexpr int kMaxList = kMaxK + kPad;
constexpr int kWaveQueries = 16;   // queries per wavefront (the N of the 16x16x4 tile)
constexpr int kTile = 16;          // candidates per tile (the M of the 16x16x4 tile)
constexpr int kFilterWaves = 4;
constexpr int kFilterBlock = 64 * kFilterWaves;
constexpr int kBlockQueries = kWaveQueries * kFilterWaves;   // 64 queries per workgroup

struct KnnBlock { int32_t cluster; int32_t q0; };   // queries members[start[cluster] + q0 ..] of one workgroup

// |x|^2 of every point in float32 (t = 0..d-1 in order) and the largest one per cluster
__global__ void __launch_bounds__(256) k_knn_norms(const float* __restrict__ X, int64_t n, int32_t d, const int32_t* __restrict__ cluster_of,
                                                   float* __restrict__ norm, uint32_t* __restrict__ max_norm_bits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float* x = X + i * d;
    float s = 0.f;
    int t = 0;
    if ((d & 3) == 0)
        for (; t < d; t += 4) {
            const float4 a = *(const float4*)(x + t);
            s = fmaf(a.x, a.x, s); s = fmaf(a.y, a.y, s); s = fmaf(a.z, a.z, s); s = fmaf(a.w, a.w, s);
        }
    for (; t < d; ++t) s = fmaf(x[t], x[t], s);
    norm[i] = s;
    atomicMax(&max_norm_bits[cluster_of[i]], __float_as_uint(s));   // non-negative floats order like their bit patterns
}

__global__ void __launch_bounds__(256) k_knn_count(const int32_t* __restrict__ cluster_of, int64_t n, int32_t R, uint32_t* __restrict__ counts,
                                                   int* __restrict__ bad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t r = cluster_of[i];
    if (r < 0 || r >= R) { *bad = 1; return; }
    atomicAdd(&counts[r], 1u);
}

// members grouped by cluster (any order inside a cluster: ties are broken by the point index, not by position)
__global__ void __launch_bounds__(256) k_knn_group(const int32_t* __restrict__ cluster_of, int64_t n, const uint32_t* __restrict__ start,
                                                   uint32_t* __restrict__ cursor, int32_t* __restrict__ members) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t r = cluster_of[i];
    members[start[r] + atomicAdd(&cursor[r], 1u)] = (int32_t)i;
}

// ---------------------------------------------------------------- stage 1: the float32 filter on the matrix cores
// One workgroup = 64 queries of one cluster (4 wavefronts x 16), looping over the cluster's points 16 at a time.
// 16x16x4 tile: A = the 16 candidates (lane l supplies A[i = l % 16][k = l / 16]), B = the 16 queries (lane l supplies
// B[k = l / 16][j = l % 16]), D[i][j] in lane l for j = l % 16, i = 4 (l / 16) + v, v = 0..3.  The queries' rows stay in
// registers for the whole loop (D4 = ceil(d / 4) values per lane); the candidates' rows are staged through LDS,
// double-buffered (their point ids one tile further ahead, so that the row loads do not wait for an index load),
// rows padded to 4 D4 + 2 words so that the 32 lanes of a half wavefront hit 32 different banks.  (Four planes by
// column mod 4 with one 16-byte LDS load per four multiplications measured 10-60 % slower: bank conflicts.)
//
// Selection: every query owns an unsorted array of (key, point) pairs in LDS with room for K' + kSpare entries and a
// threshold tau (inf until K' pairs are there).  A candidate with key < tau is appended (one LDS counter increment, two
// stores: no search, no shifting).  When fewer than 16 free slots are left (one tile can bring 16 per query) the
// wavefront compacts that query's array together: every lane takes an entry, counts the entries that precede it in
// (key, point), the K' first stay, tau becomes the K'-th key.  Everything rejected or dropped has key >= the final tau.
constexpr int kSpare = 40;
template <int D4>
__global__ void __launch_bounds__(kFilterBlock) k_knn_filter(const float* __restrict__ X, int32_t d, const float* __restrict__ norm,
                                                            const int32_t* __restrict__ members, const uint32_t* __restrict__ start,
                                                            const KnnBlock* __restrict__ blocks, int32_t list_len,
                                                            int32_t* __restrict__ cand, float* __restrict__ tau_out) {
    constexpr int kRow = 4 * D4 + 2;
    constexpr int kTileWords = kTile * kRow;
    const int cap = list_len + kSpare;                        // <= 128: two entries per lane in a compaction
    extern __shared__ float lds[];
    float* tile = lds;                                        // [2][kTile][kRow]
    float* tnorm = tile + 2 * kTileWords;                     // [2][kTile]
    int32_t* tile_pt = (int32_t*)(tnorm + 2 * kTile);         // [2][kTile] point of each staged candidate (-1: none)
    int32_t* ahead_pt = tile_pt + 2 * kTile;                  // [2][kTile] points of the tile after the staged one
    float* akey = (float*)(ahead_pt + 2 * kTile);             // [kBlockQueries][cap]
    int32_t* apt = (int32_t*)(akey + kBlockQueries * cap);    // [kBlockQueries][cap]
    uint32_t* fill = (uint32_t*)(apt + kBlockQueries * cap);  // [kBlockQueries]
    float* qtau = (float*)(fill + kBlockQueries);             // [kBlockQueries]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const KnnBlock blk = blocks[blockIdx.x];
    const uint32_t c0 = start[blk.cluster], c1 = start[blk.cluster + 1];
    const int32_t n_r = (int32_t)(c1 - c0);
    // this lane's query and its slice of the row
    const int jq = wave * kWaveQueries + (lane & 15);          // query of the workgroup this lane works for
    const int32_t qpos = blk.q0 + jq;
    const int32_t qpt = qpos < n_r ? members[c0 + qpos] : -1;
    float breg[D4];
#pragma unroll
    for (int t = 0; t < D4; ++t) {
        const int col = 4 * t + (lane >> 4);
        breg[t] = (qpt >= 0 && col < d) ? X[(int64_t)qpt * d + col] : 0.f;
    }
    for (int x = tid; x < kBlockQueries; x += kFilterBlock) { fill[x] = 0u; qtau[x] = __builtin_inff(); }
    // staging: the loads of a tile's rows go out before the tile in the other buffer is multiplied, the values are
    // written to LDS after it; the points of the tile after that are fetched one iteration earlier still
    constexpr int kPerLane = (kTile * D4 * 4 + kFilterBlock - 1) / kFilterBlock;
    float sval[kPerLane];
    int32_t spt = -1, apt_next = -1;
    float snorm = 0.f;
    auto point_at = [&](int32_t pos) { return pos < n_r ? members[c0 + pos] : -1; };
    auto fetch = [&](int which, int32_t t0) {   // rows of the tile whose points sit in ahead_pt[which]
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const int x = min(tid + u * kFilterBlock, kTile * D4 * 4 - 1);
            const int row = x / (D4 * 4), col = x % (D4 * 4);
            const int32_t pt = ahead_pt[which * kTile + row];
            sval[u] = X[(int64_t)max(pt, 0) * d + min(col, d - 1)];   // always a valid address; masked when it is stored
        }
        if (tid < kTile) {
            spt = ahead_pt[which * kTile + tid];
            snorm = spt >= 0 ? norm[spt] : 0.f;
            apt_next = point_at(t0 + kTile + tid);            // the points of the tile after this one
        }
    };
    auto stash = [&](int buf, int which) {
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const int x = tid + u * kFilterBlock;
            const int row = x / (D4 * 4), col = x % (D4 * 4);
            if (x < kTile * D4 * 4)   // (nothing touches the loaded value before this point: the load stays in flight)
                tile[buf * kTileWords + row * kRow + col] = (ahead_pt[which * kTile + row] >= 0 && col < d) ? sval[u] : 0.f;
        }
        if (tid < kTile) {
            tile_pt[buf * kTile + tid] = spt;
            tnorm[buf * kTile + tid] = snorm;
            ahead_pt[(which ^ 1) * kTile + tid] = apt_next;
        }
    };
    if (tid < kTile) ahead_pt[tid] = point_at(tid);
    __syncthreads();
    fetch(0, 0);
    stash(0, 0);     // tile 0 in buffer 0, the points of tile 1 in ahead_pt[1]
    __syncthreads();
    // compaction of query j's array by the whole wavefront (j is the same for all lanes)
    auto compact = [&](int j) {
        float* ak = akey + j * cap;
        int32_t* ap = apt + j * cap;
        const int cnt = (int)min(fill[j], (uint32_t)cap);
        float k0 = __builtin_inff(), k1 = __builtin_inff();
        int32_t p0 = 0x7fffffff, p1 = 0x7fffffff;
        if (lane < cnt) { k0 = ak[lane]; p0 = ap[lane]; }
        if (lane + 64 < cnt) { k1 = ak[lane + 64]; p1 = ap[lane + 64]; }
        int r0 = 0, r1 = 0;   // entries that precede this lane's in (key, point); the others' entries come by lane broadcast
        const int first = min(cnt, 64), second = max(cnt - 64, 0);
        for (int o = 0; o < first; ++o) {
            const float ko = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(k0), o));
            const int32_t po = __builtin_amdgcn_readlane(p0, o);
            r0 += (ko < k0 || (ko == k0 && po < p0)) ? 1 : 0;
            r1 += (ko < k1 || (ko == k1 && po < p1)) ? 1 : 0;
        }
        for (int o = 0; o < second; ++o) {
            const float ko = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(k1), o));
            const int32_t po = __builtin_amdgcn_readlane(p1, o);
            r0 += (ko < k0 || (ko == k0 && po < p0)) ? 1 : 0;
            r1 += (ko < k1 || (ko == k1 && po < p1)) ? 1 : 0;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (lane < cnt && r0 < list_len) { ak[r0] = k0; ap[r0] = p0; }
        if (lane + 64 < cnt && r1 < list_len) { ak[r1] = k1; ap[r1] = p1; }
        if (cnt >= list_len) {
            if (lane < cnt && r0 == list_len - 1) qtau[j] = k0;
            if (lane + 64 < cnt && r1 == list_len - 1) qtau[j] = k1;
            if (lane == 0) fill[j] = (uint32_t)list_len;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    int buf = 0;
    for (int32_t t0 = 0; t0 < n_r; t0 += kTile, buf ^= 1) {
        const bool more = t0 + kTile < n_r;
        if (more) fetch(buf ^ 1, t0 + kTile);   // the next tile's rows are on their way while this one is multiplied
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        const float* arow = tile + buf * kTileWords + (lane & 15) * kRow + (lane >> 4);
#pragma unroll
        for (int t = 0; t < D4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(arow[4 * t], breg[t], acc, 0, 0, 0);
        const float tau = qtau[jq];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 4 * (lane >> 4) + v;
            const int32_t cpt = tile_pt[buf * kTile + i];
            const float key = tnorm[buf * kTile + i] - 2.f * acc[v];
            if (cpt >= 0 && cpt != qpt && qpt >= 0 && key < tau) {
                const uint32_t slot = atomicAdd(&fill[jq], 1u);   // a tile brings at most 16 per query: room is kept below
                akey[jq * cap + slot] = key;
                apt[jq * cap + slot] = cpt;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // queries of this wavefront whose array could not take another tile
        unsigned long long need = __ballot((lane < kWaveQueries) && fill[wave * kWaveQueries + lane] + kTile > (uint32_t)cap);
        while (need) {
            const int j = __builtin_ctzll(need);
            need &= need - 1;
            compact(wave * kWaveQueries + j);
        }
        if (more) stash(buf ^ 1, buf ^ 1);
        __syncthreads();   // the other buffer is staged, this one is free
    }
    // the K' best of every query and the K'-th key (inf while fewer than K' were ever there: then nothing was left out)
    for (int j = 0; j < kWaveQueries; ++j) compact(wave * kWaveQueries + j);
    if ((lane >> 4) == 0 && qpt >= 0) {
        const int64_t p = (int64_t)c0 + qpos;
        const int cnt = (int)min(fill[jq], (uint32_t)list_len);
        for (int x = 0; x < list_len; ++x) cand[p * list_len + x] = x < cnt ? apt[jq * cap + x] : -1;
        tau_out[p] = qtau[jq];
    }
}

__host__ __device__ inline size_t knn_filter_lds_bytes(int d4, int list_len) {
    return ((size_t)2 * kTile * (4 * d4 + 2) + 6 * kTile + (size_t)2 * kBlockQueries * (list_len + kSpare) + 2 * kBlockQueries) * 4;
}

// the oracle's distance: difference, product and running sum each rounded once, in float64, t = 0..d-1 in order
__device__ __forceinline__ double exact_distance(const float* __restrict__ x, const float* __restrict__ y, int32_t d) {
    double acc = 0.0;
    int t = 0;
    if ((d & 3) == 0) {   // rows are 16-byte aligned: four values per load, still added one by one in order
        for (; t < d; t += 4) {
            const float4 a = *(const float4*)(x + t), b = *(const float4*)(y + t);
            double diff = (double)a.x - (double)b.x;
            acc = __dadd_rn(acc, __dmul_rn(diff, diff));
            diff = (double)a.y - (double)b.y;
            acc = __dadd_rn(acc, __dmul_rn(diff, diff));
            diff = (double)a.z - (double)b.z;
            acc = __dadd_rn(acc, __dmul_rn(diff, diff));
            diff = (double)a.w - (double)b.w;
            acc = __dadd_rn(acc, __dmul_rn(diff, diff));
        }
        return acc;
    }
    for (; t < d; ++t) {
        const double diff = (double)x[t] - (double)y[t];
        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
    }
    return acc;
}

// ---------------------------------------------------------------- stage 2: exact distances of the candidates
// One wavefront per query, one lane per candidate.  rank = number of candidates that come before in (distance, point).
// The answer is certified when the k-th exact key, D_k - |q|^2, lies below tau by more than eps: every point the
// filter left out has float32 key >= tau, hence exact key >= tau - eps.  eps = 4 (d + 4) 2^-24 max|x|^2 bounds the
// rounding of the float32 norm, dot product and their combination for any pair of the cluster.
__global__ void __launch_bounds__(256) k_knn_refine(const float* __restrict__ X, int32_t d, const int32_t* __restrict__ members,
                                                    const int32_t* __restrict__ cluster_of, const uint32_t* __restrict__ max_norm_bits,
                                                    const int32_t* __restrict__ cand, const float* __restrict__ tau, int64_t n,
                                                    int32_t k, int32_t list_len, int32_t* __restrict__ out,
                                                    int32_t* __restrict__ flagged, uint32_t* __restrict__ n_flagged) {
    const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // position in the member order
    const int lane = threadIdx.x & 63;
    if (p >= n) return;
    const int32_t q = members[p];
    const float* xq = X + (int64_t)q * d;
    const int32_t c = lane < list_len ? cand[p * list_len + lane] : -1;
    const double D = c >= 0 ? exact_distance(xq, X + (int64_t)c * d, d) : __builtin_inf();
    int rank = 0, cnt = 0;
    for (int o = 0; o < list_len; ++o) {
        const double Do = __shfl(D, o, 64);
        const int32_t co = __shfl(c, o, 64);
        if (co >= 0) {
            ++cnt;
            if (Do < D || (Do == D && co < c)) ++rank;
        }
    }
    if (c >= 0 && rank < k) out[(int64_t)q * k + rank] = c;
    if (lane >= cnt && lane < k) out[(int64_t)q * k + lane] = -1;   // cluster smaller than k + 1
    // certification by the lane that holds the k-th neighbour (only needed when something was left out)
    const float t = tau[p];
    if (c >= 0 && rank == min(k, cnt) - 1 && t < __builtin_inff() && cnt >= k) {
        double qn = 0.0;
        for (int x = 0; x < d; ++x) qn = fma((double)xq[x], (double)xq[x], qn);
        const double M = (double)__uint_as_float(max_norm_bits[cluster_of[q]]);
        const double eps = 4.0 * (double)(d + 4) * 5.9604644775390625e-08 * M * 1.01 + 1e-12 * M;
        if (!(D - qn + eps < (double)t)) flagged[atomicAdd(n_flagged, 1u)] = q;
    }
}

// ---------------------------------------------------------------- stage 3: flagged queries, exactly, against the whole cluster
// One workgroup per flagged query: k rounds, each picking the smallest (distance, point) above the one picked before.
__global__ void __launch_bounds__(256) k_knn_exact(const float* __restrict__ X, int32_t d, const int32_t* __restrict__ members,
                                                   const uint32_t* __restrict__ start, const int32_t* __restrict__ cluster_of,
                                                   const int32_t* __restrict__ flagged, int32_t k, int32_t* __restrict__ out) {
    __shared__ double sD[256];
    __shared__ int32_t sP[256];
    const int32_t q = flagged[blockIdx.x];
    const int32_t r = cluster_of[q];
    const uint32_t c0 = start[r], c1 = start[r + 1];
    const float* xq = X + (int64_t)q * d;
    double lastD = -1.0;
    int32_t lastP = -1;
    for (int m = 0; m < k; ++m) {
        double bestD = __builtin_inf();
        int32_t bestP = -1;
        for (uint32_t pos = c0 + threadIdx.x; pos < c1; pos += 256) {
            const int32_t c = members[pos];
            if (c == q) continue;
            const double D = exact_distance(xq, X + (int64_t)c * d, d);
            const bool after = D > lastD || (D == lastD && c > lastP);
            const bool better = D < bestD || (D == bestD && (bestP < 0 || c < bestP));
            if (after && better) { bestD = D; bestP = c; }
        }
        sD[threadIdx.x] = bestD;
        sP[threadIdx.x] = bestP;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) {
                const double Do = sD[threadIdx.x + w];
                const int32_t Po = sP[threadIdx.x + w];
                const bool take = Po >= 0 && (sP[threadIdx.x] < 0 || Do < sD[threadIdx.x] || (Do == sD[threadIdx.x] && Po < sP[threadIdx.x]));
                if (take) { sD[threadIdx.x] = Do; sP[threadIdx.x] = Po; }
            }
            __syncthreads();
        }
        lastD = sD[0];
        lastP = sP[0];
        if (threadIdx.x == 0) out[(int64_t)q * k + m] = lastP;   // -1 once the cluster is exhausted
        __syncthreads();
        if (lastP < 0) {   // nothing left: the remaining slots stay empty
            for (int x = m + 1 + threadIdx.x; x < k; x += 256) out[(int64_t)q * k + x] = -1;
            break;
        }
    }
}

}  // namespace nomad_knn

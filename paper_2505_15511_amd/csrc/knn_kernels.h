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
constexpr int32_t kEmptyPoint = 0x7fffff00;   // stand-ins for empty list slots: above every point index (n < 2^31 - 256)
// The filter's workgroup is 8 wavefronts.  Up to d = 384 each wavefront has 16 queries of its own and the whole of their
// rows in registers (128 queries share every staged tile).  At wider rows a lane's share of its query's row (d / 4
// values) would leave one wavefront per SIMD, so two wavefronts share 16 queries and hold half of the columns each
// (64 queries per workgroup): each multiplies its half, the two partial tiles are exchanged through LDS and added.
__host__ __device__ constexpr int knn_filter_waves(int) { return 8; }
__host__ __device__ constexpr int knn_filter_split(int d4) { return d4 >= 128 ? 2 : 1; }
__host__ __device__ constexpr int knn_filter_block_queries(int d4) { return kWaveQueries * knn_filter_waves(d4) / knn_filter_split(d4); }
// LDS buffers for the staged candidate tile: two, or one at the widest rows (see the kernel)
__host__ __device__ constexpr int knn_filter_buffers(int d4) { return d4 > 64 ? 1 : 2; }

// wavefronts per SIMD the filter is compiled for: narrow rows and short lists fit two workgroups per compute unit (128
// registers per lane), and the second workgroup is what hides the first one's tile barriers
__host__ __device__ constexpr int knn_filter_waves_per_simd(int d4, int L) { return d4 <= 32 && L <= 12 ? 4 : 2; }   // (also the L = 4 lists of a one-neighbour search)

struct KnnBlock { int32_t cluster; int32_t q0; };   // queries q0 .. of group `cluster`: one workgroup's share

// Queries and candidates, both cut into the same groups (group g: queries qmembers[qstart[g] .. qstart[g+1]), candidates
// cmembers[cstart[g] .. cstart[g+1])).  Nearest neighbours inside clusters: both are the data set grouped by cluster.
// K-Means assignment: one group, the queries are the points, the candidates the centroids.  Neighbourhoods of a sample
// of query points among all points: one group, the queries a gathered copy of the sampled rows.
struct KnnSets {
    const float* XQ;             // query rows
    const float* XC;             // candidate rows
    const int32_t* qmembers;     // query row of every position, or nullptr = the position itself
    const int32_t* cmembers;     // candidate row of every position, or nullptr = the position itself
    const uint32_t* qstart;      // [groups + 1]
    const uint32_t* cstart;      // [groups + 1]
    const float* cnorm;          // |c'|^2 of every candidate row (centred, float32)
    const float* centre;         // [groups][d] what both sides are centred on
    const int32_t* group_of_q;   // group of every query row, or nullptr = group 0
    const uint32_t* max_norm_bits;   // [groups] largest centred |.|^2 over the group's queries and candidates
    int64_t n_q, n_c;            // rows of XQ, XC
    int32_t d;
    int32_t same_set;            // 1: queries and candidates are the same rows: a row is not its own neighbour
    const int32_t* self_row;     // or, per query row, the candidate row that is the query itself (nullptr: see same_set)
    float* key2;                 // nullptr, or [2 n_q]: the filter leaves every query's two smallest float32 keys here and the
                                 // refinement of a k = 1 search reads them (a clear winner needs no float64 distance)
};

// bound on |float32 key - exact key| of the filter for rows of d values whose centred squared norms are at most M
__device__ __forceinline__ double knn_filter_eps(int32_t d, double M) {
    return (4.0 * (double)(d + 4) + 8.0) * 5.9604644775390625e-08 * M * 1.01 + 1e-12 * M;
}
__device__ __forceinline__ int32_t knn_row(const int32_t* members, uint32_t pos) { return members ? members[pos] : (int32_t)pos; }

// Distances do not change when a cluster is moved as a whole, and the float32 error of the filter grows with |x|^2:
// the filter therefore works on rows centred on their cluster, x' = fl(x - c_r), c_r = the cluster's mean in float32.
// Column sums of a cluster, a slab of rows per block, one thread per column:
constexpr int kCentroidRows = 1024;
__global__ void __launch_bounds__(256) k_knn_centroid_sums(const float* __restrict__ X, int32_t d, const int32_t* __restrict__ members,
                                                           const uint32_t* __restrict__ start, const KnnBlock* __restrict__ slabs,
                                                           float* __restrict__ centre) {
    const KnnBlock sl = slabs[blockIdx.x];   // rows q0 .. q0 + kCentroidRows of cluster sl.cluster
    const uint32_t c0 = start[sl.cluster], c1 = start[sl.cluster + 1];
    const uint32_t r0 = c0 + (uint32_t)sl.q0, r1 = min(c1, r0 + (uint32_t)kCentroidRows);
    for (int col = threadIdx.x; col < d; col += 256) {
        float s = 0.f;
        uint32_t r = r0;
        for (; r + 16 <= r1; r += 16) {   // sixteen rows in flight
            int32_t row[16];
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) row[u] = knn_row(members, r + u);
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = X[(int64_t)row[u] * d + col];
#pragma unroll
            for (int u = 0; u < 16; ++u) s += v[u];
        }
        for (; r < r1; ++r) s += X[(int64_t)knn_row(members, r) * d + col];
        atomicAdd(&centre[(int64_t)sl.cluster * d + col], s);
    }
}
__global__ void __launch_bounds__(256) k_knn_centroid_finish(float* __restrict__ centre, const uint32_t* __restrict__ start, int32_t R, int32_t d) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= (int64_t)R * d) return;
    const int32_t r = (int32_t)(x / d);
    const uint32_t cnt = start[r + 1] - start[r];
    centre[x] = cnt ? centre[x] / (float)cnt : 0.f;
}

// |x'|^2 of every centred row in float32 and the largest one per cluster.  Sixteen lanes share a row (a wavefront reads
// four consecutive rows, each lane every sixteenth column or 16-byte chunk) and add their partial sums pairwise; any
// summation order stays within the d u |x'|^2 that the filter's error bound allows for the norm.
constexpr int kNormLanes = 16;
constexpr int kNormRows = 256 / kNormLanes;   // rows per workgroup
__global__ void __launch_bounds__(256) k_knn_norms(const float* __restrict__ X, int64_t n, int32_t d, const int32_t* __restrict__ cluster_of,
                                                   const float* __restrict__ centre, float* __restrict__ norm,
                                                   uint32_t* __restrict__ max_norm_bits) {
    const int64_t i = (int64_t)blockIdx.x * kNormRows + threadIdx.x / kNormLanes;
    const int part = threadIdx.x % kNormLanes;
    const bool valid = i < n;
    int32_t g = 0;
    float s = 0.f;
    if (valid) {
        const float* x = X + i * d;
        g = cluster_of ? cluster_of[i] : 0;
        const float* c = centre + (int64_t)g * d;
        if ((d & 3) == 0) {
            for (int t = 4 * part; t < d; t += 4 * kNormLanes) {
                const float4 xv = *(const float4*)(x + t), cv = *(const float4*)(c + t);
                float v = xv.x - cv.x;
                s = fmaf(v, v, s);
                v = xv.y - cv.y;
                s = fmaf(v, v, s);
                v = xv.z - cv.z;
                s = fmaf(v, v, s);
                v = xv.w - cv.w;
                s = fmaf(v, v, s);
            }
        } else {
            for (int t = part; t < d; t += kNormLanes) {
                const float v = x[t] - c[t];
                s = fmaf(v, v, s);
            }
        }
    }
    for (int w = kNormLanes / 2; w > 0; w >>= 1) s += __shfl_xor(s, w, kNormLanes);   // every lane of the row: the row's sum
    if (valid && part == 0 && norm) norm[i] = s;
    // non-negative floats order like their bit patterns; one atomic per wavefront where it lies inside one group
    const unsigned long long live = __ballot(valid);
    if (!live) return;
    const int first = __ffsll((long long)live) - 1;
    const int32_t g0 = __shfl(g, first, 64);
    uint32_t bits = valid ? __float_as_uint(s) : 0u;
    if (__all(!valid || g == g0)) {
        for (int w = 32; w > 0; w >>= 1) bits = max(bits, (uint32_t)__shfl_xor((int)bits, w, 64));
        if ((int)(threadIdx.x & 63) == first && bits > max_norm_bits[g0]) atomicMax(&max_norm_bits[g0], bits);
    } else if (valid && part == 0 && bits > max_norm_bits[g]) {   // the maximum only grows: a stale read costs one atomic, not the result
        atomicMax(&max_norm_bits[g], bits);
    }
}

// cluster sizes; a block counts kCountSpan labels in LDS first where the clusters are few enough to fit there
constexpr int kCountSpan = 16384;
constexpr int kCountLds = 4096;
__global__ void __launch_bounds__(256) k_knn_count(const int32_t* __restrict__ cluster_of, int64_t n, int32_t R, uint32_t* __restrict__ counts,
                                                   int* __restrict__ bad) {
    __shared__ uint32_t h[kCountLds];
    const bool local = R <= kCountLds;
    if (local) {
        for (int r = threadIdx.x; r < R; r += 256) h[r] = 0u;
        __syncthreads();
    }
    const int64_t i0 = (int64_t)blockIdx.x * kCountSpan, i1 = min(n, i0 + kCountSpan);
    for (int64_t i = i0 + threadIdx.x; i < i1; i += 256) {
        const int32_t r = cluster_of[i];
        if (r < 0 || r >= R) { *bad = 1; continue; }
        if (local) atomicAdd(&h[r], 1u);
        else atomicAdd(&counts[r], 1u);
    }
    if (local) {
        __syncthreads();
        for (int r = threadIdx.x; r < R; r += 256)
            if (h[r]) atomicAdd(&counts[r], h[r]);
    }
}

// members grouped by cluster (any order inside a cluster: ties are broken by the point index, not by position).  A
// workgroup takes kGroupSpan points: ranks inside the workgroup from an LDS counter per cluster, then one global
// reservation per cluster it met (clusters beyond kCountLds: one global atomic per point).
constexpr int kGroupSpan = 4096;
__global__ void __launch_bounds__(256) k_knn_group(const int32_t* __restrict__ cluster_of, int64_t n, int32_t R, const uint32_t* __restrict__ start,
                                                   uint32_t* __restrict__ cursor, int32_t* __restrict__ members) {
    __shared__ uint32_t h[kCountLds];     // count, then global base, of every cluster inside this workgroup's span
    const int64_t i0 = (int64_t)blockIdx.x * kGroupSpan;
    constexpr int kPer = kGroupSpan / 256;
    if (R > kCountLds) {
        for (int u = 0; u < kPer; ++u) {
            const int64_t i = i0 + u * 256 + threadIdx.x;
            if (i < n) { const int32_t r = cluster_of[i]; members[start[r] + atomicAdd(&cursor[r], 1u)] = (int32_t)i; }
        }
        return;
    }
    for (int r = threadIdx.x; r < R; r += 256) h[r] = 0u;
    __syncthreads();
    int32_t cl[kPer];
    uint32_t rk[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int64_t i = i0 + u * 256 + threadIdx.x;
        cl[u] = i < n ? cluster_of[i] : -1;
        rk[u] = cl[u] >= 0 ? atomicAdd(&h[cl[u]], 1u) : 0u;
    }
    __syncthreads();
    for (int r = threadIdx.x; r < R; r += 256)
        if (h[r]) h[r] = start[r] + atomicAdd(&cursor[r], h[r]);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kPer; ++u)
        if (cl[u] >= 0) members[h[cl[u]] + rk[u]] = (int32_t)(i0 + u * 256 + threadIdx.x);
}

// ---------------------------------------------------------------- stage 1: the float32 filter on the matrix cores
// One workgroup = 128 queries of one cluster (8 wavefronts x 16; 64 at the widest rows), looping over the cluster's
// points 16 at a time.
// 16x16x4 tile: A = the 16 candidates (lane l supplies A[i = l % 16][k = l / 16]), B = the 16 queries (lane l supplies
// B[k = l / 16][j = l % 16]), D[i][j] in lane l for j = l % 16, i = 4 (l / 16) + v, v = 0..3.  The queries' rows stay in
// registers for the whole loop (D4 = ceil(d / 4) values per lane).
//
// The candidates' rows are scattered over memory (a cluster's points are wherever the data set has them).  Thread t
// always copies the same 16-byte chunks of one row (32 threads per row); the
// loads of tile T+2 go out while tile T is multiplied (two register sets, the loop unrolled by two), tile T+1 is
// written to the other LDS buffer after the multiplications; the point behind each row is fetched one tile further
// ahead still, first thing in the iteration, so that no row load waits for an index.  LDS rows are padded to 4 D4 + 2
// words: the 32 lanes of a half wavefront then read 32 different banks.
//
// Selection: each of the four lanes of a query sees a quarter of the candidates (four per tile) and keeps the L
// smallest keys of that quarter, with their points, sorted in registers; a new key is pushed through the list with
// compare-and-swap steps, for all lanes at once whenever any lane of the wavefront has a key below its list's last.
// Every wavefront does the same work in every tile, so the tile barrier costs no waiting (an earlier version that
// compacted per-query arrays in LDS on demand spent 70 % of its time at that barrier).  At the end the four lists of
// a query are merged: the K' smallest keys go on, tau = min(K'-th key of the union, the four lists' last keys):
// every candidate that is not passed on has key >= tau.
template <int D4, int L>
__global__ void __launch_bounds__(64 * knn_filter_waves(D4), knn_filter_waves_per_simd(D4, L)) k_knn_filter(const KnnSets P, const KnnBlock* __restrict__ blocks, int32_t list_len,
                                                                         int32_t* __restrict__ cand, float* __restrict__ tau_out) {
    const float* __restrict__ X = P.XC;        // candidate rows (the loop's stream)
    const float* __restrict__ norm = P.cnorm;
    const int32_t d = P.d;
    constexpr int kFilterBlock = 64 * knn_filter_waves(D4);
    constexpr int kRow = 4 * D4 + 2;
    constexpr int kTileWords = kTile * kRow;
    constexpr int kRowThreads = kFilterBlock / kTile;          // 32 threads copy one row
    constexpr int kChunks = (D4 + kRowThreads - 1) / kRowThreads;   // 16-byte chunks per thread and tile
    constexpr bool kTwoAhead = D4 <= 64;                      // two tiles of rows in flight where the registers allow it
    constexpr int kBuffers = knn_filter_buffers(D4);          // LDS tile buffers
    constexpr int kMerge = 4 * L;                             // entries of a query's four lists
    extern __shared__ float lds[];
    float* tile = lds;                                        // [kBuffers][kTile][kRow]
    float* tnorm = tile + kBuffers * kTileWords;              // [2][kTile]
    int32_t* tile_pt = (int32_t*)(tnorm + 2 * kTile);         // [2][kTile] point of each staged candidate (-1: none)
    float* mkey = (float*)(tile_pt + 2 * kTile);              // [waves][4][kMerge] merge scratch of four queries per wavefront
    int32_t* mpt = (int32_t*)(mkey + knn_filter_waves(D4) * 4 * kMerge);   // [waves][4][kMerge]
    floatx4* xch = (floatx4*)(mpt + knn_filter_waves(D4) * 4 * kMerge);    // [waves][64] partial tiles (split rows only; 16-byte aligned)
    constexpr int kSplit = knn_filter_split(D4);                       // wavefronts that share 16 queries
    constexpr int KH = D4 / kSplit;                                    // 4-column steps per wavefront
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = wave % kSplit;                                    // which part of the columns this wavefront multiplies
    const KnnBlock blk = blocks[blockIdx.x];
    const uint32_t c0 = P.cstart[blk.cluster], c1 = P.cstart[blk.cluster + 1];
    const int32_t n_r = (int32_t)(c1 - c0);                    // candidates of the group
    const uint32_t q0g = P.qstart[blk.cluster];
    const int32_t n_qg = (int32_t)(P.qstart[blk.cluster + 1] - q0g);   // queries of the group
    // this lane's query and its slice of the row
    const int32_t qpos = blk.q0 + (wave / kSplit) * kWaveQueries + (lane & 15);
    const int32_t qpt = qpos < n_qg ? knn_row(P.qmembers, q0g + qpos) : -1;
    // the candidate that is the query itself, if any
    const int32_t self = qpt < 0 ? -1 : P.self_row ? P.self_row[qpt] : P.same_set ? qpt : -1;
    const float* ctr = P.centre + (int64_t)blk.cluster * d;    // the group's centre: every row enters as x - centre
    float breg[KH];
#pragma unroll
    for (int t = 0; t < KH; ++t) {
        const int col = 4 * (half * KH + t) + (lane >> 4);
        breg[t] = (qpt >= 0 && col < d) ? P.XQ[(int64_t)qpt * d + col] - ctr[col] : 0.f;
    }
    float lk[L];      // this lane's L smallest keys so far, ascending
    int32_t lp[L];    // and their points
#pragma unroll
    for (int x = 0; x < L; ++x) { lk[x] = __builtin_inff(); lp[x] = -1; }

    // ---- staging
    const int srow = tid / kRowThreads, sthr = tid % kRowThreads;   // this thread's row of every tile and its place in it
    const bool vec = (d & 3) == 0;                                  // rows are 16-byte aligned
    struct Staged { float4 v[kChunks]; int32_t pt; float nrm; };
    // the centre at this thread's columns: in registers, or at the widest rows (where registers are short) in LDS
    constexpr bool kKeepCentre = D4 < 192;
    float* lds_centre = (float*)(xch + (kSplit == 2 ? knn_filter_waves(D4) * 64 : 0));   // [4 D4] (widest rows only)
    if (!kKeepCentre) {
        for (int col = tid; col < 4 * D4; col += kFilterBlock) lds_centre[col] = col < d ? ctr[col] : 0.f;
        __syncthreads();
    }
    auto centre_at = [&](int u) {
        const int col = 4 * (sthr + u * kRowThreads);
        return make_float4(col < d ? ctr[col] : 0.f, col + 1 < d ? ctr[col + 1] : 0.f, col + 2 < d ? ctr[col + 2] : 0.f,
                           col + 3 < d ? ctr[col + 3] : 0.f);
    };
    float4 cchunk[kKeepCentre ? kChunks : 1];
    if (kKeepCentre) {
#pragma unroll
        for (int u = 0; u < kChunks; ++u) cchunk[u] = centre_at(u);
    }
    auto point_at = [&](int32_t pos) { return pos < n_r ? knn_row(P.cmembers, c0 + pos) : -1; };
    // loads of this thread's chunks of the row of point pt (any valid row when pt < 0; masked when it is stored)
    auto fetch = [&](Staged& S, int32_t pt) {
        S.pt = pt;
        const float* row = X + (int64_t)max(pt, 0) * d;
        S.nrm = norm[max(pt, 0)];
#pragma unroll
        for (int u = 0; u < kChunks; ++u) {
            const int col = 4 * (sthr + u * kRowThreads);
            if (vec) {
                S.v[u] = *(const float4*)(row + min(col, d - 4));
            } else {
                S.v[u].x = row[min(col, d - 1)];
                S.v[u].y = row[min(col + 1, d - 1)];
                S.v[u].z = row[min(col + 2, d - 1)];
                S.v[u].w = row[min(col + 3, d - 1)];
            }
        }
    };
    // (nothing touches the loaded values before they are stored: the loads stay in flight until then)
    auto stash = [&](const Staged& S, int buf) {
        float* dst = tile + buf * kTileWords + srow * kRow;
#pragma unroll
        for (int u = 0; u < kChunks; ++u) {
            const int col = 4 * (sthr + u * kRowThreads);
            if (col < 4 * D4) {
                const bool live = S.pt >= 0;
                const float4 cc = kKeepCentre ? cchunk[kKeepCentre ? u : 0] : *(const float4*)(lds_centre + col);
                float2 lo = make_float2((live && col < d) ? S.v[u].x - cc.x : 0.f, (live && col + 1 < d) ? S.v[u].y - cc.y : 0.f);
                float2 hi = make_float2((live && col + 2 < d) ? S.v[u].z - cc.z : 0.f, (live && col + 3 < d) ? S.v[u].w - cc.w : 0.f);
                *(float2*)(dst + col) = lo;        // rows start on even words: 8-byte stores
                *(float2*)(dst + col + 2) = hi;
            }
        }
        // a row that stands for no candidate gets an infinite norm: its key is infinite whatever the (zero) product
        if (sthr == 0) { tile_pt[buf * kTile + srow] = S.pt; tnorm[buf * kTile + srow] = S.pt >= 0 ? S.nrm : __builtin_inff(); }
    };
    // multiply the tile in LDS buffer `buf` with this wavefront's queries, push what beats the lists' last keys
    auto consume = [&](int buf) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        const float* arow = tile + buf * kTileWords + (lane & 15) * kRow + (lane >> 4) + 4 * half * KH;
        if (D4 < 64) {
#pragma unroll
            for (int t = 0; t < KH; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(arow[4 * t], breg[t], acc, 0, 0, 0);
        } else {
            // Rows of 256 columns and more: the candidates' values come from LDS in batches of kBatch, the next batch on its way while this one
            // is multiplied (left to itself the compiler reads each value right before its multiplication and waits for it).
            constexpr int kBatch = 8;
            float a_cur[kBatch], a_nxt[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) a_cur[u] = arow[4 * u];
#pragma unroll
            for (int tb = 0; tb < KH; tb += kBatch) {
                if (tb + kBatch < KH) {
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) a_nxt[u] = arow[4 * (tb + kBatch + u)];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < kBatch; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[u], breg[tb + u], acc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < kBatch; ++u) a_cur[u] = a_nxt[u];
            }
        }
        if (kSplit == 2) {   // the other half of the columns: a + b and b + a are the same number, both wavefronts go on alike
            xch[wave * 64 + lane] = acc;
            __syncthreads();
            const floatx4 other = xch[(wave ^ 1) * 64 + lane];
            acc[0] += other[0]; acc[1] += other[1]; acc[2] += other[2]; acc[3] += other[3];
        }
        float ck[4];      // this lane's four candidates of the tile
        int32_t cp[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = 4 * (lane >> 4) + v;
            cp[v] = tile_pt[buf * kTile + i];
            ck[v] = tnorm[buf * kTile + i] - 2.f * acc[v];
            if (cp[v] == self) ck[v] = __builtin_inff();   // (lanes without a query collect keys nobody reads)
        }
        if (L == 2) {
            // One neighbour wanted: a lane keeps its best two, and the tile's four candidates go in one after the other
            // without asking whether any lane has a hit (two comparisons and six selections each).
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool lt0 = ck[v] < lk[0], lt1 = ck[v] < lk[1];
                lk[1] = lt0 ? lk[0] : (lt1 ? ck[v] : lk[1]);
                lp[1] = lt0 ? lp[0] : (lt1 ? cp[v] : lp[1]);
                lk[0] = lt0 ? ck[v] : lk[0];
                lp[0] = lt0 ? cp[v] : lp[0];
            }
            return;
        }
        // Insertion passes run for the whole wavefront, so they are spent on the lane's best remaining candidate: some lane
        // has a hit in most tiles, a lane with two in one tile is rare, and the second pass is skipped when there is none.
#pragma nounroll   // a real loop: unrolled, every early exit would copy the whole list into the registers of the next tile
        for (int pass = 0; pass < 4; ++pass) {
            float xk = ck[0];
            int32_t xp = cp[0];
            int sel = 0;
#pragma unroll
            for (int v = 1; v < 4; ++v) {
                const bool less = ck[v] < xk;
                xk = less ? ck[v] : xk;
                xp = less ? cp[v] : xp;
                sel = less ? v : sel;
            }
            if (!__any(xk < lk[L - 1])) break;
#pragma unroll
            for (int v = 0; v < 4; ++v) ck[v] = sel == v ? __builtin_inff() : ck[v];
            // From the last slot down: a slot takes its left neighbour if the new key goes before that one, the new key if
            // it goes exactly here (L independent comparisons, no value carried along; an infinite key changes nothing).
#pragma unroll
            for (int x = L - 1; x >= 1; --x) {
                const bool left = xk < lk[x - 1], here = xk < lk[x];
                lk[x] = left ? lk[x - 1] : (here ? xk : lk[x]);
                lp[x] = left ? lp[x - 1] : (here ? xp : lp[x]);
            }
            {
                const bool here = xk < lk[0];
                lk[0] = here ? xk : lk[0];
                lp[0] = here ? xp : lp[0];
            }
        }
    };

    // tile T sits in LDS buffer T & 1
    if (kTwoAhead) {
        // Registers: S0 / S1 hold the rows of the even / odd tile that is on its way, pt_ahead the point of this
        // thread's row one tile beyond those.
        Staged S0, S1;
        fetch(S0, point_at(srow));                         // tile 0
        stash(S0, 0);
        fetch(S1, point_at(kTile + srow));                 // tile 1, stored at the end of iteration 0
        int32_t pt_ahead = point_at(2 * kTile + srow);     // tile 2's point
        __syncthreads();
        for (int32_t t0 = 0; t0 < n_r; t0 += 2 * kTile) {
            // ---- even tile T (buffer 0): tile T+2's rows go out into S0, tile T+1 (S1) is stored afterwards
            {
                const int32_t pt_use = pt_ahead;
                pt_ahead = point_at(t0 + 3 * kTile + srow);
                fetch(S0, pt_use);
                consume(0);
                stash(S1, 1);
                __syncthreads();
            }
            if (t0 + kTile >= n_r) break;
            // ---- odd tile T+1 (buffer 1): tile T+3's rows go out into S1, tile T+2 (S0) is stored afterwards
            {
                const int32_t pt_use = pt_ahead;
                pt_ahead = point_at(t0 + 4 * kTile + srow);
                fetch(S1, pt_use);
                consume(1);
                stash(S0, 0);
                __syncthreads();
            }
        }
    } else {
        // Wide rows: one tile of rows in flight (its multiplications take thousands of cycles) and a single LDS
        // buffer, which is what lets more than one workgroup share a compute unit: the next tile waits in registers
        // until every wavefront is done with the current one.
        Staged S;
        fetch(S, point_at(srow));
        stash(S, 0);
        int32_t pt_ahead = point_at(kTile + srow);         // tile 1's point
        __syncthreads();
        for (int32_t t0 = 0; t0 < n_r; t0 += kTile) {
            const int32_t pt_use = pt_ahead;
            pt_ahead = point_at(t0 + 2 * kTile + srow);
            fetch(S, pt_use);                              // tile T+1
            consume(0);
            __syncthreads();
            stash(S, 0);
            __syncthreads();
        }
    }

    // ---- merge the four lists of every query, four queries of the wavefront at a time: sixteen lanes per query, each
    // with up to kPerLane of the query's 4 L entries, which it ranks by counting the entries that precede them in
    // (key, point).  (Of two wavefronts that share their queries both hold the same lists: one of them reports.)
    if (half != 0) return;
    constexpr int kPerLane = (kMerge + 15) / 16;
    float* mk = mkey + wave * 4 * kMerge;        // [4 queries][kMerge]
    int32_t* mp = mpt + wave * 4 * kMerge;
    // the smallest of the four lists' last keys: what this query's lanes may have turned away
    float thr = lk[L - 1];
    thr = fminf(thr, __shfl_xor(thr, 16, 64));
    thr = fminf(thr, __shfl_xor(thr, 32, 64));
    for (int jb = 0; jb < kWaveQueries; jb += 4) {
        if (((lane & 15) >> 2) == (jb >> 2)) {   // the lanes of queries jb .. jb + 3 lay their lists out
            float* dk = mk + (lane & 3) * kMerge + (lane >> 4) * L;
            int32_t* dp = mp + (lane & 3) * kMerge + (lane >> 4) * L;
#pragma unroll
            for (int x = 0; x < L; ++x) { dk[x] = lk[x]; dp[x] = lp[x]; }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int g = lane >> 4, sub = lane & 15;            // this lane now works for query jb + g
        const float* qk = mk + g * kMerge;
        const int32_t* qp = mp + g * kMerge;
        // an empty slot (point -1) sorts after every real entry; empty slots get distinct stand-in points so that the
        // ranks stay a permutation and every one of the K' output slots is written
        float ek[kPerLane];
        int32_t ep[kPerLane];
        int er[kPerLane];
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const int e = sub + 16 * u;
            ek[u] = e < kMerge ? qk[e] : __builtin_inff();
            ep[u] = e < kMerge ? qp[e] : -1;
            if (ep[u] < 0) ep[u] = kEmptyPoint + e;
            er[u] = 0;
        }
#pragma unroll 4
        for (int o = 0; o < kMerge; ++o) {
            const float ko = qk[o];
            int32_t po = qp[o];
            if (po < 0) po = kEmptyPoint + o;
#pragma unroll
            for (int u = 0; u < kPerLane; ++u) er[u] += (ko < ek[u] || (ko == ek[u] && po < ep[u])) ? 1 : 0;
        }
        // the query's point, position and threshold, from a lane that owns it
        const int32_t jq_pt = __shfl(qpt, jb + g, 64);
        const int32_t jq_pos = __shfl(qpos, jb + g, 64);
        const float jq_thr = __shfl(thr, jb + g, 64);
        if (jq_pt >= 0) {
            const int64_t p = (int64_t)q0g + jq_pos;
            // fewer entries than K' (the best-two lists of a one-neighbour search): the lists' last keys alone bound what was
            // turned away; the slots beyond the entries keep their "no candidate" filling
            if (kMerge < list_len && sub == 0) tau_out[p] = jq_thr;
#pragma unroll
            for (int u = 0; u < kPerLane; ++u) {
                if (sub + 16 * u >= kMerge) continue;
                if (er[u] < list_len) cand[p * list_len + er[u]] = ep[u] >= kEmptyPoint ? -1 : ep[u];
                // tau: the K'-th key of the union (inf if there is none) and the lists' last keys
                if (er[u] == list_len - 1) tau_out[p] = fminf(ek[u], jq_thr);
                if (P.key2 && er[u] < 2) P.key2[2 * p + er[u]] = ek[u];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

__host__ __device__ inline size_t knn_filter_lds_bytes(int d4, int L) {
    return ((size_t)knn_filter_buffers(d4) * kTile * (4 * d4 + 2) + 4 * kTile + (size_t)2 * knn_filter_waves(d4) * 16 * L) * 4 +
           (knn_filter_split(d4) == 2 ? (size_t)knn_filter_waves(d4) * 64 * 16 : 0) + (d4 >= 192 ? (size_t)16 * d4 : 0);
}
// entries per lane's list for K' = list_len candidates per query: half of K', so that the four lists of a query hold 2 K'
__host__ inline int knn_filter_list_class(int list_len) { return list_len <= 9 ? 2 : list_len <= 16 ? 8 : list_len <= 24 ? 12 : 20; }

// the oracle's distance: difference, product and running sum each rounded once, in float64, t = 0..d-1 in order
__device__ __forceinline__ double exact_distance(const float* __restrict__ x, const float* __restrict__ y, int32_t d) {
    double acc = 0.0;
    int t = 0;
    if ((d & 3) == 0) {   // rows are 16-byte aligned: four values per load, still added one by one in order
        for (; t + 16 <= d; t += 16) {   // eight loads in flight before the first dependent addition
            float4 a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = *(const float4*)(x + t + 4 * u); b[u] = *(const float4*)(y + t + 4 * u); }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                double diff = (double)a[u].x - (double)b[u].x;
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                diff = (double)a[u].y - (double)b[u].y;
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                diff = (double)a[u].z - (double)b[u].z;
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                diff = (double)a[u].w - (double)b[u].w;
                acc = __dadd_rn(acc, __dmul_rn(diff, diff));
            }
        }
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
// One lane per candidate.  rank = number of candidates that come before in (distance, point).
// The answer is certified when the k-th exact key, D_k - |q|^2, lies below tau by more than eps: every point the
// filter left out has float32 key >= tau, hence exact key >= tau - eps.  With x' = fl(x - centre) the rows the filter
// saw and M = max |x'|^2 over the cluster, eps = (4 (d + 4) + 8) 2^-24 M bounds the rounding of the float32 norm,
// dot product and their combination (4 (d + 4) u M) plus what centring in float32 moves a distance by (8 u M).
// G lanes per query (16, 32 or 64, at least the list length): short lists share a wavefront between several queries.
template <int G>
__global__ void __launch_bounds__(256) k_knn_refine(const KnnSets P, const int32_t* __restrict__ cand, const float* __restrict__ tau,
                                                    int32_t k, int32_t list_len, int32_t* __restrict__ out,
                                                    int32_t* __restrict__ flagged, uint32_t* __restrict__ n_flagged) {
    const int64_t p = (int64_t)blockIdx.x * (256 / G) + (threadIdx.x / G);   // position in the grouped query order
    const int lane = threadIdx.x % G;
    const int32_t d = P.d;
    if (p >= P.n_q) return;
    int32_t q = knn_row(P.qmembers, (uint32_t)p);
    if (G == 64) q = __builtin_amdgcn_readfirstlane(q);   // the same for the whole wavefront
    const float* xq = P.XQ + (int64_t)q * d;
    int32_t c = lane < list_len ? cand[p * list_len + lane] : -1;
    if (c >= P.n_c) c = -1;   // never an address outside the candidate rows, whatever the list holds
    if (k == 1 && P.key2) {
        // One neighbour wanted: if the smallest float32 key lies below the second by more than twice the filter's error
        // bound, its candidate is the nearest in exact arithmetic too (every other candidate's key, kept or turned away,
        // is at least the second key), and no float64 distance is needed.
        const int32_t g1 = P.group_of_q ? P.group_of_q[q] : 0;
        const double eps1 = knn_filter_eps(d, (double)__uint_as_float(P.max_norm_bits[g1]));
        const double key0 = (double)P.key2[2 * p], key1 = (double)P.key2[2 * p + 1];
        if (key1 - key0 > 2.0 * eps1) {   // false for NaN (no candidate at all: inf - inf)
            if (lane == 0) out[(int64_t)q] = c;   // list slot 0 holds the smallest key's candidate
            return;
        }
    }
    const double D = c >= 0 ? exact_distance(xq, P.XC + (int64_t)c * d, d) : __builtin_inf();
    int rank = 0, cnt = 0;
    for (int o = 0; o < list_len; ++o) {
        const double Do = __shfl(D, o, G);
        const int32_t co = __shfl(c, o, G);
        if (co >= 0) {
            ++cnt;
            if (Do < D || (Do == D && co < c)) ++rank;
        }
    }
    if (c >= 0 && rank < k) out[(int64_t)q * k + rank] = c;
    if (lane >= cnt && lane < k) out[(int64_t)q * k + lane] = -1;   // fewer than k candidates in the group
    // certification by the lane that holds the k-th neighbour (only needed when something was left out).  |q'|^2 of the
    // centred query as the filter saw it: the group's lanes add a strided share each (the order is free: the value only
    // enters an inequality with slack).
    const float t = tau[p];
    const int32_t g = P.group_of_q ? P.group_of_q[q] : 0;
    double qn = 0.0;
    if (t < __builtin_inff() && cnt >= k) {   // the same for every lane of the group
        const float* ctr = P.centre + (int64_t)g * d;
        for (int x = lane; x < d; x += G) {
            const double v = (double)(xq[x] - ctr[x]);
            qn = fma(v, v, qn);
        }
        for (int w = G / 2; w > 0; w >>= 1) qn += __shfl_xor(qn, w, G);
    }
    if (c >= 0 && rank == min(k, cnt) - 1 && t < __builtin_inff() && cnt >= k) {
        const double eps = knn_filter_eps(d, (double)__uint_as_float(P.max_norm_bits[g]));
        if (!(D - qn + eps < (double)t)) flagged[atomicAdd(n_flagged, 1u)] = q;
    }
}

// ---------------------------------------------------------------- stage 3: flagged queries, exactly, against the whole cluster
// One workgroup per flagged query.  Every thread walks its share of the group once and keeps its own k smallest
// (distance, point) pairs sorted in registers (KL >= k slots); the k smallest of the group are among those, and k rounds
// pick them: each thread offers its smallest pair above the one picked before, the workgroup takes the smallest offer.
template <int KL>
__global__ void __launch_bounds__(256) k_knn_exact(const KnnSets P, const int32_t* __restrict__ flagged, int32_t k, int32_t* __restrict__ out) {
    __shared__ double sD[256];
    __shared__ int32_t sP[256];
    const int32_t d = P.d;
    const int32_t q = flagged[blockIdx.x];
    const int32_t r = P.group_of_q ? P.group_of_q[q] : 0;
    const uint32_t c0 = P.cstart[r], c1 = P.cstart[r + 1];
    const float* xq = P.XQ + (int64_t)q * d;
    const int32_t self = P.self_row ? P.self_row[q] : P.same_set ? q : -1;
    double lD[KL];      // ascending in (distance, point); empty slots: (inf, -1) at the end
    int32_t lP[KL];
#pragma unroll
    for (int x = 0; x < KL; ++x) { lD[x] = __builtin_inf(); lP[x] = -1; }
    double wD = __builtin_inf();   // the pair in slot k - 1 (point -1 while the list is not full)
    int32_t wP = -1;
    for (uint32_t pos = c0 + threadIdx.x; pos < c1; pos += 256) {
        const int32_t c = knn_row(P.cmembers, pos);
        if (c == self) continue;
        double xD = exact_distance(xq, P.XC + (int64_t)c * d, d);
        int32_t xP = c;
        // slot k - 1 is the list's last used slot: what does not come before it cannot be among this thread's k smallest
        if (!(wP < 0 || xD < wD || (xD == wD && xP < wP))) continue;
#pragma unroll
        for (int x = 0; x < KL; ++x) {
            if (x < k) {
                const bool take = xP >= 0 && (lP[x] < 0 || xD < lD[x] || (xD == lD[x] && xP < lP[x]));
                const double oD = lD[x];
                const int32_t oP = lP[x];
                lD[x] = take ? xD : oD;
                lP[x] = take ? xP : oP;
                xD = take ? oD : xD;
                xP = take ? oP : xP;
            }
        }
#pragma unroll
        for (int x = 0; x < KL; ++x)
            if (x == k - 1) { wD = lD[x]; wP = lP[x]; }
    }
    double lastD = -1.0;
    int32_t lastP = -1;
    for (int m = 0; m < k; ++m) {
        double bestD = __builtin_inf();
        int32_t bestP = -1;
#pragma unroll
        for (int x = KL - 1; x >= 0; --x) {   // descending, so that the first pair after the last pick is what remains
            const bool after = lP[x] >= 0 && (lD[x] > lastD || (lD[x] == lastD && lP[x] > lastP));
            bestD = after ? lD[x] : bestD;
            bestP = after ? lP[x] : bestP;
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
        if (threadIdx.x == 0) out[(int64_t)q * k + m] = lastP;   // -1 once the group is exhausted
        __syncthreads();
        if (lastP < 0) {   // nothing left: the remaining slots stay empty
            for (int x = m + 1 + threadIdx.x; x < k; x += 256) out[(int64_t)q * k + x] = -1;
            break;
        }
    }
}

// ---------------------------------------------------------------- Lloyd's iterations (the K-Means index of Section 3.2)
__global__ void __launch_bounds__(256) k_iota(int32_t* __restrict__ v, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) v[i] = (int32_t)i;
}

// ---- stable sort of the points by label (the M step adds a cluster's rows in ascending point order)
// Least-significant-digit radix passes of 8 bits over (label, point) pairs.  A workgroup of 256 lanes owns kSortSpan
// consecutive positions of a pass's input: it counts its digits (k_sort_count), an exclusive scan over the counts in
// (digit, workgroup) order gives every workgroup the first output slot of each of its digits (two levels), and the
// scatter (k_sort_scatter) ranks the pairs of a chunk of 256 in input order: inside a wavefront by the lanes below
// with the same digit (eight ballots), across wavefronts by their counts taken in wavefront order, across chunks by a
// running slot per digit.  Equal digits keep their input order in every pass, so equal labels end up in ascending
// point order.
constexpr int kSortSpan = 2048;

__global__ void __launch_bounds__(256) k_sort_count(const int32_t* __restrict__ keys, int64_t n, int shift, uint32_t n_blocks,
                                                    uint32_t* __restrict__ hist) {   // hist [256][n_blocks]
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0u;
    __syncthreads();
    const int64_t i0 = (int64_t)blockIdx.x * kSortSpan;
    for (int u = 0; u < kSortSpan / 256; ++u) {
        const int64_t i = i0 + u * 256 + threadIdx.x;
        if (i < n) atomicAdd(&h[((uint32_t)keys[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * n_blocks + blockIdx.x] = h[threadIdx.x];
}

// Exclusive scan of the m counters in two levels: every workgroup scans a tile of kScanTile consecutive counters in
// place and reports the tile's total (k_sort_scan_tiles); one workgroup scans the totals (k_sort_scan); the scatter adds
// a counter's tile offset when it reads it.
constexpr int kScanTile = 2048;

__global__ void __launch_bounds__(256) k_sort_scan_tiles(uint32_t* __restrict__ hist, uint64_t m, uint32_t* __restrict__ tile_total) {
    __shared__ uint32_t wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t x0 = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * 8;
    uint32_t v[8];
    uint32_t own = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) { v[u] = x0 + u < m ? hist[x0 + u] : 0u; own += v[u]; }
    uint32_t incl = own;
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        const uint32_t up = __shfl_up(incl, dlt, 64);
        if (lane >= dlt) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t run = incl - own;
    for (int w = 0; w < wave; ++w) run += wave_sum[w];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        if (x0 + u < m) hist[x0 + u] = run;
        run += v[u];
    }
    if (threadIdx.x == 255) tile_total[blockIdx.x] = run;
}

// exclusive scan of m counters in place; one workgroup, every lane a contiguous share
__global__ void __launch_bounds__(1024) k_sort_scan(uint32_t* __restrict__ hist, uint64_t m) {
    __shared__ uint32_t part[1024];
    const uint64_t per = (m + 1023) / 1024;
    const uint64_t a = min(m, (uint64_t)threadIdx.x * per), b = min(m, a + per);
    uint32_t own = 0;
    for (uint64_t x = a; x < b; ++x) own += hist[x];
    part[threadIdx.x] = own;
    __syncthreads();
    for (int dlt = 1; dlt < 1024; dlt <<= 1) {
        const uint32_t v = (int)threadIdx.x >= dlt ? part[threadIdx.x - dlt] : 0u;
        __syncthreads();
        part[threadIdx.x] += v;
        __syncthreads();
    }
    uint32_t run = part[threadIdx.x] - own;
    for (uint64_t x = a; x < b; ++x) { const uint32_t c = hist[x]; hist[x] = run; run += c; }
}

// vals_in == nullptr: the value of position i is i (first pass)
__global__ void __launch_bounds__(256) k_sort_scatter(const int32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in, int64_t n,
                                                      int shift, uint32_t n_blocks, const uint32_t* __restrict__ first_slot,
                                                      const uint32_t* __restrict__ tile_offset, int32_t* __restrict__ keys_out,
                                                      int32_t* __restrict__ vals_out) {
    __shared__ uint32_t running[256];       // next output slot of every digit for this workgroup
    __shared__ uint32_t wave_cnt[4][256];   // pairs of the chunk with each digit, per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    {
        const size_t x = (size_t)threadIdx.x * n_blocks + blockIdx.x;   // the counters in (digit, workgroup) order
        running[threadIdx.x] = first_slot[x] + tile_offset[x / kScanTile];
    }
    const int64_t i0 = (int64_t)blockIdx.x * kSortSpan;
    for (int u = 0; u < kSortSpan / 256; ++u) {
#pragma unroll
        for (int w = 0; w < 4; ++w) wave_cnt[w][threadIdx.x] = 0u;
        __syncthreads();
        const int64_t i = i0 + u * 256 + threadIdx.x;
        const bool has = i < n;
        const int32_t key = has ? keys_in[i] : 0;
        const int32_t val = has ? (vals_in ? vals_in[i] : (int32_t)i) : 0;
        const uint32_t dgt = ((uint32_t)key >> shift) & 255u;
        unsigned long long same = __ballot(has);   // lanes of this wavefront that hold a pair with this lane's digit
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const bool set = (dgt >> bit) & 1u;
            const unsigned long long m = __ballot(set);
            same &= set ? m : ~m;
        }
        const uint32_t below = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
        if (has && below == 0u) wave_cnt[wave][dgt] = (uint32_t)__popcll(same);
        __syncthreads();
        if (has) {
            uint32_t pos = running[dgt] + below;
            for (int w = 0; w < wave; ++w) pos += wave_cnt[w][dgt];
            keys_out[pos] = key;
            vals_out[pos] = val;
        }
        __syncthreads();
        running[threadIdx.x] += wave_cnt[0][threadIdx.x] + wave_cnt[1][threadIdx.x] + wave_cnt[2][threadIdx.x] + wave_cnt[3][threadIdx.x];
    }
}

// how many points changed their cluster
__global__ void __launch_bounds__(256) k_kmeans_changed(const int32_t* __restrict__ a, const int32_t* __restrict__ b, int64_t n,
                                                        unsigned long long* __restrict__ changed) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool diff = i < n && a[i] != b[i];
    const unsigned long long m = __ballot(diff);
    if ((threadIdx.x & 63) == 0 && m) atomicAdd(changed, (unsigned long long)__popcll(m));
}

// M step: centroid j = float32(sum of its rows / count), the rows added in ascending point order in float64 (ids: the
// points sorted by cluster, ascending inside a cluster; one thread per (cluster, column)); an empty cluster keeps its row.
__global__ void __launch_bounds__(256) k_kmeans_update(const float* __restrict__ X, int32_t d, const int32_t* __restrict__ ids,
                                                       const uint32_t* __restrict__ start, int32_t K, float* __restrict__ C) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= (int64_t)K * d) return;
    const int32_t j = (int32_t)(x / d), col = (int32_t)(x % d);
    const uint32_t r0 = start[j], r1 = start[j + 1];
    if (r1 == r0) return;
    double sum = 0.0;
    uint32_t r = r0;
    if (r + 64 <= r1) {   // batches of 64 rows in flight, the additions in order; the next batch's ids travel with this batch's rows
        int32_t idn[64];
#pragma unroll
        for (int u = 0; u < 64; ++u) idn[u] = ids[r + u];
        for (; r + 64 <= r1; r += 64) {
            float v[64];
#pragma unroll
            for (int u = 0; u < 64; ++u) v[u] = X[(int64_t)idn[u] * d + col];
            if (r + 128 <= r1) {
#pragma unroll
                for (int u = 0; u < 64; ++u) idn[u] = ids[r + 64 + u];
            }
#pragma unroll
            for (int u = 0; u < 64; ++u) sum = __dadd_rn(sum, (double)v[u]);
        }
    }
    for (; r + 8 <= r1; r += 8) {
        int32_t id[8];
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) id[u] = ids[r + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = X[(int64_t)id[u] * d + col];
#pragma unroll
        for (int u = 0; u < 8; ++u) sum = __dadd_rn(sum, (double)v[u]);
    }
    for (; r < r1; ++r) sum = __dadd_rn(sum, (double)X[(int64_t)ids[r] * d + col]);
    C[x] = (float)(sum / (double)(r1 - r0));
}

// The start from a locality-sensitive hash: bit j of a point = [ sum_t h_{j,t} (x_t - a_{j,t}) > 0 ], a_j the anchor row of
// plane j, the sum over t = 0..d-1 in order with difference, product and running sum each rounded once in float64;
// bucket = floor(code K / 2^b).  One thread per point, one accumulator per plane, the row read once.
constexpr int kMaxPlanes = 30;
__global__ void __launch_bounds__(256) k_lsh_buckets(const float* __restrict__ X, int64_t n, int32_t d, const float* __restrict__ planes,
                                                     const int32_t* __restrict__ anchors, int32_t b, int32_t K, int32_t* __restrict__ bucket) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    double acc[kMaxPlanes];
#pragma unroll
    for (int j = 0; j < kMaxPlanes; ++j) acc[j] = 0.0;
    const float* x = X + i * d;
    for (int t = 0; t < d; ++t) {
        const double xt = (double)x[t];
#pragma unroll
        for (int j = 0; j < kMaxPlanes; ++j)
            if (j < b) {
                const double diff = __dsub_rn(xt, (double)X[(int64_t)anchors[j] * d + t]);
                acc[j] = __dadd_rn(acc[j], __dmul_rn((double)planes[(int64_t)j * d + t], diff));
            }
    }
    uint64_t code = 0;
#pragma unroll
    for (int j = 0; j < kMaxPlanes; ++j)
        if (j < b && acc[j] > 0.0) code |= (uint64_t)1 << j;
    bucket[i] = (int32_t)((code * (uint64_t)K) >> b);
}

// Anchors the caller did not draw: plane j goes through the median of a strided sample along its normal.  The sample is the
// m = min(kLshSample, n) points floor(s n / m); projection = sum_t h_{j,t} x_t over t = 0..d-1 in order (product and
// running sum each rounded once in float64); the anchor is the sample point of rank floor(m / 2) in ascending
// (projection, point).  One workgroup per plane: four sample points per thread, ranks by counting.
constexpr int kLshSample = 1024;
__global__ void __launch_bounds__(256) k_lsh_median_anchors(const float* __restrict__ X, int64_t n, int32_t d, const float* __restrict__ planes,
                                                            int32_t* __restrict__ anchors) {
    __shared__ double sproj[kLshSample];
    const int j = blockIdx.x;
    const int m = (int)min((int64_t)kLshSample, n);
    const float* h = planes + (int64_t)j * d;
    for (int s = threadIdx.x; s < m; s += 256) {
        const float* x = X + (((int64_t)s * n) / m) * d;
        double acc = 0.0;
        for (int t = 0; t < d; ++t) acc = __dadd_rn(acc, __dmul_rn((double)h[t], (double)x[t]));
        sproj[s] = acc;
    }
    __syncthreads();
    for (int s = threadIdx.x; s < m; s += 256) {   // sample points are in ascending index order: ties go to the lower s
        const double p = sproj[s];
        int rank = 0;
        for (int o = 0; o < m; ++o) rank += (sproj[o] < p || (sproj[o] == p && o < s)) ? 1 : 0;
        if (rank == m / 2) anchors[j] = (int32_t)(((int64_t)s * n) / m);
    }
}

// centroid j starts as the data point floor(j n / K): what an empty bucket keeps
__global__ void __launch_bounds__(256) k_lsh_fallback(const float* __restrict__ X, int64_t n, int32_t d, int32_t K, float* __restrict__ C) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= (int64_t)K * d) return;
    const int64_t j = x / d;
    C[x] = X[((j * n) / K) * d + x % d];
}

// sum over the points of the exact distance to their centroid (added in no particular order)
__global__ void __launch_bounds__(256) k_kmeans_inertia(const float* __restrict__ X, const float* __restrict__ C, int32_t d,
                                                        const int32_t* __restrict__ labels, int64_t n, double* __restrict__ out) {
    __shared__ double part[256];
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    part[threadIdx.x] = i < n ? exact_distance(X + i * d, C + (int64_t)labels[i] * d, d) : 0.0;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) atomicAdd(out, part[0]);
}

}  // namespace nomad_knn

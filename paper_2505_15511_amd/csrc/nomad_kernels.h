// Device kernels of libnomad for gfx950 (64-wide wavefronts).
//
// Notation follows the paper (arxiv 2505.15511): theta = embedding rows, q = Cauchy kernel
// (Eq. 1), ij = directed kNN edge with head i and tail j, m = sampled negative, mu_r / p_r = mean
// and mass of cell r, |M| = noise-sample count, s = negatives drawn per edge.
//
// Two mappings of edges to lanes:
//   k_edges_binned / k_edges_pooled (the deterministic epoch): one directed edge per lane, consecutive
//     lanes on consecutive CSR positions; forces to tails and negatives leave as records binned by
//     destination tile; head sums are segmented scans in lane order.
//   k_edges (atomic mode, the loss, and the fallback without binning): a *row group* of LPR adjacent
//     lanes walks the CSR row of one head i, LPR edges at a time; head sums are reduced inside the
//     row group with a fixed xor butterfly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "edge_plan.h"
#include "philox.h"

namespace nomad {

constexpr int kBlock = 256;
// 64-bit fixed point used for order-independent accumulation of the negatives' gradient in
// deterministic mode: one unit = 2^-36.  Every single contribution is bounded by p(j|i) <= 1 in
// magnitude, so 2^27 contributions per point still fit.
constexpr double kFixInv = 1.0 / 68719476736.0;       // 2^-36

// v * 2^36 rounded to the nearest integer (ties to even) as a 64-bit two's complement number, for |v| < 2^15.
// Adding 1.5 * 2^52 in double precision leaves that integer in the low mantissa bits: three instructions
// where the float -> int64 conversion takes a dozen.
__device__ __forceinline__ unsigned long long to_fixed(float v) {
    const double d = fma((double)v, 68719476736.0, 6755399441055744.0);
    return (unsigned long long)(__double_as_longlong(d) - 0x4338000000000000LL);
}

// ------------------------------------------------------------------ sampler
// Counter = (edge lo, edge hi, epoch, slot block), key = the 64-bit seed (philox.h).

// Population a head samples its negatives from: the points of its own group.
struct Population {
    uint32_t base;           // first position in `members` (or first point index when contiguous)
    uint32_t count;          // n_loc(i)
    const int32_t* members;  // ascending point list, or nullptr when the group is an index range
};

__device__ __forceinline__ int32_t draw_index(uint32_t x, const Population& pop) {
    const uint32_t u = __umulhi(x, pop.count);
    return pop.members ? pop.members[pop.base + u] : (int32_t)(pop.base + u);
}

template <int LPR>
__device__ __forceinline__ float rowgroup_sum(float v) {
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float cauchy(float dx, float dy) {
    return __builtin_amdgcn_rcpf(fmaf(dx, dx, fmaf(dy, dy, 1.0f)));
}

// ------------------------------------------------------------------ validation and set-up
enum Flag {
    kFlagRowPtr = 0,     // row_ptr not monotone / does not start at 0
    kFlagCol = 1,        // column out of range
    kFlagSelfLoop = 2,
    kFlagWeight = 3,     // negative / non-finite weight or non-positive row sum
    kFlagCluster = 4,    // cluster id out of range
    kFlagGroup = 5,      // group label out of range
    kFlagCount = 8
};

__global__ void k_check_row_ptr(const int32_t* __restrict__ row_ptr, int64_t n, int* flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && row_ptr[0] != 0) flags[kFlagRowPtr] = 1;
    if (i < n && row_ptr[i + 1] < row_ptr[i]) flags[kFlagRowPtr] = 1;
}

// one thread per row: columns in range, no self loops; normalised weights p(j|i), from the caller's weights w or,
// with by_rank, from the position of the edge in its row: the inverse-rank model of Eq. 7 read with ranks 1..k_i and
// the row's own k_i-term normaliser, exp(1/rho) / sum_{rho'} exp(1/rho')
__global__ void k_check_rows(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                             const float* __restrict__ w, float* __restrict__ pe, int64_t n, int by_rank, int* flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t a = row_ptr[i], b = row_ptr[i + 1];
    if (by_rank) {
        double z = 0.0;
        for (int32_t e = a; e < b; ++e) {
            const int32_t j = col[e];
            if (j < 0 || j >= n) flags[kFlagCol] = 1;
            else if (j == i) flags[kFlagSelfLoop] = 1;
            z += exp(1.0 / (double)(e - a + 1));
        }
        for (int32_t e = a; e < b; ++e) pe[e] = (float)(exp(1.0 / (double)(e - a + 1)) / z);
        return;
    }
    double sum = 0.0;
    for (int32_t e = a; e < b; ++e) {
        const int32_t j = col[e];
        if (j < 0 || j >= n) flags[kFlagCol] = 1;
        else if (j == i) flags[kFlagSelfLoop] = 1;
        if (w) {
            const float x = w[e];
            if (!(x >= 0.0f) || !(x <= 3.0e38f)) flags[kFlagWeight] = 1;
            sum += (double)x;
        }
    }
    if (w && b > a) {
        if (!(sum > 0.0)) { flags[kFlagWeight] = 1; return; }
        for (int32_t e = a; e < b; ++e) pe[e] = (float)((double)w[e] / sum);
    }
}

// cluster sizes, first index of each cluster, number of index positions where the cluster /
// the group changes (tells whether clusters and groups are contiguous index ranges)
__global__ void k_cluster_census(const int32_t* __restrict__ cluster_of, const int32_t* __restrict__ group_of_cluster,
                                 int64_t n, int32_t R, uint32_t* counts, uint32_t* first, uint32_t* gfirst,
                                 unsigned long long* boundaries, int* flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t c = cluster_of[i];
    if (c < 0 || c >= R) { flags[kFlagCluster] = 1; return; }
    // Points are usually numbered cluster by cluster: when the lanes of a wavefront that are still here all hold the same
    // cluster, its first lane reports for all of them (one atomic instead of 64 on one address).
    const unsigned long long here = __ballot(1);
    const int leader = __ffsll((long long)here) - 1;
    const int32_t c0 = __shfl(c, leader, 64);
    if (__ballot(c != c0) == 0ull) {
        if ((int)(threadIdx.x & 63) == leader) {
            atomicAdd(&counts[c], (uint32_t)__popcll(here));
            atomicMin(&first[c], (uint32_t)i);   // the lowest lane holds the lowest index
            if (group_of_cluster) atomicMin(&gfirst[group_of_cluster[c]], (uint32_t)i);
        }
    } else {
        atomicAdd(&counts[c], 1u);
        atomicMin(&first[c], (uint32_t)i);
        if (group_of_cluster) atomicMin(&gfirst[group_of_cluster[c]], (uint32_t)i);
    }
    if (i > 0) {
        const int32_t p = cluster_of[i - 1];
        if (p >= 0 && p < R) {
            if (p != c) atomicAdd(&boundaries[0], 1ull);
            if (group_of_cluster && group_of_cluster[p] != group_of_cluster[c]) atomicAdd(&boundaries[1], 1ull);
        }
    }
}

// hinfo[i] = (population base, population size, omega, group label) of the group of point i (see EdgeArgs::hinfo)
__global__ void __launch_bounds__(kBlock) k_head_info(const int32_t* __restrict__ cluster_of, const int32_t* __restrict__ group_of_cluster,
                                                      const uint32_t* __restrict__ gbase, const uint32_t* __restrict__ gcount,
                                                      const float* __restrict__ gomega, int64_t n, float4* __restrict__ hinfo) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t g = group_of_cluster[cluster_of[i]];
    hinfo[i] = make_float4(__uint_as_float(gbase[g]), __uint_as_float(gcount[g]), gomega[g], __int_as_float(g));
}

// ------------------------------------------------------------------ K1: cell means
// Two stages, both in a fixed order: (a) one block per chunk of a cell's member list sums its
// points in float64 (lane-strided partials, xor butterfly inside the wavefront, wavefront totals
// added in wavefront order); (b) one wavefront per cell adds the chunk totals the same way.
struct MeanChunk { int32_t cell; uint32_t begin; uint32_t end; };

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ void __launch_bounds__(kBlock) k_mean_chunks(const float2* __restrict__ theta,
                                                        const int32_t* __restrict__ members,
                                                        const MeanChunk* __restrict__ chunks, double2* __restrict__ partial) {
    __shared__ double sx[kBlock / 64], sy[kBlock / 64];
    const MeanChunk ch = chunks[blockIdx.x];
    double ax = 0.0, ay = 0.0;
    for (uint32_t p = ch.begin + threadIdx.x; p < ch.end; p += kBlock) {
        const float2 v = theta[members ? (uint32_t)members[p] : p];
        ax += (double)v.x;
        ay += (double)v.y;
    }
    ax = wave_sum(ax);
    ay = wave_sum(ay);
    if ((threadIdx.x & 63) == 0) { sx[threadIdx.x >> 6] = ax; sy[threadIdx.x >> 6] = ay; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double tx = 0.0, ty = 0.0;
        for (int w = 0; w < kBlock / 64; ++w) { tx += sx[w]; ty += sy[w]; }
        partial[blockIdx.x] = make_double2(tx, ty);
    }
}

// cinfo[slot of r] = (mu_x, mu_y, p_r, group label as bits), the table ordered group by group when
// cells are grouped; one wavefront per cell
__global__ void __launch_bounds__(kBlock) k_mean_finish(const double2* __restrict__ partial,
                                                        const uint32_t* __restrict__ chunk_start,
                                                        const uint32_t* __restrict__ counts,
                                                        const int32_t* __restrict__ group_of_cluster,
                                                        const int32_t* __restrict__ cell_slot, int32_t R, double inv_n,
                                                        float2* __restrict__ mu, float4* __restrict__ cinfo) {
    const int32_t r = (int32_t)((blockIdx.x * (uint32_t)kBlock + threadIdx.x) >> 6);
    if (r >= R) return;
    const int lane = threadIdx.x & 63;
    double ax = 0.0, ay = 0.0;
    for (uint32_t c = chunk_start[r] + lane; c < chunk_start[r + 1]; c += 64) {
        ax += partial[c].x;
        ay += partial[c].y;
    }
    ax = wave_sum(ax);
    ay = wave_sum(ay);
    if (lane == 0) {
        const uint32_t cnt = counts[r];
        const float mx = cnt ? (float)(ax / (double)cnt) : 0.0f;
        const float my = cnt ? (float)(ay / (double)cnt) : 0.0f;
        mu[r] = make_float2(mx, my);
        cinfo[cell_slot ? cell_slot[r] : r] =
            make_float4(mx, my, (float)((double)cnt * inv_n), __int_as_float(group_of_cluster ? group_of_cluster[r] : 0));
    }
}

// ------------------------------------------------------------------ K2: mean-field sums (Eq. 5)
// One lane per head; the cell table is staged through LDS, 1,024 cells at a time, and read with
// wave-uniform addresses, eight cells per batch.  The table is ordered group by group, so the cells a head does NOT approximate
// (its own group) are one slot range [lo, hi).  Points are usually numbered cluster by cluster,
// which makes that range the same for all 64 lanes of most wavefronts: those skip the range and
// need no per-cell test; mixed wavefronts test every cell.  Partial sums are folded into the
// totals every 64 cells to keep float32 round-off from growing with |R|.
struct MeanFieldSum { float a, bx, by; };

constexpr int kMeanFieldBlock = 1024;   // lanes per workgroup = cells staged per step
constexpr int kMeanFieldHeads = 1;      // heads per lane (2 measured 10 % slower: the loop is bound by vector ALU issue, not by LDS)

template <bool TEST>
__device__ __forceinline__ void mean_field_add(float q, float dx, float dy, const float4 c, int32_t gi, MeanFieldSum& s) {
    const float w = (TEST && __float_as_int(c.w) == gi) ? 0.0f : c.z;
    const float wq = w * q;
    s.a += wq;
    const float wq2 = wq * q;
    s.bx = fmaf(wq2, dx, s.bx);
    s.by = fmaf(wq2, dy, s.by);
}

template <bool TEST>
__device__ __forceinline__ void mean_field_cell(const float2 ti, const float4 c, int32_t gi, MeanFieldSum& s) {
    const float dx = ti.x - c.x, dy = ti.y - c.y;
    mean_field_add<TEST>(cauchy(dx, dy), dx, dy, c, gi, s);
}

// Two cells share one reciprocal (the slowest instruction of the loop): with t = 1 + d^2,
// 1/t0 = t1 / (t0 t1) and 1/t1 = t0 / (t0 t1).
template <bool TEST>
__device__ __forceinline__ void mean_field_pair(const float2 ti, const float4 c0, const float4 c1, int32_t gi, MeanFieldSum& s) {
    const float dx0 = ti.x - c0.x, dy0 = ti.y - c0.y, dx1 = ti.x - c1.x, dy1 = ti.y - c1.y;
    const float t0 = fmaf(dx0, dx0, fmaf(dy0, dy0, 1.0f)), t1 = fmaf(dx1, dx1, fmaf(dy1, dy1, 1.0f));
    const float r = __builtin_amdgcn_rcpf(t0 * t1);
    mean_field_add<TEST>(r * t1, dx0, dy0, c0, gi, s);
    mean_field_add<TEST>(r * t0, dx1, dy1, c1, gi, s);
}

// cells [r_begin, r_end) of the staged part of the table (LDS; `cells` points at the slot that holds cell 0),
// for the kMeanFieldHeads heads of this lane
template <bool TEST>
__device__ __forceinline__ void mean_field_range(const float2 (&ti)[kMeanFieldHeads], const float4* cells, int32_t r_begin, int32_t r_end,
                                                 const int32_t (&gi)[kMeanFieldHeads], MeanFieldSum (&total)[kMeanFieldHeads]) {
    for (int32_t r0 = r_begin; r0 < r_end; r0 += 64) {
        MeanFieldSum s[kMeanFieldHeads];
#pragma unroll
        for (int h = 0; h < kMeanFieldHeads; ++h) s[h] = MeanFieldSum{0.f, 0.f, 0.f};
        const int32_t r1 = min(r_end, r0 + 64);
        int32_t r = r0;
        for (; r + 8 <= r1; r += 8) {
#pragma unroll
            for (int u = 0; u < 8; u += 2) {
                const float4 c0 = cells[r + u], c1 = cells[r + u + 1];
#pragma unroll
                for (int h = 0; h < kMeanFieldHeads; ++h) mean_field_pair<TEST>(ti[h], c0, c1, gi[h], s[h]);
            }
        }
        for (; r < r1; ++r) {
            const float4 c = cells[r];
#pragma unroll
            for (int h = 0; h < kMeanFieldHeads; ++h) mean_field_cell<TEST>(ti[h], c, gi[h], s[h]);
        }
#pragma unroll
        for (int h = 0; h < kMeanFieldHeads; ++h) { total[h].a += s[h].a; total[h].bx += s[h].bx; total[h].by += s[h].by; }
    }
}

__global__ void __launch_bounds__(kMeanFieldBlock) k_mean_field(const float2* __restrict__ theta,
                                                                const int32_t* __restrict__ cluster_of,
                                                                const int32_t* __restrict__ group_of_cluster,
                                                                const float4* __restrict__ cinfo, const int2* __restrict__ group_slots,
                                                                int32_t R, int64_t i_begin, int64_t n, float* __restrict__ A,
                                                                float2* __restrict__ B) {
    // Every wavefront needs the whole cell table.  Reading it straight from memory with wave-uniform loads makes
    // each of the n/64 wavefronts pull all |R| x 16 bytes through the scalar cache (240 GB per launch at 60 M points
    // and 16,384 cells); staged through LDS the table is read once per workgroup and broadcast to the lanes.
    __shared__ float4 cells[kMeanFieldBlock];
    // the heads of a lane are adjacent points, so that a wavefront covers 128 consecutive points (one group, usually)
    // heads i_begin .. n-1 (n = one past the last head of this launch)
    const int64_t i0 = i_begin + ((int64_t)blockIdx.x * kMeanFieldBlock + threadIdx.x) * kMeanFieldHeads;
    float2 ti[kMeanFieldHeads];
    int32_t gi[kMeanFieldHeads];
    MeanFieldSum t[kMeanFieldHeads];
#pragma unroll
    for (int h = 0; h < kMeanFieldHeads; ++h) {
        const int64_t ic = min(i0 + h, n - 1);   // heads past the end: a copy of the last one, not stored
        ti[h] = theta[ic];
        gi[h] = group_of_cluster[cluster_of[ic]];
        t[h] = MeanFieldSum{0.f, 0.f, 0.f};
    }
    const int32_t g0 = __builtin_amdgcn_readfirstlane(gi[0]);
    bool same = true;
#pragma unroll
    for (int h = 0; h < kMeanFieldHeads; ++h) same = same && gi[h] == g0;
    const bool uniform = __all(same);
    int2 own = make_int2(0, 0);           // slot range to skip: the own group of a wavefront whose heads share it
    if (uniform) own = group_slots[g0];
    for (int32_t c0 = 0; c0 < R; c0 += kMeanFieldBlock) {
        __syncthreads();
        if (c0 + (int32_t)threadIdx.x < R) cells[threadIdx.x] = cinfo[c0 + threadIdx.x];
        __syncthreads();
        const int32_t c1 = min(R, c0 + kMeanFieldBlock);
        const float4* base = cells - c0;
        if (uniform) {
            mean_field_range<false>(ti, base, c0, min(c1, max(c0, own.x)), gi, t);
            mean_field_range<false>(ti, base, max(c0, min(c1, own.y)), c1, gi, t);
        } else {
            mean_field_range<true>(ti, base, c0, c1, gi, t);
        }
    }
#pragma unroll
    for (int h = 0; h < kMeanFieldHeads; ++h) {
        const int64_t i = i0 + h;
        if (i < n) {
            A[i] = t[h].a;
            B[i] = make_float2(t[h].bx, t[h].by);
        }
    }
}

// ------------------------------------------------------------------ K3: the edge pass
struct EdgeArgs {
    const int32_t* row_ptr;
    const int32_t* col;
    const float* pe;               // normalised weights, or nullptr for 1/deg
    const float2* theta;
    const int32_t* cluster_of;     // used only when grouped
    const int32_t* group_of_cluster;  // nullptr = single group
    const uint32_t* gbase;         // per group: population base
    const uint32_t* gcount;        // per group: population size
    const float* gomega;           // per group: weight of one sampled negative
    const int32_t* gmembers;       // nullptr when every group is an index range
    const float4* hinfo;           // grouped: per point (population base, population size, omega, group) of its group,
                                   // so that the edge pass needs one lookup per head instead of a chain of four
    const float2* mu;              // cell means (sampled far field only)
    int32_t far;                   // sampled far field: negatives from all points, other groups' through their cell mean
    const float* A;                // mean-field sums (grouped only)
    const float2* B;
    float noise_count;             // |M|
    float omega0;                  // single-group omega
    uint32_t key0, key1, epoch;
    uint32_t pool_size, pool_block;   // pooled sampler (0, 0 = i.i.d. negatives per edge)
    uint32_t pool_mode;               // 0: 16-bit picks, consecutive blocks; 1: distinct picks, interleaved blocks
    uint32_t pool_line_bits;          // distinct picks: log2 of the points per pool line
    uint32_t pool_segment_bits;       // distinct picks: log2 of the positions dealt to a block together
    uint32_t pool_blocks;             // distinct picks: number of blocks NB
    const uint32_t* pool_keys;        // stratified pools: this epoch's (A0, A1, A2, C0, C1, C2, r, 0), written by k_pool_keys
    int32_t s;
    int64_t n;
    int64_t row_begin, row_end;    // heads this launch covers (a sub-step of a minibatch epoch; else 0, n)
    // outputs
    float2* g;                     // atomic mode: accumulators of every force
    float2* ghead;                 // deterministic mode: head-side sums
    unsigned long long* gfix;      // deterministic fallback: fixed-point sums of tail and negative forces [n*2]
    double* loss_partial;          // loss mode: one partial per block
    float* cS;                     // gradient through the means: 2 p_e / S_e of every edge, or nullptr
};

enum EdgeMode { kModeAtomic = 0, kModeDet = 1, kModeLoss = 2 };

// Per-head constants of the edge pass.
struct HeadCtx {
    float2 ti;
    float inv_deg;
    float omega;          // weight of one sampled negative (Eq. 6 estimate)
    float MA, MBx, MBy;   // |M| A_i and |M| B_i (Eq. 5 and its derivative factor)
    int32_t group;        // group label of the head (0 without groups)
    Population pop;
};

__device__ __forceinline__ HeadCtx load_head(const EdgeArgs& P, int64_t i, int32_t ea, int32_t eb) {
    HeadCtx h;
    h.ti = P.theta[i];
    h.inv_deg = eb > ea ? 1.0f / (float)(eb - ea) : 0.f;
    h.MA = h.MBx = h.MBy = 0.f;
    h.group = 0;
    if (P.group_of_cluster && P.far) {   // every head samples all points; Eq. 5's sum is left to the samples
        h.group = __float_as_int(P.hinfo[i].w);
        h.pop.base = 0;
        h.pop.count = (uint32_t)P.n;
        h.pop.members = nullptr;
        h.omega = P.omega0;
    } else if (P.group_of_cluster) {
        const float4 hi = P.hinfo[i];
        h.group = __float_as_int(hi.w);
        h.pop.base = __float_as_uint(hi.x);
        h.pop.count = __float_as_uint(hi.y);
        h.pop.members = P.gmembers;
        h.omega = hi.z;
        h.MA = P.noise_count * P.A[i];
        const float2 b = P.B[i];
        h.MBx = P.noise_count * b.x;
        h.MBy = P.noise_count * b.y;
    } else {
        h.pop.base = 0;
        h.pop.count = (uint32_t)P.n;
        h.pop.members = nullptr;
        h.omega = P.omega0;
    }
    return h;
}

// Everything one directed edge e = (i -> j) contributes, for a compile-time number S of negatives:
//   a        attraction coefficient 2 p q_ij (1 - q_ij / S_e)         (gradient of Eq. 4's numerator and q_ij in S_e)
//   m[k], (rx,ry)[k]  the sampled negatives and the force each receives, b_k (theta_i - theta_m)
//   (hx,hy)  total force on the head: a d_ij - sum_k r_k - 2 p |M| B_i / S_e
template <int S>
struct EdgeOut {
    float a, dx, dy, hx, hy, log_term;
    float c;              // 2 p_e / S_e: what the edge multiplies d S_e / d(anything) with
    int32_t j;
    int32_t m[S];
    float rx[S], ry[S];
};

// The arithmetic of one edge, given the embedding rows it touches (tj the tail, tm[k] the negatives).
template <int S, bool LOSS>
__device__ __forceinline__ void edge_math(const HeadCtx& h, float pe, float2 tj, const float2 (&tm)[S > 0 ? S : 1],
                                          EdgeOut<(S > 0 ? S : 1)>& o) {
    o.dx = h.ti.x - tj.x;
    o.dy = h.ti.y - tj.y;
    const float qij = cauchy(o.dx, o.dy);
    float qm[S > 0 ? S : 1];
    float qsum = 0.f;
#pragma unroll
    for (int k = 0; k < S; ++k) {
        o.rx[k] = h.ti.x - tm[k].x;
        o.ry[k] = h.ti.y - tm[k].y;
        qm[k] = cauchy(o.rx[k], o.ry[k]);
        qsum += qm[k];
    }
    const float rest = h.MA + h.omega * qsum;   // S_e - q_ij: the noise part of the denominator
    const float Se = qij + rest;
    if (LOSS) {
        o.log_term = pe * logf(Se / qij);   // -log q + log S = log(S (1 + d^2))
        return;
    }
    const float inv_S = __builtin_amdgcn_rcpf(Se);   // 1 ulp; S_e >= q_ij > 0
    o.a = 2.0f * pe * qij * rest * inv_S;       // 1 - q_ij / S_e = (S_e - q_ij) / S_e without the cancellation
    float fx = o.a * o.dx, fy = o.a * o.dy;
    const float bscale = 2.0f * pe * h.omega * inv_S;
#pragma unroll
    for (int k = 0; k < S; ++k) {
        const float b = bscale * qm[k] * qm[k];
        o.rx[k] *= b;
        o.ry[k] *= b;
        fx -= o.rx[k];
        fy -= o.ry[k];
    }
    o.c = 2.0f * pe * inv_S;
    o.hx = fx - o.c * h.MBx;
    o.hy = fy - o.c * h.MBy;
}

// Pooled sampler: pool entry of slot k given the four words of the per-edge Philox call k >> 3
// (16-bit half k & 1 of word (k >> 1) & 3, scaled to the pool size), and the point behind a pool entry
// (word u & 3 of Philox(counter (block, 0xFFFFFFFF, epoch, u >> 2)) mapped onto the population).
__device__ __forceinline__ uint32_t pool_slot(const uint32_t (&w)[4], int k, uint32_t pool_size) {
    const uint32_t x16 = (w[(k >> 1) & 3] >> (16 * (k & 1))) & 0xFFFFu;
    return (x16 * pool_size) >> 16;
}

__device__ __forceinline__ int32_t pool_point(const EdgeArgs& P, const Population& pop, uint32_t block, uint32_t u) {
    uint32_t w[4];
    philox4x32_10(block, 0xFFFFFFFFu, P.epoch, u >> 2, P.key0, P.key1, w);
    return draw_index(w[u & 3u], pop);
}

// ---- pooled sampler with distinct picks (see nomad.h).  One population: all n points.
constexpr uint32_t kPoolEntryStream = 0xFFFFFFFFu, kPoolPickStream = 0xFFFFFFFEu;

// entry of slot k given the edge's word W: (u_0 + k c) mod pool_size, u_0 = top log2(pool_size) bits of W,
// c = 2 (bits 1 .. log2(pool_size) - 1 of W) + 1
__device__ __forceinline__ uint32_t distinct_pick(uint32_t W, int k, uint32_t pool_size) {
    const uint32_t u0 = W >> (__clz(pool_size) + 1);     // 32 - log2(pool_size)
    const uint32_t c = (W & (pool_size - 2u)) | 1u;      // = 2 ((W >> 1) & (pool_size / 2 - 1)) + 1
    return (u0 + (uint32_t)k * c) & (pool_size - 1u);
}

// ---- stratified pools (pool_mode 2, see nomad.h): the lines of an epoch's pools are dealt from a keyed permutation
constexpr uint32_t kPoolKeyStream = 0xFFFFFFFDu;

// this epoch's keys: multipliers (odd), increments, cyclic shift of the lines
__global__ void k_pool_keys(uint32_t key0, uint32_t key1, uint32_t epoch, uint32_t n, uint32_t* __restrict__ keys) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    uint32_t a[4], b[4];
    philox4x32_10(0u, kPoolKeyStream, epoch, 0u, key0, key1, a);
    philox4x32_10(1u, kPoolKeyStream, epoch, 0u, key0, key1, b);
    keys[0] = a[0] | 1u; keys[1] = a[2] | 1u; keys[2] = b[0] | 1u;
    keys[3] = a[1]; keys[4] = a[3]; keys[5] = b[1];
    keys[6] = __umulhi(b[2], n);
    keys[7] = 0u;
}

// the keyed bijection of 0 .. n_lines-1: three rounds of x <- (A_k x + C_k) mod 2^b, x <- x xor (x >> max(1, b / 2)) on
// b = max(1, ceil(log2 n_lines)) bits, repeated until the value lies below n_lines
__device__ __forceinline__ uint32_t line_permutation(uint32_t x, uint32_t n_lines, const uint32_t* __restrict__ keys) {
    const uint32_t b = n_lines > 2u ? 32u - (uint32_t)__clz(n_lines - 1u) : 1u;
    const uint32_t mask = b >= 32u ? 0xFFFFFFFFu : (1u << b) - 1u, sh = b / 2u > 1u ? b / 2u : 1u;
    const uint32_t A0 = keys[0], A1 = keys[1], A2 = keys[2], C0 = keys[3], C1 = keys[4], C2 = keys[5];
    do {
        x = (A0 * x + C0) & mask; x ^= x >> sh;
        x = (A1 * x + C1) & mask; x ^= x >> sh;
        x = (A2 * x + C2) & mask; x ^= x >> sh;
    } while (x >= n_lines);
    return x;
}

// first point of the line with running number `index` (= beta L + gamma) of this epoch
__device__ __forceinline__ uint32_t stratified_line_start(const EdgeArgs& P, uint64_t index) {
    const uint32_t n = (uint32_t)P.n, n_lines = (n + (1u << P.pool_line_bits) - 1u) >> P.pool_line_bits;
    const uint32_t x = line_permutation((uint32_t)(index % n_lines), n_lines, P.pool_keys);
    return (uint32_t)((((uint64_t)x << P.pool_line_bits) + P.pool_keys[6]) % n);
}

// point behind entry u of block beta's pool: point number (u div L) of line (u mod L)
__device__ __forceinline__ int32_t distinct_pool_point(const EdgeArgs& P, uint32_t beta, uint32_t u) {
    const uint32_t lg = 31u - (uint32_t)__clz(P.pool_size), lg_lines = lg - P.pool_line_bits;
    const uint32_t gamma = u & ((1u << lg_lines) - 1u), o = u >> lg_lines;
    uint32_t pt;
    if (P.pool_mode == 2) {
        pt = stratified_line_start(P, ((uint64_t)beta << lg_lines) + gamma) + o;
    } else {
        uint32_t w[4];
        philox4x32_10(beta, kPoolEntryStream, P.epoch, gamma >> 2, P.key0, P.key1, w);
        pt = __umulhi(w[gamma & 3u], (uint32_t)P.n) + o;
    }
    if (pt >= (uint32_t)P.n) pt -= (uint32_t)P.n;
    return (int32_t)pt;
}

// block and rank of CSR position e
__device__ __forceinline__ void distinct_block_of(const EdgeArgs& P, uint32_t e, uint32_t& beta, uint32_t& rank) {
    const uint32_t sigma = e >> P.pool_segment_bits;
    beta = sigma % P.pool_blocks;
    rank = ((sigma / P.pool_blocks) << P.pool_segment_bits) + (e & ((1u << P.pool_segment_bits) - 1u));
}

__device__ __forceinline__ uint32_t distinct_edge_word(const EdgeArgs& P, uint32_t beta, uint32_t rank) {
    uint32_t w[4];
    philox4x32_10(beta, kPoolPickStream, P.epoch, (rank & 1023u) + 1024u * (rank >> 12), P.key0, P.key1, w);
    return w[(rank >> 10) & 3u];
}

// Negative of slot k of CSR position e in epoch P.epoch (general form, any s).
__device__ __forceinline__ int32_t negative_of_slot(const EdgeArgs& P, const Population& pop, int32_t e, int k) {
    uint32_t w[4];
    if (P.pool_mode != 0) {
        uint32_t beta, rank;
        distinct_block_of(P, (uint32_t)e, beta, rank);
        return distinct_pool_point(P, beta, distinct_pick(distinct_edge_word(P, beta, rank), k, P.pool_size));
    }
    if (P.pool_size == 0) {
        philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)(k >> 2), P.key0, P.key1, w);
        return draw_index(w[k & 3], pop);
    }
    philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)(k >> 3), P.key0, P.key1, w);
    return pool_point(P, pop, (uint32_t)e / P.pool_block, pool_slot(w, k, P.pool_size));
}

// The s negatives of CSR position e in epoch P.epoch.
template <int S>
__device__ __forceinline__ void draw_negatives(const EdgeArgs& P, const Population& pop, int32_t e, int32_t (&m)[S > 0 ? S : 1]) {
    if (P.pool_size == 0) {
#pragma unroll
        for (int b = 0; b < (S + 3) / 4; ++b) {
            uint32_t w[4];
            philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)b, P.key0, P.key1, w);
#pragma unroll
            for (int l = 0; l < 4; ++l)
                if (4 * b + l < S) m[4 * b + l] = draw_index(w[l], pop);
        }
    } else if (P.pool_mode != 0) {
        uint32_t beta, rank;
        distinct_block_of(P, (uint32_t)e, beta, rank);
        const uint32_t W = distinct_edge_word(P, beta, rank);
#pragma unroll
        for (int k = 0; k < S; ++k) m[k] = distinct_pool_point(P, beta, distinct_pick(W, k, P.pool_size));
    } else {
        uint32_t w[4];
        philox4x32_10((uint32_t)e, 0u, P.epoch, 0u, P.key0, P.key1, w);   // S <= 8 here: one call
#pragma unroll
        for (int k = 0; k < S; ++k) m[k] = pool_point(P, pop, (uint32_t)e / P.pool_block, pool_slot(w, k, P.pool_size));
    }
}

// Where negative m sits for a head of group `group`.  Sampled far field: a point of another group stands for its
// cell and enters through the cell mean (Eq. 5 estimated from the samples); it then receives no force (m = -1).
__device__ __forceinline__ float2 negative_row(const EdgeArgs& P, int32_t group, int32_t& m) {
    if (P.far) {
        const int32_t r = P.cluster_of[m];
        if (P.group_of_cluster[r] != group) { m = -1; return P.mu[r]; }
    }
    return P.theta[m];
}

template <int S, bool LOSS>
__device__ __forceinline__ void edge_terms(const EdgeArgs& P, const HeadCtx& h, int32_t e, EdgeOut<(S > 0 ? S : 1)>& o) {
    const int32_t j = P.col[e];
    o.j = j;
    const float2 tj = P.theta[j];
    const float pe = P.pe ? P.pe[e] : h.inv_deg;
    draw_negatives<S>(P, h.pop, e, o.m);
    float2 tm[S > 0 ? S : 1];
#pragma unroll
    for (int k = 0; k < S; ++k) tm[k] = negative_row(P, h.group, o.m[k]);
    edge_math<S, LOSS>(h, pe, tj, tm, o);
}

// Blocks are handed to the 8 XCDs round-robin; giving XCD x the x-th contiguous eighth of the
// rows keeps each L2 on its own slice of theta and of the index stream.
__device__ __forceinline__ uint32_t xcd_contiguous_block(uint32_t b, uint32_t nblocks) {
    const uint32_t per = (nblocks + 7u) >> 3;
    return (b & 7u) * per + (b >> 3);
}

// Dynamic-s variant of the per-edge arithmetic (s = 0 or s > 8): the negatives are drawn twice,
// once for S_e and once for the forces, so nothing has to be kept per slot.  `emit(m, rx, ry)`
// receives the force on each negative.
template <bool LOSS, typename Emit>
__device__ __forceinline__ void edge_terms_dynamic(const EdgeArgs& P, const HeadCtx& h, int32_t e, int32_t s, float& a,
                                                   float& dx, float& dy, float& hx, float& hy, float& log_term, Emit emit) {
    const int32_t j = P.col[e];
    const float2 tj = P.theta[j];
    const float pe = P.pe ? P.pe[e] : h.inv_deg;
    dx = h.ti.x - tj.x;
    dy = h.ti.y - tj.y;
    const float qij = cauchy(dx, dy);
    float qsum = 0.f;
    for (int k = 0; k < s; ++k) {
        int32_t mk = negative_of_slot(P, h.pop, e, k);
        const float2 tm = negative_row(P, h.group, mk);
        qsum += cauchy(h.ti.x - tm.x, h.ti.y - tm.y);
    }
    const float rest = h.MA + h.omega * qsum;   // S_e - q_ij
    const float Se = qij + rest;
    if (LOSS) { log_term = pe * logf(Se / qij); return; }
    const float inv_S = __builtin_amdgcn_rcpf(Se);   // 1 ulp; S_e >= q_ij > 0
    a = 2.0f * pe * qij * rest * inv_S;
    float fx = a * dx, fy = a * dy;
    const float bscale = 2.0f * pe * h.omega * inv_S;
    for (int k = 0; k < s; ++k) {
        int32_t mk = negative_of_slot(P, h.pop, e, k);
        const float2 tm = negative_row(P, h.group, mk);
        const float gx = h.ti.x - tm.x, gy = h.ti.y - tm.y;
        const float q = cauchy(gx, gy);
        const float bb = bscale * q * q;
        fx -= bb * gx;
        fy -= bb * gy;
        if (mk >= 0) emit(mk, bb * gx, bb * gy);
    }
    const float c = 2.0f * pe * inv_S;
    hx = fx - c * h.MBx;
    hy = fy - c * h.MBy;
    if (P.cS) P.cS[e] = c;
}

__device__ __forceinline__ void add_fixed(unsigned long long* gfix, int64_t m, float rx, float ry) {
    atomicAdd(&gfix[2 * m], to_fixed(rx));
    atomicAdd(&gfix[2 * m + 1], to_fixed(ry));
}

// The edge pass with forces scattered straight from the kernel: global fp32 atomics (kModeAtomic),
// or global 64-bit fixed-point atomics (kModeDet: order-independent, the fallback of the binned
// path below); kModeLoss only sums the loss terms.  S > 0: compile-time number of negatives; S = 0: run-time s.
template <int S, int MODE, int LPR>
__global__ void __launch_bounds__(kBlock) k_edges(const EdgeArgs P) {
    constexpr int ROWS = kBlock / LPR;
    constexpr int SS = S > 0 ? S : 1;
    const uint32_t lb = xcd_contiguous_block(blockIdx.x, gridDim.x);
    const int64_t i = P.row_begin + (int64_t)lb * ROWS + (threadIdx.x / LPR);
    const int lane = threadIdx.x % LPR;
    float hx = 0.f, hy = 0.f;
    double lsum = 0.0;
    if (i < P.row_end) {
        const int32_t ea = P.row_ptr[i], eb = P.row_ptr[i + 1];
        const HeadCtx h = load_head(P, i, ea, eb);
        for (int32_t e = ea + lane; e < eb; e += LPR) {
            float a = 0.f, dx = 0.f, dy = 0.f, ehx = 0.f, ehy = 0.f, lt = 0.f;
            if (S > 0) {
                EdgeOut<SS> o;
                edge_terms<SS, MODE == kModeLoss>(P, h, e, o);
                if (MODE == kModeLoss) { lsum += (double)o.log_term; continue; }
                a = o.a; dx = o.dx; dy = o.dy; ehx = o.hx; ehy = o.hy;
                if (P.cS) P.cS[e] = o.c;
#pragma unroll
                for (int k = 0; k < SS; ++k) {
                    if (o.m[k] < 0) continue;   // stood for a cell mean: no force
                    if (MODE == kModeAtomic) {
                        unsafeAtomicAdd(&P.g[o.m[k]].x, o.rx[k]);
                        unsafeAtomicAdd(&P.g[o.m[k]].y, o.ry[k]);
                    } else {
                        add_fixed(P.gfix, o.m[k], o.rx[k], o.ry[k]);
                    }
                }
            } else {
                edge_terms_dynamic<MODE == kModeLoss>(P, h, e, P.s, a, dx, dy, ehx, ehy, lt, [&](int32_t mk, float rx, float ry) {
                    if (MODE == kModeAtomic) {
                        unsafeAtomicAdd(&P.g[mk].x, rx);
                        unsafeAtomicAdd(&P.g[mk].y, ry);
                    } else {
                        add_fixed(P.gfix, mk, rx, ry);
                    }
                });
                if (MODE == kModeLoss) { lsum += (double)lt; continue; }
            }
            const int32_t j = P.col[e];   // the tail takes the opposite of the attraction
            if (MODE == kModeAtomic) {
                unsafeAtomicAdd(&P.g[j].x, -a * dx);
                unsafeAtomicAdd(&P.g[j].y, -a * dy);
            } else {
                add_fixed(P.gfix, j, -a * dx, -a * dy);
            }
            hx += ehx;
            hy += ehy;
        }
    }
    if (MODE == kModeLoss) {
        __shared__ double sl[kBlock / 64];
        lsum = wave_sum(lsum);
        if ((threadIdx.x & 63) == 0) sl[threadIdx.x >> 6] = lsum;
        __syncthreads();
        if (threadIdx.x == 0) {
            double tsum = 0.0;
            for (int w = 0; w < kBlock / 64; ++w) tsum += sl[w];
            P.loss_partial[lb] = tsum;
        }
        return;
    }
    hx = rowgroup_sum<LPR>(hx);
    hy = rowgroup_sum<LPR>(hy);
    if (lane == 0 && i < P.row_end) {
        if (MODE == kModeAtomic) {
            unsafeAtomicAdd(&P.g[i].x, hx);
            unsafeAtomicAdd(&P.g[i].y, hy);
        } else {
            P.ghead[i] = make_float2(hx, hy);
        }
    }
}

// ------------------------------------------------------------------ K3 + K4, binned: the fast deterministic path
// Global atomics run at a fixed ~21 G/s on this GPU whatever the locality, far too slow for the
// E*(s+1) forces an epoch sends to tails and negatives.  Instead the edge pass *bins* every such
// force by the destination's tile of 2^tile_bits points and a second kernel accumulates each tile
// in LDS (a segmented sum over destination tiles):
//
//   k_edges_binned   one persistent workgroup per compute unit, each owning a contiguous range of
//                    CSR positions; in every round each lane takes one directed edge.  The round's
//                    records (destination, force x, force y) are counting-sorted by tile in LDS and
//                    then written with consecutive lanes on consecutive records, so the records of
//                    one tile leave the workgroup as one contiguous run instead of one partial line
//                    per lane.  Every (workgroup, tile) pair appends to its own chain of chunks of
//                    kChunk records; a workgroup takes chunks from a private range of the pool,
//                    sized at set-up for the records its edges can emit, so handing out a chunk is
//                    an LDS operation: no global atomics, no spin loops, only workgroup barriers.
//                    Head sums are reduced over the lanes of a row with a segmented scan in lane
//                    order; rows that lie inside one wavefront store their sum directly, the few
//                    that straddle a wavefront hand their partial sums on as records.
//   k_tile_accumulate one workgroup per tile walks the chains of all workgroups for its tile and
//                    adds the records into 2 x 64-bit fixed-point accumulators per point in LDS.
//                    Integer addition is associative, so the result does not depend on the order
//                    records were appended or read in.  It then adds the head sums and writes g.
// (tile and chunk sizes and the LDS budgets: edge_plan.h)
constexpr uint32_t kNoChunk = 0xFFFFFFFFu;

struct BinArgs {
    const int32_t* head;          // [E] head of every CSR position
    uint32_t* pool;               // [max_chunks][kChunk][3]: (index inside the tile, force x, force y)
    uint32_t* chunk_prev;         // [max_chunks] previous chunk of the same chain
    uint32_t* chain_head;         // [n_bins][n_wg] last chunk of every (tile, workgroup) chain, kNoChunk if empty
    uint32_t* chain_fill;         // [n_bins][n_wg] records in that last chunk (all earlier chunks are full)
    const uint32_t* wg_pool_begin;// [n_wg + 1] each workgroup's private range of chunk ids
    float2* ghead;                // head sums of rows that lie inside one wavefront (others: records)
    int64_t E;
    int64_t e_begin, e_end;       // CSR positions this launch covers (a sub-step of a minibatch epoch; else 0, E)
    uint32_t max_chunks;
    uint32_t n_bins;
    int tile_bits;
    int* overflow;                // set if a workgroup's chunk range were ever exceeded (it cannot be)
};


// Workgroup barrier that orders LDS accesses only.  The edge pass never reads back, inside the
// kernel, anything it wrote to global memory, so its barriers need not wait for outstanding global
// loads and stores (a full __syncthreads() would drain them every round).
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// LDS tables of one edge-pass workgroup (see k_edges_binned): per tile the record count of the round
// (after the scan: first sorted slot), the fill of the open chunk, the open chunk and the first chunk
// allocated this round; then the round's records sorted by tile.
struct BinLds {
    uint32_t* start;    // [B+1]
    uint32_t* fill;     // [B] records in the open chunk (kChunk: none open / full)
    uint32_t* chunk;    // [B] open chunk of this (workgroup, tile)
    uint32_t* base;     // [B] first chunk allocated this round
    uint32_t* rec_pt;   // [nrec] destination point
    uint32_t* rec_x;    // [nrec] force x (float bits)
    uint32_t* rec_y;    // [nrec]
    uint32_t B;
    int tile_bits;
};

__device__ __forceinline__ BinLds carve_bin_lds(uint32_t* mem, uint32_t B, uint32_t nrec, int tile_bits) {
    BinLds L;
    L.start = mem; L.fill = L.start + B + 1; L.chunk = L.fill + B; L.base = L.chunk + B;
    L.rec_pt = L.base + B; L.rec_x = L.rec_pt + nrec; L.rec_y = L.rec_x + nrec;
    L.B = B; L.tile_bits = tile_bits;
    return L;
}

template <int BS>
__device__ __forceinline__ void init_bin_lds(const BinLds& L) {
    for (uint32_t b = threadIdx.x; b < L.B; b += BS) { L.start[b] = 0; L.fill[b] = kChunk; L.chunk[b] = kNoChunk; L.base[b] = 0; }
    if (threadIdx.x == 0) L.start[L.B] = 0;
}

// rank of a new record among this round's records of its tile
__device__ __forceinline__ uint32_t take_rank(const BinLds& L, uint32_t pt) { return atomicAdd(&L.start[pt >> L.tile_bits], 1u); }

// One round of the binned scatter for a workgroup of BS lanes.  Every lane brings up to NR records
// (valid[k], destination pt[k], force (fx[k], fy[k]), rank[k] from take_rank).  The records are
// counting-sorted by tile in LDS and appended to the (workgroup, tile) chains with consecutive lanes
// on consecutive records.  FLUSH_ITERS * BS bounds the records of one round.  All lanes must call.
template <int NR, int BS, int FLUSH_ITERS>
__device__ __forceinline__ void sort_and_flush(const BinLds& L, const BinArgs& Q, uint32_t pool_end, uint32_t* pool_cursor,
                                               uint32_t* wave_total, const bool (&valid)[NR], const uint32_t (&pt)[NR],
                                               const uint32_t (&rank)[NR], const float (&fx)[NR], const float (&fy)[NR]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t B = L.B;
    const int tb = L.tile_bits;
    const uint32_t per = (B + BS - 1) / BS;   // tiles owned by one thread, contiguous
    const uint32_t b0 = min(B, (uint32_t)tid * per), b1 = min(B, b0 + per);
    lds_barrier();
    // ---- exclusive scan of the per-tile counts
    uint32_t cnt_own[kMaxBinsPerThread];
    uint32_t own_sum = 0;
#pragma unroll
    for (int x = 0; x < kMaxBinsPerThread; ++x) {
        cnt_own[x] = (b0 + x < b1) ? L.start[b0 + x] : 0u;
        own_sum += cnt_own[x];
    }
    uint32_t incl = own_sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t u = __shfl_up(incl, d, 64);
        if (lane >= d) incl += u;
    }
    if (lane == 63) wave_total[wave] = incl;
    lds_barrier();
    uint32_t run = incl - own_sum;
    for (int v = 0; v < wave; ++v) run += wave_total[v];
    if (tid == BS - 1) L.start[B] = run + own_sum;
    // tiles whose open chunk cannot take this round's records get new chunks, linked to the chain
#pragma unroll
    for (int x = 0; x < kMaxBinsPerThread; ++x) {
        const uint32_t b = b0 + x;
        if (b < b1) {
            const uint32_t c = cnt_own[x];
            L.start[b] = run;
            run += c;
            const uint32_t fl = L.fill[b];
            if (c != 0 && fl + c > (uint32_t)kChunk) {
                const uint32_t k = (fl + c - 1) / kChunk;
                const uint32_t nb = atomicAdd(pool_cursor, k);
                L.base[b] = nb;
                if (nb + k > pool_end) *Q.overflow = 1;
                uint32_t prev = L.chunk[b];
                for (uint32_t y = 0; y < k && nb + y < pool_end; ++y) { Q.chunk_prev[nb + y] = prev; prev = nb + y; }
            }
        }
    }
    lds_barrier();
    // ---- records to their sorted slots
    {
        uint32_t p[NR];
#pragma unroll
        for (int k = 0; k < NR; ++k) p[k] = valid[k] ? L.start[pt[k] >> tb] + rank[k] : 0u;
#pragma unroll
        for (int k = 0; k < NR; ++k)
            if (valid[k]) { L.rec_pt[p[k]] = pt[k]; L.rec_x[p[k]] = __float_as_uint(fx[k]); L.rec_y[p[k]] = __float_as_uint(fy[k]); }
    }
    lds_barrier();
    // ---- consecutive lanes write consecutive sorted records to the chains
    const uint32_t total = L.start[B];
#pragma nounroll
    for (int it = 0; it < FLUSH_ITERS; ++it) {
        const uint32_t p = (uint32_t)tid + (uint32_t)it * BS;
        if (p < total) {
            const uint32_t dpt = L.rec_pt[p];
            const uint32_t b = dpt >> tb;
            const uint32_t pos = L.fill[b] + (p - L.start[b]);
            uint32_t ch, off;
            if (pos < (uint32_t)kChunk) { ch = L.chunk[b]; off = pos; }
            else { ch = L.base[b] + (pos - kChunk) / kChunk; off = (pos - kChunk) % kChunk; }
            if (ch < pool_end) {   // kNoChunk is above any valid id
                uint32_t* dst = Q.pool + ((size_t)ch * kChunk + off) * 3;
                dst[0] = dpt & ((1u << tb) - 1u);
                dst[1] = L.rec_x[p];
                dst[2] = L.rec_y[p];
            }
        }
    }
    lds_barrier();
    // ---- chain state after this round; counts back to zero
#pragma unroll
    for (int x = 0; x < kMaxBinsPerThread; ++x) {
        const uint32_t b = b0 + x;
        if (b < b1) {
            const uint32_t c = cnt_own[x];
            if (c != 0) {
                const uint32_t fl = L.fill[b];
                if (fl + c > (uint32_t)kChunk) {
                    const uint32_t k = (fl + c - 1) / kChunk;
                    L.chunk[b] = L.base[b] + k - 1;
                    L.fill[b] = fl + c - k * kChunk;
                } else {
                    L.fill[b] = fl + c;
                }
            }
            L.start[b] = 0;
        }
    }
    lds_barrier();
}

// The same round without the counting sort, for graphs whose rounds reach few of many tiles (more tiles than a round
// has records, and negatives drawn near the head): a record's place in its chain is the chain's fill plus the rank
// it took from the tile's counter, so once the chains have been extended every lane writes its own records.  The
// records of one tile still land side by side; what is given up is that consecutive lanes write them, what is saved
// are the scan over all tiles, the staging in LDS and two of the round's six barriers.  All lanes must call.
template <int NR, int BS>
__device__ __forceinline__ void direct_flush(const BinLds& L, const BinArgs& Q, uint32_t pool_end, uint32_t* pool_cursor,
                                             const bool (&valid)[NR], const uint32_t (&pt)[NR], const uint32_t (&rank)[NR],
                                             const float (&fx)[NR], const float (&fy)[NR]) {
    const uint32_t B = L.B;
    const int tb = L.tile_bits;
    lds_barrier();   // the round's counts are complete
    for (uint32_t b = threadIdx.x; b < B; b += BS) {
        const uint32_t c = L.start[b], fl = L.fill[b];
        if (c != 0 && fl + c > (uint32_t)kChunk) {
            const uint32_t k = (fl + c - 1) / kChunk;
            const uint32_t nb = atomicAdd(pool_cursor, k);
            L.base[b] = nb;
            if (nb + k > pool_end) *Q.overflow = 1;
            uint32_t prev = L.chunk[b];
            for (uint32_t y = 0; y < k && nb + y < pool_end; ++y) { Q.chunk_prev[nb + y] = prev; prev = nb + y; }
        }
    }
    lds_barrier();
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        if (valid[k]) {
            const uint32_t b = pt[k] >> tb;
            const uint32_t pos = L.fill[b] + rank[k];
            uint32_t ch, off;
            if (pos < (uint32_t)kChunk) { ch = L.chunk[b]; off = pos; }
            else { ch = L.base[b] + (pos - kChunk) / kChunk; off = (pos - kChunk) % kChunk; }
            if (ch < pool_end) {   // kNoChunk is above any valid id
                uint32_t* dst = Q.pool + ((size_t)ch * kChunk + off) * 3;
                dst[0] = pt[k] & ((1u << tb) - 1u);
                dst[1] = __float_as_uint(fx[k]);
                dst[2] = __float_as_uint(fy[k]);
            }
        }
    }
    lds_barrier();   // the tables have been read
    for (uint32_t b = threadIdx.x; b < B; b += BS) {
        const uint32_t c = L.start[b];
        if (c != 0) {
            const uint32_t fl = L.fill[b];
            if (fl + c > (uint32_t)kChunk) {
                const uint32_t k = (fl + c - 1) / kChunk;
                L.chunk[b] = L.base[b] + k - 1;
                L.fill[b] = fl + c - k * kChunk;
            } else {
                L.fill[b] = fl + c;
            }
            L.start[b] = 0;
        }
    }
    lds_barrier();
}

// the last chunk of every chain and how full it is (end of the edge pass)
template <int BS>
__device__ __forceinline__ void publish_chains(const BinLds& L, const BinArgs& Q, uint32_t pool_end) {
    const uint32_t W = gridDim.x, w = blockIdx.x;
    for (uint32_t b = threadIdx.x; b < L.B; b += BS) {
        const uint32_t ch = L.chunk[b];
        Q.chain_head[(size_t)b * W + w] = ch < pool_end ? ch : kNoChunk;
        Q.chain_fill[(size_t)b * W + w] = L.fill[b];
    }
}

// Head sum of each row: segmented inclusive scan over the lanes of the row, in lane order.  The last
// lane of a row then holds the row's sum; it is stored directly when the whole row lies inside this
// wavefront (positions wave_e0 .. wave_e0+63, below e_end), else it has to be handed on as a record
// (returns true on that lane).  A row is a run of consecutive CSR positions ea .. eb-1, so the first lane of a
// lane's segment follows from ea: no lane has to look at its neighbours' heads.
__device__ __forceinline__ bool reduce_head_sums(const BinArgs& Q, bool has, int32_t i, int32_t ea, int32_t eb, int64_t e64,
                                                 int64_t e_end, float& hx, float& hy) {
    const int lane = threadIdx.x & 63;
    const int64_t wave_e0 = e64 - lane;
    const int seg0 = has ? (int)max((int64_t)ea - wave_e0, (int64_t)0) : lane;   // first lane of this lane's row
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const float ux = __shfl_up(hx, d, 64), uy = __shfl_up(hy, d, 64);
        if (lane - d >= seg0) { hx += ux; hy += uy; }
    }
    const bool row_end = has && (lane == 63 || e64 + 1 >= min((int64_t)eb, e_end));
    const bool inside = (int64_t)ea >= wave_e0 && (int64_t)eb <= min(wave_e0 + 64, e_end);
    if (row_end && inside) Q.ghead[i] = make_float2(hx, hy);
    return row_end && !inside;
}

// What one lane has in flight for its edge of the next round: issued a round ahead, so that the
// gathers of round r+1 are served while round r is being sorted and written out.  GATHER: also the
// rows of the negatives (i.i.d. sampler); the pooled sampler reads them from its pool in LDS.
template <int S, bool GATHER>
struct EdgeFetch {
    bool has;
    int32_t e, i, j, ea, eb;
    float pe;
    HeadCtx h;
    int32_t m[S > 0 ? S : 1];
    float2 tj, tm[S > 0 ? S : 1];   // sampled far field: tm[k].x carries the cell of m[k] until the round resolves it
};

template <int S, bool GATHER>
__device__ __forceinline__ void issue_edge(const EdgeArgs& P, bool has, int32_t e, int32_t i, int32_t j, EdgeFetch<S, GATHER>& f) {
    f.has = has;
    f.e = e; f.i = has ? i : -1; f.j = j; f.ea = 0; f.eb = 0; f.pe = 0.f;
    if (!has) return;
    f.ea = P.row_ptr[i];
    f.eb = P.row_ptr[i + 1];
    f.h = load_head(P, i, f.ea, f.eb);
    f.tj = P.theta[j];
    f.pe = P.pe ? P.pe[e] : f.h.inv_deg;
    if (GATHER) {
        draw_negatives<S>(P, f.h.pop, e, f.m);
        if (P.far) {
#pragma unroll
            for (int k = 0; k < S; ++k) f.tm[k] = make_float2(__int_as_float(P.cluster_of[f.m[k]]), 0.f);
        } else {
#pragma unroll
            for (int k = 0; k < S; ++k) f.tm[k] = P.theta[f.m[k]];
        }
    }
}

// Sampled far field: with the cells of the negatives in hand, fetch what each stands for: the mean of its cell
// when the cell belongs to another group than the head's (then m = -1: no force goes back), else its own row.
template <int S>
__device__ __forceinline__ void resolve_far_negatives(const EdgeArgs& P, EdgeFetch<S, true>& f) {
    int32_t grp[S > 0 ? S : 1];
    float2 mean[S > 0 ? S : 1];
#pragma unroll
    for (int k = 0; k < S; ++k) {
        const int32_t r = __float_as_int(f.tm[k].x);
        grp[k] = P.group_of_cluster[r];
        mean[k] = P.mu[r];
    }
#pragma unroll
    for (int k = 0; k < S; ++k) {
        if (grp[k] != f.h.group) { f.tm[k] = mean[k]; f.m[k] = -1; }
        else f.tm[k] = P.theta[f.m[k]];
    }
}

template <int S, int BS, bool SORT = true, int ROUNDS = 1>
__global__ void __launch_bounds__(BS) k_edges_binned(const EdgeArgs P, const BinArgs Q) {
    static_assert(!SORT || ROUNDS == 1, "the sorted form stages one round's records in LDS");
    constexpr int SS = S > 0 ? S : 1;
    constexpr int kWaves = BS / 64;
    constexpr int NREC = BS * (S + 1) + 2 * kWaves;
    constexpr int NR = S + 2;   // per lane and round: the tail, the negatives, and possibly a partial head sum
    extern __shared__ uint32_t lds_bins[];
    const BinLds L = carve_bin_lds(lds_bins, Q.n_bins, SORT ? NREC : 0, Q.tile_bits);
    __shared__ uint32_t wave_total[kWaves];
    __shared__ uint32_t pool_cursor;
    const int tid = threadIdx.x;
    const uint32_t W = gridDim.x, w = blockIdx.x;
    const uint32_t pool_end = min(Q.wg_pool_begin[w + 1], Q.max_chunks);
    init_bin_lds<BS>(L);
    if (tid == 0) pool_cursor = Q.wg_pool_begin[w];
    lds_barrier();

    // The CSR positions are dealt to the workgroups in slabs of BS positions, round-robin: slab w, w + W, ...
    // (every workgroup then sends records to every tile at about the same rate, whatever the locality of the
    // graph, which keeps the chains the tile pass walks equally long).
    const int64_t n_slabs = (Q.e_end - Q.e_begin + BS - 1) / BS;
    const int64_t stride = (int64_t)W * BS;
    // Software pipeline over rounds: (head, tail) indices are read two rounds ahead, the embedding rows
    // one round ahead.
    EdgeFetch<S, true> f;
    int32_t i_next = 0, j_next = 0;
    {
        const int64_t e0 = Q.e_begin + (int64_t)w * BS + tid, e1 = e0 + stride;
        int32_t i0 = 0, j0 = 0;
        if (e0 < Q.e_end) { i0 = Q.head[e0]; j0 = P.col[e0]; }
        if (e1 < Q.e_end) { i_next = Q.head[e1]; j_next = P.col[e1]; }
        issue_edge<S, true>(P, e0 < Q.e_end, (int32_t)e0, i0, j0, f);
    }
    // The unsorted form takes ROUNDS rounds between two flushes (no barrier in between: a record only takes its rank
    // from the tile's counter when it is made); slabs past the end are empty rounds.
    for (int64_t slab0 = w; slab0 < n_slabs; slab0 += (int64_t)W * ROUNDS) {
        bool valid[NR * ROUNDS];
        uint32_t dst_pt[NR * ROUNDS], rank[NR * ROUNDS];
        float fx[NR * ROUNDS], fy[NR * ROUNDS];
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            // one edge per lane; records: slot 0 the tail (force -a d_ij), slots 1..S the negatives
            const int64_t slab = slab0 + (int64_t)r * W;
            const int64_t e64 = Q.e_begin + slab * BS + tid;
            const int64_t e_end = min(Q.e_begin + (slab + 1) * BS, Q.e_end);
            const bool has = f.has;
            const int32_t i = f.i, ea = f.ea, eb = f.eb;
            const int base = r * NR;
#pragma unroll
            for (int k = 0; k < NR; ++k) { valid[base + k] = k <= S && has; dst_pt[base + k] = 0u; rank[base + k] = 0u; fx[base + k] = 0.f; fy[base + k] = 0.f; }
            float hx = 0.f, hy = 0.f;
            if (has) {
                if (P.far) resolve_far_negatives<S>(P, f);
                EdgeOut<SS> o;
                edge_math<S, false>(f.h, f.pe, f.tj, f.tm, o);
                hx = o.hx;
                hy = o.hy;
                if (P.cS) P.cS[f.e] = o.c;
                dst_pt[base] = (uint32_t)f.j; fx[base] = -o.a * o.dx; fy[base] = -o.a * o.dy;
#pragma unroll
                for (int k = 0; k < S; ++k) {
                    valid[base + k + 1] = f.m[k] >= 0;
                    dst_pt[base + k + 1] = f.m[k] >= 0 ? (uint32_t)f.m[k] : 0u;
                    fx[base + k + 1] = o.rx[k];
                    fy[base + k + 1] = o.ry[k];
                }
            }
            // the loads of the next round go out before this round is sorted and written
            {
                const int64_t e1 = e64 + stride, e2 = e1 + stride;
                const int32_t i1 = i_next, j1 = j_next;
                if (e2 < Q.e_end) { i_next = Q.head[e2]; j_next = P.col[e2]; }
                issue_edge<S, true>(P, e1 < Q.e_end, (int32_t)e1, i1, j1, f);
            }
            valid[base + S + 1] = reduce_head_sums(Q, has, i, ea, eb, e64, e_end, hx, hy);
            dst_pt[base + S + 1] = valid[base + S + 1] ? (uint32_t)i : 0u;
            fx[base + S + 1] = hx;
            fy[base + S + 1] = hy;
#pragma unroll
            for (int k = 0; k < NR; ++k)
                if (valid[base + k]) rank[base + k] = take_rank(L, dst_pt[base + k]);
        }
        if (SORT) sort_and_flush<NR * ROUNDS, BS, (NREC + BS - 1) / BS>(L, Q, pool_end, &pool_cursor, wave_total, valid, dst_pt, rank, fx, fy);
        else direct_flush<NR * ROUNDS, BS>(L, Q, pool_end, &pool_cursor, valid, dst_pt, rank, fx, fy);
    }
    publish_chains<BS>(L, Q, pool_end);
}

// ------------------------------------------------------------------ K3 + K4 with the pooled sampler
// The negatives of a block of ROUNDS * 1024 consecutive CSR positions come from the block's pool of
// P.pool_size points, which lives in LDS: pool_th (their embedding rows, one gather per pool entry and block
// instead of one per negative) and pool_acc (64-bit fixed-point sums of the forces they receive, handed on as
// one record per pool entry and block).  The rounds of a block run without barriers.  Records (one tail per
// edge, the pool entries, the few partial head sums) are not sorted: a record takes its rank among the block's
// records of its tile from an LDS counter when it is made, and once the tiles' chains have been extended every
// lane writes its own records at fill + rank.  Tails of one wavefront mostly share a tile and get consecutive
// ranks, so their writes still coalesce; a pool entry's record is alone in its tile whichever way it is written.
constexpr int kMaxPoolPerLane = 4;   // pool entries one lane fetches and hands on: pool_size <= 4 * workgroup size


// What a lane of the pooled edge pass has in flight for its next edge (no groups there: one population, no mean field).
struct PoolFetch {
    bool has;
    int32_t e, i, j, ea, eb;
    float pe;
    float2 ti, tj;
};

__device__ __forceinline__ void issue_pool_edge(const EdgeArgs& P, bool has, int32_t e, int32_t i, int32_t j, PoolFetch& f) {
    f.has = has;
    f.e = e; f.i = has ? i : -1; f.j = j; f.ea = 0; f.eb = 0; f.pe = 0.f;
    f.ti = make_float2(0.f, 0.f);
    f.tj = make_float2(0.f, 0.f);
    if (!has) return;
    f.ea = P.row_ptr[i];
    f.eb = P.row_ptr[i + 1];
    f.ti = P.theta[i];
    f.tj = P.theta[j];
    if (P.pe) f.pe = P.pe[e];
}

template <int S, int ROUNDS, int BS>
__global__ void __launch_bounds__(BS) k_edges_pooled(const EdgeArgs P, const BinArgs Q) {
    constexpr int SS = S > 0 ? S : 1;
    constexpr int NP = kMaxPoolPerLane;
    constexpr int kSide = 2 * (BS / 64) * ROUNDS;    // partial head sums a block can produce
    extern __shared__ unsigned long long lds_pool[];
    const uint32_t PS = P.pool_size, B = Q.n_bins;
    const int tb = Q.tile_bits;
    unsigned long long* pool_acc = lds_pool;                         // [2 PS] fixed-point force sums
    float2* pool_th = (float2*)(pool_acc + 2 * (size_t)PS);          // [PS] embedding rows of the pool
    uint32_t* pool_pt = (uint32_t*)(pool_th + PS);                   // [PS] the points
    uint32_t* cnt = pool_pt + PS;                                    // [B] records of this block per tile
    uint32_t* fill = cnt + B;                                        // [B] records in the open chunk (kChunk: none open / full)
    uint32_t* chunk = fill + B;                                      // [B] open chunk of this (workgroup, tile)
    uint32_t* base = chunk + B;                                      // [B] first chunk allocated for this block
    uint32_t* side_pt = base + B;                                    // [kSide] partial head sums: the head
    float* side_x = (float*)(side_pt + kSide);                       // [kSide]
    float* side_y = side_x + kSide;                                  // [kSide]
    __shared__ uint32_t pool_cursor, side_n;
    const int tid = threadIdx.x;
    const uint32_t W = gridDim.x, w = blockIdx.x;
    constexpr int64_t G = (int64_t)BS * ROUNDS;                       // = P.pool_block
    // the blocks that meet this launch's positions are dealt to the workgroups round-robin: first_block + w, + W, ...
    // (blocks are counted from CSR position 0 whatever the launch covers: a block's pool does not depend on it)
    const int64_t first_block = Q.e_begin / G;
    const int64_t n_blocks = (Q.e_end + G - 1) / G;   // one past the last block
    const uint32_t pool_end = min(Q.wg_pool_begin[w + 1], Q.max_chunks);
    for (uint32_t b = tid; b < B; b += BS) { cnt[b] = 0; fill[b] = kChunk; chunk[b] = kNoChunk; base[b] = 0; }
    for (uint32_t u = tid; u < 2 * PS; u += BS) pool_acc[u] = 0ull;
    if (tid == 0) { pool_cursor = Q.wg_pool_begin[w]; side_n = 0; }

    // One Philox call yields four consecutive pool entries, so lane t fetches entries 4t .. 4t+3 (lanes beyond
    // pool_size / 4 idle); a block's pool is fetched while the block before it is written out.
    uint32_t next_pt[NP];
    float2 next_th[NP];
    auto fetch_pool = [&](int64_t blk) {
#pragma unroll
        for (int k = 0; k < NP; ++k) { next_pt[k] = 0u; next_th[k] = make_float2(0.f, 0.f); }
        const uint32_t u0 = 4u * (uint32_t)tid;
        if (u0 < PS && blk < n_blocks) {
            uint32_t wd[4];
            philox4x32_10((uint32_t)blk, 0xFFFFFFFFu, P.epoch, (uint32_t)tid, P.key0, P.key1, wd);
#pragma unroll
            for (int k = 0; k < NP; ++k)
                if (u0 + k < PS) { next_pt[k] = __umulhi(wd[k], (uint32_t)P.n); next_th[k] = P.theta[next_pt[k]]; }
        }
    };
    auto stage_pool = [&]() {
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const uint32_t u = 4u * (uint32_t)tid + (uint32_t)k;
            if (u < PS) { pool_pt[u] = next_pt[k]; pool_th[u] = next_th[k]; }
        }
    };
    fetch_pool(first_block + w);
    stage_pool();
    // edge pipeline: (head, tail) indices two rounds ahead, embedding rows one round ahead; the position after the
    // last one of a block is the first of this workgroup's next block
    auto next_position = [&](int64_t e) { return (e + BS) % G < BS ? e + BS + (int64_t)(W - 1) * G : e + BS; };
    auto covered = [&](int64_t e) { return e >= Q.e_begin && e < Q.e_end; };
    PoolFetch f;
    int32_t i_next = 0, j_next = 0;
    {
        const int64_t e0 = (first_block + w) * G + tid, e1 = next_position(e0);
        int32_t i0 = 0, j0 = 0;
        if (covered(e0)) { i0 = Q.head[e0]; j0 = P.col[e0]; }
        if (covered(e1)) { i_next = Q.head[e1]; j_next = P.col[e1]; }
        issue_pool_edge(P, covered(e0), (int32_t)e0, i0, j0, f);
    }
    // a record goes to position fill + rank of its tile's chain
    auto emit = [&](bool valid, uint32_t pt, uint32_t rank, float x, float y) {
        if (!valid) return;
        const uint32_t b = pt >> tb;
        const uint32_t pos = fill[b] + rank;
        uint32_t ch, off;
        if (pos < (uint32_t)kChunk) { ch = chunk[b]; off = pos; }
        else { ch = base[b] + (pos - kChunk) / kChunk; off = (pos - kChunk) % kChunk; }
        if (ch < pool_end) {   // kNoChunk is above any valid id
            uint32_t* dst = Q.pool + ((size_t)ch * kChunk + off) * 3;
            dst[0] = pt & ((1u << tb) - 1u);
            dst[1] = __float_as_uint(x);
            dst[2] = __float_as_uint(y);
        }
    };
    HeadCtx h;
    h.omega = P.omega0;
    h.MA = h.MBx = h.MBy = 0.f;
    for (int64_t blk = first_block + w; blk < n_blocks; blk += W) {
        const int64_t e_end = min((blk + 1) * G, Q.e_end);
        lds_barrier();   // the block's pool is in LDS, the tile tables are those left by the block before
        bool tv[ROUNDS];
        uint32_t tpt[ROUNDS], trk[ROUNDS];
        float tfx[ROUNDS], tfy[ROUNDS];
        // ---- ROUNDS rounds of one edge per lane, no barriers in between
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int64_t e64 = blk * G + (int64_t)r * BS + tid;
            const bool has = f.has;
            const int32_t i = f.i, ea = f.ea, eb = f.eb;
            float hx = 0.f, hy = 0.f;
            tv[r] = has; tpt[r] = 0u; trk[r] = 0u; tfx[r] = 0.f; tfy[r] = 0.f;
            if (has) {
                uint32_t slot[SS];
                float2 tm[SS];
                {
                    uint32_t wd[4];
                    philox4x32_10((uint32_t)f.e, 0u, P.epoch, 0u, P.key0, P.key1, wd);   // S <= 8: one call
#pragma unroll
                    for (int k = 0; k < S; ++k) slot[k] = pool_slot(wd, k, PS);
                }
#pragma unroll
                for (int k = 0; k < S; ++k) tm[k] = pool_th[slot[k]];
                h.ti = f.ti;
                EdgeOut<SS> o;
                edge_math<S, false>(h, P.pe ? f.pe : 1.0f / (float)(eb - ea), f.tj, tm, o);
                hx = o.hx;
                hy = o.hy;
#pragma unroll
                for (int k = 0; k < S; ++k) {
                    atomicAdd(&pool_acc[2 * slot[k]], to_fixed(o.rx[k]));
                    atomicAdd(&pool_acc[2 * slot[k] + 1], to_fixed(o.ry[k]));
                }
                tpt[r] = (uint32_t)f.j; tfx[r] = -o.a * o.dx; tfy[r] = -o.a * o.dy;
                trk[r] = atomicAdd(&cnt[tpt[r] >> tb], 1u);
            }
            {
                const int64_t e1 = next_position(e64), e2 = next_position(e1);
                const int32_t i1 = i_next, j1 = j_next;
                if (covered(e2)) { i_next = Q.head[e2]; j_next = P.col[e2]; }
                issue_pool_edge(P, covered(e1), (int32_t)e1, i1, j1, f);
            }
            if (reduce_head_sums(Q, has, i, ea, eb, e64, e_end, hx, hy)) {
                const uint32_t k = atomicAdd(&side_n, 1u);
                side_pt[k] = (uint32_t)i; side_x[k] = hx; side_y[k] = hy;
            }
        }
        fetch_pool(blk + W);
        lds_barrier();   // every force of the block is in pool_acc, the side list is complete
        // ---- one record per pool entry that received a force, one per partial head sum
        bool pv[NP];
        uint32_t ppt[NP], prk[NP];
        float pfx[NP], pfy[NP];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const uint32_t u = (uint32_t)tid + (uint32_t)k * BS;
            pv[k] = false; ppt[k] = 0u; prk[k] = 0u; pfx[k] = 0.f; pfy[k] = 0.f;
            if (u < PS) {
                const long long ax = (long long)pool_acc[2 * u], ay = (long long)pool_acc[2 * u + 1];
                pv[k] = (ax | ay) != 0;
                if (pv[k]) {
                    pool_acc[2 * u] = 0ull;
                    pool_acc[2 * u + 1] = 0ull;
                    ppt[k] = pool_pt[u];
                    pfx[k] = (float)((double)ax * kFixInv);
                    pfy[k] = (float)((double)ay * kFixInv);
                    prk[k] = atomicAdd(&cnt[ppt[k] >> tb], 1u);
                }
            }
        }
        const bool sv = (uint32_t)tid < side_n;
        uint32_t spt = 0u, srk = 0u;
        float sx = 0.f, sy = 0.f;
        if (sv) { spt = side_pt[tid]; sx = side_x[tid]; sy = side_y[tid]; srk = atomicAdd(&cnt[spt >> tb], 1u); }
        lds_barrier();   // the counts are complete
        // ---- tiles whose open chunk cannot take this block's records get new chunks, linked to the chain
        for (uint32_t b = tid; b < B; b += BS) {
            const uint32_t c = cnt[b], fl = fill[b];
            if (c != 0 && fl + c > (uint32_t)kChunk) {
                const uint32_t k = (fl + c - 1) / kChunk;
                const uint32_t nb = atomicAdd(&pool_cursor, k);
                base[b] = nb;
                if (nb + k > pool_end) *Q.overflow = 1;
                uint32_t prev = chunk[b];
                for (uint32_t y = 0; y < k && nb + y < pool_end; ++y) { Q.chunk_prev[nb + y] = prev; prev = nb + y; }
            }
        }
        lds_barrier();
        // ---- every lane writes its own records
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) emit(tv[r], tpt[r], trk[r], tfx[r], tfy[r]);
#pragma unroll
        for (int k = 0; k < NP; ++k) emit(pv[k], ppt[k], prk[k], pfx[k], pfy[k]);
        emit(sv, spt, srk, sx, sy);
        lds_barrier();   // the tables have been read
        // ---- chain state after this block, counts back to zero; the next block's pool into LDS
        for (uint32_t b = tid; b < B; b += BS) {
            const uint32_t c = cnt[b];
            if (c != 0) {
                const uint32_t fl = fill[b];
                if (fl + c > (uint32_t)kChunk) {
                    const uint32_t k = (fl + c - 1) / kChunk;
                    chunk[b] = base[b] + k - 1;
                    fill[b] = fl + c - k * kChunk;
                } else {
                    fill[b] = fl + c;
                }
                cnt[b] = 0;
            }
        }
        if (tid == 0) side_n = 0;
        stage_pool();
    }
    lds_barrier();
    for (uint32_t b = tid; b < B; b += BS) {
        const uint32_t ch = chunk[b];
        Q.chain_head[(size_t)b * W + w] = ch < pool_end ? ch : kNoChunk;
        Q.chain_fill[(size_t)b * W + w] = fill[b];
    }
}

// ------------------------------------------------------------------ K3 + K4, pooled sampler with distinct picks
// Same plan as k_edges_pooled (pool rows and their force sums in LDS, unsorted records ranked per tile, chains
// extended once per block) for the sampler whose picks of one edge lie in different pool lines (nomad.h).  What
// differs: a block's positions are Q segments spread over the edge list (position of rank r * 1024 + lane: segment
// rank >> seg_bits of the block, offset rank & (segment - 1)); one Philox call serves a lane's picks of four rounds
// (word r & 3 of call number lane + 1024 (r >> 2)); a pool line is pool_line consecutive points, read by adjacent
// lanes (one or two 128-byte lines per pool line instead of one per entry), and its entries' records leave as one
// contiguous run; positions, indices and byte offsets are 32-bit (needs 8 n < 2^32, checked by the host).

struct DistinctFetch {   // what a lane has in flight for its edge of the next round
    bool has;
    uint32_t e, i, j, ea, eb;
    float pe;
    float2 ti, tj;
};

template <typename T>
__device__ __forceinline__ T load_at(const T* base, uint32_t index) {   // 64-bit base + 32-bit byte offset
    return *(const T*)((const char*)base + (size_t)(index * (uint32_t)sizeof(T)));
}

template <int S, int ROUNDS>
__global__ void __launch_bounds__(1024) k_edges_pooled_distinct(const EdgeArgs P, const BinArgs Q) {
    constexpr int SS = S > 0 ? S : 1;
    constexpr int BS = 1024;
    constexpr int NP = kMaxPoolPerLane;
    constexpr int kSide = 32 * ROUNDS;                                 // partial head sums a block can produce
    extern __shared__ unsigned long long lds_pool[];
    const uint32_t PS = P.pool_size, B = Q.n_bins, n = (uint32_t)P.n, E = (uint32_t)Q.E, NB = P.pool_blocks;
    const uint32_t line_bits = P.pool_line_bits, seg_bits = P.pool_segment_bits;
    const uint32_t L = PS >> line_bits, lg_lines = 31u - (uint32_t)__clz(L);
    const int tb = Q.tile_bits;
    unsigned long long* pool_acc = lds_pool;                         // [2 PS] fixed-point force sums
    float2* pool_th = (float2*)(pool_acc + 2 * (size_t)PS);          // [PS] embedding rows of the pool
    uint32_t* pool_pt = (uint32_t*)(pool_th + PS);                   // [PS] the points
    uint32_t* line_start = pool_pt + PS;                             // [L] first point of every line of the NEXT block
    uint32_t* cnt = line_start + L;                                  // [B] records of this block per tile
    uint32_t* fill = cnt + B;                                        // [B] records in the open chunk (kChunk: none open / full)
    uint32_t* chunk = fill + B;                                      // [B] open chunk of this (workgroup, tile)
    uint32_t* base = chunk + B;                                      // [B] first chunk allocated for this block
    uint32_t* side_pt = base + B;                                    // [kSide] partial head sums: the head
    float* side_x = (float*)(side_pt + kSide);
    float* side_y = side_x + kSide;
    __shared__ uint32_t pool_cursor, side_n;
    const uint32_t tid = threadIdx.x;
    const uint32_t W = gridDim.x, w = blockIdx.x;
    const uint32_t pool_end = min(Q.wg_pool_begin[w + 1], Q.max_chunks);
    for (uint32_t b = tid; b < B; b += BS) { cnt[b] = 0; fill[b] = kChunk; chunk[b] = kNoChunk; base[b] = 0; }
    for (uint32_t u = tid; u < 2 * PS; u += BS) pool_acc[u] = 0ull;
    if (tid == 0) { pool_cursor = Q.wg_pool_begin[w]; side_n = 0; }

    // ---- the pool of a block: line starts (one Philox call per four lines), then every lane fetches up to NP entries;
    // lane index idx = tid + 1024 k stands for point number idx % pool_line of line idx / pool_line, i.e. entry
    // (idx % pool_line) L + idx / pool_line: adjacent lanes read adjacent points
    auto draw_lines = [&](uint32_t blk) {
        if (P.pool_mode == 2) {   // stratified pools: the block's lines, dealt from this epoch's permutation of the lines
            if (blk < NB)         // (up to 4096 lines when a line is a single point: more than one per lane)
                for (uint32_t g = tid; g < L; g += BS) line_start[g] = stratified_line_start(P, (uint64_t)blk * L + g);
        } else if (4u * tid < L && blk < NB) {
            uint32_t wd[4];
            philox4x32_10(blk, kPoolEntryStream, P.epoch, tid, P.key0, P.key1, wd);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (4u * tid + k < L) line_start[4u * tid + k] = __umulhi(wd[k], n);
        }
    };
    uint32_t next_pt[NP];
    float2 next_th[NP];
    auto fetch_pool = [&](uint32_t blk) {
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            next_pt[k] = 0u;
            next_th[k] = make_float2(0.f, 0.f);
            const uint32_t idx = tid + (uint32_t)k * BS;
            if (idx < PS && blk < NB) {
                uint32_t pt = line_start[idx >> line_bits] + (idx & ((1u << line_bits) - 1u));
                if (pt >= n) pt -= n;
                next_pt[k] = pt;
                next_th[k] = load_at(P.theta, pt);
            }
        }
    };
    auto entry_of = [&](uint32_t idx) { return ((idx & ((1u << line_bits) - 1u)) << lg_lines) + (idx >> line_bits); };
    auto stage_pool = [&]() {
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const uint32_t idx = tid + (uint32_t)k * BS;
            if (idx < PS) { const uint32_t u = entry_of(idx); pool_pt[u] = next_pt[k]; pool_th[u] = next_th[k]; }
        }
    };
    // ---- positions: rank r * 1024 + tid of block blk
    auto position = [&](uint32_t blk, int r, bool& has) {
        const uint32_t rank = (uint32_t)r * BS + tid;
        const uint32_t e = ((blk + (rank >> seg_bits) * NB) << seg_bits) + (rank & ((1u << seg_bits) - 1u));
        has = blk < NB && e < E;
        return e;
    };
    auto issue = [&](bool has, uint32_t e, uint32_t i, uint32_t j, DistinctFetch& f) {
        f.has = has; f.e = e; f.i = i; f.j = j; f.ea = 0; f.eb = 0; f.pe = 0.f;
        f.ti = make_float2(0.f, 0.f);
        f.tj = make_float2(0.f, 0.f);
        if (!has) return;
        f.ea = (uint32_t)load_at(P.row_ptr, i);
        f.eb = (uint32_t)load_at(P.row_ptr + 1, i);
        f.ti = load_at(P.theta, i);
        f.tj = load_at(P.theta, j);
        if (P.pe) f.pe = load_at(P.pe, e);
    };
    draw_lines(w);
    lds_barrier();
    fetch_pool(w);
    stage_pool();
    DistinctFetch f;
    uint32_t i_next = 0, j_next = 0;
    {
        bool h0, h1;
        const uint32_t e0 = position(w, 0, h0);
        const uint32_t e1 = position(w + W * (1 / ROUNDS), 1 % ROUNDS, h1);
        uint32_t i0 = 0, j0 = 0;
        if (h0) { i0 = (uint32_t)load_at(Q.head, e0); j0 = (uint32_t)load_at(P.col, e0); }
        if (h1) { i_next = (uint32_t)load_at(Q.head, e1); j_next = (uint32_t)load_at(P.col, e1); }
        issue(h0, e0, i0, j0, f);
    }
    auto emit = [&](bool valid, uint32_t pt, uint32_t rank, float x, float y) {
        if (!valid) return;
        const uint32_t b = pt >> tb;
        const uint32_t pos = fill[b] + rank;
        uint32_t ch, off;
        if (pos < (uint32_t)kChunk) { ch = chunk[b]; off = pos; }
        else { ch = base[b] + (pos - kChunk) / kChunk; off = (pos - kChunk) % kChunk; }
        if (ch < pool_end) {   // kNoChunk is above any valid id
            uint32_t* dst = Q.pool + ((size_t)ch * kChunk + off) * 3;
            dst[0] = pt & ((1u << tb) - 1u);
            dst[1] = __float_as_uint(x);
            dst[2] = __float_as_uint(y);
        }
    };
    HeadCtx h;
    h.omega = P.omega0;
    h.MA = h.MBx = h.MBy = 0.f;
    for (uint32_t blk = w; blk < NB; blk += W) {
        lds_barrier();   // the block's pool is in LDS, the tile tables are those left by the block before
        bool tv[ROUNDS];
        uint32_t tpt[ROUNDS], trk[ROUNDS];
        float tfx[ROUNDS], tfy[ROUNDS];
        uint32_t wd[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            if ((r & 3) == 0) philox4x32_10(blk, kPoolPickStream, P.epoch, tid + 1024u * (uint32_t)(r >> 2), P.key0, P.key1, wd);
            const bool has = f.has;
            const uint32_t e = f.e, i = f.i, ea = f.ea, eb = f.eb;
            float hx = 0.f, hy = 0.f;
            tv[r] = has; tpt[r] = 0u; trk[r] = 0u; tfx[r] = 0.f; tfy[r] = 0.f;
            if (has) {
                uint32_t slot[SS];
                float2 tm[SS];
#pragma unroll
                for (int k = 0; k < S; ++k) slot[k] = distinct_pick(wd[r & 3], k, PS);
#pragma unroll
                for (int k = 0; k < S; ++k) tm[k] = pool_th[slot[k]];
                h.ti = f.ti;
                EdgeOut<SS> o;
                edge_math<S, false>(h, P.pe ? f.pe : __builtin_amdgcn_rcpf((float)(eb - ea)), f.tj, tm, o);
                hx = o.hx;
                hy = o.hy;
#pragma unroll
                for (int k = 0; k < S; ++k) {
                    atomicAdd(&pool_acc[2 * slot[k]], to_fixed(o.rx[k]));
                    atomicAdd(&pool_acc[2 * slot[k] + 1], to_fixed(o.ry[k]));
                }
                tpt[r] = f.j; tfx[r] = -o.a * o.dx; tfy[r] = -o.a * o.dy;
                trk[r] = atomicAdd(&cnt[tpt[r] >> tb], 1u);
            }
            {   // the loads of the next round go out before this round's head sums are reduced
                bool h1, h2;
                const uint32_t e1 = position(blk + W * ((r + 1) / ROUNDS), (r + 1) % ROUNDS, h1);   // one round ahead
                const uint32_t e2 = position(blk + W * ((r + 2) / ROUNDS), (r + 2) % ROUNDS, h2);   // two rounds ahead
                const uint32_t i1 = i_next, j1 = j_next;
                if (h2) { i_next = (uint32_t)load_at(Q.head, e2); j_next = (uint32_t)load_at(P.col, e2); }
                issue(h1, e1, i1, j1, f);
            }
            if (reduce_head_sums(Q, has, (int32_t)i, (int32_t)ea, (int32_t)eb, (int64_t)e, (int64_t)E, hx, hy)) {
                const uint32_t k = atomicAdd(&side_n, 1u);
                side_pt[k] = i; side_x[k] = hx; side_y[k] = hy;
            }
        }
        draw_lines(blk + W);
        lds_barrier();   // every force of the block is in pool_acc, the side list and the next block's lines are complete
        // ---- one record per pool entry that received a force, one per partial head sum
        bool pv[NP];
        uint32_t ppt[NP], prk[NP];
        float pfx[NP], pfy[NP];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const uint32_t idx = tid + (uint32_t)k * BS;
            pv[k] = false; ppt[k] = 0u; prk[k] = 0u; pfx[k] = 0.f; pfy[k] = 0.f;
            if (idx < PS) {
                const uint32_t u = entry_of(idx);
                const long long ax = (long long)pool_acc[2 * u], ay = (long long)pool_acc[2 * u + 1];
                pv[k] = (ax | ay) != 0;
                if (pv[k]) {
                    pool_acc[2 * u] = 0ull;
                    pool_acc[2 * u + 1] = 0ull;
                    ppt[k] = pool_pt[u];
                    pfx[k] = (float)((double)ax * kFixInv);
                    pfy[k] = (float)((double)ay * kFixInv);
                    prk[k] = atomicAdd(&cnt[ppt[k] >> tb], 1u);
                }
            }
        }
        const bool sv = tid < side_n;
        uint32_t spt = 0u, srk = 0u;
        float sx = 0.f, sy = 0.f;
        if (sv) { spt = side_pt[tid]; sx = side_x[tid]; sy = side_y[tid]; srk = atomicAdd(&cnt[spt >> tb], 1u); }
        fetch_pool(blk + W);
        lds_barrier();   // the counts are complete
        // ---- tiles whose open chunk cannot take this block's records get new chunks, linked to the chain
        for (uint32_t b = tid; b < B; b += BS) {
            const uint32_t c = cnt[b], fl = fill[b];
            if (c != 0 && fl + c > (uint32_t)kChunk) {
                const uint32_t k = (fl + c - 1) / kChunk;
                const uint32_t nb = atomicAdd(&pool_cursor, k);
                base[b] = nb;
                if (nb + k > pool_end) *Q.overflow = 1;
                uint32_t prev = chunk[b];
                for (uint32_t y = 0; y < k && nb + y < pool_end; ++y) { Q.chunk_prev[nb + y] = prev; prev = nb + y; }
            }
        }
        lds_barrier();
        // ---- every lane writes its own records
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) emit(tv[r], tpt[r], trk[r], tfx[r], tfy[r]);
#pragma unroll
        for (int k = 0; k < NP; ++k) emit(pv[k], ppt[k], prk[k], pfx[k], pfy[k]);
        emit(sv, spt, srk, sx, sy);
        lds_barrier();   // the tables have been read
        // ---- chain state after this block, counts back to zero; the next block's pool into LDS
        for (uint32_t b = tid; b < B; b += BS) {
            const uint32_t c = cnt[b];
            if (c != 0) {
                const uint32_t fl = fill[b];
                if (fl + c > (uint32_t)kChunk) {
                    const uint32_t k = (fl + c - 1) / kChunk;
                    chunk[b] = base[b] + k - 1;
                    fill[b] = fl + c - k * kChunk;
                } else {
                    fill[b] = fl + c;
                }
                cnt[b] = 0;
            }
        }
        if (tid == 0) side_n = 0;
        stage_pool();
    }
    lds_barrier();
    for (uint32_t b = tid; b < B; b += BS) {
        const uint32_t ch = chunk[b];
        Q.chain_head[(size_t)b * W + w] = ch < pool_end ? ch : kNoChunk;
        Q.chain_fill[(size_t)b * W + w] = fill[b];
    }
}

// chunk-id range of each workgroup for the kernel above: blocks w, w + W, ...; records per block: one tail per
// position, two partial head sums per wavefront and round, one per pool entry
__global__ void k_wg_pools_distinct(uint32_t n_blocks, int W, int64_t block_edges, uint32_t pool_size, uint32_t n_bins,
                                    uint32_t* __restrict__ wg_pool_begin, unsigned long long* __restrict__ total) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const uint64_t per_block = (uint64_t)block_edges + pooled_side_records(block_edges) + pool_size;
    const uint64_t blocks = ((uint64_t)n_blocks + W - 1) / W;
    const uint64_t per_wg = blocks * per_block / kChunk + n_bins + 1;
    for (int w = 0; w <= W; ++w) wg_pool_begin[w] = (uint32_t)min(per_wg * (uint64_t)w, (uint64_t)0xFFFFFFFFull);
    *total = per_wg * (uint64_t)W;
}

// private chunk-id range of each workgroup: enough for every record its slabs can emit (s+1 per
// position, plus at most two partial head sums per wavefront and round), plus one partly filled chunk
// per tile.  The same bound for every workgroup, valid for a launch over any sub-range of the positions.
__global__ void k_wg_pools(int64_t E, int W, int records_per_edge, int block, uint32_t n_bins, uint32_t* __restrict__ wg_pool_begin,
                           unsigned long long* __restrict__ total) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const uint64_t n_slabs = (uint64_t)((E + block - 1) / block);
    const uint64_t rounds = (n_slabs + W - 1) / W;   // slabs w, w + W, ...
    const uint64_t records = rounds * ((uint64_t)block * records_per_edge + 2 * (block / 64));
    const uint64_t per_wg = records / kChunk + n_bins + 1;
    for (int w = 0; w <= W; ++w) wg_pool_begin[w] = (uint32_t)min(per_wg * (uint64_t)w, (uint64_t)0xFFFFFFFFull);
    *total = per_wg * (uint64_t)W;
}

// the same bound for the pooled edge pass: workgroups own whole blocks of `block_edges` positions; records per
// block = one tail per edge, two partial head sums per wavefront and round, one per pool entry.  A sub-range of
// the positions may cut one more block than the full range has.
__global__ void k_wg_pools_pooled(int64_t E, int W, int64_t block_edges, uint32_t pool_size, uint32_t n_bins,
                                  uint32_t* __restrict__ wg_pool_begin, unsigned long long* __restrict__ total) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    const uint64_t n_blocks = (uint64_t)((E + block_edges - 1) / block_edges) + 1;
    const uint64_t per_block = (uint64_t)block_edges + pooled_side_records(block_edges) + pool_size;
    const uint64_t blocks = (n_blocks + W - 1) / W;   // blocks first + w, first + w + W, ...
    const uint64_t per_wg = blocks * per_block / kChunk + n_bins + 1;
    for (int w = 0; w <= W; ++w) wg_pool_begin[w] = (uint32_t)min(per_wg * (uint64_t)w, (uint64_t)0xFFFFFFFFull);
    *total = per_wg * (uint64_t)W;
}

// head[e] = row of CSR position e (one thread per row)
__global__ void __launch_bounds__(kBlock) k_edge_heads(const int32_t* __restrict__ row_ptr, int64_t n, int32_t* __restrict__ head) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) head[e] = (int32_t)i;
}

// ------------------------------------------------------------------ opt-in: gradient through the cell means
// mu_r = (1/n_r) sum_{l in r} theta_l.  d(n L)/d mu_r = |M| p_r sum_{i: r approximated for i} c_i q(theta_i, mu_r)^2
// (theta_i - mu_r) with c_i = sum_{e in row i} 2 p_e / S_e (Eq. 4 with Eq. 5 differentiated in mu_r), and every
// member of cell r receives 1/n_r of it.  Three steps: c_i from the edge pass's per-edge values (row order), the
// sum over heads for every cell (the mean-field pass with the roles of heads and cells exchanged), the per-cell
// vector that the tile pass adds to its points.

// c_i of the heads row_begin .. row_end-1: the row's values added in CSR order
__global__ void __launch_bounds__(kBlock) k_head_coefficients(const int32_t* __restrict__ row_ptr, const float* __restrict__ cS,
                                                             int64_t row_begin, int64_t row_end, float* __restrict__ chead) {
    const int64_t i = row_begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= row_end) return;
    float c = 0.f;
    for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) c += cS[e];
    chead[i] = c;
}

// 2^-24 fixed point for the per-cell sums (the sums over up to n heads can be large; what is left after the division
// by n_r is far below the gradient's resolution)
constexpr double kCellFixInv = 1.0 / 16777216.0;
__device__ __forceinline__ unsigned long long to_cell_fixed(float v) {
    const double d = fma((double)v, 16777216.0, 6755399441055744.0);
    return (unsigned long long)(__double_as_longlong(d) - 0x4338000000000000LL);
}

constexpr int kMeanGradHeads = 16384;   // heads per workgroup

// One lane per cell, the heads of the workgroup's chunk staged through LDS 256 at a time:
// Gfix[r] += sum_i [group(i) != group(r)] c_i q(theta_i, mu_r)^2 (theta_i - mu_r), in fixed point (order-independent).
__global__ void __launch_bounds__(kBlock) k_mean_gradient(const float2* __restrict__ theta, const float* __restrict__ chead,
                                                         const float4* __restrict__ hinfo, const float2* __restrict__ mu,
                                                         const int32_t* __restrict__ group_of_cluster, int32_t R, int64_t i_begin,
                                                         int64_t i_end, unsigned long long* __restrict__ Gfix) {
    __shared__ float4 heads[kBlock];   // (theta_i, c_i, group of i)
    const int32_t r = (int32_t)blockIdx.x * kBlock + threadIdx.x;
    const bool live = r < R;
    const float2 m = live ? mu[r] : make_float2(0.f, 0.f);
    const int32_t gr = live ? group_of_cluster[r] : -1;
    const int64_t h0 = i_begin + (int64_t)blockIdx.y * kMeanGradHeads, h1 = min(i_end, h0 + kMeanGradHeads);
    float Gx = 0.f, Gy = 0.f;
    for (int64_t b0 = h0; b0 < h1; b0 += kBlock) {
        __syncthreads();
        const int64_t i = b0 + threadIdx.x;
        float4 hd = make_float4(0.f, 0.f, 0.f, __int_as_float(-1));
        if (i < h1) {
            const float2 t = theta[i];
            hd = make_float4(t.x, t.y, chead[i], hinfo[i].w);
        }
        heads[threadIdx.x] = hd;
        __syncthreads();
        const int cnt = (int)min((int64_t)kBlock, h1 - b0);
        float sx = 0.f, sy = 0.f;   // folded into the totals every 256 heads to keep float32 round-off from growing
        for (int k = 0; k < cnt; ++k) {
            const float4 hk = heads[k];
            const float dx = hk.x - m.x, dy = hk.y - m.y;
            const float q = cauchy(dx, dy);
            const float w = (__float_as_int(hk.w) == gr) ? 0.f : hk.z * q * q;
            sx = fmaf(w, dx, sx);
            sy = fmaf(w, dy, sy);
        }
        Gx += sx;
        Gy += sy;
    }
    if (live && (Gx != 0.f || Gy != 0.f)) {
        atomicAdd(&Gfix[2 * r], to_cell_fixed(Gx));
        atomicAdd(&Gfix[2 * r + 1], to_cell_fixed(Gy));
    }
}

// gmean[r] = |M| p_r G_r / n_r: what every member of cell r adds to its gradient; the sums are cleared for the next use
__global__ void __launch_bounds__(kBlock) k_mean_gradient_finish(unsigned long long* __restrict__ Gfix, const uint32_t* __restrict__ counts,
                                                                int32_t R, double noise_over_n, float2* __restrict__ gmean) {
    const int32_t r = (int32_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const double gx = (double)(long long)Gfix[2 * r] * kCellFixInv, gy = (double)(long long)Gfix[2 * r + 1] * kCellFixInv;
    Gfix[2 * r] = 0ull;
    Gfix[2 * r + 1] = 0ull;
    // |M| p_r / n_r = |M| / n for every non-empty cell
    gmean[r] = counts[r] ? make_float2((float)(gx * noise_over_n), (float)(gy * noise_over_n)) : make_float2(0.f, 0.f);
}

// g_l += gmean[cell of l] (the scatter paths whose last kernel does not take the step itself)
__global__ void __launch_bounds__(kBlock) k_add_mean_gradient(float2* __restrict__ g, const int32_t* __restrict__ cluster_of,
                                                             const float2* __restrict__ gmean, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float2 m = gmean[cluster_of[i]];
    float2 v = g[i];
    v.x += m.x;
    v.y += m.y;
    g[i] = v;
}

// With `theta` given it also takes the SGD step of Section 3.4 for its points, theta <- theta - eta g (the
// edge pass that read theta has finished by then).
// An epoch's edge pass may run in phases over ranges of CSR positions, each followed by this kernel, so that the
// record pool holds one phase at a time: `carry` ([2 n] fixed-point sums) takes the tile's sums of every phase but the
// last (kPhaseFirst stores them, kPhaseMiddle adds them), and the last phase (kPhaseLast) adds what was carried before
// it goes on as the single-phase form (kPhaseOnly) does.  Integer sums: the result does not depend on the phases.
enum TilePhase { kPhaseOnly = 0, kPhaseFirst = 1, kPhaseMiddle = 2, kPhaseLast = 3 };

__global__ void __launch_bounds__(kBinBlock) k_tile_accumulate(const BinArgs Q, uint32_t n_wg, float2* __restrict__ g, int64_t n,
                                                              float2* __restrict__ theta, float eta,
                                                              const int32_t* __restrict__ cluster_of, const float2* __restrict__ gmean,
                                                              unsigned long long* __restrict__ carry, int phase) {
    extern __shared__ unsigned long long acc[];   // [2 << tile_bits]
    constexpr int kPerLane = kChunk / 64;         // records one lane takes from a full chunk
    const uint32_t b = blockIdx.x;
    const int tile = 1 << Q.tile_bits;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int l = threadIdx.x; l < 2 * tile; l += kBinBlock) acc[l] = 0ull;
    __syncthreads();
    // A wavefront walks the chains of kChains workgroups side by side: the loads of a step (next chunk ids and up to
    // kPerLane records per lane and chain) all go out before any is used, so the latency of following a chain is
    // paid once per step for all of them.  Chunk ids and fills are wave-uniform.
    constexpr int kChains = 8;
    for (uint32_t w0 = (uint32_t)wave * kChains; w0 < n_wg; w0 += (kBinBlock / 64) * kChains) {
        uint32_t ch[kChains], cnt[kChains];
#pragma unroll
        for (int k = 0; k < kChains; ++k) {
            const bool live = w0 + k < n_wg;
            ch[k] = live ? Q.chain_head[(size_t)b * n_wg + w0 + k] : kNoChunk;
            cnt[k] = live ? Q.chain_fill[(size_t)b * n_wg + w0 + k] : 0u;
            ch[k] = __builtin_amdgcn_readfirstlane(ch[k]);
            cnt[k] = __builtin_amdgcn_readfirstlane(cnt[k]);
        }
        bool any = true;
        while (any) {
            uint32_t prev[kChains];
            uint32_t rec[kChains][kPerLane][3];
#pragma unroll
            for (int k = 0; k < kChains; ++k) {
                prev[k] = kNoChunk;
                if (ch[k] != kNoChunk) {
                    prev[k] = Q.chunk_prev[ch[k]];
                    const uint32_t* src = Q.pool + (size_t)ch[k] * kChunk * 3;
#pragma unroll
                    for (int u = 0; u < kPerLane; ++u) {
                        const uint32_t r = (uint32_t)u * 64u + lane;
                        if (r < cnt[k]) { rec[k][u][0] = src[3 * r]; rec[k][u][1] = src[3 * r + 1]; rec[k][u][2] = src[3 * r + 2]; }
                    }
                }
            }
            any = false;
#pragma unroll
            for (int k = 0; k < kChains; ++k) {
                if (ch[k] != kNoChunk) {
#pragma unroll
                    for (int u = 0; u < kPerLane; ++u) {
                        const uint32_t r = (uint32_t)u * 64u + lane;
                        if (r < cnt[k]) {
                            const uint32_t ml = rec[k][u][0] & (uint32_t)(tile - 1);
                            atomicAdd(&acc[2 * ml], to_fixed(__uint_as_float(rec[k][u][1])));
                            atomicAdd(&acc[2 * ml + 1], to_fixed(__uint_as_float(rec[k][u][2])));
                        }
                    }
                    ch[k] = __builtin_amdgcn_readfirstlane(prev[k]);
                    cnt[k] = kChunk;
                    any = any || ch[k] != kNoChunk;
                }
            }
        }
    }
    __syncthreads();
    const int64_t p0 = (int64_t)b << Q.tile_bits;
    if (phase == kPhaseFirst || phase == kPhaseMiddle) {   // not the last phase of the step: carry the sums on
        for (int l = threadIdx.x; l < 2 * tile && 2 * p0 + l < 2 * n; l += kBinBlock) {
            const unsigned long long before = phase == kPhaseMiddle ? carry[2 * p0 + l] : 0ull;
            carry[2 * p0 + l] = before + acc[l];
        }
        return;
    }
    if (phase == kPhaseLast) {
        for (int l = threadIdx.x; l < 2 * tile && 2 * p0 + l < 2 * n; l += kBinBlock) acc[l] += carry[2 * p0 + l];
        __syncthreads();
    }
    for (int l = threadIdx.x; l < tile && p0 + l < n; l += kBinBlock) {
        const float2 hd = Q.ghead[p0 + l];
        Q.ghead[p0 + l] = make_float2(0.f, 0.f);   // consumed: rows that hand their head sum on as records rely on this
        float2 gi = make_float2((float)((double)hd.x + (double)(long long)acc[2 * l] * kFixInv),
                                (float)((double)hd.y + (double)(long long)acc[2 * l + 1] * kFixInv));
        if (gmean) {   // gradient through the means: every member's share of its cell's term
            const float2 gm = gmean[cluster_of[p0 + l]];
            gi.x += gm.x;
            gi.y += gm.y;
        }
        g[p0 + l] = gi;
        if (theta) {
            float2 t = theta[p0 + l];
            t.x = fmaf(-eta, gi.x, t.x);
            t.y = fmaf(-eta, gi.y, t.y);
            theta[p0 + l] = t;
        }
    }
}

// fixed-order sum of the per-block loss partials (one block)
__global__ void __launch_bounds__(kBlock) k_loss_finish(const double* __restrict__ partial, uint32_t count, double inv_n,
                                                        double* __restrict__ out) {
    __shared__ double sl[kBlock / 64];
    double acc = 0.0;
    for (uint32_t b = threadIdx.x; b < count; b += kBlock) acc += partial[b];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) sl[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kBlock / 64; ++w) t += sl[w];
        *out = t * inv_n;
    }
}

// ------------------------------------------------------------------ K4 (fallback): combine
// g = head sum + fixed-point sum of tail and negative forces; clears both for the next launch.
__global__ void __launch_bounds__(kBlock) k_combine_fixed(float2* __restrict__ ghead, unsigned long long* __restrict__ gfix,
                                                          float2* __restrict__ g, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float2 h = ghead[i];
    ghead[i] = make_float2(0.f, 0.f);   // consumed: a sub-step over other heads must not see this one again
    const double sx = (double)(long long)gfix[2 * i] * kFixInv, sy = (double)(long long)gfix[2 * i + 1] * kFixInv;
    gfix[2 * i] = 0ull;
    gfix[2 * i + 1] = 0ull;
    g[i] = make_float2((float)((double)h.x + sx), (float)((double)h.y + sy));
}

// ------------------------------------------------------------------ K5: SGD step (Section 3.4)
__global__ void __launch_bounds__(kBlock) k_update(float2* __restrict__ theta, const float2* __restrict__ g, float eta, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float2 t = theta[i];
    const float2 gi = g[i];
    t.x = fmaf(-eta, gi.x, t.x);
    t.y = fmaf(-eta, gi.y, t.y);
    theta[i] = t;
}

__global__ void __launch_bounds__(kBlock) k_zero_f2(float2* __restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = make_float2(0.f, 0.f);
}

__global__ void __launch_bounds__(kBlock) k_zero_u64(unsigned long long* __restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

// ------------------------------------------------------------------ test hook: negatives of an edge range
__global__ void __launch_bounds__(kBlock) k_negatives(const EdgeArgs P, int64_t e_begin, int64_t e_end, int32_t* __restrict__ out) {
    const int64_t e = e_begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= e_end) return;
    // head of e: last row whose offset is <= e
    int64_t lo = 0, hi = P.n;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)P.row_ptr[mid] <= e) lo = mid; else hi = mid;
    }
    const int64_t i = lo;
    Population pop;
    if (P.group_of_cluster && !P.far) {
        const int32_t gi = P.group_of_cluster[P.cluster_of[i]];
        pop.base = P.gbase[gi];
        pop.count = P.gcount[gi];
        pop.members = P.gmembers;
    } else {
        pop.base = 0;
        pop.count = (uint32_t)P.n;
        pop.members = nullptr;
    }
    for (int k = 0; k < P.s; ++k) out[(e - e_begin) * P.s + k] = negative_of_slot(P, pop, (int32_t)e, k);
}

}  // namespace nomad

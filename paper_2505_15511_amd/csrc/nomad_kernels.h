// Device kernels of libnomad for gfx950 (64-wide wavefronts).
//
// Notation follows the paper (arxiv 2505.15511): theta = embedding rows, q = Cauchy kernel
// (Eq. 1), ij = directed kNN edge with head i and tail j, m = sampled negative, mu_r / p_r = mean
// and mass of cell r, |M| = noise-sample count, s = negatives drawn per edge.
//
// Mapping: a *row group* of LPR adjacent lanes walks the CSR row of one head i, LPR edges at a
// time, so neighbour indices are read as contiguous 4*LPR-byte runs and consecutive row groups
// read consecutive runs.  Head-side sums are reduced inside the row group with a fixed xor
// butterfly, which makes them independent of scheduling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nomad {

constexpr int kBlock = 256;
// 64-bit fixed point used for order-independent accumulation of the negatives' gradient in
// deterministic mode: one unit = 2^-36.  Every single contribution is bounded by p(j|i) <= 1 in
// magnitude, so 2^27 contributions per point still fit.
constexpr float kFixScale = 68719476736.0f;          // 2^36
constexpr double kFixInv = 1.0 / 68719476736.0;

// ------------------------------------------------------------------ sampler
// Philox4x32 with 10 rounds (Salmon et al., SC'11): the counter-based generator behind the
// uniform noise distribution over tails (Section 3.3).  Counter = (edge lo, edge hi, epoch,
// slot block), key = the 64-bit seed.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

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
    kFlagAsymmetric = 6, // reverse edge missing or parallel edges
    kFlagCount = 8
};

__global__ void k_check_row_ptr(const int32_t* __restrict__ row_ptr, int64_t n, int* flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && row_ptr[0] != 0) flags[kFlagRowPtr] = 1;
    if (i < n && row_ptr[i + 1] < row_ptr[i]) flags[kFlagRowPtr] = 1;
}

// one thread per row: columns in range, no self loops; normalised weights p(j|i)
__global__ void k_check_rows(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                             const float* __restrict__ w, float* __restrict__ pe, int64_t n, int* flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t a = row_ptr[i], b = row_ptr[i + 1];
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
    atomicAdd(&counts[c], 1u);
    atomicMin(&first[c], (uint32_t)i);
    if (group_of_cluster) atomicMin(&gfirst[group_of_cluster[c]], (uint32_t)i);
    if (i > 0) {
        const int32_t p = cluster_of[i - 1];
        if (p >= 0 && p < R) {
            if (p != c) atomicAdd(&boundaries[0], 1ull);
            if (group_of_cluster && group_of_cluster[p] != group_of_cluster[c]) atomicAdd(&boundaries[1], 1ull);
        }
    }
}

// reverse-edge index: rev[e] = position of (j -> i) for e = (i -> j)
__global__ void k_build_rev(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col, int64_t n,
                            int32_t* __restrict__ rev, int* flags) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
        const int32_t j = col[e];
        int32_t found = -1, hits = 0;
        for (int32_t f = row_ptr[j]; f < row_ptr[j + 1]; ++f)
            if (col[f] == i) { if (found < 0) found = f; ++hits; }
        if (hits != 1) flags[kFlagAsymmetric] = 1;
        rev[e] = found < 0 ? e : found;
    }
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

// cinfo[r] = (mu_x, mu_y, p_r, group label as bits); one wavefront per cell
__global__ void __launch_bounds__(kBlock) k_mean_finish(const double2* __restrict__ partial,
                                                        const uint32_t* __restrict__ chunk_start,
                                                        const uint32_t* __restrict__ counts,
                                                        const int32_t* __restrict__ group_of_cluster, int32_t R, double inv_n,
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
        cinfo[r] = make_float4(mx, my, (float)((double)cnt * inv_n), __int_as_float(group_of_cluster ? group_of_cluster[r] : 0));
    }
}

// ------------------------------------------------------------------ K2: mean-field sums (Eq. 5)
// One lane per head; the cell table is read with wave-uniform addresses.  Partial sums are folded
// into the totals every 64 cells to keep float32 round-off from growing with |R|.
__global__ void __launch_bounds__(kBlock) k_mean_field(const float2* __restrict__ theta,
                                                       const int32_t* __restrict__ cluster_of,
                                                       const int32_t* __restrict__ group_of_cluster,
                                                       const float4* __restrict__ cinfo, int32_t R, int64_t n,
                                                       float* __restrict__ A, float2* __restrict__ B) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float2 ti = theta[i];
    const int32_t gi = group_of_cluster[cluster_of[i]];
    float At = 0.f, Bx = 0.f, By = 0.f;
    for (int32_t r0 = 0; r0 < R; r0 += 64) {
        float a = 0.f, bx = 0.f, by = 0.f;
        const int32_t r1 = min(R, r0 + 64);
        for (int32_t r = r0; r < r1; ++r) {
            const float4 c = cinfo[r];
            const float w = (__float_as_int(c.w) == gi) ? 0.0f : c.z;
            const float dx = ti.x - c.x, dy = ti.y - c.y;
            const float q = cauchy(dx, dy);
            const float wq = w * q;
            a += wq;
            const float wq2 = wq * q;
            bx = fmaf(wq2, dx, bx);
            by = fmaf(wq2, dy, by);
        }
        At += a; Bx += bx; By += by;
    }
    A[i] = At;
    B[i] = make_float2(Bx, By);
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
    const float* A;                // mean-field sums (grouped only)
    const float2* B;
    float noise_count;             // |M|
    float omega0;                  // single-group omega
    uint32_t key0, key1, epoch;
    int32_t s;
    int64_t n;
    uint32_t rows_per_xcd_span;    // for the block -> row remap
    // outputs
    float2* g;                     // atomic mode: accumulators of every force
    float2* ghead;                 // deterministic mode: head-side sums
    float* coef;                   // deterministic mode: a_e per edge
    unsigned long long* gfix;      // deterministic mode: fixed-point negative sums [n*2]
    double* loss_partial;          // loss mode: one partial per block
};

enum EdgeMode { kModeAtomic = 0, kModeDet = 1, kModeLoss = 2 };

// Blocks are handed to the 8 XCDs round-robin; giving XCD x the x-th contiguous eighth of the
// rows keeps each L2 on its own slice of theta and of the index stream.
__device__ __forceinline__ uint32_t xcd_contiguous_block(uint32_t b, uint32_t nblocks) {
    const uint32_t per = (nblocks + 7u) >> 3;
    return (b & 7u) * per + (b >> 3);
}

template <int S, int MODE, int LPR>
__global__ void __launch_bounds__(kBlock) k_edges(const EdgeArgs P) {
    constexpr int ROWS = kBlock / LPR;
    constexpr int SS = S > 0 ? S : 1;
    const uint32_t lb = xcd_contiguous_block(blockIdx.x, gridDim.x);
    const int64_t i = (int64_t)lb * ROWS + (threadIdx.x / LPR);
    const int lane = threadIdx.x % LPR;
    float hx = 0.f, hy = 0.f;
    double lsum = 0.0;
    if (i < P.n) {
        const int32_t ea = P.row_ptr[i], eb = P.row_ptr[i + 1];
        const float2 ti = P.theta[i];
        const float inv_deg = eb > ea ? 1.0f / (float)(eb - ea) : 0.f;
        Population pop;
        float omega, MA = 0.f, MBx = 0.f, MBy = 0.f;
        if (P.group_of_cluster) {
            const int32_t gi = P.group_of_cluster[P.cluster_of[i]];
            pop.base = P.gbase[gi];
            pop.count = P.gcount[gi];
            pop.members = P.gmembers;
            omega = P.gomega[gi];
            MA = P.noise_count * P.A[i];
            const float2 b = P.B[i];
            MBx = P.noise_count * b.x;
            MBy = P.noise_count * b.y;
        } else {
            pop.base = 0;
            pop.count = (uint32_t)P.n;
            pop.members = nullptr;
            omega = P.omega0;
        }
        const int32_t s = S > 0 ? S : P.s;
        for (int32_t e = ea + lane; e < eb; e += LPR) {
            const int32_t j = P.col[e];
            const float2 tj = P.theta[j];
            const float pe = P.pe ? P.pe[e] : inv_deg;
            const float dx = ti.x - tj.x, dy = ti.y - tj.y;
            const float qij = cauchy(dx, dy);
            int32_t m[SS];
            float ex[SS], ey[SS], qm[SS];
            float qsum = 0.f;
            if (S > 0) {
#pragma unroll
                for (int b = 0; b < (S + 3) / 4; ++b) {
                    uint32_t w[4];
                    philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)b, P.key0, P.key1, w);
#pragma unroll
                    for (int l = 0; l < 4; ++l)
                        if (4 * b + l < S) m[4 * b + l] = draw_index(w[l], pop);
                }
#pragma unroll
                for (int k = 0; k < S; ++k) {
                    const float2 tm = P.theta[m[k]];
                    ex[k] = ti.x - tm.x;
                    ey[k] = ti.y - tm.y;
                    qm[k] = cauchy(ex[k], ey[k]);
                    qsum += qm[k];
                }
            } else {
                for (int b = 0; 4 * b < s; ++b) {
                    uint32_t w[4];
                    philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)b, P.key0, P.key1, w);
                    for (int l = 0; l < 4 && 4 * b + l < s; ++l) {
                        const float2 tm = P.theta[draw_index(w[l], pop)];
                        qsum += cauchy(ti.x - tm.x, ti.y - tm.y);
                    }
                }
            }
            const float Se = qij + MA + omega * qsum;
            if (MODE == kModeLoss) {
                // -log q + log S = log(S (1 + d^2))
                lsum += (double)(pe * logf(Se / qij));
                continue;
            }
            const float inv_S = 1.0f / Se;
            const float a = 2.0f * pe * qij * (1.0f - qij * inv_S);
            float fx = a * dx, fy = a * dy;           // attraction on the head; the tail gets the opposite
            if (MODE == kModeAtomic) {
                unsafeAtomicAdd(&P.g[j].x, -fx);
                unsafeAtomicAdd(&P.g[j].y, -fy);
            } else {
                P.coef[e] = a;
            }
            const float bscale = 2.0f * pe * omega * inv_S;
            if (S > 0) {
#pragma unroll
                for (int k = 0; k < S; ++k) {
                    const float b = bscale * qm[k] * qm[k];
                    const float rx = b * ex[k], ry = b * ey[k];
                    fx -= rx;
                    fy -= ry;
                    if (MODE == kModeAtomic) {
                        unsafeAtomicAdd(&P.g[m[k]].x, rx);
                        unsafeAtomicAdd(&P.g[m[k]].y, ry);
                    } else {
                        atomicAdd(&P.gfix[2 * (int64_t)m[k]], (unsigned long long)__float2ll_rn(rx * kFixScale));
                        atomicAdd(&P.gfix[2 * (int64_t)m[k] + 1], (unsigned long long)__float2ll_rn(ry * kFixScale));
                    }
                }
            } else {
                for (int b = 0; 4 * b < s; ++b) {
                    uint32_t w[4];
                    philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)b, P.key0, P.key1, w);
                    for (int l = 0; l < 4 && 4 * b + l < s; ++l) {
                        const int32_t mk = draw_index(w[l], pop);
                        const float2 tm = P.theta[mk];
                        const float gx = ti.x - tm.x, gy = ti.y - tm.y;
                        const float q = cauchy(gx, gy);
                        const float bb = bscale * q * q;
                        const float rx = bb * gx, ry = bb * gy;
                        fx -= rx;
                        fy -= ry;
                        if (MODE == kModeAtomic) {
                            unsafeAtomicAdd(&P.g[mk].x, rx);
                            unsafeAtomicAdd(&P.g[mk].y, ry);
                        } else {
                            atomicAdd(&P.gfix[2 * (int64_t)mk], (unsigned long long)__float2ll_rn(rx * kFixScale));
                            atomicAdd(&P.gfix[2 * (int64_t)mk + 1], (unsigned long long)__float2ll_rn(ry * kFixScale));
                        }
                    }
                }
            }
            const float c = 2.0f * pe * inv_S;        // mean-field term: -2 p |M| B_i / S
            hx += fx - c * MBx;
            hy += fy - c * MBy;
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
    if (lane == 0 && i < P.n) {
        if (MODE == kModeAtomic) {
            unsafeAtomicAdd(&P.g[i].x, hx);
            unsafeAtomicAdd(&P.g[i].y, hy);
        } else {
            P.ghead[i] = make_float2(hx, hy);
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

// ------------------------------------------------------------------ K4: deterministic scatter
// g_j = head sum + sum over the row of j of a_{rev(e')} (theta_j - theta_{col(e')}) + negatives.
// The tail forces are *pulled*: the force edge (i -> j) puts on its tail j is read by row j through
// the reverse edge (j -> i), in CSR order, so the sum has one fixed order.  The negatives' sums
// arrive in 64-bit fixed point (integer addition is associative) and are cleared here for the
// next epoch.
template <int LPR>
__global__ void __launch_bounds__(kBlock) k_tail_pull(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                      const int32_t* __restrict__ rev, const float* __restrict__ coef,
                                                      const float2* __restrict__ theta, const float2* __restrict__ ghead,
                                                      unsigned long long* __restrict__ gfix, float2* __restrict__ g, int64_t n) {
    constexpr int ROWS = kBlock / LPR;
    const uint32_t lb = xcd_contiguous_block(blockIdx.x, gridDim.x);
    const int64_t j = (int64_t)lb * ROWS + (threadIdx.x / LPR);
    const int lane = threadIdx.x % LPR;
    float ax = 0.f, ay = 0.f;
    if (j < n) {
        const float2 tj = theta[j];
        for (int32_t e = row_ptr[j] + lane; e < row_ptr[j + 1]; e += LPR) {
            const float2 ti = theta[col[e]];
            const float a = coef[rev[e]];
            ax = fmaf(a, tj.x - ti.x, ax);
            ay = fmaf(a, tj.y - ti.y, ay);
        }
    }
    ax = rowgroup_sum<LPR>(ax);
    ay = rowgroup_sum<LPR>(ay);
    if (lane == 0 && j < n) {
        const float2 h = ghead[j];
        const double nx = (double)(long long)gfix[2 * j] * kFixInv;
        const double ny = (double)(long long)gfix[2 * j + 1] * kFixInv;
        gfix[2 * j] = 0ull;
        gfix[2 * j + 1] = 0ull;
        g[j] = make_float2((float)((double)h.x + (double)ax + nx), (float)((double)h.y + (double)ay + ny));
    }
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
    if (P.group_of_cluster) {
        const int32_t gi = P.group_of_cluster[P.cluster_of[i]];
        pop.base = P.gbase[gi];
        pop.count = P.gcount[gi];
        pop.members = P.gmembers;
    } else {
        pop.base = 0;
        pop.count = (uint32_t)P.n;
        pop.members = nullptr;
    }
    for (int b = 0; 4 * b < P.s; ++b) {
        uint32_t w[4];
        philox4x32_10((uint32_t)e, 0u, P.epoch, (uint32_t)b, P.key0, P.key1, w);
        for (int l = 0; l < 4 && 4 * b + l < P.s; ++l) out[(e - e_begin) * P.s + 4 * b + l] = draw_index(w[l], pop);
    }
}

}  // namespace nomad

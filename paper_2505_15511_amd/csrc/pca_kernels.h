// Device code of the PCA initialisation (Section 3.5: the projection starts from a PCA of the data).
//
//   mean        column sums in float64, a slab of rows per block, the slabs added in order
//   covariance  C = (1/n) sum_i (x_i - mean)(x_i - mean)^T: a dense contraction over the points, on the float64 matrix
//               cores (v_mfma_f64_16x16x4f64), one wavefront per 64x64 tile of C and slab of rows, slabs added in order
//   axes        the leading eigenvectors of C by subspace iteration with a Rayleigh-Ritz step per iteration: a block of
//               kRitz vectors, Z = C Q on the whole chip, the small dense algebra (projected eigenproblem by Jacobi
//               rotations, re-orthonormalisation by Gram-Schmidt twice) in one workgroup
//   scores      theta_i = ((x_i - mean) . axis_1, (x_i - mean) . axis_2), float64, oriented and scaled, rounded once
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nomad_pca {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int kMeanRows = 1024;   // rows per partial column sum
constexpr int kColBlock = 64;     // a wavefront's tile of C is kColBlock x kColBlock (4 x 4 matrix-core tiles)
constexpr int kRitz = 8;          // vectors iterated together (convergence goes with lambda_9 / lambda_2)
constexpr int kMaxDim = 768;      // rows of Q per thread of the single-workgroup step: kMaxDim / 256
constexpr int kRowsPerThread = kMaxDim / 256;

__global__ void __launch_bounds__(256) k_pca_colsum(const float* __restrict__ X, int64_t n, int32_t d, double* __restrict__ partial) {
    const int64_t r0 = (int64_t)blockIdx.x * kMeanRows, r1 = min(n, r0 + kMeanRows);
    for (int col = threadIdx.x; col < d; col += 256) {
        double s = 0.0;
        int64_t r = r0;
        for (; r + 16 <= r1; r += 16) {   // sixteen rows in flight; added in row order
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = X[(r + u) * d + col];
#pragma unroll
            for (int u = 0; u < 16; ++u) s += (double)v[u];
        }
        for (; r < r1; ++r) s += (double)X[r * d + col];
        partial[(int64_t)blockIdx.x * d + col] = s;
    }
}

__global__ void __launch_bounds__(256) k_pca_mean(const double* __restrict__ partial, int32_t blocks, int32_t d, int64_t n,
                                                  double* __restrict__ mean) {
    const int col = blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= d) return;
    double s = 0.0;
    int b = 0;
    for (; b + 16 <= blocks; b += 16) {   // sixteen partial sums in flight; added in block order
        double v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = partial[(int64_t)(b + u) * d + col];
#pragma unroll
        for (int u = 0; u < 16; ++u) s += v[u];
    }
    for (; b < blocks; ++b) s += partial[(int64_t)b * d + col];
    mean[col] = s / (double)n;
}

// column blocks (a, b), a <= b, of tile pair number `pair` when there are nb column blocks
__host__ __device__ inline void cov_pair(int pair, int nb, int& a, int& b) {
    a = 0;
    while (pair >= nb - a) { pair -= nb - a; ++a; }
    b = a + pair;
}

// One wavefront: tile pair blockIdx.x / slabs, rows slab * slab_rows ...  Operand layout of the 16x16x4 float64
// instruction: lane l supplies A[i = l % 16][k = l / 16] and B[k = l / 16][j = l % 16]; it receives D[i = l / 16 + 4 v][j = l % 16]
// in element v.  Here k runs over four consecutive rows of X, i and j over columns: D += Xc^T Xc.
__global__ void __launch_bounds__(64) k_pca_cov(const float* __restrict__ X, int64_t n, int32_t d, const double* __restrict__ mean,
                                                int32_t slabs, int64_t slab_rows, double* __restrict__ partial) {
    const int pair = blockIdx.x / slabs, slab = blockIdx.x % slabs;
    int a, b;
    cov_pair(pair, (d + kColBlock - 1) / kColBlock, a, b);
    const int lane = threadIdx.x, lr = lane >> 4, lc = lane & 15;
    int cola[4], colb[4];
    double ma[4], mb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        cola[u] = a * kColBlock + 16 * u + lc;
        colb[u] = b * kColBlock + 16 * u + lc;
        ma[u] = cola[u] < d ? mean[cola[u]] : 0.0;
        mb[u] = colb[u] < d ? mean[colb[u]] : 0.0;
    }
    doublex4 acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = doublex4{0.0, 0.0, 0.0, 0.0};
    const int64_t r0 = (int64_t)slab * slab_rows, r1 = min(n, r0 + slab_rows);
    // loads run kAhead steps (of four rows) ahead of the multiplications: a step is 16 matrix instructions, about half a
    // microsecond, and the rows come from HBM
    constexpr int kAhead = 4;
    float fa[kAhead][4], fb[kAhead][4];
    auto fetch = [&](int slot, int64_t r) {   // this lane's row of the step that starts at row r; NaN stands for "no such element"
        const int64_t row = r + lr;
        const bool rv = row < r1;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            fa[slot][u] = (rv && cola[u] < d) ? X[row * d + cola[u]] : __builtin_nanf("");
            fb[slot][u] = (rv && colb[u] < d) ? X[row * d + colb[u]] : __builtin_nanf("");
        }
    };
#pragma unroll
    for (int s = 0; s < kAhead; ++s) fetch(s, r0 + 4 * s);
    for (int64_t r = r0; r < r1; r += 4 * kAhead) {
#pragma unroll
        for (int s = 0; s < kAhead; ++s) {   // slot s holds the step at row r + 4 s
            double xa[4], xb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {   // an absent element contributes nothing
                xa[u] = fa[s][u] == fa[s][u] ? (double)fa[s][u] - ma[u] : 0.0;
                xb[u] = fb[s][u] == fb[s][u] ? (double)fb[s][u] - mb[u] : 0.0;
            }
            fetch(s, r + 4 * (s + kAhead));   // beyond the slab: all NaN, no memory access
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = __builtin_amdgcn_mfma_f64_16x16x4f64(xa[x], xb[y], acc[x][y], 0, 0, 0);
        }
    }
    double* out = partial + (int64_t)blockIdx.x * (kColBlock * kColBlock);
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int v = 0; v < 4; ++v) out[(16 * x + lr + 4 * v) * kColBlock + 16 * y + lc] = acc[x][y][v];
}

// C = (1/n) sum over the slabs, in slab order; both triangles written
__global__ void __launch_bounds__(256) k_pca_cov_reduce(const double* __restrict__ partial, int32_t n_pairs, int32_t slabs, int32_t d,
                                                        int64_t n, double* __restrict__ C) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x >= (int64_t)n_pairs * kColBlock * kColBlock) return;
    const int pair = (int)(x / (kColBlock * kColBlock)), e = (int)(x % (kColBlock * kColBlock));
    int a, b;
    cov_pair(pair, (d + kColBlock - 1) / kColBlock, a, b);
    const int gi = a * kColBlock + e / kColBlock, gj = b * kColBlock + e % kColBlock;
    if (gi >= d || gj >= d) return;
    double s = 0.0;
    const double* src = partial + (int64_t)pair * slabs * (kColBlock * kColBlock) + e;
    int sl = 0;
    for (; sl + 16 <= slabs; sl += 16) {   // sixteen partial tiles in flight; added in slab order
        double v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = src[(int64_t)(sl + u) * (kColBlock * kColBlock)];
#pragma unroll
        for (int u = 0; u < 16; ++u) s += v[u];
    }
    for (; sl < slabs; ++sl) s += src[(int64_t)sl * (kColBlock * kColBlock)];
    s /= (double)n;
    C[(int64_t)gi * d + gj] = s;
    if (a != b) C[(int64_t)gj * d + gi] = s;
}

// Z = C Q: one wavefront per row of C; Q and Z are [d][kRitz] row-major (columns >= p stay zero)
__global__ void __launch_bounds__(256) k_pca_apply(const double* __restrict__ C, const double* __restrict__ Q, int32_t d,
                                                   double* __restrict__ Z) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= d) return;
    double s[kRitz];
#pragma unroll
    for (int m = 0; m < kRitz; ++m) s[m] = 0.0;
    for (int col = lane; col < d; col += 64) {
        const double c = C[(int64_t)row * d + col];
#pragma unroll
        for (int m = 0; m < kRitz; ++m) s[m] = fma(c, Q[col * kRitz + m], s[m]);
    }
#pragma unroll
    for (int m = 0; m < kRitz; ++m)
        for (int w = 32; w > 0; w >>= 1) s[m] += __shfl_xor(s[m], w, 64);
    if (lane == 0)
#pragma unroll
        for (int m = 0; m < kRitz; ++m) Z[row * kRitz + m] = s[m];
}

// sums of COUNT per-thread values over the 256 threads of the workgroup, into out[0..COUNT) in LDS (COUNT <= 64)
template <int COUNT>
__device__ __forceinline__ void block_sums(const double (&v)[COUNT], double (*scratch)[64], double* out) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int c = 0; c < COUNT; ++c) {
        double s = v[c];
        for (int w = 32; w > 0; w >>= 1) s += __shfl_xor(s, w, 64);
        if (lane == 0) scratch[wave][c] = s;
    }
    __syncthreads();
    if ((int)threadIdx.x < COUNT) out[threadIdx.x] = scratch[0][threadIdx.x] + scratch[1][threadIdx.x] + scratch[2][threadIdx.x] + scratch[3][threadIdx.x];
    __syncthreads();
}

// Eigenpairs of the symmetric p x p matrix H (p <= kRitz) by cyclic Jacobi rotations, eigenvalues descending; one thread.
// W is orthogonal whatever the number of sweeps; lam and W are the eigenpairs to the accuracy the sweeps reached.
__device__ inline void jacobi_eigen(double (*H)[kRitz], int p, double (*W)[kRitz], double* lam) {
    for (int i = 0; i < kRitz; ++i)
        for (int j = 0; j < kRitz; ++j) W[i][j] = i == j ? 1.0 : 0.0;
    // Two sweeps per call are enough: the caller iterates, and its basis is nearly the Ritz basis from the second
    // call on (H nearly diagonal, where the rotations converge quadratically).  Rotations that would change nothing at
    // float64 resolution are skipped.
    for (int sweep = 0; sweep < 2; ++sweep) {
        bool rotated = false;
        for (int i = 0; i < p; ++i)
            for (int j = i + 1; j < p; ++j) {
                const double hij = H[i][j];
                if (hij * hij <= 1e-34 * fabs(H[i][i] * H[j][j]) || hij == 0.0) continue;
                rotated = true;
                const double theta = (H[j][j] - H[i][i]) / (2.0 * hij);
                const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                const double c = 1.0 / sqrt(t * t + 1.0), s = t * c;
                for (int k = 0; k < p; ++k) {   // H <- H J
                    const double hki = H[k][i], hkj = H[k][j];
                    H[k][i] = c * hki - s * hkj;
                    H[k][j] = s * hki + c * hkj;
                }
                for (int k = 0; k < p; ++k) {   // H <- J^T H
                    const double hik = H[i][k], hjk = H[j][k];
                    H[i][k] = c * hik - s * hjk;
                    H[j][k] = s * hik + c * hjk;
                }
                for (int k = 0; k < p; ++k) {   // W <- W J
                    const double wki = W[k][i], wkj = W[k][j];
                    W[k][i] = c * wki - s * wkj;
                    W[k][j] = s * wki + c * wkj;
                }
            }
        if (!rotated) break;
    }
    for (int i = 0; i < p; ++i) lam[i] = H[i][i];
    for (int i = 0; i < p; ++i) {   // selection sort, descending
        int best = i;
        for (int j = i + 1; j < p; ++j)
            if (lam[j] > lam[best]) best = j;
        if (best != i) {
            const double t = lam[i]; lam[i] = lam[best]; lam[best] = t;
            for (int k = 0; k < p; ++k) { const double w = W[k][i]; W[k][i] = W[k][best]; W[k][best] = w; }
        }
    }
    for (int i = p; i < kRitz; ++i) lam[i] = 0.0;
}

// One Rayleigh-Ritz step in one workgroup.  In: Q [d][kRitz] (orthonormal columns, or any start block) and Z = C Q.
// H = Q^T Z, H = W diag(lam) W^T; Ritz vectors Q W with images Z W; residual = max over the first two pairs of
// |Z w - lam Q w| / lam_1; the next Q = the orthonormalised Z W (Gram-Schmidt, every column projected twice; a column
// that vanishes -- C of lower rank than the block -- is replaced by a coordinate vector).
// Znext = C^s Q for some s >= 1 (Z itself when s = 1): the next basis is the orthonormalised Znext W, s power steps at once.
__global__ void __launch_bounds__(256) k_pca_ritz(double* __restrict__ Q, const double* __restrict__ Z, const double* __restrict__ Znext,
                                                  int32_t d, int32_t p, double* __restrict__ lam_out, double* __restrict__ resid_out) {
    __shared__ double scratch[4][64];
    __shared__ double sums[64];
    __shared__ double H[kRitz][kRitz], W[kRitz][kRitz], lam[kRitz];
    const int tid = threadIdx.x;
    double q[kRowsPerThread][kRitz], z[kRowsPerThread][kRitz];
#pragma unroll
    for (int x = 0; x < kRowsPerThread; ++x) {
        const int row = tid + 256 * x;
#pragma unroll
        for (int m = 0; m < kRitz; ++m) {
            q[x][m] = row < d ? Q[row * kRitz + m] : 0.0;
            z[x][m] = row < d ? Z[row * kRitz + m] : 0.0;
        }
    }
    {
        double h[kRitz * kRitz];
#pragma unroll
        for (int a = 0; a < kRitz; ++a)
#pragma unroll
            for (int b = 0; b < kRitz; ++b) {
                double s = 0.0;
#pragma unroll
                for (int x = 0; x < kRowsPerThread; ++x) s = fma(q[x][a], z[x][b], s);
                h[a * kRitz + b] = s;
            }
        block_sums<kRitz * kRitz>(h, scratch, sums);
    }
    if (tid == 0) {
        for (int a = 0; a < kRitz; ++a)
            for (int b = 0; b < kRitz; ++b) H[a][b] = 0.5 * (sums[a * kRitz + b] + sums[b * kRitz + a]);
        jacobi_eigen(H, p, W, lam);
    }
    __syncthreads();
    // Ritz vectors and their images
    double rq[kRowsPerThread][kRitz], rz[kRowsPerThread][kRitz];
#pragma unroll
    for (int x = 0; x < kRowsPerThread; ++x)
#pragma unroll
        for (int m = 0; m < kRitz; ++m) {
            double sq = 0.0, sz = 0.0;
#pragma unroll
            for (int a = 0; a < kRitz; ++a) {
                sq = fma(q[x][a], W[a][m], sq);
                sz = fma(z[x][a], W[a][m], sz);
            }
            rq[x][m] = sq;
            rz[x][m] = sz;
        }
    {
        double r[2] = {0.0, 0.0};
#pragma unroll
        for (int x = 0; x < kRowsPerThread; ++x)
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const double e = rz[x][m] - lam[m] * rq[x][m];
                r[m] = fma(e, e, r[m]);
            }
        block_sums<2>(r, scratch, sums);
        if (tid == 0) {
            const double worst = sqrt(fmax(sums[0], sums[1]));
            resid_out[0] = lam[0] > 0.0 ? worst / lam[0] : 0.0;
            for (int m = 0; m < kRitz; ++m) lam_out[m] = lam[m];
        }
    }
    if (Znext != Z) {
#pragma unroll
        for (int x = 0; x < kRowsPerThread; ++x) {
            const int row = tid + 256 * x;
#pragma unroll
            for (int m = 0; m < kRitz; ++m) z[x][m] = row < d ? Znext[row * kRitz + m] : 0.0;
#pragma unroll
            for (int m = 0; m < kRitz; ++m) {
                double sz = 0.0;
#pragma unroll
                for (int a = 0; a < kRitz; ++a) sz = fma(z[x][a], W[a][m], sz);
                rz[x][m] = sz;
            }
        }
    }
    // the next basis: orthonormalise the images column by column (q is reused for the finished columns)
#pragma unroll
    for (int m = 0; m < kRitz; ++m) {
        if (m >= p) {
#pragma unroll
            for (int x = 0; x < kRowsPerThread; ++x) q[x][m] = 0.0;
            continue;
        }
        double v[kRowsPerThread];
#pragma unroll
        for (int x = 0; x < kRowsPerThread; ++x) v[x] = rz[x][m];   // by now: column m of Znext W
        for (int attempt = 0; attempt < 4; ++attempt) {
            double before[1] = {0.0};
#pragma unroll
            for (int x = 0; x < kRowsPerThread; ++x) before[0] = fma(v[x], v[x], before[0]);
            block_sums<1>(before, scratch, sums);
            const double norm_before = sums[0];
            __syncthreads();
            for (int pass = 0; pass < 2; ++pass) {
                double dots[kRitz];
#pragma unroll
                for (int j = 0; j < kRitz; ++j) {
                    double s = 0.0;
                    if (j < m)
#pragma unroll
                        for (int x = 0; x < kRowsPerThread; ++x) s = fma(v[x], q[x][j], s);
                    dots[j] = s;
                }
                block_sums<kRitz>(dots, scratch, sums);
#pragma unroll
                for (int j = 0; j < kRitz; ++j)
                    if (j < m)
#pragma unroll
                        for (int x = 0; x < kRowsPerThread; ++x) v[x] = fma(-sums[j], q[x][j], v[x]);
                __syncthreads();
            }
            double after[1] = {0.0};
#pragma unroll
            for (int x = 0; x < kRowsPerThread; ++x) after[0] = fma(v[x], v[x], after[0]);
            block_sums<1>(after, scratch, sums);
            const double norm_after = sums[0];
            __syncthreads();
            if (norm_after > 1e-24 * norm_before && norm_after > 0.0) {
                const double inv = 1.0 / sqrt(norm_after);
#pragma unroll
                for (int x = 0; x < kRowsPerThread; ++x) q[x][m] = v[x] * inv;
                break;
            }
            // nothing left of this column: start again from a coordinate vector
            const int unit = (m * 37 + attempt * 101) % d;
#pragma unroll
            for (int x = 0; x < kRowsPerThread; ++x) {
                v[x] = (tid + 256 * x) == unit ? 1.0 : 0.0;
                q[x][m] = 0.0;
            }
        }
    }
#pragma unroll
    for (int x = 0; x < kRowsPerThread; ++x) {
        const int row = tid + 256 * x;
        if (row < d)
#pragma unroll
            for (int m = 0; m < kRitz; ++m) Q[row * kRitz + m] = q[x][m];
    }
}

// factor[m] for m = 0, 1: the sign that makes the axis' entry of largest magnitude (the first among equals) positive,
// times std0 / sqrt(lam_1) when std0 > 0.  One thread.
__global__ void k_pca_orient(const double* __restrict__ Q, int32_t d, const double* __restrict__ lam, float std0, double* __restrict__ factor) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const double scale = std0 > 0.f ? (double)std0 / sqrt(lam[0]) : 1.0;
    for (int m = 0; m < 2; ++m) {
        int best = 0;
        for (int r = 1; r < d; ++r)
            if (fabs(Q[r * kRitz + m]) > fabs(Q[best * kRitz + m])) best = r;
        factor[m] = (Q[best * kRitz + m] > 0.0 ? 1.0 : -1.0) * scale;
    }
}

// theta_i = factor * ((x_i - mean) . axis_1, (x_i - mean) . axis_2): a wavefront per row, kProjectRows rows in turn
constexpr int kProjectRows = 16;
__global__ void __launch_bounds__(256) k_pca_project(const float* __restrict__ X, int64_t n, int32_t d, const double* __restrict__ mean,
                                                     const double* __restrict__ Q, const double* __restrict__ factor,
                                                     float2* __restrict__ theta) {
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const double f0 = factor[0], f1 = factor[1];
    for (int x = 0; x < kProjectRows; x += 4) {   // four rows at a time: their loads are in flight together
        const int64_t row0 = w * kProjectRows + x;
        if (row0 >= n) return;
        double s0[4] = {0.0, 0.0, 0.0, 0.0}, s1[4] = {0.0, 0.0, 0.0, 0.0};
        for (int col = lane; col < d; col += 64) {
            const double m = mean[col], q0 = Q[col * kRitz], q1 = Q[col * kRitz + 1];
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = row0 + u < n ? X[(row0 + u) * d + col] : 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const double c = (double)v[u] - m;
                s0[u] = fma(c, q0, s0[u]);
                s1[u] = fma(c, q1, s1[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            for (int o = 32; o > 0; o >>= 1) {
                s0[u] += __shfl_xor(s0[u], o, 64);
                s1[u] += __shfl_xor(s1[u], o, 64);
            }
            if (lane == 0 && row0 + u < n) theta[row0 + u] = make_float2((float)(s0[u] * f0), (float)(s1[u] * f1));
        }
    }
}

}  // namespace nomad_pca

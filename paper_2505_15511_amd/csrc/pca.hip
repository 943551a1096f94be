// libnomad: the PCA initialisation behind the C ABI of include/nomad.h (host side).
#include <hip/hip_runtime.h>

#include <cmath>
#include <random>
#include <vector>

#include "host_util.h"
#include "nomad.h"
#include "pca_kernels.h"

using namespace nomad_pca;

#pragma GCC visibility push(default)
extern "C" int nomad_pca_init(const float* X, int64_t n, int32_t d, float std0, float* theta_out, double* stats, int mem, int32_t device,
                              void* stream) {
    if (!X || !theta_out || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return NOMAD_E_INVALID_ARG;
    if (n < 2 || d < 2 || d > kMaxDim || device < 0 || !(std0 == std0)) return NOMAD_E_INVALID_ARG;
    if (n >= ((int64_t)1 << 31) - 256) return NOMAD_E_TOO_LARGE;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return NOMAD_E_HIP;
    KTRY(hipSetDevice(device));
    hipStream_t st = (hipStream_t)stream;
    Buffers buf;
    const float* dX = X;
    float* dTheta = theta_out;
    if (mem == NOMAD_HOST) {
        float *x = nullptr, *t = nullptr;
        KTRY(buf.alloc(&x, (size_t)n * d));
        KTRY(buf.alloc(&t, (size_t)n * 2));
        KTRY(hipMemcpyAsync(x, X, sizeof(float) * (size_t)n * d, hipMemcpyHostToDevice, st));
        dX = x; dTheta = t;
    }
    const int32_t p = std::min<int32_t>(kRitz, d);
    // mean
    const int32_t mean_blocks = (int32_t)blocks_of(n, kMeanRows);
    double *mean_partial = nullptr, *mean = nullptr;
    KTRY(buf.alloc(&mean_partial, (size_t)mean_blocks * d));
    KTRY(buf.alloc(&mean, (size_t)d));
    hipLaunchKernelGGL(k_pca_colsum, dim3((uint32_t)mean_blocks), dim3(256), 0, st, dX, n, d, mean_partial);
    hipLaunchKernelGGL(k_pca_mean, dim3(blocks_of(d, 256)), dim3(256), 0, st, (const double*)mean_partial, mean_blocks, d, n, mean);
    // covariance: enough (tile pair, slab) wavefronts to fill the chip, slabs of at least 256 rows
    const int32_t nb = (d + kColBlock - 1) / kColBlock, n_pairs = nb * (nb + 1) / 2;
    int64_t slabs64 = std::max<int64_t>(1, (2048 + n_pairs - 1) / n_pairs);
    slabs64 = std::min<int64_t>(slabs64, (n + 255) / 256);
    const int64_t slab_rows = (((n + slabs64 - 1) / slabs64) + 3) / 4 * 4;
    const int32_t slabs = (int32_t)((n + slab_rows - 1) / slab_rows);
    double *cov_partial = nullptr, *Cm = nullptr;
    KTRY(buf.alloc(&cov_partial, (size_t)n_pairs * slabs * kColBlock * kColBlock));
    KTRY(buf.alloc(&Cm, (size_t)d * d));
    hipLaunchKernelGGL(k_pca_cov, dim3((uint32_t)(n_pairs * slabs)), dim3(64), 0, st, dX, n, d, (const double*)mean, slabs, slab_rows, cov_partial);
    hipLaunchKernelGGL(k_pca_cov_reduce, dim3(blocks_of((int64_t)n_pairs * kColBlock * kColBlock, 256)), dim3(256), 0, st,
                       (const double*)cov_partial, n_pairs, slabs, d, n, Cm);
    // leading eigenvectors: subspace iteration from a fixed pseudo-random block
    double *Q = nullptr, *Z = nullptr, *Z2 = nullptr, *Z3 = nullptr, *lam = nullptr, *resid = nullptr, *factor = nullptr;
    KTRY(buf.alloc(&Q, (size_t)d * kRitz));
    KTRY(buf.alloc(&Z, (size_t)d * kRitz));
    KTRY(buf.alloc(&Z2, (size_t)d * kRitz));
    KTRY(buf.alloc(&Z3, (size_t)d * kRitz));
    KTRY(buf.alloc(&lam, (size_t)kRitz));
    KTRY(buf.alloc(&resid, 1));
    KTRY(buf.alloc(&factor, 2));
    std::vector<double> hQ((size_t)d * kRitz, 0.0);
    std::mt19937_64 gen(0x6e6f6d6164ULL);
    for (int32_t r = 0; r < d; ++r)
        for (int32_t m = 0; m < p; ++m) hQ[(size_t)r * kRitz + m] = (double)(gen() >> 11) * (2.0 / 9007199254740992.0) - 1.0;
    KTRY(hipMemcpyAsync(Q, hQ.data(), sizeof(double) * hQ.size(), hipMemcpyHostToDevice, st));
    // kPower applications of C per Rayleigh-Ritz step (that step is one workgroup, an application the whole chip).  Started
    // from Ritz vectors, column m picks up the directions before it only at rounding level times (lambda_1 / lambda_m)^kPower,
    // which Gram-Schmidt applied twice removes again.
    constexpr int kPower = 4;
    const double tol = 1e-12;
    const int max_iters = 2000, check_every = 4;
    int iters = 0;
    double hresid = 1.0, hlam[kRitz] = {0};
    while (iters < max_iters) {
        for (int x = 0; x < check_every; ++x) {
            hipLaunchKernelGGL(k_pca_apply, dim3(blocks_of(d, 4)), dim3(256), 0, st, (const double*)Cm, (const double*)Q, d, Z);
            double *from = Z, *to = Z2;
            for (int s = 1; s < kPower; ++s) {
                hipLaunchKernelGGL(k_pca_apply, dim3(blocks_of(d, 4)), dim3(256), 0, st, (const double*)Cm, (const double*)from, d, to);
                from = to;
                to = to == Z2 ? Z3 : Z2;
            }
            hipLaunchKernelGGL(k_pca_ritz, dim3(1), dim3(256), 0, st, Q, (const double*)Z, (const double*)from, d, p, lam, resid);
        }
        iters += check_every;
        KTRY(hipMemcpyAsync(&hresid, resid, sizeof(double), hipMemcpyDeviceToHost, st));
        KTRY(hipStreamSynchronize(st));
        if (!(hresid > tol)) break;
    }
    KTRY(hipMemcpyAsync(hlam, lam, sizeof(hlam), hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (std0 > 0.f && !(hlam[0] > 0.0)) return NOMAD_E_INVALID_ARG;   // no variance to scale
    // scores
    hipLaunchKernelGGL(k_pca_orient, dim3(1), dim3(64), 0, st, (const double*)Q, d, (const double*)lam, std0, factor);
    hipLaunchKernelGGL(k_pca_project, dim3(blocks_of(n, 4 * kProjectRows)), dim3(256), 0, st, dX, n, d, (const double*)mean, (const double*)Q,
                       (const double*)factor, (float2*)dTheta);
    KTRY(hipGetLastError());
    if (mem == NOMAD_HOST) KTRY(hipMemcpyAsync(theta_out, dTheta, sizeof(float) * (size_t)n * 2, hipMemcpyDeviceToHost, st));
    KTRY(hipStreamSynchronize(st));
    if (stats) {
        stats[0] = hlam[0];
        stats[1] = hlam[1];
        stats[2] = hresid;
        stats[3] = (double)iters;
    }
    return NOMAD_OK;
}
#pragma GCC visibility pop

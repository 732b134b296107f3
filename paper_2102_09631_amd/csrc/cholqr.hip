// Tall-skinny orthonormalisation of the h x r iterate by CholeskyQR2.
// The iterate is held transposed (Yt: r x h, row j = column j of Y), so the
// Gram matrix is S[i][j] = sum_k Yt[i][k] Yt[j][k].  One round is
//   S = Y^T Y  ->  S = R^T R (upper R)  ->  Y <- Y R^{-1},
// done twice.  The r x r factorisation runs in fp64 inside one workgroup's LDS.
#include "dad_internal.h"

namespace dad {

constexpr int GRAM_COLS = 256;  // columns of Yt per workgroup of the Gram kernel

// gram_part[b][i*r+j] = sum over this block's columns of Yt[i][k]*Yt[j][k]
// Products of two fp32 values are exact in fp64, so the Gram matrix carries no rounding beyond the
// final sums; CholeskyQR then tolerates condition numbers far beyond the fp32 limit of ~4e3.
__global__ __launch_bounds__(256) void k_gram_partial(const float* __restrict__ Yt, double* __restrict__ gram_part,
                                                      int64_t h, int r) {
    constexpr int KC = 64;
    __shared__ float Ys[DAD_MAX_RANK][KC + 1];
    const int t = threadIdx.x;
    const int64_t kbeg = (int64_t)blockIdx.x * GRAM_COLS;
    const int64_t kend = (kbeg + GRAM_COLS < h) ? kbeg + GRAM_COLS : h;
    const int nent = r * r;
    double acc[DAD_MAX_RANK * DAD_MAX_RANK / 256];
#pragma unroll
    for (int m = 0; m < DAD_MAX_RANK * DAD_MAX_RANK / 256; ++m) acc[m] = 0.0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += KC) {
        for (int e = t; e < r * KC; e += 256) {
            int i = e / KC, kk = e % KC;
            int64_t k = k0 + kk;
            Ys[i][kk] = (k < kend) ? Yt[(int64_t)i * h + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < DAD_MAX_RANK * DAD_MAX_RANK / 256; ++m) {
            int e = t + 256 * m;
            if (e < nent) {
                int i = e / r, j = e % r;
                double a = acc[m];
#pragma unroll 16
                for (int kk = 0; kk < KC; ++kk) a = fma((double)Ys[i][kk], (double)Ys[j][kk], a);
                acc[m] = a;
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int m = 0; m < DAD_MAX_RANK * DAD_MAX_RANK / 256; ++m) {
        int e = t + 256 * m;
        if (e < nent) gram_part[(int64_t)blockIdx.x * nent + e] = acc[m];
    }
}

// One workgroup: S = sum_b gram_part[b] (fp64, b ascending), S = R^T R, rinv = R^{-1} (upper, fp32 out).
// A pivot that is not > 0 (or is NaN) latches *flag = 1 and is replaced by 1 so the kernel still
// finishes with finite arithmetic; the outputs are then meaningless.
__global__ __launch_bounds__(256) void k_chol_rinv(const double* __restrict__ gram_part, int nblocks,
                                                   float* __restrict__ rinv, int r, int* __restrict__ flag) {
    __shared__ double S[DAD_MAX_RANK][DAD_MAX_RANK + 1];  // upper: R; strict lower [j][i]: Rinv[i][j]
    __shared__ double dinv[DAD_MAX_RANK];                 // Rinv[j][j]
    const int t = threadIdx.x;
    const int nent = r * r;
    for (int e = t; e < nent; e += 256) {
        double a = 0.0;
        for (int b = 0; b < nblocks; ++b) a += gram_part[(int64_t)b * nent + e];
        S[e / r][e % r] = a;
    }
    __syncthreads();
    for (int k = 0; k < r; ++k) {
        double piv = S[k][k];
        __syncthreads();
        if (!(piv > 0.0)) {
            if (t == 0) *flag = 1;
            piv = 1.0;
        }
        const double d = sqrt(piv);
        if (t == 0) S[k][k] = d;
        for (int j = k + 1 + t; j < r; j += 256) S[k][j] = S[k][j] / d;
        __syncthreads();
        const int m = r - k - 1;  // trailing block, upper part only
        for (int e = t; e < m * m; e += 256) {
            int i = k + 1 + e / m, j = k + 1 + e % m;
            if (i <= j) S[i][j] -= S[k][i] * S[k][j];
        }
        __syncthreads();
    }
    // Back substitution, one column of R^{-1} per thread.
    if (t < r) {
        const int j = t;
        const double djj = 1.0 / S[j][j];
        dinv[j] = djj;
        for (int i = j - 1; i >= 0; --i) {
            double a = S[i][j] * djj;  // k = j term: R[i][j] * Rinv[j][j]
            for (int k = i + 1; k < j; ++k) a += S[i][k] * S[j][k];  // Rinv[k][j] lives at S[j][k]
            S[j][i] = -a / S[i][i];
        }
    }
    __syncthreads();
    for (int e = t; e < nent; e += 256) {
        int i = e / r, j = e % r;
        double v = (i == j) ? dinv[j] : (i < j ? S[j][i] : 0.0);
        rinv[e] = (float)v;
    }
}

// Gt[j][k] = sum_{i<=j} rinv[i][j] * Yt[i][k]   (Y <- Y R^{-1}); Gt may alias Yt.
__global__ __launch_bounds__(256) void k_apply_rinv(const float* Yt, float* Gt, const float* __restrict__ rinv,
                                                    int64_t h, int r) {
    constexpr int KC = 64;
    __shared__ float Ys[DAD_MAX_RANK][KC + 1];
    __shared__ float Rs[DAD_MAX_RANK][DAD_MAX_RANK + 1];
    const int t = threadIdx.x;
    const int kl = t & 63, jg = t >> 6;
    const int64_t k0 = (int64_t)blockIdx.x * KC;
    for (int e = t; e < r * KC; e += 256) {
        int i = e / KC, kk = e % KC;
        Ys[i][kk] = (k0 + kk < h) ? Yt[(int64_t)i * h + k0 + kk] : 0.f;
    }
    for (int e = t; e < r * r; e += 256) Rs[e / r][e % r] = rinv[e];
    __syncthreads();
    const int64_t k = k0 + kl;
    for (int j = jg; j < r; j += 4) {
        float a = 0.f;
        for (int i = 0; i <= j; ++i) a = fmaf(Rs[i][j], Ys[i][kl], a);
        if (k < h) Gt[(int64_t)j * h + k] = a;
    }
}

dad_status launch_cholqr2(const float* Yt, float* Gt, int64_t h, int r, double* gram_part, int gram_blocks,
                          float* rinv, int* flag, hipStream_t s) {
    const float* src = Yt;
    for (int round = 0; round < 2; ++round) {
        hipLaunchKernelGGL(k_gram_partial, dim3((unsigned)gram_blocks), dim3(256), 0, s, src, gram_part, h, r);
        DAD_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_chol_rinv, dim3(1), dim3(256), 0, s, (const double*)gram_part, gram_blocks, rinv, r, flag);
        DAD_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_apply_rinv, dim3((unsigned)ceil_div(h, 64)), dim3(256), 0, s, src, Gt, (const float*)rinv,
                           h, r);
        DAD_LAUNCH_CHECK();
        src = Gt;
    }
    return DAD_OK;
}

int gram_blocks_for(int64_t h) { return (int)ceil_div(h, GRAM_COLS); }

}  // namespace dad

// Cholesky factorisation and inverse of an r x r Gram matrix (r <= DAD_MAX_RANK) by one workgroup
// of 256 threads, shared by the orthonormalisation kernels.
#pragma once

#include "dad_internal.h"

namespace dad {

struct FactorShared {
    double colS[2][2][DAD_MAX_RANK];  // columns k, k+1 of the running S, double buffered over steps
    double rowT[2][2][DAD_MAX_RANK];  // rows k, k+1 of the running inverse
};

// Sums `nblocks` r x r fp64 partials (block order ascending) and factorises the sum:
// S = L L^T and X = L^{-1} by one right-looking sweep over k in fp64 registers.  Threads form a
// 16 x 16 grid (ti, tj); thread (ti, tj) owns the entries (ti + 16a, tj + 16b), a, b < NA, of every
// r x r matrix (NA = 2 covers r <= 32, NA = 4 r <= 64).  Pivot k needs column k of the running S
// and row k of the running inverse T (T starts as I), published through LDS; then
//     L[i][k] = S[i][k] / sqrt(S[k][k]),  X[k][j] = T[k][j] / sqrt(S[k][k]),
//     S[i][j] -= L[i][k] L[j][k],         T[i][j] -= L[i][k] X[k][j]      for i > k.
// R^{-1} = X^T (upper triangular, row-major r x r) is written in the type RT.  A pivot that is not
// > 0 (or NaN) latches *flag and is replaced by 1 so the sweep still ends with finite arithmetic.
// piv_range, when given, receives two doubles:
//   [0] the smallest pivot (square of a diagonal entry of R), 0 after a breakdown;
//   [1] trace(S) * ||R^{-1}||_F^2 / r^2 = (||R||_F ||R^{-1}||_F / r)^2, which is 1 for a factorised
//       iterate with orthogonal columns of equal length and bounds its squared condition number
//       from ABOVE (cond_2(Y)^2 = cond_2(R)^2 <= ||R||_F^2 ||R^{-1}||_F^2); +inf after a breakdown.
//       (The ratio of the pivots would only bound it from below: a unit-diagonal R with large
//       entries above the diagonal has equal pivots and a condition number that grows like 2^r.)
// Every thread of the workgroup must call it; the caller synchronises before `f` is reused.
template <int NA, typename RT>
__device__ __forceinline__ void factor_partials(FactorShared& f, const double* __restrict__ gram_part, int nblocks, int r,
                                                RT* __restrict__ rinv, int* __restrict__ flag,
                                                double* __restrict__ piv_range = nullptr) {
    const int t = threadIdx.x, ti = t >> 4, tj = t & 15;
    const int nent = r * r;
    double S[NA][NA], T[NA][NA];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < NA; ++b) {
            S[a][b] = 0.0;
            T[a][b] = (ti + 16 * a == tj + 16 * b) ? 1.0 : 0.0;
        }
    constexpr int NB = NA == 2 ? 8 : 4;  // partials in flight per thread
    for (int b0 = 0; b0 < nblocks; b0 += NB) {
        double v[NB][NA][NA];
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int b = 0; b < NA; ++b) {
                    const int i = ti + 16 * a, j = tj + 16 * b;
                    v[u][a][b] = (b0 + u < nblocks && i < r && j < r)
                                     ? __builtin_nontemporal_load(gram_part + (int64_t)(b0 + u) * nent + i * r + j)
                                     : 0.0;
                }
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int b = 0; b < NA; ++b) S[a][b] += v[u][a][b];
    }
    // identity beyond r keeps the padded rows and columns inert
    double tr_part = 0.0, xsq_part = 0.0;  // this thread's share of trace(S) and of ||R^{-1}||_F^2
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < NA; ++b) {
            const int i = ti + 16 * a, j = tj + 16 * b;
            if (i >= r || j >= r) S[a][b] = (i == j) ? 1.0 : 0.0;
            else if (i == j) tr_part += S[a][b];
        }

    // Two pivots per step: columns k, k+1 of S and rows k, k+1 of T are published together and every
    // thread redoes the small update of the second by the first (same operations, in the same order,
    // as two single steps), which halves the number of barriers on this serial path.  For odd r the
    // last step's second pivot is the inert identity padding.
    bool bad = false;
    double pmin = 1.7976931348623157e308, pmax = 0.0;
    for (int k = 0; k < r; k += 2) {
        const int buf = (k >> 1) & 1, ka = k >> 4, kt = k & 15;
        if (tj == kt || tj == kt + 1) {
            const int which = tj - kt;
#pragma unroll
            for (int b = 0; b < NA; ++b)
                if (b == ka) {
#pragma unroll
                    for (int a = 0; a < NA; ++a) f.colS[buf][which][ti + 16 * a] = S[a][b];
                }
        }
        if (ti == kt || ti == kt + 1) {
            const int which = ti - kt;
#pragma unroll
            for (int a = 0; a < NA; ++a)
                if (a == ka) {
#pragma unroll
                    for (int b = 0; b < NA; ++b) f.rowT[buf][which][tj + 16 * b] = T[a][b];
                }
        }
        __syncthreads();
        const double* c0 = f.colS[buf][0];
        const double* c1 = f.colS[buf][1];
        const double* t0 = f.rowT[buf][0];
        const double* t1 = f.rowT[buf][1];
        // every LDS operand of the step is read up front and pinned, so that the reads are issued
        // together and waited for once instead of one at a time inside the selects below
        double piv0 = c0[k], ck1 = c0[k + 1], piv1 = c1[k + 1];
        double ci0[NA], ci1[NA], cj0[NA], cj1[NA], tj0[NA], tj1[NA];
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            ci0[a] = c0[ti + 16 * a];
            ci1[a] = c1[ti + 16 * a];
            cj0[a] = c0[tj + 16 * a];
            cj1[a] = c1[tj + 16 * a];
            tj0[a] = t0[tj + 16 * a];
            tj1[a] = t1[tj + 16 * a];
        }
        asm volatile("" : "+v"(piv0), "+v"(ck1), "+v"(piv1));
#pragma unroll
        for (int a = 0; a < NA; ++a)
            asm volatile("" : "+v"(ci0[a]), "+v"(ci1[a]), "+v"(cj0[a]), "+v"(cj1[a]), "+v"(tj0[a]), "+v"(tj1[a]));
        if (!(piv0 > 0.0)) {
            bad = true;
            piv0 = 1.0;
        }
        pmin = piv0 < pmin ? piv0 : pmin;
        pmax = piv0 > pmax ? piv0 : pmax;
        const double d0 = rsqrt(piv0);
        const double m = ck1 * d0;  // L[k+1][k]
        piv1 = fma(-m, m, piv1);
        if (!(piv1 > 0.0)) {
            bad = true;
            piv1 = 1.0;
        }
        if (k + 1 < r) {  // not the inert padding of an odd r
            pmin = piv1 < pmin ? piv1 : pmin;
            pmax = piv1 > pmax ? piv1 : pmax;
        }
        const double d1 = rsqrt(piv1);
        double l0[NA], l1[NA], lt0[NA], lt1[NA], x0[NA], x1[NA];
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            const int i = ti + 16 * a;
            const double v0 = ci0[a] * d0;
            const double v1 = fma(-v0, m, ci1[a]) * d1;
            l0[a] = (i > k) ? v0 : 0.0;
            l1[a] = (i > k + 1) ? v1 : 0.0;
            lt0[a] = cj0[a] * d0;
            lt1[a] = fma(-lt0[a], m, cj1[a]) * d1;
            x0[a] = tj0[a] * d0;
            x1[a] = fma(-m, x0[a], tj1[a]) * d1;
        }
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < NA; ++b) {
                S[a][b] = fma(-l1[a], lt1[b], fma(-l0[a], lt0[b], S[a][b]));
                T[a][b] = fma(-l1[a], x1[b], fma(-l0[a], x0[b], T[a][b]));
            }
        if (ti == kt) {  // R^{-1}[j][k] = X[k][j]
#pragma unroll
            for (int b = 0; b < NA; ++b) {
                const int j = tj + 16 * b;
                if (j < r) {
                    rinv[j * r + k] = (RT)x0[b];
                    xsq_part += x0[b] * x0[b];
                    if (k + 1 < r) {
                        rinv[j * r + k + 1] = (RT)x1[b];
                        xsq_part += x1[b] * x1[b];
                    }
                }
            }
        }
    }
    if (bad && t == 0) *flag = 1;
    if (piv_range) {  // uniform over the workgroup
        __syncthreads();  // the last step's reads of the published columns and rows are done
        double* tr_s = &f.colS[0][0][0];  // 256 doubles each
        double* xs_s = &f.rowT[0][0][0];
        tr_s[t] = tr_part;
        xs_s[t] = xsq_part;
        __syncthreads();
        if (t < 64) {
            double tr = (tr_s[t] + tr_s[t + 64]) + (tr_s[t + 128] + tr_s[t + 192]);
            double xs = (xs_s[t] + xs_s[t + 64]) + (xs_s[t + 128] + xs_s[t + 192]);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                tr += __shfl_down(tr, o, 64);
                xs += __shfl_down(xs, o, 64);
            }
            if (t == 0) {
                piv_range[0] = bad ? 0.0 : pmin;  // a breakdown reads as infinitely ill conditioned
                piv_range[1] = bad ? __builtin_huge_val() : tr * xs / ((double)r * (double)r);
            }
        }
    }
    (void)pmax;
}

}  // namespace dad

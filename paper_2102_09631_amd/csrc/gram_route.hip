// Rank-r compression for few rows (N <= DAD_GRAM_MAX_ROWS): the association Algorithm 2 prints,
// with C = A A^T formed once (Algorithm 2, precomputation; Eq. 6), taken one step further by also
// forming E = Delta Delta^T, so that the whole block power iteration runs on N x N and N x r
// matrices and each factor is read twice (once for its Gram matrix, once for the result) instead
// of 2 n_iter + 1 times.  With M = A^T Delta and every iterate written as G_k = Delta^T T_k:
//     H0 = Delta G0                                   (N x r)
//     Z_1 = C H0,  Z_k = C (E T_{k-1})                Y_k = M^T M G_{k-1} = Delta^T Z_k
//     Y_k^T Y_k = Z_k^T E Z_k = R^T R,  T_k = Z_k R^{-1}      (Cholesky QR in the row space)
//     Gt = T_n^T Delta,   Pt = (E T_n)^T A.
// The span of the iterate, hence Pt^T Gt, is that of dad_compress_rank; the arithmetic between the
// two passes over the factors is fp64 (products of fp32 values are exact in fp64, so C and E carry
// no rounding beyond their final sums).  Launches:
//   k_gram_tiles   64 x 64 tiles of C and of [Delta; G0][Delta; G0]^T (upper triangle of tiles),
//                  split over the columns, fp64 matrix instruction
//   k_gram_gather  sums the column splits in a fixed order, mirrors, and files E and H0
//   k_ns_step      CV: Z = (C F) R^-1 | EZ: F = E Z, Gram, last workgroup factorises |
//                  REFINE: second Cholesky round in place for the returned iterate, a hand-over
//                  of the first factor when its pivots are within 1e6 of each other |
//                  APPLY: fp32 T = Z R^-1, V = F R^-1
//   k_ns_project   Gt = T^T Delta and Pt = V^T A, one 16-column strip per workgroup
#include "chol_factor.h"
#include "dad_internal.h"

namespace dad {

typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int GT = 64;        // tile edge of the Gram kernel
constexpr int GK = 64;        // columns per LDS stage
constexpr int GLD = GK + 4;   // LDS pitch in floats: rows land 4 banks apart, 16 rows x 4 columns conflict free

// ------------------------------------------------------------------------------------ Gram tiles

// Number of tile pairs (ti <= tj) of an nt x nt tile grid, and the pair with a given index.
static inline int tri_count(int nt) { return nt * (nt + 1) / 2; }
__device__ __forceinline__ void tri_decode(int id, int nt, int& ti, int& tj) {
    ti = 0;
    while (id >= nt - ti) {
        id -= nt - ti;
        ++ti;
    }
    tj = ti + id;
}

// Thread t's 16 entries (row t / 4, columns 16 (t % 4) ..) of the 64 x 64 block at rows row0..,
// columns k0.. of the virtual matrix [X; aug] (X: N x h of T, aug: naug x h fp32; rows beyond both
// and columns from kend on read as zero), as fp32 in registers.
template <typename T>
__device__ __forceinline__ void load_rows(float (&v)[16], const T* __restrict__ X, const float* __restrict__ aug,
                                          int64_t N, int naug, int64_t h, int64_t row0, int64_t k0, int64_t kend,
                                          bool vec) {
    const int t = threadIdx.x, row = t >> 2, seg = (t & 3) * 16;
    const int64_t gi = row0 + row, k = k0 + seg;
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = 0.f;
    if (gi < N) {
        const T* p = X + gi * h + k;
        if (vec && k + 16 <= kend) {
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 x = reinterpret_cast<const float4*>(p)[q];
                    v[4 * q] = x.x, v[4 * q + 1] = x.y, v[4 * q + 2] = x.z, v[4 * q + 3] = x.w;
                }
            } else {
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const uint4 x = reinterpret_cast<const uint4*>(p)[q];
                    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[8 * q + 2 * e] = __uint_as_float(w[e] << 16);
                        v[8 * q + 2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (k + i < kend) v[i] = ld<T>(p, i);
        }
    } else if (gi < N + naug) {
        const float* p = aug + (gi - N) * h + k;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (k + i < kend) v[i] = p[i];
    }
}

__device__ __forceinline__ void store_rows(float (*Xs)[GLD], const float (&v)[16]) {
    const int t = threadIdx.x, row = t >> 2, seg = (t & 3) * 16;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(&Xs[row][seg + 4 * q]) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}

struct GramJobs {
    int jobsC, jobsE;      // tile pairs of C (nt x nt tiles) and of the augmented E (nta x nta)
    int nt, nta;
    int splitsC, splitsE;  // column chunks per tile pair
    int64_t ck;            // columns per chunk (multiple of GK)
};

// One workgroup = one tile pair x one column chunk.  Wave w owns the 32 x 32 quarter (w / 2, w % 2)
// of the tile as 2 x 2 blocks of the 16x16x4 fp64 matrix instruction: lane l supplies row l % 16 of
// a block at column 4 kk + l / 16; result element v of lane l is entry (4 v + l / 16, l % 16).
template <typename T>
__global__ __launch_bounds__(256) void k_gram_tiles(const T* __restrict__ A, const T* __restrict__ D,
                                                    const float* __restrict__ G0, int64_t N, int64_t h_in, int64_t h_out,
                                                    int r, GramJobs J, double* __restrict__ part, int vecA, int vecD,
                                                    int* __restrict__ hdr) {
    __shared__ float Is[GT][GLD];
    __shared__ float Js[GT][GLD];
    if (blockIdx.x == 0 && threadIdx.x < 64) hdr[threadIdx.x] = 0;  // flag and ticket of this call
    int b = blockIdx.x;
    const bool isC = b < J.jobsC * J.splitsC;
    const T* X;
    int64_t h;
    int naug, ti, tj, split;
    bool vec;
    if (isC) {
        tri_decode(b / J.splitsC, J.nt, ti, tj);
        split = b % J.splitsC;
        X = A, h = h_in, naug = 0, vec = vecA;
    } else {
        const int e = b - J.jobsC * J.splitsC;
        tri_decode(e / J.splitsE, J.nta, ti, tj);
        split = e % J.splitsE;
        X = D, h = h_out, naug = r, vec = vecD;
    }
    const int64_t kbeg = (int64_t)split * J.ck;
    const int64_t kend = kbeg + J.ck < h ? kbeg + J.ck : h;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wr = 32 * (wave >> 1), wc = 32 * (wave & 1), li = lane & 15, lk = lane >> 4;
    f64x4 acc[2][2];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q) acc[p][q] = f64x4{0.0, 0.0, 0.0, 0.0};
    // a diagonal pair multiplies one block of rows by itself; the next stage's loads are in flight
    // while the current one is multiplied
    const bool diag = ti == tj;
    const float (*Jp)[GLD] = diag ? Is : Js;
    float vi[16], vj[16];
    load_rows<T>(vi, X, G0, N, naug, h, (int64_t)ti * GT, kbeg, kend, vec);
    if (!diag) load_rows<T>(vj, X, G0, N, naug, h, (int64_t)tj * GT, kbeg, kend, vec);
    for (int64_t k0 = kbeg; k0 < kend; k0 += GK) {
        __syncthreads();
        store_rows(Is, vi);
        if (!diag) store_rows(Js, vj);
        __syncthreads();
        if (k0 + GK < kend) {
            load_rows<T>(vi, X, G0, N, naug, h, (int64_t)ti * GT, k0 + GK, kend, vec);
            if (!diag) load_rows<T>(vj, X, G0, N, naug, h, (int64_t)tj * GT, k0 + GK, kend, vec);
        }
#pragma unroll 4
        for (int kk = 0; kk < GK / 4; ++kk) {
            const double a0 = (double)Is[wr + li][4 * kk + lk], a1 = (double)Is[wr + 16 + li][4 * kk + lk];
            const double b0 = (double)Jp[wc + li][4 * kk + lk], b1 = (double)Jp[wc + 16 + li][4 * kk + lk];
            acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
        }
    }
    double* out = part + (int64_t)b * (GT * GT);
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int v = 0; v < 4; ++v) out[(wr + 16 * p + 4 * v + lk) * GT + wc + 16 * q + li] = acc[p][q][v];
}

// Four workgroups per tile pair: entry (i, j) of the pair = sum of its column splits (ascending),
// filed at (i, j) and, off the diagonal tiles, at (j, i).  Of the augmented matrix the N x N corner
// is E and the N x r border H0 = Delta G0; the r x r corner is not needed.
__global__ __launch_bounds__(256) void k_gram_gather(const double* __restrict__ part, GramJobs J, int64_t N, int r,
                                                     double* __restrict__ C, double* __restrict__ E,
                                                     double* __restrict__ H0) {
    const int job = blockIdx.x >> 2, quarter = blockIdx.x & 3;
    const bool isC = job < J.jobsC;
    int ti, tj, splits;
    const double* src;
    if (isC) {
        tri_decode(job, J.nt, ti, tj);
        splits = J.splitsC;
        src = part + (int64_t)job * splits * (GT * GT);
    } else {
        tri_decode(job - J.jobsC, J.nta, ti, tj);
        splits = J.splitsE;
        src = part + ((int64_t)J.jobsC * J.splitsC + (int64_t)(job - J.jobsC) * splits) * (GT * GT);
    }
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int e = quarter * 1024 + m * 256 + threadIdx.x;
        double s = 0.0;
        for (int q0 = 0; q0 < splits; q0 += 8) {  // eight loads in flight, summed in ascending order
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {  // always a valid address, so that no load waits on a branch
                const int q = q0 + u < splits ? q0 + u : splits - 1;
                v[u] = __builtin_nontemporal_load(src + (int64_t)q * (GT * GT) + e);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) s += q0 + u < splits ? v[u] : 0.0;
        }
        const int64_t i = (int64_t)ti * GT + e / GT, j = (int64_t)tj * GT + e % GT;
        if (isC) {
            if (i < N && j < N) {
                C[i * N + j] = s;
                if (ti != tj) C[j * N + i] = s;
            }
        } else if (i < N) {
            if (j < N) {
                E[i * N + j] = s;
                if (ti != tj) E[j * N + i] = s;
            } else if (j < N + r) {
                H0[i * r + (j - N)] = s;
            }
        }
    }
}

// ------------------------------------------------------------------------------------ row-space steps

enum { NS_CV = 0, NS_EZ = 1, NS_REFINE = 2, NS_APPLY = 3 };

constexpr int NS_ROWS = 16;   // rows of the N x r matrices per workgroup
constexpr int NS_IN = 8192;   // entries of the right operand per LDS stage (NS_IN / (16 NA) rows)
constexpr int NS_LD = DAD_MAX_RANK + 1;
// Largest (||R||_F ||R^-1||_F / r)^2 of the first factor, an upper bound of cond(Y)^2, up to which one
// round is taken to be enough: the orthonormality error of one fp64 round is about 1e-16 cond(Y)^2.
constexpr double NS_REFINE_SPREAD = 1e6;

// Lives in dynamic LDS (about 100 KB).  The product phase and the phases after it never overlap in
// time, so they share storage.
template <int NA>
struct NsShared {
    static constexpr int CH = NS_IN / (16 * NA);  // rows of the right operand per stage: 256 or 128
    union {
        struct {
            double In[NS_IN];             // CH rows x r of the right operand, as in memory
            double Ss[NS_ROWS][CH + 1];   // 16 rows x CH columns of the symmetric matrix
        } m;
        struct {
            double Zs[NS_ROWS][NS_LD];
            double Fs[NS_ROWS][NS_LD];
            FactorShared f;
        } g;
    };
    double Rs[16 * NA][16 * NA + 1];  // R^-1 (upper triangular; the zeros below the diagonal are stored)
    int last;
};

// out[col] = sum_{i <= col} tile[row][i] * R^-1[i][col] for the NA columns this thread owns; eight
// terms are read from LDS together (the index is clamped; terms beyond the column are masked).
template <int NA>
__device__ __forceinline__ void tri_apply(const double (*tile)[NS_LD], const double (*Rs)[16 * NA + 1], int row, int cg,
                                          int r, double (&out)[NA]) {
#pragma unroll
    for (int b = 0; b < NA; ++b) {
        const int col = cg + 16 * b;
        double s0 = 0.0, s1 = 0.0;
        if (col < r) {
            for (int i0 = 0; i0 <= col; i0 += 8) {
                double a[8], c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = i0 + u <= col ? i0 + u : col;
                    a[u] = tile[row][i];
                    c[u] = Rs[i][col];
                }
#pragma unroll
                for (int u = 0; u < 8; u += 2) {
                    s0 = fma(i0 + u <= col ? a[u] : 0.0, c[u], s0);
                    s1 = fma(i0 + u + 1 <= col ? a[u + 1] : 0.0, c[u + 1], s1);
                }
            }
        }
        out[b] = s0 + s1;
    }
}

// Workgroup g handles rows [16 g, 16 g + 16) of the N x r matrices; thread (row = t / 16, cg = t % 16)
// owns columns cg + 16 b, b < NA.
//   NS_CV      Z = (S In) Rin^-1        S = C, In = previous F (or H0 with rin == nullptr: identity)
//   NS_EZ      F = S Z                  S = E; then Gram partial Z^T F, last workgroup -> rout
//   NS_REFINE  Z <- Z Rin^-1, F <- F Rin^-1 in place; Gram partial of the result -> rout
//   NS_APPLY   Tf = Z Rin^-1, Vf = F Rin^-1 as fp32 with row pitch `pitch` (columns r.. zero)
// The product streams S and In through LDS in stages of CH rows; the loads of the next stage are
// in flight while the current one is multiplied.
template <int NA, int MODE>
__global__ __launch_bounds__(256) void k_ns_step(const double* __restrict__ S, const double* In, double* Z, double* F,
                                                 const double* __restrict__ rin, double* __restrict__ rout,
                                                 float* __restrict__ Tf, float* __restrict__ Vf, int pitch, int64_t N,
                                                 int r, double* __restrict__ gram_part, int* __restrict__ counter,
                                                 int* __restrict__ flag, double* __restrict__ piv_range) {
    extern __shared__ __attribute__((aligned(16))) char ns_smem[];
    NsShared<NA>& sh = *reinterpret_cast<NsShared<NA>*>(ns_smem);
    constexpr int CH = NsShared<NA>::CH;
    const int t = threadIdx.x, row = t >> 4, cg = t & 15;
    const int64_t g0 = (int64_t)blockIdx.x * NS_ROWS, gi = g0 + row;
    const bool live = gi < N;
    if (MODE == NS_REFINE) {
        // The first round reports an upper bound of the iterate's squared condition number; when it is
        // small the first factor already orthonormalises to fp32 accuracy and more, and the second
        // round reduces to handing that factor on.
        if (piv_range[0] > 0.0 && piv_range[1] <= NS_REFINE_SPREAD) {
            if (blockIdx.x == 0)
                for (int e = t; e < r * r; e += 256) rout[e] = rin[e];
            return;
        }
    }
    // R^-1 travels global -> registers now (clamped addresses, so that the loads go out together)
    // and registers -> LDS just before the barrier in front of its first use.
    double rv[NA * NA];
    const bool use_r = MODE != NS_EZ && rin != nullptr;
    if (use_r) {
#pragma unroll
        for (int m = 0; m < NA * NA; ++m) rv[m] = rin[t + 256 * m < r * r ? t + 256 * m : r * r - 1];
    }
    auto store_r = [&]() {
        if (!use_r) return;
#pragma unroll
        for (int m = 0; m < NA * NA; ++m) {
            const int e = t + 256 * m, i = e / r, j = e % r;
            if (e < r * r) sh.Rs[i][j] = rv[m];
        }
    };
    double acc[NA];
#pragma unroll
    for (int b = 0; b < NA; ++b) acc[b] = 0.0;
    double zown[NA];  // this thread's entries of Z (all modes but NS_CV)
    if (MODE != NS_CV) {
#pragma unroll
        for (int b = 0; b < NA; ++b) {
            const double v = Z[(live ? gi : N - 1) * r + (cg + 16 * b < r ? cg + 16 * b : r - 1)];
            zown[b] = (live && cg + 16 * b < r) ? v : 0.0;
        }
    }
    if (MODE == NS_CV || MODE == NS_EZ) {
        const double* src = MODE == NS_CV ? In : Z;
        const int64_t total = N * r;
        typedef double f64x2 __attribute__((ext_vector_type(2)));
        constexpr int NI = NS_IN / 512;  // pairs of right-operand entries per thread and stage
        constexpr int NSS = CH / 16;     // entries of S per thread and stage
        f64x2 pin[NI];
        double ps[NSS];
        // Every load has a valid (clamped) address and its value is selected only when it is written
        // to LDS a stage later: a load under a branch, or a select right behind it, would be waited
        // for before the next load is issued.
        const int64_t lastpair = total >= 2 ? ((total - 2) & ~(int64_t)1) : 0;  // the buffer is padded to 256 B
        double tail = 0.0;
        auto fetch = [&](int64_t n0) {
            tail = src[total - 1];
#pragma unroll
            for (int m = 0; m < NI; ++m) {
                const int64_t idx = n0 * r + 2 * (t + 256 * m);  // even: CH is even, and src is 16-byte aligned
                pin[m] = *reinterpret_cast<const f64x2*>(src + (idx < lastpair ? idx : lastpair));
            }
#pragma unroll
            for (int m = 0; m < NSS; ++m) {
                const int e = t + 256 * m, rr = e / CH, cc = e % CH;
                const int64_t gr = g0 + rr < N ? g0 + rr : N - 1, gc = n0 + cc < N ? n0 + cc : N - 1;
                ps[m] = S[gr * N + gc];
            }
        };
        auto commit = [&](int64_t n0) {
#pragma unroll
            for (int m = 0; m < NI; ++m) {
                const int e = 2 * (t + 256 * m);
                const int64_t idx = n0 * r + e;
                f64x2 v = {0.0, 0.0};
                if (e < CH * r) {
                    if (idx + 1 < total)
                        v = pin[m];
                    else if (idx < total)
                        v.x = tail;
                }
                *reinterpret_cast<f64x2*>(&sh.m.In[e]) = v;
            }
#pragma unroll
            for (int m = 0; m < NSS; ++m) {
                const int e = t + 256 * m, rr = e / CH, cc = e % CH;
                sh.m.Ss[rr][cc] = (g0 + rr < N && n0 + cc < N) ? ps[m] : 0.0;
            }
        };
        constexpr int LC = 4 * NA, TR = NA;  // lanes along the columns; rows per lane
        const int lane = t & 63, wave = t >> 6, tc = lane % LC, tr = lane / LC;
        int pcol[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) pcol[j] = tc + LC * j < r ? tc + LC * j : 0;  // columns from r on are not kept
        double pacc[TR][4];
#pragma unroll
        for (int a = 0; a < TR; ++a)
#pragma unroll
            for (int j = 0; j < 4; ++j) pacc[a][j] = 0.0;
        fetch(0);
        for (int64_t n0 = 0; n0 < N; n0 += CH) {
            __syncthreads();
            commit(n0);
            __syncthreads();
            if (n0 + CH < N) fetch(n0 + CH);
            // LDS bandwidth bounds this product, so each lane owns a TR x 4 block of the 16 x r result
            // (TR + 4 reads for 4 TR multiply-adds) and the four waves split the rows of the stage.
            const int64_t rest = N - n0;
            const int nlim = rest < CH ? (int)((rest + 15) & ~(int64_t)15) : CH;  // rows beyond N hold zeros
            const int per = nlim / 4;
            for (int n = wave * per; n < (wave + 1) * per; n += 4) {
                double c[4][TR], v[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
#pragma unroll
                    for (int a = 0; a < TR; ++a) c[u][a] = sh.m.Ss[TR * tr + a][n + u];
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[u][j] = sh.m.In[(n + u) * r + pcol[j]];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int a = 0; a < TR; ++a)
#pragma unroll
                        for (int j = 0; j < 4; ++j) pacc[a][j] = fma(c[u][a], v[u][j], pacc[a][j]);
            }
        }
        __syncthreads();  // the product's LDS is free from here on
        // the four waves' partial sums meet in LDS and are added in wave order
        double (*red)[NS_ROWS][NS_LD] = reinterpret_cast<double (*)[NS_ROWS][NS_LD]>(sh.m.In);
#pragma unroll
        for (int a = 0; a < TR; ++a)
#pragma unroll
            for (int j = 0; j < 4; ++j) red[wave][TR * tr + a][tc + LC * j] = pacc[a][j];
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NA; ++b) {
            const int col = cg + 16 * b;
            acc[b] = ((red[0][row][col] + red[1][row][col]) + red[2][row][col]) + red[3][row][col];
        }
        __syncthreads();
    }
    if (MODE == NS_CV) {
        if (rin) {
#pragma unroll
            for (int b = 0; b < NA; ++b) sh.g.Zs[row][cg + 16 * b] = acc[b];
            store_r();
            __syncthreads();
            tri_apply<NA>(sh.g.Zs, sh.Rs, row, cg, r, acc);
        }
        if (live) {
#pragma unroll
            for (int b = 0; b < NA; ++b)
                if (cg + 16 * b < r) Z[gi * r + cg + 16 * b] = acc[b];
        }
        return;
    }
    // the three other modes work on this workgroup's rows of Z and F
#pragma unroll
    for (int b = 0; b < NA; ++b) {
        const int col = cg + 16 * b;
        const bool in = live && col < r;
        sh.g.Zs[row][col] = zown[b];
        double fv = 0.0;
        if (MODE != NS_EZ) fv = F[(live ? gi : N - 1) * r + (col < r ? col : r - 1)];
        sh.g.Fs[row][col] = in ? (MODE == NS_EZ ? acc[b] : fv) : 0.0;
        if (MODE == NS_EZ && in) F[gi * r + col] = acc[b];
    }
    store_r();
    __syncthreads();
    if (MODE == NS_REFINE || MODE == NS_APPLY) {
        double z[NA], f[NA];
        tri_apply<NA>(sh.g.Zs, sh.Rs, row, cg, r, z);
        tri_apply<NA>(sh.g.Fs, sh.Rs, row, cg, r, f);
        if (MODE == NS_APPLY) {
            if (live) {
#pragma unroll
                for (int b = 0; b < NA; ++b)
                    if (cg + 16 * b < pitch) {  // tri_apply leaves zero in the columns from r on
                        Tf[gi * pitch + cg + 16 * b] = (float)z[b];
                        Vf[gi * pitch + cg + 16 * b] = (float)f[b];
                    }
            }
            return;
        }
        __syncthreads();
#pragma unroll
        for (int b = 0; b < NA; ++b) {
            const int col = cg + 16 * b;
            sh.g.Zs[row][col] = z[b];  // zero outside the live rows and columns
            sh.g.Fs[row][col] = f[b];
            if (live && col < r) {
                Z[gi * r + col] = z[b];
                F[gi * r + col] = f[b];
            }
        }
        __syncthreads();
    }
    // Gram partial of these 16 rows: thread (ti, tj) owns entries (ti + 16 a, tj + 16 b) of Z^T F
    {
        const int ti = row, tj = cg;
        double* mine = gram_part + (int64_t)blockIdx.x * r * r;
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < NA; ++b) {
                const int i = ti + 16 * a, j = tj + 16 * b;
                if (i < r && j < r) {
                    double s = 0.0;
#pragma unroll
                    for (int n = 0; n < NS_ROWS; ++n) s = fma(sh.g.Zs[n][i], sh.g.Fs[n][j], s);
                    mine[i * r + j] = s;
                }
            }
    }
    __threadfence();
    __syncthreads();
    if (t == 0) sh.last = (atomicAdd(counter, 1) == (int)gridDim.x - 1);
    __syncthreads();
    if (!sh.last) return;
    __threadfence();
    factor_partials<NA, double>(sh.g.f, gram_part, (int)gridDim.x, r, rout, flag, piv_range);
    if (t == 0) *counter = 0;
}

// ------------------------------------------------------------------------------------ projection

constexpr int PJ_COLS = 16;       // columns per workgroup
constexpr int PJ_STAGE = 8192;    // floats of W per LDS stage (PJ_STAGE / RP rows)

// out_t[j][c] = sum_n W[n][j] X[n][c] for one 16-column strip of X (N x h of T); W is N x RP fp32
// (columns r.. are zero).  Strips [0, strips_in) belong to (A, Vf) -> Pt, the rest to (Delta, Tf)
// -> Gt.  Thread (rg = t / 16, col = t % 16) takes the rows rg, rg + 16, ... with RP accumulators:
// narrow strips give a few hundred workgroups, and a wave reads four rows of W per LDS access.
// The 16 row groups are summed in a fixed order (8..15 onto 0..7, then 0..7 in sequence).
template <typename T, int RP>
__global__ __launch_bounds__(256) void k_ns_project(const T* __restrict__ A, const T* __restrict__ D,
                                                    const float* __restrict__ Vf, const float* __restrict__ Tf,
                                                    float* __restrict__ Pt, float* __restrict__ Gt, int64_t N,
                                                    int64_t h_in, int64_t h_out, int r, int strips_in) {
    constexpr int SR = PJ_STAGE / RP;  // rows per stage
    constexpr int TRW = SR / 16;       // rows per thread and stage
    // one buffer: the staged rows of W during the loop, the partial sums of the row groups after it
    __shared__ __attribute__((aligned(16))) float buf[PJ_STAGE];
    float (*Ws)[RP] = reinterpret_cast<float (*)[RP]>(buf);
    float (*red)[RP][PJ_COLS] = reinterpret_cast<float (*)[RP][PJ_COLS]>(buf);  // 8 x RP x 16 <= PJ_STAGE
    const bool left = (int)blockIdx.x < strips_in;
    const T* X = left ? A : D;
    const float* W = left ? Vf : Tf;
    float* out = left ? Pt : Gt;
    const int64_t h = left ? h_in : h_out;
    const int64_t c0 = (int64_t)(left ? blockIdx.x : blockIdx.x - strips_in) * PJ_COLS;
    const int t = threadIdx.x, col = t & 15, rg = t >> 4;
    const int64_t c = c0 + col;
    const bool colok = c < h;
    const int64_t cc = colok ? c : h - 1;
    const int64_t wtotal = N * RP;
    float acc[RP];
#pragma unroll
    for (int j = 0; j < RP; ++j) acc[j] = 0.f;
    for (int64_t n0 = 0; n0 < N; n0 += SR) {
        // clamped addresses and no selects behind the loads, so that all of them go out together:
        // rows from N on meet zero rows of W, columns from h on are not stored
        float4 wv[PJ_STAGE / 1024];
#pragma unroll
        for (int m = 0; m < PJ_STAGE / 1024; ++m) {
            const int64_t idx = n0 * RP + 4 * (t + 256 * m);
            wv[m] = *reinterpret_cast<const float4*>(W + (idx < wtotal ? idx : wtotal - 4));
        }
        float x[TRW];
#pragma unroll
        for (int i = 0; i < TRW; ++i) {
            const int64_t n = n0 + rg + 16 * i;
            x[i] = ld<T>(X, (n < N ? n : N - 1) * h + cc);
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < PJ_STAGE / 1024; ++m) {
            const float keep = n0 * RP + 4 * (t + 256 * m) < wtotal ? 1.f : 0.f;  // rows from N on become zero
            reinterpret_cast<float4*>(buf)[t + 256 * m] =
                make_float4(keep * wv[m].x, keep * wv[m].y, keep * wv[m].z, keep * wv[m].w);
        }
        __syncthreads();
        const int64_t rest = N - n0;
#pragma unroll
        for (int i = 0; i < TRW; ++i) {
            if (16 * i < rest) {  // uniform: skips the row groups of a short last stage
                const float4* w4 = reinterpret_cast<const float4*>(Ws[rg + 16 * i]);
#pragma unroll
                for (int q = 0; q < RP / 4; ++q) {
                    const float4 w = w4[q];
                    acc[4 * q] = fmaf(w.x, x[i], acc[4 * q]);
                    acc[4 * q + 1] = fmaf(w.y, x[i], acc[4 * q + 1]);
                    acc[4 * q + 2] = fmaf(w.z, x[i], acc[4 * q + 2]);
                    acc[4 * q + 3] = fmaf(w.w, x[i], acc[4 * q + 3]);
                }
            }
        }
    }
    __syncthreads();
    if (rg >= 8) {
#pragma unroll
        for (int j = 0; j < RP; ++j) red[rg - 8][j][col] = acc[j];
    }
    __syncthreads();
    if (rg < 8) {
#pragma unroll
        for (int j = 0; j < RP; ++j) acc[j] += red[rg][j][col];
    }
    __syncthreads();
    if (rg < 8) {
#pragma unroll
        for (int j = 0; j < RP; ++j) red[rg][j][col] = acc[j];
    }
    __syncthreads();
    // RP x 16 results, 8 partials each
    for (int e = t; e < RP * PJ_COLS; e += 256) {
        const int j = e / PJ_COLS, cl = e % PJ_COLS;
        float s = red[0][j][cl];
#pragma unroll
        for (int g = 1; g < 8; ++g) s += red[g][j][cl];
        if (j < r && c0 + cl < h) out[(int64_t)j * h + c0 + cl] = s;
    }
}

// ------------------------------------------------------------------------------------ plan

struct GramPlan {
    GramJobs J;
    int rows16;
    size_t off_hdr, off_part, off_C, off_E, off_H0, off_Z, off_F, off_gp, off_rinv, off_Tf, off_Vf, total;
};

// Row pitch of the fp32 copies the projection reads: the accumulator count of its instantiation.
static inline int proj_pitch(int r) { return r <= 16 ? 16 : r <= 32 ? 32 : 64; }

static GramPlan plan_gram(int64_t N, int64_t h_in, int64_t h_out, int r) {
    GramPlan p;
    GramJobs& J = p.J;
    J.nt = (int)ceil_div(N, GT);
    J.nta = (int)ceil_div(N + r, GT);
    J.jobsC = tri_count(J.nt);
    J.jobsE = tri_count(J.nta);
    // the longest column chunk that still gives about three workgroups per compute unit
    const int64_t hmax = h_in > h_out ? h_in : h_out;
    int64_t ck = (int64_t)align_up((size_t)hmax, GK);
    for (;;) {
        const int64_t wgs = J.jobsC * ceil_div(h_in, ck) + J.jobsE * ceil_div(h_out, ck);
        if (wgs >= 768 || ck <= 2 * GK) break;
        ck = (int64_t)align_up((size_t)(ck / 2), GK);
    }
    J.ck = ck;
    J.splitsC = (int)ceil_div(h_in, ck);
    J.splitsE = (int)ceil_div(h_out, ck);
    p.rows16 = (int)ceil_div(N, 16);
    size_t o = 0;
    p.off_hdr = o, o += 256;
    p.off_part = o, o += ((size_t)J.jobsC * J.splitsC + (size_t)J.jobsE * J.splitsE) * GT * GT * 8;
    p.off_C = o, o += align_up((size_t)N * N * 8, 256);
    p.off_E = o, o += align_up((size_t)N * N * 8, 256);
    p.off_H0 = o, o += align_up((size_t)N * r * 8, 256);
    p.off_Z = o, o += align_up((size_t)N * r * 8, 256);
    p.off_F = o, o += align_up((size_t)N * r * 8, 256);
    p.off_gp = o, o += align_up((size_t)p.rows16 * r * r * 8, 256);
    p.off_rinv = o, o += 2 * (size_t)DAD_MAX_RANK * DAD_MAX_RANK * 8;
    p.off_Tf = o, o += align_up((size_t)N * proj_pitch(r) * 4, 256);
    p.off_Vf = o, o += align_up((size_t)N * proj_pitch(r) * 4, 256);
    p.total = o;
    return p;
}

template <int NA>
static dad_status ns_steps(const GramPlan& p, char* ws, int64_t N, int r, int n_iter, hipStream_t s) {
    const double* C = reinterpret_cast<const double*>(ws + p.off_C);
    const double* E = reinterpret_cast<const double*>(ws + p.off_E);
    const double* H0 = reinterpret_cast<const double*>(ws + p.off_H0);
    double* Z = reinterpret_cast<double*>(ws + p.off_Z);
    double* F = reinterpret_cast<double*>(ws + p.off_F);
    double* gp = reinterpret_cast<double*>(ws + p.off_gp);
    double* rinv[2] = {reinterpret_cast<double*>(ws + p.off_rinv),
                       reinterpret_cast<double*>(ws + p.off_rinv) + DAD_MAX_RANK * DAD_MAX_RANK};
    float* Tf = reinterpret_cast<float*>(ws + p.off_Tf);
    float* Vf = reinterpret_cast<float*>(ws + p.off_Vf);
    int* flag = reinterpret_cast<int*>(ws + p.off_hdr);
    int* counter = flag + 16;
    double* piv = reinterpret_cast<double*>(ws + p.off_hdr + 128);  // smallest and largest pivot of the last factor
    const dim3 grid((unsigned)p.rows16), block(256);
    const size_t lds = sizeof(NsShared<NA>);
    int cur = 0;  // rinv[cur] holds the factor of the latest Gram matrix
    for (int it = 0; it < n_iter; ++it) {
        {
            ProfScope ps(KID_NS_STEP, s);
            hipLaunchKernelGGL((k_ns_step<NA, NS_CV>), grid, block, lds, s, C, it == 0 ? H0 : (const double*)F, Z, F,
                               it == 0 ? (const double*)nullptr : (const double*)rinv[cur], (double*)nullptr,
                               (float*)nullptr, (float*)nullptr, 0, N, r, gp, counter, flag, piv);
        }
        DAD_LAUNCH_CHECK();
        cur ^= 1;
        {
            ProfScope ps(KID_NS_STEP, s);
            hipLaunchKernelGGL((k_ns_step<NA, NS_EZ>), grid, block, lds, s, E, (const double*)nullptr, Z, F,
                               (const double*)nullptr, rinv[cur], (float*)nullptr, (float*)nullptr, 0, N, r, gp, counter,
                               flag, piv);
        }
        DAD_LAUNCH_CHECK();
    }
    {   // second Cholesky round for the iterate that is returned
        ProfScope ps(KID_NS_STEP, s);
        hipLaunchKernelGGL((k_ns_step<NA, NS_REFINE>), grid, block, lds, s, (const double*)nullptr, (const double*)nullptr,
                           Z, F, (const double*)rinv[cur], rinv[cur ^ 1], (float*)nullptr, (float*)nullptr, 0, N, r, gp,
                           counter, flag, piv);
    }
    DAD_LAUNCH_CHECK();
    cur ^= 1;
    {
        ProfScope ps(KID_NS_STEP, s);
        hipLaunchKernelGGL((k_ns_step<NA, NS_APPLY>), grid, block, lds, s, (const double*)nullptr, (const double*)nullptr, Z,
                           F, (const double*)rinv[cur], (double*)nullptr, Tf, Vf, proj_pitch(r), N, r, gp, counter, flag, piv);
    }
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

template <typename T>
static dad_status run_gram(const GramPlan& p, const T* A, const T* D, int64_t N, int64_t h_in, int64_t h_out, int r,
                           int n_iter, const float* G0, float* Pt, float* Gt, char* ws, hipStream_t s) {
    double* part = reinterpret_cast<double*>(ws + p.off_part);
    int* hdr = reinterpret_cast<int*>(ws + p.off_hdr);
    const int q = 16 / (int)sizeof(T);  // elements per 16-byte load
    const int vecA = h_in % q == 0, vecD = h_out % q == 0;
    {
        ProfScope ps(KID_GRAM_TILES, s);
        const unsigned grid = (unsigned)(p.J.jobsC * p.J.splitsC + p.J.jobsE * p.J.splitsE);
        hipLaunchKernelGGL((k_gram_tiles<T>), dim3(grid), dim3(256), 0, s, A, D, G0, N, h_in, h_out, r, p.J, part, vecA,
                           vecD, hdr);
    }
    DAD_LAUNCH_CHECK();
    {
        ProfScope ps(KID_GRAM_GATHER, s);
        hipLaunchKernelGGL(k_gram_gather, dim3((unsigned)(4 * (p.J.jobsC + p.J.jobsE))), dim3(256), 0, s, part, p.J, N, r,
                           reinterpret_cast<double*>(ws + p.off_C), reinterpret_cast<double*>(ws + p.off_E),
                           reinterpret_cast<double*>(ws + p.off_H0));
    }
    DAD_LAUNCH_CHECK();
    dad_status rc = r <= 32 ? ns_steps<2>(p, ws, N, r, n_iter, s) : ns_steps<4>(p, ws, N, r, n_iter, s);
    if (rc != DAD_OK) return rc;
    const int strips_in = (int)ceil_div(h_in, PJ_COLS), strips_out = (int)ceil_div(h_out, PJ_COLS);
    const float* Tf = reinterpret_cast<const float*>(ws + p.off_Tf);
    const float* Vf = reinterpret_cast<const float*>(ws + p.off_Vf);
    {
        ProfScope ps(KID_NS_PROJECT, s);
        const dim3 grid((unsigned)(strips_in + strips_out)), block(256);
        if (r <= 16)
            hipLaunchKernelGGL((k_ns_project<T, 16>), grid, block, 0, s, A, D, Vf, Tf, Pt, Gt, N, h_in, h_out, r, strips_in);
        else if (r <= 32)
            hipLaunchKernelGGL((k_ns_project<T, 32>), grid, block, 0, s, A, D, Vf, Tf, Pt, Gt, N, h_in, h_out, r, strips_in);
        else
            hipLaunchKernelGGL((k_ns_project<T, 64>), grid, block, 0, s, A, D, Vf, Tf, Pt, Gt, N, h_in, h_out, r, strips_in);
    }
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

template <int NA>
static dad_status ns_prepare() {
    const int lds = (int)sizeof(NsShared<NA>);
    DAD_HIP_TRY(set_max_lds((k_ns_step<NA, NS_CV>), lds));
    DAD_HIP_TRY(set_max_lds((k_ns_step<NA, NS_EZ>), lds));
    DAD_HIP_TRY(set_max_lds((k_ns_step<NA, NS_REFINE>), lds));
    DAD_HIP_TRY(set_max_lds((k_ns_step<NA, NS_APPLY>), lds));
    return DAD_OK;
}

dad_status gram_prepare_device() {
    const dad_status rc = ns_prepare<2>();
    return rc != DAD_OK ? rc : ns_prepare<4>();
}

}  // namespace dad

using namespace dad;

static bool gram_shape_ok(int64_t N, int64_t h_in, int64_t h_out, int r) {
    if (N < 1 || N > DAD_GRAM_MAX_ROWS || h_in < 1 || h_out < 1 || r < 1 || r > DAD_MAX_RANK) return false;
    if (r > N || r > h_in || r > h_out) return false;
    return h_in <= DAD_MAX_WIDTH && h_out <= DAD_MAX_WIDTH;
}

extern "C" size_t dad_compress_gram_workspace_bytes(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt) {
    if ((dt != DAD_F32 && dt != DAD_BF16) || !gram_shape_ok(N, h_in, h_out, r)) return 0;
    return plan_gram(N, h_in, h_out, r).total;
}

extern "C" dad_status dad_compress_rank_gram(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                             dad_dtype dt, int r, int n_iter, const float* G0, float* Pt, float* Gt,
                                             void* workspace, size_t ws_bytes, void* stream) {
    if (!A || !D || !G0 || !Pt || !Gt || !workspace) return DAD_ERR_NULL;
    if (dt != DAD_F32 && dt != DAD_BF16) return DAD_ERR_DTYPE;
    if (!gram_shape_ok(N, h_in, h_out, r) || n_iter < 1) return DAD_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(D) || !aligned16(G0) || !aligned16(Pt) || !aligned16(Gt) || !aligned16(workspace))
        return DAD_ERR_ALIGN;
    const GramPlan p = plan_gram(N, h_in, h_out, r);
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    hipStream_t s = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    if (dt == DAD_F32)
        return run_gram<float>(p, static_cast<const float*>(A), static_cast<const float*>(D), N, h_in, h_out, r, n_iter,
                               G0, Pt, Gt, ws, s);
    return run_gram<bf16_t>(p, static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(D), N, h_in, h_out, r, n_iter,
                            G0, Pt, Gt, ws, s);
}

// Tall-skinny orthonormalisation of the h x r iterate by CholeskyQR2.
// The iterate is held transposed (Yt: r x h, row j = column j of Y), so the
// Gram matrix is S[i][j] = sum_k Yt[i][k] Yt[j][k].  One round is
//   S = Y^T Y  ->  S = R^T R (upper R)  ->  Y <- Y R^{-1},
// done twice (CholeskyQR2) for the iterate that is returned and once for the intermediate
// iterates of the power iteration, of which only the span matters.  Launches of CholeskyQR2:
//   1. Gram partials of Yt per 256-column slab; the workgroup that finishes last
//      sums them (fixed order), factorises and inverts R in fp64.
//   2. Y <- Y R^{-1} per slab, Gram partials of the result, last workgroup
//      factorises again.
//   3. Y <- Y R^{-1} with the second factor.
// Products of two fp32 values are exact in fp64, so the Gram matrix carries no
// rounding beyond its final sums and CholeskyQR tolerates condition numbers far
// beyond the fp32 limit.  The partials are accumulated by the fp64 matrix instruction.
#include "dad_internal.h"

namespace dad {

constexpr int QR_COLS = 64;  // columns of Yt per LDS tile
constexpr int QR_SUB = 4;    // tiles per workgroup: few, fat Gram partials keep the final sum short
constexpr int QR_LD = DAD_MAX_RANK + 1;

struct QrShared {
    union {
        float Ys[DAD_MAX_RANK][QR_COLS + 1];  // tile of Yt (or of the result)
        struct {
            double colS[2][2][DAD_MAX_RANK];  // columns k, k+1 of the running S, double buffered over steps
            double rowT[2][2][DAD_MAX_RANK];  // rows k, k+1 of the running inverse
        } f;
    };
    float Rs[DAD_MAX_RANK][QR_LD];  // R^{-1} applied by this launch
    int last;
};

// In the factorisation threads form a 16 x 16 grid (ti, tj); thread (ti, tj) owns the entries
// (ti + 16a, tj + 16b), a, b < NA, of every r x r matrix (NA = 2 covers r <= 32, NA = 4 r <= 64).
//
// The Gram partials are accumulated with the fp64 matrix instruction (16x16 output block, 4 columns
// of the tile per issue): products of fp32 values are exact in fp64.  The NA*NA blocks are dealt to
// the four waves, NA*NA/4 each; block q = wave*NBW + u covers rows 16*(q / NA), columns 16*(q % NA).
// Operand layout: lane l supplies row l%16 of its block at tile column 4*kk + l/16; result element
// v of lane l is entry (4v + l/16, l%16) of the block.
typedef double f64x4 __attribute__((ext_vector_type(4)));

template <int NA>
struct GramAcc {
    static constexpr int NBW = NA * NA / 4;
    f64x4 v[NBW];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int u = 0; u < NBW; ++u) v[u] = f64x4{0.0, 0.0, 0.0, 0.0};
    }
};

template <int NA>
__device__ __forceinline__ void gram_of_tile(const float (*Ys)[QR_COLS + 1], GramAcc<NA>& acc) {
    constexpr int NBW = GramAcc<NA>::NBW;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, lk = lane >> 4;
    const int a = (wave * NBW) / NA;  // the blocks of one wave share their row index
#pragma unroll 4
    for (int kk = 0; kk < QR_COLS / 4; ++kk) {
        const double ya = (double)Ys[16 * a + li][4 * kk + lk];
#pragma unroll
        for (int u = 0; u < NBW; ++u) {
            const int b = (wave * NBW + u) % NA;
            const double yb = (double)Ys[16 * b + li][4 * kk + lk];
            acc.v[u] = __builtin_amdgcn_mfma_f64_16x16x4f64(ya, yb, acc.v[u], 0, 0, 0);
        }
    }
}

// Runs in every workgroup after its Gram partial `acc` is complete; the workgroup that takes the
// last ticket sums all partials (block order ascending) and factorises:
// S = L L^T and X = L^{-1} by one right-looking sweep over k in fp64 registers.  Pivot k needs
// column k of the running S and row k of the running inverse T (T starts as I), published through LDS; then
//     L[i][k] = S[i][k] / sqrt(S[k][k]),  X[k][j] = T[k][j] / sqrt(S[k][k]),
//     S[i][j] -= L[i][k] L[j][k],         T[i][j] -= L[i][k] X[k][j]      for i > k.
// R^{-1} = X^T (upper triangular) is written as fp32.  A pivot that is not > 0 (or NaN) latches
// *flag and is replaced by 1 so the sweep still ends with finite arithmetic.
template <int NA>
__device__ __forceinline__ void last_block_factor(QrShared& sh, const GramAcc<NA>& acc, double* __restrict__ gram_part,
                                                  int nblocks, int r, int* __restrict__ counter,
                                                  float* __restrict__ rinv, int* __restrict__ flag) {
    const int t = threadIdx.x, ti = t >> 4, tj = t & 15;
    const int nent = r * r;
    double* mine = gram_part + (int64_t)blockIdx.x * nent;
    {
        constexpr int NBW = GramAcc<NA>::NBW;
        const int lane = t & 63, wave = t >> 6;
#pragma unroll
        for (int u = 0; u < NBW; ++u) {
            const int q = wave * NBW + u;
            const int j = 16 * (q % NA) + (lane & 15);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 16 * (q / NA) + 4 * v + (lane >> 4);
                if (i < r && j < r) mine[i * r + j] = acc.v[u][v];
            }
        }
    }
    __threadfence();
    __syncthreads();
    if (t == 0) sh.last = (atomicAdd(counter, 1) == nblocks - 1);
    __syncthreads();
    if (!sh.last) return;
    __threadfence();

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
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < NA; ++b) {
            const int i = ti + 16 * a, j = tj + 16 * b;
            if (i >= r || j >= r) S[a][b] = (i == j) ? 1.0 : 0.0;
        }

    // Two pivots per step: columns k, k+1 of S and rows k, k+1 of T are published together and every
    // thread redoes the small update of the second by the first (same operations, in the same order,
    // as two single steps), which halves the number of barriers on this serial path.  For odd r the
    // last step's second pivot is the inert identity padding.
    bool bad = false;
    for (int k = 0; k < r; k += 2) {
        const int buf = (k >> 1) & 1, ka = k >> 4, kt = k & 15;
        if (tj == kt || tj == kt + 1) {
            const int which = tj - kt;
#pragma unroll
            for (int b = 0; b < NA; ++b)
                if (b == ka) {
#pragma unroll
                    for (int a = 0; a < NA; ++a) sh.f.colS[buf][which][ti + 16 * a] = S[a][b];
                }
        }
        if (ti == kt || ti == kt + 1) {
            const int which = ti - kt;
#pragma unroll
            for (int a = 0; a < NA; ++a)
                if (a == ka) {
#pragma unroll
                    for (int b = 0; b < NA; ++b) sh.f.rowT[buf][which][tj + 16 * b] = T[a][b];
                }
        }
        __syncthreads();
        const double* c0 = sh.f.colS[buf][0];
        const double* c1 = sh.f.colS[buf][1];
        const double* t0 = sh.f.rowT[buf][0];
        const double* t1 = sh.f.rowT[buf][1];
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
        const double d0 = rsqrt(piv0);
        const double m = ck1 * d0;  // L[k+1][k]
        piv1 = fma(-m, m, piv1);
        if (!(piv1 > 0.0)) {
            bad = true;
            piv1 = 1.0;
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
                    rinv[j * r + k] = (float)x0[b];
                    if (k + 1 < r) rinv[j * r + k + 1] = (float)x1[b];
                }
            }
        }
    }
    if (bad && t == 0) *flag = 1;
    if (t == 0) *counter = 0;
}

// Up-front load of this workgroup's QR_SUB tiles; element m of tile `sub` is row (t + 256 m) / 64,
// column (t + 256 m) % 64 of that tile.
template <int SUB>
__device__ __forceinline__ void load_slab(float (&st)[SUB][16], const float* Yt, int64_t h, int r, int64_t k0) {
    const int t = threadIdx.x;
#pragma unroll
    for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int e = t + 256 * m, i = e >> 6, kk = e & 63;
            const int64_t k = k0 + sub * QR_COLS + kk;
            st[sub][m] = (i < r && k < h) ? Yt[(int64_t)i * h + k] : 0.f;
        }
}

__device__ __forceinline__ void store_tile(QrShared& sh, const float (&st)[16]) {
    const int t = threadIdx.x;
#pragma unroll
    for (int m = 0; m < 16; ++m) {
        const int e = t + 256 * m;
        sh.Ys[e >> 6][e & 63] = st[m];
    }
}

// Launch 1: Gram partial per slab + factorisation by the last workgroup.
template <int NA>
__global__ __launch_bounds__(256) void k_qr_gram(const float* __restrict__ Yt, int64_t h, int r,
                                                 double* __restrict__ gram_part, int* __restrict__ counter,
                                                 float* __restrict__ rinv, int* __restrict__ flag) {
    __shared__ QrShared sh;
    const int64_t k0 = (int64_t)blockIdx.x * QR_SUB * QR_COLS;
    float st[QR_SUB][16];
    load_slab<QR_SUB>(st, Yt, h, r, k0);
    GramAcc<NA> acc;
    acc.zero();
#pragma unroll
    for (int sub = 0; sub < QR_SUB; ++sub) {
        if (k0 + sub * QR_COLS < h) {
            if (sub) __syncthreads();
            store_tile(sh, st[sub]);
            __syncthreads();
            gram_of_tile<NA>(sh.Ys, acc);
        }
    }
    __syncthreads();
    last_block_factor<NA>(sh, acc, gram_part, gridDim.x, r, counter, rinv, flag);
}

// Launches 2 and 3: Gt[j][k] = sum_{i<=j} rinv_in[i][j] * Yt[i][k]; Gt may alias Yt (each workgroup
// reads its slab completely before it writes).  WITH_GRAM also prepares the next factor.
template <int NA, bool WITH_GRAM, int SUB>
__global__ __launch_bounds__(256) void k_qr_apply(const float* Yt, float* Gt, const float* __restrict__ rinv_in,
                                                  int64_t h, int r, double* __restrict__ gram_part,
                                                  int* __restrict__ counter, float* __restrict__ rinv_out,
                                                  int* __restrict__ flag, bf16_t* __restrict__ gt_bf16) {
    __shared__ QrShared sh;
    const int t = threadIdx.x;
    const int kl = t & 63, jg = t >> 6;
    const int64_t k0 = (int64_t)blockIdx.x * SUB * QR_COLS;
    float st[SUB][16];
    load_slab<SUB>(st, Yt, h, r, k0);
    for (int e = t; e < DAD_MAX_RANK * DAD_MAX_RANK; e += 256) {
        const int i = e >> 6, j = e & 63;
        sh.Rs[i][j] = (i < r && j < r) ? rinv_in[i * r + j] : 0.f;
    }
    GramAcc<NA> acc;
    acc.zero();
#pragma unroll
    for (int sub = 0; sub < SUB; ++sub) {
        const int64_t kc = k0 + sub * QR_COLS + kl;
        if (k0 + sub * QR_COLS < h) {
            if (sub) __syncthreads();
            store_tile(sh, st[sub]);
            __syncthreads();
            // R^{-1} is upper triangular and stored with its zeros, so the sum runs over all i
            float out[NA * 4];
#pragma unroll
            for (int m = 0; m < NA * 4; ++m) out[m] = 0.f;
#pragma unroll 4
            for (int i = 0; i < r; ++i) {
                const float y = sh.Ys[i][kl];
#pragma unroll
                for (int m = 0; m < NA * 4; ++m) out[m] = fmaf(sh.Rs[i][jg + 4 * m], y, out[m]);
            }
            __syncthreads();
#pragma unroll
            for (int m = 0; m < NA * 4; ++m) {
                const int j = jg + 4 * m;
                if (j < r) {
                    if (kc < h) {
                        Gt[(int64_t)j * h + kc] = out[m];
                        if (gt_bf16) gt_bf16[(int64_t)j * h + kc] = f32_to_bf16(out[m]);  // panel of the next thin_nn
                    }
                    if (WITH_GRAM) sh.Ys[j][kl] = (kc < h) ? out[m] : 0.f;
                }
            }
            if (WITH_GRAM) {
                __syncthreads();
                gram_of_tile<NA>(sh.Ys, acc);
            }
        }
    }
    if (WITH_GRAM) {
        __syncthreads();
        last_block_factor<NA>(sh, acc, gram_part, gridDim.x, r, counter, rinv_out, flag);
    }
}

int gram_blocks_for(int64_t h) { return (int)ceil_div(h, QR_COLS * QR_SUB); }

// `rounds` = 2: CholeskyQR2.  `rounds` = 1: a single Cholesky round, enough for an intermediate
// iterate of the power iteration, of which only the span matters.
template <int NA>
static dad_status qr(const float* Yt, float* Gt, int64_t h, int r, int rounds, double* gram_part, int nb, float* rinv,
                     int* counter, int* flag, bf16_t* gt_bf16, hipStream_t s) {
    float* rinv2 = rinv + DAD_MAX_RANK * DAD_MAX_RANK;
    const unsigned nb1 = (unsigned)ceil_div(h, QR_COLS);
    {
        ProfScope prof(KID_GRAM, s);
        hipLaunchKernelGGL(k_qr_gram<NA>, dim3((unsigned)nb), dim3(256), 0, s, Yt, h, r, gram_part, counter, rinv, flag);
    }
    DAD_LAUNCH_CHECK();
    if (rounds == 1) {
        ProfScope prof(KID_APPLY2, s);
        hipLaunchKernelGGL((k_qr_apply<NA, false, 1>), dim3(nb1), dim3(256), 0, s, Yt, Gt, (const float*)rinv, h, r,
                           gram_part, counter, rinv2, flag, gt_bf16);
        DAD_LAUNCH_CHECK();
        return DAD_OK;
    }
    {
        ProfScope prof(KID_APPLY, s);
        hipLaunchKernelGGL((k_qr_apply<NA, true, QR_SUB>), dim3((unsigned)nb), dim3(256), 0, s, Yt, Gt, (const float*)rinv,
                           h, r, gram_part, counter, rinv2, flag, (bf16_t*)nullptr);
    }
    DAD_LAUNCH_CHECK();
    {
        ProfScope prof(KID_APPLY2, s);
        hipLaunchKernelGGL((k_qr_apply<NA, false, 1>), dim3(nb1), dim3(256), 0, s, (const float*)Gt, Gt,
                           (const float*)rinv2, h, r, gram_part, counter, rinv2, flag, gt_bf16);
    }
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

dad_status launch_cholqr(const float* Yt, float* Gt, int64_t h, int r, int rounds, double* gram_part, int gram_blocks,
                         float* rinv, int* counter, int* flag, void* gt_bf16, hipStream_t s) {
    if (r <= 32) return qr<2>(Yt, Gt, h, r, rounds, gram_part, gram_blocks, rinv, counter, flag, (bf16_t*)gt_bf16, s);
    return qr<4>(Yt, Gt, h, r, rounds, gram_part, gram_blocks, rinv, counter, flag, (bf16_t*)gt_bf16, s);
}

}  // namespace dad

// Tall-skinny orthonormalisation of the h x r iterate by CholeskyQR2.
// The iterate is held transposed (Yt: r x h, row j = column j of Y), so the
// Gram matrix is S[i][j] = sum_k Yt[i][k] Yt[j][k].  One round is
//   S = Y^T Y  ->  S = R^T R (upper R)  ->  Y <- Y R^{-1},
// done twice (CholeskyQR2) for the iterate that is returned - unless the pivots of the first round
// show that one is enough - and once for the intermediate iterates of the power iteration, of
// which only the span matters.  Launches of CholeskyQR2:
//   1. Gram partials of Yt per 256-column slab; the workgroup that finishes last
//      sums them (fixed order), factorises and inverts R in fp64.
//   2. Y <- Y R^{-1} per slab, Gram partials of the result, last workgroup
//      factorises again.
//   3. Y <- Y R^{-1} with the second factor.
// Products of two fp32 values are exact in fp64, so the Gram matrix carries no
// rounding beyond its final sums and CholeskyQR tolerates condition numbers far
// beyond the fp32 limit.  The partials are accumulated by the fp64 matrix instruction.
#include "chol_factor.h"
#include "dad_internal.h"

namespace dad {

constexpr int QR_COLS = 64;  // columns of Yt per LDS tile
constexpr int QR_SUB = 4;    // tiles per workgroup: few, fat Gram partials keep the final sum short
constexpr int QR_LD = DAD_MAX_RANK + 1;
// Row pitch of the LDS tile: 4 banks from row to row, so that the 16 rows x 4 columns one operand read of
// the fp64 matrix instruction touches fall into 64 different banks (pitch 65 gave 35 % conflict cycles).
constexpr int QR_PITCH = QR_COLS + 4;

struct QrShared {
    union {
        float Ys[DAD_MAX_RANK][QR_PITCH];  // tile of Yt (or of the result)
        FactorShared f;
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
__device__ __forceinline__ void gram_of_tile(const float (*Ys)[QR_PITCH], GramAcc<NA>& acc) {
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

// Runs in every workgroup after its Gram partial `acc` is complete: the partial is published and the
// workgroup that takes the last ticket sums all partials and factorises (factor_partials); R^{-1}
// is written as fp32.
template <int NA>
__device__ __forceinline__ void last_block_factor(QrShared& sh, const GramAcc<NA>& acc, double* __restrict__ gram_part,
                                                  int nblocks, int r, int* __restrict__ counter,
                                                  float* __restrict__ rinv, int* __restrict__ flag,
                                                  double* __restrict__ piv_range) {
    const int t = threadIdx.x;
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

    factor_partials<NA, float>(sh.f, gram_part, nblocks, r, rinv, flag, piv_range);
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
// The copy of *p that belongs to job blockIdx.y of a batch (job_stride bytes per job); null stays null.
template <typename T>
__device__ __forceinline__ T* at_job(T* p, int64_t job_stride) {
    typedef typename std::remove_const<T>::type U;
    return p ? reinterpret_cast<T*>(reinterpret_cast<char*>(const_cast<U*>(p)) + blockIdx.y * job_stride) : p;
}
#define DAD_TO_JOB(p) p = at_job(p, job_stride)

template <int NA>
__global__ __launch_bounds__(256) void k_qr_gram(const float* __restrict__ Yt, int64_t h, int r,
                                                 double* __restrict__ gram_part, int* __restrict__ counter,
                                                 float* __restrict__ rinv, int* __restrict__ flag,
                                                 double* __restrict__ piv_range, int64_t job_stride, BatchInts dims,
                                                 int use_dims) {
    __shared__ QrShared sh;
    int nblocks = gridDim.x;
    if (job_stride != 0) {
        if (use_dims) {  // this job's own width; the grid is sized for the widest job
            h = dims.a[blockIdx.y];
            nblocks = (int)((h + QR_SUB * QR_COLS - 1) / (QR_SUB * QR_COLS));
            if ((int)blockIdx.x >= nblocks) return;
        }
        DAD_TO_JOB(Yt), DAD_TO_JOB(gram_part), DAD_TO_JOB(counter);
        DAD_TO_JOB(rinv), DAD_TO_JOB(flag), DAD_TO_JOB(piv_range);
    }
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
    last_block_factor<NA>(sh, acc, gram_part, nblocks, r, counter, rinv, flag, piv_range);
}

// One Cholesky round leaves G^T G - I at about eps32 * cond(Y) (the rounding of Y R^-1 in fp32); the
// second round brings it to eps32.  The first factorisation reports (||R||_F ||R^-1||_F / r)^2, an
// upper bound of cond(Y)^2 that is 1 for orthogonal columns of equal length: when it is at most
// QR_ONE_ROUND_BOUND (cond(Y) <= 4 r) the first round is kept as the result (the flat spectra of dense
// layers' gradients) and the second is not run.
constexpr double QR_ONE_ROUND_BOUND = 16.0;

__device__ __forceinline__ bool one_round_enough(const double* __restrict__ piv_first) {
    return piv_first[0] > 0.0 && piv_first[1] <= QR_ONE_ROUND_BOUND;
}

// Launches 2 and 3: Gt[j][k] = sum_{i<=j} rinv_in[i][j] * Yt[i][k]; Gt may alias Yt (each workgroup
// reads its slab completely before it writes).  WITH_GRAM also prepares the next factor.
// piv_first (CholeskyQR2 only, else null) holds the pivot range of the first factor: when one round
// is enough, the WITH_GRAM launch returns at once and the launch after it applies the first factor
// (rinv_first) to the iterate itself (Y_first) instead of the second factor to the first result.
template <int NA, bool WITH_GRAM, int SUB>
__global__ __launch_bounds__(256) void k_qr_apply(const float* Yt, float* Gt, const float* __restrict__ rinv_in,
                                                  int64_t h, int r, double* __restrict__ gram_part,
                                                  int* __restrict__ counter, float* __restrict__ rinv_out,
                                                  int* __restrict__ flag, bf16_t* __restrict__ gt_bf16,
                                                  const double* __restrict__ piv_first,
                                                  double* __restrict__ piv_second, const float* Y_first,
                                                  const float* __restrict__ rinv_first, int64_t job_stride,
                                                  BatchInts dims, int use_dims) {
    __shared__ QrShared sh;
    int nblocks = gridDim.x;
    if (job_stride != 0) {
        if (use_dims) {
            h = dims.a[blockIdx.y];
            nblocks = (int)((h + SUB * QR_COLS - 1) / (SUB * QR_COLS));
            if ((int)blockIdx.x >= nblocks) return;
        }
        DAD_TO_JOB(Yt), DAD_TO_JOB(Gt), DAD_TO_JOB(rinv_in), DAD_TO_JOB(gram_part);
        DAD_TO_JOB(counter), DAD_TO_JOB(rinv_out), DAD_TO_JOB(flag), DAD_TO_JOB(gt_bf16);
        DAD_TO_JOB(piv_first), DAD_TO_JOB(piv_second), DAD_TO_JOB(Y_first);
        DAD_TO_JOB(rinv_first);
    }
    const bool single = piv_first != nullptr && one_round_enough(piv_first);  // uniform over the grid
    if (WITH_GRAM && single) return;
    if (!WITH_GRAM && single) {
        Yt = Y_first;
        rinv_in = rinv_first;
    }
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
        last_block_factor<NA>(sh, acc, gram_part, nblocks, r, counter, rinv_out, flag, piv_second);
    }
}

int gram_blocks_for(int64_t h) { return (int)ceil_div(h, QR_COLS * QR_SUB); }

// `rounds` = 2: CholeskyQR2.  `rounds` = 1: a single Cholesky round, enough for an intermediate
// iterate of the power iteration, of which only the span matters.
template <int NA>
static dad_status qr(const float* Yt, float* Gt, int64_t h, int r, int rounds, double* gram_part, int nb, float* rinv,
                     int* counter, int* flag, bf16_t* gt_bf16, hipStream_t s, int jobs, int64_t job_stride,
                     const BatchInts* dims) {
    const BatchInts bd = dims ? *dims : BatchInts{};
    const int ud = dims ? 1 : 0;
    float* rinv2 = rinv + DAD_MAX_RANK * DAD_MAX_RANK;
    // pivot ranges of the two factors: four doubles at byte 128 of the 256-byte workspace header
    double* piv = reinterpret_cast<double*>(reinterpret_cast<char*>(flag) + 128);
    const unsigned nb1 = (unsigned)ceil_div(h, QR_COLS);
    {
        ProfScope prof(KID_GRAM, s);
        hipLaunchKernelGGL(k_qr_gram<NA>, dim3((unsigned)nb, (unsigned)jobs), dim3(256), 0, s, Yt, h, r, gram_part, counter,
                           rinv, flag, piv, job_stride, bd, ud);
    }
    DAD_LAUNCH_CHECK();
    if (rounds == 1) {
        ProfScope prof(KID_APPLY2, s);
        hipLaunchKernelGGL((k_qr_apply<NA, false, 1>), dim3(nb1, (unsigned)jobs), dim3(256), 0, s, Yt, Gt,
                           (const float*)rinv, h, r, gram_part, counter, rinv2, flag, gt_bf16, (const double*)nullptr,
                           (double*)nullptr, (const float*)nullptr, (const float*)nullptr, job_stride, bd, ud);
        DAD_LAUNCH_CHECK();
        return DAD_OK;
    }
    {
        ProfScope prof(KID_APPLY, s);
        hipLaunchKernelGGL((k_qr_apply<NA, true, QR_SUB>), dim3((unsigned)nb, (unsigned)jobs), dim3(256), 0, s, Yt, Gt,
                           (const float*)rinv, h, r, gram_part, counter, rinv2, flag, (bf16_t*)nullptr, (const double*)piv,
                           piv + 2, (const float*)nullptr, (const float*)nullptr, job_stride, bd, ud);
    }
    DAD_LAUNCH_CHECK();
    {
        ProfScope prof(KID_APPLY2, s);
        hipLaunchKernelGGL((k_qr_apply<NA, false, 1>), dim3(nb1, (unsigned)jobs), dim3(256), 0, s, (const float*)Gt, Gt,
                           (const float*)rinv2, h, r, gram_part, counter, rinv2, flag, gt_bf16, (const double*)piv,
                           (double*)nullptr, Yt, (const float*)rinv, job_stride, bd, ud);
    }
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

dad_status launch_cholqr(const float* Yt, float* Gt, int64_t h, int r, int rounds, double* gram_part, int gram_blocks,
                         float* rinv, int* counter, int* flag, void* gt_bf16, hipStream_t s, int jobs, int64_t job_stride,
                         const BatchInts* dims) {
    if (job_stride == 0) jobs = 1, dims = nullptr;
    if (r <= 32)
        return qr<2>(Yt, Gt, h, r, rounds, gram_part, gram_blocks, rinv, counter, flag, (bf16_t*)gt_bf16, s, jobs, job_stride,
                     dims);
    return qr<4>(Yt, Gt, h, r, rounds, gram_part, gram_blocks, rinv, counter, flag, (bf16_t*)gt_bf16, s, jobs, job_stride, dims);
}

}  // namespace dad

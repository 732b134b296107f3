// The thin contraction V = X G (Algorithm 2, Eq. 6: Delta G and A U) for fp32 factors on the fp32 matrix
// instruction:
//     V[n][j] = sum_k X[n][k] * Pt[j][k],      X  N x h,  Pt  r x h,  V  N x r,  all fp32.
// Both operands are contiguous along the contraction, so a stage is 32 columns of 128 rows of X and of
// the panel's rows, staged in LDS with a row pitch of 33 floats: v_mfma_f32_32x32x2_f32 takes one value
// per lane and operand (lane l: row l % 32, contraction index l / 32), and with that pitch the 64 lanes
// of a read touch 64 different banks.  A lane ends up with 16 rows of one column j, a half wave with 32
// consecutive j of one row: each store instruction writes whole rows of V.
// The other thin contraction of fp32 factors, V^T X, is G = L^T R with L = V and R = X and runs on
// k_rebuild_f32_mfma.
#include <type_traits>

#include "dad_internal.h"

namespace dad {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace tf {
constexpr int RT = 128;   // rows of X per workgroup, 32 per wave
constexpr int BK = 32;    // contraction columns per stage
constexpr int LD = BK + 1;
}  // namespace tf

// JT: 32-column blocks of the result (r <= 32 JT).  VEC: h is a multiple of 4 (rows of X and Pt are
// 16-byte aligned).  Workgroup (x, y): rows 128 x .., contraction columns y * col_chunk ..; with more
// than one column chunk the result goes to slab y of `part` ([split][N][r]) and is summed afterwards.
template <int JT, bool VEC>
__global__ __launch_bounds__(256) void k_thin_nn_f32_mfma(const float* __restrict__ X, const float* __restrict__ Pt,
                                                          float* __restrict__ out, float* __restrict__ part, int64_t N,
                                                          int64_t h, int r, int64_t col_chunk,
                                                          int* __restrict__ zero_hdr) {
    constexpr int RP = 32 * JT, ROWS = tf::RT + RP;
    constexpr int UNIT = VEC ? 4 : 1;
    constexpr int UPR = tf::BK / UNIT;                   // staging units per row
    constexpr int NLD = (ROWS * UPR + 255) / 256;        // staging accesses per thread and stage
    typedef typename std::conditional<VEC, f32x4, float>::type unit_t;
    __shared__ float lds[ROWS][tf::LD];  // rows 0..127: X, rows 128..: the panel

    // the first launch of a compress call also clears the workspace header (flag, ticket counter)
    if (zero_hdr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 64) zero_hdr[threadIdx.x] = 0;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int c = lane & 31, kh = lane >> 5;
    const int64_t n0 = (int64_t)blockIdx.x * tf::RT;
    const int64_t cbeg = (int64_t)blockIdx.y * col_chunk;
    const int64_t cend = (cbeg + col_chunk < h) ? cbeg + col_chunk : h;

    // Staging: access i of this thread is unit e = t + 256 i: row e / UPR of the stage, columns
    // (e % UPR) * UNIT ..  Addresses are clamped to valid ones and the value is zeroed by a select at
    // the LDS store, so that the loads of a stage are issued together.
    const float* src[NLD];
    int srow[NLD], scol[NLD];
    bool rowok[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int e = t + 256 * i;
        srow[i] = e / UPR;
        scol[i] = (e % UPR) * UNIT;
        if (srow[i] < tf::RT) {
            const int64_t n = n0 + srow[i];
            rowok[i] = n < N;
            src[i] = X + (rowok[i] ? n : 0) * h;
        } else {
            const int j = srow[i] - tf::RT;
            rowok[i] = j < r;  // also false for units beyond the stage (e >= ROWS * UPR)
            src[i] = Pt + (int64_t)(rowok[i] ? j : 0) * h;
        }
    }
    unit_t st[NLD];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int64_t k = k0 + scol[i];
            st[i] = *reinterpret_cast<const unit_t*>(src[i] + (k < cend ? k : cend - UNIT));  // VEC: h, chunks multiples of 4
        }
    };
    auto commit = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            if (srow[i] >= ROWS) continue;
            const bool ok = rowok[i] && k0 + scol[i] < cend;
            unit_t v = st[i];
            if (!ok) v = unit_t{};
            if constexpr (VEC) {
#pragma unroll
                for (int u = 0; u < 4; ++u) lds[srow[i]][scol[i] + u] = v[u];  // pitch 33: no 16-byte store
            } else {
                lds[srow[i]][scol[i]] = v;
            }
        }
    };

    f32x16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    fetch(cbeg);
    for (int64_t k0 = cbeg; k0 < cend; k0 += tf::BK) {
        commit(k0);
        __syncthreads();
        if (k0 + tf::BK < cend) fetch(k0 + tf::BK);  // in flight during the MFMAs below
#pragma unroll
        for (int kk = 0; kk < tf::BK; kk += 2) {
            const float x = lds[wave * 32 + c][kk + kh];
#pragma unroll
            for (int j = 0; j < JT; ++j) {
                const float p = lds[tf::RT + j * 32 + c][kk + kh];
                // X as the row operand: a lane owns one column j and 16 rows n
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, p, acc[j], 0, 0, 0);
            }
        }
        __syncthreads();  // the stage has been read; the next one may be stored
    }

    // lane: column j = 32 jt + lane % 32, rows 8 (v / 4) + 4 (lane / 32) + v % 4 of the wave's 32
    float* o = part ? part + (int64_t)blockIdx.y * N * r : out;
#pragma unroll
    for (int j = 0; j < JT; ++j) {
        const int col = j * 32 + c;
        if (col < r) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t n = n0 + wave * 32 + ((v >> 2) << 3) + (kh << 2) + (v & 3);
                if (n < N) o[n * r + col] = acc[j][v];
            }
        }
    }
}

// sp: column split as the guarded kernel's (chunk a multiple of 32); partials: [splits][N][r] floats.
dad_status f32_thin_nn(const float* X, const float* Pt, float* out, float* partials, SplitPlan sp, int64_t N, int64_t h,
                       int r, int* zero_hdr, hipStream_t s) {
    const dim3 grid((unsigned)ceil_div(N, tf::RT), (unsigned)sp.splits);
    float* part = sp.splits == 1 ? nullptr : partials;
    const bool vec = h % 4 == 0;
    {
        ProfScope prof(KID_THIN_NN, s);
#define DAD_F32_NN(JT)                                                                                                   \
    do {                                                                                                                 \
        if (vec)                                                                                                         \
            hipLaunchKernelGGL((k_thin_nn_f32_mfma<JT, true>), grid, dim3(256), 0, s, X, Pt, out, part, N, h, r, sp.chunk, \
                               zero_hdr);                                                                                \
        else                                                                                                             \
            hipLaunchKernelGGL((k_thin_nn_f32_mfma<JT, false>), grid, dim3(256), 0, s, X, Pt, out, part, N, h, r,         \
                               sp.chunk, zero_hdr);                                                                      \
    } while (0)
        if (r <= 32) DAD_F32_NN(1);
        else DAD_F32_NN(2);
#undef DAD_F32_NN
    }
    DAD_LAUNCH_CHECK();
    if (sp.splits == 1) return DAD_OK;
    return reduce_slabs(part, out, N * r, sp.splits, s);
}

}  // namespace dad

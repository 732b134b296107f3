// Algorithm 2 as printed, one singular pair at a time with peeling (Section 3.3.1, Eq. 5-7), on top
// of the thin contraction kernels.  Component j iterates
//     g <- normalise( M^T M g - sum_{i<j} sigma_i^2 g_i (g_i^T g) )          n_iter times,
// then v = Delta g, p = A^T v, sigma_j = ||p|| (= sqrt(v^T A A^T v)), q_j = p / sigma_j, and the
// pair (q_j, sigma_j g_j) is kept.  The peeled term is the deflation of M^T M by the pairs already
// found (the printed Q (G^T g) mixes vectors of two lengths); with sG_i = sigma_i g_i it is
// sum_i sG_i (sG_i^T g).  Every thin pass is HBM bound and costs the same for one column as for 32,
// so this route costs r times the block form; it exists because it is the paper's own recurrence.
#include "dad_internal.h"

namespace dad {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;  // lane 0 holds the sum
}

// Sum over the 1024 threads of the workgroup; every thread gets the result.
__device__ __forceinline__ double block_sum(double v, double* red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < 16; ++w) s += red[w];
    return s;
}

// g <- x / ||x||  (start vector of a component).  The first launch of a call also clears the header.
__global__ __launch_bounds__(1024) void k_seq_start(const float* __restrict__ x, float* __restrict__ g, int64_t h,
                                                    int* __restrict__ flag, int* __restrict__ zero_hdr) {
    __shared__ double red[16];
    if (zero_hdr && threadIdx.x < 64) zero_hdr[threadIdx.x] = 0;
    double ss = 0.0;
    for (int64_t k = threadIdx.x; k < h; k += 1024) ss += (double)x[k] * (double)x[k];
    ss = block_sum(ss, red);
    if (!(ss > 0.0)) {
        if (threadIdx.x == 0) *flag = 1;
        ss = 1.0;
    }
    const double inv = 1.0 / sqrt(ss);
    for (int64_t k = threadIdx.x; k < h; k += 1024) g[k] = (float)((double)x[k] * inv);
}

// g <- normalise( y - sum_{i<j} sG_i (sG_i . g) ),  y = M^T M g from the thin kernels.
__global__ __launch_bounds__(1024) void k_seq_update(const float* __restrict__ y, const float* __restrict__ sGt, int j,
                                                     float* __restrict__ g, int64_t h, int* __restrict__ flag) {
    __shared__ double coef[DAD_MAX_RANK];
    __shared__ double red[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = wave; i < j; i += 16) {  // one dot product per wave
        double s = 0.0;
        for (int64_t k = lane; k < h; k += 64) s += (double)sGt[(int64_t)i * h + k] * (double)g[k];
        s = wave_sum(s);
        if (lane == 0) coef[i] = s;
    }
    __syncthreads();
    double ss = 0.0;
    for (int64_t k = threadIdx.x; k < h; k += 1024) {
        double v = (double)y[k];
        for (int i = 0; i < j; ++i) v -= coef[i] * (double)sGt[(int64_t)i * h + k];
        g[k] = (float)v;  // the old g is no longer needed: the dot products are done
        ss += v * v;
    }
    ss = block_sum(ss, red);
    if (!(ss > 0.0)) {  // nothing left in this direction (or NaN): latch and leave the vector finite
        if (threadIdx.x == 0) *flag = 1;
        ss = 1.0;
    }
    const float inv = (float)(1.0 / sqrt(ss));
    for (int64_t k = threadIdx.x; k < h; k += 1024) g[k] *= inv;
}

// sigma = ||p||, q = p / sigma, sG = sigma g.
__global__ __launch_bounds__(1024) void k_seq_finish(const float* __restrict__ p, const float* __restrict__ g,
                                                     float* __restrict__ q_row, float* __restrict__ sg_row,
                                                     float* __restrict__ sigma_out, int64_t h_in, int64_t h_out,
                                                     int* __restrict__ flag) {
    __shared__ double red[16];
    double ss = 0.0;
    for (int64_t k = threadIdx.x; k < h_in; k += 1024) ss += (double)p[k] * (double)p[k];
    ss = block_sum(ss, red);
    double sigma = sqrt(ss);
    if (!(sigma > 0.0)) {
        if (threadIdx.x == 0) *flag = 1;
        sigma = 0.0;
    }
    const double inv = sigma > 0.0 ? 1.0 / sigma : 0.0;
    for (int64_t k = threadIdx.x; k < h_in; k += 1024) q_row[k] = (float)((double)p[k] * inv);
    for (int64_t k = threadIdx.x; k < h_out; k += 1024) sg_row[k] = (float)(sigma * (double)g[k]);
    if (sigma_out && threadIdx.x == 0) *sigma_out = (float)sigma;
}

// Rows 1 .. rp-1 of the one-vector panel stay zero for the whole call.
__global__ __launch_bounds__(256) void k_seq_zero(float* __restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// The thin MFMA kernels take ranks that are multiples of 8: the vector travels as row 0 of an 8-row
// panel whose other rows are zero.  The guarded kernels take the single row as it is.
static int seq_panel_rows(int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt) {
    return thin_fast_ok(N, h_in, h_out, 8, dt) ? 8 : 1;
}

struct SeqPlan {
    CompressPlan c;
    int rp;
    size_t off_panel;  // rp x h_out fp32
    size_t total;
};

static SeqPlan plan_sequential(int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt) {
    SeqPlan p;
    p.rp = seq_panel_rows(N, h_in, h_out, dt);
    p.c = plan_compress(N, h_in, h_out, p.rp, dt);
    p.off_panel = align_up(p.c.total, 256);
    p.total = p.off_panel + align_up((size_t)p.rp * h_out * 4, 256);
    return p;
}

}  // namespace dad

using namespace dad;

static bool seq_shape_ok(int64_t N, int64_t h_in, int64_t h_out, int r) {
    if (N < 1 || h_in < 1 || h_out < 1 || r < 1 || r > DAD_MAX_RANK) return false;
    if (r > N || r > h_in || r > h_out) return false;
    return N <= DAD_MAX_ROWS && h_in <= DAD_MAX_WIDTH && h_out <= DAD_MAX_WIDTH;
}

extern "C" size_t dad_compress_sequential_workspace_bytes(int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt) {
    if ((dt != DAD_F32 && dt != DAD_BF16) || !seq_shape_ok(N, h_in, h_out, 1)) return 0;
    return plan_sequential(N, h_in, h_out, dt).total;
}

extern "C" dad_status dad_compress_rank_sequential(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                                   dad_dtype dt, int r, int n_iter, const float* G0, float* Qt,
                                                   float* sGt, float* sigma, void* workspace, size_t ws_bytes,
                                                   void* stream) {
    if (!A || !D || !G0 || !Qt || !sGt || !workspace) return DAD_ERR_NULL;
    if (dt != DAD_F32 && dt != DAD_BF16) return DAD_ERR_DTYPE;
    if (!seq_shape_ok(N, h_in, h_out, r) || n_iter < 1) return DAD_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(D) || !aligned16(G0) || !aligned16(Qt) || !aligned16(sGt) || !aligned16(workspace))
        return DAD_ERR_ALIGN;
    const SeqPlan p = plan_sequential(N, h_in, h_out, dt);
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;

    hipStream_t s = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    int* flag = reinterpret_cast<int*>(ws + p.c.off_flag);
    void* V = ws + p.c.off_V;
    float* part = reinterpret_cast<float*>(ws + p.c.off_part);
    float* Ut = reinterpret_cast<float*>(ws + p.c.off_Ut);   // rp x h_in, row 0 = the vector
    float* Yt = reinterpret_cast<float*>(ws + p.c.off_Yt);   // rp x h_out
    float* panel = reinterpret_cast<float*>(ws + p.off_panel);  // rp x h_out, row 0 = g
    const int rp = p.rp;
    dad_status rc;
#define DAD_TRY(expr)                           \
    do {                                        \
        if ((rc = (expr)) != DAD_OK) return rc; \
    } while (0)
    // planes: the MFMA kernels carry w = A u as two bf16 terms (see dad_compress_rank)
    auto nn = [&](const void* X, const float* P, int64_t h, SplitPlan sp, int planes) {
        return launch_thin_nn(X, P, V, part, sp, N, h, rp, dt, p.c.fast, nullptr, planes, s);
    };
    auto tn = [&](const void* X, float* out, int64_t h, SplitPlan sp, int planes) {
        return launch_thin_tn(X, V, out, part, sp, N, h, rp, dt, p.c.fast, nullptr, planes, s);
    };
    if (rp > 1) {
        const int64_t n = (int64_t)(rp - 1) * h_out;
        ProfScope prof(KID_SEQ_VECTOR, s);
        hipLaunchKernelGGL(k_seq_zero, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, panel + h_out, n);
        DAD_LAUNCH_CHECK();
    }
    for (int j = 0; j < r; ++j) {
        {
            ProfScope prof(KID_SEQ_VECTOR, s);
            hipLaunchKernelGGL(k_seq_start, dim3(1), dim3(1024), 0, s, G0 + (int64_t)j * h_out, panel, h_out, flag,
                               j == 0 ? flag : (int*)nullptr);
        }
        DAD_LAUNCH_CHECK();
        for (int it = 0; it < n_iter; ++it) {
            DAD_TRY(nn(D, panel, h_out, p.c.nn_out, 1));  // v = Delta g
            DAD_TRY(tn(A, Ut, h_in, p.c.tn_in, 1));       // u = A^T v
            DAD_TRY(nn(A, Ut, h_in, p.c.nn_in, 2));       // w = A u
            DAD_TRY(tn(D, Yt, h_out, p.c.tn_out, 2));     // y = Delta^T w = M^T M g
            {
                ProfScope prof(KID_SEQ_VECTOR, s);
                hipLaunchKernelGGL(k_seq_update, dim3(1), dim3(1024), 0, s, Yt, sGt, j, panel, h_out, flag);
            }
            DAD_LAUNCH_CHECK();
        }
        DAD_TRY(nn(D, panel, h_out, p.c.nn_out, 1));  // v = Delta g
        DAD_TRY(tn(A, Ut, h_in, p.c.tn_in, 1));       // p = A^T v
        {
            ProfScope prof(KID_SEQ_VECTOR, s);
            hipLaunchKernelGGL(k_seq_finish, dim3(1), dim3(1024), 0, s, Ut, panel, Qt + (int64_t)j * h_in,
                               sGt + (int64_t)j * h_out, sigma ? sigma + j : (float*)nullptr, h_in, h_out, flag);
        }
        DAD_LAUNCH_CHECK();
    }
#undef DAD_TRY
    return DAD_OK;
}

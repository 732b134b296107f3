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

// Control words of a call, in the 256-byte workspace header (cleared by the first launch):
//   int 0  numeric flag            int 1  skip: the running component needs no further application
//   int 2  done: no further component is wanted (the thin launches that follow return at once)
//   byte 128: double sigma_0
// In the adaptive mode (theta >= 0; Algorithm 2's stop test and the effective rank of Section 3.3.1)
// the found vectors are projected out of the start vector and of every iterate (the projector form of
// Eq. 7's peel); with theta < 0 the peel is the subtraction sum_i sigma_i^2 g_i (g_i . g) and the counts
// are fixed.
constexpr int SEQ_SKIP = 1, SEQ_DONE = 2;

// coef[i] = (sG_i . x) / (sG_i . sG_i) for i < j: the coefficient of the found direction i in x, times
// 1 / sigma_i (the rows of sGt are sigma_i g_i); one dot-product pair per wave.
__device__ __forceinline__ void seq_projection_coefs(const float* __restrict__ sGt, const float* __restrict__ x, int j,
                                                     int64_t h, double* coef) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = wave; i < j; i += 16) {
        double sx = 0.0, ss = 0.0;
        for (int64_t k = lane; k < h; k += 64) {
            const double g = (double)sGt[(int64_t)i * h + k];
            sx += g * (double)x[k];
            ss += g * g;
        }
        sx = wave_sum(sx);
        ss = wave_sum(ss);
        if (lane == 0) coef[i] = ss > 0.0 ? sx / ss : 0.0;
    }
}

// Start of component j: g <- x / ||x||, in the adaptive mode after the found vectors are projected
// out of x.  The first launch of a call also clears the header.
__global__ __launch_bounds__(1024) void k_seq_start(const float* __restrict__ x, const float* __restrict__ sGt, int j,
                                                    float* __restrict__ g, int64_t h, int* __restrict__ hdr,
                                                    int clear_hdr, float theta, int* __restrict__ eff_rank,
                                                    int* __restrict__ iters) {
    __shared__ double red[16];
    __shared__ double coef[DAD_MAX_RANK];
    if (clear_hdr && threadIdx.x < 64) hdr[threadIdx.x] = 0;
    if (clear_hdr && threadIdx.x == 0 && eff_rank) *eff_rank = 0;
    __syncthreads();
    if (iters && threadIdx.x == 0) iters[j] = 0;
    if (hdr[SEQ_DONE]) {  // components are no longer wanted: everything up to the next start is skipped
        if (threadIdx.x == 0) hdr[SEQ_SKIP] = 1;
        return;
    }
    if (threadIdx.x == 0) hdr[SEQ_SKIP] = 0;
    const bool project = theta >= 0.f && j > 0;
    if (project) seq_projection_coefs(sGt, x, j, h, coef);
    __syncthreads();
    double ss = 0.0;
    for (int64_t k = threadIdx.x; k < h; k += 1024) {
        double v = (double)x[k];
        if (project)
            for (int i = 0; i < j; ++i) v -= coef[i] * (double)sGt[(int64_t)i * h + k];
        ss += v * v;
    }
    ss = block_sum(ss, red);
    if (!(ss > 0.0)) {
        if (threadIdx.x == 0) hdr[0] = 1;
        ss = 1.0;
    }
    const double inv = 1.0 / sqrt(ss);
    for (int64_t k = threadIdx.x; k < h; k += 1024) {
        double v = (double)x[k];
        if (project)
            for (int i = 0; i < j; ++i) v -= coef[i] * (double)sGt[(int64_t)i * h + k];
        g[k] = (float)(v * inv);
    }
}

// One application is done: y = M^T M g from the thin kernels.
//   theta < 0 : g <- normalise( y - sum_{i<j} sG_i (sG_i . g) )
//   theta >= 0: y <- y minus its components along the found vectors.  If nothing is left,
//               ||y|| < (theta sigma_0)^2, the gradient's rank is exhausted: done is set and component j
//               is dropped.  Otherwise g <- y / ||y||, and when the step from the old g (sign aligned)
//               is at most theta the remaining applications of this component are skipped.
__global__ __launch_bounds__(1024) void k_seq_update(const float* __restrict__ y, const float* __restrict__ sGt, int j,
                                                     float* __restrict__ g, int64_t h, int* __restrict__ hdr,
                                                     float theta, int* __restrict__ eff_rank, int* __restrict__ iters) {
    __shared__ double coef[DAD_MAX_RANK];
    __shared__ double red[16];
    if (hdr[SEQ_SKIP]) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool adaptive = theta >= 0.f;
    if (adaptive) {
        seq_projection_coefs(sGt, y, j, h, coef);
    } else {
        for (int i = wave; i < j; i += 16) {  // one dot product per wave
            double s = 0.0;
            for (int64_t k = lane; k < h; k += 64) s += (double)sGt[(int64_t)i * h + k] * (double)g[k];
            s = wave_sum(s);
            if (lane == 0) coef[i] = s;
        }
    }
    __syncthreads();
    if (!adaptive) {
        double ss = 0.0;
        for (int64_t k = threadIdx.x; k < h; k += 1024) {
            double v = (double)y[k];
            for (int i = 0; i < j; ++i) v -= coef[i] * (double)sGt[(int64_t)i * h + k];
            g[k] = (float)v;  // the old g is no longer needed: the dot products are done
            ss += v * v;
        }
        ss = block_sum(ss, red);
        if (!(ss > 0.0)) {  // nothing left in this direction (or NaN): latch and leave the vector finite
            if (threadIdx.x == 0) hdr[0] = 1;
            ss = 1.0;
        }
        const float inv = (float)(1.0 / sqrt(ss));
        for (int64_t k = threadIdx.x; k < h; k += 1024) g[k] *= inv;
        return;
    }
    double ss = 0.0, dot = 0.0;
    for (int64_t k = threadIdx.x; k < h; k += 1024) {
        double v = (double)y[k];
        for (int i = 0; i < j; ++i) v -= coef[i] * (double)sGt[(int64_t)i * h + k];
        ss += v * v;
        dot += v * (double)g[k];
    }
    ss = block_sum(ss, red);
    dot = block_sum(dot, red);
    if (threadIdx.x == 0 && iters) iters[j] += 1;
    if (j > 0) {
        const double s0 = *reinterpret_cast<const double*>(reinterpret_cast<const char*>(hdr) + 128);
        const double lim = (double)theta * s0;
        if (sqrt(ss) < lim * lim) {  // nothing left to iterate on
            if (threadIdx.x == 0) {
                hdr[SEQ_SKIP] = 1;
                hdr[SEQ_DONE] = 1;
                if (eff_rank) *eff_rank = j;
            }
            return;
        }
    }
    if (!(ss > 0.0)) {
        if (threadIdx.x == 0) hdr[0] = 1;
        ss = 1.0;
    }
    const double inv = 1.0 / sqrt(ss);
    const double sgn = dot < 0.0 ? -1.0 : 1.0;
    double step2 = 0.0;
    for (int64_t k = threadIdx.x; k < h; k += 1024) {
        double v = (double)y[k];
        for (int i = 0; i < j; ++i) v -= coef[i] * (double)sGt[(int64_t)i * h + k];
        const float gn = (float)(v * inv);
        const double d = sgn * (double)gn - (double)g[k];
        step2 += d * d;
        g[k] = gn;
    }
    step2 = block_sum(step2, red);
    if (threadIdx.x == 0 && sqrt(step2) <= (double)theta) hdr[SEQ_SKIP] = 1;
}

// sigma = ||p||, q = p / sigma, sG = sigma g.  Adaptive mode: a component with sigma < theta sigma_0 is
// dropped and ends the call's iteration; rows of dropped components are zero.
__global__ __launch_bounds__(1024) void k_seq_finish(const float* __restrict__ p, const float* __restrict__ g,
                                                     float* __restrict__ q_row, float* __restrict__ sg_row,
                                                     float* __restrict__ sigma_out, int64_t h_in, int64_t h_out,
                                                     int* __restrict__ hdr, int j, float theta,
                                                     int* __restrict__ eff_rank) {
    __shared__ double red[16];
    double* s0 = reinterpret_cast<double*>(reinterpret_cast<char*>(hdr) + 128);
    bool drop = hdr[SEQ_DONE] != 0;
    double sigma = 0.0;
    if (!drop) {
        double ss = 0.0;
        for (int64_t k = threadIdx.x; k < h_in; k += 1024) ss += (double)p[k] * (double)p[k];
        ss = block_sum(ss, red);
        sigma = sqrt(ss);
        if (theta >= 0.f && j > 0 && sigma < (double)theta * *s0) {
            drop = true;
            __syncthreads();  // every thread has read the flag and sigma_0
            if (threadIdx.x == 0) {
                hdr[SEQ_DONE] = 1;
                if (eff_rank) *eff_rank = j;
            }
        }
    }
    if (drop) {
        for (int64_t k = threadIdx.x; k < h_in; k += 1024) q_row[k] = 0.f;
        for (int64_t k = threadIdx.x; k < h_out; k += 1024) sg_row[k] = 0.f;
        if (sigma_out && threadIdx.x == 0) *sigma_out = 0.f;
        return;
    }
    if (!(sigma > 0.0)) {
        if (threadIdx.x == 0) hdr[0] = 1;
        sigma = 0.0;
    }
    const double inv = sigma > 0.0 ? 1.0 / sigma : 0.0;
    for (int64_t k = threadIdx.x; k < h_in; k += 1024) q_row[k] = (float)((double)p[k] * inv);
    for (int64_t k = threadIdx.x; k < h_out; k += 1024) sg_row[k] = (float)(sigma * (double)g[k]);
    if (threadIdx.x == 0) {
        if (sigma_out) *sigma_out = (float)sigma;
        if (j == 0) *s0 = sigma;
        if (eff_rank) *eff_rank = j + 1;
    }
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

// The launches of the one-vector recurrence; theta < 0: fixed counts, subtraction peel.
static dad_status sequential_launch(const SeqPlan& p, const void* A, const void* D, int64_t N, int64_t h_in,
                                    int64_t h_out, dad_dtype dt, int r, int n_iter, float theta, const float* G0,
                                    float* Qt, float* sGt, float* sigma, int* eff_rank, int* iters, void* workspace,
                                    hipStream_t s) {
    char* ws = static_cast<char*>(workspace);
    int* hdr = reinterpret_cast<int*>(ws + p.c.off_flag);
    void* V = ws + p.c.off_V;
    float* part = reinterpret_cast<float*>(ws + p.c.off_part);
    float* Ut = reinterpret_cast<float*>(ws + p.c.off_Ut);   // rp x h_in, row 0 = the vector
    float* Yt = reinterpret_cast<float*>(ws + p.c.off_Yt);   // rp x h_out
    float* panel = reinterpret_cast<float*>(ws + p.off_panel);  // rp x h_out, row 0 = g
    const int rp = p.rp;
    const bool adaptive = theta >= 0.f;
    // device-side stop flags the thin launches honour (adaptive mode only)
    const int* skip_iter = adaptive ? hdr + SEQ_SKIP : nullptr;
    const int* skip_done = adaptive ? hdr + SEQ_DONE : nullptr;
    dad_status rc;
#define DAD_TRY(expr)                           \
    do {                                        \
        if ((rc = (expr)) != DAD_OK) return rc; \
    } while (0)
    // planes: the MFMA kernels carry w = A u as two bf16 terms (see dad_compress_rank)
    auto nn = [&](const void* X, const float* P, int64_t h, SplitPlan sp, int planes, const int* skip) {
        return launch_thin_nn(X, P, V, part, sp, N, h, rp, dt, p.c.fast, nullptr, planes, s, skip);
    };
    auto tn = [&](const void* X, float* out, int64_t h, SplitPlan sp, int planes, const int* skip) {
        return launch_thin_tn(X, V, out, part, sp, N, h, rp, dt, p.c.fast, nullptr, planes, s, skip);
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
            hipLaunchKernelGGL(k_seq_start, dim3(1), dim3(1024), 0, s, G0 + (int64_t)j * h_out, (const float*)sGt, j, panel,
                               h_out, hdr, j == 0 ? 1 : 0, theta, eff_rank, iters);
        }
        DAD_LAUNCH_CHECK();
        for (int it = 0; it < n_iter; ++it) {
            DAD_TRY(nn(D, panel, h_out, p.c.nn_out, 1, skip_iter));  // v = Delta g
            DAD_TRY(tn(A, Ut, h_in, p.c.tn_in, 1, skip_iter));       // u = A^T v
            DAD_TRY(nn(A, Ut, h_in, p.c.nn_in, 2, skip_iter));       // w = A u
            DAD_TRY(tn(D, Yt, h_out, p.c.tn_out, 2, skip_iter));     // y = Delta^T w = M^T M g
            {
                ProfScope prof(KID_SEQ_VECTOR, s);
                hipLaunchKernelGGL(k_seq_update, dim3(1), dim3(1024), 0, s, (const float*)Yt, (const float*)sGt, j, panel,
                                   h_out, hdr, theta, eff_rank, iters);
            }
            DAD_LAUNCH_CHECK();
        }
        DAD_TRY(nn(D, panel, h_out, p.c.nn_out, 1, skip_done));  // v = Delta g
        DAD_TRY(tn(A, Ut, h_in, p.c.tn_in, 1, skip_done));       // p = A^T v
        {
            ProfScope prof(KID_SEQ_VECTOR, s);
            hipLaunchKernelGGL(k_seq_finish, dim3(1), dim3(1024), 0, s, (const float*)Ut, (const float*)panel,
                               Qt + (int64_t)j * h_in, sGt + (int64_t)j * h_out, sigma ? sigma + j : (float*)nullptr, h_in,
                               h_out, hdr, j, theta, eff_rank);
        }
        DAD_LAUNCH_CHECK();
    }
#undef DAD_TRY
    return DAD_OK;
}

static dad_status sequential_args_ok(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt,
                                     int r, int n_iter, const float* G0, const float* Qt, const float* sGt,
                                     const void* workspace) {
    if (!A || !D || !G0 || !Qt || !sGt || !workspace) return DAD_ERR_NULL;
    if (dt != DAD_F32 && dt != DAD_BF16) return DAD_ERR_DTYPE;
    if (!seq_shape_ok(N, h_in, h_out, r) || n_iter < 1) return DAD_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(D) || !aligned16(G0) || !aligned16(Qt) || !aligned16(sGt) || !aligned16(workspace))
        return DAD_ERR_ALIGN;
    return DAD_OK;
}

extern "C" dad_status dad_compress_rank_sequential(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                                   dad_dtype dt, int r, int n_iter, const float* G0, float* Qt,
                                                   float* sGt, float* sigma, void* workspace, size_t ws_bytes,
                                                   void* stream) {
    dad_status rc = sequential_args_ok(A, D, N, h_in, h_out, dt, r, n_iter, G0, Qt, sGt, workspace);
    if (rc != DAD_OK) return rc;
    const SeqPlan p = plan_sequential(N, h_in, h_out, dt);
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if ((rc = device_ready()) != DAD_OK) return rc;
    return sequential_launch(p, A, D, N, h_in, h_out, dt, r, n_iter, -1.f, G0, Qt, sGt, sigma, nullptr, nullptr, workspace,
                             (hipStream_t)stream);
}

extern "C" dad_status dad_compress_rank_adaptive(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                                 dad_dtype dt, int r, int max_iter, float theta, const float* G0,
                                                 float* Qt, float* sGt, float* sigma, int* effective_rank,
                                                 int* iterations, void* workspace, size_t ws_bytes, void* stream) {
    dad_status rc = sequential_args_ok(A, D, N, h_in, h_out, dt, r, max_iter, G0, Qt, sGt, workspace);
    if (rc != DAD_OK) return rc;
    if (!effective_rank) return DAD_ERR_NULL;
    if (!(theta >= 0.f) || !(theta < 1.f)) return DAD_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(effective_rank) & 3u) || (reinterpret_cast<uintptr_t>(iterations) & 3u))
        return DAD_ERR_ALIGN;
    const SeqPlan p = plan_sequential(N, h_in, h_out, dt);
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if ((rc = device_ready()) != DAD_OK) return rc;
    return sequential_launch(p, A, D, N, h_in, h_out, dt, r, max_iter, theta, G0, Qt, sGt, sigma, effective_rank,
                             iterations, workspace, (hipStream_t)stream);
}

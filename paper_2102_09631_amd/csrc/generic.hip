// Guarded LDS-tiled kernels that accept any shape and either element type.
// They serve the shapes the MFMA kernels do not take (ragged widths, fp32
// factors) and compute the same contractions with fp32 FMA.
#include "dad_internal.h"

namespace dad {

// ---------------------------------------------------------------- thin N x h by h x r
// out[n][j] = sum_k X[n][k] * Pt[j][k]   (V = Delta G and W = A U of Eq. 6); the N x r result is fp32
// whatever the factors' element type.
// With few rows (the N << h case) the contraction is also split over column chunks of `kchunk`
// (blockIdx.y); each chunk then writes an fp32 slab part[chunk][n][j] for reduce_slabs.
// MA = accumulators per thread (columns jg, jg+4, ...): 4, 8 or 16 for r <= 16, 32, 64.
template <typename T, int MA>
__global__ __launch_bounds__(256) void k_thin_nn(const T* __restrict__ X, const float* __restrict__ Pt,
                                                 float* __restrict__ out, float* __restrict__ part, int64_t N, int64_t h,
                                                 int r, int64_t kchunk, int* __restrict__ zero_hdr,
                                                 const int* __restrict__ skip) {
    if (skip && *skip) return;  // the caller's device-side stop flag is set: nothing to do
    // the first launch of a compress call also clears the workspace header (flag, ticket counter)
    if (zero_hdr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 64) zero_hdr[threadIdx.x] = 0;
    constexpr int ROWS = 64, KC = 32;
    __shared__ float Xs[ROWS][KC + 1];
    __shared__ float Ps[DAD_MAX_RANK][KC + 1];
    const int t = threadIdx.x;
    const int row = t & 63, jg = t >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * ROWS;
    float acc[MA];
#pragma unroll
    for (int m = 0; m < MA; ++m) acc[m] = 0.f;

    const int64_t kbeg = (int64_t)blockIdx.y * kchunk;
    const int64_t kend = (kbeg + kchunk < h) ? kbeg + kchunk : h;
    // Tiles travel global -> registers -> LDS.  Every load has a valid (clamped) address and its value
    // is selected only at the LDS store, so that the loads of a tile go out together, and the next
    // tile's loads are in flight while the current one is multiplied.
    constexpr int XL = ROWS * KC / 256, PL = MA / 2;  // r <= 4 MA, so r * KC / 256 <= MA / 2
    float xr[XL], pr[PL];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int m = 0; m < XL; ++m) {
            const int e = t + 256 * m, rr = e / KC, kk = e % KC;
            const int64_t n = n0 + rr < N ? n0 + rr : N - 1, k = k0 + kk < kend ? k0 + kk : kend - 1;
            xr[m] = ld<T>(X, n * h + k);
        }
#pragma unroll
        for (int m = 0; m < PL; ++m) {
            const int e = t + 256 * m, j = e / KC < r ? e / KC : r - 1, kk = e % KC;
            const int64_t k = k0 + kk < kend ? k0 + kk : kend - 1;
            pr[m] = Pt[(int64_t)j * h + k];
        }
    };
    auto commit = [&](int64_t k0) {
#pragma unroll
        for (int m = 0; m < XL; ++m) {
            const int e = t + 256 * m, rr = e / KC, kk = e % KC;
            Xs[rr][kk] = (n0 + rr < N && k0 + kk < kend) ? xr[m] : 0.f;
        }
#pragma unroll
        for (int m = 0; m < PL; ++m) {
            const int e = t + 256 * m, j = e / KC, kk = e % KC;
            if (j < r) Ps[j][kk] = (k0 + kk < kend) ? pr[m] : 0.f;
        }
    };
    fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += KC) {
        commit(k0);
        __syncthreads();
        if (k0 + KC < kend) fetch(k0 + KC);
        // rows of Ps beyond r are never written: their products land in accumulators nobody stores
#pragma unroll 8
        for (int kk = 0; kk < KC; ++kk) {
            const float x = Xs[row][kk];
#pragma unroll
            for (int m = 0; m < MA; ++m) acc[m] = fmaf(x, Ps[jg + 4 * m][kk], acc[m]);
        }
        __syncthreads();
    }
    const int64_t n = n0 + row;
    if (n < N) {
#pragma unroll
        for (int m = 0; m < MA; ++m) {
            int j = jg + 4 * m;
            if (j < r) {
                if (part)
                    part[((int64_t)blockIdx.y * N + n) * r + j] = acc[m];
                else
                    out[n * r + j] = acc[m];
            }
        }
    }
}

// ---------------------------------------------------------------- thin (N x h)^T by N x r, split over rows
// part[s][j][p] = sum_{n in chunk s} X[n][p] * V[n][j]    (U = A^T V, Y = Delta^T W, P = A^T V); V is fp32
template <typename T, int MA>
__global__ __launch_bounds__(256) void k_thin_tn(const T* __restrict__ X, const float* __restrict__ V,
                                                 float* __restrict__ part, int64_t N, int64_t h, int r,
                                                 int64_t chunk, const int* __restrict__ skip) {
    if (skip && *skip) return;
    constexpr int PW = 64, RC = 32;
    __shared__ float Xs[RC][PW];
    __shared__ float Vs[RC][DAD_MAX_RANK];
    const int t = threadIdx.x;
    const int pl = t & 63, jg = t >> 6;
    const int64_t p0 = (int64_t)blockIdx.x * PW;
    const int64_t nbeg = (int64_t)blockIdx.y * chunk;
    const int64_t nend = (nbeg + chunk < N) ? nbeg + chunk : N;
    float acc[MA];
#pragma unroll
    for (int m = 0; m < MA; ++m) acc[m] = 0.f;

    // global -> registers -> LDS with clamped addresses, the next tile in flight during the arithmetic
    // (see k_thin_nn)
    constexpr int XL = RC * PW / 256, VL = MA / 2;  // r <= 4 MA, so RC * r / 256 <= MA / 2
    float xr[XL], vr[VL];
    auto fetch = [&](int64_t n0) {
#pragma unroll
        for (int m = 0; m < XL; ++m) {
            const int e = t + 256 * m, rr = e / PW, pp = e % PW;
            const int64_t n = n0 + rr < nend ? n0 + rr : nend - 1, p = p0 + pp < h ? p0 + pp : h - 1;
            xr[m] = ld<T>(X, n * h + p);
        }
#pragma unroll
        for (int m = 0; m < VL; ++m) {
            const int e = t + 256 * m < RC * r ? t + 256 * m : RC * r - 1, rr = e / r, j = e % r;
            const int64_t n = n0 + rr < nend ? n0 + rr : nend - 1;
            vr[m] = V[n * r + j];
        }
    };
    auto commit = [&](int64_t n0) {
#pragma unroll
        for (int m = 0; m < XL; ++m) {
            const int e = t + 256 * m, rr = e / PW, pp = e % PW;
            Xs[rr][pp] = (n0 + rr < nend && p0 + pp < h) ? xr[m] : 0.f;
        }
#pragma unroll
        for (int m = 0; m < VL; ++m) {
            const int e = t + 256 * m, rr = e / r, j = e % r;
            if (e < RC * r) Vs[rr][j] = (n0 + rr < nend) ? vr[m] : 0.f;
        }
    };
    fetch(nbeg);
    for (int64_t n0 = nbeg; n0 < nend; n0 += RC) {
        commit(n0);
        __syncthreads();
        if (n0 + RC < nend) fetch(n0 + RC);
#pragma unroll 8
        for (int rr = 0; rr < RC; ++rr) {
            const float x = Xs[rr][pl];
#pragma unroll
            for (int m = 0; m < MA; ++m) acc[m] = fmaf(x, Vs[rr][jg + 4 * m], acc[m]);
        }
        __syncthreads();
    }
    const int64_t p = p0 + pl;
    if (p < h) {
#pragma unroll
        for (int m = 0; m < MA; ++m) {
            int j = jg + 4 * m;
            if (j < r) part[((int64_t)blockIdx.y * r + j) * h + p] = acc[m];
        }
    }
}

// out[i] = sum_s part[s*n + i] in a fixed order, so reruns are bit-identical.
// Small slabs (the r x h panels of the power iteration): latency bound, so the splits of one
// element are shared by the four waves of a workgroup (wave g sums s = g, g+4, ... ascending) and
// the four partial sums are combined in wave order.
// blockIdx.y: job of a batch, its pointers job_stride bytes further per job.
__global__ __launch_bounds__(256) void k_reduce_slabs(const float* part, float* out, int64_t n, int splits,
                                                      bf16_t* __restrict__ out_bf16, const int* __restrict__ skip,
                                                      int64_t job_stride, BatchInts dims, int use_dims) {
    if (skip && *skip) return;
    if (job_stride != 0) {
        if (use_dims) {  // this job's own size and slab count
            n = dims.a[blockIdx.y];
            splits = dims.b[blockIdx.y];
            if ((int64_t)blockIdx.x * 64 >= n) return;
        }
        const int64_t off = blockIdx.y * job_stride;
        part = reinterpret_cast<const float*>(reinterpret_cast<const char*>(part) + off);
        out = reinterpret_cast<float*>(reinterpret_cast<char*>(out) + off);
        if (out_bf16) out_bf16 = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(out_bf16) + off);
    }
    __shared__ float ps[4][64];
    const int e = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + e;
    float a = 0.f;
    if (i < n) {
        int s = g;
        for (; s + 28 < splits; s += 32) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(s + 4 * u) * n + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) a += v[u];
        }
        for (; s < splits; s += 4) a += part[(int64_t)s * n + i];
    }
    ps[g][e] = a;
    __syncthreads();
    if (g == 0 && i < n) {
        const float v = ((ps[0][e] + ps[1][e]) + ps[2][e]) + ps[3][e];
        out[i] = v;
        if (out_bf16) out_bf16[i] = f32_to_bf16(v);  // panel of the next thin_nn
    }
}

// Large slabs (split-K partials of the gradient rebuild): bandwidth bound, 16 bytes per thread.
__global__ __launch_bounds__(256) void k_reduce_slabs_wide(const float4* __restrict__ part, float4* __restrict__ out,
                                                           int64_t n4, int splits) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float4 a = part[i];
    for (int s = 1; s < splits; ++s) {
        const float4 v = part[(int64_t)s * n4 + i];
        a.x += v.x;
        a.y += v.y;
        a.z += v.z;
        a.w += v.w;
    }
    out[i] = a;
}

// ---------------------------------------------------------------- G = L^T R, 64 x 64 tiles, split over K
template <typename T>
__global__ __launch_bounds__(256) void k_rebuild(const T* __restrict__ L, const T* __restrict__ R,
                                                 float* __restrict__ out, int64_t K, int64_t h_in,
                                                 int64_t h_out, int64_t chunk) {
    constexpr int TM = 64, KC = 16;
    __shared__ float Ls[KC][TM];
    __shared__ float Rs[KC][TM];
    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;
    const int64_t q0 = (int64_t)blockIdx.x * TM, p0 = (int64_t)blockIdx.y * TM;
    const int64_t kbeg = (int64_t)blockIdx.z * chunk;
    const int64_t kend = (kbeg + chunk < K) ? kbeg + chunk : K;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

    // global -> registers -> LDS with clamped addresses, the next tile in flight during the arithmetic
    // (see k_thin_nn)
    constexpr int TL = KC * TM / 256;
    float lr[TL], rr_[TL];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int m = 0; m < TL; ++m) {
            const int e = t + 256 * m, kk = e / TM, c = e % TM;
            const int64_t k = k0 + kk < kend ? k0 + kk : kend - 1;
            lr[m] = ld<T>(L, k * h_in + (p0 + c < h_in ? p0 + c : h_in - 1));
            rr_[m] = ld<T>(R, k * h_out + (q0 + c < h_out ? q0 + c : h_out - 1));
        }
    };
    auto commit = [&](int64_t k0) {
#pragma unroll
        for (int m = 0; m < TL; ++m) {
            const int e = t + 256 * m, kk = e / TM, c = e % TM;
            const bool kin = k0 + kk < kend;
            Ls[kk][c] = (kin && p0 + c < h_in) ? lr[m] : 0.f;
            Rs[kk][c] = (kin && q0 + c < h_out) ? rr_[m] : 0.f;
        }
    };
    fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += KC) {
        commit(k0);
        __syncthreads();
        if (k0 + KC < kend) fetch(k0 + KC);
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
            float lv[4], rv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) lv[a] = Ls[kk][ty * 4 + a];
#pragma unroll
            for (int b = 0; b < 4; ++b) rv[b] = Rs[kk][tx * 4 + b];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(lv[a], rv[b], acc[a][b]);
        }
        __syncthreads();
    }
    float* o = out + (int64_t)blockIdx.z * h_in * h_out;
    const int64_t qb = q0 + tx * 4;
    const bool vec = (h_out & 3) == 0 && qb + 3 < h_out;  // rows stay 16-byte aligned: one store per row
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        int64_t p = p0 + ty * 4 + a;
        if (p >= h_in) continue;
        if (vec) {
            typedef float f4 __attribute__((ext_vector_type(4)));
            *reinterpret_cast<f4*>(o + p * h_out + qb) = f4{acc[a][0], acc[a][1], acc[a][2], acc[a][3]};
            continue;
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            int64_t q = qb + b;
            if (q < h_out) o[p * h_out + q] = acc[a][b];
        }
    }
}


// ---------------------------------------------------------------- host launchers

// Column split of the guarded thin_nn: with fewer than 128 row blocks the contraction is cut into
// chunks so that a few hundred workgroups run.
SplitPlan gen_thin_nn_split(int64_t N, int64_t h) {
    const int64_t rowblocks = ceil_div(N, 64);
    int64_t want = rowblocks >= 128 ? 1 : ceil_div(256, rowblocks);
    const int64_t cap = ceil_div(h, 64);
    if (want > cap) want = cap;
    SplitPlan sp;
    sp.chunk = (int64_t)align_up((size_t)ceil_div(h, want), 32);
    sp.splits = (int)ceil_div(h, sp.chunk);
    return sp;
}

dad_status gen_thin_nn(const void* X, const float* Pt, void* out, float* partials, SplitPlan sp, int64_t N, int64_t h,
                       int r, dad_dtype dt, int* zero_hdr, hipStream_t s, const int* skip) {
    dim3 grid((unsigned)ceil_div(N, 64), (unsigned)sp.splits);
    float* part = sp.splits == 1 ? nullptr : partials;
    {
        ProfScope prof(KID_THIN_NN, s);
#define DAD_GEN_NN(MA)                                                                                              \
    do {                                                                                                            \
        if (dt == DAD_BF16)                                                                                         \
            hipLaunchKernelGGL((k_thin_nn<bf16_t, MA>), grid, dim3(256), 0, s, (const bf16_t*)X, Pt, (float*)out, part, N, \
                               h, r, sp.chunk, zero_hdr, skip);                                                           \
        else                                                                                                        \
            hipLaunchKernelGGL((k_thin_nn<float, MA>), grid, dim3(256), 0, s, (const float*)X, Pt, (float*)out, part, N, h, \
                               r, sp.chunk, zero_hdr, skip);                                                              \
    } while (0)
        if (r <= 16) DAD_GEN_NN(4);
        else if (r <= 32) DAD_GEN_NN(8);
        else DAD_GEN_NN(16);
#undef DAD_GEN_NN
    }
    DAD_LAUNCH_CHECK();
    if (sp.splits == 1) return DAD_OK;
    return reduce_slabs(part, (float*)out, N * r, sp.splits, s, nullptr, skip);
}

bool reduce_slabs_is_wide(int64_t n, bool with_bf16, bool with_skip) {
    return n >= (1 << 20) && n % 4 == 0 && !with_bf16 && !with_skip;
}

dad_status reduce_slabs(const float* part, float* out, int64_t n, int splits, hipStream_t s, void* out_bf16,
                        const int* skip, int jobs, int64_t job_stride, const BatchInts* dims) {
    const bool wide = reduce_slabs_is_wide(n, out_bf16 != nullptr, skip != nullptr);
    if (job_stride == 0) jobs = 1;
    if (wide && jobs > 1) return DAD_ERR_SHAPE;  // batches are formed only of sums the small kernel takes
    ProfScope prof(wide ? KID_REDUCE_WIDE : KID_REDUCE, s);
    if (wide)
        hipLaunchKernelGGL(k_reduce_slabs_wide, dim3((unsigned)ceil_div(n / 4, 256)), dim3(256), 0, s,
                           reinterpret_cast<const float4*>(part), reinterpret_cast<float4*>(out), n / 4, splits);
    else
        hipLaunchKernelGGL(k_reduce_slabs, dim3((unsigned)ceil_div(n, 64), (unsigned)jobs), dim3(256), 0, s, part, out, n,
                           splits, (bf16_t*)out_bf16, skip, job_stride, dims ? *dims : BatchInts{}, dims ? 1 : 0);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

dad_status gen_thin_tn(const void* X, const void* V, float* out_t, float* partials, SplitPlan sp, int64_t N,
                       int64_t h, int r, dad_dtype dt, hipStream_t s, const int* skip) {
    dim3 grid((unsigned)ceil_div(h, 64), (unsigned)sp.splits);
    float* dst = sp.splits == 1 ? out_t : partials;
    {
    ProfScope prof(KID_THIN_TN, s);
#define DAD_GEN_TN(MA)                                                                                              \
    do {                                                                                                            \
        if (dt == DAD_BF16)                                                                                         \
            hipLaunchKernelGGL((k_thin_tn<bf16_t, MA>), grid, dim3(256), 0, s, (const bf16_t*)X, (const float*)V, dst, N, \
                               h, r, sp.chunk, skip);                                                               \
        else                                                                                                        \
            hipLaunchKernelGGL((k_thin_tn<float, MA>), grid, dim3(256), 0, s, (const float*)X, (const float*)V, dst, N, h, \
                               r, sp.chunk, skip);                                                                  \
    } while (0)
    if (r <= 16) DAD_GEN_TN(4);
    else if (r <= 32) DAD_GEN_TN(8);
    else DAD_GEN_TN(16);
#undef DAD_GEN_TN
    }
    DAD_LAUNCH_CHECK();
    if (sp.splits > 1) return reduce_slabs(partials, out_t, (int64_t)r * h, sp.splits, s, nullptr, skip);
    return DAD_OK;
}

dad_status gen_rebuild(const void* L, const void* R, int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt, float* G,
                       float* partials, SplitPlan sp, hipStream_t s) {
    dim3 grid((unsigned)ceil_div(h_out, 64), (unsigned)ceil_div(h_in, 64), (unsigned)sp.splits);
    float* dst = sp.splits == 1 ? G : partials;
    {
    ProfScope prof(KID_REBUILD, s);
    if (dt == DAD_BF16)
        hipLaunchKernelGGL(k_rebuild<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)L, (const bf16_t*)R, dst, K,
                           h_in, h_out, sp.chunk);
    else
        hipLaunchKernelGGL(k_rebuild<float>, grid, dim3(256), 0, s, (const float*)L, (const float*)R, dst, K, h_in,
                           h_out, sp.chunk);
    }
    DAD_LAUNCH_CHECK();
    if (sp.splits > 1) return reduce_slabs(partials, G, h_in * h_out, sp.splits, s);
    return DAD_OK;
}


}  // namespace dad

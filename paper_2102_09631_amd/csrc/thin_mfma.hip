// The two thin contractions of the structured power iteration (Algorithm 2, Eq. 6) for bf16
// factors.  Both stream a factor matrix X (N x h) once from HBM and are bandwidth bound; the
// matrix cores only do the arithmetic.
//
//   thin_nn : V[n][j]   = sum_k X[n][k] * Pt[j][k]       (V = Delta G,  W = A U)
//   thin_tn : Ot[j][p]  = sum_n V[n][j] * X[n][p]        (U = A^T V, Y = Delta^T W, P = A^T V)
//
// Loads run two tiles ahead of the arithmetic through two register sets, so each workgroup keeps
// about 40 KiB of HBM reads in flight.
#include "dad_internal.h"

namespace dad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

// ------------------------------------------------------------------------------------------------
// thin_nn
// ------------------------------------------------------------------------------------------------
namespace nn {
constexpr int RT = 128;             // rows of X per workgroup (32 per wave)
constexpr int BK = 64;              // contraction columns per stage (128 B of each row)
constexpr int XROWB = BK * 2 + 16;  // padded LDS row, bytes
constexpr int XTILEB = RT * XROWB;
}  // namespace nn

template <int RP>  // RP = r rounded up to 32 or 64
__global__ __launch_bounds__(256) void k_thin_nn_bf16(const bf16_t* __restrict__ X, const float* __restrict__ Pt,
                                                      bf16_t* __restrict__ V, int64_t N, int h, int r,
                                                      int* __restrict__ zero_hdr) {
    // the first launch of a compress call also clears the workspace header (flag, ticket counter)
    if (zero_hdr && blockIdx.x == 0 && threadIdx.x < 64) zero_hdr[threadIdx.x] = 0;
    constexpr int JT = RP / 32;
    constexpr int PLOADS = RP * nn::BK / 4 / 256;  // float4 loads of Pt per thread per stage
    constexpr int PTILEB = RP * nn::XROWB;
    constexpr int STAGEB = nn::XTILEB + PTILEB;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t n0 = (int64_t)blockIdx.x * nn::RT;
    const int nk = (h + nn::BK - 1) / nn::BK;
    // Every workgroup walks the contraction columns from its own starting stage (and wraps): at any
    // instant the workgroups then touch different column offsets of their rows, which spreads the
    // 128-byte row pieces over the memory channels instead of piling onto the few channels that one
    // common offset maps to when the row pitch is a large power of two.
    const int rot = (int)((blockIdx.x * 5u) % (unsigned)nk);

    // X staging: thread owns 16-byte chunk xc of rows xr + 32*i
    const int xc = t & 7, xr = t >> 3;
    // Pt staging: thread owns floats [4*pc, 4*pc+4) of rows pr + 16*i
    const int pc = t & 15, pr = t >> 4;

    u32x4 xs[2][4];
    f32x4 ps[2][PLOADS];

    auto gload = [&](int kt, int set) {
        int ktr = kt + rot;
        if (ktr >= nk) ktr -= nk;
        const int k0 = ktr * nn::BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t n = n0 + xr + 32 * i;
            const int k = k0 + xc * 8;
            if (n < N && k < h)
                xs[set][i] = *reinterpret_cast<const u32x4*>(X + n * h + k);
            else
                xs[set][i] = (u32x4){0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < PLOADS; ++i) {
            const int j = pr + 16 * i, k = k0 + pc * 4;
            if (j < r && k < h)
                ps[set][i] = *reinterpret_cast<const f32x4*>(Pt + (int64_t)j * h + k);
            else
                ps[set][i] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    };
    auto lstore = [&](int stage, int set) {
        char* xb = smem + stage * STAGEB;
        char* pb = xb + nn::XTILEB;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(xb + (xr + 32 * i) * nn::XROWB + xc * 16) = xs[set][i];
#pragma unroll
        for (int i = 0; i < PLOADS; ++i) {
            u32x2 w;
            w.x = pack_bf16x2(ps[set][i].x, ps[set][i].y);
            w.y = pack_bf16x2(ps[set][i].z, ps[set][i].w);
            *reinterpret_cast<u32x2*>(pb + (pr + 16 * i) * nn::XROWB + pc * 8) = w;
        }
    };

    f32x16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    auto compute = [&](int stage) {
        const char* xb = smem + stage * STAGEB;
        const char* pb = xb + nn::XTILEB;
        const int row = wave * 32 + (lane & 31), kq = (lane >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < nn::BK / 16; ++ks) {
            bf16x8 fa = *reinterpret_cast<const bf16x8*>(xb + row * nn::XROWB + ks * 32 + kq);
#pragma unroll
            for (int j = 0; j < JT; ++j) {
                bf16x8 fb = *reinterpret_cast<const bf16x8*>(pb + (j * 32 + (lane & 31)) * nn::XROWB + ks * 32 + kq);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[j], 0, 0, 0);
            }
        }
    };

    // software pipeline: LDS stage kt&1 holds tile kt, set (kt+1)&1 holds tile kt+1, the other tile kt+2
    gload(0, 0);
    lstore(0, 0);
    if (nk > 1) gload(1, 1);
    if (nk > 2) gload(2, 0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
        compute(0);
        if (kt + 1 < nk) {
            lstore(1, 1);
            if (kt + 3 < nk) gload(kt + 3, 1);
        }
        __syncthreads();
        if (kt + 1 < nk) {
            compute(1);
            if (kt + 2 < nk) {
                lstore(0, 0);
                if (kt + 4 < nk) gload(kt + 4, 0);
            }
            __syncthreads();
        }
    }

    // epilogue: fp32 -> bf16 through LDS so the tile leaves as contiguous 16-byte stores
    bf16_t* vs = reinterpret_cast<bf16_t*>(smem);  // [RT][r]
#pragma unroll
    for (int j = 0; j < JT; ++j) {
        const int col = j * 32 + (lane & 31);
        if (col < r) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wave * 32 + ((v >> 2) << 3) + ((lane >> 5) << 2) + (v & 3);
                vs[row * r + col] = f32_to_bf16(acc[j][v]);
            }
        }
    }
    __syncthreads();
    const int64_t rows_here = (N - n0 < nn::RT) ? (N - n0) : nn::RT;
    const int chunks = (int)(rows_here * r / 8);  // r % 8 == 0
    u32x4* dst = reinterpret_cast<u32x4*>(V + n0 * r);
    const u32x4* src = reinterpret_cast<const u32x4*>(vs);
    for (int e = t; e < chunks; e += 256) dst[e] = src[e];
}

// ------------------------------------------------------------------------------------------------
// thin_tn
// ------------------------------------------------------------------------------------------------
namespace tn {
constexpr int PW = 128;            // columns of X per workgroup (32 per wave)
constexpr int BK = 64;             // rows per stage
constexpr int XROWB = PW * 2;      // LDS row of the X tile, 16 chunks, XOR-swizzled
constexpr int XTILEB = BK * XROWB;
}  // namespace tn

__device__ __forceinline__ int tn_x_off(int k, int chunk) { return k * tn::XROWB + ((chunk ^ ((k & 3) << 2)) << 4); }

// Eight K-consecutive values of column m0 + lane%32 from a [k][col] tile with row pitch `rowb`;
// SWZ selects the XOR swizzle of the X tile.
template <bool SWZ>
__device__ __forceinline__ bf16x8 tn_frag(const char* tile, int rowb, int m0, int kb, int lane) {
    const int b = lane >> 4, s = lane & 15, j = s >> 2, g = s & 3;
    const int m = m0 + ((b & 1) << 4) + (g << 2);
    const int k = kb + ((b >> 1) << 3) + j;
    int chunk = m >> 3;
    if (SWZ) chunk ^= (j << 2);  // (k & 3) == j for both reads
    const char* p0 = tile + k * rowb + (chunk << 4) + ((g & 1) << 3);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0 + 4 * rowb));
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int RP>
__global__ __launch_bounds__(256) void k_thin_tn_bf16(const bf16_t* __restrict__ X, const bf16_t* __restrict__ V,
                                                      float* __restrict__ part, int64_t N, int h, int r,
                                                      int64_t chunk_rows) {
    constexpr int JT = RP / 32;
    constexpr int VROWB = RP * 2;
    constexpr int VTILEB = tn::BK * VROWB;
    constexpr int STAGEB = tn::XTILEB + VTILEB;
    constexpr int VLOADS = (tn::BK * RP / 8 + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int p0 = blockIdx.x * tn::PW;
    const int64_t nbeg = (int64_t)blockIdx.y * chunk_rows;
    const int64_t nend = (nbeg + chunk_rows < N) ? nbeg + chunk_rows : N;
    const int nk = (int)((nend - nbeg + tn::BK - 1) / tn::BK);
    const int rc = r >> 3;  // 16-byte chunks per V row

    // X staging: chunk xc of rows xr + 16*i ; (xr + 16*i) & 3 == xr & 3
    const int xc = t & 15, xr = t >> 4;
    const int x_st = tn_x_off(xr, xc);

    u32x4 xs[2][4];
    u32x4 vsr[2][VLOADS];

    auto gload = [&](int kt, int set) {
        const int64_t kb = nbeg + (int64_t)kt * tn::BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t n = kb + xr + 16 * i;
            if (n < nend)
                xs[set][i] = *reinterpret_cast<const u32x4*>(X + n * h + p0 + xc * 8);
            else
                xs[set][i] = (u32x4){0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < VLOADS; ++i) {
            const int e = t + 256 * i;
            const int row = e / rc, c = e - row * rc;
            const int64_t n = kb + row;
            if (row < tn::BK && n < nend)
                vsr[set][i] = *reinterpret_cast<const u32x4*>(V + n * r + c * 8);
            else
                vsr[set][i] = (u32x4){0, 0, 0, 0};
        }
    };
    auto lstore = [&](int stage, int set) {
        char* xb = smem + stage * STAGEB;
        char* vb = xb + tn::XTILEB;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(xb + x_st + 16 * i * tn::XROWB) = xs[set][i];
#pragma unroll
        for (int i = 0; i < VLOADS; ++i) {
            const int e = t + 256 * i;
            const int row = e / rc, c = e - row * rc;
            if (row < tn::BK) *reinterpret_cast<u32x4*>(vb + row * VROWB + c * 16) = vsr[set][i];
        }
    };

    // columns r..RP-1 of both V tiles stay zero for the whole kernel
    if (r < RP) {
        for (int e = t; e < 2 * tn::BK * RP / 8; e += 256) {
            const int stage = e / (tn::BK * RP / 8), rem = e - stage * (tn::BK * RP / 8);
            const int row = rem / (RP / 8), c = rem - row * (RP / 8);
            if (c >= rc)
                *reinterpret_cast<u32x4*>(smem + stage * STAGEB + tn::XTILEB + row * VROWB + c * 16) = (u32x4){0, 0, 0, 0};
        }
    }

    f32x16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    auto compute = [&](int stage) {
        const char* xb = smem + stage * STAGEB;
        const char* vb = xb + tn::XTILEB;
#pragma unroll
        for (int ks = 0; ks < tn::BK / 16; ++ks) {
            bf16x8 fx = tn_frag<true>(xb, tn::XROWB, wave * 32, ks * 16, lane);
#pragma unroll
            for (int j = 0; j < JT; ++j) {
                bf16x8 fv = tn_frag<false>(vb, VROWB, j * 32, ks * 16, lane);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv, fx, acc[j], 0, 0, 0);
            }
        }
    };

    gload(0, 0);
    lstore(0, 0);
    if (nk > 1) gload(1, 1);
    if (nk > 2) gload(2, 0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
        compute(0);
        if (kt + 1 < nk) {
            lstore(1, 1);
            if (kt + 3 < nk) gload(kt + 3, 1);
        }
        __syncthreads();
        if (kt + 1 < nk) {
            compute(1);
            if (kt + 2 < nk) {
                lstore(0, 0);
                if (kt + 4 < nk) gload(kt + 4, 0);
            }
            __syncthreads();
        }
    }

    // D[j][p]: lane holds column p = p0 + wave*32 + lane%32, rows j = jt*32 + 8*(v/4) + 4*(lane/32) + v%4
    float* o = part + (int64_t)blockIdx.y * r * h;
    const int p = p0 + wave * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = j * 32 + ((v >> 2) << 3) + ((lane >> 5) << 2) + (v & 3);
            if (row < r) o[(int64_t)row * h + p] = acc[j][v];
        }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
dad_status reduce_slabs(const float* part, float* out, int64_t n, int splits, hipStream_t s);

bool thin_fast_ok(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt) {
    return dt == DAD_BF16 && r % 8 == 0 && h_in % tn::PW == 0 && h_out % tn::PW == 0 && N >= 256 &&
           h_in <= (1 << 20) && h_out <= (1 << 20);
}

// Row split of thin_tn: enough workgroups to fill the chip twice over, while the fp32 partials
// (splits * h * r * 4 bytes, written and read once) stay a few percent of the factor read.
SplitPlan thin_tn_split(int64_t N, int64_t h, int r) {
    const int64_t slices = h / tn::PW;
    int64_t want = 512 / slices;  // two co-resident workgroups per CU in one round: no tail
    const int64_t cap_traffic = (int64_t)(0.08 * (double)N * 2.0 / (4.0 * r)) + 1;  // partials <= ~8% + 8%
    if (want > cap_traffic) want = cap_traffic;
    const int64_t cap_rows = ceil_div(N, 4 * tn::BK);
    if (want > cap_rows) want = cap_rows;
    if (want < 1) want = 1;
    SplitPlan sp;
    sp.chunk = (int64_t)align_up((size_t)ceil_div(N, want), tn::BK);
    sp.splits = (int)ceil_div(N, sp.chunk);
    return sp;
}

template <typename Kern>
static dad_status set_lds(Kern k, int bytes) {
    if (bytes > 64 * 1024)
        DAD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    return DAD_OK;
}

dad_status fast_thin_nn(const void* X, const float* Pt, void* out, int64_t N, int64_t h, int r, int* zero_hdr,
                        hipStream_t s) {
    dim3 grid((unsigned)ceil_div(N, nn::RT));
    ProfScope prof(KID_THIN_NN_BF16, s);
    if (r <= 32) {
        const int lds = 2 * (nn::XTILEB + 32 * nn::XROWB);
        hipLaunchKernelGGL(k_thin_nn_bf16<32>, grid, dim3(256), lds, s, (const bf16_t*)X, Pt, (bf16_t*)out, N, (int)h, r,
                           zero_hdr);
    } else {
        const int lds = 2 * (nn::XTILEB + 64 * nn::XROWB);
        hipLaunchKernelGGL(k_thin_nn_bf16<64>, grid, dim3(256), lds, s, (const bf16_t*)X, Pt, (bf16_t*)out, N, (int)h, r,
                           zero_hdr);
    }
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

dad_status fast_thin_tn(const void* X, const void* V, float* out_t, float* partials, SplitPlan sp, int64_t N, int64_t h,
                        int r, hipStream_t s) {
    dim3 grid((unsigned)(h / tn::PW), (unsigned)sp.splits);
    float* dst = sp.splits == 1 ? out_t : partials;
    {
    ProfScope prof(KID_THIN_TN_BF16, s);
    if (r <= 32) {
        const int lds = 2 * (tn::XTILEB + tn::BK * 64);
        hipLaunchKernelGGL(k_thin_tn_bf16<32>, grid, dim3(256), lds, s, (const bf16_t*)X, (const bf16_t*)V, dst, N, (int)h,
                           r, sp.chunk);
    } else {
        const int lds = 2 * (tn::XTILEB + tn::BK * 128);
        hipLaunchKernelGGL(k_thin_tn_bf16<64>, grid, dim3(256), lds, s, (const bf16_t*)X, (const bf16_t*)V, dst, N, (int)h,
                           r, sp.chunk);
    }
    }
    DAD_LAUNCH_CHECK();
    if (sp.splits > 1) return reduce_slabs(partials, out_t, (int64_t)r * h, sp.splits, s);
    return DAD_OK;
}

}  // namespace dad

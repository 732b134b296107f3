// The two thin contractions of the structured power iteration (Algorithm 2, Eq. 6) for bf16
// factors.  Both stream a factor matrix X (N x h) once from HBM and are bandwidth bound; the
// matrix cores only do the arithmetic.
//
//   thin_nn : V[n][j]   = sum_k X[n][k] * Pt[j][k]       (V = Delta G,  W = A U)
//   thin_tn : Ot[j][p]  = sum_n V[n][j] * X[n][p]        (U = A^T V, Y = Delta^T W, P = A^T V)
//
// Two families.  The *_dma kernels take whole tiles only (N a multiple of 256, h of 64): tiles go
// from HBM straight into LDS through a ring of three stages, and thin_nn takes its h x r panel as
// bf16 (its producers write that copy).  The register-staged kernels take any N and an fp32 panel:
// their loads run two tiles ahead of the arithmetic through two register sets.
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

// ------------------------------------------------------------------------------------------------
// thin_nn
// ------------------------------------------------------------------------------------------------
// Epilogue of thin_nn: the fp32 accumulators of a workgroup's RT x r tile (wave rows row0 .. row0+31,
// MFMA 32x32 result layout) leave as bf16 through LDS, so that the tile goes out as contiguous
// 16-byte stores.  planes = 2 also writes the rounding remainder: plane 0 holds hi = bf16(x), plane 1
// (N * r elements further on) lo = bf16(x - hi), and hi + lo carries 16 significand bits of x.
// vs is LDS for planes * RT * r bf16 values; the caller has finished reading its tiles.
template <int JT, int RT>
__device__ __forceinline__ void store_planes(const f32x16 (&acc)[JT], bf16_t* vs, bf16_t* __restrict__ V, int64_t N,
                                             int64_t n0, int64_t rows_here, int r, int planes, int row0, int nthreads) {
    const int t = threadIdx.x, lane = t & 63;
    bf16_t* vlo = vs + RT * r;
#pragma unroll
    for (int j = 0; j < JT; ++j) {
        const int col = j * 32 + (lane & 31);
        if (col < r) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + ((v >> 2) << 3) + ((lane >> 5) << 2) + (v & 3);
                const bf16_t hi = f32_to_bf16(acc[j][v]);
                vs[row * r + col] = hi;
                if (planes > 1) vlo[row * r + col] = f32_to_bf16(acc[j][v] - bf16_to_f32(hi));
            }
        }
    }
    __syncthreads();
    const int chunks = (int)(rows_here * r / 8);  // r % 8 == 0
    for (int p = 0; p < planes; ++p) {
        u32x4* dst = reinterpret_cast<u32x4*>(V + (int64_t)p * N * r + n0 * r);
        const u32x4* src = reinterpret_cast<const u32x4*>(vs + p * RT * r);
        for (int e = t; e < chunks; e += nthreads) dst[e] = src[e];
    }
}

namespace nn {
constexpr int RT = 128;             // rows of X per workgroup (32 per wave)
constexpr int BK = 64;              // contraction columns per stage (128 B of each row)
constexpr int XROWB = BK * 2 + 16;  // padded LDS row, bytes
constexpr int XTILEB = RT * XROWB;
}  // namespace nn

template <int RP>  // RP = r rounded up to 32 or 64
__global__ __launch_bounds__(256) void k_thin_nn_bf16(const bf16_t* __restrict__ X, const float* __restrict__ Pt,
                                                      bf16_t* __restrict__ V, int64_t N, int h, int r,
                                                      int* __restrict__ zero_hdr, int planes,
                                                      const int* __restrict__ skip) {
    if (skip && *skip) return;  // the caller's device-side stop flag is set: nothing to do
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
    const int64_t rows_here = (N - n0 < nn::RT) ? (N - n0) : nn::RT;
    store_planes<JT, nn::RT>(acc, reinterpret_cast<bf16_t*>(smem), V, N, n0, rows_here, r, planes, wave * 32, 256);
}

// ------------------------------------------------------------------------------------------------
// thin_nn, direct-to-LDS variant.  The h x r panel comes as bf16 (Pb: RP x h, rows >= r zero), so both
// the X tile and the panel tile go HBM/L2 -> LDS without passing through registers, through a ring of
// three slots.  Whole tiles only: N a multiple of 32*W rows, h a multiple of 64.  Each wave loads
// exactly the 32 rows it multiplies.  16-byte chunk c of tile row m sits at chunk c ^ ((m >> 1) & 7),
// which makes the 16-byte fragment reads of 16 consecutive rows hit 16 distinct bank groups; the
// XOR is applied on the global side of the load.
// ------------------------------------------------------------------------------------------------
// SRC is `const bf16_t*` (one allocation) or RowBlocks (the sites' blocks in place; a workgroup's
// rows lie in one block because every block holds a multiple of 256 rows).
// job_stride != 0 (RowBlocks only): the blocks are independent jobs of N rows each (a batch of equal
// reductions); block j multiplies the panel and writes the V that lie j * job_stride bytes after Pb
// and V, and counts its workgroups from its own first row, so that a job's result does not depend
// on the batch it runs in.
template <int RP, int W, int NS, typename SRC>
__global__ __launch_bounds__(64 * W) void k_thin_nn_bf16_dma(const SRC X, const bf16_t* __restrict__ Pb,
                                                            bf16_t* __restrict__ V, int64_t N, int h, int r, int nt,
                                                            int planes, int64_t job_stride) {
    constexpr int JT = RP / 32, RT = 32 * W, ROWB = 128;
    constexpr int XTILEB = RT * ROWB, PTILEB = RP * ROWB, STAGEB = XTILEB + PTILEB;
    constexpr int PI = RP / 8;               // 1 KiB loads that make up the panel tile
    constexpr int PL = (PI + W - 1) / W;     // per wave (waves beyond PI repeat earlier pieces)
    constexpr int LOADS = 4 + PL;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int64_t n0 = (int64_t)blockIdx.x * RT;
    if constexpr (!std::is_pointer<SRC>::value) {
        if (job_stride != 0) {  // the job's own width, if the jobs differ in it
            int b = 0;
            while (b + 1 < X.n && X.first[b + 1] <= n0) ++b;
            if (X.h[b]) h = X.h[b];
        }
    }
    const int nk = h / nn::BK;
    RowCursor cur;
    const char* x0 = row_address(X, n0, (int64_t)h * 2, cur);
    if constexpr (!std::is_pointer<SRC>::value) {
        if (job_stride != 0) {
            n0 -= X.first[cur.blk];  // row within the job
            Pb = reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(Pb) + cur.blk * job_stride);
            V = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(V) + cur.blk * job_stride);
        }
    }
    // Every group of 256 rows starts its walk over the contraction columns at its own stage (see
    // k_thin_nn_bf16).  The start depends on the rows, not on the workgroup size, so that a row's sum
    // is taken in the same order whatever W the launch uses.
    int kidx = (int)(((unsigned)(n0 / 256) * 5u) % (unsigned)nk);

    const char* gx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 32 * wave + 8 * i + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        gx[i] = x0 + row * (int64_t)h * 2 + c * 16;
    }
    const char* gp[PL];
    int pi[PL];
#pragma unroll
    for (int i = 0; i < PL; ++i) {
        pi[i] = (wave * PL + i) % PI;
        const int row = 8 * pi[i] + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        gp[i] = reinterpret_cast<const char*>(Pb + (int64_t)row * h) + c * 16;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    auto issue = [&](int stage) {
        const uint32_t base = lds0 + stage * STAGEB;
        const int koff = kidx * ROWB;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (nt)
                dma16_nt(gx[i] + koff, base + (32 * wave + 8 * i) * ROWB);
            else
                dma16(gx[i] + koff, base + (32 * wave + 8 * i) * ROWB);
        }
#pragma unroll
        for (int i = 0; i < PL; ++i) dma16(gp[i] + koff, base + XTILEB + pi[i] * 1024);
        kidx = (kidx + 1 == nk) ? 0 : kidx + 1;
    };

    f32x16 acc[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) issue(s);

    const int mrow = lane & 31, swz = (mrow >> 1) & 7, khalf = lane >> 5;
    int slot = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + NS - 2 < nk)
            wait_vmcnt<LOADS * (NS - 2)>();
        else
            wait_vmcnt<0>();
        __syncthreads();  // tile kt complete in LDS (the panel part comes from other waves); slot of kt-1 free
        if (kt + NS - 1 < nk) issue(slot == 0 ? NS - 1 : slot - 1);
        const char* xb = smem + slot * STAGEB + (wave * 32 + mrow) * ROWB;
        const char* pb = smem + slot * STAGEB + XTILEB + mrow * ROWB;
#pragma unroll
        for (int ks = 0; ks < nn::BK / 16; ++ks) {
            const int c = ((ks * 2 + khalf) ^ swz) << 4;
            bf16x8 fa = *reinterpret_cast<const bf16x8*>(xb + c);
#pragma unroll
            for (int j = 0; j < JT; ++j) {
                bf16x8 fb = *reinterpret_cast<const bf16x8*>(pb + j * 32 * ROWB + c);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[j], 0, 0, 0);
            }
        }
        slot = slot == NS - 1 ? 0 : slot + 1;
    }
    __syncthreads();

    // epilogue: fp32 -> bf16 through LDS so the tile leaves as contiguous 16-byte stores
    store_planes<JT, RT>(acc, reinterpret_cast<bf16_t*>(smem), V, N, n0, RT, r, planes, wave * 32, 64 * W);
}

// Start of a compress call on the direct-to-LDS path: Gb <- bf16(G0) with rows r..RP-1 zero, the same
// zero rows in Ub, and the workspace header cleared.
// With a table of start matrices (batch of jobs) job blockIdx.y takes G0 from the table and the other
// pointers job_stride bytes further per job.
__global__ __launch_bounds__(256) void k_panel_init(const float* __restrict__ G0, bf16_t* __restrict__ Gb,
                                                    bf16_t* __restrict__ Ub, int64_t h_in, int64_t h_out, int r, int rp,
                                                    int* __restrict__ hdr, PtrTable g0s, int64_t job_stride,
                                                    BatchInts dims, int use_dims) {
    if (job_stride != 0) {
        if (use_dims) {  // a = h_in, b = h_out of this job
            h_in = dims.a[blockIdx.y];
            h_out = dims.b[blockIdx.y];
        }
        const int64_t off = blockIdx.y * job_stride;
        G0 = static_cast<const float*>(g0s.p[blockIdx.y]);
        Gb = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(Gb) + off);
        Ub = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(Ub) + off);
        hdr = reinterpret_cast<int*>(reinterpret_cast<char*>(hdr) + off);
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < 64) hdr[threadIdx.x] = 0;
    if (i < (int64_t)rp * h_out) Gb[i] = (i < (int64_t)r * h_out) ? f32_to_bf16(G0[i]) : (bf16_t)0;
    const int64_t pad0 = (int64_t)r * h_in;
    if (i < (int64_t)(rp - r) * h_in) Ub[pad0 + i] = (bf16_t)0;
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

// NV = number of bf16 planes of V (1, or 2 when V = hi + lo): the planes are N * r elements apart and
// both are multiplied into the same accumulators.
template <int RP, int NV>
__global__ __launch_bounds__(256) void k_thin_tn_bf16(const bf16_t* __restrict__ X, const bf16_t* __restrict__ V,
                                                      float* __restrict__ part, int64_t N, int h, int r,
                                                      int64_t chunk_rows, const int* __restrict__ skip) {
    if (skip && *skip) return;
    constexpr int JT = RP / 32;
    constexpr int VROWB = RP * 2;
    constexpr int VTILEB = tn::BK * VROWB;
    constexpr int STAGEB = tn::XTILEB + NV * VTILEB;
    constexpr int VLOADS = (tn::BK * RP / 8 + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int p0 = blockIdx.x * tn::PW;
    const int64_t nbeg = (int64_t)blockIdx.y * chunk_rows;
    const int64_t nend = (nbeg + chunk_rows < N) ? nbeg + chunk_rows : N;
    const int nk = (int)((nend - nbeg + tn::BK - 1) / tn::BK);
    const int rc = r >> 3;  // 16-byte chunks per V row
    const int64_t plane = N * (int64_t)r;

    // X staging: chunk xc of rows xr + 16*i ; (xr + 16*i) & 3 == xr & 3
    const int xc = t & 15, xr = t >> 4;
    const int x_st = tn_x_off(xr, xc);

    u32x4 xs[2][4];
    u32x4 vsr[2][NV][VLOADS];

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
        for (int q = 0; q < NV; ++q)
#pragma unroll
            for (int i = 0; i < VLOADS; ++i) {
                const int e = t + 256 * i;
                const int row = e / rc, c = e - row * rc;
                const int64_t n = kb + row;
                if (row < tn::BK && n < nend)
                    vsr[set][q][i] = *reinterpret_cast<const u32x4*>(V + q * plane + n * r + c * 8);
                else
                    vsr[set][q][i] = (u32x4){0, 0, 0, 0};
            }
    };
    auto lstore = [&](int stage, int set) {
        char* xb = smem + stage * STAGEB;
        char* vb = xb + tn::XTILEB;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(xb + x_st + 16 * i * tn::XROWB) = xs[set][i];
#pragma unroll
        for (int q = 0; q < NV; ++q)
#pragma unroll
            for (int i = 0; i < VLOADS; ++i) {
                const int e = t + 256 * i;
                const int row = e / rc, c = e - row * rc;
                if (row < tn::BK) *reinterpret_cast<u32x4*>(vb + q * VTILEB + row * VROWB + c * 16) = vsr[set][q][i];
            }
    };

    // columns r..RP-1 of all V tiles stay zero for the whole kernel
    if (r < RP) {
        constexpr int PER = tn::BK * RP / 8;  // 16-byte chunks per V tile
        for (int e = t; e < 2 * NV * PER; e += 256) {
            const int stage = e / (NV * PER), rem = e - stage * (NV * PER);
            const int q = rem / PER, rem2 = rem - q * PER;
            const int row = rem2 / (RP / 8), c = rem2 - row * (RP / 8);
            if (c >= rc)
                *reinterpret_cast<u32x4*>(smem + stage * STAGEB + tn::XTILEB + q * VTILEB + row * VROWB + c * 16) =
                    (u32x4){0, 0, 0, 0};
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
            for (int j = 0; j < JT; ++j)
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    bf16x8 fv = tn_frag<false>(vb + q * VTILEB, VROWB, j * 32, ks * 16, lane);
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
// thin_tn, direct-to-LDS variant: whole 64-row tiles only (N and the row chunk multiples of 64) and
// r in {16, 32, 64}.  X and V tiles go HBM -> LDS without passing through registers, through a ring
// of three slots, so two tiles per workgroup are always in flight and two workgroups share a CU.
// The swizzle of the X tile is applied on the global side, as in the rebuild kernel.
// ------------------------------------------------------------------------------------------------
// SRC as in k_thin_nn_bf16_dma; a row chunk may span several blocks, the walk jumps at their ends.
// job_stride != 0 (RowBlocks only): block blockIdx.y of X is a job of its own with N rows, whose V and
// partial slabs lie blockIdx.y * job_stride bytes after V and part.
template <int R, int PW, int BK, int NV, typename SRC>
__global__ __launch_bounds__(256) void k_thin_tn_bf16_dma(const SRC X, const bf16_t* __restrict__ V,
                                                          float* __restrict__ part, int64_t N, int h,
                                                          int64_t chunk_rows, int strips, int splits, int nt,
                                                          int64_t job_stride) {
    constexpr int JT = R > 32 ? 2 : 1;
    constexpr int MT = PW / 128;                  // 32-column tiles per wave
    constexpr int XROWB = PW * 2;
    constexpr int XTILEB = BK * XROWB;
    constexpr int XL = XTILEB / 1024 / 4;         // X loads per wave per tile
    constexpr int RPL = 1024 / XROWB;             // tile rows covered by one load
    constexpr int CPR = PW / 8;                   // 16-byte chunks per row
    constexpr int VROWB = R * 2;
    constexpr int VTILEB = BK * VROWB;
    constexpr int VSLOT = NV * VTILEB + 256;  // R = 16: fragment reads of the unused columns 16..31 run past the tile
    constexpr int STAGEB = XTILEB + VSLOT;
    constexpr int NS = 3;
    constexpr int VP = VTILEB / 1024;             // 1 KiB pieces of the V tile
    constexpr int VL = VP > 4 ? VP / 4 : 1;       // V loads per wave per tile (fewer pieces than waves: repeats)
    constexpr int LOADS = XL + NV * VL;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    if constexpr (!std::is_pointer<SRC>::value) {
        if (job_stride != 0 && X.h[blockIdx.y]) {  // the job's own width and row split; the grid is sized for the largest job
            h = X.h[blockIdx.y];
            splits = X.splits[blockIdx.y];
            chunk_rows = X.chunk[blockIdx.y];
            strips = h / PW;
            if ((int)blockIdx.x >= strips * splits) return;
        }
    }
    // Workgroups are handed to the eight XCDs round-robin by their linear index.  All column strips
    // of one row chunk go to the same XCD, so that the chunk of V they share is fetched into one L2.
    int strip, split;
    if ((splits & 7) == 0) {
        const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
        split = xcd + 8 * (q / strips);
        strip = q % strips;
    } else {
        strip = blockIdx.x % strips;
        split = blockIdx.x / strips;
    }
    const int p0 = strip * PW;
    const int64_t nbeg = (int64_t)split * chunk_rows;
    const int64_t nend = (nbeg + chunk_rows < N) ? nbeg + chunk_rows : N;
    const int nk = (int)((nend - nbeg) / BK);

    // X: load i of this wave covers tile rows (wave*XL + i)*RPL .. ; lane -> row += lane/CPR, LDS chunk lane%CPR
    int64_t row0 = 0;  // the job's first row in X
    if constexpr (!std::is_pointer<SRC>::value) {
        if (job_stride != 0) {
            row0 = X.first[blockIdx.y];
            V = reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(V) + blockIdx.y * job_stride);
            part = reinterpret_cast<float*>(reinterpret_cast<char*>(part) + blockIdx.y * job_stride);
        }
    }
    RowCursor cur;
    const char* x0 = row_address(X, row0 + nbeg, (int64_t)h * 2, cur);
    int64_t row_next = row0 + nbeg;  // first row of the next tile to be issued
    const char* gx[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        const int row = (wave * XL + i) * RPL + lane / CPR;
        const int c = (lane % CPR) ^ ((row & 3) << 2);
        gx[i] = x0 + (row * (int64_t)h + p0 + c * 8) * 2;
    }
    // V: a tile is BK*R*2 contiguous bytes of each of the NV planes (N*R elements apart); load i of
    // this wave covers the 1 KiB piece vi[i] of every plane
    const char* gv[NV][VL];
    int vi[VL];
#pragma unroll
    for (int i = 0; i < VL; ++i) {
        vi[i] = (wave * VL + i) % VP;
#pragma unroll
        for (int q = 0; q < NV; ++q)
            gv[q][i] = reinterpret_cast<const char*>(V + (int64_t)q * N * R + nbeg * R) + vi[i] * 1024 + lane * 16;
    }
    const int64_t adv_x = (int64_t)BK * h * 2;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    auto issue = [&](int stage) {
        const uint32_t base = lds0 + stage * STAGEB;
        if constexpr (!std::is_pointer<SRC>::value) {
            if (row_next == cur.end) {
                const int64_t jump = block_jump(X, (int64_t)h * 2, cur);
#pragma unroll
                for (int i = 0; i < XL; ++i) gx[i] += jump;
            }
            row_next += BK;
        }
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            if (nt)
                dma16_nt(gx[i], base + (wave * XL + i) * 1024);
            else
                dma16(gx[i], base + (wave * XL + i) * 1024);
            gx[i] += adv_x;
        }
#pragma unroll
        for (int q = 0; q < NV; ++q)
#pragma unroll
            for (int i = 0; i < VL; ++i) {
                dma16(gv[q][i], base + XTILEB + q * VTILEB + vi[i] * 1024);
                gv[q][i] += VTILEB;
            }
    };

    f32x16 acc[MT][JT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int j = 0; j < JT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][j][v] = 0.f;

#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) issue(s);

    int slot = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + NS - 2 < nk)
            wait_vmcnt<LOADS * (NS - 2)>();
        else
            wait_vmcnt<0>();
        __syncthreads();  // tile kt is complete in LDS, and the slot of tile kt-1 is free
        if (kt + NS - 1 < nk) issue(slot == 0 ? NS - 1 : slot - 1);
        const char* xb = smem + slot * STAGEB;
        const char* vb = xb + XTILEB;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fv[NV][JT];
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int j = 0; j < JT; ++j) fv[q][j] = tn_frag<false>(vb + q * VTILEB, VROWB, j * 32, ks * 16, lane);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                bf16x8 fx = tn_frag<true>(xb, XROWB, (wave * MT + m) * 32, ks * 16, lane);
#pragma unroll
                for (int j = 0; j < JT; ++j)
#pragma unroll
                    for (int q = 0; q < NV; ++q)
                        acc[m][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[q][j], fx, acc[m][j], 0, 0, 0);
            }
        }
        slot = slot == NS - 1 ? 0 : slot + 1;
    }

    float* o = part + (int64_t)split * R * h;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int p = p0 + (wave * MT + m) * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < JT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = j * 32 + ((v >> 2) << 3) + ((lane >> 5) << 2) + (v & 3);
                if (row < R) o[(int64_t)row * h + p] = acc[m][j][v];
            }
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------

// A factor larger than most of the 256 MB Infinity Cache is loaded with the non-temporal hint (4-8 %
// faster); a smaller one is not, because the next pass over it still finds part of it cached.
static bool stream_once(int64_t N, int64_t h) { return N * h * 2 > (int64_t)200 << 20; }

bool thin_fast_ok(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt) {
    return dt == DAD_BF16 && r % 8 == 0 && h_in % tn::PW == 0 && h_out % tn::PW == 0 && N >= 256 &&
           h_in <= (1 << 20) && h_out <= (1 << 20);
}

// Column-strip width of thin_tn.  512-byte row segments use the HBM channels better than 256-byte
// ones when the row pitch is a power of two, and halve the re-reads of V.
int thin_tn_pw(int64_t h) { return h % 256 == 0 ? 256 : 128; }

// Row split of thin_tn: about one workgroup per CU, while the fp32 partials (splits * h * r * 4
// bytes, written and read once) stay a few percent of the factor read.
SplitPlan thin_tn_split(int64_t N, int64_t h, int r) {
    const int64_t slices = h / thin_tn_pw(h);
    int64_t want = 256 / slices;  // one workgroup per CU in a single round (measured faster than two)
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

dad_status fast_thin_nn(const void* X, const float* Pt, void* out, int64_t N, int64_t h, int r, int* zero_hdr,
                        int planes, hipStream_t s, const int* skip) {
    dim3 grid((unsigned)ceil_div(N, nn::RT));
    ProfScope prof(KID_THIN_NN_BF16, s);
    if (r <= 32) {
        const int lds = 2 * (nn::XTILEB + 32 * nn::XROWB);
        hipLaunchKernelGGL(k_thin_nn_bf16<32>, grid, dim3(256), lds, s, (const bf16_t*)X, Pt, (bf16_t*)out, N, (int)h, r,
                           zero_hdr, planes, skip);
    } else {
        const int lds = 2 * (nn::XTILEB + 64 * nn::XROWB);
        hipLaunchKernelGGL(k_thin_nn_bf16<64>, grid, dim3(256), lds, s, (const bf16_t*)X, Pt, (bf16_t*)out, N, (int)h, r,
                           zero_hdr, planes, skip);
    }
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

bool thin_dma_ok(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt) {
    return thin_fast_ok(N, h_in, h_out, r, dt) && N % 256 == 0 && h_in % nn::BK == 0 && h_out % nn::BK == 0;
}

// g0s != null: a batch of `jobs` jobs (G0 unused).
// dims (optional): job j has widths dims->a[j] (h_in) and dims->b[j] (h_out); h_in, h_out are then the largest.
dad_status launch_panel_init(const float* G0, void* Gb, void* Ub, int64_t h_in, int64_t h_out, int r, int* hdr,
                             hipStream_t s, const PtrTable* g0s, int jobs, int64_t job_stride, const BatchInts* dims) {
    PtrTable none = {};
    if (!g0s) jobs = 1, job_stride = 0, dims = nullptr;
    const int rp = r <= 32 ? 32 : 64;
    int64_t n = (int64_t)rp * h_out;
    if ((int64_t)(rp - r) * h_in > n) n = (int64_t)(rp - r) * h_in;
    ProfScope prof(KID_PANEL_INIT, s);
    hipLaunchKernelGGL(k_panel_init, dim3((unsigned)ceil_div(n, 256), (unsigned)jobs), dim3(256), 0, s, G0, (bf16_t*)Gb,
                       (bf16_t*)Ub, h_in, h_out, r, rp, hdr, g0s ? *g0s : none, job_stride, dims ? *dims : BatchInts{},
                       dims ? 1 : 0);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

constexpr int nn_dma_lds(int rp, int w, int ns) { return ns * (32 * w * 128 + rp * 128); }
constexpr int tn_dma_lds(int r, int pw, int bk, int nv) { return 3 * (bk * pw * 2 + nv * bk * r * 2 + 256); }

template <int RP, int W, int NS>
static dad_status dma_thin_nn_cfg(const void* X, const RowBlocks* xb, const void* Pb, void* out, int64_t N, int64_t h,
                                  int r, int planes, int jobs, int64_t job_stride, hipStream_t s) {
    const int lds = nn_dma_lds(RP, W, NS);
    const dim3 grid((unsigned)(jobs * (N / (32 * W)))), block(64 * W);
    const int nt = stream_once(jobs * N, h) ? 1 : 0;
    if (xb)
        hipLaunchKernelGGL((k_thin_nn_bf16_dma<RP, W, NS, RowBlocks>), grid, block, lds, s, *xb, (const bf16_t*)Pb,
                           (bf16_t*)out, N, (int)h, r, nt, planes, jobs > 1 || job_stride ? job_stride : (int64_t)0);
    else
        hipLaunchKernelGGL((k_thin_nn_bf16_dma<RP, W, NS, const bf16_t*>), grid, block, lds, s, (const bf16_t*)X,
                           (const bf16_t*)Pb, (bf16_t*)out, N, (int)h, r, nt, planes, (int64_t)0);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

// Rows per workgroup: 256 (eight waves) when that still gives one workgroup per CU, fewer for
// shorter factors so that the chip stays filled (a site's 8192 rows: 256 single-wave workgroups).
// xb, when not null, gives X as row blocks (X itself is then unused).  job_stride != 0: the blocks
// are `jobs` independent problems of N rows each (see the kernel); the rows per workgroup are chosen
// from one job's N, as a single call would.
dad_status dma_thin_nn(const void* X, const RowBlocks* xb, const void* Pb, void* out, int64_t N, int64_t h, int r,
                       int planes, hipStream_t s, int jobs, int64_t job_stride) {
    if (job_stride != 0 && !xb) return DAD_ERR_SHAPE;
    if (job_stride == 0) jobs = 1;
    ProfScope prof(KID_THIN_NN_BF16, s);
    const int64_t want = 256;          // workgroups
    // A batch fills the chip with the rows of all its jobs (the result does not depend on W).  Jobs of
    // unequal widths: every job gets at least 256 workgroups where its rows allow, so that the units,
    // which take workgroups round-robin, each receive workgroups of every job and finish together.
    const bool per_job = job_stride != 0 && xb->h[0] != 0;
    const int64_t rows = per_job ? N : jobs * N;
#define DAD_NN_W(W) \
    (r <= 32 ? dma_thin_nn_cfg<32, W, 3>(X, xb, Pb, out, N, h, r, planes, jobs, job_stride, s) \
             : dma_thin_nn_cfg<64, W, 3>(X, xb, Pb, out, N, h, r, planes, jobs, job_stride, s))
    if (rows / 256 >= want) return DAD_NN_W(8);
    if (rows / 128 >= want) return DAD_NN_W(4);
    if (rows / 64 >= want) return DAD_NN_W(2);
    return DAD_NN_W(1);
#undef DAD_NN_W
}

// True when fast_thin_tn (without a skip word) takes the direct-to-LDS kernel.
bool thin_tn_dma_ok(int64_t N, int r, SplitPlan sp) {
    return (r == 16 || r == 32 || r == 64) && N % tn::BK == 0 && sp.chunk % tn::BK == 0;
}

// xb, when not null, gives X as row blocks (X itself is then unused); only the direct-to-LDS kernel
// reads blocks, so the caller has checked thin_tn_dma_ok and passes no skip word.
// job_stride != 0: the blocks are `jobs` independent problems of N rows each, and V, out_t, partials
// and out_bf16 of job j lie j * job_stride bytes after the pointers given.
dad_status fast_thin_tn(const void* X, const RowBlocks* xb, const void* V, float* out_t, float* partials, SplitPlan sp,
                        int64_t N, int64_t h, int r, void* out_bf16, int planes, hipStream_t s, const int* skip,
                        int jobs, int64_t job_stride) {
    float* dst = sp.splits == 1 ? out_t : partials;
    if (xb && (skip || !thin_tn_dma_ok(N, r, sp))) return DAD_ERR_SHAPE;
    if (job_stride != 0 && !xb) return DAD_ERR_SHAPE;
    if (job_stride == 0) jobs = 1;
    // jobs of different widths (xb->h set): the grid is sized for the job with the most workgroups, every job
    // writes slabs (also one with a single chunk), and the sum runs with each job's own size and count
    const bool per_job = job_stride != 0 && xb->h[0] != 0;
    int64_t max_blocks = 0;
    BatchInts rd = {};
    if (per_job) {
        for (int j = 0; j < jobs; ++j) {
            const int64_t nb = (int64_t)(xb->h[j] / thin_tn_pw(h)) * xb->splits[j];
            if (nb > max_blocks) max_blocks = nb;
            rd.a[j] = r * xb->h[j];
            rd.b[j] = xb->splits[j];
        }
        dst = partials;
    }
    if (!skip && thin_tn_dma_ok(N, r, sp)) {
        ProfScope prof(KID_THIN_TN_BF16, s);
        const int pw = thin_tn_pw(h);
        const int bk = pw == 128 ? 64 : 32;
        const int lds = tn_dma_lds(r, pw, bk, planes);
        const int strips = (int)(h / pw);
#define DAD_TN_LAUNCH_NV(RR, PP, BB, NV)                                                                          \
    do {                                                                                                          \
        const dim3 grid((unsigned)(per_job ? max_blocks : strips * sp.splits), (unsigned)jobs);                  \
        const int nt = stream_once(jobs * N, h) ? 1 : 0;                                                          \
        if (xb)                                                                                                   \
            hipLaunchKernelGGL((k_thin_tn_bf16_dma<RR, PP, BB, NV, RowBlocks>), grid, dim3(256), lds, s, *xb,     \
                               (const bf16_t*)V, dst, N, (int)h, sp.chunk, strips, sp.splits, nt, job_stride);    \
        else                                                                                                      \
            hipLaunchKernelGGL((k_thin_tn_bf16_dma<RR, PP, BB, NV, const bf16_t*>), grid, dim3(256), lds, s,      \
                               (const bf16_t*)X, (const bf16_t*)V, dst, N, (int)h, sp.chunk, strips, sp.splits, nt, \
                               (int64_t)0);                                                                       \
    } while (0)
#define DAD_TN_LAUNCH(RR, PP, BB)                  \
    do {                                           \
        if (planes > 1)                            \
            DAD_TN_LAUNCH_NV(RR, PP, BB, 2);       \
        else                                       \
            DAD_TN_LAUNCH_NV(RR, PP, BB, 1);       \
    } while (0)
        if (pw == 128) {
            if (r == 16) DAD_TN_LAUNCH(16, 128, 64);
            else if (r == 32) DAD_TN_LAUNCH(32, 128, 64);
            else DAD_TN_LAUNCH(64, 128, 64);
        } else {
            if (r == 16) DAD_TN_LAUNCH(16, 256, 32);
            else if (r == 32) DAD_TN_LAUNCH(32, 256, 32);
            else DAD_TN_LAUNCH(64, 256, 32);
        }
#undef DAD_TN_LAUNCH_NV
#undef DAD_TN_LAUNCH
    } else {  // ragged row count or a rank the direct-to-LDS kernel is not built for
        ProfScope prof(KID_THIN_TN_BF16, s);
        const dim3 grid((unsigned)(h / tn::PW), (unsigned)sp.splits);
        const int rp = r <= 32 ? 32 : 64;
        const int lds = 2 * (tn::XTILEB + planes * tn::BK * rp * 2);  // at most 64 KiB
#define DAD_TN_REG(RP, NV)                                                                                            \
    hipLaunchKernelGGL((k_thin_tn_bf16<RP, NV>), grid, dim3(256), lds, s, (const bf16_t*)X, (const bf16_t*)V, dst, N, \
                       (int)h, r, sp.chunk, skip)
        if (r <= 32) {
            if (planes > 1) DAD_TN_REG(32, 2);
            else DAD_TN_REG(32, 1);
        } else {
            if (planes > 1) DAD_TN_REG(64, 2);
            else DAD_TN_REG(64, 1);
        }
#undef DAD_TN_REG
    }
    DAD_LAUNCH_CHECK();
    if (per_job) return reduce_slabs(partials, out_t, (int64_t)r * h, sp.splits, s, out_bf16, skip, jobs, job_stride, &rd);
    if (sp.splits > 1) return reduce_slabs(partials, out_t, (int64_t)r * h, sp.splits, s, out_bf16, skip, jobs, job_stride);
    if (out_bf16) return reduce_slabs(out_t, out_t, (int64_t)r * h, 1, s, out_bf16, skip, jobs, job_stride);  // copy only
    return DAD_OK;
}

// Once per device: the direct-to-LDS kernels use more than the 64 KiB of dynamic LDS a kernel gets
// without asking.
dad_status thin_prepare_device() {
#define DAD_NN_ATTR(RP, W)                                                                             \
    DAD_HIP_TRY(set_max_lds((k_thin_nn_bf16_dma<RP, W, 3, const bf16_t*>), nn_dma_lds(RP, W, 3))); \
    DAD_HIP_TRY(set_max_lds((k_thin_nn_bf16_dma<RP, W, 3, RowBlocks>), nn_dma_lds(RP, W, 3)))
    DAD_NN_ATTR(32, 1); DAD_NN_ATTR(32, 2); DAD_NN_ATTR(32, 4); DAD_NN_ATTR(32, 8);
    DAD_NN_ATTR(64, 1); DAD_NN_ATTR(64, 2); DAD_NN_ATTR(64, 4); DAD_NN_ATTR(64, 8);
#undef DAD_NN_ATTR
#define DAD_TN_ATTR(R, PW, BK)                                                                              \
    DAD_HIP_TRY(set_max_lds((k_thin_tn_bf16_dma<R, PW, BK, 1, const bf16_t*>), tn_dma_lds(R, PW, BK, 1))); \
    DAD_HIP_TRY(set_max_lds((k_thin_tn_bf16_dma<R, PW, BK, 2, const bf16_t*>), tn_dma_lds(R, PW, BK, 2))); \
    DAD_HIP_TRY(set_max_lds((k_thin_tn_bf16_dma<R, PW, BK, 1, RowBlocks>), tn_dma_lds(R, PW, BK, 1)));     \
    DAD_HIP_TRY(set_max_lds((k_thin_tn_bf16_dma<R, PW, BK, 2, RowBlocks>), tn_dma_lds(R, PW, BK, 2)))
    DAD_TN_ATTR(16, 128, 64); DAD_TN_ATTR(32, 128, 64); DAD_TN_ATTR(64, 128, 64);
    DAD_TN_ATTR(16, 256, 32); DAD_TN_ATTR(32, 256, 32); DAD_TN_ATTR(64, 256, 32);
#undef DAD_TN_ATTR
    return DAD_OK;
}

}  // namespace dad

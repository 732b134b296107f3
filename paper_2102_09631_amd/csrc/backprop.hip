// One step of the delta recursion (Section 3.1, Eq. 3):
//     D_out[n][p] = ( sum_q D_next[n][q] * W_next[p][q] ) * phi'(Z[n][p]).
// Both operands of the contraction are contiguous along q, so MFMA fragments are plain 16-byte
// LDS reads (no transposition as in the gradient rebuild).  The derivative of the activation is
// applied to the fp32 accumulators, and the result leaves as bf16 rows: written at a site's row
// offset inside the stacked buffer, it is that site's part of the stacked delta.
#include "dad_internal.h"

namespace dad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// phi'(z).  FAST uses the hardware exponential (a few ulp), enough for a result rounded to bf16;
// the guarded kernel, which also serves fp32, uses the library functions.
template <int ACT, bool FAST>
__device__ __forceinline__ float act_derivative(float z) {
    if (ACT == DAD_ACT_RELU) return z > 0.f ? 1.f : 0.f;
    if (ACT == DAD_ACT_TANH) {
        // 1 - tanh^2 = 4 e / (1 + e)^2 with e = exp(-2|z|) <= 1: no overflow, no cancellation
        const float e = FAST ? __expf(-2.f * fabsf(z)) : expf(-2.f * fabsf(z));
        const float d = 1.f + e;
        return 4.f * e / (d * d);
    }
    if (ACT == DAD_ACT_SIGMOID) {
        // s (1 - s) = e / (1 + e)^2 with e = exp(-|z|)
        const float e = FAST ? __expf(-fabsf(z)) : expf(-fabsf(z));
        const float d = 1.f + e;
        return e / (d * d);
    }
    return 1.f;
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel: whole 256 x 256 output tiles (N and h multiples of 256), h_next a multiple of 32.
// Eight waves (2 x 4, each 128 rows x 64 columns).  Per stage the tile rows of D_next and of W_next
// contribute 64 contraction elements each: 128 bytes, a whole cache line per row, which the memory
// pipeline moves at twice the rate of half lines (32-element stages through a deeper ring measured
// 25 % slower).  Two 64 KiB stages alternate; the tiles go from memory straight into LDS.  LDS row =
// eight 16-byte chunks; chunk c of row r sits in slot c ^ ((r >> 1) & 7), applied on the global side
// of the load, so that the 16 lanes of one pass of a fragment read (16 consecutive rows, same chunk)
// fall on 16 different bank groups.
// ---------------------------------------------------------------------------------------------
namespace bp {
constexpr int TILE = 256;
constexpr int BK = 64;
constexpr int ROWB = BK * 2;
constexpr int TILEB = TILE * ROWB;   // one operand tile per stage
constexpr int STAGEB = 2 * TILEB;
constexpr int STAGES = 2;
constexpr int THREADS = 512;
}  // namespace bp

template <int ACT>
__global__ __launch_bounds__(bp::THREADS) void k_backprop_bf16(const bf16_t* __restrict__ Dn, const bf16_t* __restrict__ Wn,
                                                              const bf16_t* __restrict__ Z, bf16_t* __restrict__ Dout,
                                                              int h, int hn, int tiles_n, int total) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 2, wn = wave & 3;

    // workgroups of one XCD (ids congruent mod 8) take neighbouring tiles: the same rows of D_next
    // against successive column tiles, and all of them the same slab of W_next
    int lid = blockIdx.x;
    {
        const int per = total >> 3, main = per << 3;
        if ((int)blockIdx.x < main) lid = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    }
    const int pm = lid / tiles_n, qn = lid - pm * tiles_n;
    const int64_t n0 = (int64_t)pm * bp::TILE;
    const int p0 = qn * bp::TILE;
    const int nk = hn / bp::BK;

    // load i of this wave covers tile rows 32*wave + 8*i .. +7: lane -> row += lane/8, slot lane%8
    const char* ga[4];
    const char* gb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 32 * wave + 8 * i + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        ga[i] = reinterpret_cast<const char*>(Dn + (n0 + row) * (int64_t)hn) + c * 16;
        gb[i] = reinterpret_cast<const char*>(Wn + (int64_t)(p0 + row) * hn) + c * 16;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    auto issue = [&](int stage) {
        const uint32_t base = lds0 + stage * bp::STAGEB + (32 * wave) * bp::ROWB;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma16(ga[i], base + 8 * i * bp::ROWB);
            ga[i] += bp::ROWB;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma16(gb[i], base + bp::TILEB + 8 * i * bp::ROWB);
            gb[i] += bp::ROWB;
        }
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (nk > 0) issue(0);

    // fragment of 32 rows starting at row0: lane -> row row0 + lane%32, contraction elements
    // 16*ks + 8*(lane/32) .. +7, i.e. chunk 2*ks + lane/32 of that row
    const int frow = lane & 31, fsw = (frow >> 1) & 7, fhalf = lane >> 5;
    auto frag = [&](const char* tile, int row0, int ks) -> bf16x8 {
        const int slot = (2 * ks + fhalf) ^ fsw;
        return *reinterpret_cast<const bf16x8*>(tile + (row0 + frow) * bp::ROWB + (slot << 4));
    };

    // Each stage is four MFMA K-steps; fragment sets 0 and 1 alternate.  The last step of a stage is
    // multiplied after the next stage's barrier, so the matrix cores have independent MFMAs to chew on
    // while the first fragments of the new stage travel from LDS.
    // Within a step the six fragment reads are spread between the eight MFMAs of the other set.
    bf16x8 fa0[4], fb0[2], fa1[4], fb1[2];
#pragma unroll
    for (int a = 0; a < 4; ++a) fa1[a] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};  // the first stage multiplies zeros
#pragma unroll
    for (int b = 0; b < 2; ++b) fb1[b] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    auto read_frags = [&](bf16x8 (&fa)[4], bf16x8 (&fb)[2], const char* ta, int ks) {
        const char* tb = ta + bp::TILEB;
#pragma unroll
        for (int a = 0; a < 4; ++a) fa[a] = frag(ta, wm * 128 + a * 32, ks);
#pragma unroll
        for (int b = 0; b < 2; ++b) fb[b] = frag(tb, wn * 64 + b * 32, ks);
    };
    auto mma = [&](const bf16x8 (&fa)[4], const bf16x8 (&fb)[2]) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                // W fragment as the row operand: a lane then owns four consecutive p of one n
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[b], fa[a], acc[a][b], 0, 0, 0);
    };
    for (int kt = 0; kt < nk; ++kt) {
        wait_vmcnt<0>();
        __syncthreads();  // tile kt is complete in LDS, and every wave has its fragments of tile kt-1
        if (kt + 1 < nk) issue((kt + 1) & 1);
        const char* ta = smem + (kt & 1) * bp::STAGEB;
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa0, fb0, ta, 0);
        mma(fa1, fb1);
        interleave_reads_mfma<6, 8, true>();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa1, fb1, ta, 1);
        mma(fa0, fb0);
        interleave_reads_mfma<6, 8, false>();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa0, fb0, ta, 2);
        mma(fa1, fb1);
        interleave_reads_mfma<6, 8, false>();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa1, fb1, ta, 3);
        mma(fa0, fb0);
        interleave_reads_mfma<6, 8, false>();
        __builtin_amdgcn_sched_barrier(0);
    }
    // this wave's 16 pieces of Z (eight lanes per row, 16 bytes each) are requested now, so that
    // their latency passes while the last MFMAs drain and the accumulators are staged
    u32x4 zraw[2][8];
#pragma unroll
    for (int rnd = 0; rnd < 2; ++rnd)
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int64_t n = n0 + wm * 128 + rnd * 64 + pass * 8 + (lane >> 3);
            zraw[rnd][pass] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4*>(Z + n * h + p0 + wn * 64 + (lane & 7) * 8));
        }
    if (nk > 0) mma(fa1, fb1);
    __syncthreads();  // every wave is done with the ring: its memory now stages the output

    // Epilogue.  Each wave owns 16 KiB of LDS: an fp32 [64 n][64 p] block, two rounds for its 128 rows.
    // Element (n, p) sits at float4 column (p/4) ^ (n & 15) of row n (conflict-free writes, lanes of a
    // pass differ in n).  Rows are then read back eight lanes per row, so that Z is read and D_out is
    // written in whole 128-byte lines.
    float* stg = reinterpret_cast<float*>(smem) + wave * (64 * 64);
#pragma unroll
    for (int rnd = 0; rnd < 2; ++rnd) {
#pragma unroll
        for (int a2 = 0; a2 < 2; ++a2) {
            const int a = 2 * rnd + a2;
            const int nl = a2 * 32 + (lane & 31);
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int c4 = (b * 8 + 2 * g + (lane >> 5)) ^ (nl & 15);
                    f32x4 v4 = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                    *reinterpret_cast<f32x4*>(stg + nl * 64 + c4 * 4) = v4;
                }
        }
        // the block is private to the wave: program order is enough between the writes and the reads
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int nl = pass * 8 + (lane >> 3), pc = lane & 7;
            const f32x4 lo = *reinterpret_cast<const f32x4*>(stg + nl * 64 + (((2 * pc) ^ (nl & 15)) << 2));
            const f32x4 hi = *reinterpret_cast<const f32x4*>(stg + nl * 64 + (((2 * pc + 1) ^ (nl & 15)) << 2));
            const int64_t n = n0 + wm * 128 + rnd * 64 + nl;
            const int p = p0 + wn * 64 + pc * 8;
            const u32x4 zr = zraw[rnd][pass];
            float o[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            uint32_t packed[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float z0 = __uint_as_float(zr[e] << 16), z1 = __uint_as_float(zr[e] & 0xffff0000u);
                const float r0 = o[2 * e] * act_derivative<ACT, true>(z0), r1 = o[2 * e + 1] * act_derivative<ACT, true>(z1);
                packed[e] = pack_bf16x2(r0, r1);
            }
            // written once, read by a later call: keep it out of the caches the operand tiles live in
            __builtin_nontemporal_store(u32x4{packed[0], packed[1], packed[2], packed[3]},
                                        reinterpret_cast<u32x4*>(Dout + n * h + p));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Guarded kernel for any shape and either element type: 64 x 64 output tile, fp32 FMA from LDS.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_backprop(const T* __restrict__ Dn, const T* __restrict__ Wn,
                                                  const T* __restrict__ Z, T* __restrict__ Dout, int64_t N, int64_t h,
                                                  int64_t hn, int act) {
    constexpr int TM = 64, KC = 16;
    __shared__ float As[TM][KC + 1];
    __shared__ float Bs[TM][KC + 1];
    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;
    const int64_t p0 = (int64_t)blockIdx.x * TM, n0 = (int64_t)blockIdx.y * TM;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;
    // Tiles travel global -> registers -> LDS: every load has a valid (clamped) address and its value
    // is selected only at the LDS store, so that the loads of a tile go out together, and the next
    // tile's loads are in flight while the current one is multiplied.
    constexpr int TL = TM * KC / 256;
    float ar[TL], br[TL];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int m = 0; m < TL; ++m) {
            const int e = t + 256 * m, rr = e / KC, kk = e % KC;
            const int64_t k = k0 + kk < hn ? k0 + kk : hn - 1;
            ar[m] = ld<T>(Dn, (n0 + rr < N ? n0 + rr : N - 1) * hn + k);
            br[m] = ld<T>(Wn, (p0 + rr < h ? p0 + rr : h - 1) * hn + k);
        }
    };
    auto commit = [&](int64_t k0) {
#pragma unroll
        for (int m = 0; m < TL; ++m) {
            const int e = t + 256 * m, rr = e / KC, kk = e % KC;
            const bool kin = k0 + kk < hn;
            As[rr][kk] = (kin && n0 + rr < N) ? ar[m] : 0.f;
            Bs[rr][kk] = (kin && p0 + rr < h) ? br[m] : 0.f;
        }
    };
    // the 4 x 4 values of Z this thread needs at the end are requested up front as well
    float zr[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t n = n0 + ty * 4 + a, pp = p0 + tx * 4 + b;
            zr[a][b] = ld<T>(Z, (n < N ? n : N - 1) * h + (pp < h ? pp : h - 1));
        }
    fetch(0);
    for (int64_t k0 = 0; k0 < hn; k0 += KC) {
        commit(k0);
        __syncthreads();
        if (k0 + KC < hn) fetch(k0 + KC);
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) av[a] = As[ty * 4 + a][kk];
#pragma unroll
            for (int b = 0; b < 4; ++b) bv[b] = Bs[tx * 4 + b][kk];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int64_t n = n0 + ty * 4 + a;
        if (n >= N) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int64_t p = p0 + tx * 4 + b;
            if (p >= h) continue;
            const float z = zr[a][b];
            float d = 1.f;
            if (act == DAD_ACT_RELU) d = act_derivative<DAD_ACT_RELU, false>(z);
            else if (act == DAD_ACT_TANH) d = act_derivative<DAD_ACT_TANH, false>(z);
            else if (act == DAD_ACT_SIGMOID) d = act_derivative<DAD_ACT_SIGMOID, false>(z);
            st<T>(Dout, n * h + p, acc[a][b] * d);
        }
    }
}

static bool backprop_fast_ok(int64_t N, int64_t h, int64_t hn, dad_dtype dt) {
    return dt == DAD_BF16 && N % bp::TILE == 0 && h % bp::TILE == 0 && hn % bp::BK == 0 && hn >= bp::BK &&
           (N / bp::TILE) * (h / bp::TILE) < (1 << 30) && h <= (1 << 20) && hn <= (1 << 20);
}

template <int ACT>
static dad_status launch_backprop_fast(const void* Dn, const void* Wn, const void* Z, void* Dout, int64_t N, int64_t h,
                                       int64_t hn, hipStream_t s) {
    const int lds = bp::STAGES * bp::STAGEB;
    const int tiles_n = (int)(h / bp::TILE);
    const int total = (int)((N / bp::TILE) * tiles_n);
    ProfScope prof(KID_BACKPROP_BF16, s);
    hipLaunchKernelGGL(k_backprop_bf16<ACT>, dim3((unsigned)total), dim3(bp::THREADS), lds, s, (const bf16_t*)Dn,
                       (const bf16_t*)Wn, (const bf16_t*)Z, (bf16_t*)Dout, (int)h, (int)hn, tiles_n, total);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

dad_status backprop_prepare_device() {
    const int lds = bp::STAGES * bp::STAGEB;
    DAD_HIP_TRY(set_max_lds(k_backprop_bf16<DAD_ACT_IDENTITY>, lds));
    DAD_HIP_TRY(set_max_lds(k_backprop_bf16<DAD_ACT_RELU>, lds));
    DAD_HIP_TRY(set_max_lds(k_backprop_bf16<DAD_ACT_TANH>, lds));
    DAD_HIP_TRY(set_max_lds(k_backprop_bf16<DAD_ACT_SIGMOID>, lds));
    return DAD_OK;
}

}  // namespace dad

using namespace dad;

extern "C" dad_status dad_backprop_delta(const void* D_next, const void* W_next, const void* Z, int64_t N, int64_t h,
                                         int64_t h_next, dad_dtype dt, dad_activation act, void* D_out, void* stream) {
    if (!D_next || !W_next || !Z || !D_out) return DAD_ERR_NULL;
    if (dt != DAD_F32 && dt != DAD_BF16) return DAD_ERR_DTYPE;
    if (act != DAD_ACT_IDENTITY && act != DAD_ACT_RELU && act != DAD_ACT_TANH && act != DAD_ACT_SIGMOID)
        return DAD_ERR_SHAPE;
    if (N < 1 || h < 1 || h_next < 1 || N > DAD_MAX_ROWS || h > DAD_MAX_WIDTH || h_next > DAD_MAX_WIDTH)
        return DAD_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    const bool fast = backprop_fast_ok(N, h, h_next, dt);
    if (fast && (!aligned16(D_next) || !aligned16(W_next) || !aligned16(Z) || !aligned16(D_out))) return DAD_ERR_ALIGN;
    if (!fast && ceil_div(N, 64) > 65535) return DAD_ERR_SHAPE;  // grid.y limit of the guarded kernel
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    if (fast) {
        switch (act) {
            case DAD_ACT_RELU: return launch_backprop_fast<DAD_ACT_RELU>(D_next, W_next, Z, D_out, N, h, h_next, s);
            case DAD_ACT_TANH: return launch_backprop_fast<DAD_ACT_TANH>(D_next, W_next, Z, D_out, N, h, h_next, s);
            case DAD_ACT_SIGMOID: return launch_backprop_fast<DAD_ACT_SIGMOID>(D_next, W_next, Z, D_out, N, h, h_next, s);
            default: return launch_backprop_fast<DAD_ACT_IDENTITY>(D_next, W_next, Z, D_out, N, h, h_next, s);
        }
    }
    dim3 grid((unsigned)ceil_div(h, 64), (unsigned)ceil_div(N, 64));
    ProfScope prof(KID_BACKPROP, s);
    if (dt == DAD_BF16)
        hipLaunchKernelGGL(k_backprop<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)D_next, (const bf16_t*)W_next,
                           (const bf16_t*)Z, (bf16_t*)D_out, N, h, h_next, (int)act);
    else
        hipLaunchKernelGGL(k_backprop<float>, grid, dim3(256), 0, s, (const float*)D_next, (const float*)W_next,
                           (const float*)Z, (float*)D_out, N, h, h_next, (int)act);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

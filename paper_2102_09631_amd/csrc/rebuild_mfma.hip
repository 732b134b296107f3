// Full gradient rebuild G = L^T R (Eq. 4) for bf16 factors on the gfx950 matrix cores.
//
// Both operands are stored with the contraction index K (the sample/token row)
// as the slow axis, while a bf16 MFMA operand wants each lane to hold eight
// consecutive K values of one output row/column.  Tiles are therefore staged in
// LDS exactly as they sit in memory ([k][column], 16-byte chunks XOR-swizzled by
// the row to spread banks) and read back with the LDS transpose-read, which
// hands every lane four K-consecutive values of its column.
//
// One workgroup = 4 waves (2 x 2), one 256 x 256 output tile, a contiguous chunk
// of K.  Split-K partials are written as fp32 slabs and summed in fixed order by
// k_reduce_slabs, so results are reproducible bit for bit.
#include "dad_internal.h"

namespace dad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace rb {
constexpr int TILE = 256;             // output tile edge
constexpr int BK = 32;                // K rows per pipeline stage
constexpr int ROWB = TILE * 2;        // bytes per LDS row
constexpr int TILEB = BK * ROWB;      // bytes per operand tile
constexpr int STAGEB = 2 * TILEB;     // L tile + R tile
constexpr int NSTAGE = 2;
}  // namespace rb

// byte offset of 16-byte chunk `chunk` of row k inside an operand tile
__device__ __forceinline__ int rb_lds_off(int k, int chunk) { return k * rb::ROWB + ((chunk ^ ((k & 3) << 2)) << 4); }

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

// Eight K-consecutive bf16 of column (m0 + lane%32), K rows kb + 8*(lane/32) .. +7, from a [k][col] tile.
__device__ __forceinline__ bf16x8 rb_frag(const char* tile, int m0, int kb, int lane) {
    const int b = lane >> 4, s = lane & 15, j = s >> 2, g = s & 3;
    const int m = m0 + ((b & 1) << 4) + (g << 2);
    const int k = kb + ((b >> 1) << 3) + j;
    const char* p0 = tile + rb_lds_off(k, m >> 3) + ((g & 1) << 3);
    const char* p1 = tile + rb_lds_off(k + 4, m >> 3) + ((g & 1) << 3);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p1));
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// grid.x = tiles * splits.  Logical ids are laid out so that the workgroups that share an XCD
// (ids congruent mod 8) walk neighbouring tiles of the same K chunk and hit each other's L2 lines.
__global__ __launch_bounds__(256) void k_rebuild_bf16(const bf16_t* __restrict__ L, const bf16_t* __restrict__ R,
                                                      float* __restrict__ out, int64_t K, int h_in, int h_out,
                                                      int64_t chunk, int tiles_m, int tiles_n, int total) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware remap: hardware hands consecutive block ids to the 8 XCDs round-robin.
    int lid = blockIdx.x;
    {
        const int per = total >> 3, main = per << 3;
        if ((int)blockIdx.x < main) lid = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    }
    const int tiles = tiles_m * tiles_n;
    const int split = lid / tiles, tile = lid - split * tiles;
    int pm, qn;
    if (tiles_m <= tiles_n) {
        pm = tile % tiles_m;
        qn = tile / tiles_m;
    } else {
        qn = tile % tiles_n;
        pm = tile / tiles_n;
    }
    const int p0 = pm * rb::TILE, q0 = qn * rb::TILE;
    const int64_t kbeg = (int64_t)split * chunk;
    const int64_t kend = (kbeg + chunk < K) ? kbeg + chunk : K;
    const int nk = (int)((kend - kbeg + rb::BK - 1) / rb::BK);

    // global -> register staging: thread owns chunk c of rows r0 + 8*i
    const int c = t & 31, r0 = t >> 5;
    const bf16_t* gl = L + (kbeg + r0) * (int64_t)h_in + p0 + c * 8;
    const bf16_t* gr = R + (kbeg + r0) * (int64_t)h_out + q0 + c * 8;
    const int st_off = rb_lds_off(r0, c);  // (r0 + 8*i) & 3 == r0 & 3
    u32x4 sl[4], sr[4];

    auto gload = [&](int kt) {
        const int64_t kb = kbeg + (int64_t)kt * rb::BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t row = kb + r0 + 8 * i;
            if (row < kend) {
                sl[i] = *reinterpret_cast<const u32x4*>(gl + ((int64_t)kt * rb::BK + 8 * i) * h_in);
                sr[i] = *reinterpret_cast<const u32x4*>(gr + ((int64_t)kt * rb::BK + 8 * i) * h_out);
            } else {
                sl[i] = (u32x4){0, 0, 0, 0};
                sr[i] = (u32x4){0, 0, 0, 0};
            }
        }
    };
    auto lstore = [&](int stage) {
        char* base = smem + stage * rb::STAGEB;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<u32x4*>(base + st_off + 8 * i * rb::ROWB) = sl[i];
            *reinterpret_cast<u32x4*>(base + rb::TILEB + st_off + 8 * i * rb::ROWB) = sr[i];
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    gload(0);
    lstore(0);
    __syncthreads();
    if (nk > 1) gload(1);

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const char* tl = smem + cur * rb::STAGEB;
        const char* tr = tl + rb::TILEB;
#pragma unroll
        for (int ks = 0; ks < rb::BK / 16; ++ks) {
            bf16x8 fa[4], fb[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) fa[a] = rb_frag(tl, wm * 128 + a * 32, ks * 16, lane);
#pragma unroll
            for (int b = 0; b < 4; ++b) fb[b] = rb_frag(tr, wn * 128 + b * 32, ks * 16, lane);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            lstore(cur ^ 1);
            if (kt + 2 < nk) gload(kt + 2);
        }
        __syncthreads();
    }

    float* o = out + (int64_t)split * h_in * h_out;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int q = q0 + wn * 128 + b * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int p = p0 + wm * 128 + a * 32 + ((v >> 2) << 3) + ((lane >> 5) << 2) + (v & 3);
                o[(int64_t)p * h_out + q] = acc[a][b][v];
            }
        }
}

dad_status reduce_slabs(const float* part, float* out, int64_t n, int splits, hipStream_t s);

bool rebuild_fast_ok(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt) {
    return dt == DAD_BF16 && h_in % rb::TILE == 0 && h_out % rb::TILE == 0 && K >= 256 && h_in <= (1 << 20) &&
           h_out <= (1 << 20);
}

// Number of K chunks: fill the 256 CUs with whole rounds of workgroups while keeping the fp32
// partial traffic (splits * h_in * h_out * 4 bytes) small next to the operand reads.
SplitPlan rebuild_fast_split(int64_t K, int64_t h_in, int64_t h_out) {
    const int64_t tiles = (h_in / rb::TILE) * (h_out / rb::TILE);
    int best = 1;
    double best_score = -1.0;
    for (int s = 1; s <= 64; ++s) {
        if (s > 1 && K / s < 1024) break;
        const int64_t wg = tiles * s;
        const double eff = (double)wg / (double)(ceil_div(wg, 256) * 256);
        const double ops = (double)K * (h_in + h_out) * 2.0;
        const double extra = s > 1 ? (2.0 * s + 1.0) * h_in * h_out * 4.0 : 0.0;
        const double score = eff / (1.0 + extra / ops);
        if (score > best_score * 1.02) {
            best_score = score;
            best = s;
        }
    }
    SplitPlan sp;
    sp.chunk = (int64_t)align_up((size_t)ceil_div(K, best), rb::BK);
    sp.splits = (int)ceil_div(K, sp.chunk);
    return sp;
}

dad_status fast_rebuild(const void* L, const void* R, int64_t K, int64_t h_in, int64_t h_out, float* G, float* partials,
                        SplitPlan sp, hipStream_t s) {
    static bool attr_set = false;
    const int lds = rb::NSTAGE * rb::STAGEB;
    if (!attr_set) {
        DAD_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_rebuild_bf16),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_set = true;
    }
    const int tm = (int)(h_in / rb::TILE), tn = (int)(h_out / rb::TILE);
    const int total = tm * tn * sp.splits;
    float* dst = sp.splits == 1 ? G : partials;
    {
        ProfScope prof(KID_REBUILD_BF16, s);
        hipLaunchKernelGGL(k_rebuild_bf16, dim3((unsigned)total), dim3(256), lds, s, (const bf16_t*)L, (const bf16_t*)R,
                           dst, K, (int)h_in, (int)h_out, sp.chunk, tm, tn, total);
    }
    DAD_LAUNCH_CHECK();
    if (sp.splits > 1) return reduce_slabs(partials, G, h_in * h_out, sp.splits, s);
    return DAD_OK;
}

}  // namespace dad

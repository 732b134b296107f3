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
#include <type_traits>

#include "dad_internal.h"

namespace dad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace rb {
constexpr int TILE = 256;             // output tile edge
constexpr int BK = 32;                // K rows per pipeline stage
constexpr int ROWB = TILE * 2;        // bytes per LDS row
constexpr int TILEB = BK * ROWB;      // bytes per operand tile
constexpr int STAGEB = 2 * TILEB;     // L tile + R tile
constexpr int NSTAGE = 2;
}  // namespace rb

// byte offset of 16-byte chunk `chunk` of row k inside an operand tile whose rows are ROWB bytes
template <int ROWB = rb::ROWB>
__device__ __forceinline__ int rb_lds_off(int k, int chunk) { return k * ROWB + ((chunk ^ ((k & 3) << 2)) << 4); }

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

// Eight K-consecutive bf16 of column (m0 + lane%32), K rows kb + 8*(lane/32) .. +7, from a [k][col] tile.
template <int ROWB = rb::ROWB>
__device__ __forceinline__ bf16x8 rb_frag(const char* tile, int m0, int kb, int lane) {
    const int b = lane >> 4, s = lane & 15, j = s >> 2, g = s & 3;
    const int m = m0 + ((b & 1) << 4) + (g << 2);
    const int k = kb + ((b >> 1) << 3) + j;
    const char* p0 = tile + rb_lds_off<ROWB>(k, m >> 3) + ((g & 1) << 3);
    const char* p1 = tile + rb_lds_off<ROWB>(k + 4, m >> 3) + ((g & 1) << 3);
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

// ---------------------------------------------------------------------------------------------
// Variant for K chunks that are whole multiples of BK: the operand tiles go from HBM straight into
// LDS (no register staging), through a ring of DMA_STAGES buffers, so three tiles per workgroup are
// in flight while the fourth is multiplied.  The XOR swizzle is applied on the global side: the
// lane that owns LDS chunk position c' of row k fetches global chunk c' ^ ((k & 3) << 2).
// The loads are issued through inline assembly because the compiler would otherwise wait for ALL
// outstanding LDS-bound loads before any LDS read; the waits are placed by hand instead.
//
// Eight waves (2 x 4, each 128 x 64 of the tile) rather than four: a wave can keep at most fifteen
// LDS reads in flight, and with one wave per SIMD the transpose-reads deliver only ~64 B/clk per CU,
// exactly what four 128 x 128 waves need at full MFMA rate; two waves per SIMD roughly double it.
namespace rb {
constexpr int DMA_STAGES = 4;
constexpr int DMA_LOADS = 4;  // 16-byte loads per thread per stage, for both tile sizes
}  // namespace rb

// T = tile edge, WM x WN waves, each (T/WM) x (T/WN) of the tile.  T = 256 with 2 x 4 waves is the
// kernel for large gradients.  T = 128 with 2 x 2 waves (two workgroups per CU) serves gradients with
// few 256-tiles, where filling the chip would otherwise take so many K chunks that their fp32
// partial slabs outweigh the operand reads.
// SRC is `const bf16_t*` (operands in one allocation each) or RowBlocks (the sites' blocks in
// place, the same row split for both operands, every block a multiple of 256 rows): a K chunk may
// span blocks, and the operand pointers jump at a block's end.
// The XCD-aware order of the workgroups of a launch: ids congruent mod 8 share an XCD and get
// consecutive logical ids.
__device__ __forceinline__ int rb_logical_id(int total) {
    const int per = total >> 3, main = per << 3;
    return (int)blockIdx.x < main ? (int)((blockIdx.x & 7) * per + (blockIdx.x >> 3)) : (int)blockIdx.x;
}

// One workgroup's tile: `lid` is its logical index among the tiles_m * tiles_n * splits of this product.
template <int T, int WM, int WN, typename SRC>
__device__ __forceinline__ void rebuild_tile_dma(const SRC& L, const SRC& R, float* __restrict__ out, int64_t K, int h_in,
                                                 int h_out, int64_t chunk, int tiles_m, int tiles_n, int lid) {
    constexpr int WAVES = WM * WN;
    constexpr int FA = T / (32 * WM), FB = T / (32 * WN);  // 32-wide fragments per wave
    constexpr int ROWB = T * 2;                            // bytes per LDS row
    constexpr int TILEB = rb::BK * ROWB;
    constexpr int STAGEB = 2 * TILEB;
    constexpr int CPR = ROWB / 16;                         // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;                          // tile rows covered by one load of a wave
    static_assert(rb::BK == 2 * RPI * WAVES, "two loads per wave and operand cover a stage");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;

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
    const int p0 = pm * T, q0 = qn * T;
    const int64_t kbeg = (int64_t)split * chunk;
    const int64_t kend = (kbeg + chunk < K) ? kbeg + chunk : K;
    const int nk = (int)((kend - kbeg) / rb::BK);  // host guarantees whole tiles

    // this lane's two rows per operand tile: row = 2*RPI*wave + RPI*i + lane/CPR, LDS chunk position lane%CPR
    RowCursor cur_l, cur_r;
    const char* l0 = row_address(L, kbeg, (int64_t)h_in * 2, cur_l);
    const char* r0 = row_address(R, kbeg, (int64_t)h_out * 2, cur_r);
    int64_t row_next = kbeg;  // first row of the next tile to be issued
    const char* gl[2];
    const char* gr[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = 2 * RPI * wave + RPI * i + lane / CPR;
        const int c = (lane % CPR) ^ ((row & 3) << 2);
        gl[i] = l0 + (row * (int64_t)h_in + p0 + c * 8) * 2;
        gr[i] = r0 + (row * (int64_t)h_out + q0 + c * 8) * 2;
    }
    const int64_t adv_l = (int64_t)rb::BK * h_in * 2, adv_r = (int64_t)rb::BK * h_out * 2;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    auto issue = [&](int stage) {  // loads the next tile in sequence into ring slot `stage`
        // wave-uniform by construction; readfirstlane lets the compiler keep it in a scalar register
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGEB + (2 * RPI * wave) * ROWB);
        if constexpr (!std::is_pointer<SRC>::value) {
            if (row_next == cur_l.end) {
                const int64_t jl = block_jump(L, (int64_t)h_in * 2, cur_l);
                const int64_t jr = block_jump(R, (int64_t)h_out * 2, cur_r);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    gl[i] += jl;
                    gr[i] += jr;
                }
            }
            row_next += rb::BK;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dma16(gl[i], base + RPI * i * ROWB);
            gl[i] += adv_l;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            dma16(gr[i], base + TILEB + RPI * i * ROWB);
            gr[i] += adv_r;
        }
    };

    f32x16 acc[FA][FB];
#pragma unroll
    for (int a = 0; a < FA; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

#pragma unroll
    for (int s = 0; s < rb::DMA_STAGES - 1; ++s)
        if (s < nk) issue(s);

    // Each K tile is two MFMA K-steps (ks = 0, 1) with fragment sets 0 and 1.  The second step of a
    // tile is multiplied after the next tile's barrier, so the matrix cores have independent MFMAs to
    // chew on while the first fragments of the new tile travel from LDS:
    //   barrier | DMA(kt+3) | read set0(kt,0) x MFMA set1(kt-1,1) | read set1(kt,1) x MFMA set0(kt,0) | ...
    // where "x" is an instruction-by-instruction interleave: one or two fragment reads between
    // consecutive MFMAs (measured 6-7 % faster than reads and MFMAs in blocks: 67 % instead of 60 % of
    // peak on all-zero operands, 49 % instead of 46 % on the benchmark's).
    bf16x8 fa0[FA], fb0[FB], fa1[FA], fb1[FB];
    // set 1 starts as zeros, so that the first tile's "previous K-step" multiplies into zero accumulators
#pragma unroll
    for (int a = 0; a < FA; ++a) fa1[a] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < FB; ++b) fb1[b] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    auto read_frags = [&](bf16x8 (&fa)[FA], bf16x8 (&fb)[FB], const char* tl, int ks) {
        const char* tr = tl + TILEB;
#pragma unroll
        for (int a = 0; a < FA; ++a) fa[a] = rb_frag<ROWB>(tl, wm * (FA * 32) + a * 32, ks * 16, lane);
#pragma unroll
        for (int b = 0; b < FB; ++b) fb[b] = rb_frag<ROWB>(tr, wn * (FB * 32) + b * 32, ks * 16, lane);
    };
    auto mma = [&](const bf16x8 (&fa)[FA], const bf16x8 (&fb)[FB]) {
#pragma unroll
        for (int a = 0; a < FA; ++a)
#pragma unroll
            for (int b = 0; b < FB; ++b)
                // R fragment as the MFMA's row operand: each lane then owns four consecutive q of one p
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[b], fa[a], acc[a][b], 0, 0, 0);
    };

    // One K tile; STAGE is a compile-time ring slot so every LDS address is lane offset + constant.
    auto step = [&](int kt, auto stage_c) {
        constexpr int STAGE = decltype(stage_c)::value;
        // tile kt has landed once at most DMA_STAGES-2 younger tiles are outstanding
        if (kt + rb::DMA_STAGES - 2 < nk)
            wait_vmcnt<rb::DMA_LOADS * (rb::DMA_STAGES - 2)>();
        else
            wait_vmcnt<0>();
        __syncthreads();  // everyone's part of tile kt is in LDS, and tile kt-1's slot is free
        if (kt + rb::DMA_STAGES - 1 < nk) issue((STAGE + rb::DMA_STAGES - 1) % rb::DMA_STAGES);
        const char* tl = smem + STAGE * STAGEB;
        constexpr int NR = 2 * (FA + FB), NM = FA * FB;  // LDS reads and MFMAs per K-step
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa0, fb0, tl, 0);
        mma(fa1, fb1);
        interleave_reads_mfma<NR, NM, true>();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fa1, fb1, tl, 1);
        mma(fa0, fb0);
        interleave_reads_mfma<NR, NM, false>();
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int kt = 0; kt < nk; kt += rb::DMA_STAGES) {
        step(kt, std::integral_constant<int, 0>{});
        if (kt + 1 < nk) step(kt + 1, std::integral_constant<int, 1>{});
        if (kt + 2 < nk) step(kt + 2, std::integral_constant<int, 2>{});
        if (kt + 3 < nk) step(kt + 3, std::integral_constant<int, 3>{});
    }
    if (nk > 0) mma(fa1, fb1);

    // D[q][p] layout: lane holds p = lane % 32 and q = 8*g + 4*(lane/32) + 0..3 for g = 0..3: 16-byte stores
    float* o = out + (int64_t)split * h_in * h_out;
#pragma unroll
    for (int a = 0; a < FA; ++a)
#pragma unroll
        for (int b = 0; b < FB; ++b) {
            const int p = p0 + wm * (FA * 32) + a * 32 + (lane & 31);
            const int qb = q0 + wn * (FB * 32) + b * 32 + ((lane >> 5) << 2);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v4 = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                *reinterpret_cast<f32x4*>(o + (int64_t)p * h_out + qb + 8 * g) = v4;
            }
        }
}

template <int T, int WM, int WN, typename SRC>
__global__ __launch_bounds__(64 * WM * WN) void k_rebuild_bf16_dma(const SRC L, const SRC R,
                                                                  float* __restrict__ out, int64_t K, int h_in,
                                                                  int h_out, int64_t chunk, int tiles_m,
                                                                  int tiles_n, int total) {
    rebuild_tile_dma<T, WM, WN, SRC>(L, R, out, K, h_in, h_out, chunk, tiles_m, tiles_n, rb_logical_id(total));
}

// Several products in one launch (the full gradients of the layers of a block): gradients with few
// 256-tiles fill the chip together, so each needs fewer K chunks and writes fewer fp32 slabs.
namespace rb {
constexpr int MAX_JOBS = 16;
}
struct RebuildJob {
    const bf16_t* L;
    const bf16_t* R;
    float* out;  // G, or the first of its slabs
    int64_t K, chunk;
    int h_in, h_out, tiles_m, tiles_n;
};
struct RebuildJobs {
    int first_block[rb::MAX_JOBS];  // first logical id of each job; entries beyond the last job hold INT_MAX
    RebuildJob j[rb::MAX_JOBS];
};

template <int T, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void k_rebuild_bf16_dma_jobs(RebuildJobs tb, int total) {
    const int lid = rb_logical_id(total);
    int ji = 0;
#pragma unroll
    for (int i = 1; i < rb::MAX_JOBS; ++i) ji += tb.first_block[i] <= lid ? 1 : 0;
    const RebuildJob& jb = tb.j[ji];
    const bf16_t* L = jb.L;
    const bf16_t* R = jb.R;
    rebuild_tile_dma<T, WM, WN, const bf16_t*>(L, R, jb.out, jb.K, jb.h_in, jb.h_out, jb.chunk, jb.tiles_m, jb.tiles_n,
                                               lid - tb.first_block[ji]);
}



bool rebuild_fast_ok(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt) {
    if (dt != DAD_BF16 || K < 256 || h_in > (1 << 20) || h_out > (1 << 20)) return false;
    if (h_in % 256 == 0 && h_out % 256 == 0) return true;
    return h_in % 128 == 0 && h_out % 128 == 0 && K % rb::BK == 0;  // 128-tiles: whole K stages only
}

// Score of a tiling: share of the CU slots that whole rounds of workgroups fill, discounted by the
// fp32 partial traffic (splits * h_in * h_out * 4 bytes written, read, and the result written) next
// to the operand reads, and for 128-tiles by their doubled L2->LDS traffic per flop.
static double rebuild_score(int64_t K, int64_t h_in, int64_t h_out, int tile, int s) {
    const int64_t wg = (h_in / tile) * (h_out / tile) * s;
    const int64_t slots = tile == 256 ? 256 : 512;
    const double eff = (double)wg / (double)(ceil_div(wg, slots) * slots);
    const double ops = (double)K * (h_in + h_out) * 2.0;
    const double extra = s > 1 ? (2.0 * s + 1.0) * h_in * h_out * 4.0 : 0.0;
    return eff / (1.0 + extra / ops) * (tile == 256 ? 1.0 : 0.8);
}

// Tile edge and number of K chunks.
SplitPlan rebuild_fast_split(int64_t K, int64_t h_in, int64_t h_out, int* tile_out) {
    int best = 1, best_tile = 0;
    double best_score = -1.0;
    for (int tile : {256, 128}) {
        if (h_in % tile || h_out % tile) continue;
        if (tile == 128 && K % rb::BK) continue;
        for (int s = 1; s <= 64; ++s) {
            if (s > 1 && K / s < 1024) break;
            const double score = rebuild_score(K, h_in, h_out, tile, s);
            if (score > best_score * 1.02) {
                best_score = score;
                best = s;
                best_tile = tile;
            }
        }
    }
    SplitPlan sp;
    sp.chunk = (int64_t)align_up((size_t)ceil_div(K, best), rb::BK);
    sp.splits = (int)ceil_div(K, sp.chunk);
    *tile_out = best_tile;
    return sp;
}

template <int T, int WM, int WN>
static dad_status launch_rebuild_dma(const void* L, const void* R, const RowBlocks* lb, const RowBlocks* rbk, float* dst,
                                     int64_t K, int64_t h_in, int64_t h_out, SplitPlan sp, hipStream_t s) {
    const int lds = rb::DMA_STAGES * 2 * rb::BK * T * 2;
    const int tm = (int)(h_in / T), tn = (int)(h_out / T);
    const int total = tm * tn * sp.splits;
    ProfScope prof(KID_REBUILD_BF16_DMA, s);
    if (lb)
        hipLaunchKernelGGL((k_rebuild_bf16_dma<T, WM, WN, RowBlocks>), dim3((unsigned)total), dim3(64 * WM * WN), lds, s,
                           *lb, *rbk, dst, K, (int)h_in, (int)h_out, sp.chunk, tm, tn, total);
    else
        hipLaunchKernelGGL((k_rebuild_bf16_dma<T, WM, WN, const bf16_t*>), dim3((unsigned)total), dim3(64 * WM * WN), lds,
                           s, (const bf16_t*)L, (const bf16_t*)R, dst, K, (int)h_in, (int)h_out, sp.chunk, tm, tn, total);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

// True when fast_rebuild takes the direct-to-LDS kernel.
bool rebuild_dma_ok(int64_t K, SplitPlan sp) { return K % rb::BK == 0 && sp.chunk % rb::BK == 0; }

// lb / rbk, when not null, give both operands as row blocks (L and R are then unused); only the
// direct-to-LDS kernel reads blocks.
dad_status fast_rebuild(const void* L, const void* R, const RowBlocks* lb, const RowBlocks* rbk, int64_t K, int64_t h_in,
                        int64_t h_out, float* G, float* partials, SplitPlan sp, int tile, hipStream_t s) {
    float* dst = sp.splits == 1 ? G : partials;
    dad_status rc;
    if ((lb != nullptr) != (rbk != nullptr) || (lb && !rebuild_dma_ok(K, sp))) return DAD_ERR_SHAPE;
    if (rebuild_dma_ok(K, sp)) {
        rc = tile == 128 ? launch_rebuild_dma<128, 2, 2>(L, R, lb, rbk, dst, K, h_in, h_out, sp, s)
                         : launch_rebuild_dma<256, 2, 4>(L, R, lb, rbk, dst, K, h_in, h_out, sp, s);
        if (rc != DAD_OK) return rc;
    } else {  // ragged K: register-staged kernel, 256-tiles (the plan never picks 128-tiles here)
        const int lds = rb::NSTAGE * rb::STAGEB;
        const int tm = (int)(h_in / rb::TILE), tn = (int)(h_out / rb::TILE);
        const int total = tm * tn * sp.splits;
        ProfScope prof(KID_REBUILD_BF16, s);
        hipLaunchKernelGGL(k_rebuild_bf16, dim3((unsigned)total), dim3(256), lds, s, (const bf16_t*)L, (const bf16_t*)R,
                           dst, K, (int)h_in, (int)h_out, sp.chunk, tm, tn, total);
        DAD_LAUNCH_CHECK();
    }
    if (sp.splits > 1) return reduce_slabs(partials, G, h_in * h_out, sp.splits, s);
    return DAD_OK;
}

// True when a product can join a launch of several: whole 256-tiles and whole K stages.
bool rebuild_group_ok(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt) {
    return dt == DAD_BF16 && K >= 256 && K % rb::BK == 0 && h_in % 256 == 0 && h_out % 256 == 0 && h_in <= (1 << 20) &&
           h_out <= (1 << 20);
}

// Number of K chunks for n products launched together (the same for all of them): the score of
// rebuild_fast_split on the totals.
int rebuild_group_splits(int n, const int64_t* K, const int64_t* h_in, const int64_t* h_out) {
    int64_t tiles = 0, kmin = K[0];
    double ops = 0.0, outs = 0.0;
    for (int i = 0; i < n; ++i) {
        tiles += (h_in[i] / 256) * (h_out[i] / 256);
        ops += (double)K[i] * (h_in[i] + h_out[i]) * 2.0;
        outs += (double)h_in[i] * h_out[i] * 4.0;
        if (K[i] < kmin) kmin = K[i];
    }
    int best = 1;
    double best_score = -1.0;
    for (int s = 1; s <= 64; ++s) {
        if (s > 1 && kmin / s < 1024) break;
        const int64_t wg = tiles * s;
        const double eff = (double)wg / (double)(ceil_div(wg, 256) * 256);
        const double extra = s > 1 ? (2.0 * s + 1.0) * outs : 0.0;
        const double score = eff / (1.0 + extra / ops);
        if (score > best_score * 1.02) {
            best_score = score;
            best = s;
        }
    }
    return best;
}

SplitPlan rebuild_group_plan(int64_t K, int splits) {
    SplitPlan sp;
    sp.chunk = (int64_t)align_up((size_t)ceil_div(K, splits), rb::BK);
    sp.splits = (int)ceil_div(K, sp.chunk);
    return sp;
}

// n products (every one passes rebuild_group_ok; sp[i] from rebuild_group_plan) in launches of up to
// rb::MAX_JOBS; a product with sp[i].splits > 1 goes through slabs[i] and reduce_slabs.
dad_status launch_rebuild_group(int n, const void* const* L, const void* const* R, float* const* G, const int64_t* K,
                                const int64_t* h_in, const int64_t* h_out, const SplitPlan* sp, float* const* slabs,
                                hipStream_t s) {
    const int lds = rb::DMA_STAGES * 2 * rb::BK * 256 * 2;
    for (int first = 0; first < n; first += rb::MAX_JOBS) {
        const int cnt = n - first < rb::MAX_JOBS ? n - first : rb::MAX_JOBS;
        RebuildJobs tb;
        int64_t blocks = 0;
        for (int i = 0; i < rb::MAX_JOBS; ++i) {
            if (i >= cnt) {
                tb.first_block[i] = 0x7fffffff;
                tb.j[i] = RebuildJob{};
                continue;
            }
            const int k = first + i;
            RebuildJob& jb = tb.j[i];
            jb.L = static_cast<const bf16_t*>(L[k]);
            jb.R = static_cast<const bf16_t*>(R[k]);
            jb.out = sp[k].splits == 1 ? G[k] : slabs[k];
            jb.K = K[k];
            jb.chunk = sp[k].chunk;
            jb.h_in = (int)h_in[k];
            jb.h_out = (int)h_out[k];
            jb.tiles_m = (int)(h_in[k] / 256);
            jb.tiles_n = (int)(h_out[k] / 256);
            tb.first_block[i] = (int)blocks;
            blocks += (int64_t)jb.tiles_m * jb.tiles_n * sp[k].splits;
            if (blocks > ((int64_t)1 << 30)) return DAD_ERR_SHAPE;
        }
        {
            ProfScope prof(KID_REBUILD_BF16_DMA, s);
            hipLaunchKernelGGL((k_rebuild_bf16_dma_jobs<256, 2, 4>), dim3((unsigned)blocks), dim3(512), lds, s, tb, (int)blocks);
        }
        DAD_LAUNCH_CHECK();
    }
    for (int i = 0; i < n; ++i) {
        if (sp[i].splits == 1) continue;
        const dad_status rc = reduce_slabs(slabs[i], G[i], h_in[i] * h_out[i], sp[i].splits, s);
        if (rc != DAD_OK) return rc;
    }
    return DAD_OK;
}

dad_status rebuild_prepare_device() {
    DAD_HIP_TRY(set_max_lds((k_rebuild_bf16_dma_jobs<256, 2, 4>), rb::DMA_STAGES * 2 * rb::BK * 256 * 2));
    DAD_HIP_TRY(set_max_lds((k_rebuild_bf16_dma<256, 2, 4, const bf16_t*>), rb::DMA_STAGES * 2 * rb::BK * 256 * 2));
    DAD_HIP_TRY(set_max_lds((k_rebuild_bf16_dma<128, 2, 2, const bf16_t*>), rb::DMA_STAGES * 2 * rb::BK * 128 * 2));
    DAD_HIP_TRY(set_max_lds((k_rebuild_bf16_dma<256, 2, 4, RowBlocks>), rb::DMA_STAGES * 2 * rb::BK * 256 * 2));
    DAD_HIP_TRY(set_max_lds((k_rebuild_bf16_dma<128, 2, 2, RowBlocks>), rb::DMA_STAGES * 2 * rb::BK * 128 * 2));
    DAD_HIP_TRY(set_max_lds(k_rebuild_bf16, rb::NSTAGE * rb::STAGEB));
    return DAD_OK;
}

}  // namespace dad

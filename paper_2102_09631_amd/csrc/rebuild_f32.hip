// Gradient rebuild G = L^T R (Eq. 4) for fp32 operands on the fp32 matrix instruction: the full
// gradient of the fp32 workloads (K = N) and the rank-r gradient P G^T of every workload (K = r; the
// sites' local rebuild of Algorithm 1).
//
// v_mfma_f32_32x32x2_f32 takes ONE value per lane and operand: lane l supplies A[l % 32][l / 32] and
// B[l / 32][l % 32], i.e. 32 consecutive floats of one K row of a factor per half wave - exactly how
// the factors lie in memory, so no transposition is needed anywhere.  Tiles of 16 K rows are staged in
// LDS as they are (16-byte global loads; one-float accesses to global memory cost the memory
// pipeline as much as 16-byte ones and held a register-only version at a third of this one's rate)
// and the operands are read from there one float per lane, conflict free.  R supplies the MFMA's
// row operand, so that a lane ends up with four consecutive q of one p and the result leaves as
// 16-byte stores.  Every staged element outside the matrices is zero, so any K, h_in, h_out is served
// (widths that are not multiples of 4 take one-float global accesses).
//
// One launch can serve several layers (a table of jobs in the kernel argument): the rank-r rebuild of
// one layer writes a few MB and is launch bound on its own.
#include <type_traits>

#include "dad_internal.h"

namespace dad {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace rf {
constexpr int WM = 2, WN = 2;          // waves per workgroup
constexpr int KC = 16;                 // K rows per LDS stage
constexpr int MAX_JOBS = 32;
}  // namespace rf

struct RebuildF32Job {
    const float* L;
    const float* R;
    float* out;        // G, or the first of `splits` slabs of h_in * h_out floats
    int64_t K, chunk;  // chunk = K rows per split (a multiple of 8 unless splits == 1)
    int h_in, h_out, tiles_n, tiles, splits, pad;
};

struct RebuildF32Jobs {
    int first_block[rf::MAX_JOBS];  // first workgroup of each job; entries beyond the last job hold INT_MAX
    RebuildF32Job j[rf::MAX_JOBS];
};

// FM x FN accumulator tiles of 32 x 32 per wave: 2 x 4 (a wave owns 64 x 128, a workgroup 128 x 256;
// six LDS reads feed eight MFMAs per pair of K rows) for large outputs, 1 x 2 (workgroup 64 x 128)
// when the larger tile would leave most of the chip without a workgroup.  VEC: rows of both factors
// and of G are 16-byte aligned (h_in and h_out multiples of 4).
template <int FM, int FN, bool VEC>
__global__ __launch_bounds__(256) void k_rebuild_f32_mfma(RebuildF32Jobs tb) {
    constexpr int TM = rf::WM * FM * 32, TN = rf::WN * FN * 32, TW = TM + TN;
    constexpr int UNIT = VEC ? 4 : 1;                       // floats per staging access
    constexpr int NLD = rf::KC * TW / UNIT / 256;            // staging accesses per thread and stage
    static_assert(NLD * 256 * UNIT == rf::KC * TW, "the staging loads cover a stage");
    __shared__ __attribute__((aligned(16))) float lds[2][rf::KC][TW];  // [k][ L columns | R columns ]

    // which job: the whole table of first blocks is fetched at once and compared without a loop
    int ji = 0;
#pragma unroll
    for (int i = 1; i < rf::MAX_JOBS; ++i) ji += tb.first_block[i] <= (int)blockIdx.x ? 1 : 0;
    const RebuildF32Job& jb = tb.j[ji];
    const int local = (int)blockIdx.x - tb.first_block[ji];
    const int split = local / jb.tiles, tile = local - split * jb.tiles;
    const int pm = tile / jb.tiles_n, qn = tile - pm * jb.tiles_n;
    const int h_in = jb.h_in, h_out = jb.h_out;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / rf::WN, wn = wave % rf::WN;
    const int c = lane & 31, kh = lane >> 5;
    const int p0 = pm * TM, q0 = qn * TN;
    const int64_t kbeg = (int64_t)split * jb.chunk;
    const int64_t kend = (kbeg + jb.chunk < jb.K) ? kbeg + jb.chunk : jb.K;

    // Staging: access i of this thread is unit e = t + 256 i of the stage, row e / (TW / UNIT), and a
    // column of L or of R.  The address is clamped to a valid one and the value zeroed by a select at
    // the LDS store, so that the loads of a stage are issued together.
    typedef typename std::conditional<VEC, f32x4, float>::type unit_t;
    const float* src[NLD];
    int64_t pitch[NLD];
    int srow[NLD], scol[NLD];
    bool colok[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int e = t + 256 * i;
        srow[i] = e / (TW / UNIT);
        scol[i] = (e % (TW / UNIT)) * UNIT;
        if (scol[i] < TM) {
            const int p = p0 + scol[i];
            colok[i] = p < h_in;  // VEC: h_in % 4 == 0, so the whole unit is inside
            src[i] = jb.L + (colok[i] ? p : 0);
            pitch[i] = h_in;
        } else {
            const int q = q0 + scol[i] - TM;
            colok[i] = q < h_out;
            src[i] = jb.R + (colok[i] ? q : 0);
            pitch[i] = h_out;
        }
    }
    unit_t st[NLD];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int64_t k = k0 + srow[i];
            st[i] = *reinterpret_cast<const unit_t*>(src[i] + (k < kend ? k : kend - 1) * pitch[i]);
        }
    };
    auto commit = [&](int stage, int64_t k0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const bool ok = colok[i] && k0 + srow[i] < kend;
            unit_t v = st[i];
            if (!ok) v = unit_t{};
            *reinterpret_cast<unit_t*>(&lds[stage][srow[i]][scol[i]]) = v;
        }
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int lcol = wm * (FM * 32) + c, rcol = TM + wn * (FN * 32) + c;
    fetch(kbeg);
    int stage = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += rf::KC) {
        commit(stage, k0);
        __syncthreads();
        if (k0 + rf::KC < kend) fetch(k0 + rf::KC);  // in flight during the MFMAs below
#pragma unroll
        for (int kk = 0; kk < rf::KC; kk += 2) {
            float x[FM], y[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a) x[a] = lds[stage][kk + kh][lcol + a * 32];
#pragma unroll
            for (int b = 0; b < FN; ++b) y[b] = lds[stage][kk + kh][rcol + b * 32];
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    // L as the row operand: a lane owns one q and 16 p, a half wave 32 consecutive q
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(x[a], y[b], acc[a][b], 0, 0, 0);
        }
        stage ^= 1;  // the other buffer was last read before the barrier above
    }

    // result tile (a, b): lane holds column q = ... + lane % 32 and rows 8 (v / 4) + 4 (lane / 32) + v % 4:
    // the 32 lanes of a half wave write one whole 128-byte line of a row of G per store
    float* o = jb.out + (int64_t)split * h_in * h_out;
    const int pw = p0 + wm * (FM * 32) + (kh << 2), qw = q0 + wn * (FN * 32) + c;
    if (p0 + wm * (FM * 32) + FM * 32 <= h_in && q0 + wn * (FN * 32) + FN * 32 <= h_out) {
        float* base = o + (int64_t)pw * h_out + qw;  // interior: one address per row, FN stores at constant offsets
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float* rowp = base + (int64_t)(a * 32 + ((v >> 2) << 3) + (v & 3)) * h_out;
#pragma unroll
                for (int b = 0; b < FN; ++b) rowp[b * 32] = acc[a][b][v];
            }
        return;
    }
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) {
            const int q = qw + b * 32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int p = pw + a * 32 + ((v >> 2) << 3) + (v & 3);
                if (p < h_in && q < h_out) o[(int64_t)p * h_out + q] = acc[a][b][v];
            }
        }
}

// A job may take the large tile when its widths allow 16-byte accesses (the one-float staging of odd
// widths needs too many registers for it).  Its result does not depend on the tile: every element is
// summed over k in ascending pairs either way.
static bool rebuild_f32_vec(int64_t h_in, int64_t h_out) { return h_in % 4 == 0 && h_out % 4 == 0; }
static int64_t rebuild_f32_big_tiles(int64_t h_in, int64_t h_out) { return ceil_div(h_in, 128) * ceil_div(h_out, 256); }

// Split of the contraction for one fp32 rebuild: about two workgroups per compute unit, chunks of at
// least 256 rows (even, so that the pairs of K rows of one MFMA stay inside a chunk).
SplitPlan rebuild_f32_split(int64_t K, int64_t h_in, int64_t h_out) {
    // planned for the job on its own: the large tile if that alone gives 512 workgroups
    const bool big = rebuild_f32_vec(h_in, h_out) && rebuild_f32_big_tiles(h_in, h_out) >= 512;
    const int64_t tiles = big ? rebuild_f32_big_tiles(h_in, h_out) : ceil_div(h_in, 64) * ceil_div(h_out, 128);
    int64_t want = ceil_div(512, tiles);
    const int64_t max_splits = ceil_div(K, 256);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    SplitPlan sp;
    sp.chunk = (int64_t)align_up((size_t)ceil_div(K, want), 8);
    sp.splits = (int)ceil_div(K, sp.chunk);
    return sp;
}

// Launches n jobs (G_i = L_i^T R_i, each with its own split plan; a job with splits > 1 writes slabs
// at slabs[i] and is summed by reduce_slabs afterwards) in as few launches as the job table allows.
dad_status launch_rebuild_f32(int n, const void* const* L, const void* const* R, float* const* G, const int64_t* K,
                              const int64_t* h_in, const int64_t* h_out, const SplitPlan* sp, float* const* slabs,
                              hipStream_t s, int kid) {
    // the large tile for the 16-byte jobs when together they fill the chip twice over with it
    int64_t big_total = 0;
    for (int i = 0; i < n; ++i)
        if (rebuild_f32_vec(h_in[i], h_out[i])) big_total += rebuild_f32_big_tiles(h_in[i], h_out[i]) * sp[i].splits;
    const bool use_big = big_total >= 512;
    RebuildF32Jobs tb;
    int nj = 0, blocks = 0;
    bool big = false, vec = false;  // tile and access width of the jobs in the table
    auto flush = [&]() -> dad_status {
        if (nj == 0) return DAD_OK;
        for (int i = nj; i < rf::MAX_JOBS; ++i) tb.first_block[i] = 0x7fffffff;
        ProfScope prof(kid, s);
        if (big)
            hipLaunchKernelGGL((k_rebuild_f32_mfma<2, 4, true>), dim3((unsigned)blocks), dim3(256), 0, s, tb);
        else if (vec)
            hipLaunchKernelGGL((k_rebuild_f32_mfma<1, 2, true>), dim3((unsigned)blocks), dim3(256), 0, s, tb);
        else
            hipLaunchKernelGGL((k_rebuild_f32_mfma<1, 2, false>), dim3((unsigned)blocks), dim3(256), 0, s, tb);
        DAD_LAUNCH_CHECK();
        nj = 0;
        blocks = 0;
        return DAD_OK;
    };
    for (int i = 0; i < n; ++i) {
        // the entry points have checked that every pointer is 16-byte aligned
        const bool job_vec = rebuild_f32_vec(h_in[i], h_out[i]);
        const bool job_big = job_vec && use_big;
        const int64_t tm = ceil_div(h_in[i], job_big ? 128 : 64), tn = ceil_div(h_out[i], job_big ? 256 : 128);
        const int64_t nb = tm * tn * sp[i].splits;
        if (nb > (int64_t)1 << 30) return DAD_ERR_SHAPE;
        if (nj == rf::MAX_JOBS || blocks + nb > ((int64_t)1 << 30) || (nj > 0 && (job_big != big || job_vec != vec))) {
            const dad_status rc = flush();
            if (rc != DAD_OK) return rc;
        }
        big = job_big;
        vec = job_vec;
        tb.first_block[nj] = blocks;
        RebuildF32Job& jb = tb.j[nj++];
        jb.L = static_cast<const float*>(L[i]);
        jb.R = static_cast<const float*>(R[i]);
        jb.out = sp[i].splits == 1 ? G[i] : slabs[i];
        jb.K = K[i];
        jb.chunk = sp[i].chunk;
        jb.h_in = (int)h_in[i];
        jb.h_out = (int)h_out[i];
        jb.tiles_n = (int)tn;
        jb.tiles = (int)(tm * tn);
        jb.splits = sp[i].splits;
        jb.pad = 0;
        blocks += (int)nb;
    }
    dad_status rc = flush();
    if (rc != DAD_OK) return rc;
    for (int i = 0; i < n; ++i)
        if (sp[i].splits > 1 && (rc = reduce_slabs(slabs[i], G[i], h_in[i] * h_out[i], sp[i].splits, s)) != DAD_OK) return rc;
    return DAD_OK;
}

}  // namespace dad

// Internal declarations shared by the translation units of libdad (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "dad.h"

namespace dad {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest, ties to even; NaN stays NaN.  This is the hardware conversion
// (v_cvt_pk_bf16_f32); it agrees bit for bit with the integer formulation
// u += 0x7fff + ((u >> 16) & 1) on finite values, ties, denormals and infinities.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

// Two values at once: a in the low half, b in the high half.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> __device__ __forceinline__ float ld(const T* p, int64_t i);
template <> __device__ __forceinline__ float ld<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }

template <typename T> __device__ __forceinline__ void st(T* p, int64_t i, float v);
template <> __device__ __forceinline__ void st<float>(float* p, int64_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t* p, int64_t i, float v) { p[i] = f32_to_bf16(v); }

// 16 bytes per lane from global memory straight into LDS: lane i's data lands at lds_addr + 16*i
// (lds_addr must be wave-uniform).  Issued through inline assembly because the compiler would
// otherwise wait for ALL outstanding LDS-bound loads before any LDS read; callers place the waits
// themselves with wait_vmcnt<N>() (N = number of younger loads that may still be in flight).
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);  // uniform by contract; this makes it a scalar register
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory");
}

// The same with the non-temporal hint, for data that is streamed once.
__device__ __forceinline__ void dma16_nt(const void* gptr, uint32_t lds_addr) {
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(lds_addr), "v"(gptr) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// Places NR LDS reads and NM matrix instructions of one scheduling region alternately in the
// instruction stream (reads first or matrix instructions first), so that a wave's fragment reads are
// issued in the shadow of its own MFMAs instead of in a block before them.
template <int NR, int NM, bool READ_FIRST, int I = 0>
__device__ __forceinline__ void interleave_reads_mfma() {
    constexpr int N = NR >= NM ? NM : NR;
    if constexpr (I < N) {
        constexpr int nr = NR >= NM ? (NR + NM - 1 - I) / NM : 1;
        constexpr int nm = NR >= NM ? 1 : (NM + NR - 1 - I) / NR;
        if (READ_FIRST) {
            __builtin_amdgcn_sched_group_barrier(0x100, nr, 0);  // DS read
            __builtin_amdgcn_sched_group_barrier(0x008, nm, 0);  // MFMA
        } else {
            __builtin_amdgcn_sched_group_barrier(0x008, nm, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, nr, 0);
        }
        interleave_reads_mfma<NR, NM, READ_FIRST, I + 1>();
    }
}

// A row-major matrix given as n contiguous row blocks (the sites' blocks in stacking order) instead
// of one allocation.  Passed to kernels by value; first[n] is the total row count.  Kernels that take
// it walk rows in whole stages, so every block's row count must be a multiple of BLOCK_ROW_QUANTUM.
constexpr int MAX_ROW_BLOCKS = 32;
constexpr int64_t BLOCK_ROW_QUANTUM = 256;
struct RowBlocks {
    const char* base[MAX_ROW_BLOCKS];
    int64_t first[MAX_ROW_BLOCKS + 1];
    int n;
    // Only for the jobs of a batch (kernels launched with job_stride != 0), whose widths may differ:
    // block j is a matrix of its own with h[j] columns, and thin_tn splits its rows into splits[j]
    // chunks of chunk[j] rows.
    int h[MAX_ROW_BLOCKS];
    int splits[MAX_ROW_BLOCKS];
    int chunk[MAX_ROW_BLOCKS];
};

// One caller pointer per job of a batch (a batch: up to MAX_ROW_BLOCKS equal reductions whose
// launches are merged; everything else of a job lives in its workspace region, at a fixed stride).
struct PtrTable {
    const void* p[MAX_ROW_BLOCKS];
};

// Two integers per job of a batch (widths, slab counts, block counts: what a launch needs per job).
struct BatchInts {
    int a[MAX_ROW_BLOCKS];
    int b[MAX_ROW_BLOCKS];
};

// Where a kernel's walk over rows stands: the block it is in and the row at which that block ends.
struct RowCursor {
    int blk;
    int64_t end;
};

// Address of row `row` (pitch in bytes); sets the cursor.  One allocation: a single endless block.
__device__ __forceinline__ const char* row_address(const uint16_t* X, int64_t row, int64_t pitch, RowCursor& c) {
    c.blk = 0;
    c.end = INT64_MAX;
    return reinterpret_cast<const char*>(X) + row * pitch;
}
__device__ __forceinline__ const char* row_address(const RowBlocks& X, int64_t row, int64_t pitch, RowCursor& c) {
    int b = 0;
    while (b + 1 < X.n && X.first[b + 1] <= row) ++b;
    c.blk = b;
    c.end = X.first[b + 1];
    return X.base[b] + (row - X.first[b]) * pitch;
}
// A pointer that has walked to the end of block c.blk continues in the next block after adding this.
__device__ __forceinline__ int64_t block_jump(const uint16_t*, int64_t, RowCursor&) { return 0; }
__device__ __forceinline__ int64_t block_jump(const RowBlocks& X, int64_t pitch, RowCursor& c) {
    const int b = c.blk;
    const int64_t jump = (X.base[b + 1] - X.base[b]) - (X.first[b + 1] - X.first[b]) * pitch;
    c.blk = b + 1;
    c.end = X.first[b + 2];
    return jump;
}

inline size_t elem_size(dad_dtype dt) { return dt == DAD_BF16 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define DAD_HIP_TRY(expr)                          \
    do {                                           \
        if ((expr) != hipSuccess) return DAD_ERR_HIP; \
    } while (0)

#define DAD_LAUNCH_CHECK()                                 \
    do {                                                   \
        if (hipGetLastError() != hipSuccess) return DAD_ERR_HIP; \
    } while (0)

// Raises a kernel's dynamic-LDS limit (needed above 64 KiB) on the current device.
template <typename Kern>
inline hipError_t set_max_lds(Kern k, int bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// Per-device set-up of each translation unit's kernels; called once per device by the entry points
// (api.hip: device_ready) or by dad_init.
dad_status thin_prepare_device();
dad_status rebuild_prepare_device();
dad_status gram_prepare_device();
dad_status backprop_prepare_device();

// Makes the current device ready for launches (kernel attributes set, the address of this device's
// copy of the static scratch array resolved); cheap after the first call on a device.
// scratch_out, when not null, receives that address.
dad_status device_ready(void** scratch_out = nullptr);

// ---------------------------------------------------------------- optional per-kernel timing

enum KernelId {
    KID_STACK = 0, KID_THIN_NN_BF16, KID_THIN_TN_BF16, KID_REDUCE, KID_GRAM, KID_APPLY, KID_APPLY2, KID_REBUILD_BF16,
    KID_THIN_NN, KID_THIN_TN, KID_REBUILD, KID_PANEL_INIT, KID_REBUILD_BF16_DMA, KID_BACKPROP_BF16, KID_BACKPROP,
    KID_GRAM_TILES, KID_GRAM_GATHER, KID_NS_STEP, KID_NS_PROJECT, KID_REBUILD_F32, KID_REDUCE_WIDE, KID_SEQ_VECTOR,
    KID_COUNT
};

// Brackets the kernel launched inside its scope with two events when timing is enabled.
class ProfScope {
public:
    ProfScope(int id, hipStream_t s);
    ~ProfScope();
    ProfScope(const ProfScope&) = delete;
    ProfScope& operator=(const ProfScope&) = delete;

private:
    int id_;
    hipStream_t s_;
    void* a_;
};

// ---------------------------------------------------------------- workspace plans

// Split of a contraction over `rows` rows into `splits` contiguous chunks of
// `chunk` rows (the last may be short).
struct SplitPlan {
    int splits;
    int64_t chunk;
};

// Layout of the dad_compress_rank workspace (byte offsets from its start).
struct CompressPlan {
    size_t off_flag;      // 256 B header: int flag at +0, int ticket counter at +64, pivot ranges (4 doubles) at +128
    size_t off_V;         // N x r intermediate: fp32, or on the MFMA path up to two bf16 planes (hi, lo) N*r apart
    size_t off_part;      // split partials, fp32
    size_t off_Ut;        // r x h_in fp32
    size_t off_Yt;        // r x h_out fp32
    size_t off_gram;      // gram partials, fp64
    size_t off_rinv;      // two DAD_MAX_RANK^2 fp32 inverse factors
    size_t off_Gb;        // bf16 copy of the current right block, RP x h_out (direct-to-LDS path only)
    size_t off_Ub;        // bf16 copy of U, RP x h_in
    bool dma;             // thin_nn takes its panel as bf16 and loads straight into LDS
    size_t total;
    SplitPlan tn_in;      // split of  A^T V   (width h_in)
    SplitPlan tn_out;     // split of  Delta^T W (width h_out)
    SplitPlan nn_in;      // column split of  A U  (guarded kernel only; chunk = columns)
    SplitPlan nn_out;     // column split of  Delta G
    int gram_blocks;
    bool fast;            // MFMA kernels apply to these sizes
};

// part_floor: least size of the split-partials region (a batch of jobs of several widths).
CompressPlan plan_compress(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt, size_t part_floor = 0);

// True when the bf16 MFMA thin kernels serve these sizes (otherwise the guarded kernels do).
bool thin_fast_ok(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt);

struct RebuildPlan {
    SplitPlan split;
    size_t total;  // bytes of partials (0 when splits == 1)
    bool fast;     // bf16 MFMA kernels
    bool f32;      // fp32 MFMA kernel (every fp32 shape)
    int tile;      // output tile edge of the bf16 MFMA kernel (256 or 128)
};

RebuildPlan plan_rebuild(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt);

// ---------------------------------------------------------------- launchers (host)

// out[i] = sum over s of part[s*n + i] in a fixed order; out_bf16 (optional) gets a bf16 copy.
// skip (optional, everywhere below): a device word; when it is non-zero at run time the kernels
// return at once (the adaptive one-vector iteration stops on the device with a fixed launch sequence).
// jobs / job_stride: the same sum for `jobs` problems whose pointers lie job_stride bytes apart;
// dims (optional): job j sums dims->b[j] slabs of dims->a[j] floats (n is then the largest a[j]).
dad_status reduce_slabs(const float* part, float* out, int64_t n, int splits, hipStream_t s, void* out_bf16 = nullptr,
                        const int* skip = nullptr, int jobs = 1, int64_t job_stride = 0, const BatchInts* dims = nullptr);


// out[n][j] = sum_k X[n][k] * Pt[j][k];  X is N x h (dt), Pt r x h fp32.  out is N x r: fp32 from the
// guarded kernels (fast = false); from the MFMA kernels `planes` bf16 planes N*r elements apart,
// plane 0 = the rounded value, plane 1 (planes = 2) = the rounded remainder.
// zero_hdr, when not null, is the 256-byte workspace header the launch clears on the side.
// partials/sp: fp32 slabs and column split of the guarded kernel (ignored by the MFMA kernel).
dad_status launch_thin_nn(const void* X, const float* Pt, void* out, float* partials, SplitPlan sp, int64_t N,
                          int64_t h, int r, dad_dtype dt, bool fast, int* zero_hdr, int planes, hipStream_t s,
                          const int* skip = nullptr);

// out_t[j][p] = sum_n X[n][p] * V[n][j];  X N x h (dt), V N x r as launch_thin_nn wrote it with the
// same `fast` and `planes` (the planes are summed), out_t r x h fp32.
// out_bf16 (optional, fast path only) receives a bf16 copy of out_t.
dad_status launch_thin_tn(const void* X, const void* V, float* out_t, float* partials, SplitPlan sp,
                          int64_t N, int64_t h, int r, dad_dtype dt, bool fast, void* out_bf16, int planes,
                          hipStream_t s, const int* skip = nullptr);

// Orthonormalisation Yt (r x h) -> Gt (r x h), rows of Gt orthonormal; rounds = 2 is CholeskyQR2.
// gt_bf16 (optional) receives a bf16 copy of Gt.
// jobs / job_stride: `jobs` independent iterates whose pointers (all of them) lie job_stride bytes apart;
// dims (optional): iterate j is r x dims->a[j] (h is then the largest of them).
dad_status launch_cholqr(const float* Yt, float* Gt, int64_t h, int r, int rounds, double* gram_part, int gram_blocks,
                         float* rinv, int* counter, int* flag, void* gt_bf16, hipStream_t s, int jobs = 1,
                         int64_t job_stride = 0, const BatchInts* dims = nullptr);

dad_status launch_rebuild(const void* L, const void* R, int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt,
                          float* G, float* partials, const RebuildPlan& plan, hipStream_t s);


// G_i = L_i^T R_i for n fp32 jobs in as few launches as possible (csrc/rebuild_f32.hip); a job with
// sp[i].splits > 1 goes through slabs[i] (splits * h_in * h_out floats) and reduce_slabs.
SplitPlan rebuild_f32_split(int64_t K, int64_t h_in, int64_t h_out);
// kid: the timing id the launches are booked under.
dad_status launch_rebuild_f32(int n, const void* const* L, const void* const* R, float* const* G, const int64_t* K,
                              const int64_t* h_in, const int64_t* h_out, const SplitPlan* sp, float* const* slabs,
                              hipStream_t s, int kid = KID_REBUILD_F32);

}  // namespace dad

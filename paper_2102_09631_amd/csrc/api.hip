// C ABI of libdad: argument checks on the host, then kernel launches on the caller's stream.
#include <atomic>
#include <mutex>
#include <vector>

#include "dad_internal.h"

// Scratch of dad_compress_rank_noalloc: one copy per device, held from the load of the library's
// code object until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; device_ready() resolves each device's address once and every launch and
// kernel argument uses that pointer.
static __device__ __align__(256) unsigned char scratch[DAD_STATIC_SCRATCH_BYTES];

namespace dad {

// implemented in the kernel translation units
dad_status gen_thin_nn(const void*, const float*, void*, float*, SplitPlan, int64_t, int64_t, int, dad_dtype, int*,
                       hipStream_t, const int*);
SplitPlan gen_thin_nn_split(int64_t N, int64_t h);
dad_status gen_thin_tn(const void*, const void*, float*, float*, SplitPlan, int64_t, int64_t, int, dad_dtype,
                       hipStream_t, const int*);
dad_status gen_rebuild(const void*, const void*, int64_t, int64_t, int64_t, dad_dtype, float*, float*, SplitPlan,
                       hipStream_t);
dad_status launch_stack(int, const void* const*, const void* const*, const int64_t*, int64_t, int64_t, dad_dtype,
                        void*, void*, hipStream_t);
dad_status f32_thin_nn(const float*, const float*, float*, float*, SplitPlan, int64_t, int64_t, int, int*, hipStream_t);
int gram_blocks_for(int64_t h);
bool thin_fast_ok(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt);
SplitPlan thin_tn_split(int64_t N, int64_t h, int r);
dad_status fast_thin_nn(const void*, const float*, void*, int64_t, int64_t, int, int*, int, hipStream_t, const int*);
dad_status fast_thin_tn(const void*, const RowBlocks*, const void*, float*, float*, SplitPlan, int64_t, int64_t, int,
                        void*, int, hipStream_t, const int*, int jobs = 1, int64_t job_stride = 0);
bool reduce_slabs_is_wide(int64_t n, bool with_bf16, bool with_skip);
bool thin_tn_dma_ok(int64_t N, int r, SplitPlan sp);
bool thin_dma_ok(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt);
dad_status launch_panel_init(const float*, void*, void*, int64_t, int64_t, int, int*, hipStream_t,
                             const PtrTable* g0s = nullptr, int jobs = 1, int64_t job_stride = 0,
                             const BatchInts* dims = nullptr);
dad_status dma_thin_nn(const void*, const RowBlocks*, const void*, void*, int64_t, int64_t, int, int, hipStream_t,
                       int jobs = 1, int64_t job_stride = 0);
bool rebuild_fast_ok(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt);
SplitPlan rebuild_fast_split(int64_t K, int64_t h_in, int64_t h_out, int* tile);
dad_status fast_rebuild(const void*, const void*, const RowBlocks*, const RowBlocks*, int64_t, int64_t, int64_t, float*,
                        float*, SplitPlan, int, hipStream_t);
bool rebuild_dma_ok(int64_t K, SplitPlan sp);
bool rebuild_group_ok(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt);
int rebuild_group_splits(int n, const int64_t* K, const int64_t* h_in, const int64_t* h_out);
SplitPlan rebuild_group_plan(int64_t K, int splits);
dad_status launch_rebuild_group(int n, const void* const* L, const void* const* R, float* const* G, const int64_t* K,
                                const int64_t* h_in, const int64_t* h_out, const SplitPlan* sp, float* const* slabs,
                                hipStream_t s);

static SplitPlan split_rows(int64_t rows, int64_t tiles, int64_t target_blocks, int64_t min_chunk, int64_t quantum) {
    int64_t want = ceil_div(target_blocks, tiles);
    int64_t max_splits = ceil_div(rows, min_chunk);
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    int64_t chunk = align_up((size_t)ceil_div(rows, want), (size_t)quantum);
    SplitPlan sp;
    sp.chunk = chunk;
    sp.splits = (int)ceil_div(rows, chunk);
    return sp;
}

CompressPlan plan_compress(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt, size_t part_floor) {
    CompressPlan p;
    p.fast = thin_fast_ok(N, h_in, h_out, r, dt);
    p.tn_in = p.fast ? thin_tn_split(N, h_in, r) : split_rows(N, ceil_div(h_in, 64), 1024, 32, 32);
    p.tn_out = p.fast ? thin_tn_split(N, h_out, r) : split_rows(N, ceil_div(h_out, 64), 1024, 32, 32);
    p.nn_in = gen_thin_nn_split(N, h_in);
    p.nn_out = gen_thin_nn_split(N, h_out);
    p.gram_blocks = gram_blocks_for(h_out);
    size_t o = 0;
    p.off_flag = o;
    o += 256;
    p.off_V = o;
    o += align_up((size_t)N * r * 4, 256);  // fp32, or two bf16 planes
    size_t part_in = (size_t)p.tn_in.splits * r * h_in * 4, part_out = (size_t)p.tn_out.splits * r * h_out * 4;
    p.off_part = o;
    size_t part_max = part_in > part_out ? part_in : part_out;
    if (part_floor > part_max) part_max = part_floor;  // a batch of jobs of several widths shares one layout
    if (!p.fast) {  // column-split slabs of the guarded thin_nn share the region
        const size_t nn_in = p.nn_in.splits > 1 ? (size_t)p.nn_in.splits * N * r * 4 : 0;
        const size_t nn_out = p.nn_out.splits > 1 ? (size_t)p.nn_out.splits * N * r * 4 : 0;
        if (nn_in > part_max) part_max = nn_in;
        if (nn_out > part_max) part_max = nn_out;
    }
    o += align_up(part_max, 256);
    p.off_Ut = o;
    o += align_up((size_t)r * h_in * 4, 256);
    p.off_Yt = o;
    o += align_up((size_t)r * h_out * 4, 256);
    p.off_gram = o;
    o += align_up((size_t)p.gram_blocks * r * r * 8, 256);
    p.off_rinv = o;
    o += 2 * DAD_MAX_RANK * DAD_MAX_RANK * 4;
    p.dma = thin_dma_ok(N, h_in, h_out, r, dt);
    const size_t rp = r <= 32 ? 32 : 64;
    p.off_Gb = o;
    if (p.dma) o += align_up(rp * (size_t)h_out * 2, 256);
    p.off_Ub = o;
    if (p.dma) o += align_up(rp * (size_t)h_in * 2, 256);
    p.total = o;
    return p;
}

RebuildPlan plan_rebuild(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt) {
    RebuildPlan p;
    p.fast = rebuild_fast_ok(K, h_in, h_out, dt);
    p.f32 = !p.fast && dt == DAD_F32;
    p.tile = 0;
    p.split = p.fast  ? rebuild_fast_split(K, h_in, h_out, &p.tile)
              : p.f32 ? rebuild_f32_split(K, h_in, h_out)
                      : split_rows(K, ceil_div(h_in, 64) * ceil_div(h_out, 64), 2048, 512, 16);
    p.total = p.split.splits > 1 ? (size_t)p.split.splits * h_in * h_out * 4 : 0;
    return p;
}

static bool dtype_ok(dad_dtype dt) { return dt == DAD_F32 || dt == DAD_BF16; }

// ---------------------------------------------------------------- per-device set-up
constexpr int MAX_DEVICES = 64;
constexpr int SIDE_STREAMS = DAD_MAX_LANES - 1;
struct DeviceState {
    std::atomic<int> ready{0};
    void* scratch = nullptr;  // this device's copy of the static scratch array
    // dad_compress_rank_grouped: side streams (default priority) the lanes beyond the first run on,
    // one fork event and one join event per side stream
    hipStream_t side[SIDE_STREAMS] = {};
    hipEvent_t fork = nullptr;
    hipEvent_t join[SIDE_STREAMS] = {};
    std::mutex lanes_mu;  // one grouped call at a time enqueues on a device's side streams
};
static DeviceState g_dev[MAX_DEVICES];
static std::mutex g_dev_mu;

dad_status device_ready(void** scratch_out) {
    int dev = -1;
    DAD_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return DAD_ERR_HIP;
    DeviceState& st = g_dev[dev];
    if (!st.ready.load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lk(g_dev_mu);
        if (!st.ready.load(std::memory_order_relaxed)) {
            dad_status rc;
            if ((rc = thin_prepare_device()) != DAD_OK) return rc;
            if ((rc = rebuild_prepare_device()) != DAD_OK) return rc;
            if ((rc = gram_prepare_device()) != DAD_OK) return rc;
            if ((rc = backprop_prepare_device()) != DAD_OK) return rc;
            void* ptr = nullptr;
            DAD_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            if (!ptr) return DAD_ERR_HIP;
            st.scratch = ptr;
            DAD_HIP_TRY(hipEventCreateWithFlags(&st.fork, hipEventDisableTiming));
            for (int i = 0; i < SIDE_STREAMS; ++i) {
                DAD_HIP_TRY(hipStreamCreateWithFlags(&st.side[i], hipStreamNonBlocking));
                DAD_HIP_TRY(hipEventCreateWithFlags(&st.join[i], hipEventDisableTiming));
            }
            st.ready.store(1, std::memory_order_release);
        }
    }
    if (scratch_out) *scratch_out = st.scratch;
    return DAD_OK;
}

// Copies the flag word of a workspace header to a caller-owned word.
__global__ void k_copy_flag(const int* __restrict__ hdr, int* __restrict__ out) { *out = *hdr; }

// Grouped compress: the group's sticky flag is cleared at the start of the call and set after every
// layer whose own flag was latched (several lanes may store the same 1).  `jobs` headers, stride
// bytes apart, are looked at (the jobs of a batch).
__global__ void k_clear_flag(int* __restrict__ flag) { *flag = 0; }
__global__ void k_latch_flag(const int* __restrict__ hdr, int* __restrict__ group_flag, int jobs, int64_t stride) {
    for (int j = 0; j < jobs; ++j)
        if (*reinterpret_cast<const int*>(reinterpret_cast<const char*>(hdr) + j * stride)) *group_flag = 1;
}

// End of a batch: the jobs' pairs leave their workspace regions for the callers' buffers.
__global__ __launch_bounds__(256) void k_batch_copy_out(const char* __restrict__ ws, int64_t stride, size_t off_p,
                                                        size_t off_g, int64_t n_p, int64_t n_g, PtrTable pt,
                                                        PtrTable gt, BatchInts dims, int use_dims) {
    const int j = blockIdx.y;
    if (use_dims) {  // this job's own sizes; the grid is sized for the largest
        n_p = dims.a[j];
        n_g = dims.b[j];
    }
    const float* sp = reinterpret_cast<const float*>(ws + j * stride + off_p);
    const float* sg = reinterpret_cast<const float*>(ws + j * stride + off_g);
    float* dp = static_cast<float*>(const_cast<void*>(pt.p[j]));
    float* dg = static_cast<float*>(const_cast<void*>(gt.p[j]));
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;  // n_p, n_g are multiples of 4, buffers 16-byte aligned
    typedef float f4 __attribute__((ext_vector_type(4)));
    if (i < n_p) *reinterpret_cast<f4*>(dp + i) = *reinterpret_cast<const f4*>(sp + i);
    if (i < n_g) *reinterpret_cast<f4*>(dg + i) = *reinterpret_cast<const f4*>(sg + i);
}

}  // namespace dad

using namespace dad;

extern "C" {

const char* dad_status_string(dad_status s) {
    switch (s) {
        case DAD_OK: return "DAD_OK";
        case DAD_ERR_NULL: return "DAD_ERR_NULL: required pointer is NULL";
        case DAD_ERR_SHAPE: return "DAD_ERR_SHAPE: size out of range";
        case DAD_ERR_ALIGN: return "DAD_ERR_ALIGN: device pointer not 16-byte aligned";
        case DAD_ERR_WORKSPACE: return "DAD_ERR_WORKSPACE: workspace too small (or sizes beyond the static scratch)";
        case DAD_ERR_DTYPE: return "DAD_ERR_DTYPE: unknown element type";
        case DAD_ERR_NUMERIC: return "DAD_ERR_NUMERIC: orthonormalisation broke down (iterate lost rank)";
        case DAD_ERR_HIP: return "DAD_ERR_HIP: HIP runtime call failed";
    }
    return "unknown dad_status";
}

dad_status dad_stack_factors(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                             int64_t h_in, int64_t h_out, dad_dtype dt, void* A_out, void* D_out, void* stream) {
    if (!A_sites || !D_sites || !rows || !A_out || !D_out) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    if (S < 1 || S > DAD_MAX_SITES || h_in < 1 || h_out < 1) return DAD_ERR_SHAPE;
    for (int s = 0; s < S; ++s) {
        if (rows[s] < 0) return DAD_ERR_SHAPE;
        if (rows[s] > 0 && (!A_sites[s] || !D_sites[s])) return DAD_ERR_NULL;
    }
    if (!aligned16(A_out) || !aligned16(D_out)) return DAD_ERR_ALIGN;
    for (int s = 0; s < S; ++s)
        if (rows[s] > 0 && (!aligned16(A_sites[s]) || !aligned16(D_sites[s]))) return DAD_ERR_ALIGN;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    return launch_stack(S, A_sites, D_sites, rows, h_in, h_out, dt, A_out, D_out, (hipStream_t)stream);
}

static bool compress_shape_ok(int64_t N, int64_t h_in, int64_t h_out, int r) {
    if (N < 1 || h_in < 1 || h_out < 1 || r < 1 || r > DAD_MAX_RANK) return false;
    if (r > N || r > h_in || r > h_out) return false;
    // what the launch grids hold: ceil(N / 64) in grid.x, ceil(h / 64) in grid.y
    if (N > DAD_MAX_ROWS || h_in > DAD_MAX_WIDTH || h_out > DAD_MAX_WIDTH) return false;
    return true;
}

size_t dad_compress_workspace_bytes(int64_t N, int64_t h_in, int64_t h_out, int r, dad_dtype dt) {
    if (!dtype_ok(dt) || !compress_shape_ok(N, h_in, h_out, r)) return 0;
    return plan_compress(N, h_in, h_out, r, dt).total;
}

// Host-side argument checks shared by dad_compress_rank and dad_compress_rank_noalloc.
static dad_status compress_args_ok(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt,
                                   int r, int n_iter, const float* G0, const float* Pt, const float* Gt) {
    if (!A || !D || !G0 || !Pt || !Gt) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    if (!compress_shape_ok(N, h_in, h_out, r) || n_iter < 1) return DAD_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(D) || !aligned16(G0) || !aligned16(Pt) || !aligned16(Gt)) return DAD_ERR_ALIGN;
    return DAD_OK;
}

// The launches of one compress call; every argument has been checked and the device is ready.
// A batch: `jobs` reductions of equal sizes on the direct-to-LDS path whose launches are merged (one
// launch does the same step of every job; a job's arithmetic is that of a call of its own).  Job j
// works in the workspace region j * stride bytes after the first and has block j of Ab / Db as its
// factors; the pairs are formed in the regions (P in the U slot, G in place in the Y slot) and
// copied to the callers' buffers at the end.
// per_job: the jobs differ in their widths (equal N and r): h_in/h_out and the row splits of thin_tn
// are per job (tables inside Ab / Db and `widths`), every buffer of the shared layout is sized for the
// largest job, and the h_in / h_out arguments of compress_launch are the largest widths.
struct Batch {
    int jobs;
    int64_t stride;
    PtrTable g0, pt, gt;
    bool per_job;
    BatchInts widths;  // a = h_in, b = h_out
};

// Ab / Db, when not null, give the factors as row blocks read in place (A and D are then unused); the
// caller has checked compress_in_place().  With `batch` the blocks are the jobs of a batch, N is one
// job's row count and G0, Pt, Gt are unused.
static dad_status compress_launch(const CompressPlan& p, const void* A, const void* D, int64_t N, int64_t h_in,
                                  int64_t h_out, dad_dtype dt, int r, int n_iter, const float* G0, float* Pt, float* Gt,
                                  void* workspace, hipStream_t s, const RowBlocks* Ab = nullptr,
                                  const RowBlocks* Db = nullptr, const Batch* batch = nullptr) {
    char* ws = static_cast<char*>(workspace);
    int* flag = reinterpret_cast<int*>(ws + p.off_flag);
    void* V = ws + p.off_V;
    float* part = reinterpret_cast<float*>(ws + p.off_part);
    float* Ut = reinterpret_cast<float*>(ws + p.off_Ut);
    float* Yt = reinterpret_cast<float*>(ws + p.off_Yt);
    double* gram = reinterpret_cast<double*>(ws + p.off_gram);
    float* rinv = reinterpret_cast<float*>(ws + p.off_rinv);
    dad_status rc;

    int* counter = flag + 16;
    // bf16 copies of the two h x r panels, made by their producers (direct-to-LDS path only)
    void* Gb = p.dma ? ws + p.off_Gb : nullptr;
    void* Ub = p.dma ? ws + p.off_Ub : nullptr;

    const int jobs = batch ? batch->jobs : 1;
    const int64_t jstride = batch ? batch->stride : 0;
    if (batch) {  // the pair is formed inside the regions
        Pt = Ut;
        Gt = Yt;
    }
    struct Factor {
        const void* ptr;          // one allocation, or
        const RowBlocks* blocks;  // row blocks (ptr unused)
    };
    const Factor FA = {A, Ab}, FD = {D, Db};
    // fp32 factors, r >= 16: both thin contractions run on the fp32 matrix instruction (same-box
    // measurements: equal to the guarded kernels on 64-row stacks, 10-30 % faster from 256 rows on).
    // Below r = 16 a 32-wide MFMA block is mostly padding and the guarded kernels, which have an
    // instance for narrow panels, measured 4-10 % faster on the two MLP workloads (r = 4, 8).
    const bool f32_mfma = !p.fast && dt == DAD_F32 && r >= 16;
    // V <- X * panel (N x r); the direct-to-LDS kernel takes the bf16 copy of the panel
    auto nn = [&](const Factor& X, const float* panel, const void* panel_bf16, int64_t h, SplitPlan sp, int* hdr,
                  int planes) {
        if (p.dma) return dma_thin_nn(X.ptr, X.blocks, panel_bf16, V, N, h, r, planes, s, jobs, jstride);
        if (f32_mfma)
            return f32_thin_nn(static_cast<const float*>(X.ptr), panel, static_cast<float*>(V), part, sp, N, h, r, hdr, s);
        return launch_thin_nn(X.ptr, panel, V, part, sp, N, h, r, dt, p.fast, hdr, planes, s);
    };
    // out (r x h) <- V^T X, with an optional bf16 copy
    auto tn = [&](const Factor& X, float* out, int64_t h, SplitPlan sp, void* out_bf16, int planes) {
        if (X.blocks)
            return fast_thin_tn(nullptr, X.blocks, V, out, part, sp, N, h, r, out_bf16, planes, s, nullptr, jobs, jstride);
        if (f32_mfma) {  // V^T X is the rebuild L^T R with L = V (N x r) and R = X
            const void* L = V;
            const int64_t r64 = r;
            return launch_rebuild_f32(1, &L, &X.ptr, &out, &N, &r64, &h, &sp, &part, s, KID_THIN_TN);
        }
        return launch_thin_tn(X.ptr, V, out, part, sp, N, h, r, dt, p.fast, out_bf16, planes, s);
    };
    // On the MFMA path the N x r intermediates are bf16.  V = Delta G goes as one plane.  W = A U goes
    // as two (rounded value + rounded remainder): activations with a non-zero mean (ReLU, GELU) give
    // the rows of W a large common component, and one bf16 rounding of it drowns the row-to-row
    // differences that the next contraction with Delta extracts.
    const int PV = 1, PW = 2;
#define DAD_TRY(expr)                      \
    do {                                   \
        if ((rc = (expr)) != DAD_OK) return rc; \
    } while (0)
    // the workspace header is cleared by the first launch of the call
    const bool per_job = batch && batch->per_job;
    BatchInts out_w = {}, copy_n = {};  // per job: h_out (orthonormalisation), element counts of the pair
    if (per_job)
        for (int j = 0; j < jobs; ++j) {
            out_w.a[j] = batch->widths.b[j];
            copy_n.a[j] = r * batch->widths.a[j];
            copy_n.b[j] = r * batch->widths.b[j];
        }
    if (p.dma)
        DAD_TRY(launch_panel_init(G0, Gb, Ub, h_in, h_out, r, flag, s, batch ? &batch->g0 : nullptr, jobs, jstride,
                                  per_job ? &batch->widths : nullptr));
    const float* G = G0;
    for (int it = 0; it < n_iter; ++it) {
        DAD_TRY(nn(FD, G, Gb, h_out, p.nn_out, it == 0 ? flag : nullptr, PV));  // V = Delta G
        DAD_TRY(tn(FA, Ut, h_in, p.tn_in, Ub, PV));                             // U = A^T V
        DAD_TRY(nn(FA, Ut, Ub, h_in, p.nn_in, nullptr, PW));                    // W = A U
        DAD_TRY(tn(FD, Yt, h_out, p.tn_out, nullptr, PW));                      // Y = Delta^T W
        // G = orth(Y): up to two Cholesky rounds for the iterate that is returned, one for the others
        DAD_TRY(launch_cholqr(Yt, Gt, h_out, r, (it + 1 == n_iter) ? 2 : 1, gram, p.gram_blocks, rinv, counter, flag, Gb,
                              s, jobs, jstride, per_job ? &out_w : nullptr));
        G = Gt;
    }
    DAD_TRY(nn(FD, Gt, Gb, h_out, p.nn_out, nullptr, PV));  // V = Delta G
    DAD_TRY(tn(FA, Pt, h_in, p.tn_in, nullptr, PV));        // P = A^T V
    if (batch) {
        const int64_t n_p = (int64_t)r * h_in, n_g = (int64_t)r * h_out;
        const int64_t n_max = n_p > n_g ? n_p : n_g;
        hipLaunchKernelGGL(k_batch_copy_out, dim3((unsigned)ceil_div(n_max / 4, 256), (unsigned)jobs), dim3(256), 0, s,
                           (const char*)ws, jstride, p.off_Ut, p.off_Yt, n_p, n_g, batch->pt, batch->gt, copy_n,
                           per_job ? 1 : 0);
        DAD_LAUNCH_CHECK();
    }
    return DAD_OK;
#undef DAD_TRY
}

// ---------------------------------------------------------------- factors given as site blocks

// Checks of a site table (the rules of dad_stack_factors); *N receives the total row count.
// With check_pointers false only S and the row counts are looked at (workspace size queries).
static dad_status sites_ok(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                           bool check_pointers, int64_t* N) {
    if (!rows || (check_pointers && (!A_sites || !D_sites))) return DAD_ERR_NULL;
    if (S < 1 || S > DAD_MAX_SITES) return DAD_ERR_SHAPE;
    int64_t total = 0;
    for (int s = 0; s < S; ++s) {
        if (rows[s] < 0 || rows[s] > DAD_MAX_ROWS) return DAD_ERR_SHAPE;
        total += rows[s];
        if (total > DAD_MAX_ROWS) return DAD_ERR_SHAPE;
    }
    if (check_pointers)
        for (int s = 0; s < S; ++s) {
            if (rows[s] == 0) continue;
            if (!A_sites[s] || !D_sites[s]) return DAD_ERR_NULL;
            if (!aligned16(A_sites[s]) || !aligned16(D_sites[s])) return DAD_ERR_ALIGN;
        }
    *N = total;
    return DAD_OK;
}

// The kernels that read blocks in place walk rows in whole stages of up to 256 rows.
static bool rows_allow_blocks(int S, const int64_t* rows) {
    int used = 0;
    for (int s = 0; s < S; ++s) {
        if (rows[s] == 0) continue;
        if (rows[s] % BLOCK_ROW_QUANTUM) return false;
        if (++used > MAX_ROW_BLOCKS) return false;
    }
    return used > 0;
}

static void fill_blocks(int S, const void* const* sites, const int64_t* rows, RowBlocks* b) {
    int n = 0;
    int64_t row = 0;
    for (int s = 0; s < S; ++s) {
        if (rows[s] == 0) continue;
        b->base[n] = static_cast<const char*>(sites[s]);
        b->first[n] = row;
        row += rows[s];
        ++n;
    }
    for (int i = n; i <= MAX_ROW_BLOCKS; ++i) b->first[i] = row;
    for (int i = n; i < MAX_ROW_BLOCKS; ++i) b->base[i] = nullptr;
    b->n = n;
}

// One layer of a compress call: stacked factors, or site blocks read in place, or site blocks that
// the call first stacks behind the layer's plan in its workspace.
struct LayerPlan {
    int64_t N;
    CompressPlan cp;
    bool sites, in_place;
    size_t off_A, off_D, total;
};

static bool compress_in_place(const CompressPlan& p, int64_t N, int r, int S, const int64_t* rows) {
    return p.dma && thin_tn_dma_ok(N, r, p.tn_in) && thin_tn_dma_ok(N, r, p.tn_out) && rows_allow_blocks(S, rows);
}

// Shapes only (d.S, d.rows, d.N, widths); DAD_ERR_* on sizes out of range.
static dad_status plan_layer(const dad_compress_desc& d, dad_dtype dt, int r, LayerPlan* lp) {
    lp->sites = d.S > 0;
    lp->N = d.N;
    if (d.S < 0) return DAD_ERR_SHAPE;
    if (lp->sites) {
        const dad_status rc = sites_ok(d.S, nullptr, nullptr, d.rows, false, &lp->N);
        if (rc != DAD_OK) return rc;
    }
    if (!compress_shape_ok(lp->N, d.h_in, d.h_out, r)) return DAD_ERR_SHAPE;
    lp->cp = plan_compress(lp->N, d.h_in, d.h_out, r, dt);
    lp->in_place = lp->sites && compress_in_place(lp->cp, lp->N, r, d.S, d.rows);
    size_t o = align_up(lp->cp.total, 256);
    lp->off_A = o;
    if (lp->sites && !lp->in_place) o += align_up((size_t)lp->N * d.h_in * elem_size(dt), 256);
    lp->off_D = o;
    if (lp->sites && !lp->in_place) o += align_up((size_t)lp->N * d.h_out * elem_size(dt), 256);
    lp->total = o;
    return DAD_OK;
}

// Pointer checks of one layer (after plan_layer).
static dad_status layer_args_ok(const dad_compress_desc& d, const LayerPlan& lp, dad_dtype dt, int r, int n_iter) {
    if (lp.sites) {
        int64_t N = 0;
        const dad_status rc = sites_ok(d.S, d.A_sites, d.D_sites, d.rows, true, &N);
        if (rc != DAD_OK) return rc;
        if (!d.G0 || !d.Pt || !d.Gt) return DAD_ERR_NULL;
        if (n_iter < 1) return DAD_ERR_SHAPE;
        if (!aligned16(d.G0) || !aligned16(d.Pt) || !aligned16(d.Gt)) return DAD_ERR_ALIGN;
        return DAD_OK;
    }
    return compress_args_ok(d.A, d.D, d.N, d.h_in, d.h_out, dt, r, n_iter, d.G0, d.Pt, d.Gt);
}

// The launches of one layer on stream s; ws is the layer's region (lp.total bytes).
static dad_status launch_layer(const dad_compress_desc& d, const LayerPlan& lp, dad_dtype dt, int r, int n_iter,
                               void* ws, hipStream_t s) {
    if (!lp.sites)
        return compress_launch(lp.cp, d.A, d.D, lp.N, d.h_in, d.h_out, dt, r, n_iter, d.G0, d.Pt, d.Gt, ws, s);
    if (lp.in_place) {
        RowBlocks a = {}, b = {};
        fill_blocks(d.S, d.A_sites, d.rows, &a);
        fill_blocks(d.S, d.D_sites, d.rows, &b);
        return compress_launch(lp.cp, nullptr, nullptr, lp.N, d.h_in, d.h_out, dt, r, n_iter, d.G0, d.Pt, d.Gt, ws, s, &a,
                               &b);
    }
    void* A = static_cast<char*>(ws) + lp.off_A;
    void* D = static_cast<char*>(ws) + lp.off_D;
    const dad_status rc = launch_stack(d.S, d.A_sites, d.D_sites, d.rows, d.h_in, d.h_out, dt, A, D, s);
    if (rc != DAD_OK) return rc;
    return compress_launch(lp.cp, A, D, lp.N, d.h_in, d.h_out, dt, r, n_iter, d.G0, d.Pt, d.Gt, ws, s);
}

dad_status dad_compress_rank(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out, dad_dtype dt,
                             int r, int n_iter, const float* G0, float* Pt, float* Gt, void* workspace,
                             size_t ws_bytes, void* stream) {
    if (!workspace) return DAD_ERR_NULL;
    dad_status rc = compress_args_ok(A, D, N, h_in, h_out, dt, r, n_iter, G0, Pt, Gt);
    if (rc != DAD_OK) return rc;
    if (!aligned16(workspace)) return DAD_ERR_ALIGN;
    const CompressPlan p = plan_compress(N, h_in, h_out, r, dt);
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if ((rc = device_ready()) != DAD_OK) return rc;
    return compress_launch(p, A, D, N, h_in, h_out, dt, r, n_iter, G0, Pt, Gt, workspace, (hipStream_t)stream);
}

dad_status dad_compress_rank_noalloc(const void* A, const void* D, int64_t N, int64_t h_in, int64_t h_out,
                                     dad_dtype dt, int r, int n_iter, const float* G0, float* Pt, float* Gt,
                                     int* numeric_flag, void* stream) {
    dad_status rc = compress_args_ok(A, D, N, h_in, h_out, dt, r, n_iter, G0, Pt, Gt);
    if (rc != DAD_OK) return rc;
    if (numeric_flag && (reinterpret_cast<uintptr_t>(numeric_flag) & 3u)) return DAD_ERR_ALIGN;
    const CompressPlan p = plan_compress(N, h_in, h_out, r, dt);
    if (p.total > (size_t)DAD_STATIC_SCRATCH_BYTES) return DAD_ERR_WORKSPACE;
    void* ws = nullptr;  // the current device's copy of `scratch`
    if ((rc = device_ready(&ws)) != DAD_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    rc = compress_launch(p, A, D, N, h_in, h_out, dt, r, n_iter, G0, Pt, Gt, ws, s);
    if (rc != DAD_OK || !numeric_flag) return rc;
    hipLaunchKernelGGL(k_copy_flag, dim3(1), dim3(1), 0, s, (const int*)ws, numeric_flag);
    DAD_LAUNCH_CHECK();
    return DAD_OK;
}

size_t dad_compress_sites_workspace_bytes(int S, const int64_t* rows, int64_t h_in, int64_t h_out, int r, dad_dtype dt) {
    if (!dtype_ok(dt) || S < 1) return 0;
    dad_compress_desc d = {};
    d.S = S, d.rows = rows, d.h_in = h_in, d.h_out = h_out;
    LayerPlan lp;
    return plan_layer(d, dt, r, &lp) == DAD_OK ? lp.total : 0;
}

dad_status dad_compress_rank_sites(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                                   int64_t h_in, int64_t h_out, dad_dtype dt, int r, int n_iter, const float* G0,
                                   float* Pt, float* Gt, void* workspace, size_t ws_bytes, void* stream) {
    if (!workspace) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    if (S < 1) return DAD_ERR_SHAPE;
    dad_compress_desc d = {};
    d.S = S, d.A_sites = A_sites, d.D_sites = D_sites, d.rows = rows, d.h_in = h_in, d.h_out = h_out;
    d.G0 = G0, d.Pt = Pt, d.Gt = Gt;
    LayerPlan lp;
    dad_status rc = plan_layer(d, dt, r, &lp);
    if (rc != DAD_OK) return rc;
    if ((rc = layer_args_ok(d, lp, dt, r, n_iter)) != DAD_OK) return rc;
    if (!aligned16(workspace)) return DAD_ERR_ALIGN;
    if (ws_bytes < lp.total) return DAD_ERR_WORKSPACE;
    if ((rc = device_ready()) != DAD_OK) return rc;
    return launch_layer(d, lp, dt, r, n_iter, workspace, (hipStream_t)stream);
}

// The layers of a grouped call are dealt to the lanes in units: a unit is one layer, or a batch of
// up to MAX_ROW_BLOCKS consecutive stacked layers that the direct-to-LDS kernels serve and whose
// launches are merged, one launch doing the same step of every job.  The jobs of a batch have equal
// N (and r); their widths are either all equal (the S site reductions of one layer in Algorithm 1)
// or all multiples of 256 (the layers of a small block).  Only small layers are batched: their
// launches are short and bound by latency, while a larger layer keeps the chip busy on its own and
// gains more from running beside another layer on a second lane.  Jobs of equal widths are balanced,
// so factors of up to 256 MiB per job are taken (the sites of the benchmark's layers: 1.5 times faster
// than 8 lanes); with unequal widths every job keeps the decomposition of a call of its own, the
// workgroups of a launch then differ in length, and only layers of at most 64 MiB are taken (four layers
// with an encoder block's widths, batch against four lanes on one box: 57 against 109 us per layer at
// 15 MiB, 76 against 108 at 60 MiB, 119 against 122 at 120 MiB; on a box with faster launches the lanes
// won at 120 MiB).
constexpr double BATCH_MAX_BYTES = 256.0 * 1024 * 1024;
constexpr double BATCH_MAX_BYTES_MIXED = 64.0 * 1024 * 1024;

static double factor_bytes(const dad_compress_desc& d, int64_t N, dad_dtype dt) {
    return (double)N * (double)(d.h_in + d.h_out) * (double)elem_size(dt);
}

struct Unit {
    int first, count;
    bool per_job;         // the jobs differ in their widths
    CompressPlan layout;  // workspace layout of every job's region (sized for the largest job)
    size_t bytes;         // of its lane region
};

static bool batchable(const dad_compress_desc& d, const LayerPlan& lp, int r, dad_dtype dt) {
    return !lp.sites && lp.cp.dma && thin_tn_dma_ok(lp.N, r, lp.cp.tn_in) && thin_tn_dma_ok(lp.N, r, lp.cp.tn_out) &&
           !reduce_slabs_is_wide((int64_t)r * d.h_in, false, false) && !reduce_slabs_is_wide((int64_t)r * d.h_out, false, false) &&
           lp.N < ((int64_t)1 << 31) && factor_bytes(d, lp.N, dt) <= BATCH_MAX_BYTES;
}

// A layer that may share a batch with layers of other widths.
static bool mixable(const dad_compress_desc& d, int64_t N, dad_dtype dt) {
    return d.h_in % 256 == 0 && d.h_out % 256 == 0 && factor_bytes(d, N, dt) <= BATCH_MAX_BYTES_MIXED;
}

// Layout of the grouped workspace: 256-byte group header (sticky numeric flag at +0), then one region
// per lane, each large enough for any unit of the group.
static dad_status grouped_plans(int n, const dad_compress_desc* descs, dad_dtype dt, int r, std::vector<LayerPlan>* plans,
                                std::vector<Unit>* units, size_t* lane_bytes) {
    plans->resize((size_t)n);
    units->clear();
    bool open = false, uniform = true, all256 = false;  // state of the last unit while it can still grow
    for (int i = 0; i < n; ++i) {
        LayerPlan& lp = (*plans)[(size_t)i];
        const dad_status rc = plan_layer(descs[i], dt, r, &lp);
        if (rc != DAD_OK) return rc;
        const bool can = batchable(descs[i], lp, r, dt);
        bool joined = false;
        if (open && can) {
            Unit& u = units->back();
            const dad_compress_desc& f = descs[u.first];
            const bool same = f.h_in == descs[i].h_in && f.h_out == descs[i].h_out;
            if (u.count < MAX_ROW_BLOCKS && (*plans)[(size_t)u.first].N == lp.N &&
                ((uniform && same) || (all256 && mixable(descs[i], lp.N, dt)))) {
                ++u.count;
                uniform = uniform && same;
                joined = true;
            }
        }
        if (!joined) {
            units->push_back(Unit{i, 1, false, lp.cp, lp.total});
            open = can;
            uniform = true;
            all256 = can && mixable(descs[i], lp.N, dt);
        }
        units->back().per_job = !uniform;
    }
    size_t lane = 0;
    for (Unit& u : *units) {
        if (u.count > 1) {  // one layout for all jobs of the batch
            int64_t hi = 0, ho = 0;
            size_t part = 0;
            for (int j = u.first; j < u.first + u.count; ++j) {
                const CompressPlan& c = (*plans)[(size_t)j].cp;
                if (descs[j].h_in > hi) hi = descs[j].h_in;
                if (descs[j].h_out > ho) ho = descs[j].h_out;
                const size_t pi = (size_t)c.tn_in.splits * r * descs[j].h_in * 4, po = (size_t)c.tn_out.splits * r * descs[j].h_out * 4;
                if (pi > part) part = pi;
                if (po > part) part = po;
            }
            u.layout = plan_compress((*plans)[(size_t)u.first].N, hi, ho, r, dt, part);
            u.bytes = (size_t)u.count * align_up(u.layout.total, 256);
        }
        if (u.bytes > lane) lane = u.bytes;
    }
    *lane_bytes = align_up(lane, 256);
    return DAD_OK;
}

size_t dad_compress_grouped_workspace_bytes(int n, const dad_compress_desc* descs, dad_dtype dt, int r, int lanes) {
    if (n < 1 || n > DAD_MAX_GROUP || !descs || !dtype_ok(dt) || lanes < 1 || lanes > DAD_MAX_LANES) return 0;
    std::vector<LayerPlan> plans;
    std::vector<Unit> units;
    size_t lane_bytes = 0;
    if (grouped_plans(n, descs, dt, r, &plans, &units, &lane_bytes) != DAD_OK) return 0;
    const int used = lanes < (int)units.size() ? lanes : (int)units.size();
    return 256 + (size_t)used * lane_bytes;
}

// The launches of one batch on stream s; ws holds u.count regions.
static dad_status launch_batch(const dad_compress_desc* descs, const Unit& u, const std::vector<LayerPlan>& plans,
                               dad_dtype dt, int r, int n_iter, void* ws, hipStream_t s) {
    const int64_t N = plans[(size_t)u.first].N;
    RowBlocks a = {}, b = {};
    Batch batch = {};
    batch.jobs = u.count;
    batch.stride = (int64_t)align_up(u.layout.total, 256);
    batch.per_job = u.per_job;
    int64_t hi = 0, ho = 0;
    for (int j = 0; j < MAX_ROW_BLOCKS; ++j) {
        const bool in = j < u.count;
        const dad_compress_desc& d = descs[u.first + (in ? j : 0)];
        const CompressPlan& c = plans[(size_t)(u.first + (in ? j : 0))].cp;
        a.base[j] = in ? static_cast<const char*>(d.A) : nullptr;
        b.base[j] = in ? static_cast<const char*>(d.D) : nullptr;
        a.first[j] = b.first[j] = (in ? j : u.count) * N;
        batch.g0.p[j] = in ? d.G0 : nullptr;
        batch.pt.p[j] = in ? d.Pt : nullptr;
        batch.gt.p[j] = in ? d.Gt : nullptr;
        if (in && u.per_job) {
            a.h[j] = (int)d.h_in, a.splits[j] = c.tn_in.splits, a.chunk[j] = (int)c.tn_in.chunk;
            b.h[j] = (int)d.h_out, b.splits[j] = c.tn_out.splits, b.chunk[j] = (int)c.tn_out.chunk;
            batch.widths.a[j] = (int)d.h_in;
            batch.widths.b[j] = (int)d.h_out;
        }
        if (in && d.h_in > hi) hi = d.h_in;
        if (in && d.h_out > ho) ho = d.h_out;
    }
    a.first[MAX_ROW_BLOCKS] = b.first[MAX_ROW_BLOCKS] = (int64_t)u.count * N;
    a.n = b.n = u.count;
    return compress_launch(u.layout, nullptr, nullptr, N, hi, ho, dt, r, n_iter, nullptr, nullptr, nullptr, ws, s, &a, &b,
                           &batch);
}

dad_status dad_compress_rank_grouped(int n, const dad_compress_desc* descs, dad_dtype dt, int r, int n_iter, int lanes,
                                     void* workspace, size_t ws_bytes, void* stream) {
    if (!descs || !workspace) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    if (n < 1 || n > DAD_MAX_GROUP || lanes < 1 || lanes > DAD_MAX_LANES) return DAD_ERR_SHAPE;
    std::vector<LayerPlan> plans;
    std::vector<Unit> units;
    size_t lane_bytes = 0;
    dad_status rc = grouped_plans(n, descs, dt, r, &plans, &units, &lane_bytes);
    if (rc != DAD_OK) return rc;
    for (int i = 0; i < n; ++i)
        if ((rc = layer_args_ok(descs[i], plans[(size_t)i], dt, r, n_iter)) != DAD_OK) return rc;
    if (!aligned16(workspace)) return DAD_ERR_ALIGN;
    const int nu = (int)units.size();
    const int used = lanes < nu ? lanes : nu;
    if (ws_bytes < 256 + (size_t)used * lane_bytes) return DAD_ERR_WORKSPACE;
    if ((rc = device_ready()) != DAD_OK) return rc;
    int dev = 0;
    DAD_HIP_TRY(hipGetDevice(&dev));
    DeviceState& st = g_dev[dev];
    hipStream_t main = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    int* group_flag = reinterpret_cast<int*>(ws);

    std::lock_guard<std::mutex> lk(st.lanes_mu);
    hipLaunchKernelGGL(k_clear_flag, dim3(1), dim3(1), 0, main, group_flag);
    DAD_LAUNCH_CHECK();
    // fork: the side streams start after everything already enqueued on the caller's stream
    if (used > 1) {
        DAD_HIP_TRY(hipEventRecord(st.fork, main));
        for (int l = 1; l < used; ++l) DAD_HIP_TRY(hipStreamWaitEvent(st.side[l - 1], st.fork, 0));
    }
    for (int k = 0; k < nu; ++k) {  // unit k on lane k mod `used`; a lane's units follow each other on its stream
        const int l = k % used;
        hipStream_t s = l == 0 ? main : st.side[l - 1];
        void* lane_ws = ws + 256 + (size_t)l * lane_bytes;
        const Unit& u = units[(size_t)k];
        const LayerPlan& lp = plans[(size_t)u.first];
        rc = u.count > 1 ? launch_batch(descs, u, plans, dt, r, n_iter, lane_ws, s)
                         : launch_layer(descs[u.first], lp, dt, r, n_iter, lane_ws, s);
        if (rc != DAD_OK) break;
        hipLaunchKernelGGL(k_latch_flag, dim3(1), dim3(1), 0, s, (const int*)lane_ws, group_flag, u.count,
                           (int64_t)align_up(u.layout.total, 256));
        if (hipGetLastError() != hipSuccess) {
            rc = DAD_ERR_HIP;
            break;
        }
    }
    // join, also after a failed enqueue: the caller's stream must not run ahead of the side streams
    for (int l = 1; l < used; ++l) {
        if (hipEventRecord(st.join[l - 1], st.side[l - 1]) != hipSuccess ||
            hipStreamWaitEvent(main, st.join[l - 1], 0) != hipSuccess)
            rc = rc == DAD_OK ? DAD_ERR_HIP : rc;
    }
    return rc;
}

dad_status dad_init(void) { return device_ready(); }

static bool rebuild_shape_ok(int64_t K, int64_t h_in, int64_t h_out) {
    return K >= 1 && h_in >= 1 && h_out >= 1 && K <= DAD_MAX_ROWS && h_in <= DAD_MAX_WIDTH && h_out <= DAD_MAX_WIDTH;
}

size_t dad_reconstruct_workspace_bytes(int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt) {
    if (!dtype_ok(dt) || !rebuild_shape_ok(K, h_in, h_out)) return 0;
    return plan_rebuild(K, h_in, h_out, dt).total;
}

dad_status dad_reconstruct_grad(const void* L, const void* R, int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt,
                                float* G, void* workspace, size_t ws_bytes, void* stream) {
    if (!L || !R || !G) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    if (!rebuild_shape_ok(K, h_in, h_out)) return DAD_ERR_SHAPE;
    const RebuildPlan p = plan_rebuild(K, h_in, h_out, dt);
    if (p.total > 0 && !workspace) return DAD_ERR_NULL;
    if (!aligned16(L) || !aligned16(R) || !aligned16(G) || (workspace && !aligned16(workspace))) return DAD_ERR_ALIGN;
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    return launch_rebuild(L, R, K, h_in, h_out, dt, G, static_cast<float*>(workspace), p, (hipStream_t)stream);
}

// Full rebuild on site blocks: in place on the direct-to-LDS bf16 kernel, else stacked into the
// workspace behind the split slabs first.
struct RebuildSitesPlan {
    int64_t N;
    RebuildPlan rp;
    bool in_place;
    size_t off_A, off_D, total;
};

static dad_status plan_rebuild_sites(int S, const int64_t* rows, int64_t h_in, int64_t h_out, dad_dtype dt,
                                     RebuildSitesPlan* p) {
    const dad_status rc = sites_ok(S, nullptr, nullptr, rows, false, &p->N);
    if (rc != DAD_OK) return rc;
    if (!rebuild_shape_ok(p->N, h_in, h_out)) return DAD_ERR_SHAPE;
    p->rp = plan_rebuild(p->N, h_in, h_out, dt);
    p->in_place = p->rp.fast && rebuild_dma_ok(p->N, p->rp.split) && rows_allow_blocks(S, rows);
    size_t o = align_up(p->rp.total, 256);
    p->off_A = o;
    if (!p->in_place) o += align_up((size_t)p->N * h_in * elem_size(dt), 256);
    p->off_D = o;
    if (!p->in_place) o += align_up((size_t)p->N * h_out * elem_size(dt), 256);
    p->total = o;
    return DAD_OK;
}

size_t dad_reconstruct_sites_workspace_bytes(int S, const int64_t* rows, int64_t h_in, int64_t h_out, dad_dtype dt) {
    if (!dtype_ok(dt)) return 0;
    RebuildSitesPlan p;
    return plan_rebuild_sites(S, rows, h_in, h_out, dt, &p) == DAD_OK ? p.total : 0;
}

dad_status dad_reconstruct_grad_sites(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                                      int64_t h_in, int64_t h_out, dad_dtype dt, float* G, void* workspace,
                                      size_t ws_bytes, void* stream) {
    if (!G) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    RebuildSitesPlan p;
    dad_status rc = plan_rebuild_sites(S, rows, h_in, h_out, dt, &p);
    if (rc != DAD_OK) return rc;
    int64_t N = 0;
    if ((rc = sites_ok(S, A_sites, D_sites, rows, true, &N)) != DAD_OK) return rc;
    if (p.total > 0 && !workspace) return DAD_ERR_NULL;
    if (!aligned16(G) || (workspace && !aligned16(workspace))) return DAD_ERR_ALIGN;
    if (ws_bytes < p.total) return DAD_ERR_WORKSPACE;
    if ((rc = device_ready()) != DAD_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    if (p.in_place) {
        RowBlocks a = {}, b = {};
        fill_blocks(S, A_sites, rows, &a);
        fill_blocks(S, D_sites, rows, &b);
        return fast_rebuild(nullptr, nullptr, &a, &b, p.N, h_in, h_out, G, reinterpret_cast<float*>(ws), p.rp.split,
                            p.rp.tile, s);
    }
    void* A = ws + p.off_A;
    void* D = ws + p.off_D;
    if ((rc = launch_stack(S, A_sites, D_sites, rows, h_in, h_out, dt, A, D, s)) != DAD_OK) return rc;
    return launch_rebuild(A, D, p.N, h_in, h_out, dt, G, reinterpret_cast<float*>(ws), p.rp, s);
}

// Checks of one job of the grouped rebuild; *plan receives its plan.
static dad_status rebuild_job_ok(const dad_rebuild_desc& d, dad_dtype dt, RebuildPlan* plan) {
    if (!d.L || !d.R || !d.G) return DAD_ERR_NULL;
    if (!rebuild_shape_ok(d.K, d.h_in, d.h_out)) return DAD_ERR_SHAPE;
    if (!aligned16(d.L) || !aligned16(d.R) || !aligned16(d.G)) return DAD_ERR_ALIGN;
    *plan = plan_rebuild(d.K, d.h_in, d.h_out, dt);
    return DAD_OK;
}

// Plan of a grouped rebuild.  fp32 jobs all run together (one job table) with their slabs side by
// side.  bf16 jobs run unit by unit on the stream and share one region: a unit is a run of up to 16
// consecutive jobs with whole 256-tiles and K stages, launched together with a common number of K
// chunks chosen for the run as a whole (few-tile gradients then fill the chip together and write
// fewer slabs), or a single job planned as dad_reconstruct_grad plans it.
struct RebuildUnit {
    int first, count;
};
struct GroupedRebuild {
    std::vector<RebuildPlan> single;  // per job, as a call of its own
    std::vector<RebuildUnit> units;   // bf16 only
    std::vector<SplitPlan> split;     // per job: the split it runs with
    std::vector<size_t> off;          // per job: byte offset of its slabs in the workspace
    size_t bytes = 0;
};

static void plan_grouped_rebuild(int n, const dad_rebuild_desc* descs, dad_dtype dt, GroupedRebuild* g) {
    const size_t N = (size_t)n;
    g->single.resize(N), g->split.resize(N), g->off.assign(N, 0);
    for (int i = 0; i < n; ++i) {
        g->single[(size_t)i] = plan_rebuild(descs[i].K, descs[i].h_in, descs[i].h_out, dt);
        g->split[(size_t)i] = g->single[(size_t)i].split;
    }
    if (dt == DAD_F32) {
        size_t off = 0;
        for (int i = 0; i < n; ++i) {
            g->off[(size_t)i] = off;
            off += align_up(g->single[(size_t)i].total, 256);
        }
        g->bytes = off;
        return;
    }
    for (int i = 0; i < n;) {
        int cnt = 1;
        if (rebuild_group_ok(descs[i].K, descs[i].h_in, descs[i].h_out, dt))
            while (i + cnt < n && cnt < 16 && rebuild_group_ok(descs[i + cnt].K, descs[i + cnt].h_in, descs[i + cnt].h_out, dt))
                ++cnt;
        g->units.push_back(RebuildUnit{i, cnt});
        size_t need = g->single[(size_t)i].total;
        if (cnt > 1) {
            std::vector<int64_t> K((size_t)cnt), hi((size_t)cnt), ho((size_t)cnt);
            for (int j = 0; j < cnt; ++j) K[(size_t)j] = descs[i + j].K, hi[(size_t)j] = descs[i + j].h_in, ho[(size_t)j] = descs[i + j].h_out;
            const int splits = rebuild_group_splits(cnt, K.data(), hi.data(), ho.data());
            need = 0;
            for (int j = 0; j < cnt; ++j) {
                const size_t k = (size_t)(i + j);
                g->split[k] = rebuild_group_plan(descs[i + j].K, splits);
                g->off[k] = need;
                if (g->split[k].splits > 1)
                    need += align_up((size_t)g->split[k].splits * descs[i + j].h_in * descs[i + j].h_out * 4, 256);
            }
        }
        if (need > g->bytes) g->bytes = need;
        i += cnt;
    }
}

size_t dad_reconstruct_grouped_workspace_bytes(int n, const dad_rebuild_desc* descs, dad_dtype dt) {
    if (n < 1 || n > DAD_MAX_GROUP || !descs || !dtype_ok(dt)) return 0;
    for (int i = 0; i < n; ++i)
        if (!rebuild_shape_ok(descs[i].K, descs[i].h_in, descs[i].h_out)) return 0;
    GroupedRebuild g;
    plan_grouped_rebuild(n, descs, dt, &g);
    return g.bytes;
}

dad_status dad_reconstruct_grad_grouped(int n, const dad_rebuild_desc* descs, dad_dtype dt, void* workspace,
                                        size_t ws_bytes, void* stream) {
    if (!descs) return DAD_ERR_NULL;
    if (!dtype_ok(dt)) return DAD_ERR_DTYPE;
    if (n < 1 || n > DAD_MAX_GROUP) return DAD_ERR_SHAPE;
    std::vector<RebuildPlan> plans((size_t)n);
    for (int i = 0; i < n; ++i) {
        const dad_status rc = rebuild_job_ok(descs[i], dt, &plans[(size_t)i]);
        if (rc != DAD_OK) return rc;
    }
    GroupedRebuild g;
    plan_grouped_rebuild(n, descs, dt, &g);
    if (g.bytes > 0 && !workspace) return DAD_ERR_NULL;
    if (workspace && !aligned16(workspace)) return DAD_ERR_ALIGN;
    if (ws_bytes < g.bytes) return DAD_ERR_WORKSPACE;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    hipStream_t s = (hipStream_t)stream;
    char* ws = static_cast<char*>(workspace);
    // the arguments of jobs first .. first + cnt - 1 as parallel arrays
    auto run = [&](int first, int cnt, bool f32) -> dad_status {
        const size_t c = (size_t)cnt;
        std::vector<const void*> L(c), R(c);
        std::vector<float*> G(c), slabs(c);
        std::vector<int64_t> K(c), hi(c), ho(c);
        std::vector<SplitPlan> sp(c);
        for (int j = 0; j < cnt; ++j) {
            const size_t k = (size_t)j, q = (size_t)(first + j);
            L[k] = descs[first + j].L, R[k] = descs[first + j].R, G[k] = descs[first + j].G;
            K[k] = descs[first + j].K, hi[k] = descs[first + j].h_in, ho[k] = descs[first + j].h_out;
            sp[k] = g.split[q];
            slabs[k] = sp[k].splits > 1 ? reinterpret_cast<float*>(ws + g.off[q]) : nullptr;
        }
        if (f32)
            return launch_rebuild_f32(cnt, L.data(), R.data(), G.data(), K.data(), hi.data(), ho.data(), sp.data(),
                                      slabs.data(), s);
        return launch_rebuild_group(cnt, L.data(), R.data(), G.data(), K.data(), hi.data(), ho.data(), sp.data(),
                                    slabs.data(), s);
    };
    if (dt == DAD_F32) return run(0, n, true);  // every fp32 shape runs on the fp32 MFMA kernel: one job table
    for (const RebuildUnit& u : g.units) {
        dad_status rc;
        if (u.count > 1)
            rc = run(u.first, u.count, false);
        else
            rc = launch_rebuild(descs[u.first].L, descs[u.first].R, descs[u.first].K, descs[u.first].h_in,
                                descs[u.first].h_out, dt, descs[u.first].G, reinterpret_cast<float*>(ws),
                                g.single[(size_t)u.first], s);
        if (rc != DAD_OK) return rc;
    }
    return DAD_OK;
}

dad_status dad_poll_numeric_status(const void* workspace, void* stream) {
    if (!workspace) return DAD_ERR_NULL;
    int flag = 0;
    DAD_HIP_TRY(hipMemcpyAsync(&flag, workspace, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream));
    DAD_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return flag ? DAD_ERR_NUMERIC : DAD_OK;
}

}  // extern "C"

namespace dad {

dad_status launch_thin_nn(const void* X, const float* Pt, void* out, float* partials, SplitPlan sp, int64_t N,
                          int64_t h, int r, dad_dtype dt, bool fast, int* zero_hdr, int planes, hipStream_t s,
                          const int* skip) {
    if (fast) return fast_thin_nn(X, Pt, out, N, h, r, zero_hdr, planes, s, skip);
    return gen_thin_nn(X, Pt, out, partials, sp, N, h, r, dt, zero_hdr, s, skip);
}

dad_status launch_thin_tn(const void* X, const void* V, float* out_t, float* partials, SplitPlan sp, int64_t N,
                          int64_t h, int r, dad_dtype dt, bool fast, void* out_bf16, int planes, hipStream_t s,
                          const int* skip) {
    if (fast) return fast_thin_tn(X, nullptr, V, out_t, partials, sp, N, h, r, out_bf16, planes, s, skip);
    return gen_thin_tn(X, V, out_t, partials, sp, N, h, r, dt, s, skip);
}

dad_status launch_rebuild(const void* L, const void* R, int64_t K, int64_t h_in, int64_t h_out, dad_dtype dt,
                          float* G, float* partials, const RebuildPlan& plan, hipStream_t s) {
    if (plan.fast) return fast_rebuild(L, R, nullptr, nullptr, K, h_in, h_out, G, partials, plan.split, plan.tile, s);
    if (plan.f32) return launch_rebuild_f32(1, &L, &R, &G, &K, &h_in, &h_out, &plan.split, &partials, s);
    return gen_rebuild(L, R, K, h_in, h_out, dt, G, partials, plan.split, s);
}

}  // namespace dad

// Instrumentation, not part of the method: two micro-benchmarks that measure, in the caller's own
// process and on the caller's own data, the ceilings the path's kernels are priced against.
//   dad_probe_mfma_loop   : what the matrix cores sustain when nothing but MFMAs runs
//   dad_probe_read_stream : what a plain one-pass read of a buffer reaches
// The sustained MFMA rate depends on the operand values (the chip's clock under load follows the
// bit toggling of the operands), so the loop takes its fragments from a buffer of real data.
#include "dad_internal.h"

namespace dad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PROBE_FA = 4, PROBE_FB = 2;       // the register blocking of the rebuild kernel's waves
constexpr int PROBE_THREADS = 512;              // eight waves per workgroup, one workgroup per CU
constexpr size_t PROBE_FRAG_BYTES = (size_t)(PROBE_FA + PROBE_FB) * PROBE_THREADS * 16;  // per workgroup

// Every wave holds 4 + 2 operand fragments (loaded once) and 8 accumulator tiles and issues
// iters * 8 independent v_mfma_f32_32x32x16_bf16.
__global__ __launch_bounds__(PROBE_THREADS) void k_probe_mfma_loop(const bf16x8* __restrict__ src, size_t frag_sets,
                                                                   float* __restrict__ sink, int iters) {
    const size_t set = (size_t)blockIdx.x % frag_sets;
    const bf16x8* base = src + set * (PROBE_FA + PROBE_FB) * PROBE_THREADS + threadIdx.x;
    bf16x8 fa[PROBE_FA], fb[PROBE_FB];
#pragma unroll
    for (int i = 0; i < PROBE_FA; ++i) fa[i] = base[i * PROBE_THREADS];
#pragma unroll
    for (int i = 0; i < PROBE_FB; ++i) fb[i] = base[(PROBE_FA + i) * PROBE_THREADS];
    f32x16 acc[PROBE_FA][PROBE_FB];
#pragma unroll
    for (int a = 0; a < PROBE_FA; ++a)
#pragma unroll
        for (int b = 0; b < PROBE_FB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < PROBE_FA; ++a)
#pragma unroll
            for (int b = 0; b < PROBE_FB; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[b], fa[a], acc[a][b], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < PROBE_FA; ++a)
#pragma unroll
        for (int b = 0; b < PROBE_FB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[a][b][v];
    if (s == 1.2345678e33f) *sink = s;  // keeps the loop alive; practically never taken
}

// One pass over `n16` 16-byte units: every workgroup streams a contiguous share, eight units per
// thread in flight, non-temporal loads (the buffer is read once).
__global__ __launch_bounds__(256) void k_probe_read_stream(const u32x4* __restrict__ p, size_t n16, size_t per_block,
                                                           uint32_t* __restrict__ sink) {
    const size_t beg = (size_t)blockIdx.x * per_block;
    size_t end = beg + per_block;
    if (end > n16) end = n16;
    uint32_t acc = 0;
    size_t i = beg + threadIdx.x;
    for (; i + 7 * 256 < end; i += 8 * 256) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].w;
    }
    for (; i < end; i += 256) {
        const u32x4 v = __builtin_nontemporal_load(p + i);
        acc += v.x ^ v.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;  // keeps the loads alive; practically never taken
}

// Times `reps` launches between two events on `s`; the stream is synchronised.
template <typename F>
static dad_status time_launches(hipStream_t s, int reps, F&& launch, double* seconds_per_launch) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    DAD_HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return DAD_ERR_HIP;
    }
    dad_status rc = DAD_OK;
    float ms = 0.f;
    launch();  // warm-up
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) rc = DAD_ERR_HIP;
    if (rc == DAD_OK && hipEventRecord(e0, s) != hipSuccess) rc = DAD_ERR_HIP;
    for (int i = 0; rc == DAD_OK && i < reps; ++i) launch();
    if (rc == DAD_OK && (hipGetLastError() != hipSuccess || hipEventRecord(e1, s) != hipSuccess ||
                         hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
        rc = DAD_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *seconds_per_launch = (double)ms * 1e-3 / reps;
    return rc;
}

}  // namespace dad

using namespace dad;

extern "C" dad_status dad_probe_mfma_loop(const void* operands, size_t operand_bytes, int iters, void* sink,
                                          void* stream, double* tflops) {
    if (!operands || !sink || !tflops) return DAD_ERR_NULL;
    if (operand_bytes < PROBE_FRAG_BYTES || iters < 1 || iters > (1 << 24)) return DAD_ERR_SHAPE;
    if (!aligned16(operands) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return DAD_ERR_ALIGN;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, cus = 0;
    DAD_HIP_TRY(hipGetDevice(&dev));
    DAD_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus < 1) return DAD_ERR_HIP;
    const size_t sets = operand_bytes / PROBE_FRAG_BYTES;
    double sec = 0.0;
    const dad_status rc = time_launches(
        s, 2,
        [&] {
            hipLaunchKernelGGL(k_probe_mfma_loop, dim3((unsigned)cus), dim3(PROBE_THREADS), 0, s,
                               (const bf16x8*)operands, sets, (float*)sink, iters);
        },
        &sec);
    if (rc != DAD_OK) return rc;
    const double flops = 2.0 * 32 * 32 * 16 * PROBE_FA * PROBE_FB * (PROBE_THREADS / 64) * (double)iters * cus;
    *tflops = flops / sec / 1e12;
    return DAD_OK;
}

extern "C" dad_status dad_probe_read_stream(const void* src, size_t bytes, void* sink, void* stream, double* gbps) {
    if (!src || !sink || !gbps) return DAD_ERR_NULL;
    if (bytes < 16) return DAD_ERR_SHAPE;
    if (!aligned16(src) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return DAD_ERR_ALIGN;
    if (const dad_status ready = device_ready(); ready != DAD_OK) return ready;
    hipStream_t s = (hipStream_t)stream;
    const size_t n16 = bytes / 16;
    size_t blocks = 4096;  // sixteen workgroups per CU
    if (blocks > (n16 + 2047) / 2048) blocks = (n16 + 2047) / 2048;
    const size_t per_block = (n16 + blocks - 1) / blocks;
    double sec = 0.0;
    const dad_status rc = time_launches(
        s, 5,
        [&] {
            hipLaunchKernelGGL(k_probe_read_stream, dim3((unsigned)blocks), dim3(256), 0, s, (const u32x4*)src, n16,
                               per_block, (uint32_t*)sink);
        },
        &sec);
    if (rc != DAD_OK) return rc;
    *gbps = (double)(n16 * 16) / sec / 1e9;
    return DAD_OK;
}

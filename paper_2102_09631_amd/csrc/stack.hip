// dad_stack_factors: the sites' row blocks are contiguous in memory, so stacking
// is a batch of contiguous copies.  One launch moves up to MAX_SEG segments; a
// workgroup owns one 32 KiB chunk of one segment and moves it with 16-byte
// accesses when source, destination and length allow it.
#include "dad_internal.h"

namespace dad {

constexpr int MAX_SEG = 64;
constexpr int64_t CHUNK = 32768;

struct SegTable {
    const char* src[MAX_SEG];
    char* dst[MAX_SEG];
    int64_t bytes[MAX_SEG];
    int first_block[MAX_SEG + 1];  // prefix sum of chunk counts
    int unit[MAX_SEG];             // 16, 8, 4 or 2: widest access that stays aligned
    int nt[MAX_SEG];               // non-temporal stores: the stacked matrix is larger than the Infinity Cache
    int n;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Eight units per thread in flight.  The sources are read once: non-temporal loads.  The stores are
// non-temporal only when the stacked matrix does not fit the Infinity Cache anyway (6 % faster then;
// a small one is better left there for the call that reads it next).
template <typename U, bool NT>
__device__ __forceinline__ void copy_units(const char* __restrict__ s, char* __restrict__ d, int64_t bytes) {
    const U* sp = reinterpret_cast<const U*>(s);
    U* dp = reinterpret_cast<U*>(d);
    const int64_t n = bytes / (int64_t)sizeof(U);
    int64_t i = threadIdx.x;
    for (; i + 7 * 256 < n; i += 8 * 256) {
        U v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(sp + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (NT)
                __builtin_nontemporal_store(v[u], dp + i + u * 256);
            else
                dp[i + u * 256] = v[u];
        }
    }
    for (; i < n; i += 256) dp[i] = __builtin_nontemporal_load(sp + i);
}

__global__ __launch_bounds__(256) void k_stack(SegTable tb) {
    const int b = blockIdx.x;
    int seg = 0;
    while (seg + 1 < tb.n && tb.first_block[seg + 1] <= b) ++seg;
    const int64_t off = (int64_t)(b - tb.first_block[seg]) * CHUNK;
    int64_t len = tb.bytes[seg] - off;
    if (len > CHUNK) len = CHUNK;
    const char* s = tb.src[seg] + off;
    char* d = tb.dst[seg] + off;
    switch (tb.unit[seg]) {
        case 16:
            if (tb.nt[seg])
                copy_units<u32x4, true>(s, d, len);
            else
                copy_units<u32x4, false>(s, d, len);
            break;
        case 8: copy_units<u32x2, false>(s, d, len); break;
        case 4: copy_units<uint32_t, false>(s, d, len); break;
        default: copy_units<uint16_t, false>(s, d, len); break;
    }
}

static int widest_unit(const void* s, const void* d, int64_t bytes) {
    uintptr_t m = reinterpret_cast<uintptr_t>(s) | reinterpret_cast<uintptr_t>(d) | (uintptr_t)bytes;
    if ((m & 15) == 0) return 16;
    if ((m & 7) == 0) return 8;
    if ((m & 3) == 0) return 4;
    return 2;
}

dad_status launch_stack(int S, const void* const* A_sites, const void* const* D_sites, const int64_t* rows,
                        int64_t h_in, int64_t h_out, dad_dtype dt, void* A_out, void* D_out, hipStream_t st) {
    const int64_t es = (int64_t)elem_size(dt);
    SegTable tb;
    tb.n = 0;
    tb.first_block[0] = 0;
    int64_t row_off = 0;
    auto flush = [&]() -> dad_status {
        if (tb.n == 0) return DAD_OK;
        ProfScope prof(KID_STACK, st);
        hipLaunchKernelGGL(k_stack, dim3((unsigned)tb.first_block[tb.n]), dim3(256), 0, st, tb);
        DAD_LAUNCH_CHECK();
        tb.n = 0;
        tb.first_block[0] = 0;
        return DAD_OK;
    };
    auto push = [&](const void* src, char* dst, int64_t bytes, int nt) -> dad_status {
        // a segment whose chunk count would overflow the int prefix goes out in pieces
        const int64_t max_piece = CHUNK * (int64_t)(1 << 20);
        const char* sp = static_cast<const char*>(src);
        while (bytes > 0) {
            int64_t piece = bytes < max_piece ? bytes : max_piece;
            int i = tb.n;
            tb.src[i] = sp;
            tb.dst[i] = dst;
            tb.bytes[i] = piece;
            tb.unit[i] = widest_unit(sp, dst, piece);
            tb.nt[i] = nt;
            tb.first_block[i + 1] = tb.first_block[i] + (int)ceil_div(piece, CHUNK);
            tb.n = i + 1;
            if (tb.n == MAX_SEG || tb.first_block[tb.n] > (1 << 28)) {
                dad_status rc = flush();
                if (rc != DAD_OK) return rc;
            }
            sp += piece;
            dst += piece;
            bytes -= piece;
        }
        return DAD_OK;
    };
    int64_t total_rows = 0;
    for (int s = 0; s < S; ++s) total_rows += rows[s];
    const int64_t big = (int64_t)200 << 20;
    const int nt_a = total_rows * h_in * es > big, nt_d = total_rows * h_out * es > big;
    for (int s = 0; s < S; ++s) {
        if (rows[s] > 0) {
            dad_status rc = push(A_sites[s], static_cast<char*>(A_out) + row_off * h_in * es, rows[s] * h_in * es, nt_a);
            if (rc != DAD_OK) return rc;
            rc = push(D_sites[s], static_cast<char*>(D_out) + row_off * h_out * es, rows[s] * h_out * es, nt_d);
            if (rc != DAD_OK) return rc;
        }
        row_off += rows[s];
    }
    return flush();
}

}  // namespace dad

// Optional per-kernel timing: when enabled, every kernel launch of the library is bracketed by a
// pair of HIP events on the launch stream; dad_profile_get sums the elapsed times per kernel.
// Disabled (the default) it costs one branch per launch.
#include <atomic>
#include <mutex>
#include <vector>

#include "dad_internal.h"

namespace dad {

static const char* const kKernelNames[KID_COUNT] = {
    "k_stack",       "k_thin_nn_bf16", "k_thin_tn_bf16", "k_reduce_slabs", "k_qr_gram", "k_qr_apply<NA,true>",
    "k_qr_apply<NA,false>",  "k_rebuild_bf16", "k_thin_nn",      "k_thin_tn",      "k_rebuild",      "k_panel_init",  "k_rebuild_bf16_dma", "k_backprop_bf16", "k_backprop",
    "k_gram_tiles", "k_gram_gather", "k_ns_step", "k_ns_project", "k_rebuild_f32_mfma", "k_reduce_slabs_wide", "k_seq_vector",
};

struct Pending {
    int id;
    hipEvent_t a, b;
};

static std::mutex g_mu;
static std::atomic<bool> g_on{false};  // read on every launch without the mutex
static std::vector<Pending> g_pending;
static std::vector<hipEvent_t> g_free;
static double g_ms[KID_COUNT];
static int64_t g_n[KID_COUNT];

static hipEvent_t get_event() {
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

ProfScope::ProfScope(int id, hipStream_t s) : id_(id), s_(s), a_(nullptr) {
    if (!g_on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t a = get_event();
    if (a && hipEventRecord(a, s) == hipSuccess) a_ = a;
}

ProfScope::~ProfScope() {
    if (!a_) return;
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t b = get_event();
    if (b && hipEventRecord(b, s_) == hipSuccess) g_pending.push_back({id_, (hipEvent_t)a_, b});
}

static dad_status drain() {
    for (const Pending& p : g_pending) {
        float ms = 0.f;
        DAD_HIP_TRY(hipEventSynchronize(p.b));
        DAD_HIP_TRY(hipEventElapsedTime(&ms, p.a, p.b));
        g_ms[p.id] += ms;
        g_n[p.id] += 1;
        g_free.push_back(p.a);
        g_free.push_back(p.b);
    }
    g_pending.clear();
    return DAD_OK;
}

}  // namespace dad

using namespace dad;

extern "C" {

dad_status dad_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(g_mu);
    dad_status rc = drain();
    g_on.store(on != 0, std::memory_order_relaxed);
    return rc;
}

dad_status dad_profile_reset(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    dad_status rc = drain();
    for (int i = 0; i < KID_COUNT; ++i) {
        g_ms[i] = 0.0;
        g_n[i] = 0;
    }
    return rc;
}

int dad_profile_kernel_count(void) { return KID_COUNT; }

const char* dad_profile_kernel_name(int id) { return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : ""; }

dad_status dad_profile_get(int id, double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return DAD_ERR_NULL;
    if (id < 0 || id >= KID_COUNT) return DAD_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_mu);
    dad_status rc = drain();
    *total_ms = g_ms[id];
    *launches = g_n[id];
    return rc;
}

}  // extern "C"

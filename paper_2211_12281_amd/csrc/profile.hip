// Optional HIP-event instrumentation of the dominant kernels, for benchmarks.
#include "kge_internal.h"
#include <vector>

namespace {
struct Rec { int slot; hipEvent_t a, b; };
unsigned g_mask = 0;                     // bit s: slot s is instrumented
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;

hipEvent_t get_event() {
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

KgeProfScope::KgeProfScope(int slot, hipStream_t st) : slot_(slot), st_(st), a_(nullptr), b_(nullptr) {
    if (!((g_mask >> slot) & 1u)) return;
    a_ = get_event(); b_ = get_event();
    if (a_ && b_) (void)hipEventRecord((hipEvent_t)a_, st_);
}

KgeProfScope::~KgeProfScope() {
    if (!a_ || !b_) return;
    (void)hipEventRecord((hipEvent_t)b_, st_);
    g_recs.push_back(Rec{slot_, (hipEvent_t)a_, (hipEvent_t)b_});
}

extern "C" int kge_profile_enable(int on) {
    g_mask = on < 0 ? ~0u : (unsigned)on;
    return KGE_OK;
}

extern "C" int kge_profile_collect(int slot, double *total_ms, int64_t *launches) {
    if (slot < 0 || slot >= KGE_PROF_SLOTS || !total_ms || !launches) return KGE_E_INVALID_ARG;
    double tot = 0.0; int64_t n = 0;
    std::vector<Rec> keep;
    for (const Rec &r : g_recs) {
        if (r.slot != slot) { keep.push_back(r); continue; }
        if (hipEventSynchronize(r.b) != hipSuccess) return KGE_E_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return KGE_E_HIP;
        tot += ms; ++n;
        g_pool.push_back(r.a); g_pool.push_back(r.b);
    }
    g_recs.swap(keep);
    *total_ms = tot; *launches = n;
    return KGE_OK;
}

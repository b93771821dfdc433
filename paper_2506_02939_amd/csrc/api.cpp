// Host-only entry points of libpamm: status names, workspace queries and the generator sampler.
#include <unordered_map>

#include "pamm_plan.h"
#include "pamm_profile.h"

using namespace pamm;

namespace pamm {
Profiler g_profiler;
pamm_debug_plan g_plan_override = {0, 0, 0, 0, 0, 0};
}

extern "C" const char* pamm_status_string(pamm_status s) {
    switch (s) {
        case PAMM_OK: return "PAMM_OK";
        case PAMM_ERR_INVALID_ARG: return "PAMM_ERR_INVALID_ARG";
        case PAMM_ERR_UNSUPPORTED: return "PAMM_ERR_UNSUPPORTED";
        case PAMM_ERR_WORKSPACE: return "PAMM_ERR_WORKSPACE";
        case PAMM_ERR_DEVICE: return "PAMM_ERR_DEVICE";
    }
    return "PAMM_ERR_UNKNOWN";
}

extern "C" size_t pamm_compress_workspace(int64_t b, int64_t n, int64_t k, pamm_dtype dt) {
    CompressPlan p;
    return plan_compress(b, n, k, dt, &p) == PAMM_OK ? p.total : 0;
}

extern "C" size_t pamm_grad_workspace(int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt) {
    GradPlan p;
    return plan_grad(b, n, k, m, dt, &p) == PAMM_OK ? p.total : 0;
}

extern "C" size_t pamm_sketch_grad_workspace(int64_t b, int64_t n, int64_t r, int64_t m, pamm_dtype dt) {
    SketchGradPlan p;
    return plan_sketch_grad(b, n, r, m, dt, &p) == PAMM_OK ? p.total : 0;
}

namespace {

struct SplitMix64 {
    uint64_t state;
    uint64_t next() {
        state += 0x9E3779B97F4A7C15ULL;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
        return z ^ (z >> 31);
    }
    // uniform on [0, range) by rejection: discard the lowest (2^64 mod range) outputs
    uint64_t below(uint64_t range) {
        const uint64_t cut = (~range + 1) % range;
        for (;;) {
            uint64_t x = next();
            if (x >= cut) return x % range;
        }
    }
};

}  // namespace

// Partial Fisher-Yates over the virtual identity arrangement of [0,b): only displaced positions are stored,
// so the cost is O(k) whatever b is.
extern "C" pamm_status pamm_sample_indices(int64_t b, int64_t k, uint64_t seed, int32_t* idx_host) {
    if (!idx_host || b < 1 || k < 1 || k > b || b >= (int64_t(1) << 31)) return PAMM_ERR_INVALID_ARG;
    SplitMix64 rng{seed};
    std::unordered_map<int64_t, int64_t> displaced;
    displaced.reserve(size_t(2 * k));
    auto at = [&](int64_t pos) {
        auto it = displaced.find(pos);
        return it == displaced.end() ? pos : it->second;
    };
    for (int64_t t = 0; t < k; ++t) {
        const int64_t r = t + int64_t(rng.below(uint64_t(b - t)));
        const int64_t vt = at(t), vr = at(r);
        displaced[r] = vt;      // position t is never looked at again, so only r needs recording
        idx_host[t] = int32_t(vr);
    }
    return PAMM_OK;
}

extern "C" pamm_status pamm_debug_set_plan(const pamm_debug_plan* plan_host) {
    g_plan_override = plan_host ? *plan_host : pamm_debug_plan{0, 0, 0, 0, 0, 0};
    return PAMM_OK;
}

extern "C" pamm_status pamm_debug_bounded(uint64_t seed, uint64_t range, int64_t count, uint64_t* out_host) {
    if (!out_host || range == 0 || count < 0) return PAMM_ERR_INVALID_ARG;
    SplitMix64 rng{seed};
    for (int64_t i = 0; i < count; ++i) out_host[i] = rng.below(range);
    return PAMM_OK;
}

extern "C" const char* pamm_kernel_name(int id) {
    static const char* names[kNumKernels] = {"k_gather", "k_score", "k_finalize", "k_group", "k_contract", "k_prep", "k_ctb", "k_piece_sum", "k_sketch", "k_sketch_contract"};
    return (id >= 0 && id < kNumKernels) ? names[id] : "";
}

extern "C" pamm_status pamm_profile_begin(void) {
    std::lock_guard<std::mutex> lock(g_profiler.mu);
    for (auto& sp : g_profiler.spans) { (void)hipEventDestroy(sp.start); (void)hipEventDestroy(sp.stop); }
    g_profiler.spans.clear();
    g_profiler.on = true;
    return PAMM_OK;
}

extern "C" pamm_status pamm_profile_end(double* ms_total, int64_t* launches) {
    if (!ms_total || !launches) return PAMM_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_profiler.mu);
    g_profiler.on = false;
    for (int i = 0; i < kNumKernels; ++i) { ms_total[i] = 0.0; launches[i] = 0; }
    pamm_status st = PAMM_OK;
    for (auto& sp : g_profiler.spans) {
        float ms = 0.f;
        if (hipEventSynchronize(sp.stop) != hipSuccess || hipEventElapsedTime(&ms, sp.start, sp.stop) != hipSuccess) st = PAMM_ERR_DEVICE;
        else { ms_total[sp.id] += double(ms); launches[sp.id] += 1; }
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    g_profiler.spans.clear();
    return st;
}

// Optional per-kernel timing: when switched on, every kernel launch is bracketed by a pair of HIP events on the
// launch stream.  Off by default; the hot path then pays one predictable branch per launch.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>
#include <vector>

namespace pamm {

enum KernelId { kGather = 0, kScore, kFinalize, kGroup, kContract, kPrep, kCtb, kPieceSum, kSketch, kSketchContract, kNumKernels };

struct Profiler {
    bool on = false;
    std::mutex mu;
    struct Span { int id; hipEvent_t start, stop; };
    std::vector<Span> spans;

    // returns an index into spans, or -1 when profiling is off
    int begin(int id, hipStream_t s) {
        if (!on) return -1;
        std::lock_guard<std::mutex> lock(mu);
        Span sp{id, nullptr, nullptr};
        if (hipEventCreate(&sp.start) != hipSuccess || hipEventCreate(&sp.stop) != hipSuccess) return -1;
        (void)hipEventRecord(sp.start, s);
        spans.push_back(sp);
        return int(spans.size()) - 1;
    }
    void end(int token, hipStream_t s) {
        if (token < 0) return;
        std::lock_guard<std::mutex> lock(mu);
        (void)hipEventRecord(spans[size_t(token)].stop, s);
    }
};

extern Profiler g_profiler;

struct ScopedSpan {
    int token;
    hipStream_t s;
    ScopedSpan(int id, hipStream_t stream) : token(g_profiler.begin(id, stream)), s(stream) {}
    ~ScopedSpan() { g_profiler.end(token, s); }
};

}  // namespace pamm

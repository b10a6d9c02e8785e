// Per-kernel timing with HIP events on the library's own stream.
#include "ps_common.h"

namespace ps {

hipEvent_t Profiler::take()
{
    if (!pool_.empty()) {
        hipEvent_t e = pool_.back();
        pool_.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void Profiler::begin(int id, hipStream_t s)
{
    if (!enabled) return;
    open_ = Rec{id, take(), take()};
    if (open_.a) (void)hipEventRecord(open_.a, s);
}

void Profiler::end(hipStream_t s)
{
    if (!enabled || open_.id < 0) return;
    if (open_.b) (void)hipEventRecord(open_.b, s);
    recs_.push_back(open_);
    open_.id = -1;
}

hipError_t Profiler::collect(hipStream_t s)
{
    hipError_t e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    for (const Rec& r : recs_) {
        float ms = 0.f;
        if (r.a && r.b && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            total_ms[r.id] += ms;
            launches[r.id] += 1;
        }
        if (r.a) pool_.push_back(r.a);
        if (r.b) pool_.push_back(r.b);
    }
    recs_.clear();
    return hipSuccess;
}

void Profiler::reset()
{
    for (int i = 0; i < K_COUNT; ++i) {
        total_ms[i] = 0.0;
        launches[i] = 0;
    }
}

void Profiler::destroy()
{
    for (const Rec& r : recs_) {
        if (r.a) pool_.push_back(r.a);
        if (r.b) pool_.push_back(r.b);
    }
    recs_.clear();
    for (hipEvent_t e : pool_) (void)hipEventDestroy(e);
    pool_.clear();
}

}  // namespace ps

// HIP-event timing of one solve call: one pair of events around the call and
// one pair around every launch of the DP sweep kernel, all on the caller's
// stream.
#include <new>

#include "kernels.h"

namespace deft {

hipEvent_t Profiler::next()
{
    if (used_ == cap_) {
        const int ncap = cap_ ? cap_ * 2 : 64;
        hipEvent_t *n = new (std::nothrow) hipEvent_t[ncap];
        if (!n) { failed_ = true; return nullptr; }
        for (int i = 0; i < cap_; ++i) n[i] = ev_[i];
        for (int i = cap_; i < ncap; ++i) {
            if (hipEventCreate(&n[i]) != hipSuccess) {
                (void)hipGetLastError();
                for (int k = cap_; k < i; ++k) (void)hipEventDestroy(n[k]);
                delete[] n;
                failed_ = true;
                return nullptr;
            }
        }
        delete[] ev_;
        ev_ = n;
        cap_ = ncap;
    }
    return ev_[used_++];
}

bool Profiler::begin(hipStream_t st)
{
    used_ = 0;
    failed_ = false;
    have_call_ = false;
    hipEvent_t e = next();          // slot 0: start of call
    hipEvent_t f = next();          // slot 1: end of call (recorded in end())
    if (!e || !f) return false;
    if (hipEventRecord(e, st) != hipSuccess) { (void)hipGetLastError(); return false; }
    return true;
}

void Profiler::sweep_begin(hipStream_t st)
{
    hipEvent_t e = next();
    if (e && hipEventRecord(e, st) != hipSuccess) { (void)hipGetLastError(); failed_ = true; }
}

void Profiler::sweep_end(hipStream_t st) { sweep_begin(st); }

void Profiler::end(hipStream_t st)
{
    if (cap_ < 2) { failed_ = true; return; }
    if (hipEventRecord(ev_[1], st) != hipSuccess) { (void)hipGetLastError(); failed_ = true; }
    have_call_ = true;
}

deft_status_t Profiler::read(deft_knapsack_profile_t *out)
{
    if (!have_call_) return DEFT_ERR_INVALID_ARG;
    if (failed_) return DEFT_ERR_DEVICE;
    if (hipEventSynchronize(ev_[1]) != hipSuccess) { (void)hipGetLastError(); return DEFT_ERR_DEVICE; }
    float total = 0.f, sweep = 0.f;
    if (hipEventElapsedTime(&total, ev_[0], ev_[1]) != hipSuccess) { (void)hipGetLastError(); return DEFT_ERR_DEVICE; }
    int launches = 0;
    for (int i = 2; i + 1 < used_; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev_[i], ev_[i + 1]) != hipSuccess) { (void)hipGetLastError(); return DEFT_ERR_DEVICE; }
        sweep += ms;
        ++launches;
    }
    out->total_ms = total;
    out->sweep_ms = sweep;
    out->sweep_launches = launches;
    out->other_ms = total - sweep;
    return DEFT_OK;
}

void Profiler::destroy()
{
    for (int i = 0; i < cap_; ++i) (void)hipEventDestroy(ev_[i]);
    delete[] ev_;
    ev_ = nullptr;
    cap_ = used_ = 0;
}

}  // namespace deft

// HIP-event timing of solve calls: one pair of events around each call and one
// pair around every launch of the DP sweep kernel, all recorded on the caller's
// stream; nothing is waited for until the figures are read.
#include <new>

#include "kernels.h"

namespace deft {

hipEvent_t Profiler::Pool::get(int i)
{
    if (i >= cap) {
        int ncap = cap ? cap : 64;
        while (ncap <= i) ncap *= 2;
        hipEvent_t *n = new (std::nothrow) hipEvent_t[ncap];
        if (!n) return nullptr;
        for (int k = 0; k < cap; ++k) n[k] = ev[k];
        for (int k = cap; k < ncap; ++k) {
            if (hipEventCreate(&n[k]) != hipSuccess) {
                (void)hipGetLastError();
                for (int z = cap; z < k; ++z) (void)hipEventDestroy(n[z]);
                delete[] n;
                return nullptr;
            }
        }
        delete[] ev;
        ev = n;
        cap = ncap;
    }
    return ev[i];
}

void Profiler::Pool::destroy()
{
    for (int k = 0; k < cap; ++k) (void)hipEventDestroy(ev[k]);
    delete[] ev;
    ev = nullptr;
    cap = 0;
}

void Profiler::record(Pool &p, int idx, hipStream_t st)
{
    hipEvent_t e = p.get(idx);
    if (!e || hipEventRecord(e, st) != hipSuccess) {
        (void)hipGetLastError();
        failed_ = true;
    }
}

bool Profiler::begin(hipStream_t st)
{
    record(call_, ncall_, st);
    if (failed_) return false;
    ++ncall_;
    return true;
}

void Profiler::end(hipStream_t st)
{
    record(call_, ncall_, st);
    ++ncall_;
}

void Profiler::sweep_begin(hipStream_t st)
{
    record(sweep_, nsweep_, st);
    ++nsweep_;
}

void Profiler::sweep_end(hipStream_t st) { sweep_begin(st); }

deft_status_t Profiler::read(deft_knapsack_profile_t *out)
{
    if (ncall_ < 2 || (ncall_ & 1) || (nsweep_ & 1)) return DEFT_ERR_INVALID_ARG;
    if (failed_) { reset(); return DEFT_ERR_DEVICE; }
    deft_status_t rc = DEFT_OK;
    float total = 0.f, sweep = 0.f;
    if (hipEventSynchronize(call_.ev[ncall_ - 1]) != hipSuccess) rc = DEFT_ERR_DEVICE;
    for (int i = 0; rc == DEFT_OK && i < ncall_; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, call_.ev[i], call_.ev[i + 1]) != hipSuccess) rc = DEFT_ERR_DEVICE;
        total += ms;
    }
    for (int i = 0; rc == DEFT_OK && i < nsweep_; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sweep_.ev[i], sweep_.ev[i + 1]) != hipSuccess) rc = DEFT_ERR_DEVICE;
        sweep += ms;
    }
    if (rc != DEFT_OK) (void)hipGetLastError();
    out->total_ms = total;
    out->sweep_ms = sweep;
    out->sweep_launches = nsweep_ / 2;
    out->other_ms = total - sweep;
    reset();
    return rc;
}

void Profiler::destroy()
{
    call_.destroy();
    sweep_.destroy();
    reset();
}

}  // namespace deft

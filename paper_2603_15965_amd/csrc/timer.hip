// Benchmark aid: the device-side duration of one base-projection launch, read from the
// launch's own dispatch (hipExtLaunchKernelGGL with a start and a stop event), i.e. the
// interval a kernel trace reports.  Events recorded around a launch with hipEventRecord are
// marker packets of their own: they add 2-4 us of dispatch gap to the interval and cost the
// stream ~3 us each, a visible share of a 40 us step.
#include "../../include/molora.h"

#include "common.h"

#include <new>

struct molora_launch_timer {
    hipEvent_t start;
    hipEvent_t stop;
};

extern "C" {

molora_status molora_launch_timer_create(molora_launch_timer **out) {
    if (out == nullptr) return MOLORA_EINVAL;
    *out = nullptr;
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess) return MOLORA_EHIP;
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return MOLORA_EHIP;
    }
    molora_launch_timer *t = new (std::nothrow) molora_launch_timer{a, b};
    if (t == nullptr) {
        (void)hipEventDestroy(a);
        (void)hipEventDestroy(b);
        return MOLORA_EHIP;
    }
    *out = t;
    return MOLORA_OK;
}

molora_status molora_launch_timer_arm(molora_launch_timer *t) {
    if (t == nullptr) return MOLORA_EINVAL;
    molora::arm_launch_events(t->start, t->stop);
    return MOLORA_OK;
}

molora_status molora_launch_timer_elapsed_us(molora_launch_timer *t, double *us) {
    if (t == nullptr || us == nullptr) return MOLORA_EINVAL;
    *us = 0.0;
    if (hipEventSynchronize(t->stop) != hipSuccess) return MOLORA_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t->start, t->stop) != hipSuccess) {
        (void)hipGetLastError();  // armed, but no launch took the events
        return MOLORA_EHIP;
    }
    *us = 1e3 * (double)ms;
    return MOLORA_OK;
}

void molora_launch_timer_destroy(molora_launch_timer *t) {
    if (t == nullptr) return;
    (void)hipEventDestroy(t->start);
    (void)hipEventDestroy(t->stop);
    delete t;
}

}  // extern "C"

// Kernel-level timing of the library's own launches (measurement aid of the benchmark).
#include "bed.h"
#include "bed_kernel.h"

namespace {

void release(bed::LaunchTimer& t) {
    for (int i = 0; i < t.capacity; ++i) {
        if (t.start && t.start[i]) (void)hipEventDestroy(t.start[i]);
        if (t.stop && t.stop[i]) (void)hipEventDestroy(t.stop[i]);
    }
    delete[] t.start;
    delete[] t.stop;
    t = bed::LaunchTimer();
}

}  // namespace

extern "C" {

int bed_timing_begin(int capacity) {
    if (capacity < 1 || capacity > (1 << 20)) return BED_ERR_ARG;
    bed::LaunchTimer& t = bed::launch_timer();
    release(t);
    t.start = new hipEvent_t[capacity]();
    t.stop = new hipEvent_t[capacity]();
    t.capacity = capacity;
    for (int i = 0; i < capacity; ++i) {
        if (hipEventCreate(&t.start[i]) != hipSuccess || hipEventCreate(&t.stop[i]) != hipSuccess) {
            release(t);
            return BED_ERR_LAUNCH;
        }
    }
    return BED_OK;
}

int bed_timing_arm(int on) {
    bed::LaunchTimer& t = bed::launch_timer();
    if (!t.start) return BED_ERR_ARG;
    t.armed = on != 0;
    return BED_OK;
}

int bed_timing_end(float* microseconds, int max_count, int* count) {
    bed::LaunchTimer& t = bed::launch_timer();
    if (!t.start || !count || max_count < 0 || (max_count > 0 && !microseconds)) return BED_ERR_ARG;
    t.armed = false;
    const int k = t.used < max_count ? t.used : max_count;
    int status = BED_OK;
    for (int i = 0; i < k; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(t.stop[i]) != hipSuccess || hipEventElapsedTime(&ms, t.start[i], t.stop[i]) != hipSuccess) {
            status = BED_ERR_LAUNCH;
            ms = 0.f;
        }
        microseconds[i] = ms * 1000.f;
    }
    *count = t.used;
    release(t);
    return status;
}

}  // extern "C"

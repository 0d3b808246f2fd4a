// Optional per-kernel timing with HIP events on the launch stream (diagnostic;
// off by default, costs nothing when off).
#pragma once

#include "common.hpp"

namespace spo {

enum KernelClass {
    kTimeFwdSweep = 0,    // fused forward: vocabulary sweep
    kTimeRecompute = 1,   // fused backward: logits recompute -> dZ
    kTimeDHidden = 2,     // fused backward: dHidden = dZ W
    kTimeDW = 3,          // fused backward: dW += dZ^T X
    kTimeLogitsFwd = 4,   // logits-in forward row pass
    kTimeLogitsBwd = 5,   // logits-in backward row pass
    kTimeLogitsToDz = 6,  // one-call forward + backward: stored logits -> dZ
    kTimeClasses = 7
};

bool timing_enabled();
void timing_begin(int cls, hipStream_t s);
void timing_end(int cls, hipStream_t s);

struct ScopedKernelTimer {
    int cls;
    hipStream_t s;
    bool on;
    ScopedKernelTimer(int c, hipStream_t st) : cls(c), s(st), on(timing_enabled()) { if (on) timing_begin(cls, s); }
    ~ScopedKernelTimer() { if (on) timing_end(cls, s); }
};

}  // namespace spo

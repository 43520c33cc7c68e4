// Optional per-kernel timing with HIP events on the stream the kernels are
// launched on.  Off by default; when on, every launcher brackets its kernel
// with an event pair and notes the algorithmic flops and bytes of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>

namespace edl {

void prof_enable(bool on);
bool prof_enabled();
void prof_begin(const char* label, double flops, double bytes, hipStream_t st);
void prof_end(hipStream_t st);
// Waits for the recorded events, writes a JSON array of
// {"name","launches","ms","flops","bytes"} (totals per label) and clears the records.
// Returns the number of characters needed (excluding the NUL), or -1 on a HIP error.
long prof_report(char* buf, size_t cap);

// `base`, or with EDL_PROFILE_BY_SHAPE in the environment and profiling on "base M=.. C=.." (one report
// line per distinct shape); the returned string lives until the process ends.
const char* prof_shape_label(const char* base, long long M, int C);

struct ProfScope {
    hipStream_t st;
    bool on;
    ProfScope(const char* label, double flops, double bytes, hipStream_t s) : st(s), on(prof_enabled()) {
        if (on) prof_begin(label, flops, bytes, st);
    }
    ~ProfScope() {
        if (on) prof_end(st);
    }
};

}  // namespace edl

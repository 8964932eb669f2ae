// Optional per-launch timing of the library's heavy kernels with HIP events on the
// caller's stream.  Off by default; when off a launch pays one branch.  Internal.
#pragma once
#include <hip/hip_runtime.h>

namespace fise {

enum { PROF_IGEMM = 0, PROF_IGEMM_GEGLU = 1, PROF_ATTENTION = 2, PROF_IGEMM_WIDE = 3, PROF_REDUCE = 4, PROF_KINDS = 5 };

extern bool g_profile_on;
void profile_begin(int kind, double flops, double bytes, hipStream_t st);
void profile_end(hipStream_t st);

struct ProfileScope {
    hipStream_t st; bool on;
    ProfileScope(int kind, double flops, double bytes, hipStream_t s) : st(s), on(g_profile_on) {
        if (on) profile_begin(kind, flops, bytes, st);
    }
    ~ProfileScope() { if (on) profile_end(st); }
};

}  // namespace fise

// Optional per-launch timing of the library's heavy kernels with HIP events on the
// caller's stream.  Off by default; when off a launch pays one branch.  Internal.
#pragma once
#include <hip/hip_runtime.h>

namespace fise {

// one kind per kernel family, so that a kind's average can be set against a profiler's per-kernel figure
enum { PROF_IGEMM = 0,          // LDS-direct gathered GEMM, 64x64 tiles
       PROF_IGEMM_GEGLU = 1,    // the same with the GEGLU epilogue (64x128 / 32x256 tiles)
       PROF_ATTENTION = 2,      // active-query attention (without its merge launch)
       PROF_IGEMM_WIDE = 3,     // 128x128 tiles (dense-sized problems)
       PROF_REDUCE = 4,         // split-K reduce + epilogue
       PROF_IGEMM_THIN = 5,     // 32x128 tiles (at most 32 rows)
       PROF_IGEMM_STAGED = 6,   // register-staged gathered GEMM (GroupNorm prologue, 32-wide K steps)
       PROF_ATTENTION_MERGE = 7,
       PROF_EMPTY = 8,          // nothing between the two events: the bracket's own cost
       PROF_IGEMM_WSK = 9,      // wave-split gathered GEMM (per-token products, 32-row tiles, K split inside the workgroup)
       PROF_KINDS = 10 };

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

// Optional per-kernel timing: when switched on, every kernel launch of the library is bracketed by a pair
// of HIP events on the caller's stream; eqat_profile_stop() sums the elapsed times per kernel class.
#pragma once
#include <hip/hip_runtime.h>

namespace eqat {

enum ProfKernel {
    PK_INIT_MINMAX = 0, PK_QUANTIZE, PK_PREPARE, PK_GEMM_FWD, PK_GEMM_DX, PK_GEMM_DW, PK_REDUCE, PK_F32, PK_GEMV, PK_LOSS, PK_UPDATE, PK_COUNT
};

extern bool g_prof_on;
void prof_mark(int kernel, hipStream_t st, bool begin);

struct ProfScope {
    int k; hipStream_t st;
    ProfScope(int kernel, hipStream_t s) : k(kernel), st(s) { if (g_prof_on) prof_mark(k, st, true); }
    ~ProfScope() { if (g_prof_on) prof_mark(k, st, false); }
};

}  // namespace eqat

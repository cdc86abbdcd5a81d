// Optional per-kernel timing: when switched on, every kernel launch of the library is bracketed by a pair
// of HIP events on the caller's stream; eqat_profile_stop() sums the elapsed times per kernel class.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

namespace eqat {

enum ProfKernel {
    PK_INIT_MINMAX = 0, PK_QUANTIZE, PK_PREPARE, PK_GEMM_FWD, PK_GEMM_DX, PK_GEMM_DW, PK_REDUCE, PK_F32, PK_GEMV, PK_LOSS, PK_UPDATE, PK_COUNT
};

extern std::atomic<bool> g_prof_on;
// Takes a pair of events (created on first use, kept for later sessions) and records the first on `st`; -1 when timing is
// off or no event could be made.  prof_end records the second event of pair `rec`.  Safe to call from several threads.
int prof_begin(int kernel, hipStream_t st);
void prof_end(int rec, hipStream_t st);

struct ProfScope {
    int rec; hipStream_t st;
    ProfScope(int kernel, hipStream_t s) : rec(g_prof_on.load(std::memory_order_relaxed) ? prof_begin(kernel, s) : -1), st(s) {}
    ~ProfScope() { if (rec >= 0) prof_end(rec, st); }
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;
};

}  // namespace eqat

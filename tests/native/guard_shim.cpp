// C shim over csrc/lmc_guard.hpp for tests/test_host_guard.py (host logic only).
#include "../../paper_2510_09665_amd/csrc/lmc_guard.hpp"

extern "C" {
void *guard_new() { return new lmc::CopyEngineGuard(); }
void guard_free(void *g) { delete static_cast<lmc::CopyEngineGuard *>(g); }
void guard_observe(void *g, uint64_t bytes, double seconds, double now) {
    static_cast<lmc::CopyEngineGuard *>(g)->observe(bytes, seconds, now);
}
int guard_use_kernel(void *g, double now) { return static_cast<lmc::CopyEngineGuard *>(g)->use_kernel(now) ? 1 : 0; }
double guard_best(void *g) { return static_cast<lmc::CopyEngineGuard *>(g)->best_rate(); }
uint64_t guard_switches(void *g) { return static_cast<lmc::CopyEngineGuard *>(g)->switches(); }
}

// Test-only C shim around csrc/lmc_window.hpp (pure host logic), built by
// tests/test_host_window.py with g++ -fsanitize=undefined and driven from Python
// against the oracle's model.
#include <cstdint>
#include <vector>

#include "../../paper_2510_09665_amd/csrc/lmc_window.hpp"

extern "C" {
void *win_new(int64_t window) { return new lmc::OffloadWindow(window); }
void win_delete(void *w) { delete static_cast<lmc::OffloadWindow *>(w); }
void win_release(void *w, int64_t block) { static_cast<lmc::OffloadWindow *>(w)->release(lmc::FreePage{block, uint64_t(block) * 7}); }
int64_t win_take_scheduled(void *w, int64_t max, int64_t *blocks_out) {
    std::vector<lmc::FreePage> v;
    static_cast<lmc::OffloadWindow *>(w)->take_scheduled(max, &v);
    for (size_t i = 0; i < v.size(); i++) blocks_out[i] = v[i].block;
    return int64_t(v.size());
}
void win_completed(void *w, int64_t n) { static_cast<lmc::OffloadWindow *>(w)->completed(n); }
int win_acquire(void *w, int64_t n, int64_t *blocks_out) {
    std::vector<int64_t> v;
    int r = static_cast<lmc::OffloadWindow *>(w)->acquire(n, &v);
    for (size_t i = 0; i < v.size(); i++) blocks_out[i] = v[i];
    return r;
}
void win_get(void *w, int64_t *out5) {
    auto *p = static_cast<lmc::OffloadWindow *>(w);
    out5[0] = p->start(); out5[1] = p->current(); out5[2] = p->end(); out5[3] = p->tail(); out5[4] = p->state();
}
}

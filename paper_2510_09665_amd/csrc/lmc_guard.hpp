// Watches the rate of the runtime's large device-to-host copies and says when the
// library's own copy kernel should take over for a while.
//
// Why: on the machine this was written on the runtime's device-to-host copies do not keep
// their rate.  For seconds after tens of GiB of device or pinned memory had been freed (by
// this or by the previous process) they ran at 31.5 GB/s instead of 57, on and off; and in a
// mix of stores and retrieves of many requests (32 MiB copies into a fragmented pool beside
// copies the other way) whole stores ran at 12.7 GB/s, one in five, while a copy kernel's
// rate (55 GB/s) did not change.  When healthy, the runtime's copy is the faster one and
// occupies no compute unit, so it stays the first choice.
//
// Policy: remember the best rate a runtime copy has reached.  When two of the last four
// watched copies were below six tenths of it (in the slow state the small copy at the
// head of a store stays fast, so slow ones need not be neighbours), the kernel takes over
// for `hold` seconds; then the runtime is tried again, and if it is slow again at once
// the hold doubles (0.25 s ... 2 s: short, so that a healthy runtime is back in use soon
// after a false alarm or the end of an episode); four healthy copies in a row reset it.
// Plain C++, no HIP: times and rates are passed in.
#pragma once

#include <algorithm>
#include <cstdint>

namespace lmc {

class CopyEngineGuard {
public:
    static constexpr uint64_t kMinBytes = uint64_t(32) << 20;  // smaller copies are latency, not rate
    static constexpr double kMinHold = 0.25, kMaxHold = 2.0;   // seconds on the kernel before the runtime is tried again
    // A copy below this share of the best rate seen counts as slow.  The slow states measured
    // are at 0.55 (31.5 GB/s) and 0.22 (12.7 GB/s) of the link; a healthy copy that shares the
    // link with a transfer the other way still makes 0.8-0.9.
    static constexpr double kSlow = 0.6;

    // A runtime copy of `bytes` that took `seconds` has been seen finished at time `now` (s).
    void observe(uint64_t bytes, double seconds, double now) {
        if (bytes < kMinBytes || seconds <= 0.0) return;
        const double rate = double(bytes) / seconds;
        last_ = rate;
        if (rate > best_) best_ = rate;
        history_ = ((history_ << 1) | (rate < kSlow * best_ ? 1u : 0u)) & 0xFu;
        if (__builtin_popcount(history_) >= 2) {
            kernel_until_ = now + hold_;
            hold_ = std::min(hold_ * 2.0, kMaxHold);
            history_ = 0;
            switches_++;
        } else if (history_ == 0 && ++healthy_in_row_ >= 4) {
            hold_ = kMinHold;
        }
        if (history_ != 0) healthy_in_row_ = 0;
    }
    // Should a copy enqueued at time `now` be made by the kernel?
    bool use_kernel(double now) const { return now < kernel_until_; }
    double best_rate() const { return best_; }
    double last_rate() const { return last_; }
    uint64_t switches() const { return switches_; }

private:
    double best_ = 0.0, last_ = 0.0, hold_ = kMinHold, kernel_until_ = -1.0;
    unsigned history_ = 0;     // the last four watched copies, one bit each: 1 = slow
    int healthy_in_row_ = 0;
    uint64_t switches_ = 0;
};

}  // namespace lmc

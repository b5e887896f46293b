// The three-pointer window of dynamic offloading (paper section 5.3): the engine's free
// pages form a queue; only a window of them is duplicated to CPU memory.  start = head
// of the free region, current = pages before it are offloaded, end = pages before it
// are scheduled.  Positions are absolute counts of pages that ever entered the free
// region, so every pointer only moves right.  Pure host logic, no HIP.
#pragma once

#include <algorithm>
#include <cstdint>
#include <deque>
#include <vector>

namespace lmc {

struct FreePage {
    int64_t block;   // the engine's block number
    uint64_t id;     // the id under which the block's KV is cached
};

class OffloadWindow {
public:
    explicit OffloadWindow(int64_t window) : window_(window) {}

    int64_t start() const { return start_; }
    int64_t current() const { return current_; }
    int64_t issued() const { return issued_; }
    int64_t end() const { return end_; }
    int64_t tail() const { return start_ + int64_t(q_.size()); }
    // the section's state numbers: 1 initialization, 2 in progress, 4 steady; state 3
    // ("query arrival") is the pointer move made by acquire()
    int state() const { return current_ == end_ ? 4 : (current_ == start_ ? 1 : 2); }

    // The engine frees a page: it joins the tail, and the end pointer follows the tail
    // until the window is full.
    void release(FreePage p) {
        q_.push_back(p);
        if (end_ - start_ < window_) end_ = std::min(start_ + window_, tail());
    }

    // Pages scheduled but not yet handed to the store, at most max of them; they count
    // as issued from now on.
    void take_scheduled(int64_t max, std::vector<FreePage> *out) {
        const int64_t n = std::min(max, end_ - issued_);
        for (int64_t i = 0; i < n; i++) out->push_back(q_[size_t(issued_ - start_ + i)]);
        issued_ += std::max<int64_t>(n, 0);
    }

    // n more issued pages have reached CPU memory.
    void completed(int64_t n) { current_ = std::min(current_ + n, issued_); }

    // A query asks for n free pages.  0: granted (blocks appended to out; end moves
    // forward by n: state 3).  1: stall, every requested page must lie before the current
    // pointer; a request larger than the window pulls the end pointer to start + n.
    // 2: there are not n free pages at all.
    int acquire(int64_t n, std::vector<int64_t> *out) {
        if (n > tail() - start_) return 2;
        if (n > current_ - start_) {
            end_ = std::max(end_, std::min(start_ + n, tail()));
            return 1;
        }
        for (int64_t i = 0; i < n; i++) {
            out->push_back(q_.front().block);
            q_.pop_front();
        }
        start_ += n;
        end_ = std::min(end_ + n, tail());
        return 0;
    }

private:
    int64_t window_;
    int64_t start_ = 0, current_ = 0, issued_ = 0, end_ = 0;
    std::deque<FreePage> q_;   // pages at positions start_ .. tail()-1
};

}  // namespace lmc

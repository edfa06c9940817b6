// Issue pacing of chunk commands (host logic only; the caller supplies the clock).
//
// Commands that are queued back to back share the host link, finish together and leave it idle while all of
// them are issued again (512 KiB commands at depth 3: 45 of 56.5 GB/s).  Spaced by one command's own link time
// they stay staggered: one completes while the others still move, and its successor is on its way before they
// end (54 GB/s).  The spacing has to be right within a few percent (0.97 of the link time gives 52 GB/s, 1.06
// gives 52.5, 0.85 gives 47), so it is the previous command's bytes over a measured link rate with 2 % of
// headroom.  The rate only ratchets upward, from what runs sustain over windows of several queue depths between
// completions the issuing thread really waited for (only those have an exact time); a window's rate carries a
// percent or two of timing noise, so the rate moves only after three windows in a row came out above it, and then
// to the lowest of the three.  Without a measured rate nothing is paced: a rate taken from a run's own first
// windows could be a stalled one and would hold everything back.
#pragma once

#include <algorithm>
#include <cstddef>
#include <cstdint>

namespace kvb {

// What outlives a call: the link rate of one direction (bytes per second, 0 = not measured) and the ratchet's state.
struct LinkRate {
    double rate = 0.0;
    int above = 0;     // consecutive windows that ran above `rate`
    double low = 0.0;  // the lowest of them
};

class IssuePacer {
public:
    static constexpr double kHeadroom = 1.02;

    // catch_up: the factor on the spacing while two or more queue slots are free (1 = none).
    IssuePacer(LinkRate *link, bool enabled, int depth, double catch_up = 0.5)
        : link_(link), on_(enabled && depth >= 2 && link->rate > 0.0), depth_((size_t)std::max(depth, 1)),
          window_(std::max<size_t>(16, 8 * (size_t)depth)), catch_up_(catch_up)
    {
    }
    bool enabled() const { return on_; }
    // Earliest time at which the next command may be queued (a time in the past: no wait), with `in_flight` commands
    // outstanding.  One free slot is the steady state (a command has just completed): the spacing is the previous
    // command's link time.  Two or more free slots mean the queue has fallen behind (a stall on the host, the start
    // of a call): at the link's own rate it would never fill up again, so the spacing is multiplied by `catch_up`
    // until one slot is left.  Half the spacing pays for hipMemcpyAsync commands of a MiB and more (2 MiB commands:
    // 55.7 against 54.3 GB/s out, 8 MiB: 56.9 against 55.6 in); commands moved by the copy kernel catch up at no more
    // than the link's rate (factor 1), since two of them queued half a spacing apart share the link, finish together
    // and free two slots again, which repeats the pair for the rest of the call (512 KiB commands out: 47.4 GB/s
    // with the half spacing, 48.7 without).
    double due(size_t in_flight) const
    {
        if (!on_ || last_issue_ < 0.0) return -1.0;
        const double tau = last_bytes_ / (kHeadroom * link_->rate);
        return last_issue_ + (in_flight + 2 <= depth_ ? catch_up_ * tau : tau);
    }
    // A command of `bytes` is being queued at time `now`.
    void issued(double now, uint64_t bytes)
    {
        last_issue_ = now;
        last_bytes_ = (double)bytes;
    }
    // The completion of a command of `bytes` was harvested at time `now`; waited = the thread had to wait for it.
    void harvested(double now, uint64_t bytes, bool waited)
    {
        if (!on_) return;
        if (win_t0_ >= 0.0) { win_bytes_ += (double)bytes; ++win_n_; }
        if (!waited) return;
        if (win_t0_ >= 0.0 && win_n_ >= window_ && now > win_t0_) {
            const double seen = win_bytes_ / (now - win_t0_);
            if (seen > link_->rate) {
                link_->low = link_->above == 0 ? seen : std::min(link_->low, seen);
                if (++link_->above >= 3) { link_->rate = link_->low; link_->above = 0; }
            } else {
                link_->above = 0;
            }
            win_t0_ = -1.0;
        }
        if (win_t0_ < 0.0) { win_t0_ = now; win_bytes_ = 0.0; win_n_ = 0; }
    }

private:
    LinkRate *link_;
    bool on_;
    size_t depth_, window_;
    double last_issue_ = -1.0, last_bytes_ = 0.0;
    double win_t0_ = -1.0, win_bytes_ = 0.0;
    size_t win_n_ = 0;
    double catch_up_;
};

}  // namespace kvb

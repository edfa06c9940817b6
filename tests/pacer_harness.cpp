// Drives the issue pacer (paper_2604_26557_amd/csrc/pacer.hpp) with a synthetic clock and prints what it decides;
// compiled and run by tests/test_pacer_cpu.py.
#include <cstdio>
#include <cstdlib>

#include "pacer.hpp"

int main(int argc, char **argv)
{
    const double rate0 = argc > 1 ? atof(argv[1]) : 50e9;     // measured link rate, bytes per second
    const int depth = argc > 2 ? atoi(argv[2]) : 3;
    const double true_rate = argc > 3 ? atof(argv[3]) : 56e9; // what the link really sustains
    const uint64_t bytes = 512 * 1024;
    kvb::LinkRate link;
    link.rate = rate0;
    kvb::IssuePacer p(&link, true, depth);
    printf("enabled %d\n", (int)p.enabled());
    // first command: nothing to wait for
    printf("due_first %.13f\n", p.due(0));
    p.issued(1.0, bytes);
    printf("due_second %.13f\n", p.due(depth - 1));
    p.issued(p.due(depth - 1), 2 * bytes);
    printf("due_third %.13f\n", p.due(depth - 1));
    printf("due_third_behind %.13f\n", p.due(depth >= 2 ? depth - 2 : 0));
    {   // the same two commands with no catch-up (factor 1): two free slots do not shorten the spacing
        kvb::IssuePacer pk(&link, true, depth, 1.0);
        pk.issued(1.0, bytes);
        pk.issued(pk.due(depth - 1), 2 * bytes);
        printf("due_third_behind_no_catch_up %.13f\n", pk.due(depth >= 2 ? depth - 2 : 0));
    }
    // a link that sustains true_rate: completions the thread waited for arrive every bytes / true_rate
    double t = 2.0;
    for (int w = 0; w < 12; ++w) {
        const size_t n = 8 * (size_t)depth < 16 ? 16 : 8 * (size_t)depth;
        for (size_t i = 0; i < n + 1; ++i) {
            t += (double)bytes / true_rate;
            p.harvested(t, bytes, true);
        }
        printf("rate_after_window %d %.6e above %d\n", w, link.rate, link.above);
    }
    // completions noticed late in a burst (not waited for) must not end a window
    kvb::LinkRate l2;
    l2.rate = 10e9;
    kvb::IssuePacer p2(&l2, true, depth);
    t = 5.0;
    p2.harvested(t, bytes, true);
    for (int i = 0; i < 200; ++i) p2.harvested(t + 1e-9 * i, bytes, false);
    printf("rate_unwaited %.6e\n", l2.rate);
    // no measured rate, depth 1, or switched off: not paced
    kvb::LinkRate l3;
    printf("enabled_no_rate %d\n", (int)kvb::IssuePacer(&l3, true, depth).enabled());
    printf("enabled_depth1 %d\n", (int)kvb::IssuePacer(&link, true, 1).enabled());
    printf("enabled_off %d\n", (int)kvb::IssuePacer(&link, false, depth).enabled());
    return 0;
}

// Exercises the memcpy-hop worker pool (paper_2604_26557_amd/csrc/workers.hpp) the way the pipeline does: commands cut
// into pieces, pushed under one lock, counted down on the command's own counter while the pushing thread polls it.
// Built with -fsanitize=thread and run by tests/test_workers_cpu.py; prints "ok" when every byte arrived.
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "workers.hpp"

static int run_round(kvb::Workers &w, int n_cmds, size_t cmd_bytes, int ring, bool nap)
{
    std::vector<unsigned char> src((size_t)n_cmds * cmd_bytes), dst(src.size(), 0);
    for (size_t i = 0; i < src.size(); ++i) src[i] = (unsigned char)(i * 131 + 7);
    std::vector<std::atomic<int>> pending((size_t)ring);
    for (auto &p : pending) p.store(0);
    const int pieces_max = std::max(1, w.size());
    for (int c = 0; c < n_cmds; ++c) {
        std::atomic<int> &p = pending[(size_t)c % (size_t)ring];
        while (p.load(std::memory_order_acquire) != 0) std::this_thread::yield();   // the ring entry's last command is done
        if (nap && c % 7 == 0) std::this_thread::sleep_for(std::chrono::milliseconds(2));   // let the threads fall asleep
        const int pieces = (int)std::min<size_t>((size_t)pieces_max, std::max<size_t>(1, cmd_bytes / 4096));
        const size_t step = (cmd_bytes + (size_t)pieces - 1) / (size_t)pieces;
        kvb::CopyTask tasks[64];
        int n = 0;
        size_t off = 0;
        p.store(pieces, std::memory_order_release);
        for (int i = 0; i < pieces; ++i) {
            const size_t len = off < cmd_bytes ? std::min(step, cmd_bytes - off) : 0;
            if (len == 0) { p.fetch_sub(1, std::memory_order_release); continue; }
            tasks[n++] = kvb::CopyTask{dst.data() + (size_t)c * cmd_bytes + off, src.data() + (size_t)c * cmd_bytes + off, len, &p};
            off += len;
        }
        w.push(tasks, n);
    }
    for (auto &p : pending)
        while (p.load(std::memory_order_acquire) != 0) std::this_thread::yield();
    return std::memcmp(src.data(), dst.data(), src.size()) == 0 ? 0 : 1;
}

int main()
{
    int bad = 0;
    {
        kvb::Workers w;
        w.start(4);
        bad += run_round(w, 200, 64 * 1024, 6, false);
        bad += run_round(w, 40, 10000, 2, true);        // odd sizes, threads asleep between commands
        w.start(4);                                       // same size: no restart
        w.start(8);                                       // restart with more threads
        bad += run_round(w, 200, 300 * 1024, 4, false);
        w.start(1);
        bad += run_round(w, 50, 4096, 3, true);
        w.stop();
        w.stop();                                         // idempotent
        w.start(2);
        bad += run_round(w, 20, 1, 2, false);             // one-byte commands
    }                                                     // destructor stops the pool
    { kvb::Workers idle; idle.start(3); }                 // started, never used
    { kvb::Workers never; }                               // never started
    printf(bad ? "mismatch\n" : "ok\n");
    return bad;
}

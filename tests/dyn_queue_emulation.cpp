// CPU emulation of the dynamic scheduler's ready-queue protocol (paper Sec. 3.2, App. A), one std::thread
// per persistent workgroup, std::atomic in place of device-scope atomics.  Mirrors the device code's
// protocol: tickets from an atomic head, slots published as (epoch << 32 | task id + 1) after an atomic
// reservation on tail, push when a notify brings an event to zero, `done` set by whoever completes the
// last task.  Run on the row-sum graph (4n producers, n consumers) for three consecutive launches
// (epochs) without clearing the slots.  Exit code 0 iff every task ran once and every counter drained.
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>
struct Task { int wait0, notify0, id; };
int main(int argc, char** argv) {
    int n = argc > 1 ? atoi(argv[1]) : 1, NWG = argc > 2 ? atoi(argv[2]) : 64;
    // rowsum graph: 4n partial tasks (notify E[i]) then n final tasks (wait E[i])
    std::vector<Task> tasks;
    for (int i = 0; i < n; ++i) for (int j = 0; j < 4; ++j) tasks.push_back({-1, i, (int)tasks.size()});
    for (int i = 0; i < n; ++i) tasks.push_back({i, -1, (int)tasks.size()});
    std::vector<std::atomic<int>> ev(n); for (auto& e : ev) e = 4;
    std::vector<std::vector<int>> cons(n); std::vector<int> seeds;
    for (auto& t : tasks) if (t.wait0 < 0) seeds.push_back(t.id); else cons[t.wait0].push_back(t.id);
    const int cap = (int)tasks.size() + NWG + 16;
    for (uint32_t epoch = 1; epoch <= 3; ++epoch) {
        for (auto& e : ev) e = 4;
        std::vector<std::atomic<uint64_t>> slots(cap); for (auto& s : slots) s = (uint64_t)(epoch - 1) << 32;
        std::atomic<int> head{0}, tail{0}, done{0}, ndone{0};
        std::vector<std::atomic<int>> exec(tasks.size()); for (auto& e : exec) e = 0;
        auto push = [&](const int* ids, int cnt) { int base = tail.fetch_add(cnt); for (int i = 0; i < cnt; ++i) slots[base + i].store(((uint64_t)epoch << 32) | (uint32_t)(ids[i] + 1), std::memory_order_release); };
        std::vector<std::thread> th;
        std::atomic<int> timeouts{0};
        for (int wg = 0; wg < NWG; ++wg) th.emplace_back([&, wg] {
            for (int i = wg; i < (int)seeds.size(); i += NWG) push(&seeds[i], 1);
            for (;;) {
                int id = -1; int ticket = head.fetch_add(1);
                if (ticket < cap) { long spins = 0; for (;;) { uint64_t v = slots[ticket].load(std::memory_order_acquire); if ((uint32_t)(v >> 32) == epoch) { id = (int)(uint32_t)v - 1; break; } if (done.load()) break; std::this_thread::yield(); if (++spins > 20000000) { timeouts++; break; } } }
                if (id < 0) break;
                const Task& t = tasks[id];
                if (t.wait0 >= 0) while (ev[t.wait0].load() > 0) std::this_thread::yield();
                exec[id]++;
                if (t.notify0 >= 0) { if (ev[t.notify0].fetch_sub(1) == 1) push(cons[t.notify0].data(), (int)cons[t.notify0].size()); }
                int nd = ndone.fetch_add(1) + 1;
                if (nd == (int)tasks.size()) done.store(1, std::memory_order_release);
            }
        });
        for (auto& t : th) t.join();
        bool ok = timeouts == 0; for (auto& e : exec) ok = ok && e == 1; for (auto& e : ev) ok = ok && e == 0;
        printf("n=%d wgs=%d epoch=%u: %s (timeouts %d, head %d, tail %d)\n", n, NWG, epoch, ok ? "ok" : "FAIL", timeouts.load(), head.load(), tail.load());
        if (!ok) return 1;
    }
}

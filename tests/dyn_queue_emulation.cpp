// CPU emulation of the dynamic scheduler's ready-queue protocol (paper Sec. 3.2, App. A, App. E), one
// std::thread per persistent workgroup, std::atomic in place of device-scope atomics.  Mirrors the device
// code's protocol: tickets from an atomic head, slots published as (epoch << 32 | task id + 1) after an
// atomic reservation on tail, early push (a second counter per event counts producers not yet dispatched;
// the workgroup that brings it to zero pushes the consumers whose other events are that far too, a
// per-task counter that is never reset deciding which of a task's events is the last), waits kept by the
// pushed task, poppers of an empty queue leaving once the count of
// completed tasks reaches the number of tasks.  Graph: the row-sum example (4n producers
// notify E[i], n consumers wait on E[i]) plus one closing task that waits on two events (F, notified by the
// n consumers, and E[0]).  Three consecutive launches (epochs) without clearing the slots or the per-task
// counters.  Exit code 0 iff every task ran once, was pushed once, and every counter drained.
// The dispatch loop carries the device loop's own bound: more iterations than the step has tasks record an
// error, the workgroup leaves, and every wait of the others gives up on seeing the error.  With the
// environment variable STALE_WG=<w> workgroup w's pop keeps returning the id it already has (the planted
// defect: a loop that repeats its task); the run must then END, with exit code 3 (drained on the loop bound).
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>
struct Task { int wait0, wait1, notify0, id; };
// Data-dependent edges (Sec. 2.4) on the ready queue: producer (i, j), j < 4, notifies event route[i]; an event's
// count (4 x the row blocks routed to it) is known at run time only, so notifies count down from zero and the
// one that completes the count fires the event, puts the counter back and releases the consumer tasks
// [indptr[e], indptr[e+1]); the consumer grid has `surplus` tasks beyond the last range, credited as completed
// at the start and never run.
static int run_data_dependent(int n, int NWG, int m, int surplus) {
    std::vector<int> route(n), cnt(m, 0), indptr(m + 1, 0);
    unsigned seed = 12345u + (unsigned)n * 7u + (unsigned)m;
    for (int i = 0; i < n; ++i) { seed = seed * 1664525u + 1013904223u; route[i] = (int)((seed >> 16) % (unsigned)m); cnt[route[i]] += 4; }
    for (int e = 0; e < m; ++e) indptr[e + 1] = indptr[e] + cnt[e] / 4;
    const int n_prod = 4 * n, n_cons = n + surplus, total = n_prod + n_cons, cap = total + NWG + 16;
    std::vector<std::atomic<uint64_t>> slots(cap); for (auto& s : slots) s = 0;
    std::vector<std::atomic<int>> ev(m); for (auto& e : ev) e = 0;
    for (uint32_t epoch = 1; epoch <= 3; ++epoch) {
        std::atomic<int> head{0}, tail{0}, ndone{surplus}, timeouts{0};
        std::vector<std::atomic<int>> exec(total); for (auto& e : exec) e = 0;
        auto publish = [&](int base, int id) { slots[base].store(((uint64_t)epoch << 32) | (uint32_t)(id + 1), std::memory_order_release); };
        std::vector<std::thread> th;
        for (int wg = 0; wg < NWG; ++wg) th.emplace_back([&, wg] {
            for (int i = wg; i < n_prod; i += NWG) publish(tail.fetch_add(1), i);          // producers wait on nothing: seeds
            auto wait_slot = [&](int ticket) {
                if (ticket >= cap) return -1;
                long spins = 0;
                for (;;) {
                    uint64_t v = slots[ticket].load(std::memory_order_acquire);
                    if ((uint32_t)(v >> 32) == epoch) return (int)(uint32_t)v - 1;
                    if (ndone.load() >= total) return -1;
                    std::this_thread::yield();
                    if (++spins > 20000000) { timeouts++; return -1; }
                }
            };
            int id = wait_slot(head.fetch_add(1));
            while (id >= 0) {
                exec[id]++;
                if (id < n_prod) {
                    const int e = route[id / 4];
                    if (ev[e].fetch_sub(1) - 1 == -cnt[e]) {
                        ev[e].store(0);
                        const int j0 = indptr[e], k = indptr[e + 1] - j0, base = tail.fetch_add(k);
                        for (int i = 0; i < k; ++i) publish(base + i, n_prod + j0 + i);
                    }
                }
                ndone.fetch_add(1);
                id = wait_slot(head.fetch_add(1));
            }
        });
        for (auto& t : th) t.join();
        bool ok = timeouts == 0;
        for (int i = 0; i < total; ++i) ok = ok && exec[i] == (i < n_prod + n ? 1 : 0);
        for (auto& e : ev) ok = ok && e == 0;
        printf("data-dependent n=%d groups=%d wgs=%d epoch=%u: %s\n", n, m, NWG, epoch, ok ? "ok" : "FAIL");
        if (!ok) return 1;
    }
    return 0;
}

int main(int argc, char** argv) {
    int n = argc > 1 ? atoi(argv[1]) : 1, NWG = argc > 2 ? atoi(argv[2]) : 64;
    if (argc > 3) return run_data_dependent(n, NWG, atoi(argv[3]), argc > 4 ? atoi(argv[4]) : 0);
    std::vector<Task> tasks;
    const int F = n;                                   // event ids: E[0..n), F
    for (int i = 0; i < n; ++i) for (int j = 0; j < 4; ++j) tasks.push_back({-1, -1, i, (int)tasks.size()});
    for (int i = 0; i < n; ++i) tasks.push_back({i, -1, F, (int)tasks.size()});
    tasks.push_back({F, 0, -1, (int)tasks.size()});
    const int n_ev = n + 1;
    std::vector<int> init(n_ev, 0);
    for (auto& t : tasks) if (t.notify0 >= 0) init[t.notify0]++;
    struct Entry { int id, n_waited; };
    std::vector<std::vector<Entry>> cons(n_ev); std::vector<int> seeds;
    for (auto& t : tasks) {
        int w[2], k = 0;
        if (t.wait0 >= 0) w[k++] = t.wait0;
        if (t.wait1 >= 0 && t.wait1 != t.wait0) w[k++] = t.wait1;
        if (k == 0) seeds.push_back(t.id);
        for (int j = 0; j < k; ++j) cons[w[j]].push_back({t.id, k});
    }
    const int cap = (int)tasks.size() + NWG + 16;
    std::vector<std::atomic<uint64_t>> slots(cap); for (auto& s : slots) s = 0;
    std::vector<std::atomic<int>> pending(tasks.size()); for (auto& p : pending) p = 0;
    const int stale_wg = getenv("STALE_WG") ? atoi(getenv("STALE_WG")) : -1;
    std::atomic<int> error_word{0};                    // 6 = loop bound, as on the device
    for (uint32_t epoch = 1; epoch <= 3; ++epoch) {
        std::vector<std::atomic<int>> ev(n_ev), disp(n_ev);
        for (int e = 0; e < n_ev; ++e) { ev[e] = init[e]; disp[e] = init[e]; }
        std::atomic<int> head{0}, tail{0}, ndone{0};
        std::vector<std::atomic<int>> exec(tasks.size()), pushed(tasks.size());
        for (auto& e : exec) e = 0; for (auto& e : pushed) e = 0;
        auto push1 = [&](int id) { int base = tail.fetch_add(1); pushed[id]++; slots[base].store(((uint64_t)epoch << 32) | (uint32_t)(id + 1), std::memory_order_release); };
        std::vector<std::thread> th;
        std::atomic<int> timeouts{0};
        for (int wg = 0; wg < NWG; ++wg) th.emplace_back([&, wg] {
            for (int i = wg; i < (int)seeds.size(); i += NWG) push1(seeds[i]);
            auto wait_slot = [&](int ticket) {
                if (ticket >= cap) return -1;
                long spins = 0;
                for (;;) {
                    uint64_t v = slots[ticket].load(std::memory_order_acquire);
                    if ((uint32_t)(v >> 32) == epoch) return (int)(uint32_t)v - 1;
                    if (ndone.load() >= (int)tasks.size()) return -1;
                    if (error_word.load() != 0) return -1;
                    std::this_thread::yield();
                    if (++spins > 20000000) { timeouts++; return -1; }
                }
            };
            int id = wait_slot(head.fetch_add(1));
            int iterations = 0;
            while (id >= 0) {
                if (++iterations > (int)tasks.size() + 1) { int z = 0; error_word.compare_exchange_strong(z, 6); break; }
                const Task& t = tasks[id];
                const bool last = t.notify0 >= 0 && disp[t.notify0].fetch_sub(1) == 1;   // dispatched: early push
                if (last)
                    for (const Entry& c : cons[t.notify0])
                        if (c.n_waited == 1 || (pending[c.id].fetch_add(1) + 1) % c.n_waited == 0) push1(c.id);
                long spins = 0;
                for (int w : {t.wait0, t.wait1})
                    if (w >= 0) while (ev[w].load() > 0 && error_word.load() == 0) { std::this_thread::yield(); if (++spins > 20000000) { timeouts++; break; } }
                exec[id]++;
                if (t.notify0 >= 0) ev[t.notify0].fetch_sub(1);
                ndone.fetch_add(1);
                if (wg != stale_wg) id = wait_slot(head.fetch_add(1));
            }
        });
        for (auto& t : th) t.join();
        if (error_word.load() == 6) { printf("n=%d wgs=%d epoch=%u: drained on the loop bound\n", n, NWG, epoch); return 3; }
        bool ok = timeouts == 0;
        for (auto& e : exec) ok = ok && e == 1; for (auto& e : pushed) ok = ok && e == 1;
        for (auto& e : ev) ok = ok && e == 0; for (auto& e : disp) ok = ok && e == 0;
        printf("n=%d wgs=%d epoch=%u: %s (timeouts %d, head %d, tail %d)\n", n, NWG, epoch, ok ? "ok" : "FAIL", timeouts.load(), head.load(), tail.load());
        if (!ok) return 1;
    }
}

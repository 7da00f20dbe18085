// Host-only exercise of the staging-slot pool: many threads acquire, fill, "enqueue" and release
// slots against fake events that a background thread completes later.  Checks the two properties
// the search entry points rely on:
//   1. a slot is never held by two calls at once (the fill pattern survives until release);
//   2. a slot is never handed out while the work recorded behind its last use is still pending.
// Prints "ok <acquisitions> <waits>" and exits 0, or prints the violated property and exits 1.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "st_stage_pool.h"

namespace {

struct FakeEvent {
    std::atomic<int> pending{0};    // 1 from record() until the "device" completes it
    std::atomic<long> complete_at{0};
};

std::atomic<long> g_clock{0};
std::atomic<bool> g_stop{false};
std::atomic<long> g_waits{0};
FakeEvent g_events[st::kStageSlots];

bool is_done(void* e)
{
    return static_cast<FakeEvent*>(e)->pending.load(std::memory_order_acquire) == 0;
}

int wait_for(void* e)
{
    g_waits.fetch_add(1);
    while (!is_done(e)) std::this_thread::yield();
    return 0;
}

void device_thread()
{
    while (!g_stop.load()) {
        const long now = g_clock.fetch_add(1) + 1;
        for (FakeEvent& ev : g_events)
            if (ev.pending.load(std::memory_order_acquire) && ev.complete_at.load() <= now)
                ev.pending.store(0, std::memory_order_release);
        std::this_thread::yield();
    }
    for (FakeEvent& ev : g_events) ev.pending.store(0, std::memory_order_release);
}

}  // namespace

int main(int argc, char** argv)
{
    const int n_threads = argc > 1 ? atoi(argv[1]) : 12;
    const int n_iter = argc > 2 ? atoi(argv[2]) : 4000;
    constexpr size_t kBytes = 256;
    st::StagePool pool;
    std::vector<std::vector<unsigned char>> mem(st::kStageSlots, std::vector<unsigned char>(kBytes));
    std::atomic<int> holder[st::kStageSlots];
    for (int i = 0; i < st::kStageSlots; ++i) {
        st::StageSlot& s = pool.slots()[i];
        s.host = mem[i].data();
        s.dev_view = s.host;
        s.bytes = kBytes;
        s.event = &g_events[i];
        holder[i].store(-1);
    }
    std::atomic<int> failed{0};
    std::atomic<long> acquisitions{0};
    std::thread dev(device_thread);
    std::vector<std::thread> workers;
    for (int t = 0; t < n_threads; ++t) {
        workers.emplace_back([&, t] {
            unsigned rng = 12345u + 977u * (unsigned)t;
            for (int it = 0; it < n_iter && !failed.load(); ++it) {
                st::StageSlot* s = nullptr;
                if (pool.acquire(is_done, wait_for, &s) != 0 || !s) {
                    failed.store(3);
                    return;
                }
                const int idx = (int)(s - pool.slots());
                FakeEvent* ev = static_cast<FakeEvent*>(s->event);
                if (ev->pending.load(std::memory_order_acquire)) failed.store(2);  // property 2
                int expect = -1;
                if (!holder[idx].compare_exchange_strong(expect, t)) failed.store(1);  // property 1
                memset(s->host, t + 1, kBytes);
                rng = rng * 1664525u + 1013904223u;
                for (unsigned spin = 0; spin < (rng >> 24); ++spin) std::this_thread::yield();
                const unsigned char* p = static_cast<const unsigned char*>(s->host);
                for (size_t b = 0; b < kBytes; ++b)
                    if (p[b] != (unsigned char)(t + 1)) failed.store(1);
                holder[idx].store(-1);
                acquisitions.fetch_add(1);
                const bool enqueue = (rng >> 8) % 8 != 0;  // one call in eight fails before it enqueues
                if (enqueue) {
                    ev->complete_at.store(g_clock.load() + 1 + (long)((rng >> 12) % 64));
                    ev->pending.store(1, std::memory_order_release);
                }
                pool.release(s, enqueue);
            }
        });
    }
    for (std::thread& w : workers) w.join();
    g_stop.store(true);
    dev.join();
    if (failed.load()) {
        printf("violated property %d\n", failed.load());
        return 1;
    }
    printf("ok %ld %ld\n", acquisitions.load(), g_waits.load());
    return 0;
}

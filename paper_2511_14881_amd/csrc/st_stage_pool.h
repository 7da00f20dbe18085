// Pool of pinned staging slots for the per-call table uploads of the search entry points.
//
// A call fills a slot with its tables on the host, enqueues the copy (or a kernel that reads the
// slot directly) on its stream and records an event behind it.  A slot therefore goes through
// three states:
//   free      nobody uses it; if `pending`, the event recorded behind its last use may not have
//             completed yet and has to be waited for before the memory is written again
//   owned     handed to exactly one call, from acquire() until release(): the call writes the
//             host memory and enqueues the work that reads it
// Ownership is what keeps two concurrent calls from filling one slot: acquire() never hands out
// an owned slot, whatever the number of threads, and release() is the only way back.
//
// The pool knows nothing of HIP: waiting for and recording an event are callbacks, so the same
// code runs against fake events in a host-only test.
#pragma once
#include <stddef.h>

#include <mutex>
#include <thread>

namespace st {

constexpr int kStageSlots = 16;

struct StageSlot {
    void* host = nullptr;      // pinned host memory (owner: the pool's user)
    void* dev_view = nullptr;  // the same memory as the device addresses it
    size_t bytes = 0;
    void* event = nullptr;     // opaque event handle (owner: the pool's user)
    bool pending = false;      // the event has been recorded and not yet found complete
    bool owned = false;
};

class StagePool {
public:
    // is_done(event): true once the work recorded behind the slot's last use has completed.
    // wait(event): blocks until then; returns 0 or an error code that acquire() passes on.
    typedef bool (*DoneFn)(void* event);
    typedef int (*WaitFn)(void* event);

    // Hands out a slot nobody else holds.  Prefers one whose previous use has completed; else
    // takes the oldest pending one and waits for it (outside the lock: the slot is already
    // owned by the caller then); if every slot is owned by some other call it yields and retries.
    int acquire(DoneFn is_done, WaitFn wait, StageSlot** out)
    {
        for (;;) {
            StageSlot* pick = nullptr;
            bool must_wait = false;
            {
                std::lock_guard<std::mutex> lock(mu_);
                StageSlot* fallback = nullptr;
                for (int i = 0; i < kStageSlots && !pick; ++i) {
                    StageSlot& s = slot_[(next_ + i) % kStageSlots];
                    if (s.owned) continue;
                    if (!s.pending || is_done(s.event)) {
                        s.pending = false;
                        pick = &s;
                        next_ = (next_ + i + 1) % kStageSlots;
                    } else if (!fallback) {
                        fallback = &s;  // scanning starts at the oldest hand-out
                    }
                }
                if (!pick && fallback) {
                    pick = fallback;
                    must_wait = true;
                    next_ = (int)((fallback - slot_) + 1) % kStageSlots;
                }
                if (pick) pick->owned = true;
            }
            if (!pick) {
                std::this_thread::yield();
                continue;
            }
            if (must_wait) {
                const int rc = wait(pick->event);
                if (rc != 0) {
                    release(pick, false);
                    return rc;
                }
                pick->pending = false;  // owned: no other thread reads or writes the slot's fields
            }
            *out = pick;
            return 0;
        }
    }

    // Gives the slot back.  recorded = the caller has recorded the slot's event behind the work
    // that reads the slot (false: nothing was enqueued, the memory may be reused at once).
    void release(StageSlot* s, bool recorded)
    {
        std::lock_guard<std::mutex> lock(mu_);
        s->pending = recorded;
        s->owned = false;
    }

    StageSlot* slots() { return slot_; }

private:
    std::mutex mu_;
    StageSlot slot_[kStageSlots];
    int next_ = 0;
};

}  // namespace st

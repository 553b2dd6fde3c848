// counter_slots.h -- who may use which set of device counters (host-side bookkeeping, no HIP).
//
// Persistent SYRK launches take their blocks through a pair of counters in device memory, and
// launches whose blocks are cut along the contraction dimension count the finished parts of every
// block in a second array.  A set of counters must never serve two launches that can run at the same
// time.  The rule, safe by construction:
//   1. launches on one stream run one after the other, so a stream keeps the slot it was given;
//   2. a stream without a slot takes one that was never used;
//   3. failing that, the least recently used slot whose last launch is known to have finished
//      (`idle(slot)`: the caller asks the event that completes with that launch);
//   4. failing that, none: the caller launches the form that needs no counters (one workgroup per
//      block, no cut blocks).
// The owner of a slot is identified by the stream handle and, for the per-thread default stream (one
// handle that names a different stream in every host thread), the calling thread.
#pragma once
#include <stdint.h>

namespace tbs {

constexpr int kCounterSlots = 64;

struct SlotOwner {
    const void* stream = nullptr;
    uint64_t thread = 0;      // 0 unless the handle means a different stream per thread
    bool operator==(const SlotOwner& o) const { return stream == o.stream && thread == o.thread; }
};

class SlotTable {
public:
    // The slot the owner's next launch may use, or -1.  `idle(s)` is only asked about slots that
    // have been used by another owner; it must return true only if every launch that used slot s has
    // finished.  Not thread-safe: the caller serialises.
    template <class Idle>
    int acquire(const SlotOwner& who, Idle&& idle)
    {
        ++clock_;
        for (int s = 0; s < kCounterSlots; ++s)
            if (used_[s] && owner_[s] == who) return touch(s);
        for (int s = 0; s < kCounterSlots; ++s)
            if (!used_[s]) {
                used_[s] = true;
                owner_[s] = who;
                return touch(s);
            }
        // candidates in order of their last use, oldest first
        bool tried[kCounterSlots] = {};
        for (int n = 0; n < kCounterSlots; ++n) {
            int best = -1;
            for (int s = 0; s < kCounterSlots; ++s)
                if (!tried[s] && (best < 0 || last_use_[s] < last_use_[best])) best = s;
            tried[best] = true;
            if (idle(best)) {
                owner_[best] = who;
                return touch(best);
            }
        }
        return -1;
    }

    // for tests
    bool used(int s) const { return used_[s]; }
    const SlotOwner& owner(int s) const { return owner_[s]; }

private:
    int touch(int s)
    {
        last_use_[s] = clock_;
        return s;
    }
    bool used_[kCounterSlots] = {};
    SlotOwner owner_[kCounterSlots] = {};
    uint64_t last_use_[kCounterSlots] = {};
    uint64_t clock_ = 0;
};

}  // namespace tbs

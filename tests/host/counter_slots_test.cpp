// Host-only test of the rule that hands sets of device counters to launches (counter_slots.h).
// A model of the device tells which launches are still running; the test asserts that no slot is ever
// given to a launch while a launch of another stream that used the slot may still be running.
#include <cassert>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <set>
#include <vector>

#include "counter_slots.h"

using tbs::kCounterSlots;
using tbs::SlotOwner;
using tbs::SlotTable;

namespace {

struct Model {
    SlotTable table;
    // launches in flight per slot: (stream id, launch number)
    std::vector<std::set<std::pair<int, int>>> running{(size_t)kCounterSlots};
    int launches = 0, refused = 0;

    int launch(int stream, uint64_t thread = 0)
    {
        SlotOwner who;
        who.stream = reinterpret_cast<const void*>((uintptr_t)(0x1000 + 16 * stream));
        who.thread = thread;
        const int s = table.acquire(who, [&](int slot) { return running[slot].empty(); });
        if (s < 0) {
            ++refused;
            return -1;
        }
        assert(s < kCounterSlots);
        // the invariant: whatever still runs on this slot was launched on the same stream (and thread)
        for (const auto& r : running[s]) assert(r.first == stream + 100000 * (int)thread);
        running[s].insert({stream + 100000 * (int)thread, launches++});
        return s;
    }
    void finish_all_of(int stream)
    {
        for (auto& set : running)
            for (auto it = set.begin(); it != set.end();)
                it = (it->first == stream) ? set.erase(it) : ++it;
    }
};

}  // namespace

int main()
{
    {   // one stream keeps its slot, whether or not its launches have finished
        Model m;
        const int a = m.launch(1);
        assert(a >= 0 && m.launch(1) == a);
        m.finish_all_of(1);
        assert(m.launch(1) == a);
    }
    {   // different streams get different slots while there are unused ones
        Model m;
        std::set<int> seen;
        for (int s = 0; s < kCounterSlots; ++s) {
            const int slot = m.launch(s);
            assert(slot >= 0 && seen.insert(slot).second);
        }
        // all slots busy with running launches of other streams: a 65th stream gets none ...
        assert(m.launch(1000) == -1 && m.refused == 1);
        // ... and still none on a second try, nothing having finished
        assert(m.launch(1000) == -1);
        // the owners keep theirs meanwhile
        for (int s = 0; s < kCounterSlots; ++s) assert(m.launch(s) >= 0);
        // once stream 17 has drained, its slot (and only it) can move
        m.finish_all_of(17);
        const int moved = m.launch(1000);
        assert(moved >= 0);
        assert(m.table.owner(moved).stream == reinterpret_cast<const void*>((uintptr_t)(0x1000 + 16 * 1000)));
        // stream 17 comes back: every slot is busy again, it gets none
        assert(m.launch(17) == -1);
    }
    {   // idle slots are recycled oldest first
        Model m;
        for (int s = 0; s < kCounterSlots; ++s) m.launch(s);
        for (int s = 0; s < kCounterSlots; ++s) m.finish_all_of(s);
        m.launch(5);                                         // slot of stream 5 is now the most recent
        const int first = m.launch(2000);                    // takes the oldest: stream 0's
        assert(m.table.owner(first).stream == reinterpret_cast<const void*>((uintptr_t)(0x1000 + 16 * 2000)));
        assert(first == 0);
        assert(m.launch(2001) == 1);
    }
    {   // the per-thread default stream: one handle, one slot per thread
        Model m;
        const int a = m.launch(2, 1), b = m.launch(2, 2);
        assert(a >= 0 && b >= 0 && a != b);
        assert(m.launch(2, 1) == a && m.launch(2, 2) == b);
    }
    {   // random traffic: the invariant inside Model::launch holds throughout
        Model m;
        std::srand(12345);
        for (int step = 0; step < 200000; ++step) {
            const int stream = std::rand() % 90;
            if (std::rand() % 4 == 0)
                m.finish_all_of(stream);
            else
                m.launch(stream);
        }
        assert(m.launches > 1000 && m.refused > 0);
    }
    std::puts("counter slots ok");
    return 0;
}

// Driver that runs the host-side slot bookkeeping (csrc/ifx_ring.hpp) under AddressSanitizer and
// UndefinedBehaviorSanitizer against a plain list model: commits through several wraps, growth with
// the blocks moved and in place, out-of-range queries.  Compiled and run by tests/test_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <deque>
#include <vector>

#include "../../paper_2511_20714_amd/csrc/ifx_ring.hpp"

static int check(const ifx_ring &r, const std::deque<int64_t> &model, const std::vector<int64_t> &slot_model)
{
    int bad = 0;
    bad |= r.resident() != (int64_t)model.size();
    for (int64_t s = -1; s <= r.cap_blocks; ++s) {
        const int64_t want = (s >= 0 && s < r.cap_blocks) ? slot_model[(size_t)s] : -1;
        bad |= r.ordinal_in_slot(s) != want;
    }
    for (int64_t l = -1; l <= (int64_t)model.size(); ++l) {
        const int64_t slot = r.slot_of_logical(l);
        if (l < 0 || l >= (int64_t)model.size())
            bad |= slot != -1;
        else
            bad |= slot < 0 || slot >= r.cap_blocks || slot_model[(size_t)slot] != model[(size_t)l];
    }
    return bad;
}

int main()
{
    int bad = 0;
    for (int in_place = 0; in_place < 2; ++in_place)
        for (int64_t cap : {1, 2, 3, 7}) {
            ifx_ring r(cap);
            std::deque<int64_t> model;                    // resident ordinals, oldest first
            std::vector<int64_t> slots((size_t)cap, -1);  // slot -> ordinal
            int64_t next = 0;
            auto commit = [&]() {
                const int64_t s = r.next_slot();
                bad |= s < 0 || s >= r.cap_blocks;
                if ((int64_t)model.size() == r.cap_blocks) {
                    bad |= slots[(size_t)s] != model.front();  // the slot reused is the oldest block's
                    model.pop_front();
                } else {
                    bad |= slots[(size_t)s] != -1;
                }
                bad |= r.commit() != s;
                slots[(size_t)s] = next;
                model.push_back(next++);
            };
            for (int i = 0; i < 3 * cap + 2; ++i) {
                commit();
                bad |= check(r, model, slots);
            }
            for (int round = 0; round < 3; ++round) {
                const int64_t bigger = r.cap_blocks + 1 + round;
                bad |= in_place ? r.grow_in_place(r.cap_blocks) : r.grow_moved(r.cap_blocks);  // not larger: refused
                bad |= !(in_place ? r.grow_in_place(bigger) : r.grow_moved(bigger));
                slots.resize((size_t)bigger, -1);
                if (!in_place) {  // the blocks were moved to slots 0, 1, ... oldest first
                    slots.assign((size_t)bigger, -1);
                    for (size_t i = 0; i < model.size(); ++i) slots[i] = model[i];
                }
                bad |= check(r, model, slots);
                for (int i = 0; i < 2 * bigger + 1; ++i) {
                    commit();
                    bad |= check(r, model, slots);
                }
            }
            r.reset();
            bad |= r.resident() != 0 || r.next_slot() != 0 || r.ordinal_in_slot(0) != -1;
        }
    std::printf(bad ? "FAILED\n" : "ok\n");
    return bad;
}

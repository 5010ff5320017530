// Driver that runs the host-side slot bookkeeping (csrc/ifx_ring.hpp) under AddressSanitizer and
// UndefinedBehaviorSanitizer against a plain list model: commits through several wraps, copying
// growth, range runs, out-of-range queries.  Compiled and run by tests/test_sanitizers.py.
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
    for (int64_t first = 0; first <= (int64_t)model.size(); ++first)
        for (int64_t count = 0; first + count <= (int64_t)model.size() + 1; ++count) {
            int64_t rs[2] = {-7, -7}, rb[2] = {-7, -7};
            const int k = r.runs_of_logical(first, count, rs, rb);
            if (first + count > (int64_t)model.size()) {
                bad |= k != -1;
                continue;
            }
            int64_t l = first;
            for (int t = 0; t < k; ++t)
                for (int64_t b = 0; b < rb[t]; ++b, ++l) bad |= slot_model[(size_t)(rs[t] + b)] != model[(size_t)l];
            bad |= l != first + count;
        }
    return bad;
}

int main()
{
    int bad = 0;
    for (int64_t cap : {1, 2, 3, 7}) {
        ifx_ring r{cap, 0};
        std::deque<int64_t> model;                         // resident ordinals, oldest first
        std::vector<int64_t> slots((size_t)cap, -1);       // slot -> ordinal
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
        // copying growth: resident blocks move to slots 0, 1, ... oldest first
        const int64_t bigger = cap + 3;
        bad |= r.grow(cap);  // not larger: refused
        bad |= !r.grow(bigger);
        slots.assign((size_t)bigger, -1);
        for (size_t i = 0; i < model.size(); ++i) slots[i] = model[i];
        bad |= check(r, model, slots);
        for (int i = 0; i < 2 * bigger + 1; ++i) {
            commit();
            bad |= check(r, model, slots);
        }
    }
    std::printf(bad ? "FAILED\n" : "ok\n");
    return bad;
}

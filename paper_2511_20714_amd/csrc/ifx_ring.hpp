// Slot bookkeeping of one layer's cache: a ring of whole-block slots
// (paper, KV Management section: block-wise KV memory with a sliding window).
// Pure host integer code, no device calls.
#pragma once
#include <cstdint>

struct ifx_ring {
    int64_t cap_blocks;  // slots
    int64_t count;       // blocks ever committed since create / reset

    int64_t resident() const { return count < cap_blocks ? count : cap_blocks; }
    int64_t next_slot() const { return count % cap_blocks; }
    // ordinal of the oldest resident block
    int64_t oldest() const { return count - resident(); }
    // ordinal held by a physical slot, -1 if empty
    int64_t ordinal_in_slot(int64_t slot) const
    {
        if (slot < 0 || slot >= cap_blocks || slot >= count) return -1;
        // the newest ordinal congruent to slot (mod cap_blocks) that is < count
        int64_t last = count - 1;
        return last - ((last - slot) % cap_blocks);
    }
    // physical slot of the logical-th oldest resident block
    int64_t slot_of_logical(int64_t logical) const
    {
        if (logical < 0 || logical >= resident()) return -1;
        return (oldest() + logical) % cap_blocks;
    }
    int64_t commit()
    {
        int64_t s = next_slot();
        ++count;
        return s;
    }
};

// Slot bookkeeping of one layer's cache: a ring of whole-block slots
// (paper, KV Management section: block-wise KV memory with a sliding window).
// Pure host integer code, no device calls.
#pragma once
#include <cstdint>

struct ifx_ring {
    int64_t cap_blocks;  // slots
    int64_t count;       // blocks ever committed since create / reset
    int64_t base = 0;    // ordinal that slot 0 held first: 0, or the oldest resident ordinal at the last grow()

    int64_t since_base() const { return count - base; }
    int64_t resident() const { return since_base() < cap_blocks ? since_base() : cap_blocks; }
    int64_t next_slot() const { return since_base() % cap_blocks; }
    // ordinal of the oldest resident block
    int64_t oldest() const { return count - resident(); }
    // ordinal held by a physical slot, -1 if empty
    int64_t ordinal_in_slot(int64_t slot) const
    {
        if (slot < 0 || slot >= cap_blocks || slot >= since_base()) return -1;
        // the newest ordinal congruent to slot (mod cap_blocks, counted from base) that is < count
        int64_t last = since_base() - 1;
        return base + last - ((last - slot) % cap_blocks);
    }
    // physical slot of the logical-th oldest resident block
    int64_t slot_of_logical(int64_t logical) const
    {
        if (logical < 0 || logical >= resident()) return -1;
        return (oldest() - base + logical) % cap_blocks;
    }
    // More slots (paper, abstract: variable-length generation): the caller moves the resident blocks
    // to slots 0, 1, ... in logical order, and the ring counts on from there.
    bool grow(int64_t new_cap_blocks)
    {
        if (new_cap_blocks <= cap_blocks) return false;
        base = oldest();
        cap_blocks = new_cap_blocks;
        return true;
    }
    // Physical slot runs holding the resident blocks [first, first + blocks) in logical order
    // (0 = oldest): one run, or two when the range wraps around the end of the ring.
    // Returns the number of runs (0 for an empty range), -1 if the range is not resident.
    int runs_of_logical(int64_t first, int64_t blocks, int64_t (&run_slot)[2], int64_t (&run_blocks)[2]) const
    {
        if (first < 0 || blocks < 0 || first + blocks > resident()) return -1;
        if (blocks == 0) return 0;
        const int64_t s0 = (oldest() - base + first) % cap_blocks;
        run_slot[0] = s0;
        if (s0 + blocks <= cap_blocks) {
            run_blocks[0] = blocks;
            return 1;
        }
        run_blocks[0] = cap_blocks - s0;
        run_slot[1] = 0;
        run_blocks[1] = blocks - run_blocks[0];
        return 2;
    }
    int64_t commit()
    {
        int64_t s = next_slot();
        ++count;
        return s;
    }
};

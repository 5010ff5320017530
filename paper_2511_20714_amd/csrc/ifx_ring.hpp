// Slot bookkeeping of one layer's cache: whole-block slots reused in age order
// (paper, KV Management section: block-wise KV memory with a sliding window).
// Pure host integer code, no device calls.
//
// State: the slots in use, listed in the order in which they are reused
// (`perm`), and where in that list the oldest resident block sits (`head`).
// Slots are taken in increasing order until all `cap_blocks` are in use, so the
// slots in use are always 0 .. resident() - 1; from then on every commit
// overwrites the oldest resident block and the list is walked round and round.
// The list, rather than a closed formula, is what lets the capacity grow in
// place: new slots are appended behind the slots in use, in whatever order
// those are being reused at that moment, and nothing has to move.
#pragma once
#include <cstdint>
#include <vector>

struct ifx_ring {
    int64_t cap_blocks;  // slots
    int64_t count = 0;   // blocks ever committed since create / reset

    // may throw std::bad_alloc
    explicit ifx_ring(int64_t capacity_blocks) : cap_blocks(capacity_blocks) { perm.reserve((size_t)capacity_blocks); }

    int64_t resident() const { return (int64_t)perm.size(); }
    // slot the next committed block goes to
    int64_t next_slot() const { return resident() < cap_blocks ? resident() : perm[(size_t)head]; }
    // ordinal of the oldest resident block
    int64_t oldest() const { return count - resident(); }
    // physical slot of the logical-th oldest resident block, -1 if there is none
    int64_t slot_of_logical(int64_t logical) const
    {
        if (logical < 0 || logical >= resident()) return -1;
        return perm[(size_t)((head + logical) % resident())];
    }
    // ordinal held by a physical slot, -1 if empty
    int64_t ordinal_in_slot(int64_t slot) const
    {
        if (slot < 0 || slot >= resident()) return -1;  // slots in use are 0 .. resident() - 1
        for (int64_t i = 0; i < resident(); ++i)
            if (perm[(size_t)i] == slot) return oldest() + (i - head + resident()) % resident();
        return -1;
    }
    // Commit: returns the slot the block goes to.  Never allocates (the list's room was reserved
    // when the capacity was set).
    int64_t commit()
    {
        const int64_t s = next_slot();
        if (resident() < cap_blocks)
            perm.push_back(s);
        else
            head = (head + 1) % cap_blocks;
        ++count;
        return s;
    }
    void reset()
    {
        perm.clear();
        head = 0;
        count = 0;
    }
    // More slots (paper, abstract: variable-length generation), the resident blocks staying where
    // they are: the new slots are used next, then reuse goes on oldest block first.
    // May throw std::bad_alloc (nothing is changed then).
    bool grow_in_place(int64_t new_cap_blocks)
    {
        if (new_cap_blocks <= cap_blocks) return false;
        std::vector<int64_t> by_age;
        by_age.reserve((size_t)new_cap_blocks);
        for (int64_t l = 0; l < resident(); ++l) by_age.push_back(slot_of_logical(l));
        perm.swap(by_age);
        head = 0;
        cap_blocks = new_cap_blocks;
        return true;
    }
    // More slots, the caller having moved the resident blocks to slots 0, 1, ... oldest first
    // (new memory).  May throw std::bad_alloc (nothing is changed then).
    bool grow_moved(int64_t new_cap_blocks)
    {
        if (new_cap_blocks <= cap_blocks) return false;
        std::vector<int64_t> by_age;
        by_age.reserve((size_t)new_cap_blocks);
        for (int64_t l = 0; l < resident(); ++l) by_age.push_back(l);
        perm.swap(by_age);
        head = 0;
        cap_blocks = new_cap_blocks;
        return true;
    }

  private:
    std::vector<int64_t> perm;  // slots in use, in reuse order
    int64_t head = 0;           // index in perm of the oldest resident block (0 until all slots are in use)
};

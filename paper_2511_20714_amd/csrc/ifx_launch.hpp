// The launch shape of the bf16 attention kernel: how many workgroups, and which head and which
// query rows each of them takes.  Plain integer code shared by the host (which fills the shape in),
// the kernel (which decodes its workgroup number with it) and the CPU tests (which check, through
// the library's diagnostic calls, that the decoded items tile every head's rows exactly once).
//
// Workgroups are dealt round-robin to the 8 XCDs (workgroup w runs on XCD w % 8), each with an L2
// of its own.  A head's K/V stream is shared by all its workgroups, so a head is given to as few
// XCDs as possible: every XCD takes all workgroups of `whole_heads` heads of its own, then its
// share of the heads % 8 heads that are left: each of those split over `share` XCDs, `left_chunk`
// workgroups apiece (when heads % 8 divides 8), or (share == 0) their workgroups dealt out
// contiguously, `left_chunk` per XCD.
//
// A head's ceil(n / 32) wavefronts' worth of query rows go to its q_tiles = ceil(n / 256)
// workgroups as evenly as whole wavefronts allow: the first `q_more` of them take q_waves + 1
// wavefronts' rows, the others q_waves (<= 8 either way).  With full workgroups and one short one,
// the short one runs ahead of the others through the head's keys, out of reach of the L2 they
// share, and the head is fetched from memory twice.
#pragma once
#include <hip/hip_runtime.h>

namespace ifx {

struct attn_shape {
    int q_tiles;   // workgroups per head
    int q_waves, q_more;
    int whole_heads, left_heads, share, left_chunk;
    unsigned grid;  // workgroups of the launch (a few of them may find nothing to do and exit)
};

// What one workgroup does: `waves` wavefronts of 32 query rows from row0 on (the last row of the
// last one may lie past n - 1), or nothing (waves == 0).
struct attn_item {
    int head, q_tile, row0, waves;
};

inline attn_shape attn_shape_for(int n, int heads)
{
    attn_shape s;
    s.q_tiles = (n + 255) / 256;
    const int q_wavefronts = (n + 31) / 32;  // q_tiles = ceil(q_wavefronts / 8), so 1 <= q_waves <= 8
    s.q_waves = q_wavefronts / s.q_tiles;
    s.q_more = q_wavefronts % s.q_tiles;
    s.whole_heads = heads / 8;
    s.left_heads = heads % 8;
    s.share = s.left_heads > 0 && 8 % s.left_heads == 0 ? 8 / s.left_heads : 0;
    s.left_chunk = s.left_heads == 0 ? 0
                   : s.share > 0     ? (s.q_tiles + s.share - 1) / s.share
                                     : (s.left_heads * s.q_tiles + 7) / 8;
    s.grid = 8u * (unsigned)(s.whole_heads * s.q_tiles + s.left_chunk);
    return s;
}

__host__ __device__ inline attn_item attn_item_of(const attn_shape &s, unsigned workgroup)
{
    const int xcd = (int)(workgroup & 7u);
    const int idx = (int)(workgroup >> 3);
    attn_item it = {0, 0, 0, 0};
    if (idx < s.whole_heads * s.q_tiles) {
        it.head = xcd * s.whole_heads + idx / s.q_tiles;
        it.q_tile = idx % s.q_tiles;
    } else {
        const int rest = idx - s.whole_heads * s.q_tiles;
        if (s.share > 0) {
            it.head = 8 * s.whole_heads + xcd / s.share;
            it.q_tile = (xcd % s.share) * s.left_chunk + rest;
            if (it.q_tile >= s.q_tiles) return it;
        } else {
            const int item = xcd * s.left_chunk + rest;
            if (item >= s.left_heads * s.q_tiles) return it;
            it.head = 8 * s.whole_heads + item / s.q_tiles;
            it.q_tile = item % s.q_tiles;
        }
    }
    it.row0 = 32 * (it.q_tile * s.q_waves + (it.q_tile < s.q_more ? it.q_tile : s.q_more));
    it.waves = s.q_waves + (it.q_tile < s.q_more ? 1 : 0);
    return it;
}

}  // namespace ifx

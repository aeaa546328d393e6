// Static tile schedule of the attention launch (host and device).
//
// The launch runs `grid` workgroups over `total` logical tiles (a logical tile is one (batch*head,
// query tile) pair; consecutive logical tiles belong to the same head).  The hardware deals
// workgroup ids round-robin to the 8 XCDs, each with its own L2, so every XCD is given a
// contiguous range of logical tiles and the workgroups that sit on it walk that range together,
// a row of g tiles per round (g = workgroups on the XCD): at any moment they stream the K/V of the
// same one or two heads through their L2.  Odd rounds run right to left: with the causal mask the
// tiles of a head are ordered from long to short, and pairing a left-to-right round with a
// right-to-left one gives every workgroup nearly the same total length (the persistent, statically
// balanced schedule of the paper's Section 4.2).  With grid == total this is one round and the
// plain one-tile-per-workgroup launch.
//
// tile_schedule(total, grid, block, round) is the logical tile workgroup `block` processes in round
// `round`, or -1 when it has none (then it has none in any later round either).  Every logical
// tile is returned for exactly one (block, round) provided grid >= min(total, 8).
#pragma once

#if defined(__HIPCC__)
#define TILE_SCHEDULE_HD __host__ __device__
#else
#define TILE_SCHEDULE_HD
#endif

TILE_SCHEDULE_HD inline int tile_schedule(int total, int grid, int block, int round)
{
    const int XCDS = 8;
    const int x = block % XCDS, slot = block / XCDS;
    const int tq = total / XCDS, tr = total % XCDS;
    const int count = tq + (x < tr ? 1 : 0);             // tiles of this XCD ...
    const int start = x * tq + (x < tr ? x : tr);        // ... and the first of them
    const int g = grid / XCDS + (x < grid % XCDS ? 1 : 0);
    const int idx = round * g + ((round & 1) ? g - 1 - slot : slot);
    return idx < count ? start + idx : -1;
}

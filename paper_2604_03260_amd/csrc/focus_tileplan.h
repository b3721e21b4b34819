// Per query tile: which tiles of the class-ordered key arrays it must visit.
//
// A query tile holds up to L.BQ queries of ONE membership class, positions
// ascending.  Keys are partitioned by class too, so every allowed pair of
// App. D Eq. 3 (with top-k sets) is met exactly once:
//   - key class shares a group with the query class: all its keys up to the
//     tile's last query position (causal prefix), or all its keys (non-causal);
//   - otherwise: only its keys inside the union of the rows' local windows
//     (i-w < j <= i causal, |i-j| < w non-causal).
// Per-element causal/window checks on positions finish the job inside a tile.
// A launch may be restricted to one of the two disjoint parts (App. D): the classes that share
// a group (set A) or the window spans of those that share none (set B); a tile may then have nothing to visit.
#pragma once
#include "focus_internal.h"

namespace focus {

struct TilePlan {
    int t0[MAX_CLASSES];       // first key tile (global tile index inside the head)
    int cum[MAX_CLASSES + 1];  // running number of tiles over the classes
    uint8_t inter[MAX_CLASSES];
    int ibeg[MAX_CLASSES];     // tiles [ibeg, iend) of the class need no per-element causal/window test
    int iend[MAX_CLASSES];
    int cnt_hi[MAX_CLASSES];   // keys of every class in the part of a sort block below the upper bound
    int cnt_lo[MAX_CLASSES];   // ... and below the lower bound of the window span
    int cls, tile, row0, nvalid, i_lo, i_hi, total;
};

// All threads of the work-group call this (blockDim.x >= 64).  Returns false when
// the job slot is unused.
__device__ inline bool plan_query_tile(const Layout& L, const char* __restrict__ ws, int bhq, int bhk, int job,
                                       TilePlan& P)
{
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int NC = L.NC;
    const int jv = ((const int*)(ws + L.off_jobs))[(size_t)bhq * L.NT + job];
    if (jv == -1) return false;                             // class ids reach 255: the word is unsigned but for -1
    const int c = (int)((unsigned)jv >> 24), t = jv & 0xffffff;
    const int* qco = (const int*)(ws + L.off_qco) + (size_t)bhq * (NC + 1);
    const int* qcc = (const int*)(ws + L.off_qcc) + (size_t)bhq * NC;
    const int* qperm = (const int*)(ws + L.off_qperm) + (size_t)bhq * L.NQP;
    const int row0 = qco[c] + t * L.BQ;
    const int nvalid = min(L.BQ, qcc[c] - t * L.BQ);
    const int i_lo = qperm[row0];
    const int i_hi = qperm[row0 + nvalid - 1];
    // keys with position < x_hi are causal for the tile / not beyond every window (non-causal); the pass over
    // the pairs outside the window (pair_set 3, causal) ends below the window of the tile's last row instead
    const int x_hi = L.pair_set == 3 ? max(0, i_hi - L.window + 1) : L.causal ? i_hi + 1 : min(L.n, i_hi + L.window);
    const int x_lo = max(0, i_lo - L.window + 1);           // keys with position < x_lo are outside every window
    const uint8_t* kcls = (const uint8_t*)(ws + L.off_kcls) + (size_t)bhk * ((size_t)L.nblk * SB);
    const int bh_i = x_hi / SB, bl_i = x_lo / SB;
    const int part_hi = x_hi % SB, part_lo = x_lo % SB;
    // The prefix counts at sort-block boundaries come from the assign pass; the partial blocks are
    // counted here, all threads at once into a class histogram (integer atomics in LDS).
    for (int c2 = tid; c2 < NC; c2 += nthr) { P.cnt_hi[c2] = 0; P.cnt_lo[c2] = 0; }
    if (tid == 0) {
        P.cls = c; P.tile = t; P.row0 = row0; P.nvalid = nvalid; P.i_lo = i_lo; P.i_hi = i_hi;
    }
    __syncthreads();
    for (int e = tid; e < SB; e += nthr) {
        if (e < part_hi) atomicAdd(&P.cnt_hi[kcls[(size_t)bh_i * SB + e]], 1);
        if (e < part_lo) atomicAdd(&P.cnt_lo[kcls[(size_t)bl_i * SB + e]], 1);
    }
    __syncthreads();
    const int* kbc = (const int*)(ws + L.off_kbc) + (size_t)bhk * (L.nblk + 1) * NC;
    const int* kco = (const int*)(ws + L.off_kco) + (size_t)bhk * (NC + 1);
    const uint32_t* clsmask = (const uint32_t*)(ws + L.off_clsmask);
    const uint32_t mymask = clsmask[c];
    for (int c2 = tid; c2 < NC; c2 += nthr) {
        const int pre_hi = kbc[(size_t)bh_i * NC + c2] + P.cnt_hi[c2];
        // the local layout's one class holds every key: all of them count as "window only" there
        const bool inter = !L.local_only && (clsmask[c2] & mymask) != 0;
        const int koff = kco[c2];
        int a = 0, b = 0;
        // Coarse classes that share a super-group hold pairs of both sets: set B then visits their window span
        // like a class that shares nothing, and the kernels sort the pairs out one by one.
        const bool as_window = !inter || (L.coarse && L.pair_set == 2);
        if (!as_window) {
            if (L.pair_set != 2) {                         // set B skips the classes that share a group
                const int upto = L.causal ? pre_hi : kbc[(size_t)L.nblk * NC + c2];   // non-causal: the whole class
                a = koff / KT;
                b = (koff + upto + KT - 1) / KT;
            }
        } else if (L.pair_set != 1 && L.pair_set != 3) {   // sets A and 3 skip the classes that share none
            const int pre_lo = kbc[(size_t)bl_i * NC + c2] + P.cnt_lo[c2];
            if (pre_hi > pre_lo) {
                a = (koff + pre_lo) / KT;
                b = (koff + pre_hi + KT - 1) / KT;
            }
        }
        P.t0[c2] = a;
        P.cum[c2 + 1] = b - a;                             // lengths first, summed below
        P.inter[c2] = inter ? 1 : 0;
        // Tiles that need no per-element test, from prefix counts at sort-block boundaries (conservative):
        // keys before the sort block that holds i_lo+1 sit at positions <= i_lo (causal for every row);
        // for a class without a common group they must also lie above i_hi - window for every row.
        // Non-causal: for a class with a common group every tile without pads; otherwise the keys must lie
        // below i_lo + window for every row instead of at or below i_lo.
        const int safe_end = L.pair_set == 3 ? max(0, i_lo - L.window + 1) : L.causal ? i_lo + 1 : min(L.n, i_lo + L.window);
        const int cnt_below = (!L.causal && (inter || safe_end >= L.n)) ? kbc[(size_t)L.nblk * NC + c2]
                                                                        : kbc[(size_t)(safe_end / SB) * NC + c2];
        int ib = a, ie = a;
        if (inter) {
            // coarse classes only promise a common super-group: every pair is tested against the real masks
            if (!L.coarse) ie = a + min(b - a, cnt_below / KT);
        } else if (b > a) {
            const int x_in = i_hi - L.window + 1;
            const int lo_blk = (x_in <= 0) ? 0 : min(L.nblk, (x_in + SB - 1) / SB);
            ib = max(a, (koff + kbc[(size_t)lo_blk * NC + c2] + KT - 1) / KT);
            ie = min(b, (koff + cnt_below) / KT);
            if (L.local_only) {          // position order: slot = position, so the bounds are exact per key tile
                ib = max(a, (max(x_in, 0) + KT - 1) / KT);
                ie = min(b, (i_lo + 1) / KT);
            }
            if (ie < ib) ie = ib;
        }
        P.ibeg[c2] = ib;
        P.iend[c2] = ie;
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        P.cum[0] = 0;
        for (int c2 = 0; c2 < NC; ++c2) { run += P.cum[c2 + 1]; P.cum[c2 + 1] = run; }
        P.total = run;
    }
    __syncthreads();
    return true;
}

}  // namespace focus

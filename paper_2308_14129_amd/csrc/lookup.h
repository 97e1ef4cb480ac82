// Most-recent-K temporal neighbours of one query (node u, time t), one wavefront per query:
// the K events incident to u with time strictly earlier than t (the history E_t of the paper's
// Notations section, "most recent neighbours" sampling of Sec. II-B), ordered by (time, event id)
// descending.  Adjacency lists are ordered by (time, event id), so the answer is the K entries
// just below the first entry with time >= t.
//
// That boundary is found by a 64-way search over the list (each round, lane i probes the end of
// the i-th 1/64 of the remaining range; the ballot narrows the range 64-fold).  Queries of a
// batch's own events (source / destination roles) start from the event's own position in the
// list, which bounds the boundary from above: usually one probe round over the 64 entries below
// it suffices (only entries with an equal timestamp have to be stepped over).
#pragma once

#include "kernels_common.h"

namespace tig {

// One wavefront: the query (u, t) becomes row `row` of the query set (node, time, neighbour
// slots, count; the row references are filled in later).  own_pos: adjacency position of the
// query's own event in u's list (everything from there on has time >= t), or -1 if unknown.
// my_nbr / my_eid / my_ts: the slot this lane wrote (lanes below K; -1, -1, 0.0 for an unused
// slot and for the other lanes).  Returns the number of filled slots.
__device__ inline int nbr_lookup_wave(const StepArgs &a, int K, int32_t u, double t, int64_t own_pos,
                                      const QuerySet &qs, int row, int32_t &my_nbr, int32_t &my_eid, double &my_ts)
{
    my_nbr = -1;
    my_eid = -1;
    my_ts = 0.0;
    const int lane = lane_id();
    int64_t lo = 0, hi = 0;
    const bool known = u >= 0 && (int64_t)u < a.num_nodes;
    if (known) {
        lo = a.indptr[u];
        hi = a.indptr[u + 1];
    }
    const int64_t base = lo;
    // invariant: entries below lo have time < t; entries at or above hi have time >= t
    if (own_pos >= 0) {
        hi = own_pos;
        if (hi - lo > kWave) {
            const int64_t idx = hi - 1 - lane;  // the 64 entries just below
            const bool less = a.csr[idx].ts < t;
            const unsigned long long m = __ballot(less);
            if (m != 0ull) {
                // lanes grow towards earlier entries: the first set lane is the newest entry < t
                const int first = __ffsll((long long)m) - 1;
                lo = hi - first;  // entries hi-first .. hi-1 have time >= t, entry hi-first-1 < t
                hi = lo;
            } else {
                hi -= kWave;  // a run of 64+ equal timestamps: fall back to the search below
            }
        }
    }
    while (hi - lo > kWave) {
        const int64_t step = (hi - lo + kWave - 1) / kWave;
        int64_t idx = lo + (int64_t)(lane + 1) * step - 1;
        if (idx > hi - 1)
            idx = hi - 1;
        const bool less = a.csr[idx].ts < t;
        const int c = __popcll(__ballot(less));  // lists are time-ordered: lanes 0..c-1 are true
        int64_t nlo = lo + (int64_t)c * step;
        if (nlo > hi)
            nlo = hi;
        if (c < kWave) {
            int64_t nhi = lo + (int64_t)(c + 1) * step - 1;
            if (nhi > hi - 1)
                nhi = hi - 1;
            hi = nhi;
        }
        lo = nlo;
    }
    if (hi > lo) {
        const int64_t idx = lo + lane;
        const bool less = idx < hi && a.csr[idx].ts < t;
        lo += __popcll(__ballot(less));
    }
    const int64_t avail = lo - base;
    if (lane < K) {
        const int64_t p = lo - 1 - lane;
        const size_t o = (size_t)row * K + lane;
        if (p >= base) {
            const CsrEntry e = a.csr[p];
            my_nbr = e.nbr;
            my_eid = e.eid;
            my_ts = e.ts;
            qs.nbr[o] = e.nbr;
            qs.eid[o] = e.eid;
            qs.ts[o] = e.ts;
        } else {
            qs.nbr[o] = -1;
            qs.eid[o] = -1;
            qs.ts[o] = 0.0;
        }
    }
    const int cnt = (int)(avail < K ? avail : K);
    if (lane == 0) {
        qs.cnt[row] = cnt;
        qs.node[row] = known ? u : -1;
        qs.t[row] = t;
    }
    return cnt;
}

}  // namespace tig

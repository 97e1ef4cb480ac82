/*
 * TEST INFRASTRUCTURE -- part of the CPU oracle, never of the product path.
 *
 * Indexed most-recent-K temporal neighbour lookup for graphs too large for the
 * brute-force scan in tig_oracle.py (which is the definition; this routine is
 * checked bit-for-bit against it on small graphs).
 *
 * History of a query (u, t) is the set of events incident to u with a time
 * strictly earlier than t (the set E_t of the paper's Notations section); of
 * those the K most recent are returned (the "most recent neighbours" sampling
 * the paper refers to in Sec. II-B), ordered by (time, event id) descending.
 *
 * Requires events sorted by time (non-decreasing), so that each node's list in
 * event-id order is already ordered by (time, event id).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORA_API __attribute__((visibility("default")))

typedef struct {
    int64_t num_nodes;
    int64_t num_events;
    int64_t *start;      /* [num_nodes + 1] offsets into ev */
    int32_t *ev;         /* [2 * num_events] event ids, per node, ascending */
    const int32_t *src;  /* borrowed */
    const int32_t *dst;  /* borrowed */
    const double *ts;    /* borrowed */
} nbr_index;

ORA_API void nbr_index_free(nbr_index *ix)
{
    if (!ix)
        return;
    free(ix->start);
    free(ix->ev);
    free(ix);
}

/* Borrowed arrays must outlive the index.  Returns NULL on bad input / no memory. */
ORA_API nbr_index *nbr_index_build(int64_t num_nodes, int64_t num_events, const int32_t *src,
                                   const int32_t *dst, const double *ts)
{
    if (num_nodes <= 0 || num_events < 0 || !src || !dst || !ts)
        return NULL;
    for (int64_t e = 0; e < num_events; ++e) {
        if (src[e] < 0 || src[e] >= num_nodes || dst[e] < 0 || dst[e] >= num_nodes)
            return NULL;
        if (e > 0 && ts[e] < ts[e - 1])
            return NULL;
    }
    nbr_index *ix = (nbr_index *)calloc(1, sizeof(nbr_index));
    if (!ix)
        return NULL;
    ix->num_nodes = num_nodes;
    ix->num_events = num_events;
    ix->src = src;
    ix->dst = dst;
    ix->ts = ts;
    ix->start = (int64_t *)calloc((size_t)num_nodes + 1, sizeof(int64_t));
    ix->ev = (int32_t *)malloc(sizeof(int32_t) * (size_t)(2 * num_events > 0 ? 2 * num_events : 1));
    int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * (size_t)num_nodes);
    if (!ix->start || !ix->ev || !fill) {
        free(fill);
        nbr_index_free(ix);
        return NULL;
    }
    for (int64_t e = 0; e < num_events; ++e) {
        ix->start[src[e] + 1]++;
        if (dst[e] != src[e])
            ix->start[dst[e] + 1]++;
    }
    for (int64_t u = 0; u < num_nodes; ++u)
        ix->start[u + 1] += ix->start[u];
    memcpy(fill, ix->start, sizeof(int64_t) * (size_t)num_nodes);
    for (int64_t e = 0; e < num_events; ++e) { /* ascending event id */
        ix->ev[fill[src[e]]++] = (int32_t)e;
        if (dst[e] != src[e])
            ix->ev[fill[dst[e]]++] = (int32_t)e;
    }
    free(fill);
    return ix;
}

/*
 * For each query q: out_*[q*K + k], k = 0 most recent; unused slots get
 * node = -1, eid = -1, ts = 0.0; out_cnt[q] = number of valid slots.
 */
ORA_API int nbr_index_query(const nbr_index *ix, int64_t num_queries, const int32_t *q_node,
                            const double *q_time, int32_t K, int32_t *out_node, int32_t *out_eid,
                            double *out_ts, int32_t *out_cnt)
{
    if (!ix || num_queries < 0 || K <= 0 || !q_node || !q_time || !out_node || !out_eid || !out_ts ||
        !out_cnt)
        return -1;
    for (int64_t q = 0; q < num_queries; ++q) {
        const int32_t u = q_node[q];
        const double t = q_time[q];
        int64_t lo = 0, hi = 0;
        if (u >= 0 && u < ix->num_nodes) {
            lo = ix->start[u];
            hi = ix->start[u + 1];
        }
        const int64_t base = lo;
        /* number of list entries with time < t */
        while (lo < hi) {
            int64_t mid = lo + ((hi - lo) >> 1);
            if (ix->ts[ix->ev[mid]] < t)
                lo = mid + 1;
            else
                hi = mid;
        }
        int32_t cnt = 0;
        for (int32_t k = 0; k < K; ++k) {
            const int64_t p = lo - 1 - k;
            const int64_t o = q * (int64_t)K + k;
            if (p >= base) {
                const int32_t e = ix->ev[p];
                out_eid[o] = e;
                out_node[o] = ix->src[e] == u ? ix->dst[e] : ix->src[e];
                out_ts[o] = ix->ts[e];
                ++cnt;
            } else {
                out_eid[o] = -1;
                out_node[o] = -1;
                out_ts[o] = 0.0;
            }
        }
        out_cnt[q] = cnt;
    }
    return 0;
}

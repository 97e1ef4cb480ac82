/*
 * Seeded synthetic temporal-interaction-graph workloads.
 *
 * This file only draws random INPUTS (event endpoints, timestamps, edge
 * features, negatives, model weights, warm-start state).  It contains none of
 * the model's arithmetic and is the one piece shared by the CPU oracle's tests
 * and the GPU library's tests/benchmarks.
 *
 * Every value is a pure function of (seed, stream, index) through a
 * counter-based generator (splitmix64 finaliser), so results do not depend on
 * the number of OpenMP threads or on any library's random stream.
 *
 * The shapes follow the dataset table of the paper (node / edge counts and
 * feature widths of its small bipartite datasets and its large datasets) and
 * its batch sizes (Sec. III-A); no record of any dataset is reproduced.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GEN_API __attribute__((visibility("default")))

enum {
    STREAM_SRC = 1,
    STREAM_DST = 2,
    STREAM_TS = 3,
    STREAM_FEAT = 4,
    STREAM_NEG = 5,
    STREAM_STATE = 6,
    STREAM_WEIGHT_BASE = 100
};

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* 64 random bits for (seed, stream, index, attempt). */
static inline uint64_t rnd_bits(uint64_t seed, uint64_t stream, uint64_t index, uint64_t attempt)
{
    uint64_t h = mix64(seed ^ (stream * 0xD6E8FEB86659FD93ull));
    h = mix64(h + index);
    if (attempt)
        h = mix64(h ^ (attempt * 0xA24BAED4963EE407ull));
    return h;
}

/* uniform double in [0, 1) with 53 random bits */
static inline double rnd_u01(uint64_t seed, uint64_t stream, uint64_t index, uint64_t attempt)
{
    return (double)(rnd_bits(seed, stream, index, attempt) >> 11) * (1.0 / 9007199254740992.0);
}

/* ---- bounded rank-frequency Zipf: P(rank r) ~ r^-alpha, r = 1..n ---------- */

GEN_API int tig_gen_zipf_cdf(int64_t n, double alpha, double *cdf)
{
    if (n <= 0 || !cdf)
        return -1;
    double acc = 0.0;
    for (int64_t r = 0; r < n; ++r) {
        acc += pow((double)(r + 1), -alpha);
        cdf[r] = acc;
    }
    const double inv = 1.0 / acc;
    for (int64_t r = 0; r < n; ++r)
        cdf[r] *= inv;
    cdf[n - 1] = 1.0;
    return 0;
}

/* first index with cdf[idx] > u  (0-based rank) */
static inline int64_t zipf_draw(const double *cdf, int64_t n, double u)
{
    int64_t lo = 0, hi = n - 1;
    while (lo < hi) {
        int64_t mid = lo + ((hi - lo) >> 1);
        if (cdf[mid] > u)
            hi = mid;
        else
            lo = mid + 1;
    }
    return lo;
}

/*
 * Endpoints.  Bipartite (n_dst_side > 0): src ids 0..n_src_side-1 drawn from
 * cdf_src, dst ids n_src_side..n_src_side+n_dst_side-1 drawn from cdf_dst.
 * Otherwise both endpoints come from cdf_src over n_src_side ids and dst is
 * redrawn until it differs from src.  Node id = rank - 1 within its side.
 */
GEN_API int tig_gen_endpoints(uint64_t seed, int64_t num_events, int64_t n_src_side,
                              int64_t n_dst_side, const double *cdf_src, const double *cdf_dst,
                              int32_t *src, int32_t *dst)
{
    if (num_events < 0 || n_src_side <= 0 || !cdf_src || !src || !dst)
        return -1;
    if (n_dst_side > 0 && !cdf_dst)
        return -1;
    if (n_dst_side <= 0 && n_src_side < 2)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < num_events; ++e) {
        int64_t s = zipf_draw(cdf_src, n_src_side, rnd_u01(seed, STREAM_SRC, (uint64_t)e, 0));
        int64_t d;
        if (n_dst_side > 0) {
            d = n_src_side + zipf_draw(cdf_dst, n_dst_side, rnd_u01(seed, STREAM_DST, (uint64_t)e, 0));
        } else {
            uint64_t attempt = 0;
            do {
                d = zipf_draw(cdf_src, n_src_side, rnd_u01(seed, STREAM_DST, (uint64_t)e, attempt));
                ++attempt;
            } while (d == s);
        }
        src[e] = (int32_t)s;
        dst[e] = (int32_t)d;
    }
    return 0;
}

/*
 * Sorted timestamps in [0, span): normalised running sums of Exp(1) spacings
 * (the order statistics of uniforms, produced without a sort).  Chunked with a
 * fixed chunk length so the summation order, hence every bit of the result,
 * is independent of the thread count.  floor_to_int != 0 floors to whole
 * units (integer seconds), which creates equal-timestamp runs.
 */
#define TS_CHUNK (1 << 16)

GEN_API int tig_gen_timestamps(uint64_t seed, int64_t num_events, double span, int floor_to_int,
                               double *ts)
{
    if (num_events < 0 || !ts || !(span > 0.0))
        return -1;
    if (num_events == 0)
        return 0;
    const int64_t n_chunks = (num_events + TS_CHUNK - 1) / TS_CHUNK;
    double *chunk_sum = (double *)malloc(sizeof(double) * (size_t)(n_chunks + 1));
    if (!chunk_sum)
        return -2;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n_chunks; ++c) {
        const int64_t lo = c * TS_CHUNK;
        const int64_t hi = lo + TS_CHUNK < num_events ? lo + TS_CHUNK : num_events;
        double run = 0.0;
        for (int64_t e = lo; e < hi; ++e) {
            double u = rnd_u01(seed, STREAM_TS, (uint64_t)e, 0);
            run += -log(1.0 - u); /* 1-u in (0,1] */
            ts[e] = run;
        }
        chunk_sum[c] = run;
    }
    /* exclusive prefix over chunks, sequential and in order */
    double acc = 0.0;
    for (int64_t c = 0; c < n_chunks; ++c) {
        double s = chunk_sum[c];
        chunk_sum[c] = acc;
        acc += s;
    }
    /* one more spacing after the last event keeps every timestamp below span */
    const double total = acc + -log(1.0 - rnd_u01(seed, STREAM_TS, (uint64_t)num_events, 0));
    const double scale = span / total;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n_chunks; ++c) {
        const int64_t lo = c * TS_CHUNK;
        const int64_t hi = lo + TS_CHUNK < num_events ? lo + TS_CHUNK : num_events;
        const double off = chunk_sum[c];
        for (int64_t e = lo; e < hi; ++e) {
            double t = (off + ts[e]) * scale;
            if (floor_to_int)
                t = floor(t);
            if (t >= span)
                t = floor_to_int ? span - 1.0 : nextafter(span, 0.0);
            ts[e] = t;
        }
    }
    free(chunk_sum);
    /* rounding in (off + local) * scale cannot reorder by more than an ulp across a chunk
       border; enforce the non-decreasing contract exactly */
    for (int64_t e = 1; e < num_events; ++e)
        if (ts[e] < ts[e - 1])
            ts[e] = ts[e - 1];
    return 0;
}

/* i.i.d. N(0,1) as fp32, Box-Muller in double, two outputs per pair index. */
GEN_API int tig_gen_normal_f32(uint64_t seed, uint64_t stream, int64_t count, float *out)
{
    if (count < 0 || !out)
        return -1;
    const int64_t pairs = (count + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < pairs; ++p) {
        double u1 = 1.0 - rnd_u01(seed, stream, (uint64_t)p, 0); /* (0,1] */
        double u2 = rnd_u01(seed, stream, (uint64_t)p, 1);
        double r = sqrt(-2.0 * log(u1));
        double a = 6.283185307179586476925286766559 * u2;
        out[2 * p] = (float)(r * cos(a));
        if (2 * p + 1 < count)
            out[2 * p + 1] = (float)(r * sin(a));
    }
    return 0;
}

GEN_API int tig_gen_edge_feat(uint64_t seed, int64_t num_events, int64_t feat_dim, float *out)
{
    return tig_gen_normal_f32(seed, STREAM_FEAT, num_events * feat_dim, out);
}

/* uniform fp32 in [lo, hi) */
GEN_API int tig_gen_uniform_f32(uint64_t seed, uint64_t stream, int64_t count, double lo, double hi,
                                float *out)
{
    if (count < 0 || !out)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i)
        out[i] = (float)(lo + (hi - lo) * rnd_u01(seed, stream, (uint64_t)i, 0));
    return 0;
}

/*
 * One negative destination per event, uniform over [id_lo, id_lo + id_count),
 * redrawn until it differs from the event's source.
 */
GEN_API int tig_gen_negatives(uint64_t seed, int64_t first_eid, int64_t count, int64_t id_lo,
                              int64_t id_count, const int32_t *src, int32_t *neg)
{
    if (count < 0 || id_count <= 0 || !src || !neg)
        return -1;
    if (id_count == 1)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < count; ++b) {
        const uint64_t e = (uint64_t)(first_eid + b);
        uint64_t attempt = 0;
        int64_t v;
        do {
            v = id_lo + (int64_t)(rnd_u01(seed, STREAM_NEG, e, attempt) * (double)id_count);
            if (v >= id_lo + id_count)
                v = id_lo + id_count - 1;
            ++attempt;
        } while (v == (int64_t)src[e]);
        neg[b] = (int32_t)v;
    }
    return 0;
}

/*
 * Warm-start state for a window that begins at event `window_first_eid`:
 * last_update[u] = time of u's last event before the window (0 if none);
 * mem[u][:] ~ U(-0.5, 0.5) for nodes that occurred before the window, else 0.
 */
GEN_API int tig_gen_warm_state(uint64_t seed, int64_t num_nodes, int64_t mem_dim,
                               int64_t window_first_eid, const int32_t *src, const int32_t *dst,
                               const double *ts, float *mem, double *last_update)
{
    if (num_nodes <= 0 || mem_dim <= 0 || window_first_eid < 0 || !src || !dst || !ts || !mem ||
        !last_update)
        return -1;
    uint8_t *seen = (uint8_t *)calloc((size_t)num_nodes, 1);
    if (!seen)
        return -2;
    memset(last_update, 0, sizeof(double) * (size_t)num_nodes);
    for (int64_t e = 0; e < window_first_eid; ++e) { /* ascending: last write wins */
        seen[src[e]] = 1;
        seen[dst[e]] = 1;
        last_update[src[e]] = ts[e];
        last_update[dst[e]] = ts[e];
    }
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < num_nodes; ++u) {
        float *row = mem + (size_t)u * (size_t)mem_dim;
        if (seen[u]) {
            for (int64_t j = 0; j < mem_dim; ++j)
                row[j] = (float)(rnd_u01(seed, STREAM_STATE, (uint64_t)(u * mem_dim + j), 0) - 0.5);
        } else {
            for (int64_t j = 0; j < mem_dim; ++j)
                row[j] = 0.0f;
        }
    }
    free(seen);
    return 0;
}

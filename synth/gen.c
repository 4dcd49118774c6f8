/*
 * Seeded synthetic-input generators: graphs (edge lists -> canonical CSR),
 * dense feature / weight fills, and the fan-out neighbour sampler.
 *
 * This file holds no arithmetic of the GNN layer itself: it only produces the
 * inputs (a sparsity pattern and dense arrays) that both the CPU oracle and
 * the HIP library consume.  All randomness is counter based - value i of a
 * stream is a pure function of (seed, stream, i) - so results do not depend
 * on the number of OpenMP threads.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC gen.c -o libsynth.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ PRNG */

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27; z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

/* random-access splitmix64: key derived from (seed, stream), then element i */
static inline uint64_t stream_key(uint64_t seed, uint64_t stream) {
    return mix64(mix64(seed + 0x9E3779B97F4A7C15ULL) ^ (stream * 0xD1B54A32D192ED03ULL + 0x8CB92BA72F3D8DD7ULL));
}
static inline uint64_t ctr_u64(uint64_t key, uint64_t i) {
    return mix64(key + (i + 1) * 0x9E3779B97F4A7C15ULL);
}
static inline double ctr_unit(uint64_t key, uint64_t i) {            /* [0,1) */
    return (double)(ctr_u64(key, i) >> 11) * (1.0 / 9007199254740992.0);
}

uint64_t synth_hash(uint64_t seed, uint64_t stream, uint64_t i) {
    return ctr_u64(stream_key(seed, stream), i);
}

/* ------------------------------------------------------------ dense fills */

/* out[i] = lo + (hi-lo)*u_i,  u_i uniform in [0,1) */
void synth_fill_uniform(uint64_t seed, uint64_t stream, int64_t n, double lo, double hi, float *out) {
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = (float)(lo + (hi - lo) * ctr_unit(key, (uint64_t)i));
}

static inline double normal_at(uint64_t key, uint64_t i) {
    /* Box-Muller on two counter values; u1 in (0,1] so log() is finite */
    double u1 = ((double)(ctr_u64(key, 2 * i) >> 11) + 1.0) * (1.0 / 9007199254740992.0);
    double u2 = ctr_unit(key, 2 * i + 1);
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
}

void synth_fill_normal(uint64_t seed, uint64_t stream, int64_t n, double mean, double std, float *out) {
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = (float)(mean + std * normal_at(key, (uint64_t)i));
}

/* Rows of a virtual (n_total x f) normal matrix, addressed by global row id:
 * out[t*f + k] = N(mean,std) value number ids[t]*f + k of the stream. */
void synth_fill_normal_rows(uint64_t seed, uint64_t stream, const int32_t *ids, int64_t n_ids, int32_t f,
                            double mean, double std, float *out) {
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_ids; ++t)
        for (int32_t k = 0; k < f; ++k)
            out[t * f + k] = (float)(mean + std * normal_at(key, (uint64_t)ids[t] * (uint64_t)f + (uint64_t)k));
}

/* --------------------------------------------------------- edge generators */

/* R-MAT: draw t picks, at each of `scale` levels, one quadrant with
 * probabilities (a,b,c,1-a-b-c) = (row0col0,row0col1,row1col0,row1col1).
 * Draws whose endpoint falls outside [0,n) or with u==v are marked (-1,-1). */
void synth_rmat_pairs(uint64_t seed, uint64_t stream, int32_t scale, int32_t n, double a, double b, double c,
                      int64_t n_draws, int32_t *u_out, int32_t *v_out) {
    const uint64_t key = stream_key(seed, stream);
    const uint32_t ta = (uint32_t)(a * 4294967296.0);
    const uint32_t tb = (uint32_t)((a + b) * 4294967296.0);
    const uint32_t tc = (uint32_t)((a + b + c) * 4294967296.0);
    const int words = (scale + 1) / 2;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_draws; ++t) {
        uint32_t u = 0, v = 0;
        int lvl = 0;
        for (int w = 0; w < words; ++w) {
            uint64_t h = ctr_u64(key, (uint64_t)t * (uint64_t)words + (uint64_t)w);
            for (int half = 0; half < 2 && lvl < scale; ++half, ++lvl) {
                uint32_t x = (uint32_t)(half ? (h >> 32) : (h & 0xFFFFFFFFULL));
                uint32_t rb, cb;
                if (x < ta) { rb = 0; cb = 0; }
                else if (x < tb) { rb = 0; cb = 1; }
                else if (x < tc) { rb = 1; cb = 0; }
                else { rb = 1; cb = 1; }
                u = (u << 1) | rb;
                v = (v << 1) | cb;
            }
        }
        if (u >= (uint32_t)n || v >= (uint32_t)n || u == v) { u_out[t] = -1; v_out[t] = -1; }
        else { u_out[t] = (int32_t)u; v_out[t] = (int32_t)v; }
    }
}

/* G(n,M): the first m distinct unordered non-loop pairs met when walking the
 * counter stream.  Sequential (open-addressing set); meant for m up to ~1e7.
 * Returns the number of pairs written (== m unless the graph is saturated). */
int64_t synth_gnm_pairs(uint64_t seed, uint64_t stream, int32_t n, int64_t m, int32_t *u_out, int32_t *v_out) {
    const uint64_t key = stream_key(seed, stream);
    if (n < 2 || m <= 0) return 0;
    uint64_t max_pairs = (uint64_t)n * (uint64_t)(n - 1) / 2;
    if ((uint64_t)m > max_pairs) m = (int64_t)max_pairs;
    uint64_t cap = 16;
    while (cap < (uint64_t)m * 2 + 16) cap <<= 1;
    uint64_t *set = (uint64_t *)malloc(cap * sizeof(uint64_t));
    if (!set) return -1;
    memset(set, 0xFF, cap * sizeof(uint64_t));
    int64_t got = 0;
    for (uint64_t t = 0; got < m; ++t) {
        uint64_t h = ctr_u64(key, t);
        uint32_t u = (uint32_t)(((h & 0xFFFFFFFFULL) * (uint64_t)n) >> 32);
        uint32_t v = (uint32_t)(((h >> 32) * (uint64_t)n) >> 32);
        if (u == v) continue;
        if (u > v) { uint32_t s = u; u = v; v = s; }
        uint64_t k = ((uint64_t)u << 32) | v;
        uint64_t p = mix64(k) & (cap - 1);
        int dup = 0;
        while (set[p] != ~0ULL) { if (set[p] == k) { dup = 1; break; } p = (p + 1) & (cap - 1); }
        if (dup) continue;
        set[p] = k;
        u_out[got] = (int32_t)u; v_out[got] = (int32_t)v; ++got;
    }
    free(set);
    return got;
}

/* ------------------------------------------------------------ CSR builder */

static int cmp_i32(const void *x, const void *y) {
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    return (a > b) - (a < b);
}

/* Canonical CSR from an edge list.  Entry (u[t], v[t]) becomes pattern
 * element row u, column v; with symmetrize also row v, column u.  Pairs with
 * a negative endpoint are skipped.  With self_loops, (i,i) is added for every
 * i < min(n_rows,n_cols).  Per row the columns come out strictly ascending
 * (duplicates removed).
 * Two-call protocol: call with col_idx == NULL to get nnz and row_ptr, then
 * again with col_idx of that size.  Returns nnz, or <0 on failure. */
int64_t synth_build_csr(int32_t n_rows, int32_t n_cols, const int32_t *u, const int32_t *v, int64_t m,
                        int symmetrize, int self_loops, int32_t *row_ptr, int32_t *col_idx) {
    int64_t *cnt = (int64_t *)calloc((size_t)n_rows + 1, sizeof(int64_t));
    if (!cnt) return -1;
    for (int64_t t = 0; t < m; ++t) {
        int32_t a = u[t], b = v[t];
        if (a < 0 || b < 0) continue;
        if (a < n_rows && b < n_cols) cnt[a + 1]++;
        if (symmetrize && b < n_rows && a < n_cols) cnt[b + 1]++;
    }
    int32_t nself = 0;
    if (self_loops) {
        nself = n_rows < n_cols ? n_rows : n_cols;
        for (int32_t i = 0; i < nself; ++i) cnt[i + 1]++;
    }
    for (int32_t i = 0; i < n_rows; ++i) cnt[i + 1] += cnt[i];
    int64_t total = cnt[n_rows];
    int32_t *tmp = (int32_t *)malloc((size_t)(total > 0 ? total : 1) * sizeof(int32_t));
    int64_t *pos = (int64_t *)malloc(((size_t)n_rows + 1) * sizeof(int64_t));
    if (!tmp || !pos) { free(cnt); free(tmp); free(pos); return -1; }
    memcpy(pos, cnt, ((size_t)n_rows + 1) * sizeof(int64_t));
    for (int64_t t = 0; t < m; ++t) {
        int32_t a = u[t], b = v[t];
        if (a < 0 || b < 0) continue;
        if (a < n_rows && b < n_cols) tmp[pos[a]++] = b;
        if (symmetrize && b < n_rows && a < n_cols) tmp[pos[b]++] = a;
    }
    for (int32_t i = 0; i < nself; ++i) tmp[pos[i]++] = i;
    /* per-row sort + unique, in place; new length kept in pos[i] */
#pragma omp parallel for schedule(dynamic, 256)
    for (int32_t i = 0; i < n_rows; ++i) {
        int64_t lo = cnt[i], hi = cnt[i + 1];
        qsort(tmp + lo, (size_t)(hi - lo), sizeof(int32_t), cmp_i32);
        int64_t w = lo;
        for (int64_t r = lo; r < hi; ++r)
            if (r == lo || tmp[r] != tmp[r - 1]) tmp[w++] = tmp[r];
        pos[i] = w - lo;
    }
    int64_t nnz = 0;
    for (int32_t i = 0; i < n_rows; ++i) nnz += pos[i];
    if (nnz > 2147483647LL) { free(cnt); free(tmp); free(pos); return -2; }
    row_ptr[0] = 0;
    for (int32_t i = 0; i < n_rows; ++i) row_ptr[i + 1] = row_ptr[i] + (int32_t)pos[i];
    if (col_idx) {
#pragma omp parallel for schedule(dynamic, 256)
        for (int32_t i = 0; i < n_rows; ++i)
            memcpy(col_idx + row_ptr[i], tmp + cnt[i], (size_t)pos[i] * sizeof(int32_t));
    }
    free(cnt); free(tmp); free(pos);
    return nnz;
}

/* ------------------------------------------------------- fan-out sampler */

/* One hop of neighbour sampling on a square CSR `g` (global ids).
 * dst[0..n_dst) are the destination nodes (distinct global ids).  For each,
 * up to `fanout` distinct in-neighbours (columns of its row, the node itself
 * excluded) are drawn uniformly without replacement (Floyd's algorithm on the
 * counter stream); a row with at most `fanout` such neighbours keeps them all.
 * Source nodes are numbered locally: the destinations first, in order, then
 * new nodes in order of first appearance.  Output is a bipartite block in
 * canonical CSR over local column ids, with a self edge (t,t) for each
 * destination t.  src_ids must hold n_dst*(fanout+1) entries, col_idx
 * n_dst*(fanout+1) entries, row_ptr n_dst+1.  Returns n_src (<0 on failure). */
int64_t synth_sample_block(uint64_t seed, uint64_t stream, int32_t n_nodes, const int32_t *g_row_ptr,
                           const int32_t *g_col_idx, const int32_t *dst, int32_t n_dst, int32_t fanout,
                           int32_t *src_ids, int32_t *row_ptr, int32_t *col_idx) {
    const uint64_t key = stream_key(seed, stream);
    int32_t *local = (int32_t *)malloc((size_t)n_nodes * sizeof(int32_t));
    int32_t *pick = (int32_t *)malloc((size_t)(fanout + 1) * sizeof(int32_t));
    if (!local || !pick) { free(local); free(pick); return -1; }
    for (int32_t i = 0; i < n_nodes; ++i) local[i] = -1;
    int64_t n_src = 0;
    for (int32_t t = 0; t < n_dst; ++t) { local[dst[t]] = t; src_ids[n_src++] = dst[t]; }
    row_ptr[0] = 0;
    for (int32_t t = 0; t < n_dst; ++t) {
        int32_t node = dst[t];
        int32_t lo = g_row_ptr[node], hi = g_row_ptr[node + 1];
        /* position of the self entry, if present (columns ascending) */
        int32_t self_pos = -1;
        { int32_t l = lo, h = hi; while (l < h) { int32_t mid = l + (h - l) / 2; if (g_col_idx[mid] < node) l = mid + 1; else h = mid; }
          if (l < hi && g_col_idx[l] == node) self_pos = l; }
        int32_t d = (hi - lo) - (self_pos >= 0 ? 1 : 0);
        int32_t k = d < fanout ? d : fanout;
        int32_t np = 0;
        /* index q in [0,d) -> q-th neighbour skipping the self entry */
        if (d <= fanout) {
            for (int32_t q = 0; q < d; ++q) pick[np++] = q;
        } else {
            for (int32_t j = d - k; j < d; ++j) {
                uint64_t h = ctr_u64(key, (uint64_t)node * 64ULL + (uint64_t)(j - (d - k)));
                int32_t r = (int32_t)(((h >> 32) * (uint64_t)(j + 1)) >> 32);
                int found = 0;
                for (int32_t s = 0; s < np; ++s) if (pick[s] == r) { found = 1; break; }
                pick[np++] = found ? j : r;
            }
        }
        int32_t base = row_ptr[t], w = base;
        col_idx[w++] = t; /* self edge */
        for (int32_t s = 0; s < np; ++s) {
            int32_t p = lo + pick[s];
            if (self_pos >= 0 && p >= self_pos) p += 1;
            int32_t gid = g_col_idx[p];
            if (local[gid] < 0) { local[gid] = (int32_t)n_src; src_ids[n_src++] = gid; }
            col_idx[w++] = local[gid];
        }
        qsort(col_idx + base, (size_t)(w - base), sizeof(int32_t), cmp_i32);
        row_ptr[t + 1] = w;
    }
    free(local); free(pick);
    return n_src;
}

/* CPU checker: see zg_oracle.h.  Test infrastructure only; plain C, one step after the other. */
#include "zg_oracle.h"

#include <stdlib.h>
#include <string.h>

/* ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11).  One round maps (c0,c1,c2,c3) with round key (k0,k1) to
 *   (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0));
 * ten rounds, the key advanced by the Weyl constants between consecutive rounds. ---- */
static const uint32_t PHILOX_M0 = 0xD2511F53u, PHILOX_M1 = 0xCD9E8D57u;
static const uint32_t PHILOX_W0 = 0x9E3779B9u, PHILOX_W1 = 0xBB67AE85u;

void zgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)PHILOX_M0 * c0;
        uint64_t p1 = (uint64_t)PHILOX_M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += PHILOX_W0;
        k1 += PHILOX_W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint64_t zgo_mulhi64(uint64_t a, uint64_t b)
{
    return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

/* Draw for (key, hop, vertex, slot): counter words (vertex, slot, hop, 0), key words (low, high)
 * of the step key; the first two output words make the 64-bit value. */
uint64_t zgo_draw(uint64_t rng_key, int32_t hop, int32_t node, int32_t slot)
{
    uint32_t ctr[4] = {(uint32_t)node, (uint32_t)slot, (uint32_t)hop, 0u};
    uint32_t key[2] = {(uint32_t)(rng_key & 0xFFFFFFFFu), (uint32_t)(rng_key >> 32)};
    uint32_t w[4];
    zgo_philox4x32_10(ctr, key, w);
    return (uint64_t)w[0] | ((uint64_t)w[1] << 32);
}

/* Robert Floyd's algorithm for a uniform F-subset of {0..deg-1} (Bentley & Floyd, "Programming
 * pearls: a sample of brilliance", CACM 1987): for J = deg-F .. deg-1 take t uniform in [0, J];
 * insert t unless it is already in the set, in which case insert J. */
void zgo_floyd_resolve(int64_t deg, int32_t F, const int64_t *t, int64_t *pos)
{
    for (int32_t j = 0; j < F; ++j) {
        int64_t J = deg - F + j;
        int taken = 0;
        for (int32_t i = 0; i < j; ++i)
            if (pos[i] == t[j]) taken = 1;
        pos[j] = taken ? J : t[j];
    }
}

int32_t zgo_sample_positions(uint64_t rng_key, int32_t hop, int32_t node, int64_t deg, int32_t F,
                             int32_t with_replacement, int64_t *pos)
{
    if (deg <= 0 || F <= 0) return 0;
    if (with_replacement) {
        for (int32_t j = 0; j < F; ++j)
            pos[j] = (int64_t)zgo_mulhi64(zgo_draw(rng_key, hop, node, j), (uint64_t)deg);
        return F;
    }
    if (deg <= F) {
        for (int64_t j = 0; j < deg; ++j) pos[j] = j;
        return (int32_t)deg;
    }
    int64_t *t = (int64_t *)malloc(sizeof(int64_t) * (size_t)F);
    if (!t) return -1;
    for (int32_t j = 0; j < F; ++j) {
        int64_t J = deg - F + j;
        t[j] = (int64_t)zgo_mulhi64(zgo_draw(rng_key, hop, node, j), (uint64_t)(J + 1));
    }
    zgo_floyd_resolve(deg, F, t, pos);
    free(t);
    return F;
}

/* ---- helpers ---- */
static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

typedef struct { int32_t gid, local; } id_pair;

static int cmp_pair(const void *a, const void *b)
{
    int32_t x = ((const id_pair *)a)->gid, y = ((const id_pair *)b)->gid;
    return (x > y) - (x < y);
}

static int64_t row_begin(const zgo_graph *g, int64_t v)
{
    return g->offsets_is_i64 ? ((const int64_t *)g->offsets)[v] : (int64_t)((const int32_t *)g->offsets)[v];
}

void zgo_blocks_free(zgo_blocks *b)
{
    if (!b) return;
    free(b->S);
    for (int h = 0; h < ZGO_MAX_HOPS; ++h) {
        free(b->row_ptr[h]);
        free(b->nbr_gid[h]);
        free(b->col[h]);
    }
    memset(b, 0, sizeof(*b));
}

int zgo_sample_blocks(const zgo_graph *g, const int32_t *seeds, int32_t batch, const int32_t *fanouts,
                      int32_t num_hops, uint64_t rng_key, int32_t with_replacement, zgo_blocks *out)
{
    memset(out, 0, sizeof(*out));
    if (!g || !seeds || batch < 1 || num_hops < 1 || num_hops > ZGO_MAX_HOPS) return -1;
    for (int h = 0; h < num_hops; ++h)
        if (fanouts[h] < 1) return -1;

    /* D_0 = seeds in the caller's order; they must be distinct and in range. */
    int64_t n = batch;
    int32_t *S = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *chk = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    if (!S || !chk) { free(S); free(chk); return -2; }
    memcpy(S, seeds, sizeof(int32_t) * (size_t)n);
    memcpy(chk, seeds, sizeof(int32_t) * (size_t)n);
    qsort(chk, (size_t)n, sizeof(int32_t), cmp_i32);
    for (int64_t i = 0; i < n; ++i) {
        if (chk[i] < 0 || chk[i] >= g->num_nodes || (i > 0 && chk[i] == chk[i - 1])) {
            free(S); free(chk);
            return -1;
        }
    }
    free(chk);

    out->num_hops = num_hops;
    out->n[0] = n;
    out->S = S;

    for (int h = 0; h < num_hops; ++h) {
        const int32_t F = fanouts[h];
        /* row lengths k_i = min(F, deg) (with replacement: F when deg > 0) and their running sum */
        int32_t *row_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n + 1));
        if (!row_ptr) { zgo_blocks_free(out); return -2; }
        out->row_ptr[h] = row_ptr;
        row_ptr[0] = 0;
        for (int64_t i = 0; i < n; ++i) {
            int64_t v = S[i];
            int64_t deg = row_begin(g, v + 1) - row_begin(g, v);
            int64_t k = with_replacement ? (deg > 0 ? F : 0) : (deg < F ? deg : F);
            row_ptr[i + 1] = row_ptr[i] + (int32_t)k;
        }
        const int64_t E = row_ptr[n];
        out->E[h] = E;

        /* sampled neighbor ids, slot order within a row */
        int32_t *nbr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
        int32_t *col = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
        int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)F);
        if (!nbr || !col || !pos) { free(nbr); free(col); free(pos); zgo_blocks_free(out); return -2; }
        out->nbr_gid[h] = nbr;
        out->col[h] = col;
        for (int64_t i = 0; i < n; ++i) {
            int64_t v = S[i];
            int64_t begin = row_begin(g, v);
            int64_t deg = row_begin(g, v + 1) - begin;
            int32_t k = zgo_sample_positions(rng_key, h, (int32_t)v, deg, F, with_replacement, pos);
            if (k < 0 || k != row_ptr[i + 1] - row_ptr[i]) { free(pos); zgo_blocks_free(out); return -2; }
            for (int32_t j = 0; j < k; ++j) nbr[row_ptr[i] + j] = g->indices[begin + pos[j]];
        }
        free(pos);

        /* U_h: distinct sampled ids that are not in D_h, ascending */
        int32_t *sortedD = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
        int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E > 0 ? E : 1));
        if (!sortedD || !cand) { free(sortedD); free(cand); zgo_blocks_free(out); return -2; }
        memcpy(sortedD, S, sizeof(int32_t) * (size_t)n);
        qsort(sortedD, (size_t)n, sizeof(int32_t), cmp_i32);
        int64_t nc = 0;
        for (int64_t e = 0; e < E; ++e)
            if (!bsearch(&nbr[e], sortedD, (size_t)n, sizeof(int32_t), cmp_i32)) cand[nc++] = nbr[e];
        free(sortedD);
        qsort(cand, (size_t)nc, sizeof(int32_t), cmp_i32);
        int64_t nu = 0;
        for (int64_t i = 0; i < nc; ++i)
            if (i == 0 || cand[i] != cand[i - 1]) cand[nu++] = cand[i];

        /* S_h = D_h ++ U_h */
        int32_t *S2 = (int32_t *)realloc(S, sizeof(int32_t) * (size_t)(n + nu));
        if (!S2) { free(cand); zgo_blocks_free(out); return -2; }
        S = S2;
        out->S = S;
        memcpy(S + n, cand, sizeof(int32_t) * (size_t)nu);
        free(cand);
        const int64_t n_next = n + nu;

        /* local id = index in S_h */
        id_pair *map = (id_pair *)malloc(sizeof(id_pair) * (size_t)n_next);
        if (!map) { zgo_blocks_free(out); return -2; }
        for (int64_t i = 0; i < n_next; ++i) { map[i].gid = S[i]; map[i].local = (int32_t)i; }
        qsort(map, (size_t)n_next, sizeof(id_pair), cmp_pair);
        for (int64_t e = 0; e < E; ++e) {
            id_pair keyp = {nbr[e], 0};
            const id_pair *hit = (const id_pair *)bsearch(&keyp, map, (size_t)n_next, sizeof(id_pair), cmp_pair);
            col[e] = hit ? hit->local : -1;
        }
        free(map);

        n = n_next;
        out->n[h + 1] = n;
    }
    return 0;
}

void zgo_gather(const float *feat, int64_t ld, int32_t dim, const int32_t *ids, int64_t n, float *X, int64_t ldx)
{
    for (int64_t i = 0; i < n; ++i)
        for (int32_t j = 0; j < dim; ++j)
            X[i * ldx + j] = feat[(int64_t)ids[i] * ld + j];
}

void zgo_aggregate_mean(const int32_t *row_ptr, const int32_t *col, int64_t n_rows, const float *X, int64_t ldx,
                        int32_t dim, float *out, int64_t ldo)
{
    for (int64_t i = 0; i < n_rows; ++i) {
        const int32_t k = row_ptr[i + 1] - row_ptr[i];
        for (int32_t j = 0; j < dim; ++j) {
            double acc = 0.0;
            for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) acc += (double)X[(int64_t)col[e] * ldx + j];
            out[i * ldo + j] = k > 0 ? (float)(acc / (double)k) : 0.0f;
        }
    }
}

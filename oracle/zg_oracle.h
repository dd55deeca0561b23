/*
 * CPU checker for the mini-batch construction path of sampling-based GNN training
 * (multi-hop neighbor sampling -> dedup/relabel -> per-hop block CSR -> feature gather ->
 * mean aggregation; paper sections 2.2 "Sampling-based GNN iteration" and 4.1-4.3).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is plain, single-threaded, slow C
 * that follows the steps one by one with no blocking, fusion or reordering, so it can be
 * read against the paper.  Only tests, the smoke check and the CPU-baseline leg of the
 * benchmark may call it.  It shares no code with the HIP library.
 *
 * Notation: hops h = 0..H-1 counted outward from the seeds; frontier D_h (paper: source set
 * V_s^{h+1}) are the rows of hop h's block, S_h = D_h ++ (new vertices) (paper: destination
 * set V_d^{h+1}) its columns, D_{h+1} = S_h, n_h = |D_h|, E_h = number of sampled edges.
 *
 * The paper fixes the pipeline but not the sampler, the random source, orders or
 * tie-breaks; the readings taken here (each must be matched by the HIP path):
 *   - without replacement: each frontier vertex v gets min(F_h, deg v) distinct neighbor
 *     positions; deg <= F_h takes the whole row in CSR order with no random draw;
 *     otherwise Robert Floyd's subset algorithm, one draw per slot j = 0..F_h-1:
 *       J = deg - F_h + j,  t = floor(x_j * (J+1) / 2^64),  pos_j = (t already chosen) ? J : t
 *     with x_j = w0 | w1 << 32 of Philox4x32-10(counter = (v, j, h, 0), key = (lo32, hi32)
 *     of the 64-bit step key) (Salmon et al., SC'11).
 *   - with replacement (the setting of the paper's Lemma 1): F_h draws whenever deg > 0,
 *     pos_j = floor(x_j * deg / 2^64).
 *   - a row's edges stay in slot order; new vertices (not in D_h) are appended to D_h in
 *     ascending global id; the local id of a vertex is its index in S_h; seeds keep the
 *     caller's order.
 *   - mean over the sampled neighbors only (self excluded), divisor = row length, empty
 *     row -> 0; accumulation in double, result rounded once to float.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors; exhaustive uniformity of the
 * Floyd resolution over every draw sequence of small (deg, F); multiply-high against
 * big-integer arithmetic; sampled ids are true neighbors, positions distinct, row length
 * min(F, deg); S_h duplicate-free with D_h as prefix and an ascending tail; relabel is onto
 * and inverts through S_h; the full-neighborhood case (F >= max degree) equals the BFS ball
 * and the dense row-normalised adjacency product; all-ones features average to exactly 1.
 * The whole pipeline on the benchmark-sized graphs has no printed result in the paper:
 * beyond those invariants it is "parity unpinned".
 */
#ifndef ZG_ORACLE_H
#define ZG_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZGO_MAX_HOPS 8

typedef struct {
    int64_t num_nodes;
    int64_t num_edges;
    const void *offsets;    /* int32 or int64 [num_nodes+1] */
    int32_t offsets_is_i64; /* 0: int32, 1: int64 */
    const int32_t *indices; /* [num_edges] */
} zgo_graph;

typedef struct {
    int32_t num_hops;
    int64_t n[ZGO_MAX_HOPS + 1];       /* n[h] = |D_h|, n[H] = |S_{H-1}| */
    int64_t E[ZGO_MAX_HOPS];           /* sampled edges of hop h */
    int32_t *S;                        /* [n[H]] global ids; D_h is the prefix of length n[h] */
    int32_t *row_ptr[ZGO_MAX_HOPS];    /* [n[h]+1] */
    int32_t *nbr_gid[ZGO_MAX_HOPS];    /* [E[h]] sampled neighbor global ids, slot order */
    int32_t *col[ZGO_MAX_HOPS];        /* [E[h]] local ids (index into S_h) */
} zgo_blocks;

/* Philox4x32-10 block function. */
void zgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* floor(a*b / 2^64). */
uint64_t zgo_mulhi64(uint64_t a, uint64_t b);

/* The 64-bit draw x_j for (step key, hop, vertex, slot). */
uint64_t zgo_draw(uint64_t rng_key, int32_t hop, int32_t node, int32_t slot);

/* Floyd resolution given the per-slot candidates t[j] in [0, deg-F+j]: writes F distinct
 * positions in [0, deg).  Requires deg > F >= 1. */
void zgo_floyd_resolve(int64_t deg, int32_t F, const int64_t *t, int64_t *pos);

/* Neighbor positions of one frontier vertex; returns how many were written (<= F). */
int32_t zgo_sample_positions(uint64_t rng_key, int32_t hop, int32_t node, int64_t deg, int32_t F,
                             int32_t with_replacement, int64_t *pos);

/* Hops 0..H-1 from `seeds` (distinct, in range).  Fills `out` with malloc'ed arrays; release
 * with zgo_blocks_free.  Returns 0, or -1 on invalid input, -2 out of memory. */
int zgo_sample_blocks(const zgo_graph *g, const int32_t *seeds, int32_t batch, const int32_t *fanouts,
                      int32_t num_hops, uint64_t rng_key, int32_t with_replacement, zgo_blocks *out);
void zgo_blocks_free(zgo_blocks *b);

/* X[i,:] = feat[ids[i],:] for i < n (row strides in elements). */
void zgo_gather(const float *feat, int64_t ld, int32_t dim, const int32_t *ids, int64_t n, float *X, int64_t ldx);

/* out[i,:] = mean over e in [row_ptr[i], row_ptr[i+1]) of X[col[e],:]; empty row -> 0. */
void zgo_aggregate_mean(const int32_t *row_ptr, const int32_t *col, int64_t n_rows, const float *X, int64_t ldx,
                        int32_t dim, float *out, int64_t ldo);

#ifdef __cplusplus
}
#endif
#endif

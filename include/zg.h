/*
 * zg - device-resident mini-batch construction for sampling-based GNN training on AMD MI355X.
 *
 * One training iteration's mini-batch construction (paper section 2.2): multi-hop neighbor
 * sampling from a CSR graph, dedup + relabeling of every hop's vertex set, the hop's block
 * CSR, the feature-row gather and a GraphSAGE mean aggregation.  Every count and offset the
 * step produces stays in a device-resident metadata buffer (section 4.1); all kernels run with
 * launch shapes fixed by a capacity envelope provisioned once (sections 4.2, 4.3) and read the
 * true sizes on the device; the step is a captured hipGraph replayed without any host
 * synchronisation (section 4.4).
 *
 * Conventions
 *  - Plain C ABI.  Every function returns 0 (ZG_OK) or a negative zg_status; nothing throws.
 *    zg_last_error() gives a thread-local message for the last failure.
 *  - Pointers named d_* are DEVICE pointers (hipMalloc'ed or a torch CUDA tensor's data_ptr);
 *    all others are HOST pointers.  The library borrows device memory, it never frees it, and
 *    apart from zg_graph_create(ZG_GRAPH_VALIDATE) it never allocates any: the caller
 *    provides one workspace whose size zg_plan_query reports.  zg_plan additionally takes 4 KiB
 *    of pinned host memory (hipHostMalloc) for the per-step mailbox, freed by zg_plan_destroy.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - Hops h = 0..H-1 count outward from the seeds.  D_h (n_h vertices) is the frontier whose
 *    neighbors hop h samples - the rows of block h; S_h = D_h followed by the hop's newly
 *    discovered vertices in ascending global id - the columns of block h; D_{h+1} = S_h.
 *    A vertex's local id is its index in S_{H-1}; every D_h and S_h is a prefix of that list.
 *    (The paper names the mini-batch side of a hop the source set V_s and the sampled side the
 *    destination set V_d.)
 *  - fanouts[h] applies at hop h (fanouts[0] to the seeds).
 *  - The library reads no environment variable; every knob is a field of zg_envelope.
 */
#ifndef ZG_H
#define ZG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZG_MAX_HOPS 8
#define ZG_MAX_FANOUT 64
#define ZG_LOG_STRIDE 32 /* uint32 words per step in the device-side step log */

typedef struct zg_graph_s zg_graph_t;
typedef struct zg_plan_s zg_plan_t;

enum zg_status { ZG_OK = 0, ZG_EINVAL = -1, ZG_ENOMEM = -2, ZG_EHIP = -3, ZG_ESTATE = -4 };
enum zg_dtype { ZG_I32 = 0, ZG_I64 = 1 };

/* zg_graph_create flags */
#define ZG_GRAPH_VALIDATE 1u /* synchronising check: indices in range, rows ascending (hence duplicate-free) */

/* zg_envelope.flags */
#define ZG_PLAN_EAGER 1u   /* launch the step's kernels one by one instead of replaying a hipGraph */
#define ZG_PLAN_REPLACE 2u /* sample with replacement (the setting of the paper's Lemma 1) */
#define ZG_PLAN_FUSED_INPUT 8u /* X holds the rows of the frontier D_{H-1} only and the aggregation reads its input rows
                                 straight from the feature table; the rows that only feed the mean are never written out.
                                 X and agg are then the left and right halves of ONE row-major matrix at d_X, row i =
                                 [X_self(i) | mean(i)] with row stride ldx = ld_agg = 2 * (feat_dim rounded up to 4) and
                                 d_agg = d_X + ldx / 2: the input of the first GraphSAGE layer, ready for one GEMM */
#define ZG_PLAN_SAFE_TWIN 4u /* also provision the worst-case twin of the plan: the paper's "cached safe graph" (section 4.3) */
#define ZG_PLAN_AUTO_FALLBACK 16u /* (brings the twin) the step's captured graph also holds the twin's kernels, behind a
                                 device-side conditional: every workgroup of theirs returns at once unless the plan's own
                                 step raised a hop-overflow bit, in which case they redo the mini-batch on the worst-case
                                 buffers before the graph ends.  The device word zg_outputs.d_active (of zg_plan_outputs)
                                 then reads 1 and the step's valid outputs are those of zg_plan_outputs_safe; otherwise it
                                 reads 0.  A consumer kernel selects its inputs by that word: the host never looks at a
                                 flag.  zg_step_safe is refused on such a plan (ZG_ESTATE). */

#define ZG_PLAN_X_ONE_PASS 32u /* the aggregation reads the feature table and writes the rows of X that belong to the last hop's
                                 newly discovered vertices on the way; the gather copies the frontier's rows only.  This is
                                 what a plan does by default; the flag is kept for callers that state it */
#define ZG_PLAN_X_TWO_PASS 64u /* the gather copies every row of S_{H-1}; the aggregation reads X.  Results are the same
                                 bytes either way */

/* bits of the sticky device status word (zg_overflow_flag) */
#define ZG_FLAG_HOP_OVERFLOW(h) (1u << (h)) /* |S_h| exceeded its cap at hop h: outputs of the step invalid */
#define ZG_FLAG_SEED_RANGE (1u << 16)       /* a seed id outside [0, num_nodes) */
#define ZG_FLAG_SEED_DUP (1u << 17)         /* the same seed twice */
#define ZG_FLAG_INTERNAL (1u << 18)         /* a bounded device-side wait ran out (should never happen) */

enum zg_env_mode {
    ZG_ENV_MAX = 0,      /* worst case n_{h+1} = min(|V|, n_h (1 + F_h)): Eq. 1 applied hop by hop; never overflows */
    ZG_ENV_MODEL = 1,    /* Lemma 1: Poisson-binomial mean/sigma of the deduplicated size from the degree histogram,
                            cap = ceil(max((1 + margin) mean, mean + z sigma)) */
    ZG_ENV_EXPLICIT = 2, /* caller's per-hop vertex caps (e.g. zg_envelope_from_pilot) */
    ZG_ENV_GRAPH = 3     /* the same cap formula as ZG_ENV_MODEL applied to the caller's model_mean / model_sigma
                            (the output of zg_envelope_model_graph) */
};

/* Execution envelope request (section 4.3, "Metadata-Free Dispatcher"). */
typedef struct {
    int32_t mode;       /* zg_env_mode */
    uint32_t flags;     /* ZG_PLAN_* */
    double margin;      /* ZG_ENV_MODEL, ZG_ENV_GRAPH: relative head-room over the model mean; < 0 selects 0.20 (appendix B) */
    double confidence;  /* ZG_ENV_MODEL, ZG_ENV_GRAPH: p of z = Phi^-1(p^(1/m)); <= 0 selects 0.9999 */
    int64_t iterations; /* ZG_ENV_MODEL, ZG_ENV_GRAPH: m; <= 0 selects 1000 */
    int64_t node_caps[ZG_MAX_HOPS + 1]; /* ZG_ENV_EXPLICIT: cap of n_h for h = 1..H ([0] ignored); clamped to the worst case */
    double model_mean[ZG_MAX_HOPS + 1];  /* ZG_ENV_GRAPH: mean of n_h, h = 1..H ([0] ignored) */
    double model_sigma[ZG_MAX_HOPS + 1]; /* ZG_ENV_GRAPH: sigma of n_h */
    int32_t max_tickets; /* tuning knob, <= 0 selects 480: how many workgroups of one launch take a tile id from a shared
                            atomic counter (tiles grow to stay below it; the default is what an MI355X holds at once).
                            Results do not depend on it. */
    int32_t reserved;
} zg_envelope;

/* Host-side answer of zg_plan_query. */
typedef struct {
    int32_t num_hops;
    int32_t feat_dim;
    int64_t node_cap[ZG_MAX_HOPS + 1];    /* capacity of n_h, h = 0..H (node_cap[0] = batch) */
    int64_t edge_cap[ZG_MAX_HOPS];        /* node_cap[h] * fanouts[h] (exact bound) */
    int64_t maxsg_nodes[ZG_MAX_HOPS + 1]; /* worst case per hop (what ZG_ENV_MAX reserves) */
    double model_mean[ZG_MAX_HOPS + 1];   /* Lemma 1 mean of n_h (0 when the graph has no degree statistics) */
    double model_sigma[ZG_MAX_HOPS + 1];  /* Lemma 1 sigma of n_h */
    double z;                             /* Phi^-1(confidence^(1/iterations)) */
    int64_t envelope_bytes;               /* step outputs: S, block CSRs, X, agg, metadata */
    int64_t scratch_bytes;                /* id map over |V|, bitmap, scan state */
    int64_t workspace_bytes;              /* envelope + scratch + alignment: what zg_plan needs */
    int64_t maxsg_envelope_bytes;         /* envelope_bytes if ZG_ENV_MAX had been used */
    int32_t grid_sample[ZG_MAX_HOPS];     /* launch caps (workgroups) of the fixed launch skeleton: hop kernel launch h
                                             (samples hop h; for h > 0 it first ranks the vertices hop h-1 discovered) */
    int32_t grid_compact;                 /* the closing hop-kernel launch (ranks the last hop's vertices, samples nothing) */
    int32_t grid_relabel[ZG_MAX_HOPS];
    int32_t grid_gather;
    int32_t grid_aggregate;
    int64_t safe_envelope_bytes;          /* ZG_PLAN_SAFE_TWIN: bytes of the twin's outputs (part of workspace_bytes), else 0 */
} zg_plan_info;

/* Device addresses of a plan's outputs; fixed for the plan's lifetime (section 4.4, "stable buffers"). */
typedef struct {
    int32_t num_hops;
    int32_t feat_dim;
    const uint32_t *d_n;       /* [H+1] n_h of the last step */
    const uint32_t *d_E;       /* [H]   sampled edges per hop */
    const uint32_t *d_n_exact; /* [H+1] n_h before clamping to the cap */
    const uint32_t *d_flags;   /* sticky status word */
    const int32_t *d_S;        /* [node_cap[H]] global ids; local id = index */
    const int32_t *d_row_ptr[ZG_MAX_HOPS]; /* [node_cap[h]+1] */
    const int32_t *d_nbr_gid[ZG_MAX_HOPS]; /* [edge_cap[h]] sampled neighbor global ids, slot order */
    const int32_t *d_col[ZG_MAX_HOPS];     /* [edge_cap[h]] local ids: block h is (row_ptr, col), n_h x n_{h+1} */
    int64_t node_cap[ZG_MAX_HOPS + 1];
    int64_t edge_cap[ZG_MAX_HOPS];
    const float *d_X;   /* [x_row_cap, ldx] gathered feature rows of S_{H-1} (NULL if feat_dim == 0) */
    int64_t ldx;
    const float *d_agg; /* [node_cap[H-1], ld_agg] mean of block H-1 over X */
    int64_t ld_agg;
    const uint32_t *d_log; /* ring of ZG_LOG_STRIDE-word records, one per step: epoch, flags, n[0..H], E[0..H-1], n_exact[1..H] */
    int32_t log_capacity;  /* records in the ring; record of step e sits at (e % log_capacity) */
    const uint32_t *d_epoch; /* number of steps run on this plan */
    int64_t x_row_cap;       /* rows of d_X: node_cap[H], or node_cap[H-1] with ZG_PLAN_FUSED_INPUT (rows i < n_{H-1} are valid) */
    const uint32_t *d_active; /* ZG_PLAN_AUTO_FALLBACK: 1 if the last step fell back to the twin (its outputs are the valid
                                 ones), else 0; always 0 on other plans */
    int32_t x_one_pass;       /* 1 if, with the feature table bound at the time of the call, the step's aggregation reads the
                                 table and writes the new vertices' rows of X on the way (the default), 0 if the gather copies every
                                 row and the aggregation reads X (ZG_PLAN_X_TWO_PASS, or ZG_PLAN_FUSED_INPUT) */
    int32_t reserved;
} zg_outputs;

/* Fixed text for a zg_status / thread-local detail of the calling thread's last failure.  Both return
 * pointers owned by the library (the second one is valid until the thread's next failing call). */
const char *zg_strerror(int status);
const char *zg_last_error(void);

/* ---- graph ------------------------------------------------------------------------------------
 * CSR as in section 2.1: row v = the neighbor list that is sampled for v (direction is the caller's
 * choice).  d_offsets: [num_nodes+1] int32 or int64 (offsets_dtype); d_indices: [num_edges] int32;
 * num_nodes < 2^31, every degree < 2^31.  Both arrays are borrowed and must outlive the handle.
 * Synchronises (init time): the offsets are read back once to collect the degree statistics the
 * envelope model needs.  ZG_GRAPH_VALIDATE adds a device pass over the indices.
 * Errors: ZG_EINVAL (null pointer, sizes out of range, offsets[0] != 0, offsets[num_nodes] != num_edges,
 * offsets not monotone, validation found an id out of range or a row not strictly ascending), ZG_EHIP
 * (read-back failed), ZG_ENOMEM (host).  *g is NULL on failure. */
int zg_graph_create(zg_graph_t **g, int64_t num_nodes, int64_t num_edges, const void *d_offsets, int32_t offsets_dtype,
                    const int32_t *d_indices, uint32_t flags);
/* A handle that carries degree statistics only (host arrays: distinct degree values and how many
 * vertices have each): enough for zg_plan_query / capacity planning on a machine with no GPU;
 * zg_plan rejects it. */
int zg_graph_create_stats(zg_graph_t **g, int64_t num_nodes, int64_t num_edges, const int64_t *degrees,
                          const int64_t *counts, int64_t n_distinct);
/* Releases the handle (NULL is fine); the device arrays stay the caller's.  Plans made from it must be
 * destroyed first. */
int zg_graph_destroy(zg_graph_t *g);
/* Host pointers owned by the handle. */
int zg_graph_degree_histogram(const zg_graph_t *g, int64_t *n_distinct, const int64_t **degrees, const int64_t **counts);

/* ---- envelope model (host only; Lemma 1 and appendix A) -----------------------------------------
 * Standard normal quantile Phi^-1(p), 0 < p < 1. */
double zg_normal_quantile(double p);
/* Mean and sigma of the deduplicated vertex count after each hop.  With pi_v = deg(v) / sum(deg) and
 * S_h = expected number of neighbor draws up to and including hop h, a vertex is hit with probability
 * p_v = 1 - (1 - pi_v)^{S_h}; mean[h+1] = batch + sum_v p_v, sigma^2 = sum_v p_v (1 - p_v); mean[0] =
 * batch, sigma[0] = 0.  Draws of hop h: every vertex of D_h draws min(F_h, deg) (F_h if deg > 0 with
 * replacement); seeds are uniform over V, later vertices are weighted by their hit probability. */
int zg_envelope_model(const int64_t *degrees, const int64_t *counts, int64_t n_distinct, const int32_t *fanouts,
                      int32_t num_hops, int32_t batch, int32_t with_replacement, double *mean, double *sigma);

/* The same Poisson-binomial frame (the size of D_h as a sum of independent per-vertex indicators, appendix A)
 * with inclusion probabilities taken from the graph instead of the degree-proportional assumption, which is
 * crude when low-degree vertices hang on hubs: with q_u = P(u in D_h) and r_u the chance that a given neighbor
 * of u is among u's picks at hop h (min(F_h, deg)/deg without replacement, 1 - (1 - 1/deg)^{F_h} with),
 * P(v not in D_{h+1}) = (1 - q_v) prod_{u -> v} (1 - q_u r_u); mean[h+1] = sum_v q_v, sigma^2 = sum_v q_v(1 - q_v),
 * mean[0] = batch, sigma[0] = 0.  Runs on the device, one sweep over the edges per hop, and synchronises with
 * `stream` (plan time, once).  d_seed_prob: per-vertex probability of being a seed, fp32 [num_nodes] in device
 * memory, or NULL for uniform seeds (batch / num_nodes).  d_temp: caller's device scratch, 256-byte aligned, at
 * least 12 * num_nodes + 576 bytes; contents undefined afterwards.  The result is deterministic (integer sums).
 * Turn it into caps with ZG_ENV_GRAPH: copy mean / sigma into zg_envelope.model_mean / model_sigma; the planner
 * applies the cap formula of section 4.3 / Lemma 1 (margin and z) to them.
 * Errors: ZG_EINVAL (arguments, buffer), ZG_ESTATE (statistics-only handle, other device), ZG_EHIP. */
int zg_envelope_model_graph(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
                            int32_t with_replacement, const float *d_seed_prob, void *d_temp, size_t temp_bytes,
                            void *stream, double *mean, double *sigma);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): zg_envelope_model_graph without the caller's d_temp.  Its scratch is a static device array of
 * the library (12 bytes per vertex for ZG_STATIC_MODEL_MAX_NODES vertices, 12.6 MB, one copy per GPU, held until
 * the process ends), so graphs with more vertices are refused (ZG_EINVAL).  The call allocates nothing, copies
 * nothing and never synchronises: it enqueues 2 + 2 * num_hops + 1 kernels on `stream` (no memset node) and leaves
 * the result on the device, d_mean_sigma[0..H] = mean[0..H] and d_mean_sigma[H+1..2H+1] = sigma[0..H] (device
 * memory, 2 * (num_hops + 1) doubles, 8-byte aligned, valid once `stream` reaches this point).  Every call on a
 * GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race and give undefined
 * results; calls in stream order are fine, each starts from a clean state.  Same values as
 * zg_envelope_model_graph (integer sums).  Errors: ZG_EINVAL (arguments, too many vertices), ZG_ESTATE
 * (statistics-only handle, other device), ZG_EHIP. */
#define ZG_STATIC_MODEL_MAX_NODES (1 << 20)
int zg_envelope_model_graph_static(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
                                   int32_t with_replacement, const float *d_seed_prob, void *stream, double *d_mean_sigma);

/* Envelope from a pilot run (section 4.4 warm-up iterations; appendix B observes realised sizes within a few
 * percent of each other): `largest[h]`, h = 1..H, is the largest n_h seen over the pilot's mini-batches ([0]
 * ignored).  Fills *out as a ZG_ENV_EXPLICIT request with node_caps[h] = ceil((1 + margin) * largest[h]),
 * margin < 0 selecting 0.20, and the given ZG_PLAN_* flags.  Host only.  Errors: ZG_EINVAL. */
int zg_envelope_from_pilot(const int64_t *largest, int32_t num_hops, double margin, uint32_t flags, zg_envelope *out);

/* ---- plan (section 4.3: one-time provisioning of the execution envelope) ------------------------
 * Host only.  Caps, launch caps and workspace size for (fanouts, batch, envelope, feat_dim);
 * feat_dim = 0 plans the sampling/relabel/CSR part only.  1 <= num_hops <= ZG_MAX_HOPS,
 * 1 <= fanouts[h] <= ZG_MAX_FANOUT, 1 <= batch <= num_nodes, feat_dim <= 32768.
 * Errors: ZG_EINVAL (any of those limits, unknown mode, a hop's edge capacity reaching 2^31),
 * ZG_ESTATE (ZG_ENV_MODEL on a handle without degree statistics). */
int zg_plan_query(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch, const zg_envelope *env,
                  int32_t feat_dim, zg_plan_info *out);
/* Sections 4.1-4.4: lays the device-resident metadata buffer and every step buffer out at fixed addresses
 * inside d_workspace (device memory, 256-byte aligned, >= zg_plan_query's workspace_bytes), initialises the
 * scratch state on `stream`, and captures the step - a fixed launch skeleton sized by the caps - into a
 * hipGraph.  May synchronise.  The workspace belongs to the plan until zg_plan_destroy; the graph handle
 * must outlive the plan; the current device must be the graph's.
 * Errors: those of zg_plan_query, ZG_EINVAL (workspace null or misaligned), ZG_ENOMEM (workspace too small,
 * pinned host memory), ZG_ESTATE (statistics-only graph handle, other device), ZG_EHIP.  *p is NULL on failure. */
int zg_plan(zg_plan_t **p, const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
            const zg_envelope *env, int32_t feat_dim, void *d_workspace, size_t workspace_bytes, void *stream);
/* Waits until the plan's own last step has finished (its completion counter in pinned host memory, then the
 * stream that step was issued on; other plans' streams are left alone), then releases the plan.  If the device
 * does not finish within 30 s the call falls back to hipDeviceSynchronize. */
int zg_plan_destroy(zg_plan_t *p);
/* Makes gather + aggregation (section 2.2, "feature copy" and the first GraphSAGE aggregation) part of the
 * step: d_feat is the [num_nodes, ld] fp32 table in device memory (row stride ld elements, >= feat_dim),
 * borrowed until the plan is destroyed or another table is bound.  Rebuilds the captured graph: call it
 * between steps (nothing of this plan in flight).  Errors: ZG_ESTATE (plan made with feat_dim = 0),
 * ZG_EINVAL (null table, ld < feat_dim), ZG_EHIP. */
int zg_plan_bind_features(zg_plan_t *p, const float *d_feat, int64_t ld);
/* Section 4.4, "stable buffers and inputs": the device addresses the step writes to.  Host only. */
int zg_plan_outputs(const zg_plan_t *p, zg_outputs *out);

/* ---- per step ---------------------------------------------------------------------------------
 * One mini-batch: d_seeds = `batch` distinct vertex ids in device memory (or pinned host memory the
 * device can read), read when the step runs on `stream`; they must stay valid until then.  The call
 * writes (d_seeds, rng_key) into a slot of a small ring in pinned host memory that the step's first
 * kernel reads, and enqueues exactly ONE hipGraph launch - nothing else.  It never synchronises with
 * the device and never allocates; only when 255 earlier steps of this plan are still unfinished does
 * it wait, on the host, for the oldest one (a counter the device publishes in the same pinned ring); that
 * wait is bounded: after 30 s without progress the call returns ZG_ESTATE and enqueues nothing.
 * Results are in the plan's output buffers once `stream` reaches this point.  Steps of one plan must be
 * stream-ordered one after another and issued from one host thread at a time.  Invalid seeds do not fault:
 * they raise ZG_FLAG_SEED_* bits in the device status word and make the step's outputs undefined.
 * Errors: ZG_EINVAL (null), ZG_ESTATE (no captured graph; device made no progress for 30 s), ZG_EHIP (launch
 * failed; nothing was enqueued). */
int zg_step(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream);
/* Stand-alone feature gather (section 2.2, "feature copy") for the vertex list the plan's last step left
 * on the device: d_out[i,:] = d_feat[S[i],:], i < n_H (n_H is read on the device); rows >= n_H of d_out are
 * not written.  d_feat: [num_nodes, ld], d_out: [>= n_H, ld_out], both fp32 device memory, 1 <= dim <= 32768.
 * Enqueues one kernel on `stream`; never synchronises.  Errors: ZG_EINVAL, ZG_EHIP. */
int zg_gather(zg_plan_t *p, const float *d_feat, int64_t ld, int32_t dim, float *d_out, int64_t ld_out, void *stream);
/* Stand-alone GraphSAGE mean aggregation (section 2.2, "subgraph GNN training": the neighbor mean of a layer)
 * on block `hop` of the plan's last step: d_out[i,:] = mean over e in row i of d_in[col[e],:] (0 for an empty
 * row), i < n_hop; d_in: [>= n_{hop+1}, ld_in], d_out: [>= n_hop, ld_out], fp32 device memory.  Any hop works,
 * so deeper layers can aggregate their own activations.  Accumulates in fp32 in edge order.  Enqueues one
 * kernel on `stream`; never synchronises.  Errors: ZG_EINVAL (hop or dim out of range, strides), ZG_EHIP. */
int zg_aggregate_mean(zg_plan_t *p, int32_t hop, const float *d_in, int64_t ld_in, int32_t dim, float *d_out,
                      int64_t ld_out, void *stream);
/* Overflow-safe fallback (section 4.3): replays the same mini-batch on the plan's worst-case twin (needs
 * ZG_PLAN_SAFE_TWIN).  Same contract as zg_step; because the random draws are keyed by (key, hop, vertex,
 * slot), the twin produces exactly what the tight plan would have produced without the overflow.  Its
 * outputs live in the twin's own buffers (zg_plan_outputs_safe); the scratch state is shared, so the call
 * must be stream-ordered with the plan's other steps.  Errors: ZG_ESTATE (no twin, or the plan falls back
 * by itself: ZG_PLAN_AUTO_FALLBACK), otherwise as zg_step. */
int zg_step_safe(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream);
int zg_plan_outputs_safe(const zg_plan_t *p, zg_outputs *out);
/* Host only, no device call: how many steps of this plan have finished, and the ZG_FLAG_* bits the last
 * finished step raised (0 = its outputs are valid).  Both come from pinned host memory that the last kernel
 * of every step writes, so a caller that already knows step k has finished (its own event or sync) can
 * decide about the fallback without reading device memory. */
int zg_step_status(const zg_plan_t *p, uint32_t *steps_completed, uint32_t *last_flags);
/* Pilot bookkeeping (plan time): waits for `stream`, reads the unclamped sizes n_h of the plan's last step and
 * folds them into largest[0..H] by maximum (the caller zeroes the array before the first mini-batch).  Use it
 * on a ZG_ENV_MAX plan and pass the result to zg_envelope_from_pilot.  Synchronises.  Errors: ZG_EINVAL, ZG_EHIP. */
int zg_pilot_update(const zg_plan_t *p, int64_t *largest, void *stream);
/* Section 4.3, "overflow-safe fallback": device address of the plan's sticky status word (ZG_FLAG_* bits
 * accumulate over steps).  The caller reads it when it chooses (async copy + event, end of an epoch).  Host only. */
int zg_overflow_flag(const zg_plan_t *p, const uint32_t **d_flag);
/* Clears the sticky word with a one-lane kernel on `stream` (no memset node: safe under graph capture). */
int zg_overflow_clear(zg_plan_t *p, void *stream);


/* ---- measurement helpers ----------------------------------------------------------------------
 * Identifier of the sources the library was built from (a hash the build step passes in); lets a caller
 * detect a stale binary.  Library-owned string. */
const char *zg_build_id(void);
/* A plain streaming copy d_dst[i] = d_src[i] over `bytes` bytes (a multiple of 16, both pointers 16-byte
 * aligned, device memory), one kernel on `stream`: it reads `bytes` and writes `bytes` of HBM, which calibrates
 * hardware traffic counters read for the library's other kernels.  Errors: ZG_EINVAL, ZG_EHIP. */
int zg_calibration_copy(const void *d_src, void *d_dst, size_t bytes, void *stream);
/* Re-enqueues one of the two feature launches of the plan's step on the state the last step left (section 2.2, "feature
 * copy" and the first GraphSAGE aggregation), as the step runs them and without their small companion roles: which = 0
 * the gather of the frontier's rows into X, which = 1 the mean aggregation that reads its input rows from the feature
 * table and writes the remaining rows of X on the way.  Idempotent (the outputs are rewritten with the same values);
 * meant for timing the step's dominant kernels one by one.  Errors: ZG_EINVAL, ZG_ESTATE (no features bound), ZG_EHIP. */
int zg_plan_replay_features(zg_plan_t *p, int32_t which, void *stream);
/* zg_step with a stop-watch on its dominant kernel: the same step (same outputs, same mailbox and status bookkeeping),
 * its kernels enqueued one by one as a ZG_PLAN_EAGER plan does instead of replaying the captured graph, and the caller's
 * two events (hipEvent_t, created with timing enabled) recorded on `stream` right before and right after the
 * aggregation launch (section 2.2, first GraphSAGE aggregation), so that their distance is that launch's duration
 * inside a real step.  Errors: as zg_step; ZG_ESTATE if no feature table is bound; ZG_EHIP if an event could not be
 * recorded (the step is enqueued all the same and counts as a step of the plan). */
int zg_step_timed(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream, void *event_before, void *event_after);

#ifdef __cplusplus
}
#endif
#endif

// Host side of libzg: error reporting, graph handles and degree statistics, the envelope model
// (paper section 4.3, Lemma 1, appendix A) and the fixed buffer layout / launch caps of a plan.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <map>

#include "zg_internal.h"

namespace zg {

static thread_local std::string g_last_error;

void set_error(const std::string &msg) { g_last_error = msg; }

int fail(int status, const std::string &msg)
{
    set_error(msg);
    return status;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

RowTiling gather_tiling(int32_t dim, bool aligned16)
{
    RowTiling t;
    t.vec = (aligned16 && dim % 4 == 0) ? 4 : 1;
    t.dimv = (uint32_t)(dim / t.vec);
    t.inv = ((1ull << 32) + t.dimv - 1) / t.dimv;
    t.rows = std::max<uint32_t>(1, std::min<uint32_t>(kBlock, 2048u / t.dimv));
    return t;
}

RowTiling aggregate_tiling(int32_t dim, bool aligned16)
{
    RowTiling t = gather_tiling(dim, aligned16);
    // one (row, piece) pair per lane: small workgroups, many of them, hide the staging of the block's edges best
    // (measured at 128- and 600-float rows: 256 pairs per workgroup 86 / 41 us, 512 pairs 91 / 42, 1024 pairs 101 / 44).
    // Filling the lanes better for widths that leave many idle (five 600-float rows = 750 pairs instead of one = 150 of 256
    // lanes) was measured too: the kernel alone gets slower (55 -> 59 us), four plans in flight faster (77 -> 74 us per step),
    // deeper sampling slower again - not kept.
    t.rows = std::max<uint32_t>(1, std::min<uint32_t>(64, 256u / t.dimv));
    return t;
}

// frontier vertices per sampling workgroup: 1024 lanes / (lanes per vertex = power of two >= max(4, fanout))
int sample_group_log2(int fanout)
{
    int g = 2;
    while ((1 << g) < fanout) ++g;
    return g;
}

int64_t sample_tile_nodes(int fanout) { return kHopBlock >> sample_group_log2(fanout); }

// ---- envelope ----------------------------------------------------------------------------------

static int64_t sat_mul_add(int64_t n, int64_t f)
{
    // n * (1 + f) without overflow for the sizes that occur (n < 2^31, f <= 64)
    return n * (1 + f);
}

static int compute_layout_one(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
                              const zg_envelope *env, int32_t feat_dim, zg_plan_info *info, Layout *lay);

// moves a stand-alone layout: outputs to `env_base`, scratch to `scratch_base`
static void relocate(Layout &L, size_t env_base, size_t scratch_base)
{
    const size_t old_scratch = L.envelope_end;
    auto env = [&](size_t &o) { o += env_base; };
    auto scr = [&](size_t &o) { o = scratch_base + (o - old_scratch); };
    env(L.off_drmb);
    env(L.off_log);
    env(L.off_S);
    for (int h = 0; h < L.num_hops; ++h) {
        env(L.off_row_ptr[h]);
        env(L.off_nbr[h]);
        env(L.off_col[h]);
    }
    if (L.feat_dim > 0) {
        env(L.off_X);
        env(L.off_agg);
    }
    env(L.off_own);
    scr(L.off_local_id);
    scr(L.off_bitmap[0]);
    scr(L.off_bitmap[1]);
    scr(L.off_seen);
    scr(L.off_status);
    for (int l = 0; l <= L.num_hops; ++l) {
        scr(L.off_status_cnt[l]);
        scr(L.off_status_edge[l]);
    }
}

int compute_layout(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch, const zg_envelope *env,
                   int32_t feat_dim, zg_plan_info *info, Layout *lay, Layout *lay_safe)
{
    zg_plan_info pi;
    Layout L;
    int rc = compute_layout_one(g, fanouts, num_hops, batch, env, feat_dim, &pi, &L);
    if (rc != ZG_OK) return rc;
    if (env->flags & (ZG_PLAN_SAFE_TWIN | ZG_PLAN_AUTO_FALLBACK)) { // the automatic fallback brings its twin
        zg_envelope worst = *env;
        worst.mode = ZG_ENV_MAX;
        zg_plan_info pis;
        Layout Ls;
        rc = compute_layout_one(g, fanouts, num_hops, batch, &worst, feat_dim, &pis, &Ls);
        if (rc != ZG_OK) return rc;
        // [plan outputs][twin outputs][scratch, sized for the twin (it has the larger scan state)]
        const size_t env_t = L.envelope_end, env_s = Ls.envelope_end;
        const size_t scratch_bytes = Ls.total - Ls.envelope_end;
        relocate(L, 0, env_t + env_s);
        relocate(Ls, env_t, env_t + env_s);
        L.total = Ls.total = env_t + env_s + scratch_bytes;
        pi.safe_envelope_bytes = (int64_t)env_s;
        pi.scratch_bytes = (int64_t)scratch_bytes;
        pi.workspace_bytes = (int64_t)L.total;
        if (lay_safe) *lay_safe = Ls;
    }
    if (info) *info = pi;
    if (lay) *lay = L;
    return ZG_OK;
}

static int compute_layout_one(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
                              const zg_envelope *env, int32_t feat_dim, zg_plan_info *info, Layout *lay)
{
    if (!g || !fanouts || !env) return fail(ZG_EINVAL, "null argument");
    if (num_hops < 1 || num_hops > ZG_MAX_HOPS) return fail(ZG_EINVAL, "num_hops must be in 1..ZG_MAX_HOPS");
    if (batch < 1 || batch > g->num_nodes) return fail(ZG_EINVAL, "batch must be in 1..num_nodes");
    if (feat_dim < 0 || feat_dim > 32768) return fail(ZG_EINVAL, "feat_dim must be in 0..32768");
    for (int h = 0; h < num_hops; ++h)
        if (fanouts[h] < 1 || fanouts[h] > ZG_MAX_FANOUT) return fail(ZG_EINVAL, "fanout must be in 1..ZG_MAX_FANOUT");
    if (env->mode < ZG_ENV_MAX || env->mode > ZG_ENV_GRAPH) return fail(ZG_EINVAL, "unknown envelope mode");
    const bool replace = (env->flags & ZG_PLAN_REPLACE) != 0;
    const int64_t V = g->num_nodes;

    zg_plan_info pi;
    std::memset(&pi, 0, sizeof(pi));
    pi.num_hops = num_hops;
    pi.feat_dim = feat_dim;

    // worst case (Eq. 1 applied hop by hop, the frontier carried along, capped by |V|)
    pi.maxsg_nodes[0] = batch;
    for (int h = 0; h < num_hops; ++h) pi.maxsg_nodes[h + 1] = std::min<int64_t>(V, sat_mul_add(pi.maxsg_nodes[h], fanouts[h]));

    // Lemma 1 statistics (reported in every mode)
    double mean[ZG_MAX_HOPS + 1] = {}, sigma[ZG_MAX_HOPS + 1] = {};
    if (!g->degrees.empty()) {
        int rc = zg_envelope_model(g->degrees.data(), g->counts.data(), (int64_t)g->degrees.size(), fanouts, num_hops, batch,
                                   replace ? 1 : 0, mean, sigma);
        if (rc != ZG_OK) return rc;
    }
    const double conf = env->confidence > 0 ? env->confidence : 0.9999;
    const int64_t iters = env->iterations > 0 ? env->iterations : 1000;
    const double margin = env->margin >= 0 ? env->margin : 0.20;
    if (!(conf > 0.0 && conf < 1.0)) return fail(ZG_EINVAL, "confidence must be in (0,1)");
    pi.z = zg_normal_quantile(std::pow(conf, 1.0 / (double)iters));
    for (int h = 0; h <= num_hops; ++h) { // reported: the statistics the caps were (or would be) derived from
        pi.model_mean[h] = env->mode == ZG_ENV_GRAPH && h > 0 ? env->model_mean[h] : mean[h];
        pi.model_sigma[h] = env->mode == ZG_ENV_GRAPH && h > 0 ? env->model_sigma[h] : sigma[h];
    }

    auto caps_for = [&](int mode, int64_t *node_cap) -> int {
        node_cap[0] = batch;
        for (int h = 0; h < num_hops; ++h) {
            const int64_t worst = std::min<int64_t>(V, sat_mul_add(node_cap[h], fanouts[h]));
            int64_t want = worst;
            if (mode == ZG_ENV_MODEL || mode == ZG_ENV_GRAPH) {
                // section 4.3 / Lemma 1: head-room over the model mean, never less than the z-sigma band; the
                // statistics come from the degree histogram (lemma as printed) or from the caller (graph-aware model)
                if (mode == ZG_ENV_MODEL && g->degrees.empty()) return fail(ZG_ESTATE, "graph handle has no degree statistics");
                const double mu = mode == ZG_ENV_MODEL ? mean[h + 1] : env->model_mean[h + 1];
                const double sg = mode == ZG_ENV_MODEL ? sigma[h + 1] : env->model_sigma[h + 1];
                if (!(mu >= 0.0) || !(sg >= 0.0) || !std::isfinite(mu) || !std::isfinite(sg))
                    return fail(ZG_EINVAL, "model mean / sigma must be finite and non-negative");
                want = (int64_t)std::ceil(std::max((1.0 + margin) * mu, mu + pi.z * sg));
                if (want < 1) want = 1;
            } else if (mode == ZG_ENV_EXPLICIT) {
                want = env->node_caps[h + 1];
                if (want < 1) return fail(ZG_EINVAL, "explicit node cap < 1");
            }
            node_cap[h + 1] = std::max<int64_t>(node_cap[h], std::min<int64_t>(worst, want));
        }
        return ZG_OK;
    };
    int rc = caps_for(env->mode, pi.node_cap);
    if (rc != ZG_OK) return rc;

    const int64_t ldx = feat_dim > 0 ? (int64_t)align_up((size_t)feat_dim, 4) : 0;
    const bool fused = (env->flags & ZG_PLAN_FUSED_INPUT) != 0;
    // tuning knob: upper bound on the tickets (workgroups taking a tile id from one atomic counter) per kernel
    const int64_t max_tickets = env->max_tickets > 0 ? env->max_tickets : kMaxTickets;
    auto envelope_bytes_for = [&](const int64_t *node_cap) -> int64_t {
        size_t b = align_up(sizeof(Drmb), kAlign) + kGuard + align_up((size_t)kLogCapacity * ZG_LOG_STRIDE * 4, kAlign) + kGuard;
        b += align_up((size_t)node_cap[num_hops] * 4, kAlign) + kGuard;
        for (int h = 0; h < num_hops; ++h) {
            b += align_up((size_t)(node_cap[h] + 1) * 4, kAlign) + kGuard;
            b += 2 * (align_up((size_t)node_cap[h] * fanouts[h] * 4, kAlign) + kGuard);
        }
        b += align_up((size_t)node_cap[num_hops - 1] * fanouts[num_hops - 1], kAlign) + kGuard;
        if (feat_dim > 0 && fused) { // one matrix [X_self | mean]
            b += align_up((size_t)node_cap[num_hops - 1] * 2 * ldx * 4, kAlign) + kGuard;
        } else if (feat_dim > 0) {
            b += align_up((size_t)node_cap[num_hops] * ldx * 4, kAlign) + kGuard;
            b += align_up((size_t)node_cap[num_hops - 1] * ldx * 4, kAlign) + kGuard;
        }
        return (int64_t)b;
    };

    Layout L;
    L.num_hops = num_hops;
    L.feat_dim = feat_dim;
    L.ldx = ldx;
    for (int h = 0; h <= num_hops; ++h) L.node_cap[h] = pi.node_cap[h];
    for (int h = 0; h < num_hops; ++h) {
        L.fanout[h] = fanouts[h];
        L.edge_cap[h] = L.node_cap[h] * fanouts[h];
        if (L.edge_cap[h] >= (int64_t)1 << 31) return fail(ZG_EINVAL, "edge capacity of a hop reaches 2^31");
        pi.edge_cap[h] = L.edge_cap[h];
    }
    {
        // Launch l of the hop kernel (l = 0..H) samples hop l for the rows of D_l and, for l > 0, first ranks the vertices
        // hop l-1 discovered.  Rows that were already in D_{l-1} come in tiles of 1024 / G rows, a ticket covering 1..4
        // tiles (every ticket is one atomic on a shared counter, about 15 ns each on MI355X, hence the budget).  The
        // discovered vertices come in ranking tiles: W consecutive words of the hop's bitmap per workgroup, W a power of
        // two chosen so that a tile holds about one sampling pass (1024 / G vertices) of new rows at the cap, within the
        // ticket budget and between 32 and 8192 words.
        const int64_t words = (V + 31) / 32;
        L.bitmap_words = (int64_t)align_up((size_t)words, (size_t)kHopFatTileWords);
        for (int l = 0; l <= num_hops; ++l) {
            // The launch's tickets share one budget: workgroups beyond what the chip holds at once (two of 1024 lanes per
            // compute unit) only start when earlier ones have finished - a second round that doubles the launch's time.
            const int64_t rows = l == 0 ? batch : L.node_cap[l - 1];
            const int64_t T = l < num_hops ? sample_tile_nodes(fanouts[l]) : 256;
            const int64_t fattest_old = l < num_hops ? (rows + 255) / 256 : 0; // old tickets if each took 256 rows
            if (l > 0) {
                const int64_t budget = std::max<int64_t>(std::max<int64_t>(1, max_tickets / 2), max_tickets - fattest_old);
                const int64_t want = std::max<int64_t>(1, std::min<int64_t>(budget, (L.node_cap[l] + T - 1) / T));
                int64_t W = kHopMinTileWords;
                // A launch that samples for few rows over a very long bitmap (its tile count is set by the rows, not by the
                // budget) takes tiles of 16 words per lane: half the tickets, each still about one sampling pass of rows.
                // (At 110 M vertices: 210 instead of 420 tickets in the launch that ranks hop 0's ~9 k discoveries, -2 to -4 %
                // step time; the same for a launch at the ticket budget doubles its rows per ticket and costs +16 %.)
                const int64_t max_words = (l < num_hops && want < budget) ? kHopFatTileWords : kHopMaxTileWords;
                while (W < max_words && W * want < words) W *= 2;
                L.tile_words[l] = (int32_t)W;
                L.rank_tiles[l] = (words + W - 1) / W;
            }
            if (l < num_hops) {
                L.old_tiles[l] = (rows + T - 1) / T;
                L.old_tpt[l] = 1;
                // (a ticket's rows are held in 256 LDS entries)
                while (L.old_tpt[l] < kHopMaxTpt && 2 * L.old_tpt[l] * T <= 256 &&
                       (L.old_tiles[l] + L.old_tpt[l] - 1) / L.old_tpt[l] + L.rank_tiles[l] > max_tickets)
                    L.old_tpt[l] *= 2;
                L.old_tickets[l] = (L.old_tiles[l] + L.old_tpt[l] - 1) / L.old_tpt[l];
            }
        }
    }

    size_t off = 0;
    auto place = [&](size_t bytes) {
        size_t at = off;
        off += align_up(bytes, kAlign) + kGuard;
        return at;
    };
    L.off_drmb = place(sizeof(Drmb));
    L.off_log = place((size_t)kLogCapacity * ZG_LOG_STRIDE * 4);
    L.off_S = place((size_t)L.node_cap[num_hops] * 4);
    for (int h = 0; h < num_hops; ++h) {
        L.off_row_ptr[h] = place((size_t)(L.node_cap[h] + 1) * 4);
        L.off_nbr[h] = place((size_t)L.edge_cap[h] * 4);
        L.off_col[h] = place((size_t)L.edge_cap[h] * 4);
    }
    L.ld_out = ldx;
    if (feat_dim > 0 && fused) {
        // the frontier's own rows and the mean of their sampled neighbors side by side, row i = [X_self(i) | mean(i)]:
        // the input of the first GraphSAGE layer as one row-major matrix
        L.x_rows = L.node_cap[num_hops - 1];
        L.ld_out = 2 * ldx;
        L.off_X = place((size_t)L.x_rows * 2 * ldx * 4);
        L.off_agg = L.off_X + (size_t)ldx * 4;
    } else if (feat_dim > 0) {
        L.x_rows = L.node_cap[num_hops];
        L.off_X = place((size_t)L.x_rows * ldx * 4);
        L.off_agg = place((size_t)L.node_cap[num_hops - 1] * ldx * 4);
    }
    // per edge of the last hop: whether the edge was the hop's first to reach its vertex (the aggregation's cue to copy
    // the vertex's row into X).  Not zero between steps, so it sits with the plan's own buffers, not in the scratch a twin shares.
    L.off_own = place((size_t)L.edge_cap[num_hops - 1]);
    L.envelope_end = off;
    L.off_local_id = place((size_t)V * 4);
    L.off_bitmap[0] = place((size_t)L.bitmap_words * 4); // the bitmap hop h fills is [h & 1]: launch h+1 ranks and clears it
    L.off_bitmap[1] = place((size_t)L.bitmap_words * 4); // while its own sampling fills the other one
    L.off_seen = place((size_t)L.bitmap_words * 4);
    L.status_words = 0;
    for (int l = 0; l <= num_hops; ++l) L.status_words += 2 * ((size_t)L.old_tickets[l] + (size_t)L.rank_tiles[l]);
    L.off_status = place(L.status_words * 8);
    size_t w = 0;
    for (int l = 0; l <= num_hops; ++l) {
        const size_t n = (size_t)L.old_tickets[l] + (size_t)L.rank_tiles[l];
        L.off_status_cnt[l] = L.off_status + w * 8;
        L.off_status_edge[l] = L.off_status + (w + n) * 8;
        w += 2 * n;
    }
    L.total = off;

    pi.envelope_bytes = (int64_t)L.envelope_end;
    pi.scratch_bytes = (int64_t)(L.total - L.envelope_end);
    pi.workspace_bytes = (int64_t)L.total;
    pi.maxsg_envelope_bytes = envelope_bytes_for(pi.maxsg_nodes);
    for (int h = 0; h < num_hops; ++h) {
        pi.grid_sample[h] = (int32_t)(L.old_tickets[h] + L.rank_tiles[h]);
        pi.grid_relabel[h] = (int32_t)((L.edge_cap[h] + kRelabelPerBlock - 1) / kRelabelPerBlock);
    }
    pi.grid_compact = (int32_t)L.rank_tiles[num_hops];
    if (feat_dim > 0) {
        RowTiling tg = gather_tiling(feat_dim, true), ta = aggregate_tiling(feat_dim, true);
        pi.grid_gather = (int32_t)((L.x_rows + tg.rows - 1) / tg.rows);
        pi.grid_aggregate = (int32_t)((L.node_cap[num_hops - 1] + ta.rows - 1) / ta.rows);
    }
    if (info) *info = pi;
    if (lay) *lay = L;
    return ZG_OK;
}

} // namespace zg

using namespace zg;

extern "C" {

const char *zg_strerror(int status)
{
    switch (status) {
    case ZG_OK: return "ok";
    case ZG_EINVAL: return "invalid argument";
    case ZG_ENOMEM: return "workspace too small or out of host memory";
    case ZG_EHIP: return "HIP runtime error";
    case ZG_ESTATE: return "operation not valid in this state";
    default: return "unknown status";
    }
}

const char *zg_last_error(void) { return g_last_error.c_str(); }

double zg_normal_quantile(double p)
{
    // Phi(x) = erfc(-x / sqrt 2) / 2 is monotone: bisect on the lower tail, where erfc keeps its
    // relative accuracy; the upper half follows by symmetry.
    if (!(p > 0.0 && p < 1.0)) return p <= 0.0 ? -std::numeric_limits<double>::infinity() : std::numeric_limits<double>::infinity();
    if (p > 0.5) return -zg_normal_quantile(1.0 - p);
    double lo = -40.0, hi = 0.0;
    for (int it = 0; it < 200; ++it) {
        const double mid = 0.5 * (lo + hi);
        const double cdf = 0.5 * std::erfc(-mid / std::sqrt(2.0));
        if (cdf < p) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

int zg_envelope_model(const int64_t *degrees, const int64_t *counts, int64_t n_distinct, const int32_t *fanouts,
                      int32_t num_hops, int32_t batch, int32_t with_replacement, double *mean, double *sigma)
{
    if (!degrees || !counts || !fanouts || !mean || !sigma || n_distinct < 1 || num_hops < 1 || num_hops > ZG_MAX_HOPS)
        return fail(ZG_EINVAL, "zg_envelope_model: bad argument");
    double V = 0, sumdeg = 0;
    for (int64_t k = 0; k < n_distinct; ++k) {
        if (degrees[k] < 0 || counts[k] < 0) return fail(ZG_EINVAL, "zg_envelope_model: negative degree or count");
        V += (double)counts[k];
        sumdeg += (double)counts[k] * (double)degrees[k];
    }
    if (V <= 0) return fail(ZG_EINVAL, "zg_envelope_model: empty graph");
    auto draws_of = [&](int64_t d, int32_t F) -> double {
        if (with_replacement) return d > 0 ? (double)F : 0.0;
        return (double)std::min<int64_t>(d, F);
    };
    // hit probability of a vertex of degree d after S draws: 1 - (1 - d/sumdeg)^S
    auto hit = [&](int64_t d, double S) -> double {
        if (sumdeg <= 0 || d <= 0 || S <= 0) return 0.0;
        const double pi = (double)d / sumdeg;
        if (pi >= 1.0) return 1.0;
        return -std::expm1(S * std::log1p(-pi));
    };
    mean[0] = batch;
    sigma[0] = 0.0;
    double S = 0.0;
    for (int h = 0; h < num_hops; ++h) {
        double draws = 0.0;
        for (int64_t k = 0; k < n_distinct; ++k) {
            const double c = (double)counts[k];
            // seeds: uniform over V; vertices discovered so far: weighted by their hit probability
            draws += c * draws_of(degrees[k], fanouts[h]) * ((double)batch / V + hit(degrees[k], S));
        }
        S += draws;
        double mu = 0.0, var = 0.0;
        for (int64_t k = 0; k < n_distinct; ++k) {
            const double p = hit(degrees[k], S);
            mu += (double)counts[k] * p;
            var += (double)counts[k] * p * (1.0 - p);
        }
        mean[h + 1] = std::min(V, (double)batch + mu);
        sigma[h + 1] = std::sqrt(var);
    }
    return ZG_OK;
}

int zg_envelope_from_pilot(const int64_t *largest, int32_t num_hops, double margin, uint32_t flags, zg_envelope *out)
{
    if (!largest || !out) return fail(ZG_EINVAL, "null argument");
    if (num_hops < 1 || num_hops > ZG_MAX_HOPS) return fail(ZG_EINVAL, "num_hops must be in 1..ZG_MAX_HOPS");
    const double m = margin >= 0 ? margin : 0.20;
    std::memset(out, 0, sizeof(*out));
    out->mode = ZG_ENV_EXPLICIT;
    out->flags = flags;
    out->margin = m;
    for (int h = 1; h <= num_hops; ++h) {
        if (largest[h] < 0) return fail(ZG_EINVAL, "negative pilot size");
        out->node_caps[h] = std::max<int64_t>(1, (int64_t)std::ceil((1.0 + m) * (double)largest[h]));
    }
    return ZG_OK;
}

static void histogram_from_degrees(const std::vector<int64_t> &deg, zg_graph_t *g)
{
    std::map<int64_t, int64_t> hist;
    int64_t maxd = 0;
    for (int64_t d : deg) maxd = std::max(maxd, d);
    if (maxd < (int64_t)1 << 26) {
        std::vector<int64_t> dense((size_t)maxd + 1, 0);
        for (int64_t d : deg) dense[(size_t)d]++;
        for (int64_t d = 0; d <= maxd; ++d)
            if (dense[(size_t)d]) { g->degrees.push_back(d); g->counts.push_back(dense[(size_t)d]); }
        return;
    }
    for (int64_t d : deg) hist[d]++;
    for (auto &kv : hist) { g->degrees.push_back(kv.first); g->counts.push_back(kv.second); }
}

int zg_graph_create(zg_graph_t **out, int64_t num_nodes, int64_t num_edges, const void *d_offsets, int32_t offsets_dtype,
                    const int32_t *d_indices, uint32_t flags)
{
    if (!out) return fail(ZG_EINVAL, "null handle pointer");
    *out = nullptr;
    if (num_nodes < 1 || num_nodes >= ((int64_t)1 << 31)) return fail(ZG_EINVAL, "num_nodes must be in [1, 2^31)");
    if (num_edges < 0) return fail(ZG_EINVAL, "num_edges < 0");
    if (!d_offsets || (!d_indices && num_edges > 0)) return fail(ZG_EINVAL, "null device pointer");
    if (offsets_dtype != ZG_I32 && offsets_dtype != ZG_I64) return fail(ZG_EINVAL, "offsets_dtype must be ZG_I32 or ZG_I64");
    if (offsets_dtype == ZG_I32 && num_edges >= ((int64_t)1 << 31)) return fail(ZG_EINVAL, "int32 offsets cannot address num_edges");

    zg_graph_t *g = new (std::nothrow) zg_graph_t();
    if (!g) return fail(ZG_ENOMEM, "out of host memory");
    g->num_nodes = num_nodes;
    g->num_edges = num_edges;
    g->d_offsets = d_offsets;
    g->offsets_dtype = offsets_dtype;
    g->d_indices = d_indices;
    {
        const hipError_t e = hipGetDevice(&g->device);
        if (e != hipSuccess) { delete g; return fail(ZG_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e)); }
    }

    // one read-back of the offsets (init time): degree statistics for the envelope model + sanity checks
    std::vector<int64_t> deg((size_t)num_nodes);
    {
        const size_t esz = offsets_dtype == ZG_I64 ? 8 : 4;
        std::vector<char> host((size_t)(num_nodes + 1) * esz);
        hipError_t e = hipMemcpy(host.data(), d_offsets, host.size(), hipMemcpyDeviceToHost);
        if (e != hipSuccess) { delete g; return fail(ZG_EHIP, std::string("reading the offsets back: ") + hipGetErrorString(e)); }
        auto at = [&](int64_t i) -> int64_t {
            return offsets_dtype == ZG_I64 ? ((const int64_t *)host.data())[i] : (int64_t)((const int32_t *)host.data())[i];
        };
        if (at(0) != 0 || at(num_nodes) != num_edges) { delete g; return fail(ZG_EINVAL, "offsets[0] != 0 or offsets[num_nodes] != num_edges"); }
        for (int64_t v = 0; v < num_nodes; ++v) {
            const int64_t d = at(v + 1) - at(v);
            if (d < 0 || d >= ((int64_t)1 << 31)) { delete g; return fail(ZG_EINVAL, "offsets not monotone or a degree reaches 2^31"); }
            deg[(size_t)v] = d;
        }
    }
    histogram_from_degrees(deg, g);
    if (flags & ZG_GRAPH_VALIDATE) {
        int rc = validate_graph_device(g);
        if (rc != ZG_OK) { delete g; return rc; }
    }
    *out = g;
    return ZG_OK;
}

int zg_graph_create_stats(zg_graph_t **out, int64_t num_nodes, int64_t num_edges, const int64_t *degrees, const int64_t *counts,
                          int64_t n_distinct)
{
    if (!out) return fail(ZG_EINVAL, "null handle pointer");
    *out = nullptr;
    if (num_nodes < 1 || num_nodes >= ((int64_t)1 << 31) || !degrees || !counts || n_distinct < 1)
        return fail(ZG_EINVAL, "bad argument");
    int64_t v = 0, e = 0;
    for (int64_t k = 0; k < n_distinct; ++k) {
        if (degrees[k] < 0 || counts[k] < 0) return fail(ZG_EINVAL, "negative degree or count");
        v += counts[k];
        e += counts[k] * degrees[k];
    }
    if (v != num_nodes || e != num_edges) return fail(ZG_EINVAL, "histogram does not add up to num_nodes / num_edges");
    zg_graph_t *g = new (std::nothrow) zg_graph_t();
    if (!g) return fail(ZG_ENOMEM, "out of host memory");
    g->num_nodes = num_nodes;
    g->num_edges = num_edges;
    g->stats_only = true;
    g->degrees.assign(degrees, degrees + n_distinct);
    g->counts.assign(counts, counts + n_distinct);
    *out = g;
    return ZG_OK;
}

int zg_graph_destroy(zg_graph_t *g)
{
    delete g;
    return ZG_OK;
}

int zg_graph_degree_histogram(const zg_graph_t *g, int64_t *n_distinct, const int64_t **degrees, const int64_t **counts)
{
    if (!g || !n_distinct || !degrees || !counts) return fail(ZG_EINVAL, "null argument");
    *n_distinct = (int64_t)g->degrees.size();
    *degrees = g->degrees.data();
    *counts = g->counts.data();
    return ZG_OK;
}

int zg_plan_query(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch, const zg_envelope *env,
                  int32_t feat_dim, zg_plan_info *out)
{
    if (!out) return fail(ZG_EINVAL, "null output");
    return compute_layout(g, fanouts, num_hops, batch, env, feat_dim, out, nullptr);
}

} // extern "C"

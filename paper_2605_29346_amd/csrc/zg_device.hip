// HIP kernels (gfx950, wave64) and the plan / step entry points of libzg.
//
// One step = H+3 launches: the hop kernel's launches 0..H, then {gather + relabel of the last hop} and
// {aggregate + finish}.  Launch l of the hop kernel samples hop l (l < H) and, for l > 0, first ranks the vertices hop
// l-1 discovered - they are rows of block l themselves, so ranking and sampling share their chained scans; launch
// 0 also ingests the seeds and launch l >= 2 relabels the edges of hop l-2 (workgroups of a launch are split by role).
// Every kernel boundary costs about as much as the small kernels themselves at mini-batch sizes, and kernels of
// different streams do not hide it from each other, so the step is cut into as few launches as its global
// dependencies allow: "all of hop l-1 sampled" before its vertices can be ranked, and "all vertices ranked" before
// the features move.
// Every kernel is launched with a grid fixed by the plan's capacity envelope, reads the true sizes
// from the device-resident metadata buffer and lets surplus workgroups return at once (paper
// sections 4.1-4.3).  The whole step is one hipGraph (section 4.4); the step's seeds pointer and key reach it
// through a mailbox in pinned host memory.
// A plan may carry a worst-case twin (the paper's "cached safe graph", section 4.3) that replays a mini-batch
// whose sizes overflowed the envelope, on the host's request or - its kernels appended to the step's graph
// behind a device-side gate - by itself.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>

#include "zg_floyd.h"
#include "zg_internal.h"

namespace zg {

// =================================================================================================
// device helpers
// =================================================================================================
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr uint64_t kStAggregate = 1ull << 62; // tile total published
constexpr uint64_t kStPrefix = 2ull << 62;    // inclusive prefix published
constexpr uint64_t kStValueMask = (1ull << 62) - 1;
constexpr uint32_t kSpinLimit = 1u << 22;     // bounded wait: polls before giving up with ZG_FLAG_INTERNAL

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += (uint64_t)__shfl_xor((unsigned long long)v, d, 64);
    return v;
}

__device__ __forceinline__ void st_store(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint64_t st_load(uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Single-pass chained scan across workgroups: ticket `tile` (tickets are handed out in start order, so every
// predecessor is already running) publishes its total and then looks back over the predecessors' status words until
// it meets a published inclusive prefix.  A status word carries state (2 bits) and value (62 bits) together, so one
// relaxed 64-bit access is enough.  One wavefront looks back, 64 predecessors per round (sharing a look-back among
// eight wavefronts so that one round covers 512 predecessors was measured: no faster - the wait is for the
// predecessors to publish, not for the rounds - and eight times the polling).  The wait is bounded; when it runs out
// the step is flagged invalid (sticky and per-step word) and a clamped value is used.
__device__ __forceinline__ uint64_t lookback_round(uint64_t *status, int64_t base, Drmb *d, int lane, bool &found)
{
    // the 64 status words base, base-1, .. base-63 (indices below zero count as an inclusive prefix of zero)
    const int64_t idx = base - lane;
    uint64_t st;
    uint32_t spins = 0;
    for (;;) {
        st = idx >= 0 ? st_load(&status[idx]) : kStPrefix;
        const bool invalid = (st >> 62) == 0;
        if (!__any(invalid)) break;
        if (++spins > kSpinLimit) {
            if (lane == 0) { // the step's outputs are invalid: both the sticky and the per-step word say so
                atomicOr(&d->flags, ZG_FLAG_INTERNAL);
                atomicOr(&d->step_flags, ZG_FLAG_INTERNAL);
            }
            if (invalid) st = kStAggregate;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    const unsigned long long pm = __ballot((st >> 62) == 2);
    const uint64_t val = st & kStValueMask;
    found = pm != 0ull;
    if (pm) {
        const int first = __ffsll((long long)pm) - 1;
        return wave_sum64(lane <= first ? val : 0ull);
    }
    return wave_sum64(val);
}

// all 64 lanes of one wavefront: publish, then look back 64 at a time
__device__ uint64_t chained_exclusive_prefix(uint64_t *status, uint32_t tile, uint64_t total, Drmb *d, int lane)
{
    if (lane == 0) st_store(&status[tile], (tile == 0 ? kStPrefix : kStAggregate) | total);
    uint64_t excl = 0;
    if (tile > 0) {
        int64_t base = (int64_t)tile - 1;
        for (;;) {
            bool found;
            excl += lookback_round(status, base, d, lane, found);
            if (found) break;
            base -= 64;
        }
        if (lane == 0) st_store(&status[tile], kStPrefix | ((excl + total) & kStValueMask));
    }
    return excl;
}

// Philox4x32-10 (Salmon et al., SC'11) for counter (node, slot, hop, 0) and the 64-bit step key;
// returns the first two output words as one 64-bit draw.
__device__ __forceinline__ uint64_t philox_draw(uint32_t key_lo, uint32_t key_hi, uint32_t hop, uint32_t node, uint32_t slot)
{
    uint32_t c0 = node, c1 = slot, c2 = hop, c3 = 0u;
    uint32_t k0 = key_lo, k1 = key_hi;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        c0 = h1 ^ c1 ^ k0;
        c1 = l1;
        c2 = h0 ^ c3 ^ k1;
        c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return (uint64_t)c0 | ((uint64_t)c1 << 32);
}

// The G lanes of a wavefront that hold the slots of one frontier vertex, as the group interface of
// floyd_position (zg_floyd.h): slot j of the group sits in lane gbase + j.
struct WaveGroup {
    int gbase;
    __device__ __forceinline__ uint32_t candidate_of(uint32_t j, uint32_t mine) const { return __shfl(mine, gbase + (int)j, 64); }
    __device__ __forceinline__ bool flag_of(uint32_t j, bool mine) const { return __shfl((int)mine, gbase + (int)j, 64) != 0; }
    __device__ __forceinline__ bool any(bool b) const { return __any(b) != 0; }
};

// =================================================================================================
// kernels
// =================================================================================================
// Per-step inputs travel through a ring in pinned host memory that the device reads directly: the captured
// graph's arguments are frozen, and a step must be exactly one graph launch.  The host writes slot
// (steps issued % kMailboxSlots) before it launches the graph; the ingest kernel of step number e (the
// device-side step counter) reads slot e % kMailboxSlots; the last kernel of a step publishes e + 1 in
// `completed`, which the host checks (no device synchronisation) before it reuses a slot.
struct Mailbox {
    uint32_t completed;
    uint32_t issued; // steps the host has handed over so far (their slots are filled)
    uint32_t pad[2];
    uint32_t status[kMailboxSlots]; // ZG_FLAG_* bits raised by the step that used the slot
    struct {
        unsigned long long seeds; // device address of the step's seed ids
        unsigned long long key;   // step key
    } slot[kMailboxSlots];
};

// Device-side conditional of the overflow-safe fallback (paper section 4.3): the worst-case twin's kernels sit
// behind the plan's own in the same captured graph and every one of their workgroups returns at once unless
// the plan's step raised a hop-overflow bit - a fixed launch skeleton whose surplus work exits early, like
// the over-provisioned grids of section 4.2.  `gate` is the plan's metadata buffer (null: always run).
constexpr uint32_t kHopOverflowMask = 0xFFFFu;
__device__ __forceinline__ bool gate_closed(const Drmb *gate)
{
    return gate != nullptr && (gate->last_flags & kHopOverflowMask) == 0u;
}

struct IngestArgs {
    Drmb *drmb;
    const Drmb *gate;       // gated twin: the step's inputs are those of the gate owner's step that has just finished
    const Mailbox *mailbox; // the mailbox the inputs are read from (the gate owner's when gated)
    int32_t *S;
    int32_t *local_id;
    uint32_t *seen;
    uint32_t batch;
    uint32_t num_nodes;
    uint32_t blocks; // workgroups given to this role (0: role absent)
};

// The step's (seeds pointer, key).  A read of the pinned-host mailbox costs the device several microseconds, at the head
// of the step's dependency chain; when the host runs ahead of the device - the normal case in a training loop - the
// previous step has already copied this step's slot into the metadata buffer (prefetch_step_inputs) and the read
// stays in device memory.  Otherwise: the mailbox slot of the device-side step counter.
__device__ __forceinline__ void read_step_inputs(const Drmb *d, const Drmb *gate, const Mailbox *mailbox, unsigned long long *out)
{
    if (!gate && d->pre_valid && d->pre_epoch == d->epoch) {
        out[0] = d->pre_seeds;
        out[1] = d->pre_key;
        return;
    }
    const uint32_t slot = (gate ? gate->epoch - 1u : d->epoch) % kMailboxSlots;
    out[0] = __hip_atomic_load(&mailbox->slot[slot].seeds, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    out[1] = __hip_atomic_load(&mailbox->slot[slot].key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Step entry ("ingest"): seeds -> D_0 (caller's order), their local ids and "seen" bits; step key and batch size ->
// metadata buffer.  Out-of-range seeds are replaced by -1 (a vertex with no neighbors); a seed whose "seen" bit
// is already set is a duplicate.  Shares its launch with the sampling of hop 0, which reads the seeds itself.
__device__ __forceinline__ void ingest_block(const IngestArgs &a, uint32_t block, unsigned long long *s_in)
{
    const uint32_t gtid = block * blockDim.x + threadIdx.x;
    if (threadIdx.x == 0) read_step_inputs(a.drmb, a.gate, a.mailbox, s_in); // one read of the host-resident slot per workgroup
    __syncthreads();
    const int32_t *seeds = reinterpret_cast<const int32_t *>(s_in[0]);
    if (gtid == 0) {
        Drmb *d = a.drmb;
        d->n[0] = a.batch;
        d->n_exact[0] = a.batch;
        d->key_lo = (uint32_t)(s_in[1] & 0xFFFFFFFFull);
        d->key_hi = (uint32_t)(s_in[1] >> 32);
    }
    if (gtid < a.batch) {
        int32_t v = seeds[gtid];
        if ((uint32_t)v >= a.num_nodes) {
            atomicOr(&a.drmb->flags, ZG_FLAG_SEED_RANGE);
            atomicOr(&a.drmb->step_flags, ZG_FLAG_SEED_RANGE);
            v = -1;
        } else {
            const uint32_t bit = 1u << (v & 31);
            const uint32_t old = atomicOr(&a.seen[(uint32_t)v >> 5], bit);
            if (old & bit) {
                atomicOr(&a.drmb->flags, ZG_FLAG_SEED_DUP);
                atomicOr(&a.drmb->step_flags, ZG_FLAG_SEED_DUP);
            }
            a.local_id[v] = (int32_t)gtid;
        }
        a.S[gtid] = v;
    }
}

struct RelabelArgs {
    const Drmb *drmb;
    const Drmb *gate; // consulted by the gather launch (the hop kernel has its own)
    const int32_t *nbr;
    const int32_t *local_id;
    int32_t *col;
    uint32_t num_nodes;
    int32_t hop;
    uint32_t blocks; // workgroups given to this role (0: role absent)
};

// Hop h, "relabel edges": col[e] = local id of nbr_gid[e] (-1 for a vertex dropped by an overflow).
// Every sampled id is in S_h, so its map entry was written during this step (by the ingest or a ranking tile).
// Works for any workgroup size; a workgroup covers kRelabelPerBlock edges.
__device__ __forceinline__ void relabel_block(const RelabelArgs &a, uint32_t block)
{
    const uint32_t E = a.drmb->E[a.hop];
    const uint32_t e0 = block * kRelabelPerBlock;
    if (e0 >= E) return;
    const uint32_t e1 = e0 + kRelabelPerBlock < E ? e0 + kRelabelPerBlock : E;
#pragma unroll 4
    for (uint32_t e = e0 + threadIdx.x; e < e1; e += blockDim.x) {
        const int32_t g = a.nbr[e];
        a.col[e] = (uint32_t)g < a.num_nodes ? a.local_id[g] : -1;
    }
}

struct RowArgs {
    const float *src;       // gather: feature table; aggregate: input rows
    float *dst;
    const int32_t *S;       // gather: global ids of the rows to copy
    const int32_t *row_ptr; // aggregate
    const int32_t *col;     // aggregate: per edge, the index of its input row (local ids, or global ids: see n_cols)
    const uint32_t *n_rows; // device address of the row count
    const uint32_t *n_cols; // aggregate: device address of the number of valid input rows, or null if `col_limit` holds it
    uint32_t col_limit;     // aggregate: number of valid input rows when n_cols is null (num_nodes for global ids)
    float *x_dst;           // aggregate reading the table: X, whose rows of newly discovered vertices it writes on the way (or null)
    const int32_t *x_row;   // ... per edge, the row of X (the local id)
    const uint8_t *own;     // ... per edge, whether this edge is the one that writes it
    int64_t ld_x;
    int64_t ld_src, ld_dst;
    uint64_t inv;
    uint32_t dimv;
    uint32_t rows;
    uint32_t max_fanout;
    int32_t vec4;           // rows are moved in 16-byte pieces (else element by element)
    int32_t nt;             // aggregate inside a step: what it writes (means, rows of X) is stored past the caches (non-temporal)
    const int32_t *local_id; // aggregate that relabels its block's edges itself: the id map ...
    int32_t *col_out;        // ... and where col[e] = local id of nbr_gid[e] goes (null: `x_row` holds it already)
    uint32_t blocks; // workgroups given to this role (0: role absent)
};

template <int VEC> struct VecOf;
template <> struct VecOf<4> {
    typedef v4f type;
    static __device__ __forceinline__ v4f zero() { return (v4f){0.0f, 0.0f, 0.0f, 0.0f}; }
};
template <> struct VecOf<1> {
    typedef float type;
    static __device__ __forceinline__ float zero() { return 0.0f; }
};

// "Gather": X[i,:] = feat[S[i],:].  A workgroup copies `rows` consecutive output rows; lanes walk the rows
// as one flat run of 16-byte pieces so that rows whose length is not a multiple of the wave width still
// fill every lane, four loads in flight per lane before the stores.
template <int VEC, bool STREAM, bool NT_STORE = false>
__device__ __forceinline__ void gather_rows(const RowArgs &a, uint32_t row0, uint32_t rows, const int32_t *s_id)
{
    typedef typename VecOf<VEC>::type T;
    const uint32_t total = rows * a.dimv;
    for (uint32_t e0 = threadIdx.x; e0 < total; e0 += 4 * blockDim.x) {
        T val[4];
        uint32_t r[4], c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = e0 + u * blockDim.x;
            if (e < total) {
                r[u] = (uint32_t)(((uint64_t)e * a.inv) >> 32);
                c[u] = e - r[u] * a.dimv;
                const int32_t g = s_id[r[u]];
                const T *src = reinterpret_cast<const T *>(a.src + (int64_t)g * a.ld_src + (int64_t)c[u] * VEC);
                val[u] = g >= 0 ? (STREAM ? __builtin_nontemporal_load(src) : *src) : VecOf<VEC>::zero();
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t e = e0 + u * blockDim.x;
            if (e < total) {
                T *dst = reinterpret_cast<T *>(a.dst + (int64_t)(row0 + r[u]) * a.ld_dst + (int64_t)c[u] * VEC);
                if (STREAM || NT_STORE)
                    __builtin_nontemporal_store(val[u], dst);
                else
                    *dst = val[u];
            }
        }
    }
}

// "Gather": X[i,:] = feat[S[i],:].  A workgroup copies `rows` consecutive output rows; lanes walk the rows
// as one flat run of 16-byte pieces so that rows whose length is not a multiple of the wave width still
// fill every lane, four loads in flight per lane before the stores.  When the gathered matrix of this step
// is larger than the caches can hold for the aggregation that follows (decided on the device from the true
// row count), loads and stores are non-temporal: measured +15 % at 200 MB, -10 % at 90 MB.
// the same for a launch that copies the frontier's rows only (never large enough for the non-temporal path)
template <int VEC>
__device__ __forceinline__ void gather_rows_block(const RowArgs &a, uint32_t block, int32_t *s_id)
{
    const uint32_t n = *a.n_rows;
    const uint32_t row0 = block * a.rows;
    if (row0 >= n) return;
    const uint32_t rows = n - row0 < a.rows ? n - row0 : a.rows;
    if (threadIdx.x < rows) s_id[threadIdx.x] = a.S[row0 + threadIdx.x];
    __syncthreads();
    gather_rows<VEC, false, true>(a, row0, rows, s_id); // nothing in the step reads these rows of X again: stored past the caches
}

template <int VEC>
__device__ __forceinline__ void gather_block(const RowArgs &a, uint32_t block, int32_t *s_id)
{
    const uint32_t n = *a.n_rows;
    const uint32_t row0 = block * a.rows;
    if (row0 >= n) return;
    const uint32_t rows = n - row0 < a.rows ? n - row0 : a.rows;
    if (threadIdx.x < rows) s_id[threadIdx.x] = a.S[row0 + threadIdx.x];
    __syncthreads();
    if ((uint64_t)n * a.dimv * (VEC * 4) > kGatherStreamBytes)
        gather_rows<VEC, true>(a, row0, rows, s_id);
    else
        gather_rows<VEC, false>(a, row0, rows, s_id);
}

// Launch l = 0..H of the hop kernel: it samples hop l for the rows of D_l (l < H) and, for l > 0, first ranks the
// vertices that hop l-1 discovered (they are the rows of D_l that D_{l-1} did not have).
struct HopArgs {
    const void *offsets;
    const int32_t *indices;
    Drmb *drmb;
    const Drmb *gate;
    const Mailbox *mailbox;   // launch 0 reads the step's inputs itself (the gate owner's mailbox when gated)
    int32_t *S;
    int32_t *local_id;
    uint32_t *bitmap_prev;    // launches 1..H: the bitmap hop l-1 filled; ranked, consumed and cleared here
    uint32_t *bitmap_next;    // launches 0..H-1: the bitmap this launch's sampling fills
    uint32_t *seen;
    int32_t *row_ptr;         // block of hop l (launches 0..H-1)
    int32_t *nbr;
    uint8_t *own;             // last hop, when the aggregation writes X: per edge, whether it was the first to reach its vertex
    uint64_t *status_cnt;     // chained scan over the launch's tickets: vertices ranked ...
    uint64_t *status_edge;    // ... and edges sampled
    uint32_t num_nodes;
    int32_t launch;           // l
    int32_t num_hops;         // H
    int32_t fanout;
    int32_t group_log2;       // lanes per row: 2^group_log2 >= max(4, fanout)
    int32_t replace;
    uint32_t tiles_per_ticket; // consecutive tiles of old rows per ticket
    uint32_t cap_rows;        // capacity of n_l
    uint32_t edge_cap;        // capacity of E_l
    uint32_t words_per_tile;  // ranking tile (a power of two, 32..8192)
    uint32_t rank_tiles;      // 0 for launch 0
    uint32_t batch;
    uint32_t blocks;          // workgroups of this role (the launch's first ones)
};

// LDS of a hop-kernel workgroup: up to 256 rows of the block being sampled (vertex, degree, first edge offset, row
// length, first edge position), the dedup set of one sampling pass, scan scratch
constexpr int kHopRows = 256;
struct HopShared {
    uint32_t ticket;
    uint32_t base_cnt;
    unsigned long long base_edge;
    unsigned long long in[2];
    uint32_t wsum[kHopBlock / 64];
    uint32_t wk[4];
    int32_t v[kHopRows];
    uint32_t deg[kHopRows], k[kHopRows], rp[kHopRows];
    unsigned long long off[kHopRows];
    uint32_t set[kSampleHashSlots];
};

// One sampling pass over rows row0 .. row0 + 1024/G - 1 of the workgroup's LDS rows: lane (t, j) takes slot j of row
// row0 + t (vertex sh.v, degree sh.deg, sh.k slots, first edge position sh.rp): j itself if deg <= F, else Floyd's
// subset algorithm with one Philox draw per slot, all slots resolved at once (zg_floyd.h); with replacement one draw
// per slot.  The lane loads the neighbor id and stores it to nbr_gid (consecutive lanes, consecutive addresses).
// Dedup starts here: the ids go through a hash set in LDS so that each distinct id of the pass reaches the hop's bitmap
// with at most one device-scope atomic - popular vertices are sampled hundreds of times per hop and same-address atomics
// serialise at the memory side.  Ids that are already in D_l reach the bitmap too: the next launch masks it with "seen"
// (looking every id up in "seen" here was measured: one more dependent random load per edge, slower on every workload).
__device__ __forceinline__ void sample_pass(const HopArgs &a, HopShared &sh, uint32_t key_lo, uint32_t key_hi, uint32_t row0, int tid,
                                            int lane)
{
    const int glog = a.group_log2;
    const uint32_t F = (uint32_t)a.fanout;
    const int G = 1 << glog;
    const int gl = lane & (G - 1);
    const int gbase = lane & ~(G - 1);
    const uint32_t t = row0 + ((uint32_t)tid >> glog);
    const int32_t tv = sh.v[t];
    const uint32_t tdeg = sh.deg[t], tk = sh.k[t], trp = sh.rp[t];
    const unsigned long long toff = sh.off[t];
    const bool slot = (uint32_t)gl < tk;
    uint32_t pos = (uint32_t)gl;
    if (a.replace) {
        if (slot) pos = (uint32_t)__umul64hi(philox_draw(key_lo, key_hi, (uint32_t)a.launch, (uint32_t)tv, (uint32_t)gl), (uint64_t)tdeg);
    } else {
        const bool floyd = slot && tdeg > F;
        if (__any(floyd)) {
            uint32_t cand = (uint32_t)gl;
            if (floyd)
                cand = (uint32_t)__umul64hi(philox_draw(key_lo, key_hi, (uint32_t)a.launch, (uint32_t)tv, (uint32_t)gl),
                                            (uint64_t)(tdeg - F + (uint32_t)gl) + 1ull);
            WaveGroup grp{gbase};
            pos = floyd_position(grp, (uint32_t)gl, F, tdeg, floyd, cand);
        }
    }
    if (slot && trp + (uint32_t)gl < a.edge_cap) {
        const int32_t g = a.indices[toff + pos];
        a.nbr[trp + (uint32_t)gl] = g;
        if ((uint32_t)g < a.num_nodes) {
            // first lane of the pass to insert g into the LDS set marks it (at most 1024 insertions into 2048 slots)
            uint32_t h = ((uint32_t)g * 2654435761u) >> (32 - kSampleHashBits);
            bool first = false;
            for (;;) {
                const uint32_t old = atomicCAS(&sh.set[h], 0xFFFFFFFFu, (uint32_t)g);
                if (old == 0xFFFFFFFFu) {
                    first = true;
                    break;
                }
                if (old == (uint32_t)g) break;
                h = (h + 1) & (kSampleHashSlots - 1);
            }
            // The one atomic that finds the bit clear belongs to the first edge of the hop to reach the vertex.  For the last
            // hop that edge is remembered: the aggregation reads the vertex's feature row for it anyway and, if the vertex
            // turns out to be new, copies the row into X on the way (any one edge would do: they all carry the same row).
            bool mine = false;
            if (first) {
                const uint32_t bit = 1u << (g & 31);
                if (a.own)
                    mine = (atomicOr(&a.bitmap_next[(uint32_t)g >> 5], bit) & bit) == 0u;
                else
                    atomicOr(&a.bitmap_next[(uint32_t)g >> 5], bit);
            }
            if (a.own) a.own[trp + (uint32_t)gl] = mine ? 1 : 0;
        } else if (a.own) {
            a.own[trp + (uint32_t)gl] = 0;
        }
    }
}

// "Row lengths" of the workgroup's LDS rows: lanes 0..255 take the vertex sh.v[tid] (-1 beyond `nrows`), load its two
// offsets, and leave degree, first edge offset and k = min(F, deg) (F whenever deg > 0 with replacement) in LDS.
// Returns this lane's k.
template <typename OffT>
__device__ __forceinline__ uint32_t load_rows(const HopArgs &a, HopShared &sh, uint32_t nrows, int tid)
{
    if (tid >= kHopRows) return 0u;
    const int32_t v = (uint32_t)tid < nrows ? sh.v[tid] : -1;
    uint32_t deg = 0;
    unsigned long long off0 = 0;
    if (v >= 0) {
        const OffT *off = (const OffT *)a.offsets;
        const OffT o0 = off[v], o1 = off[v + 1];
        off0 = (unsigned long long)o0;
        deg = (uint32_t)(o1 - o0);
    }
    const uint32_t F = (uint32_t)a.fanout;
    const uint32_t k = a.replace ? (deg > 0 ? F : 0u) : (deg < F ? deg : F);
    sh.v[tid] = v;
    sh.deg[tid] = deg;
    sh.off[tid] = off0;
    sh.k[tid] = k;
    return k;
}

// the lowest q set bits of x
__device__ __forceinline__ uint32_t lowest_set_bits(uint32_t x, uint32_t q)
{
    uint32_t out = 0;
    while (x && q) {
        const uint32_t low = x & (0u - x);
        out |= low;
        x ^= low;
        --q;
    }
    return out;
}

// The hop kernel.  A workgroup of 1024 lanes takes a ticket; tickets are handed out in start order, so every ticket a
// workgroup ever waits for belongs to a workgroup that already runs.  In ticket order the launch's work is the row
// order of block l:
//   tickets 0 .. t_old-1   rows that were already in D_{l-1} (launch 0: the seeds), up to 256 per ticket;
//   then the ranking tiles of hop l-1's bitmap, W words each, in ascending vertex id: the bits that are not "seen"
//                          are the hop's new vertices; their rank - n_{l-1} plus the new vertices before them - is
//                          their local id and their row in block l, so they land behind D_{l-1} in ascending id.
// Two single-pass chained scans run over the tickets (status word = state + value, bounded wait): new vertices and
// sampled edges.  A ticket first finds its rows' lengths k_i = min(F, deg) ("row lengths"; 256 rows at a time, held in
// LDS), publishes both totals, takes its exclusive prefixes (wavefront 0 and wavefront 1, side by side), and then
// writes S, the id map and row_ptr ("offsets scan") and samples its rows in passes of 1024 / G rows, one lane per
// (row, slot) ("sample").  A ranking tile holds its bitmap words in registers (up to WPL per lane: 8, or 16 in the
// instantiation for sparse launches over very long bitmaps), adds the kept
// bits to "seen" and clears the words.  Vertices ranked beyond the cap are dropped (no row, local id -1, not "seen")
// and the hop's overflow bit is raised; the rows kept are a prefix of the row order, so the block stays consistent up
// to the cap.  Launch H ranks only.  The launch's surplus workgroups (the grid is sized by the caps) find no ticket
// and return.
template <typename OffT, int WPL>
__global__ __launch_bounds__(kHopBlock, 8) void k_hop(HopArgs a, RelabelArgs rel, IngestArgs ing, RowArgs gat)
{
    __shared__ HopShared sh;
    if (gate_closed(a.gate)) return;
    // Roles by workgroup index.  The closing launch may carry the copy of the frontier's feature rows (their ids are final
    // by now): its copy workgroups alternate with the ticket workgroups at the head of the grid, so that the copy - bound by
    // bandwidth - runs while the tickets - chains of dependent accesses - wait, instead of after them (tickets are handed
    // out in start order, whichever workgroups ask).  Then the remaining tickets, the relabel and ingest roles, the
    // remaining copy workgroups.
    {
        uint32_t b = blockIdx.x;
        const uint32_t pairs = a.blocks < gat.blocks ? a.blocks : gat.blocks; // (0 without the copy role)
        bool ticket_role;
        uint32_t copy_block = 0xFFFFFFFFu;
        if (b < 2u * pairs) {
            ticket_role = (b & 1u) == 0u;
            if (!ticket_role) copy_block = b >> 1;
        } else {
            b -= 2u * pairs;
            ticket_role = b < a.blocks - pairs;
            if (!ticket_role) {
                b -= a.blocks - pairs;
                if (b < rel.blocks) {
                    relabel_block(rel, b);
                    return;
                }
                b -= rel.blocks;
                if (b < ing.blocks) {
                    ingest_block(ing, b, sh.in);
                    return;
                }
                copy_block = pairs + (b - ing.blocks);
            }
        }
        if (!ticket_role) {
            if (gat.vec4)
                gather_rows_block<4>(gat, copy_block, sh.v);
            else
                gather_rows_block<1>(gat, copy_block, sh.v);
            return;
        }
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    Drmb *d = a.drmb;
    const bool first = a.launch == 0, sampling = a.launch < a.num_hops;
    if (tid == 0) sh.ticket = atomicAdd(&d->ticket[a.launch], 1u);
    if (first && tid == 64) read_step_inputs(d, a.gate, a.mailbox, sh.in);
    const uint32_t n_old = first ? a.batch : d->n[a.launch - 1]; // (in flight while the ticket comes back)
    const uint32_t key_lo_d = d->key_lo, key_hi_d = d->key_hi;
    __syncthreads();
    const uint32_t ticket = sh.ticket;
    const uint32_t T = (uint32_t)kHopBlock >> a.group_log2;  // rows per sampling pass, 16..256
    const uint32_t R = T * a.tiles_per_ticket;               // old rows per ticket, <= 256
    const uint32_t t_old = sampling ? (n_old + R - 1) / R : 0u;
    const uint32_t n_tickets = t_old + a.rank_tiles;
    if (ticket >= n_tickets) return;
    const bool old = ticket < t_old; // uniform over the workgroup
    const uint32_t key_lo = first ? (uint32_t)(sh.in[1] & 0xFFFFFFFFull) : key_lo_d;
    const uint32_t key_hi = first ? (uint32_t)(sh.in[1] >> 32) : key_hi_d;

    // ---- what this ticket's rows are
    uint32_t m;                       // rows of this ticket: old rows, or the tile's new vertices
    uint32_t lex = 0;                 // ranking tile: in-tile index of this lane's first new vertex
    uint32_t nw[WPL]; // ranking tile: this lane's new vertices (bitmap bits that are not "seen")
    uint32_t had = 0;                 // ... and which of its bitmap words were not empty
    const uint32_t r0 = ticket * R;   // old rows: the first row
    const uint32_t W = a.words_per_tile;
    const uint32_t wpl = W >= (uint32_t)kHopBlock ? W / (uint32_t)kHopBlock : 1u;
    const size_t w0 = old ? 0 : (size_t)(ticket - t_old) * W + (size_t)tid * wpl; // ranking tile: this lane's first word
#pragma unroll
    for (uint32_t r = 0; r < WPL; ++r) nw[r] = 0u;
    if (old) {
        m = n_old - r0 < R ? n_old - r0 : R;
    } else {
        const bool owner = W >= (uint32_t)kHopBlock || (uint32_t)tid < W;
        // the lane's words of the hop's bitmap, then - only where a word is not empty - the same words of "seen"
        // (wide loads: a lane's words are consecutive)
        auto load_words = [&](const uint32_t *src, uint32_t (&x)[WPL]) {
            if (wpl >= 4) {
#pragma unroll
                for (uint32_t q = 0; q < (uint32_t)WPL / 4u; ++q)
                    if (4u * q < wpl) {
                        const uint4 p = *reinterpret_cast<const uint4 *>(src + w0 + 4u * q);
                        x[4 * q] = p.x, x[4 * q + 1] = p.y, x[4 * q + 2] = p.z, x[4 * q + 3] = p.w;
                    }
            } else if (wpl == 2) {
                const uint2 p = *reinterpret_cast<const uint2 *>(src + w0);
                x[0] = p.x, x[1] = p.y;
            } else {
                x[0] = src[w0];
            }
        };
        if (owner) load_words(a.bitmap_prev, nw);
#pragma unroll
        for (uint32_t r = 0; r < WPL; ++r)
            if (nw[r]) had |= 1u << r;
        if (had) {
            if (wpl >= 4) {
#pragma unroll
                for (uint32_t q = 0; q < (uint32_t)WPL / 4u; ++q)
                    if (4u * q < wpl && ((had >> (4u * q)) & 0xFu)) {
                        const uint4 sn = *reinterpret_cast<const uint4 *>(a.seen + w0 + 4u * q);
                        nw[4 * q] &= ~sn.x, nw[4 * q + 1] &= ~sn.y, nw[4 * q + 2] &= ~sn.z, nw[4 * q + 3] &= ~sn.w;
                    }
            } else if (wpl == 2) {
                const uint2 sn = *reinterpret_cast<const uint2 *>(a.seen + w0);
                nw[0] &= ~sn.x, nw[1] &= ~sn.y;
            } else {
                nw[0] &= ~a.seen[w0];
            }
        }
        uint32_t cnt = 0;
#pragma unroll
        for (uint32_t r = 0; r < WPL; ++r) cnt += __popc(nw[r]);
        const uint32_t incl = wave_incl_scan(cnt, lane);
        if (lane == 63) sh.wsum[wave] = incl;
        __syncthreads();
        lex = incl - cnt;
        m = 0;
#pragma unroll
        for (int w = 0; w < kHopBlock / 64; ++w) {
            if (w < wave) lex += sh.wsum[w];
            m += sh.wsum[w];
        }
        __syncthreads(); // sh.wsum is used again below
    }

    // rows c0 .. c0 + 255 of the ticket into sh.v: old rows from the frontier list (launch 0: the seeds, an
    // out-of-range one becoming -1, a vertex without neighbors), new vertices expanded from the lane's bitmap words
    auto fill_rows = [&](uint32_t c0) {
        if (old) {
            if (tid < kHopRows && (uint32_t)tid < m) {
                int32_t v = first ? reinterpret_cast<const int32_t *>(sh.in[0])[r0 + tid] : a.S[r0 + tid];
                if (first && (uint32_t)v >= a.num_nodes) v = -1;
                sh.v[tid] = v;
            }
        } else {
            const uint32_t c1 = c0 + kHopRows;
            uint32_t j = lex;
#pragma unroll
            for (uint32_t r = 0; r < WPL; ++r) {
                uint32_t x = nw[r];
                const uint32_t pc = __popc(x);
                if (j + pc <= c0 || j >= c1) { // all before this batch, or this batch is full: nothing to write
                    j += pc;
                    continue;
                }
                while (x) {
                    const int b = __ffs((int)x) - 1;
                    x &= x - 1u;
                    if (j >= c0 && j < c1) sh.v[j - c0] = (int32_t)((((uint32_t)w0 + r) << 5) + (uint32_t)b);
                    ++j;
                }
            }
        }
        __syncthreads();
    };

    // ---- row lengths, 256 rows at a time; their total goes into the edge chain
    const uint32_t supers = sampling ? (m + kHopRows - 1) / kHopRows : 0u;
    uint64_t ticket_edges = 0;
    if (sampling) {
        uint32_t ksum = 0;
        for (uint32_t q = 0; q < supers; ++q) {
            const uint32_t c0 = q * kHopRows;
            fill_rows(c0);
            ksum += load_rows<OffT>(a, sh, m - c0 < (uint32_t)kHopRows ? m - c0 : (uint32_t)kHopRows, tid);
            if (q + 1 < supers) __syncthreads(); // the next fill overwrites sh.v
        }
        if (wave < 4) {
            const uint32_t ws = wave_sum(ksum);
            if (lane == 0) sh.wk[wave] = ws;
        }
        __syncthreads();
        ticket_edges = (uint64_t)sh.wk[0] + sh.wk[1] + sh.wk[2] + sh.wk[3];
    }
    // ---- both chains, side by side: wavefront 0 looks back over the new-vertex counts, wavefront 1 over the edge
    // counts.  Old rows hold no new vertex: their count chain entry is an inclusive prefix at once.
    if (wave == 0) {
        if (old) {
            if (lane == 0) st_store(&a.status_cnt[ticket], kStPrefix);
        } else {
            const uint64_t r = chained_exclusive_prefix(a.status_cnt, ticket, (uint64_t)m, d, lane);
            if (lane == 0) sh.base_cnt = (uint32_t)r;
        }
    }
    if (wave == 1 && sampling) {
        const uint64_t e = chained_exclusive_prefix(a.status_edge, ticket, ticket_edges, d, lane);
        if (lane == 0) sh.base_edge = e;
    }
    __syncthreads();
    const uint32_t rank0 = old ? r0 : n_old + sh.base_cnt;                       // row index of the ticket's first row
    const uint32_t room = rank0 < a.cap_rows ? a.cap_rows - rank0 : 0u;          // how many of its rows fit (old rows: all)
    uint64_t ebase = sampling ? sh.base_edge : 0ull;

    if (sampling) {
        // ---- offsets scan + sample, 256 rows at a time.  A single batch of rows is still in LDS from above; several
        // are redone (their loads hit the cache).
        for (uint32_t q = 0; q < supers; ++q) {
            const uint32_t c0 = q * kHopRows;
            const uint32_t nrows = m - c0 < (uint32_t)kHopRows ? m - c0 : (uint32_t)kHopRows;
            const uint32_t keep = room > c0 ? (room - c0 < nrows ? room - c0 : nrows) : 0u;
            if (supers > 1) {
                fill_rows(c0);
                (void)load_rows<OffT>(a, sh, nrows, tid);
            }
            uint32_t k = 0, kincl = 0;
            if (wave < 4) {
                k = (uint32_t)tid < keep ? sh.k[tid] : 0u; // dropped rows sample nothing
                kincl = wave_incl_scan(k, lane);
                if (lane == 63) sh.wsum[wave] = kincl;
            }
            __syncthreads();
            uint32_t total = 0;
            if (wave < 4) {
                uint32_t wbase = 0;
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    if (w < wave) wbase += sh.wsum[w];
                const uint32_t rp = (uint32_t)ebase + wbase + kincl - k;
                sh.k[tid] = k;
                sh.rp[tid] = rp;
                if ((uint32_t)tid < keep) {
                    a.row_ptr[rank0 + c0 + tid] = (int32_t)rp;
                    if (!old) {
                        const int32_t gid = sh.v[tid];
                        a.S[rank0 + c0 + tid] = gid;
                        a.local_id[gid] = (int32_t)(rank0 + c0 + tid);
                    }
                } else if ((uint32_t)tid < nrows) {
                    a.local_id[sh.v[tid]] = -1;
                }
            }
            total = sh.wsum[0] + sh.wsum[1] + sh.wsum[2] + sh.wsum[3];
            ebase += total;
            for (uint32_t row0 = 0; row0 < keep; row0 += T) {
                for (int x = tid; x < kSampleHashSlots; x += kHopBlock) sh.set[x] = 0xFFFFFFFFu;
                __syncthreads();
                sample_pass(a, sh, key_lo, key_hi, row0, tid, lane);
                __syncthreads(); // the set is reset by the next pass, the LDS rows are reused by the next batch
            }
        }
    } else {
        // ---- closing launch: ranks only
        uint32_t j = lex;
#pragma unroll
        for (uint32_t r = 0; r < WPL; ++r) {
            uint32_t x = nw[r];
            while (x) {
                const int b = __ffs((int)x) - 1;
                x &= x - 1u;
                const int32_t gid = (int32_t)((((uint32_t)w0 + r) << 5) + (uint32_t)b);
                if (j < room) {
                    a.S[rank0 + j] = gid;
                    a.local_id[gid] = (int32_t)(rank0 + j);
                } else {
                    a.local_id[gid] = -1;
                }
                ++j;
            }
        }
    }

    if (old) {
        if (first && ticket == t_old - 1 && tid == 0) { // launch 0 has no ranking tiles: the block ends with these rows
            a.row_ptr[n_old] = (int32_t)ebase;
            d->E[a.launch] = (uint32_t)ebase;
        }
        return;
    }

    // ---- the kept vertices join "seen" (not after the last hop: nothing is sampled from them), consumed words are
    // cleared for the hop after next; this lane is the only writer of its words during the launch
    if (had) {
        uint32_t left = lex < room ? room - lex : 0u; // how many of this lane's vertices are kept
#pragma unroll
        for (uint32_t r = 0; r < WPL; ++r)
            if (had & (1u << r)) {
                const uint32_t pc = __popc(nw[r]);
                if (sampling && nw[r]) {
                    const uint32_t keep = left >= pc ? nw[r] : lowest_set_bits(nw[r], left);
                    if (keep) __hip_atomic_fetch_or(&a.seen[w0 + r], keep, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); // no value comes back: nothing to wait for
                }
                left = left >= pc ? left - pc : 0u;
                a.bitmap_prev[w0 + r] = 0u;
            }
    }

    // ---- end of the block: the tile in which the cap falls closes a truncated block; the last ticket publishes the
    // hop's sizes and, when everything fitted, closes the block
    if (tid == 0) {
        if (sampling && rank0 <= a.cap_rows && (uint64_t)rank0 + m > a.cap_rows) {
            a.row_ptr[a.cap_rows] = (int32_t)ebase;
            d->E[a.launch] = (uint32_t)ebase;
        }
        if (ticket == n_tickets - 1) {
            const uint64_t exact = (uint64_t)rank0 + m;
            d->n_exact[a.launch] = (uint32_t)exact;
            d->n[a.launch] = exact < a.cap_rows ? (uint32_t)exact : a.cap_rows;
            if (exact > a.cap_rows) {
                atomicOr(&d->flags, ZG_FLAG_HOP_OVERFLOW(a.launch - 1));
                atomicOr(&d->step_flags, ZG_FLAG_HOP_OVERFLOW(a.launch - 1));
            } else if (sampling) {
                a.row_ptr[exact] = (int32_t)ebase;
                d->E[a.launch] = (uint32_t)ebase;
            }
        }
    }
}

struct FinishArgs {
    Drmb *drmb;
    const Drmb *gate;       // gated twin: the plan whose step this launch ends
    Mailbox *gate_mailbox;  // ... and its mailbox: the step counts as completed only now
    int32_t defer_completed; // plan with a gated twin behind it: leave `completed` to the twin's last launch
    Mailbox *mailbox;
    const int32_t *S;
    uint32_t *seen;
    uint32_t *log;
    uint64_t *status;       // the chained scans' status words of every launch: back to zero for the next step
    uint64_t status_words;
    int32_t num_hops;
    uint32_t blocks; // workgroups given to this role (0: role absent)
};

// End of step: the "seen" words of this step's frontier vertices (everything in D_{H-1}: the seeds and
// what hops 0..H-2 added) go back to zero - the bitmaps over |V| are never cleared as a whole -, the scan
// state (status words, tile tickets) restarts for the next step, and the step is appended to the device-side
// log; the step counter advances.
// last launch of a step that carries a gated twin: the owner's step is complete whether or not the twin ran
__device__ __forceinline__ void publish_gate_owner(const FinishArgs &a)
{
    __hip_atomic_store(&a.gate_mailbox->completed, a.gate->epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// One lane, early in the step's last launch: if the host has already handed over the next step, its mailbox slot is
// copied into the metadata buffer, so that the next step starts without a read of host memory.
__device__ __forceinline__ void prefetch_step_inputs(Drmb *d, const Mailbox *mailbox)
{
    const uint32_t next = d->epoch + 1u;
    const uint32_t issued = __hip_atomic_load(&mailbox->issued, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
    if ((int32_t)(issued - (next + 1u)) >= 0) {
        const uint32_t slot = next % kMailboxSlots;
        d->pre_seeds = __hip_atomic_load(&mailbox->slot[slot].seeds, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        d->pre_key = __hip_atomic_load(&mailbox->slot[slot].key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        d->pre_epoch = next;
        d->pre_valid = 1u;
    } else {
        d->pre_valid = 0u;
    }
}

__device__ __forceinline__ void finish_block(const FinishArgs &a, uint32_t block)
{
    const uint32_t n = a.drmb->n[a.num_hops - 1];
    const uint32_t i = block * kBlock + threadIdx.x;
    if (i < n) {
        const int32_t g = a.S[i];
        if (g >= 0) a.seen[(uint32_t)g >> 5] = 0u;
    }
    for (uint64_t w = i; w < a.status_words; w += (uint64_t)a.blocks * kBlock) a.status[w] = 0ull;
    if (i == 0) {
        Drmb *d = a.drmb;
        for (int l = 0; l <= a.num_hops; ++l) d->ticket[l] = 0u;
        const uint32_t epoch = d->epoch;
        uint32_t *rec = a.log + (size_t)(epoch % kLogCapacity) * ZG_LOG_STRIDE;
        int p = 0;
        rec[p++] = epoch;
        rec[p++] = d->step_flags;
        for (int h = 0; h <= a.num_hops; ++h) rec[p++] = d->n[h];
        for (int h = 0; h < a.num_hops; ++h) rec[p++] = d->E[h];
        for (int h = 1; h <= a.num_hops; ++h) rec[p++] = d->n_exact[h];
        d->epoch = epoch + 1;
        const uint32_t step_flags = d->step_flags;
        d->last_flags = step_flags;
        d->step_flags = 0; // for the next step: its first kernel raises seed bits from many lanes, so nobody resets there
        d->active = (step_flags & kHopOverflowMask) != 0u && a.defer_completed ? 1u : 0u;
        __hip_atomic_store(&a.mailbox->status[epoch % kMailboxSlots], step_flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (!a.defer_completed)
            __hip_atomic_store(&a.mailbox->completed, epoch + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        if (a.gate) publish_gate_owner(a);
    }
}

// "Mean-aggregate": out[i,:] = (1/k_i) * sum over row i of in[col[e],:].  A workgroup owns `rows` output
// rows; their row_ptr slice and input-row indices are staged in LDS, then each lane owns one (row, 16-byte
// column piece) pair at a time and accumulates over the row's edges in fp32, in edge order.
// Inside a step the input rows are read from the feature table (addressed by the sampled global ids: feat[nbr_gid[e]]
// is what X[col[e]] holds) and the rows of X that belong to the last hop's newly discovered vertices are written here,
// by the edge that claimed the vertex: the row passes through the registers once instead of being copied by the
// gather and read back from X (at one reference per row, a third less memory traffic for gather + aggregation).
// the lanes' loop of the aggregation: one (row, 16-byte column piece) pair at a time.  ONE_PASS: the input rows come from
// the feature table and the edge that claimed a newly discovered vertex copies the piece into X on the way.  NT: X is
// stored past the caches (nothing reads it again within the step); the table's rows are loaded through them, so that a
// row several edges share comes from memory once
template <int VEC, bool ONE_PASS, bool NT>
__device__ __forceinline__ void aggregate_rows(const RowArgs &a, uint32_t row0, uint32_t rows, int32_t e_begin, uint32_t e_count,
                                               const int32_t *s_rp, const int32_t *s_col, const int32_t *s_dst)
{
    typedef typename VecOf<VEC>::type T;
    const uint32_t total = rows * a.dimv;
    for (uint32_t e = threadIdx.x; e < total; e += kBlock) {
        const uint32_t r = (uint32_t)(((uint64_t)e * a.inv) >> 32);
        const uint32_t c = e - r * a.dimv;
        const uint32_t b = (uint32_t)(s_rp[r] - e_begin);
        uint32_t k = (uint32_t)(s_rp[r + 1] - s_rp[r]);
        if (b + k > e_count) k = b < e_count ? e_count - b : 0;
        T acc = VecOf<VEC>::zero();
        // eight of the row's edges at a time: all their loads are in flight before the first is added (in edge order)
        for (uint32_t j0 = 0; j0 < k; j0 += 8) {
            int32_t cj[8];
            T v[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) cj[u] = j0 + u < k ? s_col[b + j0 + u] : -1;
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                v[u] = VecOf<VEC>::zero();
                if (cj[u] >= 0) {
                    const T *src = reinterpret_cast<const T *>(a.src + (int64_t)cj[u] * a.ld_src + (int64_t)c * VEC);
                    v[u] = *src;
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u)
                if (cj[u] >= 0) {
                    acc += v[u];
                    if (ONE_PASS) { // the hop's first edge to a new vertex copies the piece into X on the way
                        const int32_t dj = s_dst[b + j0 + u];
                        if (dj >= 0) {
                            T *xd = reinterpret_cast<T *>(a.x_dst + (int64_t)dj * a.ld_x + (int64_t)c * VEC);
                            if (NT)
                                __builtin_nontemporal_store(v[u], xd);
                            else
                                *xd = v[u];
                        }
                    }
                }
        }
        const T res = k > 0 ? acc / (float)k : VecOf<VEC>::zero();
        T *out = reinterpret_cast<T *>(a.dst + (int64_t)(row0 + r) * a.ld_dst + (int64_t)c * VEC);
        if (NT) // (the step does not read the means again either)
            __builtin_nontemporal_store(res, out);
        else
            *out = res;
    }
}

template <int VEC>
__device__ __forceinline__ void aggregate_block(const RowArgs &a, uint32_t block, int32_t *s_mem)
{
    int32_t *s_rp = s_mem;               // [rows+1]
    int32_t *s_col = s_mem + a.rows + 1; // [rows * max_fanout]
    int32_t *s_dst = s_col + a.rows * a.max_fanout; // [rows * max_fanout] when X is written on the way: row of X, or -1
    const uint32_t n = *a.n_rows;
    const uint32_t n_in = a.n_cols ? *a.n_cols : a.col_limit;
    const uint32_t row0 = block * a.rows;
    if (row0 >= n) return;
    const uint32_t rows = n - row0 < a.rows ? n - row0 : a.rows;
    for (uint32_t t = threadIdx.x; t <= rows; t += kBlock) s_rp[t] = a.row_ptr[row0 + t];
    __syncthreads();
    const int32_t e_begin = s_rp[0];
    uint32_t e_count = (uint32_t)(s_rp[rows] - e_begin);
    if (e_count > a.rows * a.max_fanout) e_count = a.rows * a.max_fanout;
    for (uint32_t t = threadIdx.x; t < e_count; t += kBlock) { // input row of every edge, -1 = none
        const uint32_t c = (uint32_t)a.col[e_begin + t];
        const bool valid = c < n_in;
        s_col[t] = valid ? (int32_t)c : -1;
        int32_t lid = -1;
        if (a.col_out) { // "relabel edges" of this block, done here: c is the sampled global id
            lid = valid ? a.local_id[c] : -1;
            a.col_out[e_begin + t] = lid;
        } else if (a.x_dst) {
            lid = a.x_row[e_begin + t];
        }
        // the hop's first edge to a vertex writes its row of X, if the vertex is new (the frontier's rows are the gather's)
        if (a.x_dst) s_dst[t] = (valid && a.own[e_begin + t] && lid >= (int32_t)n) ? lid : -1;
    }
    __syncthreads();
    if (a.x_dst)
        aggregate_rows<VEC, true, true>(a, row0, rows, e_begin, e_count, s_rp, s_col, s_dst);
    else if (a.nt)
        aggregate_rows<VEC, false, true>(a, row0, rows, e_begin, e_count, s_rp, s_col, s_dst);
    else
        aggregate_rows<VEC, false, false>(a, row0, rows, e_begin, e_count, s_rp, s_col, s_dst);
}

// The two bandwidth-bound launches of a step, each with a small companion role on its last workgroups:
// {gather + relabel of the last hop}, then {aggregation + end-of-step clean-up}.  An absent role has zero
// workgroups (the stand-alone entry points launch the big role alone).
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_gather(RowArgs gat, RelabelArgs last)
{
    extern __shared__ int32_t s_mem[];
    if (gate_closed(last.gate)) return;
    // the relabel's workgroups come first: their chains of dependent loads then run under the copy instead of after it
    if (blockIdx.x < last.blocks)
        relabel_block(last, blockIdx.x);
    else
        gather_block<VEC>(gat, blockIdx.x - last.blocks, s_mem);
}

template <int VEC>
__global__ __launch_bounds__(kBlock) void k_aggregate(RowArgs agg, FinishArgs fin)
{
    extern __shared__ int32_t s_mem[];
    if (gate_closed(fin.gate)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) publish_gate_owner(fin);
        return;
    }
    // the launch's first workgroup starts early in the launch: its first lane looks whether the next step is already there
    if (blockIdx.x == 0 && threadIdx.x == 0 && fin.blocks && !fin.gate) prefetch_step_inputs(fin.drmb, fin.mailbox);
    if (blockIdx.x < agg.blocks)
        aggregate_block<VEC>(agg, blockIdx.x, s_mem);
    else
        finish_block(fin, blockIdx.x - agg.blocks);
}

// plain streaming copy of 16-byte pieces: the traffic counters' calibration kernel (zg_calibration_copy)
__global__ __launch_bounds__(kBlock) void k_calibrate_copy(const uint4 *src, uint4 *dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) dst[i] = src[i];
}

__global__ void k_fill_u32(uint32_t *p, uint32_t v, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// graph check: indices in range and rows strictly ascending
template <typename OffT>
__global__ void k_validate(const OffT *off, const int32_t *idx, int64_t num_nodes, uint32_t *bad)
{
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < num_nodes; v += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = (int64_t)off[v], e = (int64_t)off[v + 1];
        int32_t prev = -1;
        for (int64_t p = b; p < e; ++p) {
            const int32_t g = idx[p];
            if (g < 0 || (int64_t)g >= num_nodes) atomicOr(bad, 1u);
            if (g <= prev) atomicOr(bad, 2u);
            prev = g;
        }
    }
}

// ---- graph-aware size model (plan time) ---------------------------------------------------------
// The size model of the paper's Lemma 1 treats every neighbor draw as an independent pick of a vertex with
// probability proportional to its degree.  The kernels below keep its frame - the size of D_h is a sum of
// independent indicators, one per vertex - but take each vertex's inclusion probability from the graph itself:
// with q_u = P(u in D_h) and r_u = the chance that a given neighbor of u is among u's picks at hop h
// (min(F, deg)/deg without replacement, 1 - (1 - 1/deg)^F with), a vertex v stays out of D_{h+1} with
// probability (1 - q_v) * prod over its in-neighbors u of (1 - q_u r_u).  One sweep over the edges per hop.
// Sums are kept as 64-bit fixed point (2^-32) so that the result does not depend on the order of the atomics.
constexpr double kFix = 4294967296.0; // 2^32

__global__ void k_model_init(float *q, unsigned long long *ell, const float *seed_prob, float uniform, int64_t n)
{
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        float p = seed_prob ? seed_prob[v] : uniform;
        p = p < 0.0f ? 0.0f : (p > 1.0f ? 1.0f : p);
        q[v] = p;
        ell[v] = 0ull;
    }
}

// one wave per source vertex: every neighbor v of u receives -log(1 - q_u r_u)
template <typename OffT>
__global__ __launch_bounds__(kBlock) void k_model_push(const OffT *off, const int32_t *idx, const float *q, unsigned long long *ell,
                                                       int64_t n, int32_t fanout, int32_t replace)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 6;
    const int64_t waves = ((int64_t)gridDim.x * kBlock) >> 6;
    for (int64_t u = wave0; u < n; u += waves) {
        const float qu = q[u];
        if (qu <= 0.0f) continue;
        const int64_t b = (int64_t)off[u], e = (int64_t)off[u + 1];
        const int64_t deg = e - b;
        if (deg <= 0) continue;
        double r;
        if (replace)
            r = -expm1((double)fanout * log1p(-1.0 / (double)deg));
        else
            r = deg <= fanout ? 1.0 : (double)fanout / (double)deg;
        double x = (double)qu * r;
        if (x > 1.0 - 1e-9) x = 1.0 - 1e-9;
        const unsigned long long c = (unsigned long long)(-log1p(-x) * kFix);
        if (c == 0ull) continue;
        for (int64_t p = b + lane; p < e; p += 64) atomicAdd(&ell[idx[p]], c);
    }
}

// q_v <- 1 - (1 - q_v) exp(-ell_v); ell_v <- 0; sums[0] += q_v, sums[1] += q_v (1 - q_v)
__global__ __launch_bounds__(kBlock) void k_model_update(float *q, unsigned long long *ell, int64_t n, unsigned long long *sums)
{
    double a = 0.0, b = 0.0;
    for (int64_t v = (int64_t)blockIdx.x * kBlock + threadIdx.x; v < n; v += (int64_t)gridDim.x * kBlock) {
        const double l = (double)ell[v] / kFix;
        const double q0 = (double)q[v];
        const double q1 = q0 - (1.0 - q0) * expm1(-l);
        q[v] = (float)q1;
        ell[v] = 0ull;
        a += q1;
        b += q1 * (1.0 - q1);
    }
    // fixed-point before any cross-lane addition: integer sums are the same in any order
    unsigned long long fa = (unsigned long long)(a * kFix), fb = (unsigned long long)(b * kFix);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        fa += __shfl_xor(fa, d, 64);
        fb += __shfl_xor(fb, d, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        atomicAdd(&sums[0], fa);
        atomicAdd(&sums[1], fb);
    }
}

// results of the size model left on the device: out[0..H] = mean, out[H+1..2H+1] = sigma (sums: per hop {sum q, sum q(1-q)} in 2^-32 units)
__global__ void k_model_finish(const unsigned long long *sums, int32_t num_hops, int32_t batch, double *out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    out[0] = (double)batch;
    out[num_hops + 1] = 0.0;
    for (int h = 0; h < num_hops; ++h) {
        out[h + 1] = (double)sums[2 * h] / kFix;
        out[num_hops + 1 + h + 1] = sqrt((double)sums[2 * h + 1] / kFix);
    }
}

// Scratch of zg_envelope_model_graph_static: the per-vertex log-sums (8 bytes) and probabilities (4 bytes) for up to
// ZG_STATIC_MODEL_MAX_NODES vertices plus the per-hop sums.  One copy per GPU, held until the process ends; host code
// never uses the array's name as an address, only what hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticEllBytes = (size_t)ZG_STATIC_MODEL_MAX_NODES * 8;
constexpr size_t kStaticQBytes = (size_t)ZG_STATIC_MODEL_MAX_NODES * 4;
constexpr size_t kStaticSumsBytes = 2 * ZG_MAX_HOPS * 8;
static __device__ __align__(256) unsigned char scratch[kStaticEllBytes + kStaticQBytes + kStaticSumsBytes];

#define ZG_HIP(call)                                                                                         \
    do {                                                                                                     \
        hipError_t e_ = (call);                                                                              \
        if (e_ != hipSuccess) return fail(ZG_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));       \
    } while (0)

int validate_graph_device(const zg_graph_t *g)
{
    uint32_t *d_bad = nullptr;
    ZG_HIP(hipMalloc(&d_bad, 4));
    hipError_t e = hipMemset(d_bad, 0, 4);
    if (e == hipSuccess) {
        const int grid = (int)std::min<int64_t>(65535, (g->num_nodes + 255) / 256);
        if (g->offsets_dtype == ZG_I64)
            k_validate<int64_t><<<grid, 256>>>((const int64_t *)g->d_offsets, g->d_indices, g->num_nodes, d_bad);
        else
            k_validate<int32_t><<<grid, 256>>>((const int32_t *)g->d_offsets, g->d_indices, g->num_nodes, d_bad);
        e = hipGetLastError();
    }
    uint32_t bad = 0;
    if (e == hipSuccess) e = hipMemcpy(&bad, d_bad, 4, hipMemcpyDeviceToHost);
    (void)hipFree(d_bad);
    if (e != hipSuccess) return fail(ZG_EHIP, std::string("graph validation: ") + hipGetErrorString(e));
    if (bad & 1u) return fail(ZG_EINVAL, "graph validation: a neighbor id is out of range");
    if (bad & 2u) return fail(ZG_EINVAL, "graph validation: a row is not strictly ascending");
    return ZG_OK;
}

} // namespace zg

// =================================================================================================
// plan
// =================================================================================================
using namespace zg;

struct zg_plan_s {
    const zg_graph_t *graph = nullptr;
    Layout lay;
    char *ws = nullptr;
    uint32_t flags = 0;
    int32_t batch = 0;
    int device = -1;
    const float *d_feat = nullptr;
    int64_t ld_feat = 0;
    Mailbox *mailbox = nullptr;     // pinned host memory
    Mailbox *mailbox_dev = nullptr; // the same memory as the device addresses it
    uint32_t issued = 0;            // steps enqueued so far (mod 2^32, like the device-side step counter)
    hipStream_t last_stream = nullptr; // stream of the last enqueued step (what zg_plan_destroy waits for)
    bool stepped = false;
    zg_plan_s *twin = nullptr;      // worst-case twin (ZG_PLAN_SAFE_TWIN): own outputs, metadata and mailbox, shared scratch
    hipStream_t capture_stream = nullptr;
    hipGraph_t graph_obj = nullptr;
    hipGraphExec_t graph_exec = nullptr;

    Drmb *drmb() const { return reinterpret_cast<Drmb *>(ws + lay.off_drmb); }
    uint32_t *log() const { return reinterpret_cast<uint32_t *>(ws + lay.off_log); }
    int32_t *S() const { return reinterpret_cast<int32_t *>(ws + lay.off_S); }
    int32_t *row_ptr(int h) const { return reinterpret_cast<int32_t *>(ws + lay.off_row_ptr[h]); }
    int32_t *nbr(int h) const { return reinterpret_cast<int32_t *>(ws + lay.off_nbr[h]); }
    int32_t *col(int h) const { return reinterpret_cast<int32_t *>(ws + lay.off_col[h]); }
    float *X() const { return lay.feat_dim > 0 ? reinterpret_cast<float *>(ws + lay.off_X) : nullptr; }
    float *agg() const { return lay.feat_dim > 0 ? reinterpret_cast<float *>(ws + lay.off_agg) : nullptr; }
    int32_t *local_id() const { return reinterpret_cast<int32_t *>(ws + lay.off_local_id); }
    uint32_t *bitmap(int hop) const { return reinterpret_cast<uint32_t *>(ws + lay.off_bitmap[hop & 1]); } // the one hop `hop` fills
    uint32_t *seen() const { return reinterpret_cast<uint32_t *>(ws + lay.off_seen); }
    uint64_t *status() const { return reinterpret_cast<uint64_t *>(ws + lay.off_status); }
    uint8_t *own() const { return reinterpret_cast<uint8_t *>(ws + lay.off_own); }
    uint64_t *status_cnt(int l) const { return reinterpret_cast<uint64_t *>(ws + lay.off_status_cnt[l]); }
    uint64_t *status_edge(int l) const { return reinterpret_cast<uint64_t *>(ws + lay.off_status_edge[l]); }
};

namespace {

bool aligned16(const void *p, int64_t ld) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && (ld % 4) == 0; }

RelabelArgs relabel_args(const zg_plan_t *p, int hop, bool present, const zg_plan_t *gate = nullptr)
{
    RelabelArgs ra;
    std::memset(&ra, 0, sizeof(ra));
    ra.gate = gate ? gate->drmb() : nullptr;
    if (!present) return ra;
    ra.drmb = p->drmb();
    ra.nbr = p->nbr(hop);
    ra.local_id = p->local_id();
    ra.col = p->col(hop);
    ra.num_nodes = (uint32_t)p->graph->num_nodes;
    ra.hop = hop;
    ra.blocks = (uint32_t)((p->lay.edge_cap[hop] + kRelabelPerBlock - 1) / kRelabelPerBlock);
    return ra;
}

// Whether the step's aggregation reads the feature table and writes the newly discovered vertices' rows of X on the way
// ("one pass"), instead of the gather copying every row of S_{H-1} and the aggregation reading X ("two passes").
// ZG_PLAN_FUSED_INPUT does not materialise those rows at all.  One pass moves up to a third less memory traffic and has
// one launch fewer.  Measured on MI355X against two passes (step time on one stream / with four plans in flight):
// 56 GB table of 512-byte rows -6 % with four plans; 0.6 GB table of 2400-byte rows -7 % / -3 %; 1 GB of 400-byte rows
// -4 % / 0; 1 GB of 1 KB rows 0 / -1 %.  Hence one pass unless the flag asks for two.
bool x_written_by_aggregation(const zg_plan_t *p)
{
    if (!p->d_feat || p->lay.feat_dim <= 0 || (p->flags & ZG_PLAN_FUSED_INPUT)) return false;
    return (p->flags & ZG_PLAN_X_TWO_PASS) == 0;
}

// One pass (and ZG_PLAN_FUSED_INPUT): how the rows move.  The table's rows are loaded through the caches - about a fifth of
// the last hop's edges lead to a vertex another edge leads to as well, and its row is then found in the last-level cache
// instead of in HBM.  What the feature launches write - the frontier's rows of X, the new vertices' rows of X, the rows of
// means - nothing in the step reads again: it is stored non-temporally, whatever the row length (rows that are not whole
// 128-byte lines gain as much: 2400-byte rows 84 -> 71 us per step with four plans in flight, 400-byte rows 64 -> 59 us).
// Measured at a 56 GB table of 512-byte rows, step time with four plans in flight / on one stream: table loads and all stores
// non-temporal 183 / 215 us (X rows of new vertices only: 191 / 222 us), loads cached and stores non-temporal 174 / 214 us,
// both cached 194 / 242 us.

FinishArgs finish_args(const zg_plan_t *p, bool present, const zg_plan_t *gate = nullptr, bool defer_completed = false)
{
    FinishArgs fa;
    std::memset(&fa, 0, sizeof(fa));
    if (!present) return fa;
    const int H = p->lay.num_hops;
    fa.drmb = p->drmb();
    fa.gate = gate ? gate->drmb() : nullptr;
    fa.gate_mailbox = gate ? gate->mailbox_dev : nullptr;
    fa.defer_completed = defer_completed ? 1 : 0;
    fa.mailbox = p->mailbox_dev;
    fa.S = p->S();
    fa.seen = p->seen();
    fa.log = p->log();
    fa.status = p->status();
    fa.status_words = p->lay.status_words;
    fa.num_hops = H;
    fa.blocks = (uint32_t)((p->lay.node_cap[H - 1] + kBlock - 1) / kBlock);
    return fa;
}

RowArgs gather_args(const zg_plan_t *p, const float *d_feat, int64_t ld, int32_t dim, float *d_out, int64_t ld_out, int hop_rows,
                    int *vec)
{
    RowArgs a;
    std::memset(&a, 0, sizeof(a));
    const RowTiling t = gather_tiling(dim, *vec == 4);
    *vec = t.vec;
    a.src = d_feat;
    a.dst = d_out;
    a.S = p->S();
    a.n_rows = &p->drmb()->n[hop_rows];
    a.ld_src = ld;
    a.ld_dst = ld_out;
    a.inv = t.inv;
    a.dimv = t.dimv;
    a.rows = t.rows;
    a.blocks = (uint32_t)((p->lay.node_cap[hop_rows] + t.rows - 1) / t.rows);
    return a;
}

// input rows addressed by `col` (local ids, bounded by n[hop+1]) or, with by_gid, by nbr_gid (global ids into the table)
RowArgs aggregate_args(const zg_plan_t *p, int hop, const float *d_in, int64_t ld_in, int32_t dim, float *d_out, int64_t ld_out,
                       bool by_gid, int *vec)
{
    RowArgs a;
    std::memset(&a, 0, sizeof(a));
    const RowTiling t = aggregate_tiling(dim, *vec == 4);
    *vec = t.vec;
    a.src = d_in;
    a.dst = d_out;
    a.row_ptr = p->row_ptr(hop);
    a.col = by_gid ? p->nbr(hop) : p->col(hop);
    a.n_rows = &p->drmb()->n[hop];
    a.n_cols = by_gid ? nullptr : &p->drmb()->n[hop + 1];
    a.col_limit = (uint32_t)p->graph->num_nodes;
    a.ld_src = ld_in;
    a.ld_dst = ld_out;
    a.inv = t.inv;
    a.dimv = t.dimv;
    a.rows = t.rows;
    a.max_fanout = (uint32_t)p->lay.fanout[hop];
    a.blocks = (uint32_t)((p->lay.node_cap[hop] + t.rows - 1) / t.rows);
    return a;
}

int launch_gather(int vec, const RowArgs &gat, const RelabelArgs &ra, hipStream_t st)
{
    const unsigned grid = gat.blocks + ra.blocks;
    if (grid == 0) return ZG_OK;
    const size_t lds = (size_t)kBlock * 4;
    if (vec == 4)
        hipLaunchKernelGGL(k_gather<4>, dim3(grid), dim3(kBlock), lds, st, gat, ra);
    else
        hipLaunchKernelGGL(k_gather<1>, dim3(grid), dim3(kBlock), lds, st, gat, ra);
    ZG_HIP(hipGetLastError());
    return ZG_OK;
}

int launch_aggregate(int vec, const RowArgs &agg, const FinishArgs &fa, hipStream_t st)
{
    const unsigned grid = agg.blocks + fa.blocks;
    if (grid == 0) return ZG_OK;
    const size_t lds = agg.blocks ? ((size_t)agg.rows + 1 + (size_t)agg.rows * agg.max_fanout * (agg.x_dst ? 2 : 1)) * 4 : 0;
    if (vec == 4)
        hipLaunchKernelGGL(k_aggregate<4>, dim3(grid), dim3(kBlock), lds, st, agg, fa);
    else
        hipLaunchKernelGGL(k_aggregate<1>, dim3(grid), dim3(kBlock), lds, st, agg, fa);
    ZG_HIP(hipGetLastError());
    return ZG_OK;
}

// The step's two feature launches.  Two passes: the gather copies every row of S_{H-1} into X and the mean reads X.
// One pass (and ZG_PLAN_FUSED_INPUT): the gather copies the rows of the frontier D_{H-1} only; the mean reads its input
// rows from the table, addressed by the sampled global ids (feat[nbr_gid[e]] is the row X[col[e]] holds), and - unless
// ZG_PLAN_FUSED_INPUT leaves them out - writes the other rows of X, those of the last hop's newly discovered
// vertices, on the way.
void step_feature_args(const zg_plan_t *p, RowArgs *gat, RowArgs *agg, int *vec)
{
    const Layout &L = p->lay;
    const int H = L.num_hops;
    *vec = aligned16(p->d_feat, p->ld_feat) && aligned16(p->X(), L.ld_out) && aligned16(p->agg(), L.ld_out) ? 4 : 1;
    int v1 = *vec, v2 = *vec;
    const bool fused = (p->flags & ZG_PLAN_FUSED_INPUT) != 0, one_pass = x_written_by_aggregation(p);
    if (fused || one_pass) {
        *agg = aggregate_args(p, H - 1, p->d_feat, p->ld_feat, L.feat_dim, p->agg(), L.ld_out, true, &v1);
        // the aggregation relabels the last hop's edges itself (it holds their sampled ids anyway): no launch in between
        agg->local_id = p->local_id();
        agg->col_out = p->col(H - 1);
    } else {
        *agg = aggregate_args(p, H - 1, p->X(), L.ld_out, L.feat_dim, p->agg(), L.ld_out, false, &v1);
    }
    if (one_pass) {
        agg->x_dst = p->X();
        agg->ld_x = L.ld_out;
        agg->own = p->own();
    }
    if (fused || one_pass) agg->nt = 1;
    *gat = gather_args(p, p->d_feat, p->ld_feat, L.feat_dim, p->X(), L.ld_out, (fused || one_pass) ? H - 1 : H, &v2);
    *vec = v1; // both tilings take the same vector width for the same dim and alignment
    gat->vec4 = agg->vec4 = *vec == 4 ? 1 : 0;
}

// whether the step has no gather launch of its own: the frontier's rows are copied by workgroups of the closing hop-kernel
// launch and the aggregation relabels the last hop's edges itself (H+2 launches per step)
bool features_ride_along(const zg_plan_t *p)
{
    return p->d_feat && p->lay.feat_dim > 0 && ((p->flags & ZG_PLAN_FUSED_INPUT) || x_written_by_aggregation(p));
}

// zg_step_timed: events to record right before and right after the aggregation launch of the plan's own step
struct StepProbe {
    hipEvent_t before, after;
    hipError_t error; // what recording them returned (the step is enqueued either way)
};

// a whole step, in order, on one stream (captured once, or issued eagerly): the hop kernel's launches 0..H, then the
// two feature launches.  With `gate` the kernels are those of gate's worst-case twin `p`, run on gate's inputs and
// only if gate's step overflowed; `defer_completed` marks a plan whose gated twin follows in the same sequence.
int enqueue_body(const zg_plan_t *p, hipStream_t st, const zg_plan_t *gate = nullptr, bool defer_completed = false,
                 StepProbe *probe = nullptr)
{
    const Layout &L = p->lay;
    const zg_graph_t *g = p->graph;
    const int H = L.num_hops;
    const bool feats = p->d_feat && L.feat_dim > 0;
    const bool ride = features_ride_along(p);
    RowArgs agg, gat, no_rows;
    std::memset(&agg, 0, sizeof(agg));
    std::memset(&gat, 0, sizeof(gat));
    std::memset(&no_rows, 0, sizeof(no_rows));
    int vec = 1;
    if (feats) step_feature_args(p, &gat, &agg, &vec);
    for (int l = 0; l <= H; ++l) {
        HopArgs ha;
        std::memset(&ha, 0, sizeof(ha));
        ha.offsets = g->d_offsets;
        ha.indices = g->d_indices;
        ha.drmb = p->drmb();
        ha.gate = gate ? gate->drmb() : nullptr;
        ha.mailbox = gate ? gate->mailbox_dev : p->mailbox_dev;
        ha.S = p->S();
        ha.local_id = p->local_id();
        ha.bitmap_prev = l > 0 ? p->bitmap(l - 1) : nullptr;
        ha.bitmap_next = l < H ? p->bitmap(l) : nullptr;
        ha.seen = p->seen();
        ha.row_ptr = l < H ? p->row_ptr(l) : nullptr;
        ha.nbr = l < H ? p->nbr(l) : nullptr;
        ha.own = (l == H - 1 && x_written_by_aggregation(p)) ? p->own() : nullptr;
        ha.status_cnt = p->status_cnt(l);
        ha.status_edge = p->status_edge(l);
        ha.num_nodes = (uint32_t)g->num_nodes;
        ha.launch = l;
        ha.num_hops = H;
        ha.fanout = l < H ? L.fanout[l] : 1;
        ha.group_log2 = sample_group_log2(ha.fanout);
        ha.replace = (p->flags & ZG_PLAN_REPLACE) ? 1 : 0;
        ha.tiles_per_ticket = l < H ? (uint32_t)L.old_tpt[l] : 1u;
        ha.cap_rows = (uint32_t)L.node_cap[l];
        ha.edge_cap = l < H ? (uint32_t)L.edge_cap[l] : 0u;
        ha.words_per_tile = l > 0 ? (uint32_t)L.tile_words[l] : (uint32_t)kHopMinTileWords;
        ha.rank_tiles = (uint32_t)L.rank_tiles[l];
        ha.batch = (uint32_t)p->batch;
        ha.blocks = (uint32_t)(L.old_tickets[l] + L.rank_tiles[l]);
        // the edges of hop l-2 can be relabeled now: launch l-1 ranked the last vertices they point to
        const RelabelArgs ra = relabel_args(p, l - 2, l >= 2);
        IngestArgs ia;
        std::memset(&ia, 0, sizeof(ia));
        if (l == 0) {
            ia.drmb = p->drmb();
            ia.gate = ha.gate;
            ia.mailbox = ha.mailbox;
            ia.S = p->S();
            ia.local_id = p->local_id();
            ia.seen = p->seen();
            ia.batch = (uint32_t)p->batch;
            ia.num_nodes = (uint32_t)g->num_nodes;
            ia.blocks = (uint32_t)((p->batch + kHopBlock - 1) / kHopBlock);
        }
        // the closing launch can carry the copy of the frontier's rows: D_{H-1} is final since launch H-1 (a workgroup
        // of 1024 lanes takes four times the rows of the 256-lane gather, 256 at most: its ids sit in the LDS row slots)
        RowArgs ga = no_rows;
        if (l == H && ride) {
            ga = gat;
            ga.rows = std::min<uint32_t>(kHopRows, gat.rows * (kHopBlock / kBlock));
            ga.blocks = (uint32_t)((L.node_cap[H - 1] + ga.rows - 1) / ga.rows);
        }
        const unsigned grid = ha.blocks + ra.blocks + ia.blocks + ga.blocks;
        const bool fat = ha.words_per_tile > (uint32_t)kHopMaxTileWords; // a sparse ranking launch over a very long bitmap
        if (g->offsets_dtype == ZG_I64) {
            if (fat)
                hipLaunchKernelGGL((k_hop<int64_t, kHopFatWordsPerLane>), dim3(grid), dim3(kHopBlock), 0, st, ha, ra, ia, ga);
            else
                hipLaunchKernelGGL((k_hop<int64_t, kHopMaxWordsPerLane>), dim3(grid), dim3(kHopBlock), 0, st, ha, ra, ia, ga);
        } else {
            if (fat)
                hipLaunchKernelGGL((k_hop<int32_t, kHopFatWordsPerLane>), dim3(grid), dim3(kHopBlock), 0, st, ha, ra, ia, ga);
            else
                hipLaunchKernelGGL((k_hop<int32_t, kHopMaxWordsPerLane>), dim3(grid), dim3(kHopBlock), 0, st, ha, ra, ia, ga);
        }
        ZG_HIP(hipGetLastError());
    }
    // the tail: {gather + relabel of the last hop} - unless both ride along elsewhere -, then {aggregation + end-of-step
    // clean-up}.  (One launch for all four roles was measured: no gain - the two big roles are bound by the same memory fabric.)
    if (!ride) {
        int rc = launch_gather(vec, gat, relabel_args(p, H - 1, true, gate), st);
        if (rc != ZG_OK) return rc;
    }
    if (probe) probe->error = hipEventRecord(probe->before, st);
    int rc = launch_aggregate(vec, agg, finish_args(p, true, gate, defer_completed), st);
    if (rc == ZG_OK && probe && probe->error == hipSuccess) probe->error = hipEventRecord(probe->after, st);
    return rc;
}

// the plan's step, followed - with ZG_PLAN_AUTO_FALLBACK - by its twin's step behind the device-side gate
int enqueue_step(const zg_plan_t *p, hipStream_t st, StepProbe *probe = nullptr)
{
    const bool autofb = (p->flags & ZG_PLAN_AUTO_FALLBACK) && p->twin;
    int rc = enqueue_body(p, st, nullptr, autofb, probe);
    if (rc == ZG_OK && autofb) rc = enqueue_body(p->twin, st, p, false);
    return rc;
}

void drop_graph(zg_plan_t *p)
{
    if (p->graph_exec) (void)hipGraphExecDestroy(p->graph_exec);
    if (p->graph_obj) (void)hipGraphDestroy(p->graph_obj);
    p->graph_exec = nullptr;
    p->graph_obj = nullptr;
}

int build_graph(zg_plan_t *p)
{
    drop_graph(p);
    if (p->flags & ZG_PLAN_EAGER) return ZG_OK;
    if (!p->capture_stream) ZG_HIP(hipStreamCreateWithFlags(&p->capture_stream, hipStreamNonBlocking));
    ZG_HIP(hipStreamBeginCapture(p->capture_stream, hipStreamCaptureModeThreadLocal));
    int rc = enqueue_step(p, p->capture_stream);
    hipGraph_t gobj = nullptr;
    hipError_t e = hipStreamEndCapture(p->capture_stream, &gobj);
    if (rc != ZG_OK) {
        if (gobj) (void)hipGraphDestroy(gobj);
        return rc;
    }
    if (e != hipSuccess) return fail(ZG_EHIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
    p->graph_obj = gobj;
    ZG_HIP(hipGraphInstantiate(&p->graph_exec, p->graph_obj, nullptr, nullptr, 0));
    return ZG_OK;
}

} // namespace

extern "C" {

static int make_plan_object(zg_plan_t **out, const zg_graph_t *g, const Layout &L, uint32_t flags, int32_t batch,
                            char *ws, hipStream_t st, bool init_scratch)
{
    zg_plan_t *p = new (std::nothrow) zg_plan_t();
    if (!p) return fail(ZG_ENOMEM, "out of host memory");
    p->graph = g;
    p->lay = L;
    p->ws = ws;
    p->flags = flags;
    p->batch = batch;
    auto bail = [&](int code) {
        zg_plan_destroy(p);
        return code;
    };
    if (hipGetDevice(&p->device) != hipSuccess) return bail(fail(ZG_EHIP, "hipGetDevice failed"));
    if (p->device != g->device) return bail(fail(ZG_ESTATE, "current device differs from the graph's device"));
    {
        void *host = nullptr, *dev = nullptr;
        if (hipHostMalloc(&host, sizeof(Mailbox), hipHostMallocDefault) != hipSuccess)
            return bail(fail(ZG_ENOMEM, "hipHostMalloc of the step mailbox failed"));
        std::memset(host, 0, sizeof(Mailbox));
        p->mailbox = static_cast<Mailbox *>(host);
        if (hipHostGetDevicePointer(&dev, host, 0) != hipSuccess) return bail(fail(ZG_EHIP, "hipHostGetDevicePointer failed"));
        p->mailbox_dev = static_cast<Mailbox *>(dev);
    }
    // initial state: metadata, log, both bitmaps and the scan state zero (the id map needs no initial value:
    // an entry is only read for a vertex whose entry was written earlier in the same step)
    hipError_t e = hipMemsetAsync(p->ws + L.off_drmb, 0, sizeof(Drmb), st);
    if (e == hipSuccess) e = hipMemsetAsync(p->ws + L.off_log, 0, (size_t)kLogCapacity * ZG_LOG_STRIDE * 4, st);
    if (init_scratch) {
        if (e == hipSuccess) e = hipMemsetAsync(p->ws + L.off_seen, 0, (size_t)L.bitmap_words * 4, st);
        if (e == hipSuccess) e = hipMemsetAsync(p->ws + L.off_bitmap[0], 0, (size_t)L.bitmap_words * 4, st);
        if (e == hipSuccess) e = hipMemsetAsync(p->ws + L.off_bitmap[1], 0, (size_t)L.bitmap_words * 4, st);
        if (e == hipSuccess) e = hipMemsetAsync(p->ws + L.off_status, 0, L.status_words * 8, st);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return bail(fail(ZG_EHIP, std::string("initialising the workspace: ") + hipGetErrorString(e)));
    int rc = build_graph(p);
    if (rc != ZG_OK) return bail(rc);
    *out = p;
    return ZG_OK;
}

int zg_plan(zg_plan_t **out, const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
            const zg_envelope *env, int32_t feat_dim, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!out) return fail(ZG_EINVAL, "null handle pointer");
    *out = nullptr;
    if (!g || g->stats_only) return fail(ZG_ESTATE, "zg_plan needs a graph handle with device arrays");
    Layout L, Ls;
    int rc = compute_layout(g, fanouts, num_hops, batch, env, feat_dim, nullptr, &L, &Ls);
    if (rc != ZG_OK) return rc;
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0)
        return fail(ZG_EINVAL, "workspace must be a 256-byte aligned device pointer");
    if (workspace_bytes < L.total) return fail(ZG_ENOMEM, "workspace smaller than zg_plan_query's workspace_bytes");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(d_workspace);
    const bool with_twin = (env->flags & (ZG_PLAN_SAFE_TWIN | ZG_PLAN_AUTO_FALLBACK)) != 0;
    zg_plan_t *p = nullptr;
    // with a twin the shared scratch is sized through the twin's (larger) layout; each of the two clears the regions of
    // its own layout (they overlap, but neither covers the other's: the gaps between one's regions are inside the other's)
    rc = make_plan_object(&p, g, L, env->flags, batch, ws, st, true);
    if (rc != ZG_OK) return rc;
    if (with_twin) {
        rc = make_plan_object(&p->twin, g, Ls, env->flags & ~(ZG_PLAN_SAFE_TWIN | ZG_PLAN_AUTO_FALLBACK), batch, ws, st, true);
        if (rc == ZG_OK && (env->flags & ZG_PLAN_AUTO_FALLBACK)) rc = build_graph(p); // again, now with the twin's kernels behind
        if (rc != ZG_OK) {
            zg_plan_destroy(p);
            return rc;
        }
    }
    *out = p;
    return ZG_OK;
}

// host-only wait until the device has published `target` finished steps of the plan; false after `seconds`
static bool wait_completed(const zg_plan_t *p, uint32_t target, double seconds)
{
    const volatile uint32_t *done = &p->mailbox->completed;
    const auto t0 = std::chrono::steady_clock::now();
    uint32_t polls = 0;
    while ((int32_t)(*done - target) < 0) {
        std::this_thread::yield();
        if ((++polls & 1023u) == 0 && std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > seconds) return false;
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    return true;
}

constexpr double kHostWaitSeconds = 30.0;

int zg_plan_destroy(zg_plan_t *p)
{
    if (!p) return ZG_OK;
    // a step still in flight reads the mailbox and the captured graph: wait for this plan's own last step - its
    // completion counter first (host memory only), then the stream it was issued on, so that the launch has
    // retired as a whole.  Other plans' streams are not waited for.
    if (p->mailbox && p->stepped) {
        const bool done = wait_completed(p, p->issued, kHostWaitSeconds);
        if (!done || hipStreamSynchronize(p->last_stream) != hipSuccess) (void)hipDeviceSynchronize();
        (void)hipGetLastError();
    }
    if (p->twin) zg_plan_destroy(p->twin);
    drop_graph(p);
    if (p->capture_stream) (void)hipStreamDestroy(p->capture_stream);
    if (p->mailbox) (void)hipHostFree(p->mailbox);
    delete p;
    return ZG_OK;
}

int zg_plan_bind_features(zg_plan_t *p, const float *d_feat, int64_t ld)
{
    if (!p) return fail(ZG_EINVAL, "null plan");
    if (p->lay.feat_dim <= 0) return fail(ZG_ESTATE, "plan was made with feat_dim = 0");
    if (!d_feat || ld < p->lay.feat_dim) return fail(ZG_EINVAL, "null feature table or ld < feat_dim");
    p->d_feat = d_feat;
    p->ld_feat = ld;
    int rc = p->twin ? zg_plan_bind_features(p->twin, d_feat, ld) : ZG_OK; // first: the plan's graph may hold the twin's kernels
    if (rc == ZG_OK) rc = build_graph(p);
    return rc;
}

int zg_plan_outputs(const zg_plan_t *p, zg_outputs *o)
{
    if (!p || !o) return fail(ZG_EINVAL, "null argument");
    std::memset(o, 0, sizeof(*o));
    const Layout &L = p->lay;
    o->num_hops = L.num_hops;
    o->feat_dim = L.feat_dim;
    o->d_n = p->drmb()->n;
    o->d_E = p->drmb()->E;
    o->d_n_exact = p->drmb()->n_exact;
    o->d_flags = &p->drmb()->flags;
    o->d_S = p->S();
    for (int h = 0; h < L.num_hops; ++h) {
        o->d_row_ptr[h] = p->row_ptr(h);
        o->d_nbr_gid[h] = p->nbr(h);
        o->d_col[h] = p->col(h);
        o->edge_cap[h] = L.edge_cap[h];
    }
    for (int h = 0; h <= L.num_hops; ++h) o->node_cap[h] = L.node_cap[h];
    o->d_X = p->X();
    o->ldx = L.ld_out;
    o->d_agg = p->agg();
    o->ld_agg = L.ld_out;
    o->d_log = p->log();
    o->log_capacity = kLogCapacity;
    o->d_epoch = &p->drmb()->epoch;
    o->x_row_cap = L.x_rows;
    o->d_active = &p->drmb()->active;
    o->x_one_pass = x_written_by_aggregation(p) ? 1 : 0;
    return ZG_OK;
}

// zg_step and zg_step_timed: fill the next mailbox slot, then replay the captured graph - or, for an eager plan and for
// the timed variant, enqueue the step's kernels one by one
static int issue_step(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream, StepProbe *probe)
{
    if (!p || !d_seeds) return fail(ZG_EINVAL, "null argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    // back-pressure without touching the device: wait (host only) while every mailbox slot is taken by a
    // step that has not finished yet
    if ((uint32_t)(p->issued - p->mailbox->completed) >= (uint32_t)kMailboxSlots - 1u &&
        !wait_completed(p, p->issued - ((uint32_t)kMailboxSlots - 2u), kHostWaitSeconds))
        return fail(ZG_ESTATE, "the device finished no step of this plan for 30 s while 255 are queued; nothing was enqueued");
    const uint32_t slot = p->issued % kMailboxSlots;
    p->mailbox->slot[slot].seeds = reinterpret_cast<unsigned long long>(d_seeds);
    p->mailbox->slot[slot].key = rng_key;
    std::atomic_thread_fence(std::memory_order_seq_cst);
    p->issued += 1;
    int rc = ZG_OK;
    if (probe || (p->flags & ZG_PLAN_EAGER)) {
        rc = enqueue_step(p, st, probe);
    } else if (!p->graph_exec) {
        rc = fail(ZG_ESTATE, "plan has no captured graph");
    } else {
        hipError_t e = hipGraphLaunch(p->graph_exec, st);
        if (e != hipSuccess) rc = fail(ZG_EHIP, std::string("hipGraphLaunch: ") + hipGetErrorString(e));
    }
    if (rc != ZG_OK) {
        p->issued -= 1; // nothing was enqueued: the slot is free again
    } else {
        // only now may an earlier step copy the slot ahead of time: a slot whose launch failed is filled again later
        reinterpret_cast<std::atomic<uint32_t> *>(&p->mailbox->issued)->store(p->issued, std::memory_order_release);
        p->last_stream = st;
        p->stepped = true;
    }
    return rc;
}

int zg_step(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream)
{
    return issue_step(p, d_seeds, rng_key, stream, nullptr);
}

int zg_step_timed(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream, void *event_before, void *event_after)
{
    if (!event_before || !event_after) return fail(ZG_EINVAL, "null argument");
    if (p && !(p->d_feat && p->lay.feat_dim > 0)) return fail(ZG_ESTATE, "no feature table bound: the step has no aggregation launch");
    StepProbe probe{static_cast<hipEvent_t>(event_before), static_cast<hipEvent_t>(event_after), hipSuccess};
    const int rc = issue_step(p, d_seeds, rng_key, stream, &probe);
    if (rc == ZG_OK && probe.error != hipSuccess)
        return fail(ZG_EHIP, std::string("hipEventRecord: ") + hipGetErrorString(probe.error) + " (the step itself is enqueued)");
    return rc;
}

int zg_plan_replay_features(zg_plan_t *p, int32_t which, void *stream)
{
    if (!p) return fail(ZG_EINVAL, "null plan");
    if (!p->d_feat || p->lay.feat_dim <= 0) return fail(ZG_ESTATE, "no feature table is bound to the plan");
    if (which != 0 && which != 1) return fail(ZG_EINVAL, "which must be 0 (gather) or 1 (aggregation)");
    RowArgs gat, agg;
    int vec = 1;
    step_feature_args(p, &gat, &agg, &vec);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (which == 0) return launch_gather(vec, gat, relabel_args(p, 0, false), st);
    return launch_aggregate(vec, agg, finish_args(p, false), st);
}

int zg_pilot_update(const zg_plan_t *p, int64_t *largest, void *stream)
{
    if (!p || !largest) return fail(ZG_EINVAL, "null argument");
    uint32_t n_exact[ZG_MAX_HOPS + 1];
    hipStream_t st = static_cast<hipStream_t>(stream);
    ZG_HIP(hipMemcpyAsync(n_exact, p->drmb()->n_exact, sizeof(n_exact), hipMemcpyDeviceToHost, st));
    ZG_HIP(hipStreamSynchronize(st));
    for (int h = 0; h <= p->lay.num_hops; ++h) largest[h] = std::max<int64_t>(largest[h], (int64_t)n_exact[h]);
    return ZG_OK;
}

#ifndef ZG_BUILD_ID
#define ZG_BUILD_ID "unknown"
#endif
const char *zg_build_id(void) { return ZG_BUILD_ID; }

int zg_calibration_copy(const void *d_src, void *d_dst, size_t bytes, void *stream)
{
    if (!d_src || !d_dst || bytes == 0 || (bytes & 15u) || (reinterpret_cast<uintptr_t>(d_src) & 15u) ||
        (reinterpret_cast<uintptr_t>(d_dst) & 15u))
        return fail(ZG_EINVAL, "zg_calibration_copy: pointers and size must be non-null multiples of 16");
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n + kBlock - 1) / kBlock, 256u * 64u);
    hipLaunchKernelGGL(k_calibrate_copy, dim3(grid), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(d_src), static_cast<uint4 *>(d_dst), n);
    ZG_HIP(hipGetLastError());
    return ZG_OK;
}

int zg_envelope_model_graph(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch, int32_t with_replacement,
                            const float *d_seed_prob, void *d_temp, size_t temp_bytes, void *stream, double *mean, double *sigma)
{
    if (!g || !fanouts || !mean || !sigma || !d_temp) return fail(ZG_EINVAL, "null argument");
    if (g->stats_only) return fail(ZG_ESTATE, "the graph-aware model needs a graph handle with device arrays");
    if (num_hops < 1 || num_hops > ZG_MAX_HOPS) return fail(ZG_EINVAL, "num_hops must be in 1..ZG_MAX_HOPS");
    if (batch < 1 || batch > g->num_nodes) return fail(ZG_EINVAL, "batch must be in 1..num_nodes");
    for (int h = 0; h < num_hops; ++h)
        if (fanouts[h] < 1 || fanouts[h] > ZG_MAX_FANOUT) return fail(ZG_EINVAL, "fanout must be in 1..ZG_MAX_FANOUT");
    const int64_t n = g->num_nodes;
    const size_t need = (size_t)n * 12 + 2 * kAlign + 64;
    if ((reinterpret_cast<uintptr_t>(d_temp) % kAlign) != 0 || temp_bytes < need)
        return fail(ZG_EINVAL, "temporary buffer must be 256-byte aligned and hold 12 bytes per vertex plus 576");
    int device = -1;
    ZG_HIP(hipGetDevice(&device));
    if (device != g->device) return fail(ZG_ESTATE, "current device differs from the graph's device");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(d_temp);
    unsigned long long *ell = reinterpret_cast<unsigned long long *>(base);
    size_t at = (size_t)n * 8;
    at = (at + kAlign - 1) / kAlign * kAlign;
    float *q = reinterpret_cast<float *>(base + at);
    at += (size_t)n * 4;
    at = (at + kAlign - 1) / kAlign * kAlign;
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(base + at); // [2] per hop, reused
    const int grid = (int)std::min<int64_t>(1 << 16, (n + kBlock - 1) / kBlock);
    const int grid_push = (int)std::min<int64_t>(1 << 16, (n + (kBlock / 64) - 1) / (kBlock / 64));
    hipLaunchKernelGGL(k_model_init, dim3(grid), dim3(kBlock), 0, st, q, ell, d_seed_prob, (float)((double)batch / (double)n), n);
    ZG_HIP(hipGetLastError());
    mean[0] = (double)batch;
    sigma[0] = 0.0;
    for (int h = 0; h < num_hops; ++h) {
        hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, reinterpret_cast<uint32_t *>(sums), 0u, (size_t)4);
        if (g->offsets_dtype == ZG_I64)
            hipLaunchKernelGGL(k_model_push<int64_t>, dim3(grid_push), dim3(kBlock), 0, st, (const int64_t *)g->d_offsets, g->d_indices, q,
                               ell, n, fanouts[h], with_replacement);
        else
            hipLaunchKernelGGL(k_model_push<int32_t>, dim3(grid_push), dim3(kBlock), 0, st, (const int32_t *)g->d_offsets, g->d_indices, q,
                               ell, n, fanouts[h], with_replacement);
        hipLaunchKernelGGL(k_model_update, dim3(grid), dim3(kBlock), 0, st, q, ell, n, sums);
        ZG_HIP(hipGetLastError());
        unsigned long long host[2] = {0, 0};
        ZG_HIP(hipMemcpyAsync(host, sums, sizeof(host), hipMemcpyDeviceToHost, st));
        ZG_HIP(hipStreamSynchronize(st));
        mean[h + 1] = (double)host[0] / kFix;
        sigma[h + 1] = std::sqrt((double)host[1] / kFix);
    }
    return ZG_OK;
}

// device address of this GPU's copy of `scratch`, looked up once per device with that device current
static int static_scratch(int device, unsigned char **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static unsigned char *ptr[kMaxDevices] = {};
    if (device < 0 || device >= kMaxDevices) return fail(ZG_EINVAL, "device index out of range");
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[device]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(zg::scratch));
        if (e != hipSuccess || !p) return fail(ZG_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
        ptr[device] = static_cast<unsigned char *>(p);
    }
    *out = ptr[device];
    return ZG_OK;
}

int zg_envelope_model_graph_static(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch,
                                   int32_t with_replacement, const float *d_seed_prob, void *stream, double *d_mean_sigma)
{
    if (!g || !fanouts || !d_mean_sigma) return fail(ZG_EINVAL, "null argument");
    if (g->stats_only) return fail(ZG_ESTATE, "the graph-aware model needs a graph handle with device arrays");
    if (num_hops < 1 || num_hops > ZG_MAX_HOPS) return fail(ZG_EINVAL, "num_hops must be in 1..ZG_MAX_HOPS");
    if (batch < 1 || batch > g->num_nodes) return fail(ZG_EINVAL, "batch must be in 1..num_nodes");
    for (int h = 0; h < num_hops; ++h)
        if (fanouts[h] < 1 || fanouts[h] > ZG_MAX_FANOUT) return fail(ZG_EINVAL, "fanout must be in 1..ZG_MAX_FANOUT");
    const int64_t n = g->num_nodes;
    if (n > (int64_t)ZG_STATIC_MODEL_MAX_NODES)
        return fail(ZG_EINVAL, "zg_envelope_model_graph_static: the graph has more vertices than ZG_STATIC_MODEL_MAX_NODES, the "
                               "capacity of the library's static scratch; use zg_envelope_model_graph with a caller buffer");
    if ((reinterpret_cast<uintptr_t>(d_mean_sigma) & 7u) != 0) return fail(ZG_EINVAL, "d_mean_sigma must be 8-byte aligned");
    int device = -1;
    ZG_HIP(hipGetDevice(&device));
    if (device != g->device) return fail(ZG_ESTATE, "current device differs from the graph's device");
    unsigned char *base = nullptr;
    int rc = static_scratch(device, &base);
    if (rc != ZG_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned long long *ell = reinterpret_cast<unsigned long long *>(base);
    float *q = reinterpret_cast<float *>(base + kStaticEllBytes);
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(base + kStaticEllBytes + kStaticQBytes);
    const int grid = (int)std::min<int64_t>(1 << 16, (n + kBlock - 1) / kBlock);
    const int grid_push = (int)std::min<int64_t>(1 << 16, (n + (kBlock / 64) - 1) / (kBlock / 64));
    // the array keeps the last call's contents: the per-hop sums restart at zero here (a fill kernel, not a memset
    // node, so that the sequence may be captured), q and ell are overwritten for the first n vertices by the first kernel
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, reinterpret_cast<uint32_t *>(sums), 0u, (size_t)(4 * ZG_MAX_HOPS));
    hipLaunchKernelGGL(k_model_init, dim3(grid), dim3(kBlock), 0, st, q, ell, d_seed_prob, (float)((double)batch / (double)n), n);
    ZG_HIP(hipGetLastError());
    for (int h = 0; h < num_hops; ++h) {
        if (g->offsets_dtype == ZG_I64)
            hipLaunchKernelGGL(k_model_push<int64_t>, dim3(grid_push), dim3(kBlock), 0, st, (const int64_t *)g->d_offsets, g->d_indices, q,
                               ell, n, fanouts[h], with_replacement);
        else
            hipLaunchKernelGGL(k_model_push<int32_t>, dim3(grid_push), dim3(kBlock), 0, st, (const int32_t *)g->d_offsets, g->d_indices, q,
                               ell, n, fanouts[h], with_replacement);
        hipLaunchKernelGGL(k_model_update, dim3(grid), dim3(kBlock), 0, st, q, ell, n, sums + 2 * h);
        ZG_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(k_model_finish, dim3(1), dim3(64), 0, st, sums, num_hops, batch, d_mean_sigma);
    ZG_HIP(hipGetLastError());
    return ZG_OK;
}

int zg_step_safe(zg_plan_t *p, const int32_t *d_seeds, uint64_t rng_key, void *stream)
{
    if (!p) return fail(ZG_EINVAL, "null plan");
    if (!p->twin) return fail(ZG_ESTATE, "plan was made without ZG_PLAN_SAFE_TWIN");
    if (p->flags & ZG_PLAN_AUTO_FALLBACK)
        return fail(ZG_ESTATE, "with ZG_PLAN_AUTO_FALLBACK the twin runs inside zg_step, on the device's own decision");
    return zg_step(p->twin, d_seeds, rng_key, stream);
}

int zg_plan_outputs_safe(const zg_plan_t *p, zg_outputs *out)
{
    if (!p) return fail(ZG_EINVAL, "null plan");
    if (!p->twin) return fail(ZG_ESTATE, "plan was made without ZG_PLAN_SAFE_TWIN");
    return zg_plan_outputs(p->twin, out);
}

int zg_step_status(const zg_plan_t *p, uint32_t *steps_completed, uint32_t *last_flags)
{
    if (!p || !steps_completed || !last_flags) return fail(ZG_EINVAL, "null argument");
    const volatile Mailbox *m = p->mailbox;
    const uint32_t done = m->completed;
    std::atomic_thread_fence(std::memory_order_acquire);
    *steps_completed = done;
    *last_flags = done ? m->status[(done - 1) % kMailboxSlots] : 0u;
    return ZG_OK;
}

int zg_gather(zg_plan_t *p, const float *d_feat, int64_t ld, int32_t dim, float *d_out, int64_t ld_out, void *stream)
{
    if (!p || !d_feat || !d_out) return fail(ZG_EINVAL, "null argument");
    if (dim < 1 || dim > 32768 || ld < dim || ld_out < dim) return fail(ZG_EINVAL, "dim outside 1..32768 or a row stride < dim");
    int vec = aligned16(d_feat, ld) && aligned16(d_out, ld_out) ? 4 : 1;
    const RowArgs gat = gather_args(p, d_feat, ld, dim, d_out, ld_out, p->lay.num_hops, &vec);
    return launch_gather(vec, gat, relabel_args(p, 0, false), static_cast<hipStream_t>(stream));
}

int zg_aggregate_mean(zg_plan_t *p, int32_t hop, const float *d_in, int64_t ld_in, int32_t dim, float *d_out, int64_t ld_out,
                      void *stream)
{
    if (!p || !d_in || !d_out) return fail(ZG_EINVAL, "null argument");
    if (hop < 0 || hop >= p->lay.num_hops) return fail(ZG_EINVAL, "hop out of range");
    if (dim < 1 || dim > 32768 || ld_in < dim || ld_out < dim) return fail(ZG_EINVAL, "dim outside 1..32768 or a row stride < dim");
    int vec = aligned16(d_in, ld_in) && aligned16(d_out, ld_out) ? 4 : 1;
    const RowArgs agg = aggregate_args(p, hop, d_in, ld_in, dim, d_out, ld_out, false, &vec);
    return launch_aggregate(vec, agg, finish_args(p, false), static_cast<hipStream_t>(stream));
}

int zg_overflow_flag(const zg_plan_t *p, const uint32_t **d_flag)
{
    if (!p || !d_flag) return fail(ZG_EINVAL, "null argument");
    *d_flag = &p->drmb()->flags;
    return ZG_OK;
}

int zg_overflow_clear(zg_plan_t *p, void *stream)
{
    if (!p) return fail(ZG_EINVAL, "null plan");
    hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), &p->drmb()->flags, 0u, (size_t)1);
    ZG_HIP(hipGetLastError());
    return ZG_OK;
}

} // extern "C"

// Internal declarations shared by the host-side planner and the HIP kernels of libzg.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "zg.h"

namespace zg {

constexpr int kBlock = 256;             // threads per workgroup (4 wavefronts of 64)
constexpr int kHopBlock = 1024;         // threads per workgroup of the hop kernel: (1024 / G) vertices x G slots when it samples
constexpr int kMaxTickets = 480;        // tickets per launch of the hop kernel: what 256 compute units hold at once (2 x 1024 lanes each), less a margin
constexpr int kHopMaxTpt = 4;           // most consecutive tiles of frontier rows a workgroup takes per ticket
constexpr int kHopMaxWordsPerLane = 8;  // bitmap words a lane owns in a ranking tile (held in registers)
constexpr int kHopMinTileWords = 32;    // smallest ranking tile: 32 words = 1024 vertices
constexpr int kHopMaxTileWords = kHopBlock * kHopMaxWordsPerLane; // largest: 8192 words = 262144 vertices
constexpr int kHopFatWordsPerLane = 16; // ... 16 in a launch whose tile count is set by its (few) rows, not by the ticket budget
constexpr int kHopFatTileWords = kHopBlock * kHopFatWordsPerLane; // 16384 words = 524288 vertices
constexpr int kSampleHashBits = 11;      // LDS dedup set of a sampling workgroup: 2048 slots for <= 1024 ids
constexpr int kSampleHashSlots = 1 << kSampleHashBits;
constexpr uint64_t kGatherStreamBytes = 160ull << 20; // gathered matrices above this size are copied with non-temporal accesses
constexpr int kRelabelPerBlock = 1024;  // edges per relabel workgroup (any workgroup size)
constexpr int kMailboxSlots = 256;      // per-step inputs in flight between host and device
constexpr int kLogCapacity = 1024;      // records in the device-side step log
constexpr size_t kAlign = 256;          // every buffer starts on a 256-byte boundary ...
constexpr size_t kGuard = 256;          // ... and is followed by at least this many untouched bytes

// Device-resident metadata buffer (paper section 4.1): every size the step produces lives here, at a
// fixed address, and is only ever read by kernels.
struct Drmb {
    uint32_t n[ZG_MAX_HOPS + 1];       // n[h] = |D_h| (clamped to the cap)
    uint32_t E[ZG_MAX_HOPS];           // sampled edges of hop h
    uint32_t n_exact[ZG_MAX_HOPS + 1]; // |S_{h-1}| before clamping
    uint32_t flags;                    // sticky ZG_FLAG_* bits
    uint32_t step_flags;               // the same bits, for the current step only
    uint32_t last_flags;               // step_flags of the step that finished last (step_flags itself restarts at 0)
    uint32_t epoch;                    // steps run so far
    uint32_t key_lo, key_hi;           // step key
    uint32_t ticket[ZG_MAX_HOPS + 1];  // tile tickets of the hop kernel's launches 0..H
    uint32_t active;                   // ZG_PLAN_AUTO_FALLBACK: 1 when the last step's valid outputs are the twin's
    uint32_t pre_valid, pre_epoch;     // the next step's inputs, copied from the host mailbox ahead of time: valid for step pre_epoch
    unsigned long long pre_seeds, pre_key;
};

struct Layout {
    int32_t num_hops = 0;
    int32_t feat_dim = 0;
    int64_t ldx = 0; // feat_dim rounded up to 4 elements
    int64_t ld_out = 0; // row stride of X and agg in elements: ldx, or 2 * ldx when they are the halves of one matrix
    int64_t x_rows = 0; // rows of X: node_cap[H], or node_cap[H-1] when only the frontier's rows are materialised
    int64_t node_cap[ZG_MAX_HOPS + 1] = {};
    int64_t edge_cap[ZG_MAX_HOPS] = {};
    int32_t fanout[ZG_MAX_HOPS] = {};
    int64_t bitmap_words = 0; // padded to whole ranking tiles of the largest size
    // launch l = 0..H of the hop kernel samples hop l (l < H) and ranks the vertices that hop l-1 discovered (l > 0)
    int64_t old_tiles[ZG_MAX_HOPS] = {};        // launch l < H: tiles of 1024 / G rows of the previous frontier (cap)
    int32_t old_tpt[ZG_MAX_HOPS] = {};          // consecutive such tiles per ticket (1..kHopMaxTpt)
    int64_t old_tickets[ZG_MAX_HOPS + 1] = {};  // = ceil(tiles / tiles per ticket); 0 for launch H
    int32_t tile_words[ZG_MAX_HOPS + 1] = {};   // launch l > 0: bitmap words per ranking tile (a power of two)
    int64_t rank_tiles[ZG_MAX_HOPS + 1] = {};   // launch l > 0: ranking tiles; 0 for launch 0
    // byte offsets into the workspace
    size_t off_drmb = 0, off_log = 0, off_S = 0;
    size_t off_row_ptr[ZG_MAX_HOPS] = {}, off_nbr[ZG_MAX_HOPS] = {}, off_col[ZG_MAX_HOPS] = {};
    size_t off_X = 0, off_agg = 0;
    size_t envelope_end = 0;
    size_t off_local_id = 0, off_bitmap[2] = {}, off_seen = 0, off_status = 0;
    size_t off_own = 0; // last hop: per edge, whether it was the hop's first edge to reach its vertex
    size_t status_words = 0; // uint64 words: per launch, one vertex-count chain and one edge-count chain over its tickets
    size_t off_status_cnt[ZG_MAX_HOPS + 1] = {}, off_status_edge[ZG_MAX_HOPS + 1] = {};
    size_t total = 0;
};

void set_error(const std::string &msg);
int fail(int status, const std::string &msg);

// `lay_safe` (optional) receives the layout of the worst-case twin when env->flags has ZG_PLAN_SAFE_TWIN: its
// outputs sit behind the plan's own, both share one scratch region; lay->total is the whole workspace.
int compute_layout(const zg_graph_t *g, const int32_t *fanouts, int32_t num_hops, int32_t batch, const zg_envelope *env,
                   int32_t feat_dim, zg_plan_info *info, Layout *lay, Layout *lay_safe = nullptr);

// launch shapes of the feature kernels for a row of `dim` floats
struct RowTiling {
    int vec;            // floats per lane access: 4 when rows are 16-byte aligned, else 1
    uint32_t dimv;      // dim / vec
    uint64_t inv;       // ceil(2^32 / dimv): e / dimv == (e * inv) >> 32 for the small e used
    uint32_t rows;      // rows per workgroup
};
int sample_group_log2(int fanout);
int64_t sample_tile_nodes(int fanout);
RowTiling gather_tiling(int32_t dim, bool aligned16);
RowTiling aggregate_tiling(int32_t dim, bool aligned16);

// synchronising device-side check of the CSR arrays (indices in range, rows strictly ascending)
int validate_graph_device(const zg_graph_t *g);

} // namespace zg

struct zg_graph_s {
    int64_t num_nodes = 0, num_edges = 0;
    const void *d_offsets = nullptr;
    int32_t offsets_dtype = ZG_I32;
    const int32_t *d_indices = nullptr;
    bool stats_only = false;
    int device = -1;
    std::vector<int64_t> degrees, counts; // distinct degree values (ascending) and how many vertices have each
};

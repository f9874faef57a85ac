// Internal layout of a HAG handle: host arrays, launch schedules, device copies.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "hag.h"

namespace hag {

struct Csr {
    std::vector<int64_t> ptr;
    std::vector<int32_t> col;
};

// One unit of gather work: `cnt` consecutive column entries starting at `beg`,
// reduced into output row `row` (>= 0) or, for a piece of a split row, into
// partial slot ~row (row < 0).
struct Item {
    int64_t beg;
    int32_t cnt;
    int32_t row;
};
static_assert(sizeof(Item) == 16, "Item is loaded as one 16-byte vector");
// Set in Item::beg when the item's entries include ids >= the launch's split, i.e. rows that an
// earlier phase of the same pass produces (they come last in the item's entries).  Only the
// one-launch schedule looks at it: such an item waits for the earlier phases.
constexpr int64_t kItemDependsBit = (int64_t)1 << 62;

// Schedule of one gather launch (plus the optional second launch that folds the
// partial slots of split rows).
constexpr int kPartitions = 8;   // XCDs of the device; workgroups b of one residue mod 8 share an XCD

struct Plan {
    // items of partition k are items[part_begin[k] .. part_begin[k+1]), each partition sorted by
    // length class, longest first; partition k is executed by workgroups with index mod np == k
    std::vector<Item> items;
    int np = 1;
    std::vector<int64_t> part_begin;
    std::vector<Item> combine;   // per split row: beg = first slot, cnt = #slots, row = output row
    int64_t n_slots = 0;
    // items of a length class up to this one are not ordered by class (see build_plan): the
    // launch may only hand whole workgroups to items of longer classes
    int min_block_class = 0;
    std::vector<int32_t> slot_row;   // output row of every partial slot
    int32_t *d_slot_row = nullptr;
    // device copies
    Item *d_items = nullptr;
    Item *d_combine = nullptr;
};

// Component-local form of a graph made of many small connected components with contiguous
// node ids (a batch of small graphs): everything one component needs fits in the LDS of one
// workgroup, so a whole pass (aggregation nodes and final gather) is a single launch that
// reads every feature row from HBM once.  Ids are LOCAL to the component: originals
// 0..nv-1, then its aggregation nodes sorted by level.
struct LocalLists {
    std::vector<int32_t> ptr;    // [rows+1] offsets into col
    std::vector<uint16_t> col;   // local ids
    // lists of original nodes only: the rows of each component, longest list first, stored at
    // the component's node range as {first entry in col, length | local row index << 16}, so
    // that rows handled side by side by one wavefront are equally long and wavefronts can take
    // them in that order
    std::vector<int32_t> items;  // [2*rows]
    // transposed HAG lists only (see bwd_all): items per component that wait for no aggregation row
    std::vector<int32_t> split;  // [components]
    int32_t *d_ptr = nullptr;
    uint16_t *d_col = nullptr;
    int32_t *d_items = nullptr;
    int32_t *d_split = nullptr;
};
struct Components {
    bool enabled = false;
    bool expanded = false;                   // aggregation lists are expressed over original rows (one stage)
    int32_t count = 0;
    int32_t max_nodes = 0, max_agg = 0;      // largest nv and na over the components
    // most aggregation-list entries one component has, per pass (sizes their LDS staging area)
    int32_t max_entries_fwd = 0, max_entries_bwd = 0;
    std::vector<int32_t> node_ptr;           // [count+1] first original node of each component
    std::vector<int32_t> agg_ptr;            // [count+1] into the component-major aggregation arrays
    std::vector<uint8_t> stage;              // [a] stage of the node (1-based), component-major
    std::vector<uint8_t> n_stages;           // [count] last stage the component takes part in
    LocalLists fwd, fwd_agg;                 // Nhat_v of original nodes; staged inputs of aggregation nodes
    LocalLists bwd_agg;                      // per aggregation node, the aggregation nodes that consume it
    // Transposed pass: col = consumers of original nodes, then those of aggregation nodes; the
    // items of component k sit at slot node_ptr[k] + agg_ptr[k] and cover its original rows
    // (whole list) and its aggregation rows (the destinations that consume them, row index >= its node count):
    // first the split[k] rows that no aggregation node consumes, then the others.
    LocalLists bwd_all;
    LocalLists nfwd, nbwd;                   // the input graph and its transpose (naive baseline)
    std::vector<int32_t> meta;               // [4*count] first node, #nodes, first slot, #agg | #stages << 16
    int32_t *d_meta = nullptr;
    uint8_t *d_stage = nullptr;
};

void set_error(const std::string &msg);

// Pair counting of the search on the GPU (hag_search_device.hip): a device mirror of the lists
// of Algorithm 3 that is rewritten merge by merge and answers batches of count requests.
struct CounterInit {
    int64_t n, e, capacity;
    const int64_t *ptr;                        // [n+1] list offsets
    const int32_t *nb, *len, *norig, *prio;    // lists (original members by descending prio first), lengths
    const int64_t *out_ptr;                    // [n+1] out-lists of the original nodes ...
    const int32_t *out_col, *olen;             // ... their entries (ascending) and current lengths
};
struct Found { int32_t y, c; };
struct DeviceCounter;
DeviceCounter *counter_create(const CounterInit &in, std::string &err);   // nullptr + err on failure
void counter_destroy(DeviceCounter *d);
int counter_max_batch(const DeviceCounter *d);
// lists rows[0..r) lose p and q and gain the new node w (asynchronous; rows is copied)
bool counter_merge(DeviceCounter *d, int32_t p, int32_t q, int32_t w, const int32_t *rows, int32_t r, std::string &err);
// for each request s: found[s] = every (y, count) with count >= theta[s] among the nodes whose static
// bound reaches theta[s], in no particular order; overflow[s] set instead if there are too many
bool counter_sweep(DeviceCounter *d, int nb, const int32_t *x, const int32_t *theta,
                   std::vector<std::vector<Found>> &found, std::vector<char> &overflow, std::string &err);

}  // namespace hag

// Test and tuning knobs of the launch path.  They come from the environment ONCE, when a handle is
// built; the launch path itself never reads the environment.
struct hag_knobs {
    int64_t sub_max = 0;        // HAG_SUB_MAX: longest row one sub-group takes (0 = default rule)
    bool offset64 = false;      // HAG_OFFSET64: force the 64-bit row addressing of matrices >= 4 GiB
    int32_t component_pad = 0;  // HAG_COMPONENT_PAD: padding of an LDS row, in elements (multiple of 4, <= 64)
    bool stream_output = false; // HAG_STREAM_OUTPUT: component pass writes output rows with streaming stores
    int64_t component_parts = 0;      // HAG_COMPONENT_PARTS: column parts of the component pass (2 or 4; default none)
    int64_t component_extra_lds = 0;  // HAG_COMPONENT_EXTRA_LDS: unused LDS bytes added per workgroup (occupancy experiments)
    int64_t fuse_max_items = 0; // HAG_FUSE_MAX_ITEMS: largest pass (schedule items) that runs as one launch (0: never)
    int64_t spin_limit = 0;     // HAG_SPIN_LIMIT: polls a wavefront of the one-launch pass waits for earlier phases
    bool wait_unreachable = false;      // test only: the awaited count can never be reached, so every wait gives up
    bool deterministic_max_backward = false;
    int32_t part_shift = 0;     // HAG_PART_SHIFT: workgroup b of a partitioned launch takes the sources of class (b + shift) mod 8
};

struct hag_handle {
    int64_t n = 0, e = 0, a = 0;
    hag_knobs knobs;
    int32_t levels = 0;
    hag::Csr g;    // input graph: rows = destinations
    hag::Csr gt;   // its transpose: rows = sources, cols = destinations
    std::vector<float> inv_deg;  // 1 / max(|N(v)|, 1)
    std::vector<float> inv_deg1; // 1 / (|N(v)| + 1)

    // merge list, creation order, unified creation-order ids
    std::vector<int32_t> m_left, m_right, m_red;
    // Nhat_v in creation-order ids (kept for hag_prefix)
    // level-ordered forward form
    std::vector<int32_t> left, right;     // [a]
    std::vector<int32_t> level_ptr;       // [levels+1]
    hag::Csr hf;                          // Nhat_v, v in V
    // stages: runs of consecutive levels executed by one launch
    int32_t stages = 0;
    std::vector<int32_t> stage_ptr;       // [stages+1], in aggregation-node index space
    std::vector<uint8_t> stage_single_level;
    hag::Csr he;                          // row i: inputs of aggregation node n+i expanded to earlier stages
    // transposed HAG: row s in [0, n+a) lists the consumers of s; a consumer id < n is a
    // destination (reads gY), an id >= n is aggregation node id (reads its gradient row)
    hag::Csr ht;
    // column arrays in device order (rows cut by source partition are reordered); released after upload
    std::vector<int32_t> hf_dcol, ht_dcol, g_dcol, gt_dcol;
    hag_stats_t st{};

    // schedules
    hag::Plan p_fwd;                       // final gather over hf
    std::vector<hag::Plan> p_fwd_stage;    // [stages]; rows of he (unused for single-level stages)
    std::vector<hag::Plan> p_bwd_stage;    // [stages]; rows of ht that belong to the stage
    hag::Plan p_bwd_src;                   // rows 0..n-1 of ht
    hag::Plan p_naive_fwd, p_naive_bwd;
    int64_t max_slots = 0;
    hag::Components comp;

    // device copies
    bool uploaded = false, comp_uploaded = false;
    int device = -1;
    int32_t *d_left = nullptr, *d_right = nullptr;
    int32_t *d_hcol = nullptr, *d_tcol = nullptr, *d_gcol = nullptr, *d_gtcol = nullptr, *d_ecol = nullptr;
    int32_t *d_slot_ids = nullptr;
    float *d_inv_deg = nullptr, *d_inv_deg1 = nullptr;
    int32_t *d_sync = nullptr;   // {ticket, done, gave_up, -} of the one-launch schedule; zero between launches
    std::vector<void *> d_allocs;
};

namespace hag {
// hag_host.cpp
int finalize(hag_handle *h, uint32_t flags);  // levels, forward form, transposes, schedules, stats
void build_plan(const Csr &c, std::vector<int32_t> &dcol, int64_t row_begin, int64_t row_end, Plan &p, bool partition,
                int64_t split);
int64_t long_items(const Plan &p, int k, int64_t threshold);
// hag_device.hip
void free_device(hag_handle *h);
}  // namespace hag

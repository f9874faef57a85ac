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

// Schedule of one gather launch (plus the optional second launch that folds the
// partial slots of split rows).
struct Plan {
    // items[0 .. n_block): one whole workgroup each (long rows, longest first);
    // items[n_block ..): one sub-group of lanes each (short rows, longest first)
    std::vector<Item> items;
    int64_t n_block = 0;
    std::vector<Item> combine;   // per split row: beg = first slot, cnt = #slots, row = output row
    int64_t n_slots = 0;
    // device copies
    Item *d_items = nullptr;
    Item *d_combine = nullptr;
};

void set_error(const std::string &msg);

}  // namespace hag

struct hag_handle {
    int64_t n = 0, e = 0, a = 0;
    int32_t levels = 0;
    hag::Csr g;    // input graph: rows = destinations
    hag::Csr gt;   // its transpose: rows = sources, cols = destinations
    std::vector<float> inv_deg;  // 1 / max(|N(v)|, 1)

    // merge list, creation order, unified creation-order ids
    std::vector<int32_t> m_left, m_right, m_red;
    // Nhat_v in creation-order ids (kept for hag_prefix)
    // level-ordered forward form
    std::vector<int32_t> left, right;     // [a]
    std::vector<int32_t> level_ptr;       // [levels+1]
    hag::Csr hf;                          // Nhat_v, v in V
    // transposed HAG: row s in [0, n+a) lists the consumers of s; a consumer id < n is a
    // destination (reads gY), an id >= n is aggregation node id (reads its gradient row)
    hag::Csr ht;
    hag_stats_t st{};

    // schedules
    hag::Plan p_fwd;                       // final gather over hf
    std::vector<hag::Plan> p_bwd_level;    // [levels]; index l-1 covers rows of depth l in ht
    hag::Plan p_bwd_src;                   // rows 0..n-1 of ht
    hag::Plan p_naive_fwd, p_naive_bwd;
    int64_t max_slots = 0;

    // device copies
    bool uploaded = false;
    int device = -1;
    int32_t *d_left = nullptr, *d_right = nullptr;
    int32_t *d_hcol = nullptr, *d_tcol = nullptr, *d_gcol = nullptr, *d_gtcol = nullptr;
    int32_t *d_slot_ids = nullptr;
    float *d_inv_deg = nullptr;
    std::vector<void *> d_allocs;
};

namespace hag {
// hag_host.cpp
int finalize(hag_handle *h, uint32_t flags);  // levels, forward form, transposes, schedules, stats
void build_plan(const Csr &c, int64_t row_begin, int64_t row_end, Plan &p);
// hag_device.hip
void free_device(hag_handle *h);
}  // namespace hag

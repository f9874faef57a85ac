// Device side of libhag for gfx950 (MI355X): the kernels of Algorithm 2 and of its
// transposed pass, and the C entry points that enqueue them.
//
// The path is a sparse gather-reduce (about one add or compare per four bytes
// loaded), so it is bound by memory traffic, not by arithmetic: there is no MFMA
// here.  What matters is that every neighbour row is fetched with full-width
// coalesced 16-byte loads, that enough independent loads are in flight per wave,
// and that work is balanced across 256 compute units although row lengths are
// heavy-tailed.
#include "hag_device_common.hpp"

#include <vector>

namespace hag {

// One level of aggregation nodes (Algorithm 2, the loop over V_A): every node has exactly
// two inputs, so the work is uniform: one thread per four features of one node.
template <typename T, int RED>
__global__ __launch_bounds__(kBlock) void level_kernel(const int32_t *__restrict__ left,
                                                       const int32_t *__restrict__ right, int32_t first,
                                                       int32_t last, int32_t n, int32_t d, const T *__restrict__ x,
                                                       T *w, int32_t *wid) {
    using V = typename V4<T>::type;
    const int q = d / 4;
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t node = first + t / q;
    if (node >= last) return;
    const int c = (int)(t % q) * 4;
    const int l = left[node], r = right[node];
    V a, b;
    int4 ai, bi;
    if (l < n) {
        a = ld4(x + (size_t)l * d + c);
        ai = make_int4(l, l, l, l);
    } else {
        a = ld4(w + (size_t)(l - n) * d + c);
        if (RED == R_MAX) ai = ld4(wid + (size_t)(l - n) * d + c);
    }
    if (r < n) {
        b = ld4(x + (size_t)r * d + c);
        bi = make_int4(r, r, r, r);
    } else {
        b = ld4(w + (size_t)(r - n) * d + c);
        if (RED == R_MAX) bi = ld4(wid + (size_t)(r - n) * d + c);
    }
    if (RED == R_MAX) {
        max4(a, ai, b, bi);
        st4(wid + (size_t)node * d + c, ai);
    } else {
        add4(a, b);
    }
    st4(w + (size_t)node * d + c, a);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void fill_zero_kernel(T *p, int64_t n4) {
    using V = typename V4<T>::type;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) st4(p + i * 4, V{});
}

__device__ __forceinline__ void atomic_accumulate(float *p, float v) { unsafeAtomicAdd(p, v); }
__device__ __forceinline__ void atomic_accumulate(int32_t *p, int32_t v) { atomicAdd(p, v); }

// Transposed pass of max: each output element sends its gradient to the one source that won.
template <typename T>
__global__ __launch_bounds__(kBlock) void max_backward_kernel(const T *__restrict__ gy,
                                                              const int32_t *__restrict__ argmax, T *gx,
                                                              int64_t total, int32_t d) {
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= total) return;
    int u = argmax[i];
    if (u >= 0) atomic_accumulate(gx + (size_t)u * d + (i % d), gy[i]);
}

// Scratch for callers that cannot bring a workspace (hag_forward_static_scratch): one array per
// GPU, held from the moment the code object is loaded until the process ends.  In host code the
// array's name is only a stand-in for the symbol; the address of each GPU's copy is looked up once
// per device (hag_upload, with that device current) and kept here.
static __device__ __align__(256) unsigned char scratch[HAG_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};

// address of the current device's scratch array, looked up on first use
static int scratch_address(int device, void **out) {
    if (device < 0 || device >= kMaxDevices) { set_error("device index out of range"); return HAG_EINVAL; }
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { set_error("hipGetSymbolAddress returned no address for the scratch array"); return HAG_EHIP; }
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return HAG_OK;
}

struct Workspace {
    char *agg = nullptr;      // [a, d] aggregation-node rows (forward) or their gradients (transposed pass)
    char *part = nullptr;     // [max_slots, d]
    char *agg_id = nullptr;   // max only
    char *part_id = nullptr;  // max only
    size_t total = 0;
};

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static Workspace carve(const hag_handle *h, hag_op_t op, int64_t d, void *base) {
    Workspace w;
    size_t row = (size_t)d * 4;
    size_t s_agg = align_up((size_t)h->a * row), s_part = align_up((size_t)h->max_slots * row);
    char *p = (char *)base;
    w.agg = p; p += s_agg;
    w.part = p; p += s_part;
    if (op == HAG_MAX) {
        w.agg_id = p; p += s_agg;
        w.part_id = p; p += s_part;
    }
    w.total = (size_t)(p - (char *)base);
    return w;
}

// Longest item that a single sub-group of lanes takes; longer ones get a whole workgroup.
static int64_t block_threshold(const hag_handle *h, const Plan &p, int64_t d) {
    const int64_t sub_max = h->knobs.sub_max;
    const int64_t nsg = kBlock / pick_lpr(d);
    // A launch too small to fill the device with one sub-group per row (the stages of
    // a small HAG) lasts as long as its longest single-sub-group row: there a row gets
    // a workgroup much sooner.
    const int64_t n_all = p.part_begin[p.np] - p.part_begin[0];
    const bool small_launch = n_all <= 256 * 8 * nsg;
    return sub_max > 0 ? sub_max : small_launch ? 16 : std::max<int64_t>(64, 8 * nsg);
}

// Whether a pass over `plans` (its phases in execution order) can run as one launch: a small
// HAG whose launches are short against the gaps between them, no row cut into pieces (the fold
// of partial rows would be one more phase per launch), feature columns in one chunk.
static bool fusable(const hag_handle *h, int64_t d, const std::vector<const Plan *> &plans) {
    if (h->knobs.fuse_max_items <= 0 || !h->d_sync || h->a == 0 || d > 256) return false;
    if ((int)plans.size() > kMaxPhases || plans.size() < 2) return false;
    int64_t items = 0;
    for (const Plan *p : plans) {
        if (p->np != 1 || !p->combine.empty() || p->items.empty()) return false;
        items += (int64_t)p->items.size();
    }
    return items <= h->knobs.fuse_max_items;
}

// Fill the phase table of a one-launch pass and enqueue it.  `outs[k]` describes where phase k
// writes: all but the last write aggregation rows (unified ids, offset n).
template <typename T, int RED, int ROLE>
static int run_fused(const hag_handle *h, const std::vector<const Plan *> &plans, const std::vector<const int32_t *> &cols,
                     GatherArgs<T> base, T *agg_out, int32_t *agg_out_id, T *final_out, int32_t *final_out_id,
                     hipStream_t s) {
    FusedArgs<T> f{};
    const int lpr = pick_lpr(base.d);
    const int64_t per_block = (kBlock / kWave) * (kWave / lpr);
    int64_t blocks = 0;
    const int np = (int)plans.size();
    for (int k = 0; k < np; ++k) {
        const Plan &p = *plans[k];
        auto &ph = f.ph[k];
        ph.items = p.d_items;
        ph.col = cols[k];
        ph.n_items = (int64_t)p.items.size();
        ph.n_block = long_items(p, 0, block_threshold(h, p, base.d));
        const bool last = k == np - 1;
        ph.out = last ? final_out : agg_out;
        ph.out_id = last ? final_out_id : agg_out_id;
        ph.out_off = last ? 0 : (int32_t)h->n;
        ph.block_begin = (int32_t)blocks;
        blocks += ph.n_block + (ph.n_items - ph.n_block + per_block - 1) / per_block;
    }
    if (blocks > (1 << 24)) { set_error("launch too large"); return HAG_EINVAL; }
    f.n_phases = np;
    f.total_blocks = (int32_t)blocks;
    // As many workgroups as the device holds at once (8 per compute unit); each draws one unit per
    // ticket unless that would be more than 16 tickets per workgroup.
    f.chunk = (int32_t)std::min<int64_t>(std::max<int64_t>(blocks / (256 * 8 * 16), 1), 16);
    f.grid = (int32_t)std::min<int64_t>((blocks + f.chunk - 1) / f.chunk, 256 * 8);
    f.out_scale = base.out_scale;
    f.self = base.self;
    f.self_scale = base.self_scale;
    base.out_scale = nullptr;
    base.self = nullptr;
    base.self_scale = nullptr;
    {
        const uint64_t row_bytes = (uint64_t)base.d * 4;
        const uint64_t lo_rows = (uint64_t)std::max<int64_t>(base.split, 1);
        base.off32 = (!h->knobs.offset64 && lo_rows * row_bytes < (1ull << 32) && lo_rows <= (1ull << 24) &&
                      row_bytes < (1ull << 24)) ? 1 : 0;
    }
    base.part = nullptr;
    base.part_id = nullptr;
    base.stream_hi = 0;
    base.spin_limit = (int32_t)std::min<int64_t>(std::max<int64_t>(h->knobs.spin_limit, 1), INT32_MAX);
    base.wait_bias = h->knobs.wait_unreachable ? (1 << 30) : 0;
    f.base = base;
    f.sync = h->d_sync;
    return launch_fused<T, RED, ROLE>(f, s);
}

// run one schedule: the gather itself, then the fold of split rows
template <typename T, int RED, int ROLE>
static int run_plan(const hag_handle *h, const Plan &p, const int32_t *d_col, GatherArgs<T> a, const Workspace &w,
                    hipStream_t s, uint32_t phases = HAG_PHASE_ALL) {
    a.items = p.d_items;
    a.np = p.np;
    a.part_shift = p.np > 1 ? (int)(((h->knobs.part_shift % p.np) + p.np) % p.np) : 0;
    // rows of ids < split live in a matrix of `split` rows, the others in one of at most
    // n + a (aggregation rows) or max_slots (partial rows) rows
    {
        const uint64_t row_bytes = (uint64_t)a.d * 4;
        const uint64_t lo_rows = (uint64_t)std::max<int64_t>(a.split, 1);
        // the knob forces the 64-bit path, which otherwise only matrices of 4 GiB and more take
        a.off32 = (!h->knobs.offset64 && lo_rows * row_bytes < (1ull << 32) && lo_rows <= (1ull << 24) &&
                   row_bytes < (1ull << 24)) ? 1 : 0;
    }
    // A row is worth a whole workgroup when each of its 256/LPR sub-groups still gets about
    // eight neighbours, and needs one when a single sub-group would walk it for too long.
    {
        const int64_t threshold = block_threshold(h, p, a.d);
        for (int k = 0; k < p.np; ++k) {
            a.seg[k].begin = p.part_begin[k];
            a.seg[k].n_items = p.part_begin[k + 1] - p.part_begin[k];
            a.seg[k].n_block = long_items(p, k, threshold);
        }
    }
    a.col = d_col;
    a.part = (T *)w.part;
    a.part_id = (int32_t *)w.part_id;
    a.stream_hi = 0;
    int rc = (phases & HAG_PHASE_GATHER) ? launch_gather<T, RED, ROLE>(a, s) : HAG_OK;
    if (rc) return rc;
    if (!p.combine.empty() && (phases & HAG_PHASE_FOLD)) {
        GatherArgs<T> c = a;
        c.stream_hi = 1;
        c.items = p.d_combine;
        c.np = 1;
        c.seg[0].begin = 0;
        c.seg[0].n_block = 0;
        c.seg[0].n_items = (int64_t)p.combine.size();
        c.col = h->d_slot_ids;
        // partial results of a float max may still hold aggregation ids (see gather_body)
        c.late_id = (RED == R_MAX && std::is_same<T, float>::value) ? a.id_hi : nullptr;
        c.late_split = a.split;
        c.split = 0;               // every id refers to a partial slot
        c.src_lo = nullptr;
        c.src_hi = (const T *)w.part;
        c.id_hi = (const int32_t *)w.part_id;
        c.in_scale = nullptr;
        constexpr int FOLD_RED = RED == R_SUMIF ? R_SUM : RED;   // partial rows of a filtered sum are plain sums
        rc = launch_gather<T, FOLD_RED, G_FOLD>(c, s);
    }
    return rc;
}

static int check_common(const hag_handle *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *in, const void *out,
                        const void *ws, bool needs_ws) {
    if (!h) { set_error("handle is NULL"); return HAG_EINVAL; }
    if (!h->uploaded) { set_error("hag_upload has not been called on this handle"); return HAG_ESTATE; }
    if (op != HAG_SUM && op != HAG_MEAN && op != HAG_MAX && op != HAG_GCN) { set_error("unknown op"); return HAG_EINVAL; }
    if (dt != HAG_F32 && dt != HAG_I32) { set_error("unknown dtype"); return HAG_EINVAL; }
    if ((op == HAG_MEAN || op == HAG_GCN) && dt != HAG_F32) { set_error("mean and gcn are defined for f32 only"); return HAG_EINVAL; }
    if (d <= 0 || (d % 4) != 0) { set_error("d must be a positive multiple of 4"); return HAG_EINVAL; }
    if (d > (1 << 20)) { set_error("d too large"); return HAG_EINVAL; }
    if (h->n > 0 && (!in || !out)) { set_error("NULL feature pointer"); return HAG_EINVAL; }
    if (((uintptr_t)in | (uintptr_t)out | (uintptr_t)ws) & 15) { set_error("pointers must be 16-byte aligned"); return HAG_EINVAL; }
    if (needs_ws && !ws) { set_error("workspace is NULL but hag_workspace_bytes() > 0"); return HAG_EINVAL; }
    return HAG_OK;
}

// LDS layout of the component-local pass: [rows + zero row][agg ptr][agg list ids]
struct CompLayout {
    size_t stride = 0;                                 // row stride in LDS, in elements
    size_t lists_off = 0, total = 0;                   // bytes
    int64_t d_part = 0;                                // feature columns per workgroup
    int parts = 1;                                     // workgroups per component (column parts)
};
// An LDS row is not padded by default: 16-byte LDS reads of whole rows by sub-groups of lanes were
// measured fastest when the row stride is the row itself, and any padding made them collide in
// the banks (the handle's component_pad knob adds some for tests).
//
// Column parts (knob component_parts = 2 or 4, off by default): the feature columns of a component
// are cut in parts, each handled by a workgroup of its own with narrower LDS rows, so that more
// workgroups share a compute unit.  Measured on 5000 graphs of 74 nodes, d = 64, two parts: a pass
// takes 132 us instead of 81 us (eight lanes per row instead of sixteen double the index work per
// byte read), which outweighs the gain in occupancy.
// layout.total == 0: the pass does not apply to this call
static CompLayout component_layout(const hag_handle *h, bool naive, bool backward, hag_op_t op, int64_t d) {
    CompLayout L;
    const Components &c = h->comp;
    if (!c.enabled || !h->comp_uploaded) return L;
    // sums only.  Max stays on the generic kernels: their ordered comparison path is cheaper
    // per element than a (value, id) comparison for every LDS row (measured: the LDS variant
    // was the slower one), and its backward pass is a scatter, not a gather.
    if (op == HAG_MAX) return L;
    const size_t rows = (size_t)c.max_nodes + (naive ? 0 : (size_t)c.max_agg) + 1;
    size_t list_bytes = 0;
    if (!naive) {
        const size_t entries = backward ? c.max_entries_bwd : c.max_entries_fwd;   // aggregation lists only
        list_bytes = ((size_t)c.max_agg + 1) * 4 + ((entries + 1) & ~(size_t)1) * 2;
    }
    auto bytes_for = [&](int64_t dp) {
        size_t b = rows * ((size_t)dp + (size_t)h->knobs.component_pad) * 4 + list_bytes;
        b = (b + 15) & ~(size_t)15;
        return b + (size_t)h->knobs.component_extra_lds;   // never touched: lowers how many workgroups share a compute unit
    };
    int parts = 1;
    const int64_t forced = h->knobs.component_parts;
    for (int p : {2, 4}) {
        if (p > forced || d % p != 0 || (d / p) % 4 != 0) break;
        parts = p;
    }
    L.parts = parts;
    L.d_part = d / parts;
    L.stride = (size_t)L.d_part + (size_t)h->knobs.component_pad;
    L.lists_off = rows * L.stride * 4;
    const size_t bytes = bytes_for(L.d_part);
    if (bytes <= 63 * 1024) L.total = bytes;   // the kernel adds 256 B of static LDS; 64 KB per workgroup
    return L;
}

template <typename T, bool BACKWARD>
static int launch_component(const hag_handle *h, bool naive, hag_op_t op, int64_t d, const T *in, T *out,
                            hipStream_t s) {
    const Components &c = h->comp;
    const CompLayout L = component_layout(h, naive, BACKWARD, op, d);
    CompArgs<T> a{};
    a.meta = c.d_meta;
    a.stage = c.d_stage;
    const LocalLists &rows = BACKWARD ? (naive ? c.nbwd : c.bwd_all) : (naive ? c.nfwd : c.fwd);
    const LocalLists &aggs = BACKWARD ? c.bwd_agg : c.fwd_agg;
    a.row_items = rows.d_items;
    a.row_col = rows.d_col;
    a.row_split = rows.d_split;
    a.agg_row_ptr = aggs.d_ptr;
    a.agg_row_col = aggs.d_col;
    a.in = in;
    a.out = out;
    const float *norm = op == HAG_MEAN ? h->d_inv_deg : op == HAG_GCN ? h->d_inv_deg1 : nullptr;
    a.scale_in = BACKWARD ? norm : nullptr;
    a.scale_out = BACKWARD ? nullptr : norm;
    a.add_self = op == HAG_GCN ? 1 : 0;
    a.self_scale = nullptr;
    a.d = (int32_t)L.d_part;
    a.gd = (int32_t)d;
    a.stride = (int32_t)L.stride;
    a.use_agg = naive ? 0 : 1;
    a.reverse = BACKWARD ? 1 : 0;
    a.pairs = (!BACKWARD && !c.expanded) ? 1 : 0;
    a.stream_out = h->knobs.stream_output ? 1 : 0;
    a.lists_off = (int32_t)L.lists_off;
    a.max_agg = c.max_agg;
    return launch_component_kernel<T>(a, naive ? 2 + (BACKWARD ? 1 : 0) : (BACKWARD ? 1 : 0), L.d_part, (unsigned)c.count,
                                      (unsigned)L.parts, L.total, s);
}

template <typename T, int RED>
static int forward_impl(const hag_handle *h, bool naive, hag_op_t op, int64_t d, const T *x, T *y, int32_t *argmax,
                        void *ws, hipStream_t s, uint32_t phases) {
    // a batch of small graphs: the whole pass is one launch out of LDS
    if (phases == HAG_PHASE_ALL && component_layout(h, naive, false, op, d).total > 0)
        return launch_component<T, false>(h, naive, op, d, x, y, s);
    Workspace w = carve(h, op, d, ws);
    const int32_t n = (int32_t)h->n;
    if (!naive && phases == HAG_PHASE_ALL) {
        // a small HAG: aggregation-node stages and the gather over V as one launch
        std::vector<const Plan *> plans;
        std::vector<const int32_t *> cols;
        for (int32_t st = 0; st < h->stages; ++st) { plans.push_back(&h->p_fwd_stage[st]); cols.push_back(h->d_ecol); }
        plans.push_back(&h->p_fwd);
        cols.push_back(h->d_hcol);
        if (fusable(h, d, plans)) {
            GatherArgs<T> b{};
            b.src_lo = x;
            b.src_hi = (const T *)w.agg;
            b.id_hi = (const int32_t *)w.agg_id;
            b.split = n;
            b.d = (int32_t)d;
            b.out_scale = op == HAG_MEAN ? h->d_inv_deg : op == HAG_GCN ? h->d_inv_deg1 : nullptr;
            b.self = op == HAG_GCN ? x : nullptr;
            return run_fused<T, RED, G_HAG_FWD>(h, plans, cols, b, (T *)w.agg, (int32_t *)w.agg_id, y, argmax, s);
        }
    }
    if (!naive && (phases & HAG_PHASE_LEVELS)) {
        for (int32_t st = 0; st < h->stages; ++st) {
            const int32_t first = h->stage_ptr[st], last = h->stage_ptr[st + 1];
            if (h->stage_single_level[st]) {
                int64_t threads = (int64_t)(last - first) * (d / 4);
                if (threads <= 0) continue;
                int64_t blocks = (threads + kBlock - 1) / kBlock;
                hipLaunchKernelGGL((level_kernel<T, RED>), dim3((unsigned)blocks), dim3(kBlock), 0, s, h->d_left,
                                   h->d_right, first, last, n, (int32_t)d, x, (T *)w.agg, (int32_t *)w.agg_id);
                HIP_TRY(hipGetLastError());
            } else {
                // several levels in one launch: every node gathers its inputs expanded down to
                // earlier stages
                GatherArgs<T> e{};
                e.src_lo = x;
                e.src_hi = (const T *)w.agg;
                e.id_hi = (const int32_t *)w.agg_id;
                e.split = n;
                e.out = (T *)w.agg;
                e.out_id = (int32_t *)w.agg_id;
                e.out_off = n;
                e.d = (int32_t)d;
                int rc = run_plan<T, RED, G_HAG_FWD_STAGE>(h, h->p_fwd_stage[st], h->d_ecol, e, w, s);
                if (rc) return rc;
            }
        }
    }
    GatherArgs<T> a{};
    a.src_lo = x;
    a.src_hi = (const T *)w.agg;
    a.id_hi = (const int32_t *)w.agg_id;
    a.split = n;
    a.out = y;
    a.out_id = argmax;
    a.out_off = 0;
    a.in_scale = nullptr;
    a.out_scale = op == HAG_MEAN ? h->d_inv_deg : op == HAG_GCN ? h->d_inv_deg1 : nullptr;
    a.self = op == HAG_GCN ? x : nullptr;
    a.d = (int32_t)d;
    if (!(phases & (HAG_PHASE_GATHER | HAG_PHASE_FOLD))) return HAG_OK;
    if (naive) return run_plan<T, RED, G_NAIVE_FWD>(h, h->p_naive_fwd, h->d_gcol, a, w, s, phases);
    return run_plan<T, RED, G_HAG_FWD>(h, h->p_fwd, h->d_hcol, a, w, s, phases);
}

template <typename T>
static int backward_impl(const hag_handle *h, bool naive, hag_op_t op, int64_t d, const T *gy, const int32_t *argmax,
                         T *gx, void *ws, hipStream_t s, uint32_t phases) {
    const int32_t n = (int32_t)h->n;
    if (op == HAG_MAX && h->knobs.deterministic_max_backward) {
        // gx[u, f] = sum over the consumers v of u of gy[v, f] where argmax[v, f] == u: a gather over the
        // transposed input graph in a fixed order (no atomics), at the price of reading the argmax row
        // of every consumer: about as much traffic as a forward pass
        if (h->n == 0) return HAG_OK;
        Workspace w = carve(h, HAG_SUM, d, ws);
        GatherArgs<T> a{};
        a.src_lo = gy;
        a.split = n;
        a.filter = argmax;
        a.slot_row = h->p_naive_bwd.d_slot_row;
        a.d = (int32_t)d;
        a.out = gx;
        a.out_off = 0;
        return run_plan<T, R_SUMIF, G_NAIVE_BWD>(h, h->p_naive_bwd, h->d_gtcol, a, w, s, phases);
    }
    if (op == HAG_MAX) {
        int64_t total = h->n * d;
        if (total == 0 || !(phases & HAG_PHASE_GATHER)) return HAG_OK;
        hipLaunchKernelGGL((fill_zero_kernel<T>), dim3((unsigned)((total / 4 + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                           s, gx, total / 4);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL((max_backward_kernel<T>), dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                           s, gy, argmax, gx, total, (int32_t)d);
        HIP_TRY(hipGetLastError());
        return HAG_OK;
    }
    if (phases == HAG_PHASE_ALL && component_layout(h, naive, true, op, d).total > 0)
        return launch_component<T, true>(h, naive, op, d, gy, gx, s);
    Workspace w = carve(h, op, d, ws);
    GatherArgs<T> a{};
    a.src_lo = gy;
    a.src_hi = (const T *)w.agg;
    a.id_hi = nullptr;
    a.split = n;
    a.in_scale = op == HAG_MEAN ? h->d_inv_deg : op == HAG_GCN ? h->d_inv_deg1 : nullptr;
    a.out_scale = nullptr;
    a.d = (int32_t)d;
    if (naive) {
        a.out = gx;
        a.out_off = 0;
        if (op == HAG_GCN) { a.self = gy; a.self_scale = h->d_inv_deg1; }
        if (!(phases & (HAG_PHASE_GATHER | HAG_PHASE_FOLD))) return HAG_OK;
        return run_plan<T, R_SUM, G_NAIVE_BWD>(h, h->p_naive_bwd, h->d_gtcol, a, w, s, phases);
    }
    if (phases == HAG_PHASE_ALL) {
        std::vector<const Plan *> plans;
        std::vector<const int32_t *> cols;
        for (int32_t st = h->stages - 1; st >= 0; --st) { plans.push_back(&h->p_bwd_stage[st]); cols.push_back(h->d_tcol); }
        plans.push_back(&h->p_bwd_src);
        cols.push_back(h->d_tcol);
        if (fusable(h, d, plans)) {
            GatherArgs<T> b = a;
            if (op == HAG_GCN) { b.self = gy; b.self_scale = h->d_inv_deg1; }
            return run_fused<T, R_SUM, G_HAG_BWD_SRC>(h, plans, cols, b, (T *)w.agg, nullptr, gx, nullptr, s);
        }
    }
    // deepest stage first: its consumers are destinations only; an earlier stage may also be
    // consumed by aggregation nodes of later stages, whose gradient rows are complete by then
    for (int32_t st = h->stages - 1; st >= 0 && (phases & HAG_PHASE_LEVELS); --st) {
        a.out = (T *)w.agg;
        a.out_off = n;
        int rc = run_plan<T, R_SUM, G_HAG_BWD_LEVEL>(h, h->p_bwd_stage[st], h->d_tcol, a, w, s);
        if (rc) return rc;
    }
    a.out = gx;
    a.out_off = 0;
    if (op == HAG_GCN) { a.self = gy; a.self_scale = h->d_inv_deg1; }
    if (!(phases & (HAG_PHASE_GATHER | HAG_PHASE_FOLD))) return HAG_OK;
    return run_plan<T, R_SUM, G_HAG_BWD_SRC>(h, h->p_bwd_src, h->d_tcol, a, w, s, phases);
}

template <typename T>
static int upload_array(hag_handle *h, const std::vector<T> &v, T **dst, hipStream_t s) {
    *dst = nullptr;
    if (v.empty()) return HAG_OK;
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, v.size() * sizeof(T));
    if (e != hipSuccess) { set_error(std::string("hipMalloc: ") + hipGetErrorString(e)); return HAG_ENOMEM; }
    h->d_allocs.push_back(p);
    HIP_TRY(hipMemcpyAsync(p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, s));
    *dst = (T *)p;
    return HAG_OK;
}

static int upload_plan(hag_handle *h, Plan &p, hipStream_t s) {
    int rc = upload_array(h, p.items, &p.d_items, s);
    if (rc) return rc;
    return upload_array(h, p.combine, &p.d_combine, s);
}

void free_device(hag_handle *h) {
    if (!h->d_allocs.empty()) {
        int cur = -1;
        bool sw = hipGetDevice(&cur) == hipSuccess && h->device >= 0 && cur != h->device;
        if (sw) (void)hipSetDevice(h->device);
        for (void *p : h->d_allocs) (void)hipFree(p);
        if (sw) (void)hipSetDevice(cur);
    }
    h->d_allocs.clear();
    h->uploaded = false;
    h->comp_uploaded = false;
}

}  // namespace hag

using namespace hag;

extern "C" {

int hag_upload(hag_t *h, void *stream) {
    if (!h) { set_error("handle is NULL"); return HAG_EINVAL; }
    if (h->uploaded) return HAG_OK;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(hipGetDevice(&h->device));
    int rc = HAG_OK;
    {
        // set-up of the static scratch array for this device (the only place that queries the symbol)
        void *unused = nullptr;
        if ((rc = scratch_address(h->device, &unused))) return rc;
    }
    std::vector<int32_t> slots((size_t)h->max_slots);
    for (size_t i = 0; i < slots.size(); ++i) slots[i] = (int32_t)i;
    if ((rc = upload_array(h, h->left, &h->d_left, s))) goto bad;
    if ((rc = upload_array(h, h->right, &h->d_right, s))) goto bad;
    if ((rc = upload_array(h, h->hf_dcol, &h->d_hcol, s))) goto bad;
    if ((rc = upload_array(h, h->ht_dcol, &h->d_tcol, s))) goto bad;
    if ((rc = upload_array(h, h->he.col, &h->d_ecol, s))) goto bad;
    if ((rc = upload_array(h, h->g_dcol, &h->d_gcol, s))) goto bad;
    if ((rc = upload_array(h, h->gt_dcol, &h->d_gtcol, s))) goto bad;
    if ((rc = upload_array(h, slots, &h->d_slot_ids, s))) goto bad;
    if ((rc = upload_array(h, h->inv_deg, &h->d_inv_deg, s))) goto bad;
    if ((rc = upload_array(h, h->inv_deg1, &h->d_inv_deg1, s))) goto bad;
    {
        // ticket, finished count and give-up flag of the one-launch schedule: zero between launches
        std::vector<int32_t> zeros(kSyncWords, 0);
        if ((rc = upload_array(h, zeros, &h->d_sync, s))) goto bad;
        (void)hipStreamSynchronize(s);   // `zeros` goes out of scope
    }
    if ((rc = upload_plan(h, h->p_fwd, s))) goto bad;
    for (auto &p : h->p_bwd_stage)
        if ((rc = upload_plan(h, p, s))) goto bad;
    for (auto &p : h->p_fwd_stage)
        if ((rc = upload_plan(h, p, s))) goto bad;
    if ((rc = upload_plan(h, h->p_bwd_src, s))) goto bad;
    if ((rc = upload_plan(h, h->p_naive_fwd, s))) goto bad;
    if ((rc = upload_plan(h, h->p_naive_bwd, s))) goto bad;
    if ((rc = upload_array(h, h->p_naive_bwd.slot_row, &h->p_naive_bwd.d_slot_row, s))) goto bad;
    if (h->comp.enabled) {
        Components &c = h->comp;
        if ((rc = upload_array(h, c.meta, &c.d_meta, s))) goto bad;
        if ((rc = upload_array(h, c.stage, &c.d_stage, s))) goto bad;
        for (LocalLists *l : {&c.fwd, &c.fwd_agg, &c.bwd_all, &c.bwd_agg, &c.nfwd, &c.nbwd}) {
            if ((rc = upload_array(h, l->split, &l->d_split, s))) goto bad;
            if ((rc = upload_array(h, l->ptr, &l->d_ptr, s))) goto bad;
            if ((rc = upload_array(h, l->col, &l->d_col, s))) goto bad;
            if ((rc = upload_array(h, l->items, &l->d_items, s))) goto bad;
        }
        h->comp_uploaded = true;
    }
    {
        hipError_t e = hipStreamSynchronize(s);  // host vectors (slots) must outlive the copies
        if (e != hipSuccess) { rc = hip_fail(e, "hipStreamSynchronize"); goto bad; }
    }
    h->uploaded = true;
    for (auto *v : {&h->hf_dcol, &h->ht_dcol, &h->g_dcol, &h->gt_dcol}) std::vector<int32_t>().swap(*v);
    return HAG_OK;
bad:
    (void)hipStreamSynchronize(s);
    free_device(h);
    return rc;
}

size_t hag_workspace_bytes(const hag_t *h, hag_op_t op, hag_dtype_t, int64_t d) {
    if (!h || d <= 0) return 0;
    return carve(h, op, d, nullptr).total;
}

static int forward_entry(const hag_t *h, bool naive, hag_op_t op, hag_dtype_t dt, int64_t d, const void *x, void *y,
                         int32_t *argmax, void *ws, void *stream, uint32_t phases) {
    int rc = check_common(h, op, dt, d, x, y, ws, hag_workspace_bytes(h, op, dt, d) > 0);
    if (rc) return rc;
    if (op == HAG_MAX && !argmax && h->n > 0) { set_error("argmax is required for max"); return HAG_EINVAL; }
    if ((uintptr_t)argmax & 15) { set_error("argmax must be 16-byte aligned"); return HAG_EINVAL; }
    if (x == y && h->n > 0) { set_error("x and y must not alias"); return HAG_EINVAL; }
    hipStream_t s = (hipStream_t)stream;
    if (dt == HAG_F32) {
        if (op == HAG_MAX) return forward_impl<float, R_MAX>(h, naive, op, d, (const float *)x, (float *)y, argmax, ws, s, phases);
        return forward_impl<float, R_SUM>(h, naive, op, d, (const float *)x, (float *)y, argmax, ws, s, phases);
    }
    if (op == HAG_MAX) return forward_impl<int32_t, R_MAX>(h, naive, op, d, (const int32_t *)x, (int32_t *)y, argmax, ws, s, phases);
    return forward_impl<int32_t, R_SUM>(h, naive, op, d, (const int32_t *)x, (int32_t *)y, argmax, ws, s, phases);
}

static int backward_entry(const hag_t *h, bool naive, hag_op_t op, hag_dtype_t dt, int64_t d, const void *gy,
                          const int32_t *argmax, void *gx, void *ws, void *stream, uint32_t phases) {
    const bool needs_ws = (op != HAG_MAX || (h && h->knobs.deterministic_max_backward)) && hag_workspace_bytes(h, op, dt, d) > 0;
    int rc = check_common(h, op, dt, d, gy, gx, ws, needs_ws);
    if (rc) return rc;
    if (op == HAG_MAX && !argmax && h->n > 0) { set_error("argmax is required for max"); return HAG_EINVAL; }
    if (gy == gx && h->n > 0) { set_error("gy and gx must not alias"); return HAG_EINVAL; }
    hipStream_t s = (hipStream_t)stream;
    if (dt == HAG_F32) return backward_impl<float>(h, naive, op, d, (const float *)gy, argmax, (float *)gx, ws, s, phases);
    return backward_impl<int32_t>(h, naive, op, d, (const int32_t *)gy, argmax, (int32_t *)gx, ws, s, phases);
}

int hag_forward(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *x, void *y, int32_t *argmax,
                void *ws, void *stream) {
    return forward_entry(h, false, op, dt, d, x, y, argmax, ws, stream, HAG_PHASE_ALL);
}
int hag_forward_static_scratch(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *x, void *y,
                               int32_t *argmax, void *stream) {
    if (!h) { set_error("handle is NULL"); return HAG_EINVAL; }
    if (!h->uploaded) { set_error("hag_upload has not been called on this handle"); return HAG_ESTATE; }
    if (d <= 0 || d > (1 << 20)) { set_error("d out of range"); return HAG_EINVAL; }
    const size_t need = hag_workspace_bytes(h, op, dt, d);
    if (need > (size_t)HAG_STATIC_SCRATCH_BYTES) {
        set_error("this pass needs " + std::to_string(need) + " bytes of scratch, the static array holds " +
                  std::to_string((size_t)HAG_STATIC_SCRATCH_BYTES) + ": use hag_forward with a workspace");
        return HAG_EINVAL;
    }
    // the address was looked up by hag_upload on the handle's device; no runtime query here
    void *ws = (h->device >= 0 && h->device < kMaxDevices) ? g_scratch_ptr[h->device] : nullptr;
    if (!ws) { set_error("static scratch of the handle's device was not set up"); return HAG_ESTATE; }
    return forward_entry(h, false, op, dt, d, x, y, argmax, ws, stream, HAG_PHASE_ALL);
}
int hag_set_option(hag_t *h, int32_t option, int64_t value) {
    if (!h) { set_error("handle is NULL"); return HAG_EINVAL; }
    switch (option) {
        case HAG_OPT_ONE_LAUNCH_MAX_ITEMS: h->knobs.fuse_max_items = std::max<int64_t>(value, 0); return HAG_OK;
        case HAG_OPT_SPIN_LIMIT: h->knobs.spin_limit = std::max<int64_t>(value, 1); return HAG_OK;
        case HAG_OPT_TEST_WAIT_UNREACHABLE: h->knobs.wait_unreachable = value != 0; return HAG_OK;
        case HAG_OPT_DETERMINISTIC_MAX_BACKWARD: h->knobs.deterministic_max_backward = value != 0; return HAG_OK;
        case HAG_OPT_PARTITION_SHIFT: h->knobs.part_shift = (int32_t)(value & 7); return HAG_OK;
    }
    set_error("unknown option");
    return HAG_EINVAL;
}

int hag_check(const hag_t *h, void *stream) {
    if (!h) { set_error("handle is NULL"); return HAG_EINVAL; }
    if (!h->uploaded) { set_error("hag_upload has not been called on this handle"); return HAG_ESTATE; }
    hipStream_t s = (hipStream_t)stream;
    std::vector<int32_t> words(kSyncWords, 0);
    HIP_TRY(hipMemcpyAsync(words.data(), h->d_sync, sizeof(int32_t) * kSyncWords, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    bool clean = true;
    for (int k = 0; k < kSyncWords; ++k) clean = clean && words[k] == 0;
    if (clean) return HAG_OK;
    // a wait gave up (or a launch did not finish): put the words back to zero for the next launch
    HIP_TRY(hipMemsetAsync(h->d_sync, 0, sizeof(int32_t) * kSyncWords, s));
    HIP_TRY(hipStreamSynchronize(s));
    set_error(words[kSyncGaveUp] ? "a one-launch pass gave up waiting for its earlier phases: its output is not valid"
                       : "a one-launch pass did not run to its end");
    return HAG_ETIMEOUT;
}

int hag_forward_phases(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *x, void *y,
                       int32_t *argmax, void *ws, void *stream, uint32_t phases) {
    return forward_entry(h, false, op, dt, d, x, y, argmax, ws, stream, phases);
}
int hag_naive_forward(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *x, void *y, int32_t *argmax,
                      void *ws, void *stream) {
    return forward_entry(h, true, op, dt, d, x, y, argmax, ws, stream, HAG_PHASE_ALL);
}
int hag_backward(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *gy, const int32_t *argmax,
                 void *gx, void *ws, void *stream) {
    return backward_entry(h, false, op, dt, d, gy, argmax, gx, ws, stream, HAG_PHASE_ALL);
}
int hag_backward_phases(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *gy, const int32_t *argmax,
                        void *gx, void *ws, void *stream, uint32_t phases) {
    return backward_entry(h, false, op, dt, d, gy, argmax, gx, ws, stream, phases);
}
int hag_naive_backward(const hag_t *h, hag_op_t op, hag_dtype_t dt, int64_t d, const void *gy, const int32_t *argmax,
                       void *gx, void *ws, void *stream) {
    return backward_entry(h, true, op, dt, d, gy, argmax, gx, ws, stream, HAG_PHASE_ALL);
}

}  // extern "C"


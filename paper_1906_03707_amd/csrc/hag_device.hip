// Device side of libhag for gfx950 (MI355X): the kernels of Algorithm 2 and of its
// transposed pass, and the C entry points that enqueue them.
//
// The path is a sparse gather-reduce (about one add or compare per four bytes
// loaded), so it is bound by memory traffic, not by arithmetic: there is no MFMA
// here.  What matters is that every neighbour row is fetched with full-width
// coalesced 16-byte loads, that enough independent loads are in flight per wave,
// and that work is balanced across 256 compute units although row lengths are
// heavy-tailed.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <string>
#include <type_traits>

#include "hag_internal.hpp"

namespace hag {

constexpr int kBlock = 256;  // 4 wavefronts of 64 lanes
constexpr int kWave = 64;

enum { R_SUM = 0, R_MAX = 1 };
// which phase a gather launch belongs to: only a tag, so that every phase has a kernel symbol
// of its own in profiler output
enum { G_HAG_FWD = 0, G_HAG_BWD_LEVEL = 1, G_HAG_BWD_SRC = 2, G_NAIVE_FWD = 3, G_NAIVE_BWD = 4, G_FOLD = 5, G_HAG_FWD_STAGE = 6 };

template <typename T> struct V4;
template <> struct V4<float> { using type = float4; };
template <> struct V4<int32_t> { using type = int4; };

template <typename T>
struct GatherArgs {
    const Item *items;
    int np;                   // 1 or kPartitions: workgroup b works on partition b mod np
    struct {
        int64_t begin;        // first item of the partition
        int64_t n_block;      // its first n_block items take one workgroup each
        int64_t n_items;      // all its items
    } seg[kPartitions];
    const int32_t *col;
    const T *src_lo;          // rows of ids < split
    const T *src_hi;          // rows of ids >= split, row (id - split)
    const int32_t *id_hi;     // R_MAX: winning original ids stored beside src_hi rows
    int32_t split;
    T *out;                   // final rows, row (item.row - out_off)
    int32_t *out_id;          // R_MAX
    int32_t out_off;
    T *part;                  // partial slots of split rows
    int32_t *part_id;         // R_MAX
    const float *in_scale;    // optional: multiplies rows of ids < split (mean, transposed pass)
    const float *out_scale;   // optional: multiplies final rows (mean, forward), indexed by item.row
    const T *self;            // optional: row item.row of this matrix is added to a final row (gcn) ...
    const float *self_scale;  // ... after being multiplied by self_scale[item.row], if given
    int32_t d;
    int32_t off32;            // both gathered matrices are smaller than 4 GiB: 32-bit byte offsets
    int32_t stream_hi;        // rows of src_hi are read once (fold of partial rows): streaming loads
};

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ int4 ld4(const int32_t *p) { return *reinterpret_cast<const int4 *>(p); }
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ void st4(int32_t *p, int4 v) { *reinterpret_cast<int4 *>(p) = v; }

typedef float f4v_t __attribute__((ext_vector_type(4)));
typedef int i4v_t __attribute__((ext_vector_type(4)));
// streaming stores: the row is not read again by this launch and should not displace the
// gathered matrices from the caches
__device__ __forceinline__ void st4_stream(float *p, float4 v) {
    f4v_t x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<f4v_t *>(p));
}
__device__ __forceinline__ void st4_stream(int32_t *p, int4 v) {
    i4v_t x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<i4v_t *>(p));
}

__device__ __forceinline__ float4 ld4_stream(const float *p) {
    const f4v_t x = __builtin_nontemporal_load(reinterpret_cast<const f4v_t *>(p));
    return make_float4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ int4 ld4_stream(const int32_t *p) {
    const i4v_t x = __builtin_nontemporal_load(reinterpret_cast<const i4v_t *>(p));
    return make_int4(x.x, x.y, x.z, x.w);
}

__device__ __forceinline__ void add4(float4 &a, const float4 &b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
// int32 sums wrap modulo 2^32: add as unsigned
__device__ __forceinline__ void add4(int4 &a, const int4 &b) {
    a.x = (int)((unsigned)a.x + (unsigned)b.x); a.y = (int)((unsigned)a.y + (unsigned)b.y);
    a.z = (int)((unsigned)a.z + (unsigned)b.z); a.w = (int)((unsigned)a.w + (unsigned)b.w);
}
__device__ __forceinline__ void scale4(float4 &a, float s) { a.x *= s; a.y *= s; a.z *= s; a.w *= s; }
__device__ __forceinline__ void scale4(int4 &, float) {}

// (value, id) max with ties to the smaller id; id < 0 means "nothing yet"
template <typename S>
__device__ __forceinline__ void max1(S &v, int &vi, S w, int wi) {
    bool take = (wi >= 0) && (vi < 0 || w > v || (w == v && wi < vi));
    v = take ? w : v;
    vi = take ? wi : vi;
}
// the same when the candidate's id is known to exceed every id already folded in
template <typename S>
__device__ __forceinline__ void max_first1(S &v, int &vi, S w, int wi) {
    bool take = (wi >= 0) && (vi < 0 || w > v);
    v = take ? w : v;
    vi = take ? wi : vi;
}
template <typename V>
__device__ __forceinline__ void max_first4(V &v, int4 &vi, const V &w, int wi) {
    max_first1(v.x, vi.x, w.x, wi); max_first1(v.y, vi.y, w.y, wi);
    max_first1(v.z, vi.z, w.z, wi); max_first1(v.w, vi.w, w.w, wi);
}
template <typename V>
__device__ __forceinline__ void max4(V &v, int4 &vi, const V &w, const int4 &wi) {
    max1(v.x, vi.x, w.x, wi.x); max1(v.y, vi.y, w.y, wi.y);
    max1(v.z, vi.z, w.z, wi.z); max1(v.w, vi.w, w.w, wi.w);
}

// (value, id) max where the id of an aggregation row (id >= split) stands for the winning
// original id stored beside that row, and is only looked up when a tie makes it matter.
// acc_id is an original id, or an aggregation id whose stored winner has not been needed yet.
// Original ids of a list arrive in ascending order before any aggregation id, so a tie
// between two original ids keeps the accumulator.
template <typename S>
__device__ __forceinline__ void settle_tie1(S v, int &vi, S w, int wi, const int32_t *id_hi, int split, size_t d,
                                            int col) {
    if (vi >= 0 && w == v) {
        const int other = id_hi[(size_t)(wi - split) * d + col];
        const int mine = vi < split ? vi : id_hi[(size_t)(vi - split) * d + col];
        vi = min(mine, other);
    }
}
template <typename V>
__device__ __forceinline__ void lazy_max4(V &v, int4 &vi, const V &w, int wi, const int32_t *id_hi, int split,
                                          size_t d, int cb) {
    if (wi >= split && (w.x == v.x || w.y == v.y || w.z == v.z || w.w == v.w)) {   // rare
        settle_tie1(v.x, vi.x, w.x, wi, id_hi, split, d, cb);
        settle_tie1(v.y, vi.y, w.y, wi, id_hi, split, d, cb + 1);
        settle_tie1(v.z, vi.z, w.z, wi, id_hi, split, d, cb + 2);
        settle_tie1(v.w, vi.w, w.w, wi, id_hi, split, d, cb + 3);
    }
    max_first4(v, vi, w, wi);   // a tie keeps the accumulator, whose id is settled above
}
// replace aggregation ids left in acc_id by the original ids they stand for
__device__ __forceinline__ void resolve_ids(int4 &vi, const int32_t *id_hi, int split, size_t d, int cb) {
    if (vi.x >= split) vi.x = id_hi[(size_t)(vi.x - split) * d + cb];
    if (vi.y >= split) vi.y = id_hi[(size_t)(vi.y - split) * d + cb + 1];
    if (vi.z >= split) vi.z = id_hi[(size_t)(vi.z - split) * d + cb + 2];
    if (vi.w >= split) vi.w = id_hi[(size_t)(vi.w - split) * d + cb + 3];
}

__device__ __forceinline__ Item load_item(const Item *p) {
    const int4 raw = *reinterpret_cast<const int4 *>(p);
    Item it;
    it.beg = ((int64_t)(uint32_t)raw.x) | ((int64_t)raw.y << 32);
    it.cnt = raw.z;
    it.row = raw.w;
    return it;
}

// One step of the reduction: UNR neighbour rows with ids idx[0..UNR) (all valid when !TAIL;
// idx < 0 = nothing when TAIL) for the four features at element offset cb of a row.
// The gathered matrices are addressed as base + 32-bit byte offset when OFF32 (both matrices
// below 4 GiB), which costs one multiply-add per row instead of 64-bit pointer arithmetic.
template <typename T, int RED, int UNR, bool OFF32, bool TAIL, bool LAZY>
__device__ __forceinline__ void reduce_step(const GatherArgs<T> &A, const int (&idx)[UNR], int cb,
                                            typename V4<T>::type &acc, int4 &acc_id) {
    using V = typename V4<T>::type;
    const uint32_t row_bytes = (uint32_t)A.d * 4u, cb_bytes = (uint32_t)cb * 4u;
    const size_t d = (size_t)A.d;
    V val[UNR];
    // Lists are sorted, so ids >= split (rows of the second matrix) come last: most steps see
    // none in the whole wavefront and take the single-matrix path.
    int hi_any = 0;
#pragma unroll
    for (int k = 0; k < UNR; ++k) hi_any |= (idx[k] >= A.split);
    const bool single = !__any(hi_any);
    if (single) {
#pragma unroll
        for (int k = 0; k < UNR; ++k) {
            val[k] = V{};
            if (!TAIL || idx[k] >= 0) {
                if (OFF32) val[k] = ld4(reinterpret_cast<const T *>(reinterpret_cast<const char *>(A.src_lo) +
                                                                     ((uint32_t)idx[k] * row_bytes + cb_bytes)));
                else val[k] = ld4(A.src_lo + (size_t)idx[k] * d + cb);
            }
        }
    } else {
        // mixed: select the address, not the path, so the loads still issue together
        const T *ptr[UNR];
#pragma unroll
        for (int k = 0; k < UNR; ++k) {
            const int id = TAIL ? max(idx[k], 0) : idx[k];
            const bool lo = id < A.split;
            const T *base_ptr = lo ? A.src_lo : A.src_hi;
            ptr[k] = base_ptr + (size_t)(lo ? id : id - A.split) * d + cb;
        }
#pragma unroll
        for (int k = 0; k < UNR; ++k) {
            val[k] = V{};
            if (!TAIL || idx[k] >= 0) val[k] = A.stream_hi ? ld4_stream(ptr[k]) : ld4(ptr[k]);
        }
    }
    if (A.in_scale) {
#pragma unroll
        for (int k = 0; k < UNR; ++k)
            if (idx[k] >= 0 && idx[k] < A.split) scale4(val[k], A.in_scale[idx[k]]);
    }
    if (RED == R_MAX) {
        if (single) {
            // Only original rows here, and a list holds its original ids in ascending order
            // before any aggregation node: whatever the accumulator holds came from a smaller
            // id, so a tie keeps it and "greater than" is the whole test.
#pragma unroll
            for (int k = 0; k < UNR; ++k) max_first4(acc, acc_id, val[k], idx[k]);
        } else if (LAZY) {
#pragma unroll
            for (int k = 0; k < UNR; ++k) lazy_max4(acc, acc_id, val[k], idx[k], A.id_hi, A.split, d, cb);
        } else {
#pragma unroll
            for (int k = 0; k < UNR; ++k) {
                int4 vid = make_int4(idx[k], idx[k], idx[k], idx[k]);   // -1 stays "nothing"
                if (idx[k] >= A.split) vid = ld4(A.id_hi + (size_t)(idx[k] - A.split) * d + cb);
                max4(acc, acc_id, val[k], vid);
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < UNR; ++k) add4(acc, val[k]);
    }
}

// Reduce `cnt` neighbour rows whose ids start at col[beg] into (acc, acc_id), for the four
// features starting at element cb of a row.  Called by all LPR lanes of a sub-group together
// (sub-groups of one wavefront may have different cnt: the loop then simply runs with part of
// the wavefront masked off).  Column ids are read LPR at a time (coalesced) and handed round
// inside the sub-group; UNR neighbour rows are requested before the first is consumed; full
// groups of UNR ids take a path without any per-row predicate.
template <typename T, int RED, int LPR, int UNR, bool OFF32, bool LAZY>
__device__ __forceinline__ void reduce_rows(const GatherArgs<T> &A, int64_t beg, int cnt, int sl, int cb,
                                            typename V4<T>::type &acc, int4 &acc_id) {
    for (int base = 0; base < cnt; base += LPR) {
        const int here = min(LPR, cnt - base);
        const int mine = (sl < here) ? A.col[beg + base + sl] : -1;
        const int full = here & ~(UNR - 1);
        int j = 0;
        for (; j < full; j += UNR) {
            int idx[UNR];
#pragma unroll
            for (int k = 0; k < UNR; ++k) idx[k] = __shfl(mine, j + k, LPR);
            reduce_step<T, RED, UNR, OFF32, false, LAZY>(A, idx, cb, acc, acc_id);
        }
        if (j < here) {
            int idx[UNR];
#pragma unroll
            for (int k = 0; k < UNR; ++k) idx[k] = __shfl(mine, j + k, LPR);
            reduce_step<T, RED, UNR, OFF32, true, LAZY>(A, idx, cb, acc, acc_id);
        }
    }
}

template <typename T, int RED>
__device__ __forceinline__ void store_result(const GatherArgs<T> &A, int row, int cbase, typename V4<T>::type acc,
                                             int4 acc_id) {
    const size_t d = (size_t)A.d;
    if (row >= 0) {
        if (A.self) {
            auto own = ld4(A.self + (size_t)row * d + cbase);
            if (A.self_scale) scale4(own, A.self_scale[row]);
            add4(acc, own);
        }
        if (A.out_scale) scale4(acc, A.out_scale[row]);
        const size_t o = (size_t)(row - A.out_off) * d + cbase;
        st4(A.out + o, acc);
        if (RED == R_MAX) st4(A.out_id + o, acc_id);
    } else {
        const size_t o = (size_t)(~row) * d + cbase;
        // written once, read once by the fold launch: kept out of the caches, partial rows
        // leave the gathered matrices there (unconditional: a run-time choice between the two
        // store forms made the compiler keep the kernel's arguments in scratch memory)
        st4_stream(A.part + o, acc);
        if (RED == R_MAX) st4_stream(A.part_id + o, acc_id);
    }
}

// Gather-reduce.  Lane sl of a sub-group of LPR lanes owns the four consecutive features
// starting at (blockIdx.y * LPR + sl) * 4, so a neighbour row is fetched by LPR adjacent
// lanes as one contiguous run of 16-byte loads.
//   workgroups [0, n_block): one long item each; its 256/LPR sub-groups take equal slices
//     of the neighbour list and fold their partial rows through LDS in a fixed order;
//   later workgroups: one short item per sub-group.
template <typename T, int RED, int LPR, int ROLE>
__global__ __launch_bounds__(kBlock) void gather_kernel(GatherArgs<T> A) {
    using V = typename V4<T>::type;
    constexpr int SG = kWave / LPR;       // sub-groups per wavefront
    constexpr int NSG = kBlock / LPR;     // sub-groups per workgroup
    constexpr int UNR = 4;
    // Max over fp32 rows looks up the winner stored beside an aggregation row only on a tie
    // (exact ties are rare in real-valued features).  int32 features tie all the time, and
    // the fold of partial slots has ids beside every row, so both read them always.
    constexpr bool LAZY = RED == R_MAX && std::is_same<T, float>::value && ROLE != G_FOLD;
    __shared__ V red_val[kBlock];
    __shared__ int4 red_id[RED == R_MAX ? kBlock : 1];
    const int lane = threadIdx.x & (kWave - 1);
    const int sl = lane % LPR;
    const int cbase = (blockIdx.y * LPR + sl) * 4;
    const bool col_ok = cbase < A.d;
    const int cb = col_ok ? cbase : 0;      // lanes past the last feature read column 0 and store nothing
    V acc{};
    int4 acc_id = make_int4(-1, -1, -1, -1);

    const int part = blockIdx.x % A.np;
    const int64_t vb = blockIdx.x / A.np;            // index of this workgroup inside its partition
    const int64_t p_begin = A.seg[part].begin, p_block = A.seg[part].n_block, p_items = A.seg[part].n_items;
    if (vb < p_block) {
        const Item it = load_item(A.items + p_begin + vb);
        const int sg = threadIdx.x / LPR;
        int per = (it.cnt + NSG - 1) / NSG;
        per = (per + UNR - 1) / UNR * UNR;
        const int lo = min(it.cnt, sg * per), hi = min(it.cnt, lo + per);
        if (A.off32) reduce_rows<T, RED, LPR, UNR, true, LAZY>(A, it.beg + lo, hi - lo, sl, cb, acc, acc_id);
        else reduce_rows<T, RED, LPR, UNR, false, LAZY>(A, it.beg + lo, hi - lo, sl, cb, acc, acc_id);
        if (LAZY) resolve_ids(acc_id, A.id_hi, A.split, (size_t)A.d, cb);
        red_val[threadIdx.x] = acc;
        if (RED == R_MAX) red_id[threadIdx.x] = acc_id;
        __syncthreads();
        if (threadIdx.x < LPR && col_ok) {
#pragma unroll
            for (int s = 1; s < NSG; ++s) {
                if (RED == R_MAX) max4(acc, acc_id, red_val[s * LPR + sl], red_id[s * LPR + sl]);
                else add4(acc, red_val[s * LPR + sl]);
            }
            store_result<T, RED>(A, it.row, cbase, acc, acc_id);
        }
        return;
    }
    const int wave = threadIdx.x / kWave;
    const int sg = lane / LPR;
    const int64_t local = p_block + ((vb - p_block) * (kBlock / kWave) + wave) * SG + sg;
    const bool has_item = local < p_items;
    Item it{0, 0, 0};
    if (has_item) it = load_item(A.items + p_begin + local);
    if (A.off32) reduce_rows<T, RED, LPR, UNR, true, LAZY>(A, it.beg, it.cnt, sl, cb, acc, acc_id);
    else reduce_rows<T, RED, LPR, UNR, false, LAZY>(A, it.beg, it.cnt, sl, cb, acc, acc_id);
    if (LAZY) resolve_ids(acc_id, A.id_hi, A.split, (size_t)A.d, cb);
    if (has_item && col_ok) store_result<T, RED>(A, it.row, cbase, acc, acc_id);
}

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

// ------------------------------------------------------------------------------------------
// Component-local pass: a batch of small graphs.  One workgroup per connected component.  Its
// feature rows and the short lists of its aggregation nodes are read from HBM once into LDS,
// its aggregation nodes are evaluated in LDS stage by stage (Algorithm 2's loop over V_A,
// never touching global memory), and every output row is then reduced out of LDS.  The
// transposed pass walks the transposed lists with the stages in reverse order, but splits the
// gradient of an aggregation row in two: the part that comes from destinations depends on
// nothing and is summed in the same walk as the original rows that no aggregation node
// consumes (all these lists are long and alike); only the few terms that come from other
// aggregation rows are then added stage by stage, and the remaining original rows follow.
// A workgroup is short-lived and several share a compute unit, so what bounds the pass is the
// number of dependent LDS / memory round trips per workgroup as much as the LDS bytes moved:
// list ids are requested one step ahead of their use, the lists of the first rows already
// while the rows are staged.  In the row loop a read costs one add that moves the row's byte
// offset across lanes, one 16-byte LDS read and four adds; rows are not padded.
// ------------------------------------------------------------------------------------------
template <typename T>
struct CompArgs {
    const int32_t *meta;         // per component: first node, #nodes, first aggregation slot, #agg | #stages << 16
    const uint8_t *stage;        // stage of each aggregation slot (ascending inside a component)
    // lists of the rows written to global memory: per node slot {first entry in row_col,
    // length | local row index << 16}, each component's rows sorted longest list first
    const int32_t *row_items;
    const uint16_t *row_col;
    // Transposed pass over a HAG: the items of a component (at slot v0 + a0) cover its
    // aggregation rows too (row index >= nv: the sum over the destinations that consume the
    // row, kept in LDS); the first row_split[c] items depend on no aggregation row, the others
    // are the original rows that aggregation nodes consume.  NULL: nv items at slot v0.
    const int32_t *row_split;
    const int32_t *agg_row_ptr;  // lists of the aggregation rows kept in LDS (component-major index)
    const uint16_t *agg_row_col;
    const T *in;
    T *out;
    const float *scale_in, *scale_out;
    const float *self_scale;     // gcn: the node's own staged row times self_scale[v] (1 if NULL) is added
    int32_t add_self;
    int32_t d, stride;           // feature width; row stride in LDS, in elements
    int32_t lists_off;           // offset of the staged aggregation lists, in bytes
    int32_t max_agg;             // most aggregation rows a component has
    int32_t use_agg, reverse;
    int32_t pairs;               // forward pass: every staged list has exactly two entries
    int32_t stream_out;          // output rows are written with streaming stores
};

// Value of lane J of the caller's sub-group of LPR lanes.  A sub-group of 16 lanes is one row of
// the data-parallel-primitive network and one of 4 lanes is a quad, so there the broadcast is
// a plain vector move that leaves the LDS pipe to the row reads; other widths use the
// cross-lane read through LDS.  All lanes of the wavefront must be active.
template <int LPR, int J>
__device__ __forceinline__ int sub_bcast(int v) {
    // every lane is written, so the "old" operand and the bound control do not matter; zero
    // fill lets the compiler fold the move into the instruction that consumes it
    if constexpr (LPR == 16) return __builtin_amdgcn_update_dpp(0, v, 0x150 + J, 0xf, 0xf, true);   // row_newbcast:J
    else if constexpr (LPR == 4) return __builtin_amdgcn_update_dpp(0, v, J * 0x55, 0xf, 0xf, true);  // quad_perm:[J,J,J,J]
    else return __shfl(v, J, LPR);
}

// acc += the LDS rows whose byte offsets lanes J0..J0+3 of the sub-group hold in m
template <typename T, int LPR, int J0>
__device__ __forceinline__ void lds_add4rows(const unsigned char *colbuf, int m, typename V4<T>::type &acc) {
    using V = typename V4<T>::type;
    const int u0 = sub_bcast<LPR, J0>(m), u1 = sub_bcast<LPR, J0 + 1>(m);
    const int u2 = sub_bcast<LPR, J0 + 2>(m), u3 = sub_bcast<LPR, J0 + 3>(m);
    const V a = *reinterpret_cast<const V *>(colbuf + u0);
    const V b = *reinterpret_cast<const V *>(colbuf + u1);
    const V c = *reinterpret_cast<const V *>(colbuf + u2);
    const V e = *reinterpret_cast<const V *>(colbuf + u3);
    add4(acc, a); add4(acc, b); add4(acc, c); add4(acc, e);
}

// Row ids and what a list entry becomes in registers: the byte offset of its LDS row, so that
// the multiplication is done once per entry by the lane that loaded it, not once per row read.
struct RowOffsets {
    int row_bytes;   // LDS row stride in bytes
    int zero;        // offset of the row of zeros / "nothing"
};

// A lane's share of entries [first, first + 4*LPR) of the list col[beg .. beg+cnt): four row
// offsets, that of the zero row past the end.
template <int LPR>
__device__ __forceinline__ void load_ids(int (&m)[4], const uint16_t *col, int beg, int cnt, int first, int sl,
                                         RowOffsets ro) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int e = first + t * LPR + sl;
        m[t] = (e < cnt) ? (int)col[beg + e] * ro.row_bytes : ro.zero;
    }
}

// Add the LDS rows listed in col[beg .. beg+cnt) into acc, for the four features at column 4*k.
// Called by all lanes of a wavefront with a common maxcnt; m holds the first 4*LPR ids
// (load_ids with first = 0).  Entries past cnt read the zero row, so the inner loop has no
// branches.  The next 4*LPR ids are requested before the current ones are consumed.
template <typename T, int LPR>
__device__ __forceinline__ void lds_reduce(const T *buf, RowOffsets ro, const uint16_t *col, int beg, int cnt,
                                           int maxcnt, int sl, int k, const int (&m0)[4],
                                           typename V4<T>::type &acc) {
    using V = typename V4<T>::type;
    constexpr int CH = 4 * LPR;
    const unsigned char *colbuf = reinterpret_cast<const unsigned char *>(buf + 4 * k);
    int m[4] = {m0[0], m0[1], m0[2], m0[3]}, nx[4] = {ro.zero, ro.zero, ro.zero, ro.zero};
    for (int base = 0; base < maxcnt; base += CH) {
        if (base + CH < maxcnt) load_ids<LPR>(nx, col, beg, cnt, base + CH, sl, ro);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int b = base + t * LPR;
            const int lim = min(LPR, maxcnt - b);   // <= 0 past the end
            if constexpr (LPR == 16) {
                if (lim > 0) lds_add4rows<T, LPR, 0>(colbuf, m[t], acc);
                if (lim > 4) lds_add4rows<T, LPR, 4>(colbuf, m[t], acc);
                if (lim > 8) lds_add4rows<T, LPR, 8>(colbuf, m[t], acc);
                if (lim > 12) lds_add4rows<T, LPR, 12>(colbuf, m[t], acc);
            } else if constexpr (LPR == 4) {
                if (lim > 0) lds_add4rows<T, LPR, 0>(colbuf, m[t], acc);
            } else {
                for (int j = 0; j < lim; j += 4) {
                    int u[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) u[r] = __shfl(m[t], j + r, LPR);
#pragma unroll
                    for (int r = 0; r < 4; ++r) add4(acc, *reinterpret_cast<const V *>(colbuf + u[r]));
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) m[t] = nx[t];
    }
}

// largest value of x over the sub-groups of the caller's wavefront (x is the same in all lanes
// of a sub-group); the result is wave-uniform
template <int LPR>
__device__ __forceinline__ int wave_max_over_subgroups(int x) {
    int r = 0;
#pragma unroll
    for (int s = 0; s < kWave / LPR; ++s) r = max(r, __builtin_amdgcn_readlane(x, s * LPR));
    return r;
}

// A wavefront's walk over the rows it reduces: rows come SG = 64/LPR at a time ("group"), group
// g goes to wavefront g mod NW.  The walk keeps the item and the first list ids of the current
// group and the item of the next one in registers, each requested a step before it is needed.
template <int LPR>
struct RowPipe {
    static constexpr int SG = kWave / LPR;
    int2 item, item_next;
    int ids[4];
    int n_groups;
    __device__ __forceinline__ int2 load_item(const int32_t *items, int count, int g, int sgw) const {
        const int slot = g * SG + sgw;
        return (g < n_groups && slot < count) ? *reinterpret_cast<const int2 *>(items + 2 * (size_t)slot) : int2{0, 0};
    }
    __device__ __forceinline__ void start(const int32_t *items, int count, const uint16_t *col, int wave, int nw, int sgw,
                                          int sl, RowOffsets ro) {
        n_groups = (count + SG - 1) / SG;
        item = load_item(items, count, wave, sgw);
        item_next = load_item(items, count, wave + nw, sgw);
        load_ids<LPR>(ids, col, item.x, item.y & 0xffff, 0, sl, ro);
    }
};

// Reduce `count` rows, described by items {first list entry, length | row << 16}, out of LDS.
// A row index below nv is an original node: the result goes to global memory (with the
// epilogue of the op); an index from nv on is an aggregation row and stays in LDS.
template <typename T, int LPR, int NW>
__device__ __forceinline__ void component_rows(const CompArgs<T> &A, T *buf, RowPipe<LPR> &pipe, const int32_t *items,
                                               int count, const uint16_t *col, int v0, int nv, RowOffsets ro, int wave,
                                               int sgw, int sl) {
    using V = typename V4<T>::type;
    constexpr int SG = kWave / LPR;
    const int q = A.d / 4, stride = A.stride;
    for (int g = wave; g < pipe.n_groups; g += NW) {
        // the lists of this wavefront's next group and the item of the one after it
        int ids_next[4];
        load_ids<LPR>(ids_next, col, pipe.item_next.x, pipe.item_next.y & 0xffff, 0, sl, ro);
        const int2 item_after = pipe.load_item(items, count, g + 2 * NW, sgw);
        const bool has = g * SG + sgw < count;
        const int beg = pipe.item.x, cnt = pipe.item.y & 0xffff, v = pipe.item.y >> 16;
        const int maxcnt = wave_max_over_subgroups<LPR>(cnt);
        for (int kb = 0; kb < q; kb += LPR) {
            const int k = min(kb + sl, q - 1);
            V acc{};
            lds_reduce<T, LPR>(buf, ro, col, beg, cnt, maxcnt, sl, k, pipe.ids, acc);
            if (has && kb + sl < q) {
                if (v >= nv) {
                    *reinterpret_cast<V *>(buf + v * stride + 4 * k) = acc;
                } else {
                    if (A.add_self) {
                        // the staged row already carries scale_in, which is the factor the own row needs
                        add4(acc, *reinterpret_cast<const V *>(buf + v * stride + 4 * k));
                    }
                    if (A.scale_out) scale4(acc, A.scale_out[v0 + v]);
                    if (A.stream_out) st4_stream(A.out + (size_t)(v0 + v) * A.d + 4 * k, acc);
                    else st4(A.out + (size_t)(v0 + v) * A.d + 4 * k, acc);
                }
            }
        }
        pipe.item = pipe.item_next;
        pipe.item_next = item_after;
#pragma unroll
        for (int t = 0; t < 4; ++t) pipe.ids[t] = ids_next[t];
    }
}

// Aggregation rows [r0, r1) of one stage, a sub-group per row: row j becomes the sum of the LDS
// rows in its staged list (plus its present content if `accumulate`).
template <typename T, int LPR, int NSG>
__device__ __forceinline__ void component_stage(const CompArgs<T> &A, T *buf, const int32_t *l_agg_ptr,
                                                const uint16_t *l_agg_col, int r0, int r1, int nv, int zrow,
                                                RowOffsets ro, int sg,
                                                int sl, bool accumulate) {
    using V = typename V4<T>::type;
    const int q = A.d / 4, stride = A.stride;
    for (int jb = r0; jb < r1; jb += NSG) {
        const int j = jb + sg;
        const bool has = j < r1;
        const int beg = has ? l_agg_ptr[j] : 0;
        const int cnt = has ? l_agg_ptr[j + 1] - beg : 0;
        const int maxcnt = wave_max_over_subgroups<LPR>(cnt);
        int m[4];
        load_ids<LPR>(m, l_agg_col, beg, cnt, 0, sl, ro);
        for (int kb = 0; kb < q; kb += LPR) {
            const int k = min(kb + sl, q - 1);
            V acc = *reinterpret_cast<const V *>(buf + (has && accumulate ? nv + j : zrow) * stride + 4 * k);
            lds_reduce<T, LPR>(buf, ro, l_agg_col, beg, cnt, maxcnt, sl, k, m, acc);
            if (has && kb + sl < q) *reinterpret_cast<V *>(buf + (nv + j) * stride + 4 * k) = acc;
        }
    }
}

// ROLE only gives each use its own symbol in profiles: 0 = HAG forward, 1 = HAG transposed
// pass, 2 = input graph forward (baseline), 3 = its transposed pass.
template <typename T, int LPR, int BLOCK, int ROLE>
__global__ __launch_bounds__(BLOCK) void component_kernel(CompArgs<T> A) {
    using V = typename V4<T>::type;
    constexpr int NSG = BLOCK / LPR;       // sub-groups per workgroup
    constexpr int NW = BLOCK / kWave;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int st_begin[64];           // stage st is aggregation rows [st_begin[st-1], st_begin[st])
    T *buf = reinterpret_cast<T *>(smem);
    int32_t *l_agg_ptr = reinterpret_cast<int32_t *>(smem + A.lists_off);   // [na+1], rebased
    uint16_t *l_agg_col = reinterpret_cast<uint16_t *>(l_agg_ptr + A.max_agg + 1);
    const int c = blockIdx.x;
    const int4 meta = *reinterpret_cast<const int4 *>(A.meta + 4 * (size_t)c);   // v0, nv, a0, na | stages << 16
    const int v0 = meta.x, nv = meta.y, a0 = meta.z;
    const int na = A.use_agg ? (meta.w & 0xffff) : 0;
    const int n_stages = A.use_agg ? (meta.w >> 16) : 0;
    const int q = A.d / 4, stride = A.stride;
    const int zrow = nv + na;              // a row of zeros / "nothing"
    const RowOffsets ro{stride * (int)sizeof(T), zrow * stride * (int)sizeof(T)};
    const int tid = threadIdx.x, sg = tid / LPR, sl = tid % LPR;
    const int wave = tid / kWave, sgw = (tid & (kWave - 1)) / LPR;

    // Rows are taken SG at a time, longest list first, group g by wavefront g mod NW.  The
    // first group's lists are requested now, the second group's items too.
    const int32_t *items = A.row_items + 2 * (size_t)(A.row_split ? v0 + a0 : v0);
    const int n_first = A.row_split ? A.row_split[c] : nv;       // rows that wait for no aggregation row
    const int n_second = A.row_split ? nv + na - n_first : 0;    // rows that do
    RowPipe<LPR> pipe;
    pipe.start(items, n_first, A.row_col, wave, NW, sgw, sl, ro);

    // stage the component: rows (forward: activations; transposed pass: seeds), the zero row,
    // and the short lists of its aggregation rows
    for (int i = tid; i < nv * q; i += BLOCK) {
        const int r = i / q, k = i - r * q;
        V x = ld4(A.in + (size_t)(v0 + r) * A.d + 4 * k);
        if (A.scale_in) scale4(x, A.scale_in[v0 + r]);
        *reinterpret_cast<V *>(buf + r * stride + 4 * k) = x;
    }
    for (int k = tid; k < q; k += BLOCK) {
        *reinterpret_cast<V *>(buf + zrow * stride + 4 * k) = V{};
    }
    if (na > 0) {
        const int e0 = A.agg_row_ptr[a0], ne = A.agg_row_ptr[a0 + na] - e0;
        for (int i = tid; i <= na; i += BLOCK) l_agg_ptr[i] = A.agg_row_ptr[a0 + i] - e0;
        for (int i = tid; i < ne; i += BLOCK) l_agg_col[i] = A.agg_row_col[e0 + i];
        // every stage 1..n_stages of a component has rows, sorted by stage
        for (int j = tid; j < na; j += BLOCK) {
            const int s0 = A.stage[a0 + j];
            const int s1 = (j + 1 < na) ? (int)A.stage[a0 + j + 1] : n_stages + 1;
            for (int t = s0; t < s1; ++t) st_begin[t] = j + 1;
        }
        if (tid == 0) st_begin[0] = 0;
    }
    __syncthreads();

    // Forward pass: aggregation rows, stage by stage (Algorithm 2's loop over V_A; the host
    // may have expanded the lists down to original rows, then there is a single stage).
    for (int st = 1; st <= (A.reverse ? 0 : n_stages); ++st) {
        const int r0 = st_begin[st - 1], r1 = st_begin[st];
        if (A.pairs) {
            // two-input form: list j is entries 2j and 2j+1
            for (int j = r0 + sg; j < r1; j += NSG) {
                const uint32_t pair = *reinterpret_cast<const uint32_t *>(l_agg_col + 2 * j);
                const int a = (int)(pair & 0xffffu), b = (int)(pair >> 16);
                for (int k = sl; k < q; k += LPR) {
                    V x = *reinterpret_cast<const V *>(buf + a * stride + 4 * k);
                    add4(x, *reinterpret_cast<const V *>(buf + b * stride + 4 * k));
                    *reinterpret_cast<V *>(buf + (nv + j) * stride + 4 * k) = x;
                }
            }
        } else {
            component_stage<T, LPR, NSG>(A, buf, l_agg_ptr, l_agg_col, r0, r1, nv, zrow, ro, sg, sl, false);
        }
        __syncthreads();
    }

    // forward: y[v] over Nhat_v.  Transposed pass: gx[u] over u's consumers for the rows that
    // no aggregation node consumes, and the destination part of every aggregation row.
    component_rows<T, LPR, NW>(A, buf, pipe, items, n_first, A.row_col, v0, nv, ro, wave, sgw, sl);

    if (n_second > 0) {
        pipe.start(items + 2 * (size_t)n_first, n_second, A.row_col, wave, NW, sgw, sl, ro);
        __syncthreads();
        // From the last stage but one down to the first, each aggregation row adds the
        // finished rows of the aggregation nodes built from it (none of this when the host
        // has expanded the lists of the rows below to all aggregation nodes above them).
        for (int st = n_stages - 1; st >= 1; --st) {
            component_stage<T, LPR, NSG>(A, buf, l_agg_ptr, l_agg_col, st_begin[st - 1], st_begin[st], nv, zrow, ro, sg, sl,
                                         true);
            __syncthreads();
        }
        // the original rows that aggregation nodes consume
        component_rows<T, LPR, NW>(A, buf, pipe, items + 2 * (size_t)n_first, n_second, A.row_col, v0, nv, ro, wave,
                                   sgw, sl);
    }
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

// ------------------------------------------------------------------------------------------
// launch helpers
// ------------------------------------------------------------------------------------------
static int hip_fail(hipError_t e, const char *what) {
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    return HAG_EHIP;
}
#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t _e = (expr);                         \
        if (_e != hipSuccess) return hip_fail(_e, #expr); \
    } while (0)

static int pick_lpr(int64_t d) {
    int64_t q = d / 4;
    int l = 4;
    while (l < 64 && l < q) l <<= 1;
    return l;
}

template <typename T, int RED, int LPR, int ROLE>
static int launch_gather_lpr(const GatherArgs<T> &a, hipStream_t s) {
    constexpr int SG = kWave / LPR;
    const int64_t per_block = (kBlock / kWave) * SG;
    int64_t most = 0;   // workgroups of the busiest partition; the grid gives every partition that many
    for (int k = 0; k < a.np; ++k)
        most = std::max(most, a.seg[k].n_block + (a.seg[k].n_items - a.seg[k].n_block + per_block - 1) / per_block);
    const int64_t gx = most * a.np;
    const int64_t gy = (a.d / 4 + LPR - 1) / LPR;
    if (gx <= 0) return HAG_OK;
    if (gx > 0x7fffffffLL || gy > 65535) { set_error("launch too large"); return HAG_EINVAL; }
    hipLaunchKernelGGL((gather_kernel<T, RED, LPR, ROLE>), dim3((unsigned)gx, (unsigned)gy), dim3(kBlock), 0, s, a);
    HIP_TRY(hipGetLastError());
    return HAG_OK;
}

template <typename T, int RED, int ROLE>
static int launch_gather(const GatherArgs<T> &a, hipStream_t s) {
    switch (pick_lpr(a.d)) {
        case 4: return launch_gather_lpr<T, RED, 4, ROLE>(a, s);
        case 8: return launch_gather_lpr<T, RED, 8, ROLE>(a, s);
        case 16: return launch_gather_lpr<T, RED, 16, ROLE>(a, s);
        case 32: return launch_gather_lpr<T, RED, 32, ROLE>(a, s);
        default: return launch_gather_lpr<T, RED, 64, ROLE>(a, s);
    }
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

// run one schedule: the gather itself, then the fold of split rows
template <typename T, int RED, int ROLE>
static int run_plan(const hag_handle *h, const Plan &p, const int32_t *d_col, GatherArgs<T> a, const Workspace &w,
                    hipStream_t s, uint32_t phases = HAG_PHASE_ALL) {
    a.items = p.d_items;
    a.np = p.np;
    // rows of ids < split live in a matrix of `split` rows, the others in one of at most
    // n + a (aggregation rows) or max_slots (partial rows) rows
    {
        const uint64_t row_bytes = (uint64_t)a.d * 4;
        const uint64_t lo_rows = (uint64_t)std::max<int64_t>(a.split, 1);
        // HAG_OFFSET64=1 forces the 64-bit path, which otherwise only matrices of 4 GiB and more take
        const char *e64 = std::getenv("HAG_OFFSET64");
        const bool force64 = e64 && std::atoi(e64) != 0;
        a.off32 = (!force64 && lo_rows * row_bytes < (1ull << 32)) ? 1 : 0;
    }
    // A row is worth a whole workgroup when each of its 256/LPR sub-groups still gets about
    // eight neighbours, and needs one when a single sub-group would walk it for too long.
    {
        const char *esub = std::getenv("HAG_SUB_MAX");     // read per call: a test may change it
        const int64_t sub_max = esub ? std::atoll(esub) : 0LL;
        const int64_t nsg = kBlock / pick_lpr(a.d);
        // A launch too small to fill the device with one sub-group per row (the stages of
        // a small HAG) lasts as long as its longest single-sub-group row: there a row gets
        // a workgroup much sooner.
        const int64_t n_all = p.part_begin[p.np] - p.part_begin[0];
        const bool small_launch = n_all <= 256 * 8 * nsg;
        const int64_t threshold = sub_max > 0 ? sub_max : small_launch ? 16 : std::max<int64_t>(64, 8 * nsg);
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
        c.split = 0;               // every id refers to a partial slot
        c.src_lo = nullptr;
        c.src_hi = (const T *)w.part;
        c.id_hi = (const int32_t *)w.part_id;
        c.in_scale = nullptr;
        rc = launch_gather<T, RED, G_FOLD>(c, s);
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
};
// Padding of an LDS row, in elements (a multiple of 4); none by default: 16-byte LDS reads of
// whole rows by sub-groups of lanes were measured fastest when the row stride is the row
// itself, and any padding made them collide in the banks.  Read per call.
static size_t component_pad() {
    const char *e = std::getenv("HAG_COMPONENT_PAD");
    const long v = e ? std::atol(e) : 0;
    return (size_t)(v < 0 ? 0 : v > 64 ? 64 : v) & ~(size_t)3;
}
// layout.total == 0: the pass does not apply to this call
static CompLayout component_layout(const hag_handle *h, bool naive, bool backward, hag_op_t op, int64_t d) {
    CompLayout L;
    const Components &c = h->comp;
    if (!c.enabled || !h->comp_uploaded) return L;
    // sums only.  Max stays on the generic kernels: their ordered comparison path is cheaper
    // per element than a (value, id) comparison for every LDS row (measured: the LDS variant
    // was the slower one), and its backward pass is a scatter, not a gather.
    if (op == HAG_MAX) return L;
    const size_t stride = (size_t)d + component_pad();
    L.stride = stride;
    const size_t rows = (size_t)c.max_nodes + (naive ? 0 : (size_t)c.max_agg) + 1;
    size_t bytes = rows * stride * 4;
    L.lists_off = bytes;
    if (!naive) {
        const size_t entries = backward ? c.max_entries_bwd : c.max_entries_fwd;   // aggregation lists only
        bytes += ((size_t)c.max_agg + 1) * 4 + ((entries + 1) & ~(size_t)1) * 2;
    }
    bytes = (bytes + 15) & ~(size_t)15;
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
    a.d = (int32_t)d;
    a.stride = (int32_t)L.stride;
    a.use_agg = naive ? 0 : 1;
    a.reverse = BACKWARD ? 1 : 0;
    a.pairs = (!BACKWARD && !c.expanded) ? 1 : 0;
    { const char *e = std::getenv("HAG_STREAM_OUTPUT"); a.stream_out = e ? std::atoi(e) : 0; }   // read per call
    a.lists_off = (int32_t)L.lists_off;
    a.max_agg = c.max_agg;
    // 4 wavefronts per workgroup: 8 were measured slower even where LDS lets only 6 workgroups share
    // a compute unit (fewer, longer row groups per wavefront balance worse)
    const dim3 grid((unsigned)c.count), block(kBlock);
#define HAG_COMPONENT_LAUNCH(LPR_)                                                                                  \
    if (naive) hipLaunchKernelGGL((component_kernel<T, LPR_, kBlock, 2 + (BACKWARD ? 1 : 0)>), grid, block, L.total, s, a); \
    else hipLaunchKernelGGL((component_kernel<T, LPR_, kBlock, BACKWARD ? 1 : 0>), grid, block, L.total, s, a)
    switch (pick_lpr(d)) {
        case 4: HAG_COMPONENT_LAUNCH(4); break;
        case 8: HAG_COMPONENT_LAUNCH(8); break;
        case 16: HAG_COMPONENT_LAUNCH(16); break;
        case 32: HAG_COMPONENT_LAUNCH(32); break;
        default: HAG_COMPONENT_LAUNCH(64); break;
    }
#undef HAG_COMPONENT_LAUNCH
    HIP_TRY(hipGetLastError());
    return HAG_OK;
}

template <typename T, int RED>
static int forward_impl(const hag_handle *h, bool naive, hag_op_t op, int64_t d, const T *x, T *y, int32_t *argmax,
                        void *ws, hipStream_t s, uint32_t phases) {
    // a batch of small graphs: the whole pass is one launch out of LDS
    if (phases == HAG_PHASE_ALL && component_layout(h, naive, false, op, d).total > 0)
        return launch_component<T, false>(h, naive, op, d, x, y, s);
    Workspace w = carve(h, op, d, ws);
    const int32_t n = (int32_t)h->n;
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
    if ((rc = upload_plan(h, h->p_fwd, s))) goto bad;
    for (auto &p : h->p_bwd_stage)
        if ((rc = upload_plan(h, p, s))) goto bad;
    for (auto &p : h->p_fwd_stage)
        if ((rc = upload_plan(h, p, s))) goto bad;
    if ((rc = upload_plan(h, h->p_bwd_src, s))) goto bad;
    if ((rc = upload_plan(h, h->p_naive_fwd, s))) goto bad;
    if ((rc = upload_plan(h, h->p_naive_bwd, s))) goto bad;
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
    int rc = check_common(h, op, dt, d, gy, gx, ws, op != HAG_MAX && hag_workspace_bytes(h, op, dt, d) > 0);
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

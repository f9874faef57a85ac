// Shared by the device translation units of libhag: argument blocks of the kernels, small
// vector helpers, and the launch functions each unit defines for the others.
#pragma once
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

// R_SUMIF: sum of the rows' elements whose entry in a second, int32 matrix (GatherArgs::filter, same
// shape and row index as src_lo) equals the id of the output row: the backward pass of max as a
// gather, gx[u, f] = sum over consumers v of u of gy[v, f] where argmax[v, f] == u, in a fixed order
enum { R_SUM = 0, R_MAX = 1, R_SUMIF = 2 };
// which phase a gather launch belongs to: only a tag, so that every phase has a kernel symbol
// of its own in profiler output
enum { G_HAG_FWD = 0, G_HAG_BWD_LEVEL = 1, G_HAG_BWD_SRC = 2, G_NAIVE_FWD = 3, G_NAIVE_BWD = 4, G_FOLD = 5, G_HAG_FWD_STAGE = 6 };

template <typename T> struct V4;
template <> struct V4<float> { using type = float4; };
template <> struct V4<int32_t> { using type = int4; };

template <typename T>
struct GatherArgs {
    const Item *items;
    int np;                   // 1 or kPartitions: workgroup b works on partition (b + part_shift) mod np
    int part_shift;           // 0 <= part_shift < np
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
    // Fold of partial (value, id) rows of a float max: a stored id >= late_split is an aggregation
    // node standing for the winner stored in late_id (row id - late_split); NULL: stored ids are final
    const int32_t *late_id;
    int32_t late_split;
    const int32_t *filter;    // R_SUMIF: [rows of src_lo, d]
    const int32_t *slot_row;  // R_SUMIF: output row of every partial slot
    // One-launch schedule only (sync_complete NULL otherwise): an item marked as depending on earlier
    // phases waits until sync_complete[k] > wait_bias for every earlier phase k < wait_n, polling at
    // most spin_limit times in all; a wait that gives up sets *sync_gave_up and goes on (every access
    // stays in bounds; the result is then not valid).
    const int32_t *sync_complete;
    int32_t *sync_gave_up;
    int32_t coherent_out;     // this phase's rows are read by later phases of the same launch
    int32_t wait_n;
    int32_t wait_bias;        // 0; tests make it large, so that no phase ever counts as complete
    int32_t spin_limit;
};

// One pass (all aggregation-node stages and the gather over V) as a single launch.  Workgroups
// take tickets in the order they start; ticket ranges map to phases, earlier phases first, so
// whatever a workgroup waits for belongs to workgroups that are already running and never wait
// for it.
constexpr int kMaxPhases = 8;
// Layout of the schedule's device words.  What is polled (the completion flags) sits in cache lines of
// its own, apart from what is updated with atomics (ticket, counts): thousands of waiting wavefronts
// reading a line would otherwise hold up the very updates they wait for.
constexpr int kSyncLine = 32;   // words per 128-byte line
constexpr int kSyncTicket = 0, kSyncFinished = kSyncLine, kSyncGaveUp = 2 * kSyncLine, kSyncDone = 4 * kSyncLine,
              kSyncComplete = kSyncDone + kMaxPhases * kSyncLine, kSyncWords = kSyncComplete + kMaxPhases * kSyncLine;
template <typename T>
struct FusedArgs {
    GatherArgs<T> base;       // everything the phases share; the per-phase fields below overwrite theirs
    struct Phase {
        const Item *items;
        const int32_t *col;
        int64_t n_block, n_items;
        T *out;
        int32_t *out_id;
        int32_t out_off;
        int32_t block_begin;  // first ticket of the phase = number of workgroups of all earlier phases
    } ph[kMaxPhases];
    int32_t n_phases;
    int32_t total_blocks;     // units of work (one workgroup's worth each) over all phases
    int32_t chunk;            // consecutive units a workgroup draws per ticket
    int32_t grid;             // workgroups launched
    // epilogue of the last phase (the rows of V)
    const float *out_scale;
    const T *self;
    const float *self_scale;
    // device words ticket, finished, gave_up, done[k], complete[k] (k < kMaxPhases; offsets kSync*, one
    // 128-byte line each): all but gave_up are zero at launch and put back to zero by the last
    // workgroup of the launch to finish; done[k] counts the finished workgroups of phase k, whose
    // last one sets complete[k]
    int32_t *sync;
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

// Rows that one phase of a one-launch pass writes and a later phase of the same launch reads, on
// another compute unit and possibly another XCD: element-wise device-scope accesses, which are
// written through to, and read from, the level all XCDs share instead of a private cache.
__device__ __forceinline__ float4 ld4_coherent(const float *p) {
    float4 v;
    v.x = __hip_atomic_load(p + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.y = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.z = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.w = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return v;
}
__device__ __forceinline__ int4 ld4_coherent(const int32_t *p) {
    int4 v;
    v.x = __hip_atomic_load(p + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.y = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.z = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.w = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return v;
}
__device__ __forceinline__ void st4_coherent(float *p, float4 v) {
    __hip_atomic_store(p + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st4_coherent(int32_t *p, int4 v) {
    __hip_atomic_store(p + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool COH>
__device__ __forceinline__ int ld1_id(const int32_t *p) {
    if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
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
// the same for a candidate known to be valid, with the emptiness of the accumulator given as a flag
template <typename V>
__device__ __forceinline__ void max_filled4(V &v, int4 &vi, const V &w, int wi, bool empty) {
    const bool tx = empty | (w.x > v.x), ty = empty | (w.y > v.y), tz = empty | (w.z > v.z), tw = empty | (w.w > v.w);
    v.x = tx ? w.x : v.x; vi.x = tx ? wi : vi.x;
    v.y = ty ? w.y : v.y; vi.y = ty ? wi : vi.y;
    v.z = tz ? w.z : v.z; vi.z = tz ? wi : vi.z;
    v.w = tw ? w.w : v.w; vi.w = tw ? wi : vi.w;
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
template <bool COH, typename S>
__device__ __forceinline__ void settle_tie1(S v, int &vi, S w, int wi, const int32_t *id_hi, int split, size_t d,
                                            int col) {
    if (vi >= 0 && w == v) {
        const int other = ld1_id<COH>(id_hi + (size_t)(wi - split) * d + col);
        const int mine = vi < split ? vi : ld1_id<COH>(id_hi + (size_t)(vi - split) * d + col);
        vi = min(mine, other);
    }
}
template <bool COH, typename V>
__device__ __forceinline__ void lazy_max4(V &v, int4 &vi, const V &w, int wi, const int32_t *id_hi, int split,
                                          size_t d, int cb) {
    if (wi >= split && (w.x == v.x || w.y == v.y || w.z == v.z || w.w == v.w)) {   // rare
        settle_tie1<COH>(v.x, vi.x, w.x, wi, id_hi, split, d, cb);
        settle_tie1<COH>(v.y, vi.y, w.y, wi, id_hi, split, d, cb + 1);
        settle_tie1<COH>(v.z, vi.z, w.z, wi, id_hi, split, d, cb + 2);
        settle_tie1<COH>(v.w, vi.w, w.w, wi, id_hi, split, d, cb + 3);
    }
    max_first4(v, vi, w, wi);   // a tie keeps the accumulator, whose id is settled above
}
// (value, id) max of partial results whose ids may still be aggregation ids (>= split) standing for the
// winner stored in `late`: a tie between two such partial results is settled on the original ids
template <typename S>
__device__ __forceinline__ void late_max1(S &v, int &vi, S w, int wi, const int32_t *late, int split, size_t d, int col) {
    if (wi < 0) return;
    if (vi >= 0 && w == v && (wi >= split || vi >= split)) {   // rare
        if (wi >= split) wi = late[(size_t)(wi - split) * d + col];
        if (vi >= split) vi = late[(size_t)(vi - split) * d + col];
    }
    const bool take = vi < 0 || w > v || (w == v && wi < vi);
    v = take ? w : v;
    vi = take ? wi : vi;
}
template <typename V>
__device__ __forceinline__ void late_max4(V &v, int4 &vi, const V &w, const int4 &wi, const int32_t *late, int split,
                                          size_t d, int cb) {
    late_max1(v.x, vi.x, w.x, wi.x, late, split, d, cb);
    late_max1(v.y, vi.y, w.y, wi.y, late, split, d, cb + 1);
    late_max1(v.z, vi.z, w.z, wi.z, late, split, d, cb + 2);
    late_max1(v.w, vi.w, w.w, wi.w, late, split, d, cb + 3);
}
// replace aggregation ids left in acc_id by the original ids they stand for
template <bool COH>
__device__ __forceinline__ void resolve_ids(int4 &vi, const int32_t *id_hi, int split, size_t d, int cb) {
    if (vi.x >= split) vi.x = ld1_id<COH>(id_hi + (size_t)(vi.x - split) * d + cb);
    if (vi.y >= split) vi.y = ld1_id<COH>(id_hi + (size_t)(vi.y - split) * d + cb + 1);
    if (vi.z >= split) vi.z = ld1_id<COH>(id_hi + (size_t)(vi.z - split) * d + cb + 2);
    if (vi.w >= split) vi.w = ld1_id<COH>(id_hi + (size_t)(vi.w - split) * d + cb + 3);
}

struct DevItem {
    int64_t beg;
    int32_t cnt, row;
    bool depends;             // reads rows produced by an earlier phase of the pass
};
__device__ __forceinline__ DevItem load_item(const Item *p) {
    const int4 raw = *reinterpret_cast<const int4 *>(p);
    DevItem it;
    it.beg = ((int64_t)(uint32_t)raw.x) | ((int64_t)(raw.y & 0x3fffffff) << 32);
    it.depends = (raw.y >> 30) & 1;          // kItemDependsBit
    it.cnt = raw.z;
    it.row = raw.w;
    return it;
}


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
    int32_t d, stride;           // feature columns this workgroup handles (columns blockIdx.y * d ...); row stride in LDS, in elements
    int32_t gd;                  // row stride of the matrices in global memory, in elements (the full feature width)
    int32_t lists_off;           // offset of the staged aggregation lists, in bytes
    int32_t max_agg;             // most aggregation rows a component has
    int32_t use_agg, reverse;
    int32_t pairs;               // forward pass: every staged list has exactly two entries
    int32_t stream_out;          // output rows are written with streaming stores
};

static inline int hip_fail(hipError_t e, const char *what) {
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    return HAG_EHIP;
}
#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t _e = (expr);                         \
        if (_e != hipSuccess) return hip_fail(_e, #expr); \
    } while (0)

// lanes that share one feature row: the power of two that covers d/4 float4 columns, 4..64
static inline int pick_lpr(int64_t d) {
    int64_t q = d / 4;
    int l = 4;
    while (l < 64 && l < q) l <<= 1;
    return l;
}

// Defined in the gather units (one per element type and reduction), used by hag_device.hip.
template <typename T, int RED, int ROLE>
int launch_gather(const GatherArgs<T> &a, hipStream_t s);
// ROLE: G_HAG_FWD (forward pass) or G_HAG_BWD_SRC (transposed pass)
template <typename T, int RED, int ROLE>
int launch_fused(const FusedArgs<T> &a, hipStream_t s);

// Defined in the component units (one per element type).  role: 0 = HAG forward, 1 = HAG
// transposed pass, 2 = input graph forward (baseline), 3 = its transposed pass.
template <typename T>
int launch_component_kernel(const CompArgs<T> &a, int role, int64_t d, unsigned components, unsigned column_parts,
                            size_t lds_bytes, hipStream_t s);

}  // namespace hag

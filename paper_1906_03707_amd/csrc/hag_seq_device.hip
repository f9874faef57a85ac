// Device path for a SEQUENTIAL Aggregate (Section 3.1): an LSTM aggregator over ordered neighbour
// lists, run over a prefix HAG found by hag_seq_search (or over the plain lists).
//
// A prefix HAG turns the lists into a forest of states: the state after the one-element prefix (u)
// has no predecessor, an aggregation node w = (v1, v2) is "the state of v1, then x[v2]" (Equation 2:
// cover(w) = (cover(v1), cover(v2))), and every v continues from the state of its list's head
// through the rest of its list (Algorithm 2: aggregation nodes first, then the nodes of V).  The
// forest is cut into PATHS: every state hands its running (h, c) on to one continuation (its
// largest subtree, or one node's private remainder) without a trip through memory, and is written
// to memory only if something else needs it (another path starts there, or it is some a_v).  A path
// that starts from a written state is one level above the path that wrote it; one launch runs all
// paths of a level, 64 per workgroup, each step a gathered matrix product on the matrix cores:
//     gates^T [4H, paths] = Wp [4H, D+H] . Z^T [D+H, paths],    Z[j] = (x[in_j], h_j),
// 32 gate rows x 32 paths per wavefront tile with v_mfma_f32_32x32x2_f32 (fp32 in, fp32 out).  The rows of
// Wp are ordered (hidden unit, gate), so a lane ends up holding all four gates of its hidden units
// for its path and the cell's element-wise part runs in registers.  A wavefront keeps its slice of
// Wp in registers for the whole launch; the operand rows of a tile of paths are staged in LDS.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "hag_device_common.hpp"

struct hag_seq {
    int64_t n = 0, e = 0, n_merges = 0, n_states = 0;
    std::vector<int32_t> final_state; // per node: state row holding a_v, -1 for an empty list, -2: written by its path
    // paths, level by level, longest first within a level: 4 per path, (state row it starts from or -1,
    // first step, steps, node whose a_v its last h is or -1); per step the input row and the state row the
    // step's (h, c) is written to (-1: not needed outside the path)
    std::vector<int32_t> paths, step_x, step_out;
    std::vector<int64_t> level_ptr;   // paths of level l: [level_ptr[l], level_ptr[l+1])
    std::vector<int64_t> tile_ptr;    // tiles of 64 paths of level l: [tile_ptr[l], tile_ptr[l+1]) (a tile never mixes levels)
    // The same paths in the order of the one-launch pass: grouped by the DEPTH of the state they start from (the
    // number of evaluations behind it; 0 for the zero state), longest first within a group.  A path that writes a
    // state starts from a shallower one, so here too a path depends only on earlier groups; and the order follows
    // the time at which start states become available, which keeps tiles from waiting.
    std::vector<int32_t> paths_by_depth;
    std::vector<int64_t> depth_ptr, depth_tile_ptr;
    int64_t longest = 0;
    bool one_launch = true;           // HAG_SEQ_ONE_LAUNCH (default 1): all levels in one launch, paths waiting for the states they start from
    int32_t spin_limit = 1 << 21;     // HAG_SPIN_LIMIT: polls (about half a microsecond apart) after which such a wait gives up
    bool wait_unreachable = false;    // tests only: flags are never set, so every wait gives up
    int32_t *d_final = nullptr, *d_paths = nullptr, *d_step_x = nullptr, *d_step_out = nullptr;   // d_paths: padded to whole tiles per level
    int32_t *d_paths_by_depth = nullptr;                    // likewise per depth group
    // for the backward pass: per step where its h_{t-1} lives (>= 0: that step's tape row, -1: the zero state,
    // <= -2: state row -(value) - 2), and the steps grouped by the input row they read (for the gradient of x)
    std::vector<int32_t> step_prev, xt_ptr, xt_idx;
    std::vector<int32_t> pending_init;   // per state: the paths that start from it
    int32_t *d_step_prev = nullptr, *d_xt_ptr = nullptr, *d_xt_idx = nullptr, *d_pending_init = nullptr;
    int64_t resident_reverse[3] = {0, 0, 0};   // reverse kernel variants <false,1>, <false,2>, <true,2>
    int64_t resident[6] = {0, 0, 0, 0, 0, 0};
    int64_t resident_tape[6] = {0, 0, 0, 0, 0, 0};   // likewise for the variants that write the tape   // per kernel variant: workgroups the device holds at once (set by hag_seq_upload)
    int32_t *d_gave_up = nullptr;     // set by a wait that gave up; read and cleared by hag_seq_check
    int device = -1;
};

namespace hag {

constexpr int kSeqJobs = 64;      // paths per tile
constexpr int kSeqMaxK = 256;     // D + H at most (128 for the variants that hold Wp in registers)

// Wp / bp from the usual layout: w_ih [4H, D], w_hh [4H, H], b [4H], gate-major rows (input, forget,
// cell, output gate).
__global__ __launch_bounds__(256) void seq_pack_kernel(const float *__restrict__ w_ih, const float *__restrict__ w_hh,
                                                      const float *__restrict__ b, float *__restrict__ wp,
                                                      float *__restrict__ bp, int d, int hidden, int kp, int operand_order,
                                                      int32_t *__restrict__ flags, int64_t n_flags) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)4 * hidden * kp;
    // the "state is written" flags of this pass start at zero
    for (int64_t f = i; f < n_flags; f += (int64_t)gridDim.x * 256) flags[f] = 0;
    if (i >= total) return;
    int r = (int)(i / kp), k = (int)(i % kp);
    if (operand_order) {
        // the kernel that streams Wp reads it in the order its matrix instructions consume it:
        // [gate tile][4 k-steps][lane][step in the group], lane l supplying row l % 32 and column 2 * step + l / 32
        const int per_tile = 32 * kp, tile = (int)(i / per_tile), rest = (int)(i % per_tile);
        const int q = rest / 256, lane = (rest % 256) / 4, step = 4 * q + (rest & 3);
        r = tile * 32 + (lane & 31);
        k = 2 * step + (lane >> 5);
    }
    const int unit = r >> 2, gate = r & 3, src_row = gate * hidden + unit;
    float v = 0.f;
    if (k < d) v = w_ih[(size_t)src_row * d + k];
    else if (k < d + hidden) v = w_hh[(size_t)src_row * hidden + (k - d)];
    wp[i] = v;
    if (k == 0) bp[r] = b[src_row];                        // (every row has exactly one element with k == 0 in either order)
}

// Gate functions on the hardware's exp2 and reciprocal: absolute error of a few 1e-7 on outputs in (0, 1) and
// (-1, 1), against ~150 instructions per hidden unit for the library versions, which made the element-wise
// part as long as the matrix products.
__device__ __forceinline__ float seq_sigmoid(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }
__device__ __forceinline__ float seq_tanh(float z) {
    const float e = __expf(-2.f * fabsf(z));             // in (0, 1]: no overflow, no cancellation in 1 + e
    return copysignf((1.f - e) * __builtin_amdgcn_rcpf(1.f + e), z);
}

typedef float seq_acc_t __attribute__((ext_vector_type(16)));

struct SeqChainArgs {
    const int32_t *chains;   // paths, 4 per path, in tiles of 64 (padded with empty paths), longest first within a level
    int64_t n_path_tiles;
    int32_t *flags;          // per state row: set once the row is written (NULL: every start state was written by an earlier launch)
    int32_t *gave_up;        // set by a wait that gives up
    int32_t spin_limit;      // polls of a flag before giving up
    int32_t publish;         // 0 in a test of the time-out: no flag is ever set
    const int32_t *step_x;   // per step: input row
    const int32_t *step_out; // per step: state row to write, or -1
    const float *x, *wp, *bp;
    float *h, *c;            // [n_states, H]: read where a path starts (written by a lower level), written where a step says so
    float *a_out;            // [n, H]
    float *tape_g, *tape_c, *tape_h;   // training: per step the activated gates [H][4], the new c [H] and the new h [H] (NULL: inference)
    int32_t d, hidden;
};

// State rows that another workgroup of the same launch reads, possibly on another XCD: device-scope accesses,
// which are written through to, and read from, the level all XCDs share instead of a private cache; eight bytes
// at a time (the widest access that has a device-scope form).
__device__ __forceinline__ float4 seq_ld4_device(const float *p) {
    const unsigned long long a = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long b = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float4(__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)), __uint_as_float((unsigned)b), __uint_as_float((unsigned)(b >> 32)));
}
__device__ __forceinline__ void seq_st4_device(float *p, float4 v) {
    const unsigned long long a = (unsigned long long)__float_as_uint(v.x) | ((unsigned long long)__float_as_uint(v.y) << 32);
    const unsigned long long b = (unsigned long long)__float_as_uint(v.z) | ((unsigned long long)__float_as_uint(v.w) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p) + 1, b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Hides a value's origin from the optimiser, so that what is derived from it is computed where it is used
// instead of being held in a register across the products.
__device__ __forceinline__ int seq_opaque(int v) { asm volatile("" : "+v"(v)); return v; }

// One level of paths.  A workgroup of 8 wavefronts takes tiles of 64 paths and walks ALL their steps:
// the running states never leave the compute unit (h in the staged operand rows, c beside them in LDS),
// so a step costs one input row of global traffic, plus the two state rows where something else needs
// them.  Paths are sorted by length, so the paths of a tile end within a step or two of each other; a
// path that has ended keeps its state while the others finish.  KSTEPS = KP / 2 matrix-core steps per
// 32 x 32 product.  WIDE (hidden > 32, up to 8 gate tiles of 8 hidden units): wavefront w holds gate
// tile w and multiplies it with both halves of the path tile; otherwise (up to 4 gate tiles) wavefront w
// holds gate tile w % 4 and takes the half w / 4 of the path tile.  Either way a wavefront keeps one gate
// tile of Wp in registers (64 of the 128 it may use at four wavefronts per SIMD, 32 more for the
// accumulators), so the staging and element-wise phases of one workgroup hide behind the products of the other.
//
// BIG (hidden up to 128, D + H up to 256): 16 wavefronts, wavefront w takes gate tile w and both halves of the
// path tile; Wp no longer fits the registers of a compute unit, so every wavefront streams its gate tile,
// stored in the order the matrix instructions consume it, from the L2 cache once per step (16-byte loads, one
// group of four k-steps ahead): 4H (D + H) * 4 bytes per 64 cells, against 2 * 4H (D + H) * 64 flops.
template <int KSTEPS, bool WIDE, bool BIG, bool TAPE>
__global__ __launch_bounds__(BIG ? 1024 : 512, (TAPE && !BIG) ? 2 : 4) void seq_chain_kernel(SeqChainArgs A) {
    static_assert(!BIG || WIDE, "the streamed variant uses the wide tiling");
    constexpr int KP = 2 * KSTEPS, ZS = KP + 2;
    constexpr int HMAX = BIG ? 128 : (WIDE ? 64 : 32);
    constexpr int HS = HMAX + 1, JG = WIDE ? 2 : 1;
    constexpr int TPP = BIG ? 16 : 8;                      // threads per path in the staging phases
    __shared__ float z[kSeqJobs * ZS];
    __shared__ float cs[kSeqJobs * HS];
    __shared__ __align__(16) float sb[4 * (BIG ? 128 : 64)];
    __shared__ int32_t sdesc[kSeqJobs * 4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hidden = A.hidden, d = A.d, n_tiles = hidden / 8;
    const int tile = WIDE ? wave : (wave & 3), group0 = WIDE ? 0 : (wave >> 2);
    float wreg[BIG ? 1 : KSTEPS];
    if constexpr (!BIG) {
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s)
            wreg[s] = tile < n_tiles ? A.wp[(size_t)(tile * 32 + (lane & 31)) * KP + 2 * s + (lane >> 5)] : 0.f;
    }
    if ((int)threadIdx.x < 4 * hidden) sb[threadIdx.x] = A.bp[threadIdx.x];
    constexpr int ZV = KP / (4 * TPP);
    for (int64_t ct = blockIdx.x; ct < A.n_path_tiles; ct += gridDim.x) {
        {
            const int tid0 = seq_opaque(threadIdx.x);
            if (tid0 < kSeqJobs * 4) sdesc[tid0] = A.chains[ct * (kSeqJobs * 4) + tid0];
        }
        __syncthreads();
        if (A.flags) {
            // All levels in one launch: wait until the states this tile's paths start from are written.  They
            // belong to tiles with a smaller index, which this or another resident workgroup finishes without
            // waiting for this one, so the wait ends; it is bounded all the same, and a time-out is recorded.
            const int tid0 = seq_opaque(threadIdx.x);
            if (tid0 < kSeqJobs) {
                const int start = sdesc[tid0 * 4];
                if (start >= 0) {
                    bool ready = false;
                    for (int spin = 0; spin < A.spin_limit; ++spin) {
                        if (__hip_atomic_load(A.flags + start, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { ready = true; break; }
                        // once any wait of the pass has given up its output is void: the others do not sit theirs out
                        if (__hip_atomic_load(A.gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                        __builtin_amdgcn_s_sleep(16);
                    }
                    if (!ready) __hip_atomic_store(A.gave_up, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();
            // the awaited rows are read with device-scope loads, which do not look into a private cache, so no
            // cache is invalidated here; the fence keeps those loads behind the polls
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        }
        // (thread indices are derived again in every phase, and the descriptor is re-read from LDS where it is needed rather than held in registers, which are short)
        const int steps = sdesc[2];                        // the tile's first path is its longest
        // the state the path starts from, the first input row, zero padding
        {
            const int tid = seq_opaque(threadIdx.x), sj = tid / TPP, part = tid % TPP;
            const int start = sdesc[sj * 4], beg = sdesc[sj * 4 + 1], len = sdesc[sj * 4 + 2];
            const int row0 = len > 0 ? A.step_x[beg] : -1;
#pragma unroll 1                                           // (one vector in flight: this runs once per tile, and registers are short)
            for (int i = 0; i < ZV; ++i) {
                const int k = part * 4 + 4 * TPP * i;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < d) { if (row0 >= 0) v = *reinterpret_cast<const float4 *>(A.x + (size_t)row0 * d + k); }
                else if (k < d + hidden && start >= 0)
                    v = A.flags ? seq_ld4_device(A.h + (size_t)start * hidden + (k - d)) : *reinterpret_cast<const float4 *>(A.h + (size_t)start * hidden + (k - d));
                *reinterpret_cast<float2 *>(&z[sj * ZS + k]) = make_float2(v.x, v.y);
                *reinterpret_cast<float2 *>(&z[sj * ZS + k + 2]) = make_float2(v.z, v.w);
            }
            for (int u = part * 4; u < hidden; u += 4 * TPP) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (start >= 0) v = A.flags ? seq_ld4_device(A.c + (size_t)start * hidden + u) : *reinterpret_cast<const float4 *>(A.c + (size_t)start * hidden + u);
                cs[sj * HS + u] = v.x; cs[sj * HS + u + 1] = v.y; cs[sj * HS + u + 2] = v.z; cs[sj * HS + u + 3] = v.w;
            }
        }
        __syncthreads();
        for (int t = 0; t < steps; ++t) {
            // the next step's input row is requested before this step's products and lands in LDS after them
            // (its first 64 columns, that is: holding more across the products would spill registers)
            constexpr int ZE = ZV < 2 ? ZV : 2;
            float4 xr[ZE];
            const int tid = seq_opaque(threadIdx.x), sj = tid / TPP, part = tid % TPP;
            const int len = sdesc[sj * 4 + 2], at = sdesc[sj * 4 + 1] + t;
            const int row1 = t + 1 < len ? A.step_x[at + 1] : -1;
#pragma unroll
            for (int i = 0; i < ZE; ++i) {
                const int k = part * 4 + 4 * TPP * i;
                xr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < d && row1 >= 0) xr[i] = *reinterpret_cast<const float4 *>(A.x + (size_t)row1 * d + k);
            }
            seq_acc_t acc[JG];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float4 bias = tile < n_tiles ? *reinterpret_cast<const float4 *>(&sb[(tile * 8 + 2 * m + (lane >> 5)) * 4])
                                                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int g = 0; g < JG; ++g) { acc[g][4 * m] = bias.x; acc[g][4 * m + 1] = bias.y; acc[g][4 * m + 2] = bias.z; acc[g][4 * m + 3] = bias.w; }
            }
            const float *zl = &z[(group0 * 32 + (lane & 31)) * ZS + (lane >> 5)];
            if constexpr (!BIG) {
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
                    for (int g = 0; g < JG; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[s], zl[g * 32 * ZS + 2 * s], acc[g], 0, 0, 0);
                }
            } else if (tile < n_tiles) {                   // (a wavefront without a gate tile has nothing to stream)
                const float4 *wq = reinterpret_cast<const float4 *>(A.wp) + (size_t)tile * (KSTEPS / 4) * 64 + lane;
                float4 wa = wq[0];
                constexpr int UNR = KSTEPS == 96 ? 12 : 16;   // a divisor of the trip count: how far the loads run ahead within the registers there are
#pragma unroll UNR
                for (int q = 0; q < KSTEPS / 4; ++q) {
                    const float4 wn = wq[(q + 1 < KSTEPS / 4 ? q + 1 : q) * 64];
                    const float w4[4] = {wa.x, wa.y, wa.z, wa.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
#pragma unroll
                        for (int g = 0; g < JG; ++g)
                            acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(w4[r], zl[g * 32 * ZS + 2 * (4 * q + r)], acc[g], 0, 0, 0);
                    }
                    wa = wn;
                }
            }
            __syncthreads();                               // every product has read z
            // the state row this step writes, if any: asked for now, used after the next barrier
            int keep = -1;
            {
                const int tid1 = seq_opaque(threadIdx.x), sj1 = tid1 / TPP;
                if (t < sdesc[sj1 * 4 + 2]) keep = A.step_out[sdesc[sj1 * 4 + 1] + t];
            }
            // element-wise part: lane l holds, for path l % 32 of its half, gate rows 8 * (r / 4) + 4 * (l / 32) + r % 4 of the
            // gate tile, i.e. the four gates (r % 4) of hidden units 2 * (r / 4) + l / 32 of the tile; the new h goes straight
            // into the operand rows of the next step
            if (tile < n_tiles) {
#pragma unroll
                for (int g = 0; g < JG; ++g) {
                    const int j = (group0 + g) * 32 + (lane & 31);
                    if (t < sdesc[j * 4 + 2]) {
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            const int unit = tile * 8 + 2 * m + (lane >> 5);
                            const float c_new = seq_sigmoid(acc[g][4 * m + 1]) * cs[j * HS + unit] +
                                                seq_sigmoid(acc[g][4 * m + 0]) * seq_tanh(acc[g][4 * m + 2]);
                            cs[j * HS + unit] = c_new;
                            if constexpr (TAPE) {
                                // what the backward pass needs of this cell, indexed by the step
                                const float gi = seq_sigmoid(acc[g][4 * m + 0]), gf = seq_sigmoid(acc[g][4 * m + 1]);
                                const float gg = seq_tanh(acc[g][4 * m + 2]), go = seq_sigmoid(acc[g][4 * m + 3]);
                                const float h_new = go * seq_tanh(c_new);
                                const size_t cell = (size_t)(sdesc[j * 4 + 1] + t) * hidden + unit;
                                *reinterpret_cast<float4 *>(A.tape_g + cell * 4) = make_float4(gi, gf, gg, go);
                                z[j * ZS + d + unit] = h_new;              // (c and h go to the tape as whole rows, below)
                                continue;
                            }
                            z[j * ZS + d + unit] = seq_sigmoid(acc[g][4 * m + 3]) * seq_tanh(c_new);
                        }
                    }
                }
            }
            {
                const int tid2 = seq_opaque(threadIdx.x), sj2 = tid2 / TPP, part2 = tid2 % TPP;
                if (row1 >= 0) {
#pragma unroll
                    for (int i = 0; i < ZV; ++i) {
                        const int k = part2 * 4 + 4 * TPP * i;
                        if (k < d) {
                            const float4 v = i < ZE ? xr[i < ZE ? i : 0] : *reinterpret_cast<const float4 *>(A.x + (size_t)row1 * d + k);
                            *reinterpret_cast<float2 *>(&z[sj2 * ZS + k]) = make_float2(v.x, v.y);
                            *reinterpret_cast<float2 *>(&z[sj2 * ZS + k + 2]) = make_float2(v.z, v.w);
                        }
                    }
                }
            }
            __syncthreads();                               // the operand rows and cell states of the next step are complete
            if constexpr (TAPE) {
                // the step's c and h rows of the tape, from LDS: whole rows, a few lines per path instead of one request per element
                const int tid4 = seq_opaque(threadIdx.x), sj4 = tid4 / TPP, part4 = tid4 % TPP;
                if (t < sdesc[sj4 * 4 + 2]) {
                    const size_t row = (size_t)(sdesc[sj4 * 4 + 1] + t) * hidden;
                    for (int u = part4 * 4; u < hidden; u += 4 * TPP) {
                        const float *ph = &z[sj4 * ZS + d + u], *pc = &cs[sj4 * HS + u];
                        *reinterpret_cast<float4 *>(A.tape_h + row + u) = make_float4(ph[0], ph[1], ph[2], ph[3]);
                        *reinterpret_cast<float4 *>(A.tape_c + row + u) = make_float4(pc[0], pc[1], pc[2], pc[3]);
                    }
                }
            }
            if (keep >= 0) {                               // a state that another path starts from, or some a_v
                const int tid3 = seq_opaque(threadIdx.x), sj3 = tid3 / TPP, part3 = tid3 % TPP;
                for (int u = part3 * 4; u < hidden; u += 4 * TPP) {
                    const float *ph = &z[sj3 * ZS + d + u], *pc = &cs[sj3 * HS + u];
                    if (A.flags) {
                        seq_st4_device(A.h + (size_t)keep * hidden + u, make_float4(ph[0], ph[1], ph[2], ph[3]));
                        seq_st4_device(A.c + (size_t)keep * hidden + u, make_float4(pc[0], pc[1], pc[2], pc[3]));
                    } else {
                        *reinterpret_cast<float4 *>(A.h + (size_t)keep * hidden + u) = make_float4(ph[0], ph[1], ph[2], ph[3]);
                        *reinterpret_cast<float4 *>(A.c + (size_t)keep * hidden + u) = make_float4(pc[0], pc[1], pc[2], pc[3]);
                    }
                }
                if (A.flags) {
                    // the threads of a path are adjacent lanes of one wavefront: once the wavefront has seen its stores complete,
                    // the whole row is out, and one of them sets the state's flag
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    if (A.publish && part3 == 0) __hip_atomic_store(A.flags + keep, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        // a_v = the last h of the path, where the path ends a node's list
        const int tid = seq_opaque(threadIdx.x), sj = tid / TPP, part = tid % TPP;
        const int node = sdesc[sj * 4 + 3];
        if (node >= 0) {
            for (int u = part * 4; u < hidden; u += 4 * TPP) {
                const float *ph = &z[sj * ZS + d + u];
                *reinterpret_cast<float4 *>(A.a_out + (size_t)node * hidden + u) = make_float4(ph[0], ph[1], ph[2], ph[3]);
            }
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void seq_output_kernel(const int32_t *__restrict__ final_state, const float *__restrict__ h,
                                                        float *__restrict__ out, int64_t n, int hidden) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n * hidden) return;
    const int64_t v = i / hidden;
    const int s = final_state[v];
    if (s == -2) return;                                   // written by the node's path
    out[i] = s >= 0 ? h[(size_t)s * hidden + (i % hidden)] : 0.f;
}


// ---------------------------------------------------------------------------------------------------------
// Backward pass (backpropagation through time along the same paths, last step first).  For the cell of a step,
// with the gradients dh, dc of its outputs:  t = tanh(c'),  d_o = dh t,  dc += dh o (1 - t^2),
//   d(pre-activations) = (dc g i(1-i),  dc c f(1-f),  dc i (1-g^2),  d_o o(1-o)),   dc_prev = dc f,
//   (dx, dh_prev) = Wp^T d(pre-activations),   dWp += d(pre-activations) (x, h_prev)^T,   db += d(pre-activations).
// A state that other paths start from (or that is some a_v) collects their gradients in its row of gh / gc; levels
// run last to first, so a path finds those rows complete when it reaches the step that wrote the state.

struct SeqRevArgs {
    const int32_t *paths;    // this level's paths in tiles of 64
    int64_t n_path_tiles;
    const int32_t *step_out;
    const float *wqt;        // Wp^T in the order the matrix instructions consume it
    float *tape_g;           // in: the activated gates of every step; out: the gradients of its pre-activations
    const float *tape_c;     // c' of every step
    const float *c_state;    // c rows of the kept states
    const float *g_a;        // [n, H]
    float *gh, *gc;          // [n_states, H]
    float *dx;               // [cells, d]: every step's gradient of its input row
    // all levels in one launch (NULL: one launch per level): per kept state the number of paths that start from it and
    // have not sent their gradients yet; tiles are taken last first
    int32_t *pending;
    int32_t *gave_up;
    int32_t spin_limit, reversed;
    int32_t publish;         // 0 in a test of the time-out: no path is ever counted off
    int32_t d, hidden, kp;
};


__global__ __launch_bounds__(256) void seq_copy_i32_kernel(const int32_t *__restrict__ src, int32_t *__restrict__ dst, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void seq_fill_kernel(float *p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0.f;
}

// Wp^T for the backward product, from the usual layout: [kp / 32 row tiles][4H / 8 groups of four k-steps][64 lanes][4];
// lane l supplies row (tile * 32 + l % 32) of Wp^T, i.e. column z of Wp = (w_ih | w_hh | 0), and Wp's row 2 * step + l / 32,
// rows of Wp being ordered (unit, gate).
__global__ __launch_bounds__(256) void seq_pack_transposed_kernel(const float *__restrict__ w_ih, const float *__restrict__ w_hh,
                                                                 float *__restrict__ wqt, int d, int hidden, int kp) {
    const int64_t total = (int64_t)kp * 4 * hidden;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int per_tile = 32 * 4 * hidden, tile = (int)(i / per_tile), rest = (int)(i % per_tile);
        const int q = rest / 256, lane = (rest % 256) / 4, step = 4 * q + (rest & 3);
        const int r = 2 * step + (lane >> 5), z = tile * 32 + (lane & 31);
        const int row = (r & 3) * hidden + (r >> 2);
        float v = 0.f;
        if (z < d) v = w_ih[(size_t)row * d + z];
        else if (z < d + hidden) v = w_hh[(size_t)row * hidden + (z - d)];
        wqt[i] = v;
    }
}

// a_v that is a shared state's h (the node's whole list is a shared prefix): its gradient goes to the state's row
__global__ __launch_bounds__(256) void seq_final_grad_kernel(const int32_t *__restrict__ final_state, const float *__restrict__ g_a,
                                                            float *gh, int64_t n, int hidden) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n * hidden; i += (int64_t)gridDim.x * 256) {
        const int st = final_state[i / hidden];
        if (st >= 0) __hip_atomic_fetch_add(gh + (size_t)st * hidden + (i % hidden), g_a[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// WIDE_H: hidden above 64 (up to 128): rows of 4 * 128 + 2 staged gradients, one workgroup per compute unit.
template <bool WIDE_H, int NPI>
__global__ __launch_bounds__(512, WIDE_H ? 2 : 4) void seq_reverse_kernel(SeqRevArgs A) {
    constexpr int ZG = 4 * (WIDE_H ? 128 : 64) + 2, IT = WIDE_H ? 4 : 2;
    // per path: the pre-activation gradients of the current step (the product's operand), then the product's result
    // (dx, dh_prev); the running dh and dc themselves stay in the registers of the path's eight threads
    __shared__ __align__(16) float zg[kSeqJobs * ZG];
    __shared__ int32_t sdesc[kSeqJobs * 4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hidden = A.hidden, d = A.d, n_rt = A.kp / 32;          // 2 or 4 row tiles of the product
    // the product has n_rt row tiles x 2 halves of the paths; wavefront w takes pairs w and, with more than 8 (NPI = 2), w + 8
    const int sj = threadIdx.x >> 3, part = threadIdx.x & 7;         // element-wise phases: 8 threads per path, all in one wavefront
    for (int64_t ci = blockIdx.x; ci < A.n_path_tiles; ci += gridDim.x) {
        const int64_t ct = A.reversed ? A.n_path_tiles - 1 - ci : ci;
        if (threadIdx.x < kSeqJobs * 4) sdesc[threadIdx.x] = A.paths[ct * (kSeqJobs * 4) + threadIdx.x];
        __syncthreads();
        const int steps = sdesc[2];
        const int start = sdesc[sj * 4], beg = sdesc[sj * 4 + 1], len = sdesc[sj * 4 + 2], node = sdesc[sj * 4 + 3];
        float dhv[IT][4], dcv[IT][4];                        // units part * 4 + 32 * it + e
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int u = part * 4 + 32 * it;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (node >= 0 && u < hidden) v = *reinterpret_cast<const float4 *>(A.g_a + (size_t)node * hidden + u);
            dhv[it][0] = v.x; dhv[it][1] = v.y; dhv[it][2] = v.z; dhv[it][3] = v.w;
            dcv[it][0] = dcv[it][1] = dcv[it][2] = dcv[it][3] = 0.f;
        }
        for (int t = steps - 1; t >= 0; --t) {
            if (t < len) {
                const size_t cell = (size_t)beg + t;
                if (t + 1 < len) {
                    // the product of the step before left (dx, dh_prev) of this path in its row: dx goes out, dh_prev is this
                    // step's dh.  Only this path's own lanes touch the row between the barriers, and they read it before
                    // they overwrite it below (one wavefront, program order).
                    for (int k = part * 4; k < d; k += 32) {
                        const float *pz = &zg[sj * ZG + k];
                        *reinterpret_cast<float4 *>(A.dx + (cell + 1) * d + k) = make_float4(pz[0], pz[1], pz[2], pz[3]);
                    }
#pragma unroll
                    for (int it = 0; it < IT; ++it) {
                        const int u = part * 4 + 32 * it;
                        if (u >= hidden) continue;
#pragma unroll
                        for (int e = 0; e < 4; ++e) dhv[it][e] = zg[sj * ZG + d + u + e];
                    }
                }
                const int keep = A.step_out[cell];
                if (A.pending && keep >= 0) {
                    // One launch for all levels: the paths that start from this state belong to tiles taken before this one,
                    // which never wait for it, so the count reaches zero; the wait is bounded all the same.  Their sums are
                    // then read with device-scope loads.
                    bool ready = false;
                    for (int spin = 0; spin < A.spin_limit; ++spin) {
                        if (__hip_atomic_load(A.pending + keep, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <= 0) { ready = true; break; }
                        if (__hip_atomic_load(A.gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                        __builtin_amdgcn_s_sleep(16);
                    }
                    if (!ready) __hip_atomic_store(A.gave_up, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                }
#pragma unroll
                for (int it = 0; it < IT; ++it) {
                    const int u = part * 4 + 32 * it;
                    if (u >= hidden) continue;
                    float cn[4], cp[4];
                    if (keep >= 0) {                       // what the other users of this state sent back
                        const float4 a = A.pending ? seq_ld4_device(A.gh + (size_t)keep * hidden + u) : *reinterpret_cast<const float4 *>(A.gh + (size_t)keep * hidden + u);
                        const float4 b = A.pending ? seq_ld4_device(A.gc + (size_t)keep * hidden + u) : *reinterpret_cast<const float4 *>(A.gc + (size_t)keep * hidden + u);
                        dhv[it][0] += a.x; dhv[it][1] += a.y; dhv[it][2] += a.z; dhv[it][3] += a.w;
                        dcv[it][0] += b.x; dcv[it][1] += b.y; dcv[it][2] += b.z; dcv[it][3] += b.w;
                    }
                    {
                        const float4 a = *reinterpret_cast<const float4 *>(A.tape_c + cell * hidden + u);
                        cn[0] = a.x; cn[1] = a.y; cn[2] = a.z; cn[3] = a.w;
                        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (t > 0) b = *reinterpret_cast<const float4 *>(A.tape_c + (cell - 1) * hidden + u);
                        else if (start >= 0) b = *reinterpret_cast<const float4 *>(A.c_state + (size_t)start * hidden + u);
                        cp[0] = b.x; cp[1] = b.y; cp[2] = b.z; cp[3] = b.w;
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float4 *pg = reinterpret_cast<float4 *>(A.tape_g + (cell * hidden + u + e) * 4);
                        const float4 g4 = *pg;             // i, f, g, o
                        const float tc = seq_tanh(cn[e]);
                        const float d_o = dhv[it][e] * tc;
                        const float dcc = dcv[it][e] + dhv[it][e] * g4.w * (1.f - tc * tc);
                        const float4 dg = make_float4(dcc * g4.z * g4.x * (1.f - g4.x), dcc * cp[e] * g4.y * (1.f - g4.y),
                                                      dcc * g4.x * (1.f - g4.z * g4.z), d_o * g4.w * (1.f - g4.w));
                        *pg = dg;                          // kept for the weight gradients
                        *reinterpret_cast<float2 *>(&zg[sj * ZG + (u + e) * 4]) = make_float2(dg.x, dg.y);
                        *reinterpret_cast<float2 *>(&zg[sj * ZG + (u + e) * 4 + 2]) = make_float2(dg.z, dg.w);
                        dcv[it][e] = dcc * g4.y;
                    }
                }
            }
            __syncthreads();
            // (dx, dh_prev)^T [kp, paths] = Wp^T [kp, 4H] . dG^T [4H, paths]
            seq_acc_t acc[NPI];
#pragma unroll
            for (int pi = 0; pi < NPI; ++pi) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[pi][r] = 0.f;
                const int pair = wave + 8 * pi;
                if (pair >= 2 * n_rt) continue;
                const int rt = pair % n_rt, grp = pair / n_rt;
                const float4 *wq = reinterpret_cast<const float4 *>(A.wqt) + (size_t)rt * (hidden / 2) * 64 + lane;
                const float *zl = &zg[(grp * 32 + (lane & 31)) * ZG + (lane >> 5)];
                float4 wa = wq[0];
                for (int q = 0; q < hidden / 2; ++q) {
                    const float4 wn = wq[(q + 1 < hidden / 2 ? q + 1 : q) * 64];
                    acc[pi] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa.x, zl[2 * (4 * q + 0)], acc[pi], 0, 0, 0);
                    acc[pi] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa.y, zl[2 * (4 * q + 1)], acc[pi], 0, 0, 0);
                    acc[pi] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa.z, zl[2 * (4 * q + 2)], acc[pi], 0, 0, 0);
                    acc[pi] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa.w, zl[2 * (4 * q + 3)], acc[pi], 0, 0, 0);
                    wa = wn;
                }
            }
            __syncthreads();                               // every product has read the staged gradients
#pragma unroll
            for (int pi = 0; pi < NPI; ++pi) {
                const int pair = wave + 8 * pi;
                if (pair >= 2 * n_rt) continue;
                const int rt = pair % n_rt, grp = pair / n_rt;
                const int j = grp * 32 + (lane & 31);
                if (t < sdesc[j * 4 + 2]) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = rt * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                        if (row < d + hidden) zg[j * ZG + row] = acc[pi][r];
                    }
                }
            }
            __syncthreads();
        }
        // the first step's dx, and what is left: the gradient of the state the path started from
        if (len > 0) {
            for (int k = part * 4; k < d; k += 32) {
                const float *pz = &zg[sj * ZG + k];
                *reinterpret_cast<float4 *>(A.dx + (size_t)beg * d + k) = make_float4(pz[0], pz[1], pz[2], pz[3]);
            }
            if (start >= 0) {
#pragma unroll
                for (int it = 0; it < IT; ++it) {
                    const int u = part * 4 + 32 * it;
                    if (u >= hidden) continue;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        __hip_atomic_fetch_add(A.gh + (size_t)start * hidden + u + e, zg[sj * ZG + d + u + e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_fetch_add(A.gc + (size_t)start * hidden + u + e, dcv[it][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
                if (A.pending) {
                    // the eight threads of the path are lanes of one wavefront: once it has seen its atomics complete, one
                    // of them counts the path off
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    if (part == 0 && A.publish) __hip_atomic_fetch_sub(A.pending + start, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        __syncthreads();
    }
}

// g_x[u] = the sum of the dx rows of the steps that read x[u]; one thread per (u, four columns)
__global__ __launch_bounds__(256) void seq_input_grad_kernel(const int32_t *__restrict__ xt_ptr, const int32_t *__restrict__ xt_idx,
                                                            const float *__restrict__ dx, float *__restrict__ g_x, int64_t n, int d) {
    const int q = d / 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n * q; i += (int64_t)gridDim.x * 256) {
        const int64_t u = i / q;
        const int k = (int)(i % q) * 4;
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int32_t e = xt_ptr[u]; e < xt_ptr[u + 1]; ++e) {
            const float4 v = *reinterpret_cast<const float4 *>(dx + (size_t)xt_idx[e] * d + k);
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        *reinterpret_cast<float4 *>(g_x + (size_t)u * d + k) = sum;
    }
}

// dWp [4H, kp] = sum over steps of dG[step] (x[in], h_prev)^T and dbp = sum of dG[step], on the matrix cores: the sum over
// steps is the contraction.  A workgroup of 8 wavefronts stages 32 steps at a time in LDS (their dG rows and their
// gathered (x[in], h_prev) rows), wavefront w accumulates row tile w of dWp (32 rows of dG) against all column tiles
// (kp / 32, 16 registers each); every workgroup ends with its own partial sums, which a second kernel adds up in a
// fixed order (so the weight gradients do not depend on timing) and writes in the layout of w_ih, w_hh and b.
struct SeqWgradArgs {
    const float *dg, *x, *tape_h, *h_state;
    const int32_t *step_x, *step_prev;
    int64_t cells;
    int32_t d, hidden, kp;
    float *partial;          // [gridDim.x][4H * kp + 4H]
};
constexpr int kSeqWgradCells = 32;
constexpr int kSeqWgradGroups = 768;        // workgroups along x at most (three per compute unit)
constexpr int64_t kSeqWgradPartialFloats = 64 << 20;   // and no more partial sums than this many floats

// NCT: column tiles of 32 (kp / 32 rounded up to 4 or 8).  blockIdx.y selects a slab of 256 rows of dWp (hidden > 64 has two).
template <int NCT, bool SLABS>
__global__ __launch_bounds__(512, 2) void seq_weight_grad_kernel(SeqWgradArgs A) {
    constexpr int CK = kSeqWgradCells, ZW = NCT * 32, RZ = NCT / 2;
    __shared__ __align__(16) float sdg[CK][256];
    __shared__ __align__(16) float sz[CK][ZW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rows = 4 * A.hidden, d = A.d, hidden = A.hidden, kp = A.kp;
    const int row0 = SLABS ? blockIdx.y * 256 : 0, n_rt = (rows - row0 < 256 ? rows - row0 : 256) / 32, n_ct = kp / 32;
    seq_acc_t acc[NCT];
#pragma unroll
    for (int c = 0; c < NCT; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    float accb = 0.f;                                      // thread i < 256: the sum of dG[.][row0 + i]
    const int64_t chunks = (A.cells + CK - 1) / CK;
    // the next 32 steps' rows are requested into registers before the products of the current ones
    float4 rg[4], rz[RZ];
    auto request = [&](int64_t ch) {
        const int64_t c0 = ch * CK;
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const int i = threadIdx.x + 512 * v4, c = i / 64, k = (i % 64) * 4;
            rg[v4] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ch < chunks && c0 + c < A.cells && row0 + k < rows) rg[v4] = *reinterpret_cast<const float4 *>(A.dg + (size_t)(c0 + c) * rows + row0 + k);
        }
#pragma unroll
        for (int v4 = 0; v4 < RZ; ++v4) {
            const int i = threadIdx.x + 512 * v4, c = i / (ZW / 4), k = (i % (ZW / 4)) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ch < chunks && c0 + c < A.cells) {
                if (k < d) v = *reinterpret_cast<const float4 *>(A.x + (size_t)A.step_x[c0 + c] * d + k);
                else if (k < d + hidden) {
                    const int pv = A.step_prev[c0 + c];
                    if (pv >= 0) v = *reinterpret_cast<const float4 *>(A.tape_h + (size_t)pv * hidden + (k - d));
                    else if (pv <= -2) v = *reinterpret_cast<const float4 *>(A.h_state + (size_t)(-pv - 2) * hidden + (k - d));
                }
            }
            rz[v4] = v;
        }
    };
    request(blockIdx.x);
    for (int64_t ch = blockIdx.x; ch < chunks; ch += gridDim.x) {
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const int i = threadIdx.x + 512 * v4;
            *reinterpret_cast<float4 *>(&sdg[i / 64][(i % 64) * 4]) = rg[v4];
        }
#pragma unroll
        for (int v4 = 0; v4 < RZ; ++v4) {
            const int i = threadIdx.x + 512 * v4;
            *reinterpret_cast<float4 *>(&sz[i / (ZW / 4)][(i % (ZW / 4)) * 4]) = rz[v4];
        }
        __syncthreads();
        request(ch + gridDim.x);
        if (wave < n_rt) {
#pragma unroll
            for (int st = 0; st < CK / 2; ++st) {
                const int c = 2 * st + (lane >> 5);
                const float a = sdg[c][wave * 32 + (lane & 31)];
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
                    if (ct < n_ct) acc[ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, sz[c][ct * 32 + (lane & 31)], acc[ct], 0, 0, 0);
            }
        }
        if ((int)threadIdx.x < 32 * n_rt) {
#pragma unroll
            for (int c = 0; c < CK; ++c) accb += sdg[c][threadIdx.x];
        }
        __syncthreads();
    }
    float *out = A.partial + (size_t)blockIdx.x * ((size_t)rows * kp + rows);
    if (wave < n_rt) {
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            if (ct >= n_ct) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + wave * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                out[(size_t)row * kp + ct * 32 + (lane & 31)] = acc[ct][r];
            }
        }
    }
    if ((int)threadIdx.x < 32 * n_rt) out[(size_t)rows * kp + row0 + threadIdx.x] = accb;
}

// adds the workgroups' partial sums in index order and writes the usual layout: rows (unit, gate) -> gate-major rows,
// columns split into the input and the hidden part
__global__ __launch_bounds__(256) void seq_weight_grad_reduce_kernel(const float *__restrict__ partial, int groups, float *__restrict__ g_w_ih,
                                                                    float *__restrict__ g_w_hh, float *__restrict__ g_b, int d, int hidden,
                                                                    int kp) {
    const int64_t per = (int64_t)4 * hidden * kp + 4 * hidden;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < per; i += (int64_t)gridDim.x * 256) {
        float sum = 0.f;
        for (int g = 0; g < groups; ++g) sum += partial[(size_t)g * per + i];
        if (i < (int64_t)4 * hidden * kp) {
            const int r = (int)(i / kp), k = (int)(i % kp);
            const int row = (r & 3) * hidden + (r >> 2);
            if (k < d) g_w_ih[(size_t)row * d + k] = sum;
            else if (k < d + hidden) g_w_hh[(size_t)row * hidden + (k - d)] = sum;
        } else {
            const int r = (int)(i - (int64_t)4 * hidden * kp);
            g_b[(r & 3) * hidden + (r >> 2)] = sum;
        }
    }
}

}  // namespace hag

using namespace hag;

extern "C" {

int hag_seq_search(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity, int64_t *n_merges, int32_t *left,
                   int32_t *right, int32_t *redundancy, int64_t *hrowptr, int32_t *hcol);

int hag_seq_create(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity, hag_seq_t **out) {
    if (!out) { set_error("out is NULL"); return HAG_EINVAL; }
    *out = nullptr;
    if (n < 0 || capacity < 0 || !rowptr) { set_error("n < 0, capacity < 0 or rowptr is NULL"); return HAG_EINVAL; }
    try {
        const int64_t e = rowptr[n];
        std::vector<int64_t> hrowptr(n + 1, 0);
        std::vector<int32_t> hcol((size_t)std::max<int64_t>(e, 1));
        const int64_t cap = std::min(capacity, e);
        std::vector<int32_t> left((size_t)std::max<int64_t>(cap, 1)), right(left.size()), red(left.size());
        int64_t a = 0;
        // capacity 0 still goes through the search: it validates the lists and copies them
        int rc = hag_seq_search(n, rowptr, col, cap, &a, left.data(), right.data(), red.data(), hrowptr.data(), hcol.data());
        if (rc) return rc;
        if (n + a + e + n >= (int64_t)INT32_MAX) { set_error("too many states for 32-bit ids"); return HAG_EINVAL; }
        auto *h = new hag_seq();
        h->n = n; h->e = e; h->n_merges = a;
        if (const char *v = getenv("HAG_SEQ_ONE_LAUNCH")) h->one_launch = atoi(v) != 0;
        if (const char *v = getenv("HAG_SPIN_LIMIT")) h->spin_limit = (int32_t)std::min<long long>(std::max<long long>(atoll(v), 1), INT32_MAX);
        const bool share = capacity > 0;
        // shared states: the one-element prefixes in use, then the aggregation nodes (a state's predecessor
        // has a smaller index)
        std::vector<int32_t> first_id(n, -1);
        int32_t n_first = 0;
        auto need_first = [&](int32_t u) { if (first_id[u] < 0) first_id[u] = n_first++; };
        if (share) {
            for (int64_t i = 0; i < a; ++i) if (left[i] < n) need_first(left[i]);
            for (int64_t v = 0; v < n; ++v)
                if (hrowptr[v + 1] > hrowptr[v] && hcol[hrowptr[v]] < n) need_first(hcol[hrowptr[v]]);
        }
        const int64_t S = (int64_t)n_first + a;
        h->n_states = S;
        auto state_of = [&](int32_t id) { return id < n ? first_id[id] : n_first + (id - (int32_t)n); };
        std::vector<int32_t> prev((size_t)S, -1), xrow((size_t)S, 0), depth((size_t)S, 1);
        for (int64_t u = 0; u < n; ++u) if (first_id[u] >= 0) xrow[first_id[u]] = (int32_t)u;
        for (int64_t i = 0; i < a; ++i) {
            const int32_t st = n_first + (int32_t)i;
            prev[st] = state_of(left[i]); xrow[st] = right[i]; depth[st] = depth[prev[st]] + 1;
        }
        // every node's private remainder: what follows the shared state of its list's head
        struct R { int32_t start, beg, len, node; };
        std::vector<R> rem;
        std::vector<int32_t> consumers((size_t)S, 0), tail((size_t)S, -1);   // tail: the longest remainder starting at the state
        std::vector<int64_t> weight((size_t)S, 1);
        std::vector<uint8_t> is_final((size_t)S, 0);
        h->final_state.assign(n, -1);
        for (int64_t v = 0; v < n; ++v) {
            const int64_t b0 = hrowptr[v], b1 = hrowptr[v + 1];
            if (b1 == b0) continue;
            if (!share) { rem.push_back(R{-1, (int32_t)b0, (int32_t)(b1 - b0), (int32_t)v}); h->final_state[v] = -2;
                          h->longest = std::max<int64_t>(h->longest, b1 - b0); continue; }
            const int32_t st = state_of(hcol[b0]);
            h->longest = std::max<int64_t>(h->longest, depth[st] + (b1 - b0 - 1));
            if (b1 - b0 == 1) { h->final_state[v] = st; is_final[st] = 1; continue; }
            h->final_state[v] = -2;
            ++consumers[st];
            weight[st] += b1 - b0 - 1;
            if (tail[st] < 0 || rem[tail[st]].len < (int32_t)(b1 - b0 - 1)) tail[st] = (int32_t)rem.size();
            rem.push_back(R{st, (int32_t)(b0 + 1), (int32_t)(b1 - b0 - 1), (int32_t)v});
        }
        // a state hands its running (h, c) to the successor with the most evaluations below it, or, with no
        // successor state, to its longest remainder
        std::vector<int32_t> cont((size_t)S, -1);
        for (int64_t st = S - 1; st >= 0; --st) {
            const int32_t p = prev[st];
            if (p < 0) continue;
            weight[p] += weight[st];
            ++consumers[p];
            if (cont[p] < 0 || weight[cont[p]] <= weight[st]) cont[p] = (int32_t)st;   // ties: the smaller index
        }
        std::vector<uint8_t> rem_used(rem.size(), 0);
        std::vector<int32_t> level((size_t)S, 0);
        struct P { int32_t start, head, len, node, level, rem; };   // head: first state (-1: a bare remainder `rem`)
        std::vector<P> ps;
        for (int64_t st = 0; st < S; ++st) {
            const int32_t p = prev[st];
            const bool is_head = p < 0 || cont[p] != st;
            level[st] = p < 0 ? 0 : (is_head ? level[p] + 1 : level[p]);
            if (!is_head) continue;
            int32_t len = 0, t = (int32_t)st, r = -1;
            for (;; t = cont[t]) { ++len; if (cont[t] < 0) break; }
            if (tail[t] >= 0) { r = tail[t]; rem_used[r] = 1; len += rem[r].len; }
            ps.push_back(P{p, (int32_t)st, len, r >= 0 ? rem[r].node : -1, level[st], r});
        }
        for (size_t r = 0; r < rem.size(); ++r)
            if (!rem_used[r]) ps.push_back(P{rem[r].start, -1, rem[r].len, rem[r].node, rem[r].start < 0 ? 0 : level[rem[r].start] + 1, (int32_t)r});
        std::stable_sort(ps.begin(), ps.end(), [](const P &p, const P &q) { return p.level != q.level ? p.level < q.level : p.len > q.len; });
        int32_t levels = 0;
        for (const P &p : ps) levels = std::max(levels, p.level + 1);
        h->level_ptr.assign((size_t)levels + 1, 0);
        h->paths.reserve(ps.size() * 4);
        for (const P &p : ps) {
            ++h->level_ptr[(size_t)p.level + 1];
            const int32_t beg = (int32_t)h->step_x.size();
            if (p.head >= 0) {
                for (int32_t t = p.head; t >= 0; t = cont[t]) {
                    // the continuation takes the state along; anything else that needs it reads it from memory
                    const bool handed_on = cont[t] >= 0 || (p.rem >= 0);
                    const bool kept = is_final[t] || consumers[t] > (handed_on ? 1 : 0);
                    h->step_x.push_back(xrow[t]);
                    h->step_out.push_back(kept ? t : -1);
                }
            }
            if (p.rem >= 0)
                for (int32_t k = 0; k < rem[p.rem].len; ++k) { h->step_x.push_back(hcol[rem[p.rem].beg + k]); h->step_out.push_back(-1); }
            h->paths.push_back(p.start); h->paths.push_back(beg); h->paths.push_back(p.len); h->paths.push_back(p.node);
        }
        for (int32_t l = 0; l < levels; ++l) h->level_ptr[(size_t)l + 1] += h->level_ptr[l];
        h->tile_ptr.assign((size_t)levels + 1, 0);
        for (int32_t l = 0; l < levels; ++l)
            h->tile_ptr[(size_t)l + 1] = h->tile_ptr[l] + (h->level_ptr[(size_t)l + 1] - h->level_ptr[l] + kSeqJobs - 1) / kSeqJobs;
        {
            const int64_t np = (int64_t)(h->paths.size() / 4);
            std::vector<int32_t> key((size_t)np), order((size_t)np);
            int32_t groups = 0;
            for (int64_t i = 0; i < np; ++i) {
                const int32_t start = h->paths[i * 4];
                key[i] = start < 0 ? 0 : depth[start];
                order[i] = (int32_t)i;
                groups = std::max(groups, key[i] + 1);
            }
            std::stable_sort(order.begin(), order.end(), [&](int32_t p, int32_t q) {
                return key[p] != key[q] ? key[p] < key[q] : h->paths[(size_t)p * 4 + 2] > h->paths[(size_t)q * 4 + 2];
            });
            h->depth_ptr.assign((size_t)groups + 1, 0);
            h->paths_by_depth.reserve(h->paths.size());
            for (int32_t i : order) {
                ++h->depth_ptr[(size_t)key[i] + 1];
                h->paths_by_depth.insert(h->paths_by_depth.end(), h->paths.begin() + (size_t)i * 4, h->paths.begin() + (size_t)i * 4 + 4);
            }
            h->depth_tile_ptr.assign((size_t)groups + 1, 0);
            for (int32_t g = 0; g < groups; ++g) {
                h->depth_tile_ptr[(size_t)g + 1] = h->depth_tile_ptr[g] + (h->depth_ptr[(size_t)g + 1] + kSeqJobs - 1) / kSeqJobs;
                h->depth_ptr[(size_t)g + 1] += h->depth_ptr[g];
            }
        }
        {
            const int64_t cells = (int64_t)h->step_x.size(), np = (int64_t)(h->paths.size() / 4);
            h->step_prev.assign((size_t)cells, -1);
            h->pending_init.assign((size_t)std::max<int64_t>(h->n_states, 1), 0);
            for (int64_t i = 0; i < np; ++i) {
                const int32_t start = h->paths[i * 4], beg = h->paths[i * 4 + 1], len = h->paths[i * 4 + 2];
                if (start >= 0 && len > 0) ++h->pending_init[start];
                for (int32_t t = 0; t < len; ++t) h->step_prev[(size_t)beg + t] = t > 0 ? beg + t - 1 : (start >= 0 ? -start - 2 : -1);
            }
            h->xt_ptr.assign((size_t)n + 1, 0);
            for (int64_t a2 = 0; a2 < cells; ++a2) ++h->xt_ptr[(size_t)h->step_x[a2] + 1];
            for (int64_t u = 0; u < n; ++u) h->xt_ptr[(size_t)u + 1] += h->xt_ptr[u];
            h->xt_idx.resize((size_t)cells);
            std::vector<int32_t> at(h->xt_ptr.begin(), h->xt_ptr.end() - 1);
            for (int64_t a2 = 0; a2 < cells; ++a2) h->xt_idx[(size_t)at[h->step_x[a2]]++] = (int32_t)a2;
        }
        *out = h;
        return HAG_OK;
    } catch (const std::bad_alloc &) {
        set_error("out of host memory");
        return HAG_ENOMEM;
    } catch (const std::exception &ex) {
        set_error(ex.what());
        return HAG_EINVAL;
    }
}

void hag_seq_free(hag_seq_t *h) {
    if (!h) return;
    if (h->d_final) (void)hipFree(h->d_final);
    if (h->d_paths) (void)hipFree(h->d_paths);
    if (h->d_paths_by_depth) (void)hipFree(h->d_paths_by_depth);
    if (h->d_step_prev) (void)hipFree(h->d_step_prev);
    if (h->d_xt_ptr) (void)hipFree(h->d_xt_ptr);
    if (h->d_xt_idx) (void)hipFree(h->d_xt_idx);
    if (h->d_pending_init) (void)hipFree(h->d_pending_init);
    if (h->d_step_x) (void)hipFree(h->d_step_x);
    if (h->d_step_out) (void)hipFree(h->d_step_out);
    if (h->d_gave_up) (void)hipFree(h->d_gave_up);
    delete h;
}

int64_t hag_seq_cells(const hag_seq_t *h) { return h ? (int64_t)h->step_x.size() : 0; }
int64_t hag_seq_ranks(const hag_seq_t *h) { return h ? h->longest : 0; }
int64_t hag_seq_launches(const hag_seq_t *h) {
    if (!h) return 0;
    const int64_t levels = (int64_t)h->level_ptr.size() - 1;
    return h->one_launch ? std::min<int64_t>(levels, 1) : levels;
}
int64_t hag_seq_merges(const hag_seq_t *h) { return h ? h->n_merges : 0; }

// Padded D + H, which also names the kernel variant: 64 and 128 hold Wp in registers (hidden <= 64), 192 and 256 stream it.
static int64_t seq_kp(int64_t d, int64_t hidden) {
    if (hidden <= 64 && d + hidden <= 128) return d + hidden <= 64 ? 64 : 128;
    return d + hidden <= 192 ? 192 : 256;
}
// Index into hag_seq::resident / the variant table below.
static int seq_variant(int64_t kp, int64_t hidden) { return kp > 128 ? (kp == 192 ? 4 : 5) : (kp == 64 ? 0 : 2) + (hidden > 32 ? 1 : 0); }
typedef void (*seq_kernel_t)(SeqChainArgs);
static const seq_kernel_t kSeqVariants[6] = {seq_chain_kernel<32, false, false, false>, seq_chain_kernel<32, true, false, false>,
                                             seq_chain_kernel<64, false, false, false>, seq_chain_kernel<64, true, false, false>,
                                             seq_chain_kernel<96, true, true, false>,   seq_chain_kernel<128, true, true, false>};
typedef void (*seq_reverse_t)(SeqRevArgs);
static const seq_reverse_t kSeqReverseVariants[3] = {seq_reverse_kernel<false, 1>, seq_reverse_kernel<false, 2>, seq_reverse_kernel<true, 2>};
// the same with the tape written (training)
static const seq_kernel_t kSeqTapeVariants[6] = {seq_chain_kernel<32, false, false, true>, seq_chain_kernel<32, true, false, true>,
                                                 seq_chain_kernel<64, false, false, true>, seq_chain_kernel<64, true, false, true>,
                                                 seq_chain_kernel<96, true, true, true>,   seq_chain_kernel<128, true, true, true>};

int hag_seq_get_plan(const hag_seq_t *h, int32_t order, int64_t *n_states, int64_t *n_paths, const int32_t **paths,
                     const int32_t **step_x, const int32_t **step_out, int64_t *n_levels, const int64_t **level_ptr,
                     const int32_t **final_state) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (order != 0 && order != 1) { set_error("order must be 0 (levels) or 1 (depth of the start state)"); return HAG_EINVAL; }
    if (n_states) *n_states = h->n_states;
    if (n_paths) *n_paths = (int64_t)(h->paths.size() / 4);
    if (paths) *paths = order ? h->paths_by_depth.data() : h->paths.data();
    if (step_x) *step_x = h->step_x.data();
    if (step_out) *step_out = h->step_out.data();
    if (n_levels) *n_levels = (int64_t)(order ? h->depth_ptr.size() : h->level_ptr.size()) - 1;
    if (level_ptr) *level_ptr = order ? h->depth_ptr.data() : h->level_ptr.data();
    if (final_state) *final_state = h->final_state.data();
    return HAG_OK;
}

int hag_seq_upload(hag_seq_t *h) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (h->d_final) return HAG_OK;
    HIP_TRY(hipGetDevice(&h->device));
    auto put = [](int32_t **dst, const std::vector<int32_t> &src) -> hipError_t {
        hipError_t e = hipMalloc(dst, std::max<size_t>(src.size(), 1) * sizeof(int32_t));
        if (e == hipSuccess && !src.empty()) e = hipMemcpy(*dst, src.data(), src.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        return e;
    };
    {
        // every group padded to whole tiles with empty paths (no start state, no steps, no node)
        auto padded = [](const std::vector<int32_t> &paths, const std::vector<int64_t> &ptr, const std::vector<int64_t> &tiles) {
            std::vector<int32_t> out;
            out.reserve((size_t)tiles.back() * kSeqJobs * 4);
            for (size_t l = 0; l + 1 < ptr.size(); ++l) {
                out.insert(out.end(), paths.begin() + ptr[l] * 4, paths.begin() + ptr[l + 1] * 4);
                while ((int64_t)out.size() < tiles[l + 1] * kSeqJobs * 4) { out.push_back(-1); out.push_back(0); out.push_back(0); out.push_back(-1); }
            }
            return out;
        };
        HIP_TRY(put(&h->d_paths, padded(h->paths, h->level_ptr, h->tile_ptr)));
        HIP_TRY(put(&h->d_paths_by_depth, padded(h->paths_by_depth, h->depth_ptr, h->depth_tile_ptr)));
    }
    HIP_TRY(put(&h->d_step_x, h->step_x));
    HIP_TRY(put(&h->d_step_out, h->step_out));
    HIP_TRY(put(&h->d_step_prev, h->step_prev));
    HIP_TRY(put(&h->d_xt_ptr, h->xt_ptr));
    HIP_TRY(put(&h->d_xt_idx, h->xt_idx));
    HIP_TRY(put(&h->d_pending_init, h->pending_init));
    HIP_TRY(put(&h->d_gave_up, std::vector<int32_t>(1, 0)));
    {
        // workgroups of each kernel variant that the device holds at once (at most the two per compute unit the
        // kernel is tuned for): the grid of a one-launch pass
        int cus = 0;
        HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device));
        for (int k = 0; k < 6; ++k) {
            int per_cu = 0;
            HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kSeqVariants[k], k >= 4 ? 1024 : 512, 0));
            h->resident[k] = (int64_t)std::min(per_cu, 2) * cus;
            HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kSeqTapeVariants[k], k >= 4 ? 1024 : 512, 0));
            h->resident_tape[k] = (int64_t)std::min(per_cu, 2) * cus;
            if (k < 3) {
                HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kSeqReverseVariants[k], 512, 0));
                h->resident_reverse[k] = (int64_t)std::min(per_cu, k == 2 ? 1 : 2) * cus;
            }
        }
    }
    HIP_TRY(put(&h->d_final, h->final_state));
    return HAG_OK;
}

int hag_seq_set_option(hag_seq_t *h, int32_t option, int64_t value) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    switch (option) {
        case HAG_OPT_SEQ_ONE_LAUNCH: h->one_launch = value != 0; return HAG_OK;
        case HAG_OPT_SPIN_LIMIT: h->spin_limit = (int32_t)std::min<int64_t>(std::max<int64_t>(value, 1), INT32_MAX); return HAG_OK;
        case HAG_OPT_TEST_WAIT_UNREACHABLE: h->wait_unreachable = value != 0; return HAG_OK;
        default: set_error("unknown option"); return HAG_EINVAL;
    }
}

int hag_seq_check(const hag_seq_t *h, void *stream) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (!h->d_final) { set_error("hag_seq_upload has not been called on this handle"); return HAG_ESTATE; }
    hipStream_t s = (hipStream_t)stream;
    int32_t word = 0;
    HIP_TRY(hipMemcpyAsync(&word, h->d_gave_up, sizeof(word), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (!word) return HAG_OK;
    HIP_TRY(hipMemsetAsync(h->d_gave_up, 0, sizeof(word), s));
    HIP_TRY(hipStreamSynchronize(s));
    set_error("a pass of the LSTM aggregator gave up waiting for a state: its output is not valid");
    return HAG_ETIMEOUT;
}

size_t hag_seq_workspace_bytes(const hag_seq_t *h, int64_t d, int64_t hidden) {
    if (!h || d <= 0 || hidden <= 0) return 0;
    const size_t states = (size_t)std::max<int64_t>(h->n_states, 1) * (size_t)hidden * sizeof(float);
    const size_t wp = (size_t)4 * hidden * seq_kp(d, hidden) * sizeof(float), bp = (size_t)4 * hidden * sizeof(float);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t flags = (size_t)std::max<int64_t>(h->n_states, 1) * sizeof(int32_t);
    return up(wp) + up(bp) + 2 * up(states) + up(flags);
}

static int seq_forward(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih, const float *w_hh,
                       const float *b, float *a_out, void *workspace, void *stream, float *tape_g, float *tape_c, float *tape_h) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (!h->d_final) { set_error("hag_seq_upload has not been called on this handle"); return HAG_ESTATE; }
    if (d <= 0 || d % 4 != 0 || hidden <= 0 || hidden % 8 != 0 || hidden > 128 || d + hidden > kSeqMaxK) {
        set_error("d must be a multiple of 4, hidden a multiple of 8 up to 128, d + hidden at most 256");
        return HAG_EINVAL;
    }
    if (h->n == 0) return HAG_OK;
    if (!x || !w_ih || !w_hh || !b || !a_out || !workspace) { set_error("NULL pointer"); return HAG_EINVAL; }
    if (((uintptr_t)x | (uintptr_t)workspace | (uintptr_t)a_out) & 15) { set_error("x, a_out and workspace must be 16-byte aligned"); return HAG_EINVAL; }
    hipStream_t s = (hipStream_t)stream;
    const int kp = (int)seq_kp(d, hidden);
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    char *w = (char *)workspace;
    float *wp = (float *)w; w += up((size_t)4 * hidden * kp * sizeof(float));
    float *bp = (float *)w; w += up((size_t)4 * hidden * sizeof(float));
    const size_t states = up((size_t)std::max<int64_t>(h->n_states, 1) * (size_t)hidden * sizeof(float));
    float *hst = (float *)w; w += states;
    float *cst = (float *)w; w += states;
    int32_t *flags = (int32_t *)w;                          // [n_states]
    {
        const int64_t total = (int64_t)4 * hidden * kp;
        hipLaunchKernelGGL(seq_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w_ih, w_hh, b, wp, bp, (int)d,
                           (int)hidden, kp, kp > 128 ? 1 : 0, flags, h->n_states);
        HIP_TRY(hipGetLastError());
    }
    const int64_t levels = (int64_t)h->tile_ptr.size() - 1;
    const int variant = seq_variant(kp, hidden);
    const bool big = variant >= 4;
    const int64_t resident = tape_g ? h->resident_tape[variant] : h->resident[variant];
    const bool fused = levels > 1 && h->one_launch && resident > 0;
    for (int64_t l = 0; l < (fused ? 1 : levels); ++l) {
        SeqChainArgs c;
        const int64_t t0 = fused ? 0 : h->tile_ptr[l], t1 = fused ? h->depth_tile_ptr.back() : h->tile_ptr[l + 1];
        c.chains = fused ? h->d_paths_by_depth : h->d_paths + t0 * kSeqJobs * 4;
        c.n_path_tiles = t1 - t0;
        c.flags = fused ? flags : nullptr;
        c.spin_limit = h->spin_limit;
        c.publish = h->wait_unreachable ? 0 : 1;
        c.gave_up = h->d_gave_up;
        c.step_x = h->d_step_x; c.step_out = h->d_step_out;
        c.x = x; c.wp = wp; c.bp = bp; c.h = hst; c.c = cst; c.a_out = a_out;
        c.tape_g = tape_g; c.tape_c = tape_c; c.tape_h = tape_h;
        c.d = (int32_t)d; c.hidden = (int32_t)hidden;
        if (c.n_path_tiles <= 0) continue;
        const dim3 grid((unsigned)std::min<int64_t>(c.n_path_tiles, fused ? resident : (big ? 256 : 512))), block(big ? 1024 : 512);
        hipLaunchKernelGGL(tape_g ? kSeqTapeVariants[variant] : kSeqVariants[variant], grid, block, 0, s, c);
        HIP_TRY(hipGetLastError());
    }
    {
        const int64_t total = h->n * hidden;
        hipLaunchKernelGGL(seq_output_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, h->d_final, hst, a_out, h->n,
                           (int)hidden);
        HIP_TRY(hipGetLastError());
    }
    return HAG_OK;
}

int hag_seq_lstm_forward(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih, const float *w_hh,
                         const float *b, float *a_out, void *workspace, void *stream) {
    return seq_forward(h, d, hidden, x, w_ih, w_hh, b, a_out, workspace, stream, nullptr, nullptr, nullptr);
}

// workgroups (along x) of the weight-gradient kernel at most: each leaves one set of partial sums
static int64_t seq_wgrad_groups(size_t per) { return std::max<int64_t>(std::min<int64_t>(kSeqWgradGroups, kSeqWgradPartialFloats / (int64_t)per), 1); }

// Layout of the training workspace: the forward workspace, then the tape and the backward pass's own buffers.
struct SeqTrainLayout { size_t fwd, tape_g, tape_c, tape_h, dx, gh, gc, pending, wqt, partial, total; };
static SeqTrainLayout seq_train_layout(const hag_seq_t *h, int64_t d, int64_t hidden) {
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t cells = std::max<size_t>(h->step_x.size(), 1), states = (size_t)std::max<int64_t>(h->n_states, 1);
    const size_t kp = (size_t)seq_kp(d, hidden), H = (size_t)hidden, f = sizeof(float);
    SeqTrainLayout L;
    size_t at = up(hag_seq_workspace_bytes(h, d, hidden));
    L.fwd = 0;
    L.tape_g = at; at += up(cells * 4 * H * f);
    L.tape_c = at; at += up(cells * H * f);
    L.tape_h = at; at += up(cells * H * f);
    L.dx = at; at += up(cells * (size_t)d * f);
    L.gh = at; at += up(states * H * f);
    L.gc = at; at += up(states * H * f);
    L.pending = at; at += up(states * sizeof(int32_t));
    L.wqt = at; at += up(kp * 4 * H * f);
    L.partial = at; at += up((size_t)seq_wgrad_groups(4 * H * kp + 4 * H) * (4 * H * kp + 4 * H) * f);
    L.total = at;
    return L;
}
static bool seq_backward_supported(int64_t d, int64_t hidden) {
    return d > 0 && d % 4 == 0 && hidden > 0 && hidden % 8 == 0 && hidden <= 128 && d + hidden <= kSeqMaxK;
}

size_t hag_seq_train_workspace_bytes(const hag_seq_t *h, int64_t d, int64_t hidden) {
    if (!h || !seq_backward_supported(d, hidden)) return 0;
    return seq_train_layout(h, d, hidden).total;
}

int hag_seq_lstm_forward_train(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih, const float *w_hh,
                               const float *b, float *a_out, void *workspace, void *stream) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (!seq_backward_supported(d, hidden)) {
        set_error("d must be a multiple of 4, hidden a multiple of 8 up to 128, d + hidden at most 256");
        return HAG_EINVAL;
    }
    if (!workspace) { set_error("NULL pointer"); return HAG_EINVAL; }
    const SeqTrainLayout L = seq_train_layout(h, d, hidden);
    char *w = (char *)workspace;
    return seq_forward(h, d, hidden, x, w_ih, w_hh, b, a_out, workspace, stream, (float *)(w + L.tape_g), (float *)(w + L.tape_c),
                       (float *)(w + L.tape_h));
}

int hag_seq_lstm_backward(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih, const float *w_hh,
                          const float *g_a, float *g_x, float *g_w_ih, float *g_w_hh, float *g_b, void *workspace, void *stream) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (!h->d_final) { set_error("hag_seq_upload has not been called on this handle"); return HAG_ESTATE; }
    if (!seq_backward_supported(d, hidden)) {
        set_error("d must be a multiple of 4, hidden a multiple of 8 up to 128, d + hidden at most 256");
        return HAG_EINVAL;
    }
    if (h->n == 0) return HAG_OK;
    if (!x || !w_ih || !w_hh || !g_a || !g_x || !g_w_ih || !g_w_hh || !g_b || !workspace) { set_error("NULL pointer"); return HAG_EINVAL; }
    if (((uintptr_t)x | (uintptr_t)workspace | (uintptr_t)g_a | (uintptr_t)g_x) & 15) { set_error("x, g_a, g_x and workspace must be 16-byte aligned"); return HAG_EINVAL; }
    hipStream_t s = (hipStream_t)stream;
    const int kp = (int)seq_kp(d, hidden);
    const SeqTrainLayout L = seq_train_layout(h, d, hidden);
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    char *w = (char *)workspace;
    // the forward workspace as seq_forward laid it out: packed weights, packed bias, h rows, c rows
    const size_t states = up((size_t)std::max<int64_t>(h->n_states, 1) * (size_t)hidden * sizeof(float));
    const float *hst = (const float *)(w + up((size_t)4 * hidden * kp * sizeof(float)) + up((size_t)4 * hidden * sizeof(float)));
    const float *cst = (const float *)((const char *)hst + states);
    float *tape_g = (float *)(w + L.tape_g), *tape_c = (float *)(w + L.tape_c), *tape_h = (float *)(w + L.tape_h);
    float *dx = (float *)(w + L.dx), *gh = (float *)(w + L.gh), *gc = (float *)(w + L.gc), *wqt = (float *)(w + L.wqt);
    float *partial = (float *)(w + L.partial);
    const int64_t cells = (int64_t)h->step_x.size();
    auto blocks = [](int64_t total) { return dim3((unsigned)std::min<int64_t>((total + 255) / 256, 65535 * 16)); };
    // gradient rows of the kept states start at zero (gh and gc are adjacent)
    {
        const int64_t total = (int64_t)((L.pending - L.gh) / sizeof(float));
        hipLaunchKernelGGL(seq_fill_kernel, blocks(total), dim3(256), 0, s, gh, total);
        HIP_TRY(hipGetLastError());
    }
    {
        const int64_t total = (int64_t)kp * 4 * hidden;
        hipLaunchKernelGGL(seq_pack_transposed_kernel, blocks(total), dim3(256), 0, s, w_ih, w_hh, wqt, (int)d, (int)hidden, kp);
        HIP_TRY(hipGetLastError());
        const int64_t nh = h->n * hidden;
        hipLaunchKernelGGL(seq_final_grad_kernel, blocks(nh), dim3(256), 0, s, h->d_final, g_a, gh, h->n, (int)hidden);
        HIP_TRY(hipGetLastError());
    }
    const int64_t levels = (int64_t)h->tile_ptr.size() - 1;
    const int rv = hidden > 64 ? 2 : (kp > 128 ? 1 : 0);
    const int64_t resident = h->resident_reverse[rv];
    const bool fused = levels > 1 && h->one_launch && resident > 0;
    int32_t *pending = (int32_t *)(w + L.pending);
    if (fused) {
        hipLaunchKernelGGL(seq_copy_i32_kernel, blocks(h->n_states), dim3(256), 0, s, h->d_pending_init, pending, h->n_states);
        HIP_TRY(hipGetLastError());
    }
    for (int64_t l = fused ? 0 : levels - 1; l >= 0; --l) {
        SeqRevArgs r;
        // one launch: the tiles of the depth order, last first (what starts deeper comes earlier); else level by level, last first
        r.paths = fused ? h->d_paths_by_depth : h->d_paths + h->tile_ptr[l] * kSeqJobs * 4;
        r.n_path_tiles = fused ? h->depth_tile_ptr.back() : h->tile_ptr[l + 1] - h->tile_ptr[l];
        r.pending = fused ? pending : nullptr;
        r.reversed = fused ? 1 : 0;
        r.gave_up = h->d_gave_up;
        r.spin_limit = h->spin_limit;
        r.publish = h->wait_unreachable ? 0 : 1;
        r.step_out = h->d_step_out;
        r.wqt = wqt; r.tape_g = tape_g; r.tape_c = tape_c; r.c_state = cst; r.g_a = g_a; r.gh = gh; r.gc = gc; r.dx = dx;
        r.d = (int32_t)d; r.hidden = (int32_t)hidden; r.kp = kp;
        if (r.n_path_tiles <= 0) continue;
        const int64_t cap = fused ? resident : (rv == 2 ? 256 : 512);
        hipLaunchKernelGGL(kSeqReverseVariants[rv], dim3((unsigned)std::min<int64_t>(r.n_path_tiles, cap)), dim3(512), 0, s, r);
        HIP_TRY(hipGetLastError());
    }
    {
        const int64_t total = h->n * (d / 4);
        hipLaunchKernelGGL(seq_input_grad_kernel, blocks(total), dim3(256), 0, s, h->d_xt_ptr, h->d_xt_idx, dx, g_x, h->n, (int)d);
        HIP_TRY(hipGetLastError());
    }
    {
        SeqWgradArgs g;
        g.dg = tape_g; g.x = x; g.tape_h = tape_h; g.h_state = hst; g.step_x = h->d_step_x; g.step_prev = h->d_step_prev;
        g.cells = cells; g.d = (int32_t)d; g.hidden = (int32_t)hidden; g.kp = kp; g.partial = partial;
        const int64_t chunks = (cells + kSeqWgradCells - 1) / kSeqWgradCells;
        const int64_t per = (int64_t)4 * hidden * kp + 4 * hidden;
        const int groups = (int)std::max<int64_t>(std::min<int64_t>(chunks, seq_wgrad_groups((size_t)per)), 1);
        const dim3 grid((unsigned)groups, (unsigned)((4 * hidden + 255) / 256));
        if (hidden > 64) hipLaunchKernelGGL((seq_weight_grad_kernel<8, true>), grid, dim3(512), 0, s, g);
        else if (kp > 128) hipLaunchKernelGGL((seq_weight_grad_kernel<8, false>), grid, dim3(512), 0, s, g);
        else hipLaunchKernelGGL((seq_weight_grad_kernel<4, false>), grid, dim3(512), 0, s, g);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(seq_weight_grad_reduce_kernel, blocks(per), dim3(256), 0, s, partial, groups, g_w_ih, g_w_hh, g_b, (int)d,
                           (int)hidden, kp);
        HIP_TRY(hipGetLastError());
    }
    return HAG_OK;
}

}  // extern "C"

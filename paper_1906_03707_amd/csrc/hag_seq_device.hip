// Device path for a SEQUENTIAL Aggregate (Section 3.1): an LSTM aggregator over ordered neighbour
// lists, run over a prefix HAG found by hag_seq_search (or over the plain lists).
//
// Every evaluation of the LSTM cell is a "job": (input row, state it continues, state it writes).
// A prefix HAG turns the lists into a forest of jobs: the state after the one-element prefix (u) is
// a job without a predecessor, an aggregation node w = (v1, v2) is the job "state of v1, then x[v2]"
// (Equation 2: cover(w) = (cover(v1), cover(v2))), and every v continues from the state of its
// list's head through the rest of its list (Algorithm 2: aggregation nodes first, then the nodes of
// V).  Jobs are ranked by the length of the chain behind them; one launch evaluates all jobs of a
// rank as a gathered matrix product on the matrix cores:
//     gates^T [4H, jobs] = Wp [4H, D+H] . Z^T [D+H, jobs],    Z[j] = (x[in_j], h[prev_j]),
// 32 gate rows x 32 jobs per wavefront tile with v_mfma_f32_32x32x2_f32 (fp32 in, fp32 out).  The rows of
// Wp are ordered (hidden unit, gate), so a lane ends up holding all four gates of its hidden units
// for its job and the cell's element-wise part runs in registers.  A wavefront keeps its slice of
// Wp in registers for the whole launch; the gathered rows of a tile of jobs are staged in LDS.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "hag_device_common.hpp"

struct hag_seq {
    int64_t n = 0, e = 0, n_merges = 0, n_states = 0;
    std::vector<int32_t> jobs;        // 3 per job: input row, previous state (-1: none), written state
    std::vector<int64_t> rank_ptr;    // jobs of rank t: [rank_ptr[t], rank_ptr[t+1])
    std::vector<int32_t> final_state; // per node: state row holding a_v, -1 for an empty list, -2: written by its chain
    // the private part of every node's walk (what follows the shared state of its list's head): 4 per chain,
    // (state it starts from or -1, first entry in `chain_col`, entries, node), longest first
    std::vector<int32_t> chains, chain_col;
    int64_t chain_cells = 0, longest = 0;
    int32_t *d_jobs = nullptr, *d_final = nullptr, *d_chains = nullptr, *d_chain_col = nullptr;
    int device = -1;
};

namespace hag {

constexpr int kSeqJobs = 64;      // jobs per tile
constexpr int kSeqMaxK = 128;     // D + H at most

struct SeqArgs {
    const int32_t *jobs;   // this rank's jobs
    int64_t n_jobs;
    const float *x;        // [n, d]
    const float *wp;       // [4H, KP] packed weights, rows (unit, gate), columns (input, hidden, zero padding)
    const float *bp;       // [4H] packed bias
    float *h, *c;          // [n_states, H]
    int32_t d, hidden, kp;
};

// Wp / bp from the usual layout: w_ih [4H, D], w_hh [4H, H], b [4H], gate-major rows (input, forget,
// cell, output gate).
__global__ __launch_bounds__(256) void seq_pack_kernel(const float *__restrict__ w_ih, const float *__restrict__ w_hh,
                                                      const float *__restrict__ b, float *__restrict__ wp,
                                                      float *__restrict__ bp, int d, int hidden, int kp) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)4 * hidden * kp;
    if (i >= total) return;
    const int r = (int)(i / kp), k = (int)(i % kp);
    const int unit = r >> 2, gate = r & 3, src_row = gate * hidden + unit;
    float v = 0.f;
    if (k < d) v = w_ih[(size_t)src_row * d + k];
    else if (k < d + hidden) v = w_hh[(size_t)src_row * hidden + (k - d)];
    wp[i] = v;
    if (k == 0) bp[r] = b[src_row];
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

// One rank of jobs.  A workgroup of 8 wavefronts takes tiles of 64 jobs; KSTEPS = KP / 2 matrix-core steps
// per 32 x 32 product.  WIDE (hidden > 32, up to 8 gate tiles of 8 hidden units): wavefront w holds gate
// tile w and multiplies it with both halves of the job tile; otherwise (up to 4 gate tiles) wavefront w
// holds gate tile w % 4 and takes the half w / 4 of the job tile.  Either way a wavefront keeps one gate
// tile of Wp in registers, so four wavefronts fit a SIMD and the staging and element-wise phases of
// one hide behind the products of the others.
template <int KSTEPS, bool WIDE>
__global__ __launch_bounds__(512, 4) void seq_lstm_kernel(SeqArgs A) {
    constexpr int KP = 2 * KSTEPS, ZS = KP + 2;            // row stride of the staged inputs: even, and 2 banks apart per job
    constexpr int HS = (WIDE ? 64 : 32) + 1, JG = WIDE ? 2 : 1;
    __shared__ float z[kSeqJobs * ZS];
    __shared__ float hs[kSeqJobs * HS];                    // new h of the tile, [job][unit]
    __shared__ float cs[kSeqJobs * HS];                    // previous, then new cell state
    __shared__ __align__(16) float sb[4 * 64];             // packed bias (read from LDS per tile: held in registers it would cost a wavefront per SIMD)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hidden = A.hidden, d = A.d, n_tiles = hidden / 8;
    const int tile = WIDE ? wave : (wave & 3), group0 = WIDE ? 0 : (wave >> 2);
    // this wavefront's gate tile of the packed weights, in the operand layout of the matrix instruction:
    // lane l supplies row (l % 32) of the tile and column 2 * step + l / 32
    float wreg[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
        wreg[s] = tile < n_tiles ? A.wp[(size_t)(tile * 32 + (lane & 31)) * KP + 2 * s + (lane >> 5)] : 0.f;
    if ((int)threadIdx.x < 4 * hidden) sb[threadIdx.x] = A.bp[threadIdx.x];
    const int64_t n_job_tiles = (A.n_jobs + kSeqJobs - 1) / kSeqJobs;
    // Staging is done by 8 threads per job, 16 bytes at a time.  Its latency hides behind the products of the
    // other wavefronts on the SIMD (reading a tile ahead into registers instead was measured: the registers
    // it holds cost a wavefront per SIMD, which costs more).
    constexpr int ZV = KP / 32, CV = WIDE ? 2 : 1;         // 16-byte vectors per thread: inputs, previous cell state
    const int sj = threadIdx.x >> 3, part = threadIdx.x & 7;
    for (int64_t jt = blockIdx.x; jt < n_job_tiles; jt += gridDim.x) {
        const int64_t job = jt * kSeqJobs + sj;
        int in_row = -1, prev = -1, out = -1;
        if (job < A.n_jobs) { in_row = A.jobs[job * 3]; prev = A.jobs[job * 3 + 1]; out = A.jobs[job * 3 + 2]; }
        {
            float4 zr[ZV];
#pragma unroll
            for (int i = 0; i < ZV; ++i) {
                const int k = part * 4 + 32 * i;
                zr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (in_row >= 0) {
                    if (k < d) zr[i] = *reinterpret_cast<const float4 *>(A.x + (size_t)in_row * d + k);
                    else if (k < d + hidden && prev >= 0) zr[i] = *reinterpret_cast<const float4 *>(A.h + (size_t)prev * hidden + (k - d));
                }
            }
            // rows of z are only 8-byte aligned: two 8-byte stores per vector
#pragma unroll
            for (int i = 0; i < ZV; ++i) {
                const int k = part * 4 + 32 * i;
                *reinterpret_cast<float2 *>(&z[sj * ZS + k]) = make_float2(zr[i].x, zr[i].y);
                *reinterpret_cast<float2 *>(&z[sj * ZS + k + 2]) = make_float2(zr[i].z, zr[i].w);
            }
        }
#pragma unroll
        for (int i = 0; i < CV; ++i) {
            const int u = part * 4 + 32 * i;
            if (u < hidden) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (in_row >= 0 && prev >= 0) v = *reinterpret_cast<const float4 *>(A.c + (size_t)prev * hidden + u);
                cs[sj * HS + u] = v.x; cs[sj * HS + u + 1] = v.y; cs[sj * HS + u + 2] = v.z; cs[sj * HS + u + 3] = v.w;
            }
        }
        const int out_now = in_row >= 0 ? out : -1;
        __syncthreads();
        // the products start from the bias: register 4 m + gate of a lane belongs to hidden unit 2 m + lane / 32 of the tile
        seq_acc_t acc[JG];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const float4 bias = tile < n_tiles ? *reinterpret_cast<const float4 *>(&sb[(tile * 8 + 2 * m + (lane >> 5)) * 4])
                                               : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int g = 0; g < JG; ++g) { acc[g][4 * m] = bias.x; acc[g][4 * m + 1] = bias.y; acc[g][4 * m + 2] = bias.z; acc[g][4 * m + 3] = bias.w; }
        }
        const float *zl = &z[(group0 * 32 + (lane & 31)) * ZS + (lane >> 5)];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
            for (int g = 0; g < JG; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[s], zl[g * 32 * ZS + 2 * s], acc[g], 0, 0, 0);
        }
        // element-wise part: lane l holds, for job l % 32 of its half, gate rows 8 * (r / 4) + 4 * (l / 32) + r % 4 of the
        // gate tile, i.e. the four gates (r % 4) of hidden units 2 * (r / 4) + l / 32 of the tile
        if (tile < n_tiles) {
#pragma unroll
            for (int g = 0; g < JG; ++g) {
                const int j = (group0 + g) * 32 + (lane & 31);
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int unit = tile * 8 + 2 * m + (lane >> 5);
                    const float gi = acc[g][4 * m + 0];
                    const float gf = acc[g][4 * m + 1];
                    const float gg = acc[g][4 * m + 2];
                    const float go = acc[g][4 * m + 3];
                    const float c_prev = cs[j * HS + unit];   // staged above; this lane is the only one to touch the element
                    const float c_new = seq_sigmoid(gf) * c_prev + seq_sigmoid(gi) * seq_tanh(gg);
                    cs[j * HS + unit] = c_new;
                    hs[j * HS + unit] = seq_sigmoid(go) * seq_tanh(c_new);
                }
            }
        }
        __syncthreads();
        // write the new states, rows contiguous: 8 threads per job
        if (out_now >= 0) {
            for (int u = part * 4; u < hidden; u += 32) {
                const float *ph = &hs[sj * HS + u], *pc = &cs[sj * HS + u];
                *reinterpret_cast<float4 *>(A.h + (size_t)out_now * hidden + u) = make_float4(ph[0], ph[1], ph[2], ph[3]);
                *reinterpret_cast<float4 *>(A.c + (size_t)out_now * hidden + u) = make_float4(pc[0], pc[1], pc[2], pc[3]);
            }
        }
        __syncthreads();
    }
}

struct SeqChainArgs {
    const int32_t *chains;   // 4 per chain, longest first
    int64_t n_chains;
    const int32_t *col;      // the chains' input rows
    const float *x, *wp, *bp;
    const float *h, *c;      // states of the shared prefixes (read only here)
    float *a_out;            // [n, H]
    int32_t d, hidden;
};

// The private part of every node's walk, 64 nodes per workgroup tile, ALL its steps in one launch: the
// running states never leave the compute unit (h in the staged operand rows, c beside them in LDS), so
// a cell costs one input row of global traffic instead of reading and writing both state rows as well.
// Chains are sorted by length, so the chains of a tile end within a step or two of each other; a chain
// that has ended keeps its state while the others finish.  Same tiling of the products as above.
// Hides a value's origin from the optimiser, so that what is derived from it is computed where it is used
// instead of being held in a register across the products.
__device__ __forceinline__ int seq_opaque(int v) { asm volatile("" : "+v"(v)); return v; }

template <int KSTEPS, bool WIDE>
__global__ __launch_bounds__(512, 4) void seq_chain_kernel(SeqChainArgs A) {
    constexpr int KP = 2 * KSTEPS, ZS = KP + 2;
    constexpr int HS = (WIDE ? 64 : 32) + 1, JG = WIDE ? 2 : 1;
    __shared__ float z[kSeqJobs * ZS];
    __shared__ float hs[kSeqJobs * HS];
    __shared__ float cs[kSeqJobs * HS];
    __shared__ __align__(16) float sb[4 * 64];
    __shared__ int32_t sdesc[kSeqJobs * 4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hidden = A.hidden, d = A.d, n_tiles = hidden / 8;
    const int tile = WIDE ? wave : (wave & 3), group0 = WIDE ? 0 : (wave >> 2);
    float wreg[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
        wreg[s] = tile < n_tiles ? A.wp[(size_t)(tile * 32 + (lane & 31)) * KP + 2 * s + (lane >> 5)] : 0.f;
    if ((int)threadIdx.x < 4 * hidden) sb[threadIdx.x] = A.bp[threadIdx.x];
    constexpr int ZV = KP / 32;
    const int64_t n_chain_tiles = (A.n_chains + kSeqJobs - 1) / kSeqJobs;
    for (int64_t ct = blockIdx.x; ct < n_chain_tiles; ct += gridDim.x) {
        if (threadIdx.x < kSeqJobs * 4) {
            const int64_t ch = ct * kSeqJobs + threadIdx.x / 4;
            sdesc[threadIdx.x] = ch < A.n_chains ? A.chains[ch * 4 + threadIdx.x % 4] : ((threadIdx.x & 3) == 2 ? 0 : -1);
        }
        __syncthreads();
        // (thread indices are derived again in every phase, and the descriptor is re-read from LDS where it is needed rather than held in registers, which are short)
        const int steps = sdesc[2];                        // the tile's first chain is its longest
        // the state the chain starts from, the first input row, zero padding
        {
            const int tid = seq_opaque(threadIdx.x), sj = tid >> 3, part = tid & 7;
            const int start = sdesc[sj * 4], beg = sdesc[sj * 4 + 1], len = sdesc[sj * 4 + 2];
            const int row0 = len > 0 ? A.col[beg] : -1;
#pragma unroll 1                                           // (one vector in flight: this runs once per tile, and registers are short)
            for (int i = 0; i < ZV; ++i) {
                const int k = part * 4 + 32 * i;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < d) { if (row0 >= 0) v = *reinterpret_cast<const float4 *>(A.x + (size_t)row0 * d + k); }
                else if (k < d + hidden && start >= 0) v = *reinterpret_cast<const float4 *>(A.h + (size_t)start * hidden + (k - d));
                *reinterpret_cast<float2 *>(&z[sj * ZS + k]) = make_float2(v.x, v.y);
                *reinterpret_cast<float2 *>(&z[sj * ZS + k + 2]) = make_float2(v.z, v.w);
            }
            for (int u = part * 4; u < hidden; u += 32) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (start >= 0) v = *reinterpret_cast<const float4 *>(A.c + (size_t)start * hidden + u);
                cs[sj * HS + u] = v.x; cs[sj * HS + u + 1] = v.y; cs[sj * HS + u + 2] = v.z; cs[sj * HS + u + 3] = v.w;
            }
        }
        __syncthreads();
        for (int t = 0; t < steps; ++t) {
            // the next step's input row is requested before this step's products and lands in LDS after them
            // (its first 64 columns, that is: holding more across the products would spill registers)
            constexpr int ZE = ZV < 2 ? ZV : 2;
            float4 xr[ZE];
            const int tid = seq_opaque(threadIdx.x), sj = tid >> 3, part = tid & 7;
            const int len = sdesc[sj * 4 + 2];
            const int row1 = t + 1 < len ? A.col[sdesc[sj * 4 + 1] + t + 1] : -1;
#pragma unroll
            for (int i = 0; i < ZE; ++i) {
                const int k = part * 4 + 32 * i;
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
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
#pragma unroll
                for (int g = 0; g < JG; ++g) acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(wreg[s], zl[g * 32 * ZS + 2 * s], acc[g], 0, 0, 0);
            }
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
                            hs[j * HS + unit] = seq_sigmoid(acc[g][4 * m + 3]) * seq_tanh(c_new);
                        }
                    }
                }
            }
            __syncthreads();                               // every product has read z, every new h is in hs
            {
                const int tid2 = seq_opaque(threadIdx.x), sj2 = tid2 >> 3, part2 = tid2 & 7;
                if (t < sdesc[sj2 * 4 + 2]) {
                    for (int u = part2 * 4; u < hidden; u += 32) {
                        const float *ph = &hs[sj2 * HS + u];
                        *reinterpret_cast<float2 *>(&z[sj2 * ZS + d + u]) = make_float2(ph[0], ph[1]);
                        *reinterpret_cast<float2 *>(&z[sj2 * ZS + d + u + 2]) = make_float2(ph[2], ph[3]);
                    }
                }
                if (row1 >= 0) {
#pragma unroll
                    for (int i = 0; i < ZV; ++i) {
                        const int k = part2 * 4 + 32 * i;
                        if (k < d) {
                            const float4 v = i < ZE ? xr[i < ZE ? i : 0] : *reinterpret_cast<const float4 *>(A.x + (size_t)row1 * d + k);
                            *reinterpret_cast<float2 *>(&z[sj2 * ZS + k]) = make_float2(v.x, v.y);
                            *reinterpret_cast<float2 *>(&z[sj2 * ZS + k + 2]) = make_float2(v.z, v.w);
                        }
                    }
                }
            }
            __syncthreads();
        }
        // a_v = the last h of the chain
        const int tid = seq_opaque(threadIdx.x), sj = tid >> 3, part = tid & 7;
        const int node = sdesc[sj * 4 + 3];
        if (node >= 0) {
            for (int u = part * 4; u < hidden; u += 32) {
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
    if (s == -2) return;                                   // written by the node's chain
    out[i] = s >= 0 ? h[(size_t)s * hidden + (i % hidden)] : 0.f;
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
        const bool share = capacity > 0;
        // state rows: one-element prefixes in use, aggregation nodes, one running row per node
        std::vector<int32_t> first_id(n, -1);
        int32_t n_first = 0;
        auto need_first = [&](int32_t u) { if (first_id[u] < 0) first_id[u] = n_first++; };
        if (share) {
            for (int64_t i = 0; i < a; ++i) if (left[i] < n) need_first(left[i]);
            for (int64_t v = 0; v < n; ++v)
                if (hrowptr[v + 1] > hrowptr[v] && hcol[hrowptr[v]] < n) need_first(hcol[hrowptr[v]]);
        }
        const int32_t agg0 = n_first;
        h->n_states = (int64_t)n_first + a;
        std::vector<int32_t> rank_of_state((size_t)std::max<int64_t>(h->n_states, 1), 0);
        struct J { int32_t x, prev, out, rank; };
        std::vector<J> js;
        js.reserve((size_t)(e + n_first));
        for (int64_t u = 0; u < n; ++u)
            if (first_id[u] >= 0) js.push_back(J{(int32_t)u, -1, first_id[u], 0});
        auto state_of = [&](int32_t id) { return id < n ? first_id[id] : agg0 + (id - (int32_t)n); };
        for (int64_t i = 0; i < a; ++i) {
            const int32_t prev = state_of(left[i]), out_s = agg0 + (int32_t)i;
            const int32_t r = rank_of_state[prev] + 1;
            rank_of_state[out_s] = r;
            js.push_back(J{right[i], prev, out_s, r});
        }
        h->final_state.assign(n, -1);
        struct C { int32_t start, beg, len, node; };
        std::vector<C> cs;
        for (int64_t v = 0; v < n; ++v) {
            const int64_t b0 = hrowptr[v], b1 = hrowptr[v + 1];
            if (b1 == b0) continue;
            int32_t cur = -1, depth = 0;
            int64_t i = b0;
            if (share) { cur = state_of(hcol[b0]); depth = rank_of_state[cur] + 1; i = b0 + 1; }
            if (i == b1) { h->final_state[v] = cur; h->longest = std::max<int64_t>(h->longest, depth); continue; }
            cs.push_back(C{cur, (int32_t)i, (int32_t)(b1 - i), (int32_t)v});
            h->final_state[v] = -2;
            h->chain_cells += b1 - i;
            h->longest = std::max<int64_t>(h->longest, depth + (b1 - i));
        }
        std::stable_sort(cs.begin(), cs.end(), [](const C &p, const C &q) { return p.len > q.len; });
        h->chains.reserve(cs.size() * 4);
        for (const C &c : cs) { h->chains.push_back(c.start); h->chains.push_back(c.beg); h->chains.push_back(c.len); h->chains.push_back(c.node); }
        h->chain_col.assign(hcol.begin(), hcol.begin() + (size_t)hrowptr[n]);
        int32_t ranks = 0;
        for (const J &j : js) ranks = std::max(ranks, j.rank + 1);
        h->rank_ptr.assign((size_t)ranks + 1, 0);
        for (const J &j : js) ++h->rank_ptr[(size_t)j.rank + 1];
        for (int32_t t = 0; t < ranks; ++t) h->rank_ptr[(size_t)t + 1] += h->rank_ptr[t];
        std::vector<int64_t> at(h->rank_ptr.begin(), h->rank_ptr.end() - 1);
        h->jobs.resize(js.size() * 3);
        for (const J &j : js) {
            const int64_t p = at[j.rank]++;
            h->jobs[p * 3] = j.x; h->jobs[p * 3 + 1] = j.prev; h->jobs[p * 3 + 2] = j.out;
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
    if (h->d_jobs) (void)hipFree(h->d_jobs);
    if (h->d_final) (void)hipFree(h->d_final);
    if (h->d_chains) (void)hipFree(h->d_chains);
    if (h->d_chain_col) (void)hipFree(h->d_chain_col);
    delete h;
}

int64_t hag_seq_cells(const hag_seq_t *h) { return h ? (int64_t)(h->jobs.size() / 3) + h->chain_cells : 0; }
int64_t hag_seq_ranks(const hag_seq_t *h) { return h ? h->longest : 0; }
int64_t hag_seq_launches(const hag_seq_t *h) { return h ? (int64_t)h->rank_ptr.size() - 1 + (h->chains.empty() ? 0 : 1) : 0; }
int64_t hag_seq_merges(const hag_seq_t *h) { return h ? h->n_merges : 0; }

int hag_seq_upload(hag_seq_t *h) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (h->d_final) return HAG_OK;
    HIP_TRY(hipGetDevice(&h->device));
    HIP_TRY(hipMalloc(&h->d_jobs, std::max<size_t>(h->jobs.size(), 1) * sizeof(int32_t)));
    HIP_TRY(hipMalloc(&h->d_final, std::max<size_t>(h->final_state.size(), 1) * sizeof(int32_t)));
    if (!h->jobs.empty()) HIP_TRY(hipMemcpy(h->d_jobs, h->jobs.data(), h->jobs.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    if (!h->final_state.empty())
        HIP_TRY(hipMemcpy(h->d_final, h->final_state.data(), h->final_state.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    HIP_TRY(hipMalloc(&h->d_chains, std::max<size_t>(h->chains.size(), 1) * sizeof(int32_t)));
    HIP_TRY(hipMalloc(&h->d_chain_col, std::max<size_t>(h->chain_col.size(), 1) * sizeof(int32_t)));
    if (!h->chains.empty()) HIP_TRY(hipMemcpy(h->d_chains, h->chains.data(), h->chains.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    if (!h->chain_col.empty())
        HIP_TRY(hipMemcpy(h->d_chain_col, h->chain_col.data(), h->chain_col.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    return HAG_OK;
}

static int64_t seq_kp(int64_t d, int64_t hidden) { return d + hidden <= 64 ? 64 : 128; }

size_t hag_seq_workspace_bytes(const hag_seq_t *h, int64_t d, int64_t hidden) {
    if (!h || d <= 0 || hidden <= 0) return 0;
    const size_t states = (size_t)std::max<int64_t>(h->n_states, 1) * (size_t)hidden * sizeof(float);
    const size_t wp = (size_t)4 * hidden * seq_kp(d, hidden) * sizeof(float), bp = (size_t)4 * hidden * sizeof(float);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    return up(wp) + up(bp) + 2 * up(states);
}

int hag_seq_lstm_forward(const hag_seq_t *h, int64_t d, int64_t hidden, const float *x, const float *w_ih, const float *w_hh,
                         const float *b, float *a_out, void *workspace, void *stream) {
    if (!h) { set_error("NULL handle"); return HAG_EINVAL; }
    if (!h->d_final) { set_error("hag_seq_upload has not been called on this handle"); return HAG_ESTATE; }
    if (d <= 0 || d % 4 != 0 || hidden <= 0 || hidden % 8 != 0 || hidden > 64 || d + hidden > kSeqMaxK) {
        set_error("d must be a multiple of 4, hidden a multiple of 8 up to 64, d + hidden at most 128");
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
    float *cst = (float *)w;
    {
        const int64_t total = (int64_t)4 * hidden * kp;
        hipLaunchKernelGGL(seq_pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w_ih, w_hh, b, wp, bp, (int)d,
                           (int)hidden, kp);
        HIP_TRY(hipGetLastError());
    }
    const int64_t ranks = (int64_t)h->rank_ptr.size() - 1;
    for (int64_t t = 0; t < ranks; ++t) {
        SeqArgs a;
        a.jobs = h->d_jobs + h->rank_ptr[t] * 3;
        a.n_jobs = h->rank_ptr[t + 1] - h->rank_ptr[t];
        a.x = x; a.wp = wp; a.bp = bp; a.h = hst; a.c = cst;
        a.d = (int32_t)d; a.hidden = (int32_t)hidden; a.kp = kp;
        if (a.n_jobs <= 0) continue;
        const int64_t tiles = (a.n_jobs + kSeqJobs - 1) / kSeqJobs;
        const dim3 grid((unsigned)std::min<int64_t>(tiles, 256 * 2)), block(512);
        const bool wide = hidden > 32;   // more than four gate tiles
        if (kp == 64) {
            if (wide) hipLaunchKernelGGL((seq_lstm_kernel<32, true>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((seq_lstm_kernel<32, false>), grid, block, 0, s, a);
        } else {
            if (wide) hipLaunchKernelGGL((seq_lstm_kernel<64, true>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((seq_lstm_kernel<64, false>), grid, block, 0, s, a);
        }
        HIP_TRY(hipGetLastError());
    }
    if (!h->chains.empty()) {
        SeqChainArgs c;
        c.chains = h->d_chains; c.n_chains = (int64_t)(h->chains.size() / 4); c.col = h->d_chain_col;
        c.x = x; c.wp = wp; c.bp = bp; c.h = hst; c.c = cst; c.a_out = a_out;
        c.d = (int32_t)d; c.hidden = (int32_t)hidden;
        const int64_t tiles = (c.n_chains + kSeqJobs - 1) / kSeqJobs;
        const dim3 grid((unsigned)std::min<int64_t>(tiles, 256 * 2)), block(512);
        const bool wide = hidden > 32;
        if (kp == 64) {
            if (wide) hipLaunchKernelGGL((seq_chain_kernel<32, true>), grid, block, 0, s, c);
            else hipLaunchKernelGGL((seq_chain_kernel<32, false>), grid, block, 0, s, c);
        } else {
            if (wide) hipLaunchKernelGGL((seq_chain_kernel<64, true>), grid, block, 0, s, c);
            else hipLaunchKernelGGL((seq_chain_kernel<64, false>), grid, block, 0, s, c);
        }
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

}  // extern "C"

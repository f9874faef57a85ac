// Pair counting of the HAG search (Algorithm 3) on the GPU.
//
// The search asks, for one node x at a time, how often every other node shares a list
// Nhat_u with x (Redundancy(x, .) for a set Aggregate).  That count is a histogram over the
// lists that hold x: for a popular x it touches millions of list entries, which is the bulk
// of the search's time on the host and an easy job for a GPU.  The device keeps a mirror of
// the evolving lists (and of the out-lists that say which lists hold a node), applies every
// merge to the mirror with two small kernels, and answers batches of count requests.  All
// decisions stay on the host: the device only returns exact counts, so the merge sequence is
// the same with or without it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "hag_internal.hpp"

namespace hag {

namespace {

constexpr int kMaxBatch = 32;          // count requests answered per round trip
constexpr int kCountBlocks = 128;      // workgroups per request in the counting launch
constexpr int kEager = 128;            // results per request copied back with the result counts
constexpr int kFoundCap = 1 << 16;     // results kept per request; more -> the host counts that node itself
constexpr int kHotOrig = 6144;         // counters a workgroup keeps in LDS: the original nodes of highest bound ...
constexpr int kHotAgg = 2048;          // ... and the earliest aggregation nodes

struct View {
    int64_t n, m;                // original nodes; n + capacity
    const int64_t *ptr;          // [n+1] list u occupies nb[ptr[u] .. ptr[u] + len[u])
    int32_t *nb;                 // members in MIRROR ids: an original node is named by its rank in the order
                                 // (bound descending, id ascending), an aggregation node by its id (>= n)
    int32_t *len, *norig;        // current length; how many of the leading members are original nodes
    const int32_t *by_rank;      // [n] original node of each rank
    int32_t *mred;               // [capacity] creation redundancy of an aggregation node
    int64_t *out_off;            // [m] out-list of x occupies out[out_off[x] .. + olen[x]), ascending
    int32_t *out;
    int32_t *olen;
    int32_t *cnt;                // [kMaxBatch][m] counters by mirror id, all zero between batches
    const int32_t *req;          // [kMaxBatch][4] node, threshold, number of original nodes whose bound reaches it, 0
    int32_t *nfound;             // [kMaxBatch]
    Found *found;                // [kMaxBatch][kFoundCap]
};

// Request s = blockIdx.y: add one to cnt[s][y] for every member y of every list that holds
// x, skipping members whose static bound is below the threshold (they cannot reach it).
// Lists keep their original members first, by descending bound, then their aggregation
// members by creation (whose bounds never increase), so both parts can stop at the first miss.
// The lists of a popular x all hold the same few popular partners; those counters would take
// one device-wide atomic per list, all to the same address.  They are the nodes of highest
// bound and the earliest aggregation nodes, so a workgroup counts those in LDS and adds its
// totals to the global counters once.
__global__ __launch_bounds__(256) void count_kernel(View v) {
    __shared__ int32_t hot[kHotOrig + kHotAgg];
    const int s = blockIdx.y;
    const int x = v.req[4 * s], theta = v.req[4 * s + 1], rank_end = v.req[4 * s + 2];
    if (blockIdx.x == 0 && threadIdx.x == 0) v.nfound[s] = 0;
    const int32_t *o = v.out + v.out_off[x];
    const int ol = v.olen[x];
    const int waves = blockDim.x >> 6;
    if ((int)blockIdx.x * waves >= ol) return;      // no list for this workgroup
    for (int t = threadIdx.x; t < kHotOrig + kHotAgg; t += blockDim.x) hot[t] = 0;
    __syncthreads();
    int32_t *c = v.cnt + (size_t)s * (size_t)v.m;
    const int lane = threadIdx.x & 63;
    const int n_wave = gridDim.x * waves;
    const int n = (int)v.n;
    for (int i = blockIdx.x * waves + (threadIdx.x >> 6); i < ol; i += n_wave) {
        const int u = o[i];
        const int32_t *l = v.nb + v.ptr[u];
        const int no = v.norig[u], L = v.len[u];
        for (int j0 = 0; j0 < no; j0 += 64) {
            const int j = j0 + lane;
            bool ok = false;
            if (j < no) {
                const int y = l[j];                  // a rank: ascending along the list
                ok = y < rank_end;
                if (ok) {
                    if (y < kHotOrig) atomicAdd(&hot[y], 1);
                    else atomicAdd(&c[y], 1);
                }
            }
            if (!__all(ok)) break;
        }
        for (int j0 = no; j0 < L; j0 += 64) {
            const int j = j0 + lane;
            bool ok = false;
            if (j < L) {
                const int y = l[j];
                const int ai = y - n;
                ok = v.mred[ai] >= theta;
                if (ok) {
                    if (ai < kHotAgg) atomicAdd(&hot[kHotOrig + ai], 1);
                    else atomicAdd(&c[y], 1);
                }
            }
            if (!__all(ok)) break;
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kHotOrig + kHotAgg; t += blockDim.x) {
        const int k = hot[t];
        if (k) atomicAdd(&c[t < kHotOrig ? t : n + (t - kHotOrig)], k);
    }
}

// Request s = blockIdx.y: report every (y, count) with count >= threshold and clear all counters.
__global__ __launch_bounds__(256) void collect_kernel(View v) {
    const int s = blockIdx.y;
    const int theta = v.req[4 * s + 1];
    int32_t *c = v.cnt + (size_t)s * (size_t)v.m;
    for (int64_t y = (int64_t)blockIdx.x * 256 + threadIdx.x; y < v.m; y += (int64_t)gridDim.x * 256) {
        const int k = c[y];
        if (k == 0) continue;
        c[y] = 0;
        if (k >= theta) {
            const int at = atomicAdd(&v.nfound[s], 1);
            if (at < kFoundCap) v.found[(size_t)s * kFoundCap + at] = Found{y < v.n ? v.by_rank[y] : (int32_t)y, k};
        }
    }
}

// The rewrite loop of Algorithm 3 on the mirror: every list named in rows[0..r) holds p and
// q (mirror ids); remove both and append w.  One wavefront per list, compacting in place: a chunk of 64
// members is read by one instruction before any of them is written, and is written to
// positions no later chunk reads.
__global__ __launch_bounds__(256) void rewrite_kernel(View v, int64_t rows_at, int r, int p, int q, int w) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= r) return;
    const int u = v.out[rows_at + i];
    int32_t *l = v.nb + v.ptr[u];
    const int L = v.len[u];
    int k = 0;
    for (int j0 = 0; j0 < L; j0 += 64) {
        const int j = j0 + lane;
        const int y = j < L ? l[j] : -1;
        const bool keep = j < L && y != p && y != q;
        const unsigned long long mask = __ballot(keep);
        const int pos = k + __popcll(mask & ((1ull << lane) - 1ull));
        if (keep) l[pos] = y;
        k += __popcll(mask);
    }
    if (lane == 0 && k < L) {
        l[k] = w;
        v.len[u] = k + 1;
        v.norig[u] -= (p < v.n) + (q < v.n);     // a rank is below n just as the id it stands for
    }
}

// Out-lists after a merge: rows[0..r) leave the out-lists of p (workgroup 0) and q
// (workgroup 1) and become the out-list of w, which already sits at out[rows_at ..).
__global__ __launch_bounds__(1024) void out_remove_kernel(View v, int64_t rows_at, int r, int p, int q, int w) {
    __shared__ int wave_total[16];
    const int x = blockIdx.x == 0 ? p : q;
    int32_t *o = v.out + v.out_off[x];
    const int l = v.olen[x];
    const int32_t *rows = v.out + rows_at;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int k = 0;
    for (int i0 = 0; i0 < l; i0 += 1024) {
        const int i = i0 + (int)threadIdx.x;
        const int val = i < l ? o[i] : -1;
        bool keep = i < l;
        if (keep) {
            int lo = 0, hi = r;                  // first entry of rows that is >= val
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (rows[mid] < val) lo = mid + 1; else hi = mid;
            }
            keep = !(lo < r && rows[lo] == val);
        }
        const unsigned long long mask = __ballot(keep);
        if (lane == 0) wave_total[wave] = __popcll(mask);
        __syncthreads();                         // every member of the chunk has been read
        int before = 0, total = 0;
        for (int t = 0; t < 16; ++t) {
            before += t < wave ? wave_total[t] : 0;
            total += wave_total[t];
        }
        if (keep) o[k + before + __popcll(mask & ((1ull << lane) - 1ull))] = val;
        k += total;
        __syncthreads();                         // wave_total is reused by the next chunk
    }
    if (threadIdx.x == 0) {
        v.olen[x] = k;
        if (blockIdx.x == 0) {
            v.olen[w] = r;
            v.out_off[w] = rows_at;
            v.mred[w - v.n] = r;
        }
    }
}

}  // namespace

struct DeviceCounter {
    View v{};
    int64_t e = 0, capacity = 0;
    int64_t pool_used = 0;            // entries of the aggregation nodes' out-lists appended so far
    hipStream_t stream = nullptr;
    std::vector<void *> allocs;
    // pinned host buffers
    int32_t *h_req = nullptr, *h_nfound = nullptr, *h_rows = nullptr;
    Found *h_eager = nullptr, *h_found = nullptr;
    std::vector<int32_t> prio_desc;   // the static bounds of the original nodes, descending
    std::vector<int32_t> rank;        // mirror id of every original node
    // how many results the host takes from the first copy / at all (tests lower both through
    // HAG_SEARCH_EAGER_LIMIT / HAG_SEARCH_FOUND_LIMIT to reach the second copy and the host fallback)
    int eager_limit = kEager, found_limit = kFoundCap;
};

#define CNT_TRY(expr)                                                              \
    do {                                                                           \
        hipError_t _e = (expr);                                                    \
        if (_e != hipSuccess) {                                                    \
            err = std::string(#expr) + ": " + hipGetErrorString(_e);               \
            return false;                                                          \
        }                                                                          \
    } while (0)

static bool counter_setup(DeviceCounter *d, const CounterInit &in, std::string &err) {
    const int64_t n = in.n, e = in.e, m = in.n + in.capacity;
    d->e = e;
    d->capacity = in.capacity;
    d->v.n = n;
    d->v.m = m;
    if (const char *v = std::getenv("HAG_SEARCH_EAGER_LIMIT")) d->eager_limit = std::max(0, std::min(kEager, std::atoi(v)));
    if (const char *v = std::getenv("HAG_SEARCH_FOUND_LIMIT")) d->found_limit = std::max(0, std::min(kFoundCap, std::atoi(v)));
    CNT_TRY(hipStreamCreate(&d->stream));
    auto dev_alloc = [&](void **p, size_t bytes) {
        hipError_t rc = hipMalloc(p, std::max<size_t>(bytes, 256));
        if (rc == hipSuccess) d->allocs.push_back(*p);
        return rc;
    };
    int64_t *ptr = nullptr;
    int32_t *by_rank = nullptr, *req = nullptr;
    std::vector<int32_t> h_by_rank((size_t)n);
    std::vector<int32_t> &h_rank = d->rank;
    h_rank.resize((size_t)n);
    for (int64_t i = 0; i < n; ++i) h_by_rank[i] = (int32_t)i;
    std::sort(h_by_rank.begin(), h_by_rank.end(),
              [&](int32_t a, int32_t b) { return in.prio[a] != in.prio[b] ? in.prio[a] > in.prio[b] : a < b; });
    d->prio_desc.resize((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        h_rank[h_by_rank[i]] = (int32_t)i;
        d->prio_desc[i] = in.prio[h_by_rank[i]];
    }
    CNT_TRY(dev_alloc((void **)&ptr, (size_t)(n + 1) * 8));
    CNT_TRY(dev_alloc((void **)&d->v.nb, (size_t)e * 4));
    CNT_TRY(dev_alloc((void **)&d->v.len, (size_t)n * 4));
    CNT_TRY(dev_alloc((void **)&d->v.norig, (size_t)n * 4));
    CNT_TRY(dev_alloc((void **)&by_rank, (size_t)n * 4));
    CNT_TRY(dev_alloc((void **)&d->v.mred, (size_t)in.capacity * 4));
    CNT_TRY(dev_alloc((void **)&d->v.out_off, (size_t)m * 8));
    // out-lists of the original nodes first, then room for those of the aggregation nodes: a
    // merge of redundancy r shortens the lists by r entries in total, so the r's sum to at most e
    CNT_TRY(dev_alloc((void **)&d->v.out, (size_t)e * 8));
    CNT_TRY(dev_alloc((void **)&d->v.olen, (size_t)m * 4));
    CNT_TRY(dev_alloc((void **)&d->v.cnt, (size_t)kMaxBatch * (size_t)m * 4));
    CNT_TRY(dev_alloc((void **)&req, (size_t)kMaxBatch * 16));
    CNT_TRY(dev_alloc((void **)&d->v.nfound, (size_t)kMaxBatch * 4));
    CNT_TRY(dev_alloc((void **)&d->v.found, (size_t)kMaxBatch * kFoundCap * sizeof(Found)));
    d->v.ptr = ptr;
    d->v.by_rank = by_rank;
    d->v.req = req;
    CNT_TRY(hipHostMalloc((void **)&d->h_req, (size_t)kMaxBatch * 16, hipHostMallocDefault));
    CNT_TRY(hipHostMalloc((void **)&d->h_nfound, (size_t)kMaxBatch * 4, hipHostMallocDefault));
    CNT_TRY(hipHostMalloc((void **)&d->h_eager, (size_t)kMaxBatch * kEager * sizeof(Found), hipHostMallocDefault));
    CNT_TRY(hipHostMalloc((void **)&d->h_found, (size_t)kMaxBatch * kFoundCap * sizeof(Found), hipHostMallocDefault));
    CNT_TRY(hipHostMalloc((void **)&d->h_rows, std::max<size_t>((size_t)e * 4, 256), hipHostMallocDefault));

    CNT_TRY(hipMemcpyAsync(ptr, in.ptr, (size_t)(n + 1) * 8, hipMemcpyHostToDevice, d->stream));
    {
        // the lists in mirror ids (all members are original nodes at this point), staged through h_rows
        for (int64_t i = 0; i < e; ++i) d->h_rows[i] = h_rank[in.nb[i]];
        CNT_TRY(hipMemcpyAsync(d->v.nb, d->h_rows, (size_t)e * 4, hipMemcpyHostToDevice, d->stream));
    }
    CNT_TRY(hipMemcpyAsync(d->v.len, in.len, (size_t)n * 4, hipMemcpyHostToDevice, d->stream));
    CNT_TRY(hipMemcpyAsync(d->v.norig, in.norig, (size_t)n * 4, hipMemcpyHostToDevice, d->stream));
    CNT_TRY(hipMemcpyAsync(by_rank, h_by_rank.data(), (size_t)n * 4, hipMemcpyHostToDevice, d->stream));
    CNT_TRY(hipMemcpyAsync(d->v.out_off, in.out_ptr, (size_t)n * 8, hipMemcpyHostToDevice, d->stream));
    CNT_TRY(hipMemcpyAsync(d->v.out, in.out_col, (size_t)e * 4, hipMemcpyHostToDevice, d->stream));
    CNT_TRY(hipMemcpyAsync(d->v.olen, in.olen, (size_t)n * 4, hipMemcpyHostToDevice, d->stream));
    CNT_TRY(hipMemsetAsync(d->v.olen + n, 0, (size_t)in.capacity * 4, d->stream));
    CNT_TRY(hipMemsetAsync(d->v.cnt, 0, (size_t)kMaxBatch * (size_t)m * 4, d->stream));
    CNT_TRY(hipStreamSynchronize(d->stream));   // the host arrays may change from here on
    return true;
}

DeviceCounter *counter_create(const CounterInit &in, std::string &err) {
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count < 1) {
        err = "HAG_SEARCH_DEVICE: no HIP device";
        return nullptr;
    }
    DeviceCounter *d = new DeviceCounter;
    if (!counter_setup(d, in, err)) {
        counter_destroy(d);
        return nullptr;
    }
    return d;
}

void counter_destroy(DeviceCounter *d) {
    if (!d) return;
    if (d->stream) (void)hipStreamSynchronize(d->stream);
    for (void *p : d->allocs) (void)hipFree(p);
    for (void *p : {(void *)d->h_req, (void *)d->h_nfound, (void *)d->h_eager, (void *)d->h_found, (void *)d->h_rows})
        if (p) (void)hipHostFree(p);
    if (d->stream) (void)hipStreamDestroy(d->stream);
    delete d;
}

int counter_max_batch(const DeviceCounter *) { return kMaxBatch; }

bool counter_merge(DeviceCounter *d, int32_t p, int32_t q, int32_t w, const int32_t *rows, int32_t r, std::string &err) {
    const View &v = d->v;
    if (r < 1 || d->pool_used + r > d->e || p < 0 || q < 0 || p == q || p >= w || q >= w || w < v.n || w >= v.m) {
        err = "device mirror of the search: merge out of range";
        return false;
    }
    int32_t *stage = d->h_rows + d->pool_used;
    std::memcpy(stage, rows, (size_t)r * 4);
    const int64_t rows_at = d->e + d->pool_used;
    CNT_TRY(hipMemcpyAsync(v.out + rows_at, stage, (size_t)r * 4, hipMemcpyHostToDevice, d->stream));
    const int32_t pm = p < v.n ? d->rank[p] : p, qm = q < v.n ? d->rank[q] : q;
    hipLaunchKernelGGL(rewrite_kernel, dim3((unsigned)((r + 3) / 4)), dim3(256), 0, d->stream, v, rows_at, r, pm, qm, w);
    hipLaunchKernelGGL(out_remove_kernel, dim3(2), dim3(1024), 0, d->stream, v, rows_at, r, p, q, w);
    CNT_TRY(hipGetLastError());
    d->pool_used += r;
    return true;
}

bool counter_sweep(DeviceCounter *d, int nb, const int32_t *x, const int32_t *theta,
                   std::vector<std::vector<Found>> &found, std::vector<char> &overflow, std::string &err) {
    const View &v = d->v;
    found.assign((size_t)nb, {});
    overflow.assign((size_t)nb, 0);
    if (nb < 1) return true;
    if (nb > kMaxBatch) {
        err = "device mirror of the search: batch too large";
        return false;
    }
    for (int s = 0; s < nb; ++s) {
        if (x[s] < 0 || x[s] >= v.m || theta[s] < 1) {
            err = "device mirror of the search: request out of range";
            return false;
        }
        d->h_req[4 * s] = x[s];
        d->h_req[4 * s + 1] = theta[s];
        d->h_req[4 * s + 2] = (int32_t)(std::upper_bound(d->prio_desc.begin(), d->prio_desc.end(), theta[s],
                                                         [](int32_t t, int32_t pr) { return t > pr; }) - d->prio_desc.begin());
        d->h_req[4 * s + 3] = 0;
    }
    CNT_TRY(hipMemcpyAsync((void *)v.req, d->h_req, (size_t)nb * 16, hipMemcpyHostToDevice, d->stream));
    hipLaunchKernelGGL(count_kernel, dim3(kCountBlocks, (unsigned)nb), dim3(256), 0, d->stream, v);
    const unsigned scan_blocks = (unsigned)std::min<int64_t>((v.m + 255) / 256, 1024);
    hipLaunchKernelGGL(collect_kernel, dim3(scan_blocks, (unsigned)nb), dim3(256), 0, d->stream, v);
    CNT_TRY(hipGetLastError());
    CNT_TRY(hipMemcpyAsync(d->h_nfound, v.nfound, (size_t)nb * 4, hipMemcpyDeviceToHost, d->stream));
    CNT_TRY(hipMemcpy2DAsync(d->h_eager, kEager * sizeof(Found), v.found, kFoundCap * sizeof(Found),
                             kEager * sizeof(Found), (size_t)nb, hipMemcpyDeviceToHost, d->stream));
    CNT_TRY(hipStreamSynchronize(d->stream));
    bool more = false;
    for (int s = 0; s < nb; ++s) {
        const int k = d->h_nfound[s];
        if (k > d->found_limit) { overflow[s] = 1; continue; }
        if (k > d->eager_limit) {
            CNT_TRY(hipMemcpyAsync(d->h_found + (size_t)s * kFoundCap, v.found + (size_t)s * kFoundCap,
                                   (size_t)k * sizeof(Found), hipMemcpyDeviceToHost, d->stream));
            more = true;
        }
    }
    if (more) CNT_TRY(hipStreamSynchronize(d->stream));
    for (int s = 0; s < nb; ++s) {
        const int k = d->h_nfound[s];
        if (overflow[s] || k <= 0) continue;
        const Found *src = k > d->eager_limit ? d->h_found + (size_t)s * kFoundCap : d->h_eager + (size_t)s * kEager;
        found[s].assign(src, src + k);
    }
    return true;
}

}  // namespace hag

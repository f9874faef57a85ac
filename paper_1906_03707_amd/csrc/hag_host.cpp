// Host side of libhag: input validation, the greedy HAG search (Algorithm 3, set
// Aggregate), replay of a merge list, level ordering, transposes, launch
// schedules and statistics.  No device code here.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <memory>
#include <mutex>
#include <new>
#include <numeric>
#include <queue>
#include <thread>
#include <tuple>

#include "hag_internal.hpp"

namespace hag {

static thread_local std::string g_err;
void set_error(const std::string &msg) { g_err = msg; }

static int fail(int code, const std::string &msg) {
    set_error(msg);
    return code;
}

static int64_t env_i64(const char *name, int64_t dflt) {
    const char *s = std::getenv(name);
    return s ? std::atoll(s) : dflt;
}

static unsigned host_threads() {
    unsigned t = std::thread::hardware_concurrency();
    if (const char *s = std::getenv("HAG_NUM_THREADS")) t = (unsigned)std::max(1, std::atoi(s));
    if (const char *s = std::getenv("OMP_NUM_THREADS")) t = std::min(t, (unsigned)std::max(1, std::atoi(s)));
    return std::max(1u, std::min(t, 64u));
}

// Runs f(i, thread) for i in [0, n) on up to `threads` threads.  An exception thrown by f (in
// practice std::bad_alloc) stops the remaining work and is rethrown on the calling thread after
// all workers have joined, so that the entry points' own handlers turn it into a status code.
template <class F>
static void parallel_for(int64_t n, unsigned threads, F f) {
    threads = (unsigned)std::min<int64_t>(threads, std::max<int64_t>(n, 1));
    if (threads <= 1) {
        for (int64_t i = 0; i < n; ++i) f(i, 0u);
        return;
    }
    std::atomic<int64_t> next{0};
    std::atomic<bool> failed{false};
    std::exception_ptr first;
    std::mutex first_lock;
    std::vector<std::thread> pool;
    auto work = [&](unsigned t) {
        try {
            for (;;) {
                int64_t i = next.fetch_add(1);
                if (i >= n || failed.load(std::memory_order_relaxed)) break;
                f(i, t);
            }
        } catch (...) {
            std::lock_guard<std::mutex> g(first_lock);
            if (!first) first = std::current_exception();
            failed.store(true);
        }
    };
    try {
        for (unsigned t = 1; t < threads; ++t) pool.emplace_back(work, t);
    } catch (...) {   // could not start every worker: the ones that run finish the job
    }
    work(0u);
    for (auto &th : pool) th.join();
    if (first) std::rethrow_exception(first);
}

// ------------------------------------------------------------------------------------------
// validation + copy of the input graph
// ------------------------------------------------------------------------------------------
static int load_graph(int64_t n, const int64_t *rowptr, const int32_t *col, uint32_t flags, Csr &g) {
    if (n < 0) return fail(HAG_EINVAL, "n < 0");
    if (!rowptr) return fail(HAG_EINVAL, "rowptr is NULL");
    if (rowptr[0] != 0) return fail(HAG_EINVAL, "rowptr[0] != 0");
    for (int64_t v = 0; v < n; ++v)
        if (rowptr[v + 1] < rowptr[v]) return fail(HAG_EINVAL, "rowptr is not monotone at row " + std::to_string(v));
    int64_t e = rowptr[n];
    if (e > 0 && !col) return fail(HAG_EINVAL, "col is NULL");
    for (int64_t i = 0; i < e; ++i)
        if (col[i] < 0 || col[i] >= n) return fail(HAG_EINVAL, "col out of range at entry " + std::to_string(i));
    g.ptr.assign(n + 1, 0);
    g.col.clear();
    g.col.reserve((size_t)e);
    std::vector<int32_t> tmp;
    for (int64_t v = 0; v < n; ++v) {
        tmp.assign(col + rowptr[v], col + rowptr[v + 1]);
        std::sort(tmp.begin(), tmp.end());
        auto last = std::unique(tmp.begin(), tmp.end());
        if (last != tmp.end()) {
            if (!(flags & HAG_SEARCH_DEDUP))
                return fail(HAG_EINVAL, "duplicate neighbour in row " + std::to_string(v) + " (a neighbourhood is a set; pass HAG_SEARCH_DEDUP to drop duplicates)");
            tmp.erase(last, tmp.end());
        }
        g.col.insert(g.col.end(), tmp.begin(), tmp.end());
        g.ptr[v + 1] = (int64_t)g.col.size();
    }
    return HAG_OK;
}

// rows of `t` = columns of `c`; `rows_out` = number of rows of t
static void transpose(const Csr &c, int64_t rows_out, Csr &t) {
    int64_t rows_in = (int64_t)c.ptr.size() - 1;
    t.ptr.assign(rows_out + 1, 0);
    for (int32_t x : c.col) t.ptr[x + 1]++;
    for (int64_t i = 0; i < rows_out; ++i) t.ptr[i + 1] += t.ptr[i];
    t.col.resize(c.col.size());
    std::vector<int64_t> fill(t.ptr.begin(), t.ptr.end() - 1);
    for (int64_t r = 0; r < rows_in; ++r)
        for (int64_t i = c.ptr[r]; i < c.ptr[r + 1]; ++i) t.col[fill[c.col[i]]++] = (int32_t)r;
}

// ------------------------------------------------------------------------------------------
// Working state of Algorithm 3: the current lists Nhat_u (u in V) and, for every HAG node x,
// the sorted list out[x] of the u whose list holds x.
// ------------------------------------------------------------------------------------------
struct Builder {
    int64_t n = 0;
    const Csr *g = nullptr;
    std::vector<int32_t> nb;        // lists, in place of g->col (a list never grows)
    std::vector<int32_t> len;       // current length of each list
    Csr gt;                         // out-lists of original nodes, shrunk in place
    std::vector<int32_t> olen;
    std::vector<std::vector<int32_t>> out_agg;
    std::vector<int32_t> m_left, m_right, m_red, depth;
    std::vector<int32_t> scratch;
    // Every list keeps its original members first, ordered by descending prio (their initial
    // out-degree, an upper bound on any redundancy they can ever reach), then its aggregation
    // members in creation order (whose creation redundancies are non-increasing).  A sweep
    // that only cares about partners able to reach a threshold can then stop early.
    std::vector<int32_t> prio, norig;
    unsigned threads = 1;

    void init(const Csr &graph, bool order_by_priority = false, unsigned threads_ = 1) {
        threads = threads_;
        g = &graph;
        n = (int64_t)graph.ptr.size() - 1;
        nb = graph.col;
        len.resize(n);
        for (int64_t u = 0; u < n; ++u) len[u] = (int32_t)(graph.ptr[u + 1] - graph.ptr[u]);
        norig = len;
        transpose(graph, n, gt);
        olen.resize(n);
        for (int64_t x = 0; x < n; ++x) olen[x] = (int32_t)(gt.ptr[x + 1] - gt.ptr[x]);
        if (order_by_priority) {
            prio = olen;
            parallel_for((n + 255) / 256, threads, [&](int64_t blk, unsigned) {
                for (int64_t u = blk * 256; u < std::min<int64_t>(n, blk * 256 + 256); ++u)
                    std::sort(nb.begin() + graph.ptr[u], nb.begin() + graph.ptr[u + 1], [&](int32_t x, int32_t y) {
                        return prio[x] != prio[y] ? prio[x] > prio[y] : x < y;
                    });
            });
        }
    }
    int64_t a() const { return (int64_t)m_left.size(); }
    const int32_t *out_ptr(int32_t x) const { return x < n ? gt.col.data() + gt.ptr[x] : out_agg[x - n].data(); }
    int32_t out_len(int32_t x) const { return x < n ? olen[x] : (int32_t)out_agg[x - n].size(); }
    int32_t depth_of(int32_t x) const { return x < n ? 0 : depth[x - n]; }

    // |out(p) ∩ out(q)|; the common entries go to dst if given.  The merge loop is written
    // without data-dependent branches: which list advances is close to a coin flip.
    int32_t intersect(int32_t p, int32_t q, std::vector<int32_t> *dst) const {
        const int32_t *a_ = out_ptr(p), *b_ = out_ptr(q);
        const int32_t la = out_len(p), lb = out_len(q);
        int32_t i = 0, j = 0, c = 0;
        if (!dst && (la > 16 * lb || lb > 16 * la)) {
            // very unequal lengths: look every entry of the short list up in the rest of the long one
            const int32_t *s_ = la < lb ? a_ : b_, *l_ = la < lb ? b_ : a_;
            const int32_t ls = std::min(la, lb), ll = std::max(la, lb);
            const int32_t *from = l_, *end = l_ + ll;
            for (int32_t k = 0; k < ls && from < end; ++k) {
                from = std::lower_bound(from, end, s_[k]);
                c += (from < end && *from == s_[k]);
            }
            return c;
        }
        if (dst) {
            dst->resize((size_t)std::min(la, lb) + 1);
            int32_t *o = dst->data();
            while (i < la && j < lb) {
                const int32_t x = a_[i], y = b_[j];
                o[c] = x;
                c += (x == y);
                i += (x <= y);
                j += (y <= x);
            }
            dst->resize((size_t)c);
            return c;
        }
        while (i < la && j < lb) {
            const int32_t x = a_[i], y = b_[j];
            c += (x == y);
            i += (x <= y);
            j += (y <= x);
        }
        return c;
    }
    void remove_from_out(int32_t x, const std::vector<int32_t> &rm) {
        int32_t *o = x < n ? gt.col.data() + gt.ptr[x] : out_agg[x - n].data();
        int32_t l = out_len(x), k = 0;
        size_t j = 0;
        for (int32_t i = 0; i < l; ++i) {
            while (j < rm.size() && rm[j] < o[i]) ++j;
            if (j < rm.size() && rm[j] == o[i]) continue;
            o[k++] = o[i];
        }
        if (x < n) olen[x] = k; else out_agg[x - n].resize(k);
    }
    // the rewrite loop of Algorithm 3 for the pair (p, q); returns the redundancy
    int32_t apply_merge(int32_t p, int32_t q) {
        scratch.clear();
        int32_t r = intersect(p, q, &scratch);
        int32_t w = (int32_t)(n + a());
        // A list is ordered (original members by (prio descending, id ascending) or, without
        // priorities, by id; then aggregation members by id), so p and q are found by bisection
        // and taken out with two block moves; w has the largest id and goes to the end.
        auto position = [&](const int32_t *l, int32_t no, int32_t L, int32_t x) {
            if (x >= n) return (int32_t)(std::lower_bound(l + no, l + L, x) - l);
            if (prio.empty()) return (int32_t)(std::lower_bound(l, l + no, x) - l);
            return (int32_t)(std::lower_bound(l, l + no, x, [&](int32_t y, int32_t key) {
                return prio[y] != prio[key] ? prio[y] > prio[key] : y < key;
            }) - l);
        };
        auto rewrite = [&](int32_t u) {
            int32_t *l = nb.data() + g->ptr[u];
            const int32_t L = len[u], no = norig[u];
            int32_t i = position(l, no, L, p), j = position(l, no, L, q);
            if (i > j) std::swap(i, j);
            std::memmove(l + i, l + i + 1, sizeof(int32_t) * (size_t)(j - i - 1));
            std::memmove(l + j - 1, l + j + 1, sizeof(int32_t) * (size_t)(L - j - 1));
            l[L - 2] = w;
            len[u] = L - 1;
            norig[u] -= (p < n) + (q < n);
        };
        if (threads > 1 && r >= 1024) {
            // the lists are independent; worth the threads only for the large merges of a big graph
            const int64_t chunk = 64, chunks = (r + chunk - 1) / chunk;
            parallel_for(chunks, threads, [&](int64_t c, unsigned) {
                for (int64_t i = c * chunk; i < std::min<int64_t>(r, (c + 1) * chunk); ++i) rewrite(scratch[i]);
            });
        } else {
            for (int32_t u : scratch) rewrite(u);
        }
        remove_from_out(p, scratch);
        remove_from_out(q, scratch);
        out_agg.emplace_back(scratch);
        m_left.push_back(std::min(p, q));
        m_right.push_back(std::max(p, q));
        m_red.push_back(r);
        depth.push_back(1 + std::max(depth_of(p), depth_of(q)));
        return r;
    }
};

// ------------------------------------------------------------------------------------------
// Algorithm 3 with lazily evaluated upper bounds.
//
// The listing asks for the pair of maximal Redundancy in every iteration.  A heap over all
// co-occurring pairs is infeasible for dense graphs (sum over u of |N(u)|^2 / 2 entries), so
// the heap here is over NODES: key[x] is an upper bound on max_y Redundancy(x, y).
//
// Facts used (all follow from the rewrite loop, which only removes p and q from lists and
// adds the new node w):
//   (1) Redundancy(x, y) of an existing pair never grows, and changes only in an iteration
//       that merges x or y;
//   (2) a new node w = (p, q) has Redundancy(x, w) <= Redundancy(x, p) and <= Redundancy(x, q).
// Per node x the search keeps a short list of candidate partners (y, c) with c an upper bound
// on Redundancy(x, y) (exact at the iteration `stamp`), and `tail`, an upper bound for every
// partner that existed at x's last sweep and is not listed.  By (2) a partner created later is
// bounded by its parents, so key[x] = max(best c, tail) bounds all of x's pairs.  When x is on
// top of the heap its best entry is made exact by intersecting the two out-lists (cheap), every
// descendant of that partner born since the entry was last exact is looked up the same way
// (a node hands rows on to the nodes built from it, so only the partner's OLD count bounds
// them, not its current one), and only when the list is exhausted (best c <= tail) is x swept
// again: one counting pass over the lists that hold x.
// The heap is ordered by (key descending, id ascending), entries by (c descending, id
// ascending); this makes the accepted pair the lexicographically smallest (smaller id, larger
// id) among the pairs of maximal redundancy, i.e. the result does not depend on the laziness.
// ------------------------------------------------------------------------------------------
struct Searcher {
    Builder b;
    int64_t capacity = 0;
    int32_t max_depth = 0;
    int kKeep = 12;                               // candidates kept per sweep (more if tied)
    struct Cand { int32_t y, c; int64_t stamp; };
    std::vector<std::vector<Cand>> cand;           // sorted by (c desc, y asc)
    std::vector<int32_t> key, tail, version;
    std::vector<int64_t> mod_stamp, born;          // last iteration a node was merged / its creation
    std::vector<std::vector<int32_t>> children;    // aggregation nodes built from a node
    std::vector<int64_t> visited;                  // refresh() that last looked at a node
    int64_t visit_id = 0;
    int64_t iter = 1;
    using Entry = std::tuple<int32_t, int32_t, int32_t>;  // key, -id, version
    std::priority_queue<Entry> heap;
    unsigned threads = 1;
    bool single_thread = false;
    // optional progress log / checkpoint of the merge list (environment: HAG_SEARCH_PROGRESS=<every>,
    // HAG_SEARCH_CHECKPOINT=<file>); long searches can then be resumed with hag_from_merges
    int64_t progress_every = 0;
    std::chrono::steady_clock::time_point t_start;
    int64_t n_sweep = 0, n_batch = 0, n_refresh = 0;
    std::atomic<int64_t> n_empty{0};
    double t_sweep = 0, t_refresh = 0, t_merge = 0;
    std::vector<std::vector<int32_t>> cnt, touched;
    std::vector<std::vector<Found>> found_host;
    // optional: counting on the GPU (HAG_SEARCH_DEVICE); the host lists stay authoritative
    DeviceCounter *dev = nullptr;
    std::string dev_err;
    std::vector<std::vector<Found>> found_dev;
    std::vector<char> overflow_dev;

    void report_progress() {
        double el = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_start).count();
        std::fprintf(stderr, "[hag_search] %lld merges, redundancy %d, %.1f s, %lld sweeps (%lld empty) in %lld batches (%.1f s), %lld refreshes (%.1f s), merges %.1f s\n",
                     (long long)b.a(), b.m_red.back(), el, (long long)n_sweep, (long long)n_empty.load(), (long long)n_batch, t_sweep, (long long)n_refresh, t_refresh, t_merge);
        if (const char *path = std::getenv("HAG_SEARCH_CHECKPOINT")) {
            std::string tmp = std::string(path) + ".tmp";
            if (FILE *f = std::fopen(tmp.c_str(), "wb")) {
                int64_t a = b.a();
                std::fwrite(&a, sizeof a, 1, f);
                std::fwrite(b.m_left.data(), sizeof(int32_t), (size_t)a, f);
                std::fwrite(b.m_right.data(), sizeof(int32_t), (size_t)a, f);
                std::fclose(f);
                std::rename(tmp.c_str(), path);
            }
        }
    }

    static bool better(const Cand &p, const Cand &q) { return p.c != q.c ? p.c > q.c : p.y < q.y; }
    int32_t best_c(int32_t x) const { return cand[x].empty() ? 0 : cand[x][0].c; }
    void rekey(int32_t x) { key[x] = std::max(best_c(x), tail[x]); }
    void push(int32_t x) {
        version[x]++;
        if (key[x] >= 2) heap.emplace(key[x], -x, version[x]);
    }
    bool mergeable(int32_t x) const { return max_depth <= 0 || b.depth_of(x) < max_depth; }

    // One counting pass over the lists that hold x, restricted to partners whose static bound
    // reaches theta = a fixed share (theta_pct) of x's key.  Counts >= theta are exact and complete; if none
    // reaches theta, theta-1 becomes the bound for everything and x is swept again later with
    // a lower threshold.
    int32_t theta_pct = 50;
    int32_t theta_of(int32_t x) const { return std::max(2, (int32_t)(((int64_t)key[x] * theta_pct + 99) / 100)); }

    void sweep(int32_t x, unsigned t) {
        auto &c = cnt[t];
        auto &tl = touched[t];
        tl.clear();
        const int32_t theta = theta_of(x);
        const int32_t *o = b.out_ptr(x);
        const int32_t ol = b.out_len(x);
        const int32_t n = (int32_t)b.n;
        for (int32_t i = 0; i < ol; ++i) {
            const int32_t u = o[i];
            const int32_t *l = b.nb.data() + b.g->ptr[u];
            const int32_t no = b.norig[u], L = b.len[u];
            int32_t lo = 0, hi = no;          // first original member with prio < theta
            while (lo < hi) {
                int32_t mid = (lo + hi) >> 1;
                if (b.prio[l[mid]] >= theta) lo = mid + 1; else hi = mid;
            }
            for (int32_t j = 0; j < lo; ++j) {
                int32_t y = l[j];
                if (c[y]++ == 0) tl.push_back(y);
            }
            for (int32_t j = no; j < L; ++j) {
                int32_t y = l[j];
                if (b.m_red[y - n] < theta) break;
                if (c[y]++ == 0) tl.push_back(y);
            }
        }
        auto &fd = found_host[t];
        fd.clear();
        for (int32_t y : tl) {
            if (c[y] >= theta) fd.push_back(Found{y, c[y]});
            c[y] = 0;
        }
        finish_sweep(x, theta, fd);
    }

    // `found` = every (y, count) with count >= theta: rebuild x's candidate list and tail from it
    void finish_sweep(int32_t x, int32_t theta, const std::vector<Found> &found) {
        auto &lst = cand[x];
        lst.clear();
        int32_t below = theta - 1;   // bound for everything not listed
        for (const Found &f : found) {
            if (f.y == x || !mergeable(f.y)) continue;
            if (f.c >= theta) lst.push_back(Cand{f.y, f.c, iter});
        }
        if (lst.empty()) n_empty++;
        std::sort(lst.begin(), lst.end(), better);
        if ((int)lst.size() > kKeep) {
            int32_t cut = lst[kKeep].c;            // first dropped count; keep only strictly larger
            size_t keep = (size_t)kKeep;
            while (keep > 0 && lst[keep - 1].c == cut) --keep;
            if (keep == 0) {                        // more than kKeep partners tied at the top
                keep = (size_t)kKeep;
                while (keep < lst.size() && lst[keep].c == cut) ++keep;
                cut = keep < lst.size() ? lst[keep].c : below;
            }
            lst.resize(keep);
            below = std::max(below, cut);
        }
        tail[x] = below;
        rekey(x);
    }

    // the same for a batch of nodes, counted on the device
    bool sweep_on_device(const std::vector<int32_t> &xs) {
        std::vector<int32_t> theta(xs.size());
        for (size_t i = 0; i < xs.size(); ++i) theta[i] = theta_of(xs[i]);
        if (!counter_sweep(dev, (int)xs.size(), xs.data(), theta.data(), found_dev, overflow_dev, dev_err)) return false;
        for (size_t i = 0; i < xs.size(); ++i) {
            if (overflow_dev[i]) sweep(xs[i], 0);
            else finish_sweep(xs[i], theta[i], found_dev[i]);
        }
        return true;
    }

    // Make x's best entry exact, or report that x needs a sweep.  Returns 1 if the best entry
    // is exact and beats the tail (x may be accepted), 0 if the key changed (push x back),
    // -1 if the list is exhausted.
    int refresh(int32_t x) {
        auto &lst = cand[x];
        if (lst.empty() || lst[0].c <= tail[x]) return tail[x] >= 2 || !lst.empty() ? -1 : 0;
        Cand &e = lst[0];
        if (mod_stamp[x] < e.stamp && mod_stamp[e.y] < e.stamp) return 1;
        ++n_refresh;
        const int64_t since = e.stamp;
        const int32_t y = e.y;
        e.c = b.intersect(x, y, nullptr);
        e.stamp = iter;
        // Descendants of y born since the entry was exact.  Fact (2) bounds each of them by the
        // OLD count of (x, y) only: a node hands rows on to its children, so its current count
        // says nothing about theirs, and the whole subtree has to be looked at.  A descendant
        // that is already listed carries a bound for its own subtree.
        std::vector<int32_t> stack;
        {
            // children are listed in creation order, so those born since the stamp are a suffix
            const auto &ch = children[y];
            auto first = std::partition_point(ch.begin(), ch.end(), [&](int32_t w) { return born[w] < since; });
            stack.assign(first, ch.end());
        }
        ++visit_id;
        while (!stack.empty()) {
            int32_t w = stack.back();
            stack.pop_back();
            if (visited[w] == visit_id) continue;      // reachable through both of its parents
            visited[w] = visit_id;
            bool listed = false;
            for (const Cand &q : lst) listed |= (q.y == w);
            if (listed) continue;
            for (int32_t w2 : children[w]) stack.push_back(w2);
            if (w == x || !mergeable(w)) continue;
            int32_t cw = b.intersect(x, w, nullptr);
            if (cw > tail[x]) lst.push_back(Cand{w, cw, iter});
        }
        std::sort(lst.begin(), lst.end(), better);
        while (!lst.empty() && lst.back().c <= tail[x]) lst.pop_back();   // covered by the tail bound
        rekey(x);
        return 0;
    }

    // false only if the device mirror failed (dev_err says why)
    bool run() {
        int64_t n = b.n, m = n + capacity;
        key.assign(m, 0); tail.assign(m, 0); version.assign(m, 0);
        mod_stamp.assign(m, 0); born.assign(m, 0);
        cand.assign(m, {}); children.assign(m, {});
        visited.assign(m, 0);
        threads = single_thread ? 1u : host_threads();
        progress_every = single_thread ? 0 : env_i64("HAG_SEARCH_PROGRESS", 0);
        kKeep = (int)std::max<int64_t>(1, env_i64("HAG_SEARCH_KEEP", 12));
        // threshold of a sweep, in percent of the node's key: a higher one makes a sweep cheaper and more
        // likely to come back empty; measured best at half the key on the host, at two thirds on the device
        theta_pct = (int32_t)std::min<int64_t>(100, std::max<int64_t>(1, env_i64("HAG_SEARCH_THETA_PCT", dev ? 65 : 50)));
        t_start = std::chrono::steady_clock::now();
        cnt.assign(threads, std::vector<int32_t>(m, 0));
        touched.assign(threads, {});
        found_host.assign(threads, {});
        const size_t batch_max = dev ? (size_t)counter_max_batch(dev) : (size_t)threads;
        for (int64_t x = 0; x < n; ++x) { tail[x] = b.olen[x]; key[x] = tail[x]; push((int32_t)x); }
        std::vector<int32_t> batch, dirty;
        while (b.a() < capacity) {
            int32_t chosen = -1;
            while (!heap.empty()) {
                auto [k, negx, ver] = heap.top();
                int32_t x = -negx;
                heap.pop();
                if (ver != version[x]) continue;
                auto t0 = std::chrono::steady_clock::now();
                int rc = refresh(x);
                t_refresh += std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
                if (rc == 1) { chosen = x; break; }
                if (rc == 0) { push(x); continue; }
                // x needs a sweep; sweep it together with the next few exhausted nodes
                batch.assign(1, x);
                dirty.clear();
                while (!heap.empty() && batch.size() < batch_max) {
                    auto [k2, negx2, ver2] = heap.top();
                    int32_t x2 = -negx2;
                    if (ver2 != version[x2]) { heap.pop(); continue; }
                    if (k2 < key[x] / 2) break;
                    heap.pop();
                    batch.push_back(x2);
                }
                for (int32_t z : batch) {
                    bool exhausted = cand[z].empty() || cand[z][0].c <= tail[z];
                    if (exhausted && key[z] >= 2) dirty.push_back(z);
                    else heap.emplace(key[z], -z, version[z]);
                }
                auto t1 = std::chrono::steady_clock::now();
                if (dev) {
                    if (!sweep_on_device(dirty)) return false;
                } else {
                    parallel_for((int64_t)dirty.size(), threads, [&](int64_t i, unsigned t) { sweep(dirty[i], t); });
                }
                t_sweep += std::chrono::duration<double>(std::chrono::steady_clock::now() - t1).count();
                n_sweep += (int64_t)dirty.size();
                n_batch += dirty.empty() ? 0 : 1;
                for (int32_t z : dirty) push(z);
            }
            if (chosen < 0 || key[chosen] < 2) break;
            int32_t p = chosen, q = cand[chosen][0].y;
            auto t2 = std::chrono::steady_clock::now();
            const int32_t r = b.apply_merge(p, q);
            if (dev && !counter_merge(dev, p, q, (int32_t)(b.n + b.a() - 1), b.scratch.data(), r, dev_err)) return false;
            t_merge += std::chrono::duration<double>(std::chrono::steady_clock::now() - t2).count();
            if (progress_every > 0 && b.a() % progress_every == 0) report_progress();
            int32_t w = (int32_t)(b.n + b.a() - 1);
            mod_stamp[p] = mod_stamp[q] = iter;
            born[w] = iter;
            children[p].push_back(w);
            children[q].push_back(w);
            ++iter;
            for (int32_t x : {p, q}) {
                tail[x] = std::min(tail[x], b.out_len(x));
                for (Cand &e : cand[x]) e.c = std::min(e.c, b.out_len(x));
                rekey(x);
                push(x);
            }
            tail[w] = mergeable(w) ? b.out_len(w) : 0;
            rekey(w);
            push(w);
        }
        return true;
    }
};

// ------------------------------------------------------------------------------------------
// schedules
// ------------------------------------------------------------------------------------------
// Items are ordered by length class, longest first, and keep their row order inside a class.
// Classes are octaves: fine enough that the sub-groups of a wavefront get items of similar
// length, coarse enough that a class is a dense sweep over the rows, so that rows launched
// together are neighbours and share sources (measured on the 114M-edge graph: quarter-octave
// classes cost 5 % at d = 128 and 512, and gain 1-3 % at d = 16).
static int length_class(int32_t cnt) {
    if (cnt <= 1) return cnt;
    return 32 - __builtin_clz((unsigned)cnt);
}

// Schedule of one gather launch over rows [row_begin, row_end) of `c`.
//
// One item per row; rows beyond `block_max` entries are cut into pieces that write partial
// rows, folded by a second launch.  Which items get a whole workgroup and which a single
// sub-group of lanes is decided at launch time (see long_items()).
//
// Source partitioning.  MI355X has 8 XCDs with a private 4 MB L2 each, and workgroups are
// handed to XCDs round-robin, so the workgroups b of one residue mod 8 share an XCD.  When the
// gathered matrix is much larger than one L2, every row of at least `part_min` entries is cut by
// the class of the SOURCE id (source_class) into 8 segments and segment k is scheduled on workgroups with b mod 8 == k:
// each L2 then only ever sees one eighth of the source rows, which raises its hit rate.
// `dcol` (a copy of c.col) is reordered inside such rows so that a segment is contiguous.
// The segments write partial rows that the fold launch adds up.  Items of unpartitioned rows
// are dealt round-robin to the 8 lists.
// The class (0..7) of a source row: which partition, and so which XCD's L2, reads it.  Runs of
// 2^shift consecutive ids share a class and the run number is folded three bits at a time, so that
// no address bit of a row is the same for all rows of a class.  (With the class taken from the low
// bits of the id, all rows one XCD reads agree in address bits 9..11 when a row has 512 bytes;
// measured on MI355X, such a launch is 5 % slower or faster depending on the parity of class minus
// XCD number, and 15 % slower at 64-byte rows, where two classes also share every cache line.)
// shift < 0 selects that old rule, for comparison.
static inline int source_class(int32_t id, int shift) {
    const uint32_t u = (uint32_t)id;
    if (shift < 0) return (int)(u & 7u);
    const uint32_t w = u >> shift;
    return (int)((w ^ (w >> 3) ^ (w >> 6) ^ (w >> 9) ^ (w >> 12) ^ (w >> 15) ^ (w >> 18) ^ (w >> 21) ^ (w >> 24)) & 7u);
}

void build_plan(const Csr &c, std::vector<int32_t> &dcol, int64_t row_begin, int64_t row_end, Plan &p,
                bool partition, int64_t split) {
    const int class_shift = (int)std::min<int64_t>(env_i64("HAG_PART_CLASS_SHIFT", 5), 20);
    const int64_t block_max = env_i64("HAG_BLOCK_MAX", 2048);
    const int64_t part_min = env_i64("HAG_PART_MIN", 64);
    // cutting by source only pays when the rows long enough to be cut hold most of the entries;
    // otherwise keep one list, which also keeps neighbouring rows on neighbouring workgroups
    if (partition) {
        int64_t total = c.ptr[row_end] - c.ptr[row_begin], in_long = 0, n_long = 0;
        for (int64_t r = row_begin; r < row_end; ++r) {
            int64_t cnt = c.ptr[r + 1] - c.ptr[r];
            if (cnt >= part_min) { in_long += cnt; ++n_long; }
        }
        // ... and are long enough on average that an eighth of a row is still worth a partial row
        partition = total > 0 && in_long * 100 >= total * env_i64("HAG_PART_SHARE_PCT", 30) &&
                    in_long >= n_long * env_i64("HAG_PART_MEAN_MIN", 128);
    }
    const int np = partition ? kPartitions : 1;
    std::vector<std::vector<Item>> lists(np);
    p.items.clear();
    p.combine.clear();
    p.n_slots = 0;
    p.np = np;
    std::vector<int32_t> slot_row;                        // output row of every partial slot
    auto cut = [&](int part, int64_t beg, int64_t cnt, bool partial, int64_t row) {
        // appends the items of one contiguous run of entries; returns nothing, bumps n_slots
        if (!partial && cnt <= block_max) {
            lists[part].push_back(Item{beg, (int32_t)cnt, (int32_t)row});
            return;
        }
        int64_t pieces = std::max<int64_t>(1, (cnt + block_max - 1) / block_max);
        int64_t per = (cnt + pieces - 1) / pieces;
        for (int64_t k = 0; k < pieces; ++k) {
            int64_t b0 = beg + k * per, b1 = std::min(beg + cnt, b0 + per);
            lists[part].push_back(Item{b0, (int32_t)(b1 - b0), (int32_t)~(p.n_slots++)});
            slot_row.push_back((int32_t)row);
        }
    };
    if (np > 1) {
        // reorder the rows that are cut by source: (class, id); rows are independent
        const int64_t chunk = 256, chunks = (row_end - row_begin + chunk - 1) / chunk;
        parallel_for(chunks, host_threads(), [&](int64_t ci, unsigned) {
            const int64_t r0 = row_begin + ci * chunk, r1 = std::min(row_end, r0 + chunk);
            for (int64_t r = r0; r < r1; ++r) {
                const int64_t beg = c.ptr[r], cnt = c.ptr[r + 1] - beg;
                if (cnt < part_min) continue;
                int32_t *row = dcol.data() + beg;
                std::sort(row, row + cnt, [class_shift](int32_t x, int32_t y) {
                    int px = source_class(x, class_shift), py = source_class(y, class_shift);
                    return px != py ? px < py : x < y;
                });
            }
        });
    }
    int rr = 0, rr_run = 0;     // whole rows go to the lists in runs of 64, which keeps neighbours together
    auto next_list = [&] { if (++rr_run == 64) { rr_run = 0; rr = (rr + 1) % np; } };
    for (int64_t r = row_begin; r < row_end; ++r) {
        int64_t beg = c.ptr[r], cnt = c.ptr[r + 1] - beg;
        if (np > 1 && cnt >= part_min) {
            const int32_t *row = dcol.data() + beg;
            int64_t first_slot = p.n_slots, i = 0;
            while (i < cnt) {
                int part = source_class(row[i], class_shift);
                int64_t j = i;
                while (j < cnt && source_class(row[j], class_shift) == part) ++j;
                cut(part, beg + i, j - i, true, r);
                i = j;
            }
            p.combine.push_back(Item{first_slot, (int32_t)(p.n_slots - first_slot), (int32_t)r});
        } else if (cnt > block_max) {
            int64_t first_slot = p.n_slots;
            cut(rr, beg, cnt, true, r);
            next_list();
            p.combine.push_back(Item{first_slot, (int32_t)(p.n_slots - first_slot), (int32_t)r});
        } else {
            cut(rr, beg, cnt, false, r);
            next_list();
        }
    }
    if (np > 1) {
        // even out the lists: move whole-row items from long lists to short ones (their source
        // ids are mixed anyway), so that every XCD gets about the same number of entries
        std::vector<int64_t> load(np, 0);
        int64_t total = 0;
        for (int k = 0; k < np; ++k) for (const Item &it : lists[k]) load[k] += it.cnt + 8;
        for (int k = 0; k < np; ++k) total += load[k];
        int64_t target = total / np;
        std::vector<Item> pool;
        for (int k = 0; k < np; ++k) {
            auto &l = lists[k];
            for (size_t i = l.size(); i-- > 0 && load[k] > target;)
                if (l[i].row >= 0) { load[k] -= l[i].cnt + 8; pool.push_back(l[i]); l.erase(l.begin() + i); }
        }
        for (const Item &it : pool) {
            int k = (int)(std::min_element(load.begin(), load.end()) - load.begin());
            lists[k].push_back(it);
            load[k] += it.cnt + 8;
        }
    }
    // entries are ascending inside an item (inside each source segment of a cut row), so ids >= split
    // come last: mark the items that read rows an earlier phase of the pass produces
    for (auto &l : lists)
        for (Item &it : l)
            if (it.cnt > 0 && dcol[(size_t)(it.beg + it.cnt - 1)] >= split) it.beg |= kItemDependsBit;
    // Order inside a partition: by length class, longest first, rows in their given order inside a
    // class.  With `bucket_rows` > 0 the short items (fewer than 128 entries, the bulk of a large
    // graph once its rows are cut by source) are ordered by (row / bucket_rows, class) instead: a
    // bucket of neighbouring rows is then swept once, all its lengths together, instead of once per
    // length class, so the sources that neighbouring rows share are fetched into L2 once.
    // (measured on the 114M-edge graph, d = 128, forward + backward: 5.74 -> 5.58 ms with the HAG,
    // 6.05 -> 5.92 ms without, for buckets of 2048 to 8192 rows; 32768: 5.61 / 5.98.)  Only for
    // plans cut by source: elsewhere rows are short and the length classes keep wavefronts balanced.
    const int64_t bucket_rows = np > 1 ? env_i64("HAG_BUCKET_ROWS", 4096) : 0;
    constexpr int kShortClass = 7;                        // lengths 64..127
    auto true_row = [&](const Item &it) -> int64_t { return it.row >= 0 ? it.row : slot_row[(size_t)~it.row]; };
    auto before = [&](const Item &x, const Item &y) {
        const int cx = length_class(x.cnt), cy = length_class(y.cnt);
        const bool sx = bucket_rows > 0 && cx <= kShortClass, sy = bucket_rows > 0 && cy <= kShortClass;
        if (sx != sy) return !sx;                         // long classes first
        if (sx) {
            const int64_t bx = true_row(x) / bucket_rows, by = true_row(y) / bucket_rows;
            if (bx != by) return bx < by;
        }
        return cx > cy;
    };
    p.min_block_class = bucket_rows > 0 ? kShortClass : 0;
    p.slot_row = slot_row;
    p.part_begin.assign(np + 1, 0);
    for (int k = 0; k < np; ++k) {
        std::stable_sort(lists[k].begin(), lists[k].end(), before);
        p.items.insert(p.items.end(), lists[k].begin(), lists[k].end());
        p.part_begin[k + 1] = (int64_t)p.items.size();
    }
}

// Number of leading items of partition k whose length class exceeds that of `threshold` entries.
int64_t long_items(const Plan &p, int k, int64_t threshold) {
    const int cls = std::max(length_class((int32_t)std::min<int64_t>(threshold, INT32_MAX)), p.min_block_class);
    auto b = p.items.begin() + p.part_begin[k], e = p.items.begin() + p.part_begin[k + 1];
    auto it = std::partition_point(b, e, [cls](const Item &x) { return length_class(x.cnt) > cls; });
    return (int64_t)(it - b);
}

// ------------------------------------------------------------------------------------------
// finalisation: levels, level-ordered forward form, transposes, schedules, statistics
// ------------------------------------------------------------------------------------------
// Detect a batch of small graphs: the node ids split into many small contiguous ranges that no
// edge crosses.  Aggregation nodes never cross components (their inputs
// co-occur in some list, hence lie in one component).  Fills h->comp or leaves it disabled.
static void build_components(hag_handle *h) {
    Components &c = h->comp;
    c = Components{};
    const int64_t n = h->n, a = h->a;
    if (env_i64("HAG_COMPONENT", 1) == 0 || n < 1024) return;
    std::vector<int32_t> parent(n);
    std::iota(parent.begin(), parent.end(), 0);
    auto find = [&](int32_t x) {
        while (parent[x] != x) { parent[x] = parent[parent[x]]; x = parent[x]; }
        return x;
    };
    for (int64_t v = 0; v < n; ++v)
        for (int64_t i = h->g.ptr[v]; i < h->g.ptr[v + 1]; ++i) {
            int32_t ra = find((int32_t)v), rb = find(h->g.col[i]);
            if (ra != rb) parent[std::max(ra, rb)] = std::min(ra, rb);   // root = smallest id
        }
    // blocks: the finest cut of 0..n-1 into contiguous ranges that no edge crosses (a block is one
    // connected component or several interleaved ones)
    std::vector<int32_t> last_of(n, -1);        // largest id of the component rooted at r
    for (int64_t v = 0; v < n; ++v) last_of[find((int32_t)v)] = (int32_t)v;
    std::vector<int32_t> comp_of(n + a);
    c.node_ptr.clear();
    int32_t block_end = -1;
    for (int64_t v = 0; v < n; ++v) {
        if (v > block_end) c.node_ptr.push_back((int32_t)v);
        block_end = std::max(block_end, last_of[find((int32_t)v)]);
        comp_of[v] = (int32_t)c.node_ptr.size() - 1;
    }
    c.node_ptr.push_back((int32_t)n);
    c.count = (int32_t)c.node_ptr.size() - 1;
    if (c.count < 64) return;                   // too few workgroups to fill the device
    // aggregation nodes per component, sorted by level (level order is already by level)
    std::vector<int32_t> agg_count(c.count, 0);
    for (int64_t i = 0; i < a; ++i) {
        comp_of[n + i] = comp_of[h->left[i]];
        if (comp_of[h->right[i]] != comp_of[n + i]) return;   // cannot happen for a valid HAG
        agg_count[comp_of[n + i]]++;
    }
    c.agg_ptr.assign(c.count + 1, 0);
    for (int32_t k = 0; k < c.count; ++k) {
        c.agg_ptr[k + 1] = c.agg_ptr[k] + agg_count[k];
        c.max_nodes = std::max(c.max_nodes, c.node_ptr[k + 1] - c.node_ptr[k]);
        c.max_agg = std::max(c.max_agg, agg_count[k]);
    }
    if (c.max_nodes + c.max_agg > 4096) return;  // local ids are 16 bit and must fit LDS anyway
    // local id of every unified id
    std::vector<int32_t> local(n + a), fill(c.agg_ptr.begin(), c.agg_ptr.end() - 1);
    // One stage per level, in the paper's two-input form (unless the lists are expanded, below)
    c.stage.resize(a);
    c.n_stages.assign(c.count, 0);
    if (h->levels > 63) return;                  // the kernel keeps one offset per level in LDS
    std::vector<int32_t> slot_of(a);             // component-major index of aggregation node i
    for (int64_t v = 0; v < n; ++v) local[v] = (int32_t)v - c.node_ptr[comp_of[v]];
    for (int32_t lv = 0; lv < h->levels; ++lv)
        for (int32_t i = h->level_ptr[lv]; i < h->level_ptr[lv + 1]; ++i) {
            int32_t k = comp_of[n + i];
            int32_t slot = fill[k]++;
            slot_of[i] = slot;
            local[n + i] = (c.node_ptr[k + 1] - c.node_ptr[k]) + (slot - c.agg_ptr[k]);
            c.stage[slot] = (uint8_t)(lv + 1);
            c.n_stages[k] = std::max(c.n_stages[k], (uint8_t)(lv + 1));
        }
    if (h->hf.col.size() + 2 * (size_t)a >= (size_t)INT32_MAX) return;
    // the two inputs of every aggregation node, and the consumers of every node (transposed HAG)
    Csr pairs, consumers;
    pairs.ptr.resize(a + 1);
    pairs.col.resize(2 * (size_t)a);
    for (int64_t i = 0; i <= a; ++i) pairs.ptr[i] = 2 * i;
    for (int64_t i = 0; i < a; ++i) { pairs.col[2 * i] = h->left[i]; pairs.col[2 * i + 1] = h->right[i]; }
    // Expanded form: every aggregation row as the sum of the original rows it covers
    // (Section 3.1: aggr(w) is the aggregate over cover(w)), so that all of them are computed
    // in one stage, and, transposed, every original row that aggregation nodes consume takes
    // the destination parts of all aggregation nodes above it.  Used when the covers are
    // small (a handful of nodes each), which removes every dependent stage but one.
    Csr cover;
    bool expanded = true;
    {
        const int64_t forced = env_i64("HAG_COMPONENT_EXPAND", -1);
        const size_t limit = forced == 1 ? (size_t)INT32_MAX / 2 : forced == 0 ? 0 : 4 * (size_t)a + 64;
        cover.ptr.assign(1, 0);
        for (int64_t i = 0; i < a && expanded; ++i) {
            for (int32_t u : {h->left[i], h->right[i]}) {
                if (u < n) {
                    cover.col.push_back(u);
                } else {
                    // u's cover is already complete and lies before the insertion point
                    const size_t b = (size_t)cover.ptr[u - n], e = (size_t)cover.ptr[u - n + 1];
                    cover.col.reserve(cover.col.size() + (e - b));
                    for (size_t t = b; t < e; ++t) cover.col.push_back(cover.col[t]);
                }
            }
            cover.ptr.push_back((int64_t)cover.col.size());
            if (cover.col.size() > limit) expanded = false;
        }
        if (a == 0) expanded = false;
    }
    if (expanded) {
        std::fill(c.stage.begin(), c.stage.end(), (uint8_t)1);
        for (int32_t k = 0; k < c.count; ++k) c.n_stages[k] = agg_count[k] > 0 ? 1 : 0;
    }
    c.expanded = expanded;
    // aggregation nodes above every original node (those whose cover holds it)
    Csr above;
    if (expanded) {
        above.ptr.assign(n + 1, 0);
        for (int32_t u : cover.col) above.ptr[u + 1]++;
        for (int64_t u = 0; u < n; ++u) above.ptr[u + 1] += above.ptr[u];
        above.col.resize(cover.col.size());
        std::vector<int64_t> at(above.ptr.begin(), above.ptr.end() - 1);
        for (int64_t i = 0; i < a; ++i)
            for (int64_t t = cover.ptr[i]; t < cover.ptr[i + 1]; ++t) above.col[at[cover.col[t]]++] = (int32_t)(n + i);
    }
    consumers.ptr.assign(n + a + 1, 0);
    for (int32_t x : h->hf.col) consumers.ptr[x + 1]++;
    for (int32_t x : pairs.col) consumers.ptr[x + 1]++;
    for (int64_t x = 0; x < n + a; ++x) consumers.ptr[x + 1] += consumers.ptr[x];
    consumers.col.resize((size_t)consumers.ptr[n + a]);
    {
        std::vector<int64_t> at(consumers.ptr.begin(), consumers.ptr.end() - 1);
        for (int64_t v = 0; v < n; ++v)
            for (int64_t i = h->hf.ptr[v]; i < h->hf.ptr[v + 1]; ++i) consumers.col[at[h->hf.col[i]]++] = (int32_t)v;
        for (int64_t i = 0; i < a; ++i) {
            consumers.col[at[h->left[i]]++] = (int32_t)(n + i);
            consumers.col[at[h->right[i]]++] = (int32_t)(n + i);
        }
    }
    // rows of src in the given order of rows, ids made local
    auto localise = [&](const Csr &src, const std::vector<int64_t> &rows, LocalLists &dst) {
        dst.ptr.assign(1, 0);
        dst.col.clear();
        for (int64_t r : rows) {
            for (int64_t i = src.ptr[r]; i < src.ptr[r + 1]; ++i) dst.col.push_back((uint16_t)local[src.col[i]]);
            dst.ptr.push_back((int32_t)dst.col.size());
        }
    };
    std::vector<int64_t> orig_rows(n), agg_rows(a), agg_rows_t(a);
    std::iota(orig_rows.begin(), orig_rows.end(), 0);
    for (int64_t i = 0; i < a; ++i) { agg_rows[slot_of[i]] = i; agg_rows_t[slot_of[i]] = n + i; }
    localise(h->hf, orig_rows, c.fwd);
    localise(expanded ? cover : pairs, agg_rows, c.fwd_agg);
    LocalLists bwd_orig;
    localise(consumers, orig_rows, bwd_orig);
    // consumers of an aggregation row: destinations first (they were filled in first), then
    // aggregation nodes; the two parts are used apart
    LocalLists bwd_agg_full;
    localise(consumers, agg_rows_t, bwd_agg_full);
    std::vector<int32_t> agg_mid((size_t)a);
    c.bwd_agg.ptr.assign(1, 0);
    c.bwd_agg.col.clear();
    for (int64_t slot = 0; slot < a; ++slot) {
        const int32_t k = comp_of[agg_rows_t[slot]], nv = c.node_ptr[k + 1] - c.node_ptr[k];
        int32_t m = bwd_agg_full.ptr[slot];
        while (m < bwd_agg_full.ptr[slot + 1] && bwd_agg_full.col[m] < nv) ++m;
        agg_mid[slot] = m;
        if (!expanded)
            c.bwd_agg.col.insert(c.bwd_agg.col.end(), bwd_agg_full.col.begin() + m,
                                 bwd_agg_full.col.begin() + bwd_agg_full.ptr[slot + 1]);
        c.bwd_agg.ptr.push_back((int32_t)c.bwd_agg.col.size());
    }
    localise(h->g, orig_rows, c.nfwd);
    localise(h->gt, orig_rows, c.nbwd);
    {
        // transposed pass: one item list per component over original and aggregation rows
        LocalLists &l = c.bwd_all;
        const int32_t off_agg = (int32_t)bwd_orig.col.size();
        l.col = bwd_orig.col;
        l.col.insert(l.col.end(), bwd_agg_full.col.begin(), bwd_agg_full.col.end());
        l.items.resize(2 * (size_t)(n + a));
        l.split.resize((size_t)c.count);
        struct Row { int32_t beg, len, row; };
        std::vector<Row> first, second;
        for (int32_t k = 0; k < c.count; ++k) {
            const int32_t v0 = c.node_ptr[k], nv = c.node_ptr[k + 1] - v0, a0 = c.agg_ptr[k], a1 = c.agg_ptr[k + 1];
            first.clear();
            second.clear();
            for (int32_t j = a0; j < a1; ++j)
                first.push_back({off_agg + bwd_agg_full.ptr[j], agg_mid[j] - bwd_agg_full.ptr[j], nv + (j - a0)});
            for (int32_t v = 0; v < nv; ++v) {
                const int32_t b = bwd_orig.ptr[v0 + v], e = bwd_orig.ptr[v0 + v + 1];
                const bool feeds_agg = e > b && bwd_orig.col[e - 1] >= nv;   // aggregation consumers come last
                if (feeds_agg && expanded) {
                    // destinations, then every aggregation node above v instead of the direct ones
                    const int32_t nb = (int32_t)l.col.size();
                    for (int32_t t = b; t < e && bwd_orig.col[t] < nv; ++t) l.col.push_back(bwd_orig.col[t]);
                    for (int64_t t = above.ptr[v0 + v]; t < above.ptr[v0 + v + 1]; ++t)
                        l.col.push_back((uint16_t)local[above.col[t]]);
                    second.push_back({nb, (int32_t)l.col.size() - nb, v});
                } else {
                    (feeds_agg ? second : first).push_back({b, e - b, v});
                }
            }
            auto longer = [](const Row &x, const Row &y) { return x.len > y.len; };
            std::stable_sort(first.begin(), first.end(), longer);
            std::stable_sort(second.begin(), second.end(), longer);
            l.split[k] = (int32_t)first.size();
            int32_t *o = l.items.data() + 2 * (size_t)(v0 + a0);
            for (const std::vector<Row> *part : {&first, &second})
                for (const Row &r : *part) { *o++ = r.beg; *o++ = r.len | (r.row << 16); }
        }
    }
    if (c.bwd_all.col.size() >= (size_t)INT32_MAX) return;
    for (LocalLists *l : {&c.fwd, &c.nfwd, &c.nbwd}) {
        l->items.resize(2 * (size_t)n);
        std::vector<int32_t> o((size_t)c.max_nodes);
        for (int32_t k = 0; k < c.count; ++k) {
            const int32_t v0 = c.node_ptr[k], nv = c.node_ptr[k + 1] - v0;
            auto len = [&](int32_t x) { return l->ptr[v0 + x + 1] - l->ptr[v0 + x]; };
            std::iota(o.begin(), o.begin() + nv, 0);
            std::stable_sort(o.begin(), o.begin() + nv, [&](int32_t x, int32_t y) { return len(x) > len(y); });
            for (int32_t i = 0; i < nv; ++i) {
                l->items[2 * (size_t)(v0 + i)] = l->ptr[v0 + o[i]];
                l->items[2 * (size_t)(v0 + i) + 1] = len(o[i]) | (o[i] << 16);   // both below 4096
            }
        }
    }
    for (int32_t k = 0; k < c.count; ++k) {
        int32_t a0 = c.agg_ptr[k], a1 = c.agg_ptr[k + 1];
        auto span = [&](const LocalLists &l, int32_t lo, int32_t hi) { return l.ptr[hi] - l.ptr[lo]; };
        c.max_entries_fwd = std::max(c.max_entries_fwd, span(c.fwd_agg, a0, a1));
        c.max_entries_bwd = std::max(c.max_entries_bwd, span(c.bwd_agg, a0, a1));
    }
    c.meta.resize(4 * (size_t)c.count);
    for (int32_t k = 0; k < c.count; ++k) {
        c.meta[4 * k + 0] = c.node_ptr[k];
        c.meta[4 * k + 1] = c.node_ptr[k + 1] - c.node_ptr[k];
        c.meta[4 * k + 2] = c.agg_ptr[k];
        c.meta[4 * k + 3] = (c.agg_ptr[k + 1] - c.agg_ptr[k]) | ((int32_t)c.n_stages[k] << 16);
    }
    c.enabled = true;
}

static int finalize_from_builder(hag_handle *h, Builder &b) {
    const int64_t n = b.n, a = b.a();
    h->n = n;
    h->a = a;
    h->e = (int64_t)h->g.col.size();
    h->m_left = b.m_left;
    h->m_right = b.m_right;
    h->m_red = b.m_red;
    {
        hag_knobs &k = h->knobs;
        k.sub_max = env_i64("HAG_SUB_MAX", 0);
        k.offset64 = env_i64("HAG_OFFSET64", 0) != 0;
        const int64_t pad = env_i64("HAG_COMPONENT_PAD", 0);
        k.component_pad = (int32_t)((pad < 0 ? 0 : pad > 64 ? 64 : pad) & ~(int64_t)3);
        k.stream_output = env_i64("HAG_STREAM_OUTPUT", 0) != 0;
        k.component_parts = env_i64("HAG_COMPONENT_PARTS", 0);
        k.component_extra_lds = std::max<int64_t>(env_i64("HAG_COMPONENT_EXTRA_LDS", 0), 0) & ~(int64_t)15;
        k.part_shift = (int32_t)(env_i64("HAG_PART_SHIFT", 0) & 7);
        k.fuse_max_items = env_i64("HAG_FUSE_MAX_ITEMS", 0);   // off: measured slower than one launch per stage
        k.spin_limit = env_i64("HAG_SPIN_LIMIT", 1 << 18);
    }
    // depth(original) = 0, depth(w) = 1 + max over its inputs; creation order is topological
    std::vector<int32_t> order(a);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return b.depth[x] < b.depth[y]; });
    std::vector<int32_t> newid(a);
    for (int64_t i = 0; i < a; ++i) newid[order[i]] = (int32_t)(n + i);
    auto remap = [&](int32_t x) { return x < n ? x : newid[x - n]; };
    h->levels = a ? b.depth[order[a - 1]] : 0;
    h->left.resize(a);
    h->right.resize(a);
    h->level_ptr.assign(h->levels + 1, 0);
    for (int64_t i = 0; i < a; ++i) {
        int32_t c = order[i];
        int32_t l = remap(b.m_left[c]), r = remap(b.m_right[c]);
        h->left[i] = std::min(l, r);
        h->right[i] = std::max(l, r);
        h->level_ptr[b.depth[c]] = (int32_t)(i + 1);
    }
    for (int32_t l = 1; l <= h->levels; ++l) h->level_ptr[l] = std::max(h->level_ptr[l], h->level_ptr[l - 1]);
    // Nhat_v, level-order ids, ascending
    h->hf.ptr.assign(n + 1, 0);
    for (int64_t v = 0; v < n; ++v) h->hf.ptr[v + 1] = h->hf.ptr[v] + b.len[v];
    h->hf.col.resize((size_t)h->hf.ptr[n]);
    for (int64_t v = 0; v < n; ++v) {
        int32_t *dst = h->hf.col.data() + h->hf.ptr[v];
        const int32_t *src = b.nb.data() + h->g.ptr[v];
        for (int32_t i = 0; i < b.len[v]; ++i) dst[i] = remap(src[i]);
        std::sort(dst, dst + b.len[v]);
    }
    // Stages: consecutive levels executed by one launch.  A node of a stage is expressed over
    // nodes of earlier stages (and originals) by expanding its inputs that lie in the same
    // stage, which by cover()'s definition (Section 3.1) leaves aggr(w) unchanged.  A level
    // joins the running stage while the extra row reads this causes stay small against the
    // cost of one more launch; a stage of a single level keeps the two-input form.
    {
        const int64_t extra_rows = env_i64("HAG_STAGE_EXTRA_ROWS", 32768);
        const double extra_frac = 0.25;
        const int64_t max_expand = 256;
        Csr &he = h->he;
        he.ptr.assign(1, 0);
        he.col.clear();
        h->stage_ptr.assign(1, 0);
        std::vector<int32_t> node_level(a);
        for (int32_t l = 1; l <= h->levels; ++l)
            for (int32_t i = h->level_ptr[l - 1]; i < h->level_ptr[l]; ++i) node_level[i] = l;
        int32_t base_level = 0;              // levels <= base_level belong to closed stages
        int64_t stage_reads = 0, stage_nodes = 0;
        std::vector<int32_t> tmp;
        auto expand_level = [&](int32_t l, std::vector<int64_t> &ptr_out, std::vector<int32_t> &col_out) {
            int64_t worst = 0;
            ptr_out.clear();
            col_out.clear();
            for (int32_t i = h->level_ptr[l - 1]; i < h->level_ptr[l]; ++i) {
                size_t before = col_out.size();
                for (int32_t u : {h->left[i], h->right[i]}) {
                    if (u >= n && node_level[u - n] > base_level)
                        col_out.insert(col_out.end(), he.col.begin() + he.ptr[u - n], he.col.begin() + he.ptr[u - n + 1]);
                    else
                        col_out.push_back(u);
                }
                std::sort(col_out.begin() + before, col_out.end());
                worst = std::max<int64_t>(worst, (int64_t)(col_out.size() - before));
                ptr_out.push_back((int64_t)col_out.size());
            }
            return worst;
        };
        std::vector<int64_t> lp;
        std::vector<int32_t> lc;
        for (int32_t l = 1; l <= h->levels; ++l) {
            int64_t nodes = h->level_ptr[l] - h->level_ptr[l - 1];
            int64_t worst = expand_level(l, lp, lc);
            bool first = (l == base_level + 1);
            int64_t reads = stage_reads + (int64_t)lc.size(), cnt = stage_nodes + nodes;
            bool ok = first || (worst <= max_expand && reads <= 2 * cnt + extra_rows + (int64_t)(extra_frac * 2 * cnt));
            if (!ok) {                       // close the stage before this level and start a new one
                h->stage_ptr.push_back(h->level_ptr[l - 1]);
                base_level = l - 1;
                stage_reads = stage_nodes = 0;
                expand_level(l, lp, lc);
            }
            int64_t off = (int64_t)he.col.size();
            he.col.insert(he.col.end(), lc.begin(), lc.end());
            for (int64_t q : lp) he.ptr.push_back(off + q);
            stage_reads += (int64_t)lc.size();
            stage_nodes += nodes;
        }
        if (a > 0) h->stage_ptr.push_back((int32_t)a);
        h->stages = (int32_t)h->stage_ptr.size() - 1;
        h->stage_single_level.assign(h->stages, 0);
        for (int32_t st = 0; st < h->stages; ++st)
            h->stage_single_level[st] = node_level[h->stage_ptr[st]] == node_level[h->stage_ptr[st + 1] - 1];
    }
    // transposed HAG (in its staged form): consumers of every source
    {
        Csr all;  // rows: destinations 0..n-1 then aggregation nodes; cols: their (expanded) in-neighbours
        all.ptr.resize(n + a + 1);
        all.col.reserve(h->hf.col.size() + h->he.col.size());
        all.col = h->hf.col;
        for (int64_t v = 0; v <= n; ++v) all.ptr[v] = h->hf.ptr[v];
        all.col.insert(all.col.end(), h->he.col.begin(), h->he.col.end());
        for (int64_t i = 0; i < a; ++i) all.ptr[n + i + 1] = h->hf.ptr[n] + h->he.ptr[i + 1];
        transpose(all, n + a, h->ht);
    }
    transpose(h->g, n, h->gt);
    h->inv_deg.resize(n);
    h->inv_deg1.resize(n);
    for (int64_t v = 0; v < n; ++v) {
        int64_t d = h->g.ptr[v + 1] - h->g.ptr[v];
        h->inv_deg[v] = 1.0f / (float)std::max<int64_t>(d, 1);
        h->inv_deg1[v] = 1.0f / (float)(d + 1);
    }
    // schedules
    const bool part = env_i64("HAG_PARTITION", 1) != 0 && (n + a) >= env_i64("HAG_PARTITION_MIN_ROWS", 16384);
    h->hf_dcol = h->hf.col;
    h->ht_dcol = h->ht.col;
    h->g_dcol = h->g.col;
    h->gt_dcol = h->gt.col;
    std::vector<int32_t> he_dcol = h->he.col;   // never partitioned: stays as it is
    build_plan(h->hf, h->hf_dcol, 0, n, h->p_fwd, part, n);
    h->p_fwd_stage.assign(h->stages, Plan{});
    h->p_bwd_stage.assign(h->stages, Plan{});
    for (int32_t st = 0; st < h->stages; ++st) {
        // (a single-level stage runs as level_kernel when launched on its own; the one-launch
        // schedule takes its rows as gather items like any other stage)
        build_plan(h->he, he_dcol, h->stage_ptr[st], h->stage_ptr[st + 1], h->p_fwd_stage[st], false, n);
        for (Item &it : h->p_fwd_stage[st].items) if (it.row >= 0) it.row += (int32_t)n;   // unified ids
        for (Item &it : h->p_fwd_stage[st].combine) it.row += (int32_t)n;
        build_plan(h->ht, h->ht_dcol, n + h->stage_ptr[st], n + h->stage_ptr[st + 1], h->p_bwd_stage[st], part, n);
    }
    build_plan(h->ht, h->ht_dcol, 0, n, h->p_bwd_src, part, n);
    build_plan(h->g, h->g_dcol, 0, n, h->p_naive_fwd, part, INT64_MAX);
    build_plan(h->gt, h->gt_dcol, 0, n, h->p_naive_bwd, part, INT64_MAX);
    h->max_slots = std::max({h->p_fwd.n_slots, h->p_bwd_src.n_slots, h->p_naive_fwd.n_slots, h->p_naive_bwd.n_slots});
    for (auto &p : h->p_bwd_stage) h->max_slots = std::max(h->max_slots, p.n_slots);
    for (auto &p : h->p_fwd_stage) h->max_slots = std::max(h->max_slots, p.n_slots);
    build_components(h);
    // statistics (Section 4.1: k in-neighbours cost k-1 binary aggregations; Section 5.4: one
    // row transfer per aggregated neighbour)
    hag_stats_t &s = h->st;
    s = hag_stats_t{};
    s.n = n; s.e = h->e; s.a = a; s.levels = h->levels; s.stages = h->stages;
    s.h = (int64_t)h->hf.col.size();
    s.e_hag = s.h + 2 * a;
    for (int64_t v = 0; v < n; ++v) {
        int64_t d = h->g.ptr[v + 1] - h->g.ptr[v], dh = h->hf.ptr[v + 1] - h->hf.ptr[v];
        s.aggr_naive += std::max<int64_t>(d - 1, 0);
        s.aggr_hag += std::max<int64_t>(dh - 1, 0);
        s.max_degree = std::max(s.max_degree, d);
        s.max_hag_degree = std::max(s.max_hag_degree, dh);
    }
    s.aggr_hag += a;
    s.xfer_naive = s.e;
    s.xfer_hag = s.e_hag;
    s.components = h->comp.enabled ? h->comp.count : 0;
    return HAG_OK;
}

static int replay(hag_handle *h, int64_t n_merges, const int32_t *left, const int32_t *right) {
    Builder b;
    b.init(h->g, false, host_threads());
    for (int64_t i = 0; i < n_merges; ++i) {
        int64_t lim = b.n + i;
        if (left[i] < 0 || right[i] < 0 || left[i] >= lim || right[i] >= lim)
            return fail(HAG_EINVAL, "merge " + std::to_string(i) + " refers to a node that does not exist yet");
        if (left[i] == right[i]) return fail(HAG_EINVAL, "merge " + std::to_string(i) + " has equal inputs");
        if (b.apply_merge(left[i], right[i]) < 1)
            return fail(HAG_EINVAL, "merge " + std::to_string(i) + " is used by no list");
    }
    return finalize_from_builder(h, b);
}

}  // namespace hag

using namespace hag;

extern "C" {

const char *hag_last_error(void) { return g_err.c_str(); }

int hag_search(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t capacity, uint32_t flags,
               int32_t max_depth, hag_t **out) {
    if (!out) return fail(HAG_EINVAL, "out is NULL");
    *out = nullptr;
    if (capacity < 0) return fail(HAG_EINVAL, "capacity < 0");
    if (max_depth < 0) return fail(HAG_EINVAL, "max_depth < 0");
    if (n + capacity >= (int64_t)INT32_MAX) return fail(HAG_EINVAL, "n + capacity must be below 2^31");
    try {
        std::unique_ptr<hag_handle> h(new hag_handle);
        int rc = load_graph(n, rowptr, col, flags, h->g);
        if (rc) return rc;
        Searcher s;
        s.capacity = capacity;
        s.max_depth = max_depth;
        s.b.init(h->g, true, host_threads());
        if (capacity > 0 && (flags & HAG_SEARCH_DEVICE) && n > 0) {
            const Builder &b = s.b;
            CounterInit in{n, (int64_t)b.nb.size(), capacity, h->g.ptr.data(), b.nb.data(), b.len.data(),
                           b.norig.data(), b.prio.data(), b.gt.ptr.data(), b.gt.col.data(), b.olen.data()};
            s.dev = counter_create(in, s.dev_err);
            if (!s.dev) return fail(HAG_EHIP, s.dev_err);
        }
        // released on every way out of this scope, exceptions included
        std::unique_ptr<DeviceCounter, void (*)(DeviceCounter *)> dev_guard(s.dev, counter_destroy);
        const bool ok = capacity > 0 ? s.run() : true;
        dev_guard.reset();
        s.dev = nullptr;
        if (!ok) return fail(HAG_EHIP, s.dev_err);
        rc = finalize_from_builder(h.get(), s.b);
        if (rc) return rc;
        *out = h.release();
        return HAG_OK;
    } catch (const std::bad_alloc &) {
        return fail(HAG_ENOMEM, "out of host memory");
    } catch (const std::exception &ex) {   // e.g. a worker thread could not be started
        return fail(HAG_ENOMEM, std::string("host resources exhausted: ") + ex.what());
    }
}

int hag_search_batched(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t n_graphs,
                       const int64_t *graph_ptr, double capacity_fraction, uint32_t flags, int32_t max_depth,
                       hag_t **out) {
    if (!out) return fail(HAG_EINVAL, "out is NULL");
    *out = nullptr;
    if (n_graphs < 0 || !graph_ptr) return fail(HAG_EINVAL, "bad graph_ptr");
    if (capacity_fraction < 0) return fail(HAG_EINVAL, "capacity_fraction < 0");
    if (max_depth < 0) return fail(HAG_EINVAL, "max_depth < 0");
    if (graph_ptr[0] != 0 || graph_ptr[n_graphs] != n) return fail(HAG_EINVAL, "graph_ptr must span 0..n");
    for (int64_t gi = 0; gi < n_graphs; ++gi)
        if (graph_ptr[gi + 1] < graph_ptr[gi]) return fail(HAG_EINVAL, "graph_ptr is not monotone");
    try {
        std::unique_ptr<hag_handle> h(new hag_handle);
        int rc = load_graph(n, rowptr, col, flags, h->g);
        if (rc) return rc;
        for (int64_t gi = 0; gi < n_graphs; ++gi)
            for (int64_t v = graph_ptr[gi]; v < graph_ptr[gi + 1]; ++v)
                for (int64_t i = h->g.ptr[v]; i < h->g.ptr[v + 1]; ++i)
                    if (h->g.col[i] < graph_ptr[gi] || h->g.col[i] >= graph_ptr[gi + 1])
                        return fail(HAG_EINVAL, "edge crosses graphs at row " + std::to_string(v));
        // search every graph on its own (local ids), in parallel
        struct Local { std::vector<int32_t> l, r; };
        std::vector<Local> res(n_graphs);
        parallel_for(n_graphs, host_threads(), [&](int64_t gi, unsigned) {
            int64_t v0 = graph_ptr[gi], nv = graph_ptr[gi + 1] - v0;
            Csr sub;
            sub.ptr.resize(nv + 1);
            for (int64_t v = 0; v <= nv; ++v) sub.ptr[v] = h->g.ptr[v0 + v] - h->g.ptr[v0];
            sub.col.resize((size_t)sub.ptr[nv]);
            for (size_t i = 0; i < sub.col.size(); ++i) sub.col[i] = (int32_t)(h->g.col[h->g.ptr[v0] + i] - v0);
            Searcher s;
            s.capacity = (int64_t)std::floor(capacity_fraction * (double)nv);
            s.max_depth = max_depth;
            s.single_thread = true;
            s.b.init(sub, true);
            if (s.capacity > 0) s.run();
            res[gi].l = s.b.m_left;
            res[gi].r = s.b.m_right;
        });
        // concatenate: local aggregation node j of graph gi becomes n + offset[gi] + j
        std::vector<int32_t> left, right;
        int64_t off = 0;
        for (int64_t gi = 0; gi < n_graphs; ++gi) {
            int64_t v0 = graph_ptr[gi], nv = graph_ptr[gi + 1] - v0;
            auto map = [&](int32_t x) { return (int32_t)(x < nv ? v0 + x : n + off + (x - nv)); };
            for (size_t j = 0; j < res[gi].l.size(); ++j) {
                left.push_back(map(res[gi].l[j]));
                right.push_back(map(res[gi].r[j]));
            }
            off += (int64_t)res[gi].l.size();
        }
        rc = replay(h.get(), (int64_t)left.size(), left.data(), right.data());
        if (rc) return rc;
        *out = h.release();
        return HAG_OK;
    } catch (const std::bad_alloc &) {
        return fail(HAG_ENOMEM, "out of host memory");
    } catch (const std::exception &ex) {   // e.g. a worker thread could not be started
        return fail(HAG_ENOMEM, std::string("host resources exhausted: ") + ex.what());
    }
}

int hag_from_merges(int64_t n, const int64_t *rowptr, const int32_t *col, int64_t n_merges, const int32_t *left,
                    const int32_t *right, uint32_t flags, hag_t **out) {
    if (!out) return fail(HAG_EINVAL, "out is NULL");
    *out = nullptr;
    if (n_merges < 0 || (n_merges > 0 && (!left || !right))) return fail(HAG_EINVAL, "bad merge list");
    if (n + n_merges >= (int64_t)INT32_MAX) return fail(HAG_EINVAL, "n + n_merges must be below 2^31");
    try {
        std::unique_ptr<hag_handle> h(new hag_handle);
        int rc = load_graph(n, rowptr, col, flags, h->g);
        if (rc) return rc;
        rc = replay(h.get(), n_merges, left, right);
        if (rc) return rc;
        *out = h.release();
        return HAG_OK;
    } catch (const std::bad_alloc &) {
        return fail(HAG_ENOMEM, "out of host memory");
    } catch (const std::exception &ex) {   // e.g. a worker thread could not be started
        return fail(HAG_ENOMEM, std::string("host resources exhausted: ") + ex.what());
    }
}

int hag_prefix(const hag_t *src, int64_t n_merges, hag_t **out) {
    if (!out) return fail(HAG_EINVAL, "out is NULL");
    *out = nullptr;
    if (!src) return fail(HAG_EINVAL, "handle is NULL");
    if (n_merges < 0 || n_merges > src->a) return fail(HAG_EINVAL, "n_merges out of range");
    try {
        std::unique_ptr<hag_handle> h(new hag_handle);
        h->g = src->g;
        int rc = replay(h.get(), n_merges, src->m_left.data(), src->m_right.data());
        if (rc) return rc;
        *out = h.release();
        return HAG_OK;
    } catch (const std::bad_alloc &) {
        return fail(HAG_ENOMEM, "out of host memory");
    } catch (const std::exception &ex) {   // e.g. a worker thread could not be started
        return fail(HAG_ENOMEM, std::string("host resources exhausted: ") + ex.what());
    }
}

void hag_free(hag_t *h) {
    if (!h) return;
    free_device(h);
    delete h;
}

int hag_stats(const hag_t *h, hag_stats_t *out) {
    if (!h || !out) return fail(HAG_EINVAL, "NULL argument");
    *out = h->st;
    return HAG_OK;
}

int hag_get_merges(const hag_t *h, int64_t *n_merges, const int32_t **left, const int32_t **right,
                   const int32_t **redundancy) {
    if (!h) return fail(HAG_EINVAL, "handle is NULL");
    if (n_merges) *n_merges = h->a;
    if (left) *left = h->m_left.data();
    if (right) *right = h->m_right.data();
    if (redundancy) *redundancy = h->m_red.data();
    return HAG_OK;
}

int hag_get_forward(const hag_t *h, const int32_t **agg_left, const int32_t **agg_right, const int32_t **level_ptr,
                    int32_t *n_levels, const int64_t **hrowptr, const int32_t **hcol) {
    if (!h) return fail(HAG_EINVAL, "handle is NULL");
    if (agg_left) *agg_left = h->left.data();
    if (agg_right) *agg_right = h->right.data();
    if (level_ptr) *level_ptr = h->level_ptr.data();
    if (n_levels) *n_levels = h->levels;
    if (hrowptr) *hrowptr = h->hf.ptr.data();
    if (hcol) *hcol = h->hf.col.data();
    return HAG_OK;
}

int64_t hag_algorithmic_bytes(const hag_t *h, int which, hag_op_t op, int64_t d) {
    if (!h || d <= 0) return -1;
    const int64_t n = h->n, a = h->a, row = 4 * d;
    bool naive = which >= 2, bwd = which & 1;
    int64_t edges = naive ? h->e : h->st.e_hag;   // one row read per edge
    int64_t rows_out = naive ? n : n + a;         // one row write per produced node
    int64_t ptrs = bwd && !naive ? n + a + 1 : n + 1;
    if (op == HAG_MAX && bwd)                     // argmax read, gy read, gx cleared, gx updated
        return 4 * row * n;
    int64_t bytes = row * edges + row * rows_out + 4 * edges + 8 * ptrs;
    if (op == HAG_MAX) bytes += row * rows_out;   // winning ids written beside the values
    if (op == HAG_GCN) bytes += row * n;          // the node's own row
    return bytes;
}

}  // extern "C"

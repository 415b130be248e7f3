// Host-side CBM builder: binary CSR -> compression tree -> delta lists -> GPU work lists.
//
// Follows Section 2 of the paper (extended Hamming-distance graph with a virtual
// null row, spanning tree rooted at the virtual vertex, delta lists per tree
// edge, Eq. (2)) and the alpha rule of Section 2.2 ("Edge Pruning"), but never
// materialises the all-pairs distance graph: an edge (y,x) can beat the virtual
// edge of x only if  w(y,x) = nnz(a_x) + nnz(a_y) - 2|a_x n a_y| < nnz(a_x),
// i.e. |a_x n a_y| > nnz(a_y)/2, so only rows sharing a column are candidates.
// The tree is grown Prim-style from the virtual vertex with a cap on depth, then
// cut into vertical paths (one GPU work item each) whose length is chosen by a
// small latency/bandwidth cost model of the kernels.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <queue>
#include <thread>

#include "cbm_internal.h"

namespace {

constexpr int32_t kDefaultMaxDepth = 16;
constexpr int32_t kDefaultHubCap = 512;
constexpr int32_t kDefaultMaxCand = 8;
constexpr int64_t kLocalityMinEntries = 24;  // mean entries per work item from which a round is scheduled by locality
constexpr double kLocalityEntries = 230.0;   // such a round's bandwidth grows by 1/230 of the base per entry in a work item
constexpr int64_t kBundleMinEntries = 96;   // mean entries per work item from which a round's paths are bundled
constexpr int64_t kShareSortItems = 8192;   // work items in an XCD's share of a round up to which they run strictly longest first
constexpr long kShareBucket = 32;           // ... beyond that: by length in buckets of this many entries, locality order inside
constexpr int64_t kLongSingleRow = 64;      // mean entries of a round of single rows from which the sweep kernel may take it (narrow X)
constexpr int64_t kBundleMinItems = 256;    // ... and the work items it must have: a round of a few long paths gains nothing from sweeps in step
constexpr int64_t kDeviceSearchMinRows = 65536;  // from here on a handle bound for a GPU searches its candidates there
constexpr int64_t kSampleMinRows = 65536;  // automatic mode samples the compressibility of matrices this large first
constexpr int32_t kSplitLenDefault = 512;  // most delta entries in one segment of a split row
constexpr int32_t kSplitMinDefault = 128;  // rows with more delta entries than this are split
constexpr int32_t kPhasesDefault = 4;      // sub-ranges of an XCD's column range, for rows of >= kFineMin entries
constexpr int32_t kFineMinDefault = 1024;

// Cost model of one product (reference: k = 128, i.e. 512-byte rows).  A launch costs a fixed
// overhead plus the larger of its bandwidth time and the latency of its longest work item: a work
// item walks its entries in batches of 8 row loads, so an entry costs about one eighth of a memory
// round trip.  Measured on MI355X: ~7 us per dependent launch, ~0.2 us per entry, ~6 TB/s.
constexpr double kLaunchUs = 7.0;
constexpr double kEntryUs = 0.2;
constexpr double kBytesPerUs = 6.0e6;
constexpr double kRefRowBytes = 512.0;
constexpr int64_t kPathChoices[] = {16, 32, 64, 128, 256};

long env_or(const char* name, long dflt) {
    const char* v = std::getenv(name);
    return v ? std::atol(v) : dflt;
}
// a tuning knob from the environment, held to the range the work lists can encode
long env_clamped(const char* name, long dflt, long lo, long hi) { return std::min(hi, std::max(lo, env_or(name, dflt))); }

template <class F>
void parallel_chunks(int nthreads, int64_t total, int64_t chunk, F&& fn) {
    if (total <= 0) return;
    std::atomic<int64_t> next{0};
    auto worker = [&](int tid) {
        for (;;) {
            int64_t b = next.fetch_add(chunk);
            if (b >= total) break;
            fn(b, std::min(total, b + chunk), tid);
        }
    };
    int nt = (int)std::max<int64_t>(1, std::min<int64_t>(nthreads, (total + chunk - 1) / chunk));
    if (nt == 1) {
        worker(0);
        return;
    }
    std::vector<std::thread> pool;
    pool.reserve(nt);
    for (int t = 0; t < nt; ++t) pool.emplace_back(worker, t);
    for (auto& th : pool) th.join();
}

// |a n b| for two sorted lists; binary search when one is much longer.
int64_t intersect_size(const int32_t* a, int64_t na, const int32_t* b, int64_t nb) {
    if (na > nb) {
        std::swap(a, b);
        std::swap(na, nb);
    }
    if (na == 0) return 0;
    int64_t c = 0;
    if (nb > 32 * na) {
        const int32_t* lo = b;
        const int32_t* end = b + nb;
        for (int64_t i = 0; i < na; ++i) {
            lo = std::lower_bound(lo, end, a[i]);
            if (lo == end) break;
            if (*lo == a[i]) ++c;
        }
        return c;
    }
    int64_t i = 0, j = 0;
    while (i < na && j < nb) {
        int32_t x = a[i], y = b[j];
        c += (x == y);
        i += (x <= y);
        j += (y <= x);
    }
    return c;
}

// Transpose of a CSR pattern (fewer than 2^32 entries): tptr / trow = rows holding each column, ascending inside a
// column.  A counting sort whose row blocks (equal shares of the entries, in row order) are counted and scattered by
// one thread each; a block's start inside a column is the column's start plus what the earlier blocks put there.
void transpose_pattern(int nthreads, int64_t m, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                       std::vector<int64_t>& tptr, std::vector<int32_t>& trow) {
    const int64_t nz = rowptr[m];
    tptr.assign(n + 1, 0);
    trow.resize(nz);
    int nt = nz < (1 << 20) ? 1 : std::max(1, std::min(nthreads, 64));
    while (nt > 1 && (int64_t)nt * n * 4 > ((int64_t)1 << 30)) --nt;  // at most 1 GiB of per-block offsets
    std::vector<int64_t> rb(nt + 1, m);
    rb[0] = 0;
    for (int t = 1; t < nt; ++t) rb[t] = std::lower_bound(rowptr, rowptr + m + 1, nz * t / nt) - rowptr;
    std::vector<std::vector<uint32_t>> off(nt);
    auto run = [&](auto&& fn) {
        if (nt == 1) {
            fn(0);
            return;
        }
        std::vector<std::thread> pool;
        for (int t = 0; t < nt; ++t) pool.emplace_back(fn, t);
        for (auto& th : pool) th.join();
    };
    run([&](int t) {
        off[t].assign(n, 0);
        for (int64_t p = rowptr[rb[t]]; p < rowptr[rb[t + 1]]; ++p) ++off[t][colidx[p]];
    });
    for (int64_t j = 0; j < n; ++j) {
        int64_t at = tptr[j];
        for (int t = 0; t < nt; ++t) {
            const uint32_t c = off[t][j];
            off[t][j] = (uint32_t)at;
            at += c;
        }
        tptr[j + 1] = at;
    }
    run([&](int t) {
        for (int64_t i = rb[t]; i < rb[t + 1]; ++i)
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) trow[off[t][colidx[p]]++] = (int32_t)i;
    });
}

struct Cand {
    int32_t child, parent, w;
};

struct HeapEdge {
    uint64_t key;  // (w << 1) | non-virtual : draws go to the virtual edge (Section 2.2)
    int32_t x, y;  // y = -1: virtual
    bool operator>(const HeapEdge& o) const {
        if (key != o.key) return key > o.key;
        if (x != o.x) return x > o.x;
        return y > o.y;
    }
};

struct Builder {
    cbm_handle* h;
    int64_t m, n, nnz = 0;
    int nthreads;
    int32_t alpha, min_saving, max_depth, hub_cap, max_cand;
    bool auto_depth;
    const int64_t* rowptr = nullptr;  // the matrix that is compressed: A, or A v I
    const int32_t* colidx = nullptr;
    std::vector<int64_t> own_rowptr;
    std::vector<int32_t> own_colidx;
    bool verbose = false;
    std::chrono::steady_clock::time_point last;

    const int32_t* row(int64_t i) const { return colidx + rowptr[i]; }
    int64_t rlen(int64_t i) const { return h->rownnz[i]; }
    int64_t dlen(int64_t x) const { return h->dptr[x + 1] - h->dptr[x]; }
    void lap(const char* what) {
        auto now = std::chrono::steady_clock::now();
        if (verbose)
            std::fprintf(stderr, "[cbm_build] %-22s %.3f s\n", what, std::chrono::duration<double>(now - last).count());
        last = now;
    }

    cbm_status validate(const int64_t* in_rowptr, const int32_t* in_colidx);
    void self_loops(const int64_t* in_rowptr, const int32_t* in_colidx);
    void transpose_matrix();
    std::vector<int32_t> loc;  // position of every row in a breadth-first walk of the graph (square matrices)
    void locality_order();
    std::vector<int64_t> optr;  // candidate edges bucketed by parent
    std::vector<int32_t> ochild, ow;
    bool device_candidates = false;  // run the candidate search on the GPU
    bool device_optional = false;    // ... and fall back to the host threads if that fails
    bool locality = false;           // rounds of long work items will be scheduled by graph locality
    bool sample_first = false;       // estimate what a tree could save from a sample of rows before the full search
    bool skip_tree = false;          // the sample said: nothing to gain, store every row in full
    cbm_status find_candidates();
    std::vector<int32_t> kept_parent, kept_level;  // the best of the grown trees while "no tree" is being priced
    std::vector<int64_t> kept_dptr;
    void prim(int64_t seeds);
    void prim(int64_t seeds, std::vector<int32_t>& parent, std::vector<int32_t>& level, std::vector<int64_t>& dptr) const;
    void arborescence();
    void all_roots();
    void delta_lists();
    // paths
    std::vector<int64_t> cptr;
    std::vector<int32_t> cidx, order, rho, cont, next, round;
    int64_t split_min = 0, split_len = 0;
    bool bundle = false;  // rounds of long work items are emitted as bundles: a path's deltas in one sweep over the columns
    int64_t bundle_min = kBundleMinEntries;  // mean entries per work item from which a round is bundled (CBM_BUNDLE_MIN)
    int64_t bundle_min_items = kBundleMinItems;  // work items a round needs before its paths are cut for bundling (CBM_BUNDLE_MIN_ITEMS)
    int64_t locality_min = kLocalityMinEntries;  // ... from which a round is scheduled by locality (CBM_LOCALITY_MIN)
    std::vector<uint8_t> cap_rows_in_round;  // rounds whose paths plan() holds to CBM_BUNDLE_ROWS rows
    void choose_bundled_rounds(int64_t path_max, int32_t* nrounds);
    bool is_split(int64_t x) const { return dlen(x) > split_min; }
    void tree_index();
    double plan(int64_t path_max, int32_t* nrounds_out);
    double last_round_us = 0.0, last_round_bytes_us = 0.0;  // of the last round: modelled time; its bandwidth term alone
    bool prune_last_round(int64_t path_max);
    double csr_cost() const;
    cbm_status emit(int32_t nrounds);
};

cbm_status Builder::validate(const int64_t* in_rowptr, const int32_t* in_colidx) {
    if (in_rowptr[0] != 0) return CBM_ERR_INVALID_CSR;
    for (int64_t i = 0; i < m; ++i)
        if (in_rowptr[i + 1] < in_rowptr[i]) return CBM_ERR_INVALID_CSR;
    std::atomic<bool> bad{false};
    parallel_chunks(nthreads, m, 4096, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            int64_t prev = -1;
            for (int64_t p = in_rowptr[i]; p < in_rowptr[i + 1]; ++p) {
                int64_t c = in_colidx[p];
                if (c <= prev || c >= n) {
                    bad = true;
                    return;
                }
                prev = c;
            }
        }
    });
    return bad ? CBM_ERR_INVALID_CSR : CBM_OK;
}

void Builder::self_loops(const int64_t* in_rowptr, const int32_t* in_colidx) {
    own_rowptr.assign(m + 1, 0);
    for (int64_t i = 0; i < m; ++i) {
        const int32_t* b = in_colidx + in_rowptr[i];
        const int32_t* e = in_colidx + in_rowptr[i + 1];
        bool has = std::binary_search(b, e, (int32_t)i);
        own_rowptr[i + 1] = own_rowptr[i] + (e - b) + (has ? 0 : 1);
    }
    own_colidx.resize(own_rowptr[m]);
    parallel_chunks(nthreads, m, 4096, [&](int64_t b0, int64_t e0, int) {
        for (int64_t i = b0; i < e0; ++i) {
            const int32_t* b = in_colidx + in_rowptr[i];
            const int32_t* e = in_colidx + in_rowptr[i + 1];
            int32_t* out = own_colidx.data() + own_rowptr[i];
            const int32_t* pos = std::lower_bound(b, e, (int32_t)i);
            out = std::copy(b, pos, out);
            if (pos == e || *pos != (int32_t)i) *out++ = (int32_t)i;
            std::copy(pos, e, out);
        }
    });
    rowptr = own_rowptr.data();
    colidx = own_colidx.data();
}

// Replace the matrix by its transpose (n x m).  Rows are scanned in order, so every new row comes out sorted.
void Builder::transpose_matrix() {
    std::vector<int64_t> tp;
    std::vector<int32_t> tc;
    transpose_pattern(nthreads, m, n, rowptr, colidx, tp, tc);
    own_rowptr.swap(tp);
    own_colidx.swap(tc);
    rowptr = own_rowptr.data();
    colidx = own_colidx.data();
    std::swap(m, n);
}

// Breadth-first order of the rows over the graph itself (row i's columns are its neighbours): rows close in this
// order have overlapping neighbourhoods, so their delta lists gather overlapping rows of X.
void Builder::locality_order() {
    loc.assign(m, -1);
    std::vector<int32_t> queue;
    queue.reserve(m);
    int32_t pos = 0;
    for (int64_t s0 = 0; s0 < m; ++s0) {
        if (loc[s0] >= 0) continue;
        loc[s0] = pos++;
        queue.clear();
        queue.push_back((int32_t)s0);
        for (size_t qh = 0; qh < queue.size(); ++qh) {
            const int32_t x = queue[qh];
            for (int64_t p = rowptr[x]; p < rowptr[x + 1]; ++p) {
                const int32_t y = colidx[p];
                if (y < m && loc[y] < 0) {
                    loc[y] = pos++;
                    queue.push_back(y);
                }
            }
        }
    }
}

void Builder::all_roots() {
    h->parent.assign(m, -1);
    h->level.assign(m, 1);
    h->dptr.assign(m + 1, 0);
    for (int64_t x = 0; x < m; ++x) h->dptr[x + 1] = h->dptr[x] + rlen(x);
}

// Candidate parents: for every row, the rows that share columns with it, ranked by exact Hamming distance.
cbm_status Builder::find_candidates() {
    // transpose: rows holding each column
    std::vector<int64_t> tptr;
    std::vector<int32_t> trow;
    transpose_pattern(nthreads, m, n, rowptr, colidx, tptr, trow);
    lap("transpose");

    // candidate parents of one row: rows sharing columns, ranked by exact Hamming distance (the best come out in sc)
    struct Scored {
        int64_t score;  // saving = nnz(a_x) - w(y,x) = 2|a_x n a_y| - nnz(a_y) (upper bound, then exact)
        int32_t y;
    };
    auto row_candidates = [&](int64_t x, std::vector<int32_t>& cnt, std::vector<int32_t>& tch, std::vector<Scored>& sc) {
        sc.clear();
        const int64_t nx = rlen(x);
        if (nx < 1) return;
        tch.clear();
        int64_t nhub = 0;
        for (const int32_t* pj = row(x); pj != row(x) + nx; ++pj) {
            int64_t deg = tptr[*pj + 1] - tptr[*pj];
            if (hub_cap >= 0 && deg > hub_cap) {  // a hub column: too many rows to expand
                ++nhub;
                continue;
            }
            for (int64_t q = tptr[*pj]; q < tptr[*pj + 1]; ++q) {
                int32_t y = trow[q];
                if (cnt[y]++ == 0) tch.push_back(y);
            }
        }
        for (int32_t y : tch) {
            int64_t ipart = cnt[y];
            cnt[y] = 0;
            if (y == x) continue;
            int64_t ny = rlen(y);
            int64_t iub = ipart + std::min<int64_t>(nhub, std::min(ny, nx) - ipart);
            int64_t ub = 2 * iub - ny;
            if (ub >= min_saving) sc.push_back({ub, y});
        }
        if (sc.empty()) return;
        auto better = [](const Scored& a, const Scored& b2) {
            return a.score != b2.score ? a.score > b2.score : a.y < b2.y;
        };
        if (nhub > 0) {
            // shared hub columns were not counted: settle the best few by exact intersection
            size_t keep = max_cand < 0 ? sc.size() : std::min<size_t>(sc.size(), 2 * (size_t)max_cand);
            if (keep < sc.size()) {
                std::nth_element(sc.begin(), sc.begin() + keep, sc.end(), better);
                sc.resize(keep);
            }
            size_t w = 0;
            for (auto& s : sc) {
                int64_t ny = rlen(s.y);
                int64_t I = intersect_size(row(x), nx, row(s.y), ny);
                s.score = 2 * I - ny;
                if (s.score >= min_saving) sc[w++] = s;
            }
            sc.resize(w);
        }
        size_t keep = max_cand < 0 ? sc.size() : std::min<size_t>(sc.size(), (size_t)max_cand);
        if (keep < sc.size()) {
            std::nth_element(sc.begin(), sc.begin() + keep, sc.end(), better);
            sc.resize(keep);
        }
    };
    std::vector<std::vector<int32_t>> counters(nthreads), touched(nthreads);

    // Automatic mode on a large matrix: look at every 64th row first.  The best candidate of a row bounds what any
    // tree can save on it; if the sample says the whole matrix would shed under 2 % of its entries, no tree can pay
    // for a dependent launch, and the full search (the bulk of the build time) is skipped.
    if (sample_first) {
        const int64_t stride = 64, nsample = (m + stride - 1) / stride;
        std::vector<int64_t> saved(nthreads, 0), seen(nthreads, 0);
        parallel_chunks(nthreads, nsample, 16, [&](int64_t b, int64_t e, int tid) {
            auto& cnt = counters[tid];
            if (cnt.empty()) cnt.assign(m, 0);
            std::vector<Scored> sc;
            for (int64_t i = b; i < e; ++i) {
                const int64_t x = i * stride;
                row_candidates(x, cnt, touched[tid], sc);
                int64_t best = 0;
                for (auto& c : sc) best = std::max(best, c.score);
                saved[tid] += best;
                seen[tid] += rlen(x);
            }
        });
        int64_t sv = 0, sn = 0;
        for (int t = 0; t < nthreads; ++t) {
            sv += saved[t];
            sn += seen[t];
        }
        if (verbose)
            std::fprintf(stderr, "[cbm_build] sample of %ld rows: at most %.2f %% of their entries can be saved\n", (long)nsample,
                         sn > 0 ? 100.0 * sv / sn : 0.0);
        lap("candidate sample");
        if (sv * 50 < sn) {
            skip_tree = true;
            return CBM_OK;
        }
    }

    std::vector<std::vector<Cand>> cand_per_thread(nthreads);
    if (device_candidates) {
        std::vector<int32_t> cn, cy, cw;
        const cbm_status st = cbm_device_candidates(h->opts.device, m, n, rowptr, colidx, tptr.data(), trow.data(), hub_cap,
                                                    min_saving, max_cand, &cn, &cy, &cw);
        if (st != CBM_OK && !device_optional) return st;
        if (st != CBM_OK) {
            if (verbose) std::fprintf(stderr, "[cbm_build] candidate search on the GPU failed (%d): host threads instead\n", (int)st);
            device_candidates = false;
        } else {
            auto& out = cand_per_thread[0];
            for (int64_t x = 0; x < m; ++x)
                for (int32_t i = 0; i < cn[x]; ++i) out.push_back({(int32_t)x, cy[x * max_cand + i], cw[x * max_cand + i]});
        }
    }
    if (!device_candidates) {
        parallel_chunks(nthreads, m, 64, [&](int64_t b, int64_t e, int tid) {
            auto& cnt = counters[tid];
            auto& out = cand_per_thread[tid];
            if (cnt.empty()) cnt.assign(m, 0);
            std::vector<Scored> sc;
            for (int64_t x = b; x < e; ++x) {
                row_candidates(x, cnt, touched[tid], sc);
                const int64_t nx = rlen(x);
                for (auto& c : sc) out.push_back({(int32_t)x, c.y, (int32_t)(nx - c.score)});
            }
        });
    }
    std::vector<int64_t>().swap(tptr);
    std::vector<int32_t>().swap(trow);
    lap("candidates");

    // bucket candidate edges by parent: Prim pushes the out-edges of each newly attached row
    optr.assign(m + 1, 0);
    for (auto& v : cand_per_thread)
        for (auto& c : v) ++optr[c.parent + 1];
    for (int64_t i = 0; i < m; ++i) optr[i + 1] += optr[i];
    ochild.resize(optr[m]);
    ow.resize(optr[m]);
    {
        std::vector<int64_t> fill(optr.begin(), optr.end() - 1);
        for (auto& v : cand_per_thread) {
            for (auto& c : v) {
                int64_t p = fill[c.parent]++;
                ochild[p] = c.child;
                ow[p] = c.w;
            }
            std::vector<Cand>().swap(v);
        }
    }
    return CBM_OK;
}

// Prim growth from the virtual vertex over the candidate edges, depth-capped.  `seeds` rows, evenly
// spread over the index range, are forced to be stored in full before anything else is attached:
// with a depth cap, growing from many seeds at once gives wider levels (more parallel work per
// dependent launch) and often fewer deltas than growing from the few cheapest rows only.
// Also leaves in dptr[] the delta count of every row (the weight of its tree edge).
void Builder::prim(int64_t seeds) { prim(seeds, h->parent, h->level, h->dptr); }

// The same into arrays of the caller's (reads the builder only: several growths can run side by side).
void Builder::prim(int64_t seeds, std::vector<int32_t>& parent, std::vector<int32_t>& level, std::vector<int64_t>& dptr) const {
    parent.assign(m, -1);
    level.assign(m, 0);
    std::vector<int32_t> wsel(m, 0);
    std::vector<HeapEdge> init;
    init.reserve(m);
    for (int64_t x = 0; x < m; ++x) init.push_back({(uint64_t)rlen(x) << 1, (int32_t)x, -1});
    if (seeds > 0 && seeds < m)
        for (int64_t i = 0; i < seeds; ++i) init[(size_t)(i * m / seeds)].key = 0;  // popped before any other edge
    std::priority_queue<HeapEdge, std::vector<HeapEdge>, std::greater<HeapEdge>> pq(std::greater<HeapEdge>(),
                                                                                    std::move(init));
    while (!pq.empty()) {
        HeapEdge e = pq.top();
        pq.pop();
        if (level[e.x] != 0) continue;
        int32_t lvl = e.y < 0 ? 1 : level[e.y] + 1;
        parent[e.x] = e.y;
        level[e.x] = lvl;
        wsel[e.x] = e.y < 0 ? (int32_t)rlen(e.x) : (int32_t)(e.key >> 1);
        if (max_depth > 0 && lvl >= max_depth) continue;  // nothing may hang below the cap
        for (int64_t p = optr[e.x]; p < optr[e.x + 1]; ++p)
            if (level[ochild[p]] == 0) pq.push({((uint64_t)ow[p] << 1) | 1u, ochild[p], e.x});
    }
    dptr.assign(m + 1, 0);
    for (int64_t x = 0; x < m; ++x) dptr[x + 1] = dptr[x] + wsel[x];
}

// Exact minimum-cost arborescence of the candidate digraph rooted at the virtual vertex (Section 2.2,
// "Edge Pruning": once edges are pruned by direction the chain of compression is an MCA).  Edmonds'
// algorithm in Tarjan's form: every vertex keeps a meldable heap (leftist, with a lazy offset) of its
// incoming edges; walking backwards along cheapest incoming edges either reaches finished ground or
// closes a cycle, which is contracted (union-find, heaps melded, the chosen edge's cost taken off every
// edge entering that vertex).  Contractions are undone in reverse order to read off the real edges.
// Cost of an edge = (m + 1) * w + [non-virtual]: total weight first, then as few real edges as possible
// (draws go to the virtual vertex).
void Builder::arborescence() {
    const int64_t V = m + 1, root = m;  // vertex m is the virtual null row
    const int64_t E = m + (int64_t)ochild.size();
    std::vector<int32_t> src(E), dst(E), lc(E, -1), rc(E, -1), rank(E, 1);
    std::vector<int64_t> key(E), lazy(E, 0);
    std::vector<int32_t> ew(E);  // Hamming weight of the edge (delta count)
    for (int64_t x = 0; x < m; ++x) {  // virtual edges
        src[x] = (int32_t)root;
        dst[x] = (int32_t)x;
        ew[x] = (int32_t)rlen(x);
        key[x] = (int64_t)rlen(x) * V;
    }
    {
        int64_t e = m;
        for (int64_t y = 0; y < m; ++y)
            for (int64_t p = optr[y]; p < optr[y + 1]; ++p, ++e) {
                src[e] = (int32_t)y;
                dst[e] = ochild[p];
                ew[e] = ow[p];
                key[e] = (int64_t)ow[p] * V + 1;
            }
    }
    auto push_down = [&](int32_t a) {
        if (lazy[a] == 0) return;
        for (int32_t c : {lc[a], rc[a]})
            if (c >= 0) {
                key[c] += lazy[a];
                lazy[c] += lazy[a];
            }
        lazy[a] = 0;
    };
    std::function<int32_t(int32_t, int32_t)> meld = [&](int32_t a, int32_t b) -> int32_t {
        if (a < 0) return b;
        if (b < 0) return a;
        if (key[b] < key[a] || (key[b] == key[a] && b < a)) std::swap(a, b);
        push_down(a);
        rc[a] = meld(rc[a], b);
        if (lc[a] < 0 || rank[lc[a]] < rank[rc[a]]) std::swap(lc[a], rc[a]);
        rank[a] = rc[a] < 0 ? 1 : rank[rc[a]] + 1;
        return a;
    };
    std::vector<int32_t> heap(V, -1);
    for (int64_t e = 0; e < E; ++e) heap[dst[e]] = meld(heap[dst[e]], (int32_t)e);

    // union-find with rollback (union by size, no path compression)
    std::vector<int32_t> up(V), sz(V, 1);
    for (int64_t v = 0; v < V; ++v) up[v] = (int32_t)v;
    std::vector<std::pair<int32_t, int32_t>> log;  // (child root, parent root) of every union
    auto find = [&](int32_t v) {
        while (up[v] != v) v = up[v];
        return v;
    };
    auto unite = [&](int32_t a, int32_t b) {  // a, b are roots; returns the new root
        if (sz[a] < sz[b]) std::swap(a, b);
        up[b] = a;
        sz[a] += sz[b];
        log.push_back({b, a});
        return a;
    };
    struct Cycle {
        size_t log_size;                                     // union-find state before the contraction
        std::vector<std::pair<int32_t, int32_t>> members;    // (component at that time, its chosen in-edge)
        int32_t merged;                                      // component after the contraction
    };
    std::vector<Cycle> cycles;
    std::vector<int32_t> chosen(V, -1);  // chosen in-edge of a live component
    std::vector<int32_t> state(V, 0);    // 0 = untouched, 1 = on the current walk, 2 = finished
    state[root] = 2;
    std::vector<int32_t> walk;
    for (int64_t s = 0; s < m; ++s) {
        int32_t u = find((int32_t)s);
        if (state[u] != 0) continue;
        walk.clear();
        for (;;) {
            if (state[u] == 2) break;  // reached finished ground
            if (state[u] == 1) {
                // u closes a cycle with the top of the walk: contract everything above u on the walk, and u
                Cycle c;
                c.log_size = log.size();
                int32_t merged = u, h2 = -1;
                for (;;) {
                    const int32_t w = walk.back();
                    walk.pop_back();
                    c.members.push_back({w, chosen[w]});
                    h2 = meld(h2, heap[w]);
                    if (w == u) break;
                }
                for (auto& mw : c.members)
                    if (mw.first != merged) merged = unite(find(merged), find(mw.first));
                merged = find(merged);
                heap[merged] = h2;
                state[merged] = 0;
                chosen[merged] = -1;
                c.merged = merged;
                cycles.push_back(std::move(c));
                u = merged;
                continue;
            }
            state[u] = 1;
            walk.push_back(u);
            // cheapest edge entering u from outside u
            int32_t e = heap[u];
            while (e >= 0 && find(src[e]) == u) {
                push_down(e);
                e = heap[u] = meld(lc[e], rc[e]);
            }
            // every vertex has its virtual edge, so a heap never runs dry before the root is reached
            push_down(e);
            heap[u] = meld(lc[e], rc[e]);
            lc[e] = rc[e] = -1;
            chosen[u] = e;
            if (heap[u] >= 0) {  // reduced costs for the other edges entering u
                key[heap[u]] -= key[e];
                lazy[heap[u]] -= key[e];
            }
            u = find(src[e]);
        }
        for (int32_t w : walk) state[w] = 2;
    }
    // undo the contractions, newest first: inside a cycle every member keeps its chosen edge except the
    // member that the cycle's own in-edge really enters
    for (size_t i = cycles.size(); i-- > 0;) {
        Cycle& c = cycles[i];
        const int32_t e_in = chosen[c.merged];
        while (log.size() > c.log_size) {
            auto [child, parent] = log.back();
            log.pop_back();
            up[child] = child;
            sz[parent] -= sz[child];
        }
        for (auto& mw : c.members) chosen[mw.first] = mw.second;
        chosen[find(dst[e_in])] = e_in;
    }
    h->parent.assign(m, -1);
    h->level.assign(m, 0);
    h->dptr.assign(m + 1, 0);
    for (int64_t x = 0; x < m; ++x) {
        const int32_t e = chosen[x];
        h->parent[x] = src[e] == root ? -1 : src[e];
        h->dptr[x + 1] = h->dptr[x] + ew[e];
    }
    // levels by walking down from the rows stored in full
    std::vector<int64_t> cp(m + 1, 0);
    for (int64_t x = 0; x < m; ++x)
        if (h->parent[x] >= 0) ++cp[h->parent[x] + 1];
    for (int64_t x = 0; x < m; ++x) cp[x + 1] += cp[x];
    std::vector<int32_t> ch(cp[m]);
    {
        std::vector<int64_t> fill(cp.begin(), cp.end() - 1);
        for (int64_t x = 0; x < m; ++x)
            if (h->parent[x] >= 0) ch[fill[h->parent[x]]++] = (int32_t)x;
    }
    std::vector<int32_t> frontier;
    for (int64_t x = 0; x < m; ++x)
        if (h->parent[x] < 0) {
            h->level[x] = 1;
            frontier.push_back((int32_t)x);
        }
    for (size_t i = 0; i < frontier.size(); ++i) {
        const int32_t x = frontier[i];
        for (int64_t q = cp[x]; q < cp[x + 1]; ++q) {
            h->level[ch[q]] = h->level[x] + 1;
            frontier.push_back(ch[q]);
        }
    }
}

// Delta lists (Eq. (2)) of every tree edge by list merge -- or, for a handle that searched its candidates on the GPU,
// by the GPU's kernel, which writes the same lists in the same order (the host merge is the fallback).
void Builder::delta_lists() {
    bool any_parent = false;  // with every row stored in full the lists are the rows themselves: nothing to send anywhere
    for (int64_t x = 0; x < m && !any_parent; ++x) any_parent = h->parent[x] >= 0;
    if (device_candidates && any_parent) {
        const cbm_status st = cbm_device_deltas(h->opts.device, m, rowptr, colidx, h->parent.data(), &h->nplus, &h->nminus,
                                                &h->dptr, &h->dcol);
        if (st == CBM_OK) {
            lap("delta lists (GPU)");
            return;
        }
        if (verbose) std::fprintf(stderr, "[cbm_build] delta lists on the GPU failed (%d): host threads instead\n", (int)st);
    }
    h->nplus.assign(m, 0);
    h->nminus.assign(m, 0);
    parallel_chunks(nthreads, m, 1024, [&](int64_t b, int64_t e, int) {
        for (int64_t x = b; x < e; ++x) {
            int32_t y = h->parent[x];
            if (y < 0) {
                h->nplus[x] = (int32_t)rlen(x);
                continue;
            }
            int64_t I = intersect_size(row(x), rlen(x), row(y), rlen(y));
            h->nplus[x] = (int32_t)(rlen(x) - I);
            h->nminus[x] = (int32_t)(rlen(y) - I);
        }
    });
    h->dptr.assign(m + 1, 0);
    for (int64_t x = 0; x < m; ++x) h->dptr[x + 1] = h->dptr[x] + h->nplus[x] + h->nminus[x];
    h->dcol.resize(h->dptr[m]);
    parallel_chunks(nthreads, m, 1024, [&](int64_t b, int64_t e, int) {
        for (int64_t x = b; x < e; ++x) {
            uint32_t* plus = h->dcol.data() + h->dptr[x];
            int32_t y = h->parent[x];
            if (y < 0) {
                for (int64_t i = 0; i < rlen(x); ++i) plus[i] = (uint32_t)row(x)[i];
                continue;
            }
            uint32_t* minus = plus + h->nplus[x];
            const int32_t *a = row(x), *ae = a + rlen(x), *c = row(y), *ce = c + rlen(y);
            while (a != ae && c != ce) {
                if (*a == *c) {
                    ++a;
                    ++c;
                } else if (*a < *c) {
                    *plus++ = (uint32_t)*a++;
                } else {
                    *minus++ = (uint32_t)*c++ | CBM_DELTA_MINUS;
                }
            }
            while (a != ae) *plus++ = (uint32_t)*a++;
            while (c != ce) *minus++ = (uint32_t)*c++ | CBM_DELTA_MINUS;
        }
    });
    lap("delta lists");
}

// Children lists, level order, and for every row the child that should continue its path: the
// non-split child whose subtree needs the most rounds (a Strahler-number rule, so the number of
// dependent rounds is as small as the tree allows).
void Builder::tree_index() {
    int32_t depth = 0;
    for (int64_t x = 0; x < m; ++x) depth = std::max(depth, h->level[x]);
    cptr.assign(m + 1, 0);
    for (int64_t x = 0; x < m; ++x)
        if (h->parent[x] >= 0) ++cptr[h->parent[x] + 1];
    for (int64_t x = 0; x < m; ++x) cptr[x + 1] += cptr[x];
    cidx.resize(cptr[m]);
    {
        std::vector<int64_t> fill(cptr.begin(), cptr.end() - 1);
        for (int64_t x = 0; x < m; ++x)
            if (h->parent[x] >= 0) cidx[fill[h->parent[x]]++] = (int32_t)x;
    }
    order.resize(m);  // rows by level: parents before children
    {
        std::vector<int64_t> lpos(depth + 2, 0);
        for (int64_t x = 0; x < m; ++x) ++lpos[h->level[x] + 1];
        for (int l = 0; l <= depth; ++l) lpos[l + 1] += lpos[l];
        for (int64_t x = 0; x < m; ++x) order[lpos[h->level[x]]++] = (int32_t)x;
    }
    rho.assign(m, 1);
    cont.assign(m, -1);
    for (int64_t i = m - 1; i >= 0; --i) {
        const int32_t x = order[i];
        int32_t best = -1, need = 1;
        if (!is_split(x))
            for (int64_t q = cptr[x]; q < cptr[x + 1]; ++q) {
                const int32_t c = cidx[q];
                if (!is_split(c) && (best < 0 || rho[c] > rho[best])) best = c;
            }
        for (int64_t q = cptr[x]; q < cptr[x + 1]; ++q) {
            const int32_t c = cidx[q];
            need = std::max(need, c == best ? rho[c] : rho[c] + 1);
        }
        rho[x] = need;
        cont[x] = best;
    }
}

// Cut the tree into paths of at most path_max entries (deltas + one marker per row); fills next[]
// and round[] and returns the modelled time of one product in microseconds.
double Builder::plan(int64_t path_max, int32_t* nrounds_out) {
    next = cont;
    round.assign(m, 0);
    std::vector<int64_t> run(m, 0);  // entries of the path up to and including x
    std::vector<int32_t> prow(m, 0);  // rows of the path up to and including x
    int32_t nrounds = 0;
    for (int64_t i = 0; i < m; ++i) {
        const int32_t x = order[i];
        const int32_t y = h->parent[x];
        const bool continues = y >= 0 && next[y] == x;
        if (continues) {
            round[x] = round[y];
            run[x] = run[y] + dlen(x) + 1;
            prow[x] = prow[y] + 1;
        } else {
            round[x] = y < 0 ? 1 : round[y] + 1;
            run[x] = dlen(x) + 1;
            prow[x] = 1;
        }
        if (next[x] >= 0 && run[x] + dlen(next[x]) + 1 > path_max) next[x] = -1;  // cut: the child heads a new path
        // a round that is going to be bundled holds paths of at most CBM_BUNDLE_ROWS rows
        if (next[x] >= 0 && (size_t)round[x] < cap_rows_in_round.size() && cap_rows_in_round[round[x]] && prow[x] >= CBM_BUNDLE_ROWS)
            next[x] = -1;
        nrounds = std::max(nrounds, round[x]);
    }
    *nrounds_out = nrounds;
    // cost: per round, entries gathered and the longest path; split rows add one segment launch and combines
    std::vector<int64_t> entries(nrounds + 1, 0), rows(nrounds + 1, 0), longest(nrounds + 1, 0), comb(nrounds + 1, 0);
    std::vector<int64_t> heads(nrounds + 1, 0), written(nrounds + 1, 0);
    int64_t seg_entries = 0;
    bool fixup = false;
    for (int64_t i = 0; i < m; ++i) {
        const int32_t x = order[i];
        const int r = round[x];
        const int64_t nc = cptr[x + 1] - cptr[x];
        fixup = fixup || nc > 1 || (nc == 1 && next[x] < 0);
        if (is_split(x)) {
            seg_entries += dlen(x);
            comb[r] += (dlen(x) + split_len - 1) / split_len + CBM_XCD;
            continue;
        }
        entries[r] += dlen(x);
        const bool head = h->parent[x] < 0 || next[h->parent[x]] != x;
        rows[r] += 1 + (h->parent[x] >= 0 && head);  // Y write (+ parent read for a head)
        heads[r] += head;
        ++written[r];
        if (next[x] < 0) longest[r] = std::max(longest[r], run[x]);
    }
    double us = 0.0;
    if (seg_entries > 0)
        us += kLaunchUs + std::max((double)split_len * kEntryUs, seg_entries * kRefRowBytes / (2.0 * kBytesPerUs));
    for (int r = 1; r <= nrounds; ++r) {
        double round_us = 0.0, bytes_us = 0.0;
        if (entries[r] + rows[r] > 0) {
            // a round of long work items is scheduled by graph locality (see emit): more of its gathers hit in L2
            const bool local = locality && heads[r] >= 64 * CBM_XCD && entries[r] + written[r] >= locality_min * heads[r];
            // measured on the protein recipe: 1.25x the base rate at 68 entries per work item, 1.6x at 130, 2.4x at 320
            const double per_item = heads[r] > 0 ? (double)(entries[r] + written[r]) / (double)heads[r] : 0.0;
            // ... and less when there are too few long items to fill the chip (2,500 of them: 0.6 of the rate of 12,000)
            const double fill = (double)heads[r] / ((double)heads[r] + 2048.0);
            const double rate = local ? kBytesPerUs * (1.0 + std::min(1.5, per_item / kLocalityEntries)) * fill / 0.85 : kBytesPerUs;
            bytes_us = (entries[r] + rows[r]) * kRefRowBytes / rate;
            round_us += kLaunchUs + std::max(longest[r] * kEntryUs, bytes_us);
        }
        if (comb[r] > 0) {
            round_us += kLaunchUs + comb[r] * kRefRowBytes / kBytesPerUs;
            bytes_us += comb[r] * kRefRowBytes / kBytesPerUs;
        }
        us += round_us;
        last_round_us = round_us;
        last_round_bytes_us = bytes_us;
    }
    if (fixup && h->square_self_loops) us += kLaunchUs;
    return us;
}

// Rounds whose work items are long (kBundleMinEntries entries on average) and hold more than one row are going to be
// bundled; their paths are then cut again so that none has more than CBM_BUNDLE_ROWS rows.  (The rows cut off head new
// paths one round later; emit() bundles a round only if every path in it obeys the limit, so a round that the second
// cut changes in an unforeseen way simply stays in the plain layout.)  The limit is given up if it would lengthen the
// product by more than an eighth of its rounds.
void Builder::choose_bundled_rounds(int64_t path_max, int32_t* nrounds) {
    std::vector<int64_t> ent(*nrounds + 1, 0), items(*nrounds + 1, 0);
    std::vector<uint8_t> multi(*nrounds + 1, 0);
    for (int64_t x = 0; x < m; ++x) {
        if (is_split(x)) continue;
        const int32_t y = h->parent[x];
        const bool head = y < 0 || next[y] != x;
        ent[round[x]] += dlen(x) + 1;
        items[round[x]] += head;
        multi[round[x]] |= !head;
    }
    cap_rows_in_round.assign(*nrounds + 2, 0);
    bool any = false;
    for (int r = 1; r <= *nrounds; ++r)
        if (multi[r] && items[r] >= bundle_min_items && ent[r] >= bundle_min * items[r]) cap_rows_in_round[r] = 1, any = true;
    if (!any) return;
    const int32_t before = *nrounds;
    plan(path_max, nrounds);  // (the limits stay in force for every later plan() of this build)
    if (*nrounds > before + std::max(1, before / 8)) {
        // a very deep tree: the row limit would add dependent launches, which cost more than the sweeps save
        cap_rows_in_round.clear();
        plan(path_max, nrounds);
    }
}

// The paper prunes compression opportunities that do not pay for their overhead (Section 2.2, "Edge
// Pruning").  Here the overhead that matters is a whole dependent launch: if storing the heads of the LAST
// round in full costs less (a few more gathered rows in round 1) than that round's launch and latency, do
// so; the round disappears.  The round's gathered rows do not: its paths move to round 1 with their
// entries, so what is saved is the launch, the latency of its longest path where that exceeds the
// bandwidth term, and one parent-row read per head.  Returns true if the tree changed.
bool Builder::prune_last_round(int64_t path_max) {
    int32_t nr = 0;
    plan(path_max, &nr);
    if (nr <= 1) return false;
    int64_t extra = 0;
    std::vector<int32_t> heads;
    for (int64_t x = 0; x < m; ++x) {
        if (round[x] != nr) continue;
        const int32_t y = h->parent[x];
        if (y >= 0 && next[y] == x) continue;  // continues a path of this round: moves with its head
        heads.push_back((int32_t)x);
        extra += rlen(x) - dlen(x);
    }
    const double saved = last_round_us - last_round_bytes_us + heads.size() * kRefRowBytes / kBytesPerUs;
    if (saved <= extra * kRefRowBytes / kBytesPerUs) return false;
    if (verbose)
        std::fprintf(stderr, "[cbm_build] round %d (%zu heads, saves %.1f us) dropped: heads stored in full, +%ld deltas\n", nr,
                     heads.size(), saved, (long)extra);
    std::vector<int64_t> len(m);
    for (int64_t x = 0; x < m; ++x) len[x] = dlen(x);
    for (int32_t x : heads) {
        h->parent[x] = -1;
        len[x] = rlen(x);
    }
    for (int64_t x = 0; x < m; ++x) h->dptr[x + 1] = h->dptr[x] + len[x];
    for (int64_t i = 0; i < m; ++i) {  // the old level order is still parents-first
        const int32_t x = order[i];
        h->level[x] = h->parent[x] < 0 ? 1 : h->level[h->parent[x]] + 1;
    }
    tree_index();
    return true;
}

// Modelled time of one product with every row stored in full (plain CSR on the same kernels).
double Builder::csr_cost() const {
    int64_t seg = 0, ent = 0, longest = 0;
    for (int64_t x = 0; x < m; ++x) {
        if (rlen(x) > split_min) {
            seg += rlen(x);
        } else {
            ent += rlen(x) + 1;
            longest = std::max(longest, rlen(x) + 1);
        }
    }
    double us = kLaunchUs + std::max(longest * kEntryUs, ent * kRefRowBytes / kBytesPerUs);
    if (seg > 0)
        us += 2 * kLaunchUs + std::max((double)split_len * kEntryUs, seg * kRefRowBytes / (2.0 * kBytesPerUs));
    return us;
}

// Write the entry stream and the work-item lists for the paths chosen by plan().
cbm_status Builder::emit(int32_t nrounds) {
    const int phases = (int)env_clamped("CBM_PHASES", kPhasesDefault, 1, 64);
    const int64_t fine_min = env_clamped("CBM_FINE_MIN", kFineMinDefault, 1, (long)CBM_TASK_LEN_MASK);
    // rows that a row of ANOTHER work item is compressed against keep their unscaled sum in Y
    std::vector<uint8_t> internal(m, 0);
    h->internal_rows.clear();
    for (int64_t x = 0; x < m; ++x) {
        const int64_t nc = cptr[x + 1] - cptr[x];
        internal[x] = nc > 1 || (nc == 1 && next[x] < 0);
        if (internal[x]) h->internal_rows.push_back((int32_t)x);
    }
    h->levels.assign(nrounds, CbmLevel{});
    h->tasks.clear();
    h->comb.clear();
    h->stream.clear();
    h->num_slots = 0;
    h->seg_deltas = 0;
    int64_t split_rows = 0;
    std::vector<std::vector<CbmTask>> rtasks(nrounds + 1), rcomb(nrounds + 1);
    std::vector<std::vector<int32_t>> rrows(nrounds + 1);  // rows of each path, beside rtasks
    std::vector<std::vector<CbmTask>> seg_tasks((size_t)CBM_XCD * (phases + 1));  // [xcd][phase]; last = unphased
    // Pass 1, in order: where every work item's entries go in the stream (heads of paths and split rows only).
    struct Piece {
        int32_t x;
        int64_t base;  // first entry in the stream
    };
    std::vector<Piece> paths, splits;
    int64_t at = 0;
    for (int64_t i = 0; i < m; ++i) {
        const int32_t x = order[i];
        const int32_t y = h->parent[x];
        if (y >= 0 && next[y] == x) continue;  // not a head
        CbmLevel& R = h->levels[round[x] - 1];
        if (is_split(x)) {
            splits.push_back({x, at});
            at += dlen(x);
            continue;
        }
        const int64_t start = at;
        int32_t path_rows = 0;
        for (int32_t v = x; v >= 0; v = next[v]) {
            at += dlen(v) + 1;
            R.deltas += dlen(v);
            ++R.rows_written;
            ++path_rows;
        }
        // the entry count shares a word with the work item's flags
        if (at - start > (int64_t)CBM_TASK_LEN_MASK) return CBM_ERR_UNSUPPORTED;
        paths.push_back({x, start});
        rtasks[round[x]].push_back({x, y, (uint32_t)start, (uint32_t)(at - start)});
        rrows[round[x]].push_back(path_rows);
        R.parent_reads += y >= 0;
    }
    if (at >= (int64_t)UINT32_MAX) return CBM_ERR_UNSUPPORTED;
    // Which rounds are bundled: those of long work items with more than one row.  (Measured on the protein graph: rounds
    // averaging 134 to 165 entries per work item run 11 to 21 % faster bundled, rounds averaging 105 to 120 run 5 to 10 %
    // slower -- fewer loads in flight per work item than the row-by-row kernel keeps; rounds of short items, as on the
    // collaboration graph, 8 % slower.)
    std::vector<uint8_t> round_bundled(nrounds + 1, 0);
    h->bundled = false;
    for (int r = 1; r <= nrounds && bundle; ++r) {
        int64_t ent = 0;
        int32_t most = 1;
        for (size_t i = 0; i < rtasks[r].size(); ++i) {
            ent += rtasks[r][i].len_flags & CBM_TASK_LEN_MASK;
            most = std::max(most, rrows[r][i]);
        }
        if (verbose)
            std::fprintf(stderr, "[cbm_build] round %d: %zu work items, %.1f entries each, at most %d rows in a path\n", r, rtasks[r].size(),
                         rtasks[r].empty() ? 0.0 : (double)ent / (double)rtasks[r].size(), (int)most);
        // (a round of long single rows has the same entries in either layout: the launch picks the kernel by the width of X)
        h->levels[r - 1].long_single_rows = most == 1 && !rtasks[r].empty() && ent >= kLongSingleRow * (int64_t)rtasks[r].size();
        if (most > 1 && most <= CBM_BUNDLE_ROWS && ent >= bundle_min * (int64_t)rtasks[r].size()) {
            round_bundled[r] = 1;
            h->levels[r - 1].bundled = true;
            h->bundled = true;
        }
    }
    h->stream.resize((size_t)at);
    // A row's deltas go into the stream in ONE ascending sweep over the columns (Delta+ and Delta- merged; the sign
    // travels with the entry).  Work items that run at the same time then move through X in step, low rows first,
    // and find each other's rows in L2: 4 to 6 % off the protein product against "Delta+ then Delta-".
    const bool merge_sort = std::getenv("CBM_NO_MERGE_SORT") == nullptr;
    // Pass 2, on all threads: the entries themselves.  A path is its rows' deltas, each followed by the row's marker;
    // a split row is its deltas re-sorted by column.
    parallel_chunks(nthreads, (int64_t)paths.size(), 256, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            uint32_t* out = h->stream.data() + paths[i].base;
            if (round_bundled[round[paths[i].x]]) {
                // every delta of the path (at most CBM_BUNDLE_ROWS rows), tagged with its row's place in the path, in one
                // ascending sweep; then the rows' markers, in row order
                uint32_t* first = out;
                uint32_t slot = 0;
                for (int32_t v = paths[i].x; v >= 0; v = next[v], ++slot)
                    for (int64_t q = h->dptr[v]; q < h->dptr[v + 1]; ++q) *out++ = h->dcol[q] | (slot << CBM_BUNDLE_SLOT_SHIFT);
                std::sort(first, out, [](uint32_t a, uint32_t b2) { return (a & CBM_BUNDLE_INDEX_MASK) < (b2 & CBM_BUNDLE_INDEX_MASK); });
                for (int32_t v = paths[i].x; v >= 0; v = next[v])
                    *out++ = (uint32_t)v | CBM_ENTRY_MARK | (internal[v] ? CBM_ENTRY_INTERNAL : 0u);
                continue;
            }
            for (int32_t v = paths[i].x; v >= 0; v = next[v]) {
                uint32_t* first = out;
                out = std::copy(h->dcol.begin() + h->dptr[v], h->dcol.begin() + h->dptr[v + 1], out);
                if (merge_sort && h->nminus[v] > 0)
                    std::sort(first, out, [](uint32_t a, uint32_t b2) { return (a & CBM_ENTRY_INDEX_MASK) < (b2 & CBM_ENTRY_INDEX_MASK); });
                *out++ = (uint32_t)v | CBM_ENTRY_MARK | (internal[v] ? CBM_ENTRY_INTERNAL : 0u);
            }
        }
    });
    parallel_chunks(nthreads, (int64_t)splits.size(), 4, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t x = splits[i].x;
            uint32_t* out = h->stream.data() + splits[i].base;
            std::copy(h->dcol.begin() + h->dptr[x], h->dcol.begin() + h->dptr[x + 1], out);
            if (h->nminus[x] > 0)  // Delta+ alone is already in column order
                std::sort(out, out + dlen(x), [](uint32_t a, uint32_t b2) {
                    return (a & CBM_ENTRY_INDEX_MASK) < (b2 & CBM_ENTRY_INDEX_MASK);
                });
        }
    });
    // Pass 3, in order: a long row is cut into segments that depend on nothing.  Its entries, sorted by column,
    // are cut at the CBM_XCD column-range boundaries first: all segments of one column range run on one XCD
    // (workgroup id mod 8), so the popular rows of X in that range stay in that XCD's L2.  Very long rows are cut
    // finer still: each XCD's range is walked in `phases` sub-ranges, one after the other, so that at any time an
    // XCD gathers from 1/(8 phases) of X.
    // The boundaries give every range an equal share of the split rows' entries (equal widths would overload one XCD
    // on a matrix whose popular columns sit together in the index range); cut[f] = first column of fine piece f.
    std::vector<uint32_t> cut((size_t)CBM_XCD * phases + 1, 0);
    {
        const int P = CBM_XCD * phases;
        std::vector<int64_t> upto((size_t)n + 1, 0);  // entries of split rows in columns < c
        for (const Piece& sp : splits)
            for (int64_t i = 0; i < dlen(sp.x); ++i) ++upto[(h->stream[sp.base + i] & CBM_ENTRY_INDEX_MASK) + 1];
        for (int64_t c2 = 0; c2 < n; ++c2) upto[c2 + 1] += upto[c2];
        const int64_t total = upto[n];
        for (int f = 1; f < P; ++f)
            cut[f] = total > 0 ? (uint32_t)(std::lower_bound(upto.begin(), upto.end(), (total * f + P - 1) / P) - upto.begin())
                               : (uint32_t)((int64_t)f * n / P);
        cut[P] = (uint32_t)n;
        for (int f = 1; f <= P; ++f) cut[f] = std::min<uint32_t>((uint32_t)n, std::max(cut[f], cut[f - 1]));
    }
    for (const Piece& sp : splits) {
        const int32_t x = sp.x;
        const int32_t y = h->parent[x];
        CbmLevel& R = h->levels[round[x] - 1];
        ++split_rows;
        const int64_t len = dlen(x);
        const int64_t base = sp.base;
        const uint32_t* ent = h->stream.data() + base;
        const int64_t slot0 = h->num_slots;
        const int fine = len >= fine_min ? phases : 1;  // pieces per XCD range
        const int npieces = CBM_XCD * fine;
        int64_t pos = 0;
        for (int f = 0; f < npieces; ++f) {
            const uint32_t hi = cut[(size_t)(f + 1) * (phases / fine)];  // columns < hi
            const int64_t end = std::partition_point(ent + pos, ent + len, [&](uint32_t e2) { return (e2 & CBM_ENTRY_INDEX_MASK) < hi; }) - ent;
            auto& list = seg_tasks[(size_t)(f / fine) * (phases + 1) + (fine > 1 ? f % fine : phases)];
            for (int64_t b = pos; b < end; b += split_len) {
                const int64_t e = std::min(end, b + split_len);
                list.push_back({(int32_t)h->num_slots, -1, (uint32_t)(base + b), (uint32_t)(e - b) | CBM_TASK_SEGMENT});
                ++h->num_slots;
            }
            pos = end;
        }
        const int64_t nseg = h->num_slots - slot0;
        h->seg_deltas += len;
        rcomb[round[x]].push_back({x, y, (uint32_t)slot0, (uint32_t)nseg | (internal[x] ? CBM_TASK_INTERNAL : 0u)});
        R.comb_segments += nseg;
        R.comb_parent_reads += y >= 0;
    }
    if ((int64_t)h->stream.size() >= (int64_t)UINT32_MAX) return CBM_ERR_UNSUPPORTED;
    // longest first: wave-mates get similar lengths and the tail of a launch is short
    auto longest_first = [](const CbmTask& a, const CbmTask& b2) {
        return (a.len_flags & CBM_TASK_LEN_MASK) > (b2.len_flags & CBM_TASK_LEN_MASK);
    };
    for (int j = 0; j < CBM_XCD; ++j) {  // segment work items first: one block per XCD, phases in order
        h->seg_begin[j] = (int64_t)h->tasks.size();
        for (int ph = 0; ph <= phases; ++ph) {
            auto& list = seg_tasks[(size_t)j * (phases + 1) + ph];
            std::stable_sort(list.begin(), list.end(), longest_first);
            h->tasks.insert(h->tasks.end(), list.begin(), list.end());
        }
        h->seg_count[j] = (int64_t)h->tasks.size() - h->seg_begin[j];
    }
    const bool by_locality = !loc.empty();
    for (int r = 1; r <= nrounds; ++r) {
        CbmLevel& R = h->levels[r - 1];
        auto& lt = rtasks[r];
        R.task_begin = (int64_t)h->tasks.size();
        R.task_count = (int64_t)lt.size();
        int64_t round_entries = 0;
        for (auto& t : lt) round_entries += (t.len_flags & CBM_TASK_LEN_MASK);
        // worth it for rounds of long work items (protein: 8 % faster); rounds of short ones lose more to the
        // ragged tail of each XCD's block than they gain (and a graph without a tree has no such order at all)
        if (by_locality && (int64_t)lt.size() >= 64 * CBM_XCD && round_entries >= locality_min * (int64_t)lt.size()) {
            // neighbours in the graph next to each other, one contiguous share of the entries per XCD: what the
            // work items running on an XCD at one time gather overlaps, and stays in that XCD's L2
            std::stable_sort(lt.begin(), lt.end(), [&](const CbmTask& a, const CbmTask& b2) { return loc[a.row] < loc[b2.row]; });
            const int64_t total = round_entries;
            R.by_xcd = true;
            size_t i = 0;
            int64_t seen = 0;
            for (int j = 0; j < CBM_XCD; ++j) {
                R.xcd_begin[j] = R.task_begin + (int64_t)i;
                const int64_t want = total * (j + 1) / CBM_XCD;
                while (i < lt.size() && (j == CBM_XCD - 1 || seen < want)) seen += (lt[i++].len_flags & CBM_TASK_LEN_MASK);
                R.xcd_count[j] = R.task_begin + (int64_t)i - R.xcd_begin[j];
            }
            // Inside a share the longest work items go first: which XCD gathers what is what the locality is about, and
            // a long item that starts last is the tail of the whole launch (protein product: 1.05 -> 0.80 ms; only the
            // longer half first gains half of that).  A share of very many short items has no tail to speak of and lives
            // on neighbours running side by side instead (collaboration graph with every row stored in full: 0.44 ms in
            // locality order, 0.54 ms longest-first): there the order is by length only in buckets of 32 entries,
            // locality order inside a bucket.  CBM_SHARE_SORT: 0 = locality order, 1 = longest first, n = buckets of n.
            const long share_mode = env_clamped("CBM_SHARE_SORT", -1, -1, 1 << 20);
            for (int j = 0; j < CBM_XCD; ++j) {
                auto b = lt.begin() + (R.xcd_begin[j] - R.task_begin);
                const long mode = share_mode >= 0 ? share_mode : (R.xcd_count[j] <= kShareSortItems ? 1 : kShareBucket);
                if (mode == 1)
                    std::stable_sort(b, b + R.xcd_count[j], longest_first);
                else if (mode > 1)
                    std::stable_sort(b, b + R.xcd_count[j], [&](const CbmTask& x, const CbmTask& y) {
                        return (x.len_flags & CBM_TASK_LEN_MASK) / mode > (y.len_flags & CBM_TASK_LEN_MASK) / mode;
                    });
            }
        } else {
            std::stable_sort(lt.begin(), lt.end(), longest_first);
        }
        h->tasks.insert(h->tasks.end(), lt.begin(), lt.end());
        R.comb_begin = (int64_t)h->comb.size();
        R.comb_count = (int64_t)rcomb[r].size();
        h->comb.insert(h->comb.end(), rcomb[r].begin(), rcomb[r].end());
    }
    h->stats.num_split_rows = split_rows;
    return CBM_OK;
}

}  // namespace

// Column-blocked CBM: the columns are cut into B equal ranges and the part of every row inside a range becomes a row
// of its own; the B m part-rows, stacked block after block (part-row b m + i = row i inside range b), are compressed
// as ONE matrix by the builder above -- its candidate search only ever pairs rows that share columns, so trees form
// inside ranges -- and a product is the sum of the B partial rows of every row.  The format lives in h->inner.
static cbm_status cbm_build_blocked(int64_t m, int64_t n, const int64_t* in_rowptr, const int32_t* in_colidx, cbm_handle* h) {
    auto t0 = std::chrono::steady_clock::now();
    const cbm_build_opts& o = h->opts;
    const int64_t B = o.column_blocks;
    if (o.flags & CBM_FLAG_TRANSPOSE) return CBM_ERR_INVALID_ARG;
    if (o.add_self_loops && m != n) return CBM_ERR_INVALID_ARG;
    if (B > 64 || B * m > (int64_t)CBM_ENTRY_INDEX_MASK || n > (int64_t)CBM_ENTRY_INDEX_MASK) return CBM_ERR_UNSUPPORTED;
    Builder P;  // borrowed for its CSR checks and the A v I step
    P.h = h;
    P.m = m;
    P.n = n;
    P.nthreads = o.num_threads > 0 ? o.num_threads : (int)std::max(1u, std::thread::hardware_concurrency());
    cbm_status st = P.validate(in_rowptr, in_colidx);
    if (st != CBM_OK) return st;
    P.rowptr = in_rowptr;
    P.colidx = in_colidx;
    if (o.add_self_loops) P.self_loops(in_rowptr, in_colidx);
    const int64_t nnz = P.rowptr[m];
    if (nnz >= (int64_t)UINT32_MAX) return CBM_ERR_UNSUPPORTED;
    h->m = m;
    h->n = n;
    h->blocks = (int32_t)B;
    h->square_self_loops = o.add_self_loops != 0;
    // the part-rows, block after block
    std::vector<int64_t> srp((size_t)(B * m) + 1, 0);
    std::vector<int32_t> sci((size_t)nnz);
    auto lo_of = [&](int64_t b) { return (int32_t)((b * n + B - 1) / B); };  // block b = columns [lo_of(b), lo_of(b + 1))
    parallel_chunks(P.nthreads, m, 4096, [&](int64_t r0, int64_t r1, int) {
        for (int64_t i = r0; i < r1; ++i) {
            const int32_t* row = P.colidx + P.rowptr[i];
            const int32_t* end = P.colidx + P.rowptr[i + 1];
            for (int64_t b = 0; b < B; ++b) {
                const int32_t* lo = std::lower_bound(row, end, lo_of(b));
                const int32_t* hi = std::lower_bound(lo, end, lo_of(b + 1));
                srp[(size_t)(b * m + i) + 1] = hi - lo;
            }
        }
    });
    for (int64_t v = 0; v < B * m; ++v) srp[v + 1] += srp[v];
    parallel_chunks(P.nthreads, m, 4096, [&](int64_t r0, int64_t r1, int) {
        for (int64_t i = r0; i < r1; ++i) {
            const int32_t* row = P.colidx + P.rowptr[i];
            const int32_t* end = P.colidx + P.rowptr[i + 1];
            for (int64_t b = 0; b < B; ++b) {
                const int32_t* lo = std::lower_bound(row, end, lo_of(b));
                const int32_t* hi = std::lower_bound(lo, end, lo_of(b + 1));
                std::copy(lo, hi, sci.begin() + srp[(size_t)(b * m + i)]);
            }
        }
    });
    cbm_handle* in = new cbm_handle();
    h->inner = in;  // owned from here on: freed with the outer handle, also on failure
    in->opts = o;
    in->opts.column_blocks = 0;
    in->opts.add_self_loops = 0;
    st = cbm_build_host(B * m, n, srp.data(), sci.data(), in);
    if (st != CBM_OK) return st;
    // weights by index: an entry's index is a column (< n) or a part-row b m + i, whose weights are those of row i
    std::vector<float> dinv, rinv(m);
    for (int64_t i = 0; i < m; ++i) {
        const int64_t len = P.rowptr[i + 1] - P.rowptr[i];
        rinv[i] = len > 0 ? (float)(1.0 / (double)len) : 0.0f;
    }
    in->rinv.resize((size_t)(B * m));
    for (int64_t v = 0; v < B * m; ++v) in->rinv[v] = rinv[v % m];
    if (h->square_self_loops) {  // D = row sums of A v I
        in->square_self_loops = true;
        in->dinv.resize((size_t)(B * m));
        for (int64_t v = 0; v < B * m; ++v) {
            const int64_t i = v % m;
            in->dinv[v] = (float)(1.0 / std::sqrt((double)(P.rowptr[i + 1] - P.rowptr[i])));
        }
        in->stats.bytes_cbm += 4 * (int64_t)in->dinv.size();
    }
    h->rownnz.resize(m);
    for (int64_t i = 0; i < m; ++i) h->rownnz[i] = (int32_t)(P.rowptr[i + 1] - P.rowptr[i]);
    cbm_stats_t& s = h->stats;
    s = in->stats;
    s.m = m;
    s.n = n;
    s.nnz = nnz;
    s.scalar_ops += (B - 1) * m;  // the additions of the block sum
    s.bytes_csr = 8 * (m + 1) + 4 * in_rowptr[m];
    s.add_self_loops = o.add_self_loops != 0;
    s.column_blocks = (int32_t)B;
    s.build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return CBM_OK;
}

cbm_status cbm_build_host(int64_t m, int64_t n, const int64_t* in_rowptr, const int32_t* in_colidx, cbm_handle* h) {
    auto t0 = std::chrono::steady_clock::now();
    const cbm_build_opts& o = h->opts;
    if (o.alpha < 0 || o.max_depth < -1 || o.hub_cap < -1 || o.max_candidates < -1 || o.seed_roots < -1 ||
        o.num_threads < 0 || o.column_blocks < 0)
        return CBM_ERR_INVALID_ARG;
    if (o.column_blocks > 1) return cbm_build_blocked(m, n, in_rowptr, in_colidx, h);
    if (m > (int64_t)CBM_ENTRY_INDEX_MASK || n > (int64_t)CBM_ENTRY_INDEX_MASK) return CBM_ERR_UNSUPPORTED;
    if (o.add_self_loops && m != n) return CBM_ERR_INVALID_ARG;
    Builder B;
    B.h = h;
    B.m = m;
    B.n = n;
    B.nthreads = o.num_threads > 0 ? o.num_threads : (int)std::max(1u, std::thread::hardware_concurrency());
    B.alpha = o.alpha;
    B.min_saving = std::max(o.alpha, 1);  // strict gain at alpha = 0: draws go to the virtual edge
    B.auto_depth = o.max_depth == 0;
    B.max_depth = o.max_depth == 0 ? kDefaultMaxDepth : o.max_depth;  // -1 = unlimited
    B.hub_cap = o.hub_cap == 0 ? kDefaultHubCap : o.hub_cap;
    B.max_cand = o.max_candidates == 0 ? kDefaultMaxCand : o.max_candidates;
    B.verbose = std::getenv("CBM_VERBOSE") != nullptr;
    B.last = t0;
    // segments and unsplit rows both have to fit the 24-bit entry count of a work item
    B.split_len = env_clamped("CBM_SPLIT_LEN", kSplitLenDefault, 1, 1 << 20);
    B.split_min = env_clamped("CBM_SPLIT_MIN", kSplitMinDefault, 1, 1 << 20);
    h->m = m;
    h->n = n;
    h->eff_alpha = B.alpha;
    h->eff_max_depth = B.max_depth;
    h->eff_hub_cap = B.hub_cap;
    h->eff_max_cand = B.max_cand;
    h->square_self_loops = o.add_self_loops != 0;

    cbm_status st = B.validate(in_rowptr, in_colidx);
    if (st != CBM_OK) return st;
    B.rowptr = in_rowptr;
    B.colidx = in_colidx;
    if (o.add_self_loops) B.self_loops(in_rowptr, in_colidx);
    B.nnz = B.rowptr[m];
    if (B.nnz >= (int64_t)UINT32_MAX) return CBM_ERR_UNSUPPORTED;
    if (h->square_self_loops) {  // D^-1/2 of A v I: D is the row sums of the matrix as given, transposed or not
        h->dinv.resize(m);
        for (int64_t i = 0; i < m; ++i) h->dinv[i] = (float)(1.0 / std::sqrt((double)(B.rowptr[i + 1] - B.rowptr[i])));
    }
    if (o.flags & CBM_FLAG_TRANSPOSE) {
        B.transpose_matrix();
        m = B.m;
        n = B.n;
        h->m = m;
        h->n = n;
    }
    h->rownnz.resize(m);
    for (int64_t i = 0; i < m; ++i) h->rownnz[i] = (int32_t)(B.rowptr[i + 1] - B.rowptr[i]);
    B.lap("validate + A v I");

    h->rinv.resize(m);  // 1/nnz per row: the mean aggregator's row weight
    for (int64_t i = 0; i < m; ++i) h->rinv[i] = B.rlen(i) > 0 ? (float)(1.0 / (double)B.rlen(i)) : 0.0f;

    // ---- tree, paths, rounds ---------------------------------------------------------------------
    // The tree is cut into vertical paths.  A path is ONE work item: its running sum stays in
    // registers from row to row (c_x = c_y + deltas, Eq. (5)), so only the head of a path waits for
    // another work item, the one that produced its parent's row.  Paths whose head hangs off a row of
    // a round-r path run in round r + 1, and every round is one kernel launch.  Longer paths mean fewer
    // rounds but a longer chain of dependent batches inside one work item.  The number of seeded roots
    // and the path length cap are the pair the cost model likes best; with the default depth option the
    // model may also find that no tree pays for its extra launches (small graphs): then every row is
    // stored in full.  A depth cap of 1 means exactly that and needs no candidate search.
    int32_t nrounds = 0;
    int64_t best_len = kPathChoices[0], best_split = B.split_min;
    // rows longer than the split threshold are cut into per-XCD segments: worth a launch or two of their own on
    // graphs with many long rows, a loss where only a handful exist
    std::vector<int64_t> split_choices = {kSplitMinDefault, kSplitLenDefault};
    if (std::getenv("CBM_SPLIT_MIN")) split_choices = {B.split_min};
    bool tree = B.max_depth != 1 && m > 1;
    B.locality = m == n && !std::getenv("CBM_NO_LOCALITY");
    B.bundle = tree && n <= (int64_t)CBM_BUNDLE_INDEX_MASK && !std::getenv("CBM_NO_BUNDLE");
    B.bundle_min = env_clamped("CBM_BUNDLE_MIN", kBundleMinEntries, 1, 1 << 20);
    B.bundle_min_items = env_clamped("CBM_BUNDLE_MIN_ITEMS", kBundleMinItems, 1, 1 << 30);
    B.locality_min = env_clamped("CBM_LOCALITY_MIN", kLocalityMinEntries, 1, 1 << 20);
    const bool exact_tree = (o.flags & CBM_FLAG_EXACT_TREE) != 0;
    if (o.flags & CBM_FLAG_DEVICE_BUILD) {  // asked for: an error if it cannot be had
        if ((o.flags & (CBM_FLAG_HOST_ONLY | CBM_FLAG_HOST_SEARCH)) || B.max_cand < 1 || B.max_cand > 16) return CBM_ERR_INVALID_ARG;
        B.device_candidates = true;
    } else if (!(o.flags & (CBM_FLAG_HOST_ONLY | CBM_FLAG_HOST_SEARCH)) && m >= kDeviceSearchMinRows && B.max_cand >= 1 &&
               B.max_cand <= 16) {
        // not asked for: a handle that is going to a GPU anyway searches there too when the matrix is large, and
        // falls back to the host threads if the GPU cannot take it (memory); both give the same candidates
        B.device_candidates = true;
        B.device_optional = true;
    }
    if (tree && exact_tree) {
        if ((st = B.find_candidates()) != CBM_OK) return st;
        B.arborescence();
        B.tree_index();
        double best_us = 1e300;
        for (int64_t cap : kPathChoices) {
            int32_t nr = 0;
            const double us = B.plan(cap, &nr);
            if (us < best_us) {
                best_us = us;
                best_len = cap;
            }
        }
        B.lap("exact arborescence");
    } else if (tree) {
        B.sample_first = B.auto_depth && m >= kSampleMinRows && !std::getenv("CBM_NO_SAMPLE");
        if ((st = B.find_candidates()) != CBM_OK) return st;
    }
    if (tree && !exact_tree && B.skip_tree) tree = false;
    if (tree && !exact_tree) {
        const int64_t forced_len = env_clamped("CBM_PATH_MAX", 0, 0, 1 << 20);
        const int64_t forced_seeds = o.seed_roots > 0 ? o.seed_roots : o.seed_roots < 0 ? 0 : env_or("CBM_SEED_ROOTS", -1);
        double best_us = 1e300;
        // the trees grown from 0, m/128, m/32, m/8 seeded roots, side by side (or the one the caller asked for)
        struct Grown {
            int64_t seeds;
            std::vector<int32_t> parent, level;
            std::vector<int64_t> dptr;
        };
        std::vector<Grown> grown;
        for (int64_t seeds : {(int64_t)0, m / 128, m / 32, m / 8}) {
            grown.push_back({forced_seeds >= 0 ? forced_seeds : seeds, {}, {}, {}});
            if (forced_seeds >= 0 || m < 1024) break;
        }
        {
            std::vector<std::thread> pool;
            for (size_t i = 1; i < grown.size() && B.nthreads > 1; ++i)
                pool.emplace_back([&, i] { B.prim(grown[i].seeds, grown[i].parent, grown[i].level, grown[i].dptr); });
            B.prim(grown[0].seeds, grown[0].parent, grown[0].level, grown[0].dptr);
            for (auto& th : pool) th.join();
            for (size_t i = 1; i < grown.size() && B.nthreads <= 1; ++i)
                B.prim(grown[i].seeds, grown[i].parent, grown[i].level, grown[i].dptr);
        }
        size_t best_tree = 0;
        for (size_t gi = 0; gi < grown.size(); ++gi) {
            const int64_t seeds = grown[gi].seeds;
            h->parent.swap(grown[gi].parent);
            h->level.swap(grown[gi].level);
            h->dptr.swap(grown[gi].dptr);
            for (int64_t split : split_choices) {
                B.split_min = split;
                B.tree_index();
                for (int64_t cap : kPathChoices) {
                    if (forced_len > 0) cap = forced_len;
                    int32_t nr = 0;
                    const double us = B.plan(cap, &nr);
                    if (B.verbose)
                        std::fprintf(stderr,
                                     "[cbm_build] seeds %7ld split above %3ld path cap %4ld: %3d rounds, %ld deltas, model %.1f us\n",
                                     (long)seeds, (long)split, (long)cap, nr, (long)h->dptr[m], us);
                    if (us < best_us) {
                        best_us = us;
                        best_len = cap;
                        best_split = split;
                        best_tree = gi;
                    }
                    if (forced_len > 0) break;
                }
            }
            h->parent.swap(grown[gi].parent);
            h->level.swap(grown[gi].level);
            h->dptr.swap(grown[gi].dptr);
        }
        B.kept_parent.swap(grown[best_tree].parent);  // the winner, for after the comparison with "no tree"
        B.kept_level.swap(grown[best_tree].level);
        B.kept_dptr.swap(grown[best_tree].dptr);
        grown.clear();
        if (B.auto_depth && forced_len <= 0) {
            B.all_roots();
            for (int64_t split : split_choices) {
                B.split_min = split;
                const double csr_us = B.csr_cost();
                if (B.verbose)
                    std::fprintf(stderr, "[cbm_build] all rows in full, split above %ld: model %.1f us (best tree: %.1f us)\n",
                                 (long)split, csr_us, best_us);
                if (csr_us <= best_us) {
                    best_us = csr_us;
                    best_split = split;
                    tree = false;
                }
            }
        }
        B.lap("tree + path model");
    } else if (!tree) {
        B.all_roots();
        double best_us = 1e300;
        for (int64_t split : split_choices) {
            B.split_min = split;
            const double us = B.csr_cost();
            if (us < best_us) {
                best_us = us;
                best_split = split;
            }
        }
    }
    B.split_min = best_split;
    if (tree && exact_tree) {
        // keep the arborescence as found
        if (B.bundle) {
            int32_t nr = 0;
            B.plan(best_len, &nr);
            B.choose_bundled_rounds(best_len, &nr);
        }
    } else if (tree) {
        h->parent.swap(B.kept_parent);
        h->level.swap(B.kept_level);
        h->dptr.swap(B.kept_dptr);
        B.tree_index();
        if (B.bundle) {  // before the last round is priced: the row limit of bundled rounds moves some rows one round down
            int32_t nr = 0;
            B.plan(best_len, &nr);
            B.choose_bundled_rounds(best_len, &nr);
        }
        while (B.auto_depth && B.prune_last_round(best_len)) {  // part of the automatic policy only
        }
    } else {
        B.all_roots();
    }
    std::vector<int64_t>().swap(B.optr);
    std::vector<int32_t>().swap(B.ochild);
    std::vector<int32_t>().swap(B.ow);
    if (!tree) B.bundle = false;  // every row stored in full: nothing to bundle
    B.delta_lists();
    B.tree_index();
    B.plan(best_len, &nrounds);
    if (tree && B.locality) B.locality_order();
    cbm_stats_t& s = h->stats;
    std::memset(&s, 0, sizeof(s));
    st = B.emit(nrounds);
    if (st != CBM_OK) return st;
    B.lap("paths + work lists");

    // ---- counters (Properties 1 and 2) -----------------------------------------------------------
    s.m = m;
    s.n = n;
    s.nnz = B.nnz;
    int32_t depth = 0;
    for (int64_t x = 0; x < m; ++x) {
        depth = std::max(depth, h->level[x]);
        s.num_delta_plus += h->nplus[x];
        s.num_delta_minus += h->nminus[x];
        if (h->parent[x] < 0) {
            ++s.num_roots;
            s.scalar_ops += B.rlen(x);
        } else {
            s.scalar_ops += 1 + h->nplus[x] + h->nminus[x];
        }
    }
    s.num_internal = (int64_t)h->internal_rows.size();
    s.num_tasks = (int64_t)h->tasks.size();
    s.bytes_csr = 8 * (m + 1) + 4 * in_rowptr[m];
    s.bytes_cbm = 4 * (int64_t)h->stream.size() + (int64_t)sizeof(CbmTask) * (int64_t)(h->tasks.size() + h->comb.size()) +
                  4 * (int64_t)h->internal_rows.size() + 4 * (int64_t)h->dinv.size();
    s.depth = depth;
    s.rounds = nrounds;
    s.alpha = B.alpha;
    s.add_self_loops = o.add_self_loops != 0;
    s.column_blocks = 1;
    for (const CbmLevel& L : h->levels) s.bundled_rounds += L.bundled;
    s.build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return CBM_OK;
}

cbm_status cbm_decompress_host(const cbm_handle* h, int64_t* rowptr, int32_t* colidx) {
    if (h->blocks > 1) {  // rebuild the part-rows from the inner format, then put every row's parts back together
        const cbm_handle* in = h->inner;
        const int64_t m = h->m, B = h->blocks;
        std::vector<int64_t> srp((size_t)(B * m) + 1);
        std::vector<int32_t> sci((size_t)std::max<int64_t>(1, in->stats.nnz));
        const cbm_status st = cbm_decompress_host(in, srp.data(), sci.data());
        if (st != CBM_OK) return st;
        rowptr[0] = 0;
        for (int64_t i = 0; i < m; ++i) {
            int32_t* out = colidx + rowptr[i];
            for (int64_t b = 0; b < B; ++b)  // ranges ascend, so the parts in block order are the sorted row
                out = std::copy(sci.begin() + srp[(size_t)(b * m + i)], sci.begin() + srp[(size_t)(b * m + i) + 1], out);
            rowptr[i + 1] = out - colidx;
        }
        return CBM_OK;
    }
    const int64_t m = h->m;
    rowptr[0] = 0;
    for (int64_t x = 0; x < m; ++x) rowptr[x + 1] = rowptr[x] + h->rownnz[x];
    // parents before children: visit rows by level; a row is rebuilt from its parent's rebuilt
    // list and its own two delta lists only (Eq. (2))
    std::vector<int32_t> order(m);
    for (int64_t x = 0; x < m; ++x) order[x] = (int32_t)x;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return h->level[a] < h->level[b]; });
    for (int32_t x : order) {
        const uint32_t* plus = h->dcol.data() + h->dptr[x];
        const uint32_t* pe = plus + h->nplus[x];
        const uint32_t* minus = pe;
        const uint32_t* me = minus + h->nminus[x];
        int32_t* out = colidx + rowptr[x];
        int32_t* oe = colidx + rowptr[x + 1];
        int32_t y = h->parent[x];
        const int32_t* a = y >= 0 ? colidx + rowptr[y] : nullptr;
        const int32_t* ae = y >= 0 ? colidx + rowptr[y + 1] : nullptr;
        // (a_y \ Delta-) merged with Delta+
        while (a != ae || plus != pe) {
            if (a != ae && minus != me && (uint32_t)*a == (*minus & ~CBM_DELTA_MINUS)) {
                ++a;
                ++minus;
                continue;
            }
            int32_t v;
            if (plus == pe || (a != ae && (uint32_t)*a < *plus))
                v = *a++;
            else
                v = (int32_t)*plus++;
            if (out == oe) return CBM_ERR_STATE;
            *out++ = v;
        }
        if (out != oe || minus != me) return CBM_ERR_STATE;
    }
    return CBM_OK;
}

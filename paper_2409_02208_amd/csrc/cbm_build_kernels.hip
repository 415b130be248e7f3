// The builder's GPU side: the candidate search, and the delta lists of the chosen tree.
//
// The compression tree is chosen among "candidate" edges (y, x): rows y that share columns with
// row x, ranked by the Hamming distance of Lemma 2.1, w(y,x) = nnz(a_x) + nnz(a_y) - 2 |a_x n a_y|.
// Finding them is the pattern of the sparse product A A^T: for every column j of row x, every row y
// of column j shares one more column with x.  One workgroup owns one row at a time and counts either
// in an LDS hash table (rows that meet a few thousand others at most) or in a dense array of its own
// (one counter per row of the matrix: the chip's memory is large enough to give every resident
// workgroup such an array), then scores the rows it met, keeps the best few and settles them by exact
// list intersection where columns were skipped as hubs.  The selection rule and the tie-breaks are
// those of the host search, so both produce the same candidate set.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "cbm_internal.h"

namespace {

constexpr int kHashBits = 13;
constexpr int kHashSlots = 1 << kHashBits;           // counters a workgroup keeps in LDS (keys + counts: 64 KiB)
constexpr unsigned kHashLimit = kHashSlots - 1024;  // distinct rows from which the table is given up: up to 256 lanes x 4
                                                     // insertions may still land after that, and it must never fill
constexpr int kCandMax = 16;          // most candidates kept per row
constexpr int kSelMax = 2 * kCandMax;  // most candidates settled by exact intersection

struct CandArgs {
    int64_t m;
    const int64_t* rowptr;  // the compressed matrix (A or A v I), CSR
    const int32_t* colidx;
    const int64_t* tptr;  // its transpose: rows holding each column
    const int32_t* trow;
    const int32_t* order;  // rows in the order workgroups take them (heaviest first)
    int64_t nheavy;        // the first nheavy of them expand to too many rows for an LDS table: dense counters at once
    int32_t* overflow;     // [m] rows whose LDS table filled up: left to the dense pass
    unsigned long long* noverflow;
    int64_t hub_cap;       // columns held by more rows than this are not expanded (< 0: no cap)
    int64_t min_saving;    // a candidate must save at least this many deltas
    int32_t keep;          // candidates kept per row, <= kCandMax
    unsigned long long* next;  // work queue: index into order[] of the next row
    uint32_t* cnt;             // [workgroup][m] shared-column counters, all zero between rows
    int32_t* touched;          // [workgroup][m] rows with a non-zero counter
    unsigned long long* pass;  // [workgroup][m] keys of the rows that may save enough
    int32_t* out_n;            // [m] candidates found
    int32_t* out_y;            // [m][keep] candidate parents
    int32_t* out_w;            // [m][keep] their distance w(y,x)
};

// larger key = better candidate: higher saving first, then the smaller row index
__device__ __forceinline__ unsigned long long make_key(int64_t saving, int32_t y) {
    return ((unsigned long long)saving << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)y);
}
__device__ __forceinline__ int32_t key_row(unsigned long long key) { return (int32_t)(0xFFFFFFFFu - (uint32_t)key); }

__device__ __forceinline__ unsigned long long wave_max(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, off, 64);
        const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), off, 64);
        const unsigned long long o = ((unsigned long long)hi << 32) | lo;
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ int64_t wave_sum(int64_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, off, 64);
        const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)((uint64_t)v >> 32), off, 64);
        v += (int64_t)(((uint64_t)hi << 32) | lo);
    }
    return v;
}

// Shared-column counters of one row.  Most rows touch a few thousand others at most: the TABLE pass counts those in
// an LDS hash table (open addressing; a key is claimed with compare-and-swap, then its count is bumped) and puts a row
// that touches more on a list.  The dense pass (TABLE = false, no LDS, more workgroups per CU) then takes the heavy
// rows and that list, counting in the workgroup's dense array of m counters in device memory.
template <bool TABLE>
__global__ __launch_bounds__(256) void cbm_candidates_kernel(const CandArgs a) {
    extern __shared__ int s_table[];  // kHashSlots keys (-1 = free), then kHashSlots counts
    int* s_key = s_table;
    unsigned* s_cnt = reinterpret_cast<unsigned*>(s_table + kHashSlots);
    __shared__ unsigned long long s_row;
    __shared__ unsigned s_ntouched, s_npass, s_nhub, s_distinct, s_overflow;
    __shared__ unsigned long long s_sel[kSelMax];
    __shared__ long long s_saving[kSelMax];
    __shared__ unsigned long long s_red[4];
    uint32_t* cnt = a.cnt + (size_t)blockIdx.x * a.m;
    int32_t* touched = a.touched + (size_t)blockIdx.x * a.m;
    unsigned long long* pass = a.pass + (size_t)blockIdx.x * a.m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (TABLE)
        for (int i = tid; i < kHashSlots; i += 256) {
            s_key[i] = -1;
            s_cnt[i] = 0;
        }
    // work list: TABLE: order[nheavy..m); dense: order[0..nheavy), then the rows the table pass gave up on
    const unsigned long long nwork = TABLE ? (unsigned long long)(a.m - a.nheavy) : (unsigned long long)a.nheavy + *a.noverflow;

    for (;;) {
        __syncthreads();  // everyone is done with the shared state of the previous row
        if (tid == 0) {
            s_row = atomicAdd(a.next, 1ull);
            s_ntouched = 0;
            s_npass = 0;
            s_nhub = 0;
            s_distinct = 0;
            s_overflow = 0;
        }
        __syncthreads();
        if (s_row >= nwork) return;  // the queue only grows: every workgroup gets here
        const int32_t x = TABLE ? a.order[a.nheavy + s_row]
                                : s_row < (unsigned long long)a.nheavy ? a.order[s_row] : a.overflow[s_row - a.nheavy];
        const int64_t xb = a.rowptr[x], nx = a.rowptr[x + 1] - xb;
        if (nx < 1) {
            if (tid == 0) a.out_n[x] = 0;
            continue;
        }
        const int grp = tid >> 4, gl = tid & 15;
        constexpr bool in_lds = TABLE;

        // 1a. count shared columns in the LDS table: a column per group of 16 lanes, the column's rows over the lanes
        if (in_lds) {
            unsigned myhub = 0;
            volatile unsigned* overflow = &s_overflow;  // set by any lane, read by all: never kept in a register
            for (int64_t p = grp; p < nx && !*overflow; p += 16) {
                const int32_t j = a.colidx[xb + p];
                const int64_t tb = a.tptr[j], deg = a.tptr[j + 1] - tb;
                if (a.hub_cap >= 0 && deg > a.hub_cap) {
                    if (gl == 0) ++myhub;
                    continue;
                }
                for (int64_t q = gl; q < deg && !*overflow; q += 16) {
                    const int32_t y = a.trow[tb + q];
                    unsigned slot = ((unsigned)y * 2654435761u) >> (32 - kHashBits);
                    // The table always keeps free slots (kHashLimit), so a probe sequence meets one; the bound on
                    // the walk makes the loop end whatever happens, and a row that hits it is counted again densely.
                    int probe = 0;
                    for (; probe < kHashSlots; ++probe) {
                        int key = *(volatile int*)&s_key[slot];
                        if (key == -1) key = atomicCAS(&s_key[slot], -1, y);
                        if (key == -1 || key == y) {
                            atomicAdd(&s_cnt[slot], 1u);
                            if (key == -1 && atomicAdd(&s_distinct, 1u) >= kHashLimit) *overflow = 1;
                            break;
                        }
                        slot = (slot + 1) & (kHashSlots - 1);
                    }
                    if (probe == kHashSlots) *overflow = 1;
                }
            }
            if (myhub) atomicAdd(&s_nhub, myhub);
            __syncthreads();
            if (*overflow) {  // too many distinct rows: empty the table and leave this row to the dense pass
                for (int i = tid; i < kHashSlots; i += 256) {
                    s_key[i] = -1;
                    s_cnt[i] = 0;
                }
                if (tid == 0) a.overflow[atomicAdd(a.noverflow, 1ull)] = x;
                continue;
            }
        }

        // 1b. ... or in the dense array
        if (!in_lds) {
            unsigned myhub = 0;
            for (int64_t p = grp; p < nx; p += 16) {
                const int32_t j = a.colidx[xb + p];
                const int64_t tb = a.tptr[j], deg = a.tptr[j + 1] - tb;
                if (a.hub_cap >= 0 && deg > a.hub_cap) {  // a hub column: too many rows to expand
                    if (gl == 0) ++myhub;
                    continue;
                }
                for (int64_t q = gl; q < deg; q += 64) {  // four counters in flight per lane
                    int32_t y[4];
                    uint32_t old[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) y[u] = q + 16 * u < deg ? a.trow[tb + q + 16 * u] : -1;
#pragma unroll
                    for (int u = 0; u < 4; ++u) old[u] = y[u] >= 0 ? atomicAdd(&cnt[y[u]], 1u) : 1u;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (old[u] == 0u) touched[atomicAdd(&s_ntouched, 1u)] = y[u];
                }
            }
            if (myhub) atomicAdd(&s_nhub, myhub);
            __syncthreads();
        }
        const unsigned ntouched = in_lds ? (unsigned)kHashSlots : s_ntouched;
        const int64_t nhub = s_nhub;

        // 2. score what was touched (upper bound of the saving where hub columns were skipped) and leave every counter
        //    zero for the next row: table slots are read and freed; a dense counter is read and cleared by one
        //    exchange, where the atomics counted it
        for (unsigned i = tid; i < ntouched; i += 256) {
            int32_t y;
            int64_t shared;
            if (in_lds) {
                y = s_key[i];
                if (y == -1) continue;
                shared = (int64_t)s_cnt[i];
                s_key[i] = -1;
                s_cnt[i] = 0;
            } else {
                y = touched[i];
                shared = (int64_t)atomicExch(&cnt[y], 0u);
            }
            if (y == x) continue;
            const int64_t ny = a.rowptr[y + 1] - a.rowptr[y];
            const int64_t room = (ny < nx ? ny : nx) - shared;  // columns the two rows could still share among the hubs
            const int64_t most = shared + (nhub < room ? nhub : room);
            const int64_t ub = 2 * most - ny;  // saving = nnz(a_x) - w(y,x) = 2 |a_x n a_y| - nnz(a_y)
            if (ub >= a.min_saving) pass[atomicAdd(&s_npass, 1u)] = make_key(ub, y);
        }
        __syncthreads();
        const unsigned npass = s_npass;
        if (npass == 0) {
            if (tid == 0) a.out_n[x] = 0;
            continue;
        }

        // 3. the best `nsel` of them: all, or repeated maximum below the previous maximum (keys are distinct)
        const unsigned want = (unsigned)(nhub > 0 ? 2 * a.keep : a.keep);
        const unsigned nsel = npass < want ? npass : want;
        if (npass <= nsel) {
            for (unsigned i = tid; i < npass; i += 256) s_sel[i] = pass[i];
        } else {
            unsigned long long bound = ~0ull;
            for (unsigned r = 0; r < nsel; ++r) {
                unsigned long long best = 0;
                for (unsigned i = tid; i < npass; i += 256) {
                    const unsigned long long key = pass[i];
                    if (key < bound && key > best) best = key;
                }
                best = wave_max(best);
                if (lane == 0) s_red[wave] = best;
                __syncthreads();
                best = s_red[0];
                for (int w = 1; w < 4; ++w) best = s_red[w] > best ? s_red[w] : best;
                if (tid == 0) s_sel[r] = best;
                bound = best;
                __syncthreads();
            }
        }
        __syncthreads();

        // 4. where hub columns were skipped, the exact saving by list intersection: a candidate per wave,
        //    the shorter list searched in the longer
        if (nhub > 0) {
            for (unsigned s = wave; s < nsel; s += 4) {
                const int32_t y = key_row(s_sel[s]);
                const int64_t yb = a.rowptr[y], ny = a.rowptr[y + 1] - yb;
                const int32_t* sh = a.colidx + xb;
                const int32_t* lg = a.colidx + yb;
                int64_t nsh = nx, nlg = ny;
                if (nlg < nsh) {
                    const int32_t* t = sh;
                    sh = lg;
                    lg = t;
                    nsh = ny;
                    nlg = nx;
                }
                int64_t found = 0;
                for (int64_t i = lane; i < nsh; i += 64) {
                    const int32_t v = sh[i];
                    int64_t lo = 0, hi = nlg;
                    while (lo < hi) {
                        const int64_t mid = (lo + hi) >> 1;
                        if (lg[mid] < v)
                            lo = mid + 1;
                        else
                            hi = mid;
                    }
                    found += (lo < nlg && lg[lo] == v);
                }
                found = wave_sum(found);
                if (lane == 0) s_saving[s] = 2 * found - ny;
            }
        } else {
            for (unsigned s = tid; s < nsel; s += 256) s_saving[s] = (long long)(s_sel[s] >> 32);
        }
        __syncthreads();

        // 5. the best `keep` by exact saving (ties: smaller row index)
        if (tid == 0) {
            unsigned long long fin[kSelMax];
            int nf = 0;
            for (unsigned s = 0; s < nsel; ++s)
                if (s_saving[s] >= a.min_saving) fin[nf++] = make_key(s_saving[s], key_row(s_sel[s]));
            for (int i = 1; i < nf; ++i) {  // insertion sort, descending
                const unsigned long long key = fin[i];
                int j = i - 1;
                while (j >= 0 && fin[j] < key) {
                    fin[j + 1] = fin[j];
                    --j;
                }
                fin[j + 1] = key;
            }
            const int nout = nf < a.keep ? nf : a.keep;
            for (int i = 0; i < nout; ++i) {
                a.out_y[(int64_t)x * a.keep + i] = key_row(fin[i]);
                a.out_w[(int64_t)x * a.keep + i] = (int32_t)(nx - (int64_t)(fin[i] >> 32));
            }
            a.out_n[x] = nout;
        }
    }
}


// ---- delta lists (Eq. (2)) on the GPU -----------------------------------------------------------------
// One wave per row x with tree parent y: Delta+ = a_x \ a_y, Delta- = a_y \ a_x.  Both lists are sorted, so
// membership is a binary search in the other list; a wave takes 64 elements at a time, and the elements that
// are NOT found keep their order in the output (ballot + prefix count).  COUNT = true only counts.
__device__ __forceinline__ bool sorted_contains(const int32_t* __restrict__ a, int64_t n, int32_t v) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1; else hi = mid;
    }
    return lo < n && a[lo] == v;
}

template <bool COUNT>
__global__ __launch_bounds__(256) void cbm_delta_kernel(int64_t m, const int64_t* __restrict__ rowptr,
                                                        const int32_t* __restrict__ colidx,
                                                        const int32_t* __restrict__ parent, int32_t* __restrict__ nplus,
                                                        int32_t* __restrict__ nminus, const int64_t* __restrict__ dptr,
                                                        uint32_t* __restrict__ dcol) {
    const int64_t x = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (x >= m) return;
    const int lane = threadIdx.x & 63;
    const int32_t y = parent[x];
    const int32_t* ax = colidx + rowptr[x];
    const int64_t nx = rowptr[x + 1] - rowptr[x];
    if (y < 0) {  // compressed against the virtual null row: the row itself
        if (COUNT) {
            if (lane == 0) {
                nplus[x] = (int32_t)nx;
                nminus[x] = 0;
            }
        } else {
            for (int64_t i = lane; i < nx; i += 64) dcol[dptr[x] + i] = (uint32_t)ax[i];
        }
        return;
    }
    const int32_t* ay = colidx + rowptr[y];
    const int64_t ny = rowptr[y + 1] - rowptr[y];
    int64_t at = COUNT ? 0 : dptr[x];
    int32_t count[2] = {0, 0};
    for (int side = 0; side < 2; ++side) {  // 0: elements of a_x missing from a_y; 1: elements of a_y missing from a_x
        const int32_t* a = side ? ay : ax;
        const int32_t* b = side ? ax : ay;
        const int64_t na = side ? ny : nx, nb = side ? nx : ny;
        for (int64_t i0 = 0; i0 < na; i0 += 64) {
            const int64_t i = i0 + lane;
            const int32_t v = i < na ? a[i] : 0;
            const bool out = i < na && !sorted_contains(b, nb, v);
            const unsigned long long mask = __ballot(out);
            if (!COUNT && out)
                dcol[at + __popcll(mask & ((1ull << lane) - 1ull))] = (uint32_t)v | (side ? CBM_DELTA_MINUS : 0u);
            at += __popcll(mask);
            count[side] += __popcll(mask);
        }
    }
    if (COUNT && lane == 0) {
        nplus[x] = count[0];
        nminus[x] = count[1];
    }
}

struct DeviceBuffers {
    std::vector<void*> ptrs;
    ~DeviceBuffers() {
        for (void* p : ptrs) hipFree(p);
    }
    template <typename T>
    hipError_t alloc(T** out, size_t count) {
        *out = nullptr;
        hipError_t e = hipMalloc((void**)out, std::max<size_t>(count, 1) * sizeof(T));
        if (e == hipSuccess) ptrs.push_back(*out);
        return e;
    }
};

#define CAND_TRY(call, status)                                     \
    do {                                                          \
        hipError_t err_ = (call);                                 \
        if (err_ != hipSuccess) {                                 \
            cbm_set_error_detail(#call, hipGetErrorString(err_)); \
            if (cur != dev) hipSetDevice(cur);                    \
            return (status);                                      \
        }                                                         \
    } while (0)

}  // namespace

cbm_status cbm_device_candidates(int device, int64_t m, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                                 const int64_t* tptr, const int32_t* trow, int64_t hub_cap, int64_t min_saving,
                                 int32_t keep, std::vector<int32_t>* out_n, std::vector<int32_t>* out_y,
                                 std::vector<int32_t>* out_w) {
    if (keep < 1 || keep > kCandMax) return CBM_ERR_INVALID_ARG;
    out_n->assign(m, 0);
    out_y->assign((size_t)m * keep, 0);
    out_w->assign((size_t)m * keep, 0);
    if (m == 0) return CBM_OK;
    int cur = -1, dev = device;
    {
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) {
            cbm_set_error_detail("hipGetDevice", hipGetErrorString(e));
            return CBM_ERR_HIP;
        }
    }
    if (dev < 0) dev = cur;
    if (cur != dev) CAND_TRY(hipSetDevice(dev), CBM_ERR_HIP);
    const int64_t nnz = rowptr[m];
    const bool verbose = std::getenv("CBM_VERBOSE") != nullptr;
    auto last = std::chrono::steady_clock::now();
    auto lap = [&](const char* what) {
        const auto now = std::chrono::steady_clock::now();
        if (verbose)
            std::fprintf(stderr, "[cbm_build]   device candidates: %-18s %.3f s\n", what,
                         std::chrono::duration<double>(now - last).count());
        last = now;
    };

    // heaviest rows first: the expansion of row x touches sum over its non-hub columns of the column's rows
    std::vector<int32_t> order(m);
    int64_t nheavy = 0;
    {
        std::vector<int64_t> work(m);
        const int nt = (int)std::max(1u, std::min(32u, std::thread::hardware_concurrency()));
        std::vector<std::thread> pool;
        for (int t = 0; t < nt; ++t)
            pool.emplace_back([&, t] {
                for (int64_t x = m * t / nt; x < m * (t + 1) / nt; ++x) {
                    int64_t w = 0;
                    for (int64_t p = rowptr[x]; p < rowptr[x + 1]; ++p) {
                        const int64_t deg = tptr[colidx[p] + 1] - tptr[colidx[p]];
                        if (hub_cap < 0 || deg <= hub_cap) w += deg;
                    }
                    work[x] = w;
                }
            });
        for (auto& th : pool) th.join();
        // Which rows go straight to the dense counters?  A row whose expansion is shorter than the table is safe in the
        // table.  In between it depends on the graph: where neighbourhoods overlap (the expansion of a row of a
        // nearest-neighbour graph revisits the same few thousand rows) the table holds rows that expand to a quarter of
        // a million; where they do not (power-law graphs) such rows overflow it.  Count the distinct rows of a few.
        int64_t heavy_from = 1 << 18;
        {
            std::vector<int32_t> mid;
            for (int64_t x = 0; x < m; ++x)
                if (work[x] >= (int64_t)kHashLimit && work[x] < heavy_from) mid.push_back((int32_t)x);
            const size_t nsample = std::min<size_t>(48, mid.size());
            size_t spilled = 0;
            std::vector<uint8_t> seen(nsample ? m : 0, 0);
            std::vector<int32_t> hit;
            for (size_t i = 0; i < nsample; ++i) {
                const int32_t x = mid[i * mid.size() / nsample];
                hit.clear();
                for (int64_t p = rowptr[x]; p < rowptr[x + 1]; ++p) {
                    const int32_t j = colidx[p];
                    if (hub_cap >= 0 && tptr[j + 1] - tptr[j] > hub_cap) continue;
                    for (int64_t q = tptr[j]; q < tptr[j + 1]; ++q)
                        if (!seen[trow[q]]) {
                            seen[trow[q]] = 1;
                            hit.push_back(trow[q]);
                        }
                }
                spilled += hit.size() > kHashLimit;
                for (int32_t y : hit) seen[y] = 0;
            }
            if (nsample > 0 && 2 * spilled >= nsample) heavy_from = kHashLimit;
        }
        std::vector<std::pair<int64_t, int32_t>> heavy;
        size_t w = 0;
        for (int64_t x = 0; x < m; ++x)
            if (work[x] >= heavy_from) heavy.push_back({work[x], (int32_t)x});
        std::sort(heavy.begin(), heavy.end(), [](const auto& p, const auto& q) { return p.first > q.first; });
        nheavy = (int64_t)heavy.size();
        for (auto& p : heavy) order[w++] = p.second;
        for (int64_t x = 0; x < m; ++x)
            if (work[x] < heavy_from) order[w++] = (int32_t)x;
    }
    lap("row order");
    // one counter array, one touched list and one key list of m entries per workgroup
    size_t free_b = 0, total_b = 0;
    CAND_TRY(hipMemGetInfo(&free_b, &total_b), CBM_ERR_HIP);
    const size_t fixed = (size_t)(m + 1) * 8 + (size_t)nnz * 4 + (size_t)(n + 1) * 8 + (size_t)nnz * 4 + (size_t)m * 4 +
                         (size_t)m * 4 * (1 + 2 * (size_t)keep);
    const size_t per_wg = (size_t)m * 16;
    const size_t budget = std::min<size_t>((size_t)24 << 30, free_b / 2 > fixed ? free_b / 2 - fixed : 0);
    int64_t nwg = (int64_t)std::min<size_t>(1024, budget / per_wg);
    nwg = std::min<int64_t>(nwg, m);
    if (nwg < 1) {
        cbm_set_error_detail("cbm_device_candidates", "not enough device memory for one workgroup's counters");
        if (cur != dev) hipSetDevice(cur);
        return CBM_ERR_ALLOC;
    }

    DeviceBuffers buf;
    CandArgs a{};
    int64_t *d_rowptr, *d_tptr;
    int32_t *d_colidx, *d_trow, *d_order;
    CAND_TRY(buf.alloc(&d_rowptr, m + 1), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_colidx, nnz), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_tptr, n + 1), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_trow, nnz), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_order, m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.next, 2), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.overflow, m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.cnt, (size_t)nwg * m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.touched, (size_t)nwg * m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.pass, (size_t)nwg * m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.out_n, m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.out_y, (size_t)m * keep), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&a.out_w, (size_t)m * keep), CBM_ERR_ALLOC);
    CAND_TRY(hipMemcpy(d_rowptr, rowptr, (size_t)(m + 1) * 8, hipMemcpyHostToDevice), CBM_ERR_HIP);
    if (nnz > 0) {
        CAND_TRY(hipMemcpy(d_colidx, colidx, (size_t)nnz * 4, hipMemcpyHostToDevice), CBM_ERR_HIP);
        CAND_TRY(hipMemcpy(d_trow, trow, (size_t)nnz * 4, hipMemcpyHostToDevice), CBM_ERR_HIP);
    }
    CAND_TRY(hipMemcpy(d_tptr, tptr, (size_t)(n + 1) * 8, hipMemcpyHostToDevice), CBM_ERR_HIP);
    CAND_TRY(hipMemcpy(d_order, order.data(), (size_t)m * 4, hipMemcpyHostToDevice), CBM_ERR_HIP);
    CAND_TRY(hipMemset(a.next, 0, 2 * sizeof(unsigned long long)), CBM_ERR_HIP);
    a.noverflow = a.next + 1;
    CAND_TRY(hipMemset(a.cnt, 0, (size_t)nwg * m * sizeof(uint32_t)), CBM_ERR_HIP);
    CAND_TRY(hipDeviceSynchronize(), CBM_ERR_HIP);
    lap("alloc + upload");
    a.m = m;
    a.rowptr = d_rowptr;
    a.colidx = d_colidx;
    a.tptr = d_tptr;
    a.trow = d_trow;
    a.order = d_order;
    a.nheavy = nheavy;
    a.hub_cap = hub_cap;
    a.min_saving = min_saving;
    a.keep = keep;
    const size_t lds = (size_t)kHashSlots * 8;
    CAND_TRY(hipFuncSetAttribute((const void*)cbm_candidates_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
             CBM_ERR_HIP);
    hipLaunchKernelGGL(cbm_candidates_kernel<true>, dim3((unsigned)nwg), dim3(256), lds, 0, a);
    CAND_TRY(hipGetLastError(), CBM_ERR_HIP);
    if (verbose) {
        CAND_TRY(hipDeviceSynchronize(), CBM_ERR_HIP);
        unsigned long long nov = 0;
        CAND_TRY(hipMemcpy(&nov, a.noverflow, sizeof(nov), hipMemcpyDeviceToHost), CBM_ERR_HIP);
        std::fprintf(stderr, "[cbm_build]   device candidates: %ld heavy rows, %llu rows left by the table pass\n", (long)nheavy, nov);
        lap("table pass");
    }
    CAND_TRY(hipMemsetAsync(a.next, 0, sizeof(unsigned long long), 0), CBM_ERR_HIP);  // the dense pass has its own queue
    hipLaunchKernelGGL(cbm_candidates_kernel<false>, dim3((unsigned)nwg), dim3(256), 0, 0, a);
    CAND_TRY(hipGetLastError(), CBM_ERR_HIP);
    CAND_TRY(hipDeviceSynchronize(), CBM_ERR_HIP);
    lap("dense pass");
    CAND_TRY(hipMemcpy(out_n->data(), a.out_n, (size_t)m * 4, hipMemcpyDeviceToHost), CBM_ERR_HIP);
    CAND_TRY(hipMemcpy(out_y->data(), a.out_y, (size_t)m * keep * 4, hipMemcpyDeviceToHost), CBM_ERR_HIP);
    CAND_TRY(hipMemcpy(out_w->data(), a.out_w, (size_t)m * keep * 4, hipMemcpyDeviceToHost), CBM_ERR_HIP);
    lap("download");
    if (cur != dev) hipSetDevice(cur);
    return CBM_OK;
}

// Delta lists of every tree edge on the GPU: the same lists, in the same order, as the host merge.
cbm_status cbm_device_deltas(int device, int64_t m, const int64_t* rowptr, const int32_t* colidx, const int32_t* parent,
                             std::vector<int32_t>* nplus, std::vector<int32_t>* nminus, std::vector<int64_t>* dptr,
                             std::vector<uint32_t>* dcol) {
    nplus->assign(m, 0);
    nminus->assign(m, 0);
    dptr->assign(m + 1, 0);
    dcol->clear();
    if (m == 0) return CBM_OK;
    int cur = -1, dev = device;
    {
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) {
            cbm_set_error_detail("hipGetDevice", hipGetErrorString(e));
            return CBM_ERR_HIP;
        }
    }
    if (dev < 0) dev = cur;
    if (cur != dev) CAND_TRY(hipSetDevice(dev), CBM_ERR_HIP);
    const int64_t nnz = rowptr[m];
    DeviceBuffers buf;
    int64_t *d_rowptr = nullptr, *d_dptr = nullptr;
    int32_t *d_colidx = nullptr, *d_parent = nullptr, *d_np = nullptr, *d_nm = nullptr;
    uint32_t* d_dcol = nullptr;
    CAND_TRY(buf.alloc(&d_rowptr, (size_t)m + 1), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_colidx, (size_t)nnz), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_parent, (size_t)m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_np, (size_t)m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_nm, (size_t)m), CBM_ERR_ALLOC);
    CAND_TRY(buf.alloc(&d_dptr, (size_t)m + 1), CBM_ERR_ALLOC);
    CAND_TRY(hipMemcpy(d_rowptr, rowptr, ((size_t)m + 1) * 8, hipMemcpyHostToDevice), CBM_ERR_HIP);
    if (nnz > 0) CAND_TRY(hipMemcpy(d_colidx, colidx, (size_t)nnz * 4, hipMemcpyHostToDevice), CBM_ERR_HIP);
    CAND_TRY(hipMemcpy(d_parent, parent, (size_t)m * 4, hipMemcpyHostToDevice), CBM_ERR_HIP);
    const dim3 grid((unsigned)((m + 3) / 4));
    hipLaunchKernelGGL(cbm_delta_kernel<true>, grid, dim3(256), 0, 0, m, d_rowptr, d_colidx, d_parent, d_np, d_nm,
                       (const int64_t*)nullptr, (uint32_t*)nullptr);
    CAND_TRY(hipGetLastError(), CBM_ERR_HIP);
    CAND_TRY(hipMemcpy(nplus->data(), d_np, (size_t)m * 4, hipMemcpyDeviceToHost), CBM_ERR_HIP);
    CAND_TRY(hipMemcpy(nminus->data(), d_nm, (size_t)m * 4, hipMemcpyDeviceToHost), CBM_ERR_HIP);
    for (int64_t x = 0; x < m; ++x) (*dptr)[x + 1] = (*dptr)[x] + (*nplus)[x] + (*nminus)[x];
    const int64_t nd = (*dptr)[m];
    dcol->resize((size_t)nd);
    if (nd > 0) {
        CAND_TRY(buf.alloc(&d_dcol, (size_t)nd), CBM_ERR_ALLOC);
        CAND_TRY(hipMemcpy(d_dptr, dptr->data(), ((size_t)m + 1) * 8, hipMemcpyHostToDevice), CBM_ERR_HIP);
        hipLaunchKernelGGL(cbm_delta_kernel<false>, grid, dim3(256), 0, 0, m, d_rowptr, d_colidx, d_parent, d_np, d_nm,
                           (const int64_t*)d_dptr, d_dcol);
        CAND_TRY(hipGetLastError(), CBM_ERR_HIP);
        CAND_TRY(hipMemcpy(dcol->data(), d_dcol, (size_t)nd * 4, hipMemcpyDeviceToHost), CBM_ERR_HIP);
    }
    if (cur != dev) hipSetDevice(cur);
    return CBM_OK;
}

// CBM product kernels for gfx950 (wave64) and their launch logic.
//
// The compression tree is cut into vertical paths; a path is one work item, and the paths whose head
// hangs off a row of a round-r path form round r + 1: one launch per round (Algorithm 1 visits tree
// edges in topological order; work items of one round do not depend on each other).  A launch fuses
// the two stages of Section 2.2: for each row x of a path
//     Y[x,:] = Y[r_x,:] + sum_{j in Delta+} X[j,:] - sum_{j in Delta-} X[j,:]        (Eq. (5))
// with the running sum kept in registers from row to row, so a compressed row costs at most one
// parent-row read, never a read-modify-write.  A group of LANES lanes owns one work item and four
// columns per lane; a wave carries 64/LANES work items.  Entries are fetched
// cooperatively (one coalesced load per LANES entries) and broadcast inside the group.
// Long rows are cut into segments by column range, one range per XCD, summed by a combine launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "cbm_internal.h"

#define HIP_TRY(call, status)                                      \
    do {                                                          \
        hipError_t err_ = (call);                                 \
        if (err_ != hipSuccess) {                                 \
            cbm_set_error_detail(#call, hipGetErrorString(err_)); \
            return (status);                                      \
        }                                                         \
    } while (0)

// Partial sums of split rows for cbm_spmm_noalloc: the callers of that entry point cannot allocate, so the
// library brings this array along.  Every GPU the library runs on holds its own copy until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress -- never a device address.
#define CBM_STATIC_SCRATCH_FLOATS (16 * 1024 * 1024)  // 64 MiB
static __device__ __align__(256) float cbm_static_scratch[CBM_STATIC_SCRATCH_FLOATS];

namespace {

// device address of cbm_static_scratch on each GPU (each holds the array at an address of its own)
constexpr int kMaxDevices = 64;
float* g_static_scratch[kMaxDevices] = {};
std::mutex g_static_scratch_mutex;

// Address of the static scratch on `device`, which must be the current device; resolved once per device.
cbm_status static_scratch_address(int device, float** out) {
    if (device < 0 || device >= kMaxDevices) return CBM_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[device]) {
        float* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(cbm_static_scratch)), CBM_ERR_HIP);
        if (!ptr) {
            cbm_set_error_detail("hipGetSymbolAddress(cbm_static_scratch)", "null address");
            return CBM_ERR_HIP;
        }
        g_static_scratch[device] = ptr;
    }
    *out = g_static_scratch[device];
    return CBM_OK;
}

// Four columns of a row: what one lane holds.
struct alignas(16) Vec4 {
    float v[4];
};
typedef float float4a __attribute__((ext_vector_type(4)));

// Which four columns a lane holds, and how it moves them.
// RAGGED = false: k is a multiple of 4 and every row starts on a 16-byte boundary; lane l of a group holds the
// consecutive columns 4l .. 4l+3 of the group's column chunk: one aligned 128-bit access.
// RAGGED = true: any k, leading dimension and base address; lane l holds columns l, l + LANES, l + 2 LANES,
// l + 3 LANES of the chunk, so every access is a 32-bit one that the group's lanes make to consecutive words.
template <bool RAGGED, int LANES>
__device__ __forceinline__ Vec4 ld_row(const float* row, int c0, int k) {
    Vec4 r;
    if (!RAGGED) {
        const float4a t = *reinterpret_cast<const float4a*>(row + c0);
#pragma unroll
        for (int c = 0; c < 4; ++c) r.v[c] = t[c];
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) r.v[c] = c0 + c * LANES < k ? row[c0 + c * LANES] : 0.0f;
    }
    return r;
}
// Streaming store: rows of Y and partial sums are written once and not re-read by the same launch, so
// they should not displace the gathered rows of X from L2.
template <bool RAGGED, int LANES>
__device__ __forceinline__ void st_row(float* row, int c0, int k, const Vec4& x) {
    if (!RAGGED) {
        float4a t;
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = x.v[c];
        __builtin_nontemporal_store(t, reinterpret_cast<float4a*>(row + c0));
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c0 + c * LANES < k) __builtin_nontemporal_store(x.v[c], row + c0 + c * LANES);
    }
}
// first column of lane `sl` in column chunk `chunk` (a chunk = 4 LANES columns either way)
template <bool RAGGED, int LANES>
__device__ __forceinline__ int first_column(int chunk, int sl) {
    return RAGGED ? chunk * 4 * LANES + sl : (chunk * LANES + sl) * 4;
}

// MODE 0: Y = M X (M = the compressed matrix).
// MODE 1: Y = D^-1/2 M D^-1/2 X with M = A v I (the normalised adjacency).  MODE 2: MODE 1 then max(., 0).
// MODE 3: Y = D^-1 M X (mean over each row's entries: the GraphSAGE mean aggregator).
// MODE 4: Y = M X + s X (s = 1 + eps: the GIN aggregator).
// Column weights multiply gathered rows, row weights the stored row; the self term of MODE 4 is the
// row's own X row, fetched by its marker entry like any gathered row.
// A row that ANOTHER work item is compressed against (INTERNAL) is written as the bare running sum,
// because that work item continues from it (the row scale belongs to the update step, Section 2.2);
// cbm_finish_kernel applies the row weight / self term to those rows once every round is done.
template <int MODE>
struct Mode {
    static constexpr bool wcol = MODE == 1 || MODE == 2;
    static constexpr bool wrow = MODE == 1 || MODE == 2 || MODE == 3;
    static constexpr bool relu = MODE == 2;
    static constexpr bool self = MODE == 4;
    static constexpr bool weights = wcol || wrow;
};

// out = finish(acc): acc (+ self_w * own X row) (* row weight) (then ReLU)
template <bool RAGGED, int LANES, int MODE>
__device__ __forceinline__ void store_row(float* row, int c0, int k, Vec4 acc, bool finish, float w, const Vec4& own,
                                          float self_w) {
    if (finish) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (Mode<MODE>::self) acc.v[c] = fmaf(self_w, own.v[c], acc.v[c]);
            if (Mode<MODE>::wrow) acc.v[c] *= w;
            if (Mode<MODE>::relu) acc.v[c] = fmaxf(acc.v[c], 0.0f);
        }
    }
    st_row<RAGGED, LANES>(row, c0, k, acc);
}

// One work item = one path of the compression tree (or one segment of a split row): start from
// the parent's row, walk the entry stream; a delta entry gathers a row of X, a marker entry stores
// the running sum as a finished row of Y and the walk goes on from the same registers.
//
// A group of LANES lanes owns the work item.  Entries are fetched LANES at a time (one coalesced
// load, two chunks ahead; their d^-1/2 weights one chunk ahead) and broadcast inside the group.
// X rows are loaded in batches of U; two batches ping-pong so that the loads of batch b+1 are in
// flight while batch b is accumulated: a long path is a chain of dependent adds, but never a chain
// of dependent loads.  Two builds of every variant: batches of 8 rows at 4 waves per SIMD for
// launches with few, long work items (the loads in flight come from inside each item), batches
// of 2 at 8 waves per SIMD for launches with many work items (they come from occupancy).
// Some launches map workgroups to work items per XCD: workgroup b runs on XCD b mod 8 and takes its
// items from that XCD's block of the task list -- the segments of one column range of X, or one share
// of a round whose work items were put in graph-locality order.
struct CbmSegMap {
    int64_t begin[CBM_XCD];
    int64_t count[CBM_XCD];
    int use;
};

// Waves per SIMD the register allocation is held to: 4 with batches of 8 rows, 8 with batches of 2 --
// one less for the few variants that would otherwise spill registers.
constexpr int level_min_waves(bool ragged, int lanes, int mode, int umax) {
    const bool weighted = mode >= 1 && mode <= 3;
    if (umax >= 8) return ((lanes == 16 || (ragged && lanes == 8)) && weighted) ? 3 : 4;
    return 8;
}

template <bool RAGGED, int LANES, int MODE, int UMAX>
__global__ __launch_bounds__(256, level_min_waves(RAGGED, LANES, MODE, UMAX)) void cbm_level_kernel(const CbmTask* __restrict__ tasks, int64_t ntasks,
                                                        const CbmSegMap map,
                                                        const uint32_t* __restrict__ stream,
                                                        const float* __restrict__ X, int64_t ldx, float* Y,
                                                        int64_t ldy, float* scratch, int64_t ld_scratch,
                                                        const float* __restrict__ ws, const float* __restrict__ rw,
                                                        float self_w, int k) {
    using M = Mode<MODE>;
    constexpr int G = 64 / LANES;                  // work items per wave
    constexpr int U = LANES < UMAX ? LANES : UMAX;  // X rows per batch
    constexpr int BPC = LANES / U;                  // batches per chunk of entries
    const int lane = threadIdx.x & 63;
    const int sub = lane / LANES;
    const int sl = lane % LANES;
    int64_t t;
    if (map.use) {
        const int xcd = blockIdx.x % CBM_XCD;  // gridDim.x is a multiple of 8, so this is the linear id mod 8
        const int64_t tl = ((int64_t)(blockIdx.x / CBM_XCD) * 4 + (threadIdx.x >> 6)) * G + sub;
        if (tl >= map.count[xcd]) return;
        t = map.begin[xcd] + tl;
    } else {
        t = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * G + sub;
        if (t >= ntasks) return;  // a whole group leaves together: no lane it exchanges with is gone
    }
    const CbmTask tk = tasks[t];
    const uint32_t len = tk.len_flags & CBM_TASK_LEN_MASK;
    const int c0 = first_column<RAGGED, LANES>(blockIdx.y, sl);
    const bool colok = c0 < k;

    Vec4 acc;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc.v[c] = 0.0f;
    if (tk.parent >= 0 && colok) acc = ld_row<RAGGED, LANES>(Y + (int64_t)tk.parent * ldy, c0, k);

    const uint32_t* es = stream + tk.start;
    // lanes past the end of the stream hold entry 0 with weight 0: a delta that is never loaded
    auto load_e = [&](int chunk) -> uint32_t {
        const uint32_t idx = (uint32_t)chunk * LANES + sl;
        return idx < len ? __builtin_nontemporal_load(es + idx) : 0u;  // read once: keep it out of the way of X
    };
    const float* wes = ws + tk.start;
    auto load_w = [&](uint32_t e, int chunk) -> float {  // signed column weight of a delta, row weight of a marker
        if (!M::weights) return 0.0f;
        const uint32_t idx = (uint32_t)chunk * LANES + sl;
        if (idx >= len) return 0.0f;
        if (M::wcol) return __builtin_nontemporal_load(wes + idx);  // stored per entry, beside the stream
        return (e & CBM_ENTRY_MARK) ? rw[e & CBM_ENTRY_INDEX_MASK] : 0.0f;
    };
    uint32_t e0 = load_e(0), e1 = load_e(1), e2 = load_e(2);
    float w0 = load_w(e0, 0), w1 = load_w(e1, 1);
    float wprev = 0.0f;  // weights of the chunk before the current one: its last batch is consumed after the rotation
    int cur = 0;         // chunk whose entries are in e0 / w0

    struct Batch {
        Vec4 x[U];
        uint32_t e[U];
    };
    const int nb = (int)((len + U - 1) / U);
    auto fetch = [&](Batch& S, int b) {
        if (b > 0 && b % BPC == 0) {  // batch b opens the next chunk: rotate the entry pipeline
            const int chunk = b / BPC;
            e0 = e1;
            wprev = w0;
            w0 = w1;
            e1 = e2;
            e2 = load_e(chunk + 2);
            w1 = load_w(e1, chunk + 1);
            cur = chunk;
        }
        const int off = (b % BPC) * U;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            S.e[u] = (uint32_t)__shfl((int)e0, off + u, LANES);
            // a delta gathers its column's row of X; in MODE 4 a marker gathers the row's own X row
            const bool gather = !(S.e[u] & CBM_ENTRY_MARK) ||
                                (M::self && !(S.e[u] & CBM_ENTRY_INTERNAL));
            if ((uint32_t)(b * U + u) < len && gather && colok) {
                S.x[u] = ld_row<RAGGED, LANES>(X + (int64_t)(S.e[u] & CBM_ENTRY_INDEX_MASK) * ldx, c0, k);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) S.x[u].v[c] = 0.0f;
            }
        }
    };
    auto consume = [&](const Batch& S, int b) {
        // weights are broadcast here, not at fetch time: one register per lane instead of U per batch
        const float wsrc = (b / BPC == cur) ? w0 : wprev;
        const int off = (b % BPC) * U;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float w = M::weights ? __shfl(wsrc, off + u, LANES) : 0.0f;
            if (S.e[u] & CBM_ENTRY_MARK) {
                if (colok)
                    store_row<RAGGED, LANES, MODE>(Y + (int64_t)(S.e[u] & CBM_ENTRY_INDEX_MASK) * ldy, c0, k, acc,
                                                   !(S.e[u] & CBM_ENTRY_INTERNAL), w, S.x[u], self_w);
            } else if (M::wcol) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc.v[c] = fmaf(w, S.x[u].v[c], acc.v[c]);
            } else {
                const uint32_t sgn = S.e[u] & CBM_DELTA_MINUS;
#pragma unroll
                for (int c = 0; c < 4; ++c) acc.v[c] += __uint_as_float(__float_as_uint(S.x[u].v[c]) ^ sgn);
            }
        }
    };
    Batch A, B;
    if (nb > 0) fetch(A, 0);
    for (int b = 0; b < nb; b += 2) {
        if (b + 1 < nb) fetch(B, b + 1);
        consume(A, b);
        if (b + 2 < nb) fetch(A, b + 2);
        if (b + 1 < nb) consume(B, b + 1);
    }
    // scratch rows (16-byte aligned, padded to a multiple of four columns) use the same lane-to-column map
    if ((tk.len_flags & CBM_TASK_SEGMENT) && colok)
        st_row<RAGGED, LANES>(scratch + (int64_t)tk.row * ld_scratch, c0, k, acc);
}

// Bundled paths.  The rows r_1 -> r_2 -> ... of a path are compressed against one another, so
//     Y[r_j,:] = Y[parent,:] + sum_{i <= j} ( sum_{Delta+(r_i)} X - sum_{Delta-(r_i)} X ).
// The kernel above walks them row by row: three or four short sweeps over the columns per work item, and work items at
// different rows of their paths ask for unrelated parts of X (26-34 % L2 hits against 71 % for a round of rows stored
// in full, which are one long sweep each).  Here ALL deltas of a path of at most CBM_BUNDLE_ROWS rows come in one
// ascending sweep, each tagged with the row it belongs to; the group keeps one partial sum per row and, when the deltas
// are done, forms the running sums and stores the rows (the path's markers follow its deltas in the stream).  Work
// items that start together then move through X together.  The sweep itself is a plain loop: no markers inside it.
// (waves per SIMD the register allocation is held to: the variants that would spill at four get three)
constexpr int bundle_min_waves(bool ragged, int lanes, int mode, int umax, int split) {
    return umax >= 8 ? (ragged || (lanes <= 16 && split == 1) ? 3 : 4) : 6;
}

// SPLIT = 2 or 4: a work item is shared by that many neighbouring groups of the wave, which take its deltas in turn
// (every SPLIT-th place) and add their partial sums across the groups at the end.  The item's gathers are the same, its
// chain of dependent batches 1/SPLIT as long, and a wave holds 1/SPLIT as many work items of unequal length.
template <bool RAGGED, int LANES, int MODE, int UMAX, int SPLIT>
__global__ __launch_bounds__(256, bundle_min_waves(RAGGED, LANES, MODE, UMAX, SPLIT)) void cbm_bundle_kernel(
    const CbmTask* __restrict__ tasks, int64_t ntasks, const CbmSegMap map, const uint32_t* __restrict__ stream,
    const float* __restrict__ X, int64_t ldx, float* Y, int64_t ldy, const float* __restrict__ ws, const float* __restrict__ rw,
    float self_w, int k) {
    using M = Mode<MODE>;
    constexpr int S = SPLIT;                      // groups per work item
    constexpr int G = 64 / LANES / S;             // work items per wave
    static_assert(G >= 1 && (S == 1 || S == 2 || S == 4), "the groups of a shared work item lie in one wave");
    constexpr int U = LANES / S < UMAX ? LANES / S : UMAX;  // rows a group loads per batch
    constexpr int BPC = LANES / (U * S);          // batches per chunk of LANES entries
    constexpr int R = CBM_BUNDLE_ROWS;
    static_assert(R == 4, "the choice among the partial sums below is written for four rows");
    const int lane = threadIdx.x & 63;
    const int sub = lane / LANES / S;             // the work item's place in the wave
    const int half = S > 1 ? (lane / LANES) & (S - 1) : 0;  // which of the item's groups
    const int sl = lane % LANES;
    int64_t t;
    if (map.use) {
        const int xcd = blockIdx.x % CBM_XCD;
        const int64_t tl = ((int64_t)(blockIdx.x / CBM_XCD) * 4 + (threadIdx.x >> 6)) * G + sub;
        if (tl >= map.count[xcd]) return;
        t = map.begin[xcd] + tl;
    } else {
        t = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * G + sub;
        if (t >= ntasks) return;
    }
    const CbmTask tk = tasks[t];
    const uint32_t total = tk.len_flags & CBM_TASK_LEN_MASK;
    // the last entries are the markers of the path's rows, in row order (1 .. R of them: the builder guarantees it)
    uint32_t nrows = 0;
#pragma unroll
    for (int s = 1; s <= R; ++s)
        if ((uint32_t)s <= total && (stream[tk.start + total - s] & CBM_ENTRY_MARK)) nrows = (uint32_t)s;
        else break;
    const uint32_t len = total - nrows;  // the deltas
    const int c0 = first_column<RAGGED, LANES>(blockIdx.y, sl);
    const bool colok = c0 < k;

    Vec4 run;  // the parent's row: the running sum starts there
#pragma unroll
    for (int c = 0; c < 4; ++c) run.v[c] = 0.0f;
    if (tk.parent >= 0 && colok) run = ld_row<RAGGED, LANES>(Y + (int64_t)tk.parent * ldy, c0, k);
    Vec4 acc[R];  // the partial sum of each row's own deltas
#pragma unroll
    for (int s = 0; s < R; ++s)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[s].v[c] = 0.0f;

    const uint32_t* es = stream + tk.start;
    const float* wes = ws + tk.start;
    auto load_e = [&](int chunk) -> uint32_t {
        const uint32_t idx = (uint32_t)chunk * LANES + sl;
        return idx < len ? __builtin_nontemporal_load(es + idx) : 0u;
    };
    auto load_w = [&](uint32_t e, int chunk) -> float {  // what the gathered row is multiplied by: +-d_j^-1/2, or +-1
        const uint32_t idx = (uint32_t)chunk * LANES + sl;
        if (idx >= len) return 0.0f;
        if (M::wcol) return __builtin_nontemporal_load(wes + idx);
        return __uint_as_float(0x3f800000u | (e & CBM_DELTA_MINUS));  // the fused multiply-add is then an exact add or subtract
    };
    uint32_t e0 = load_e(0), e1 = load_e(1), e2 = load_e(2);
    float w0 = load_w(e0, 0), w1 = load_w(e1, 1);
    float wprev = 0.0f;
    int cur = 0;

    struct Batch {
        Vec4 x[U];
        uint32_t e[U];
    };
    const int nb = (int)((len + U * S - 1) / (U * S));  // a batch = U entries for every group of the item
    auto fetch = [&](Batch& Bt, int b) {
        if (b > 0 && b % BPC == 0) {
            const int chunk = b / BPC;
            e0 = e1;
            wprev = w0;
            w0 = w1;
            e1 = e2;
            e2 = load_e(chunk + 2);
            w1 = load_w(e1, chunk + 1);
            cur = chunk;
        }
        const int off = (b % BPC) * U * S + half;  // this group's entries of the batch: every S-th from here
#pragma unroll
        for (int u = 0; u < U; ++u) {
            Bt.e[u] = (uint32_t)__shfl((int)e0, off + u * S, LANES);
            if ((uint32_t)(b * U * S + u * S + half) < len && colok) {
                Bt.x[u] = ld_row<RAGGED, LANES>(X + (int64_t)(Bt.e[u] & CBM_BUNDLE_INDEX_MASK) * ldx, c0, k);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) Bt.x[u].v[c] = 0.0f;
            }
        }
    };
    auto consume = [&](const Batch& Bt, int b) {
        const float wsrc = (b / BPC == cur) ? w0 : wprev;
        const int off = (b % BPC) * U * S + half;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float w = __shfl(wsrc, off + u * S, LANES);  // (0 past the end of the deltas, where the row is zero too)
            const uint32_t slot = (Bt.e[u] >> CBM_BUNDLE_SLOT_SHIFT) & (uint32_t)(R - 1);  // the same for the whole group
            auto add = [&](Vec4& a) {
#pragma unroll
                for (int c = 0; c < 4; ++c) a.v[c] = fmaf(w, Bt.x[u].v[c], a.v[c]);
            };
            if (slot & 2u) { if (slot & 1u) add(acc[3]); else add(acc[2]); }
            else { if (slot & 1u) add(acc[1]); else add(acc[0]); }
        }
    };
    Batch A, B;
    if (nb > 0) fetch(A, 0);
    for (int b = 0; b < nb; b += 2) {
        if (b + 1 < nb) fetch(B, b + 1);
        consume(A, b);
        if (b + 2 < nb) fetch(A, b + 2);
        if (b + 1 < nb) consume(B, b + 1);
    }
    if (S > 1) {  // the other groups' shares of every row's deltas (the same additions in every group: equal sums)
#pragma unroll
        for (int s2 = 0; s2 < R; ++s2)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                acc[s2].v[c] += __shfl_xor(acc[s2].v[c], LANES, 64);
                if (S > 2) acc[s2].v[c] += __shfl_xor(acc[s2].v[c], 2 * LANES, 64);
            }
    }
    // the rows of the path, in order: running sum, then the store its marker asks for (a wide item's two groups hold
    // the same sums and store alternate rows)
    uint32_t em[R];
    float wm[R];
    Vec4 own[R];
#pragma unroll
    for (int s = 0; s < R; ++s) {  // everything the stores need, in flight together
        em[s] = 0u;
        wm[s] = 0.0f;
#pragma unroll
        for (int c = 0; c < 4; ++c) own[s].v[c] = 0.0f;
        if ((uint32_t)s < nrows) {
            em[s] = es[len + s];
            if (M::wcol) wm[s] = wes[len + s];
        }
    }
#pragma unroll
    for (int s = 0; s < R; ++s) {
        if ((uint32_t)s < nrows) {
            const uint32_t row = em[s] & CBM_ENTRY_INDEX_MASK;
            if (!M::wcol && M::wrow) wm[s] = rw[row];
            if (M::self && !(em[s] & CBM_ENTRY_INTERNAL) && colok && (s & (S - 1)) == half)
                own[s] = ld_row<RAGGED, LANES>(X + (int64_t)row * ldx, c0, k);
        }
    }
#pragma unroll
    for (int s = 0; s < R; ++s) {
        if ((uint32_t)s < nrows) {
#pragma unroll
            for (int c = 0; c < 4; ++c) run.v[c] += acc[s].v[c];
            if (colok && (s & (S - 1)) == half)
                store_row<RAGGED, LANES, MODE>(Y + (int64_t)(em[s] & CBM_ENTRY_INDEX_MASK) * ldy, c0, k, run,
                                               !(em[s] & CBM_ENTRY_INTERNAL), wm[s], own[s], self_w);
        }
    }
}

// Rows whose delta list was cut into segments: Y[x,:] = Y[r_x,:] + sum of the row's segment sums.
template <bool RAGGED, int LANES, int MODE>
__global__ __launch_bounds__(256) void cbm_combine_kernel(const CbmTask* __restrict__ comb, int64_t ncomb,
                                                          const float* __restrict__ X, int64_t ldx, float* Y,
                                                          int64_t ldy, const float* scratch, int64_t ld_scratch,
                                                          const float* __restrict__ rw, float self_w, int k) {
    constexpr int G = 64 / LANES;
    const int lane = threadIdx.x & 63;
    const int64_t t = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * G + lane / LANES;
    const int c0 = first_column<RAGGED, LANES>(blockIdx.y, lane % LANES);
    if (t >= ncomb || c0 >= k) return;
    const CbmTask tk = comb[t];
    const uint32_t nseg = tk.len_flags & CBM_TASK_LEN_MASK;
    Vec4 acc;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc.v[c] = 0.0f;
    if (tk.parent >= 0) acc = ld_row<RAGGED, LANES>(Y + (int64_t)tk.parent * ldy, c0, k);
    const float* part = scratch + (int64_t)tk.start * ld_scratch;
    for (uint32_t s0 = 0; s0 < nseg; s0 += 8) {  // eight independent loads in flight, added in segment order
        Vec4 p[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (s0 + u < nseg) {
                p[u] = ld_row<RAGGED, LANES>(part + (int64_t)(s0 + u) * ld_scratch, c0, k);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) p[u].v[c] = 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc.v[c] += p[u].v[c];
    }
    const bool finish = !(tk.len_flags & CBM_TASK_INTERNAL);
    Vec4 own;
#pragma unroll
    for (int c = 0; c < 4; ++c) own.v[c] = 0.0f;
    if (Mode<MODE>::self && finish) own = ld_row<RAGGED, LANES>(X + (int64_t)tk.row * ldx, c0, k);
    store_row<RAGGED, LANES, MODE>(Y + (int64_t)tk.row * ldy, c0, k, acc, finish, Mode<MODE>::wrow ? rw[tk.row] : 1.0f, own,
                                   self_w);
}

// Deferred finish of the rows other work items were compressed against: row weight (MODE 1-3) or self term (MODE 4).
template <int MODE>
__global__ __launch_bounds__(256) void cbm_finish_kernel(const int32_t* __restrict__ rows, int64_t nrows,
                                                         const float* __restrict__ X, int64_t ldx, float* Y, int64_t ldy,
                                                         const float* __restrict__ rw, float self_w, int k) {
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= nrows) return;
    const int32_t x = rows[r];
    const float s = Mode<MODE>::wrow ? rw[x] : 1.0f;
    float* y = Y + (int64_t)x * ldy;
    for (int c = threadIdx.x & 63; c < k; c += 64) {
        float v = y[c];
        if (Mode<MODE>::self) v = fmaf(self_w, X[(int64_t)x * ldx + c], v);
        if (Mode<MODE>::wrow) v *= s;
        if (Mode<MODE>::relu) v = fmaxf(v, 0.0f);
        y[c] = v;
    }
}

// Weight of every stream entry for the normalised product: +-d_j^-1/2 for a delta on column j, d_x^-1/2 for the
// marker of row x.  Stored once per handle so that the product kernel reads weights as it reads entries --
// coalesced -- instead of gathering one word per delta.
__global__ __launch_bounds__(256) void cbm_entry_weights_kernel(const uint32_t* __restrict__ stream, int64_t nent,
                                                                const float* __restrict__ dinv, float* __restrict__ w,
                                                                uint32_t delta_mask) {  // 26 bits in a handle that bundles
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nent) return;
    const uint32_t e = stream[i];
    const float d = dinv[e & ((e & CBM_ENTRY_MARK) ? CBM_ENTRY_INDEX_MASK : delta_mask)];
    w[i] = (!(e & CBM_ENTRY_MARK) && (e & CBM_DELTA_MINUS)) ? -d : d;
}

// 256 CUs x 4 SIMDs x 8 waves = 8192 resident waves at most; from eight times that on, a launch is "many waves"
constexpr int64_t kManyWavesDefault = 65536;

struct LaunchCtx {
    const cbm_handle* h;
    const float* X;
    int64_t ldx;
    int k;
    float* Y;
    int64_t ldy;
    float* scratch;  // partial sums of split rows: the handle's own array, or the library's static one
    int64_t ld_scratch;
    hipStream_t stream;
    const float* ws;  // per-entry weights of the stream (MODE 1/2)
    const float* rw;  // row weights (MODE 1/2/3)
    float self_w;     // MODE 4
};

// launches of up to this many waves (counted with one group per work item) share every work item among four groups
constexpr int64_t kWideMaxWavesDefault = 32768;

inline int64_t wide_max_waves() {  // (read at every launch, so that a test can run both forms in one process)
    const char* e = std::getenv("CBM_WIDE_MAX_WAVES");
    return e ? std::atoll(e) : kWideMaxWavesDefault;
}

template <bool RAGGED, int LANES, int MODE, int UMAX, int SPLIT>
void launch_bundles_as(const LaunchCtx& c, const CbmLevel& L) {
    constexpr int G = 64 / LANES / SPLIT;
    const int ychunks = (c.k + LANES * 4 - 1) / (LANES * 4);
    CbmSegMap map{};
    if (L.by_xcd) {
        int64_t most = 0;
        for (int j = 0; j < CBM_XCD; ++j) {
            map.begin[j] = L.xcd_begin[j];
            map.count[j] = L.xcd_count[j];
            most = std::max(most, map.count[j]);
        }
        map.use = 1;
        dim3 grid((unsigned)(CBM_XCD * ((most + 4 * G - 1) / (4 * G))), (unsigned)ychunks);
        hipLaunchKernelGGL((cbm_bundle_kernel<RAGGED, LANES, MODE, UMAX, SPLIT>), grid, dim3(256), 0, c.stream, c.h->d_tasks,
                           (int64_t)c.h->tasks.size(), map, c.h->d_stream, c.X, c.ldx, c.Y, c.ldy, c.ws, c.rw, c.self_w, c.k);
        return;
    }
    dim3 grid((unsigned)((L.task_count + 4 * G - 1) / (4 * G)), (unsigned)ychunks);
    hipLaunchKernelGGL((cbm_bundle_kernel<RAGGED, LANES, MODE, UMAX, SPLIT>), grid, dim3(256), 0, c.stream, c.h->d_tasks + L.task_begin,
                       L.task_count, map, c.h->d_stream, c.X, c.ldx, c.Y, c.ldy, c.ws, c.rw, c.self_w, c.k);
}

template <bool RAGGED, int LANES, int MODE, int UMAX>
void launch_bundles(const LaunchCtx& c, const CbmLevel& L) {
    // Narrow feature matrices only (k <= 64: four or eight work items in a wave): the rounds of a tree are then short of
    // work and last as long as their longest item's chain of dependent batches, whatever k is (protein recipe: 0.43-0.47 ms
    // for every k from 8 to 64).  Four groups per item: 0.32 ms at k = 64, 0.28 ms at k <= 32.  With two work items in a
    // wave to begin with (k = 128, or 256 in chunks of 128) the rounds are bound by lines in flight and sharing items out
    // is a loss (0.80 -> 0.94 ms with two groups per item).
    if constexpr (LANES <= 16 && UMAX >= 8) {
        const int64_t ychunks = (c.k + LANES * 4 - 1) / (LANES * 4);
        if (L.task_count / (64 / LANES) * ychunks <= wide_max_waves()) return launch_bundles_as<RAGGED, LANES, MODE, UMAX, 4>(c, L);
    }
    launch_bundles_as<RAGGED, LANES, MODE, UMAX, 1>(c, L);
}

template <bool RAGGED, int LANES, int MODE, int UMAX>
void launch_level(const LaunchCtx& c, const CbmLevel& L) {
    constexpr int G = 64 / LANES;
    const int ychunks = (c.k + LANES * 4 - 1) / (LANES * 4);
    CbmSegMap map{};
    if (L.task_count <= 0) return;
    if (L.bundled) return launch_bundles<RAGGED, LANES, MODE, UMAX>(c, L);
    if constexpr (LANES <= 16 && UMAX >= 8) {
        // narrow X, a round of long single rows (the roots of a tree): the sweep kernel shares each row among four
        // groups of the wave; the kernel below would walk it with one (protein recipe, k = 64: that round 0.077 ms, the product
        // 0.317 -> 0.288 ms)
        const int64_t ychunks2 = (c.k + LANES * 4 - 1) / (LANES * 4);
        if (L.long_single_rows && L.task_count / (64 / LANES) * ychunks2 <= wide_max_waves())
            return launch_bundles_as<RAGGED, LANES, MODE, UMAX, 4>(c, L);
    }
    if (L.by_xcd) {  // one block of the (locality-ordered) work items per XCD
        int64_t most = 0;
        for (int j = 0; j < CBM_XCD; ++j) {
            map.begin[j] = L.xcd_begin[j];
            map.count[j] = L.xcd_count[j];
            most = std::max(most, map.count[j]);
        }
        map.use = 1;
        dim3 grid((unsigned)(CBM_XCD * ((most + 4 * G - 1) / (4 * G))), (unsigned)ychunks);
        hipLaunchKernelGGL((cbm_level_kernel<RAGGED, LANES, MODE, UMAX>), grid, dim3(256), 0, c.stream, c.h->d_tasks,
                           (int64_t)c.h->tasks.size(), map, c.h->d_stream, c.X, c.ldx, c.Y, c.ldy, c.scratch,
                           c.ld_scratch, c.ws, c.rw, c.self_w, c.k);
        return;
    }
    dim3 grid((unsigned)((L.task_count + 4 * G - 1) / (4 * G)), (unsigned)ychunks);
    hipLaunchKernelGGL((cbm_level_kernel<RAGGED, LANES, MODE, UMAX>), grid, dim3(256), 0, c.stream,
                       c.h->d_tasks + L.task_begin, L.task_count, map, c.h->d_stream, c.X, c.ldx, c.Y, c.ldy,
                       c.scratch, c.ld_scratch, c.ws, c.rw, c.self_w, c.k);
}
// all segments of all split rows, one block of work items per XCD
template <bool RAGGED, int LANES, int MODE, int UMAX>
void launch_segments(const LaunchCtx& c, const CbmLevel&) {
    constexpr int G = 64 / LANES;
    const int ychunks = (c.k + LANES * 4 - 1) / (LANES * 4);
    CbmSegMap map{};
    int64_t most = 0;
    for (int j = 0; j < CBM_XCD; ++j) {
        map.begin[j] = c.h->seg_begin[j];
        map.count[j] = c.h->seg_count[j];
        most = std::max(most, map.count[j]);
    }
    map.use = 1;
    dim3 grid((unsigned)(CBM_XCD * ((most + 4 * G - 1) / (4 * G))), (unsigned)ychunks);
    hipLaunchKernelGGL((cbm_level_kernel<RAGGED, LANES, MODE, UMAX>), grid, dim3(256), 0, c.stream, c.h->d_tasks,
                       (int64_t)c.h->tasks.size(), map, c.h->d_stream, c.X, c.ldx, c.Y, c.ldy, c.scratch,
                       c.ld_scratch, c.ws, c.rw, c.self_w, c.k);
}
template <bool RAGGED, int LANES, int MODE>
void launch_combine(const LaunchCtx& c, const CbmLevel& L) {
    constexpr int G = 64 / LANES;
    const int ychunks = (c.k + LANES * 4 - 1) / (LANES * 4);
    dim3 grid((unsigned)((L.comb_count + 4 * G - 1) / (4 * G)), (unsigned)ychunks);
    hipLaunchKernelGGL((cbm_combine_kernel<RAGGED, LANES, MODE>), grid, dim3(256), 0, c.stream,
                       c.h->d_comb + L.comb_begin, L.comb_count, c.X, c.ldx, c.Y, c.ldy, c.scratch,
                       c.ld_scratch, c.rw, c.self_w, c.k);
}

using LevelFn = void (*)(const LaunchCtx&, const CbmLevel&);
struct Variant {
    LevelFn level, combine, segments;  // batches of 8 rows
    LevelFn level_many, segments_many;  // batches of 2 rows, full occupancy: for launches of many work items
    int group;                          // work items per wave
};

template <bool RAGGED, int LANES, int MODE>
Variant variant() {
    return {launch_level<RAGGED, LANES, MODE, 8>, launch_combine<RAGGED, LANES, MODE>, launch_segments<RAGGED, LANES, MODE, 8>,
            launch_level<RAGGED, LANES, MODE, 2>, launch_segments<RAGGED, LANES, MODE, 2>, 64 / LANES};
}
template <bool RAGGED, int LANES>
Variant pick_mode(int mode) {
    switch (mode) {
        case 0: return variant<RAGGED, LANES, 0>();
        case 1: return variant<RAGGED, LANES, 1>();
        case 2: return variant<RAGGED, LANES, 2>();
        case 3: return variant<RAGGED, LANES, 3>();
        default: return variant<RAGGED, LANES, 4>();
    }
}
template <bool RAGGED>
Variant pick_lanes(int lanes, int mode) {
    switch (lanes) {
        case 8: return pick_mode<RAGGED, 8>(mode);
        case 16: return pick_mode<RAGGED, 16>(mode);
        case 32: return pick_mode<RAGGED, 32>(mode);
        default: return pick_mode<RAGGED, 64>(mode);
    }
}

struct ProfScope {
    const cbm_handle* h;
    hipStream_t s;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(const cbm_handle* h_, hipStream_t s_, cbm_launch_record rec) : h(h_), s(s_) {
        if (!h->profiling) return;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
            a = b = nullptr;
            return;
        }
        hipEventRecord(a, s);
        h->prof_records.push_back(rec);
    }
    ~ProfScope() {
        if (!a) return;
        hipEventRecord(b, s);
        h->prof_events.push_back(a);
        h->prof_events.push_back(b);
    }
};

}  // namespace

cbm_status cbm_upload(cbm_handle* h) {
    if (h->blocks > 1) {  // the format lives in the inner handle
        const cbm_status st = cbm_upload(h->inner);
        if (st != CBM_OK) return st;
        h->device = h->inner->device;
        h->on_device = true;
        return CBM_OK;
    }
    int dev = h->opts.device;
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur), CBM_ERR_HIP);
    if (dev < 0) dev = cur;
    if (cur != dev) HIP_TRY(hipSetDevice(dev), CBM_ERR_HIP);
    h->device = dev;
    auto up = [&](auto** dptr, const auto& vec) -> cbm_status {
        using T = std::remove_reference_t<decltype(**dptr)>;
        *dptr = nullptr;
        size_t bytes = vec.size() * sizeof(T);
        if (bytes == 0) bytes = sizeof(T);  // keep every pointer valid
        HIP_TRY(hipMalloc((void**)dptr, bytes), CBM_ERR_ALLOC);
        if (!vec.empty())
            HIP_TRY(hipMemcpy(*dptr, vec.data(), vec.size() * sizeof(T), hipMemcpyHostToDevice), CBM_ERR_HIP);
        return CBM_OK;
    };
    cbm_status st = CBM_OK;
    if ((st = up(&h->d_tasks, h->tasks)) != CBM_OK || (st = up(&h->d_comb, h->comb)) != CBM_OK ||
        (st = up(&h->d_stream, h->stream)) != CBM_OK || (st = up(&h->d_dinv, h->dinv)) != CBM_OK ||
        (st = up(&h->d_rinv, h->rinv)) != CBM_OK ||
        (st = up(&h->d_internal, h->internal_rows)) != CBM_OK) {
        cbm_release_device(h);
        if (cur != dev) hipSetDevice(cur);
        return st;
    }
    if (h->square_self_loops && !h->stream.empty()) {
        const int64_t nent = (int64_t)h->stream.size();
        hipError_t e = hipMalloc((void**)&h->d_wstream, nent * sizeof(float));
        if (e == hipSuccess) {
            hipLaunchKernelGGL(cbm_entry_weights_kernel, dim3((unsigned)((nent + 255) / 256)), dim3(256), 0, 0, h->d_stream,
                               nent, h->d_dinv, h->d_wstream, h->bundled ? CBM_BUNDLE_INDEX_MASK : CBM_ENTRY_INDEX_MASK);
            e = hipGetLastError();
            if (e == hipSuccess) e = hipDeviceSynchronize();
        }
        if (e != hipSuccess) {
            cbm_set_error_detail("entry weights", hipGetErrorString(e));
            cbm_release_device(h);
            if (cur != dev) hipSetDevice(cur);
            return CBM_ERR_HIP;
        }
    }
    {   // set-up is the place to look up the static scratch of this GPU, so that cbm_spmm_noalloc need not
        float* unused = nullptr;
        if (static_scratch_address(dev, &unused) != CBM_OK) {
            cbm_release_device(h);
            if (cur != dev) hipSetDevice(cur);
            return CBM_ERR_HIP;
        }
    }
    h->on_device = true;
    if (cur != dev) hipSetDevice(cur);
    return CBM_OK;
}

void cbm_release_device(cbm_handle* h) {
    if (h->d_partial) hipFree(h->d_partial);
    h->d_partial = nullptr;
    h->partial_k = 0;
    for (void* e : h->prof_events) hipEventDestroy((hipEvent_t)e);
    h->prof_events.clear();
    if (h->d_tasks) hipFree(h->d_tasks);
    if (h->d_comb) hipFree(h->d_comb);
    if (h->d_stream) hipFree(h->d_stream);
    if (h->d_dinv) hipFree(h->d_dinv);
    if (h->d_rinv) hipFree(h->d_rinv);
    if (h->d_wstream) hipFree(h->d_wstream);
    if (h->d_internal) hipFree(h->d_internal);
    if (h->d_scratch) hipFree(h->d_scratch);
    h->d_tasks = h->d_comb = nullptr;
    h->d_stream = nullptr;
    h->d_dinv = nullptr;
    h->d_rinv = nullptr;
    h->d_wstream = nullptr;
    h->d_internal = nullptr;
    h->d_scratch = nullptr;
    h->scratch_k = 0;
    h->on_device = false;
}

// Make the handle's split-row scratch at least num_slots x k floats (rounded up to four columns).
cbm_status cbm_reserve_scratch(const cbm_handle* h, int32_t k) {
    const int64_t ld_scratch = ((int64_t)k + 3) & ~(int64_t)3;
    if (h->blocks > 1) {  // the partial rows of the B m part-rows, and whatever the inner format needs
        if (h->partial_k < ld_scratch) {
            if (h->d_partial) hipFree(h->d_partial);
            h->d_partial = nullptr;
            h->partial_k = 0;
            HIP_TRY(hipMalloc((void**)&h->d_partial, (size_t)h->blocks * h->m * ld_scratch * sizeof(float) + 16), CBM_ERR_ALLOC);
            h->partial_k = ld_scratch;
        }
        return cbm_reserve_scratch(h->inner, k);
    }
    if (h->num_slots <= 0 || h->scratch_k >= ld_scratch) return CBM_OK;
    // hipFree waits for the device: no product enqueued earlier is still reading the old array when it goes
    if (h->d_scratch) hipFree(h->d_scratch);
    h->d_scratch = nullptr;
    h->scratch_k = 0;
    HIP_TRY(hipMalloc((void**)&h->d_scratch, (size_t)h->num_slots * ld_scratch * sizeof(float)), CBM_ERR_ALLOC);
    h->scratch_k = ld_scratch;
    return CBM_OK;
}

namespace {
// Column-blocked handle: Y[i,:] = sum over the B column ranges of the partial row of part-row b m + i
// (+ self_w X[i,:], then ReLU): B loads in flight per element, added in block order.
template <bool VEC>
__global__ __launch_bounds__(256) void cbm_block_sum_kernel(int64_t m, int blocks, const float* __restrict__ P, int64_t ldp,
                                                            const float* __restrict__ X, int64_t ldx, float* __restrict__ Y,
                                                            int64_t ldy, float self_w, int relu, int k) {
    constexpr int W = VEC ? 4 : 1;
    const int per_row = (k + W - 1) / W;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= m * per_row) return;
    const int64_t i = idx / per_row;
    const int c = (int)(idx % per_row) * W;
    float acc[W];
#pragma unroll
    for (int j = 0; j < W; ++j) acc[j] = 0.0f;
    for (int b0 = 0; b0 < blocks; b0 += 8) {
        float part[8][W];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool on = b0 + u < blocks;
            const float* src = P + ((int64_t)(on ? b0 + u : b0) * m + i) * ldp + c;
            if (VEC) {
                const float4a t = __builtin_nontemporal_load(reinterpret_cast<const float4a*>(src));
#pragma unroll
                for (int j = 0; j < W; ++j) part[u][j] = on ? t[j] : 0.0f;
            } else {
                part[u][0] = on ? __builtin_nontemporal_load(src) : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int j = 0; j < W; ++j) acc[j] += part[u][j];
    }
#pragma unroll
    for (int j = 0; j < W; ++j) {
        if (self_w != 0.0f) acc[j] = fmaf(self_w, X[i * ldx + c + j], acc[j]);
        if (relu) acc[j] = fmaxf(acc[j], 0.0f);
    }
    if (VEC) {
        float4a t;
#pragma unroll
        for (int j = 0; j < W; ++j) t[j] = acc[j];
        *reinterpret_cast<float4a*>(Y + i * ldy + c) = t;
    } else {
        Y[i * ldy + c] = acc[0];
    }
}

cbm_status launch_blocked(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy, CbmEpilogue epi,
                          float self_weight, hipStream_t stream) {
    if (const cbm_status st = cbm_reserve_scratch(h, k); st != CBM_OK) return st;
    const int64_t ldp = h->partial_k;
    // the part-rows carry column weights and row weight (the row weight distributes over the sum of the parts); ReLU and
    // the self term have to wait for the whole row
    const CbmEpilogue inner_epi = epi == CBM_EPI_ROWSCALE_RELU ? CBM_EPI_ROWSCALE : epi == CBM_EPI_SELF ? CBM_EPI_NONE : epi;
    if (const cbm_status st = cbm_launch_product(h->inner, X, ldx, k, h->d_partial, ldp, inner_epi, 0.0f, stream, false); st != CBM_OK)
        return st;
    const bool vec = k % 4 == 0 && ldy % 4 == 0 && ((uintptr_t)Y & 15) == 0;
    const int64_t threads = h->m * (vec ? k / 4 : k);
    if (threads > 0) {
        cbm_launch_record rec{};
        rec.kind = 4;
        rec.tasks = h->m;
        rec.algorithmic_bytes = 0;  // the partial rows are this variant's overhead
        ProfScope ps(h->inner, stream, rec);
        const dim3 grid((unsigned)((threads + 255) / 256));
        const float sw = epi == CBM_EPI_SELF ? self_weight : 0.0f;
        const int relu = epi == CBM_EPI_ROWSCALE_RELU;
        if (vec)
            hipLaunchKernelGGL(cbm_block_sum_kernel<true>, grid, dim3(256), 0, stream, h->m, (int)h->blocks, h->d_partial, ldp, X, ldx,
                               Y, ldy, sw, relu, (int)k);
        else
            hipLaunchKernelGGL(cbm_block_sum_kernel<false>, grid, dim3(256), 0, stream, h->m, (int)h->blocks, h->d_partial, ldp, X,
                               ldx, Y, ldy, sw, relu, (int)k);
    }
    HIP_TRY(hipGetLastError(), CBM_ERR_HIP);
    return CBM_OK;
}
}  // namespace

size_t cbm_static_scratch_bytes() { return (size_t)CBM_STATIC_SCRATCH_FLOATS * sizeof(float); }

cbm_status cbm_launch_product(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                              CbmEpilogue epi, float self_weight, void* stream_, bool static_scratch) {
    hipStream_t stream = (hipStream_t)stream_;
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur), CBM_ERR_HIP);
    if (cur != h->device) return CBM_ERR_STATE;  // the caller's current device must be the handle's
    if (h->blocks > 1) {
        if (static_scratch) {
            cbm_set_error_detail("cbm_spmm_noalloc", "a column-blocked handle keeps B partial rows per row: more than the static scratch is for");
            return CBM_ERR_UNSUPPORTED;
        }
        return launch_blocked(h, X, ldx, k, Y, ldy, epi, self_weight, stream);
    }

    const int64_t ld_scratch = ((int64_t)k + 3) & ~(int64_t)3;
    float* scratch = nullptr;
    if (static_scratch) {
        // nothing on this path allocates: the partial sums go to the library's static array, which every call on
        // this GPU shares.  Segments overwrite their scratch rows in full before the combine launches read them,
        // so nothing has to be cleared between calls.
        if (h->profiling) return CBM_ERR_STATE;  // per-launch events are created on the fly
        if (h->num_slots > 0) {
            if ((uint64_t)h->num_slots * (uint64_t)ld_scratch > (uint64_t)CBM_STATIC_SCRATCH_FLOATS) {
                char msg[160];
                std::snprintf(msg, sizeof(msg), "%lld scratch rows of %lld floats exceed the static scratch of %lld floats",
                              (long long)h->num_slots, (long long)ld_scratch, (long long)CBM_STATIC_SCRATCH_FLOATS);
                cbm_set_error_detail("cbm_spmm_noalloc", msg);
                return CBM_ERR_UNSUPPORTED;
            }
            if (const cbm_status st = static_scratch_address(cur, &scratch); st != CBM_OK) return st;
        }
    } else {
        // scratch rows for split rows: sized by cbm_reserve, else for this k on first use
        if (const cbm_status st = cbm_reserve_scratch(h, k); st != CBM_OK) return st;
        scratch = h->d_scratch;
    }

    // every lane holds four columns; rows that all start on 16-byte boundaries and hold a multiple of four columns
    // take the aligned variant (128-bit accesses), anything else the ragged one (32-bit accesses, strided columns)
    const bool aligned = k % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && ((uintptr_t)X & 15) == 0 && ((uintptr_t)Y & 15) == 0;
    // at least 8 lanes per work item, idle ones included: entries are fetched a group's width at a time, and groups
    // of 4 spend more on that than they save (k <= 16: 25-30 % slower, measured)
    int lanes = 8;
    while (lanes < 64 && lanes * 4 < k) lanes *= 2;
    // a feature matrix whose width is a multiple of 128 goes through in column chunks of 128, one after the other
    // (the chunk index is the slow grid dimension): half the bytes per gathered row, so twice the rows of X stay in
    // L2 (k = 256, 512: 5 % faster).  With a partly filled last chunk, walking the entries again costs more than that.
    if (lanes == 64 && k % 128 == 0) lanes = 32;
    const int mode = (int)epi;
    const Variant var = aligned ? pick_lanes<false>(lanes, mode) : pick_lanes<true>(lanes, mode);
    if (h->profiling) {
        for (void* e : h->prof_events) hipEventDestroy((hipEvent_t)e);
        h->prof_events.clear();
        h->prof_records.clear();
    }
    // a launch of this many waves or more hides latency by occupancy: small batches, more waves per SIMD
    static const int64_t many_waves = [] {
        const char* e = std::getenv("CBM_MANY_WAVES");
        return e ? std::atoll(e) : (int64_t)kManyWavesDefault;
    }();
    const int64_t ychunks = ((int64_t)k + lanes * 4 - 1) / (lanes * 4);
    auto many = [&](int64_t items) { return items / var.group * ychunks >= many_waves; };
    const bool wcol = mode == 1 || mode == 2, wrow = wcol || mode == 3;
    const LaunchCtx ctx{h, X, ldx, k, Y, ldy, scratch, ld_scratch, stream, h->d_wstream, mode == 3 ? h->d_rinv : h->d_dinv, self_weight};
    const int64_t rowb = 4 * (int64_t)k;
    const int64_t per_delta = rowb + 4 + (wcol ? 4 : 0);
    const int64_t per_row = rowb + 4 + (wrow ? 4 : 0) + (mode == 4 ? rowb : 0);  // Y write, marker, weight, own X row
    if (h->num_slots > 0) {
        cbm_launch_record rec{};
        rec.kind = 1;
        rec.per_xcd = 1;
        rec.tasks = h->num_slots;
        rec.deltas = h->seg_deltas;
        // the method's bytes only: the partial sums of split rows are this implementation's overhead
        rec.algorithmic_bytes = h->seg_deltas * per_delta;
        ProfScope ps(h, stream, rec);
        (many(h->num_slots) ? var.segments_many : var.segments)(ctx, CbmLevel{});
    }
    for (size_t l = 0; l < h->levels.size(); ++l) {
        const CbmLevel& L = h->levels[l];
        if (L.task_count > 0) {
            cbm_launch_record rec{};
            rec.kind = 0;
            rec.per_xcd = L.by_xcd ? 1 : 0;
            rec.level = (int32_t)l + 1;
            rec.tasks = L.task_count;
            rec.deltas = L.deltas;
            // per delta: one X row + its entry (+ d^-1/2); per row: one Y write + its marker entry (+ d^-1/2);
            // per work item with a parent: the parent's row
            rec.algorithmic_bytes = L.deltas * per_delta + L.rows_written * per_row + L.parent_reads * rowb;
            ProfScope ps(h, stream, rec);
            (many(L.task_count) ? var.level_many : var.level)(ctx, L);
        }
        if (L.comb_count > 0) {
            cbm_launch_record rec{};
            rec.kind = 2;
            rec.level = (int32_t)l + 1;
            rec.tasks = L.comb_count;
            // split rows: the Y write and the parent read belong to the method, the partial sums do not
            rec.algorithmic_bytes = L.comb_parent_reads * rowb + L.comb_count * per_row;
            ProfScope ps(h, stream, rec);
            var.combine(ctx, L);
        }
    }
    if (mode != 0 && !h->internal_rows.empty()) {
        const int64_t nr = (int64_t)h->internal_rows.size();
        cbm_launch_record rec{};
        rec.kind = 3;
        rec.tasks = nr;
        rec.algorithmic_bytes = 0;  // the deferred finish is overhead of this implementation
        ProfScope ps(h, stream, rec);
        dim3 grid((unsigned)((nr + 3) / 4));
        auto fin = mode == 1 ? cbm_finish_kernel<1> : mode == 2 ? cbm_finish_kernel<2> : mode == 3 ? cbm_finish_kernel<3>
                                                                                                   : cbm_finish_kernel<4>;
        hipLaunchKernelGGL(fin, grid, dim3(256), 0, stream, h->d_internal, nr, X, ldx, Y, ldy, ctx.rw, self_weight, k);
    }
    HIP_TRY(hipGetLastError(), CBM_ERR_HIP);
    return CBM_OK;
}

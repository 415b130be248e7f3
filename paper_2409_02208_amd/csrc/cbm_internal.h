// Internal layout shared by the host builder, the kernel launchers and the C ABI.
#pragma once

#include <cstdint>
#include <vector>

#include "cbm.h"

// One GPU work item: start from the parent's finished row, then walk `len` entries of the
// entry stream beginning at stream[start].
//   parent  >= 0: row whose result is loaded first;  -1: none (virtual null row).
//   len     low 24 bits = number of entries; high bits = CBM_TASK_* flags.
// An entry is either a delta -- a column index with the sign in bit 31 (set = Delta-): gather that
// row of X -- or a marker (CBM_ENTRY_MARK): store the running sum as row (entry & index mask) of Y
// and keep going; the next rows of the path continue from the same registers.
// A SEGMENT task has no markers: its sum goes to scratch row `row` when the entries end.
struct CbmTask {
    int32_t row;
    int32_t parent;
    uint32_t start;
    uint32_t len_flags;
};

constexpr uint32_t CBM_TASK_LEN_MASK = 0x00ffffffu;
constexpr uint32_t CBM_TASK_INTERNAL = 0x01000000u;  // some row is compressed against this one
constexpr uint32_t CBM_TASK_SEGMENT = 0x02000000u;   // `row` is a scratch slot, not a matrix row
constexpr uint32_t CBM_DELTA_MINUS = 0x80000000u;
constexpr uint32_t CBM_ENTRY_MARK = 0x40000000u;      // entry stores a row instead of gathering one
constexpr uint32_t CBM_ENTRY_INTERNAL = 0x20000000u;  // marker: another work item reads this row, keep it unscaled
constexpr uint32_t CBM_ENTRY_INDEX_MASK = 0x1fffffffu;
// Bundled paths: the rows of a path are taken in groups of CBM_BUNDLE_ROWS, and a group's deltas come in ONE ascending
// sweep over the columns, each entry saying in bits 26-28 which row of the group it belongs to; the group's markers
// follow, tagged alike, in row order.  Rows and columns are limited to 26 bits in a handle that bundles.
constexpr uint32_t CBM_BUNDLE_SLOT_SHIFT = 26;
constexpr uint32_t CBM_BUNDLE_INDEX_MASK = 0x03ffffffu;
constexpr int32_t CBM_BUNDLE_ROWS = 4;  // most rows in a bundled path (a power of two)
constexpr int CBM_XCD = 8;  // accelerator complex dies of an MI355X; workgroup (linear id) b runs on XCD b mod 8

struct CbmLevel {
    // one ROUND of dependent work (the struct keeps its first name: a round of single-row paths is a tree level)
    int64_t task_begin = 0, task_count = 0;        // into tasks[]: paths headed in this round
    int64_t comb_begin = 0, comb_count = 0;        // into comb[]: split rows of this round
    int64_t deltas = 0;                            // delta entries gathered by the round's main launch
    int64_t parent_reads = 0;                      // tasks in the main launch with a parent
    int64_t rows_written = 0;                      // matrix rows written by the main launch
    int64_t comb_segments = 0;                     // scratch rows read by the combine launch
    int64_t comb_parent_reads = 0;
    bool bundled = false;                          // the round's paths are emitted as bundles (see CBM_BUNDLE_SLOT_SHIFT)
    bool long_single_rows = false;                 // every path is one row (deltas, then its marker: the same entries in either
                                                   // layout), long on average, columns below 2^26: either kernel can run the round
    // work items in locality order, cut into one contiguous block per XCD (absolute indices into tasks[])
    bool by_xcd = false;
    int64_t xcd_begin[CBM_XCD] = {}, xcd_count[CBM_XCD] = {};
};

struct cbm_handle {
    int64_t m = 0, n = 0;
    cbm_build_opts opts{};
    int32_t eff_alpha = 0, eff_max_depth = 0, eff_hub_cap = 0, eff_max_cand = 0;
    bool square_self_loops = false;

    // ---- host copy of the format -------------------------------------------------
    std::vector<int32_t> rownnz;   // nnz of each compressed row (A or A v I)
    std::vector<int32_t> parent;   // -1 = virtual null row
    std::vector<int32_t> level;    // 1 = stored in full
    std::vector<int32_t> nplus, nminus;
    std::vector<int64_t> dptr;     // m + 1
    std::vector<uint32_t> dcol;    // Delta+ then Delta- of each row, sign in bit 31 (host copy, by row)
    std::vector<uint32_t> stream;  // the same deltas in work-item order, with row markers (uploaded)
    std::vector<float> dinv;       // d_x^-1/2 (square_self_loops only)
    std::vector<float> rinv;       // 1 / nnz of each compressed row, 0 for an empty row
    std::vector<CbmTask> tasks;
    std::vector<CbmTask> comb;     // split rows: start = first scratch slot, len = number of segments
    std::vector<int32_t> internal_rows;
    std::vector<CbmLevel> levels;  // levels[0] is round 1
    int64_t num_slots = 0;         // scratch rows needed by split rows
    int64_t seg_begin[CBM_XCD] = {}, seg_count[CBM_XCD] = {};  // segment work items in tasks[], per column range
    int64_t seg_deltas = 0;        // delta entries gathered by the segment launch
    bool bundled = false;          // some round's paths are emitted as bundles: delta columns are 26-bit in this handle
    cbm_stats_t stats{};

    // ---- device arrays (owned) ---------------------------------------------------
    int device = -1;
    bool on_device = false;
    CbmTask* d_tasks = nullptr;
    CbmTask* d_comb = nullptr;
    uint32_t* d_stream = nullptr;
    float* d_dinv = nullptr;
    float* d_rinv = nullptr;
    float* d_wstream = nullptr;  // weight of every stream entry (normalised product), computed on the device at upload
    int32_t* d_internal = nullptr;
    mutable float* d_scratch = nullptr;  // num_slots x scratch_k floats, sized on first use
    mutable int64_t scratch_k = 0;

    // ---- column-blocked handle: the format itself lives in `inner`, built on the B m part-rows ----
    int32_t blocks = 1;
    cbm_handle* inner = nullptr;          // owned
    mutable float* d_partial = nullptr;   // B m x partial_k floats: the part-rows' sums, sized on first use
    mutable int64_t partial_k = 0;

    // ---- per-launch profiling ----------------------------------------------------
    bool profiling = false;
    mutable std::vector<cbm_launch_record> prof_records;
    mutable std::vector<void*> prof_events;  // hipEvent_t pairs
};

// Detail text of the most recent failure on this thread (which HIP call, which error).
void cbm_set_error_detail(const char* what, const char* detail);
const char* cbm_get_error_detail();

// host builder (cbm_builder.cpp)
cbm_status cbm_build_host(int64_t m, int64_t n, const int64_t* rowptr, const int32_t* colidx, cbm_handle* h);
cbm_status cbm_decompress_host(const cbm_handle* h, int64_t* rowptr, int32_t* colidx);

// device side (cbm_kernels.hip)
enum CbmEpilogue { CBM_EPI_NONE = 0, CBM_EPI_ROWSCALE = 1, CBM_EPI_ROWSCALE_RELU = 2, CBM_EPI_MEAN = 3, CBM_EPI_SELF = 4 };
cbm_status cbm_upload(cbm_handle* h);
void cbm_release_device(cbm_handle* h);
// Candidate search of the builder on the GPU (same candidate set as the host search): for every row the
// best `keep` (<= 16) rows to compress it against, out_y / out_w = parent and distance, out_n = how many.
cbm_status cbm_device_candidates(int device, int64_t m, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                                 const int64_t* tptr, const int32_t* trow, int64_t hub_cap, int64_t min_saving,
                                 int32_t keep, std::vector<int32_t>* out_n, std::vector<int32_t>* out_y,
                                 std::vector<int32_t>* out_w);
// grow the handle's split-row scratch to k columns (no-op when it is wide enough or no row is split)
cbm_status cbm_reserve_scratch(const cbm_handle* h, int32_t k);
// Delta lists (Eq. (2)) of every tree edge on the GPU: nplus / nminus / dptr / dcol exactly as the host merge writes them.
cbm_status cbm_device_deltas(int device, int64_t m, const int64_t* rowptr, const int32_t* colidx, const int32_t* parent,
                             std::vector<int32_t>* nplus, std::vector<int32_t>* nminus, std::vector<int64_t>* dptr,
                             std::vector<uint32_t>* dcol);
cbm_status cbm_launch_product(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                              CbmEpilogue epi, float self_weight, void* stream, bool static_scratch = false);
size_t cbm_static_scratch_bytes();
// dense fp32 MFMA matmul (cbm_gemm.hip)
cbm_status cbm_launch_gemm(int64_t M, int32_t N, int32_t K, const float* A, int64_t lda, const float* B, int64_t ldb,
                           float* C, int64_t ldc, void* stream);

// extern "C" boundary of libcbm: argument checks, handle lifetime, dispatch.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>

#include "cbm_internal.h"

namespace {
thread_local char g_detail[512] = "";
}

void cbm_set_error_detail(const char* what, const char* detail) {
    std::snprintf(g_detail, sizeof(g_detail), "%s: %s", what ? what : "", detail ? detail : "");
}
const char* cbm_get_error_detail() { return g_detail; }

namespace {

cbm_status check_product_args(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy) {
    if (!h || k <= 0 || ldx < k || ldy < k) return CBM_ERR_INVALID_ARG;
    if ((!X && h->n > 0) || (!Y && h->m > 0)) return CBM_ERR_INVALID_ARG;  // an empty operand may be NULL
    if (!h->on_device) return CBM_ERR_STATE;
    if (X && Y && h->m > 0 && h->n > 0) {  // Y is written while X is still being gathered: they must not overlap
        const uintptr_t xb = (uintptr_t)X, xe = xb + ((uintptr_t)(h->n - 1) * ldx + k) * sizeof(float);
        const uintptr_t yb = (uintptr_t)Y, ye = yb + ((uintptr_t)(h->m - 1) * ldy + k) * sizeof(float);
        if (xb < ye && yb < xe) return CBM_ERR_INVALID_ARG;
    }
    return CBM_OK;
}

}  // namespace

extern "C" {

cbm_status cbm_build(int64_t m, int64_t n, const int64_t* rowptr, const int32_t* colidx, const cbm_build_opts* opts,
                     cbm_handle** out) {
    if (!out || m < 0 || n < 0 || !rowptr || (!colidx && rowptr[m] > 0)) return CBM_ERR_INVALID_ARG;
    cbm_handle* h = new (std::nothrow) cbm_handle();
    if (!h) return CBM_ERR_ALLOC;
    if (opts) h->opts = *opts;
    if (!opts) h->opts.device = -1;
    cbm_status st;
    try {
        st = cbm_build_host(m, n, rowptr, colidx, h);
        if (st == CBM_OK && !(h->opts.flags & CBM_FLAG_HOST_ONLY)) st = cbm_upload(h);
    } catch (const std::bad_alloc&) {
        st = CBM_ERR_ALLOC;
    } catch (...) {
        st = CBM_ERR_STATE;
    }
    if (st != CBM_OK) {
        cbm_free(h);
        return st;
    }
    *out = h;
    return CBM_OK;
}

cbm_status cbm_spmm(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                    void* hip_stream) {
    cbm_status st = check_product_args(h, X, ldx, k, Y, ldy);
    if (st != CBM_OK) return st;
    return cbm_launch_product(h, X, ldx, k, Y, ldy, CBM_EPI_NONE, 0.0f, hip_stream);
}

cbm_status cbm_spmm_noalloc(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                            void* hip_stream) {
    cbm_status st = check_product_args(h, X, ldx, k, Y, ldy);
    if (st != CBM_OK) return st;
    return cbm_launch_product(h, X, ldx, k, Y, ldy, CBM_EPI_NONE, 0.0f, hip_stream, /*static_scratch=*/true);
}

cbm_status cbm_spmm_normalized(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                               void* hip_stream) {
    cbm_status st = check_product_args(h, X, ldx, k, Y, ldy);
    if (st != CBM_OK) return st;
    if (!h->square_self_loops) return CBM_ERR_STATE;
    return cbm_launch_product(h, X, ldx, k, Y, ldy, CBM_EPI_ROWSCALE, 0.0f, hip_stream);
}

cbm_status cbm_spmm_normalized_relu(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y,
                                    int64_t ldy, void* hip_stream) {
    cbm_status st = check_product_args(h, X, ldx, k, Y, ldy);
    if (st != CBM_OK) return st;
    if (!h->square_self_loops) return CBM_ERR_STATE;
    return cbm_launch_product(h, X, ldx, k, Y, ldy, CBM_EPI_ROWSCALE_RELU, 0.0f, hip_stream);
}

cbm_status cbm_spmm_mean(const cbm_handle* h, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                         void* hip_stream) {
    cbm_status st = check_product_args(h, X, ldx, k, Y, ldy);
    if (st != CBM_OK) return st;
    return cbm_launch_product(h, X, ldx, k, Y, ldy, CBM_EPI_MEAN, 0.0f, hip_stream);
}

cbm_status cbm_spmm_gin(const cbm_handle* h, float eps, const float* X, int64_t ldx, int32_t k, float* Y, int64_t ldy,
                        void* hip_stream) {
    cbm_status st = check_product_args(h, X, ldx, k, Y, ldy);
    if (st != CBM_OK) return st;
    if (h->m != h->n) return CBM_ERR_STATE;
    return cbm_launch_product(h, X, ldx, k, Y, ldy, CBM_EPI_SELF, 1.0f + eps, hip_stream);
}

cbm_status cbm_reserve(cbm_handle* h, int32_t max_k) {
    if (!h || max_k <= 0) return CBM_ERR_INVALID_ARG;
    if (!h->on_device) return CBM_ERR_STATE;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return CBM_ERR_HIP;
    if (cur != h->device) return CBM_ERR_STATE;
    return cbm_reserve_scratch(h, max_k);  // (a column-blocked handle: its partial rows and the inner scratch)
}

cbm_status cbm_dense_matmul(int64_t M, int32_t N, int32_t K, const float* A, int64_t lda, const float* B, int64_t ldb,
                            float* C, int64_t ldc, void* hip_stream) {
    if (M < 0 || N < 0 || K < 0 || lda < K || ldb < N || ldc < N) return CBM_ERR_INVALID_ARG;
    if ((M > 0 && N > 0) && (!C || (K > 0 && (!A || !B)))) return CBM_ERR_INVALID_ARG;
    return cbm_launch_gemm(M, N, K, A, lda, B, ldb, C, ldc, hip_stream);
}

size_t cbm_gcn2_workspace_bytes(const cbm_handle* h, int32_t f_in, int32_t hidden, int32_t f_out) {
    if (!h || f_in <= 0 || hidden <= 0 || f_out <= 0) return 0;
    // Z0 (n x hidden), H (n x hidden), Z1 (n x f_out), each rounded up to 256 bytes
    auto r = [](size_t b) { return (b + 255) & ~(size_t)255; };
    const size_t n = (size_t)h->n;
    return 2 * r(n * (size_t)hidden * 4) + r(n * (size_t)f_out * 4);
}

cbm_status cbm_gcn2_forward(const cbm_handle* h, const float* X, int32_t f_in, const float* W0, int32_t hidden,
                            const float* W1, int32_t f_out, float* out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    if (!h || !X || !W0 || !W1 || !out || !workspace || f_in <= 0 || hidden <= 0 || f_out <= 0)
        return CBM_ERR_INVALID_ARG;
    if (!h->on_device || !h->square_self_loops) return CBM_ERR_STATE;
    if (workspace_bytes < cbm_gcn2_workspace_bytes(h, f_in, hidden, f_out) || ((uintptr_t)workspace & 15))
        return CBM_ERR_INVALID_ARG;
    auto r = [](size_t b) { return (b + 255) & ~(size_t)255; };
    const int64_t n = h->n;
    {   // out is written while the workspace is read, the workspace while X and the weights are read: none may overlap
        struct Span {
            uintptr_t b, e;
        };
        auto span = [](const void* p, size_t bytes) { return Span{(uintptr_t)p, (uintptr_t)p + bytes}; };
        const Span wsp = span(workspace, workspace_bytes), outp = span(out, (size_t)n * f_out * 4);
        const Span in[3] = {span(X, (size_t)n * f_in * 4), span(W0, (size_t)f_in * hidden * 4), span(W1, (size_t)hidden * f_out * 4)};
        auto overlap = [](Span a, Span b) { return a.b < b.e && b.b < a.e; };
        if (overlap(wsp, outp)) return CBM_ERR_INVALID_ARG;
        for (const Span& s : in)
            if (overlap(s, wsp) || overlap(s, outp)) return CBM_ERR_INVALID_ARG;
    }
    cbm_status st;
    // both products share the handle's split-row scratch: size it once for the wider of the two, before anything is enqueued
    if ((st = cbm_reserve_scratch(h, hidden > f_out ? hidden : f_out)) != CBM_OK) return st;
    char* ws = (char*)workspace;
    float* Z0 = (float*)ws;
    float* H = (float*)(ws + r((size_t)n * hidden * 4));
    float* Z1 = (float*)(ws + 2 * r((size_t)n * hidden * 4));
    if ((st = cbm_launch_gemm(n, hidden, f_in, X, f_in, W0, hidden, Z0, hidden, hip_stream)) != CBM_OK) return st;
    if ((st = cbm_launch_product(h, Z0, hidden, hidden, H, hidden, CBM_EPI_ROWSCALE_RELU, 0.0f, hip_stream)) != CBM_OK)
        return st;
    if ((st = cbm_launch_gemm(n, f_out, hidden, H, hidden, W1, f_out, Z1, f_out, hip_stream)) != CBM_OK) return st;
    return cbm_launch_product(h, Z1, f_out, f_out, out, f_out, CBM_EPI_ROWSCALE, 0.0f, hip_stream);
}

cbm_status cbm_stats(const cbm_handle* h, cbm_stats_t* out) {
    if (!h || !out) return CBM_ERR_INVALID_ARG;
    *out = h->stats;
    return CBM_OK;
}

cbm_status cbm_get_tree(const cbm_handle* h, int32_t* parent, int32_t* nplus, int32_t* nminus, int32_t* level) {
    if (!h) return CBM_ERR_INVALID_ARG;
    if (h->blocks > 1) h = h->inner;  // the tree over the B m part-rows
    const size_t bytes = (size_t)h->m * sizeof(int32_t);
    if (parent && bytes) std::memcpy(parent, h->parent.data(), bytes);
    if (nplus && bytes) std::memcpy(nplus, h->nplus.data(), bytes);
    if (nminus && bytes) std::memcpy(nminus, h->nminus.data(), bytes);
    if (level && bytes) std::memcpy(level, h->level.data(), bytes);
    return CBM_OK;
}

cbm_status cbm_decompress(const cbm_handle* h, int64_t* rowptr, int32_t* colidx) {
    if (!h || !rowptr || (!colidx && h->stats.nnz > 0)) return CBM_ERR_INVALID_ARG;
    return cbm_decompress_host(h, rowptr, colidx);
}

cbm_status cbm_profile_enable(cbm_handle* h, int32_t on) {
    if (!h) return CBM_ERR_INVALID_ARG;
    if (!h->on_device) return CBM_ERR_STATE;
    h->profiling = on != 0;
    if (h->inner) h->inner->profiling = on != 0;
    return CBM_OK;
}

cbm_status cbm_profile_read(cbm_handle* h, cbm_launch_record* records, int32_t cap, int32_t* count) {
    if (!h || !count || cap < 0 || (cap > 0 && !records)) return CBM_ERR_INVALID_ARG;
    if (h->inner) h = h->inner;  // a column-blocked handle's launches are recorded where they are made
    const size_t nrec = h->prof_records.size();
    if (h->prof_events.size() != 2 * nrec) return CBM_ERR_STATE;
    for (size_t i = 0; i < nrec; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, (hipEvent_t)h->prof_events[2 * i], (hipEvent_t)h->prof_events[2 * i + 1]) !=
            hipSuccess)
            return CBM_ERR_HIP;  // e.g. the stream has not been synchronised yet
        h->prof_records[i].milliseconds = ms;
        if ((int32_t)i < cap) records[i] = h->prof_records[i];
    }
    *count = (int32_t)nrec;
    return CBM_OK;
}

void cbm_free(cbm_handle* h) {
    if (!h) return;
    cbm_release_device(h);
    if (h->inner) {
        cbm_release_device(h->inner);
        delete h->inner;
    }
    delete h;
}

const char* cbm_last_error_detail(void) { return cbm_get_error_detail(); }

const char* cbm_status_string(cbm_status s) {
    switch (s) {
        case CBM_OK: return "ok";
        case CBM_ERR_INVALID_ARG: return "invalid argument";
        case CBM_ERR_INVALID_CSR: return "invalid CSR (row offsets not monotone, or columns unsorted / repeated / out of range)";
        case CBM_ERR_ALLOC: return "allocation failed";
        case CBM_ERR_HIP: return "HIP runtime error";
        case CBM_ERR_UNSUPPORTED: return "size not supported";
        case CBM_ERR_STATE: return "handle cannot perform this operation";
    }
    return "unknown status";
}

}  // extern "C"

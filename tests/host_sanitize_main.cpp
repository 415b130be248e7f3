// Host builder + decompress on random matrices, built with ASan/UBSan by test_host_sanitizers.py; also checks that
// every work item, entry and scratch slot the builder emits is in range (what the kernels rely on).
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <vector>
#include "cbm_internal.h"
void cbm_set_error_detail(const char*, const char*) {}
// the GPU candidate search is not part of a host-only build
cbm_status cbm_device_candidates(int, int64_t, int64_t, const int64_t*, const int32_t*, const int64_t*, const int32_t*, int64_t,
                                 int64_t, int32_t, std::vector<int32_t>*, std::vector<int32_t>*, std::vector<int32_t>*) {
    return CBM_ERR_STATE;
}
cbm_status cbm_device_deltas(int, int64_t, const int64_t*, const int32_t*, const int32_t*, std::vector<int32_t>*, std::vector<int32_t>*,
                             std::vector<int64_t>*, std::vector<uint32_t>*) {
    return CBM_ERR_STATE;
}
const char* cbm_get_error_detail() { return ""; }
int main() {
    std::mt19937 rng(1);
    for (int trial = 0; trial < 60; ++trial) {
        int m = 1 + rng() % 400, n = (trial % 3 == 0) ? m : 1 + rng() % 400;
        double dens = (rng() % 100) / 300.0;
        std::vector<int64_t> rp(m + 1, 0);
        std::vector<int32_t> ci;
        for (int i = 0; i < m; ++i) {
            std::set<int> s;
            int cnt = (int)(dens * n);
            if (trial % 7 == 0 && i == 3) cnt = n;  // a long row -> segments
            for (int c = 0; c < cnt; ++c) s.insert(rng() % n);
            if (trial % 5 == 0 && i > 0 && i % 4 == 0) { s.clear(); for (int64_t p = rp[i-1]; p < rp[i]; ++p) s.insert(ci[p]); }  // duplicate rows
            for (int c : s) ci.push_back(c);
            rp[i + 1] = (int64_t)ci.size();
        }
        cbm_handle h;
        h.opts = cbm_build_opts{};
        h.opts.alpha = trial % 4;
        h.opts.add_self_loops = (m == n) && (trial % 2);
        h.opts.max_depth = (trial % 6 == 0) ? -1 : (trial % 6 == 1) ? 1 : (trial % 6 == 2) ? 0 : 16;
        h.opts.seed_roots = (trial % 3) - 1;
        h.opts.hub_cap = (trial % 4 == 0) ? 3 : 0;
        h.opts.num_threads = 1 + trial % 4;
        h.opts.flags = CBM_FLAG_HOST_ONLY;
        h.opts.column_blocks = (trial % 5 == 1) ? 3 : (trial % 11 == 2) ? 64 : 0;  // column-blocked builds too
        cbm_status st = cbm_build_host(m, n, rp.data(), ci.data(), &h);
        if (st != CBM_OK) { printf("build failed %d\n", st); return 1; }
        std::vector<int64_t> orp(m + 1);
        std::vector<int32_t> oci(h.stats.nnz + 1);
        st = cbm_decompress_host(&h, orp.data(), oci.data());
        if (st != CBM_OK) { printf("decompress failed %d\n", st); return 1; }
        if (!h.opts.add_self_loops && (orp != rp || !std::equal(ci.begin(), ci.end(), oci.begin()))) { printf("round trip differs\n"); return 1; }
        struct Owner {  // the inner handle of a column-blocked build is heap-allocated and owned by the outer one
            cbm_handle* p;
            ~Owner() { delete p; }
        } owner{h.inner};
        if (h.inner) {  // the emitted work lists are the inner handle's: B m part-rows
            const cbm_handle& in = *h.inner;
            h.tasks = in.tasks;
            h.comb = in.comb;
            h.stream = in.stream;
            h.num_slots = in.num_slots;
            m = (int)in.m;
        }
        // bounds of the emitted stream / tasks
        for (auto& t : h.tasks) {
            uint32_t len = t.len_flags & CBM_TASK_LEN_MASK;
            if ((size_t)t.start + len > h.stream.size()) { printf("task out of stream\n"); return 1; }
            if (t.parent >= m) { printf("bad parent\n"); return 1; }
            for (uint32_t i = 0; i < len; ++i) {
                uint32_t e = h.stream[t.start + i];
                const bool bundled = h.inner ? h.inner->bundled : h.bundled;  // then delta columns are 26-bit, with row tags above
                uint32_t idx = e & ((e & CBM_ENTRY_MARK) || !bundled ? CBM_ENTRY_INDEX_MASK : CBM_BUNDLE_INDEX_MASK);
                if (e & CBM_ENTRY_MARK) { if ((int64_t)idx >= m) { printf("marker row out of range\n"); return 1; } }
                else if ((int64_t)idx >= n) { printf("column out of range\n"); return 1; }
            }
            if ((t.len_flags & CBM_TASK_SEGMENT) && t.row >= h.num_slots) { printf("slot out of range\n"); return 1; }
        }
        // a bundled round: every path has its deltas first (row tags within the limit), then at most CBM_BUNDLE_ROWS markers
        for (auto& L : (h.inner ? h.inner->levels : h.levels)) {
            if (!L.bundled) continue;
            for (int64_t ti = L.task_begin; ti < L.task_begin + L.task_count; ++ti) {
                const CbmTask& t = h.tasks[ti];
                uint32_t len = t.len_flags & CBM_TASK_LEN_MASK, nmark = 0;
                bool seen_marker = false;
                for (uint32_t i = 0; i < len; ++i) {
                    const uint32_t e = h.stream[t.start + i];
                    if (e & CBM_ENTRY_MARK) { seen_marker = true; ++nmark; }
                    else if (seen_marker) { printf("delta after a marker in a bundle\n"); return 1; }
                    else if (((e >> CBM_BUNDLE_SLOT_SHIFT) & 7u) >= (uint32_t)CBM_BUNDLE_ROWS) { printf("row tag out of range\n"); return 1; }
                }
                if (nmark < 1 || nmark > (uint32_t)CBM_BUNDLE_ROWS) { printf("bundle of %u rows\n", nmark); return 1; }
            }
        }
        for (auto& c : h.comb) if ((int64_t)c.start + (c.len_flags & CBM_TASK_LEN_MASK) > h.num_slots) { printf("comb slots\n"); return 1; }
    }
    printf("asan run ok\n");
    return 0;
}

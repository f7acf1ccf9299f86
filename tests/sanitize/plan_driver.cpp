// Runs the host planner (csrc/plan.cpp, no GPU code) under AddressSanitizer and
// UndefinedBehaviorSanitizer: plans for every rule, sender-side degrees, group-interleaved fused
// tensors and rejected descriptors; every query; every element's index map against the element
// count per shard.  Built and started by tests/test_host_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "rose_internal.h"

static void fail(const char *what, int rc) {
    std::printf("FAILED: %s (%d)\n", what, rc);
    std::exit(1);
}

static rose_tensor_desc desc(int64_t rows, int64_t cols, int32_t rule, std::vector<int64_t> sec = {}, int32_t groups = 0) {
    rose_tensor_desc t;
    std::memset(&t, 0, sizeof t);
    t.rows = rows;
    t.cols = cols;
    t.rule = (rose_rule)rule;
    t.n_sections = (int32_t)sec.size();
    for (size_t i = 0; i < sec.size(); ++i) t.section_rows[i] = sec[i];
    t.src_groups = groups;
    return t;
}

static void walk(const std::vector<rose_tensor_desc> &ts, int32_t tp, int32_t tp_src, int32_t src_rank) {
    rose_plan *p = nullptr;
    rose_status s = rose_shard_plan_create_src(ts.data(), (int32_t)ts.size(), tp, tp_src, src_rank, &p);
    if (s != ROSE_OK) fail("create", s);
    int64_t v = 0;
    size_t bytes = 0;
    if (rose_plan_n_tensors(p) != (int32_t)ts.size() || rose_plan_tp(p) != tp) fail("counts", 0);
    if (rose_plan_workspace_bytes(p, &bytes) != ROSE_OK || bytes < 8192) fail("workspace", 0);
    if (rose_plan_n_tiles(p, &v) != ROSE_OK || v < 1) fail("tiles", 0);
    for (int32_t d = 0; d < tp; ++d)
        if (rose_plan_bucket_capacity(p, d, &v) != ROSE_OK || v < 0) fail("capacity", d);
    for (int32_t t = 0; t < (int32_t)ts.size(); ++t) {
        int64_t base = 0, src = 0;
        if (rose_plan_tensor_base(p, t, &base) != ROSE_OK) fail("base", t);
        if (rose_plan_src_numel(p, t, &src) != ROSE_OK) fail("src numel", t);
        std::vector<int64_t> seen(tp, 0);
        const int64_t n = src;                      // the map takes an index inside the sender's slice
        int64_t sent = 0;
        for (int64_t g = 0; g < n; ++g) {
            int32_t d0 = 0, nd = 0, loc = 0;
            if (rose_plan_map_index(p, t, g, &d0, &nd, &loc) != ROSE_OK) fail("map", (int)g);
            if (nd == 0) continue;                  // not sent by this sender
            ++sent;
            for (int32_t d = d0; d < d0 + nd; ++d) {
                int64_t ln = 0;
                if (rose_plan_local_numel(p, t, d, &ln) != ROSE_OK) fail("local numel", d);
                if (loc < 0 || loc >= ln) fail("local index out of range", (int)g);
                ++seen[d];
            }
        }
        const bool sends = ts[t].rule != ROSE_REPLICATED || t % tp_src == src_rank;
        if (sent != (sends ? n : 0)) fail("a sender sends its whole slice, or nothing of a replicated tensor", t);
    }
    delete p;                                        // the plan owns no device memory before its first device call
}

int main() {
    std::vector<rose_tensor_desc> ts = {
        desc(3, 41, ROSE_REPLICATED), desc(0, 16, ROSE_SPLIT_ROWS), desc(16, 37, ROSE_SPLIT_ROWS),
        desc(5, 64, ROSE_SPLIT_COLS), desc(64, 9, ROSE_FUSED_ROWS, {32, 16, 16}), desc(2, 20000, ROSE_SPLIT_COLS),
        desc(1, 3 * 8192 + 5, ROSE_REPLICATED),
    };
    for (int32_t tp : {1, 2, 4, 8})
        for (int32_t tp_src : {1, 2, 4, 8})
            for (int32_t s = 0; s < tp_src; ++s) walk(ts, tp, tp_src, s);
    std::vector<rose_tensor_desc> g = {desc(128, 12, ROSE_FUSED_ROWS, {64, 32, 32}, 8)};
    for (int32_t tp : {1, 2, 4, 8})
        for (int32_t tp_src : {1, 2, 4, 8})
            for (int32_t s = 0; s < tp_src; ++s) walk(g, tp, tp_src, s);
    // descriptors the planner must turn down without touching anything
    rose_plan *p = nullptr;
    std::vector<rose_tensor_desc> bad = {desc(6, 4, ROSE_SPLIT_ROWS)};
    if (rose_shard_plan_create(bad.data(), 1, 4, &p) != ROSE_ERR_SHAPE || p) fail("non-divisible rows", 0);
    bad = {desc(1, (int64_t)1 << 31, ROSE_REPLICATED)};
    if (rose_shard_plan_create(bad.data(), 1, 1, &p) != ROSE_ERR_UNSUPPORTED || p) fail("too large", 0);
    bad = {desc(12, 4, ROSE_FUSED_ROWS, {8, 8})};
    if (rose_shard_plan_create(bad.data(), 1, 2, &p) != ROSE_ERR_SHAPE || p) fail("sections", 0);
    if (rose_shard_plan_create(nullptr, 1, 2, &p) != ROSE_ERR_ARG) fail("null", 0);
    if (rose_shard_plan_create(ts.data(), (int32_t)ts.size(), 32, &p) != ROSE_ERR_UNSUPPORTED) fail("tp", 0);
    std::printf("ok\n");
    return 0;
}

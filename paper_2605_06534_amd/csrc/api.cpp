// C ABI: argument checks, the plan's device tables, and hand-off to the kernel launchers.
#include <hip/hip_runtime_api.h>

#include <cstring>

#include "rose_internal.h"

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr int32_t kNeighboursBelowPpm = 75000, kTimedBelowPpm = 40000;   // see encode_common

// Copy the piece and tile tables to the current device once; later calls on the same device
// reuse them.  A plan is bound to the first device it is used on.  `may_allocate` = false: only
// report whether the plan is resident here (nothing is allocated, ROSE_ERR_SCRATCH if it is not).
rose_status device_tables_locked(const rose_plan *p, bool may_allocate);
rose_status device_tables(const rose_plan *p, bool may_allocate = true) {
    std::lock_guard<std::mutex> lock(p->mu);
    try {
        return device_tables_locked(p, may_allocate);
    } catch (...) {                                     // host memory ran out while building the tables
        return ROSE_ERR_HIP;
    }
}

rose_status device_tables_locked(const rose_plan *p, bool may_allocate) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return ROSE_ERR_HIP;
    if (p->device == dev) return ROSE_OK;
    if (p->device != -1) return ROSE_ERR_ARG;
    if (!may_allocate) return ROSE_ERR_SCRATCH;

    // elements of a shard's copy of each tensor, per receiving stage (0: the stage does not hold it)
    std::vector<int32_t> numel((size_t)p->pp_dst * p->n_tensors, 0);
    for (int32_t i = 0; i < p->n_tensors; ++i) {
        const rose_tensor_desc &t = p->tensors[i];
        numel[(size_t)p->stage_dst_of[i] * p->n_tensors + i] =
            (int32_t)(t.rows * t.cols / (t.rule == ROSE_REPLICATED ? 1 : p->tp));
    }
    // replicated tensors the sender holds: a refresh copies them whole, sent from here or not
    std::vector<int32_t> repl;
    std::vector<int64_t> repl_numel;
    for (int32_t i = 0; i < p->n_tensors; ++i) {
        const rose_tensor_desc &t = p->tensors[i];
        if (t.rule == ROSE_REPLICATED && t.rows * t.cols > 0 && p->stage_src_of[i] == p->stage_src) {
            repl.push_back(i);
            repl_numel.push_back(t.rows * t.cols);
        }
    }
    rose::Piece *dp = nullptr;
    int32_t *dt = nullptr, *dn = nullptr, *dr = nullptr;
    int64_t *drn = nullptr;
    unsigned long long *dv = nullptr;
    int resident[8];
    void *sws = nullptr;
    size_t sws_bytes = 0;
    const size_t pb = p->pieces.size() * sizeof(rose::Piece), tb = p->tile_piece.size() * sizeof(int32_t);
    const size_t nb = numel.size() * sizeof(int32_t), vb = kVerdictSlots * sizeof(unsigned long long);
    bool ok = hipMalloc(reinterpret_cast<void **>(&dp), pb) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&dt), tb) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&dn), nb) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&dv), vb) == hipSuccess &&
              hipMemcpy(dp, p->pieces.data(), pb, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(dt, p->tile_piece.data(), tb, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(dn, numel.data(), nb, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemset(dv, 0, vb) == hipSuccess;
    if (ok && !repl.empty()) {
        ok = hipMalloc(reinterpret_cast<void **>(&dr), repl.size() * sizeof(int32_t)) == hipSuccess &&
             hipMalloc(reinterpret_cast<void **>(&drn), repl.size() * sizeof(int64_t)) == hipSuccess &&
             hipMemcpy(dr, repl.data(), repl.size() * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess &&
             hipMemcpy(drn, repl_numel.data(), repl.size() * sizeof(int64_t), hipMemcpyHostToDevice) == hipSuccess;
    }
    ok = ok && rose::encode_resident_all(resident) == 0 && rose::static_scratch(&sws, &sws_bytes) == 0;
    if (!ok) {
        if (dp) (void)hipFree(dp);
        if (dt) (void)hipFree(dt);
        if (dn) (void)hipFree(dn);
        if (dv) (void)hipFree(dv);
        if (dr) (void)hipFree(dr);
        if (drn) (void)hipFree(drn);
        return ROSE_ERR_HIP;
    }
    p->d_pieces = dp;
    p->d_tile_piece = dt;
    p->d_local_numel = dn;
    p->d_verdict = dv;
    p->d_repl_list = dr;
    p->d_repl_numel = drn;
    p->n_repl = (int32_t)repl.size();
    std::memcpy(p->resident, resident, sizeof resident);
    p->static_ws = sws;
    p->static_ws_bytes = sws_bytes;
    p->device = dev;
    return ROSE_OK;
}

rose_status check_bucket(const rose_bucket &b) {
    if (b.capacity < 0 || !b.seg_off) return ROSE_ERR_ARG;
    if (b.capacity > 0 && (!b.idx || !b.val)) return ROSE_ERR_ARG;
    if (!aligned(b.idx, 16) || !aligned(b.val, 16) || !aligned(b.seg_off, 8)) return ROSE_ERR_ALIGN;
    return ROSE_OK;
}

}  // namespace

extern "C" rose_status rose_plan_upload(const rose_plan *p) {
    if (!p) return ROSE_ERR_ARG;
    return device_tables(p);
}

extern "C" void rose_shard_plan_destroy(rose_plan *p) {
    if (!p) return;
    if (p->d_pieces) (void)hipFree(p->d_pieces);
    if (p->d_tile_piece) (void)hipFree(p->d_tile_piece);
    if (p->d_local_numel) (void)hipFree(p->d_local_numel);
    if (p->d_verdict) (void)hipFree(p->d_verdict);
    if (p->d_repl_list) (void)hipFree(p->d_repl_list);
    if (p->d_repl_numel) (void)hipFree(p->d_repl_numel);
    delete p;
}

// The tile order a launch into these buckets uses: the caller's choice, else by density.
static int pick_tile_order(const rose_plan *p, const rose_bucket *buckets) {
    int order = p->tile_order.load(std::memory_order_relaxed);
    if (order != ROSE_TILE_ORDER_AUTO_PICK) return order;
    int32_t ppm = p->seen_density_ppm.load(std::memory_order_relaxed);
    if (ppm < 0 && p->capacity_sum > 0) {
        // nothing read back yet: the buckets cannot hold more than their capacities, which bounds the density
        double room = 0;
        for (int32_t d = 0; d < p->n_buckets; ++d) room += (double)(buckets[d].capacity > 0 ? buckets[d].capacity : 0);
        const double bound = 1e6 * room / (double)p->capacity_sum;
        ppm = bound >= 1e6 ? -1 : (int32_t)bound;
    }
    return ppm < 0 ? ROSE_TILE_ORDER_SPREAD
                   : ppm < kTimedBelowPpm ? ROSE_TILE_ORDER_TIMED
                                          : ppm < kNeighboursBelowPpm ? ROSE_TILE_ORDER_NEIGHBOURS : ROSE_TILE_ORDER_SPREAD;
}

extern "C" rose_status rose_plan_pick_tile_order(const rose_plan *p, const rose_bucket *buckets, int32_t *order) {
    if (!p || !buckets || !order) return ROSE_ERR_ARG;
    *order = pick_tile_order(p, buckets);
    return ROSE_OK;
}

// workspace = nullptr: the library's built-in scratch (the call must not allocate)
static rose_status encode_common(const rose_plan *p, const void *const *old_ptrs, const void *const *new_ptrs,
                                 int32_t new_dtype, const rose_bucket *buckets, void *workspace,
                                 size_t workspace_bytes, bool refresh, bool arith, void *stream) {
    const bool built_in = workspace == nullptr && workspace_bytes == (size_t)-1;
    if (!p || !old_ptrs || !new_ptrs || !buckets || (!workspace && !built_in)) return ROSE_ERR_ARG;
    if (new_dtype != ROSE_BF16 && new_dtype != ROSE_FP32_RNE) return ROSE_ERR_ARG;
    size_t need = 0;
    rose_plan_workspace_bytes(p, &need);
    if (!aligned(old_ptrs, 8) || !aligned(new_ptrs, 8)) return ROSE_ERR_ALIGN;
    rose::EncodeArgs a;
    std::memset(&a, 0, sizeof a);
    for (int32_t d = 0; d < p->n_buckets; ++d) {
        rose_status s = check_bucket(buckets[d]);
        if (s != ROSE_OK) return s;
        a.bucket[d].idx = buckets[d].idx;
        a.bucket[d].val = buckets[d].val;
        a.bucket[d].capacity = buckets[d].capacity;
        a.bucket[d].seg_off = buckets[d].seg_off;
    }
    rose_status s = device_tables(p, !built_in);
    if (s != ROSE_OK) return s;
    if (built_in) {
        if (need > p->static_ws_bytes) return ROSE_ERR_SCRATCH;
        workspace = p->static_ws;
        workspace_bytes = p->static_ws_bytes;
    }
    if (workspace_bytes < need) return ROSE_ERR_ARG;
    if (!aligned(workspace, 256)) return ROSE_ERR_ALIGN;
    std::memcpy(a.chain_first, p->chain_first, sizeof a.chain_first);
    std::memcpy(a.block_first, p->block_first, sizeof a.block_first);
    a.pieces = p->d_pieces;
    a.tile_piece = p->d_tile_piece;
    a.old_ptrs = old_ptrs;
    a.new_ptrs = new_ptrs;
    char *ws = static_cast<char *>(workspace);
    a.abort_flag = reinterpret_cast<unsigned int *>(ws + rose::kWsAbortOff);
    a.ticket = reinterpret_cast<unsigned int *>(ws + rose::kWsTicketOff);
    a.tile_desc = reinterpret_cast<unsigned long long *>(ws + rose::kWsHeaderBytes);
    a.n_tiles = (int32_t)p->tile_piece.size();
    a.n_blocks = p->block_first[p->n_buckets];
    a.block_desc = a.tile_desc + a.n_tiles;
    a.tp = p->n_buckets;
    a.n_tensors = p->n_tensors;
    rose::RefreshArgs r{p->d_repl_list, p->d_repl_numel, p->n_repl};
    const bool f32 = new_dtype == ROSE_FP32_RNE;
    const int resident = p->resident[(f32 ? 1 : 0) + (refresh ? 2 : 0) + (arith ? 4 : 0)];
    // Tile order: the caller's choice, else picked from the density the plan's last checked launch showed
    // (7B-style workload, neighbours against spread on the same buffers: 2.7 / 1.8 / 1.4 / 1.0 % faster at
    // 1 / 2 / 5 / 7 %, 2 / 13 % slower at 8 / 10 %; timed against neighbours: 1.6 / 5 / 8 / 7 / 1 % faster at
    // 0.5 / 1 / 2 / 3 / 4 %, 2 % slower at 5 %).
    const int order = pick_tile_order(p, buckets);
    return rose::launch_encode(a, f32, refresh ? &r : nullptr, arith ? 1 : 0, resident,
                               p->worker_cap.load(std::memory_order_relaxed), order, stream) == 0
               ? ROSE_OK
               : ROSE_ERR_HIP;
}

extern "C" rose_status rose_delta_encode(const rose_plan *p, const void *const *old_ptrs,
                                         const void *const *new_ptrs, int32_t new_dtype,
                                         const rose_bucket *buckets, void *workspace,
                                         size_t workspace_bytes, void *stream) {
    return encode_common(p, old_ptrs, new_ptrs, new_dtype, buckets, workspace, workspace_bytes, false, false, stream);
}

extern "C" rose_status rose_delta_encode_refresh(const rose_plan *p, void *const *old_ptrs,
                                                 const void *const *new_ptrs, int32_t new_dtype,
                                                 const rose_bucket *buckets, void *workspace,
                                                 size_t workspace_bytes, void *stream) {
    return encode_common(p, const_cast<const void *const *>(old_ptrs), new_ptrs, new_dtype, buckets, workspace,
                         workspace_bytes, true, false, stream);
}

extern "C" rose_status rose_delta_encode_ex(const rose_plan *p, void *const *old_ptrs, const void *const *new_ptrs,
                                            int32_t new_dtype, uint32_t flags, const rose_bucket *buckets,
                                            void *workspace, size_t workspace_bytes, void *stream) {
    if (flags & ~(uint32_t)(ROSE_ENCODE_REFRESH | ROSE_ENCODE_ARITH)) return ROSE_ERR_ARG;
    return encode_common(p, const_cast<const void *const *>(old_ptrs), new_ptrs, new_dtype, buckets, workspace,
                         workspace_bytes, (flags & ROSE_ENCODE_REFRESH) != 0, (flags & ROSE_ENCODE_ARITH) != 0, stream);
}

extern "C" rose_status rose_delta_encode_static(const rose_plan *p, void *const *old_ptrs,
                                                const void *const *new_ptrs, int32_t new_dtype, uint32_t flags,
                                                const rose_bucket *buckets, void *stream) {
    if (flags & ~(uint32_t)(ROSE_ENCODE_REFRESH | ROSE_ENCODE_ARITH)) return ROSE_ERR_ARG;
    return encode_common(p, const_cast<const void *const *>(old_ptrs), new_ptrs, new_dtype, buckets, nullptr, (size_t)-1,
                         (flags & ROSE_ENCODE_REFRESH) != 0, (flags & ROSE_ENCODE_ARITH) != 0, stream);
}

static rose_status apply_common(const rose_plan *p, int32_t d, const rose_bucket *bucket, int32_t payload,
                                void *const *dst_ptrs, void *stream) {
    if (!p || !bucket || !dst_ptrs || d < 0 || d >= p->n_buckets) return ROSE_ERR_ARG;
    if (payload != ROSE_PAYLOAD_NEW && payload != ROSE_PAYLOAD_ARITH) return ROSE_ERR_ARG;
    rose_status s = check_bucket(*bucket);
    if (s != ROSE_OK) return s;
    if (!aligned(dst_ptrs, 8)) return ROSE_ERR_ALIGN;
    rose::BucketDev b{bucket->idx, bucket->val, bucket->capacity, bucket->seg_off};
    s = device_tables(p);
    if (s != ROSE_OK) return s;
    const int32_t *local_numel = p->d_local_numel + (size_t)(d / p->tp) * p->n_tensors;
    int64_t shard_elems = 0;
    for (int32_t i = 0; i < p->n_tensors; ++i)
        if (p->stage_dst_of[i] == d / p->tp) {
            const rose_tensor_desc &t = p->tensors[i];
            shard_elems += t.rows * t.cols / (t.rule == ROSE_REPLICATED ? 1 : p->tp);
        }
    return rose::launch_apply(b, p->n_tensors, local_numel, dst_ptrs, payload, shard_elems, stream) == 0 ? ROSE_OK
                                                                                                       : ROSE_ERR_HIP;
}

extern "C" rose_status rose_delta_apply(const rose_plan *p, int32_t d, const rose_bucket *bucket,
                                        void *const *dst_ptrs, void *stream) {
    return apply_common(p, d, bucket, ROSE_PAYLOAD_NEW, dst_ptrs, stream);
}

extern "C" rose_status rose_delta_apply_ex(const rose_plan *p, int32_t d, const rose_bucket *bucket, int32_t payload,
                                           void *const *dst_ptrs, void *stream) {
    return apply_common(p, d, bucket, payload, dst_ptrs, stream);
}

extern "C" rose_status rose_dense_copy(const rose_plan *p, int32_t d, const void *const *new_ptrs,
                                       int32_t new_dtype, void *const *dst_ptrs, void *stream) {
    if (!p || !new_ptrs || !dst_ptrs || d < 0 || d >= p->n_buckets) return ROSE_ERR_ARG;
    if (new_dtype != ROSE_BF16 && new_dtype != ROSE_FP32_RNE) return ROSE_ERR_ARG;
    if (!aligned(new_ptrs, 8) || !aligned(dst_ptrs, 8)) return ROSE_ERR_ALIGN;
    rose::CopyArgs a;
    std::memset(&a, 0, sizeof a);
    rose_status s = device_tables(p);
    if (s != ROSE_OK) return s;
    a.pieces = p->d_pieces;
    a.tile_piece = p->d_tile_piece;
    a.new_ptrs = new_ptrs;
    a.dst_ptrs = dst_ptrs;
    a.tile_begin = p->chain_first[d];
    a.n_tiles = p->chain_first[d + 1] - p->chain_first[d];
    return rose::launch_dense_copy(a, new_dtype == ROSE_FP32_RNE, stream) == 0 ? ROSE_OK : ROSE_ERR_HIP;
}

extern "C" rose_status rose_bucket_check(const rose_plan *p, const rose_bucket *bucket, void *stream,
                                         int64_t *required) {
    if (!p || !bucket || !bucket->seg_off) return ROSE_ERR_ARG;
    int64_t total = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(&total, bucket->seg_off + p->n_tensors, sizeof total, hipMemcpyDeviceToHost, st) != hipSuccess)
        return ROSE_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return ROSE_ERR_HIP;
    if (required) *required = total;
    if (total < 0) return ROSE_ERR_HIP;     // the encode launch gave up (see rose_delta_encode)
    if (p->capacity_sum > 0) {
        // what this bucket says about the update's density, taking the buckets to be about equal
        const double ppm = 1e6 * (double)total * p->n_buckets / (double)p->capacity_sum;
        p->seen_density_ppm.store(ppm > 1e6 ? 1000000 : (int32_t)ppm, std::memory_order_relaxed);
    }
    return total > bucket->capacity ? ROSE_ERR_CAPACITY : ROSE_OK;
}

extern "C" rose_status rose_bw_probe(const void *src, void *dst, size_t bytes, uint64_t *sink, void *stream) {
    if (!src || (bytes & 15u)) return ROSE_ERR_ARG;
    if (!dst && !sink) return ROSE_ERR_ARG;
    if (!aligned(src, 16) || !aligned(dst, 16) || !aligned(sink, 8)) return ROSE_ERR_ALIGN;
    return rose::launch_bw_probe(src, dst, bytes, sink, stream) == 0 ? ROSE_OK : ROSE_ERR_HIP;
}

static rose_status probe_mixed(const void *src_a, const void *src_b, void *dst, size_t read_bytes,
                               size_t write_bytes_per_chunk, int timed, uint64_t *sink, void *stream) {
    if (!src_a || !src_b || !dst || !sink) return ROSE_ERR_ARG;
    if ((read_bytes % ROSE_PROBE_CHUNK) || (write_bytes_per_chunk & 15u) || write_bytes_per_chunk > ROSE_PROBE_CHUNK)
        return ROSE_ERR_ARG;
    if (!aligned(src_a, 16) || !aligned(src_b, 16) || !aligned(dst, 16) || !aligned(sink, 8)) return ROSE_ERR_ALIGN;
    return rose::launch_bw_probe_mixed(src_a, src_b, dst, read_bytes / ROSE_PROBE_CHUNK,
                                       (uint32_t)(write_bytes_per_chunk / 16), timed, sink, stream) == 0
               ? ROSE_OK
               : ROSE_ERR_HIP;
}

extern "C" rose_status rose_bw_probe_mixed(const void *src_a, const void *src_b, void *dst, size_t read_bytes,
                                           size_t write_bytes_per_chunk, uint64_t *sink, void *stream) {
    return probe_mixed(src_a, src_b, dst, read_bytes, write_bytes_per_chunk, 0, sink, stream);
}

extern "C" rose_status rose_bw_probe_mixed_timed(const void *src_a, const void *src_b, void *dst, size_t read_bytes,
                                                 size_t write_bytes_per_chunk, uint64_t *sink, void *stream) {
    return probe_mixed(src_a, src_b, dst, read_bytes, write_bytes_per_chunk, 1, sink, stream);
}

extern "C" rose_status rose_bw_probe_lines(void *dst, size_t bytes, uint32_t touched_per_2_32, void *stream) {
    if (!dst || (bytes & 63u)) return ROSE_ERR_ARG;
    if (!aligned(dst, 64)) return ROSE_ERR_ALIGN;
    return rose::launch_bw_probe_lines(dst, bytes / 64, touched_per_2_32, stream) == 0 ? ROSE_OK : ROSE_ERR_HIP;
}

extern "C" rose_status rose_object_bytes(const rose_plan *p, int64_t n_entries, size_t *bytes) {
    if (!p || !bytes || n_entries < 0) return ROSE_ERR_ARG;
    *bytes = rose::object_bytes_for(p->n_tensors, n_entries);
    return ROSE_OK;
}

static rose_status pack_common(const rose_plan *p, int32_t d, const rose_bucket *bucket, int32_t payload,
                               int64_t first_entry, int64_t n_entries, void *object, size_t object_bytes,
                               void *stream) {
    if (!p || !bucket || !object || d < 0 || d >= p->n_buckets || first_entry < 0 || n_entries < 0) return ROSE_ERR_ARG;
    if (payload != ROSE_PAYLOAD_NEW && payload != ROSE_PAYLOAD_ARITH) return ROSE_ERR_ARG;
    rose_status s = check_bucket(*bucket);
    if (s != ROSE_OK) return s;
    if (!aligned(object, 16)) return ROSE_ERR_ALIGN;
    if (first_entry + n_entries > bucket->capacity) return ROSE_ERR_ARG;
    if (object_bytes < rose::object_bytes_for(p->n_tensors, n_entries)) return ROSE_ERR_CAPACITY;
    rose::BucketDev b{bucket->idx, bucket->val, bucket->capacity, bucket->seg_off};
    return rose::launch_pack(b, d, p->n_tensors, first_entry, n_entries, payload, object, stream) == 0 ? ROSE_OK
                                                                                                       : ROSE_ERR_HIP;
}

extern "C" rose_status rose_bucket_pack(const rose_plan *p, int32_t d, const rose_bucket *bucket, int64_t first_entry,
                                        int64_t n_entries, void *object, size_t object_bytes, void *stream) {
    return pack_common(p, d, bucket, ROSE_PAYLOAD_NEW, first_entry, n_entries, object, object_bytes, stream);
}

extern "C" rose_status rose_bucket_pack_ex(const rose_plan *p, int32_t d, const rose_bucket *bucket, int32_t payload,
                                           int64_t first_entry, int64_t n_entries, void *object, size_t object_bytes,
                                           void *stream) {
    return pack_common(p, d, bucket, payload, first_entry, n_entries, object, object_bytes, stream);
}

extern "C" rose_status rose_object_apply(const rose_plan *p, const void *object, size_t object_bytes,
                                         void *const *dst_ptrs, void *stream) {
    if (!p || !object || !dst_ptrs) return ROSE_ERR_ARG;
    if (!aligned(object, 16) || !aligned(dst_ptrs, 8)) return ROSE_ERR_ALIGN;
    if (object_bytes < rose::object_bytes_for(p->n_tensors, 0)) return ROSE_ERR_ARG;
    rose_status s = device_tables(p);
    if (s != ROSE_OK) return s;
    // the validation pass leaves its verdict in one of the plan's words; tickets tell the calls apart
    const uint64_t ticket = p->verdict_ticket.fetch_add(1, std::memory_order_relaxed) + 1;
    return rose::launch_apply_object(object, object_bytes, p->n_tensors, p->n_buckets, p->tp, p->d_local_numel, dst_ptrs,
                                     p->d_verdict + ticket % kVerdictSlots, ticket, stream) == 0
               ? ROSE_OK
               : ROSE_ERR_HIP;
}

extern "C" rose_status rose_object_check(const rose_plan *p, const void *object, size_t object_bytes, void *stream,
                                         int32_t *shard, int64_t *first_entry, int64_t *n_entries,
                                         int32_t *payload) {
    if (!p || !object || object_bytes < 64) return ROSE_ERR_ARG;
    uint32_t h[16];
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(h, object, sizeof h, hipMemcpyDeviceToHost, st) != hipSuccess) return ROSE_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return ROSE_ERR_HIP;
    int64_t n = 0;
    if (!rose::object_header_valid(h, p->n_tensors, object_bytes, &n)) return ROSE_ERR_ARG;
    if ((int32_t)h[2] < 0 || (int32_t)h[2] >= p->n_buckets) return ROSE_ERR_ARG;
    if (shard) *shard = (int32_t)h[2];
    if (first_entry) *first_entry = (int64_t)((uint64_t)h[4] | ((uint64_t)h[5] << 32));
    if (n_entries) *n_entries = n;
    if (payload) *payload = (int32_t)h[8];
    return ROSE_OK;
}

// shard_plan: host-side planner (Sec. 4.2 "Shard-aware Weight Transfer": the sharded dimension
// of each parameter gives per-rank slice ranges).  Pure integer work, no HIP calls.
//
// Every (tensor, shard) segment is described in the SHARD-LOCAL index order, as a few pieces
// whose source elements are contiguous or equal runs at a fixed stride.  A tile is a run of
// kTile local indices of one piece, so a tile has one destination, its entries come out in
// ascending local index, and its loads are contiguous.  Tiles are numbered shard-major
// (all of shard 0's segments in tensor order, then shard 1's, ...): one prefix-sum chain per
// shard yields each entry's final position in that shard's bucket.
#include <cstring>
#include <new>

#include "rose_internal.h"

namespace rose {

void make_magic(uint32_t divisor, uint32_t *magic, uint32_t *shift) {
    // Round-up method for dividends below 2^31: with l = ceil(log2 divisor),
    // m = floor(2^(31+l) / divisor) + 1 fits 32 bits and k / divisor = (k * m) >> (31 + l).
    uint32_t l = 0;
    while ((1ull << l) < divisor) ++l;
    if (l == 0) l = 1;  // divisor 1: m = 2^32 would not fit; callers never divide by 1
    uint64_t m = ((1ull << (31 + l)) / divisor) + 1;
    *magic = (uint32_t)m;
    *shift = l - 1;     // after taking the high 32 bits of the product
}

static bool magic_ok(uint32_t divisor, uint32_t magic, uint32_t shift, uint32_t limit) {
    // exhaustive over the quotient boundaries inside [0, limit)
    for (uint64_t q = 0; q * divisor < limit; ++q) {
        uint64_t a = q * divisor, b = a + divisor - 1;
        if (b >= limit) b = limit - 1;
        if (magic_div((uint32_t)a, magic, shift) != q) return false;
        if (magic_div((uint32_t)b, magic, shift) != q) return false;
    }
    return true;
}

}  // namespace rose

using rose::Piece;

// bound_local: also require the shard-local size to fit an int32 index (the destination side; a
// sender's slice is addressed with 64-bit offsets and may be larger)
static rose_status check_desc(const rose_tensor_desc &t, int32_t tp, bool bound_local) {
    if (t.rows < 0 || t.cols < 0) return ROSE_ERR_ARG;
    switch (t.rule) {
    case ROSE_REPLICATED: break;
    case ROSE_SPLIT_ROWS: if (t.rows % tp) return ROSE_ERR_SHAPE; break;
    case ROSE_SPLIT_COLS: if (t.cols % tp) return ROSE_ERR_SHAPE; break;
    case ROSE_FUSED_ROWS: {
        if (t.n_sections < 1 || t.n_sections > ROSE_MAX_SECTIONS) return ROSE_ERR_ARG;
        int64_t sum = 0;
        for (int j = 0; j < t.n_sections; ++j) {
            if (t.section_rows[j] < 0) return ROSE_ERR_ARG;
            if (t.section_rows[j] % tp) return ROSE_ERR_SHAPE;
            sum += t.section_rows[j];
        }
        if (sum != t.rows) return ROSE_ERR_SHAPE;
        break;
    }
    default: return ROSE_ERR_ARG;
    }
    if (t.src_groups != 0) {
        if (t.rule != ROSE_FUSED_ROWS || t.src_groups < 0) return ROSE_ERR_ARG;
        for (int j = 0; j < t.n_sections; ++j)
            if (t.section_rows[j] % t.src_groups) return ROSE_ERR_SHAPE;
    }
    // guard rows * cols against int64 overflow, then bound the shard-local size
    if (t.cols != 0 && t.rows > (int64_t)(INT64_MAX / 4) / t.cols) return ROSE_ERR_UNSUPPORTED;
    int64_t local = t.rows * t.cols / (t.rule == ROSE_REPLICATED ? 1 : tp);
    if (bound_local && local >= (int64_t)1 << 31) return ROSE_ERR_UNSUPPORTED;
    return ROSE_OK;
}

static int64_t local_numel(const rose_tensor_desc &t, int32_t tp) {
    return t.rows * t.cols / (t.rule == ROSE_REPLICATED ? 1 : tp);
}

// does sender `src_rank` of `tp_src` send tensor ordinal ti?  A replicated tensor is held by every
// sender and sent by exactly one (dealt round robin); every other tensor is sent by all, each its slice.
static bool sends(const rose_tensor_desc &t, int32_t ti, int32_t tp_src, int32_t src_rank) {
    return t.rule != ROSE_REPLICATED || ti % tp_src == src_rank;
}

// Pipeline stage that holds a tensor (Sec. 4.2: the engine maps between TP and PP layouts of both
// sides): the decoder layers are dealt to the pp stages in equal consecutive groups, tensors marked
// ROSE_LAYER_FIRST (the embedding) go with the first stage, ROSE_LAYER_LAST (final norm, head) with
// the last.  With one stage everything is held by it, whatever the layer field says.
static int32_t stage_of(int32_t layer, int32_t n_layers, int32_t pp) {
    if (pp <= 1 || layer == ROSE_LAYER_FIRST) return 0;
    if (layer == ROSE_LAYER_LAST) return pp - 1;
    return layer / (n_layers / pp);
}

// pieces of segment (t, d) that sender s of S holds, in ascending local index, for prefix chain
// `chain` (= bucket); `here` = false: the sender does not hold the tensor, or the bucket's stage
// does not receive it (an empty segment)
static void segment_pieces(const rose_tensor_desc &t, int32_t ti, int32_t d, int32_t D, int32_t S, int32_t s,
                           int32_t chain, bool here, std::vector<Piece> &out) {
    size_t first = out.size();
    // a part of `len` elements in runs of `run`: the sender's slice advances by src_stride per run,
    // the destination's local index by lstride per run (both equal to run when contiguous)
    auto add = [&](int64_t src_off, int64_t src_stride, int64_t local_base, int64_t lstride, int64_t run,
                   int64_t len) {
        if (len <= 0) return;
        Piece p;
        std::memset(&p, 0, sizeof p);
        p.src_off = src_off;
        p.tensor = ti;
        p.shard = chain;
        p.local_base = (int32_t)local_base;
        p.len = (int32_t)len;
        const bool src_strided = run < len && src_stride != run;
        const bool dst_strided = run < len && lstride != run;
        const bool strided = src_strided || dst_strided;
        p.run = (int32_t)(strided ? run : len);
        p.stride = src_strided ? src_stride : p.run;
        p.lstride = (int32_t)(dst_strided ? lstride : p.run);
        if (src_strided) p.flags |= rose::kPieceStrided;
        if (dst_strided) p.flags |= rose::kPieceDstStrided;
        if (strided && run >= 2) rose::make_magic((uint32_t)run, &p.magic, &p.shift);
        bool vec = (src_off % rose::kVec == 0) && (local_base % rose::kVec == 0) &&
                   (!strided || run % rose::kVec == 0) && (!src_strided || src_stride % rose::kVec == 0) &&
                   (!dst_strided || lstride % rose::kVec == 0);
        if (strided && vec && !rose::magic_ok((uint32_t)run, p.magic, p.shift, (uint32_t)len)) vec = false;
        if (vec) p.flags |= rose::kPieceVec;
        out.push_back(p);
    };
    // rows (or columns) [lo, hi) that both the sender's block and the destination's block hold
    auto overlap = [](int64_t a0, int64_t a1, int64_t b0, int64_t b1, int64_t *lo, int64_t *hi) {
        *lo = a0 > b0 ? a0 : b0;
        *hi = a1 < b1 ? a1 : b1;
        return *hi > *lo;
    };
    const int64_t R = t.rows, C = t.cols;
    int64_t lo, hi;
    if (here && sends(t, ti, S, s)) {
        switch (t.rule) {
        case ROSE_REPLICATED:
            add(0, R * C, 0, R * C, R * C, R * C);
            if (out.size() > first) out.back().flags |= rose::kPieceReplicated;
            break;
        case ROSE_SPLIT_ROWS:
            if (overlap(s * (R / S), (s + 1) * (R / S), d * (R / D), (d + 1) * (R / D), &lo, &hi))
                add((lo - s * (R / S)) * C, 0, (lo - d * (R / D)) * C, 0, (hi - lo) * C, (hi - lo) * C);
            break;
        case ROSE_SPLIT_COLS:
            if (overlap(s * (C / S), (s + 1) * (C / S), d * (C / D), (d + 1) * (C / D), &lo, &hi))
                add(lo - s * (C / S), C / S, lo - d * (C / D), C / D, hi - lo, R * (hi - lo));
            break;
        case ROSE_FUSED_ROWS: {
            if (t.src_groups > 0) {
                // The sender keeps the tensor interleaved by head group and holds whole groups
                // [g0, g1).  In the destination's order (section, then row) the parts it holds of
                // section j are, group by group, the overlap of the group's rows with shard d's.
                const int64_t G = t.src_groups;
                const int64_t g0 = s * (G / S), g1 = (s + 1) * (G / S);
                int64_t group_rows = 0;
                for (int j = 0; j < t.n_sections; ++j) group_rows += t.section_rows[j] / G;
                int64_t before = 0, loc_row = 0;  // rows of earlier sections per group / per shard
                for (int j = 0; j < t.n_sections; ++j) {
                    const int64_t per_g = t.section_rows[j] / G, per_d = t.section_rows[j] / D;
                    for (int64_t g = g0; g < g1; ++g) {
                        if (overlap(g * per_g, (g + 1) * per_g, d * per_d, (d + 1) * per_d, &lo, &hi)) {
                            const int64_t src_row = (g - g0) * group_rows + before + (lo - g * per_g);
                            add(src_row * C, 0, (loc_row + lo - d * per_d) * C, 0, (hi - lo) * C, (hi - lo) * C);
                        }
                    }
                    before += per_g;
                    loc_row += per_d;
                }
                break;
            }
            int64_t src_row = 0, loc_row = 0;     // first row of section j in the sender's slice / the shard
            for (int j = 0; j < t.n_sections; ++j) {
                const int64_t per_s = t.section_rows[j] / S, per_d = t.section_rows[j] / D;
                if (overlap(s * per_s, (s + 1) * per_s, d * per_d, (d + 1) * per_d, &lo, &hi))
                    add((src_row + lo - s * per_s) * C, 0, (loc_row + lo - d * per_d) * C, 0, (hi - lo) * C,
                        (hi - lo) * C);
                src_row += per_s;
                loc_row += per_d;
            }
            break;
        }
        }
    }
    if (out.size() == first) {   // empty segment: keep one empty piece so the segment has a tile
        Piece p;
        std::memset(&p, 0, sizeof p);
        p.tensor = ti;
        p.shard = chain;
        p.run = 0;
        out.push_back(p);
    }
    out[first].flags |= rose::kPieceFirst;
}

extern "C" rose_status rose_shard_plan_create_pp(const rose_tensor_desc *tensors, int32_t n_tensors, int32_t tp,
                                                 int32_t tp_src, int32_t src_rank, int32_t n_layers, int32_t pp_src,
                                                 int32_t stage_src, int32_t pp_dst, rose_plan **out) {
    if (!out) return ROSE_ERR_ARG;
    *out = nullptr;
    if (!tensors || n_tensors < 1 || tp < 1 || tp_src < 1 || src_rank < 0 || src_rank >= tp_src) return ROSE_ERR_ARG;
    if (pp_src < 1 || pp_dst < 1 || stage_src < 0 || stage_src >= pp_src || n_layers < 0) return ROSE_ERR_ARG;
    if (tp > ROSE_MAX_TP || tp_src > ROSE_MAX_TP || pp_dst > ROSE_MAX_TP || tp * pp_dst > ROSE_MAX_TP ||
        pp_src > (1 << 20))
        return ROSE_ERR_UNSUPPORTED;
    const bool staged = pp_src > 1 || pp_dst > 1;
    if (staged && (n_layers < 1 || n_layers % pp_src || n_layers % pp_dst)) return ROSE_ERR_SHAPE;
    for (int32_t i = 0; i < n_tensors; ++i) {
        rose_status s = check_desc(tensors[i], tp, true);
        if (s == ROSE_OK) s = check_desc(tensors[i], tp_src, false);
        if (s == ROSE_OK && tensors[i].src_groups > 0 && tensors[i].src_groups % tp_src) s = ROSE_ERR_SHAPE;
        if (s == ROSE_OK && staged && tensors[i].layer != ROSE_LAYER_FIRST && tensors[i].layer != ROSE_LAYER_LAST &&
            (tensors[i].layer < 0 || tensors[i].layer >= n_layers))
            s = ROSE_ERR_ARG;
        if (s != ROSE_OK) return s;
    }
    rose_plan *p = new (std::nothrow) rose_plan;
    if (!p) return ROSE_ERR_ARG;
    try {
        p->tp = tp;
        p->tp_src = tp_src;
        p->src_rank = src_rank;
        p->n_layers = n_layers;
        p->pp_src = pp_src;
        p->stage_src = stage_src;
        p->pp_dst = pp_dst;
        p->n_buckets = tp * pp_dst;
        p->n_tensors = n_tensors;
        p->tensors.assign(tensors, tensors + n_tensors);
        p->stage_src_of.resize(n_tensors);
        p->stage_dst_of.resize(n_tensors);
        p->global_base.resize(n_tensors + 1);
        p->global_base[0] = 0;
        for (int32_t i = 0; i < n_tensors; ++i) {
            p->global_base[i + 1] = p->global_base[i] + tensors[i].rows * tensors[i].cols;
            p->stage_src_of[i] = stage_of(tensors[i].layer, n_layers, pp_src);
            p->stage_dst_of[i] = stage_of(tensors[i].layer, n_layers, pp_dst);
        }
        int64_t n_tiles = 0;
        for (int32_t b = 0; b < p->n_buckets; ++b) {
            const int32_t stage_dst = b / tp, d = b % tp;
            p->chain_first[b] = (int32_t)n_tiles;
            for (int32_t i = 0; i < n_tensors; ++i) {
                size_t first = p->pieces.size();
                const bool here = p->stage_src_of[i] == stage_src && p->stage_dst_of[i] == stage_dst;
                segment_pieces(tensors[i], i, d, tp, tp_src, src_rank, b, here, p->pieces);
                for (size_t k = first; k < p->pieces.size(); ++k) {
                    Piece &pc = p->pieces[k];
                    int64_t nt = pc.len == 0 ? 1 : ((int64_t)pc.len + rose::kTile - 1) / rose::kTile;
                    if (n_tiles + nt >= ((int64_t)1 << 31) - 1) {
                        delete p;
                        return ROSE_ERR_UNSUPPORTED;
                    }
                    pc.first_tile = (int32_t)n_tiles;
                    n_tiles += nt;
                    p->tile_piece.insert(p->tile_piece.end(), (size_t)nt, (int32_t)k);
                }
            }
        }
        for (int32_t b = p->n_buckets; b <= ROSE_MAX_TP; ++b) p->chain_first[b] = (int32_t)n_tiles;
        for (const Piece &pc : p->pieces) p->capacity_sum += pc.len;
        int32_t n_blocks = 0;
        for (int32_t b = 0; b <= ROSE_MAX_TP; ++b) {
            p->block_first[b] = n_blocks;
            if (b < p->n_buckets) n_blocks += (p->chain_first[b + 1] - p->chain_first[b] + rose::kBlock - 1) / rose::kBlock;
        }
    } catch (...) {
        delete p;
        return ROSE_ERR_ARG;
    }
    *out = p;
    return ROSE_OK;
}

extern "C" rose_status rose_shard_plan_create_src(const rose_tensor_desc *tensors, int32_t n_tensors, int32_t tp,
                                                  int32_t tp_src, int32_t src_rank, rose_plan **out) {
    return rose_shard_plan_create_pp(tensors, n_tensors, tp, tp_src, src_rank, 0, 1, 0, 1, out);
}

extern "C" rose_status rose_shard_plan_create(const rose_tensor_desc *tensors, int32_t n_tensors,
                                              int32_t tp, rose_plan **out) {
    return rose_shard_plan_create_pp(tensors, n_tensors, tp, 1, 0, 0, 1, 0, 1, out);
}

extern "C" int32_t rose_plan_n_tensors(const rose_plan *p) { return p ? p->n_tensors : -1; }
extern "C" int32_t rose_plan_tp(const rose_plan *p) { return p ? p->tp : -1; }
extern "C" int32_t rose_plan_n_buckets(const rose_plan *p) { return p ? p->n_buckets : -1; }

extern "C" rose_status rose_plan_stage_of(const rose_plan *p, int32_t t, int32_t *stage_src, int32_t *stage_dst) {
    if (!p || t < 0 || t >= p->n_tensors) return ROSE_ERR_ARG;
    if (stage_src) *stage_src = p->stage_src_of[t];
    if (stage_dst) *stage_dst = p->stage_dst_of[t];
    return ROSE_OK;
}

// does an encode launch with these flags dereference the old / new pointers of tensor t?
static bool tensor_is_read(const rose_plan *p, int32_t t, uint32_t flags) {
    const rose_tensor_desc &d = p->tensors[t];
    if (p->stage_src_of[t] != p->stage_src || d.rows * d.cols == 0) return false;
    if (sends(d, t, p->tp_src, p->src_rank)) return true;
    return (flags & ROSE_ENCODE_REFRESH) != 0;     // held but not sent (replicated): only the refresh copy touches it
}

extern "C" rose_status rose_plan_tensor_is_read(const rose_plan *p, int32_t t, uint32_t flags, int32_t *is_read) {
    if (!p || !is_read || t < 0 || t >= p->n_tensors) return ROSE_ERR_ARG;
    if (flags & ~(uint32_t)(ROSE_ENCODE_REFRESH | ROSE_ENCODE_ARITH)) return ROSE_ERR_ARG;
    *is_read = tensor_is_read(p, t, flags) ? 1 : 0;
    return ROSE_OK;
}

extern "C" rose_status rose_plan_set_tile_order(rose_plan *p, int32_t order) {
    if (!p || order < ROSE_TILE_ORDER_AUTO_PICK || order > ROSE_TILE_ORDER_TIMED) return ROSE_ERR_ARG;
    p->tile_order.store(order, std::memory_order_relaxed);
    return ROSE_OK;
}

extern "C" rose_status rose_plan_set_worker_cap(rose_plan *p, int32_t workers) {
    if (!p || workers < 0) return ROSE_ERR_ARG;
    p->worker_cap.store(workers, std::memory_order_relaxed);
    return ROSE_OK;
}

extern "C" rose_status rose_plan_tensor_base(const rose_plan *p, int32_t t, int64_t *global_base) {
    if (!p || !global_base || t < 0 || t > p->n_tensors) return ROSE_ERR_ARG;
    *global_base = p->global_base[t];
    return ROSE_OK;
}

extern "C" rose_status rose_plan_local_numel(const rose_plan *p, int32_t t, int32_t d, int64_t *numel) {
    if (!p || !numel || t < 0 || t >= p->n_tensors || d < 0 || d >= p->n_buckets) return ROSE_ERR_ARG;
    *numel = p->stage_dst_of[t] == d / p->tp ? local_numel(p->tensors[t], p->tp) : 0;
    return ROSE_OK;
}

extern "C" rose_status rose_plan_bucket_capacity(const rose_plan *p, int32_t d, int64_t *max_entries) {
    if (!p || !max_entries || d < 0 || d >= p->n_buckets) return ROSE_ERR_ARG;
    int64_t s = 0;                              // everything this sender can send to shard d
    for (const Piece &pc : p->pieces)
        if (pc.shard == d) s += pc.len;
    *max_entries = s;
    return ROSE_OK;
}

extern "C" rose_status rose_plan_src_numel(const rose_plan *p, int32_t t, int64_t *numel) {
    if (!p || !numel || t < 0 || t >= p->n_tensors) return ROSE_ERR_ARG;
    *numel = p->stage_src_of[t] == p->stage_src ? local_numel(p->tensors[t], p->tp_src) : 0;
    return ROSE_OK;
}

extern "C" rose_status rose_plan_n_tiles(const rose_plan *p, int64_t *n_tiles) {
    if (!p || !n_tiles) return ROSE_ERR_ARG;
    *n_tiles = (int64_t)p->tile_piece.size();
    return ROSE_OK;
}

extern "C" rose_status rose_plan_workspace_bytes(const rose_plan *p, size_t *bytes) {
    if (!p || !bytes) return ROSE_ERR_ARG;
    // header + one 64-bit descriptor per tile + one per block of tiles
    *bytes = rose::kWsHeaderBytes +
             (p->tile_piece.size() + (size_t)p->block_first[p->n_buckets]) * sizeof(unsigned long long);
    return ROSE_OK;
}

// Test hook: answers from the piece tables the kernels use, not from the rule formulas, so a
// wrong table shows up on the host.
extern "C" rose_status rose_plan_map_index(const rose_plan *p, int32_t t, int64_t g, int32_t *d_first,
                                           int32_t *n_dest, int32_t *local) {
    if (!p || !d_first || !n_dest || !local || t < 0 || t >= p->n_tensors) return ROSE_ERR_ARG;
    if (p->stage_src_of[t] != p->stage_src) return ROSE_ERR_ARG;          // not held by this sender
    if (g < 0 || g >= local_numel(p->tensors[t], p->tp_src)) return ROSE_ERR_ARG;
    int found = 0;
    for (const Piece &pc : p->pieces) {
        if (pc.tensor != t || pc.len == 0) continue;
        int64_t rel = g - pc.src_off;
        if (rel < 0) continue;
        int64_t k;
        if (pc.flags & rose::kPieceStrided) {
            int64_t row = rel / pc.stride, in = rel % pc.stride;
            if (in >= pc.run) continue;
            k = row * pc.run + in;
        } else {
            k = rel;
        }
        if (k >= pc.len) continue;
        int32_t loc = pc.local_base + (int32_t)k;
        if (pc.flags & rose::kPieceDstStrided) loc = pc.local_base + (int32_t)((k / pc.run) * pc.lstride + k % pc.run);
        if (!found) {
            *d_first = pc.shard;
            *local = loc;
        } else if (*local != loc || pc.shard != *d_first + found) {
            return ROSE_ERR_ARG;   // tables inconsistent
        }
        ++found;
    }
    if (!found) {
        // a replicated tensor that another sender sends has no destination from here
        if (sends(p->tensors[t], t, p->tp_src, p->src_rank)) return ROSE_ERR_ARG;
        *d_first = 0;
        *local = 0;
    }
    *n_dest = found;
    return ROSE_OK;
}

extern "C" const char *rose_status_str(rose_status s) {
    switch (s) {
    case ROSE_OK: return "ok";
    case ROSE_ERR_ARG: return "invalid argument";
    case ROSE_ERR_SHAPE: return "shape not divisible by the tensor-parallel degree";
    case ROSE_ERR_CAPACITY: return "bucket capacity exceeded";
    case ROSE_ERR_ALIGN: return "pointer not aligned";
    case ROSE_ERR_HIP: return "HIP runtime error";
    case ROSE_ERR_UNSUPPORTED: return "unsupported size";
    case ROSE_ERR_SCRATCH:
        return "the plan is not resident on this device (rose_plan_upload), or it needs more scratch than the "
               "library's built-in buffer holds";
    }
    return "unknown status";
}

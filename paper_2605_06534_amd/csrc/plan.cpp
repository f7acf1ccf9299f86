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

static rose_status check_desc(const rose_tensor_desc &t, int32_t tp) {
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
    // guard rows * cols against int64 overflow, then bound the shard-local size
    if (t.cols != 0 && t.rows > (int64_t)(INT64_MAX / 4) / t.cols) return ROSE_ERR_UNSUPPORTED;
    int64_t local = t.rows * t.cols / (t.rule == ROSE_REPLICATED ? 1 : tp);
    if (local >= (int64_t)1 << 31) return ROSE_ERR_UNSUPPORTED;
    return ROSE_OK;
}

static int64_t local_numel(const rose_tensor_desc &t, int32_t tp) {
    return t.rows * t.cols / (t.rule == ROSE_REPLICATED ? 1 : tp);
}

// pieces of segment (t, d), in ascending local index
static void segment_pieces(const rose_tensor_desc &t, int32_t ti, int32_t d, int32_t tp,
                           std::vector<Piece> &out) {
    size_t first = out.size();
    auto add = [&](int64_t src_off, int64_t local_base, int64_t len, int64_t run, int64_t stride) {
        if (len <= 0) return;
        Piece p;
        std::memset(&p, 0, sizeof p);
        p.src_off = src_off;
        p.tensor = ti;
        p.shard = d;
        p.local_base = (int32_t)local_base;
        p.len = (int32_t)len;
        bool strided = run < len && stride != run;
        p.run = (int32_t)(strided ? run : len);
        p.stride = strided ? stride : len;
        if (strided) {
            p.flags |= rose::kPieceStrided;
            if (run >= 2) rose::make_magic((uint32_t)run, &p.magic, &p.shift);
        }
        bool vec = (src_off % rose::kVec == 0) && (local_base % rose::kVec == 0) &&
                   (!strided || (run % rose::kVec == 0 && stride % rose::kVec == 0));
        if (strided && vec && !rose::magic_ok((uint32_t)run, p.magic, p.shift, (uint32_t)len)) vec = false;
        if (vec) p.flags |= rose::kPieceVec;
        out.push_back(p);
    };
    const int64_t R = t.rows, C = t.cols;
    switch (t.rule) {
    case ROSE_REPLICATED: add(0, 0, R * C, R * C, R * C); break;
    case ROSE_SPLIT_ROWS: add(d * (R / tp) * C, 0, (R / tp) * C, (R / tp) * C, 0); break;
    case ROSE_SPLIT_COLS: add(d * (C / tp), 0, R * (C / tp), C / tp, C); break;
    case ROSE_FUSED_ROWS: {
        int64_t sec_row = 0, loc_row = 0;
        for (int j = 0; j < t.n_sections; ++j) {
            int64_t per = t.section_rows[j] / tp;
            add((sec_row + d * per) * C, loc_row * C, per * C, per * C, 0);
            sec_row += t.section_rows[j];
            loc_row += per;
        }
        break;
    }
    }
    if (out.size() == first) {   // empty segment: keep one empty piece so the segment has a tile
        Piece p;
        std::memset(&p, 0, sizeof p);
        p.tensor = ti;
        p.shard = d;
        p.run = 0;
        out.push_back(p);
    }
    out[first].flags |= rose::kPieceFirst;
}

extern "C" rose_status rose_shard_plan_create(const rose_tensor_desc *tensors, int32_t n_tensors,
                                              int32_t tp, rose_plan **out) {
    if (!out) return ROSE_ERR_ARG;
    *out = nullptr;
    if (!tensors || n_tensors < 1 || tp < 1) return ROSE_ERR_ARG;
    if (tp > ROSE_MAX_TP) return ROSE_ERR_UNSUPPORTED;
    for (int32_t i = 0; i < n_tensors; ++i) {
        rose_status s = check_desc(tensors[i], tp);
        if (s != ROSE_OK) return s;
    }
    rose_plan *p = new (std::nothrow) rose_plan;
    if (!p) return ROSE_ERR_ARG;
    try {
        p->tp = tp;
        p->n_tensors = n_tensors;
        p->tensors.assign(tensors, tensors + n_tensors);
        p->global_base.resize(n_tensors + 1);
        p->global_base[0] = 0;
        for (int32_t i = 0; i < n_tensors; ++i)
            p->global_base[i + 1] = p->global_base[i] + tensors[i].rows * tensors[i].cols;
        int64_t n_tiles = 0;
        for (int32_t d = 0; d < tp; ++d) {
            p->chain_first[d] = (int32_t)n_tiles;
            for (int32_t i = 0; i < n_tensors; ++i) {
                size_t first = p->pieces.size();
                segment_pieces(tensors[i], i, d, tp, p->pieces);
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
        for (int32_t d = tp; d <= ROSE_MAX_TP; ++d) p->chain_first[d] = (int32_t)n_tiles;
        int32_t n_blocks = 0;
        for (int32_t d = 0; d <= ROSE_MAX_TP; ++d) {
            p->block_first[d] = n_blocks;
            if (d < tp) n_blocks += (p->chain_first[d + 1] - p->chain_first[d] + rose::kBlock - 1) / rose::kBlock;
        }
    } catch (...) {
        delete p;
        return ROSE_ERR_ARG;
    }
    *out = p;
    return ROSE_OK;
}

extern "C" int32_t rose_plan_n_tensors(const rose_plan *p) { return p ? p->n_tensors : -1; }
extern "C" int32_t rose_plan_tp(const rose_plan *p) { return p ? p->tp : -1; }

extern "C" rose_status rose_plan_tensor_base(const rose_plan *p, int32_t t, int64_t *global_base) {
    if (!p || !global_base || t < 0 || t > p->n_tensors) return ROSE_ERR_ARG;
    *global_base = p->global_base[t];
    return ROSE_OK;
}

extern "C" rose_status rose_plan_local_numel(const rose_plan *p, int32_t t, int32_t d, int64_t *numel) {
    if (!p || !numel || t < 0 || t >= p->n_tensors || d < 0 || d >= p->tp) return ROSE_ERR_ARG;
    *numel = local_numel(p->tensors[t], p->tp);
    return ROSE_OK;
}

extern "C" rose_status rose_plan_bucket_capacity(const rose_plan *p, int32_t d, int64_t *max_entries) {
    if (!p || !max_entries || d < 0 || d >= p->tp) return ROSE_ERR_ARG;
    int64_t s = 0;
    for (const auto &t : p->tensors) s += local_numel(t, p->tp);
    *max_entries = s;
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
             (p->tile_piece.size() + (size_t)p->block_first[p->tp]) * sizeof(unsigned long long);
    return ROSE_OK;
}

// Test hook: answers from the piece tables the kernels use, not from the rule formulas, so a
// wrong table shows up on the host.
extern "C" rose_status rose_plan_map_index(const rose_plan *p, int32_t t, int64_t g, int32_t *d_first,
                                           int32_t *n_dest, int32_t *local) {
    if (!p || !d_first || !n_dest || !local || t < 0 || t >= p->n_tensors) return ROSE_ERR_ARG;
    const rose_tensor_desc &td = p->tensors[t];
    if (g < 0 || g >= td.rows * td.cols) return ROSE_ERR_ARG;
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
        if (!found) {
            *d_first = pc.shard;
            *local = pc.local_base + (int32_t)k;
        } else if (*local != pc.local_base + (int32_t)k || pc.shard != *d_first + found) {
            return ROSE_ERR_ARG;   // tables inconsistent
        }
        ++found;
    }
    if (!found) return ROSE_ERR_ARG;
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
    }
    return "unknown status";
}

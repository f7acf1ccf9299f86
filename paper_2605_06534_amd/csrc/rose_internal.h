// Internal declarations shared by the host planner, the C ABI and the kernel launchers.
#pragma once

#include <atomic>
#include <cstddef>
#include <cstdint>
#include <mutex>
#include <vector>

#include "rose_delta.h"

namespace rose {

// Tile geometry of the encode / dense-copy kernels: one workgroup of kThreads lanes walks one
// tile; a lane takes kIters vectors of kVec 16-bit elements (one 128-bit load each).
#ifndef ROSE_THREADS
#define ROSE_THREADS 256
#endif
constexpr int kThreads = ROSE_THREADS;
constexpr int kWaves = kThreads / 64;
constexpr int kVec = 8;
#ifndef ROSE_ITERS
#define ROSE_ITERS 4
#endif
constexpr int kIters = ROSE_ITERS;
constexpr int kWaveSpan = 64 * kVec * kIters;      // elements one wave covers in a tile
constexpr int kTile = kThreads * kVec * kIters;    // elements per tile

enum : int32_t {
    kPieceFirst = 1,    // first piece of its (tensor, shard) segment
    kPieceVec = 2,      // offsets and run lengths are multiples of kVec: 128-bit loads are legal
    kPieceStrided = 4,  // runs of `run` elements every `stride` source elements
    kPieceReplicated = 16, // piece of a replicated tensor: several destinations read the same source
    kPieceDstStrided = 8 // runs of `run` elements every `lstride` LOCAL indices (the sender's slice
                        // covers only part of each row of the destination shard)
};

// One part of a (tensor, shard) segment: element k = 0 .. len-1 of the piece lies at
//   source element  src_off + k                              (contiguous)
//                   src_off + (k / run) * stride + k % run   (kPieceStrided: a column block of a
//                                                             row-parallel matrix)
//   local index     local_base + k                           (contiguous)
//                   local_base + (k / run) * lstride + k % run   (kPieceDstStrided)
// Both are ascending in k.
struct Piece {
    int64_t src_off;
    int64_t stride;
    int32_t tensor;
    int32_t shard;
    int32_t local_base;
    int32_t len;
    int32_t run;
    uint32_t magic;      // k / run == mulhi(k, magic) >> shift for k < 2^31 (run >= 2)
    uint32_t shift;
    int32_t first_tile;
    int32_t flags;
    int32_t lstride;
};
static_assert(sizeof(Piece) == 56, "Piece layout is shared with device code");

struct BucketDev {
    int32_t *idx;
    uint16_t *val;
    int64_t capacity;
    int64_t *seg_off;
};

struct EncodeArgs {
    BucketDev bucket[ROSE_MAX_TP];
    int32_t chain_first[ROSE_MAX_TP + 1];   // first tile of each shard's chain; [tp] = n_tiles
    const Piece *pieces;
    const int32_t *tile_piece;
    const void *const *old_ptrs;
    const void *const *new_ptrs;
    int32_t block_first[ROSE_MAX_TP + 1];   // first block descriptor of each shard's chain
    unsigned long long *tile_desc;          // one descriptor per tile
    unsigned long long *block_desc;         // one descriptor per block of kBlock tiles of a chain
    unsigned int *abort_flag;               // workspace header: set when a wait gave up
    int32_t n_tiles;
    int32_t n_blocks;
    int32_t n_tensors;
    int32_t tp;
    int32_t n_server_wgs;                   // workgroups 0 .. n_server_wgs-1 serve prefixes, the rest walk tiles
    int32_t n_servers;                      // waves that serve prefixes (kWaves per serving workgroup)
    int32_t n_tickets;                      // tickets the counter hands out
    int32_t adjacent;                       // a ticket's tiles are neighbours in the bucket (see ticket_tile)
    int32_t batch;                          // tiles per ticket
    int32_t timed;                          // bucket stores go out in shared windows of time (see encode_body)
    unsigned int *ticket;                   // workspace header: the ticket counter
};

// Tiles of one chain are grouped in blocks of kBlock; a serving wave gathers a block's counts
// and hands every tile of the block its prefix.
constexpr int kBlock = 64;

// workspace layout (bytes): header, tile descriptors, block descriptors
// A ticket hands a worker a batch of tiles: the tiles at one position of as many consecutive blocks
// (a "group" of blocks has kBlock tickets).  All tickets come from one counter, in order.  The
// counter serves one ticket in about 14 ns, whoever asks: with 3 tiles (96 KB of input) per ticket it
// alone caps a launch at about 6 TB/s, which the other tile orders do not reach anyway; the timed
// order does, and takes 4.
#ifndef ROSE_BATCH
#define ROSE_BATCH 3
#endif
#ifndef ROSE_BATCH_TIMED
#define ROSE_BATCH_TIMED 4
#endif
constexpr int kBatch = ROSE_BATCH, kBatchTimed = ROSE_BATCH_TIMED;

constexpr size_t kWsAbortOff = 0;
constexpr int kWsCarefulWord = 2;      // 32-bit word 2 of the header counts same-group ticket pairs (diagnostic)
constexpr int kWsAheadWord = 3;        // 32-bit word 3: how often tiles were counted ahead of a wait (diagnostic)
constexpr size_t kWsTicketOff = 4096;
constexpr size_t kWsHeaderBytes = 8192;

struct CopyArgs {
    const Piece *pieces;
    const int32_t *tile_piece;
    const void *const *new_ptrs;
    void *const *dst_ptrs;
    int32_t tile_begin;
    int32_t n_tiles;
};

// host side of the magic-number division used for strided pieces
void make_magic(uint32_t divisor, uint32_t *magic, uint32_t *shift);
inline uint32_t magic_div(uint32_t k, uint32_t magic, uint32_t shift) {
    return (uint32_t)(((uint64_t)k * magic) >> 32) >> shift;
}

// kernel launchers (kernels.hip); all return a hipError_t as int
// replicated tensors to copy new -> old after an encode with refresh (device arrays of n entries)
struct RefreshArgs {
    const int32_t *list;
    const int64_t *numel;
    int32_t n;
};
// resident: workgroups of this kernel variant that fit on the device at once (encode_resident_all);
// worker_cap: 0, or the most workgroups that may walk tiles; order: ROSE_TILE_ORDER_SPREAD, _NEIGHBOURS or _TIMED
int launch_encode(const EncodeArgs &a, int new_is_f32, const RefreshArgs *refresh, int arith, int resident,
                  int worker_cap, int order, void *stream);
// resident workgroups of each of the eight encode kernel variants on the current device
// (index: fp32 input + 2 * refresh + 4 * arithmetic payload)
int encode_resident_all(int resident[8]);
// Address and size of the library's built-in scratch array on the current device (one array per
// device, found once per device with hipGetSymbolAddress and kept).
int static_scratch(void **ptr, size_t *bytes);
// shard_elems: elements of the destination shard's tensors together (the kernel compares the entry
// count with it to choose how it walks the entries)
int launch_apply(const BucketDev &b, int32_t n_tensors, const int32_t *local_numel, void *const *dst_ptrs,
                 int arith, int64_t shard_elems, void *stream);
int launch_dense_copy(const CopyArgs &a, int new_is_f32, void *stream);
int launch_pack(const BucketDev &b, int32_t shard, int32_t n_tensors, int64_t first, int64_t n, int32_t payload,
                void *object, void *stream);
// local_numel: [n_stages][n_tensors]; the object's shard word b selects row b / tp.  verdict: one word of
// device memory that belongs to this call until its kernels have run; ticket: a value no other call
// that shares the word uses.
int launch_apply_object(const void *object, size_t object_bytes, int32_t n_tensors, int32_t n_buckets, int32_t tp,
                        const int32_t *local_numel, void *const *dst_ptrs, unsigned long long *verdict,
                        unsigned long long ticket, void *stream);
size_t object_bytes_for(int32_t n_tensors, int64_t n);
bool object_header_valid(const uint32_t *header, int32_t n_tensors, size_t object_bytes, int64_t *n);
int launch_bw_probe(const void *src, void *dst, size_t bytes, uint64_t *sink, void *stream);
int launch_bw_probe_lines(void *dst, size_t n_lines, uint32_t threshold, void *stream);
int launch_bw_probe_mixed(const void *a, const void *b, void *dst, size_t n_chunks, uint32_t w16, int timed,
                          uint64_t *sink, void *stream);

}  // namespace rose

// words of device memory that object applies use to hand the validation pass's verdict to the apply pass
constexpr int kVerdictSlots = 4096;

struct rose_plan {
    int32_t tp_src = 1, src_rank = 0;          // the sender holds shard src_rank of tp_src of every tensor
    int32_t tp = 0;
    // pipeline stages (Sec. 4.2: TP and PP on both sides): the sender is stage stage_src of pp_src and holds
    // the tensors of that stage only; the receiving side has pp_dst stages of tp shards each.  Bucket (and
    // prefix chain) b = stage * tp + shard.
    int32_t n_layers = 0, pp_src = 1, stage_src = 0, pp_dst = 1;
    int32_t n_buckets = 0;                     // tp * pp_dst
    int32_t n_tensors = 0;
    std::vector<rose_tensor_desc> tensors;
    std::vector<int32_t> stage_src_of, stage_dst_of;   // [n_tensors] stage that holds each tensor on either side
    std::vector<int64_t> global_base;          // [n_tensors + 1]
    std::vector<rose::Piece> pieces;
    std::vector<int32_t> tile_piece;           // piece of each tile
    int32_t chain_first[ROSE_MAX_TP + 1] = {0};
    int32_t block_first[ROSE_MAX_TP + 1] = {0};
    mutable std::atomic<int32_t> worker_cap{0};     // rose_plan_set_worker_cap
    mutable std::atomic<int32_t> tile_order{0};     // rose_plan_set_tile_order
    mutable std::atomic<int32_t> seen_density_ppm{-1};   // changed elements per million as estimated from the last
                                                         // bucket total that rose_bucket_check read back (-1: none yet)
    int64_t capacity_sum = 0;                            // entries of all buckets together if every element changed
    mutable std::atomic<uint64_t> verdict_ticket{0};
    // device copies of pieces / tile_piece, made on first use on a device (the only device the plan is used on)
    mutable std::mutex mu;
    mutable int device = -1;
    mutable rose::Piece *d_pieces = nullptr;
    mutable int32_t *d_tile_piece = nullptr;
    mutable int32_t *d_local_numel = nullptr;  // [pp_dst][n_tensors] elements of a shard's copy of each tensor
                                               // (0 where the stage does not hold the tensor)
    mutable int32_t *d_repl_list = nullptr;    // replicated tensors this sender holds (ordinals) and their sizes
    mutable int64_t *d_repl_numel = nullptr;
    mutable int32_t n_repl = 0;
    mutable unsigned long long *d_verdict = nullptr;   // [kVerdictSlots]
    mutable int resident[8] = {0};             // see encode_resident_all
    mutable void *static_ws = nullptr;         // the library's built-in scratch on `device`
    mutable size_t static_ws_bytes = 0;
};

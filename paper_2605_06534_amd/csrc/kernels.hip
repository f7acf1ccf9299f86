// HIP kernels for gfx950 (wave64): diff + mask + count + scan + shard-aware bucket write
// (Sec. 4.2 "Sparsity-aware Weight Transfer", App. F D2S), scatter-apply (App. F S2D), the dense
// shard copy (Sec. 4.2 "Shard-aware Weight Transfer"), transport objects (Sec. 4.2 "Asynchronous
// Weight Transfer") and bandwidth probes.
//
// Everything here is bound by HBM traffic; there is no contraction, so no MFMA.  The encode
// kernel reads each weight once with 128-bit loads and writes only the changed entries.
#include <hip/hip_runtime.h>

#include <mutex>

#include "rose_internal.h"

namespace rose {

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------

typedef unsigned long long u64;

__device__ __forceinline__ uint32_t rne_bf16(uint32_t u) {
    // fp32 pattern -> bf16 pattern, nearest, ties to even: add half an ulp of the kept part
    // minus one, plus the lowest kept bit, then truncate.  NaN keeps its top bits, quieted.
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x0040u) : r;
}

__device__ __forceinline__ uint32_t pack_rne(uint32_t lo, uint32_t hi) {
    return (rne_bf16(lo) & 0xFFFFu) | (rne_bf16(hi) << 16);
}

// 8-bit mask of the 16-bit lanes of x that are non-zero (bit e = element e, little endian).
// A packed 16-bit min with 1 turns the two halves of a dword into 0 / 1 (bits 0 and 16) in one
// instruction; the four dwords are merged first (even elements in bits 0,2,4,6, odd ones in
// 16,18,20,22) and the odd ones folded down at the end.
__device__ __forceinline__ uint32_t nz16_pair(uint32_t x) {
    uint32_t b;
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(b) : "v"(x), "v"(0x00010001u));
    return b;
}
__device__ __forceinline__ uint32_t nz16_mask(uint4 x) {
    const uint32_t t = nz16_pair(x.x) | (nz16_pair(x.y) << 2) | (nz16_pair(x.z) << 4) | (nz16_pair(x.w) << 6);
    return (t | (t >> 15)) & 0xFFu;
}

// element e (0..7) of a vector of eight 16-bit patterns
__device__ __forceinline__ uint32_t pick16(uint4 v, uint32_t e) {
    uint32_t a = (e & 4u) ? ((e & 2u) ? v.w : v.z) : ((e & 2u) ? v.y : v.x);
    return (e & 1u) ? (a >> 16) : (a & 0xFFFFu);
}

// ---------------------------------------------------------------------------------------------
// Arithmetic payload (Sec. 4.2 writes the update as W_t = W_{t-1} + dW_t).  An entry carries
// d = bf16(new - old) if d is a number and bf16(old + d) is exactly the new pattern; otherwise it
// carries the new pattern and bit 31 of its index says so (escape).  Sums and differences of two
// bf16 values are formed in fp32 and rounded to nearest even: the fp32 result is exact unless the
// operands lie more than 16 binades apart, and then it sits so close to the larger operand that
// the second rounding cannot cross a tie, so the result is the correctly rounded bf16 one.
// Subnormals are kept (the kernels are built with IEEE denormal handling for fp32).
// ---------------------------------------------------------------------------------------------
#ifndef ROSE_ARITH_HWCVT
#define ROSE_ARITH_HWCVT 1     // 1: round with the packed fp32 -> bf16 conversion instruction (checked against
                               // the integer rounding below and the CPU reference on all 2^32 pattern pairs;
                               // 7B workload at 5 %: encode 5.60 ms instead of 6.14 ms)
#endif
// the two fp32 values rounded to bf16 (nearest even), packed: lo in bits 0..15, hi in 16..31.
// A NaN stays a NaN (its low 16 bits are zero here, so the rounding add cannot carry out of them).
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
#if ROSE_ARITH_HWCVT
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
    return r;
#else
    const uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    const uint32_t ra = a + 0x7FFFu + ((a >> 16) & 1u), rb = b + 0x7FFFu + ((b >> 16) & 1u);
    return (ra >> 16) | (rb & 0xFFFF0000u);
#endif
}
// payloads of the two elements of a dword; *b01 gets 1 in bit 0 / bit 16 for an escaped element
__device__ __forceinline__ uint32_t arith_pair(uint32_t o, uint32_t n, uint32_t *b01) {
    const float ol = __uint_as_float(o << 16), oh = __uint_as_float(o & 0xFFFF0000u);
    const float nl = __uint_as_float(n << 16), nh = __uint_as_float(n & 0xFFFF0000u);
    const uint32_t d = pack_bf16_pair(nl - ol, nh - oh);
    const uint32_t back = pack_bf16_pair(ol + __uint_as_float(d << 16), oh + __uint_as_float(d & 0xFFFF0000u));
    // a half of (mx ^ 0x7F80...) is non-zero where d is a NaN: magnitude above the pattern of infinity
    uint32_t mx;
    asm("v_pk_max_u16 %0, %1, %2" : "=v"(mx) : "v"(d & 0x7FFF7FFFu), "v"(0x7F807F80u));
    const uint32_t bad = (back ^ n) | (mx ^ 0x7F807F80u);
    const uint32_t b = nz16_pair(bad);
    *b01 = b;
    const uint32_t take_new = b * 0xFFFFu;              // 0xFFFF in the halves that escape
    return (n & take_new) | (d & ~take_new);
}
// the same for a vector of eight; esc8 bit e = element e escapes
__device__ __forceinline__ uint4 arith_vec(uint4 o, uint4 n, uint32_t *esc8) {
    uint32_t b0, b1, b2, b3;
    uint4 p;
    p.x = arith_pair(o.x, n.x, &b0);
    p.y = arith_pair(o.y, n.y, &b1);
    p.z = arith_pair(o.z, n.z, &b2);
    p.w = arith_pair(o.w, n.w, &b3);
    const uint32_t t = b0 | (b1 << 2) | (b2 << 4) | (b3 << 6);
    *esc8 = (t | (t >> 15)) & 0xFFu;
    return p;
}

// inclusive prefix sum over the 64 lanes of a wave with DPP moves (no LDS traffic): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then the row totals are broadcast into the following
// rows (lane 15 of a row into the next row, lane 31 into the upper half).  A lane without a
// source keeps the 0 passed as the old value.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return x;
}

// Cache policy of the encode kernel's streams (measured on the 7B workload: both hints together
// take 0.27 ms off 5.65 ms; either alone gains nothing): the two tensors are read once and the
// bucket entries are written once, so both are marked non-temporal.
#ifndef ROSE_NT_LOADS
#define ROSE_NT_LOADS 1
#endif
#ifndef ROSE_REFRESH_NT
#define ROSE_REFRESH_NT 1
#endif
#ifndef ROSE_REFRESH_WHOLE
#define ROSE_REFRESH_WHOLE 160         // entries per tile above which refresh rewrites the whole tile
                                       // (7B workload: 7.7 ms at 1 %, 8.0 ms at 5 %; 10.7 ms at 5 % without)
#endif
#ifndef ROSE_NT_STORES
#define ROSE_NT_STORES 1
#endif
// 128-bit load / store through the global address space (pointers fetched from a table would
// otherwise be treated as generic and use the slower flat instructions)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u32x4 global_u32x4;
__device__ __forceinline__ uint4 gload16(const void *p) {
    u32x4 v = *reinterpret_cast<const global_u32x4 *>(reinterpret_cast<uintptr_t>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
// the same for data that is read once: tells the caches not to keep it
__device__ __forceinline__ uint4 gload16_stream(const void *p) {
#if ROSE_NT_LOADS
    u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const global_u32x4 *>(reinterpret_cast<uintptr_t>(p)));
#else
    u32x4 v = *reinterpret_cast<const global_u32x4 *>(reinterpret_cast<uintptr_t>(p));
#endif
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void gstore16(void *p, uint4 v) {
    u32x4 w = {v.x, v.y, v.z, v.w};
    *reinterpret_cast<global_u32x4 *>(reinterpret_cast<uintptr_t>(p)) = w;
}

// Uniform (per-workgroup) table reads through the constant address space, so that they become
// scalar loads served by the scalar cache instead of vector loads.  Only used for tables that no
// kernel writes: the plan's piece / tile tables and the caller's pointer tables.
typedef __attribute__((address_space(4))) const uint32_t const_u32;
typedef __attribute__((address_space(4))) const uint64_t const_u64;
__device__ __forceinline__ uint32_t cload32(const void *p) {
    return *reinterpret_cast<const_u32 *>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ uint64_t cload64(const void *p) {
    return *reinterpret_cast<const_u64 *>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ Piece load_piece(const Piece *p) {
    static_assert(sizeof(Piece) == 7 * 8, "piece is read as seven 64-bit words");
    static_assert(kTile <= (1 << 13), "a ring entry keeps the offset inside a tile in 13 bits");
    uint64_t w[7];
#pragma unroll
    for (int i = 0; i < 7; ++i) w[i] = cload64(reinterpret_cast<const uint64_t *>(p) + i);
    Piece pc;
    __builtin_memcpy(&pc, w, sizeof pc);
    return pc;
}

// source element of piece-relative local index k
__device__ __forceinline__ int64_t src_index(const Piece &pc, uint32_t k, bool use_magic) {
    if (pc.flags & kPieceStrided) {
        uint32_t q = use_magic ? (__umulhi(k, pc.magic) >> pc.shift) : (k / (uint32_t)pc.run);
        return pc.src_off + (int64_t)q * pc.stride + (k - q * (uint32_t)pc.run);
    }
    return pc.src_off + k;
}

// shard-local index of element k of the piece
__device__ __forceinline__ uint32_t dst_index(const Piece &pc, uint32_t k, bool use_magic) {
    if (pc.flags & kPieceDstStrided) {
        uint32_t q = use_magic ? (__umulhi(k, pc.magic) >> pc.shift) : (k / (uint32_t)pc.run);
        return (uint32_t)pc.local_base + q * (uint32_t)pc.lstride + (k - q * (uint32_t)pc.run);
    }
    return (uint32_t)pc.local_base + k;
}

// Tile loaders.  A lane's vector j holds the eight 16-bit patterns at piece-relative local indices
// k .. k+7 with k = k_wave + (j * 64 + lane) * 8.
//
// load_raw / load_tile_fast (used by the dense copy): the whole tile lies inside the piece and
// every vector is 16-byte aligned, so all loads are 128-bit loads issued back to back.  Loading
// (raw registers) is split from conversion (fp32 -> bf16) so that a tile's loads can be issued long
// before its data is needed; the encode kernel has its own loader for that (load_raw_pair).
template <int SRC_F32> struct RawTile;
template <> struct RawTile<0> { uint4 v[kIters]; };
template <> struct RawTile<1> { uint4 lo[kIters], hi[kIters]; };

// `limit` is the piece length for a tile that reaches past the end of its piece (vectors that do
// not fit entirely read as zero) and 0xFFFFFFFF for a full tile.
__device__ __forceinline__ void load_raw(const void *base, const Piece &pc, uint32_t k_wave, int lane,
                                         uint32_t limit, RawTile<0> &r) {
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        const uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
        r.v[j] = make_uint4(0, 0, 0, 0);
        if (k + kVec <= limit) r.v[j] = gload16(static_cast<const uint16_t *>(base) + src_index(pc, k, true));
    }
}
__device__ __forceinline__ void load_raw(const void *base, const Piece &pc, uint32_t k_wave, int lane,
                                         uint32_t limit, RawTile<1> &r) {
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        const uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
        r.lo[j] = r.hi[j] = make_uint4(0, 0, 0, 0);
        if (k + kVec <= limit) {
            const uint32_t *p = static_cast<const uint32_t *>(base) + src_index(pc, k, true);
            r.lo[j] = gload16(p);
            r.hi[j] = gload16(p + 4);
        }
    }
}
__device__ __forceinline__ uint4 raw_to_bf16(const RawTile<0> &r, int j) { return r.v[j]; }
__device__ __forceinline__ uint4 raw_to_bf16(const RawTile<1> &r, int j) {
    return make_uint4(pack_rne(r.lo[j].x, r.lo[j].y), pack_rne(r.lo[j].z, r.lo[j].w),
                      pack_rne(r.hi[j].x, r.hi[j].y), pack_rne(r.hi[j].z, r.hi[j].w));
}

template <int SRC_F32>
__device__ __forceinline__ void load_tile_fast(const void *base, const Piece &pc, uint32_t k_wave, int lane,
                                               uint4 (&out)[kIters]) {
    RawTile<SRC_F32> r;
    load_raw(base, pc, k_wave, lane, 0xFFFFFFFFu, r);
#pragma unroll
    for (int j = 0; j < kIters; ++j) out[j] = raw_to_bf16(r, j);
}

// General path (ragged last tile of a piece, shapes or pointers that are not multiples of 16
// bytes): one vector, element by element; patterns past the end of the piece read as zero.
template <int SRC_F32>
__device__ __forceinline__ uint4 load_vec_general(const void *base, const Piece &pc, uint32_t k) {
    // deliberately one element at a time in a rolled loop: this path is rare and must stay small
    uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
#pragma unroll 1
    for (uint32_t i = 0; i < (uint32_t)kVec; ++i) {
        uint32_t v = 0;
        if (k + i < (uint32_t)pc.len) {
            int64_t s = src_index(pc, k + i, false);
            v = SRC_F32 ? rne_bf16(static_cast<const uint32_t *>(base)[s])
                        : (uint32_t) static_cast<const uint16_t *>(base)[s];
        }
        v <<= (i & 1u) * 16u;
        const uint32_t q = i >> 1;
        w0 |= (q == 0) ? v : 0u;
        w1 |= (q == 1) ? v : 0u;
        w2 |= (q == 2) ? v : 0u;
        w3 |= (q == 3) ? v : 0u;
    }
    return make_uint4(w0, w1, w2, w3);
}

__device__ __forceinline__ uint4 xor4(uint4 a, uint4 b) { return make_uint4(a.x ^ b.x, a.y ^ b.y, a.z ^ b.z, a.w ^ b.w); }

// ---------------------------------------------------------------------------------------------
// Prefix sums across workgroups.
//
// Every tile needs the number of entries that earlier tiles of its chain (= destination shard)
// produce.  Tiles are grouped in blocks of kBlock consecutive tiles of a chain.  A worker publishes
// each tile's count ("aggregate") in the tile's descriptor word and moves on.  A few workgroups of
// the grid do not walk tiles: each of their waves SERVES blocks (block s, s + n_servers, ...): it
// reads the block's 64 aggregates with one load per poll, scans them, publishes the block total,
// looks back over earlier BLOCK words (64 blocks = 4096 tiles per load) for the block's offset and
// writes every tile of the block its exclusive prefix into the tile's word.  Workers read only
// their own tiles' words, so no worker ever walks a chain or waits for a slower worker's tile
// other than through the answer it needs.
//
// A descriptor is one 64-bit word, status in the top two bits, value below, written and read with
// relaxed device-scope atomics: the word carries all a reader needs, nothing else is ordered by it.
//
// Progress: the whole grid (workers and servers) is resident at once: the launcher sizes it from
// the occupancy query.  A worker publishes a tile's count before it ever waits for that tile's
// prefix, and the rules at struct Walk keep it from waiting for a block that still needs a count
// from the waiter itself; a server waits for counts of its current block and for earlier blocks.
// So every wait is for something a running wave produces without waiting on the waiter.  Waits
// are bounded anyway:
// after ROSE_SPIN_LIMIT failed polls, or once the abort flag is set, a wave stops waiting, sets
// the flag, and the launch is reported as failed; every wave always reaches the end of the kernel.
// ---------------------------------------------------------------------------------------------
constexpr u64 kStatusShift = 62;
constexpr u64 kStatusAggregate = 1;   // tile word: the tile's count;  block word: the block's count
constexpr u64 kStatusPrefix = 2;      // tile word: the tile's exclusive prefix;  block word: count of
                                      // this block and all earlier blocks of the chain
constexpr u64 kValueMask = (1ull << kStatusShift) - 1;

#ifndef ROSE_DIAG
#define ROSE_DIAG 0           // timing experiments only: 1 no waiting for prefixes, 2 no bucket writes,
                              // 4 no publishing, 8 no parking in LDS
#endif
#ifndef ROSE_WRITE_PERIOD_LOG2
#define ROSE_WRITE_PERIOD_LOG2 12     // ticks of the 100 MHz clock between windows (2^12: 41 us)
#endif
#ifndef ROSE_WRITE_RING_NUM
#define ROSE_WRITE_RING_NUM 6        // eighths of the ring that may fill up between windows
#endif
#ifndef ROSE_WRITE_OPEN_LOG2
#define ROSE_WRITE_OPEN_LOG2 10       // ticks a window is open (2^10: 10 us)
#endif
#ifndef ROSE_COUNT_AHEAD
#define ROSE_COUNT_AHEAD 1    // count the rest of a ticket's tiles before waiting for room (dense inputs)
#endif
#ifndef ROSE_SPIN_LIMIT
#define ROSE_SPIN_LIMIT (1u << 22)   // failed polls after which a wave gives up and flags the launch
#endif

__device__ __forceinline__ void desc_store(u64 *p, u64 v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 desc_load(u64 *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The workspace is one array of 64-bit words: header (abort flag, ticket counters), tile words,
// block words.  All of it starts at zero.
__global__ void reset_kernel(u64 *workspace, int64_t n_words) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i < n_words; i += (int64_t)gridDim.x * blockDim.x) workspace[i] = 0;
}

// After encode: if any wave gave up waiting, mark every bucket as invalid (total = -1) so that
// rose_bucket_check reports it and apply does nothing.
__global__ void finalize_kernel(EncodeArgs a) {
    if (threadIdx.x < (unsigned)a.tp && *a.abort_flag) a.bucket[threadIdx.x].seg_off[a.n_tensors] = -1;
}

// Asking for a ticket without waiting for it.  The counter's answer is in flight from one
// iteration of the worker loop to the next; a value in flight must not live in a register the
// compiler knows about (it may copy such a register at any time, before the answer has arrived).
// So each encode kernel keeps one VGPR out of the compiler's hands (amdgpu_num_vgpr stops the
// allocator below it) and the two routines here name it directly.
//   ticket_request: lane 0 of the calling wave adds 1 to *counter; the old value will arrive in
//                   lane 0 of the reserved register.  Nothing waits.
//   ticket_take:    waits for every outstanding vector memory operation of the wave, then reads
//                   the reserved register.
// A kernel with 4 waves per SIMD has 128 registers per lane (CLASS = 0), one with 3 has 168 (1),
// one with 2 has 256 (2).
#define ROSE_TICKET_VGPR_0 "v127"
#define ROSE_TICKET_VGPR_1 "v167"
#define ROSE_TICKET_VGPR_2 "v255"
constexpr int kNumVgpr0 = 126, kNumVgpr1 = 166, kNumVgpr2 = 254;     // what the compiler may use
#define ROSE_TICKET_REQUEST(REG)                                                                              \
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 1\n\tglobal_atomic_add " REG                         \
                 ", %1, %2, %3 sc0\n\ts_mov_b64 exec, %0"                                                     \
                 : "=&s"(saved) : "v"(zero), "v"(one), "s"(counter) : "memory", REG)
#define ROSE_TICKET_TAKE(REG) asm volatile("s_waitcnt vmcnt(0)\n\tv_mov_b32 %0, " REG : "=v"(t) : : "memory")
template <int CLASS>
__device__ __forceinline__ void ticket_request(unsigned int *counter) {
    unsigned long long saved;
    const unsigned int zero = 0, one = 1;
    if constexpr (CLASS == 2) ROSE_TICKET_REQUEST(ROSE_TICKET_VGPR_2);
    else if constexpr (CLASS == 1) ROSE_TICKET_REQUEST(ROSE_TICKET_VGPR_1);
    else ROSE_TICKET_REQUEST(ROSE_TICKET_VGPR_0);
}
template <int CLASS>
__device__ __forceinline__ unsigned int ticket_take() {
    unsigned int t;
    if constexpr (CLASS == 2) ROSE_TICKET_TAKE(ROSE_TICKET_VGPR_2);
    else if constexpr (CLASS == 1) ROSE_TICKET_TAKE(ROSE_TICKET_VGPR_1);
    else ROSE_TICKET_TAKE(ROSE_TICKET_VGPR_0);
    return t;
}
#undef ROSE_TICKET_REQUEST
#undef ROSE_TICKET_TAKE

__device__ __forceinline__ bool has_prefix(u64 word) { return (word >> kStatusShift) == kStatusPrefix; }

// bounded wait bookkeeping; returns false when the wave must stop waiting
__device__ __forceinline__ bool keep_waiting(unsigned int *abort_flag, unsigned int &spins, int lane) {
    if (++spins > ROSE_SPIN_LIMIT ||
        ((spins & 63u) == 0 && __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
        if (lane == 0) __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
    __builtin_amdgcn_s_sleep(2);
    return true;
}

// sum of a 64-bit value over the wave
__device__ __forceinline__ u64 wave_sum64(u64 v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
    return v;
}

// Offset of block `blk` (index into block_desc) inside its chain whose first block is
// `blk_first`: the published total of all earlier blocks.  One wave; each step reads 64 earlier
// block words (nearest first), needs every word nearer than the first prefix to hold at least an
// aggregate, and sums them.
__device__ __forceinline__ bool block_look_back(u64 *block_desc, unsigned int *abort_flag, int32_t blk,
                                                int32_t blk_first, int lane, u64 *out) {
    u64 excl = 0;
    int32_t look = blk - 1;
    unsigned int spins = 0;
    for (;;) {
        int32_t at = look - lane;
        u64 v = (at >= blk_first) ? desc_load(block_desc + at) : (kStatusPrefix << kStatusShift);
        u64 st = v >> kStatusShift;
        u64 pref = __ballot(st == kStatusPrefix);
        u64 empty = __ballot(st == 0);
        int first_pref = pref ? __ffsll((long long)pref) - 1 : 64;
        u64 need = (first_pref >= 63) ? ~0ull : ((1ull << (first_pref + 1)) - 1);
        if (empty & need) {
            if (!keep_waiting(abort_flag, spins, lane)) return false;
            continue;
        }
        excl += wave_sum64((lane <= first_pref) ? (v & kValueMask) : 0);
        if (pref) break;
        look -= 64;
    }
    *out = excl;
    return true;
}

// A serving wave: blocks server, server + n_servers, ... in increasing order.
__device__ __forceinline__ void serve_blocks(const EncodeArgs &a, int32_t server, int lane) {
    int32_t shard = 0;
    for (int32_t blk = server; blk < a.n_blocks; blk += a.n_servers) {
        while (blk >= a.block_first[shard + 1]) ++shard;          // blocks are numbered chain by chain
        const int32_t blk_first = a.block_first[shard];
        const int32_t first_tile = a.chain_first[shard] + (blk - blk_first) * kBlock;
        const int32_t n = min(kBlock, a.chain_first[shard + 1] - first_tile);   // tiles in this block
        unsigned int spins = 0;
        bool ok = true;
        u64 agg = 0;
        for (;;) {   // lane i takes the count of the block's tile i
            u64 v = (lane < n) ? desc_load(a.tile_desc + first_tile + lane) : (kStatusAggregate << kStatusShift);
            if (__ballot((v >> kStatusShift) == 0) == 0) {
                agg = v & kValueMask;
                break;
            }
            if (!keep_waiting(a.abort_flag, spins, lane)) {
                ok = false;
                break;
            }
        }
        const uint32_t incl = wave_incl_scan((uint32_t)agg);    // <= 64 tiles * kTile entries
        const uint32_t block_total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        u64 block_excl = 0;
        if (ok && blk > blk_first) {
            if (lane == 0) desc_store(a.block_desc + blk, (kStatusAggregate << kStatusShift) | block_total);
            ok = block_look_back(a.block_desc, a.abort_flag, blk, blk_first, lane, &block_excl);
        }
        // published even after giving up, so that nobody keeps waiting on this block
        if (lane == 0) desc_store(a.block_desc + blk, (kStatusPrefix << kStatusShift) | (block_excl + block_total));
        if (lane < n)
            desc_store(a.tile_desc + first_tile + lane,
                       (kStatusPrefix << kStatusShift) | (block_excl + (incl - (uint32_t)agg)));
    }
}

// ---------------------------------------------------------------------------------------------
// encode: persistent workgroups.  The first n_server_wgs workgroups serve prefixes (above), the
// others are workers that walk the tiles their tickets name (see ticket_tile and struct Walk).
//
// Worker, per tile: (1) the tile's 128-bit loads were issued one tile earlier; XOR old and new
// into an 8-bit change mask per vector, (2) copy out parked tiles whose prefixes have arrived,
// poll for the others, ask for a ticket, (3) issue the NEXT tile's loads, (4) wave prefix sums of
// the popcounts, wave totals through LDS, (5) publish the tile's count, (6) park the tile's
// entries, compacted, in an LDS ring and go on (the order of the memory operations matters: see
// the comment in encode_body).  The wait for a tile's prefix is deferred: parked tiles are polled
// one lane per tile, every iteration, without waiting; only when the ring (kRing entries) or the
// queue of parked tiles (kQueue) is full, and at the end, does a workgroup wait.  This keeps
// loads in flight while counts travel between workgroups.  A tile with more than kRing entries
// (only possible if the ring is configured smaller than a tile) is written straight from
// registers after a drain.
// Inside a tile wave w covers a contiguous part and walks it in kIters steps of 512 elements,
// so the order (wave, step, lane, element) is ascending local index.
// ---------------------------------------------------------------------------------------------
#ifndef ROSE_RING
#define ROSE_RING 8192
#endif
#ifndef ROSE_QUEUE
#define ROSE_QUEUE 64         // (16 to 64 measure the same in the spread order; the timed order holds tiles back for a
                              // whole period between windows)
#endif
constexpr int kRing = ROSE_RING;        // entries parked per workgroup (power of two)
constexpr int kQueue = ROSE_QUEUE;      // tiles parked per workgroup (<= 64)
static_assert((kRing & (kRing - 1)) == 0 && (kQueue & (kQueue - 1)) == 0 && kQueue <= 64,
              "ring and queue sizes must be powers of two, the queue at most a wave");

enum : int { kLoadVec = 0, kLoadGeneral = 1 };
enum : int { kDrainOldest = 0, kDrainAll = 1, kDrainReady = 2 };
#ifndef ROSE_ALIGN_STORES
#define ROSE_ALIGN_STORES 1
#endif


struct TileCtx {
    Piece pc;
    const uint16_t *old_base;
    const void *new_base;
    uint32_t k_tile;
    uint32_t limit;     // see load_raw
    uint32_t vec;       // 128-bit loads are legal for this tile
    int32_t piece;      // index of pc in the piece table
};

__device__ __forceinline__ TileCtx tile_ctx(const EncodeArgs &a, int32_t tile) {
    TileCtx c;
    c.piece = cload32(a.tile_piece + tile);
    c.pc = load_piece(a.pieces + c.piece);
    c.old_base = reinterpret_cast<const uint16_t *>(cload64(a.old_ptrs + c.pc.tensor));
    c.new_base = reinterpret_cast<const void *>(cload64(a.new_ptrs + c.pc.tensor));
    c.k_tile = (uint32_t)(tile - c.pc.first_tile) * (uint32_t)kTile;
    c.limit = (c.k_tile + (uint32_t)kTile <= (uint32_t)c.pc.len) ? 0xFFFFFFFFu : (uint32_t)c.pc.len;
    // uniform choice: aligned piece and aligned tensors -> 128-bit loads
    c.vec = ((c.pc.flags & kPieceVec) && ((((uintptr_t)c.old_base) | ((uintptr_t)c.new_base)) & 15u) == 0 &&
             c.k_tile + (uint32_t)kVec <= (uint32_t)c.pc.len) ? 1u : 0u;
    return c;
}

// What a worker keeps of a tile while it handles it (uniform, a few scalars: the full context is
// only needed to issue the loads and in rare paths, which build it again).
struct TileMeta {
    uint32_t out_base;  // local index of the tile's first element (piece with contiguous local indices),
                        // else the tile's first element number k inside its piece
    int32_t piece;      // -1, or the piece whose table entry maps element numbers to local indices
    int32_t shard;
    int32_t seg;        // tensor whose segment starts with this tile, else -1
    uint32_t limit;     // see load_raw
    uint32_t vec;       // bit 0: 128-bit loads are legal; bit 1: piece of a replicated tensor
    uint32_t k_tile;
};
__device__ __forceinline__ TileMeta tile_meta(const TileCtx &c, int32_t tile) {
    TileMeta m;
    const bool dst_strided = (c.pc.flags & kPieceDstStrided) != 0;
    m.out_base = dst_strided ? c.k_tile : (uint32_t)c.pc.local_base + c.k_tile;
    m.piece = dst_strided ? c.piece : -1;
    m.shard = c.pc.shard;
    m.seg = ((c.pc.flags & kPieceFirst) && tile == c.pc.first_tile) ? c.pc.tensor : -1;
    m.limit = c.limit;
    m.vec = c.vec | ((c.pc.flags & kPieceReplicated) ? 2u : 0u);
    m.k_tile = c.k_tile;
    return m;
}

// Issue a tile's 128-bit loads of the old and the new tensor: both use the same element offsets,
// which are worked out once.  t_off = wave * kWaveSpan + lane * kVec.
template <int NEW_F32>
__device__ __forceinline__ void raw_zero(int j, RawTile<0> &ro, RawTile<NEW_F32> &rn) {
    ro.v[j] = make_uint4(0, 0, 0, 0);
    if constexpr (NEW_F32) rn.lo[j] = rn.hi[j] = make_uint4(0, 0, 0, 0);
    else rn.v[j] = make_uint4(0, 0, 0, 0);
}
// one vector of the old and of the new tensor at element `off` from uniform bases
template <int NEW_F32, typename OFF>
__device__ __forceinline__ void load_raw_at(const uint16_t *o, const void *n, OFF off, int j, RawTile<0> &ro,
                                            RawTile<NEW_F32> &rn) {
    ro.v[j] = gload16_stream(o + off);
    if constexpr (NEW_F32) {
        rn.lo[j] = gload16_stream(static_cast<const uint32_t *>(n) + off);
        rn.hi[j] = gload16_stream(static_cast<const uint32_t *>(n) + off + 4);
    } else {
        rn.v[j] = gload16_stream(static_cast<const uint16_t *>(n) + off);
    }
}
// All of a tile's loads are issued unconditionally (no zeroing, no predication: nothing but the
// loads themselves ever writes the load registers).  A vector that does not fit entirely inside
// the piece is loaded from the tile's first vector instead, which tile_ctx guarantees to exist
// for a tile with vec set; the caller discards such vectors.
template <int NEW_F32>
__device__ __forceinline__ void load_raw_pair(const TileCtx &c, uint32_t t_off, RawTile<0> &ro, RawTile<NEW_F32> &rn) {
    const bool full = c.limit == 0xFFFFFFFFu;
    // One instruction sequence for both kinds of piece: a contiguous piece is walked as a strided
    // one whose row number is always 0 (magic 0).
    const bool strided = (c.pc.flags & kPieceStrided) != 0;
    const uint32_t magic = strided ? c.pc.magic : 0u, shift = strided ? c.pc.shift : 0u;
    const uint32_t run = strided ? (uint32_t)c.pc.run : 0u;
    const int64_t stride = strided ? c.pc.stride : 0;
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        uint32_t k = c.k_tile + t_off + (uint32_t)j * 64 * kVec;
        if (!full && k + kVec > c.limit) k = c.k_tile;
        const uint32_t q = __umulhi(k, magic) >> shift;
        const int64_t e = c.pc.src_off + (int64_t)q * stride + (k - q * run);
        load_raw_at<NEW_F32>(c.old_base, c.new_base, e, j, ro, rn);
    }
}

// The j-th tile of a ticket, or -1 if there is none.  A ticket stands for a.batch tiles (kBatch below; the
// launcher picks it).  A group of kBatch consecutive blocks has
// kBatch * kBlock tile positions ("slots", block after block) and kBlock tickets.  Two orders:
// spread (a.adjacent = 0): ticket n of the group stands for position n of each of the group's blocks, so
// that a block's 64 tiles are walked by 64 workers at once and its prefixes are ready one tile-time
// later; neighbours (a.adjacent = 1): ticket n stands for the kBatch NEIGHBOURING slots
// n * kBatch .. n * kBatch + kBatch - 1.  Neighbouring slots are
// neighbouring tiles of one chain (except where a chain ends inside the group: a chain's short last
// block has no tile for its last positions), so the entries of a ticket's tiles follow each other in
// the bucket and are written as one run: only the two ends of a ticket's run share 64-byte lines of
// the bucket with another workgroup's.  (Measured on the 7B-style workload with every run padded to
// whole lines, which is what no shared lines at all would give: 3 % faster at 1 - 5 %, 7 % at 10 %.)
// The price: a block's prefixes are ready kBatch tile-times later, so more entries wait in the ring,
// which pays while the ring holds them (see launch_encode for who picks the order).  Uniform.
__device__ __forceinline__ int32_t ticket_tile(const EncodeArgs &a, int32_t ticket, int32_t j) {
    ticket = __builtin_amdgcn_readfirstlane(ticket);    // uniform anyway: keeps the table look-ups scalar
    j = __builtin_amdgcn_readfirstlane(j);
    int32_t blk = (ticket / kBlock) * a.batch + j, pos = ticket & (kBlock - 1);
    if (a.adjacent) {
        const int32_t slot = (ticket & (kBlock - 1)) * a.batch + j;
        blk = (ticket / kBlock) * a.batch + slot / kBlock;
        pos = slot & (kBlock - 1);
    }
    if (blk >= a.n_blocks) return -1;
    int32_t shard = 0;
    while (blk >= a.block_first[shard + 1]) ++shard;
    const int32_t t = a.chain_first[shard] + (blk - a.block_first[shard]) * kBlock + pos;
    return t < a.chain_first[shard + 1] ? t : -1;
}

// A worker's position in the tile order it is given by its tickets (uniform state).
//
// Waiting and tickets.  A worker may wait for the prefix of a parked tile X only while every tile
// it holds a ticket for and has not published lies in a later block than X: then the earliest
// block that is not fully published never depends on a waiting worker, and all waits end.  Tickets
// are taken in order, so the tiles of a worker's tickets lie in later and later groups, except
// when two tickets in a row fall into the SAME group (few workers are taking tickets, e.g. while
// most of them wait).  Such a pair is handled with care: from the moment the second ticket is
// accepted nothing waits until the counts of all tiles of both tickets are published by a
// count-only pass; then those tiles are walked again ("redo", without publishing) in the normal
// way.  While redoing, no further ticket is asked for.
// The same machinery serves tiles so dense that the ring does not hold a ticket's worth of them: a
// worker that would have to wait for room with fewer tiles parked than a ticket has, and with tiles
// of the current ticket still uncounted, counts those first and walks the ticket again from the
// current tile on.  (Waiting there is allowed by the rule above, but every later group of workers
// would wait for those counts in turn, and the groups would run one after the other.)
struct Walk {
    int32_t ticket, j;          // ticket in use (-1: none yet) and its batch slot
    int32_t next_ticket;        // ticket fetched ahead of time
    int32_t redo_through;       // last ticket of a redo
    bool have_next;
    bool exhausted;             // the counter has run out
    bool careful;               // a same-group ticket was accepted; its counts are not published yet
    bool redo;                  // tiles up to the end of ticket redo_through are published already
};
enum : int { kWalkTile = 0, kWalkNeedTicket = 1, kWalkDone = 2 };

// take in the counter's answer n
__device__ __forceinline__ void walk_accept(const EncodeArgs &a, Walk &w, uint32_t n) {
    if (n >= (uint32_t)a.n_tickets) {
        w.exhausted = true;
    } else if ((int32_t)n <= w.ticket) {
        // One counter hands the tickets out in order, so a worker's tickets increase.  A value that
        // does not is not a ticket (the register it arrives in is only reserved by asking the
        // compiler, see ticket_request): walk no further and mark the launch as failed.
        __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        w.exhausted = true;
    } else {
        w.next_ticket = (int32_t)n;
        w.have_next = true;
        if (w.ticket >= 0 && (int32_t)n / kBlock == w.ticket / kBlock) w.careful = true;
    }
}

// Advance to the next tile.  kWalkNeedTicket: the current ticket is used up and no further one
// is at hand (ask the counter, then call again); kWalkDone: no tiles are left.
__device__ __forceinline__ int walk_step(const EncodeArgs &a, Walk &w, int32_t *tile) {
    for (;;) {
        while (w.j + 1 < a.batch) {
            ++w.j;
            const int32_t t = ticket_tile(a, w.ticket, w.j);
            if (t >= 0) {
                *tile = t;
                return kWalkTile;
            }
        }
        w.j = a.batch;
        if (w.redo && w.ticket == w.redo_through) w.redo = false;
        if (!w.have_next) return w.exhausted ? kWalkDone : kWalkNeedTicket;
        w.ticket = w.next_ticket;
        w.have_next = false;
        w.j = -1;
    }
}

template <int NEW_F32, int REFRESH, int ARITH>
__device__ __forceinline__ void encode_body(const EncodeArgs &a) {
    // register class, see ticket_request
    constexpr int WIDE = (NEW_F32 && REFRESH && ARITH) ? 2 : (NEW_F32 || (REFRESH && ARITH)) ? 1 : 0;
    __shared__ uint32_t s_ring[kRing];      // an entry: offset inside its tile (13 bits) << 16 | value;
                                            // bit 31: the entry escapes (arithmetic payload only)
    __shared__ uint32_t s_wave_total[2][kWaves];
    __shared__ u64 s_excl[2][kQueue];       // prefixes of the tiles an iteration copies out, oldest first
    __shared__ u64 s_excl_sync[kQueue];     // the same for a blocking drain
    __shared__ int32_t s_nready[2];
    __shared__ uint32_t s_q_count[kQueue];
    __shared__ uint32_t s_q_off[kQueue];
    __shared__ uint32_t s_q_base[kQueue];   // see TileMeta::out_base
    __shared__ int32_t s_q_piece[kQueue];   // see TileMeta::piece
    __shared__ int32_t s_q_shard[kQueue];
    __shared__ int32_t s_q_seg[kQueue];     // tensor whose segment starts with this tile, else -1
    __shared__ int32_t s_q_last[kQueue];    // 1 if the tile is the last of its chain
    __shared__ int32_t s_ok, s_ready;
    __shared__ int32_t s_ticket[2], s_ticket_sync;
    __shared__ uint32_t s_count_only[kWaves];
    __shared__ u64 s_direct_excl;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int32_t)blockIdx.x < a.n_server_wgs) {
        serve_blocks(a, (int32_t)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(wave), lane);
        return;
    }

    // Uniform bookkeeping, kept identical in every thread.  The queue is a circular FIFO whose i-th
    // oldest tile sits in slot (q_head + i) mod kQueue; the ring holds their entries in that order.
    //
    // Order of the memory operations of one iteration.  The hardware counts outstanding vector
    // memory operations in issue order, and the compiler can only wait for "all but the newest
    // n" with an n it can count at compile time; behind loops and branches it has to wait for
    // everything.  So results are taken in only at the top of an iteration, where everything in
    // flight is wanted anyway, and the long-latency loads of the next tile are issued after the
    // iteration's other memory operations (bucket stores, the poll, the ticket request):
    //   top   the tile's data has landed; so have last iteration's poll answers and ticket
    //   (a)   change masks of this tile (frees the load registers)
    //   (b)   copy out the parked tiles announced at the last barrier; wave 0 takes in the poll
    //         answers and announces (through LDS, valid after this iteration's barrier) which
    //         parked tiles can be copied out next time
    //   (c)   wave 0 polls the parked tiles without a prefix; thread 0 asks for a ticket
    //   (d)   the NEXT tile's loads are issued
    //   (e)   scan, barrier, publish this tile's count, park its entries (LDS only)
    int q_head = 0, q_len = 0;
    uint32_t ring_used = 0, ring_head = 0;
    int parity = 0;
    int n_announced = 0;        // oldest parked tiles whose prefixes lie in s_excl[parity ^ 1]
    // wave 0 only: lane i tracks the i-th oldest parked tile
    int32_t wq_tile = 0;
    u64 wq_w = 0;               // the newest copy of its descriptor word: the prefix once the status says so
    u64 polled = 0;             // written only by the poll's load (in flight across the iteration boundary)
    int n_polled = 0;           // lanes of wave 0 whose tiles the poll in flight covers
    bool ticket_out = false;    // a ticket has been asked for and not yet taken in

    // copy the n oldest parked tiles to the buckets (prefixes in excl[0..n)); returns ring entries freed.
    // Tiles that follow each other in the bucket (up to four: same shard, each starting where the one
    // before ends; their entries follow each other in the ring as well) are written as one run.
    auto copy_out = [&](int n, const u64 *excl_by_age, bool ok) -> uint32_t {
        uint32_t freed = 0;
        for (int i = 0; i < n;) {
            const int slot = (q_head + i) & (kQueue - 1);
            // everything about the tiles is uniform: kept in scalar registers, the bucket's
            // pointers come through scalar loads
            const uint32_t cnt0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_q_count[slot]);
            if (!ok || (ROSE_DIAG & 2)) {
                freed += cnt0;
                ++i;
                continue;
            }
            const u64 excl = ((u64)(uint32_t)__builtin_amdgcn_readfirstlane((int)(excl_by_age[i] >> 32)) << 32) |
                             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)excl_by_age[i]);
            const uint32_t off = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_q_off[slot]);
            const int32_t shard = __builtin_amdgcn_readfirstlane(s_q_shard[slot]);
            const BucketDev b = a.bucket[shard];
            const int32_t piece = __builtin_amdgcn_readfirstlane(s_q_piece[slot]);
            // the run: this tile and the parked tiles behind it that continue it (c1..c3: where the
            // second to fourth tile's entries start inside the run; b0..b3: see TileMeta::out_base)
            uint32_t cnt = cnt0, c1 = 0xFFFFFFFFu, c2 = 0xFFFFFFFFu, c3 = 0xFFFFFFFFu;
            const uint32_t b0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_q_base[slot]);
            uint32_t b1 = 0, b2 = 0, b3 = 0;
            int g = 1;
            if (threadIdx.x == 0) {
                const int32_t seg = s_q_seg[slot];
                if (seg >= 0) b.seg_off[seg] = (int64_t)excl;
                if (s_q_last[slot]) b.seg_off[a.n_tensors] = (int64_t)(excl + cnt0);
            }
            while (piece < 0 && g < 4 && i + g < n) {
                const int s2 = (q_head + i + g) & (kQueue - 1);
                const u64 e2 = ((u64)(uint32_t)__builtin_amdgcn_readfirstlane((int)(excl_by_age[i + g] >> 32)) << 32) |
                               (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)excl_by_age[i + g]);
                if (__builtin_amdgcn_readfirstlane(s_q_shard[s2]) != shard || e2 != excl + cnt ||
                    __builtin_amdgcn_readfirstlane(s_q_piece[s2]) >= 0)
                    break;
                const uint32_t cg = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_q_count[s2]);
                const uint32_t bg = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_q_base[s2]);
                if (threadIdx.x == 0) {
                    const int32_t seg = s_q_seg[s2];
                    if (seg >= 0) b.seg_off[seg] = (int64_t)e2;
                    if (s_q_last[s2]) b.seg_off[a.n_tensors] = (int64_t)(e2 + cg);
                }
                if (g == 1) { c1 = cnt; b1 = bg; }
                else if (g == 2) { c2 = cnt; b2 = bg; }
                else { c3 = cnt; b3 = bg; }
                cnt += cg;
                ++g;
            }
            freed += cnt;
            // local index of the element at offset o of the tile
            uint32_t l_base = b0, l_run = 0, l_magic = 0, l_shift = 0, l_stride = 0;
            if (piece >= 0) {                          // the piece's local indices come in strided runs
                const Piece pc = load_piece(a.pieces + piece);
                l_base = (uint32_t)pc.local_base;
                l_run = (uint32_t)pc.run;
                l_magic = pc.magic;
                l_shift = pc.shift;
                l_stride = (uint32_t)pc.lstride;
            }
            // A wave's store covers 64 entries = 256 bytes of indices, 128 of values.  The run starts at an
            // arbitrary entry of the bucket, so the threads are lined up with the BUCKET, not with the run:
            // thread t of a round handles the entry whose position is t more than a multiple of 32
            // entries.  Every store but the first and last of a run then fills whole 64-byte lines
            // (otherwise each wave's store starts and ends inside a line and the line's 32-byte halves
            // are written twice: 1.20 x the bytes at the memory).
            const uint32_t phase = ROSE_ALIGN_STORES ? (uint32_t)excl & 31u : 0u;
            for (uint32_t kk = threadIdx.x; kk < cnt + phase; kk += kThreads) {
                const uint32_t k = kk - phase;         // (wraps below phase: caught by the first test)
                const u64 pos = excl + k;
                if (kk >= phase && pos < (u64)b.capacity) {
                    const uint32_t entry = s_ring[(off + k) & (kRing - 1)];
                    const uint32_t base = k < c1 ? b0 : k < c2 ? b1 : k < c3 ? b2 : b3;
                    uint32_t local = base + (ARITH ? (entry >> 16) & (uint32_t)(kTile - 1) : entry >> 16);
                    if (piece >= 0) {                  // base is the tile's first element number here
                        // (runs of one element have no magic divisor: the quotient is the number itself)
                        const uint32_t q = l_run == 1u ? local : (__umulhi(local, l_magic) >> l_shift);
                        local = l_base + q * l_stride + (local - q * l_run);
                    }
                    if constexpr (ARITH) local |= entry & 0x80000000u;
#if ROSE_NT_STORES
                    __builtin_nontemporal_store((int32_t)local, b.idx + pos);
                    __builtin_nontemporal_store((uint16_t)entry, b.val + pos);
#else
                    b.idx[pos] = (int32_t)local;
                    b.val[pos] = (uint16_t)entry;
#endif
                }
            }
            i += g;
        }
        return freed;
    };
    auto pop = [&](int n) {      // forget the n oldest tiles (wave 0 shifts its lanes down)
        q_head = (q_head + n) & (kQueue - 1);
        q_len -= n;
        if (wave == 0) {
            wq_tile = __shfl(wq_tile, lane + n, 64);
            wq_w = __shfl(wq_w, lane + n, 64);
        }
    };

    // Blocking drain, for when there is no room to park (or at the end): waits until the oldest
    // parked tile (all = false) or every parked tile (all = true) has its prefix, and copies out
    // every leading tile whose prefix is known; these include the announced ones.
    // mode kDrainOldest / kDrainAll as described; kDrainReady waits for nothing: it looks once and
    // copies out what has its prefix by now.
    auto drain = [&](int mode) {
        const bool all = mode == kDrainAll;
        __syncthreads();                               // parked entries visible; earlier copies done
        if (wave == 0) {
            bool ok = true;
            int n_ready = q_len;
#if !(ROSE_DIAG & 1)
            unsigned int spins = 0;
            for (;;) {
                if (lane < q_len && !has_prefix(wq_w)) wq_w = desc_load(a.tile_desc + wq_tile);
                const u64 unknown = __ballot(lane < q_len && !has_prefix(wq_w));
                n_ready = unknown ? __ffsll((long long)unknown) - 1 : q_len;
                if (mode == kDrainReady || (all ? (n_ready == q_len) : (n_ready >= 1 || q_len == 0))) break;
                if (!keep_waiting(a.abort_flag, spins, lane)) {
                    ok = false;         // give up: drop everything that is parked
                    n_ready = q_len;
                    break;
                }
            }
#else
            wq_w = kStatusPrefix << kStatusShift;
#endif
            if (lane < n_ready) s_excl_sync[lane] = wq_w & kValueMask;
            if (lane == 0) {
                s_ok = ok ? 1 : 0;
                s_ready = n_ready;
            }
        }
        __syncthreads();
        const int n_ready = __builtin_amdgcn_readfirstlane(s_ready);
        const uint32_t freed = copy_out(n_ready, s_excl_sync, s_ok != 0);
        __syncthreads();                               // ring and queue slots may be reused
        pop(n_ready);
        ring_used -= freed;
        n_announced = 0;
        n_polled = 0;                                  // the lanes of wave 0 have moved
    };

    // Tiles come from tickets (dynamic, so that faster workgroups take more): thread 0 asks for a
    // ticket well before it is needed; the answer is handed to the others through LDS at the
    // barrier of the following iteration.
    Walk walk;
    walk.ticket = -1;
    walk.j = a.batch;
    walk.next_ticket = 0;
    walk.redo_through = 0;
    walk.have_next = false;
    walk.exhausted = false;
    walk.careful = false;
    walk.redo = false;
    // all threads; two barriers; no waiting for other workgroups.  Takes in the ticket that is on
    // its way, if any, else asks for one.
    auto settle_ticket = [&]() {
        if (threadIdx.x == 0) {
            if (!ticket_out) ticket_request<WIDE>(a.ticket);
            s_ticket_sync = (int32_t)ticket_take<WIDE>();
        }
        ticket_out = false;
        __syncthreads();
        walk_accept(a, walk, (uint32_t)__builtin_amdgcn_readfirstlane(s_ticket_sync));
        __syncthreads();
    };
    // Count-only pass over one tile (all threads, rolled loads: this is rare): publishes its count.
    auto publish_count = [&](int32_t t) {
        const TileCtx c = tile_ctx(a, __builtin_amdgcn_readfirstlane(t));
        uint32_t cnt = 0;
        if ((c.vec & 1u) && c.limit == 0xFFFFFFFFu) {
            // a whole tile with 128-bit loads (cached: the tile is read again soon); kept rolled, one
            // pair of vectors at a time, because the next tile's loads occupy the load registers
#pragma unroll 1
            for (int j = 0; j < kIters; ++j) {
                const uint32_t k = c.k_tile + (uint32_t)wave * kWaveSpan + (uint32_t)(j * 64 + lane) * kVec;
                const int64_t e = src_index(c.pc, k, true);
                const uint4 o = gload16(c.old_base + e);
                uint4 n;
                if constexpr (NEW_F32) {
                    const uint32_t *p32 = static_cast<const uint32_t *>(c.new_base) + e;
                    const uint4 lo = gload16(p32), hi = gload16(p32 + 4);
                    n = make_uint4(pack_rne(lo.x, lo.y), pack_rne(lo.z, lo.w), pack_rne(hi.x, hi.y), pack_rne(hi.z, hi.w));
                } else {
                    n = gload16(static_cast<const uint16_t *>(c.new_base) + e);
                }
                cnt += __popc(nz16_mask(xor4(o, n)));
            }
        } else {
#pragma unroll 1
            for (int j = 0; j < kIters; ++j) {
                const uint32_t k = c.k_tile + (uint32_t)wave * kWaveSpan + (uint32_t)(j * 64 + lane) * kVec;
                const uint4 o = load_vec_general<0>(c.old_base, c.pc, k);
                const uint4 n = load_vec_general<NEW_F32>(c.new_base, c.pc, k);
                cnt += __popc(nz16_mask(xor4(o, n)));
            }
        }
        const uint32_t wave_cnt = (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(cnt), 63);
        __syncthreads();                               // earlier readers of s_count_only are done
        if (lane == 0) s_count_only[wave] = wave_cnt;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t total = 0;
            for (int w = 0; w < kWaves; ++w) total += s_count_only[w];
            if (!(ROSE_DIAG & 4)) desc_store(a.tile_desc + t, (kStatusAggregate << kStatusShift) | total);
        }
    };
    int32_t tile = -1;
    for (;;) {
        const int st = walk_step(a, walk, &tile);
        if (st == kWalkTile) break;
        if (st == kWalkDone) return;
        settle_ticket();
    }
    walk.careful = false;                              // nothing is parked yet, nothing has waited
    bool cur_redo = false;
    const uint32_t t_off = (uint32_t)wave * kWaveSpan + (uint32_t)lane * kVec;
    RawTile<0> raw_old;
    RawTile<NEW_F32> raw_new;
#pragma unroll
    for (int j = 0; j < kIters; ++j) raw_zero(j, raw_old, raw_new);
    // the tile's context, its loads (if 128-bit loads are legal for it), and what is kept of it
    auto start_tile = [&](int32_t t) -> TileMeta {
        const TileCtx c = tile_ctx(a, __builtin_amdgcn_readfirstlane(t));
        if (c.vec) load_raw_pair<NEW_F32>(c, t_off, raw_old, raw_new);
        return tile_meta(c, t);
    };
    TileMeta cur, nxt;
    bool loaded = false;                               // the tile's loads have been issued

    for (;;) {
        // All of the following are the same in every lane; saying so keeps them, and everything
        // derived from them, in scalar registers.
        tile = __builtin_amdgcn_readfirstlane(tile);
        q_head = __builtin_amdgcn_readfirstlane(q_head);
        q_len = __builtin_amdgcn_readfirstlane(q_len);
        ring_used = (uint32_t)__builtin_amdgcn_readfirstlane((int)ring_used);
        ring_head = (uint32_t)__builtin_amdgcn_readfirstlane((int)ring_head);
        parity = __builtin_amdgcn_readfirstlane(parity);
        n_announced = __builtin_amdgcn_readfirstlane(n_announced);
        n_polled = __builtin_amdgcn_readfirstlane(n_polled);
        walk.ticket = __builtin_amdgcn_readfirstlane(walk.ticket);
        walk.j = __builtin_amdgcn_readfirstlane(walk.j);
        walk.next_ticket = __builtin_amdgcn_readfirstlane(walk.next_ticket);
        walk.redo_through = __builtin_amdgcn_readfirstlane(walk.redo_through);
        {
            const int flags = __builtin_amdgcn_readfirstlane((int)loaded | (int)cur_redo << 1 | (int)ticket_out << 2 |
                                                             (int)walk.have_next << 3 | (int)walk.exhausted << 4 |
                                                             (int)walk.careful << 5 | (int)walk.redo << 6);
            loaded = flags & 1;
            cur_redo = flags & 2;
            ticket_out = flags & 4;
            walk.have_next = flags & 8;
            walk.exhausted = flags & 16;
            walk.careful = flags & 32;
            walk.redo = flags & 64;
        }
        cur = loaded ? nxt : start_tile(tile);         // not loaded: the first tile, or one named late
        // ---- (a) change masks ----
        const uint32_t k_wave = cur.k_tile + (uint32_t)wave * kWaveSpan;
        uint4 nv[kIters];                              // the new patterns
        uint4 pv[ARITH ? kIters : 1];                  // arithmetic payloads (difference, or new where it escapes)
        uint32_t esc_all = 0;                          // bit 8 j + e: element e of vector j escapes
        uint32_t mask[kIters];
        // Always taken from the load registers, also for a tile that has no 128-bit loads (its
        // result is replaced below): this way every path consumes what was loaded, and the
        // compiler never has to wait for memory before the registers are loaded again.
#pragma unroll
        for (int j = 0; j < kIters; ++j) {
            nv[j] = raw_to_bf16(raw_new, j);
            mask[j] = nz16_mask(xor4(raw_old.v[j], nv[j]));
            if constexpr (ARITH) {
                uint32_t esc8;
                pv[j] = arith_vec(raw_old.v[j], nv[j], &esc8);
                esc_all |= esc8 << (8 * j);
            }
        }
        // pin the above here: the load registers are dead from this point on, whatever the
        // scheduler would prefer
#pragma unroll
        for (int j = 0; j < kIters; ++j)
            asm volatile("" : "+v"(mask[j]), "+v"(nv[j].x), "+v"(nv[j].y), "+v"(nv[j].z), "+v"(nv[j].w));
        if constexpr (ARITH) {
#pragma unroll
            for (int j = 0; j < kIters; ++j) asm volatile("" : "+v"(pv[j].x), "+v"(pv[j].y), "+v"(pv[j].z), "+v"(pv[j].w));
            asm volatile("" : "+v"(esc_all));
        }
        if (cur.vec & 1u) {
            if (cur.limit != 0xFFFFFFFFu) {            // vectors past the end of the piece hold nothing
#pragma unroll
                for (int j = 0; j < kIters; ++j)
                    if (k_wave + (uint32_t)(j * 64 + lane) * kVec + kVec > cur.limit) mask[j] = 0;
            }
            // a piece whose length is not a multiple of 8: the one vector that straddles its end
            if (cur.limit != 0xFFFFFFFFu && (cur.limit & (kVec - 1))) {
                const uint32_t ks = cur.limit & ~(uint32_t)(kVec - 1);
                const TileCtx c = tile_ctx(a, __builtin_amdgcn_readfirstlane(tile));
                if (ks >= k_wave && ks < k_wave + (uint32_t)kWaveSpan && ((ks - k_wave) / kVec) % 64 == (uint32_t)lane) {
                    const uint32_t js = (ks - k_wave) / (64 * kVec);
                    uint4 o = load_vec_general<0>(c.old_base, c.pc, ks);
                    uint4 n = load_vec_general<NEW_F32>(c.new_base, c.pc, ks);
                    uint32_t m = nz16_mask(xor4(o, n));
                    uint32_t esc8 = 0;
                    uint4 pay = n;
                    if constexpr (ARITH) pay = arith_vec(o, n, &esc8);
#pragma unroll
                    for (int jj = 0; jj < kIters; ++jj) {
                        if ((uint32_t)jj == js) {
                            nv[jj] = n;
                            mask[jj] = m;
                            if constexpr (ARITH) {
                                pv[jj] = pay;
                                esc_all = (esc_all & ~(0xFFu << (8 * jj))) | (esc8 << (8 * jj));
                            }
                        }
                    }
                }
            }
        } else {
            // shapes or pointers that are not multiples of 16 bytes.  Kept as a rolled loop (one
            // vector in flight) so that this rare path does not set the kernel's register budget;
            // the selects put the result into static slots
            const TileCtx c = tile_ctx(a, __builtin_amdgcn_readfirstlane(tile));
#pragma unroll 1
            for (int j = 0; j < kIters; ++j) {
                uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
                uint4 o = load_vec_general<0>(c.old_base, c.pc, k);
                uint4 n = load_vec_general<NEW_F32>(c.new_base, c.pc, k);
                uint32_t m = nz16_mask(xor4(o, n));
                uint32_t esc8 = 0;
                uint4 pay = n;
                if constexpr (ARITH) pay = arith_vec(o, n, &esc8);
#pragma unroll
                for (int jj = 0; jj < kIters; ++jj) {
                    if (jj == j) {
                        nv[jj] = n;
                        mask[jj] = m;
                        if constexpr (ARITH) {
                            pv[jj] = pay;
                            esc_all = (esc_all & ~(0xFFu << (8 * jj))) | (esc8 << (8 * jj));
                        }
                    }
                }
            }
        }

        // ---- (b) poll answers and ticket of the previous iteration; copy out what was announced ----
        const bool accept_now = ticket_out;
        if (accept_now && threadIdx.x == 0) {
            s_ticket[parity] = (int32_t)ticket_take<WIDE>();   // nothing else is in flight here
        }
        ticket_out = false;
        if (wave == 0 && lane < n_polled && !has_prefix(wq_w)) wq_w = polled;
#if ROSE_DIAG & 1
        wq_w = kStatusPrefix << kStatusShift;
#endif
        if (n_announced > 0) {
            ring_used -= copy_out(n_announced, s_excl[parity ^ 1], true);
            pop(n_announced);
            n_announced = 0;
        }
        if (wave == 0) {
            const u64 unknown = __ballot(lane < q_len && !has_prefix(wq_w));
            int n_ready = unknown ? __ffsll((long long)unknown) - 1 : q_len;
            // Timed order: bucket stores go out in windows of time that all workgroups share (a
            // constant-rate clock every wave can read): a steady trickle of writes among the reads
            // costs the memory far more than the same bytes written in bursts (a plain streaming
            // kernel that reads two streams at 7.1 TB/s loses 22 % when it writes 1.5 % of what it
            // reads tile by tile, and 6 % when it writes the same bytes in such windows).  Outside a
            // window parked tiles simply stay parked, unless the ring or the queue is more than three
            // quarters full.
            if (a.timed) {
                const uint32_t now = (uint32_t)__builtin_amdgcn_s_memrealtime();
                const bool open = (now & ((1u << ROSE_WRITE_PERIOD_LOG2) - 1u)) < (1u << ROSE_WRITE_OPEN_LOG2);
                const bool pressure = q_len > kQueue * 3 / 4 || ring_used > (uint32_t)kRing * ROSE_WRITE_RING_NUM / 8;
                if (!open && !pressure) n_ready = 0;
            }
            if (lane < n_ready) s_excl[parity][lane] = wq_w & kValueMask;
            if (lane == 0) s_nready[parity] = n_ready;
            // ---- (c) poll: one lane per parked tile that has no prefix yet ----
            if (lane < q_len && !has_prefix(wq_w)) polled = desc_load(a.tile_desc + wq_tile);
        }
        n_polled = q_len;
        // ask for the next ticket as soon as the one fetched ahead has been taken into use
        if (!walk.have_next && !accept_now && !walk.exhausted && !walk.redo) {
            if (threadIdx.x == 0) ticket_request<WIDE>(a.ticket);
            ticket_out = true;
        }

        // ---- (d) the next tile's loads go out now and stay in flight during everything below ----
        int32_t next = -1;
        const int32_t ticket_before = walk.ticket;
        int next_state = walk_step(a, walk, &next);     // kWalkNeedTicket: decided after the barrier
        next_state = __builtin_amdgcn_readfirstlane(next_state);   // uniform anyway: scalar branches below
        next = __builtin_amdgcn_readfirstlane(next);
        bool nxt_redo = walk.redo;
        loaded = next_state == kWalkTile;
        if (loaded) nxt = start_tile(next);

        // ---- (e) exclusive rank of each of this lane's vectors inside the wave's span: the
        // per-vector counts (<= 8, wave totals <= 512) are scanned two at a time in 16-bit fields
        uint32_t rank[kIters];
        uint32_t wave_total = 0;
#pragma unroll
        for (int j = 0; j < kIters; j += 2) {
            const uint32_t c0 = __popc(mask[j]);
            const uint32_t c1 = (j + 1 < kIters) ? __popc(mask[j + 1]) : 0u;
            const uint32_t inc = wave_incl_scan(c0 | (c1 << 16));
            const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
            rank[j] = wave_total + (inc & 0xFFFFu) - c0;
            wave_total += tot & 0xFFFFu;
            if (j + 1 < kIters) {
                rank[j + 1] = wave_total + (inc >> 16) - c1;
                wave_total += tot >> 16;
            }
        }
        if (lane == 0) s_wave_total[parity][wave] = wave_total;
        __syncthreads();
        if (accept_now) walk_accept(a, walk, (uint32_t)__builtin_amdgcn_readfirstlane(s_ticket[parity]));
        n_announced = __builtin_amdgcn_readfirstlane(s_nready[parity]);
        uint32_t wave_excl = 0, tile_total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            uint32_t c = s_wave_total[parity][w];
            if (w < wave) wave_excl += c;
            tile_total += c;
        }
        tile_total = (uint32_t)__builtin_amdgcn_readfirstlane((int)tile_total);   // uniform: scalar bookkeeping below
        parity ^= 1;

        // publish the count: a serving wave turns it into this tile's prefix
        if (threadIdx.x == 0 && !cur_redo && !(ROSE_DIAG & 4))
            desc_store(a.tile_desc + tile, (kStatusAggregate << kStatusShift) | tile_total);

        // Room to park?  Making room may wait, and nothing may wait while a ticket is on its way
        // (it could be of the current ticket's group): take it in first.
        const bool big = tile_total > (uint32_t)kRing;
        if (ticket_out && !walk.careful && (big || q_len == kQueue || ring_used + tile_total > (uint32_t)kRing))
            settle_ticket();
        // A same-group ticket has just been accepted: nothing may wait now.  This tile is not
        // parked; it is walked again after the count-only pass at the end of the iteration.
        // Tiles so dense that the ring does not hold a ticket's worth (fewer tiles are parked than a
        // ticket has, and there is no room for this one), with tiles of the current ticket still
        // uncounted: waiting now would make every worker of a later group wait for those counts
        // while this one waits for the prefix of the same ticket's first tile, and the groups of
        // workers would take turns instead of running side by side.  So the rest of the ticket is
        // counted first and the ticket's tiles, this one included, are walked again without
        // publishing, exactly as for a same-group pair (below).
        bool dense = false;
#if ROSE_COUNT_AHEAD
        // the next tile is of the same ticket: not all of the ticket is counted
        const bool mid_ticket = !walk.careful && !cur_redo && !walk.redo && !big && next_state == kWalkTile &&
                                walk.ticket == ticket_before;
        if (a.adjacent) {
            // A ticket's tiles are neighbours, so its uncounted tiles may lie in the very block whose
            // prefixes a wait would be for: in the middle of a ticket nothing may wait at all.  First
            // look, without waiting, whether prefixes have arrived since the last poll.
            if (__builtin_expect(mid_ticket && (q_len == kQueue || ring_used + tile_total > (uint32_t)kRing), 0)) {
                if (q_len > 0) drain(kDrainReady);
                dense = q_len == kQueue || ring_used + tile_total > (uint32_t)kRing;
            }
        } else if (__builtin_expect(ring_used + tile_total > (uint32_t)kRing && q_len < a.batch, 0)) {
            dense = mid_ticket;
        }
#endif
        const bool skip = walk.careful || dense;
        if (skip) {
        } else if (big) {
            if (q_len > 0) drain(kDrainAll);
        } else {
            while (q_len == kQueue || ring_used + tile_total > (uint32_t)kRing) drain(kDrainOldest);
        }

        const int32_t chain_last = a.chain_first[cur.shard + 1] - 1;
        const int32_t seg = cur.seg;
        if (skip) {
        } else if (!big) {
            // park the entries: ring slot = ring_head + rank inside the tile
            const uint32_t base = ring_head + wave_excl;
#pragma unroll
            for (int j = 0; j < kIters; ++j) {
                uint32_t m = mask[j];
                uint32_t slot = base + rank[j];
                const uint32_t in_tile0 = t_off + (uint32_t)(j * 64) * kVec;
                while (m && !(ROSE_DIAG & 8)) {
                    const uint32_t e = __ffs(m) - 1;
                    m &= m - 1;
                    if constexpr (ARITH)
                        s_ring[slot & (kRing - 1)] = ((in_tile0 + e) << 16) | (pick16(pv[j], e) & 0xFFFFu) |
                                                     ((esc_all >> (8 * j + e)) << 31);
                    else
                        s_ring[slot & (kRing - 1)] = ((in_tile0 + e) << 16) | (pick16(nv[j], e) & 0xFFFFu);
                    ++slot;
                }
            }
            if (threadIdx.x == 0) {
                const int slot = (q_head + q_len) & (kQueue - 1);
                s_q_count[slot] = tile_total;
                s_q_off[slot] = ring_head;
                s_q_base[slot] = cur.out_base;
                s_q_piece[slot] = cur.piece;
                s_q_shard[slot] = cur.shard;
                s_q_seg[slot] = seg;
                s_q_last[slot] = tile == chain_last;
            }
            if (wave == 0 && lane == q_len) {
                wq_tile = tile;
                wq_w = 0;
            }
            ++q_len;
            ring_used += tile_total;
            ring_head = (ring_head + tile_total) & (kRing - 1);
        } else {
            // more entries than the ring holds: wait for the prefix now, write from registers
            if (wave == 0) {
                bool ok = true;
                u64 excl = 0;
#if !(ROSE_DIAG & 1)
                unsigned int spins = 0;
                for (;;) {
                    u64 v = desc_load(a.tile_desc + tile);
                    if ((v >> kStatusShift) == kStatusPrefix) {
                        excl = v & kValueMask;
                        break;
                    }
                    if (!keep_waiting(a.abort_flag, spins, lane)) {
                        ok = false;
                        break;
                    }
                }
#endif
                if (lane == 0) {
                    s_direct_excl = excl;
                    s_ok = ok ? 1 : 0;
                }
            }
            __syncthreads();
            const u64 tile_excl = s_direct_excl;
            const BucketDev b = a.bucket[cur.shard];
            const Piece big_pc = load_piece(a.pieces + (cur.piece >= 0 ? cur.piece : 0));
            if (s_ok && !(ROSE_DIAG & 2)) {
                if (threadIdx.x == 0) {
                    if (seg >= 0) b.seg_off[seg] = (int64_t)tile_excl;
                    if (tile == chain_last) b.seg_off[a.n_tensors] = (int64_t)(tile_excl + tile_total);
                }
                const u64 wave_base = tile_excl + wave_excl;
#pragma unroll
                for (int j = 0; j < kIters; ++j) {
                    uint32_t m = mask[j];
                    u64 pos = wave_base + rank[j];
                    // cur.out_base + offset is the local index, or (strided local indices) the
                    // element number that the piece maps to one
                    const uint32_t local0 = cur.out_base + t_off + (uint32_t)(j * 64) * kVec;
                    while (m) {
                        const uint32_t e = __ffs(m) - 1;
                        m &= m - 1;
                        if (pos < (u64)b.capacity) {
                            uint32_t local = cur.piece >= 0 ? dst_index(big_pc, local0 + e, false) : local0 + e;
                            if constexpr (ARITH) {
                                local |= (esc_all >> (8 * j + e)) << 31;
                                b.val[pos] = (uint16_t)pick16(pv[j], e);
                            } else {
                                b.val[pos] = (uint16_t)pick16(nv[j], e);
                            }
                            b.idx[pos] = (int32_t)local;
                        }
                        ++pos;
                    }
                }
            }
            __syncthreads();                           // s_direct_excl / s_ok are reused
        }

        // Sender refresh (W_{t-1} <- W_t for what this tile covers): only now that the tile is known
        // not to be walked again, and never for replicated tensors, which other destinations' tiles
        // still have to read (a small kernel after this one copies those).
        if constexpr (REFRESH) {
            if (!skip && !(cur.vec & 2u)) {
                const TileCtx c = tile_ctx(a, __builtin_amdgcn_readfirstlane(tile));
                uint16_t *ob = const_cast<uint16_t *>(c.old_base);
                // a tile with many changes is written whole: full lines cost the memory less than
                // many partial ones
                const bool whole = (cur.vec & 1u) && c.limit == 0xFFFFFFFFu && tile_total > (uint32_t)ROSE_REFRESH_WHOLE;
#pragma unroll
                for (int j = 0; j < kIters; ++j) {
                    if (mask[j] || whole) {
                        const uint32_t k = c.k_tile + t_off + (uint32_t)(j * 64) * kVec;
                        if ((cur.vec & 1u) && (c.limit == 0xFFFFFFFFu || k + kVec <= c.limit)) {
#if ROSE_REFRESH_NT
                            {
                                u32x4 w = {nv[j].x, nv[j].y, nv[j].z, nv[j].w};
                                __builtin_nontemporal_store(w, reinterpret_cast<global_u32x4 *>(reinterpret_cast<uintptr_t>(ob + src_index(c.pc, k, true))));
                            }
#else
                            gstore16(ob + src_index(c.pc, k, true), nv[j]);     // unchanged elements keep their bits
#endif
                        } else {
                            uint32_t m = mask[j];
                            while (m) {
                                const uint32_t e = __ffs(m) - 1;
                                m &= m - 1;
                                ob[src_index(c.pc, k + e, false)] = (uint16_t)pick16(nv[j], e);
                            }
                        }
                    }
                }
            }
        }

        // The rare cases that the next tile could not be named before the barrier above, or that a
        // same-group ticket has arrived: settle them now; the next tile's loads are then issued at
        // the top of the next iteration.
        bool late = false;
        bool redo_cur = skip;                          // this iteration's tile was not parked
        for (;;) {
            if (walk.careful || dense) {
                // the ticket in use (tA) and the one just accepted (tB) are of one group: publish
                // the counts of everything not yet published, then walk those tiles again.  The
                // dense case (above) is the same with no second ticket: the rest of tA is counted
                // and tA is walked again from this iteration's tile on.
                const bool pair = walk.careful;
                const int32_t tA = walk.ticket, tB = walk.next_ticket;
                const int32_t j_end = pair ? 2 * a.batch : a.batch;
                int32_t j_from = a.batch;               // first slot of tA to walk again
                if (redo_cur)
                    for (int32_t j = 0; j < a.batch; ++j)
                        if (ticket_tile(a, tA, j) == tile) j_from = j;
                redo_cur = false;
                // slot j_from itself is published (it is this iteration's tile); when tA is used up
                // (j_from = kBatch) every slot of tB is still to be counted
#pragma unroll 1
                for (int32_t j = j_from < a.batch ? j_from + 1 : a.batch; j < j_end; ++j) {
                    const int32_t t = j < a.batch ? ticket_tile(a, tA, j) : ticket_tile(a, tB, j - a.batch);
                    if (t >= 0) publish_count(t);
                }
                __syncthreads();
                if (threadIdx.x == 0)                  // diagnostic words: how often each happened
                    __hip_atomic_fetch_add(a.abort_flag + (pair ? kWsCarefulWord : kWsAheadWord), 1u, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                walk.careful = false;
                dense = false;
                walk.redo = true;
                walk.redo_through = pair ? tB : tA;
                walk.j = j_from - 1;
                next_state = walk_step(a, walk, &next);
                late = true;
            }
            if (next_state != kWalkNeedTicket) break;
            if (!walk.have_next && !walk.exhausted) {
                settle_ticket();
                if (walk.careful) continue;
            }
            next_state = walk_step(a, walk, &next);
            late = true;
        }
        if (late) {
            nxt_redo = walk.redo;
            loaded = false;
        }
        if (next_state == kWalkDone) break;
        cur_redo = nxt_redo;
        tile = next;
    }
    while (q_len > 0) drain(kDrainAll);
}

// The instantiations get their own register budgets: 4 waves per SIMD (128 VGPRs) fit the bf16
// kernels without spills; the fp32-master kernels hold twice the raw data, and the kernel that both
// refreshes and forms arithmetic payloads keeps new values and payloads side by side: those get 3
// (the one that does all three at once: 2).
// REFRESH = 1 also writes the new bf16 values over the old ones; ARITH = 1 emits arithmetic payloads.
template <int NEW_F32, int REFRESH, int ARITH> __global__ void encode_kernel(EncodeArgs a);
#define ROSE_ENCODE_KERNEL(F32, REFRESH, ARITH, WAVES, VGPRS)                                                         \
    template <>                                                                                                       \
    __global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES), amdgpu_num_vgpr(VGPRS))) \
    void encode_kernel<F32, REFRESH, ARITH>(EncodeArgs a) {                                                           \
        encode_body<F32, REFRESH, ARITH>(a);                                                                          \
    }
ROSE_ENCODE_KERNEL(0, 0, 0, 4, kNumVgpr0)
ROSE_ENCODE_KERNEL(0, 1, 0, 4, kNumVgpr0)
ROSE_ENCODE_KERNEL(0, 0, 1, 4, kNumVgpr0)
ROSE_ENCODE_KERNEL(0, 1, 1, 3, kNumVgpr1)
ROSE_ENCODE_KERNEL(1, 0, 0, 3, kNumVgpr1)
ROSE_ENCODE_KERNEL(1, 1, 0, 3, kNumVgpr1)
ROSE_ENCODE_KERNEL(1, 0, 1, 3, kNumVgpr1)
ROSE_ENCODE_KERNEL(1, 1, 1, 2, kNumVgpr2)
#undef ROSE_ENCODE_KERNEL

// Replicated tensors after an encode with refresh: old <- bf16(new), whole tensors (they are small).
__global__ __launch_bounds__(256) void refresh_replicated_kernel(const int32_t *list, const int64_t *numel, int32_t n,
                                                                 void *const *old_ptrs, const void *const *new_ptrs,
                                                                 int new_is_f32) {
    for (int32_t i = blockIdx.y; i < n; i += gridDim.y) {
        const int32_t t = list[i];
        uint16_t *o = static_cast<uint16_t *>(old_ptrs[t]);
        const int64_t cnt = numel[i];
        for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < cnt; k += (int64_t)gridDim.x * blockDim.x)
            o[k] = new_is_f32 ? (uint16_t)rne_bf16(static_cast<const uint32_t *>(new_ptrs[t])[k])
                              : static_cast<const uint16_t *>(new_ptrs[t])[k];
    }
}

// ---------------------------------------------------------------------------------------------
// apply (App. F S2D): every entry's value goes to its local index of the receiver's copy.
//
// Scattered 2-byte stores reach memory as byte-masked partial writes of the lines they touch,
// which the memory side turns into slow read-modify-writes (measured: about 3 TB/s of line
// traffic).  So the kernel does the read-modify-write itself, one 64-byte line at a time, with
// 128-bit accesses marked non-temporal (a line is touched once per launch; with the hints this
// path was never slower than direct stores between 1 % and 10 % density, without them it lost
// below 3 %): a wave takes 64 consecutive entries (ascending local index inside a segment,
// so the entries of a line are neighbours), finds the distinct lines they touch, loads those lines
// into LDS, patches the entries in, and stores the lines back whole.
//
// A line's entries may straddle two waves' chunks (a line holds at most 32 entries, a chunk 64):
// the line belongs to the wave that holds its FIRST entry; that wave also applies the entries of
// its last line that lie in the next chunk, and the next wave skips them.  Entries whose own
// 16-byte part of the line is not entirely inside the tensor (the last few elements of a tensor
// whose size is not a multiple of 8) and entries of tensors that are not 16-byte aligned are stored
// directly; the line path never touches those bytes.
// ---------------------------------------------------------------------------------------------
#ifndef ROSE_APPLY_NT
#define ROSE_APPLY_NT 14     // non-temporal hints: 1 entry loads, 2 line loads, 4 line stores, 8 direct stores
                             // (measured best on the 7B workload at 1 - 10 % density)
#endif
#ifndef ROSE_APPLY_BLOCKS
#define ROSE_APPLY_BLOCKS (256 * 512)           // most workgroups an apply launch uses (7B workload, four shards, one
                                                // chunk per wave: 2.40 / 3.64 / 4.92 ms at 1 / 2 / 5 % with 256 * 128,
                                                // 2.36 / 3.48 / 4.51 ms with 256 * 512 or more)
#endif
constexpr int kApplyThreads = 256;
constexpr int kApplyWaves = kApplyThreads / 64;
#ifndef ROSE_APPLY_LINE
#define ROSE_APPLY_LINE 64                      // bytes moved around an entry: 64 or 32 (32 halves the bytes at low
                                                // density and is slower all the same: 7B workload 3.61 instead of
                                                // 2.43 ms at 1 %, 7.91 instead of 5.20 ms at 5 %: the memory moves
                                                // 64-byte units)
#endif
constexpr int kLineElems = ROSE_APPLY_LINE / 2; // line of 16-bit elements
constexpr int kLineShift = ROSE_APPLY_LINE == 128 ? 6 : ROSE_APPLY_LINE == 64 ? 5 : 4;
constexpr int kLineParts = kLineElems / 8;      // 16-byte parts of a line
constexpr int kLinesPerRound = 64 / kLineParts; // lines a wave moves with one load per lane
static_assert(ROSE_APPLY_LINE == 128 || ROSE_APPLY_LINE == 64 || ROSE_APPLY_LINE == 32, "line size");


__device__ __forceinline__ void lds_wave_fence() {
    // LDS operations of one wave are carried out in order; this keeps the compiler from moving
    // them across and waits for the ones issued so far.
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// Largest t in [0, n) with seg_off[t] <= e, for a wave-uniform e < seg_off[n]: a 64-ary search,
// one parallel probe per round (two rounds up to 4096 tensors).
__device__ __forceinline__ int32_t wave_find_segment(const int64_t *seg_off, int32_t n, int64_t e, int lane) {
    int32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int32_t step = (hi - lo + 63) >> 6;
        const int32_t probe = lo + lane * step;
        const bool le = probe < hi && seg_off[probe] <= e;   // true on a prefix of the lanes, lane 0 included
        const int k = __popcll(__ballot(le)) - 1;
        lo += k * step;
        hi = hi < lo + step ? hi : lo + step;
    }
    return lo;
}

// value an entry leaves at its element: the payload itself, or (arithmetic payload, no escape)
// bf16(current + payload), see arith_pair
__device__ __forceinline__ uint16_t apply_value(uint32_t cur, uint32_t val, bool add) {
    if (!add) return (uint16_t)val;
    return (uint16_t)pack_bf16_pair(__uint_as_float(cur << 16) + __uint_as_float(val << 16), 0.0f);
}

// arith != 0: the bucket holds arithmetic payloads (bit 31 of an index marks an entry that carries
// the new pattern instead)
//
// The entries are cut into RUNS of chunks of 64, dealt round robin to the grid's waves, so that at any
// time the waves work inside one band of the bucket that moves forward.  How long a run should be
// depends on the density (measured on the 7B-style workload, 4 shards: runs of 1 / 8 chunks take
// 2.36 / 2.58 ms at 1 %, 4.51 / 5.56 ms at 5 %, 7.30 / 6.0 ms at 10 %): where nearly every line of the
// destination is touched, long runs make a wave stream through a contiguous piece of it; where the
// touched lines lie apart, one chunk per wave and as many workgroups as there are chunks do best.  The
// kernel picks the run length from the density it sees (entries against the elements of the shard).
// Inside a run what a chunk needs from its neighbours is at hand: the next chunk's entries are
// requested one chunk ahead (they are also the look-ahead for a line that straddles the two chunks),
// the previous chunk's last index stays in a register, and the segment the wave is in (tensor, ends,
// destination pointer, size) is uniform state that moves forward and is fetched with scalar loads.
// All of a chunk's line loads are issued before the first is taken in.
#ifndef ROSE_APPLY_RUN
#define ROSE_APPLY_RUN 8        // chunks per run in the dense regime
#endif
#ifndef ROSE_APPLY_DENSE_DIV
#define ROSE_APPLY_DENSE_DIV 13 // dense regime: at least one entry per this many elements of the shard
#endif
#ifndef ROSE_APPLY_DENSE_BLOCKS
#define ROSE_APPLY_DENSE_BLOCKS (256 * 128)     // workgroups that take part in the dense regime
#endif
constexpr int kLineRounds = 64 / kLinesPerRound;     // rounds of one load per lane that move up to 64 lines
// shard_elems: elements of the destination shard's tensors together (for the density estimate; objects,
// which hold a part of a stream, pass a value that keeps them out of the dense regime)
__device__ __forceinline__ void apply_body(const BucketDev &b, int32_t n_tensors, const int32_t *local_numel,
                                           void *const *dst_ptrs, int arith, int64_t shard_elems) {
    __shared__ uint4 s_line[kApplyWaves][64][kLineParts];   // wave, line slot, 16-byte part
    __shared__ u64 s_addr[kApplyWaves][64];             // address of the line
    __shared__ int32_t s_parts[kApplyWaves][64];        // 16-byte parts of the line inside the tensor
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t total = b.seg_off[n_tensors];
    if (total > b.capacity) total = b.capacity;
    if (total <= 0) return;
    const bool dense = total >= shard_elems / ROSE_APPLY_DENSE_DIV;
    uint32_t n_wgs = gridDim.x;
    if (dense && n_wgs > (uint32_t)ROSE_APPLY_DENSE_BLOCKS) n_wgs = ROSE_APPLY_DENSE_BLOCKS;
    const uint32_t wg = blockIdx.x;
    if (wg >= n_wgs) return;
    const int64_t n_waves = (int64_t)n_wgs * kApplyWaves;
    const int64_t run = dense ? (int64_t)ROSE_APPLY_RUN * 64 : 64;
    const int32_t idx_mask = arith ? 0x7FFFFFFF : -1;
    int32_t t_u = 0, t_have = -1, numel_u = 0;          // uniform: segment of the chunk's first entry, and the
    int64_t seg_start_u = 0, seg_end_u = 0;             // tensor whose pointer and size are loaded
    uint16_t *dst_u = nullptr;

    for (int64_t rbase = ((int64_t)wg * kApplyWaves + wave) * run; rbase < total; rbase += n_waves * run) {
        int64_t wbase = rbase;
        const int64_t wend = rbase + run < total ? rbase + run : total;
        if (wbase >= seg_end_u) {                       // (empty segments are stepped over by the search)
            t_u = __builtin_amdgcn_readfirstlane(wave_find_segment(b.seg_off, n_tensors, wbase, lane));
            seg_start_u = (int64_t)cload64(b.seg_off + t_u);
            seg_end_u = (int64_t)cload64(b.seg_off + t_u + 1);
        }
        // the run's first chunk, and the last index before the run
        int32_t cur_idx_raw = 0, prev_last = 0;
        uint32_t cur_val = 0;
        if (wbase + lane < total) {
#if ROSE_APPLY_NT & 1
            cur_idx_raw = __builtin_nontemporal_load(b.idx + wbase + lane);
            cur_val = __builtin_nontemporal_load(b.val + wbase + lane);
#else
            cur_idx_raw = b.idx[wbase + lane];
            cur_val = b.val[wbase + lane];
#endif
        }
        if (wbase > 0) prev_last = b.idx[wbase - 1] & idx_mask;

        for (;;) {
            const int64_t e = wbase + lane, e2 = e + 64;
            const bool valid = e < total;
            // the next chunk's entries: requested now, needed as look-ahead below and as the entries
            // of the next round (the run's last chunk only looks into them)
            int32_t nxt_idx_raw = 0;
            uint32_t nxt_val = 0;
            if (e2 < total && (lane < kLineElems || wbase + 64 < wend)) {     // whole only if the run goes on
#if ROSE_APPLY_NT & 1
                nxt_idx_raw = __builtin_nontemporal_load(b.idx + e2);
                nxt_val = __builtin_nontemporal_load(b.val + e2);
#else
                nxt_idx_raw = b.idx[e2];
                nxt_val = b.val[e2];
#endif
            }
            const int32_t idx_raw = cur_idx_raw;
            const uint32_t val = cur_val;
            const bool look = lane < kLineElems && e2 < total;
            const int32_t idx2_raw = look ? nxt_idx_raw : 0;
            const uint32_t val2 = look ? nxt_val : 0u;
            const int32_t idx = idx_raw & idx_mask, idx2 = idx2_raw & idx_mask;
            const bool add = arith && idx_raw >= 0, add2 = arith && idx2_raw >= 0;

            // tensor of the chunk's first entry, then of each lane's entry
            while (wbase >= seg_end_u) {                // ends: wbase < total <= seg_off[n_tensors]
                ++t_u;
                seg_start_u = seg_end_u;
                seg_end_u = (int64_t)cload64(b.seg_off + t_u + 1);
            }
            int32_t t = t_u;
            int64_t seg_end = seg_end_u;
            uint16_t *dst;
            int32_t numel;
            const int64_t chunk_last = wbase + 63 < total ? wbase + 63 : total - 1;
            if (chunk_last < seg_end_u) {               // the whole chunk lies in one segment: all uniform
                if (t_have != t_u) {
                    dst_u = reinterpret_cast<uint16_t *>(cload64(dst_ptrs + t_u));
                    numel_u = (int32_t)cload32(local_numel + t_u);
                    t_have = t_u;
                }
                dst = valid ? dst_u : nullptr;
                numel = valid ? numel_u : 0;
            } else {
                while (valid && e >= seg_end) {
                    ++t;
                    seg_end = b.seg_off[t + 1];
                }
                dst = valid ? static_cast<uint16_t *>(dst_ptrs[t]) : nullptr;
                numel = valid ? local_numel[t] : 0;
            }
            // may this entry go through the line path?  (depends on the entry alone)
            const bool ok = valid && (((uintptr_t)dst) & 15u) == 0 && idx >= 0 && (idx | 7) < numel;
            const u64 key = valid ? (((u64)(uint32_t)t << 32) | (uint32_t)(idx >> kLineShift)) : ~0ull;

            // same line as the entry before?  lane 0 looks at the last entry of the previous chunk
            u64 prev_key = __shfl_up(key, 1, 64);
            if (lane == 0)
                prev_key = wbase > seg_start_u ? (((u64)(uint32_t)t << 32) | (uint32_t)(prev_last >> kLineShift)) : ~0ull - 1;
            const bool same = valid && key == prev_key;
            // leading lanes that continue the previous chunk's last line were applied with that chunk
            const u64 not_same = __ballot(!same);
            const int first_own = not_same ? __ffsll((long long)not_same) - 1 : 64;
            const bool owned = ok && lane >= first_own;
            const bool direct = valid && !ok && idx >= 0 && idx < numel;   // an index outside the tensor is dropped

            // entries of the next chunk that still lie in this chunk's last line
            const u64 key63 = __shfl(key, 63, 64);
            const bool own63 = __shfl((int)owned, 63, 64) != 0;
            const int64_t seg_end63 = __shfl(seg_end, 63, 64);
            const int32_t numel63 = __shfl(numel, 63, 64);
            const bool ext = own63 && look && e2 < seg_end63 &&
                             ((key63 & ~0xffffffffull) | (uint32_t)(idx2 >> kLineShift)) == key63 && idx2 >= 0 &&
                             (idx2 | 7) < numel63;

            // distinct lines of the owned entries
            const bool prev_owned = __shfl_up((int)owned, 1, 64) != 0 && lane > 0;
            const bool head = owned && (!prev_owned || !same);
            const u64 heads = __ballot(head);
            const int n_lines = __popcll(heads);
            const int slot = __popcll(heads & ((2ull << lane) - 1)) - 1;      // line slot of an owned lane
            if (head) {
                const int32_t line_first = (idx >> kLineShift) << kLineShift;
                s_addr[wave][slot] = (u64)(uintptr_t)(dst + line_first);
                int32_t parts = (numel - line_first) >> 3;
                s_parts[wave][slot] = parts > kLineParts ? kLineParts : parts;
            }
            lds_wave_fence();

            // load the lines: kLineParts lanes per line, kLinesPerRound lines per round; every
            // round's load is issued before the first one is put into LDS
            const int part = lane % kLineParts;
            uint4 lv[kLineRounds];
            u64 la[kLineRounds];
            bool on[kLineRounds];
#pragma unroll
            for (int r = 0; r < kLineRounds; ++r) {
                const int sl = r * kLinesPerRound + lane / kLineParts;
                on[r] = sl < n_lines && part < s_parts[wave][sl];
                la[r] = on[r] ? s_addr[wave][sl] + (u64)(part * 16) : 0;
            }
#pragma unroll
            for (int r = 0; r < kLineRounds; ++r) {
                lv[r] = make_uint4(0, 0, 0, 0);
                if (on[r]) {
#if ROSE_APPLY_NT & 2
                    lv[r] = gload16_stream(reinterpret_cast<const void *>((uintptr_t)la[r]));
#else
                    lv[r] = gload16(reinterpret_cast<const void *>((uintptr_t)la[r]));
#endif
                }
            }
#pragma unroll
            for (int r = 0; r < kLineRounds; ++r)
                if (on[r]) s_line[wave][r * kLinesPerRound + lane / kLineParts][part] = lv[r];
            lds_wave_fence();

            // patch
            uint16_t *lines16 = reinterpret_cast<uint16_t *>(&s_line[wave][0][0]);
            if (owned) {
                uint16_t *q = lines16 + slot * kLineElems + (idx & (kLineElems - 1));
                *q = apply_value(*q, val, add);
            }
            if (ext) {
                uint16_t *q = lines16 + (n_lines - 1) * kLineElems + (idx2 & (kLineElems - 1));
                *q = apply_value(*q, val2, add2);
            }
            lds_wave_fence();

            // store the lines back whole
#pragma unroll
            for (int r = 0; r < kLineRounds; ++r) {
                if (on[r]) {
                    const uint4 v4 = s_line[wave][r * kLinesPerRound + lane / kLineParts][part];
#if ROSE_APPLY_NT & 4
                    u32x4 w = {v4.x, v4.y, v4.z, v4.w};
                    __builtin_nontemporal_store(w, reinterpret_cast<global_u32x4 *>((uintptr_t)la[r]));
#else
                    gstore16(reinterpret_cast<void *>((uintptr_t)la[r]), v4);
#endif
                }
            }
            if (direct) {
                const uint16_t v = apply_value(add ? dst[idx] : 0u, val, add);
#if ROSE_APPLY_NT & 8
                __builtin_nontemporal_store(v, dst + idx);
#else
                dst[idx] = v;
#endif
            }
            lds_wave_fence();                           // the LDS slots are reused by the next chunk

            wbase += 64;
            if (wbase >= wend) break;
            prev_last = __builtin_amdgcn_readlane(idx, 63); // the chunk was full: another one follows
            cur_idx_raw = nxt_idx_raw;
            cur_val = nxt_val;
        }
    }
}

__global__ __launch_bounds__(kApplyThreads) void apply_kernel(BucketDev b, int32_t n_tensors,
                                                              const int32_t *local_numel, void *const *dst_ptrs, int arith,
                                                              int64_t shard_elems) {
    apply_body(b, n_tensors, local_numel, dst_ptrs, arith, shard_elems);
}

// ---------------------------------------------------------------------------------------------
// Transport objects (Sec. 4.2 "Asynchronous Weight Transfer": fixed-size buckets that describe
// themselves): a range of a destination's entries with a header and its own segment table, see
// the layout in the header file.  pack copies; apply checks the header on the device and then
// runs the ordinary apply on the arrays inside the object.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline size_t up16(size_t x) { return (x + 15) & ~(size_t)15; }
__host__ __device__ inline size_t object_idx_off(int32_t n_tensors) { return up16(64 + 8 * ((size_t)n_tensors + 1)); }
__host__ __device__ inline size_t object_size(int32_t n_tensors, int64_t n) {
    return object_idx_off(n_tensors) + up16(4 * (size_t)n) + up16(2 * (size_t)n);
}

__global__ __launch_bounds__(256) void pack_kernel(BucketDev b, int32_t shard, int32_t n_tensors, int64_t first,
                                                   int64_t n, int32_t payload, char *obj) {
    int64_t total = b.seg_off[n_tensors];
    if (total > b.capacity) total = b.capacity;
    const bool ok = total >= 0 && first + n <= total;          // else: an object nobody will apply
    const size_t a_off = object_idx_off(n_tensors), b_off = a_off + up16(4 * (size_t)n);
    if (blockIdx.x == 0) {
        if (threadIdx.x < 16) {
            uint32_t w = 0;
            if (threadIdx.x == 0) w = ok ? ROSE_OBJECT_MAGIC : 0u;
            if (threadIdx.x == 1) w = 1u;
            if (threadIdx.x == 2) w = (uint32_t)shard;
            if (threadIdx.x == 3) w = (uint32_t)n_tensors;
            if (threadIdx.x == 4) w = (uint32_t)(u64)first;
            if (threadIdx.x == 5) w = (uint32_t)((u64)first >> 32);
            if (threadIdx.x == 6) w = (uint32_t)(u64)n;
            if (threadIdx.x == 7) w = (uint32_t)((u64)n >> 32);
            if (threadIdx.x == 8) w = (uint32_t)payload;
            reinterpret_cast<uint32_t *>(obj)[threadIdx.x] = w;
        }
        int64_t *seg = reinterpret_cast<int64_t *>(obj + 64);
        for (int32_t t = threadIdx.x; t <= n_tensors; t += blockDim.x) {
            int64_t v = b.seg_off[t] - first;
            seg[t] = v < 0 ? 0 : (v > n ? n : v);
        }
        // the index and value arrays end on 16-byte boundaries: zero the slack
        int32_t *idx = reinterpret_cast<int32_t *>(obj + a_off);
        uint16_t *val = reinterpret_cast<uint16_t *>(obj + b_off);
        if (threadIdx.x < 4 && n + threadIdx.x < (int64_t)(up16(4 * (size_t)n) / 4)) idx[n + threadIdx.x] = 0;
        if (threadIdx.x < 8 && n + threadIdx.x < (int64_t)(up16(2 * (size_t)n) / 2)) val[n + threadIdx.x] = 0;
    }
    if (!ok) return;
    int32_t *idx = reinterpret_cast<int32_t *>(obj + a_off);
    uint16_t *val = reinterpret_cast<uint16_t *>(obj + b_off);
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        idx[e] = b.idx[first + e];
        val[e] = b.val[first + e];
    }
}

// true if the 64-byte header describes an object of this plan that fits object_bytes
__host__ __device__ inline bool object_header_ok(const uint32_t *h, int32_t n_tensors, size_t object_bytes, int64_t *n_out) {
    const int64_t first = (int64_t)((u64)h[4] | ((u64)h[5] << 32));
    const int64_t n = (int64_t)((u64)h[6] | ((u64)h[7] << 32));
    *n_out = n;
    if (h[0] != ROSE_OBJECT_MAGIC || h[1] != 1u || (int32_t)h[3] != n_tensors || first < 0 || n < 0) return false;
    if (h[8] > 1u) return false;                                        // payload kind: 0 new pattern, 1 arithmetic
    if (n > (int64_t)(object_bytes / 6)) return false;
    return object_size(n_tensors, n) <= object_bytes;
}

// the arrays inside an object whose header has passed object_header_ok
__device__ __forceinline__ BucketDev object_arrays(const char *obj, int32_t n_tensors, int64_t n) {
    const size_t a_off = object_idx_off(n_tensors), b_off = a_off + up16(4 * (size_t)n);
    BucketDev b;
    b.idx = reinterpret_cast<int32_t *>(const_cast<char *>(obj + a_off));
    b.val = reinterpret_cast<uint16_t *>(const_cast<char *>(obj + b_off));
    b.capacity = n;
    b.seg_off = reinterpret_cast<int64_t *>(const_cast<char *>(obj + 64));
    return b;
}

// Object apply runs as three launches on the stream: the verdict word is cleared, a pass over the
// segment table and all indices writes `ticket` into it if the object is not in order, and the apply
// pass leaves at once if it finds the ticket there.
__global__ void object_clear_kernel(u64 *verdict) { *verdict = 0; }

// Segment table: starts at 0, never decreases, ends at n.  Indices (escape bit masked off for
// arithmetic payloads): strictly ascending inside a segment, which is what lets the apply pass
// give every 64-byte piece of a tensor to exactly one wave.  An index may only fail to exceed its
// predecessor where a segment starts.
__global__ __launch_bounds__(256) void object_validate_kernel(const char *obj, size_t object_bytes, int32_t n_tensors,
                                                              int32_t n_buckets, u64 *verdict, u64 ticket) {
    uint32_t h[9];
    for (int i = 0; i < 9; ++i) h[i] = reinterpret_cast<const uint32_t *>(obj)[i];
    int64_t n;
    if (!object_header_ok(h, n_tensors, object_bytes, &n) || h[2] >= (uint32_t)n_buckets) return;   // apply rejects it too
    const BucketDev b = object_arrays(obj, n_tensors, n);
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (int64_t t = gid; t < n_tensors; t += stride) {
        const int64_t lo = b.seg_off[t], hi = b.seg_off[t + 1];
        bad |= lo < 0 || hi < lo || hi > n;
    }
    const int32_t m = h[8] ? 0x7FFFFFFF : -1;
    for (int64_t e = gid + 1; e < n; e += stride) {
        if ((b.idx[e] & m) <= (b.idx[e - 1] & m)) {
            // allowed only if some segment starts at e: smallest t with seg_off[t] >= e
            int32_t lo = 0, hi = n_tensors;
            while (lo < hi) {
                const int32_t mid = (lo + hi) >> 1;
                if (b.seg_off[mid] < e) lo = mid + 1; else hi = mid;
            }
            bad |= b.seg_off[lo] != e;
        }
    }
    if (bad) *verdict = ticket;
}

__global__ __launch_bounds__(kApplyThreads) void apply_object_kernel(const char *obj, size_t object_bytes, int32_t n_tensors,
                                                                     int32_t n_buckets, int32_t tp,
                                                                     const int32_t *local_numel, void *const *dst_ptrs,
                                                                     const u64 *verdict, u64 ticket) {
    uint32_t h[9];
    for (int i = 0; i < 9; ++i) h[i] = reinterpret_cast<const uint32_t *>(obj)[i];
    int64_t n;
    if (!object_header_ok(h, n_tensors, object_bytes, &n)) return;     // uniform: every thread leaves
    if (h[2] >= (uint32_t)n_buckets) return;
    if (*verdict == ticket) return;                                    // the validation pass found it out of order
    const BucketDev b = object_arrays(obj, n_tensors, n);
    if (b.seg_off[0] != 0 || b.seg_off[n_tensors] != n) return;
    apply_body(b, n_tensors, local_numel + (size_t)(h[2] / (uint32_t)tp) * n_tensors, dst_ptrs, (int)h[8], INT64_MAX);
}

// ---------------------------------------------------------------------------------------------
// dense copy of one shard: the same tiles as encode, moved instead of compared.
// ---------------------------------------------------------------------------------------------
template <int NEW_F32>
__global__ __launch_bounds__(kThreads) void dense_copy_kernel(CopyArgs a) {
    const int32_t tile = a.tile_begin + (int32_t)blockIdx.x;
    const Piece pc = load_piece(a.pieces + cload32(a.tile_piece + tile));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const void *new_base = reinterpret_cast<const void *>(cload64(a.new_ptrs + pc.tensor));
    uint16_t *dst = reinterpret_cast<uint16_t *>(cload64(a.dst_ptrs + pc.tensor));
    const uint32_t k_tile = (uint32_t)(tile - pc.first_tile) * (uint32_t)kTile;
    const uint32_t k_wave = k_tile + (uint32_t)wave * kWaveSpan;
    const bool fast = (pc.flags & kPieceVec) && k_tile + (uint32_t)kTile <= (uint32_t)pc.len &&
                      ((((uintptr_t)new_base) | ((uintptr_t)dst)) & 15u) == 0;
    if (fast) {
        uint4 nv[kIters];
        load_tile_fast<NEW_F32>(new_base, pc, k_wave, lane, nv);
#pragma unroll
        for (int j = 0; j < kIters; ++j)
            gstore16(dst + dst_index(pc, k_wave + (uint32_t)(j * 64 + lane) * kVec, true), nv[j]);
    } else {
#pragma unroll 1
        for (int j = 0; j < kIters; ++j) {
            uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
            uint4 n = load_vec_general<NEW_F32>(new_base, pc, k);
#pragma unroll
            for (uint32_t i = 0; i < (uint32_t)kVec; ++i)
                if (k + i < (uint32_t)pc.len) dst[dst_index(pc, k + i, false)] = (uint16_t)pick16(n, i);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bandwidth probe: grid-stride 128-bit copy, or read-only with a checksum
// ---------------------------------------------------------------------------------------------
constexpr int kBwThreads = 256;

__global__ __launch_bounds__(256) void bw_copy_kernel(const uint4 *src, uint4 *dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * (kBwThreads * 4) + threadIdx.x;
    const size_t step = (size_t)gridDim.x * (kBwThreads * 4);
    for (; i < n16; i += step) {
        uint4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            size_t at = i + (size_t)j * kBwThreads;
            v[j] = at < n16 ? src[at] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            size_t at = i + (size_t)j * kBwThreads;
            if (at < n16) dst[at] = v[j];
        }
    }
}

// (non-temporal loads, eight in flight per lane: 7.1 TB/s; ordinary loads, four in flight: 6.1 - 6.2)
__global__ __launch_bounds__(256) void bw_read_kernel(const uint4 *src, size_t n16, u64 *sink) {
    size_t i = (size_t)blockIdx.x * (kBwThreads * 8) + threadIdx.x;
    const size_t step = (size_t)gridDim.x * (kBwThreads * 8);
    uint32_t acc = 0;
    for (; i < n16; i += step) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            size_t at = i + (size_t)j * kBwThreads;
            v[j] = at < n16 ? gload16_stream(src + at) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    // The data-dependent test keeps the loads alive; it is true for about one lane in 2^32, so
    // the probe is not slowed down by atomics on one address.
    if (acc == 0x9E3779B9u) atomicAdd(sink, 1ull);
}

// Mixed probe: the traffic of an encode launch without any of its work.  Reads two streams in
// 16 KB chunks (non-temporal, like encode) and writes w16 16-byte vectors per chunk, contiguous
// across chunks, to a third.  TIMED = 0: every chunk's output is written at once.  TIMED = 1: it is
// held back (nothing is stored anywhere: the probe only remembers which chunks are due) and written
// in the windows of time of the encode kernel's timed tile order, or when 64 chunks are due.
template <int TIMED>
__global__ __launch_bounds__(256) void bw_mix_kernel(const uint4 *a, const uint4 *b, uint4 *dst, size_t n_chunks,
                                                     uint32_t w16, u64 *sink) {
    uint4 acc = make_uint4(0, 0, 0, 0);
    size_t due_from = blockIdx.x;                      // the oldest chunk whose output has not been written
    uint32_t n_due = 0;
    auto write_chunk = [&](size_t c) {
        for (uint32_t k = threadIdx.x; k < w16; k += kBwThreads) {
            u32x4 w = {acc.x, acc.y, acc.z, acc.w};
            __builtin_nontemporal_store(w, reinterpret_cast<global_u32x4 *>(reinterpret_cast<uintptr_t>(dst + c * (size_t)w16 + k)));
        }
    };
    for (size_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        uint4 va[4], vb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            va[j] = gload16_stream(a + c * 1024 + j * kBwThreads + threadIdx.x);
            vb[j] = gload16_stream(b + c * 1024 + j * kBwThreads + threadIdx.x);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = xor4(acc, xor4(va[j], vb[j]));
        if (!TIMED) {
            write_chunk(c);
        } else {
            ++n_due;
            const uint32_t now = (uint32_t)__builtin_amdgcn_s_memrealtime();
            const bool open = (now & ((1u << ROSE_WRITE_PERIOD_LOG2) - 1u)) < (1u << ROSE_WRITE_OPEN_LOG2);
            if (open || n_due >= 64u) {
                for (; n_due > 0; --n_due, due_from += gridDim.x) write_chunk(due_from);
            }
        }
    }
    if (TIMED)
        for (; n_due > 0; --n_due, due_from += gridDim.x) write_chunk(due_from);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) atomicAdd(sink, 1ull);
}

// Line probe: the memory traffic of an apply launch without its work.  A wave takes 128 consecutive
// lines of 64 bytes, 16 per round (4 lanes per line); the lines whose hash is below the threshold are
// loaded (all loads first, non-temporal like apply's), changed and stored back.
__device__ __forceinline__ uint32_t line_hash(size_t i) {
    uint32_t x = (uint32_t)i * 0x9E3779B1u ^ (uint32_t)((uint64_t)i >> 32);
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
__global__ __launch_bounds__(256) void bw_lines_kernel(uint4 *dst, size_t n_lines, uint32_t threshold) {
    const int lane = threadIdx.x & 63;
    const size_t base = ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 128;
    uint4 v[8];
    bool on[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const size_t line = base + (size_t)(r * 16 + lane / 4);
        on[r] = line < n_lines && line_hash(line) < threshold;
        v[r] = make_uint4(0, 0, 0, 0);
        if (on[r]) v[r] = gload16_stream(dst + line * 4 + (lane & 3));
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (on[r]) {
            const size_t line = base + (size_t)(r * 16 + lane / 4);
            u32x4 w = {v[r].x + 1u, v[r].y, v[r].z, v[r].w};
            __builtin_nontemporal_store(w, reinterpret_cast<global_u32x4 *>(reinterpret_cast<uintptr_t>(dst + line * 4 + (lane & 3))));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
// workgroups per CU the encode grid may use (bounded by what fits at once)
#ifndef ROSE_WGS_PER_CU
#define ROSE_WGS_PER_CU 8
#endif

// the encode kernel variant for (fp32 master input, sender refresh, arithmetic payload)
typedef void (*EncodeKernel)(EncodeArgs);
static EncodeKernel encode_variant(int new_is_f32, int refresh, int arith) {
    static const EncodeKernel table[8] = {encode_kernel<0, 0, 0>, encode_kernel<1, 0, 0>, encode_kernel<0, 1, 0>,
                                          encode_kernel<1, 1, 0>, encode_kernel<0, 0, 1>, encode_kernel<1, 0, 1>,
                                          encode_kernel<0, 1, 1>, encode_kernel<1, 1, 1>};
    return table[(new_is_f32 ? 1 : 0) + (refresh ? 2 : 0) + (arith ? 4 : 0)];
}

// Number of workgroups of each encode kernel variant that fit on the current device at once.
int encode_resident_all(int resident[8]) {
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int)e;
    for (int v = 0; v < 8; ++v) {
        int per_cu = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, encode_variant(v & 1, v & 2, v & 4), kThreads, 0);
        if (e != hipSuccess) return (int)e;
        if (per_cu < 1 || cus < 1) return (int)hipErrorInvalidValue;
        if (per_cu > ROSE_WGS_PER_CU) per_cu = ROSE_WGS_PER_CU;
        resident[v] = cus * per_cu;
    }
    return 0;
}

// Built-in scratch for callers that cannot allocate (rose_delta_encode_static).  In host code the
// array's name only stands for the symbol: its address on a device comes from hipGetSymbolAddress
// with that device current, each device has its own copy, and only that pointer is ever handed to
// a kernel.
static __device__ __align__(256) unsigned long long scratch[ROSE_STATIC_SCRATCH_BYTES / sizeof(unsigned long long)];
constexpr int kMaxDevices = 64;
int static_scratch(void **ptr, size_t *bytes) {
    static std::mutex mu;
    static void *per_device[kMaxDevices] = {nullptr};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return (int)hipErrorInvalidValue;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    *bytes = sizeof(scratch);
    return 0;
}

#ifndef ROSE_SERVER_WGS
#define ROSE_SERVER_WGS 16          // workgroups of the grid that serve prefixes (kWaves servers each)
#endif

int launch_encode(const EncodeArgs &args, int new_is_f32, const RefreshArgs *refresh, int arith, int resident,
                  int worker_cap, int order, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    EncodeArgs a = args;
    a.adjacent = order == ROSE_TILE_ORDER_SPREAD ? 0 : 1;
    a.timed = order == ROSE_TILE_ORDER_TIMED ? 1 : 0;
    a.batch = a.timed ? kBatchTimed : kBatch;
    if (resident < 1) return (int)hipErrorInvalidValue;
    // servers: one wave per block at most, ROSE_SERVER_WGS workgroups at most, and never more than
    // a quarter of what is resident.  They are the first workgroups of the grid, so they are
    // resident before any worker waits for them.
    int server_wgs = (a.n_blocks + kWaves - 1) / kWaves;
    if (server_wgs > ROSE_SERVER_WGS) server_wgs = ROSE_SERVER_WGS;
    if (server_wgs > resident / 4) server_wgs = resident / 4;
    if (server_wgs < 1) server_wgs = 1;
    int workers = resident - server_wgs;
    if (workers > a.n_tiles) workers = a.n_tiles;
    // the caller's cap: fewer workers than the device holds (never fewer than the progress
    // argument below needs)
    if (worker_cap > kBlock && worker_cap < workers) workers = worker_cap;
    // Progress with dynamic tickets: see the comment at struct Walk.  A worker that waits holds no
    // unpublished tile in the block it waits for or in an earlier one; what it waits for can still
    // need tickets of a partly handed-out group to be taken, by a worker that holds none of that
    // group's kBlock tickets.  Hence: more workers than tickets in a group.
    if (workers < 1) return (int)hipErrorInvalidValue;
    if (workers < a.n_tiles && workers <= kBlock) return (int)hipErrorInvalidValue;   // device holds too few workgroups
    a.n_server_wgs = server_wgs;
    a.n_servers = server_wgs * kWaves;
    a.n_tickets = ((a.n_blocks + a.batch - 1) / a.batch) * kBlock;
    // header, tile words and block words are one array
    const int64_t n_words = (int64_t)(kWsHeaderBytes / sizeof(u64)) + a.n_tiles + a.n_blocks;
    int reset_blocks = (int)((n_words + 1023) / 1024);
    if (reset_blocks > 2048) reset_blocks = 2048;
    hipLaunchKernelGGL(reset_kernel, dim3(reset_blocks), dim3(256), 0, st, reinterpret_cast<u64 *>(a.abort_flag), n_words);
    const dim3 grid(workers + server_wgs), block(kThreads);
    hipLaunchKernelGGL(encode_variant(new_is_f32, refresh ? 1 : 0, arith), grid, block, 0, st, a);
    if (refresh) {
        if (refresh->n > 0)
            hipLaunchKernelGGL(refresh_replicated_kernel, dim3(8, refresh->n > 1024 ? 1024 : refresh->n), dim3(256), 0, st,
                               refresh->list, refresh->numel, refresh->n, const_cast<void *const *>(a.old_ptrs),
                               a.new_ptrs, new_is_f32);
    }
    hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(64), 0, st, a);
    return (int)hipGetLastError();
}

int launch_apply(const BucketDev &b, int32_t n_tensors, const int32_t *local_numel, void *const *dst_ptrs,
                 int arith, int64_t shard_elems, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t chunks = (b.capacity + kApplyThreads - 1) / kApplyThreads;
    int blocks = chunks < 1 ? 1 : (chunks > ROSE_APPLY_BLOCKS ? ROSE_APPLY_BLOCKS : (int)chunks);
    hipLaunchKernelGGL(apply_kernel, dim3(blocks), dim3(kApplyThreads), 0, st, b, n_tensors, local_numel, dst_ptrs, arith,
                       shard_elems);
    return (int)hipGetLastError();
}

int launch_pack(const BucketDev &b, int32_t shard, int32_t n_tensors, int64_t first, int64_t n, int32_t payload,
                void *object, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t want = (n + 1023) / 1024;
    int blocks = want < 1 ? 1 : (want > 256 * 16 ? 256 * 16 : (int)want);
    hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, st, b, shard, n_tensors, first, n, payload, static_cast<char *>(object));
    return (int)hipGetLastError();
}

int launch_apply_object(const void *object, size_t object_bytes, int32_t n_tensors, int32_t n_buckets, int32_t tp,
                        const int32_t *local_numel, void *const *dst_ptrs, unsigned long long *verdict,
                        unsigned long long ticket, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t chunks = ((int64_t)(object_bytes / 6) + kApplyThreads - 1) / kApplyThreads;
    int blocks = chunks < 1 ? 1 : (chunks > ROSE_APPLY_BLOCKS ? ROSE_APPLY_BLOCKS : (int)chunks);
    const int vblocks = blocks > 4096 ? 4096 : blocks;
    hipLaunchKernelGGL(object_clear_kernel, dim3(1), dim3(1), 0, st, verdict);
    hipLaunchKernelGGL(object_validate_kernel, dim3(vblocks), dim3(256), 0, st, static_cast<const char *>(object),
                       object_bytes, n_tensors, n_buckets, verdict, ticket);
    hipLaunchKernelGGL(apply_object_kernel, dim3(blocks), dim3(kApplyThreads), 0, st, static_cast<const char *>(object),
                       object_bytes, n_tensors, n_buckets, tp, local_numel, dst_ptrs, verdict, ticket);
    return (int)hipGetLastError();
}

size_t object_bytes_for(int32_t n_tensors, int64_t n) { return object_size(n_tensors, n); }
bool object_header_valid(const uint32_t *h, int32_t n_tensors, size_t object_bytes, int64_t *n) {
    return object_header_ok(h, n_tensors, object_bytes, n);
}

int launch_dense_copy(const CopyArgs &a, int new_is_f32, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.n_tiles <= 0) return 0;
    if (new_is_f32)
        hipLaunchKernelGGL(dense_copy_kernel<1>, dim3(a.n_tiles), dim3(kThreads), 0, st, a);
    else
        hipLaunchKernelGGL(dense_copy_kernel<0>, dim3(a.n_tiles), dim3(kThreads), 0, st, a);
    return (int)hipGetLastError();
}

int launch_bw_probe(const void *src, void *dst, size_t bytes, uint64_t *sink, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    size_t n16 = bytes / 16;
    if (n16 == 0) return 0;
    size_t want = (n16 + kBwThreads * 4 - 1) / (kBwThreads * 4);
    int blocks = want > 256 * 32 ? 256 * 32 : (int)want;
    if (dst)
        hipLaunchKernelGGL(bw_copy_kernel, dim3(blocks), dim3(kBwThreads), 0, st,
                           static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    else
        hipLaunchKernelGGL(bw_read_kernel, dim3(blocks), dim3(kBwThreads), 0, st,
                           static_cast<const uint4 *>(src), n16, reinterpret_cast<u64 *>(sink));
    return (int)hipGetLastError();
}

int launch_bw_probe_lines(void *dst, size_t n_lines, uint32_t threshold, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_lines == 0) return 0;
    const size_t blocks = (n_lines + 511) / 512;
    if (blocks > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(bw_lines_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<uint4 *>(dst), n_lines, threshold);
    return (int)hipGetLastError();
}

int launch_bw_probe_mixed(const void *a, const void *b, void *dst, size_t n_chunks, uint32_t w16, int timed,
                          uint64_t *sink, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_chunks == 0) return 0;
    int blocks = n_chunks > 256 * 32 ? 256 * 32 : (int)n_chunks;
    if (timed)
        hipLaunchKernelGGL(bw_mix_kernel<1>, dim3(blocks), dim3(kBwThreads), 0, st, static_cast<const uint4 *>(a),
                           static_cast<const uint4 *>(b), static_cast<uint4 *>(dst), n_chunks, w16,
                           reinterpret_cast<u64 *>(sink));
    else
        hipLaunchKernelGGL(bw_mix_kernel<0>, dim3(blocks), dim3(kBwThreads), 0, st, static_cast<const uint4 *>(a),
                           static_cast<const uint4 *>(b), static_cast<uint4 *>(dst), n_chunks, w16,
                           reinterpret_cast<u64 *>(sink));
    return (int)hipGetLastError();
}

}  // namespace rose

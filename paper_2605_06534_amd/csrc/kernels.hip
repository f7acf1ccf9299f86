// HIP kernels for gfx950 (wave64): diff + mask + count + scan + shard-aware bucket write
// (Sec. 4.2 "Sparsity-aware Weight Transfer", App. F D2S), scatter-apply (App. F S2D), the dense
// shard copy (Sec. 4.2 "Shard-aware Weight Transfer") and a bandwidth probe.
//
// Everything here is bound by HBM traffic; there is no contraction, so no MFMA.  The encode
// kernel reads each weight once with 128-bit loads and writes only the changed entries.
#include <hip/hip_runtime.h>

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

// 8-bit mask of the 16-bit lanes of x that are non-zero (bit e = element e, little endian)
__device__ __forceinline__ uint32_t nz16_mask(uint4 x) {
    uint32_t m = 0;
    m |= ((x.x & 0xFFFFu) != 0) ? 1u : 0u;
    m |= ((x.x >> 16) != 0) ? 2u : 0u;
    m |= ((x.y & 0xFFFFu) != 0) ? 4u : 0u;
    m |= ((x.y >> 16) != 0) ? 8u : 0u;
    m |= ((x.z & 0xFFFFu) != 0) ? 16u : 0u;
    m |= ((x.z >> 16) != 0) ? 32u : 0u;
    m |= ((x.w & 0xFFFFu) != 0) ? 64u : 0u;
    m |= ((x.w >> 16) != 0) ? 128u : 0u;
    return m;
}

// element e (0..7) of a vector of eight 16-bit patterns
__device__ __forceinline__ uint32_t pick16(uint4 v, uint32_t e) {
    uint32_t a = (e & 4u) ? ((e & 2u) ? v.w : v.z) : ((e & 2u) ? v.y : v.x);
    return (e & 1u) ? (a >> 16) : (a & 0xFFFFu);
}

// inclusive prefix sum over the 64 lanes of a wave
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
    const int lane = __lane_id();
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        uint32_t y = __shfl_up(x, s, 64);
        if (lane >= s) x += y;
    }
    return x;
}

// source element of piece-relative local index k
__device__ __forceinline__ int64_t src_index(const Piece &pc, uint32_t k, bool use_magic) {
    if (pc.flags & kPieceStrided) {
        uint32_t q = use_magic ? (__umulhi(k, pc.magic) >> pc.shift) : (k / (uint32_t)pc.run);
        return pc.src_off + (int64_t)q * pc.stride + (k - q * (uint32_t)pc.run);
    }
    return pc.src_off + k;
}

// Load the eight 16-bit patterns at local indices k .. k+7 of a piece (fewer at the ragged end:
// missing ones read as zero) from a bf16 tensor.
__device__ __forceinline__ uint4 load8_bf16(const uint16_t *base, const Piece &pc, uint32_t k, bool vec) {
    uint4 r = make_uint4(0, 0, 0, 0);
    if (k >= (uint32_t)pc.len) return r;
    uint32_t valid = (uint32_t)pc.len - k;
    if (vec && valid >= (uint32_t)kVec) {
        return *reinterpret_cast<const uint4 *>(base + src_index(pc, k, true));
    }
    uint32_t e[kVec];
#pragma unroll
    for (int i = 0; i < kVec; ++i) e[i] = ((uint32_t)i < valid) ? base[src_index(pc, k + i, false)] : 0u;
    r.x = e[0] | (e[1] << 16);
    r.y = e[2] | (e[3] << 16);
    r.z = e[4] | (e[5] << 16);
    r.w = e[6] | (e[7] << 16);
    return r;
}

// Same for an fp32 master tensor: the eight values are rounded to bf16 on the way in.
__device__ __forceinline__ uint4 load8_f32(const uint32_t *base, const Piece &pc, uint32_t k, bool vec) {
    uint4 r = make_uint4(0, 0, 0, 0);
    if (k >= (uint32_t)pc.len) return r;
    uint32_t valid = (uint32_t)pc.len - k;
    if (vec && valid >= (uint32_t)kVec) {
        const uint4 *p = reinterpret_cast<const uint4 *>(base + src_index(pc, k, true));
        uint4 a = p[0], b = p[1];
        r.x = pack_rne(a.x, a.y);
        r.y = pack_rne(a.z, a.w);
        r.z = pack_rne(b.x, b.y);
        r.w = pack_rne(b.z, b.w);
        return r;
    }
    uint32_t e[kVec];
#pragma unroll
    for (int i = 0; i < kVec; ++i)
        e[i] = ((uint32_t)i < valid) ? rne_bf16(base[src_index(pc, k + i, false)]) : 0u;
    r.x = e[0] | (e[1] << 16);
    r.y = e[2] | (e[3] << 16);
    r.z = e[4] | (e[5] << 16);
    r.w = e[6] | (e[7] << 16);
    return r;
}

// ---------------------------------------------------------------------------------------------
// look-back descriptors: one 64-bit word per tile, status in the top two bits, count below.
// Published and polled with relaxed device-scope atomics: the word carries everything a
// successor needs, so no other memory has to be ordered with it.
// ---------------------------------------------------------------------------------------------
constexpr u64 kStatusShift = 62;
constexpr u64 kStatusAggregate = 1;   // value = this tile's own count
constexpr u64 kStatusPrefix = 2;      // value = count of this tile and all before it in the chain
constexpr u64 kValueMask = (1ull << kStatusShift) - 1;

__device__ __forceinline__ void desc_store(u64 *p, u64 v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 desc_load(u64 *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void reset_kernel(u64 *desc, unsigned int *ticket, int32_t n_tiles) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) *ticket = 0;
    for (; i < n_tiles; i += (int64_t)gridDim.x * blockDim.x) desc[i] = 0;
}

// ---------------------------------------------------------------------------------------------
// encode: one workgroup per tile, tiles handed out by a ticket so that a tile's predecessors in
// its chain have always started.
//   1. issue all 128-bit loads of the tile (old and new), 2. XOR -> 8-bit change mask per vector,
//   3. wave prefix sums of the popcounts, wave totals through LDS, 4. wave 0 publishes the tile
//   count and looks back along the shard's chain for its exclusive prefix, 5. every lane writes its
//   changed (local index, new pattern) pairs at bucket position prefix + rank.
// Inside a tile wave w covers a contiguous quarter and walks it in kIters steps of 512 elements,
// so the order (wave, step, lane, element) is ascending local index.
// ---------------------------------------------------------------------------------------------
template <int NEW_F32>
__global__ __launch_bounds__(kThreads) void encode_kernel(EncodeArgs a) {
    __shared__ int32_t s_tile;
    __shared__ uint32_t s_wave_total[kWaves];
    __shared__ u64 s_excl;

    if (threadIdx.x == 0)
        s_tile = (int32_t)__hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int32_t tile = __builtin_amdgcn_readfirstlane(s_tile);   // uniform: keep it scalar
    if (tile >= a.n_tiles) return;

    const Piece pc = a.pieces[a.tile_piece[tile]];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint16_t *old_base = static_cast<const uint16_t *>(a.old_ptrs[pc.tensor]);
    const void *new_base = a.new_ptrs[pc.tensor];
    const bool vec = (pc.flags & kPieceVec) &&
                     ((((uintptr_t)old_base) | ((uintptr_t)new_base)) & 15u) == 0;
    const uint32_t k_wave = (uint32_t)(tile - pc.first_tile) * (uint32_t)kTile + (uint32_t)wave * kWaveSpan;

    uint4 nv[kIters];
    uint32_t mask[kIters];
    {
        uint4 ov[kIters];
#pragma unroll
        for (int j = 0; j < kIters; ++j) {
            uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
            ov[j] = load8_bf16(old_base, pc, k, vec);
            nv[j] = NEW_F32 ? load8_f32(static_cast<const uint32_t *>(new_base), pc, k, vec)
                            : load8_bf16(static_cast<const uint16_t *>(new_base), pc, k, vec);
        }
#pragma unroll
        for (int j = 0; j < kIters; ++j) {
            uint4 x = make_uint4(ov[j].x ^ nv[j].x, ov[j].y ^ nv[j].y, ov[j].z ^ nv[j].z, ov[j].w ^ nv[j].w);
            mask[j] = nz16_mask(x);
        }
    }

    // exclusive rank of each of this lane's vectors inside the wave's span
    uint32_t rank[kIters];
    uint32_t wave_total = 0;
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        uint32_t c = __popc(mask[j]);
        uint32_t inc = wave_incl_scan(c);
        rank[j] = wave_total + inc - c;
        wave_total += __shfl(inc, 63, 64);
    }
    if (lane == 0) s_wave_total[wave] = wave_total;
    __syncthreads();

    uint32_t wave_excl = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        uint32_t c = s_wave_total[w];
        if (w < wave) wave_excl += c;
        tile_total += c;
    }

    const int32_t chain_first = a.chain_first[pc.shard];
    if (wave == 0) {
        u64 excl = 0;
        if (tile > chain_first) {
            if (lane == 0) desc_store(a.desc + tile, (kStatusAggregate << kStatusShift) | tile_total);
            int32_t look = tile - 1;      // lane 0 reads the nearest predecessor
            for (;;) {
                int32_t at = look - lane;
                u64 v = (at >= chain_first) ? desc_load(a.desc + at) : (kStatusPrefix << kStatusShift);
                u64 st = v >> kStatusShift;
                u64 empty = __ballot(st == 0);
                u64 pref = __ballot(st == kStatusPrefix);
                // lanes nearer than the first prefix must all be published
                int first_pref = pref ? __ffsll((long long)pref) - 1 : 64;
                u64 need = (first_pref >= 63) ? ~0ull : ((1ull << (first_pref + 1)) - 1);
                if (empty & need) {
                    __builtin_amdgcn_s_sleep(1);
                    continue;
                }
                u64 contrib = (lane <= first_pref) ? (v & kValueMask) : 0;
                // wave sum of 64-bit values
#pragma unroll
                for (int s = 32; s >= 1; s >>= 1) contrib += __shfl_xor(contrib, s, 64);
                excl += contrib;
                if (pref) break;
                look -= 64;
            }
        }
        if (lane == 0) {
            desc_store(a.desc + tile, (kStatusPrefix << kStatusShift) | (excl + tile_total));
            s_excl = excl;
        }
    }
    __syncthreads();
    const u64 tile_excl = s_excl;

    const BucketDev b = a.bucket[pc.shard];
    if (threadIdx.x == 0) {
        if ((pc.flags & kPieceFirst) && tile == pc.first_tile) b.seg_off[pc.tensor] = (int64_t)tile_excl;
        if (tile == a.chain_first[pc.shard + 1] - 1) b.seg_off[a.n_tensors] = (int64_t)(tile_excl + tile_total);
    }

    const u64 wave_base = tile_excl + wave_excl;
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        uint32_t m = mask[j];
        u64 pos = wave_base + rank[j];
        uint32_t local0 = (uint32_t)pc.local_base + k_wave + (uint32_t)(j * 64 + lane) * kVec;
        while (m) {
            uint32_t e = __ffs(m) - 1;
            m &= m - 1;
            if (pos < (u64)b.capacity) {
                b.idx[pos] = (int32_t)(local0 + e);
                b.val[pos] = (uint16_t)pick16(nv[j], e);
            }
            ++pos;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// apply: persistent grid over chunks of a bucket's entries; entries are in ascending local index
// inside a segment, so neighbouring lanes store into the same or neighbouring lines.
// ---------------------------------------------------------------------------------------------
constexpr int kApplyPerLane = 4;
constexpr int kApplyChunk = kThreads * kApplyPerLane;

__global__ __launch_bounds__(kThreads) void apply_kernel(BucketDev b, int32_t n_tensors, void *const *dst_ptrs) {
    int64_t total = b.seg_off[n_tensors];
    if (total > b.capacity) total = b.capacity;
    for (int64_t e0 = (int64_t)blockIdx.x * kApplyChunk; e0 < total; e0 += (int64_t)gridDim.x * kApplyChunk) {
        // tensor of the chunk's first entry: largest t with seg_off[t] <= e0 (uniform search)
        int32_t lo = 0, hi = n_tensors;
        while (hi - lo > 1) {
            int32_t mid = (lo + hi) >> 1;
            if (b.seg_off[mid] <= e0) lo = mid; else hi = mid;
        }
        int64_t e = e0 + (int64_t)threadIdx.x * kApplyPerLane;
        if (e >= total) continue;
        int32_t t = lo;
        int64_t seg_end = b.seg_off[t + 1];
        int32_t ix[kApplyPerLane];
        uint32_t vv[kApplyPerLane];
        if (e + kApplyPerLane <= total) {
            int4 i4 = *reinterpret_cast<const int4 *>(b.idx + e);
            uint2 v2 = *reinterpret_cast<const uint2 *>(b.val + e);
            ix[0] = i4.x; ix[1] = i4.y; ix[2] = i4.z; ix[3] = i4.w;
            vv[0] = v2.x & 0xFFFFu; vv[1] = v2.x >> 16; vv[2] = v2.y & 0xFFFFu; vv[3] = v2.y >> 16;
        } else {
#pragma unroll
            for (int i = 0; i < kApplyPerLane; ++i) {
                bool ok = e + i < total;
                ix[i] = ok ? b.idx[e + i] : 0;
                vv[i] = ok ? b.val[e + i] : 0u;
            }
        }
        uint16_t *dst = nullptr;
        bool have = false;
#pragma unroll
        for (int i = 0; i < kApplyPerLane; ++i) {
            int64_t ei = e + i;
            if (ei >= total) break;
            while (ei >= seg_end) {
                ++t;
                seg_end = b.seg_off[t + 1];
                have = false;
            }
            if (!have) {
                dst = static_cast<uint16_t *>(dst_ptrs[t]);
                have = true;
            }
            dst[ix[i]] = (uint16_t)vv[i];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// dense copy of one shard: the same tiles as encode, moved instead of compared.
// ---------------------------------------------------------------------------------------------
template <int NEW_F32>
__global__ __launch_bounds__(kThreads) void dense_copy_kernel(CopyArgs a) {
    const int32_t tile = a.tile_begin + (int32_t)blockIdx.x;
    const Piece pc = a.pieces[a.tile_piece[tile]];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const void *new_base = a.new_ptrs[pc.tensor];
    uint16_t *dst = static_cast<uint16_t *>(a.dst_ptrs[pc.tensor]);
    const bool vec = (pc.flags & kPieceVec) && ((((uintptr_t)new_base) | ((uintptr_t)dst)) & 15u) == 0;
    const uint32_t k_wave = (uint32_t)(tile - pc.first_tile) * (uint32_t)kTile + (uint32_t)wave * kWaveSpan;
    uint4 nv[kIters];
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
        nv[j] = NEW_F32 ? load8_f32(static_cast<const uint32_t *>(new_base), pc, k, vec)
                        : load8_bf16(static_cast<const uint16_t *>(new_base), pc, k, vec);
    }
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
        uint32_t k = k_wave + (uint32_t)(j * 64 + lane) * kVec;
        if (k >= (uint32_t)pc.len) continue;
        uint32_t valid = (uint32_t)pc.len - k;
        uint16_t *out = dst + (uint32_t)pc.local_base + k;
        if (vec && valid >= (uint32_t)kVec) {
            *reinterpret_cast<uint4 *>(out) = nv[j];
        } else {
            for (uint32_t i = 0; i < valid && i < (uint32_t)kVec; ++i) out[i] = (uint16_t)pick16(nv[j], i);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bandwidth probe: grid-stride 128-bit copy, or read-only with a checksum
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void bw_copy_kernel(const uint4 *src, uint4 *dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * (kThreads * 4) + threadIdx.x;
    const size_t step = (size_t)gridDim.x * (kThreads * 4);
    for (; i < n16; i += step) {
        uint4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            size_t at = i + (size_t)j * kThreads;
            v[j] = at < n16 ? src[at] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            size_t at = i + (size_t)j * kThreads;
            if (at < n16) dst[at] = v[j];
        }
    }
}

__global__ __launch_bounds__(kThreads) void bw_read_kernel(const uint4 *src, size_t n16, u64 *sink) {
    size_t i = (size_t)blockIdx.x * (kThreads * 4) + threadIdx.x;
    const size_t step = (size_t)gridDim.x * (kThreads * 4);
    uint32_t acc = 0;
    for (; i < n16; i += step) {
        uint4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            size_t at = i + (size_t)j * kThreads;
            v[j] = at < n16 ? src[at] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) acc += v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    // the checksum keeps the loads alive: one atomic per wave
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(sink, (u64)acc);
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
int launch_encode(const EncodeArgs &a, int new_is_f32, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    int reset_blocks = (a.n_tiles + 1023) / 1024;
    if (reset_blocks < 1) reset_blocks = 1;
    if (reset_blocks > 2048) reset_blocks = 2048;
    hipLaunchKernelGGL(reset_kernel, dim3(reset_blocks), dim3(256), 0, st, a.desc, a.ticket, a.n_tiles);
    if (new_is_f32)
        hipLaunchKernelGGL(encode_kernel<1>, dim3(a.n_tiles), dim3(kThreads), 0, st, a);
    else
        hipLaunchKernelGGL(encode_kernel<0>, dim3(a.n_tiles), dim3(kThreads), 0, st, a);
    return (int)hipGetLastError();
}

int launch_apply(const BucketDev &b, int32_t n_tensors, void *const *dst_ptrs, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t chunks = (b.capacity + kApplyChunk - 1) / kApplyChunk;
    int blocks = chunks < 1 ? 1 : (chunks > 256 * 16 ? 256 * 16 : (int)chunks);
    hipLaunchKernelGGL(apply_kernel, dim3(blocks), dim3(kThreads), 0, st, b, n_tensors, dst_ptrs);
    return (int)hipGetLastError();
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
    size_t want = (n16 + kThreads * 4 - 1) / (kThreads * 4);
    int blocks = want > 256 * 32 ? 256 * 32 : (int)want;
    if (dst)
        hipLaunchKernelGGL(bw_copy_kernel, dim3(blocks), dim3(kThreads), 0, st,
                           static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
    else
        hipLaunchKernelGGL(bw_read_kernel, dim3(blocks), dim3(kThreads), 0, st,
                           static_cast<const uint4 *>(src), n16, reinterpret_cast<u64 *>(sink));
    return (int)hipGetLastError();
}

}  // namespace rose

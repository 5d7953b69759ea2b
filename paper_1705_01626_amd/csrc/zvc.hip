// Zero-value compression (ZVC) for AMD gfx950 (wave64): kernels and C ABI.
//
// The operation is the one of the paper's section 5.1 ("Zero-value
// compression"): one 32-bit presence mask per 32 consecutive elements plus the
// non-zero elements packed in order.  The paper builds it as a fixed-function
// pipeline beside the memory controllers (section 5.2); this file is a GPU
// kernel design instead:
//
//   * one pass over the input.  A workgroup owns a tile of 16 KB of input; each
//     lane loads 16 bytes at a time (fully coalesced), tests its elements for a
//     non-zero bit pattern with integer compares, and the wave derives packed
//     positions from ballots + mbcnt (the GPU form of the paper's per-sector
//     prefix sum over mask bits);
//   * the offset of a tile's first kept element in the packed stream -- the
//     paper's "offset to the next mask", a serial chain in hardware -- is a
//     device-wide exclusive scan of per-tile counts done in the same pass with
//     decoupled look-back over one 64-bit state word per tile;
//   * kept elements are staged in LDS at their tile-local rank and leave as
//     aligned 16-byte stores; masks leave as one contiguous run per wave.
//
// Decompression mirrors it: per-tile popcount of the masks, the same scan, the
// tile's packed run staged into LDS with aligned 16-byte loads, and every lane
// rebuilds 16 bytes of output from "bit ? next stored element : zero".

#include "zvc.h"

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>

namespace {

// ------------------------------------------------------------------ geometry
constexpr int kThreads = 256;                 // 4 waves of 64 lanes
constexpr int kWaveSize = 64;
constexpr int kWaves = kThreads / kWaveSize;
constexpr int kLoads = 4;                     // 16-byte loads per lane per tile
constexpr int kTileBytes = kThreads * 16 * kLoads;  // 16 KB of input per tile
constexpr size_t kHeaderBytes = 256;          // workspace header, then tile states

template <int W>
struct Geometry {
    static constexpr int kElemsPerLane = 16 / W;                 // per 16-byte load: 4 | 8
    static constexpr int kLanesPerGroup = 32 / kElemsPerLane;    // lanes covering one mask: 8 | 4
    static constexpr int kGroupsPerLoad = kWaveSize / kLanesPerGroup;  // masks per wave-load: 8 | 16
    static constexpr int kTileElems = kTileBytes / W;            // 4096 | 8192
    static constexpr int kTileGroups = kTileElems / 32;          // 128 | 256
    static_assert(kLoads <= kLanesPerGroup, "mask hand-off needs one lane per load");
    static_assert(kTileGroups <= kThreads, "one thread per mask in the decoder");
};

// Workspace header.  Lives at the start of the caller's workspace.
struct WsHeader {
    unsigned int ticket;           // next tile to hand out
    unsigned int done;             // finished workgroups (count-only pass)
    unsigned long long nnz;        // accumulator of the count-only pass
    unsigned long long size_word;  // compressed size for zvc_offload's read-back
    unsigned long long pad[29];
};
static_assert(sizeof(WsHeader) == kHeaderBytes, "header is 256 bytes");

// Tile state word: status in the two top bits, a count in the rest.
constexpr unsigned long long kStatusShift = 62;
constexpr unsigned long long kStatusInvalid = 0;    // nothing published yet
constexpr unsigned long long kStatusAggregate = 1;  // value = this tile's own count
constexpr unsigned long long kStatusPrefix = 2;     // value = count of this and all earlier tiles
constexpr unsigned long long kValueMask = (1ull << kStatusShift) - 1;

__host__ __device__ inline size_t div_up(size_t a, size_t b) { return a / b + (a % b != 0); }

inline size_t tiles_for(size_t n, int w) {
    const size_t tile_elems = static_cast<size_t>(kTileBytes / w);
    return div_up(n, tile_elems);
}

// ------------------------------------------------------------ device helpers
__device__ inline unsigned long long load_state(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store_state(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Number of set bits of `ballot` in lanes below the calling lane.
__device__ inline unsigned lanes_below(unsigned long long ballot) {
    return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(ballot >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(ballot), 0u));
}

__device__ inline unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) v += __shfl_xor(v, off);
    return v;
}

// 16 bytes of input for the lane whose first element is e0.  Elements at or
// past n read as zero.  The 16-byte access is used only when the base pointer
// is 16-byte aligned (ALIGNED) and the whole chunk is inside the tensor.
template <int W, bool ALIGNED>
__device__ inline uint4 load_chunk(const unsigned char* __restrict__ in, size_t e0, size_t n) {
    constexpr int E = 16 / W;
    if (ALIGNED && e0 + E <= n) return *reinterpret_cast<const uint4*>(in + e0 * W);
    unsigned d[4] = {0u, 0u, 0u, 0u};
    if (W == 4) {
        const unsigned* p = reinterpret_cast<const unsigned*>(in);
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (e0 + c < n) d[c] = p[e0 + c];
    } else {
        const unsigned short* p = reinterpret_cast<const unsigned short*>(in);
#pragma unroll
        for (int c = 0; c < 8; ++c)
            if (e0 + c < n) d[c >> 1] |= static_cast<unsigned>(p[e0 + c]) << (16 * (c & 1));
    }
    return make_uint4(d[0], d[1], d[2], d[3]);
}

// Presence bits of the lane's 16 bytes: bit c set <=> element c is non-zero as
// an integer (section 5.2: words compared to zero form the mask bits).
template <int W>
__device__ inline unsigned presence_bits(const uint4& v) {
    if (W == 4) {
        return (v.x != 0u ? 1u : 0u) | (v.y != 0u ? 2u : 0u) | (v.z != 0u ? 4u : 0u) |
               (v.w != 0u ? 8u : 0u);
    }
    const unsigned d[4] = {v.x, v.y, v.z, v.w};
    unsigned bits = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        bits |= ((d[k] & 0xFFFFu) != 0u ? 1u : 0u) << (2 * k);
        bits |= ((d[k] >> 16) != 0u ? 1u : 0u) << (2 * k + 1);
    }
    return bits;
}

template <int W>
__device__ inline unsigned element_of(const uint4& v, int c) {
    const unsigned d[4] = {v.x, v.y, v.z, v.w};
    if (W == 4) return d[c];
    return (d[c >> 1] >> (16 * (c & 1))) & 0xFFFFu;
}

// Decoupled look-back (single-pass scan): sum of the counts of all tiles
// before `tile`.  Called by one whole wave.  Lane k inspects predecessor
// tile-1-k (then 64 further back per round); a predecessor with a prefix ends
// the walk, aggregates in front of it are added.  Every predecessor holds a
// ticket taken before ours, so it is resident and will publish.
__device__ inline unsigned long long look_back(const unsigned long long* states, unsigned tile,
                                               int lane) {
    unsigned long long exclusive = 0;
    long long base = static_cast<long long>(tile) - 1;
    while (true) {
        const long long idx = base - lane;
        // tiles before the first behave as a published prefix of zero
        unsigned long long st = (kStatusPrefix << kStatusShift);
        if (idx >= 0) st = load_state(states + idx);
        const unsigned long long status = st >> kStatusShift;
        const unsigned long long invalid = __ballot(status == kStatusInvalid);
        const unsigned long long prefix = __ballot(status == kStatusPrefix);
        // lanes up to and including the nearest prefix must all be published
        const int first_prefix = prefix ? __ffsll(static_cast<long long>(prefix)) - 1 : kWaveSize;
        const unsigned long long needed =
            first_prefix >= kWaveSize - 1 ? ~0ull : ((2ull << first_prefix) - 1ull);
        if (invalid & needed) {
            __builtin_amdgcn_s_sleep(1);
            continue;
        }
        const unsigned long long take = (lane <= first_prefix) ? (st & kValueMask) : 0ull;
        exclusive += wave_sum(take);
        if (first_prefix < kWaveSize) break;
        base -= kWaveSize;
    }
    return exclusive;
}

// Publishes this tile's count, finds the count of all earlier tiles, publishes
// the inclusive prefix.  Called by wave 0 of the workgroup.
__device__ inline unsigned long long tile_exclusive_prefix(unsigned long long* states,
                                                           unsigned tile, unsigned tile_total,
                                                           int lane) {
    unsigned long long exclusive = 0;
    if (tile == 0) {
        if (lane == 0) store_state(states, (kStatusPrefix << kStatusShift) | tile_total);
    } else {
        if (lane == 0)
            store_state(states + tile, (kStatusAggregate << kStatusShift) | tile_total);
        exclusive = look_back(states, tile, lane);
        if (lane == 0)
            store_state(states + tile, (kStatusPrefix << kStatusShift) | (exclusive + tile_total));
    }
    return exclusive;
}

// ------------------------------------------------------------------- kernels

// Puts the workspace header and the first `slots` tile states back to zero.
__global__ void reset_kernel(unsigned long long* ws_words, size_t header_words, size_t slots) {
    const size_t total = header_words + slots;
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < total;
         i += static_cast<size_t>(gridDim.x) * blockDim.x)
        ws_words[i] = 0ull;
}

__global__ void write_word_kernel(unsigned long long* dst, unsigned long long v) { *dst = v; }

// Section 5.1 encoder.  One workgroup per tile, tiles handed out by ticket.
template <int W, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void compress_kernel(
    const unsigned char* __restrict__ in, size_t n, unsigned* __restrict__ masks,
    unsigned char* __restrict__ values, WsHeader* hdr, unsigned long long* states,
    unsigned long long* d_bytes, unsigned num_tiles, size_t num_groups) {
    using G = Geometry<W>;
    constexpr int E = G::kElemsPerLane;
    constexpr int LPG = G::kLanesPerGroup;

    __shared__ __align__(16) unsigned char s_stage[kTileBytes + 16];
    __shared__ unsigned s_tile;
    __shared__ unsigned s_wave_total[kWaves];
    __shared__ unsigned long long s_prefix;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid / kWaveSize;

    if (tid == 0) s_tile = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const unsigned tile = s_tile;
    const size_t tile_elem0 = static_cast<size_t>(tile) * G::kTileElems;

    // ---- load, zero test, in-wave ranks, masks
    uint4 data[kLoads];
    unsigned bits[kLoads];
    unsigned rank[kLoads];   // wave-local packed position of the lane's first kept element
    unsigned running = 0;    // wave-uniform: kept elements of earlier loads of this wave
    unsigned my_mask = 0;
    const int lane_in_group = lane % LPG;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const size_t e0 =
            tile_elem0 + (static_cast<size_t>(wave * kLoads + j) * kWaveSize + lane) * E;
        data[j] = load_chunk<W, ALIGNED>(in, e0, n);
        bits[j] = presence_bits<W>(data[j]);
        unsigned below = 0, load_total = 0;
#pragma unroll
        for (int c = 0; c < E; ++c) {
            const unsigned long long b = __ballot((bits[j] >> c) & 1u);
            below += lanes_below(b);
            load_total += static_cast<unsigned>(__popcll(b));
        }
        rank[j] = running + below;
        running += load_total;
        // the group's mask: OR of the lanes' bit fields, each at its position
        unsigned m = bits[j] << (E * lane_in_group);
#pragma unroll
        for (int off = 1; off < LPG; off <<= 1) m |= __shfl_xor(m, off);
        if (lane_in_group == j) my_mask = m;
    }
    if (lane_in_group < kLoads) {
        const size_t g = static_cast<size_t>(tile) * G::kTileGroups +
                         static_cast<size_t>(wave * kLoads + lane_in_group) * G::kGroupsPerLoad +
                         lane / LPG;
        if (g < num_groups) masks[g] = my_mask;
    }

    // ---- tile-level scan of the wave totals
    if (lane == 0) s_wave_total[wave] = running;
    __syncthreads();
    unsigned wave_offset = 0, tile_total = 0;
#pragma unroll
    for (int v = 0; v < kWaves; ++v) {
        const unsigned t = s_wave_total[v];
        if (v < wave) wave_offset += t;
        tile_total += t;
    }

    // ---- device-wide exclusive scan (decoupled look-back), wave 0
    if (wave == 0) {
        const unsigned long long ex = tile_exclusive_prefix(states, tile, tile_total, lane);
        if (lane == 0) s_prefix = ex;
    }
    __syncthreads();
    const unsigned long long exclusive = s_prefix;

    // ---- stage kept elements in LDS.  LDS byte p corresponds to global byte
    //      (dst - shift) + p, so 16-byte chunks are aligned on both sides.
    unsigned char* dst = values + exclusive * W;
    const unsigned shift = static_cast<unsigned>(reinterpret_cast<uintptr_t>(dst) & 15u);
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        unsigned r = wave_offset + rank[j];
#pragma unroll
        for (int c = 0; c < E; ++c) {
            if ((bits[j] >> c) & 1u) {
                const unsigned v = element_of<W>(data[j], c);
                if (W == 4)
                    *reinterpret_cast<unsigned*>(s_stage + shift + r * 4u) = v;
                else
                    *reinterpret_cast<unsigned short*>(s_stage + shift + r * 2u) =
                        static_cast<unsigned short>(v);
                ++r;
            }
        }
    }
    __syncthreads();

    // ---- copy out: whole 16-byte chunks, ragged ends element by element
    const unsigned end = shift + tile_total * W;
    const unsigned chunks = (end + 15u) / 16u;
    unsigned char* gbase = dst - shift;
    for (unsigned q = tid; q < chunks; q += kThreads) {
        const unsigned lo = q * 16u, hi = lo + 16u;
        if (lo >= shift && hi <= end) {
            *reinterpret_cast<uint4*>(gbase + lo) = *reinterpret_cast<const uint4*>(s_stage + lo);
        } else {
            const unsigned a = lo > shift ? lo : shift;
            const unsigned b = hi < end ? hi : end;
            for (unsigned o = a; o < b; o += W) {
                if (W == 4)
                    *reinterpret_cast<unsigned*>(gbase + o) =
                        *reinterpret_cast<const unsigned*>(s_stage + o);
                else
                    *reinterpret_cast<unsigned short*>(gbase + o) =
                        *reinterpret_cast<const unsigned short*>(s_stage + o);
            }
        }
    }

    // ---- section 5.4: the compressed size, reported by the last tile
    if (tile == num_tiles - 1 && tid == 0)
        *d_bytes = 4ull * num_groups + static_cast<unsigned long long>(W) * (exclusive + tile_total);
}

// Section 5.2 decoder.  values_avail = number of stored elements that may be
// read; anything the masks ask for beyond it decodes as zero.
template <int W, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void decompress_kernel(
    const unsigned* __restrict__ masks, const unsigned char* __restrict__ values,
    unsigned long long values_avail, size_t n, unsigned char* __restrict__ out, WsHeader* hdr,
    unsigned long long* states, size_t num_groups) {
    using G = Geometry<W>;
    constexpr int E = G::kElemsPerLane;
    constexpr int LPG = G::kLanesPerGroup;

    __shared__ __align__(16) unsigned char s_stage[kTileBytes + 16];
    __shared__ unsigned s_mask[G::kTileGroups];
    __shared__ unsigned s_group_offset[G::kTileGroups];
    __shared__ unsigned s_tile;
    __shared__ unsigned s_wave_total[kWaves];
    __shared__ unsigned long long s_prefix;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid / kWaveSize;

    if (tid == 0) s_tile = atomicAdd(&hdr->ticket, 1u);
    __syncthreads();
    const unsigned tile = s_tile;
    const size_t tile_elem0 = static_cast<size_t>(tile) * G::kTileElems;

    // ---- one thread per mask: popcount, exclusive scan over the tile
    unsigned m = 0;
    const size_t g = static_cast<size_t>(tile) * G::kTileGroups + tid;
    if (tid < G::kTileGroups && g < num_groups) {
        m = masks[g];
        const unsigned tail = static_cast<unsigned>(n % 32);
        if (g == num_groups - 1 && tail != 0) m &= (1u << tail) - 1u;  // bits past n never count
    }
    const unsigned cnt = __popc(m);
    unsigned incl = cnt;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
        const unsigned t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == kWaveSize - 1) s_wave_total[wave] = incl;
    __syncthreads();
    unsigned wave_offset = 0, tile_total = 0;
#pragma unroll
    for (int v = 0; v < kWaves; ++v) {
        const unsigned t = s_wave_total[v];
        if (v < wave) wave_offset += t;
        tile_total += t;
    }
    if (tid < G::kTileGroups) {
        s_mask[tid] = m;
        s_group_offset[tid] = wave_offset + incl - cnt;
    }

    if (wave == 0) {
        const unsigned long long ex = tile_exclusive_prefix(states, tile, tile_total, lane);
        if (lane == 0) s_prefix = ex;
    }
    __syncthreads();
    const unsigned long long exclusive = s_prefix;

    // ---- stage the tile's stored elements in LDS (aligned 16-byte chunks,
    //      ragged ends element by element, nothing past values_avail)
    const unsigned char* src = values + exclusive * W;
    const unsigned shift = static_cast<unsigned>(reinterpret_cast<uintptr_t>(src) & 15u);
    unsigned long long readable = values_avail > exclusive ? values_avail - exclusive : 0ull;
    if (readable > tile_total) readable = tile_total;
    const unsigned end = shift + tile_total * W;
    const unsigned end_valid = shift + static_cast<unsigned>(readable) * W;
    const unsigned chunks = (end + 15u) / 16u;
    const unsigned char* gbase = src - shift;
    for (unsigned q = tid; q < chunks; q += kThreads) {
        const unsigned lo = q * 16u, hi = lo + 16u;
        if (lo >= shift && hi <= end_valid) {
            *reinterpret_cast<uint4*>(s_stage + lo) = *reinterpret_cast<const uint4*>(gbase + lo);
        } else {
            const unsigned a = lo > shift ? lo : shift;
            const unsigned b = hi < end ? hi : end;
            for (unsigned o = a; o < b; o += W) {
                if (W == 4)
                    *reinterpret_cast<unsigned*>(s_stage + o) =
                        o < end_valid ? *reinterpret_cast<const unsigned*>(gbase + o) : 0u;
                else
                    *reinterpret_cast<unsigned short*>(s_stage + o) =
                        o < end_valid ? *reinterpret_cast<const unsigned short*>(gbase + o)
                                      : static_cast<unsigned short>(0);
            }
        }
    }
    __syncthreads();

    // ---- expand: each lane rebuilds 16 bytes of output per load
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int seg = wave * kLoads + j;
        const size_t e0 = tile_elem0 + (static_cast<size_t>(seg) * kWaveSize + lane) * E;
        if (e0 >= n) continue;
        const int gi = seg * G::kGroupsPerLoad + lane / LPG;
        const unsigned bit0 = static_cast<unsigned>(lane % LPG) * E;
        const unsigned gm = s_mask[gi];
        unsigned r = s_group_offset[gi] + __popc(gm & ((1u << bit0) - 1u));
        const unsigned field = gm >> bit0;
        unsigned d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int c = 0; c < E; ++c) {
            if ((field >> c) & 1u) {
                if (W == 4) {
                    d[c] = *reinterpret_cast<const unsigned*>(s_stage + shift + r * 4u);
                } else {
                    const unsigned v =
                        *reinterpret_cast<const unsigned short*>(s_stage + shift + r * 2u);
                    d[c >> 1] |= v << (16 * (c & 1));
                }
                ++r;
            }
        }
        if (ALIGNED && e0 + E <= n) {
            *reinterpret_cast<uint4*>(out + e0 * W) = make_uint4(d[0], d[1], d[2], d[3]);
        } else {
#pragma unroll
            for (int c = 0; c < E; ++c) {
                if (e0 + c < n) {
                    if (W == 4)
                        reinterpret_cast<unsigned*>(out)[e0 + c] = d[c];
                    else
                        reinterpret_cast<unsigned short*>(out)[e0 + c] =
                            static_cast<unsigned short>((d[c >> 1] >> (16 * (c & 1))) & 0xFFFFu);
                }
            }
        }
    }
}

// Count-only pass (section 5.4's size, without producing the stream).
template <int W, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void count_kernel(const unsigned char* __restrict__ in,
                                                         size_t n, WsHeader* hdr,
                                                         unsigned long long* d_bytes,
                                                         size_t num_groups) {
    constexpr int E = 16 / W;
    __shared__ unsigned long long s_wave[kWaves];
    const size_t chunks = div_up(n, E);
    unsigned long long count = 0;
    for (size_t q = blockIdx.x * static_cast<size_t>(kThreads) + threadIdx.x; q < chunks;
         q += static_cast<size_t>(gridDim.x) * kThreads) {
        const uint4 v = load_chunk<W, ALIGNED>(in, q * E, n);
        count += __popc(presence_bits<W>(v));
    }
    count = wave_sum(count);
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x / kWaveSize;
    if (lane == 0) s_wave[wave] = count;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long block_total = 0;
        for (int v = 0; v < kWaves; ++v) block_total += s_wave[v];
        atomicAdd(&hdr->nnz, block_total);
        __threadfence();
        const unsigned finished = atomicAdd(&hdr->done, 1u);
        if (finished == gridDim.x - 1) {
            const unsigned long long total = atomicAdd(&hdr->nnz, 0ull);
            *d_bytes = 4ull * num_groups + static_cast<unsigned long long>(W) * total;
        }
    }
}

// -------------------------------------------------------------- host helpers
inline bool aligned_to(const void* p, size_t a) {
    return reinterpret_cast<uintptr_t>(p) % a == 0;
}

inline bool ranges_overlap(const void* a, size_t an, const void* b, size_t bn) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return an != 0 && bn != 0 && a0 < b0 + bn && b0 < a0 + an;
}

inline zvc_status hip_ok(hipError_t e) { return e == hipSuccess ? ZVC_OK : ZVC_E_HIP; }

zvc_status launch_reset(void* d_ws, size_t slots, hipStream_t stream) {
    const size_t words = kHeaderBytes / 8 + slots;
    const unsigned blocks = static_cast<unsigned>(div_up(words, 256) < 1024 ? div_up(words, 256) : 1024);
    hipLaunchKernelGGL(reset_kernel, dim3(blocks), dim3(256), 0, stream,
                       static_cast<unsigned long long*>(d_ws), kHeaderBytes / 8, slots);
    return hip_ok(hipGetLastError());
}

zvc_status check_workspace(const void* d_ws, size_t ws, size_t n, int w) {
    if (d_ws == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_ws, 256)) return ZVC_E_ALIGN;
    if (ws < zvc_workspace_bytes(n, w)) return ZVC_E_WORKSPACE;
    return ZVC_OK;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

const char* zvc_status_string(zvc_status st) {
    switch (st) {
        case ZVC_OK: return "ZVC_OK";
        case ZVC_E_ARG: return "ZVC_E_ARG: invalid argument";
        case ZVC_E_WIDTH: return "ZVC_E_WIDTH: element width must be 2 or 4 bytes";
        case ZVC_E_CAPACITY: return "ZVC_E_CAPACITY: output buffer below the worst-case size";
        case ZVC_E_WORKSPACE: return "ZVC_E_WORKSPACE: workspace too small";
        case ZVC_E_ALIGN: return "ZVC_E_ALIGN: pointer alignment";
        case ZVC_E_HIP: return "ZVC_E_HIP: a HIP runtime call failed";
        case ZVC_E_CORRUPT: return "ZVC_E_CORRUPT: compressed stream inconsistent with its size";
    }
    return "ZVC: unknown status";
}

size_t zvc_mask_bytes(size_t n) { return 4 * div_up(n, 32); }

size_t zvc_max_compressed_bytes(size_t n, int w) {
    if (w != 2 && w != 4) return 0;
    return zvc_mask_bytes(n) + static_cast<size_t>(w) * n;
}

size_t zvc_workspace_bytes(size_t n, int w) {
    if (w != 2 && w != 4) return 0;
    return kHeaderBytes + 8 * tiles_for(n, w);
}

zvc_status zvc_check_stream(const void* h_comp, uint64_t bytes, size_t n, int w) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (h_comp == nullptr && bytes != 0) return ZVC_E_ARG;
    const size_t groups = div_up(n, 32);
    if (bytes < 4 * groups) return ZVC_E_CORRUPT;
    const unsigned char* p = static_cast<const unsigned char*>(h_comp);
    uint64_t kept = 0;
    for (size_t g = 0; g < groups; ++g) {
        uint32_t m;
        std::memcpy(&m, p + 4 * g, 4);
        if (g == groups - 1 && n % 32 != 0 && (m >> (n % 32)) != 0) return ZVC_E_CORRUPT;
        kept += static_cast<uint64_t>(__builtin_popcount(m));
    }
    return bytes == 4 * groups + static_cast<uint64_t>(w) * kept ? ZVC_OK : ZVC_E_CORRUPT;
}

zvc_status zvc_workspace_init(void* d_ws, size_t ws, hipStream_t stream) {
    if (d_ws == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_ws, 256)) return ZVC_E_ALIGN;
    if (ws < kHeaderBytes) return ZVC_E_WORKSPACE;
    return launch_reset(d_ws, (ws - kHeaderBytes) / 8, stream);
}

zvc_status zvc_compressed_size(const void* d_in, size_t n, int w, uint64_t* d_bytes, void* d_ws,
                               size_t ws, hipStream_t stream) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (d_bytes == nullptr || (d_in == nullptr && n != 0)) return ZVC_E_ARG;
    if (!aligned_to(d_in, static_cast<size_t>(w)) || !aligned_to(d_bytes, 8)) return ZVC_E_ALIGN;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    unsigned long long* out = reinterpret_cast<unsigned long long*>(d_bytes);
    if (n == 0) {
        hipLaunchKernelGGL(write_word_kernel, dim3(1), dim3(1), 0, stream, out, 0ull);
        return hip_ok(hipGetLastError());
    }
    if (zvc_status st = launch_reset(d_ws, 0, stream)) return st;
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);
    const unsigned char* in = static_cast<const unsigned char*>(d_in);
    const size_t groups = div_up(n, 32);
    const size_t chunks = div_up(n * static_cast<size_t>(w), 16);
    size_t blocks = div_up(chunks, static_cast<size_t>(kThreads) * 8);
    if (blocks > 4096) blocks = 4096;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    const bool al = aligned_to(d_in, 16);
    if (w == 4) {
        if (al) hipLaunchKernelGGL((count_kernel<4, true>), grid, block, 0, stream, in, n, hdr, out, groups);
        else hipLaunchKernelGGL((count_kernel<4, false>), grid, block, 0, stream, in, n, hdr, out, groups);
    } else {
        if (al) hipLaunchKernelGGL((count_kernel<2, true>), grid, block, 0, stream, in, n, hdr, out, groups);
        else hipLaunchKernelGGL((count_kernel<2, false>), grid, block, 0, stream, in, n, hdr, out, groups);
    }
    return hip_ok(hipGetLastError());
}

zvc_status zvc_compress(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                        uint64_t* d_bytes, void* d_ws, size_t ws, hipStream_t stream) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (d_bytes == nullptr || ((d_in == nullptr || d_out == nullptr) && n != 0)) return ZVC_E_ARG;
    if (!aligned_to(d_in, static_cast<size_t>(w)) || !aligned_to(d_out, 4) ||
        !aligned_to(d_bytes, 8))
        return ZVC_E_ALIGN;
    if (out_cap < zvc_max_compressed_bytes(n, w)) return ZVC_E_CAPACITY;
    if (ranges_overlap(d_in, n * static_cast<size_t>(w), d_out, zvc_max_compressed_bytes(n, w)))
        return ZVC_E_ARG;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    unsigned long long* out_bytes = reinterpret_cast<unsigned long long*>(d_bytes);
    if (n == 0) {
        hipLaunchKernelGGL(write_word_kernel, dim3(1), dim3(1), 0, stream, out_bytes, 0ull);
        return hip_ok(hipGetLastError());
    }
    const size_t tiles = tiles_for(n, w);
    if (tiles > 0x7FFFFFFFull) return ZVC_E_ARG;
    if (zvc_status st = launch_reset(d_ws, tiles, stream)) return st;
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);
    unsigned long long* states =
        reinterpret_cast<unsigned long long*>(static_cast<unsigned char*>(d_ws) + kHeaderBytes);
    const size_t groups = div_up(n, 32);
    const unsigned char* in = static_cast<const unsigned char*>(d_in);
    unsigned* masks = static_cast<unsigned*>(d_out);
    unsigned char* values = static_cast<unsigned char*>(d_out) + 4 * groups;
    const dim3 grid(static_cast<unsigned>(tiles)), block(kThreads);
    const unsigned nt = static_cast<unsigned>(tiles);
    const bool al = aligned_to(d_in, 16);
    if (w == 4) {
        if (al) hipLaunchKernelGGL((compress_kernel<4, true>), grid, block, 0, stream, in, n, masks, values, hdr, states, out_bytes, nt, groups);
        else hipLaunchKernelGGL((compress_kernel<4, false>), grid, block, 0, stream, in, n, masks, values, hdr, states, out_bytes, nt, groups);
    } else {
        if (al) hipLaunchKernelGGL((compress_kernel<2, true>), grid, block, 0, stream, in, n, masks, values, hdr, states, out_bytes, nt, groups);
        else hipLaunchKernelGGL((compress_kernel<2, false>), grid, block, 0, stream, in, n, masks, values, hdr, states, out_bytes, nt, groups);
    }
    return hip_ok(hipGetLastError());
}

zvc_status zvc_decompress(const void* d_comp, size_t comp_bytes, size_t n, int w, void* d_out,
                          void* d_ws, size_t ws, hipStream_t stream) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if ((d_comp == nullptr || d_out == nullptr) && n != 0) return ZVC_E_ARG;
    if (!aligned_to(d_out, static_cast<size_t>(w)) || !aligned_to(d_comp, 4)) return ZVC_E_ALIGN;
    if (comp_bytes < zvc_mask_bytes(n)) return ZVC_E_CAPACITY;
    if (ranges_overlap(d_comp, comp_bytes, d_out, n * static_cast<size_t>(w))) return ZVC_E_ARG;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    if (n == 0) return ZVC_OK;
    const size_t tiles = tiles_for(n, w);
    if (tiles > 0x7FFFFFFFull) return ZVC_E_ARG;
    if (zvc_status st = launch_reset(d_ws, tiles, stream)) return st;
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);
    unsigned long long* states =
        reinterpret_cast<unsigned long long*>(static_cast<unsigned char*>(d_ws) + kHeaderBytes);
    const size_t groups = div_up(n, 32);
    const unsigned* masks = static_cast<const unsigned*>(d_comp);
    const unsigned char* values = static_cast<const unsigned char*>(d_comp) + 4 * groups;
    const unsigned long long avail = (comp_bytes - 4 * groups) / static_cast<size_t>(w);
    unsigned char* out = static_cast<unsigned char*>(d_out);
    const dim3 grid(static_cast<unsigned>(tiles)), block(kThreads);
    const bool al = aligned_to(d_out, 16);
    if (w == 4) {
        if (al) hipLaunchKernelGGL((decompress_kernel<4, true>), grid, block, 0, stream, masks, values, avail, n, out, hdr, states, groups);
        else hipLaunchKernelGGL((decompress_kernel<4, false>), grid, block, 0, stream, masks, values, avail, n, out, hdr, states, groups);
    } else {
        if (al) hipLaunchKernelGGL((decompress_kernel<2, true>), grid, block, 0, stream, masks, values, avail, n, out, hdr, states, groups);
        else hipLaunchKernelGGL((decompress_kernel<2, false>), grid, block, 0, stream, masks, values, avail, n, out, hdr, states, groups);
    }
    return hip_ok(hipGetLastError());
}

zvc_status zvc_offload(const void* d_in, size_t n, int w, void* d_stage, size_t stage_cap,
                       void* h_pinned, size_t h_cap, uint64_t* h_bytes, void* d_ws, size_t ws,
                       hipStream_t compute, hipStream_t copy) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (h_bytes == nullptr || (h_pinned == nullptr && n != 0)) return ZVC_E_ARG;
    if (h_cap < zvc_max_compressed_bytes(n, w)) return ZVC_E_CAPACITY;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);
    uint64_t* d_size = reinterpret_cast<uint64_t*>(&hdr->size_word);
    // the size word sits in the header; zvc_compress's reset runs before the
    // kernel that writes it, so it survives until the next call on this workspace
    if (zvc_status st = zvc_compress(d_in, n, w, d_stage, stage_cap, d_size, d_ws, ws, compute))
        return st;
    if (hipMemcpyAsync(h_bytes, d_size, 8, hipMemcpyDeviceToHost, compute) != hipSuccess)
        return ZVC_E_HIP;
    hipEvent_t ev;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return ZVC_E_HIP;
    zvc_status st = ZVC_OK;
    if (hipEventRecord(ev, compute) != hipSuccess || hipEventSynchronize(ev) != hipSuccess) {
        st = ZVC_E_HIP;
    } else if (*h_bytes > h_cap) {
        st = ZVC_E_CAPACITY;
    } else if (*h_bytes != 0) {
        if (copy != compute && hipStreamWaitEvent(copy, ev, 0) != hipSuccess) st = ZVC_E_HIP;
        if (st == ZVC_OK && hipMemcpyAsync(h_pinned, d_stage, *h_bytes, hipMemcpyDeviceToHost,
                                           copy) != hipSuccess)
            st = ZVC_E_HIP;
    }
    (void)hipEventDestroy(ev);
    return st;
}

zvc_status zvc_prefetch(const void* h_pinned, uint64_t bytes, size_t n, int w, void* d_stage,
                        size_t stage_cap, void* d_out, void* d_ws, size_t ws, hipStream_t copy,
                        hipStream_t compute) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if ((h_pinned == nullptr || d_stage == nullptr) && bytes != 0) return ZVC_E_ARG;
    if (bytes < zvc_mask_bytes(n) || bytes > zvc_max_compressed_bytes(n, w)) return ZVC_E_CORRUPT;
    if (stage_cap < bytes) return ZVC_E_CAPACITY;
    if ((d_out == nullptr && n != 0)) return ZVC_E_ARG;
    if (!aligned_to(d_out, static_cast<size_t>(w)) || !aligned_to(d_stage, 4)) return ZVC_E_ALIGN;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    if (n == 0) return ZVC_OK;
    if (hipMemcpyAsync(d_stage, h_pinned, bytes, hipMemcpyHostToDevice, copy) != hipSuccess)
        return ZVC_E_HIP;
    if (copy != compute) {
        hipEvent_t ev;
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return ZVC_E_HIP;
        const bool ok = hipEventRecord(ev, copy) == hipSuccess &&
                        hipStreamWaitEvent(compute, ev, 0) == hipSuccess;
        (void)hipEventDestroy(ev);
        if (!ok) return ZVC_E_HIP;
    }
    return zvc_decompress(d_stage, bytes, n, w, d_out, d_ws, ws, compute);
}

}  // extern "C"

// Zero-value compression (ZVC) for AMD gfx950 (wave64): kernels and C ABI.
//
// The operation is the one of the paper's section 5.1: one 32-bit presence mask
// per 32 consecutive elements plus the non-zero elements packed in order.  The
// paper builds it as a fixed-function pipeline beside the memory controllers
// (section 5.2); this file is a GPU kernel design instead:
//
//   * one pass over the input.  A workgroup owns a tile of 16 to 64 KB of input;
//     each lane loads one dword at a time (a wave instruction covers 256
//     contiguous bytes), so the 64-lane ballot of the zero test is two finished
//     masks and its mbcnt the packed position of the lane's element (the GPU
//     form of the paper's per-sector prefix sum over mask bits);
//   * the offset of a tile's first kept element in the packed stream -- where
//     the next mask goes, a serial chain in the paper's hardware -- is a
//     device-wide exclusive scan of per-tile counts done in the same pass:
//     every tile publishes its count, every 256th tile a running prefix, and a
//     tile adds the counts between the nearest published prefix and itself;
//   * kept elements are staged by each wave in an LDS queue in packed order and
//     leave as whole 128-byte lines; masks leave as one contiguous run per wave.
//
// Decompression: where a span's stored elements start depends on the masks
// alone, so a small pre-pass over the masks computes it for every 32 masks; the
// expand kernel's waves then work independently: each stages its packed run in
// LDS with aligned 16-byte loads and rebuilds 16 bytes of output per lane from
// "bit ? next stored element : zero".  Small tensors decode in one launch that
// uses the encoder's scan instead of the pre-pass.
//
// Three variants share these kernels: a fused ReLU + ZVC encoder
// (pre-activations in, stream of ReLU(x) out), an encoder that writes into a
// buffer below the worst case and never past it (section 9: streams kept in GPU
// memory), and the paper's own stream order (a group's mask, then its non-zeros)
// in independently decodable windows of 1 KB to 64 KB with an offset table.

#include "zvc.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <tuple>
#include <utility>
#include <cstdint>
#include <cstring>
#include <type_traits>

namespace {

// ------------------------------------------------------------------ geometry
constexpr int kThreads = 256;                 // 4 waves of 64 lanes
constexpr int kWaveSize = 64;
constexpr int kWaves = kThreads / kWaveSize;
constexpr int kFinishLanes = 64;              // arrival counters, one 128-byte line each
constexpr size_t kHeaderBytes = 256 + 128 * (kFinishLanes + 1);  // header, then the scan state
constexpr int kMinLoads = 4;                  // smallest tile: 16 KB (sizes the workspace)
constexpr int kStageLoads = 4;                // 16-byte loads a wave stages through LDS at a time
constexpr int kBlockTiles = 256;              // one running prefix is published per 256 tiles
constexpr int kMaxDevices = 64;                // GPUs per process that per-GPU host state is kept for
constexpr unsigned kDefaultPatience = 2000;   // polls a waiting tile makes before it computes a missing count itself
constexpr int kPollSleep = 8;                 // s_sleep units (64 clocks each) between polls

// The decoder's tile: LOADS 16-byte stores per lane, 256 * 16 * LOADS bytes of output.
template <int W, int LOADS>
struct Geometry {
    static constexpr int kElemsPerLane = 16 / W;                 // per 16-byte store: 4 | 8
    static constexpr int kLanesPerGroup = 32 / kElemsPerLane;    // lanes covering one mask: 8 | 4
    static constexpr int kGroupsPerLoad = kWaveSize / kLanesPerGroup;  // masks per KB of output: 8 | 16
    // per-wave LDS staging buffer: kStageLoads wave-loads plus alignment slack
    static constexpr int kStageSteps = LOADS / kStageLoads;
    // (16 bytes so the slice can mirror the destination's alignment)
    static constexpr int kWaveStageBytes = kStageLoads * kWaveSize * 16 + 16;
    static_assert(LOADS % kStageLoads == 0, "tile is staged in whole steps");
};

// The encoder's tile.  A wave reads its part of the tensor one dword per lane
// (a chunk: 256 bytes, 64 fp32 or 128 16-bit elements, 2 or 4 masks), CH chunks
// per wave, WV waves per tile (the workgroup): WV x CH / 4 KB.  With one
// element (or one pair) per lane a ballot of the zero test is two masks as they
// stand and its mbcnt is the packed position, so a chunk costs a handful of
// vector instructions.  Streaming 4-byte accesses measure as fast as 16-byte
// ones on this memory system (each wave instruction still covers whole
// 128-byte lines).
constexpr int kChunkBytes = 4 * kWaveSize;
constexpr int kStepChunks = 8;                // chunks a wave stages between two flushes: 2 KB of input
template <int W, int CH, int WV>
struct EncoderGeometry {
    static constexpr int kChunkElems = kChunkBytes / W;          // 64 | 128
    static constexpr int kChunkGroups = kChunkElems / 32;        // masks per chunk: 2 | 4
    static constexpr int kWaveElems = CH * kChunkElems;
    static constexpr int kWaveGroups = CH * kChunkGroups;
    static constexpr int kTileBytes = WV * CH * kChunkBytes;
    static constexpr int kTileElems = WV * kWaveElems;
    static constexpr int kTileGroups = WV * kWaveGroups;
    static constexpr int kSteps = CH / kStepChunks;
    static constexpr int kMaskRegs = (kWaveGroups + kWaveSize - 1) / kWaveSize;
    static constexpr int kStepGroups = kStepChunks * kChunkGroups;
    // the most a step can add to the wave's queue (windowed stream: its masks too)
    static constexpr int kStepMaxBytes = kStepChunks * kChunkBytes + 4 * kStepGroups;
    // A wave's LDS queue.  What is in it when the tile learns where its run
    // begins has cost the tile no time; what does not fit waits for that moment.
    // Room for half the wave's input (a tensor that is at most half non-zero is
    // staged whole before the scan ends) plus a little, never less than a
    // carried-over partial line plus a step.  (More workgroups per CU with a
    // smaller queue measure the same or worse.)
    static constexpr int kQueueBytes =
        CH == 64 ? 8704 : (CH * kChunkBytes / 2 > kStepMaxBytes ? CH * kChunkBytes / 2 : kStepMaxBytes) + 256;
    static_assert(kQueueBytes >= 128 + kStepMaxBytes, "a step always fits behind a carried-over partial line");
    static_assert(CH % kStepChunks == 0, "a wave's chunks are staged in whole steps");
    static_assert(kTileElems < (1 << 24), "tile totals fit the arrival word");
};

// Workspace header.  Lives at the start of the caller's workspace.
struct WsHeader {
    unsigned long long patience_plus_one;   // 0: default; else polls before a waiting tile helps itself, plus one
    unsigned long long pad0;
    unsigned long long size_word;  // compressed size for zvc_offload's read-back
    unsigned long long helped;     // predecessor counts computed by a waiting tile since the workspace's init
    unsigned long long pad[28];
    // Arrival counters, shared by the encoder and the decoder's pre-pass (calls
    // on one workspace do not overlap).  Encoder: tile t counts itself finished
    // in finish[t % 64] once it has read all the scan state it needs; the last
    // tile waits until all have, then zeroes the scan state and these counters,
    // so the next call needs no reset kernel.  Pre-pass: the workgroup that
    // completes a counter bumps finish_top, the one that completes finish_top is
    // the last.  Count-only pass: the same, with `sum` collecting the counts.
    // One counter per 128-byte line keeps the atomics on one address (about
    // 11 ns each) far apart in time.
    struct alignas(128) Line {
        unsigned value;
        unsigned pad;
        unsigned long long sum;
    } finish[kFinishLanes], finish_top;
};
static_assert(sizeof(WsHeader) == kHeaderBytes, "header size");

// Scan state in the workspace, after the header:
//   counts[t]   : 32-bit word per tile, top bit = published, rest = the tile's
//                 own count of kept elements;
//   prefixes[b] : 64-bit word per block of kBlockTiles tiles, top bit = published,
//                 rest = kept elements in all tiles up to and including the block's last.
constexpr unsigned kCountValid = 0x80000000u;
constexpr unsigned long long kPrefixValid = 1ull << 63;

__host__ __device__ inline size_t div_up(size_t a, size_t b) { return a / b + (a % b != 0); }

inline size_t tiles_for(size_t n, int w, int loads) {
    const size_t tile_elems = static_cast<size_t>(kThreads * 16 * loads / w);
    return div_up(n, tile_elems);
}
inline size_t counts_bytes(size_t tiles) { return 4 * div_up(tiles, 64) * 64; }   // padded to 256 B
inline size_t prefixes_bytes(size_t tiles) { return 8 * div_up(tiles, kBlockTiles); }
inline size_t scan_state_bytes(size_t tiles) {
    return counts_bytes(tiles) + div_up(prefixes_bytes(tiles), 256) * 256;
}
// the decoder pre-pass arrays sit at the end of the workspace, clear of the
// encoder's scan state (which is kept zeroed between calls and must not be
// scribbled on)
inline size_t pad256(size_t b) { return div_up(b, 256) * 256; }
inline size_t decoder_area_bytes(size_t chunks) {   // chunk_prefix, chunk_total, unit_end
    return pad256(8 * chunks) + pad256(4 * chunks) + pad256(4 * 128 * chunks);
}

// ------------------------------------------------------------ device helpers
__device__ inline unsigned long long load64(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store64(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store32(unsigned* p, unsigned v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// acc + number of set bits of `ballot` in lanes below the calling lane.
__device__ inline unsigned lanes_below(unsigned long long ballot, unsigned acc) {
    return __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(ballot >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(ballot), acc));
}

__device__ inline unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) v += __shfl_xor(v, off);
    return v;
}

// A value that is the same in every lane, moved to scalar registers so that
// address arithmetic built on it stays scalar.
__device__ inline unsigned uniform(unsigned v) {
    return static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
}
__device__ inline unsigned long long uniform(unsigned long long v) {
    return (static_cast<unsigned long long>(uniform(static_cast<unsigned>(v >> 32))) << 32) |
           uniform(static_cast<unsigned>(v));
}

// Lane `src` (wave-uniform) of v.
__device__ inline unsigned lane_value(unsigned v, int src) {
    return static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(v), src));
}
__device__ inline unsigned long long lane_value(unsigned long long v, int src) {
    return (static_cast<unsigned long long>(lane_value(static_cast<unsigned>(v >> 32), src)) << 32) |
           lane_value(static_cast<unsigned>(v), src);
}

// Sum over the wave of one value per lane (each below 2^26), wave-uniform
// result.  DPP adds within each row of 16 lanes (pairs, quads, half-row mirror,
// row mirror), then the four row sums are read out and added on the scalar
// unit: a dozen instructions and no lane-index registers, which matters where
// the caller holds a tile's data in registers and every cycle of the scan is
// waited for by the tile's other waves.
__device__ inline unsigned wave_sum_small(unsigned v) {
    v += static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0xB1, 0xF, 0xF, true));
    v += static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x4E, 0xF, 0xF, true));
    v += static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x141, 0xF, 0xF, true));
    v += static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), 0x140, 0xF, 0xF, true));
    return lane_value(v, 0) + lane_value(v, 16) + lane_value(v, 32) + lane_value(v, 48);
}

// Streaming 16-byte accesses, for what a call touches exactly once: the
// uncompressed tensor (read by the encoder, written by the decoder) and the
// encoder's output.  The non-temporal hint keeps such data from displacing other
// data in the caches (a plain copy kernel gains about 10 % from it here).  The
// decoder's reads of the compressed stream are ordinary loads: the masks are
// read twice (pre-pass, then expand), and the value runs of neighbouring waves
// share cache lines; with the hint those re-reads went back to memory, which
// cost 10-25 % of the decoder's time at low density.
typedef unsigned int vec4u __attribute__((ext_vector_type(4)));
__device__ inline uint4 load16_stream(const void* p) {
    const vec4u v = __builtin_nontemporal_load(reinterpret_cast<const vec4u*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline void store16_stream(void* p, const uint4& d) {
    vec4u v;
    v.x = d.x; v.y = d.y; v.z = d.z; v.w = d.w;
    __builtin_nontemporal_store(v, reinterpret_cast<vec4u*>(p));
}

// LDS written by some lanes of a wave is read by other lanes of the same wave:
// order the accesses (LDS operations of one wave execute in order).
__device__ inline void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 16 bytes of input for the lane whose first element is e0.  Elements at or
// past n read as zero.  With a 16-byte aligned base (ALIGNED) a chunk that holds
// at least one element of the tensor is loaded whole: an aligned 16-byte chunk
// never straddles a page, so the access is as safe as the load of its first
// element, and the bytes past the tensor's end are cleared in registers.
template <int W, bool ALIGNED>
__device__ inline uint4 load_chunk(const unsigned char* __restrict__ in, size_t e0, size_t n) {
    constexpr int E = 16 / W;
    unsigned d[4] = {0u, 0u, 0u, 0u};
    if (ALIGNED) {
        if (e0 >= n) return make_uint4(0u, 0u, 0u, 0u);
        const uint4 v = load16_stream(in + e0 * W);
        if (e0 + E <= n) return v;
        const unsigned valid_bytes = static_cast<unsigned>(n - e0) * W;   // 1 .. 15
        const unsigned raw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned lo = 4u * k;
            d[k] = valid_bytes >= lo + 4u ? raw[k]
                 : valid_bytes > lo      ? raw[k] & ((1u << (8u * (valid_bytes - lo))) - 1u)
                                         : 0u;
        }
        return make_uint4(d[0], d[1], d[2], d[3]);
    }
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

// Which elements are kept.  Plain ZVC (RELU = false) keeps the elements that are
// non-zero as integers (section 5.2: words compared to zero form the mask
// bits).  The fused ReLU + ZVC encoder (RELU = true) reads pre-activation
// values (IEEE-style, sign in the top bit: fp32, fp16, bf16) and keeps those
// whose sign bit is clear and which are not +0, i.e. the non-zeros of ReLU(x);
// as signed integers those are exactly the words greater than zero.
template <int W, bool RELU>
__device__ inline bool element_kept(const uint4& v, int c) {
    const unsigned d[4] = {v.x, v.y, v.z, v.w};
    if (W == 4) return RELU ? static_cast<int>(d[c]) > 0 : d[c] != 0u;
    if (c & 1) return RELU ? static_cast<int>(d[c >> 1]) > 0xFFFF : d[c >> 1] > 0xFFFFu;
    const unsigned low = d[c >> 1] & 0xFFFFu;
    return RELU ? (low - 1u) < 0x7FFFu : low != 0u;
}

// Kept-element bits of the lane's 16 bytes: bit c set <=> element c is kept.
template <int W, bool RELU>
__device__ inline unsigned presence_bits(const uint4& v) {
    unsigned bits = 0;
#pragma unroll
    for (int c = 0; c < 16 / W; ++c) bits |= (element_kept<W, RELU>(v, c) ? 1u : 0u) << c;
    return bits;
}

// A dword of a wave's LDS queue at any offset that is a multiple of W (with
// 16-bit elements the queue need not sit at the destination's offset modulo 4).
template <int W>
__device__ inline unsigned queue_dword(const unsigned char* p) {
    if (W == 4) return *reinterpret_cast<const unsigned*>(p);
    return static_cast<unsigned>(*reinterpret_cast<const unsigned short*>(p)) |
           (static_cast<unsigned>(*reinterpret_cast<const unsigned short*>(p + 2)) << 16);
}

// Writes out what a wave has staged so far.  The wave's packed run goes through
// its LDS slice like through a queue: slice offset p holds the byte that belongs
// at global address gzero + p (gzero is wave-uniform and a multiple of W; nothing
// before offset lo is ever dereferenced), and [lo, end) is staged but not yet
// written.  Every store instruction covers one 256-byte aligned block of the
// destination, a dword per lane, so whole 128-byte lines leave as whole lines
// wherever the run begins (partial-line writes cost the memory system about as
// much as whole lines).  Unless `last`, the bytes after the run's last line
// boundary stay behind: they move to the front of the slice, where the next
// step continues them, so a wave writes two partial lines per tile, not two per
// step.  Updates gzero, lo and end.
template <int W>
__device__ inline void wave_flush(unsigned char*& gzero, unsigned char* stage, unsigned& lo,
                                  unsigned& end, bool last, int lane) {
    const uintptr_t g = reinterpret_cast<uintptr_t>(gzero);
    // slice offsets of the bytes to write: [first, tail)
    int first = static_cast<int>(lo);
    const int keep_back = last ? 0 : static_cast<int>((g + end) & 127u);   // bytes after the last line boundary
    const int tail = static_cast<int>(end) - keep_back;
    if (tail <= first) {       // no line completed yet (or, with `last`, nothing staged)
        if (last) lo = end;
        return;
    }
    int stop = tail;
    if (W == 2) {
        // odd halves at either end, so that what is left is whole dwords of the destination
        if ((g + first) & 2u) {
            if (lane == 0)
                *reinterpret_cast<unsigned short*>(gzero + first) =
                    *reinterpret_cast<const unsigned short*>(stage + first);
            first += 2;
        }
        if (((g + stop) & 2u) && stop > first) {
            if (lane == 0)
                *reinterpret_cast<unsigned short*>(gzero + (stop - 2)) =
                    *reinterpret_cast<const unsigned short*>(stage + (stop - 2));
            stop -= 2;
        }
    }
    // one 256-byte aligned block of the destination per store instruction, four blocks at a
    // time so that the LDS reads of a round are under way together
    constexpr int kRound = 4;
    for (int block = first - static_cast<int>((g + first) & 255u); block < stop; block += 256 * kRound) {
        unsigned v[kRound];
#pragma unroll
        for (int j = 0; j < kRound; ++j) {
            const int at = block + 256 * j + 4 * lane;
            v[j] = 0u;
            if (at >= first && at < stop) v[j] = queue_dword<W>(stage + at);
        }
#pragma unroll
        for (int j = 0; j < kRound; ++j) {
            const int at = block + 256 * j + 4 * lane;
            if (at >= first && at < stop)
                __builtin_nontemporal_store(v[j], reinterpret_cast<unsigned*>(gzero + (block + 256 * j)) + lane);
        }
    }
    if (last) {
        lo = end;
        return;
    }
    // the unfinished line moves to the front of the slice (all lanes read before any writes:
    // source and destination may overlap)
    const unsigned rem = static_cast<unsigned>(keep_back);          // below 128
    unsigned keep = 0;
    const bool mine = static_cast<unsigned>(W * lane) < rem;
    if (mine) {
        if (W == 4) keep = *reinterpret_cast<const unsigned*>(stage + tail + W * lane);
        else keep = *reinterpret_cast<const unsigned short*>(stage + tail + W * lane);
    }
    wave_lds_sync();
    if (mine) {
        if (W == 4) *reinterpret_cast<unsigned*>(stage + W * lane) = keep;
        else *reinterpret_cast<unsigned short*>(stage + W * lane) = static_cast<unsigned short>(keep);
    }
    gzero += tail;
    lo = 0;
    end = rem;
}

// Global bytes into the LDS slice at the same offsets modulo 16, in two halves,
// so that a wave can have the loads of several steps in flight before it
// touches LDS.  wave_fetch requests the aligned
// 16-byte chunks that hold global bytes [shift, end_valid) at gbase (gbase is
// 16-byte aligned, shift < 16): chunk q goes to lane q % 64, slot q / 64.  A
// chunk is loaded whole even where the run begins or ends inside it -- an
// aligned 16-byte chunk never straddles a page, so the access is as safe as
// that of the bytes wanted -- and what lies at or past end_valid is cleared.
// wave_commit stores the chunks to LDS at the same offsets.
constexpr int kFetchSlots = (kStageLoads * kWaveSize * 16 + 16 + 15) / 16 / kWaveSize + 1;   // 5

__device__ inline void wave_fetch(uint4 (&r)[kFetchSlots], const unsigned char* gbase, unsigned end_valid,
                                  bool streaming, int lane) {
#pragma unroll
    for (int k = 0; k < kFetchSlots; ++k) {
        const unsigned q = static_cast<unsigned>(lane + k * kWaveSize);
        r[k] = make_uint4(0u, 0u, 0u, 0u);
        if (q * 16u < end_valid)
            r[k] = streaming ? load16_stream(gbase + q * 16u)
                             : *reinterpret_cast<const uint4*>(gbase + q * 16u);
    }
}

__device__ inline void wave_commit(unsigned char* stage, const uint4 (&r)[kFetchSlots], unsigned end,
                                   unsigned end_valid, int lane) {
#pragma unroll
    for (int k = 0; k < kFetchSlots; ++k) {
        const unsigned q = static_cast<unsigned>(lane + k * kWaveSize);
        if (q * 16u >= end) continue;
        uint4 v = r[k];
        if (q * 16u + 16u > end_valid) {          // only when the stream is cut short
            const unsigned valid = end_valid > q * 16u ? end_valid - q * 16u : 0u;   // bytes to keep: 0 .. 15
            unsigned d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned lo = 4u * i;
                d[i] = valid >= lo + 4u ? d[i] : valid > lo ? d[i] & ((1u << (8u * (valid - lo))) - 1u) : 0u;
            }
            v = make_uint4(d[0], d[1], d[2], d[3]);
        }
        *reinterpret_cast<uint4*>(stage + q * 16u) = v;
    }
}

// Device-wide exclusive scan of the per-tile counts, single pass (the paper's
// offset at which the next mask goes, section 5.1, for a whole tile at a time).
//
// Protocol.  Every tile publishes its own count (the wave of the tile that
// finishes its zero tests last does).  The last tile of every block of 256 also
// publishes the running total up to and including itself.  A tile
// finds the nearest published block prefix behind it and adds the counts of the
// tiles between that block and itself, two counts per 8-byte load across the
// wave.  In steady state that is a few hundred counts and the walk takes one
// pass.
//
// Why this shape (measured on MI355X): a device-scope load of a line that other
// XCDs are still writing costs a coherence round trip and slows the streaming
// traffic around it, while lines that have gone quiet are served from the local
// L2.  Counts are written once and read afterwards; running prefixes, which are
// written late, are kept sparse so that few lines are ever read while hot.  A
// classic look-back that polls a status+value word per tile, or a ticket
// counter per tile (one same-address atomic costs about 11 ns here), holds the
// whole kernel to a third of memory speed.
//
// Tiles are numbered by workgroup id.  The hardware hands workgroups out in id
// order, so a predecessor is normally already running and publishes within
// microseconds.  The wait does not rely on that: after `patience` fruitless
// polls the waiting wave computes a missing predecessor's count itself
// (`count_tile`, a re-read of that tile's input) and publishes it, so the walk
// ends whatever the dispatch order.
//
// Called by one whole wave of the tile, when the tile's own zero tests are done
// (asking for the prefixes earlier, while the tile's loads are under way, saves
// a round trip but finds a prefix further back, and the extra counts to read
// cost more than the round trip).  Returns the number of kept elements in all
// tiles before `tile` (not 0).
template <class CountTile>
__device__ inline unsigned long long scan_exclusive_prefix(unsigned* counts,
                                                           const unsigned long long* prefixes,
                                                           unsigned tile, int lane, WsHeader* hdr,
                                                           const CountTile& count_tile) {
    const int t = static_cast<int>(tile);
    // nearest published block prefix
    int bb = t / kBlockTiles - 1;
    unsigned long long base = 0;
    int lo = 0;
    while (true) {
        const int idx = bb - lane;
        const unsigned long long pv = idx >= 0 ? load64(prefixes + idx) : kPrefixValid;   // before block 0 the prefix is 0
        const unsigned long long have = __ballot((pv & kPrefixValid) != 0);
        if (have) {
            const int k = __ffsll(static_cast<long long>(have)) - 1;
            base = lane_value(pv, k) & ~kPrefixValid;
            lo = (bb - k + 1) * kBlockTiles;   // first tile after that block
            break;
        }
        bb -= kWaveSize;
    }
    // Counts of tiles lo .. t-1, a pair per 8-byte load (lo is a multiple of the
    // block size: pairs are aligned), kScanBatch loads per lane in flight at a time
    // (256 tiles a batch; asking for more at once reads more of the newest counts while they are still being written, which measures slower).  The
    // loads of a batch are added in order as far as everything they cover is
    // published; a later round asks again only from the first load that found
    // something missing, so the waiting re-reads no more than the newest counts.
    constexpr int kScanBatch = 2;
    constexpr int kLoadTiles = 2 * kWaveSize;     // tiles covered by one load of the wave
    int done_to = lo;              // wave-uniform: the counts of tiles lo .. done_to-1 are in `sum`
    unsigned sum = 0;              // a lane adds few counts, each below 2^16
    unsigned polls = 0, patience = 0;
    while (done_to < t) {
        unsigned long long pair[kScanBatch];
#pragma unroll
        for (int k = 0; k < kScanBatch; ++k) {
            const int i = done_to + k * kLoadTiles + 2 * lane;
            pair[k] = i < t ? load64(reinterpret_cast<const unsigned long long*>(counts + i))
                            : (static_cast<unsigned long long>(kCountValid) << 32) | kCountValid;
        }
        int complete = 0;          // leading loads of the batch that found everything published
        int hole = -1;             // wave-uniform: the first tile found unpublished
#pragma unroll
        for (int k = 0; k < kScanBatch; ++k) {
            if (complete != k) continue;          // wave-uniform
            const int i = done_to + k * kLoadTiles + 2 * lane;
            const unsigned c0 = static_cast<unsigned>(pair[k]);
            const unsigned c1 = i + 1 < t ? static_cast<unsigned>(pair[k] >> 32) : kCountValid;
            const unsigned long long missing = __ballot((c0 & c1 & kCountValid) == 0u);
            if (!missing) {
                sum += (c0 & ~kCountValid) + (c1 & ~kCountValid);
                complete = k + 1;
            } else {
                const int first = __ffsll(static_cast<long long>(missing)) - 1;
                hole = done_to + k * kLoadTiles + 2 * first +
                       ((lane_value(c0, first) & kCountValid) != 0u ? 1 : 0);
            }
        }
        done_to += complete * kLoadTiles;
        if (hole < 0) continue;                   // the whole batch was there: the next one, if any
        if (polls == 0) {                         // the first fruitless poll: how many may follow
            const unsigned long long p = uniform(load64(&hdr->patience_plus_one));
            patience = p != 0 ? static_cast<unsigned>(p - 1) : kDefaultPatience;
        }
        if (polls < patience) {
            ++polls;
            __builtin_amdgcn_s_sleep(kPollSleep);
            continue;
        }
        // help one unpublished predecessor, then look again without waiting anew
        const unsigned helped_count = count_tile(static_cast<unsigned>(hole), lane);
        unsigned old = 0;
        if (lane == 0) {
            old = atomicMax(counts + hole, kCountValid | helped_count);  // same value as the owner's
            atomicAdd(&hdr->helped, 1ull);
        }
        // the atomic has returned, so it has been performed before any lane polls again
        asm volatile("" : : "v"(old) : "memory");
    }
    // (halves, so that no partial sum can overflow whatever the distance walked)
    return base + wave_sum_small(sum & 0xFFFFu) +
           (static_cast<unsigned long long>(wave_sum_small(sum >> 16)) << 16);
}

// Encoder clean-up, see WsHeader::finish.  finish_arrive() is called by lane 0
// of the scan wave once the tile has read all the scan state it needs and its
// own words have been written (the s_waitcnt makes the write-through stores
// complete before the counter moves, so no late store can land after the
// clean-up).  The atomic returns nothing, so no wave ever waits for it.
__device__ inline void finish_arrive(WsHeader* hdr, unsigned tile) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __hip_atomic_fetch_add(&hdr->finish[tile % kFinishLanes].value, 1u, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}

// Called by the scan wave of the last tile at its end: waits until every tile
// of the call has arrived (none of them waits for this one, and the last tile
// is dispatched last, so the wait is short), then zeroes the scan state and the
// counters for the next call.
__device__ inline void finish_call(WsHeader* hdr, unsigned* counts, unsigned num_tiles, int lane,
                                   size_t state_bytes) {
    while (true) {
        const unsigned long long arrived = wave_sum(static_cast<unsigned long long>(
            __hip_atomic_load(&hdr->finish[lane].value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)));
        if (arrived == num_tiles) break;
        __builtin_amdgcn_s_sleep(kPollSleep);
    }
    uint4* p = reinterpret_cast<uint4*>(counts);   // counts then prefixes, 256-byte aligned
    const size_t chunks = state_bytes / 16;
    for (size_t i = lane; i < chunks; i += kWaveSize) p[i] = make_uint4(0u, 0u, 0u, 0u);
    hdr->finish[lane].value = 0u;
}

// ------------------------------------------------- encoder: loads and zero tests
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__device__ inline unsigned load_stream(const unsigned* p) { return __builtin_nontemporal_load(p); }
__device__ inline unsigned load_stream(const unsigned short* p) { return __builtin_nontemporal_load(p); }

// Dword d of a tensor that is wholly inside it.  SPLIT: 16-bit elements at an
// address that is not a multiple of 4 are fetched as two halves.
template <bool SPLIT>
__device__ __forceinline__ unsigned load_dword(const unsigned char* in, size_t d) {
    if (SPLIT) {
        const unsigned short* p = reinterpret_cast<const unsigned short*>(in) + 2 * d;
        return static_cast<unsigned>(load_stream(p)) | (static_cast<unsigned>(load_stream(p + 1)) << 16);
    }
    return load_stream(reinterpret_cast<const unsigned*>(in) + d);
}

// Dword `index` of a run of dwords that starts at `base` (wave-uniform, inside
// the tensor) and of which only dwords 0 .. room belong to the tensor, the last
// one maybe only with its low half (half_tail: 16-bit elements, odd count).
// What lies past the tensor reads as zero.  The dword that holds the tensor's
// last element is loaded whole (an aligned dword never straddles a page, so
// that is as safe as loading the element) and later lanes are redirected to
// it, so the loads need no branch; the excess is cleared in registers.  SPLIT
// fetches halves and checks each.
template <bool SPLIT>
__device__ __forceinline__ unsigned load_dword_ragged(const unsigned char* base, unsigned index,
                                                      unsigned room, bool half_tail) {
    if (SPLIT) {
        const unsigned short* p = reinterpret_cast<const unsigned short*>(base);
        const unsigned lo = index <= room ? static_cast<unsigned>(load_stream(p + 2 * index)) : 0u;
        const unsigned hi = index < room || (index == room && !half_tail)
                                ? static_cast<unsigned>(load_stream(p + 2 * index + 1)) : 0u;
        return lo | (hi << 16);
    }
    unsigned x = load_stream(reinterpret_cast<const unsigned*>(base) + (index < room ? index : room));
    if (index > room) x = 0u;
    if (half_tail && index == room) x &= 0xFFFFu;
    return x;
}

// Which elements are kept.  Plain ZVC (RELU = false) keeps the elements that are
// non-zero as integers (section 5.2: words compared to zero form the mask
// bits).  The fused ReLU + ZVC encoder (RELU = true) reads pre-activation
// values (IEEE-style, sign in the top bit: fp32, fp16, bf16) and keeps those
// whose sign bit is clear and which are not +0, i.e. the non-zeros of ReLU(x);
// as signed integers those are exactly the words greater than zero.
// kept_first: the element in the dword's low W bytes; kept_second (16-bit
// elements only): the one in its high half.
template <int W, bool RELU>
__device__ inline bool kept_first(unsigned x) {
    if (W == 4) return RELU ? static_cast<int>(x) > 0 : x != 0u;
    const unsigned low = x & 0xFFFFu;
    return RELU ? (low - 1u) < 0x7FFFu : low != 0u;
}
template <bool RELU>
__device__ inline bool kept_second(unsigned x) {
    return RELU ? static_cast<int>(x) > 0xFFFF : x > 0xFFFFu;
}

// Bits of `even` and `odd` interleaved: bit 2i of the result is bit i of even,
// bit 2i+1 is bit i of odd (wave-uniform operands, scalar unit).  With 16-bit
// elements a lane holds two neighbours, so the ballots of the first and of the
// second elements zip into the masks.
__device__ inline unsigned long long zip_bits(unsigned even, unsigned odd) {
    unsigned long long e, o;
    asm("s_bitreplicate_b64_b32 %0, %1" : "=s"(e) : "s"(even));
    asm("s_bitreplicate_b64_b32 %0, %1" : "=s"(o) : "s"(odd));
    return (e & 0x5555555555555555ull) | (o & 0xAAAAAAAAAAAAAAAAull);
}

// The 16 low bits of v moved apart: bit i goes to bit 2i.
__device__ inline unsigned spread_bits(unsigned v) {
    v = (v | (v << 8)) & 0x00FF00FFu;
    v = (v | (v << 4)) & 0x0F0F0F0Fu;
    v = (v | (v << 2)) & 0x33333333u;
    v = (v | (v << 1)) & 0x55555555u;
    return v;
}

// v in lane LANE := the wave-uniform value s (other lanes keep theirs).  The
// value usually comes straight from a vector compare; a vector instruction that
// reads such a freshly written scalar as an operand needs one wait state, which
// the compiler cannot know for an instruction it does not see, hence the s_nop.
template <int LANE>
__device__ __forceinline__ void set_lane(unsigned& v, unsigned s) {
    asm("s_nop 0\n\tv_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(s), "n"(LANE));
}
// The two halves of a ballot into lanes LANE0 and LANE1 of v (one wait state serves both).
template <int LANE0, int LANE1>
__device__ __forceinline__ void set_lanes(unsigned& v, unsigned long long ballot) {
    asm("s_nop 0\n\tv_writelane_b32 %0, %1, %3\n\tv_writelane_b32 %0, %2, %4"
        : "+v"(v)
        : "s"(static_cast<unsigned>(ballot)), "s"(static_cast<unsigned>(ballot >> 32)), "n"(LANE0), "n"(LANE1));
}

// Count of kept elements of input tile q, by one wave (scan self-help).
template <int W, int CH, int WV, bool RELU, bool SPLIT>
struct CountInputTile {
    const unsigned char* in;
    size_t n;
    __device__ unsigned operator()(unsigned q, int lane) const {
        constexpr unsigned kTileDwords = EncoderGeometry<W, CH, WV>::kTileBytes / 4;
        const size_t d0 = static_cast<size_t>(q) * kTileDwords;      // inside the tensor: q is a predecessor
        const size_t last = (n * W - 1) / 4;
        const unsigned room = last - d0 < kTileDwords ? static_cast<unsigned>(last - d0) : kTileDwords;
        const bool half_tail = W == 2 && (n & 1u) != 0u && room < kTileDwords;
        unsigned count = 0;
#pragma unroll 1
        for (unsigned i = 0; i < kTileDwords; i += kWaveSize) {
            const unsigned x = load_dword_ragged<SPLIT>(in + d0 * 4, i + lane, room, half_tail);
            count += kept_first<W, RELU>(x) ? 1u : 0u;
            if (W == 2) count += kept_second<RELU>(x) ? 1u : 0u;
        }
        return wave_sum_small(count);      // a lane counts at most 512 elements
    }
};

// ------------------------------------------------------------------- kernels

// Zeroes the workspace header and scan state (`words` 8-byte words).
__global__ void reset_kernel(unsigned long long* ws_words, size_t words) {
    for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < words;
         i += static_cast<size_t>(gridDim.x) * blockDim.x)
        ws_words[i] = 0ull;
}

__global__ void write_word_kernel(unsigned long long* dst, unsigned long long v) { *dst = v; }

// Workgroup barrier that orders LDS traffic only (__syncthreads() would also
// wait for the wave's outstanding global stores).
__device__ inline void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

struct EncoderArgs {
    const unsigned char* __restrict__ in;
    size_t n;
    unsigned* __restrict__ masks;
    unsigned char* __restrict__ values;
    WsHeader* hdr;
    unsigned* counts;
    unsigned long long* prefixes;
    unsigned long long* d_bytes;
    unsigned num_tiles;
    size_t num_groups;
    size_t state_bytes;
    unsigned long long cap_values;   // bytes that may be written at `values`
    unsigned long long* offsets;   // windowed stream only: byte offset of every window, then the total
    unsigned window_shift;         // windowed stream only: a window is 1 KB << window_shift of input
};

// Section 5.1 encoder.  One workgroup per tile; tile = workgroup id.  With
// RELU the input is the pre-activation tensor and the stream is that of
// ReLU(input): the dense ReLU output is never written or read.
//
// A wave owns CH consecutive chunks of the tile (256 bytes each, a dword per
// lane).  Its work, in the order in which it happens:
//
//   1. zero tests as the loads arrive: the ballot of a chunk's test is two
//      masks (fp32) or, zipped with the ballot of the lanes' second elements,
//      four (16-bit); its popcount adds to the wave's total.  The masks are
//      gathered into registers lane by lane and leave as coalesced stores.
//   2. the wave adds its total to the tile's arrival word in LDS; the wave that
//      arrives last publishes the tile's count for the tiles behind it, at once.
//   3. the wave stages its kept elements in its LDS queue in packed order
//      (position = ballot bits in lower lanes + kept elements of earlier
//      chunks), as many steps as the queue holds: that needs nothing from other
//      tiles, and it gives the tiles in front the time to publish their counts.
//   4. wave 0 finishes the device-wide scan (its first round trip has been
//      under way since the tile started); one barrier hands the result to the
//      other waves.
//   5. every wave writes its queue out in whole lines (wave_flush), staging
//      whatever did not fit before.
//
// WINDOWED selects the paper's own stream order (section 5.1: a group's
// non-zeros are appended right after its mask), packed back to back, plus a
// table with the byte offset of every window of 1 KB << window_shift of input
// (section 6 uses 4 KB and tries up to 64 KB).  The stream's bytes do not depend
// on the window size: the kernel works in units of 1 KB, four chunks, and stores
// the offset of every unit that begins a window.  The only differences are where things go in the
// wave's queue -- a group's mask sits before the group's elements -- and that
// masks leave with the values instead of going to a mask area.  The scan is the
// same: a window's byte offset is 4 x (groups before it) + W x (kept elements
// before it).
template <int W, int CH, int WV, bool RELU, bool WINDOWED, bool SPLIT>
__global__ __launch_bounds__(WV * kWaveSize) void compress_kernel(EncoderArgs a) {
    using G = EncoderGeometry<W, CH, WV>;
    constexpr int CG = G::kChunkGroups;
    constexpr int kAhead = CH;                    // all of a wave's loads are in flight from the start (measured: 3-6 % over 8 KB at a time)
    constexpr int kWindowChunks = 4;              // the windowed stream's unit: 1 KB of input
    static_assert(W == 2 || !SPLIT, "only 16-bit elements can sit at an odd half dword");

    __shared__ __align__(16) unsigned char s_stage[WV][G::kQueueBytes];
    __shared__ unsigned s_wave_total[WV];
    __shared__ unsigned s_arrive;                 // waves arrived << 24 | kept elements so far
    __shared__ unsigned long long s_prefix;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = static_cast<int>(uniform(static_cast<unsigned>(tid / kWaveSize)));
    const unsigned tile = blockIdx.x;
    if (tid == 0) s_arrive = 0u;

    const size_t wave_elem0 = static_cast<size_t>(tile) * G::kTileElems + static_cast<size_t>(wave) * G::kWaveElems;
    const size_t wave_group0 = static_cast<size_t>(tile) * G::kTileGroups + static_cast<size_t>(wave) * G::kWaveGroups;
    const size_t wave_dword0 = wave_elem0 / (4 / W);

    // ---- 1. loads, zero tests, masks (section 5.2: words compared to zero form the mask
    //         bits) and, fused with them where the queue has room, 3. compaction (section
    //         5.2: shift non-zeros to their packed slots)
    unsigned cur[CH];
    unsigned mask_reg[G::kMaskRegs];
    unsigned second_reg[W == 2 ? G::kMaskRegs : 1];   // 16-bit elements: the ballots of the lanes' second elements
    unsigned step_total[G::kSteps];               // wave-uniform
#pragma unroll
    for (int r = 0; r < G::kMaskRegs; ++r) mask_reg[r] = 0u;
#pragma unroll
    for (int r = 0; r < (W == 2 ? G::kMaskRegs : 1); ++r) second_reg[r] = 0u;
#pragma unroll
    for (int h = 0; h < G::kSteps; ++h) step_total[h] = 0u;
    unsigned char* stage = s_stage[wave];
    unsigned q_lo = 0, q_end = 0;                 // the wave's queue: slice offsets, wave-uniform
    unsigned zero_local = 0;                      // offset within the wave's run of slice offset 0
    unsigned window_local = 0;                    // lane i: offset within the wave's run of its window i
    // groups of the tensor among `count` groups of this wave from `first_group` on (fewer where the tensor ends)
    const auto groups_from = [&](int first_group, int count) -> unsigned {
        const size_t g = wave_group0 + static_cast<size_t>(first_group);
        return g >= a.num_groups ? 0u
             : a.num_groups - g < static_cast<size_t>(count) ? static_cast<unsigned>(a.num_groups - g)
                                                             : static_cast<unsigned>(count);
    };

    // One chunk.  TEST: its masks and its share of the totals.  STAGE: its kept
    // elements into the queue at q_end.  Both use the same ballots.
    const auto chunk = [&](auto kc, auto test_c, auto stage_c) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        constexpr bool TEST = decltype(test_c)::value, STAGE = decltype(stage_c)::value;
        const unsigned x = cur[k];
        const unsigned chunk_groups = STAGE && WINDOWED ? groups_from(k * CG, CG) : 0u;
        if (STAGE && WINDOWED && k % kWindowChunks == 0)
            set_lane<k / kWindowChunks>(window_local, zero_local + q_end);
        if constexpr (W == 4) {
            const bool keep = kept_first<4, RELU>(x);
            const unsigned long long b = __ballot(keep);
            const unsigned kept = static_cast<unsigned>(__popcll(b));
            if (TEST) {
                step_total[k / kStepChunks] += kept;
                if (!WINDOWED)
                    set_lanes<(2 * k) % kWaveSize, (2 * k + 1) % kWaveSize>(mask_reg[(2 * k) / kWaveSize], b);
            }
            if (STAGE) {
                // windowed: the lane's group has its mask, and the masks of the chunk's earlier groups, before it
                const unsigned at = 4u * lanes_below(b, 0u) + q_end + (WINDOWED ? 4u + 4u * (lane >> 5) : 0u);
                if (__builtin_expect(keep, 1)) *reinterpret_cast<unsigned*>(stage + at) = x;   // predicated, no branch
                if (WINDOWED && (lane & 31) == 0 && static_cast<unsigned>(lane >> 5) < chunk_groups)
                    *reinterpret_cast<unsigned*>(stage + at - 4u) =
                        lane == 0 ? static_cast<unsigned>(b) : static_cast<unsigned>(b >> 32);
                q_end += 4u * kept + 4u * chunk_groups;
            }
        } else {
            const bool keep0 = kept_first<2, RELU>(x), keep1 = kept_second<RELU>(x);
            const unsigned long long be = __ballot(keep0), bo = __ballot(keep1);
            const unsigned kept = static_cast<unsigned>(__popcll(be)) + static_cast<unsigned>(__popcll(bo));
            unsigned long long z0 = 0, z1 = 0;
            if (STAGE && WINDOWED) {
                z0 = zip_bits(static_cast<unsigned>(be), static_cast<unsigned>(bo));
                z1 = zip_bits(static_cast<unsigned>(be >> 32), static_cast<unsigned>(bo >> 32));
            }
            if (TEST) {
                step_total[k / kStepChunks] += kept;
                if (!WINDOWED) {
                    // The ballots as they are, 32 bits each in lanes 4k and 4k+2 (two masks' worth of
                    // first elements in mask_reg, of second elements in second_reg): they are zipped
                    // into the four masks once per wave, on the vector unit (zip_ballot_lanes),
                    // which measures 8-15 % faster than zipping every chunk on the scalar unit.
                    set_lanes<(4 * k) % kWaveSize, (4 * k + 2) % kWaveSize>(mask_reg[(4 * k) / kWaveSize], be);
                    set_lanes<(4 * k) % kWaveSize, (4 * k + 2) % kWaveSize>(second_reg[(4 * k) / kWaveSize], bo);
                }
            }
            if (STAGE) {
                const unsigned at = 2u * lanes_below(bo, lanes_below(be, 0u)) + q_end +
                                    (WINDOWED ? 4u + 4u * (lane >> 4) : 0u);
                if (WINDOWED && (lane & 15) == 0 && static_cast<unsigned>(lane >> 4) < chunk_groups) {
                    const unsigned m = lane == 0 ? static_cast<unsigned>(z0)
                                     : lane == 16 ? static_cast<unsigned>(z0 >> 32)
                                     : lane == 32 ? static_cast<unsigned>(z1) : static_cast<unsigned>(z1 >> 32);
                    *reinterpret_cast<unsigned short*>(stage + at - 4u) = static_cast<unsigned short>(m);
                    *reinterpret_cast<unsigned short*>(stage + at - 2u) = static_cast<unsigned short>(m >> 16);
                }
                if (__builtin_expect(keep0, 1)) *reinterpret_cast<unsigned short*>(stage + at) = static_cast<unsigned short>(x);
                if (__builtin_expect(keep1, 1)) *reinterpret_cast<unsigned short*>(stage + at + (keep0 ? 2u : 0u)) = static_cast<unsigned short>(x >> 16);
                q_end += 2u * kept + 4u * chunk_groups;
            }
        }
    };
    constexpr std::true_type yes{};
    constexpr std::false_type no{};

    // A wave that lies wholly inside the tensor needs no bounds checks: it keeps
    // kAhead loads in flight and tests each chunk as it arrives.  A step is
    // compacted in the same pass while the queue is sure to hold it whatever its
    // density (the first two steps always are): the compaction then happens
    // while the wave would otherwise wait for its loads, and needs nothing from
    // other tiles.  The barrier makes the cleared arrival word visible to the
    // tile's waves; it comes after the first loads have been issued, so it costs
    // them nothing.
    int staged = 0;                               // steps in the queue so far, wave-uniform
    if (wave_elem0 + G::kWaveElems <= a.n) {
        static_for<0, kAhead>([&](auto kc) __attribute__((always_inline)) {
            constexpr int k = decltype(kc)::value;
            cur[k] = load_dword<SPLIT>(a.in, wave_dword0 + static_cast<size_t>(k) * kWaveSize + lane);
            __builtin_amdgcn_sched_barrier(0);   // in the order in which the tests use them
        });
        lds_barrier();
        static_for<0, G::kSteps>([&](auto hc) __attribute__((always_inline)) {
            constexpr int h = decltype(hc)::value;
            const bool fuse = staged == h && q_end + G::kStepMaxBytes <= static_cast<unsigned>(G::kQueueBytes);
            const auto next_load = [&](auto kc) __attribute__((always_inline)) {
                constexpr int k = decltype(kc)::value;
                if constexpr (k + kAhead < CH)
                    cur[k + kAhead] =
                        load_dword<SPLIT>(a.in, wave_dword0 + static_cast<size_t>(k + kAhead) * kWaveSize + lane);
                __builtin_amdgcn_sched_barrier(0);
            };
            if (fuse) {
                static_for<h * kStepChunks, (h + 1) * kStepChunks>([&](auto kc) __attribute__((always_inline)) {
                    chunk(kc, yes, yes);
                    next_load(kc);
                });
                staged = h + 1;
            } else {
                static_for<h * kStepChunks, (h + 1) * kStepChunks>([&](auto kc) __attribute__((always_inline)) {
                    chunk(kc, yes, no);
                    next_load(kc);
                });
            }
        });
    } else if (wave_elem0 < a.n) {
        // the wave that holds the tensor's end
        const size_t last = (a.n * W - 1) / 4;                       // last dword with an element in it
        const unsigned room = static_cast<unsigned>(last - wave_dword0);
        const bool half_tail = W == 2 && (a.n & 1u) != 0u;
        const unsigned char* base = a.in + wave_dword0 * 4;
        static_for<0, CH>([&](auto kc) __attribute__((always_inline)) {
            constexpr int k = decltype(kc)::value;
            cur[k] = load_dword_ragged<SPLIT>(base, static_cast<unsigned>(k * kWaveSize + lane), room, half_tail);
            asm volatile("" : "+v"(cur[k]));     // (or the compiler keeps the masked halves of all chunks for the tests)
            __builtin_amdgcn_sched_barrier(0);
        });
        lds_barrier();
        static_for<0, CH>([&](auto kc) __attribute__((always_inline)) {
            chunk(kc, yes, no);
            __builtin_amdgcn_sched_barrier(0);
        });
    } else {
        // past the tensor's end: nothing kept, no masks (the wave still takes part in the tile's protocol)
#pragma unroll
        for (int k = 0; k < CH; ++k) cur[k] = 0u;
        lds_barrier();
    }
    unsigned wave_total = 0;
#pragma unroll
    for (int h = 0; h < G::kSteps; ++h) wave_total += step_total[h];

    // ---- 2. arrival: the last wave of the tile to get here publishes the tile's count
    unsigned arrived = 0;
    if (lane == 0) {
        s_wave_total[wave] = wave_total;
        arrived = __hip_atomic_fetch_add(&s_arrive, (1u << 24) | wave_total, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    arrived = uniform(arrived);
    const bool publisher = (arrived >> 24) == WV - 1;
    if (publisher && lane == 0)
        store32(a.counts + tile, kCountValid | ((arrived & 0xFFFFFFu) + wave_total));

    if (!WINDOWED && W == 2) {
        // zip_ballot_lanes: an even lane holds 32 bits of the first elements' ballot and the same
        // 32 bits of the second elements' ballot.  It zips the low halves into its mask, its odd
        // neighbour (which reads them with a DPP row shift) the high halves into the next mask.
#pragma unroll
        for (int r = 0; r < G::kMaskRegs; ++r) {
            // (a DPP read of a register needs two wait states after the instruction that wrote it;
            // the compiler sees the lane writes above only as opaque statements)
            asm volatile("s_nop 1" : "+v"(mask_reg[r]), "+v"(second_reg[r]));
            const unsigned first_prev =
                static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(mask_reg[r]), 0x111, 0xF, 0xF, true));
            const unsigned second_prev =
                static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(second_reg[r]), 0x111, 0xF, 0xF, true));
            const bool odd_lane = (lane & 1) != 0;
            mask_reg[r] = spread_bits(odd_lane ? first_prev >> 16 : mask_reg[r] & 0xFFFFu) |
                          (spread_bits(odd_lane ? second_prev >> 16 : second_reg[r] & 0xFFFFu) << 1);
        }
    }
    if (!WINDOWED) {
#pragma unroll
        for (int r = 0; r < G::kMaskRegs; ++r) {
            const size_t g = wave_group0 + static_cast<size_t>(r) * kWaveSize + lane;
            if (r * kWaveSize + lane < G::kWaveGroups && g < a.num_groups)
                __builtin_nontemporal_store(mask_reg[r], a.masks + g);
        }
    }

    // ---- 3. more of the compaction before the tile knows where its run begins: the steps
    //         that were not sure to fit but, now that their size is known, do
    const auto step_bytes = [&](int h) -> unsigned {
        return step_total[h] * W + (WINDOWED ? 4u * groups_from(h * G::kStepGroups, G::kStepGroups) : 0u);
    };
    const auto stage_step = [&](auto hc) __attribute__((always_inline)) {
        constexpr int h = decltype(hc)::value;
        static_for<h * kStepChunks, (h + 1) * kStepChunks>([&](auto kc) __attribute__((always_inline)) {
            chunk(kc, no, yes);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    static_for<0, G::kSteps>([&](auto hc) __attribute__((always_inline)) {
        constexpr int h = decltype(hc)::value;
        if (staged == h && q_end + step_bytes(h) <= static_cast<unsigned>(G::kQueueBytes)) {
            stage_step(hc);
            staged = h + 1;
        }
    });

    // ---- 4. device-wide exclusive scan, wave 0
    if (wave == 0) {
        unsigned long long ex = 0;
        if (tile != 0) {
            const CountInputTile<W, CH, WV, RELU, SPLIT> count_tile{a.in, a.n};
            ex = scan_exclusive_prefix(a.counts, a.prefixes, tile, lane, a.hdr, count_tile);
        }
        if (lane == 0) s_prefix = ex;
    }
    // the tile's count has reached memory before any wave of the tile goes on (see finish_arrive)
    if (publisher) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    const unsigned long long exclusive = uniform(s_prefix);
    unsigned wave_offset = 0, tile_total = 0;
#pragma unroll
    for (int v = 0; v < WV; ++v) {
        const unsigned t = uniform(s_wave_total[v]);
        if (v < wave) wave_offset += t;
        tile_total += t;
    }
    if (wave == 0 && lane == 0) {
        if (tile % kBlockTiles == kBlockTiles - 1)
            store64(a.prefixes + tile / kBlockTiles, kPrefixValid | (exclusive + tile_total));
        finish_arrive(a.hdr, tile);
    }

    //      A call with a buffer below the worst case (cap_values) writes a tile's
    //      run only if the run ends inside the buffer; the size is reported anyway.
    const unsigned long long tile_end_bytes =
        (exclusive + tile_total) * W +
        (WINDOWED ? 4ull * min(static_cast<size_t>(tile + 1) * G::kTileGroups, a.num_groups) : 0ull);
    if (tile_end_bytes <= a.cap_values) {
        unsigned char* const run_begin =
            a.values + (exclusive + wave_offset) * W +
            (WINDOWED ? 4 * (wave_group0 < a.num_groups ? wave_group0 : a.num_groups) : 0);
        unsigned char* gzero = run_begin;
        if (staged != 0) {
            wave_flush<W>(gzero, stage, q_lo, q_end, staged == G::kSteps, lane);
            zero_local = static_cast<unsigned>(gzero - run_begin);
            wave_lds_sync();
        }
        static_for<0, G::kSteps>([&](auto hc) __attribute__((always_inline)) {
            constexpr int h = decltype(hc)::value;
            if (h >= staged) {
                stage_step(hc);
                wave_lds_sync();
                wave_flush<W>(gzero, stage, q_lo, q_end, h == G::kSteps - 1, lane);
                zero_local = static_cast<unsigned>(gzero - run_begin);
                wave_lds_sync();
            }
        });
        if (WINDOWED && lane < CH / kWindowChunks) {
            // the byte offset of every window that exists: its masks before it, its kept elements before it
            const size_t unit = wave_group0 / (kWindowChunks * CG) + lane;     // 1 KB of input
            if (wave_group0 + static_cast<size_t>(lane) * (kWindowChunks * CG) < a.num_groups &&
                (unit & ((size_t{1} << a.window_shift) - 1)) == 0)
                a.offsets[unit >> a.window_shift] =
                    static_cast<unsigned long long>(run_begin - a.values) + window_local;
        }
    }

    // ---- section 5.4: the compressed size, reported by the last tile
    if (tile == a.num_tiles - 1 && tid == 0) {
        const unsigned long long total =
            4ull * a.num_groups + static_cast<unsigned long long>(W) * (exclusive + tile_total);
        *a.d_bytes = total;
        if (WINDOWED)
            a.offsets[div_up(a.num_groups, static_cast<size_t>(kWindowChunks * CG) << a.window_shift)] = total;
    }

    if (tile == a.num_tiles - 1 && wave == 0)
        finish_call(a.hdr, a.counts, a.num_tiles, lane, a.state_bytes);
}

// Decoder pre-pass (section 5.2: the popcount of a mask span is the number of
// stored words the span consumes).  Where a span's stored elements start
// depends on the masks alone, which are 1/32 (fp32) or 1/16 (16-bit) of the
// tensor, so it is computed ahead of the decoder, whose waves then depend on
// nothing but their own part of the stream.  One workgroup takes a chunk of
// kChunkMasks consecutive masks with coalesced 16-byte loads and writes
//   unit_end[u]    = stored elements of the chunk up to and including unit u
//                    (a unit is 32 masks, 1024 elements),
//   chunk_total[c] = stored elements of the chunk.
// Unless chunk_prefix is null (few chunks, see kFewChunks), the workgroup that
// finishes last (arrival counters in the header, which it also resets) turns
// the totals into chunk_prefix[c] = stored elements before chunk c.
constexpr int kUnitMasks = 32;
constexpr int kChunkLoads = 4;                                 // 16-byte loads per thread
constexpr int kChunkMasks = kThreads * 4 * kChunkLoads;        // 4096 masks = 131072 elements
constexpr int kChunkUnits = kChunkMasks / kUnitMasks;          // 128
constexpr int kUnitLanes = kUnitMasks / 4;                     // 8 lanes of one load cover a unit
// Up to this many chunks (134M elements) the expand kernel's workgroups each add
// up the chunk totals before their own chunk; above, the pre-pass does it once.
constexpr unsigned kFewChunks = 1024;

__global__ __launch_bounds__(kThreads) void mask_prefix_kernel(
    const unsigned* __restrict__ masks, size_t num_groups, unsigned tail,
    unsigned* __restrict__ unit_end, unsigned* chunk_total,
    unsigned long long* __restrict__ chunk_prefix, WsHeader* hdr, unsigned num_chunks) {
    __shared__ unsigned s_unit[kChunkUnits];
    __shared__ unsigned s_wave_total[2];
    __shared__ unsigned long long s_wave_sum[kWaves];
    __shared__ unsigned s_last;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid / kWaveSize;
    const unsigned chunk = blockIdx.x;
    const size_t g_chunk = static_cast<size_t>(chunk) * kChunkMasks;

    // ---- load k covers masks [g_chunk + 1024 k, + 1024): 4 per thread, 4 KB per workgroup
    unsigned c[kChunkLoads];
    const bool whole = g_chunk + kChunkMasks <= num_groups &&
                       !(g_chunk + kChunkMasks == num_groups && tail != 0) &&
                       (reinterpret_cast<uintptr_t>(masks) & 15u) == 0;
    if (whole) {
#pragma unroll
        for (int k = 0; k < kChunkLoads; ++k) {
            const uint4 v = *reinterpret_cast<const uint4*>(masks + g_chunk + 1024 * k + 4 * tid);
            c[k] = __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
        }
    } else {
#pragma unroll 1
        for (int k = 0; k < kChunkLoads; ++k) {
            unsigned sum = 0;
            for (int i = 0; i < 4; ++i) {
                const size_t g = g_chunk + 1024 * k + 4 * tid + i;
                if (g < num_groups) {
                    unsigned m = masks[g];
                    if (g == num_groups - 1 && tail != 0) m &= (1u << tail) - 1u;  // bits past n never count
                    sum += __popc(m);
                }
            }
            c[k] = sum;
        }
    }
    // ---- unit sums: 8 consecutive lanes of one load, two loads packed per register
    //      (a unit holds at most 1024 set bits)
#pragma unroll
    for (int q = 0; q < kChunkLoads / 2; ++q) {
        unsigned p = c[2 * q] | (c[2 * q + 1] << 16);
#pragma unroll
        for (int off = 1; off < kUnitLanes; off <<= 1) p += __shfl_xor(p, off);
        if (tid % kUnitLanes == 0) {
            s_unit[(2 * q) * (kThreads / kUnitLanes) + tid / kUnitLanes] = p & 0xFFFFu;
            s_unit[(2 * q + 1) * (kThreads / kUnitLanes) + tid / kUnitLanes] = p >> 16;
        }
    }
    __syncthreads();
    // ---- inclusive scan of the 128 unit sums (waves 0 and 1)
    const unsigned v = tid < kChunkUnits ? s_unit[tid] : 0u;
    unsigned incl = v;
#pragma unroll
    for (int off = 1; off < kWaveSize; off <<= 1) {
        const unsigned t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    if (lane == kWaveSize - 1 && wave < 2) s_wave_total[wave] = incl;
    __syncthreads();
    if (tid < kChunkUnits)
        unit_end[static_cast<size_t>(chunk) * kChunkUnits + tid] =
            incl + (wave == 1 ? s_wave_total[0] : 0u);

    // ---- few chunks: the expand kernel's workgroups add up the totals before theirs
    //      themselves (a KB or so from L2 each), which costs less than the two memory
    //      round trips below
    if (chunk_prefix == nullptr) {
        if (tid == 0) chunk_total[chunk] = s_wave_total[0] + s_wave_total[1];
        return;
    }
    // ---- the last workgroup to get here prefixes the chunk totals
    if (tid == 0) {
        store32(chunk_total + chunk, s_wave_total[0] + s_wave_total[1]);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the total is out before the count moves
        // counted like the encoder's tiles: atomics on one address cost about 11 ns
        // each here, so the arrivals are spread over 64 counters with one on top
        const unsigned slot = chunk % kFinishLanes;
        const unsigned quota = num_chunks / kFinishLanes + (slot < num_chunks % kFinishLanes ? 1u : 0u);
        unsigned last = 0;
        if (atomicAdd(&hdr->finish[slot].value, 1u) == quota - 1) {
            const unsigned slots_used = num_chunks < kFinishLanes ? num_chunks : kFinishLanes;
            last = atomicAdd(&hdr->finish_top.value, 1u) == slots_used - 1 ? 1u : 0u;
        }
        s_last = last;
    }
    __syncthreads();
    if (s_last == 0u) return;
    // 8 consecutive totals per thread and round, all loads of a round in flight together
    constexpr int kPerThread = 8;
    unsigned long long carry = 0;
    for (size_t base = 0; base < num_chunks; base += kThreads * kPerThread) {
        const size_t c0 = base + static_cast<size_t>(tid) * kPerThread;   // chunk_total is 256-byte aligned
        unsigned long long pair[kPerThread / 2];
#pragma unroll
        for (int k = 0; k < kPerThread / 2; ++k)
            pair[k] = c0 + 2 * k < num_chunks
                          ? load64(reinterpret_cast<const unsigned long long*>(chunk_total + c0 + 2 * k))
                          : 0ull;
        unsigned t[kPerThread];
        unsigned long long mine = 0;
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            t[k] = c0 + k < num_chunks ? static_cast<unsigned>(pair[k / 2] >> (32 * (k % 2))) : 0u;
            mine += t[k];
        }
        unsigned long long inc = mine;
#pragma unroll
        for (int off = 1; off < kWaveSize; off <<= 1) {
            const unsigned long long up = __shfl_up(inc, off);
            if (lane >= off) inc += up;
        }
        __syncthreads();   // s_wave_sum of the previous round has been read
        if (lane == kWaveSize - 1) s_wave_sum[wave] = inc;
        __syncthreads();
        unsigned long long before = carry + inc - mine, all = 0;
#pragma unroll
        for (int w2 = 0; w2 < kWaves; ++w2) {
            const unsigned long long ws = s_wave_sum[w2];
            if (w2 < wave) before += ws;
            all += ws;
        }
#pragma unroll
        for (int k = 0; k < kPerThread; ++k) {
            if (c0 + k < num_chunks) chunk_prefix[c0 + k] = before;
            before += t[k];
        }
        carry += all;
    }
    // ready for the next call
    if (tid < kFinishLanes) hdr->finish[tid].value = 0u;
    if (tid == 0) hdr->finish_top.value = 0u;
}

// One step of the decoder, by one wave: 4 KB of output from `m` (lane i holds
// the step's mask i, bits past n cleared) and the step's `step_total` stored
// elements, which begin at element `first` of the value area.  Stages them in
// the wave's LDS slice with aligned 16-byte loads (never past values_avail
// elements: anything the masks ask for beyond that decodes as zero); every lane
// then rebuilds 16 bytes of output per load from "bit ? next stored element :
// 0".  Slots whose bit is clear read a valid dummy address and select zero.
template <int W, bool ALIGNED>
__device__ __forceinline__ void expand_step(unsigned char* stage, const unsigned char* __restrict__ values,
                                            unsigned long long values_avail, unsigned long long first,
                                            unsigned step_total, unsigned m, size_t wave_elem0, size_t n,
                                            unsigned char* __restrict__ out, bool stream_values, int lane) {
    using G = Geometry<W, kMinLoads>;
    constexpr int E = G::kElemsPerLane;
    constexpr int LPG = G::kLanesPerGroup;
    constexpr int kStepMasks = kStageLoads * G::kGroupsPerLoad;   // 32 | 64 masks per step
    const bool full_wave = ALIGNED && wave_elem0 + static_cast<size_t>(kStageLoads) * kWaveSize * E <= n;
    const unsigned char* src = values + first * W;  // wave-uniform
    const unsigned shift = static_cast<unsigned>(reinterpret_cast<uintptr_t>(src) & 15u);
    unsigned long long readable = values_avail > first ? values_avail - first : 0ull;
    if (readable > step_total) readable = step_total;
    const unsigned end = shift + step_total * W;
    const unsigned end_valid = shift + static_cast<unsigned>(readable) * W;
    uint4 fetched[kFetchSlots];
    wave_fetch(fetched, src - shift, readable != 0 ? end_valid : 0u, stream_values, lane);
    wave_commit(stage, fetched, end, end_valid > shift ? end_valid : 0u, lane);
    // stored elements of the step before each of its masks (lane i holds mask i)
    const unsigned cnt = __popc(m);
    unsigned incl = cnt;
#pragma unroll
    for (int off = 1; off < kStepMasks; off <<= 1) {
        const unsigned t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    const unsigned before_mask = incl - cnt;
    wave_lds_sync();
#pragma unroll
    for (int jj = 0; jj < kStageLoads; ++jj) {
        const size_t e0 = wave_elem0 + (static_cast<size_t>(jj) * kWaveSize + lane) * E;
        const int gl = jj * G::kGroupsPerLoad + lane / LPG;     // the lane's mask within the step
        const unsigned gm = __shfl(m, gl);
        const unsigned bit0 = static_cast<unsigned>(lane % LPG) * E;
        unsigned at = shift + W * (__shfl(before_mask, gl) + __popc(gm & ((1u << bit0) - 1u)));
        const unsigned field = gm >> bit0;
        unsigned d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int c = 0; c < E; ++c) {
            const bool set = (field >> c) & 1u;
            const unsigned from = set ? at : shift;
            if (W == 4) {
                const unsigned v = *reinterpret_cast<const unsigned*>(stage + from);
                d[c] = set ? v : 0u;
            } else {
                const unsigned v = *reinterpret_cast<const unsigned short*>(stage + from);
                d[c >> 1] |= (set ? v : 0u) << (16 * (c & 1));
            }
            at += set ? W : 0;
        }
        if (full_wave || (ALIGNED && e0 + E <= n)) {
            store16_stream(out + e0 * W, make_uint4(d[0], d[1], d[2], d[3]));
        } else {
#pragma unroll
            for (int c = 0; c < E; ++c) {
                if (e0 + c < n) {
                    if (W == 4)
                        reinterpret_cast<unsigned*>(out)[e0 + c] = d[c];
                    else
                        reinterpret_cast<unsigned short*>(out)[e0 + c] = static_cast<unsigned short>(
                            (d[c >> 1] >> (16 * (c & 1))) & 0xFFFFu);
                }
            }
        }
    }
}

// Section 5.2 decoder.  Every wave works on its own: it expands one step, 4 KB
// of output, and knows from the pre-pass where the step's stored elements begin
// and end (expand_step does the rest).
template <int W, int LOADS, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void decompress_kernel(
    const unsigned* __restrict__ masks, const unsigned char* __restrict__ values,
    unsigned long long values_avail, size_t n, unsigned char* __restrict__ out,
    const unsigned* __restrict__ unit_end, const unsigned long long* __restrict__ chunk_prefix,
    const unsigned* __restrict__ chunk_total, size_t num_groups, bool stream_values, bool interleave) {
    using G = Geometry<W, LOADS>;
    constexpr int E = G::kElemsPerLane;
    constexpr int kStepMasks = kStageLoads * G::kGroupsPerLoad;   // 32 | 64 masks per step
    constexpr int kStepUnits = kStepMasks / kUnitMasks;           // 1 | 2
    constexpr int kSteps = G::kStageSteps;
    static_assert(kChunkMasks % (LOADS * G::kGroupsPerLoad) == 0, "a wave's masks lie in one chunk");

    __shared__ __align__(16) unsigned char s_stage[kWaves][G::kWaveStageBytes];

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = static_cast<int>(uniform(static_cast<unsigned>(tid / kWaveSize)));
    const unsigned tile = blockIdx.x;
    // Which part of the tensor (LOADS KB) the wave expands.  In a row: workgroup i
    // takes parts 4i .. 4i+3, so the eight XCDs (workgroup i runs on XCD i mod 8)
    // write 16 KB apiece side by side.  Interleaved: the waves of workgroup i take
    // parts that are i mod 8 modulo 8, so the XCDs write neighbouring 4 KB blocks at
    // the same time.  The memory system takes a stream of writes with few reads
    // among them up to 15 % faster in the second order (the host chooses).
    const size_t part = interleave ? (static_cast<size_t>(tile / 8) * kWaves + wave) * 8 + tile % 8
                                   : static_cast<size_t>(tile) * kWaves + wave;
    const size_t wave_elem0 = part * (static_cast<size_t>(LOADS) * kWaveSize * E);
    const size_t wave_group0 = wave_elem0 / 32;
    const size_t chunk = wave_group0 / kChunkMasks;     // the same for all waves of the workgroup
    const unsigned tail = static_cast<unsigned>(n % 32);

    // ---- stored elements before the wave's chunk: from the pre-pass, or (few chunks) the
    //      workgroup adds up the totals of the chunks before its own
    unsigned long long before_chunk = 0;
    if (chunk_prefix == nullptr) {
        __shared__ unsigned long long s_before;
        if (tid == 0) s_before = 0ull;
        unsigned partial = 0;                      // at most 4 totals of at most 2^17 each
        const size_t before = min(chunk, div_up(num_groups, static_cast<size_t>(kChunkMasks)));   // (a workgroup past the tensor's end)
        for (size_t c = tid; c < before; c += kThreads) partial += chunk_total[c];
        const unsigned wave_part = wave_sum_small(partial);
        lds_barrier();
        if (lane == 0 && wave_part != 0u)
            __hip_atomic_fetch_add(&s_before, static_cast<unsigned long long>(wave_part), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
        lds_barrier();
        before_chunk = s_before;
    }
    if (wave_elem0 >= n) return;                  // nothing of the tensor in this wave's part
    if (chunk_prefix != nullptr) before_chunk = chunk_prefix[chunk];

    // ---- everything the steps need from memory, requested up front
    unsigned m[kSteps], step_begin[kSteps], step_end[kSteps];
#pragma unroll
    for (int h = 0; h < kSteps; ++h) {
        const size_t g = wave_group0 + static_cast<size_t>(h) * kStepMasks + lane;
        m[h] = 0;
        if (lane < kStepMasks && g < num_groups) {
            m[h] = masks[g];
            if (g == num_groups - 1 && tail != 0) m[h] &= (1u << tail) - 1u;   // bits past n never count
        }
        const size_t u = wave_group0 / kUnitMasks + static_cast<size_t>(h) * kStepUnits;
        step_begin[h] = u % kChunkUnits != 0 ? unit_end[u - 1] : 0u;
        step_end[h] = unit_end[u + kStepUnits - 1];
    }

    static_assert(kSteps == 1, "a wave expands one step");
    expand_step<W, ALIGNED>(s_stage[wave], values, values_avail, before_chunk + step_begin[0],
                            step_end[0] - step_begin[0], m[0], wave_elem0, n, out, stream_values, lane);
}

// The same decoder in one launch, for small tensors: no pre-pass.  A workgroup
// expands 16 KB of output, in stream order.  Where its stored elements begin is
// the number of set bits in all masks before its own, which it gets the way the
// encoder's tiles get their offsets: it publishes the popcount of its own 128
// (256) masks and runs the device-wide scan over the workgroups before it
// (scan_exclusive_prefix; same scan state in the workspace, same clean-up by the
// last workgroup, same self-help if a predecessor has not been dispatched).  A
// workgroup knows its count after one small load, so the scan's chain is short;
// below a few tens of megabytes one launch beats the pre-pass's extra kernel,
// above that the pre-pass wins because its expand kernel touches no shared state.
struct CountMaskTile {
    const unsigned* masks;
    size_t num_groups;
    unsigned tail;                 // n % 32
    int tile_masks;                // masks per workgroup: 128 | 256
    // set bits in the masks of workgroup q, wave-uniform
    __device__ unsigned operator()(unsigned q, int lane) const {
        unsigned count = 0;
        for (int i = lane; i < tile_masks; i += kWaveSize) {
            const size_t g = static_cast<size_t>(q) * tile_masks + i;
            if (g < num_groups) {
                unsigned m = __builtin_nontemporal_load(masks + g);
                if (g == num_groups - 1 && tail != 0) m &= (1u << tail) - 1u;
                count += __popc(m);
            }
        }
        return wave_sum_small(count);
    }
};

template <int W, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void decompress_scan_kernel(
    const unsigned* __restrict__ masks, const unsigned char* __restrict__ values,
    unsigned long long values_avail, size_t n, unsigned char* __restrict__ out, WsHeader* hdr,
    unsigned* counts, unsigned long long* prefixes, unsigned num_tiles, size_t state_bytes,
    size_t num_groups, bool stream_values) {
    using G = Geometry<W, kMinLoads>;
    constexpr int E = G::kElemsPerLane;
    constexpr int kStepMasks = kStageLoads * G::kGroupsPerLoad;   // masks per wave: 32 | 64
    static_assert(G::kStageSteps == 1, "a wave expands one step");

    __shared__ __align__(16) unsigned char s_stage[kWaves][G::kWaveStageBytes];
    __shared__ unsigned s_wave_total[kWaves];
    __shared__ unsigned s_arrive;                 // waves arrived << 24 | set bits so far
    __shared__ unsigned long long s_prefix;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = static_cast<int>(uniform(static_cast<unsigned>(tid / kWaveSize)));
    const unsigned tile = blockIdx.x;
    if (tid == 0) s_arrive = 0u;
    const size_t wave_elem0 = (static_cast<size_t>(tile) * kWaves + wave) * (static_cast<size_t>(kMinLoads) * kWaveSize * E);
    const size_t wave_group0 = wave_elem0 / 32;
    const unsigned tail = static_cast<unsigned>(n % 32);

    // ---- the wave's masks (lane i holds mask i) and their set bits
    unsigned m = 0;
    {
        const size_t g = wave_group0 + lane;
        if (lane < kStepMasks && g < num_groups) {
            m = masks[g];
            if (g == num_groups - 1 && tail != 0) m &= (1u << tail) - 1u;   // bits past n never count
        }
    }
    lds_barrier();                                // the cleared arrival word, after the load has been issued
    const unsigned wave_total = wave_sum_small(__popc(m));

    // ---- the workgroup's count, published by the wave that arrives last; the scan, by wave 0
    unsigned arrived = 0;
    if (lane == 0) {
        s_wave_total[wave] = wave_total;
        arrived = __hip_atomic_fetch_add(&s_arrive, (1u << 24) | wave_total, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    arrived = uniform(arrived);
    const bool publisher = (arrived >> 24) == kWaves - 1;
    if (publisher && lane == 0)
        store32(counts + tile, kCountValid | ((arrived & 0xFFFFFFu) + wave_total));
    if (wave == 0) {
        unsigned long long ex = 0;
        if (tile != 0) {
            const CountMaskTile count_tile{masks, num_groups, tail, kWaves * kStepMasks};
            ex = scan_exclusive_prefix(counts, prefixes, tile, lane, hdr, count_tile);
        }
        if (lane == 0) s_prefix = ex;
    }
    // the count has reached memory before any wave of the workgroup goes on (see finish_arrive)
    if (publisher) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    const unsigned long long exclusive = uniform(s_prefix);
    unsigned wave_offset = 0, tile_total = 0;
#pragma unroll
    for (int v = 0; v < kWaves; ++v) {
        const unsigned t = uniform(s_wave_total[v]);
        if (v < wave) wave_offset += t;
        tile_total += t;
    }
    if (wave == 0 && lane == 0) {
        if (tile % kBlockTiles == kBlockTiles - 1)
            store64(prefixes + tile / kBlockTiles, kPrefixValid | (exclusive + tile_total));
        finish_arrive(hdr, tile);
    }

    if (wave_elem0 < n)
        expand_step<W, ALIGNED>(s_stage[wave], values, values_avail, exclusive + wave_offset, wave_total, m,
                                wave_elem0, n, out, stream_values, lane);

    if (tile == num_tiles - 1 && wave == 0) finish_call(hdr, counts, num_tiles, lane, state_bytes);
}

// Decoder of the windowed stream.  No scan and no pre-pass: the offset table
// says where a window's bytes are, and a window decodes from its own bytes alone
// (section 5.2: the popcount of a mask gives the offset of the next mask).  The
// kernel works in pieces of 4 KB of output (four 1 KB loads of a wave): it
// stages the piece's bytes in LDS, a few lanes walk the masks one after the
// other -- the serial chain the paper's decoder has too -- and leave every mask
// and the position of its first element for the other lanes, which then rebuild
// 16 bytes of output per load as in the planar decoder.
//   windows of 1, 2 or 4 KB: a wave takes one piece; it holds 4, 2 or 1 windows,
//     and lanes 0..3, 0..1 or 0 walk one window each (8..32 masks of 32-bit
//     elements, twice that of 16-bit ones);
//   windows of 8..64 KB: a wave takes one window and goes through its pieces
//     in order; lane 0 walks, and where its walk ends the next piece begins.
// Reads stay inside [0, stream_bytes) and inside the staged bytes whatever the
// table and the masks say; what a damaged stream asks for beyond that decodes
// as zero.
constexpr int kWindowUnitBytes = 1024;  // one load of a wave; window sizes are 1 KB << shift
constexpr unsigned kMaxWindowShift = 6; // 64 KB

template <int W, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void window_decode_kernel(
    const unsigned char* __restrict__ stream, unsigned long long stream_bytes,
    const unsigned long long* __restrict__ offsets, size_t n, size_t num_groups,
    size_t first_window, size_t num_windows, unsigned window_shift, unsigned char* __restrict__ out,
    bool interleave) {
    constexpr int E = 16 / W;
    constexpr int LPG = 32 / E;
    constexpr int GPL = kWaveSize / LPG;                    // masks per KB of output: 8 | 16
    constexpr int kPieceGroups = kStageLoads * GPL;         // masks per piece: 32 | 64
    constexpr int kUnitElems = GPL * 32;
    constexpr unsigned kPieceBytes = kStageLoads * kWindowUnitBytes;
    constexpr unsigned kMaxBytes = kPieceBytes + 4 * kPieceGroups;   // a piece with nothing dropped
    static_assert(kUnitElems * W == kWindowUnitBytes, "1 KB of output is one load of a wave");

    __shared__ __align__(16) unsigned char s_stage[kWaves][kMaxBytes + 32];   // shift < 16, then an empty mask
    __shared__ unsigned s_mask[kWaves][kPieceGroups];
    __shared__ unsigned s_first[kWaves][kPieceGroups];     // LDS offset of the group's first stored element

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = static_cast<int>(uniform(static_cast<unsigned>(tid / kWaveSize)));
    const unsigned shift_w = window_shift;
    // windows in a piece (small windows) | pieces in a window (large ones)
    const unsigned piece_windows = shift_w <= 2 ? kStageLoads >> shift_w : 1u;
    const unsigned window_pieces = shift_w <= 2 ? 1u : 1u << (shift_w - 2);
    const unsigned walker_groups = static_cast<unsigned>(kPieceGroups) / piece_windows;
    // the wave's share: dealt out in a row or, as in the planar decoder, interleaved over the XCDs
    const size_t share = interleave ? (static_cast<size_t>(blockIdx.x / 8) * kWaves + wave) * 8 + blockIdx.x % 8
                                    : static_cast<size_t>(blockIdx.x) * kWaves + wave;
    const size_t local = share * piece_windows;             // first of the wave's windows, within the range
    if (local >= num_windows) return;
    const size_t window0 = first_window + local;
    const unsigned windows_here =
        num_windows - local < piece_windows ? static_cast<unsigned>(num_windows - local) : piece_windows;
    const size_t units = div_up(num_groups, static_cast<size_t>(GPL));   // KBs of output in the tensor

    const auto clamped = [&](size_t k) {
        const unsigned long long o = offsets[k];
        return o > stream_bytes ? stream_bytes : o;
    };
    unsigned long long lo = clamped(window0);               // where the piece's bytes begin
    unsigned long long hi = clamped(window0 + windows_here);
    if (hi < lo) hi = lo;
    unsigned char* stage = s_stage[wave];

    static_assert(kMaxBytes + 16 <= kFetchSlots * kWaveSize * 16, "a piece fits the fetch slots");

    for (unsigned piece = 0; piece < window_pieces; ++piece) {
        const size_t unit0 = (window0 << shift_w) + static_cast<size_t>(piece) * kStageLoads;
        if (unit0 >= units) break;
        size_t units_left = units - unit0;
        if (shift_w <= 2 && units_left > (static_cast<size_t>(windows_here) << shift_w))
            units_left = static_cast<size_t>(windows_here) << shift_w;
        const unsigned units_here = units_left < kStageLoads ? static_cast<unsigned>(units_left) : kStageLoads;

        // ---- the piece's bytes, clamped to what can be there
        const unsigned cur_bytes = hi - lo > kMaxBytes ? kMaxBytes : static_cast<unsigned>(hi - lo);
        const unsigned char* src = stream + lo;    // wave-uniform, aligned to W
        const unsigned cur_shift = static_cast<unsigned>(reinterpret_cast<uintptr_t>(src) & 15u);
        const unsigned cur_limit = cur_shift + cur_bytes;
        {
            uint4 fetched[kFetchSlots];
            wave_fetch(fetched, src - cur_shift, cur_bytes != 0 ? cur_limit : 0u, false, lane);
            wave_commit(stage, fetched, cur_limit, cur_bytes != 0 ? cur_limit : 0u, lane);
        }
        // an empty mask behind the staged bytes: what the walk reads once it has run out of them
        if (lane == 0) {
            if (W == 4) {
                *reinterpret_cast<unsigned*>(stage + cur_limit) = 0u;
            } else {
                *reinterpret_cast<unsigned short*>(stage + cur_limit) = 0;
                *reinterpret_cast<unsigned short*>(stage + cur_limit + 2) = 0;
            }
        }
        wave_lds_sync();

        // ---- the serial walk: one lane per window of the piece
        unsigned p = cur_limit;   // a window that is not there, or whose offset is off, reads nothing
        if (static_cast<unsigned>(lane) < piece_windows) {
            const size_t group0 = unit0 * GPL + static_cast<size_t>(lane) * walker_groups;
            const unsigned valid_groups =
                static_cast<unsigned>(lane) >= windows_here || group0 >= num_groups ? 0u
                : num_groups - group0 < walker_groups ? static_cast<unsigned>(num_groups - group0)
                                                      : walker_groups;
            if (valid_groups != 0) {
                // a small window begins where the table says; a piece of a large one where the last walk ended
                const unsigned long long o = piece == 0 ? clamped(window0 + lane) : lo;
                if (o >= lo && o - lo <= cur_bytes) p = cur_shift + static_cast<unsigned>(o - lo);
            }
            for (unsigned g = 0; g < walker_groups; ++g) {
                // every step waits for the one before, so the loop has no branch: a mask that is
                // not there (past the window's groups, or past the staged bytes) is read from the
                // empty one behind them
                const unsigned at = g < valid_groups && p + 4u <= cur_limit ? p : cur_limit;
                unsigned m;
                if (W == 4)
                    m = *reinterpret_cast<const unsigned*>(stage + at);
                else
                    m = *reinterpret_cast<const unsigned short*>(stage + at) |
                        (static_cast<unsigned>(*reinterpret_cast<const unsigned short*>(stage + at + 2)) << 16);
                s_mask[wave][lane * walker_groups + g] = m;
                s_first[wave][lane * walker_groups + g] = p + 4u;
                p += 4u + W * __popc(m);
            }
        }
        wave_lds_sync();

        // ---- a large window's next piece begins where lane 0's walk ended (never beyond the
        // window).  (Asking for its bytes here, before this piece is expanded, measured no faster.)
        const bool more = piece + 1 < window_pieces && unit0 + kStageLoads < units;
        unsigned long long next_lo = lo;
        if (more) {
            const unsigned end = lane_value(p, 0);
            const unsigned long long next = lo + ((end < cur_limit ? end : cur_limit) - cur_shift);
            next_lo = next < hi ? next : hi;
        }

        // ---- expand: load jj is KB jj of the piece
        const size_t elem0 = unit0 * kUnitElems;                                  // in the tensor
        unsigned char* wout = out + ((local << shift_w) + static_cast<size_t>(piece) * kStageLoads) *
                                        kWindowUnitBytes;                         // this piece's output
        const bool full = ALIGNED && units_here == kStageLoads && elem0 + kStageLoads * kUnitElems <= n;
#pragma unroll
        for (int jj = 0; jj < kStageLoads; ++jj) {
            if (static_cast<unsigned>(jj) >= units_here) break;
            // element within the piece
            const unsigned in_step = static_cast<unsigned>((jj * kWaveSize + lane) * E);
            const int gl = jj * GPL + lane / LPG;
            const unsigned gm = s_mask[wave][gl];
            const unsigned bit0 = static_cast<unsigned>(lane % LPG) * E;
            unsigned at = s_first[wave][gl] + W * __popc(gm & ((1u << bit0) - 1u));
            const unsigned field = gm >> bit0;
            unsigned d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int c = 0; c < E; ++c) {
                const bool set = ((field >> c) & 1u) != 0u && at + W <= cur_limit;
                const unsigned from = set ? at : cur_shift;
                if (W == 4) {
                    const unsigned v = *reinterpret_cast<const unsigned*>(stage + from);
                    d[c] = set ? v : 0u;
                } else {
                    const unsigned v = *reinterpret_cast<const unsigned short*>(stage + from);
                    d[c >> 1] |= (set ? v : 0u) << (16 * (c & 1));
                }
                at += ((field >> c) & 1u) ? W : 0;
            }
            const size_t e0 = elem0 + in_step;
            if (full || (ALIGNED && e0 + E <= n)) {
                store16_stream(wout + in_step * W, make_uint4(d[0], d[1], d[2], d[3]));
            } else {
#pragma unroll
                for (int c = 0; c < E; ++c) {
                    if (e0 + c < n) {
                        if (W == 4)
                            reinterpret_cast<unsigned*>(wout)[in_step + c] = d[c];
                        else
                            reinterpret_cast<unsigned short*>(wout)[in_step + c] = static_cast<unsigned short>(
                                (d[c >> 1] >> (16 * (c & 1))) & 0xFFFFu);
                    }
                }
            }
        }
        if (!more) break;
        lo = next_lo;
        wave_lds_sync();     // the expand's reads of the stage are done before it is overwritten
    }
}

// Count-only pass (section 5.4's size, without producing the stream).  One
// workgroup per 32 KB of input, all of a thread's loads in flight together.
// A workgroup adds (1 << 40) + its count to one of 64 accumulators with a single
// atomic: the low 40 bits collect kept elements, the high bits count arrivals.
// The workgroup that completes an accumulator bumps finish_top; the one that
// completes finish_top adds the 64 sums up, reports, and leaves the accumulators
// at zero for the next call.
constexpr int kCountLoads = 8;
constexpr int kCountShift = 40;

template <int W, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void count_kernel(const unsigned char* __restrict__ in,
                                                         size_t n, WsHeader* hdr,
                                                         unsigned long long* d_bytes,
                                                         size_t num_groups, unsigned num_tiles) {
    constexpr int E = 16 / W;
    __shared__ unsigned long long s_wave[kWaves];
    __shared__ unsigned s_last;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid / kWaveSize;
    const unsigned tile = blockIdx.x;
    const size_t q0 = static_cast<size_t>(tile) * (kThreads * kCountLoads) + tid;
    uint4 v[kCountLoads];
    if (ALIGNED && (q0 - tid + kThreads * kCountLoads) * E <= n) {
#pragma unroll
        for (int j = 0; j < kCountLoads; ++j)
            v[j] = load16_stream(in + (q0 + static_cast<size_t>(j) * kThreads) * 16);
    } else {
#pragma unroll
        for (int j = 0; j < kCountLoads; ++j)
            v[j] = load_chunk<W, ALIGNED>(in, (q0 + static_cast<size_t>(j) * kThreads) * E, n);
    }
    unsigned long long count = 0;
#pragma unroll
    for (int j = 0; j < kCountLoads; ++j) count += __popc(presence_bits<W, false>(v[j]));
    count = wave_sum(count);
    if (lane == 0) s_wave[wave] = count;
    __syncthreads();
    if (tid == 0) {
        unsigned long long block_total = 0;
        for (int k = 0; k < kWaves; ++k) block_total += s_wave[k];
        const unsigned slot = tile % kFinishLanes;
        const unsigned quota = num_tiles / kFinishLanes + (slot < num_tiles % kFinishLanes ? 1u : 0u);
        const unsigned long long old =
            atomicAdd(&hdr->finish[slot].sum, (1ull << kCountShift) + block_total);
        unsigned last = 0;
        if ((old >> kCountShift) == quota - 1) {
            const unsigned slots_used = num_tiles < kFinishLanes ? num_tiles : kFinishLanes;
            last = atomicAdd(&hdr->finish_top.value, 1u) == slots_used - 1 ? 1u : 0u;
        }
        s_last = last;
    }
    __syncthreads();
    if (s_last == 0u || wave != 0) return;
    const unsigned long long part =
        __hip_atomic_load(&hdr->finish[lane].sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) &
        ((1ull << kCountShift) - 1);
    const unsigned long long total = wave_sum(part);
    hdr->finish[lane].sum = 0ull;
    if (lane == 0) {
        *d_bytes = 4ull * num_groups + static_cast<unsigned long long>(W) * total;
        hdr->finish_top.value = 0u;
    }
}

// Measurement aid, not part of the method: a plain streaming kernel that reads
// read_chunks 16-byte chunks and writes write_chunks of them, split evenly over
// the workgroups (up to 64 KB each way per workgroup, non-temporal accesses, all
// of a thread's loads in flight together, stores that depend on the loads).  It
// shows what this memory system does with the traffic of a codec call when
// nothing else is asked of the kernel.  LOADS 16-byte loads per thread: 64 KB
// per workgroup, or 16 KB for small transfers (more workgroups than CUs).
template <int LOADS>
__global__ __launch_bounds__(kThreads) void reference_stream_kernel(const uint4* __restrict__ in,
                                                                    size_t read_chunks, uint4* __restrict__ out,
                                                                    size_t write_chunks, unsigned read_per_group,
                                                                    unsigned write_per_group) {
    const size_t r0 = static_cast<size_t>(blockIdx.x) * read_per_group;
    const size_t w0 = static_cast<size_t>(blockIdx.x) * write_per_group;
    uint4 v[LOADS];
    unsigned mix = blockIdx.x;
#pragma unroll
    for (int k = 0; k < LOADS; ++k) {
        const unsigned i = threadIdx.x + k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (i < read_per_group && r0 + i < read_chunks) v[k] = load16_stream(in + r0 + i);
    }
#pragma unroll
    for (int k = 0; k < LOADS; ++k) mix ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
#pragma unroll
    for (int k = 0; k < LOADS; ++k) {
        const unsigned i = threadIdx.x + k * kThreads;
        if (i < write_per_group && w0 + i < write_chunks) {
            uint4 d = v[k];
            d.x ^= mix;
            store16_stream(out + w0 + i, d);
        }
    }
}

// -------------------------------------------------------------- host helpers
// log2(window_bytes / 1 KB) for the window sizes of the windowed stream (a power of
// two from 1 KB to 64 KB), else -1.
inline int window_shift_of(size_t window_bytes) {
    for (unsigned k = 0; k <= kMaxWindowShift; ++k)
        if (window_bytes == static_cast<size_t>(kWindowUnitBytes) << k) return static_cast<int>(k);
    return -1;
}

inline bool aligned_to(const void* p, size_t a) {
    return reinterpret_cast<uintptr_t>(p) % a == 0;
}

inline bool ranges_overlap(const void* a, size_t an, const void* b, size_t bn) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return an != 0 && bn != 0 && a0 < b0 + bn && b0 < a0 + an;
}

inline zvc_status hip_ok(hipError_t e) { return e == hipSuccess ? ZVC_OK : ZVC_E_HIP; }

// Kernel launch that reports its own status (hipGetLastError after a <<<>>> launch
// would also report, and clear, an earlier error of the calling thread).
template <typename... Params, size_t... I>
hipError_t launch_impl(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream,
                       std::tuple<Params...>& values, std::index_sequence<I...>) {
    void* pointers[] = {static_cast<void*>(&std::get<I>(values))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, pointers, 0, stream);
}
template <typename... Params, typename... Args>
hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args... args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<Params...> values{static_cast<Params>(args)...};
    return launch_impl(kernel, grid, block, stream, values, std::index_sequence_for<Params...>{});
}

// Zeroes the header and the first state_bytes bytes of scan state.
zvc_status launch_reset(void* d_ws, size_t state_bytes, hipStream_t stream) {
    const size_t words = (kHeaderBytes + state_bytes) / 8;
    const unsigned blocks = static_cast<unsigned>(div_up(words, 256) < 1024 ? div_up(words, 256) : 1024);
    return hip_ok(launch(reset_kernel, dim3(blocks), dim3(256), stream,
                         static_cast<unsigned long long*>(d_ws), words));
}

// Where the scan state of a call with `tiles` tiles lives inside the workspace.
struct ScanState {
    WsHeader* hdr;
    unsigned* counts;
    unsigned long long* prefixes;
};
inline ScanState scan_state(void* d_ws, size_t tiles) {
    unsigned char* base = static_cast<unsigned char*>(d_ws);
    return ScanState{reinterpret_cast<WsHeader*>(base),
                     reinterpret_cast<unsigned*>(base + kHeaderBytes),
                     reinterpret_cast<unsigned long long*>(base + kHeaderBytes + counts_bytes(tiles))};
}

zvc_status check_workspace(const void* d_ws, size_t ws, size_t n, int w) {
    if (d_ws == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_ws, 256)) return ZVC_E_ALIGN;
    if (ws < zvc_workspace_bytes(n, w)) return ZVC_E_WORKSPACE;
    return ZVC_OK;
}


// Shape of the encoder's tile: chunks per wave x waves per workgroup.  Each tile
// costs a fixed few nanoseconds of chip-wide time (workgroup launch plus the
// scan's state traffic), so large fp32 tensors use 64 KB tiles; smaller tensors
// use smaller tiles so that every CU still gets several.  16-bit elements are
// twice the vector work per byte, and the 32 KB tile's eight waves per SIMD
// (against four) hide it better: 32 KB tiles measure up to 9 % faster than
// 64 KB ones at 411 MB, 822 MB and 1.6 GB alike.  The limits are measured
// crossover points (8 KB tiles, and 8 or 16 waves per tile, were no faster
// at any size).
struct TileShape {
    int chunks;   // per wave: 16, 32 or 64
    int waves;    // per workgroup
};
constexpr size_t kLargeTensorBytes = size_t{160} << 20;   // (cold inputs: 64 KB tiles are 4-6 % ahead at 205 MB, 2 % behind at 103 MB)
constexpr size_t kMediumTensorBytes = size_t{12} << 20;
constexpr TileShape kMinShape{16, 4};             // 16 KB, the smallest tile (sizes the workspace)
static_assert(kMinShape.chunks * kMinShape.waves * kChunkBytes == kMinLoads * 16 * kThreads, "smallest tile");

inline TileShape choose_shape(size_t n, int w, bool split, bool windowed) {
    if (split) return kMinShape;
    const size_t bytes = n * static_cast<size_t>(w);
    // (the windowed stream's encoder gains nothing from 64 KB tiles at 822 MB and loses 20 % with
    // them on the 297 MB tensor whose channels differ widely in density)
    return bytes >= kLargeTensorBytes && w == 4 && !windowed ? TileShape{64, 4}
         : bytes >= kMediumTensorBytes ? TileShape{32, 4} : kMinShape;
}

enum class Encoder { kPlain, kRelu, kWindowed };

template <int W, int CH, int WV, bool SPLIT, bool WINDOWED_TOO = true>
hipError_t launch_compress_as(Encoder mode, hipStream_t stream, const unsigned char* in, size_t n,
                        unsigned* masks, unsigned char* values, ScanState st,
                        unsigned long long* d_bytes, unsigned tiles, size_t groups,
                        unsigned long long cap_values, unsigned long long* offsets, unsigned window_shift) {
    const EncoderArgs args{in, n, masks, values, st.hdr, st.counts, st.prefixes, d_bytes, tiles,
                           groups, scan_state_bytes(tiles), cap_values, offsets, window_shift};
    const dim3 grid(tiles), block(WV * kWaveSize);
    switch (mode) {
        case Encoder::kPlain:
            return launch(compress_kernel<W, CH, WV, false, false, SPLIT>, grid, block, stream, args);
        case Encoder::kRelu:
            return launch(compress_kernel<W, CH, WV, true, false, SPLIT>, grid, block, stream, args);
        case Encoder::kWindowed:
            if constexpr (WINDOWED_TOO)
                return launch(compress_kernel<W, CH, WV, false, true, SPLIT>, grid, block, stream, args);
            else
                return hipErrorInvalidValue;   // choose_shape() gives the windowed stream no such tile
    }
    return hipErrorInvalidValue;
}

// Tensors below this size decode in one launch (decompress_scan_kernel): measured 1-2.5 us
// faster than pre-pass + expand up to 19 MB, slower from 26 MB up.
constexpr size_t kScanDecoderBytes = size_t{16} << 20;

// Tensors below this size never decode in the interleaved order (no gain there).
inline bool interleaves(size_t n, int w) { return n * static_cast<size_t>(w) >= (size_t{64} << 20); }

template <int W, int LOADS, bool ALIGNED>
hipError_t launch_decompress_as(dim3 grid, hipStream_t stream, const unsigned* masks,
                          const unsigned char* values, unsigned long long avail, size_t n,
                          unsigned char* out, const unsigned* unit_end,
                          const unsigned long long* chunk_prefix, const unsigned* chunk_total,
                          size_t groups) {
    // Dense streams (3/4 of the elements stored, or more) are read with the streaming
    // hint: little of a cache line is then shared between waves, and the hint is worth
    // 5 % there; sparser streams are read through the caches (see load16_stream).
    const bool stream_values = avail >= n / 4 * 3;
    // Order in which the parts of the tensor are dealt out to the workgroups (see the
    // kernel): interleaved where it measures faster, 2-15 % below a twelfth and 2-5 %
    // above a third of the elements stored; in between the plain order is 1 % ahead.
    const bool interleave = (avail < n / 12 || avail > n / 3) && interleaves(n, W);
    return launch(decompress_kernel<W, LOADS, ALIGNED>, grid, dim3(kThreads), stream,
                  masks, values, avail, n, out, unit_end, chunk_prefix, chunk_total, groups, stream_values,
                  interleave);
}

// Picks the instantiation for (w, tile shape).  16-bit elements at an odd half
// dword always use the smallest tile.
template <typename... Args>
hipError_t launch_compress(int w, TileShape shape, bool split, Args... args) {
    if (split) return launch_compress_as<2, kMinShape.chunks, kMinShape.waves, true>(args...);
#define ZVC_SHAPE_CASE(C, V)                                                    \
    if (shape.chunks == C && shape.waves == V)                                  \
        return w == 4 ? launch_compress_as<4, C, V, false>(args...)             \
                      : launch_compress_as<2, C, V, false>(args...);
    if (shape.chunks == 64 && shape.waves == 4 && w == 4) return launch_compress_as<4, 64, 4, false, false>(args...);
    ZVC_SHAPE_CASE(32, 4)
    ZVC_SHAPE_CASE(16, 4)
#undef ZVC_SHAPE_CASE
    return hipErrorInvalidValue;   // choose_shape() returns nothing else
}

// The decoder has one tile size (its waves are independent; one staging step per
// wave measures best at every size) and a path for outputs that are not
// 16-byte aligned.
template <typename... Args>
hipError_t launch_decompress(int w, bool aligned, Args... args) {
    if (!aligned)
        return w == 4 ? launch_decompress_as<4, kMinLoads, false>(args...)
                      : launch_decompress_as<2, kMinLoads, false>(args...);
    return w == 4 ? launch_decompress_as<4, kMinLoads, true>(args...)
                  : launch_decompress_as<2, kMinLoads, true>(args...);
}

// `bounded`: out_cap may be anything from the size of the mask area up; the
// kernel then writes only runs that end inside it.
// `scan_state_only`: the workspace need only hold the header and the scan state
// of this call's tiles (the library's own scratch array, which no decoder uses).
zvc_status compress_impl(Encoder mode, bool bounded, const void* d_in, size_t n, int w, void* d_out,
                         size_t out_cap, uint64_t* d_bytes, uint64_t* d_offsets, void* d_ws, size_t ws,
                         hipStream_t stream, bool scan_state_only = false, unsigned window_shift = 0) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (d_bytes == nullptr || ((d_in == nullptr || d_out == nullptr) && n != 0)) return ZVC_E_ARG;
    if (!aligned_to(d_in, static_cast<size_t>(w)) || !aligned_to(d_out, 4) ||
        !aligned_to(d_bytes, 8))
        return ZVC_E_ALIGN;
    const size_t worst = zvc_max_compressed_bytes(n, w);
    if (out_cap < (bounded ? zvc_mask_bytes(n) : worst)) return ZVC_E_CAPACITY;
    if (ranges_overlap(d_in, n * static_cast<size_t>(w), d_out, out_cap < worst ? out_cap : worst))
        return ZVC_E_ARG;
    if (!scan_state_only)
        if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    unsigned long long* out_bytes = reinterpret_cast<unsigned long long*>(d_bytes);
    if (n == 0) {
        hipError_t e = launch(write_word_kernel, dim3(1), dim3(1), stream, out_bytes, 0ull);
        if (e == hipSuccess && mode == Encoder::kWindowed)
            e = launch(write_word_kernel, dim3(1), dim3(1), stream,
                       reinterpret_cast<unsigned long long*>(d_offsets), 0ull);
        return hip_ok(e);
    }
    const bool split = !aligned_to(d_in, 4);        // 16-bit elements at an odd half dword
    const TileShape shape = choose_shape(n, w, split, mode == Encoder::kWindowed);
    const size_t tiles = div_up(n * static_cast<size_t>(w), static_cast<size_t>(shape.waves) * shape.chunks * kChunkBytes);
    if (tiles > 0x7FFFFFFFull) return ZVC_E_ARG;
    if (scan_state_only && kHeaderBytes + scan_state_bytes(tiles) > ws) return ZVC_E_WORKSPACE;
    // the scan state is zero between calls: the kernel cleans up after itself
    const size_t groups = div_up(n, 32);
    const unsigned char* in = static_cast<const unsigned char*>(d_in);
    unsigned* masks = static_cast<unsigned*>(d_out);
    unsigned char* values = static_cast<unsigned char*>(d_out) + 4 * groups;
    return hip_ok(launch_compress(w, shape, split, mode, stream, in, n, masks,
                    mode == Encoder::kWindowed ? static_cast<unsigned char*>(d_out) : values,
                    scan_state(d_ws, tiles), out_bytes, static_cast<unsigned>(tiles), groups,
                    !bounded ? ~0ull : out_cap - (mode == Encoder::kWindowed ? 0 : 4 * groups),
                    reinterpret_cast<unsigned long long*>(d_offsets), window_shift));
}

// One event per host thread and GPU for ordering a copy stream after a compute
// stream (or the other way round), created at first use and kept: creating and
// destroying one per call costs several microseconds per tensor.
hipEvent_t thread_event() {
    thread_local hipEvent_t events[kMaxDevices] = {};
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return nullptr;
    if (events[device] == nullptr &&
        hipEventCreateWithFlags(&events[device], hipEventDisableTiming) != hipSuccess)
        events[device] = nullptr;
    return events[device];
}

zvc_status offload_impl(Encoder mode, const void* d_in, size_t n, int w, void* d_stage,
                        size_t stage_cap, void* h_pinned, size_t h_cap, uint64_t* h_bytes, void* d_ws,
                        size_t ws, hipStream_t compute, hipStream_t copy) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (h_bytes == nullptr || (h_pinned == nullptr && n != 0)) return ZVC_E_ARG;
    if (h_cap < zvc_max_compressed_bytes(n, w)) return ZVC_E_CAPACITY;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);
    uint64_t* d_size = reinterpret_cast<uint64_t*>(&hdr->size_word);
    // the size word sits in the header and survives until the next offload on this workspace
    if (zvc_status st = compress_impl(mode, false, d_in, n, w, d_stage, stage_cap, d_size, nullptr, d_ws,
                                      ws, compute))
        return st;
    if (hipMemcpyAsync(h_bytes, d_size, 8, hipMemcpyDeviceToHost, compute) != hipSuccess)
        return ZVC_E_HIP;
    hipEvent_t ev = thread_event();
    if (ev == nullptr) return ZVC_E_HIP;
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
    return st;
}

// Scratch of zvc_compress_static: header and scan state for tensors of up to
// ZVC_STATIC_MAX_BYTES.  Zero when the code object is loaded, which is the
// state zvc_workspace_init gives a caller's workspace, and every call leaves it
// zero again.  Each GPU holds its own copy at its own address.
constexpr size_t kStaticScratchBytes = ZVC_STATIC_SCRATCH_BYTES;   // covers 16 KB tiles (the smallest) up to the limit
static_assert(kHeaderBytes + 4 * (ZVC_STATIC_MAX_BYTES / (kMinLoads * 16 * kThreads)) + 8 * (ZVC_STATIC_MAX_BYTES / (kMinLoads * 16 * kThreads) / kBlockTiles) + 512 <= ZVC_STATIC_SCRATCH_BYTES, "scratch holds the scan state of the largest call");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];           // device address of `scratch` on each GPU, once looked up

// Device address of the current GPU's copy of `scratch` (looked up once per GPU).
zvc_status static_scratch(void** ptr) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return ZVC_E_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return ZVC_E_HIP;
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return ZVC_OK;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

const char* zvc_status_string(int status) {
    switch (status) {
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
    const size_t tiles = tiles_for(n, w, kMinLoads);
    return kHeaderBytes + scan_state_bytes(tiles) +
           decoder_area_bytes(div_up(div_up(n, 32), kChunkMasks));
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

zvc_status zvc_window_check_stream(const void* h_stream, uint64_t bytes, const uint64_t* h_offsets,
                                   size_t n, int w, size_t window_bytes) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (window_shift_of(window_bytes) < 0) return ZVC_E_ARG;
    if (h_offsets == nullptr || (h_stream == nullptr && bytes != 0)) return ZVC_E_ARG;
    const size_t windows = zvc_window_count(n, w, window_bytes);
    const size_t groups = div_up(n, 32);
    const size_t groups_per_window = window_bytes / static_cast<size_t>(w) / 32;
    const unsigned char* p = static_cast<const unsigned char*>(h_stream);
    if (h_offsets[0] != 0 || h_offsets[windows] != bytes) return ZVC_E_CORRUPT;
    for (size_t k = 0; k < windows; ++k) {
        uint64_t pos = h_offsets[k];
        const uint64_t end = h_offsets[k + 1];
        if (end < pos || end > bytes) return ZVC_E_CORRUPT;
        const size_t g0 = k * groups_per_window;
        const size_t g1 = g0 + groups_per_window < groups ? g0 + groups_per_window : groups;
        for (size_t g = g0; g < g1; ++g) {      // the walk of section 5.2: mask, then its popcount of elements
            if (pos + 4 > end) return ZVC_E_CORRUPT;
            const uint32_t m = static_cast<uint32_t>(p[pos]) | (static_cast<uint32_t>(p[pos + 1]) << 8) |
                               (static_cast<uint32_t>(p[pos + 2]) << 16) |
                               (static_cast<uint32_t>(p[pos + 3]) << 24);
            if (g == groups - 1 && n % 32 != 0 && (m >> (n % 32)) != 0) return ZVC_E_CORRUPT;
            pos += 4 + static_cast<uint64_t>(w) * static_cast<uint64_t>(__builtin_popcount(m));
        }
        if (pos != end) return ZVC_E_CORRUPT;
    }
    return ZVC_OK;
}

zvc_status zvc_workspace_init(void* d_ws, size_t ws, hipStream_t stream) {
    if (d_ws == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_ws, 256)) return ZVC_E_ALIGN;
    if (ws < kHeaderBytes) return ZVC_E_WORKSPACE;
    return launch_reset(d_ws, (ws - kHeaderBytes) / 8 * 8, stream);
}

zvc_status zvc_workspace_set_lookback_patience(void* d_ws, unsigned polls, hipStream_t stream) {
    if (d_ws == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_ws, 256)) return ZVC_E_ALIGN;
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);
    return hip_ok(launch(write_word_kernel, dim3(1), dim3(1), stream, &hdr->patience_plus_one,
                         static_cast<unsigned long long>(polls) + 1ull));
}

zvc_status zvc_reference_stream(const void* d_in, size_t read_bytes, void* d_out, size_t write_bytes,
                                hipStream_t stream) {
    if ((d_in == nullptr && read_bytes != 0) || (d_out == nullptr && write_bytes != 0)) return ZVC_E_ARG;
    if (!aligned_to(d_in, 16) || !aligned_to(d_out, 16) || read_bytes % 16 != 0 || write_bytes % 16 != 0)
        return ZVC_E_ALIGN;
    if (ranges_overlap(d_in, read_bytes, d_out, write_bytes)) return ZVC_E_ARG;
    const size_t larger = read_bytes > write_bytes ? read_bytes : write_bytes;
    if (larger == 0) return ZVC_OK;
    const bool small = larger < (size_t{32} << 20);
    const size_t group_bytes = static_cast<size_t>(kThreads) * 16 * (small ? 4 : 16);     // 16 KB | 64 KB
    const size_t groups = div_up(larger, group_bytes);
    if (groups > 0x7FFFFFFFull) return ZVC_E_ARG;
    const size_t read_chunks = read_bytes / 16, write_chunks = write_bytes / 16;
    return hip_ok(launch(small ? reference_stream_kernel<4> : reference_stream_kernel<16>,
                         dim3(static_cast<unsigned>(groups)), dim3(kThreads), stream,
                         static_cast<const uint4*>(d_in), read_chunks, static_cast<uint4*>(d_out), write_chunks,
                         static_cast<unsigned>(div_up(read_chunks, groups)),
                         static_cast<unsigned>(div_up(write_chunks, groups))));
}

zvc_status zvc_workspace_self_help_count(const void* d_ws, uint64_t* h_count) {
    if (d_ws == nullptr || h_count == nullptr) return ZVC_E_ARG;
    const WsHeader* hdr = static_cast<const WsHeader*>(d_ws);
    return hip_ok(hipMemcpy(h_count, &hdr->helped, 8, hipMemcpyDeviceToHost));
}

zvc_status zvc_compressed_size(const void* d_in, size_t n, int w, uint64_t* d_bytes, void* d_ws,
                               size_t ws, hipStream_t stream) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (d_bytes == nullptr || (d_in == nullptr && n != 0)) return ZVC_E_ARG;
    if (!aligned_to(d_in, static_cast<size_t>(w)) || !aligned_to(d_bytes, 8)) return ZVC_E_ALIGN;
    if (zvc_status st = check_workspace(d_ws, ws, n, w)) return st;
    unsigned long long* out = reinterpret_cast<unsigned long long*>(d_bytes);
    if (n == 0) {
        return hip_ok(launch(write_word_kernel, dim3(1), dim3(1), stream, out, 0ull));
    }
    WsHeader* hdr = static_cast<WsHeader*>(d_ws);   // accumulators are zero between calls
    const unsigned char* in = static_cast<const unsigned char*>(d_in);
    const size_t groups = div_up(n, 32);
    const size_t tiles = div_up(n * static_cast<size_t>(w), static_cast<size_t>(kThreads) * 16 * kCountLoads);
    if (tiles > 0x7FFFFFFFull) return ZVC_E_ARG;
    const dim3 grid(static_cast<unsigned>(tiles)), block(kThreads);
    const unsigned nt = static_cast<unsigned>(tiles);
    const bool al = aligned_to(d_in, 16);
    const auto kernel = w == 4 ? (al ? count_kernel<4, true> : count_kernel<4, false>)
                               : (al ? count_kernel<2, true> : count_kernel<2, false>);
    return hip_ok(launch(kernel, grid, block, stream, in, n, hdr, out, groups, nt));
}

zvc_status zvc_compress(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                        uint64_t* d_bytes, void* d_ws, size_t ws, hipStream_t stream) {
    return compress_impl(Encoder::kPlain, false, d_in, n, w, d_out, out_cap, d_bytes, nullptr, d_ws, ws,
                         stream);
}

zvc_status zvc_compress_static(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                               uint64_t* d_bytes, hipStream_t stream) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    if (n > ZVC_STATIC_MAX_BYTES / static_cast<size_t>(w)) return ZVC_E_WORKSPACE;
    void* ws = nullptr;
    if (zvc_status st = static_scratch(&ws)) return st;
    return compress_impl(Encoder::kPlain, false, d_in, n, w, d_out, out_cap, d_bytes, nullptr, ws,
                         kStaticScratchBytes, stream, true);
}

zvc_status zvc_relu_compress(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                             uint64_t* d_bytes, void* d_ws, size_t ws, hipStream_t stream) {
    return compress_impl(Encoder::kRelu, false, d_in, n, w, d_out, out_cap, d_bytes, nullptr, d_ws, ws,
                         stream);
}

zvc_status zvc_compress_bounded(const void* d_in, size_t n, int w, int relu, void* d_out, size_t out_cap,
                                uint64_t* d_bytes, void* d_ws, size_t ws, hipStream_t stream) {
    if (relu != 0 && relu != 1) return ZVC_E_ARG;
    return compress_impl(relu ? Encoder::kRelu : Encoder::kPlain, true, d_in, n, w, d_out, out_cap,
                         d_bytes, nullptr, d_ws, ws, stream);
}

size_t zvc_window_elements(int w, size_t window_bytes) {
    if ((w != 2 && w != 4) || window_shift_of(window_bytes) < 0) return 0;
    return window_bytes / static_cast<size_t>(w);
}

size_t zvc_window_count(size_t n, int w, size_t window_bytes) {
    if ((w != 2 && w != 4) || window_shift_of(window_bytes) < 0) return 0;
    return div_up(n * static_cast<size_t>(w), window_bytes);
}

zvc_status zvc_window_compress(const void* d_in, size_t n, int w, size_t window_bytes, void* d_out,
                               size_t out_cap, uint64_t* d_offsets, uint64_t* d_bytes, void* d_ws,
                               size_t ws, hipStream_t stream) {
    if (d_offsets == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_offsets, 8)) return ZVC_E_ALIGN;
    const int shift = window_shift_of(window_bytes);
    if (shift < 0) return ZVC_E_ARG;
    if (w == 2 || w == 4) {
        const size_t table = 8 * (zvc_window_count(n, w, window_bytes) + 1);
        if (ranges_overlap(d_offsets, table, d_out, zvc_max_compressed_bytes(n, w)) ||
            ranges_overlap(d_offsets, table, d_in, n * static_cast<size_t>(w)))
            return ZVC_E_ARG;
    }
    return compress_impl(Encoder::kWindowed, false, d_in, n, w, d_out, out_cap, d_bytes, d_offsets, d_ws, ws,
                         stream, false, static_cast<unsigned>(shift));
}

zvc_status zvc_window_decompress(const void* d_stream, size_t stream_bytes, const uint64_t* d_offsets,
                                 size_t n, int w, size_t window_bytes, size_t first_window,
                                 size_t num_windows, void* d_out, hipStream_t stream) {
    if (w != 2 && w != 4) return ZVC_E_WIDTH;
    const int shift = window_shift_of(window_bytes);
    if (shift < 0) return ZVC_E_ARG;
    const size_t windows = zvc_window_count(n, w, window_bytes);
    if (first_window > windows || num_windows > windows - first_window) return ZVC_E_ARG;
    if (num_windows == 0) return ZVC_OK;
    if (d_stream == nullptr || d_offsets == nullptr || d_out == nullptr) return ZVC_E_ARG;
    if (!aligned_to(d_out, static_cast<size_t>(w)) || !aligned_to(d_stream, static_cast<size_t>(w)) ||
        !aligned_to(d_offsets, 8))
        return ZVC_E_ALIGN;
    const size_t elems_per_window = window_bytes / static_cast<size_t>(w);
    const size_t last_elem = (first_window + num_windows) * elems_per_window < n
                                 ? (first_window + num_windows) * elems_per_window : n;
    const size_t out_bytes = (last_elem - first_window * elems_per_window) * static_cast<size_t>(w);
    if (ranges_overlap(d_stream, stream_bytes, d_out, out_bytes)) return ZVC_E_ARG;
    // a wave takes 4 KB of output, or one window if that is more
    const size_t wave_windows = shift <= 2 ? static_cast<size_t>(kStageLoads >> shift) : 1;
    // (a multiple of 8 workgroups for the interleaved order)
    const size_t blocks = div_up(div_up(num_windows, static_cast<size_t>(kWaves) * wave_windows), 8) * 8;
    if (blocks > 0x7FFFFFFFull) return ZVC_E_ARG;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    const unsigned char* in = static_cast<const unsigned char*>(d_stream);
    const unsigned long long* offs = reinterpret_cast<const unsigned long long*>(d_offsets);
    unsigned char* out = static_cast<unsigned char*>(d_out);
    const size_t groups = div_up(n, 32);
    const bool al = aligned_to(d_out, 16);
    // dense streams of large ranges decode 3-8 % faster in the interleaved order, others slower
    const bool interleave = stream_bytes / 3 > n * static_cast<size_t>(w) / 4 && out_bytes >= (size_t{64} << 20);
    const auto kernel = w == 4 ? (al ? window_decode_kernel<4, true> : window_decode_kernel<4, false>)
                               : (al ? window_decode_kernel<2, true> : window_decode_kernel<2, false>);
    return hip_ok(launch(kernel, grid, block, stream, in, static_cast<unsigned long long>(stream_bytes), offs, n,
                         groups, first_window, num_windows, static_cast<unsigned>(shift), out, interleave));
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
    const bool al = aligned_to(d_out, 16);
    // a multiple of 8 workgroups: the interleaved order deals the parts out in rounds of 8
    const size_t tiles = div_up(tiles_for(n, w, kMinLoads), 8) * 8;
    if (tiles > 0x7FFFFFFFull) return ZVC_E_ARG;
    const size_t groups = div_up(n, 32);
    const unsigned char* stream_values_at = static_cast<const unsigned char*>(d_comp) + 4 * groups;
    const unsigned long long stored_avail = (comp_bytes - 4 * groups) / static_cast<size_t>(w);
    if (n * static_cast<size_t>(w) < kScanDecoderBytes) {
        // one launch: the workgroups find their offsets with the encoder's scan (its state is at
        // the front of the workspace, zero between calls)
        const size_t scan_tiles = tiles_for(n, w, kMinLoads);
        const ScanState st = scan_state(d_ws, scan_tiles);
        const bool stream_values = stored_avail >= n / 4 * 3;
        const auto kernel = w == 4 ? (al ? decompress_scan_kernel<4, true> : decompress_scan_kernel<4, false>)
                                   : (al ? decompress_scan_kernel<2, true> : decompress_scan_kernel<2, false>);
        return hip_ok(launch(kernel, dim3(static_cast<unsigned>(scan_tiles)), dim3(kThreads), stream,
                             static_cast<const unsigned*>(d_comp), stream_values_at, stored_avail, n,
                             static_cast<unsigned char*>(d_out), st.hdr, st.counts, st.prefixes,
                             static_cast<unsigned>(scan_tiles), scan_state_bytes(scan_tiles), groups,
                             stream_values));
    }
    const size_t chunks = div_up(groups, kChunkMasks);
    if (chunks > 0xFFFFFFFFull) return ZVC_E_ARG;
    // The pre-pass arrays need no reset.  They sit at the end of the workspace, whatever its
    // size: an encoder call that this workspace is large enough for keeps its scan state
    // (which must stay zero between calls) below them, whichever call came first.
    unsigned char* area = static_cast<unsigned char*>(d_ws) + (ws - decoder_area_bytes(chunks)) / 256 * 256;
    unsigned long long* chunk_prefix =
        chunks <= kFewChunks ? nullptr : reinterpret_cast<unsigned long long*>(area);
    unsigned* chunk_total = reinterpret_cast<unsigned*>(area + pad256(8 * chunks));
    unsigned* unit_end = reinterpret_cast<unsigned*>(area + pad256(8 * chunks) + pad256(4 * chunks));
    const unsigned* masks = static_cast<const unsigned*>(d_comp);
    if (launch(mask_prefix_kernel, dim3(static_cast<unsigned>(chunks)), dim3(kThreads), stream, masks,
               groups, static_cast<unsigned>(n % 32), unit_end, chunk_total, chunk_prefix,
               static_cast<WsHeader*>(d_ws), static_cast<unsigned>(chunks)) != hipSuccess)
        return ZVC_E_HIP;
    const unsigned char* values = static_cast<const unsigned char*>(d_comp) + 4 * groups;
    const unsigned long long avail = (comp_bytes - 4 * groups) / static_cast<size_t>(w);
    return hip_ok(launch_decompress(w, al, dim3(static_cast<unsigned>(tiles)), stream, masks, values, avail, n,
                                    static_cast<unsigned char*>(d_out), unit_end, chunk_prefix, chunk_total,
                                    groups));
}

zvc_status zvc_offload(const void* d_in, size_t n, int w, void* d_stage, size_t stage_cap,
                       void* h_pinned, size_t h_cap, uint64_t* h_bytes, void* d_ws, size_t ws,
                       hipStream_t compute, hipStream_t copy) {
    return offload_impl(Encoder::kPlain, d_in, n, w, d_stage, stage_cap, h_pinned, h_cap, h_bytes, d_ws,
                        ws, compute, copy);
}

zvc_status zvc_relu_offload(const void* d_in, size_t n, int w, void* d_stage, size_t stage_cap,
                            void* h_pinned, size_t h_cap, uint64_t* h_bytes, void* d_ws, size_t ws,
                            hipStream_t compute, hipStream_t copy) {
    return offload_impl(Encoder::kRelu, d_in, n, w, d_stage, stage_cap, h_pinned, h_cap, h_bytes, d_ws,
                        ws, compute, copy);
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
        hipEvent_t ev = thread_event();
        if (ev == nullptr || hipEventRecord(ev, copy) != hipSuccess ||
            hipStreamWaitEvent(compute, ev, 0) != hipSuccess)
            return ZVC_E_HIP;
    }
    return zvc_decompress(d_stage, bytes, n, w, d_out, d_ws, ws, compute);
}

}  // extern "C"

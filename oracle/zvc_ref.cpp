// Zero-value compression (ZVC) reference oracle.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
// definition that the GPU library is checked against.  Nothing on the product
// path may include, link or call it, and it shares no code with the GPU path.
// Plain single-threaded C++17, no intrinsics, no SIMD, no blocking or fusion.
//
// What it computes (paper section 5.1, "Zero-value compression"; encoder and
// decoder pipelines of section 5.2, "(De)compression engine
// microarchitecture"):
//   * the tensor is a flat run of n elements, each w bytes wide (w = 2 or 4);
//   * every 32 consecutive elements form one group with one 32-bit presence
//     mask: bit b is 1 when element 32*g + b is non-zero, 0 when it is zero;
//   * the non-zero elements follow in their original order; zeros are dropped;
//   * decoding walks the mask bits, consuming one stored element per 1 bit and
//     emitting a zero element per 0 bit; the scheme is lossless.
//
// Readings taken where the paper leaves a choice (parity for choices 1 and 2
// is "unpinned": the paper's worked figure is not available to check them):
//   1. stream order: all masks first (4*ceil(n/32) bytes, little-endian
//      uint32), then all kept elements (w*nnz bytes).  The byte count is the
//      same as for the paper's mask-then-its-elements interleaving.
//   2. bit order: bit 0 (least significant) is the first element of the group.
//   3. "zero" is the all-zero bit pattern; -0.0, NaN and denormals are kept.
//   4. a ragged tail group has zero bits past n and stores nothing for them.
//   5. (fused ReLU + ZVC, zvc_ref_relu*) the elements are IEEE-style numbers
//      with the sign in the top bit (fp32, fp16, bf16).  ReLU keeps an element
//      unchanged when its sign bit is clear and it is not +0, and turns every
//      other element into +0.  So every positive number, denormals and +inf
//      included, is kept; -0.0 and all negative numbers become +0; a NaN is
//      kept when its sign bit is clear and dropped when it is set (max(0, NaN)
//      is 0 by IEEE maxNum and NaN in common frameworks: no choice matches
//      all, this one needs no floating-point mode).
//   6. (paper-order stream, zvc_ref_window*) section 5.1 appends a group's
//      non-zero elements right after its mask; section 6 has the DMA engine
//      work on windows of 4 KB of uncompressed data.  The windowed stream is
//      that order: window after window, inside a window group after group,
//      for each group its mask (4 bytes, little-endian, at whatever byte
//      offset it falls on) and then its kept elements.  Windows are packed
//      back to back with no padding, so the byte count equals that of reading
//      1.  A table of K+1 byte offsets (window k occupies [offsets[k],
//      offsets[k+1])) makes every window decodable on its own; the paper does
//      not say how it finds a window, the table is this build's addition and
//      is not counted in the compressed size.
//
// Entry points are extern "C" so tests can bind them with ctypes.

#include <cstddef>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// The w bytes of element i, widened to an unsigned integer.  memcpy keeps this
// an integer comparison whatever the element's floating-point meaning is.
uint32_t element_bits(const unsigned char* in, size_t i, int w) {
    uint32_t word = 0;
    if (w == 4) {
        uint32_t v;
        std::memcpy(&v, in + i * 4, 4);
        word = v;
    } else {
        uint16_t v;
        std::memcpy(&v, in + i * 2, 2);
        word = v;
    }
    return word;
}

}  // namespace

extern "C" {

// Number of 32-element groups covering n elements (section 5.1: window of 32).
uint64_t zvc_ref_groups(uint64_t n) { return n / 32 + (n % 32 != 0 ? 1 : 0); }

// Encode.  in: n elements of w bytes.  masks: room for zvc_ref_groups(n)
// words.  values: room for n*w bytes.  Returns nnz, the number of kept
// elements, or UINT64_MAX when w is not 2 or 4.
// Section 5.1: one mask per 32 values, non-zero elements appended in order.
uint64_t zvc_ref_compress(const void* in_, uint64_t n, int w, uint32_t* masks,
                          void* values_) {
    if (w != 2 && w != 4) return UINT64_MAX;
    const unsigned char* in = static_cast<const unsigned char*>(in_);
    unsigned char* values = static_cast<unsigned char*>(values_);
    const uint64_t groups = zvc_ref_groups(n);
    uint64_t kept = 0;
    for (uint64_t g = 0; g < groups; ++g) {
        uint32_t m = 0;
        for (int b = 0; b < 32; ++b) {
            const uint64_t i = 32 * g + static_cast<uint64_t>(b);
            if (i >= n) break;
            if (element_bits(in, i, w) != 0) {
                m |= (uint32_t{1} << b);
                std::memcpy(values + kept * w, in + i * w, static_cast<size_t>(w));
                ++kept;
            }
        }
        masks[g] = m;
    }
    return kept;
}

// Size of the serialised stream for n elements with nnz kept:
// one 4-byte mask per group plus w bytes per kept element (section 5.1: a
// group of 32 zeros costs 4 bytes; a fully dense group costs 4 + 32*w).
uint64_t zvc_ref_compressed_bytes(uint64_t n, int w, uint64_t nnz) {
    return 4 * zvc_ref_groups(n) + static_cast<uint64_t>(w) * nnz;
}

// Encode into one contiguous buffer laid out [masks][values] (reading 1).
// out must hold 4*groups + n*w bytes and needs no alignment.  Returns the
// number of bytes used, or UINT64_MAX on a bad width.
uint64_t zvc_ref_compress_stream(const void* in, uint64_t n, int w, void* out_) {
    if (w != 2 && w != 4) return UINT64_MAX;
    unsigned char* out = static_cast<unsigned char*>(out_);
    const uint64_t groups = zvc_ref_groups(n);
    std::vector<uint32_t> masks(groups);
    const uint64_t kept = zvc_ref_compress(in, n, w, masks.data(), out + 4 * groups);
    for (uint64_t g = 0; g < groups; ++g) {
        // little-endian serialisation of the mask word, byte by byte
        const uint32_t m = masks[g];
        out[4 * g + 0] = static_cast<unsigned char>(m & 0xFF);
        out[4 * g + 1] = static_cast<unsigned char>((m >> 8) & 0xFF);
        out[4 * g + 2] = static_cast<unsigned char>((m >> 16) & 0xFF);
        out[4 * g + 3] = static_cast<unsigned char>((m >> 24) & 0xFF);
    }
    return zvc_ref_compressed_bytes(n, w, kept);
}

// Decode (section 5.2, decompression engine: the mask's 1 bits say how many
// stored words a span uses; each output slot takes the next stored word or a
// zero).  Returns the number of stored elements consumed, or UINT64_MAX on a
// bad width.
uint64_t zvc_ref_decompress(const uint32_t* masks, const void* values_, uint64_t n,
                            int w, void* out_) {
    if (w != 2 && w != 4) return UINT64_MAX;
    const unsigned char* values = static_cast<const unsigned char*>(values_);
    unsigned char* out = static_cast<unsigned char*>(out_);
    uint64_t used = 0;
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t m = masks[i / 32];
        if ((m >> (i % 32)) & 1u) {
            std::memcpy(out + i * w, values + used * w, static_cast<size_t>(w));
            ++used;
        } else {
            std::memset(out + i * w, 0, static_cast<size_t>(w));
        }
    }
    return used;
}

// Decode from the contiguous [masks][values] stream (no alignment needed).
uint64_t zvc_ref_decompress_stream(const void* comp_, uint64_t n, int w, void* out) {
    if (w != 2 && w != 4) return UINT64_MAX;
    const unsigned char* comp = static_cast<const unsigned char*>(comp_);
    const uint64_t groups = zvc_ref_groups(n);
    std::vector<uint32_t> masks(groups);
    for (uint64_t g = 0; g < groups; ++g) {
        const unsigned char* mb = comp + 4 * g;
        masks[g] = static_cast<uint32_t>(mb[0]) | (static_cast<uint32_t>(mb[1]) << 8) |
                   (static_cast<uint32_t>(mb[2]) << 16) | (static_cast<uint32_t>(mb[3]) << 24);
    }
    return zvc_ref_decompress(masks.data(), comp + 4 * groups, n, w, out);
}

// Count of non-zero elements only (the size a compressed copy would report,
// section 5.4: the copy call returns the compressed size on completion).
uint64_t zvc_ref_count_nonzero(const void* in_, uint64_t n, int w) {
    if (w != 2 && w != 4) return UINT64_MAX;
    const unsigned char* in = static_cast<const unsigned char*>(in_);
    uint64_t kept = 0;
    for (uint64_t i = 0; i < n; ++i) kept += (element_bits(in, i, w) != 0) ? 1 : 0;
    return kept;
}

// ReLU, element by element (section 4: the zeros that ZVC removes are the
// outputs of ReLU layers; reading 5 above).  out may alias in.
int zvc_ref_relu(const void* in_, uint64_t n, int w, void* out_) {
    if (w != 2 && w != 4) return -1;
    const unsigned char* in = static_cast<const unsigned char*>(in_);
    unsigned char* out = static_cast<unsigned char*>(out_);
    const uint32_t sign = w == 4 ? 0x80000000u : 0x8000u;
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t word = element_bits(in, i, w);
        const bool positive = (word & sign) == 0 && word != 0;
        if (positive)
            std::memmove(out + i * w, in + i * w, static_cast<size_t>(w));
        else
            std::memset(out + i * w, 0, static_cast<size_t>(w));
    }
    return 0;
}

// Fused ReLU + ZVC: by definition the ZVC stream of ReLU(in).  Written as
// exactly that composition: ReLU into a temporary, then the encoder above.
uint64_t zvc_ref_relu_compress_stream(const void* in, uint64_t n, int w, void* out) {
    if (w != 2 && w != 4) return UINT64_MAX;
    std::vector<unsigned char> activated(static_cast<size_t>(n) * static_cast<size_t>(w));
    zvc_ref_relu(in, n, w, activated.data());
    return zvc_ref_compress_stream(activated.data(), n, w, out);
}

// Number of windows of window_elems elements covering n elements.
uint64_t zvc_ref_window_count(uint64_t n, uint64_t window_elems) {
    if (window_elems == 0) return 0;
    return n / window_elems + (n % window_elems != 0 ? 1 : 0);
}

// Paper-order encoder (reading 6).  window_elems must be a positive multiple of
// 32.  out: room for 4*groups + n*w bytes, no alignment needed.  offsets: room
// for window_count + 1 entries.  Returns the bytes used (= offsets[last]), or
// UINT64_MAX on a bad width or window.
uint64_t zvc_ref_window_compress(const void* in_, uint64_t n, int w, uint64_t window_elems,
                                 void* out_, uint64_t* offsets) {
    if ((w != 2 && w != 4) || window_elems == 0 || window_elems % 32 != 0) return UINT64_MAX;
    const unsigned char* in = static_cast<const unsigned char*>(in_);
    unsigned char* out = static_cast<unsigned char*>(out_);
    const uint64_t windows = zvc_ref_window_count(n, window_elems);
    uint64_t pos = 0;
    for (uint64_t k = 0; k < windows; ++k) {
        offsets[k] = pos;
        const uint64_t first = k * window_elems;
        const uint64_t last = first + window_elems < n ? first + window_elems : n;
        for (uint64_t g0 = first; g0 < last; g0 += 32) {
            // the group's mask first ...
            uint32_t m = 0;
            for (int b = 0; b < 32; ++b) {
                const uint64_t i = g0 + static_cast<uint64_t>(b);
                if (i < last && element_bits(in, i, w) != 0) m |= (uint32_t{1} << b);
            }
            out[pos + 0] = static_cast<unsigned char>(m & 0xFF);
            out[pos + 1] = static_cast<unsigned char>((m >> 8) & 0xFF);
            out[pos + 2] = static_cast<unsigned char>((m >> 16) & 0xFF);
            out[pos + 3] = static_cast<unsigned char>((m >> 24) & 0xFF);
            pos += 4;
            // ... then its non-zero elements, in order
            for (int b = 0; b < 32; ++b) {
                const uint64_t i = g0 + static_cast<uint64_t>(b);
                if (i < last && element_bits(in, i, w) != 0) {
                    std::memcpy(out + pos, in + i * w, static_cast<size_t>(w));
                    pos += static_cast<uint64_t>(w);
                }
            }
        }
    }
    offsets[windows] = pos;
    return pos;
}

// Decoder for windows first_window .. first_window + num_windows - 1 of a
// paper-order stream: reads only those windows' bytes (through the offset
// table) and writes their elements to out, which points at the first element
// of first_window.  Returns the number of elements written, or UINT64_MAX on
// bad arguments.
uint64_t zvc_ref_window_decompress(const void* stream_, const uint64_t* offsets, uint64_t n, int w,
                                   uint64_t window_elems, uint64_t first_window,
                                   uint64_t num_windows, void* out_) {
    if ((w != 2 && w != 4) || window_elems == 0 || window_elems % 32 != 0) return UINT64_MAX;
    const uint64_t windows = zvc_ref_window_count(n, window_elems);
    if (first_window > windows || num_windows > windows - first_window) return UINT64_MAX;
    const unsigned char* stream = static_cast<const unsigned char*>(stream_);
    unsigned char* out = static_cast<unsigned char*>(out_);
    uint64_t written = 0;
    for (uint64_t k = first_window; k < first_window + num_windows; ++k) {
        uint64_t pos = offsets[k];
        const uint64_t first = k * window_elems;
        const uint64_t last = first + window_elems < n ? first + window_elems : n;
        for (uint64_t g0 = first; g0 < last; g0 += 32) {
            const uint32_t m = static_cast<uint32_t>(stream[pos]) |
                               (static_cast<uint32_t>(stream[pos + 1]) << 8) |
                               (static_cast<uint32_t>(stream[pos + 2]) << 16) |
                               (static_cast<uint32_t>(stream[pos + 3]) << 24);
            pos += 4;
            for (int b = 0; b < 32; ++b) {
                const uint64_t i = g0 + static_cast<uint64_t>(b);
                if (i >= last) break;
                unsigned char* dst = out + (i - first_window * window_elems) * w;
                if ((m >> b) & 1u) {
                    std::memcpy(dst, stream + pos, static_cast<size_t>(w));
                    pos += static_cast<uint64_t>(w);
                } else {
                    std::memset(dst, 0, static_cast<size_t>(w));
                }
                ++written;
            }
        }
    }
    return written;
}

}  // extern "C"

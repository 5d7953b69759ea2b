/*
 * zvc.h -- C ABI of the zero-value compression (ZVC) library for AMD gfx950.
 *
 * ZVC (paper section 5.1, "Zero-value compression"): a tensor is treated as a
 * flat run of n elements of w bytes each.  Every 32 consecutive elements form
 * one group described by a 32-bit presence mask (bit b set <=> element
 * 32*g + b is non-zero); the non-zero elements are kept, in order, and zeros
 * are dropped.  Decompression (section 5.2, decompression engine) walks the
 * mask bits and puts back either the next kept element or a zero.  The scheme
 * is lossless.
 *
 * Compressed stream layout used by every entry point here:
 *
 *     [ masks : G = ceil(n/32) little-endian uint32 ][ values : nnz * w bytes ]
 *
 *   - bit 0 (LSB) of a mask is the first element of its group; bits that fall
 *     past n in the last group are 0;
 *   - "zero" means the all-zero bit pattern of the w-byte element: -0.0, NaN
 *     and denormals are non-zero and are kept bit for bit;
 *   - compressed_bytes = 4*G + w*nnz.  Bytes of the output buffer past that
 *     are unspecified.
 *   The paper appends each group's non-zeros right after its mask; this
 *   library stores all masks first and all values after them.  The byte count
 *   is identical; the planar order lets both parts be written coalesced.
 *
 * Conventions for every function:
 *   - `w` is the element width in bytes, 2 or 4 (anything else: ZVC_E_WIDTH).
 *     The element type is irrelevant (fp32, fp16, bf16, int: all w-byte words).
 *   - pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The
 *     caller owns every buffer; the library allocates no device memory and
 *     keeps no pointer after the call's work has completed.
 *   - d_in / d_out of the uncompressed tensor must be aligned to w bytes; the
 *     compressed buffer must be aligned to 4 bytes.  The decoders are fastest
 *     with a 16-byte aligned d_out, the encoders with a 4-byte aligned d_in
 *     (which only 16-bit elements can miss); anything less still works.
 *   - input and output ranges must not overlap.
 *   - reads are made in aligned chunks of 4 or 16 bytes: a kernel may read the
 *     whole aligned 16-byte chunk that holds the first or the last byte of a
 *     buffer it is given (such a chunk never straddles a page, so this touches no
 *     memory the bytes themselves do not), and ignores what is not the buffer's.
 *     Nothing is ever written outside the output ranges.
 *   - device work is enqueued on the given stream and the call returns
 *     without waiting for it (zvc_offload is the one exception, see there).
 *   - n = 0 is legal.
 *   - arguments are validated on the host before any GPU call; a non-OK status
 *     means nothing was enqueued (ZVC_E_HIP excepted: a HIP call failed and
 *     earlier work of this call may already be enqueued).
 *   - a workspace serves one call at a time: calls that use the same workspace
 *     must be ordered (same stream, or event dependencies).  Its contents
 *     between calls are private to the library.
 */
#ifndef ZVC_H_
#define ZVC_H_

#include <stddef.h>
#include <stdint.h>

#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum zvc_status {
    ZVC_OK = 0,
    ZVC_E_ARG = 1,       /* null pointer, overlapping or otherwise invalid argument */
    ZVC_E_WIDTH = 2,     /* w is not 2 or 4 */
    ZVC_E_CAPACITY = 3,  /* an output buffer is smaller than the required bound */
    ZVC_E_WORKSPACE = 4, /* workspace smaller than zvc_workspace_bytes(n, w) */
    ZVC_E_ALIGN = 5,     /* pointer not aligned as required */
    ZVC_E_HIP = 6,       /* a HIP runtime call failed */
    ZVC_E_CORRUPT = 7    /* a compressed stream is inconsistent with its stated size */
} zvc_status;

/* Human-readable name of a status code (static storage, never NULL; any integer
 * is accepted, unknown ones give a string that says so). */
const char* zvc_status_string(int status);

/* ---- pure host arithmetic (no GPU needed) -------------------------------- */

/* 4 * ceil(n/32): bytes of the mask part (section 5.1: one 32-bit mask per 32
 * elements). */
size_t zvc_mask_bytes(size_t n);

/* Worst-case compressed size 4*ceil(n/32) + w*n (every element non-zero: the
 * 1-bit-per-element metadata overhead of section 5.1).  0 for a bad w. */
size_t zvc_max_compressed_bytes(size_t n, int w);

/* Bytes of device workspace needed by the calls below for n elements of width
 * w.  0 for a bad w.  The workspace must be 256-byte aligned. */
size_t zvc_workspace_bytes(size_t n, int w);

/* Host-side consistency check of a compressed stream held in HOST memory:
 * ZVC_OK iff bytes == 4*G + w * (sum of popcounts of the G masks) and the last
 * mask has no bit set past n.  (The decoder of section 5.2 consumes exactly
 * popcount(mask) words per group, so any other size is a damaged stream.) */
zvc_status zvc_check_stream(const void* h_comp, uint64_t bytes, size_t n, int w);

/* ---- scan tuning and diagnostics ------------------------------------------ */

/* The device-wide scan of per-tile counts (where the next mask's elements go,
 * section 5.1) lets a tile wait for its predecessors' counts.  After `polls`
 * fruitless polls the waiting tile computes the missing count itself, so the
 * wait always ends.  Default 2000 (about a millisecond); 0 makes every wait
 * help at once, which tests use to exercise that path.  The setting belongs to
 * the workspace (a word in its header, written on `stream`; zvc_workspace_init
 * restores the default) and applies to the encoder calls that use it. */
zvc_status zvc_workspace_set_lookback_patience(void* d_ws, unsigned polls, hipStream_t stream);

/* Measurement aid, not part of the method: enqueues a plain streaming kernel
 * that reads read_bytes at d_in and writes write_bytes at d_out (what it writes
 * is a mix of what it read), both split evenly over one workgroup per 64 KB of
 * the larger side (per 16 KB below 32 MB), with 16-byte non-temporal accesses.  Given the byte counts of
 * a zvc_compress call (n*w in, the stream out) or of a zvc_decompress call (the
 * mirror) it shows what the memory system does with that traffic when the
 * kernel has nothing else to do: the same-run yardstick that the benchmark
 * prints beside every codec time.  Pointers 16-byte aligned, byte counts
 * multiples of 16 (else ZVC_E_ALIGN), ranges disjoint. */
zvc_status zvc_reference_stream(const void* d_in, size_t read_bytes, void* d_out, size_t write_bytes,
                                hipStream_t stream);

/* Number of times, since zvc_workspace_init, that a waiting tile computed a
 * predecessor's count itself.  Synchronous 8-byte device-to-host copy; call it
 * after the stream has drained. */
zvc_status zvc_workspace_self_help_count(const void* d_ws, uint64_t* h_count);

/* ---- device entry points -------------------------------------------------- */

/* Prepare a freshly allocated workspace (fills it with its initial state).
 * Call once per allocation before its first use; ws is the allocation's size
 * in bytes, at least zvc_workspace_bytes(0, 4).  Every call leaves the
 * workspace ready for the next one, so no other reset is ever needed; only
 * after a call failed with ZVC_E_HIP (or its kernels were aborted) must the
 * workspace be initialised again. */
zvc_status zvc_workspace_init(void* d_ws, size_t ws, hipStream_t stream);

/* Count-only pass: *d_bytes = 4*ceil(n/32) + w*nnz, the size zvc_compress would
 * report (section 5.4: the compressed copy returns the compressed size).
 * d_bytes is an 8-byte aligned device word, valid when `stream` reaches the end
 * of this call's work. */
zvc_status zvc_compressed_size(const void* d_in, size_t n, int w, uint64_t* d_bytes,
                               void* d_ws, size_t ws, hipStream_t stream);

/* Compress n elements at d_in into d_out (section 5.1; encoder pipeline of
 * section 5.2: zero test, prefix sum of the mask bits, shift non-zeros to
 * their packed slots, append).  out_cap is the capacity of d_out in bytes and
 * must be at least zvc_max_compressed_bytes(n, w) (else ZVC_E_CAPACITY; the
 * kernel never writes past the bound).  *d_bytes (device, 8-byte aligned)
 * receives the compressed size. */
zvc_status zvc_compress(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                        uint64_t* d_bytes, void* d_ws, size_t ws, hipStream_t stream);

/* zvc_compress for callers that cannot allocate or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * scan state lives in an array inside the library's code object, one copy per
 * GPU, ZVC_STATIC_SCRATCH_BYTES of device memory that the GPU holds until the
 * process ends.  Same stream, same arguments and errors as zvc_compress without
 * d_ws / ws; n * w may be at most ZVC_STATIC_MAX_BYTES (more: ZVC_E_WORKSPACE,
 * nothing enqueued).  Allocates nothing: no hipMalloc, no hipFree, no host
 * allocation; the first call on a GPU looks the array's address up (with that
 * GPU current, as for every call: the stream must belong to the current
 * device).  All calls on one GPU share the array: two calls that may run at the
 * same time on one GPU (different streams without an ordering between them)
 * race and give wrong streams; order them.  Every call leaves the array in its
 * initial all-zero state; only after a call's kernel was aborted is it not, and
 * then this entry point must not be used again in the process. */
#define ZVC_STATIC_MAX_BYTES ((size_t)1 << 30)
#define ZVC_STATIC_SCRATCH_BYTES ((size_t)320 << 10)
zvc_status zvc_compress_static(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                               uint64_t* d_bytes, hipStream_t stream);

/* Fused ReLU + compression: d_in holds PRE-activation values and the stream
 * written is exactly the one zvc_compress would write for ReLU(d_in), without
 * the dense ReLU output ever being stored (section 4: the zeros that ZVC
 * removes are ReLU outputs; the offload then needs one pass over the
 * activations instead of three).  Elements are IEEE-style numbers with the sign
 * in the top bit: fp32 (w = 4), fp16 or bf16 (w = 2).  An element is kept,
 * unchanged, when its sign bit is clear and it is not +0; every other element
 * counts as zero.  So positive numbers, denormals and +inf are kept, -0.0 and
 * negative numbers are dropped, and a NaN is kept exactly when its sign bit is
 * clear.  zvc_decompress of the stream gives ReLU(d_in).  Arguments, errors and
 * stream ordering as for zvc_compress. */
zvc_status zvc_relu_compress(const void* d_in, size_t n, int w, void* d_out, size_t out_cap,
                             uint64_t* d_bytes, void* d_ws, size_t ws, hipStream_t stream);

/* Compression into a buffer below the worst case, for streams that stay in GPU
 * memory (section 9, compression for GPU footprint reduction: the saving is
 * real only if the buffer is the size of the stream, which is not known before
 * the call).  relu = 0 compresses d_in as zvc_compress does, relu = 1 as
 * zvc_relu_compress does.  out_cap may be anything from zvc_mask_bytes(n) up
 * (less: ZVC_E_CAPACITY).  *d_bytes always receives the size the whole stream
 * needs.  If that is at most out_cap, d_out holds exactly the stream the
 * unbounded call writes.  If it is more, the call still returns ZVC_OK (the
 * size is not known on the host): the mask area is complete, the rest of d_out
 * up to out_cap is unspecified, and nothing at or past d_out + out_cap has been
 * written; the caller compares *d_bytes with out_cap and calls again with a
 * buffer of that size.  (zvc_compressed_size gives the exact size beforehand at
 * the price of one more read of the tensor.)  Other arguments, errors and
 * stream ordering as for zvc_compress. */
zvc_status zvc_compress_bounded(const void* d_in, size_t n, int w, int relu, void* d_out,
                                size_t out_cap, uint64_t* d_bytes, void* d_ws, size_t ws,
                                hipStream_t stream);

/* Decompress a stream produced by zvc_compress back into n elements at d_out
 * (section 5.2, decompression engine: popcount of the mask gives the words a
 * span consumes, a prefix sum gives each slot's source, slots take a stored
 * word or zero).  comp_bytes is the number of readable bytes at d_comp (at
 * least zvc_mask_bytes(n)); the kernel reads no stored element past it: if
 * damaged masks ask for more values than are there, the missing elements decode
 * as zero.  A comp_bytes larger than the stream is harmless, but the call picks
 * its access pattern from it (it tells the stream's density): pass the size
 * the encoder reported where it is known. */
zvc_status zvc_decompress(const void* d_comp, size_t comp_bytes, size_t n, int w, void* d_out,
                          void* d_ws, size_t ws, hipStream_t stream);

/* ---- the paper's own stream order, in independently decodable windows ------ */

/* Section 5.1 appends a group's non-zero elements right after its mask, and the
 * DMA engine of section 6 works on windows of uncompressed data, each decodable
 * on its own: 4 KB there, and section 7.1 reports that windows up to 64 KB make
 * little difference.  The windowed stream is that order: window after window
 * (window_bytes / w elements each, the last one possibly shorter), inside a
 * window group after group, for each group its 32-bit mask (little-endian; for
 * w = 2 it may fall on a 2-byte boundary) and then its kept elements.  Windows
 * are packed back to back, so the stream has exactly the bytes of the planar
 * one, 4*ceil(n/32) + w*nnz, and they are the same bytes whatever the window
 * size.  Beside it goes a table of zvc_window_count(n, w, window_bytes) + 1 byte
 * offsets: window k occupies [offsets[k], offsets[k+1]) and the last entry is
 * the stream's size.  The table (this library's addition, not counted in the
 * compressed size: 8 bytes per window) makes any range of windows decodable
 * without touching the rest.  The table of a larger window size is every
 * (larger / smaller)-th entry of a smaller one's, plus the final size.
 *
 * window_bytes is a power of two from ZVC_WINDOW_MIN_BYTES to
 * ZVC_WINDOW_MAX_BYTES; anything else is ZVC_E_ARG (0 from the two size
 * functions).  Decoding walks a window's masks one after the other, so small
 * windows decode fastest; the encoder's speed does not depend on the size. */
#define ZVC_WINDOW_MIN_BYTES ((size_t)1024)
#define ZVC_WINDOW_MAX_BYTES ((size_t)65536)
#define ZVC_WINDOW_PAPER_BYTES ((size_t)4096)   /* the window of section 6 */

/* Elements per window: window_bytes / w.  0 for a bad w or window size. */
size_t zvc_window_elements(int w, size_t window_bytes);

/* Number of windows for n elements of width w: ceil(n*w / window_bytes).  0 for
 * a bad w or window size. */
size_t zvc_window_count(size_t n, int w, size_t window_bytes);

/* Host-side consistency check of a windowed stream and its table, both in HOST
 * memory: ZVC_OK iff the table starts at 0, ends at `bytes`, and every window,
 * walked mask by mask (a mask, then as many elements as it has bits set), ends
 * exactly where the next one begins; the last mask has no bit set past n. */
zvc_status zvc_window_check_stream(const void* h_stream, uint64_t bytes, const uint64_t* h_offsets,
                                   size_t n, int w, size_t window_bytes);

/* Compress into the windowed stream.  d_out / out_cap / d_bytes / workspace as
 * for zvc_compress; d_offsets is a device array of
 * zvc_window_count(n, w, window_bytes) + 1 64-bit words (8-byte aligned, not
 * overlapping the other buffers). */
zvc_status zvc_window_compress(const void* d_in, size_t n, int w, size_t window_bytes, void* d_out,
                               size_t out_cap, uint64_t* d_offsets, uint64_t* d_bytes, void* d_ws,
                               size_t ws, hipStream_t stream);

/* Decompress windows first_window .. first_window + num_windows - 1 of a
 * windowed stream of n elements (a partial prefetch).  d_stream points at the
 * START of the stream (aligned to w) and stream_bytes is the number of readable
 * bytes there; d_offsets is the whole table, made for this window_bytes.  d_out
 * receives the elements of those windows only, i.e. it points at where element
 * first_window * window_bytes / w of the tensor goes.  Needs no workspace.  The
 * kernel reads nothing outside [d_stream, d_stream + stream_bytes) and the
 * table entries of the windows asked for; what a damaged table or mask asks for
 * beyond a window's bytes decodes as zero.  ZVC_E_ARG if the range does not lie
 * within the windows. */
zvc_status zvc_window_decompress(const void* d_stream, size_t stream_bytes, const uint64_t* d_offsets,
                                 size_t n, int w, size_t window_bytes, size_t first_window,
                                 size_t num_windows, void* d_out, hipStream_t stream);

/* Offload (section 3 and section 5.4: the activation map leaves GPU memory as
 * a compressed copy whose size is known on completion).  Compresses d_in into
 * the device staging buffer d_stage on `compute`, waits ON THE HOST for the
 * 8-byte size (the one host wait in this library), stores it in *h_bytes, then
 * enqueues the device-to-host copy of exactly that many bytes into h_pinned on
 * `copy` (ordered after the compression).  h_pinned should be pinned host
 * memory for the copy to be asynchronous; h_cap must be at least
 * zvc_max_compressed_bytes(n, w).  The data in h_pinned is complete when
 * `copy` has drained; d_stage may be reused only after that. */
zvc_status zvc_offload(const void* d_in, size_t n, int w, void* d_stage, size_t stage_cap,
                       void* h_pinned, size_t h_cap, uint64_t* h_bytes, void* d_ws, size_t ws,
                       hipStream_t compute, hipStream_t copy);

/* zvc_offload with the fused ReLU encoder: d_in holds pre-activations, the host
 * receives the stream of ReLU(d_in) (see zvc_relu_compress).  zvc_prefetch
 * brings back ReLU(d_in). */
zvc_status zvc_relu_offload(const void* d_in, size_t n, int w, void* d_stage, size_t stage_cap,
                            void* h_pinned, size_t h_cap, uint64_t* h_bytes, void* d_ws, size_t ws,
                            hipStream_t compute, hipStream_t copy);

/* Prefetch, the mirror of zvc_offload: enqueues the host-to-device copy of
 * `bytes` bytes from h_pinned into d_stage on `copy`, then the decompression
 * into d_out on `compute`, ordered after the copy.  No host wait.  The copy
 * overwrites d_stage as soon as `copy` gets to it: if earlier work on `compute`
 * (a previous zvc_prefetch's decompression, say) still reads d_stage, the
 * caller must make `copy` wait for that work first, or use another buffer. */
zvc_status zvc_prefetch(const void* h_pinned, uint64_t bytes, size_t n, int w, void* d_stage,
                        size_t stage_cap, void* d_out, void* d_ws, size_t ws, hipStream_t copy,
                        hipStream_t compute);

#ifdef __cplusplus
} /* extern "C" */
#endif

#endif /* ZVC_H_ */

/*
 * fftsp.h -- C ABI of the MI355X (gfx950) FFT-sparsifying gradient codec.
 *
 * The codec is the per-worker sender/receiver pair of arXiv 1811.08596, Sec. 3.1:
 * linearized gradient -> FFT -> keep the largest
 * frequency components -> range-based N-bit float -> pack; the receiver applies
 * the inverse operations in reverse order.
 *
 * Conventions shared by every entry point
 *   - Pointers named d_* are DEVICE pointers (hipMalloc / torch CUDA memory),
 *     16-byte aligned.  seg_offsets is a HOST pointer.  The caller owns every
 *     buffer; the library allocates nothing (its two 16 KiB twiddle tables are
 *     constants inside the code object).  The per-tensor entry points create
 *     three streams and four events per device on their first call outside a
 *     stream capture; they create nothing while the caller's stream is being
 *     captured (see there).
 *   - Calls only enqueue work on `stream` and return; they never synchronise and
 *     never touch the null stream.  Input buffers are not modified.  Output
 *     regions are written completely (padding bytes zero), so results are
 *     byte-comparable.  Two calls that share a workspace must be ordered by
 *     the caller (same stream, or events).
 *   - `theta` is the KEPT fraction of frequency bins in [0,1].  The paper's theta
 *     (Sec. 3.1.1) is the dropped fraction, i.e. 1 - theta of this interface.
 *   - `chunk_len` L is a power of two in [32, 2^22]; the flat gradient is cut
 *     into C = ceil(n/L) chunks, the last one zero-padded.  One chunk of length
 *     n is exactly the paper's whole-vector transform.
 *   - `bits` N is the code width: 3..16 for the offset-based N-bit float of
 *     Sec. 3.2.1 / Algorithm 1, or 32 for "quantization off" (raw binary32).
 *   - Return value: FFTSP_OK or an error; argument errors are detected on the
 *     host before anything is enqueued.  Non-finite gradient values are not
 *     detected: the call is memory-safe but its output is unspecified.
 *
 * Packed stream (little-endian, all padding zero):
 *   64-byte header: "FSP1", u32 version=1, u64 n, u32 L (0 = per-segment
 *   lengths), u32 C, u32 N, u32 m, u32 k, u32 S, f32 theta, zeros;
 *   then C records of S = align16(16 + 4*W + 4*ceil(2kN/32)) bytes,
 *   W = ceil(B/32), B = L/2+1:
 *     +0  u32 pbase, u32 vmax_bits, u32 k, u32 L-if-segmented-else-0
 *     +16 status bitmap (Sec. 3.2): bit j%32 of word j/32 set = bin j kept
 *     +16+4W codes: code i in bits [iN, iN+N) of an LSB-first u32 stream,
 *         order re0, im0, re1, im1, ... by ascending kept bin (the "dense"
 *         vector of Sec. 3.2; its positions are the prefix sum of the bitmap).
 */
#ifndef FFTSP_H
#define FFTSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t* fftsp_stream_t; /* a hipStream_t */

typedef enum {
    FFTSP_OK = 0,
    FFTSP_EINVAL = 1,       /* null/misaligned pointer, n = 0, theta outside [0,1] or NaN, bad bits */
    FFTSP_ENOSPC = 2,       /* packed_capacity smaller than fftsp_packed_bytes(...) */
    FFTSP_EWORKSPACE = 3,   /* workspace smaller than fftsp_workspace_bytes(...) */
    FFTSP_EUNSUPPORTED = 4, /* chunk_len not a power of two in [32, 2^22] */
    FFTSP_EHIP = 5,         /* a HIP runtime call or launch failed */
    FFTSP_EFORMAT = 6       /* packed stream does not match the arguments (device status word) */
} fftsp_status;

/* ---- host-side arithmetic: no device access, pure functions of their arguments ---- */

/* k = clamp(floor((double)theta * B + 1/2), 0, B): kept bins per chunk (selection rule of Sec. 3.1.1). */
int fftsp_kept_per_chunk(uint32_t chunk_len, float theta, uint32_t* k_out);
/* default mantissa width m of the N-bit float (Sec. 3.2.1, the split of the N bits); -1 if bits invalid. */
int fftsp_mantissa_bits(int bits);
/* exact size of the packed stream, 0 on invalid arguments. */
size_t fftsp_packed_bytes(size_t n, uint32_t chunk_len, float theta, int bits);
/* bytes of device workspace any entry point below needs for (n, chunk_len, bits); 0 on invalid arguments. */
size_t fftsp_workspace_bytes(size_t n, uint32_t chunk_len, int bits);

/* ---- the codec (Sec. 3.1 steps 1-4 and their inverses) ---- */

/* Sender.  d_grad: n floats.  d_packed: receives fftsp_packed_bytes(...) bytes. */
int fftsp_compress(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits,
                   void* d_packed, size_t packed_capacity,
                   void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* The sender for callers that cannot allocate device memory or pass a workspace: code recorded into a HIP graph,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same packed bytes as fftsp_compress; the
 * workspace is a fixed array of FFTSP_STATIC_SCRATCH_BYTES inside the library's code object (every GPU the
 * library runs on holds its own copy until the process ends).  The call allocates nothing, on the host side
 * of HIP or on the device (keep fftsp_profile_enable off: its events are created on demand).
 * Limit: fftsp_workspace_bytes(n, chunk_len, bits) <= FFTSP_STATIC_SCRATCH_BYTES (e.g. n = 2^20 with
 * chunk_len = 2^16, or one chunk of 2^20); beyond that the call returns FFTSP_EWORKSPACE and enqueues nothing.
 * All calls on one GPU share that GPU's array: two calls that may overlap in time (different streams, no event
 * between them) race and must be ordered by the caller.  The array keeps the last call's contents; the kernels
 * clear what they need cleared.  The device status word lives inside the array and cannot be read back. */
#define FFTSP_STATIC_SCRATCH_BYTES (16u << 20)
int fftsp_compress_static(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits,
                          void* d_packed, size_t packed_capacity, fftsp_stream_t stream);

/* Receiver.  The same (n, chunk_len, theta, bits) as the sender must be passed; a stream whose
 * header disagrees sets the device status word to FFTSP_EFORMAT and the output is unspecified
 * (reads stay inside d_packed[0, packed_bytes)).  d_grad_out: exactly n floats are written. */
int fftsp_decompress(const void* d_packed, size_t packed_bytes,
                     float* d_grad_out, size_t n, uint32_t chunk_len, float theta, int bits,
                     void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* ---- quantizer options (Sec. 3.2.1: the choice of m and eps; the static [min, max] range) ----
 *
 * The entry points above fix m from the code width and fit the range of every chunk to its largest surviving
 * component.  The _q variants take both from the caller; quantizer == NULL means the defaults.
 *   mantissa_bits: m, 1 .. bits-1 (ignored for bits = 32); 0 = fftsp_mantissa_bits(bits).
 *   range_max:     > 0: static range [-range_max, +range_max] for every chunk, as in the paper's experiments
 *                  (range estimated beforehand); components beyond it clamp to the top code (Algorithm 1) and no
 *                  reduction over the survivors is needed.  0 = fitted per chunk.  Negative, infinite or NaN:
 *                  FFTSP_EINVAL.
 * eps is not an input: for a given range it is the closed form the paper's iterative tuning converges to.
 * The receiver needs the same mantissa_bits (the stream header carries m and a mismatch raises FFTSP_EFORMAT);
 * range_max is ignored there (every record carries its pbase). */
typedef struct fftsp_quantizer {
    int mantissa_bits;
    float range_max;
} fftsp_quantizer;

int fftsp_compress_q(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits,
                     void* d_packed, size_t packed_capacity, void* d_workspace, size_t workspace_bytes,
                     const fftsp_quantizer* quantizer, fftsp_stream_t stream);
int fftsp_decompress_q(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n, uint32_t chunk_len,
                       float theta, int bits, void* d_workspace, size_t workspace_bytes,
                       const fftsp_quantizer* quantizer, fftsp_stream_t stream);
int fftsp_encode_spectrum_q(const float* d_spec, size_t n, uint32_t chunk_len, float theta, int bits,
                            void* d_packed, size_t packed_capacity, void* d_workspace, size_t workspace_bytes,
                            const fftsp_quantizer* quantizer, fftsp_stream_t stream);
int fftsp_decode_spectrum_q(const void* d_packed, size_t packed_bytes, size_t n, uint32_t chunk_len, float theta,
                            int bits, float* d_spec, void* d_workspace, size_t workspace_bytes,
                            const fftsp_quantizer* quantizer, fftsp_stream_t stream);

/* ---- receiver under an allgather (Sec. 4, "Implementation": every worker collects the packed gradients of all
 *      peers; Sec. 3.1: the receiver applies the inverse steps) ----
 *
 * The inverse transform is linear, so the peers' sparse spectra are added bin by bin and ONE inverse transform is
 * taken:   d_grad_out = scale * iFFT( sum_p D(d_packed[p]) ),   e.g. scale = 1/npeers for the average.
 * The sum starts from zero and adds the peers in list order in binary32; scale multiplies the transform's
 * normalisation 1/L (one binary32 product per output).
 *
 * d_packed: HOST array of npeers DEVICE pointers (16-byte aligned), each to a stream of packed_bytes bytes made
 * with the same (n, chunk_len, theta, bits); the array is read before the call returns.  1 <= npeers <=
 * FFTSP_MAX_PEERS (more: FFTSP_EUNSUPPORTED; call again on the remainder and add).  A stream whose header or
 * bitmaps disagree with the arguments sets the device status word to FFTSP_EFORMAT; reads stay inside each
 * stream.  The workspace must hold fftsp_workspace_bytes_accumulate(...) bytes (0 on invalid arguments). */
#define FFTSP_MAX_PEERS 32
size_t fftsp_workspace_bytes_accumulate(size_t n, uint32_t chunk_len, int bits, int npeers);
int fftsp_decompress_accumulate(const void* const* d_packed, int npeers, size_t packed_bytes, float scale,
                                float* d_grad_out, size_t n, uint32_t chunk_len, float theta, int bits,
                                void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
/* Stage-level: only the summed spectrum, C*(L+2) floats in natural bin order, unscaled (bit-exact against the
 * same binary32 sum on the host). */
int fftsp_decode_accumulate_spectrum(const void* const* d_packed, int npeers, size_t packed_bytes, size_t n,
                                     uint32_t chunk_len, float theta, int bits, float* d_spec,
                                     void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* ---- stage-level entry points (the same kernels the codec runs, exposed for parity checks) ---- */

/* Forward real DFT of each chunk (the sum of Sec. 3.1.1, sign -, unnormalised).
 * d_spec: C*(L+2) floats, chunk c at c*(L+2), bins 0..L/2 as (re,im) pairs; im of bins 0 and L/2 is +0. */
int fftsp_rfft(const float* d_grad, size_t n, uint32_t chunk_len, float* d_spec,
               void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
/* Inverse (1/L, Hermitian extension; im of bins 0 and L/2 ignored); writes the first n samples. */
int fftsp_irfft(const float* d_spec, size_t n, uint32_t chunk_len, float* d_grad_out,
                void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
/* Steps 2-4 of Sec. 3.1 on a given spectrum: magnitude top-k, Algorithm 1, packing (Sec. 3.2). */
int fftsp_encode_spectrum(const float* d_spec, size_t n, uint32_t chunk_len, float theta, int bits,
                          void* d_packed, size_t packed_capacity,
                          void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
/* Inverse of the above: unpack, Nbit_to_32bit of Algorithm 1, scatter into a zeroed spectrum. */
int fftsp_decode_spectrum(const void* d_packed, size_t packed_bytes, size_t n, uint32_t chunk_len,
                          float theta, int bits, float* d_spec,
                          void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* ---- half-precision variant (Sec. 3.1.1, "Our approach": the gradients go to 16 bits for the transform, a loss
 *      the paper calls negligible because gradients are bounded).  Definition: the chunk's DFT times 2^scale_log2,
 *      each component rounded to binary16 (nearest even, saturating at +-65504); selection, Algorithm 1 and packing
 *      as in fftsp_compress on those values; the receiver inverts and divides by 2^scale_log2.  Here the arithmetic
 *      stays binary32 and it is the stored intermediate of the two-pass transform and the stored spectrum that are
 *      binary16 (these kernels are bound by bytes, not by arithmetic), so a result differs from the definition by
 *      one more binary16 rounding inside the transform: about 5e-4 relative L2 on a spectrum, against the 1e-5 of
 *      the binary32 path.  scale_log2 in [-24, 24] is the caller's: choose it so that spectrum magnitudes
 *      (about 2^scale_log2 * sigma * sqrt(chunk_len)) sit well inside binary16's normal range [6e-5, 65504].
 *      The stream layout is that of fftsp_compress with header word 12 (offset 48) = scale_log2; fftsp_decompress
 *      rejects a stream with a non-zero scale and fftsp_decompress_h one with another scale (status
 *      FFTSP_EFORMAT).  chunk_len: power of two in [2^15, 2^22] (FFTSP_EUNSUPPORTED below: one workgroup
 *      transforms such a chunk without touching memory in between).  Everything else as fftsp_compress /
 *      fftsp_decompress, including packed and workspace sizes (fftsp_packed_bytes, fftsp_workspace_bytes). ---- */
int fftsp_compress_h(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, int scale_log2,
                     void* d_packed, size_t packed_capacity,
                     void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
int fftsp_decompress_h(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n,
                       uint32_t chunk_len, float theta, int bits, int scale_log2,
                       void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* ---- time-domain Top-k, the sparsifier the paper measures its own against (Sec. 4, "Choice of Algorithms";
 *      the Sec. 3.1.1 figure sets it beside FFT Top-k): the magnitude selection (Sec. 3.1.1), Algorithm 1 and the
 *      packing of Sec. 3.2 applied to the gradient's samples themselves, no transform.  Chunk c is samples
 *      [c*L, (c+1)*L) (the last one zero-padded for the selection; the padding is never written back); a sample
 *      ranks by |x|, ties to the lowest index; k = round-half-up(theta * L) samples are kept per chunk, theta
 *      being the KEPT fraction; bits = 32 is the paper's plain Top-k.  Record: 16-byte header as above, bitmap of
 *      ceil(L/32) words, ONE code per kept sample; stream header word 11 (offset 44) is 1, and each decompress
 *      accepts only its own kind of stream (status FFTSP_EFORMAT otherwise).  chunk_len: power of two in
 *      [32, 2^21].  Pointers, alignment, workspace, stream and error behaviour are those of
 *      fftsp_compress / fftsp_decompress; the workspace here holds no spectrum. ---- */
int fftsp_topk_kept_per_chunk(uint32_t chunk_len, float theta, uint32_t* k_out);
size_t fftsp_topk_packed_bytes(size_t n, uint32_t chunk_len, float theta, int bits);
size_t fftsp_topk_workspace_bytes(size_t n, uint32_t chunk_len, int bits);
int fftsp_topk_compress(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits,
                        void* d_packed, size_t packed_capacity,
                        void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
int fftsp_topk_decompress(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n,
                          uint32_t chunk_len, float theta, int bits,
                          void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* ---- per-tensor variant: segment i = d_grad[seg_offsets[i] .. seg_offsets[i+1]) is one chunk of
 *      L_i = max(32, next power of two >= its size); seg_offsets (nseg+1 entries, ascending) is on the HOST
 *      and is consumed before the call returns.  Sizes above 2^22 are FFTSP_EUNSUPPORTED.
 *      Records follow tensor order in the stream.  Tensors that pad to the same L_i run together as the chunks
 *      of shared launches (up to 64 at a time), so the cost grows with the number of distinct lengths rather
 *      than with the number of tensors.  These launch sets run on up to four streams at once (the caller's and
 *      streams of the library's own that fork from and join back into it, so the call is still one unit of work
 *      on the caller's stream and can be captured into a graph); the workspace holds one region per stream, each
 *      sized for the largest group.  The side streams belong to the device and are shared by all callers: calls
 *      from several host threads enqueue one after the other.  A captured call keeps the side streams inside its
 *      capture until that capture ends; a call made meanwhile on another stream, and a captured call made before
 *      the side streams exist, runs all its launch sets on the caller's stream alone (same bytes, less overlap). ---- */
size_t fftsp_packed_bytes_segments(const size_t* seg_offsets, int nseg, float theta, int bits);
size_t fftsp_workspace_bytes_segments(const size_t* seg_offsets, int nseg, int bits);
int fftsp_compress_segments(const float* d_grad, const size_t* seg_offsets, int nseg, float theta, int bits,
                            void* d_packed, size_t packed_capacity,
                            void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);
int fftsp_decompress_segments(const void* d_packed, size_t packed_bytes, float* d_grad_out,
                              const size_t* seg_offsets, int nseg, float theta, int bits,
                              void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream);

/* Synchronises `stream`'s device and reads the status word the last call on this workspace left
 * (FFTSP_OK or FFTSP_EFORMAT).  Returns FFTSP_EHIP if the copy fails. */
int fftsp_device_status(const void* d_workspace, int* status_out);

/* Per-kernel timing for benchmarks (not part of the method).  While enabled, every kernel the library
 * launches is bracketed by two HIP events on its stream (do not enable under stream capture).
 * fftsp_profile_enable(1) also discards earlier records.  fftsp_profile_report synchronises the device and
 * writes one text line per kernel, "name calls total_ms", NUL-terminated, into buf (HOST memory, cap bytes);
 * it returns the number of bytes the full report needs. */
int fftsp_profile_enable(int on);
size_t fftsp_profile_report(char* buf, size_t cap);

const char* fftsp_strerror(int status);
const char* fftsp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FFTSP_H */

// Internal declarations shared by the translation units of libfftsp.so.
// Nothing here is part of the C ABI (see include/fftsp.h).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>
#include <string>

namespace fftsp {

constexpr int kMinLogL = 5;   // chunk length 32
constexpr int kMaxLogL = 22;  // chunk length 4 Mi

// Twiddle tables, one pair per device, 2048 entries each:
//   hi[h] = exp(-2 pi i h / 2^11),  lo[l] = exp(-2 pi i l / 2^22)
// so that exp(-2 pi i E / 2^22) = hi[E >> 11] * lo[E & 2047] for any E < 2^22.
struct Tables {
    const float2* hi;
    const float2* lo;
};

// How complex values are stored where they cross HBM between kernels (the two-pass intermediate and the codec's
// own spectrum): binary32 pairs, or binary16 pairs in the half-precision variant (Sec. 3.1.1, "Our approach").
// Arithmetic is binary32 in registers and LDS either way; the variant halves the bytes, which is what bounds
// these kernels.  One = a complex value, Two = two adjacent ones (what a lane moves per access).
template <bool HALF>
struct Cx {
    using One = float2;
    using Two = float4;
};
template <>
struct Cx<true> {
    using One = uint32_t;  // bit pattern of two binary16 numbers (re low, im high)
    using Two = uint2;
};
// round to nearest even, saturating at the largest finite binary16 number
__device__ __forceinline__ uint32_t pack_half2(float2 v)
{
    const float lim = 65504.f;
    const __half2 h = __floats2half2_rn(fminf(fmaxf(v.x, -lim), lim), fminf(fmaxf(v.y, -lim), lim));
    uint32_t w;
    __builtin_memcpy(&w, &h, sizeof(w));
    return w;
}
__device__ __forceinline__ float2 unpack_half2(uint32_t w)
{
    __half2 h;
    __builtin_memcpy(&h, &w, sizeof(w));
    return __half22float2(h);
}
__device__ __forceinline__ float2 cx_load(float2 v) { return v; }
__device__ __forceinline__ float2 cx_load(uint32_t v) { return unpack_half2(v); }
__device__ __forceinline__ float4 cx_load(float4 v) { return v; }
__device__ __forceinline__ float4 cx_load(uint2 v)
{
    const float2 a = unpack_half2(v.x), b = unpack_half2(v.y);
    return make_float4(a.x, a.y, b.x, b.y);
}
template <bool HALF>
__device__ __forceinline__ typename Cx<HALF>::One cx_store(float2 v)
{
    if constexpr (HALF)
        return pack_half2(v);
    else
        return v;
}
template <bool HALF>
__device__ __forceinline__ typename Cx<HALF>::Two cx_store(float4 v)
{
    if constexpr (HALF)
        return make_uint2(pack_half2(make_float2(v.x, v.y)), pack_half2(make_float2(v.z, v.w)));
    else
        return v;
}

// Selection geometry: one workgroup of 256 lanes owns a tile of 2048 consecutive bins
// (wave w owns 512 of them as 8 rows of 64), so a wave ballot is two bitmap words.
constexpr int kTile = 2048;
constexpr int kTileThreads = 256;
constexpr int kHistBits = 12;                 // first radix-select digit: top 12 bits of the 31-bit key
constexpr int kHistBins = 1 << kHistBits;
constexpr int kKeyShift = 31 - kHistBits;     // bucket = key >> 19

constexpr size_t kControlBytes = 4096;  // control block at the start of every workspace
constexpr int kCtlGaveUpWord = 1;       // u32 index of the fused kernels' give-up word inside the control block

// The fused transforms (fused.hip) take chunk lengths 2^15 .. 2^20 and address three turn buffers of 4 MiB per XCD
// inside the intermediate's region, so they take calls whose own intermediate is at least that large (96 MiB: about
// 25 million samples); smaller calls keep the per-pass kernels and their workspace stays what those need.
constexpr size_t kFusedScratchBytes = (size_t)8 * 3 * 64 * 8192 * 8;
static inline bool fused_shape(int logL, size_t C)
{
    const int logM = logL - 1;
    return logM >= 14 && logM <= 19 && (C << logL) * 4 >= kFusedScratchBytes;
}

// Where everything lives inside the caller's workspace (byte offsets, 256-aligned).
struct Workspace {
    size_t status;    // u32[1024] control block: word 0 = device status, word 1 = "the fused transform gave up",
                      //           from word 32 on the hand-over counters of the fused kernels (fused.hip)
    size_t hist;      // u32[C][kHistBins]         (directly after status: one fill zeroes both)
    size_t sel;       // u32[C][8]  bstar, need, tau, quota, pbase, vmax, -, decode verdict
    size_t tinfo;     // u32[C][Tn][4]  n_def, vmax_def, n_cand, -
    size_t tscan;     // u32[C][Tn][2]  first rank of the tile, equal-key count before the tile
    size_t cand;      // uint2[C][Tn*kTile]  (key, max component bits) of threshold-bucket bins, tile-ordered
                      //                     (shares its bytes with mid)
    size_t prefix;    // u32[C][ceil(W/16)]  set bits before each group of 16 bitmap words (decode)
    size_t spec;      // float2[C][padded_bins(L)]  spectrum, each chunk on a 128-byte boundary
    size_t mid;       // float2[C][L/2] intermediate of the two-pass FFT
    size_t total;
};

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Per-tensor mode: the chunks of one launch are separate tensors of the same (padded) length, so where a chunk's
// samples and its record live is a table instead of c*L and c*S.  The table travels by value as a kernel argument
// (no host-to-device copy to order against the stream); longer lists are cut into launches of kMaxTableChunks.
constexpr int kMaxTableChunks = 64;
struct ChunkTable {
    uint64_t goff[kMaxTableChunks];  // element offset of the chunk's first sample in the gradient
    uint64_t roff[kMaxTableChunks];  // byte offset of the chunk's record from the first record of the launch
    uint32_t glen[kMaxTableChunks];  // samples present; the rest of the chunk is zero
};
// kernel parameter that is a ChunkTable in per-tensor launches and nothing otherwise
template <bool TABLE>
struct TableArg {
};
template <>
struct TableArg<true> {
    ChunkTable t;
};
template <bool TABLE>
inline TableArg<TABLE> table_arg(const ChunkTable* tab)
{
    TableArg<TABLE> a;
    if constexpr (TABLE) a.t = *tab;
    return a;
}

// Several senders' packed streams decoded into one spectrum (receiver under an allgather).
constexpr int kMaxPeers = 32;
struct PeerList {
    const uint8_t* p[kMaxPeers];  // first record of each peer's stream
};
// Extra workspace behind the ordinary one: per peer the group prefixes of its bitmaps and its header verdicts.
struct PeerWorkspace {
    size_t prefix;  // u32[P][C][ceil(W/16)]
    size_t verd;    // u32[P][C]
    size_t total;   // end of the whole workspace
};

static inline uint32_t tiles_per_chunk(uint32_t L) { return ((L / 2 + 1) + kTile - 1) / kTile; }
// chunk stride of the codec's own spectrum buffer, in complex bins: L/2+1 rounded up to a 128-byte multiple
static inline uint32_t padded_bins(uint32_t L) { return (L / 2 + 1 + 15u) & ~15u; }

// What a chunk's record describes: L/2+1 frequency bins, or (time-domain Top-k) the L samples themselves.
static inline uint32_t codec_bins(uint32_t L, int time_domain) { return time_domain ? L : L / 2 + 1; }
static inline uint32_t codec_tiles(uint32_t L, int time_domain)
{
    return (codec_bins(L, time_domain) + kTile - 1) / kTile;
}

// time_domain != 0: no spectrum and no FFT intermediate (the codec kernels read and write the gradient itself)
static inline Workspace make_workspace(size_t C, uint32_t L, int time_domain = 0)
{
    Workspace w;
    size_t B = codec_bins(L, time_domain), Tn = codec_tiles(L, time_domain), W = (B + 31) / 32;
    size_t off = 0;
    w.status = off; off += kControlBytes;
    w.hist = off;   off = align256(off + C * kHistBins * 4);
    w.sel = off;    off = align256(off + C * 8 * 4);
    w.tinfo = off;  off = align256(off + C * Tn * 16);
    w.tscan = off;  off = align256(off + C * Tn * 8);
    // The candidate list and the two-pass intermediate are never alive together (the sender's transform has
    // finished before the first candidate is written; the receiver has no candidates): one region serves both.
    const size_t cand_bytes = C * Tn * kTile * 8, mid_bytes = time_domain ? 0 : C * (size_t)L * 4;
    w.cand = off;
    w.mid = off;    off = align256(off + (cand_bytes > mid_bytes ? cand_bytes : mid_bytes));
    w.prefix = off; off = align256(off + C * W * 4);
    w.spec = off;   off = align256(off + (time_domain ? 0 : C * (size_t)padded_bins(L) * 8));
    w.total = off;
    return w;
}

// Where bin j of a chunk sits inside the chunk's spectrum.  pair_log = 0: natural order (the layout of the
// stage-level entry points).  pair_log = log2(N1) > 0: the two-pass FFT's own "paired" order, in which each run
// of N1 bins stores bin k1 next to bin N1-k1 (position 2*k1 / 2*k1+1; position 1 holds k1 = N1/2), so that the
// rows the real-FFT split combines are one 128-byte run for the FFT passes.  Bin L/2 keeps index L/2.
__device__ __forceinline__ uint32_t spec_index(uint32_t j, int pair_log)
{
    if (pair_log == 0) return j;
    const uint32_t N1 = 1u << pair_log, k1 = j & (N1 - 1u), hi = j - k1;
    const uint32_t pos = k1 < N1 / 2 ? 2u * k1 : (k1 == N1 / 2 ? 1u : 2u * (N1 - k1) + 1u);
    return hi + pos;
}

// Optional per-kernel event timing (prof.hip).
namespace prof {
bool enabled();
int begin(const char* name, hipStream_t s);
void end(int id, hipStream_t s);
void enable(bool on);
std::string report();
}  // namespace prof

// Launch `kernel` and, when profiling is on, bracket it with events under `name`.
#define FFTSP_LAUNCH(name, kernel, grid, block, lds, stream, ...)                    \
    do {                                                                             \
        const int fftsp_prof_id_ = ::fftsp::prof::enabled() ? ::fftsp::prof::begin(name, stream) : -1; \
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);           \
        if (fftsp_prof_id_ >= 0) ::fftsp::prof::end(fftsp_prof_id_, stream);         \
    } while (0)

// per-device tables; returns hipSuccess or the failing HIP error
hipError_t get_tables(Tables* out);

// FFT launchers (fft.hip).  Chunk c covers in[c*L, min(n, (c+1)*L)), zero beyond n.
// spec: chunk c's L/2+1 bins start at spec + 2*c*sstride floats (sstride in complex bins: L/2+1 for the dense
// layout of the stage-level entry points, a multiple of 16 inside the codec so that every chunk starts on a
// 128-byte line); mid: C*L floats of scratch (unused when L <= 2^14).
// hist (optional): u32[C][kHistBins]; the two-pass kernels clear zero_words words at zero_ptr (covering hist and
// the status words) and fill hist, setting *hist_done = 1; otherwise the caller clears and fills it.
// pair_spec != 0 asks the two-pass kernels to write the spectrum in paired order; *pair_log receives log2(N1)
// if they did, 0 otherwise (single-workgroup sizes always write natural order).
// tab != nullptr: per-tensor launch, chunk c is in[tab->goff[c] .. + tab->glen[c]) (n is not used)
// only_if (optional, two-pass sizes): device word; the kernels return at once unless it is non-zero
hipError_t launch_rfft(const float* in, size_t n, int logL, size_t C, float* spec, uint32_t sstride, float2* mid,
                       Tables t, uint32_t* hist, uint32_t* zero_ptr, size_t zero_words, int* hist_done, int pair_spec,
                       int* pair_log, const ChunkTable* tab, hipStream_t s, const uint32_t* only_if = nullptr);
// log2(N1) of the two-pass factorisation for chunk length 2^logL, 0 for single-workgroup sizes
int fft_pair_log(int logL);
// pair_spec != 0: the spectrum is in paired order (two-pass sizes only); the output is gain/L times the plain sum
hipError_t launch_irfft(const float* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out, float2* mid,
                        Tables t, int pair_spec, float gain, const ChunkTable* tab, hipStream_t s,
                        const uint32_t* only_if = nullptr);

// Fused two-pass transforms whose intermediate stays in the L2 caches (fused.hip).  They need the control block
// zeroed beforehand (launch_zero_control) and the per-pass kernels enqueued behind them with only_if = the give-up
// word, which redo the transform if the fused kernel could not finish.
struct FusedKnobs {
    int enabled;          // 0: never take the fused kernels
    uint32_t spin_limit;  // polls before a hand-over wait gives up
};
FusedKnobs fused_knobs();  // defaults overridden by the FFTSP_FUSED* environment variables (read at every call)
bool fused_applies(int logL, size_t C);
// spec: the codec's own buffer (paired order); hist: u32[C][kHistBins], already zero; ctl: the control block, zero
hipError_t launch_fused_rfft(const float* in, size_t n, int logL, size_t C, float2* spec, uint32_t sstride,
                             float2* scratch, Tables t, uint32_t* hist, uint32_t* ctl, const FusedKnobs& knobs,
                             hipStream_t s);
// the receiver's transform: spec is the codec's own decoded spectrum (paired order); ctl: the control block, zero
hipError_t launch_fused_irfft(const float2* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out,
                              float2* scratch, Tables t, float gain, uint32_t* ctl, const FusedKnobs& knobs,
                              hipStream_t s);
// zeroes the control block and the histograms behind it (one fill)
hipError_t launch_zero_control(uint8_t* ws_base, const Workspace& w, size_t C, hipStream_t s);

// Half-precision variant: chunk lengths of the two-pass FFT only (2^15 and up); spec and mid are the codec's own
// buffers, read and written as binary16 pairs (sstride in complex values); the histogram is always produced.
hipError_t launch_rfft_half(const float* in, size_t n, int logL, size_t C, void* spec, uint32_t sstride, void* mid,
                            Tables t, uint32_t* hist, uint32_t* zero_ptr, size_t zero_words, float in_scale,
                            int* pair_log, hipStream_t s);
hipError_t launch_irfft_half(const void* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out, void* mid,
                             Tables t, float gain, hipStream_t s);

// Codec launchers (codec.hip).
struct CodecArgs {
    size_t C;           // chunks
    uint32_t L;         // chunk length
    uint32_t k;         // kept bins per chunk
    int bits, m;        // code width, mantissa width
    size_t S;           // record stride in bytes
    uint32_t word3;     // 4th word of every record header
    uint32_t static_vmax;  // != 0: bit pattern of the caller's fixed range maximum (instead of the largest survivor)
    uint32_t sstride;   // distance between consecutive chunks' spectra, in complex bins
    const ChunkTable* tab;  // per-tensor launches: where each chunk's record lives (host pointer); else nullptr
    int time_domain;    // != 0: records describe the gradient's samples; `spec` of the launchers is the gradient
    size_t n;           // time domain: samples in the gradient (the last chunk may be short)
    int half;           // != 0: `spec` holds binary16 pairs (half-precision variant; two-pass chunk lengths only)
    int hdr_scale;      // stream header word 12: log2 of the factor on the spectrum (half-precision variant), else 0
    int pair_log;       // 0: spectrum in natural bin order; log2(N1): paired order (see spec_index)
    // stream header (written iff write_header)
    int write_header;
    uint64_t hdr_n;
    uint32_t hdr_L, hdr_C, hdr_k, hdr_S;
    float hdr_theta;
};
static inline PeerWorkspace make_peer_workspace(const Workspace& w, size_t C, uint32_t L, int npeers)
{
    PeerWorkspace pw;
    const size_t B = (size_t)L / 2 + 1, W = (B + 31) / 32, G = (W + 15) / 16;
    size_t off = w.total;
    pw.prefix = off; off = align256(off + (size_t)npeers * C * G * 4);
    pw.verd = off;   off = align256(off + (size_t)npeers * C * 4);
    pw.total = off;
    return pw;
}

// hist_ready != 0: the status words are cleared and the per-chunk histograms already hold the keys' top digit
hipError_t launch_encode(const float* spec, const CodecArgs& a, uint8_t* stream_base, uint8_t* records,
                         uint8_t* ws_base, const Workspace& w, int hist_ready, hipStream_t s);

// clears the device status word (for callers that decode a stream as several concurrent launch sets)
hipError_t launch_clear_status(uint8_t* ws_base, const Workspace& w, hipStream_t s);

// reset_status != 0: this call also clears the device status word (first record set of a stream)
hipError_t launch_decode(const uint8_t* stream_base, const uint8_t* records, const CodecArgs& a, float* spec,
                         uint8_t* ws_base, const Workspace& w, int check_header, int reset_status, hipStream_t s);

// npeers streams (each: 64-byte header + records) summed bin by bin, in list order, into spec; clears the status word
hipError_t launch_decode_peers(const PeerList& streams, int npeers, const CodecArgs& a, float* spec, uint8_t* ws_base,
                               const Workspace& w, const PeerWorkspace& pw, hipStream_t s);

}  // namespace fftsp

// C ABI of libfftsp.so (see include/fftsp.h): argument checks, workspace carving, launch order.
#include "../../include/fftsp.h"
#include "internal.h"
#include "twiddle_table.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

namespace fftsp {

namespace {
// Compile-time tables in device memory (twiddle_table.h): one copy per device, loaded with the code object.
// (not declared const: a const device variable that no device code names is dropped from the code object, and
// the host-side lookup of its address then finds nothing)
static __device__ twtab::Table g_tw_hi = twtab::make_table<11>();
static __device__ twtab::Table g_tw_lo = twtab::make_table<22>();
static_assert(sizeof(twtab::Pair) == sizeof(float2), "table entries are read as float2");

struct DeviceTables {
    bool ready = false;
    Tables t{nullptr, nullptr};
};
constexpr int kMaxDevices = 64;
DeviceTables g_tables[kMaxDevices];
std::mutex g_mutex;
}  // namespace

// Looks up this device's addresses of the two tables once; allocates nothing and enqueues nothing.
hipError_t get_tables(Tables* out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceTables& d = g_tables[dev];
    if (!d.ready) {
        void *hi = nullptr, *lo = nullptr;
        e = hipGetSymbolAddress(&hi, HIP_SYMBOL(g_tw_hi));
        if (e == hipSuccess) e = hipGetSymbolAddress(&lo, HIP_SYMBOL(g_tw_lo));
        if (e != hipSuccess) return e;
        d.t.hi = static_cast<const float2*>(hi);
        d.t.lo = static_cast<const float2*>(lo);
        d.ready = true;
    }
    *out = d.t;
    return hipSuccess;
}

namespace {

int log2_exact(uint32_t v)
{
    if (v == 0 || (v & (v - 1))) return -1;
    int l = 0;
    while ((1u << l) < v) ++l;
    return l;
}

int check_len(uint32_t L)
{
    const int l = log2_exact(L);
    if (l < kMinLogL || l > kMaxLogL) return -1;
    return l;
}

bool theta_ok(float t) { return t >= 0.0f && t <= 1.0f; }  // false for NaN

uint32_t kept(uint32_t L, float theta)
{
    const double B = (double)(L / 2 + 1);
    double k = std::floor((double)theta * B + 0.5);
    if (k < 0) k = 0;
    if (k > B) k = B;
    return (uint32_t)k;
}

int mantissa(int bits)
{
    if (bits == 32) return 23;
    if (bits < 3 || bits > 16) return -1;
    const int e = bits <= 6 ? 3 : (bits <= 12 ? 4 : 5);
    const int m = bits - 1 - e;
    return m < 1 ? 1 : m;
}

size_t record_stride(uint32_t L, uint32_t k, int bits)
{
    const size_t B = (size_t)L / 2 + 1, W = (B + 31) / 32;
    const size_t code_words = ((size_t)2 * k * (size_t)bits + 31) / 32;
    return (16 + 4 * W + 4 * code_words + 15) & ~(size_t)15;
}

constexpr size_t kStreamHeader = 64;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint32_t segment_length(size_t size)
{
    uint32_t L = 32;
    while ((size_t)L < size && L < (1u << 31)) L <<= 1;
    return L;
}

struct Plan {
    size_t n, C;
    uint32_t L, k;
    int logL, bits, m;
    size_t S;
    Workspace ws;
};

// common argument checks for the uniform-chunk entry points; theta/bits optional
int make_plan(Plan* p, size_t n, uint32_t L, const float* theta, const int* bits)
{
    if (n == 0) return FFTSP_EINVAL;
    p->logL = check_len(L);
    if (p->logL < 0) return FFTSP_EUNSUPPORTED;
    p->n = n;
    p->L = L;
    p->C = (n + L - 1) / L;
    p->k = 0;
    p->bits = 32;
    p->m = 23;
    if (theta) {
        if (!theta_ok(*theta)) return FFTSP_EINVAL;
        p->k = kept(L, *theta);
    }
    if (bits) {
        p->m = mantissa(*bits);
        if (p->m < 0) return FFTSP_EINVAL;
        p->bits = *bits;
    }
    p->S = record_stride(L, p->k, p->bits);
    p->ws = make_workspace(p->C, L);
    return FFTSP_OK;
}

CodecArgs codec_args(const Plan& p, float theta)
{
    CodecArgs a{};
    a.C = p.C;
    a.L = p.L;
    a.k = p.k;
    a.bits = p.bits;
    a.m = p.m;
    a.S = p.S;
    a.word3 = 0;
    a.sstride = p.L / 2 + 1;  // dense layout, natural bin order; the codec's own buffer overrides both
    a.pair_log = 0;
    a.write_header = 1;
    a.hdr_n = p.n;
    a.hdr_L = p.L;
    a.hdr_C = (uint32_t)p.C;
    a.hdr_k = p.k;
    a.hdr_S = (uint32_t)p.S;
    a.hdr_theta = theta;
    return a;
}

int hip_status(hipError_t e) { return e == hipSuccess ? FFTSP_OK : FFTSP_EHIP; }

// ---- time-domain Top-k: chunks of L samples are ranked, coded and packed as they are ----
// a chunk's selection runs in one workgroup that keeps per-tile state in LDS for up to 1025 tiles of 2048
constexpr int kTopkMaxLogL = 21;

uint32_t topk_kept(uint32_t L, float theta)
{
    double k = std::floor((double)theta * (double)L + 0.5);
    if (k < 0) k = 0;
    if (k > (double)L) k = (double)L;
    return (uint32_t)k;
}

size_t topk_record_stride(uint32_t L, uint32_t k, int bits)
{
    const size_t W = ((size_t)L + 31) / 32;
    const size_t code_words = ((size_t)k * (size_t)bits + 31) / 32;
    return (16 + 4 * W + 4 * code_words + 15) & ~(size_t)15;
}

int make_topk_plan(Plan* p, size_t n, uint32_t L, const float* theta, int bits)
{
    if (n == 0) return FFTSP_EINVAL;
    p->logL = check_len(L);
    if (p->logL < 0 || p->logL > kTopkMaxLogL) return FFTSP_EUNSUPPORTED;
    p->n = n;
    p->L = L;
    p->C = (n + L - 1) / L;
    p->k = 0;
    if (theta) {
        if (!theta_ok(*theta)) return FFTSP_EINVAL;
        p->k = topk_kept(L, *theta);
    }
    p->m = mantissa(bits);
    if (p->m < 0) return FFTSP_EINVAL;
    p->bits = bits;
    p->S = topk_record_stride(L, p->k, bits);
    p->ws = make_workspace(p->C, L, 1);
    return FFTSP_OK;
}

CodecArgs topk_args(const Plan& p, float theta)
{
    CodecArgs a = codec_args(p, theta);
    a.sstride = p.L;  // chunk c of the "spectrum" is the gradient's own samples [c*L, (c+1)*L)
    a.time_domain = 1;
    a.n = p.n;
    return a;
}

// quantizer options (Sec. 3.2.1): a chosen m replaces the default of the width, a static range replaces the
// per-chunk fit; q == nullptr keeps both defaults
int apply_quantizer(Plan* p, const fftsp_quantizer* q, uint32_t* static_vmax)
{
    *static_vmax = 0;
    if (!q) return FFTSP_OK;
    if (q->mantissa_bits != 0 && p->bits != 32) {
        if (q->mantissa_bits < 1 || q->mantissa_bits > p->bits - 1) return FFTSP_EINVAL;
        p->m = q->mantissa_bits;
    }
    const float r = q->range_max;
    if (!(r >= 0.0f) || std::isinf(r)) return FFTSP_EINVAL;
    if (r > 0.0f) std::memcpy(static_vmax, &r, sizeof(uint32_t));
    return FFTSP_OK;
}

// The receiver's inverse transform of the codec's own spectrum buffer (uniform chunks).  The decode kernels that
// ran before it on this stream have cleared the control block.
hipError_t inverse_of_decoded(const Plan& p, const float* spec, uint32_t sstride, int pair_log, float* out, uint8_t* ws,
                              Tables t, float gain, hipStream_t s)
{
    float2* mid = reinterpret_cast<float2*>(ws + p.ws.mid);
    const FusedKnobs knobs = fused_knobs();
    if (knobs.enabled && pair_log != 0 && fused_applies(p.logL, p.C)) {
        uint32_t* ctl = reinterpret_cast<uint32_t*>(ws + p.ws.status);
        hipError_t e = launch_fused_irfft(reinterpret_cast<const float2*>(spec), sstride, p.n, p.logL, p.C, out, mid, t,
                                          gain, ctl, knobs, s);
        if (e != hipSuccess) return e;
        // stand-by: the per-pass kernels redo the transform if the fused kernel gave up
        return launch_irfft(spec, sstride, p.n, p.logL, p.C, out, mid, t, 1, gain, nullptr, s, ctl + kCtlGaveUpWord);
    }
    return launch_irfft(spec, sstride, p.n, p.logL, p.C, out, mid, t, pair_log != 0, gain, nullptr, s);
}

}  // namespace
}  // namespace fftsp

using namespace fftsp;

extern "C" {

int fftsp_kept_per_chunk(uint32_t chunk_len, float theta, uint32_t* k_out)
{
    if (!k_out || !theta_ok(theta)) return FFTSP_EINVAL;
    if (check_len(chunk_len) < 0) return FFTSP_EUNSUPPORTED;
    *k_out = kept(chunk_len, theta);
    return FFTSP_OK;
}

int fftsp_mantissa_bits(int bits) { return mantissa(bits); }

size_t fftsp_packed_bytes(size_t n, uint32_t chunk_len, float theta, int bits)
{
    Plan p;
    if (make_plan(&p, n, chunk_len, &theta, &bits) != FFTSP_OK) return 0;
    return kStreamHeader + p.C * p.S;
}

size_t fftsp_workspace_bytes(size_t n, uint32_t chunk_len, int bits)
{
    Plan p;
    if (make_plan(&p, n, chunk_len, nullptr, &bits) != FFTSP_OK) return 0;
    return p.ws.total;
}

int fftsp_rfft(const float* d_grad, size_t n, uint32_t chunk_len, float* d_spec, void* d_workspace,
               size_t workspace_bytes, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, nullptr, nullptr);
    if (rc) return rc;
    if (!d_grad || !d_spec || !d_workspace || !aligned16(d_grad) || !aligned16(d_spec) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    return hip_status(launch_rfft(d_grad, n, p.logL, p.C, d_spec, p.L / 2 + 1, reinterpret_cast<float2*>(ws + p.ws.mid), t,
                                  nullptr, nullptr, 0, nullptr, 0, nullptr, nullptr, reinterpret_cast<hipStream_t>(stream)));
}

int fftsp_irfft(const float* d_spec, size_t n, uint32_t chunk_len, float* d_grad_out, void* d_workspace,
                size_t workspace_bytes, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, nullptr, nullptr);
    if (rc) return rc;
    if (!d_grad_out || !d_spec || !d_workspace || !aligned16(d_grad_out) || !aligned16(d_spec) ||
        !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    return hip_status(launch_irfft(d_spec, p.L / 2 + 1, n, p.logL, p.C, d_grad_out, reinterpret_cast<float2*>(ws + p.ws.mid), t,
                                   0, 1.0f, nullptr, reinterpret_cast<hipStream_t>(stream)));
}

int fftsp_encode_spectrum_q(const float* d_spec, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                          size_t packed_capacity, void* d_workspace, size_t workspace_bytes, const fftsp_quantizer* quantizer, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    uint32_t static_vmax = 0;
    rc = apply_quantizer(&p, quantizer, &static_vmax);
    if (rc) return rc;
    if (!d_spec || !d_packed || !d_workspace || !aligned16(d_spec) || !aligned16(d_packed) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_capacity < kStreamHeader + p.C * p.S) return FFTSP_ENOSPC;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    uint8_t* out = static_cast<uint8_t*>(d_packed);
    CodecArgs a = codec_args(p, theta);
    a.static_vmax = static_vmax;
    return hip_status(launch_encode(d_spec, a, out, out + kStreamHeader, ws, p.ws, 0,
                                    reinterpret_cast<hipStream_t>(stream)));
}

int fftsp_encode_spectrum(const float* d_spec, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                          size_t packed_capacity, void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    return fftsp_encode_spectrum_q(d_spec, n, chunk_len, theta, bits, d_packed, packed_capacity, d_workspace, workspace_bytes, nullptr, stream);
}

int fftsp_decode_spectrum_q(const void* d_packed, size_t packed_bytes, size_t n, uint32_t chunk_len, float theta,
                          int bits, float* d_spec, void* d_workspace, size_t workspace_bytes, const fftsp_quantizer* quantizer, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    uint32_t static_vmax = 0;
    rc = apply_quantizer(&p, quantizer, &static_vmax);
    if (rc) return rc;
    (void)static_vmax;  // the receiver reads the range from the records; only m matters here
    if (!d_spec || !d_packed || !d_workspace || !aligned16(d_spec) || !aligned16(d_packed) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_bytes < kStreamHeader + p.C * p.S) return FFTSP_EFORMAT;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    const uint8_t* in = static_cast<const uint8_t*>(d_packed);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t e = launch_decode(in, in + kStreamHeader, codec_args(p, theta), d_spec, ws, p.ws, 1, 1, s);
    return hip_status(e);
}

int fftsp_decode_spectrum(const void* d_packed, size_t packed_bytes, size_t n, uint32_t chunk_len, float theta,
                          int bits, float* d_spec, void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    return fftsp_decode_spectrum_q(d_packed, packed_bytes, n, chunk_len, theta, bits, d_spec, d_workspace, workspace_bytes, nullptr, stream);
}

}  // extern "C"

// the sender proper, shared by the entry points that differ only in where the workspace comes from
static int compress_impl(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                         size_t packed_capacity, void* d_workspace, size_t workspace_bytes,
                         const fftsp_quantizer* quantizer, hipStream_t s)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    uint32_t static_vmax = 0;
    rc = apply_quantizer(&p, quantizer, &static_vmax);
    if (rc) return rc;
    if (!d_grad || !d_packed || !d_workspace || !aligned16(d_grad) || !aligned16(d_packed) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_capacity < kStreamHeader + p.C * p.S) return FFTSP_ENOSPC;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    uint8_t* out = static_cast<uint8_t*>(d_packed);
    float* spec = reinterpret_cast<float*>(ws + p.ws.spec);
    int hist_done = 0;
    CodecArgs a = codec_args(p, theta);
    a.static_vmax = static_vmax;
    a.sstride = padded_bins(p.L);
    uint32_t* ctl = reinterpret_cast<uint32_t*>(ws + p.ws.status);
    uint32_t* hist = reinterpret_cast<uint32_t*>(ws + p.ws.hist);
    float2* mid = reinterpret_cast<float2*>(ws + p.ws.mid);
    const FusedKnobs knobs = fused_knobs();
    hipError_t e;
    if (knobs.enabled && fused_applies(p.logL, p.C)) {
        // both passes in one kernel, the intermediate in the L2 caches (fused.hip); the per-pass kernels stand by
        // behind it and run only if it gave up (they then clear the histograms again, not the control block)
        e = launch_zero_control(ws, p.ws, p.C, s);
        if (e == hipSuccess)
            e = launch_fused_rfft(d_grad, n, p.logL, p.C, reinterpret_cast<float2*>(spec), a.sstride, mid, t, hist, ctl,
                                  knobs, s);
        if (e == hipSuccess)
            e = launch_rfft(d_grad, n, p.logL, p.C, spec, a.sstride, mid, t, hist, hist, p.C * kHistBins, &hist_done, 1,
                            &a.pair_log, nullptr, s, ctl + kCtlGaveUpWord);
    } else {
        e = launch_rfft(d_grad, n, p.logL, p.C, spec, a.sstride, mid, t, hist, ctl,
                        (p.ws.hist - p.ws.status) / 4 + p.C * kHistBins, &hist_done, 1, &a.pair_log, nullptr, s);
    }
    if (e == hipSuccess)
        e = launch_encode(spec, a, out, out + kStreamHeader, ws, p.ws, hist_done, s);
    return hip_status(e);
}

// Workspace of fftsp_compress_static: one array per device inside the code object.  Host code never uses the
// array's name as an address: the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[FFTSP_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[64];
static std::mutex g_scratch_mutex;

static hipError_t static_scratch(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

extern "C" {

int fftsp_compress_q(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                   size_t packed_capacity, void* d_workspace, size_t workspace_bytes, const fftsp_quantizer* quantizer, fftsp_stream_t stream)
{
    return compress_impl(d_grad, n, chunk_len, theta, bits, d_packed, packed_capacity, d_workspace, workspace_bytes,
                         quantizer, reinterpret_cast<hipStream_t>(stream));
}

int fftsp_compress_static(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                          size_t packed_capacity, fftsp_stream_t stream)
{
    // sizes first: a call that cannot fit is refused before the device is touched
    Plan p;
    const int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    if (p.ws.total > (size_t)FFTSP_STATIC_SCRATCH_BYTES) return FFTSP_EWORKSPACE;
    void* ws = nullptr;
    if (static_scratch(&ws) != hipSuccess) return FFTSP_EHIP;
    return compress_impl(d_grad, n, chunk_len, theta, bits, d_packed, packed_capacity, ws,
                         (size_t)FFTSP_STATIC_SCRATCH_BYTES, nullptr, reinterpret_cast<hipStream_t>(stream));
}

int fftsp_compress(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                   size_t packed_capacity, void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    return fftsp_compress_q(d_grad, n, chunk_len, theta, bits, d_packed, packed_capacity, d_workspace, workspace_bytes, nullptr, stream);
}

int fftsp_decompress_q(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n, uint32_t chunk_len,
                     float theta, int bits, void* d_workspace, size_t workspace_bytes, const fftsp_quantizer* quantizer, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    uint32_t static_vmax = 0;
    rc = apply_quantizer(&p, quantizer, &static_vmax);
    if (rc) return rc;
    (void)static_vmax;  // the receiver reads the range from the records; only m matters here
    if (!d_grad_out || !d_packed || !d_workspace || !aligned16(d_grad_out) || !aligned16(d_packed) ||
        !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_bytes < kStreamHeader + p.C * p.S) return FFTSP_EFORMAT;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    const uint8_t* in = static_cast<const uint8_t*>(d_packed);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    float* spec = reinterpret_cast<float*>(ws + p.ws.spec);
    CodecArgs a = codec_args(p, theta);
    a.sstride = padded_bins(p.L);
    a.pair_log = fft_pair_log(p.logL);
    hipError_t e = launch_decode(in, in + kStreamHeader, a, spec, ws, p.ws, 1, 1, s);
    if (e == hipSuccess) e = inverse_of_decoded(p, spec, a.sstride, a.pair_log, d_grad_out, ws, t, 1.0f, s);
    return hip_status(e);
}

int fftsp_decompress(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n, uint32_t chunk_len,
                     float theta, int bits, void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    return fftsp_decompress_q(d_packed, packed_bytes, d_grad_out, n, chunk_len, theta, bits, d_workspace, workspace_bytes, nullptr, stream);
}

/* ---------------- receiver under an allgather: several peers' streams, one inverse transform ---------------- */

static int peer_list(PeerList* out, const void* const* d_packed, int npeers)
{
    if (!d_packed || npeers < 1) return FFTSP_EINVAL;
    if (npeers > kMaxPeers) return FFTSP_EUNSUPPORTED;
    for (int i = 0; i < kMaxPeers; ++i) out->p[i] = nullptr;
    for (int i = 0; i < npeers; ++i) {
        if (!d_packed[i] || !aligned16(d_packed[i])) return FFTSP_EINVAL;
        out->p[i] = static_cast<const uint8_t*>(d_packed[i]);
    }
    return FFTSP_OK;
}

size_t fftsp_workspace_bytes_accumulate(size_t n, uint32_t chunk_len, int bits, int npeers)
{
    Plan p;
    if (npeers < 1 || npeers > kMaxPeers || make_plan(&p, n, chunk_len, nullptr, &bits) != FFTSP_OK) return 0;
    return make_peer_workspace(p.ws, p.C, p.L, npeers).total;
}

int fftsp_decode_accumulate_spectrum(const void* const* d_packed, int npeers, size_t packed_bytes, size_t n,
                                     uint32_t chunk_len, float theta, int bits, float* d_spec, void* d_workspace,
                                     size_t workspace_bytes, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    PeerList peers;
    rc = peer_list(&peers, d_packed, npeers);
    if (rc) return rc;
    if (!d_spec || !d_workspace || !aligned16(d_spec) || !aligned16(d_workspace)) return FFTSP_EINVAL;
    if (packed_bytes < kStreamHeader + p.C * p.S) return FFTSP_EFORMAT;
    const PeerWorkspace pw = make_peer_workspace(p.ws, p.C, p.L, npeers);
    if (workspace_bytes < pw.total) return FFTSP_EWORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    return hip_status(launch_decode_peers(peers, npeers, codec_args(p, theta), d_spec, ws, p.ws, pw,
                                          reinterpret_cast<hipStream_t>(stream)));
}

int fftsp_decompress_accumulate(const void* const* d_packed, int npeers, size_t packed_bytes, float scale,
                                float* d_grad_out, size_t n, uint32_t chunk_len, float theta, int bits,
                                void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    PeerList peers;
    rc = peer_list(&peers, d_packed, npeers);
    if (rc) return rc;
    if (!d_grad_out || !d_workspace || !aligned16(d_grad_out) || !aligned16(d_workspace) || !(scale == scale))
        return FFTSP_EINVAL;
    if (packed_bytes < kStreamHeader + p.C * p.S) return FFTSP_EFORMAT;
    const PeerWorkspace pw = make_peer_workspace(p.ws, p.C, p.L, npeers);
    if (workspace_bytes < pw.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    float* spec = reinterpret_cast<float*>(ws + p.ws.spec);
    CodecArgs a = codec_args(p, theta);
    a.sstride = padded_bins(p.L);
    a.pair_log = fft_pair_log(p.logL);
    hipError_t e = launch_decode_peers(peers, npeers, a, spec, ws, p.ws, pw, s);
    if (e == hipSuccess) e = inverse_of_decoded(p, spec, a.sstride, a.pair_log, d_grad_out, ws, t, scale, s);
    return hip_status(e);
}

/* ---------------- half-precision variant: binary16 between the passes and in the spectrum ---------------- */

namespace {
constexpr int kHalfMinLogL = 15;  // the two-pass FFT starts here; shorter chunks do not need the variant
bool half_scale_ok(int s) { return s >= -24 && s <= 24; }
}  // namespace

int fftsp_compress_h(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, int scale_log2,
                     void* d_packed, size_t packed_capacity, void* d_workspace, size_t workspace_bytes,
                     fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    if (p.logL < kHalfMinLogL) return FFTSP_EUNSUPPORTED;
    if (!half_scale_ok(scale_log2)) return FFTSP_EINVAL;
    if (!d_grad || !d_packed || !d_workspace || !aligned16(d_grad) || !aligned16(d_packed) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_capacity < kStreamHeader + p.C * p.S) return FFTSP_ENOSPC;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    uint8_t* out = static_cast<uint8_t*>(d_packed);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    CodecArgs a = codec_args(p, theta);
    a.sstride = padded_bins(p.L);
    a.half = 1;
    a.hdr_scale = scale_log2;
    hipError_t e = launch_rfft_half(d_grad, n, p.logL, p.C, ws + p.ws.spec, a.sstride, ws + p.ws.mid, t,
                                    reinterpret_cast<uint32_t*>(ws + p.ws.hist),
                                    reinterpret_cast<uint32_t*>(ws + p.ws.status),
                                    (p.ws.hist - p.ws.status) / 4 + p.C * kHistBins, std::ldexp(1.0f, scale_log2),
                                    &a.pair_log, s);
    if (e == hipSuccess)
        e = launch_encode(reinterpret_cast<const float*>(ws + p.ws.spec), a, out, out + kStreamHeader, ws, p.ws, 1, s);
    return hip_status(e);
}

int fftsp_decompress_h(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n, uint32_t chunk_len,
                       float theta, int bits, int scale_log2, void* d_workspace, size_t workspace_bytes,
                       fftsp_stream_t stream)
{
    Plan p;
    int rc = make_plan(&p, n, chunk_len, &theta, &bits);
    if (rc) return rc;
    if (p.logL < kHalfMinLogL) return FFTSP_EUNSUPPORTED;
    if (!half_scale_ok(scale_log2)) return FFTSP_EINVAL;
    if (!d_grad_out || !d_packed || !d_workspace || !aligned16(d_grad_out) || !aligned16(d_packed) ||
        !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_bytes < kStreamHeader + p.C * p.S) return FFTSP_EFORMAT;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    const uint8_t* in = static_cast<const uint8_t*>(d_packed);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    CodecArgs a = codec_args(p, theta);
    a.sstride = padded_bins(p.L);
    a.pair_log = fft_pair_log(p.logL);
    a.half = 1;
    a.hdr_scale = scale_log2;
    hipError_t e = launch_decode(in, in + kStreamHeader, a, reinterpret_cast<float*>(ws + p.ws.spec), ws, p.ws, 1, 1, s);
    if (e == hipSuccess)
        e = launch_irfft_half(ws + p.ws.spec, a.sstride, n, p.logL, p.C, d_grad_out, ws + p.ws.mid, t,
                              std::ldexp(1.0f, -scale_log2), s);
    return hip_status(e);
}

/* ---------------- time-domain Top-k: the same select / quantize / pack kernels, no transform ---------------- */

int fftsp_topk_kept_per_chunk(uint32_t chunk_len, float theta, uint32_t* k_out)
{
    if (!k_out || !theta_ok(theta)) return FFTSP_EINVAL;
    const int l = check_len(chunk_len);
    if (l < 0 || l > kTopkMaxLogL) return FFTSP_EUNSUPPORTED;
    *k_out = topk_kept(chunk_len, theta);
    return FFTSP_OK;
}

size_t fftsp_topk_packed_bytes(size_t n, uint32_t chunk_len, float theta, int bits)
{
    Plan p;
    if (make_topk_plan(&p, n, chunk_len, &theta, bits) != FFTSP_OK) return 0;
    return kStreamHeader + p.C * p.S;
}

size_t fftsp_topk_workspace_bytes(size_t n, uint32_t chunk_len, int bits)
{
    Plan p;
    if (make_topk_plan(&p, n, chunk_len, nullptr, bits) != FFTSP_OK) return 0;
    return p.ws.total;
}

int fftsp_topk_compress(const float* d_grad, size_t n, uint32_t chunk_len, float theta, int bits, void* d_packed,
                        size_t packed_capacity, void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_topk_plan(&p, n, chunk_len, &theta, bits);
    if (rc) return rc;
    if (!d_grad || !d_packed || !d_workspace || !aligned16(d_grad) || !aligned16(d_packed) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_capacity < kStreamHeader + p.C * p.S) return FFTSP_ENOSPC;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    uint8_t* out = static_cast<uint8_t*>(d_packed);
    const CodecArgs a = topk_args(p, theta);
    return hip_status(launch_encode(d_grad, a, out, out + kStreamHeader, ws, p.ws, 0,
                                    reinterpret_cast<hipStream_t>(stream)));
}

int fftsp_topk_decompress(const void* d_packed, size_t packed_bytes, float* d_grad_out, size_t n, uint32_t chunk_len,
                          float theta, int bits, void* d_workspace, size_t workspace_bytes, fftsp_stream_t stream)
{
    Plan p;
    int rc = make_topk_plan(&p, n, chunk_len, &theta, bits);
    if (rc) return rc;
    if (!d_grad_out || !d_packed || !d_workspace || !aligned16(d_grad_out) || !aligned16(d_packed) ||
        !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_bytes < kStreamHeader + p.C * p.S) return FFTSP_EFORMAT;
    if (workspace_bytes < p.ws.total) return FFTSP_EWORKSPACE;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    const uint8_t* in = static_cast<const uint8_t*>(d_packed);
    const CodecArgs a = topk_args(p, theta);
    return hip_status(launch_decode(in, in + kStreamHeader, a, d_grad_out, ws, p.ws, 1, 1,
                                    reinterpret_cast<hipStream_t>(stream)));
}

/* ---------------- per-tensor variant: one single-chunk codec per segment ---------------- */

static int segments_ok(const size_t* off, int nseg)
{
    if (!off || nseg <= 0) return FFTSP_EINVAL;
    for (int i = 0; i < nseg; ++i) {
        if (off[i + 1] <= off[i]) return FFTSP_EINVAL;
        if (off[i + 1] - off[i] > ((size_t)1 << kMaxLogL)) return FFTSP_EUNSUPPORTED;
    }
    return FFTSP_OK;
}

size_t fftsp_packed_bytes_segments(const size_t* seg_offsets, int nseg, float theta, int bits)
{
    if (segments_ok(seg_offsets, nseg) != FFTSP_OK || !theta_ok(theta) || mantissa(bits) < 0) return 0;
    size_t total = kStreamHeader;
    for (int i = 0; i < nseg; ++i) {
        const uint32_t L = segment_length(seg_offsets[i + 1] - seg_offsets[i]);
        total += record_stride(L, kept(L, theta), bits);
    }
    return total;
}

// Tensors that pad to the same chunk length L run as the chunks of one launch set, at most this many at a time
// (the per-launch table holds kMaxTableChunks; long chunks are also capped at 2^26 samples per launch set so that the
// workspace stays a small multiple of the largest tensor).
static size_t batch_cap(uint32_t L)
{
    const size_t by_size = ((size_t)1 << 26) / L;
    const size_t cap = by_size < (size_t)kMaxTableChunks ? by_size : (size_t)kMaxTableChunks;
    return cap < 1 ? 1 : cap;
}

// One launch set of the per-tensor path: `count` tensors of padded length L.
struct SegBatch {
    uint32_t L;
    size_t count;
    ChunkTable tab;
};

// Groups the tensors by padded length (ascending) and cuts every group into launch sets.  Records keep tensor
// order in the stream: tensor i's record starts rec_off[i] bytes after the stream header.
static std::vector<SegBatch> plan_segments(const size_t* off, int nseg, float theta, int bits, bool with_tables)
{
    std::vector<uint32_t> len(nseg);
    std::vector<size_t> rec_off(nseg);
    std::vector<int> order(nseg);
    size_t ro = 0;
    for (int i = 0; i < nseg; ++i) {
        len[i] = segment_length(off[i + 1] - off[i]);
        rec_off[i] = ro;
        if (with_tables) ro += record_stride(len[i], kept(len[i], theta), bits);
        order[i] = i;
    }
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return len[a] < len[b]; });
    std::vector<SegBatch> out;
    for (int j = 0; j < nseg; ++j) {
        const int i = order[j];
        if (out.empty() || out.back().L != len[i] || out.back().count == batch_cap(len[i])) {
            out.emplace_back();
            out.back().L = len[i];
            out.back().count = 0;
        }
        SegBatch& b = out.back();
        if (with_tables) {
            b.tab.goff[b.count] = off[i];
            b.tab.glen[b.count] = (uint32_t)(off[i + 1] - off[i]);
            b.tab.roff[b.count] = rec_off[i];
        }
        ++b.count;
    }
    return out;
}

// The launch sets of a per-tensor call are independent chains of short kernels (most tensors are small), so they
// run on up to kSegLanes streams at once: the caller's and streams of the library's own that fork from and join
// back into the caller's through events.  The call stays one unit of work on the caller's stream and can be
// captured into a graph.  Every lane works in a workspace region of its own, sized for the largest launch set.
constexpr int kSegLanes = 4;
struct SegLanes {
    bool ready = false;
    hipStream_t s[kSegLanes - 1];
    hipEvent_t fork, join[kSegLanes - 1];
};
static SegLanes g_seg_lanes[64];
static std::mutex g_seg_mutex;  // held while a call enqueues: the events are shared by all calls on a device

static size_t segment_region_bytes(const std::vector<SegBatch>& batches)
{
    size_t best = 0;
    for (const SegBatch& b : batches) {
        const size_t t = make_workspace(b.count, b.L).total;
        best = t > best ? t : best;
    }
    return align256(best);
}

static int segment_lanes(size_t nbatches)
{
    return (int)(nbatches < (size_t)kSegLanes ? nbatches : (size_t)kSegLanes);
}

size_t fftsp_workspace_bytes_segments(const size_t* seg_offsets, int nseg, int bits)
{
    if (segments_ok(seg_offsets, nseg) != FFTSP_OK || mantissa(bits) < 0) return 0;
    const std::vector<SegBatch> batches = plan_segments(seg_offsets, nseg, 0.5f, bits, false);
    return (size_t)segment_lanes(batches.size()) * segment_region_bytes(batches);
}

// Heaviest launch set first, each onto the lane with the least work so far (work = samples); lane 0 is the caller's
// stream.  Returns the lane of every launch set.
static std::vector<int> assign_lanes(const std::vector<SegBatch>& batches, int lanes)
{
    std::vector<size_t> order(batches.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) {
        return batches[a].count * (size_t)batches[a].L > batches[b].count * (size_t)batches[b].L;
    });
    std::vector<size_t> load((size_t)lanes, 0);
    std::vector<int> lane_of(batches.size(), 0);
    for (size_t i : order) {
        int best = 0;
        for (int l = 1; l < lanes; ++l)
            if (load[(size_t)l] < load[(size_t)best]) best = l;
        lane_of[i] = best;
        // a launch set costs its samples plus a fixed price for its ten or so launches
        load[(size_t)best] += batches[i].count * (size_t)batches[i].L + ((size_t)1 << 18);
    }
    return lane_of;
}

}  // extern "C" (a template cannot have C linkage)

// The capture `s` is being recorded into: its id, 0 if none, ~0 if the capture is broken.
static hipError_t capture_of(hipStream_t s, unsigned long long* id)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    unsigned long long i = 0;
    const hipError_t e = hipStreamGetCaptureInfo(s, &st, &i);
    if (e != hipSuccess) return e;
    *id = st == hipStreamCaptureStatusNone ? 0ull : (st == hipStreamCaptureStatusActive ? i : ~0ull);
    return hipSuccess;
}

static void destroy_lanes(SegLanes& ln, int streams, int joins, bool fork)
{
    for (int i = 0; i < streams; ++i) (void)hipStreamDestroy(ln.s[i]);
    for (int i = 0; i < joins; ++i) (void)hipEventDestroy(ln.join[i]);
    if (fork) (void)hipEventDestroy(ln.fork);
}

// body(launch set index, stream, lane) enqueues one launch set; sets of one lane run in index order on its stream.
// The side streams belong to the device, not to a caller.  A caller that records its stream into a graph pulls them
// into that capture until it ends, so a call falls back to the caller's stream alone (lane 0, the same result,
// the launch sets one after the other) when a side stream is being recorded into a capture other than the
// caller's own, and when the side streams do not exist yet and the caller is recording (nothing is created while a
// capture is open).
template <typename F>
static hipError_t run_on_lanes(hipStream_t user, const std::vector<int>& lane_of, int lanes, F&& body)
{
    auto serial = [&]() {
        for (size_t bi = 0; bi < lane_of.size(); ++bi) {
            const hipError_t e = body(bi, user, 0);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    };
    if (lanes <= 1) return serial();
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_seg_mutex);
    SegLanes& ln = g_seg_lanes[dev];
    unsigned long long mine = 0;
    e = capture_of(user, &mine);
    if (e != hipSuccess) return e;
    if (!ln.ready) {
        if (mine != 0) return serial();
        int streams = 0, joins = 0;
        for (int i = 0; i < kSegLanes - 1 && e == hipSuccess; ++i) {
            e = hipStreamCreateWithFlags(&ln.s[i], hipStreamNonBlocking);  // default priority
            if (e != hipSuccess) break;
            ++streams;
            e = hipEventCreateWithFlags(&ln.join[i], hipEventDisableTiming);
            if (e == hipSuccess) ++joins;
        }
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ln.fork, hipEventDisableTiming);
        if (e != hipSuccess) {
            destroy_lanes(ln, streams, joins, false);  // the next call starts over
            return e;
        }
        ln.ready = true;
    }
    for (int l = 1; l < lanes; ++l) {
        unsigned long long theirs = 0;
        e = capture_of(ln.s[l - 1], &theirs);
        if (e != hipSuccess) return e;
        if (theirs != 0 && theirs != mine) return serial();
    }
    e = hipEventRecord(ln.fork, user);
    for (int l = 1; l < lanes && e == hipSuccess; ++l) e = hipStreamWaitEvent(ln.s[l - 1], ln.fork, 0);
    if (e != hipSuccess) return e;
    // every lane that was forked is joined again, whatever happens in between
    hipError_t first = hipSuccess;
    for (int l = 0; l < lanes; ++l) {
        hipStream_t st = l == 0 ? user : ln.s[l - 1];
        for (size_t bi = 0; bi < lane_of.size() && first == hipSuccess; ++bi)
            if (lane_of[bi] == l) first = body(bi, st, l);
        if (l > 0) {
            hipError_t j = hipEventRecord(ln.join[l - 1], st);
            if (j == hipSuccess) j = hipStreamWaitEvent(user, ln.join[l - 1], 0);
            if (first == hipSuccess) first = j;
        }
    }
    return first;
}

extern "C" {

// a lane's workspace: the usual layout, moved to the lane's region
static Workspace region_workspace(size_t count, uint32_t L, size_t region_offset)
{
    Workspace w = make_workspace(count, L);
    w.status += region_offset;
    w.hist += region_offset;
    w.sel += region_offset;
    w.tinfo += region_offset;
    w.tscan += region_offset;
    w.cand += region_offset;
    w.prefix += region_offset;
    w.spec += region_offset;
    w.mid += region_offset;
    return w;
}

static CodecArgs segment_args(const SegBatch& b, const size_t* seg_offsets, int nseg, float theta, int bits, int m)
{
    CodecArgs a{};
    a.C = b.count;
    a.L = b.L;
    a.k = kept(b.L, theta);
    a.bits = bits;
    a.m = m;
    a.S = record_stride(b.L, a.k, bits);
    a.word3 = b.L;
    a.sstride = padded_bins(b.L);
    a.tab = &b.tab;
    a.hdr_n = seg_offsets[nseg] - seg_offsets[0];
    a.hdr_L = 0;
    a.hdr_C = (uint32_t)nseg;
    a.hdr_k = 0;
    a.hdr_S = 0;
    a.hdr_theta = theta;
    return a;
}

int fftsp_compress_segments(const float* d_grad, const size_t* seg_offsets, int nseg, float theta, int bits,
                            void* d_packed, size_t packed_capacity, void* d_workspace, size_t workspace_bytes,
                            fftsp_stream_t stream)
{
    int rc = segments_ok(seg_offsets, nseg);
    if (rc) return rc;
    const int m = mantissa(bits);
    if (!theta_ok(theta) || m < 0) return FFTSP_EINVAL;
    if (!d_grad || !d_packed || !d_workspace || !aligned16(d_grad) || !aligned16(d_packed) || !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_capacity < fftsp_packed_bytes_segments(seg_offsets, nseg, theta, bits)) return FFTSP_ENOSPC;
    if (workspace_bytes < fftsp_workspace_bytes_segments(seg_offsets, nseg, bits)) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    uint8_t* out = static_cast<uint8_t*>(d_packed);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const std::vector<SegBatch> batches = plan_segments(seg_offsets, nseg, theta, bits, true);
    const size_t region = segment_region_bytes(batches);
    const int lanes = prof::enabled() ? 1 : segment_lanes(batches.size());  // per-kernel timing wants one chain
    const std::vector<int> lane_of = assign_lanes(batches, lanes);
    const hipError_t e = run_on_lanes(s, lane_of, lanes, [&](size_t bi, hipStream_t st, int lane) {
        const SegBatch& b = batches[bi];
        // every lane clears and uses the status words and histograms of its own region; nothing on the sender
        // raises a status, and the caller reads the first region's word
        const Workspace w = region_workspace(b.count, b.L, (size_t)lane * region);
        CodecArgs a = segment_args(b, seg_offsets, nseg, theta, bits, m);
        a.write_header = (bi == 0);
        float* spec = reinterpret_cast<float*>(ws + w.spec);
        int hist_done = 0;
        hipError_t pe = launch_rfft(d_grad, 0, log2_exact(b.L), b.count, spec, a.sstride,
                                    reinterpret_cast<float2*>(ws + w.mid), t, reinterpret_cast<uint32_t*>(ws + w.hist),
                                    reinterpret_cast<uint32_t*>(ws + w.status),
                                    (w.hist - w.status) / 4 + b.count * (size_t)kHistBins, &hist_done, 1, &a.pair_log,
                                    &b.tab, st);
        if (pe == hipSuccess) pe = launch_encode(spec, a, out, out + kStreamHeader, ws, w, hist_done, st);
        return pe;
    });
    return hip_status(e);
}

int fftsp_decompress_segments(const void* d_packed, size_t packed_bytes, float* d_grad_out, const size_t* seg_offsets,
                              int nseg, float theta, int bits, void* d_workspace, size_t workspace_bytes,
                              fftsp_stream_t stream)
{
    int rc = segments_ok(seg_offsets, nseg);
    if (rc) return rc;
    const int m = mantissa(bits);
    if (!theta_ok(theta) || m < 0) return FFTSP_EINVAL;
    if (!d_grad_out || !d_packed || !d_workspace || !aligned16(d_grad_out) || !aligned16(d_packed) ||
        !aligned16(d_workspace))
        return FFTSP_EINVAL;
    if (packed_bytes < fftsp_packed_bytes_segments(seg_offsets, nseg, theta, bits)) return FFTSP_EFORMAT;
    if (workspace_bytes < fftsp_workspace_bytes_segments(seg_offsets, nseg, bits)) return FFTSP_EWORKSPACE;
    Tables t;
    if (get_tables(&t) != hipSuccess) return FFTSP_EHIP;
    uint8_t* ws = static_cast<uint8_t*>(d_workspace);
    const uint8_t* in = static_cast<const uint8_t*>(d_packed);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const std::vector<SegBatch> batches = plan_segments(seg_offsets, nseg, theta, bits, true);
    const size_t region = segment_region_bytes(batches);
    const int lanes = prof::enabled() ? 1 : segment_lanes(batches.size());
    const std::vector<int> lane_of = assign_lanes(batches, lanes);
    // every launch set raises the one status word at the start of the workspace, from whatever lane it runs on:
    // it is cleared here, before the lanes fork
    hipError_t e = launch_clear_status(ws, make_workspace(1, 32), s);
    if (e == hipSuccess)
        e = run_on_lanes(s, lane_of, lanes, [&](size_t bi, hipStream_t st, int lane) {
            const SegBatch& b = batches[bi];
            Workspace w = region_workspace(b.count, b.L, (size_t)lane * region);
            w.status = 0;
            CodecArgs a = segment_args(b, seg_offsets, nseg, theta, bits, m);
            a.pair_log = fft_pair_log(log2_exact(b.L));
            float* spec = reinterpret_cast<float*>(ws + w.spec);
            hipError_t pe = launch_decode(in, in + kStreamHeader, a, spec, ws, w, bi == 0, 0, st);
            if (pe == hipSuccess)
                pe = launch_irfft(spec, a.sstride, 0, log2_exact(b.L), b.count, d_grad_out,
                                  reinterpret_cast<float2*>(ws + w.mid), t, a.pair_log != 0, 1.0f, &b.tab, st);
            return pe;
        });
    return hip_status(e);
}

int fftsp_device_status(const void* d_workspace, int* status_out)
{
    if (!d_workspace || !status_out) return FFTSP_EINVAL;
    if (hipDeviceSynchronize() != hipSuccess) return FFTSP_EHIP;
    uint32_t v = 0;
    if (hipMemcpy(&v, d_workspace, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return FFTSP_EHIP;
    *status_out = (int)v;
    return FFTSP_OK;
}

int fftsp_profile_enable(int on)
{
    prof::enable(on != 0);
    return FFTSP_OK;
}

size_t fftsp_profile_report(char* buf, size_t cap)
{
    const std::string r = prof::report();
    if (buf && cap > 0) {
        const size_t ncopy = r.size() < cap - 1 ? r.size() : cap - 1;
        std::memcpy(buf, r.data(), ncopy);
        buf[ncopy] = 0;
    }
    return r.size() + 1;
}

const char* fftsp_strerror(int status)
{
    switch (status) {
        case FFTSP_OK: return "ok";
        case FFTSP_EINVAL: return "invalid argument";
        case FFTSP_ENOSPC: return "packed buffer too small";
        case FFTSP_EWORKSPACE: return "workspace too small";
        case FFTSP_EUNSUPPORTED: return "unsupported chunk length";
        case FFTSP_EHIP: return "HIP runtime error";
        case FFTSP_EFORMAT: return "packed stream does not match the arguments";
        default: return "unknown status";
    }
}

const char* fftsp_version(void) { return "fftsp 0.1 (gfx950)"; }

}  // extern "C"

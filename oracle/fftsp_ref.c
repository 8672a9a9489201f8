/*
 * fftsp_ref.c -- CPU oracle for the FFT-sparsifying gradient codec.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the codec computes.  It exists so that the GPU library can
 * be checked against it; nothing on the product path may call it.  It shares no
 * source, table or helper with the HIP implementation.
 *
 * What it follows (arXiv 1811.08596):
 *   - Sec. 3.1, "compression framework": linearize -> FFT -> keep the largest
 *     frequency components by magnitude -> range-based N-bit float -> pack;
 *     the receiver applies the inverse steps in reverse order.
 *   - Sec. 3.1.1: the DFT sum X_k = sum_n x_n exp(-2 pi i k n / N) and the
 *     "drop the low-energy components by resetting them to zero" rule.
 *   - Sec. 3.2: status vector / prefix-sum location vector / dense vector.
 *   - Sec. 3.2.1 and Algorithm 1: the offset-based N-bit float
 *     (shift the IEEE-754 pattern right by 23-m, subtract pbase, add one;
 *     inverse: add pbase, subtract one, shift left).
 *
 * Readings taken where the paper is silent (all are this build's choices and
 * are therefore "parity unpinned" by the paper itself; the tests pin them to
 * their own stated properties):
 *   - theta in this interface is the KEPT fraction (paper's theta = 1 - kept).
 *   - the unit of selection is one complex bin of the half spectrum
 *     (j = 0..L/2), ranked by fl(re*re + fl(im*im)) evaluated with one fused
 *     multiply-add in binary32, compared as an unsigned bit pattern; ties go to
 *     the lowest bin index.
 *   - sign-magnitude code space: top bit sign, low N-1 bits magnitude code c,
 *     c = 0 is exactly zero, c = 1 is eps (pbase), c = 2^(N-1)-1 holds the
 *     top of the range; eps is the closed form that the paper's iterative
 *     tuning converges to (fftsp_ref_tune_eps implements the iteration and the
 *     tests check that both give the same pbase).  The range is the largest
 *     surviving component of the chunk by default, or the caller's static max
 *     (the *_q entry points), above which values clamp as in Algorithm 1.
 *   - default mantissa width m as a function of N (see fftsp_ref_mantissa_bits).
 *   - the byte layout of the packed stream (see the comment above encode_chunk).
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_EINVAL 1
#define REF_ENOSPC 2
#define REF_EFORMAT 6

typedef struct {
    double re, im;
} cplx;

static int is_pow2(uint64_t v) { return v && !(v & (v - 1)); }

static uint32_t f2u(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}
static float u2f(uint32_t u)
{
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* ------------------------------------------------------------------------ */
/* FFT: textbook recursive radix-2 decimation in time, in double.            */
/* W[j] = exp(sign * 2 pi i j / Lfull), j < Lfull/2, from cos/sin in double.  */
/* ------------------------------------------------------------------------ */
static void make_twiddles(cplx* W, size_t Lfull, int sign)
{
    const double two_pi = 6.283185307179586476925286766559;
    for (size_t j = 0; j < Lfull / 2; ++j) {
        double a = two_pi * (double)j / (double)Lfull;
        W[j].re = cos(a);
        W[j].im = sign * sin(a);
    }
}

/* out[0..len) = DFT of in[0], in[stride], in[2 stride], ...  (len a power of 2) */
static void fft_rec(const cplx* in, size_t stride, cplx* out, size_t len, const cplx* W, size_t wstep)
{
    if (len == 1) {
        out[0] = in[0];
        return;
    }
    size_t half = len / 2;
    fft_rec(in, stride * 2, out, half, W, wstep * 2);                 /* even samples */
    fft_rec(in + stride, stride * 2, out + half, half, W, wstep * 2); /* odd samples  */
    for (size_t j = 0; j < half; ++j) {
        cplx e = out[j], o = out[j + half], w = W[j * wstep];
        cplx t = {o.re * w.re - o.im * w.im, o.re * w.im + o.im * w.re};
        out[j].re = e.re + t.re;
        out[j].im = e.im + t.im;
        out[j + half].re = e.re - t.re;
        out[j + half].im = e.im - t.im;
    }
}

/* Forward real DFT of one chunk (Sec. 3.1.1 sum, sign -, no normalisation):
 * x has `valid` real samples, zeros up to L; spec receives bins 0..L/2 as
 * (re,im) float pairs, each component rounded once from double. */
static float round_half(double v);

/* to_half != 0: every component is scaled by 2^scale_log2 and rounded ONCE from double to binary16 (returned as the
 * binary32 number of the same value) instead of to binary32 */
static int rfft_chunk_ex(const float* x, size_t valid, uint32_t L, float* spec, int to_half, int scale_log2)
{
    cplx* in = (cplx*)malloc(sizeof(cplx) * L);
    cplx* out = (cplx*)malloc(sizeof(cplx) * L);
    cplx* W = (cplx*)malloc(sizeof(cplx) * (L / 2 + 1));
    if (!in || !out || !W) {
        free(in); free(out); free(W);
        return REF_ENOSPC;
    }
    for (size_t t = 0; t < L; ++t) {
        in[t].re = t < valid ? (double)x[t] : 0.0;
        in[t].im = 0.0;
    }
    make_twiddles(W, L, -1);
    fft_rec(in, 1, out, L, W, 1);
    size_t half = L / 2;
    for (size_t j = 0; j <= half; ++j) {
        if (to_half) {
            spec[2 * j] = round_half(ldexp(out[j].re, scale_log2));
            spec[2 * j + 1] = round_half(ldexp(out[j].im, scale_log2));
        } else {
            spec[2 * j] = (float)out[j].re;
            spec[2 * j + 1] = (float)out[j].im;
        }
    }
    /* a real signal has real DC and Nyquist bins: store +0 exactly */
    spec[1] = 0.0f;
    spec[2 * half + 1] = 0.0f;
    free(in); free(out); free(W);
    return REF_OK;
}

static int rfft_chunk(const float* x, size_t valid, uint32_t L, float* spec)
{
    return rfft_chunk_ex(x, valid, L, spec, 0, 0);
}

/* Inverse: x[t] = (1/L) sum_{j<L} Xfull[j] exp(+2 pi i j t / L), Xfull the
 * Hermitian extension of bins 0..L/2 (imaginary parts of bins 0 and L/2 are
 * ignored).  Only the first `valid` samples are written. */
static int irfft_chunk_ex(const float* spec, size_t valid, uint32_t L, float* x, int scale_log2)
{
    cplx* in = (cplx*)malloc(sizeof(cplx) * L);
    cplx* out = (cplx*)malloc(sizeof(cplx) * L);
    cplx* W = (cplx*)malloc(sizeof(cplx) * (L / 2 + 1));
    if (!in || !out || !W) {
        free(in); free(out); free(W);
        return REF_ENOSPC;
    }
    size_t half = L / 2;
    for (size_t j = 0; j <= half; ++j) {
        in[j].re = (double)spec[2 * j];
        in[j].im = (double)spec[2 * j + 1];
    }
    in[0].im = 0.0;
    in[half].im = 0.0;
    for (size_t j = 1; j < half; ++j) {
        in[L - j].re = in[j].re;
        in[L - j].im = -in[j].im;
    }
    make_twiddles(W, L, +1);
    fft_rec(in, 1, out, L, W, 1);
    for (size_t t = 0; t < valid; ++t) x[t] = (float)ldexp(out[t].re / (double)L, -scale_log2);
    free(in); free(out); free(W);
    return REF_OK;
}

static int irfft_chunk(const float* spec, size_t valid, uint32_t L, float* x)
{
    return irfft_chunk_ex(spec, valid, L, x, 0);
}

static size_t chunk_count(size_t n, uint32_t L) { return (n + L - 1) / L; }
static size_t chunk_valid(size_t n, uint32_t L, size_t c)
{
    size_t start = c * (size_t)L;
    return n - start < L ? n - start : L;
}

/* spec: C * (L+2) floats, chunk c at offset c*(L+2) */
int fftsp_ref_rfft(const float* g, size_t n, uint32_t L, float* spec, int nthreads)
{
    if (!g || !spec || n == 0 || L < 2 || !is_pow2(L)) return REF_EINVAL;
    long C = (long)chunk_count(n, L);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = rfft_chunk(g + (size_t)c * L, chunk_valid(n, L, (size_t)c), L, spec + (size_t)c * (L + 2));
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

int fftsp_ref_irfft(const float* spec, size_t n, uint32_t L, float* out, int nthreads)
{
    if (!out || !spec || n == 0 || L < 2 || !is_pow2(L)) return REF_EINVAL;
    long C = (long)chunk_count(n, L);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = irfft_chunk(spec + (size_t)c * (L + 2), chunk_valid(n, L, (size_t)c), L, out + (size_t)c * L);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

/* ------------------------------------------------------------------------ */
/* Selection (Sec. 3.1.1: keep the top fraction "in magnitude", zero the rest) */
/* ------------------------------------------------------------------------ */

/* squared modulus in binary32: im*im rounded, then ONE fused multiply-add */
uint32_t fftsp_ref_key(float re, float im)
{
    volatile float p = im * im;
    float s = fmaf(re, re, p);
    return f2u(s);
}

/* kept bins per chunk: round-half-up of theta*B in double, clamped to [0,B] */
int fftsp_ref_kept_per_chunk(uint32_t L, float theta, uint32_t* k_out)
{
    if (!k_out || L < 2 || !is_pow2(L) || !(theta >= 0.0f && theta <= 1.0f)) return REF_EINVAL;
    double B = (double)(L / 2 + 1);
    double k = floor((double)theta * B + 0.5);
    if (k < 0) k = 0;
    if (k > B) k = B;
    *k_out = (uint32_t)k;
    return REF_OK;
}

typedef struct {
    uint32_t key, idx;
} keyidx;

static int cmp_keyidx(const void* a, const void* b)
{
    const keyidx* x = (const keyidx*)a;
    const keyidx* y = (const keyidx*)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1; /* larger key first  */
    if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1; /* then lower index */
    return 0;
}

/* flags[j] = 1 for the k bins that come first when sorted by
 * (key descending, index ascending); exactly k flags are set. */
int fftsp_ref_select(const uint32_t* keys, uint32_t B, uint32_t k, uint8_t* flags)
{
    if (!keys || !flags || k > B) return REF_EINVAL;
    keyidx* a = (keyidx*)malloc(sizeof(keyidx) * (B ? B : 1));
    if (!a) return REF_ENOSPC;
    for (uint32_t j = 0; j < B; ++j) {
        a[j].key = keys[j];
        a[j].idx = j;
        flags[j] = 0;
    }
    qsort(a, B, sizeof(keyidx), cmp_keyidx);
    for (uint32_t i = 0; i < k; ++i) flags[a[i].idx] = 1;
    free(a);
    return REF_OK;
}

/* ------------------------------------------------------------------------ */
/* Range-based N-bit float (Sec. 3.2.1, Algorithm 1)                          */
/* ------------------------------------------------------------------------ */

/* default mantissa width: leave e "exponent-like" bits of span,
 * e = 3 (N<=6), 4 (7<=N<=12), 5 (N>=13); m = max(1, N-1-e); N=32 is raw fp32 */
int fftsp_ref_mantissa_bits(int bits)
{
    if (bits == 32) return 23;
    if (bits < 3 || bits > 16) return -1;
    int e = bits <= 6 ? 3 : (bits <= 12 ? 4 : 5);
    int m = bits - 1 - e;
    return m < 1 ? 1 : m;
}

/* pbase = (eps pattern) >> (23-m), Algorithm 1's init line, with eps chosen so
 * that the largest surviving component lands on the top magnitude code */
uint32_t fftsp_ref_pbase(uint32_t vmax_bits, int bits, int m)
{
    if (bits == 32) return 0;
    uint32_t s = 23u - (uint32_t)m;
    int64_t Mmax = ((int64_t)1 << (bits - 1)) - 1;
    int64_t pb = (int64_t)((vmax_bits & 0x7FFFFFFFu) >> s) - (Mmax - 1);
    return pb < 1 ? 1u : (uint32_t)pb;
}

/* 32bit_to_Nbit of Algorithm 1 on one binary32 pattern */
uint32_t fftsp_ref_quantize(uint32_t fbits, uint32_t pbase, int bits, int m)
{
    if (bits == 32) return fbits;
    uint32_t s = 23u - (uint32_t)m;
    uint32_t Mmax = (1u << (bits - 1)) - 1u;
    uint32_t a = fbits & 0x7FFFFFFFu;
    uint32_t q = a >> s;              /* 32bit_binary = pattern >> (23-m)     */
    uint32_t c;
    if (q < pbase) {
        c = 0;                        /* below eps: flushed to zero           */
    } else {
        c = q - pbase + 1u;           /* Nbit_binary = 32bit_binary - pbase + 1 */
        if (c > Mmax) c = Mmax;       /* "if value > max then value = max"     */
    }
    uint32_t sign = c ? (fbits >> 31) : 0u;
    return (sign << (bits - 1)) | c;
}

/* Nbit_to_32bit of Algorithm 1 */
uint32_t fftsp_ref_dequantize(uint32_t code, uint32_t pbase, int bits, int m)
{
    if (bits == 32) return code;
    uint32_t s = 23u - (uint32_t)m;
    uint32_t Mmax = (1u << (bits - 1)) - 1u;
    uint32_t c = code & Mmax;
    uint32_t sign = (code >> (bits - 1)) & 1u;
    if (c == 0) return 0u;
    return ((c - 1u + pbase) << s) | (sign << 31);
}

/* ------------------------------------------------------------------------ */
/* Packing (Sec. 3.2): status -> prefix sum -> dense                          */
/* ------------------------------------------------------------------------ */

/* location[i] = number of set status entries at positions < i (0-based,
 * exclusive; the paper prints the 1-based inclusive scan of the same thing) */
static uint32_t prefix_locations(const uint8_t* status, size_t len, uint32_t* location)
{
    uint32_t run = 0;
    for (size_t i = 0; i < len; ++i) {
        location[i] = run;
        run += status[i] ? 1u : 0u;
    }
    return run;
}

/* the paper's three packing steps on a plain float vector; returns the dense length.
 * location_incl receives the INCLUSIVE scan, which is what the paper's example lists. */
size_t fftsp_ref_pack_dense(const float* sparse, size_t len, uint8_t* status, uint32_t* location_incl, float* dense)
{
    uint32_t* loc = (uint32_t*)malloc(sizeof(uint32_t) * (len ? len : 1));
    if (!loc) return 0;
    for (size_t i = 0; i < len; ++i) status[i] = sparse[i] != 0.0f;
    size_t cnt = prefix_locations(status, len, loc);
    for (size_t i = 0; i < len; ++i) {
        if (status[i]) dense[loc[i]] = sparse[i];
        location_incl[i] = loc[i] + (status[i] ? 1u : 0u);
    }
    free(loc);
    return cnt;
}

static size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }

/* record stride: 16-byte record header + bitmap words + code words, 16-aligned */
size_t fftsp_ref_record_stride(uint32_t L, uint32_t k, int bits)
{
    size_t B = (size_t)L / 2 + 1;
    size_t W = (B + 31) / 32;
    size_t code_words = ((size_t)2 * k * (size_t)bits + 31) / 32;
    return align16(16 + 4 * W + 4 * code_words);
}

#define STREAM_HEADER_BYTES 64

size_t fftsp_ref_packed_bytes(size_t n, uint32_t L, float theta, int bits)
{
    uint32_t k;
    if (n == 0 || fftsp_ref_mantissa_bits(bits) < 0) return 0;
    if (fftsp_ref_kept_per_chunk(L, theta, &k)) return 0;
    return STREAM_HEADER_BYTES + chunk_count(n, L) * fftsp_ref_record_stride(L, k, bits);
}

static void put_u32(uint8_t* p, uint32_t v)
{
    p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24);
}
static uint32_t get_u32(const uint8_t* p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static void put_u64(uint8_t* p, uint64_t v)
{
    put_u32(p, (uint32_t)v);
    put_u32(p + 4, (uint32_t)(v >> 32));
}
static uint64_t get_u64(const uint8_t* p) { return (uint64_t)get_u32(p) | ((uint64_t)get_u32(p + 4) << 32); }

/* Stream header, 64 bytes, little-endian:
 *  0 "FSP1" | 4 u32 version=1 | 8 u64 n | 16 u32 L (0 = per-segment lengths) |
 *  20 u32 C | 24 u32 N | 28 u32 m | 32 u32 k (0 if segmented) |
 *  36 u32 S (0 if segmented) | 40 f32 theta (kept) | 44..63 zero            */
static void write_stream_header(uint8_t* p, uint64_t n, uint32_t L, uint32_t C, int bits, int m, uint32_t k,
                                uint32_t S, float theta)
{
    memset(p, 0, STREAM_HEADER_BYTES);
    p[0] = 'F'; p[1] = 'S'; p[2] = 'P'; p[3] = '1';
    put_u32(p + 4, 1);
    put_u64(p + 8, n);
    put_u32(p + 16, L);
    put_u32(p + 20, C);
    put_u32(p + 24, (uint32_t)bits);
    put_u32(p + 28, (uint32_t)m);
    put_u32(p + 32, k);
    put_u32(p + 36, S);
    put_u32(p + 40, f2u(theta));
}

/* set `nbits` bits of `code` at bit position `pos` of an LSB-first bit stream */
static void put_bits(uint8_t* stream, uint64_t pos, uint32_t code, int nbits)
{
    for (int b = 0; b < nbits; ++b)
        if ((code >> b) & 1u) stream[(pos + (uint64_t)b) >> 3] |= (uint8_t)(1u << ((pos + (uint64_t)b) & 7));
}
static uint32_t get_bits(const uint8_t* stream, uint64_t pos, int nbits)
{
    uint32_t v = 0;
    for (int b = 0; b < nbits; ++b)
        if ((stream[(pos + (uint64_t)b) >> 3] >> ((pos + (uint64_t)b) & 7)) & 1u) v |= 1u << b;
    return v;
}

/* One record (all little-endian, padding zero):
 *  +0 u32 pbase | +4 u32 vmax_bits | +8 u32 k | +12 u32 L if segmented else 0
 *  +16 bitmap, W = ceil(B/32) words, bit j%32 of word j/32 = bin j kept
 *  +16+4W codes: code i in bits [iN, iN+N) of an LSB-first stream, order
 *          re0, im0, re1, im1, ... by ascending kept bin
 * `rec` must have `stride` bytes. */
static int encode_chunk(const float* spec, uint32_t L, uint32_t k, int bits, int m, uint32_t word3, uint8_t* rec,
                        size_t stride, uint32_t fixed_vmax)
{
    uint32_t B = L / 2 + 1;
    size_t W = ((size_t)B + 31) / 32;
    uint32_t* keys = (uint32_t*)malloc(sizeof(uint32_t) * B);
    uint8_t* status = (uint8_t*)malloc(B);
    uint32_t* location = (uint32_t*)malloc(sizeof(uint32_t) * B);
    if (!keys || !status || !location) {
        free(keys); free(status); free(location);
        return REF_ENOSPC;
    }
    for (uint32_t j = 0; j < B; ++j) keys[j] = fftsp_ref_key(spec[2 * j], spec[2 * j + 1]);
    int e = fftsp_ref_select(keys, B, k, status);
    if (e) {
        free(keys); free(status); free(location);
        return e;
    }
    prefix_locations(status, B, location);

    /* range of the survivors: largest |component| as a bit pattern */
    uint32_t vmax = 0;
    for (uint32_t j = 0; j < B; ++j) {
        if (!status[j]) continue;
        uint32_t a = f2u(spec[2 * j]) & 0x7FFFFFFFu, b = f2u(spec[2 * j + 1]) & 0x7FFFFFFFu;
        if (a > vmax) vmax = a;
        if (b > vmax) vmax = b;
    }
    /* static range (Sec. 3.2.1: max estimated beforehand): the range no longer follows the survivors; whatever
       exceeds it is clamped to the top code by 32bit_to_Nbit */
    if (fixed_vmax) vmax = fixed_vmax;
    uint32_t pbase = fftsp_ref_pbase(vmax, bits, m);

    memset(rec, 0, stride);
    put_u32(rec + 0, pbase);
    put_u32(rec + 4, vmax);
    put_u32(rec + 8, k);
    put_u32(rec + 12, word3);
    uint8_t* bitmap = rec + 16;
    uint8_t* codes = rec + 16 + 4 * W;
    for (uint32_t j = 0; j < B; ++j) {
        if (!status[j]) continue;
        bitmap[j >> 3] |= (uint8_t)(1u << (j & 7));
        uint64_t slot = (uint64_t)location[j] * 2u;
        put_bits(codes, slot * (uint64_t)bits, fftsp_ref_quantize(f2u(spec[2 * j]), pbase, bits, m), bits);
        put_bits(codes, (slot + 1) * (uint64_t)bits, fftsp_ref_quantize(f2u(spec[2 * j + 1]), pbase, bits, m), bits);
    }
    free(keys); free(status); free(location);
    return REF_OK;
}

/* inverse of encode_chunk: zero spectrum, scatter dequantised survivors */
static int decode_chunk(const uint8_t* rec, uint32_t L, uint32_t k, int bits, int m, float* spec)
{
    uint32_t B = L / 2 + 1;
    size_t W = ((size_t)B + 31) / 32;
    uint32_t pbase = get_u32(rec + 0);
    if (get_u32(rec + 8) != k) return REF_EFORMAT;
    const uint8_t* bitmap = rec + 16;
    const uint8_t* codes = rec + 16 + 4 * W;
    uint32_t rank = 0;
    for (uint32_t j = 0; j < B; ++j) {
        spec[2 * j] = 0.0f;
        spec[2 * j + 1] = 0.0f;
        if (!((bitmap[j >> 3] >> (j & 7)) & 1u)) continue;
        if (rank >= k) return REF_EFORMAT;
        uint64_t slot = (uint64_t)rank * 2u;
        spec[2 * j] = u2f(fftsp_ref_dequantize(get_bits(codes, slot * (uint64_t)bits, bits), pbase, bits, m));
        spec[2 * j + 1] = u2f(fftsp_ref_dequantize(get_bits(codes, (slot + 1) * (uint64_t)bits, bits), pbase, bits, m));
        ++rank;
    }
    return rank == k ? REF_OK : REF_EFORMAT;
}

/* Quantizer options of Sec. 3.2.1 that the plain entry points fix: m (0 = the default for the width) and a static
 * range [-range_max, +range_max] (0 = fitted per chunk to the largest surviving component). */
static int quantizer_m(int bits, int m)
{
    if (m == 0 || bits == 32) return fftsp_ref_mantissa_bits(bits);
    if (bits < 3 || bits > 16 || m < 1 || m > bits - 1) return -1;
    return m;
}

int fftsp_ref_encode_spectrum_q(const float* spec, size_t n, uint32_t L, float theta, int bits, int m_opt,
                                float range_max, uint8_t* packed, size_t cap, int nthreads)
{
    uint32_t k;
    int m = quantizer_m(bits, m_opt);
    if (!spec || !packed || n == 0 || m < 0 || !(range_max >= 0.0f) || isinf(range_max)) return REF_EINVAL;
    if (fftsp_ref_kept_per_chunk(L, theta, &k)) return REF_EINVAL;
    size_t S = fftsp_ref_record_stride(L, k, bits);
    long C = (long)chunk_count(n, L);
    if (cap < STREAM_HEADER_BYTES + (size_t)C * S) return REF_ENOSPC;
    write_stream_header(packed, n, L, (uint32_t)C, bits, m, k, (uint32_t)S, theta);
    uint32_t fixed = range_max > 0.0f ? f2u(range_max) : 0u;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = encode_chunk(spec + (size_t)c * (L + 2), L, k, bits, m, 0, packed + STREAM_HEADER_BYTES + (size_t)c * S, S,
                             fixed);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

int fftsp_ref_encode_spectrum(const float* spec, size_t n, uint32_t L, float theta, int bits, uint8_t* packed,
                              size_t cap, int nthreads)
{
    return fftsp_ref_encode_spectrum_q(spec, n, L, theta, bits, 0, 0.0f, packed, cap, nthreads);
}

static int check_stream_header(const uint8_t* p, size_t bytes, uint64_t n, uint32_t L, uint32_t C, int bits, int m,
                               uint32_t k, uint32_t S)
{
    if (bytes < STREAM_HEADER_BYTES) return REF_EFORMAT;
    if (p[0] != 'F' || p[1] != 'S' || p[2] != 'P' || p[3] != '1') return REF_EFORMAT;
    if (get_u32(p + 4) != 1 || get_u64(p + 8) != n || get_u32(p + 16) != L || get_u32(p + 20) != C) return REF_EFORMAT;
    if (get_u32(p + 24) != (uint32_t)bits || get_u32(p + 28) != (uint32_t)m) return REF_EFORMAT;
    if (get_u32(p + 32) != k || get_u32(p + 36) != S) return REF_EFORMAT;
    return REF_OK;
}

/* frequency-domain decoder; the stream must carry the given spectrum scale (header word 12; 0 for every sender but
 * the half-precision one) */
static int decode_spectrum_scaled(const uint8_t* packed, size_t bytes, size_t n, uint32_t L, float theta, int bits,
                                  int m_opt, int scale_log2, float* spec, int nthreads);

int fftsp_ref_decode_spectrum_q(const uint8_t* packed, size_t bytes, size_t n, uint32_t L, float theta, int bits,
                                int m_opt, float* spec, int nthreads)
{
    return decode_spectrum_scaled(packed, bytes, n, L, theta, bits, m_opt, 0, spec, nthreads);
}

static int decode_spectrum_scaled(const uint8_t* packed, size_t bytes, size_t n, uint32_t L, float theta, int bits,
                                  int m_opt, int scale_log2, float* spec, int nthreads)
{
    uint32_t k;
    int m = quantizer_m(bits, m_opt);
    if (!spec || !packed || n == 0 || m < 0) return REF_EINVAL;
    if (fftsp_ref_kept_per_chunk(L, theta, &k)) return REF_EINVAL;
    size_t S = fftsp_ref_record_stride(L, k, bits);
    long C = (long)chunk_count(n, L);
    if (bytes < STREAM_HEADER_BYTES + (size_t)C * S) return REF_EFORMAT;
    int e0 = check_stream_header(packed, bytes, n, L, (uint32_t)C, bits, m, k, (uint32_t)S);
    if (e0) return e0;
    if (get_u32(packed + 44) != 0 || get_u32(packed + 48) != (uint32_t)scale_log2) return REF_EFORMAT;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = decode_chunk(packed + STREAM_HEADER_BYTES + (size_t)c * S, L, k, bits, m, spec + (size_t)c * (L + 2));
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

int fftsp_ref_decode_spectrum(const uint8_t* packed, size_t bytes, size_t n, uint32_t L, float theta, int bits,
                              float* spec, int nthreads)
{
    return fftsp_ref_decode_spectrum_q(packed, bytes, n, L, theta, bits, 0, spec, nthreads);
}

/* sender: chunk -> real FFT -> top-k -> quantize -> pack */
int fftsp_ref_compress_q(const float* g, size_t n, uint32_t L, float theta, int bits, int m_opt, float range_max,
                         uint8_t* packed, size_t cap, int nthreads)
{
    if (!g || !packed || n == 0 || L < 2 || !is_pow2(L)) return REF_EINVAL;
    size_t C = chunk_count(n, L);
    float* spec = (float*)malloc(sizeof(float) * C * ((size_t)L + 2));
    if (!spec) return REF_ENOSPC;
    int e = fftsp_ref_rfft(g, n, L, spec, nthreads);
    if (!e) e = fftsp_ref_encode_spectrum_q(spec, n, L, theta, bits, m_opt, range_max, packed, cap, nthreads);
    free(spec);
    return e;
}

int fftsp_ref_compress(const float* g, size_t n, uint32_t L, float theta, int bits, uint8_t* packed, size_t cap,
                       int nthreads)
{
    return fftsp_ref_compress_q(g, n, L, theta, bits, 0, 0.0f, packed, cap, nthreads);
}

/* receiver: unpack -> dequantize -> scatter -> inverse real FFT */
int fftsp_ref_decompress_q(const uint8_t* packed, size_t bytes, float* out, size_t n, uint32_t L, float theta, int bits,
                           int m_opt, int nthreads)
{
    if (!out || !packed || n == 0 || L < 2 || !is_pow2(L)) return REF_EINVAL;
    size_t C = chunk_count(n, L);
    float* spec = (float*)malloc(sizeof(float) * C * ((size_t)L + 2));
    if (!spec) return REF_ENOSPC;
    int e = fftsp_ref_decode_spectrum_q(packed, bytes, n, L, theta, bits, m_opt, spec, nthreads);
    if (!e) e = fftsp_ref_irfft(spec, n, L, out, nthreads);
    free(spec);
    return e;
}

int fftsp_ref_decompress(const uint8_t* packed, size_t bytes, float* out, size_t n, uint32_t L, float theta, int bits,
                         int nthreads)
{
    return fftsp_ref_decompress_q(packed, bytes, out, n, L, theta, bits, 0, nthreads);
}

/*
 * The paper's way to the smallest representable number eps for a static range [-max, +max] (Sec. 3.2.1, last
 * paragraph before Algorithm 1): start from some eps, convert the all-ones code (the most negative representable
 * number) back to binary32 with it, and move eps down if that number lies beyond the range, up otherwise, until
 * the positive and negative halves of the code space are both in use (P = 2^N / 2).  Done here as a bisection on
 * eps's bit pattern; returns eps (0 if the arguments are invalid).  The codec itself does not iterate: the
 * closed form in fftsp_ref_pbase must land on the same pbase, which is what the tests check.
 */
float fftsp_ref_tune_eps(float range_max, int bits, int m)
{
    if (bits < 3 || bits > 16 || m < 1 || m > bits - 1 || !(range_max > 0.0f) || isinf(range_max)) return 0.0f;
    const uint32_t all_ones = (1u << bits) - 1u;
    uint32_t lo = 1u << (23 - m), hi = f2u(range_max);     /* candidate eps patterns; pbase >= 1 */
    if (hi < lo) return u2f(lo);
    while (lo < hi) {
        uint32_t mid = lo + (hi - lo + 1) / 2;
        uint32_t pbase = mid >> (23 - m);                    /* init(): pbase = eps >> (23-m) */
        float actual_min = u2f(fftsp_ref_dequantize(all_ones, pbase, bits, m));
        /* the top code's pattern may run past the largest finite binary32: that is beyond any range */
        uint64_t top_pattern = ((uint64_t)pbase + (all_ones >> 1) - 1u) << (23 - m);
        if (top_pattern >= 0x7F800000u || actual_min < -range_max)
            hi = mid - 1;                                    /* reaches beyond the range: decrease eps */
        else
            lo = mid;                                        /* still inside: eps may grow */
    }
    return u2f(lo);
}

/* ------------------------------------------------------------------------ */
/* Per-tensor ("segmented") variant: segment i is g[off[i] .. off[i+1]) and   */
/* is transformed on its own with L_i = max(32, next power of two >= size).   */
/* ------------------------------------------------------------------------ */
uint32_t fftsp_ref_segment_length(size_t size)
{
    uint32_t L = 32;
    while ((size_t)L < size) L <<= 1;
    return L;
}

/*
 * Receiver under an allgather (Sec. 4, "Implementation": every worker collects all peers' packed buffers;
 * Sec. 3.1, last paragraph: the receiver applies the inverse steps).  The inverse transform is linear, so
 * instead of reconstructing every peer's gradient and adding them, the peers' sparse spectra are added bin by bin
 * and ONE inverse transform is taken:   out = scale * iFFT( sum_p D(packed_p) ).
 *
 * Readings (the paper leaves the arithmetic open; parity unpinned by the paper): the sum starts from a zero
 * spectrum and adds the peers in list order in binary32 (one rounding per addition); `scale` (e.g. 1/p for an
 * average) is applied to the binary32 result of the inverse transform with one binary32 multiplication.
 * All peers must carry the same (n, L, theta, bits).
 */
int fftsp_ref_decode_accumulate_spectrum(const uint8_t* const* packed, int npeers, size_t bytes, size_t n, uint32_t L,
                                         float theta, int bits, float* spec, int nthreads)
{
    if (!packed || npeers <= 0 || !spec || n == 0 || L < 2 || !is_pow2(L)) return REF_EINVAL;
    size_t C = chunk_count(n, L), len = C * ((size_t)L + 2);
    float* one = (float*)malloc(sizeof(float) * len);
    if (!one) return REF_ENOSPC;
    for (size_t i = 0; i < len; ++i) spec[i] = 0.0f;
    int e = 0;
    for (int p = 0; p < npeers && !e; ++p) {
        if (!packed[p]) {
            e = REF_EINVAL;
            break;
        }
        e = fftsp_ref_decode_spectrum(packed[p], bytes, n, L, theta, bits, one, nthreads);
        if (e) break;
        for (size_t i = 0; i < len; ++i) spec[i] = spec[i] + one[i];
    }
    free(one);
    return e;
}

int fftsp_ref_decompress_accumulate(const uint8_t* const* packed, int npeers, size_t bytes, float scale, float* out,
                                    size_t n, uint32_t L, float theta, int bits, int nthreads)
{
    if (!out || n == 0 || L < 2 || !is_pow2(L)) return REF_EINVAL;
    size_t C = chunk_count(n, L);
    float* spec = (float*)malloc(sizeof(float) * C * ((size_t)L + 2));
    if (!spec) return REF_ENOSPC;
    int e = fftsp_ref_decode_accumulate_spectrum(packed, npeers, bytes, n, L, theta, bits, spec, nthreads);
    if (!e) e = fftsp_ref_irfft(spec, n, L, out, nthreads);
    if (!e)
        for (size_t i = 0; i < n; ++i) out[i] = out[i] * scale;
    free(spec);
    return e;
}

size_t fftsp_ref_packed_bytes_segments(const size_t* off, int nseg, float theta, int bits)
{
    if (!off || nseg <= 0 || fftsp_ref_mantissa_bits(bits) < 0) return 0;
    size_t total = STREAM_HEADER_BYTES;
    for (int i = 0; i < nseg; ++i) {
        if (off[i + 1] <= off[i]) return 0;
        uint32_t L = fftsp_ref_segment_length(off[i + 1] - off[i]), k;
        if (fftsp_ref_kept_per_chunk(L, theta, &k)) return 0;
        total += fftsp_ref_record_stride(L, k, bits);
    }
    return total;
}

int fftsp_ref_compress_segments(const float* g, const size_t* off, int nseg, float theta, int bits, uint8_t* packed,
                                size_t cap, int nthreads)
{
    int m = fftsp_ref_mantissa_bits(bits);
    if (!g || !off || !packed || nseg <= 0 || m < 0) return REF_EINVAL;
    size_t need = fftsp_ref_packed_bytes_segments(off, nseg, theta, bits);
    if (need == 0) return REF_EINVAL;
    if (cap < need) return REF_ENOSPC;
    size_t* rec_off = (size_t*)malloc(sizeof(size_t) * (size_t)(nseg + 1));
    if (!rec_off) return REF_ENOSPC;
    rec_off[0] = STREAM_HEADER_BYTES;
    for (int i = 0; i < nseg; ++i) {
        uint32_t L = fftsp_ref_segment_length(off[i + 1] - off[i]), k;
        fftsp_ref_kept_per_chunk(L, theta, &k);
        rec_off[i + 1] = rec_off[i] + fftsp_ref_record_stride(L, k, bits);
    }
    write_stream_header(packed, off[nseg] - off[0], 0, (uint32_t)nseg, bits, m, 0, 0, theta);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (int i = 0; i < nseg; ++i) {
        size_t size = off[i + 1] - off[i];
        uint32_t L = fftsp_ref_segment_length(size), k;
        fftsp_ref_kept_per_chunk(L, theta, &k);
        float* spec = (float*)malloc(sizeof(float) * ((size_t)L + 2));
        int e = spec ? rfft_chunk(g + off[i], size, L, spec) : REF_ENOSPC;
        if (!e) e = encode_chunk(spec, L, k, bits, m, L, packed + rec_off[i], rec_off[i + 1] - rec_off[i], 0u);
        free(spec);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    free(rec_off);
    return err;
}

int fftsp_ref_decompress_segments(const uint8_t* packed, size_t bytes, float* out, const size_t* off, int nseg,
                                  float theta, int bits, int nthreads)
{
    int m = fftsp_ref_mantissa_bits(bits);
    if (!out || !off || !packed || nseg <= 0 || m < 0) return REF_EINVAL;
    size_t need = fftsp_ref_packed_bytes_segments(off, nseg, theta, bits);
    if (need == 0) return REF_EINVAL;
    if (bytes < need) return REF_EFORMAT;
    int e0 = check_stream_header(packed, bytes, off[nseg] - off[0], 0, (uint32_t)nseg, bits, m, 0, 0);
    if (e0) return e0;
    size_t* rec_off = (size_t*)malloc(sizeof(size_t) * (size_t)(nseg + 1));
    if (!rec_off) return REF_ENOSPC;
    rec_off[0] = STREAM_HEADER_BYTES;
    for (int i = 0; i < nseg; ++i) {
        uint32_t L = fftsp_ref_segment_length(off[i + 1] - off[i]), k;
        fftsp_ref_kept_per_chunk(L, theta, &k);
        rec_off[i + 1] = rec_off[i] + fftsp_ref_record_stride(L, k, bits);
    }
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (int i = 0; i < nseg; ++i) {
        size_t size = off[i + 1] - off[i];
        uint32_t L = fftsp_ref_segment_length(size), k;
        fftsp_ref_kept_per_chunk(L, theta, &k);
        float* spec = (float*)malloc(sizeof(float) * ((size_t)L + 2));
        int e = spec ? REF_OK : REF_ENOSPC;
        if (!e && get_u32(packed + rec_off[i] + 12) != L) e = REF_EFORMAT;
        if (!e) e = decode_chunk(packed + rec_off[i], L, k, bits, m, spec);
        if (!e) e = irfft_chunk(spec, size, L, out + off[i]);
        free(spec);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    free(rec_off);
    return err;
}

/* ------------------------------------------------------------------------ */
/* Time-domain Top-k: the sparsifier the paper measures its own against       */
/* (Sec. 4, "Choice of Algorithms"; the right panel of the Sec. 3.1.1 figure   */
/* that puts FFT Top-k beside direct Top-k).  The gradient samples themselves  */
/* are thresholded by magnitude; nothing is transformed.  Readings: the same   */
/* chunking, Algorithm 1 quantizer and bitmap/dense packing as the frequency   */
/* path, so that the two differ in the transform alone; N = 32 is the paper's  */
/* plain Top-k (values kept as binary32).                                      */
/*   - unit of selection: one sample; rank key = bit pattern of |x| (exact     */
/*     magnitude order); ties go to the lowest index; samples past the end of  */
/*     the gradient are zeros that take part like any other zero.              */
/*   - kept samples per chunk: round-half-up of theta * L (theta = KEPT        */
/*     fraction, as everywhere in this interface).                             */
/*   - record: +0 pbase | +4 vmax_bits | +8 k | +12 0 | bitmap ceil(L/32)     */
/*     words | ONE code per kept sample, ascending index; stream header as     */
/*     above with word 11 (offset 44) = 1 marking the time domain.             */
/* ------------------------------------------------------------------------ */
int fftsp_ref_topk_kept_per_chunk(uint32_t L, float theta, uint32_t* k_out)
{
    if (!k_out || L < 2 || !is_pow2(L) || !(theta >= 0.0f && theta <= 1.0f)) return REF_EINVAL;
    double k = floor((double)theta * (double)L + 0.5);
    if (k < 0) k = 0;
    if (k > (double)L) k = (double)L;
    *k_out = (uint32_t)k;
    return REF_OK;
}

size_t fftsp_ref_topk_record_stride(uint32_t L, uint32_t k, int bits)
{
    size_t W = ((size_t)L + 31) / 32;
    size_t code_words = ((size_t)k * (size_t)bits + 31) / 32;
    return align16(16 + 4 * W + 4 * code_words);
}

size_t fftsp_ref_topk_packed_bytes(size_t n, uint32_t L, float theta, int bits)
{
    uint32_t k;
    if (n == 0 || fftsp_ref_mantissa_bits(bits) < 0) return 0;
    if (fftsp_ref_topk_kept_per_chunk(L, theta, &k)) return 0;
    return STREAM_HEADER_BYTES + chunk_count(n, L) * fftsp_ref_topk_record_stride(L, k, bits);
}

static int topk_encode_chunk(const float* x, size_t valid, uint32_t L, uint32_t k, int bits, int m, uint8_t* rec,
                             size_t stride)
{
    size_t W = ((size_t)L + 31) / 32;
    uint32_t* pat = (uint32_t*)malloc(sizeof(uint32_t) * L);  /* sample bit patterns, zero past the end */
    uint32_t* keys = (uint32_t*)malloc(sizeof(uint32_t) * L);
    uint8_t* status = (uint8_t*)malloc(L);
    uint32_t* location = (uint32_t*)malloc(sizeof(uint32_t) * L);
    if (!pat || !keys || !status || !location) {
        free(pat); free(keys); free(status); free(location);
        return REF_ENOSPC;
    }
    for (uint32_t j = 0; j < L; ++j) {
        pat[j] = j < valid ? f2u(x[j]) : 0u;
        keys[j] = pat[j] & 0x7FFFFFFFu;
    }
    int e = fftsp_ref_select(keys, L, k, status);
    if (e) {
        free(pat); free(keys); free(status); free(location);
        return e;
    }
    prefix_locations(status, L, location);
    uint32_t vmax = 0;
    for (uint32_t j = 0; j < L; ++j)
        if (status[j] && keys[j] > vmax) vmax = keys[j];
    uint32_t pbase = fftsp_ref_pbase(vmax, bits, m);
    memset(rec, 0, stride);
    put_u32(rec + 0, pbase);
    put_u32(rec + 4, vmax);
    put_u32(rec + 8, k);
    uint8_t* bitmap = rec + 16;
    uint8_t* codes = rec + 16 + 4 * W;
    for (uint32_t j = 0; j < L; ++j) {
        if (!status[j]) continue;
        bitmap[j >> 3] |= (uint8_t)(1u << (j & 7));
        put_bits(codes, (uint64_t)location[j] * (uint64_t)bits, fftsp_ref_quantize(pat[j], pbase, bits, m), bits);
    }
    free(pat); free(keys); free(status); free(location);
    return REF_OK;
}

static int topk_decode_chunk(const uint8_t* rec, size_t valid, uint32_t L, uint32_t k, int bits, int m, float* x)
{
    size_t W = ((size_t)L + 31) / 32;
    uint32_t pbase = get_u32(rec + 0);
    if (get_u32(rec + 8) != k) return REF_EFORMAT;
    const uint8_t* bitmap = rec + 16;
    const uint8_t* codes = rec + 16 + 4 * W;
    uint32_t rank = 0;
    for (uint32_t j = 0; j < L; ++j) {
        float v = 0.0f;
        if ((bitmap[j >> 3] >> (j & 7)) & 1u) {
            if (rank >= k) return REF_EFORMAT;
            v = u2f(fftsp_ref_dequantize(get_bits(codes, (uint64_t)rank * (uint64_t)bits, bits), pbase, bits, m));
            ++rank;
        }
        if (j < valid) x[j] = v;
    }
    return rank == k ? REF_OK : REF_EFORMAT;
}

int fftsp_ref_topk_compress(const float* g, size_t n, uint32_t L, float theta, int bits, uint8_t* packed, size_t cap,
                            int nthreads)
{
    uint32_t k;
    int m = fftsp_ref_mantissa_bits(bits);
    if (!g || !packed || n == 0 || m < 0) return REF_EINVAL;
    if (fftsp_ref_topk_kept_per_chunk(L, theta, &k)) return REF_EINVAL;
    size_t S = fftsp_ref_topk_record_stride(L, k, bits);
    long C = (long)chunk_count(n, L);
    if (cap < STREAM_HEADER_BYTES + (size_t)C * S) return REF_ENOSPC;
    write_stream_header(packed, n, L, (uint32_t)C, bits, m, k, (uint32_t)S, theta);
    put_u32(packed + 44, 1);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = topk_encode_chunk(g + (size_t)c * L, chunk_valid(n, L, (size_t)c), L, k, bits, m,
                                  packed + STREAM_HEADER_BYTES + (size_t)c * S, S);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

int fftsp_ref_topk_decompress(const uint8_t* packed, size_t bytes, float* out, size_t n, uint32_t L, float theta,
                              int bits, int nthreads)
{
    uint32_t k;
    int m = fftsp_ref_mantissa_bits(bits);
    if (!out || !packed || n == 0 || m < 0) return REF_EINVAL;
    if (fftsp_ref_topk_kept_per_chunk(L, theta, &k)) return REF_EINVAL;
    size_t S = fftsp_ref_topk_record_stride(L, k, bits);
    long C = (long)chunk_count(n, L);
    if (bytes < STREAM_HEADER_BYTES + (size_t)C * S) return REF_EFORMAT;
    int e0 = check_stream_header(packed, bytes, n, L, (uint32_t)C, bits, m, k, (uint32_t)S);
    if (e0) return e0;
    if (get_u32(packed + 44) != 1) return REF_EFORMAT;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = topk_decode_chunk(packed + STREAM_HEADER_BYTES + (size_t)c * S, chunk_valid(n, L, (size_t)c), L, k, bits,
                                  m, out + (size_t)c * L);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

/* ------------------------------------------------------------------------ */
/* Half-precision variant (Sec. 3.1.1, "Our approach": the gradients go to 16  */
/* bits for the transform, whose loss is negligible because gradients are      */
/* bounded).  What the variant computes, as a definition: the exact DFT of the */
/* chunk, scaled by a caller-chosen power of two 2^s (so that small gradients  */
/* do not fall into binary16's subnormals) and each component rounded ONCE to  */
/* binary16, round-to-nearest-even, saturating at +-65504; selection,          */
/* Algorithm 1 and packing then work on those binary16 values; the receiver    */
/* inverts exactly and divides by 2^s.  Where an implementation rounds inside  */
/* its transform is its own affair: it is held to this definition within the   */
/* variant's error bound, not bit for bit.  Header word 12 (offset 48) carries */
/* s, and a decoder accepts only the scale it was asked for.                   */
/* ------------------------------------------------------------------------ */
static float round_half(double v)
{
    if (v != v) return (float)v;
    double a = fabs(v);
    double r;
    if (a >= 65504.0) {
        r = 65504.0;
    } else if (a == 0.0) {
        r = 0.0;
    } else {
        int e;
        frexp(a, &e); /* a = f * 2^e, f in [0.5, 1): floor(log2 a) = e - 1 */
        double q = (e - 1 < -14) ? ldexp(1.0, -24) : ldexp(1.0, e - 1 - 10);
        r = nearbyint(a / q) * q; /* a/q is exact; default rounding mode: ties to even */
        if (r > 65504.0) r = 65504.0;
    }
    return (float)(signbit(v) ? -r : r);
}

float fftsp_ref_round_half(double v) { return round_half(v); }

static int half_scale_ok(int s) { return s >= -24 && s <= 24; }

int fftsp_ref_rfft_h(const float* g, size_t n, uint32_t L, int scale_log2, float* spec, int nthreads)
{
    if (!g || !spec || n == 0 || L < 2 || !is_pow2(L) || !half_scale_ok(scale_log2)) return REF_EINVAL;
    long C = (long)chunk_count(n, L);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (long c = 0; c < C; ++c) {
        int e = rfft_chunk_ex(g + (size_t)c * L, chunk_valid(n, L, (size_t)c), L, spec + (size_t)c * (L + 2), 1,
                              scale_log2);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

int fftsp_ref_compress_h(const float* g, size_t n, uint32_t L, float theta, int bits, int scale_log2, uint8_t* packed,
                         size_t cap, int nthreads)
{
    if (!g || !packed || n == 0 || L < 2 || !is_pow2(L) || !half_scale_ok(scale_log2)) return REF_EINVAL;
    size_t C = chunk_count(n, L);
    float* spec = (float*)malloc(sizeof(float) * C * ((size_t)L + 2));
    if (!spec) return REF_ENOSPC;
    int e = fftsp_ref_rfft_h(g, n, L, scale_log2, spec, nthreads);
    if (!e) e = fftsp_ref_encode_spectrum(spec, n, L, theta, bits, packed, cap, nthreads);
    if (!e) put_u32(packed + 48, (uint32_t)scale_log2);
    free(spec);
    return e;
}

int fftsp_ref_decompress_h(const uint8_t* packed, size_t bytes, float* out, size_t n, uint32_t L, float theta, int bits,
                           int scale_log2, int nthreads)
{
    if (!out || !packed || n == 0 || L < 2 || !is_pow2(L) || !half_scale_ok(scale_log2)) return REF_EINVAL;
    size_t C = chunk_count(n, L);
    float* spec = (float*)malloc(sizeof(float) * C * ((size_t)L + 2));
    if (!spec) return REF_ENOSPC;
    int e = decode_spectrum_scaled(packed, bytes, n, L, theta, bits, 0, scale_log2, spec, nthreads);
    if (!e) {
        int err = 0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
        for (long c = 0; c < (long)C; ++c) {
            int ec = irfft_chunk_ex(spec + (size_t)c * (L + 2), chunk_valid(n, L, (size_t)c), L, out + (size_t)c * L,
                                    scale_log2);
            if (ec) {
#pragma omp atomic write
                err = ec;
            }
        }
        e = err;
    }
    free(spec);
    return e;
}

int fftsp_ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

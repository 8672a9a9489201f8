// Batched real FFT / inverse real FFT of power-of-two chunks for gfx950.
//
// The transform is the DFT sum of arXiv 1811.08596 Sec. 3.1.1 (sign -, unnormalised)
// applied per chunk, and its inverse (1/L) on the receiver (Sec. 3.1, last paragraph).
//
// Method (ours; the paper calls a vendor FFT): a real chunk of length L is read as
// M = L/2 complex samples z[j] = x[2j] + i x[2j+1]; an M-point complex FFT is followed
// by the even/odd split X[k] = E[k] + W_L^k O[k].  The M-point FFT is a Stockham
// autosort FFT held entirely in LDS (radix 8/4/2 register butterflies, one LDS
// round trip per stage).  M <= 2^13 fits one workgroup ("small" kernels, several
// chunks per workgroup when M is tiny).  Larger M is factored M = N1*N2 and done
// in two LDS-resident passes with a transposed intermediate:
//   pass A: for a tile of TA adjacent columns n2, N1-point FFTs over n1 (stride N2),
//           times W_M^(n2 k1), stored as mid[n2*N1 + k1] (contiguous in k1);
//   pass B: for a tile of rows k1 together with the mirrored rows N1-k1, N2-point
//           FFTs over n2; Z[k1 + N1 k2] and its partner Z[M-k] then sit in the same
//           workgroup, so the real-FFT split happens in LDS before the only store.
// The inverse runs the same two passes backwards (split first, 1/L at the end).
//
// LDS layout: element (i, b) of a batch of T transforms lives at i*T + (b ^ sw(i)),
// an XOR swizzle that keeps both "b fastest" and "i fastest" wave accesses spread
// over all banks without padding.
#include "internal.h"

namespace fftsp {
namespace {

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
// a * conj(b)
__device__ __forceinline__ float2 cmulc(float2 a, float2 b)
{
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}

// exp(-2 pi i E / 2^22), E < 2^22
__device__ __forceinline__ float2 twiddle(const Tables& t, uint32_t E)
{
    return cmul(t.hi[E >> 11], t.lo[E & 2047u]);
}

template <int LOGT>
__device__ __forceinline__ int sw_idx(int i, int b)
{
    if constexpr (LOGT == 0)
        return i;
    else if constexpr (LOGT >= 4)
        return (i << LOGT) + (b ^ (i & 15));
    else
        return (i << LOGT) + (b ^ ((i >> (4 - LOGT)) & ((1 << LOGT) - 1)));
}

// multiply by -i (forward) or +i (inverse)
template <bool INV>
__device__ __forceinline__ float2 rot90(float2 a)
{
    return INV ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
}

template <bool INV>
__device__ __forceinline__ void bf2(float2* v)
{
    float2 a = v[0], b = v[1];
    v[0] = cadd(a, b);
    v[1] = csub(a, b);
}

template <bool INV>
__device__ __forceinline__ void bf4(float2* v)
{
    float2 t0 = cadd(v[0], v[2]), t1 = csub(v[0], v[2]);
    float2 t2 = cadd(v[1], v[3]), t3 = rot90<INV>(csub(v[1], v[3]));
    v[0] = cadd(t0, t2);
    v[1] = cadd(t1, t3);
    v[2] = csub(t0, t2);
    v[3] = csub(t1, t3);
}

template <bool INV>
__device__ __forceinline__ void bf8(float2* v)
{
    const float c = 0.70710678118654752440f;
    float2 e[4] = {v[0], v[2], v[4], v[6]};
    float2 o[4] = {v[1], v[3], v[5], v[7]};
    bf4<INV>(e);
    bf4<INV>(o);
    // o[k] *= W8^k
    float2 o1 = o[1], o3 = o[3];
    if (INV) {
        o[1] = make_float2(c * (o1.x - o1.y), c * (o1.x + o1.y));
        o[3] = make_float2(-c * (o3.x + o3.y), c * (o3.x - o3.y));
    } else {
        o[1] = make_float2(c * (o1.x + o1.y), c * (o1.y - o1.x));
        o[3] = make_float2(c * (o3.y - o3.x), -c * (o3.x + o3.y));
    }
    o[2] = rot90<INV>(o[2]);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[k] = cadd(e[k], o[k]);
        v[k + 4] = csub(e[k], o[k]);
    }
}

template <int RL, bool INV>
__device__ __forceinline__ void butterfly(float2* v)
{
    if constexpr (RL == 1) bf2<INV>(v);
    if constexpr (RL == 2) bf4<INV>(v);
    if constexpr (RL == 3) bf8<INV>(v);
}

// One Stockham stage of radix 2^RL on T = 2^LOGT interleaved R-point transforms.
// NS = product of the radices already applied.  tw[e] = exp(-2 pi i e / R).
template <int LOGR, int LOGT, int NT, bool INV, int NS_LOG, int RL>
__device__ __forceinline__ void fft_stage(float2* d, const float2* tw, int tid)
{
    constexpr int R = 1 << LOGR, T = 1 << LOGT, RHO = 1 << RL, NS = 1 << NS_LOG;
    constexpr int NBF = (R / RHO) * T;
    static_assert(NBF % NT == 0, "butterflies must divide evenly over the workgroup");
    constexpr int PER = NBF / NT;
    float2 v[PER][RHO];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int w = tid + q * NT, b = w & (T - 1), j = w >> LOGT;
#pragma unroll
        for (int t = 0; t < RHO; ++t) v[q][t] = d[sw_idx<LOGT>(j + t * (R / RHO), b)];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int w = tid + q * NT, b = w & (T - 1), j = w >> LOGT;
        const int k = j & (NS - 1);
        if constexpr (NS > 1) {
#pragma unroll
            for (int t = 1; t < RHO; ++t) {
                const float2 c = tw[(t * k) << (LOGR - NS_LOG - RL)];
                v[q][t] = INV ? cmulc(v[q][t], c) : cmul(v[q][t], c);
            }
        }
        butterfly<RL, INV>(v[q]);
        const int base = ((j >> NS_LOG) << (NS_LOG + RL)) + k;
#pragma unroll
        for (int t = 0; t < RHO; ++t) d[sw_idx<LOGT>(base + t * NS, b)] = v[q][t];
    }
    __syncthreads();
}

template <int LOGR, int LOGT, int NT, bool INV, int NS_LOG = 0>
__device__ __forceinline__ void run_fft(float2* d, const float2* tw, int tid)
{
    if constexpr (NS_LOG < LOGR) {
        constexpr int rem = LOGR - NS_LOG;
        constexpr int RL = rem == 1 ? 1 : (rem % 3 == 0 ? 3 : 2);
        fft_stage<LOGR, LOGT, NT, INV, NS_LOG, RL>(d, tw, tid);
        run_fft<LOGR, LOGT, NT, INV, NS_LOG + RL>(d, tw, tid);
    }
}

template <int LOGR, int NT>
__device__ __forceinline__ void load_stage_twiddles(float2* tw, const Tables& tb, int tid)
{
    if constexpr (LOGR <= 11) {
        for (int e = tid; e < (1 << LOGR); e += NT) tw[e] = tb.hi[e << (11 - LOGR)];
    } else {
        for (int e = tid; e < (1 << LOGR); e += NT) tw[e] = twiddle(tb, (uint32_t)e << (22 - LOGR));
    }
}

__device__ __forceinline__ float2 load_pair(const float* __restrict__ in, size_t gi, size_t n, int aligned)
{
    if (gi + 1 < n) {
        if (aligned) return *reinterpret_cast<const float2*>(in + gi);
        return make_float2(in[gi], in[gi + 1]);
    }
    if (gi < n) return make_float2(in[gi], 0.f);
    return make_float2(0.f, 0.f);
}

__device__ __forceinline__ void store_pair(float* __restrict__ out, size_t gi, size_t n, int aligned, float2 v)
{
    if (gi + 1 < n) {
        if (aligned)
            *reinterpret_cast<float2*>(out + gi) = v;
        else {
            out[gi] = v.x;
            out[gi + 1] = v.y;
        }
    } else if (gi < n) {
        out[gi] = v.x;
    }
}

// X[k] from a = Z[k], b = Z[M-k], w = W_L^k   (0 < k < M)
__device__ __forceinline__ float2 split_fwd(float2 a, float2 b, float2 w)
{
    const float er = 0.5f * (a.x + b.x), ei = 0.5f * (a.y - b.y);
    const float dr = 0.5f * (a.x - b.x), di = 0.5f * (a.y + b.y);
    return make_float2(er + (w.x * di + w.y * dr), ei - (w.x * dr - w.y * di));
}

// 2 Z[k] from a = X[k], b = X[M-k], w = W_L^k  (the factor 1/2 is folded into the final 1/L)
__device__ __forceinline__ float2 split_inv(float2 a, float2 b, float2 w)
{
    const float er = a.x + b.x, ei = a.y - b.y;
    const float dr = a.x - b.x, di = a.y + b.y;
    const float orr = w.x * dr + w.y * di, oi = w.x * di - w.y * dr;  // conj(w) * d
    return make_float2(er - oi, ei + orr);
}

// ------------------------------------------------------------------ small ---
// M = 2^LOGM <= 2^13 complex points per chunk, 2^(LOGE-LOGM) chunks per workgroup.
template <int LOGM, int LOGE, int NT>
__global__ __launch_bounds__(NT) void k_fwd_small(const float* __restrict__ in, size_t n, size_t C,
                                                  float2* __restrict__ spec, Tables tb, int aligned)
{
    constexpr int M = 1 << LOGM, LOGT = LOGE - LOGM, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid = threadIdx.x;
    const size_t c0 = (size_t)blockIdx.x << LOGT;
    load_stage_twiddles<LOGM, NT>(tw, tb, tid);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, i = w & (M - 1), b = w >> LOGM;
        const size_t gi = (c0 + b) * (size_t)(2 * M) + 2 * (size_t)i;
        d[sw_idx<LOGT>(i, b)] = load_pair(in, gi, n, aligned);
    }
    __syncthreads();
    run_fft<LOGM, LOGT, NT, false>(d, tw, tid);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, k = w & (M - 1), b = w >> LOGM;
        const size_t c = c0 + b;
        if (c >= C) continue;
        float2* out = spec + c * (size_t)(M + 1);
        const float2 a = d[sw_idx<LOGT>(k, b)];
        if (k == 0) {
            out[0] = make_float2(a.x + a.y, 0.f);
            out[M] = make_float2(a.x - a.y, 0.f);
        } else {
            const float2 bq = d[sw_idx<LOGT>(M - k, b)];
            out[k] = split_fwd(a, bq, twiddle(tb, (uint32_t)k << (21 - LOGM)));
        }
    }
}

template <int LOGM, int LOGE, int NT>
__global__ __launch_bounds__(NT) void k_inv_small(const float2* __restrict__ spec, size_t n, size_t C,
                                                  float* __restrict__ out, Tables tb, int aligned)
{
    constexpr int M = 1 << LOGM, LOGT = LOGE - LOGM, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid = threadIdx.x;
    const size_t c0 = (size_t)blockIdx.x << LOGT;
    load_stage_twiddles<LOGM, NT>(tw, tb, tid);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, k = w & (M - 1), b = w >> LOGM;
        const size_t c = c0 + b;
        float2 z = make_float2(0.f, 0.f);
        if (c < C) {
            const float2* X = spec + c * (size_t)(M + 1);
            float2 a = X[k], bq = X[M - k];
            if (k == 0) {  // imaginary parts of the DC and Nyquist bins are ignored
                a.y = 0.f;
                bq.y = 0.f;
            }
            z = split_inv(a, bq, twiddle(tb, (uint32_t)k << (21 - LOGM)));
        }
        d[sw_idx<LOGT>(k, b)] = z;
    }
    __syncthreads();
    run_fft<LOGM, LOGT, NT, true>(d, tw, tid);
    const float scale = 1.0f / (float)(2 * M);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, i = w & (M - 1), b = w >> LOGM;
        const size_t gi = (c0 + b) * (size_t)(2 * M) + 2 * (size_t)i;
        float2 v = d[sw_idx<LOGT>(i, b)];
        store_pair(out, gi, n, aligned, make_float2(v.x * scale, v.y * scale));
    }
}

// --------------------------------------------------------------- two pass ---
// Forward pass A: N1-point FFTs down the columns of the N1 x N2 view of z.
template <int LOGN1, int LOGE, int NT>
__global__ __launch_bounds__(NT) void k_fwd_a(const float* __restrict__ in, size_t n, int logM,
                                              float2* __restrict__ mid, Tables tb, int aligned)
{
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1, TA = 1 << LOGT, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid = threadIdx.x;
    const uint32_t M = 1u << logM, N2 = M >> LOGN1, tiles = N2 >> LOGT;
    const size_t c = blockIdx.x / tiles;
    const uint32_t col0 = (blockIdx.x % tiles) << LOGT;
    load_stage_twiddles<LOGN1, NT>(tw, tb, tid);
    const size_t cbase = c * (size_t)(2 * (size_t)M);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
        const size_t gi = cbase + 2 * ((size_t)n1 * N2 + col0 + col);
        d[sw_idx<LOGT>(n1, col)] = load_pair(in, gi, n, aligned);
    }
    __syncthreads();
    run_fft<LOGN1, LOGT, NT, false>(d, tw, tid);
    float2* out = mid + c * (size_t)M;
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, k1 = w & (N1 - 1), col = w >> LOGN1;
        const uint32_t n2 = col0 + col;
        const float2 v = d[sw_idx<LOGT>(k1, col)];
        out[(size_t)n2 * N1 + k1] = cmul(v, twiddle(tb, (n2 * (uint32_t)k1) << (22 - logM)));
    }
}

// Row held by LDS slot s of the pass-B tile starting at row r0: slots [0,TB) are rows r0.., slots [TB,2TB)
// are their mirrors N1-row; row 0's mirror slot holds row N1/2 (both are their own partners).
template <int TB>
__device__ __forceinline__ uint32_t row_of_slot(int s, uint32_t r0, uint32_t N1)
{
    if (s < TB) return r0 + s;
    const uint32_t row = N1 - r0 - (uint32_t)(s - TB);
    return row == N1 ? N1 / 2 : row;
}

// Forward pass B: N2-point FFTs along n2 for a tile of rows and their mirrors, then the real-FFT split.
template <int LOGN2, int LOGE, int NT>
__global__ __launch_bounds__(NT) void k_fwd_b(const float2* __restrict__ mid, int logM, float2* __restrict__ spec,
                                              Tables tb)
{
    constexpr int N2 = 1 << LOGN2, LOGT = LOGE - LOGN2, T2 = 1 << LOGT, TB = T2 / 2, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid = threadIdx.x;
    const int logN1 = logM - LOGN2;
    const uint32_t M = 1u << logM, N1 = 1u << logN1, tiles = N1 >> LOGT;
    const size_t c = blockIdx.x / tiles;
    const uint32_t r0 = (blockIdx.x % tiles) * TB;
    load_stage_twiddles<LOGN2, NT>(tw, tb, tid);
    const float2* src = mid + c * (size_t)M;
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, slot = w & (T2 - 1), n2 = w >> LOGT;
        d[sw_idx<LOGT>(n2, slot)] = src[(size_t)n2 * N1 + row_of_slot<TB>(slot, r0, N1)];
    }
    __syncthreads();
    run_fft<LOGN2, LOGT, NT, false>(d, tw, tid);
    float2* out = spec + c * (size_t)(M + 1);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, slot = w & (T2 - 1), k2 = w >> LOGT;
        const uint32_t k1 = row_of_slot<TB>(slot, r0, N1);
        const uint32_t k = k1 + ((uint32_t)k2 << logN1);
        const float2 a = d[sw_idx<LOGT>(k2, slot)];
        if (k == 0) {
            out[0] = make_float2(a.x + a.y, 0.f);
            out[M] = make_float2(a.x - a.y, 0.f);
            continue;
        }
        const bool self = (k1 == 0) || (k1 == N1 / 2);
        const int ps = self ? slot : (slot ^ TB);
        const int k2p = (k1 == 0) ? ((N2 - k2) & (N2 - 1)) : (N2 - 1 - k2);
        const float2 b = d[sw_idx<LOGT>(k2p, ps)];
        out[k] = split_fwd(a, b, twiddle(tb, k << (21 - logM)));
    }
}

// Inverse pass B: undo the split, inverse N2-point FFTs over k2, times conj W_M^(n2 k1).
template <int LOGN2, int LOGE, int NT>
__global__ __launch_bounds__(NT) void k_inv_b(const float2* __restrict__ spec, int logM, float2* __restrict__ mid,
                                              Tables tb)
{
    constexpr int N2 = 1 << LOGN2, LOGT = LOGE - LOGN2, T2 = 1 << LOGT, TB = T2 / 2, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid = threadIdx.x;
    const int logN1 = logM - LOGN2;
    const uint32_t M = 1u << logM, N1 = 1u << logN1, tiles = N1 >> LOGT;
    const size_t c = blockIdx.x / tiles;
    const uint32_t r0 = (blockIdx.x % tiles) * TB;
    load_stage_twiddles<LOGN2, NT>(tw, tb, tid);
    const float2* X = spec + c * (size_t)(M + 1);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, slot = w & (T2 - 1), k2 = w >> LOGT;
        const uint32_t k = row_of_slot<TB>(slot, r0, N1) + ((uint32_t)k2 << logN1);
        d[sw_idx<LOGT>(k2, slot)] = X[k];
    }
    __syncthreads();
    float2 z[ELEMS / NT];
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, slot = w & (T2 - 1), k2 = w >> LOGT;
        const uint32_t k1 = row_of_slot<TB>(slot, r0, N1);
        const uint32_t k = k1 + ((uint32_t)k2 << logN1);
        float2 a = d[sw_idx<LOGT>(k2, slot)], b;
        if (k == 0) {
            b = X[M];
            a.y = 0.f;
            b.y = 0.f;
        } else {
            const bool self = (k1 == 0) || (k1 == N1 / 2);
            const int ps = self ? slot : (slot ^ TB);
            const int k2p = (k1 == 0) ? ((N2 - k2) & (N2 - 1)) : (N2 - 1 - k2);
            b = d[sw_idx<LOGT>(k2p, ps)];
        }
        z[q] = split_inv(a, b, twiddle(tb, k << (21 - logM)));
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, slot = w & (T2 - 1), k2 = w >> LOGT;
        d[sw_idx<LOGT>(k2, slot)] = z[q];
    }
    __syncthreads();
    run_fft<LOGN2, LOGT, NT, true>(d, tw, tid);
    float2* dst = mid + c * (size_t)M;
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, slot = w & (T2 - 1), n2 = w >> LOGT;
        const uint32_t k1 = row_of_slot<TB>(slot, r0, N1);
        const float2 v = d[sw_idx<LOGT>(n2, slot)];
        dst[(size_t)n2 * N1 + k1] = cmulc(v, twiddle(tb, ((uint32_t)n2 * k1) << (22 - logM)));
    }
}

// Inverse pass A: inverse N1-point FFTs over k1 for a tile of columns n2; writes the real samples.
template <int LOGN1, int LOGE, int NT>
__global__ __launch_bounds__(NT) void k_inv_a(const float2* __restrict__ mid, int logM, float* __restrict__ out,
                                              size_t n, Tables tb, int aligned)
{
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1, TA = 1 << LOGT, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid = threadIdx.x;
    const uint32_t M = 1u << logM, N2 = M >> LOGN1, tiles = N2 >> LOGT;
    const size_t c = blockIdx.x / tiles;
    const uint32_t col0 = (blockIdx.x % tiles) << LOGT;
    load_stage_twiddles<LOGN1, NT>(tw, tb, tid);
    const float2* src = mid + c * (size_t)M;
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, k1 = w & (N1 - 1), col = w >> LOGN1;
        d[sw_idx<LOGT>(k1, col)] = src[(size_t)(col0 + col) * N1 + k1];
    }
    __syncthreads();
    run_fft<LOGN1, LOGT, NT, true>(d, tw, tid);
    const float scale = 1.0f / (float)(2u * M);
    const size_t cbase = c * (size_t)(2 * (size_t)M);
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
        const size_t gi = cbase + 2 * ((size_t)n1 * N2 + col0 + col);
        const float2 v = d[sw_idx<LOGT>(n1, col)];
        store_pair(out, gi, n, aligned, make_float2(v.x * scale, v.y * scale));
    }
}

// ---------------------------------------------------------------- launch ----
constexpr int kNT = 256;

template <typename K>
hipError_t set_lds(K kernel, size_t bytes)
{
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

template <int LOGM>
hipError_t small_fwd(const float* in, size_t n, size_t C, float2* spec, Tables t, int aligned, hipStream_t s)
{
    constexpr int LOGE = LOGM >= 12 ? LOGM : 12;
    const size_t lds = ((size_t)(1 << LOGE) + (1 << LOGM)) * sizeof(float2);
    auto kern = k_fwd_small<LOGM, LOGE, kNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t per = (size_t)1 << (LOGE - LOGM);
    FFTSP_LAUNCH("rfft_small", kern, dim3((unsigned)((C + per - 1) / per)), dim3(kNT), lds, s, in, n, C, spec, t, aligned);
    return hipGetLastError();
}

template <int LOGM>
hipError_t small_inv(const float2* spec, size_t n, size_t C, float* out, Tables t, int aligned, hipStream_t s)
{
    constexpr int LOGE = LOGM >= 12 ? LOGM : 12;
    const size_t lds = ((size_t)(1 << LOGE) + (1 << LOGM)) * sizeof(float2);
    auto kern = k_inv_small<LOGM, LOGE, kNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t per = (size_t)1 << (LOGE - LOGM);
    FFTSP_LAUNCH("irfft_small", kern, dim3((unsigned)((C + per - 1) / per)), dim3(kNT), lds, s, spec, n, C, out, t, aligned);
    return hipGetLastError();
}

constexpr int kLogE = 13;  // 8192 complex points (64 KiB) per workgroup in the two-pass kernels

template <int LOGN1>
hipError_t fwd_a(const float* in, size_t n, int logM, size_t C, float2* mid, Tables t, int aligned, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN1)) * sizeof(float2);
    auto kern = k_fwd_a<LOGN1, kLogE, kNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t tiles = ((size_t)1 << (logM - LOGN1)) >> (kLogE - LOGN1);
    FFTSP_LAUNCH("rfft_pass_a", kern, dim3((unsigned)(C * tiles)), dim3(kNT), lds, s, in, n, logM, mid, t, aligned);
    return hipGetLastError();
}

template <int LOGN2>
hipError_t fwd_b(const float2* mid, int logM, size_t C, float2* spec, Tables t, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN2)) * sizeof(float2);
    auto kern = k_fwd_b<LOGN2, kLogE, kNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t tiles = ((size_t)1 << (logM - LOGN2)) >> (kLogE - LOGN2);
    FFTSP_LAUNCH("rfft_pass_b", kern, dim3((unsigned)(C * tiles)), dim3(kNT), lds, s, mid, logM, spec, t);
    return hipGetLastError();
}

template <int LOGN2>
hipError_t inv_b(const float2* spec, int logM, size_t C, float2* mid, Tables t, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN2)) * sizeof(float2);
    auto kern = k_inv_b<LOGN2, kLogE, kNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t tiles = ((size_t)1 << (logM - LOGN2)) >> (kLogE - LOGN2);
    FFTSP_LAUNCH("irfft_pass_b", kern, dim3((unsigned)(C * tiles)), dim3(kNT), lds, s, spec, logM, mid, t);
    return hipGetLastError();
}

template <int LOGN1>
hipError_t inv_a(const float2* mid, int logM, size_t C, float* out, size_t n, Tables t, int aligned, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN1)) * sizeof(float2);
    auto kern = k_inv_a<LOGN1, kLogE, kNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t tiles = ((size_t)1 << (logM - LOGN1)) >> (kLogE - LOGN1);
    FFTSP_LAUNCH("irfft_pass_a", kern, dim3((unsigned)(C * tiles)), dim3(kNT), lds, s, mid, logM, out, n, t, aligned);
    return hipGetLastError();
}

}  // namespace

#define FFTSP_SMALL_CASES(X) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13)

hipError_t launch_rfft(const float* in, size_t n, int logL, size_t C, float* spec, float2* mid, Tables t,
                       hipStream_t s)
{
    const int logM = logL - 1;
    const int aligned = (reinterpret_cast<uintptr_t>(in) & 7u) == 0;
    float2* sp = reinterpret_cast<float2*>(spec);
    if (C * ((size_t)1 << (logM > 13 ? logM - 13 : 0)) > 0x7fffffffu) return hipErrorInvalidValue;
    switch (logM) {
#define X(p) \
    case p: return small_fwd<p>(in, n, C, sp, t, aligned, s);
        FFTSP_SMALL_CASES(X)
#undef X
        default: break;
    }
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    switch (logN1) {
        case 7: e = fwd_a<7>(in, n, logM, C, mid, t, aligned, s); break;
        case 8: e = fwd_a<8>(in, n, logM, C, mid, t, aligned, s); break;
        case 9: e = fwd_a<9>(in, n, logM, C, mid, t, aligned, s); break;
        case 10: e = fwd_a<10>(in, n, logM, C, mid, t, aligned, s); break;
        case 11: e = fwd_a<11>(in, n, logM, C, mid, t, aligned, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    switch (logN2) {
        case 7: return fwd_b<7>(mid, logM, C, sp, t, s);
        case 8: return fwd_b<8>(mid, logM, C, sp, t, s);
        case 9: return fwd_b<9>(mid, logM, C, sp, t, s);
        case 10: return fwd_b<10>(mid, logM, C, sp, t, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_irfft(const float* spec, size_t n, int logL, size_t C, float* out, float2* mid, Tables t,
                        hipStream_t s)
{
    const int logM = logL - 1;
    const int aligned = (reinterpret_cast<uintptr_t>(out) & 7u) == 0;
    const float2* sp = reinterpret_cast<const float2*>(spec);
    if (C * ((size_t)1 << (logM > 13 ? logM - 13 : 0)) > 0x7fffffffu) return hipErrorInvalidValue;
    switch (logM) {
#define X(p) \
    case p: return small_inv<p>(sp, n, C, out, t, aligned, s);
        FFTSP_SMALL_CASES(X)
#undef X
        default: break;
    }
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    switch (logN2) {
        case 7: e = inv_b<7>(sp, logM, C, mid, t, s); break;
        case 8: e = inv_b<8>(sp, logM, C, mid, t, s); break;
        case 9: e = inv_b<9>(sp, logM, C, mid, t, s); break;
        case 10: e = inv_b<10>(sp, logM, C, mid, t, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    switch (logN1) {
        case 7: return inv_a<7>(mid, logM, C, out, n, t, aligned, s);
        case 8: return inv_a<8>(mid, logM, C, out, n, t, aligned, s);
        case 9: return inv_a<9>(mid, logM, C, out, n, t, aligned, s);
        case 10: return inv_a<10>(mid, logM, C, out, n, t, aligned, s);
        case 11: return inv_a<11>(mid, logM, C, out, n, t, aligned, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fftsp

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
//           times W_M^(n2 k1), stored as runs of N1 values per n2 (row k1 next to row N1-k1);
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
                                                  float2* __restrict__ spec, uint32_t sstride, Tables tb, int aligned)
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
        float2* out = spec + c * (size_t)sstride;
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
__global__ __launch_bounds__(NT) void k_inv_small(const float2* __restrict__ spec, uint32_t sstride, size_t n, size_t C,
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
            const float2* X = spec + c * (size_t)sstride;
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
// The two-pass kernels are persistent: a workgroup of 512 lanes walks a contiguous run of tiles and, while
// the LDS FFT of tile i runs, the global loads of tile i+1 are already in flight into registers.
//
// Twiddles outside the LDS stages are not gathered per element.  Along the index a lane walks, the exponent
// grows by a fixed step, so W^(e0 + j*step) = W^e0 * (W^step)^j: one table lookup for the base, one for the
// ratio, then a short recurrence that is re-anchored from the table every 8 steps; for the even/odd split the
// step is always 1/32 of a turn, so exact constants are used instead of a recurrence.

// Loop-invariant per-lane addresses (LDS swizzles, global offsets of 16 loads and 16 stores, four stages of
// butterfly indices) would otherwise be hoisted out of the persistent loop and held in ~100 VGPRs; making the
// lane id opaque once per iteration has them recomputed (a few integer ops) and keeps two workgroups per CU.
__device__ __forceinline__ int opaque_lane(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

constexpr int kNT = 512;   // lanes per workgroup in the two-pass kernels
constexpr int kLogE = 13;  // 8192 complex points (64 KiB) per tile
constexpr int kPer = (1 << kLogE) / kNT;
constexpr int kSplitStep = (16 * kNT) >> kLogE;  // 32nds of a turn between a lane's consecutive split twiddles
constexpr int kHistLdsWords = kHistBins / 2;  // 16-bit counters, two per word

// exp(-2 pi i q / 32), q = 0..15
__device__ constexpr float kW32re[16] = {1.0f, 0.98078528040323043f, 0.92387953251128674f, 0.83146961230254524f,
                                         0.70710678118654752f, 0.55557023301960223f, 0.38268343236508977f,
                                         0.19509032201612827f, 0.0f, -0.19509032201612827f, -0.38268343236508977f,
                                         -0.55557023301960223f, -0.70710678118654752f, -0.83146961230254524f,
                                         -0.92387953251128674f, -0.98078528040323043f};
__device__ constexpr float kW32im[16] = {-0.0f, -0.19509032201612827f, -0.38268343236508977f, -0.55557023301960223f,
                                         -0.70710678118654752f, -0.83146961230254524f, -0.92387953251128674f,
                                         -0.98078528040323043f, -1.0f, -0.98078528040323043f, -0.92387953251128674f,
                                         -0.83146961230254524f, -0.70710678118654752f, -0.55557023301960223f,
                                         -0.38268343236508977f, -0.19509032201612827f};

// The intermediate between the two passes is stored "paired": within each run of N1 values, row k1 and its
// mirror N1-k1 (the two rows the real-FFT split combines) sit next to each other,
//     position 2*k1   holds row k1        (k1 < N1/2)
//     position 2*k1+1 holds row N1-k1     (position 1 holds row N1/2, which like row 0 is its own mirror)
// so a pass-B tile of TB rows plus their mirrors is one contiguous run of 2*TB positions (128 bytes for TB = 8).
__device__ __forceinline__ uint32_t row_of_pos(uint32_t p, uint32_t N1)
{
    return (p & 1u) ? (p == 1u ? N1 / 2 : N1 - (p >> 1)) : (p >> 1);
}

// Forward pass A: N1-point FFTs down the columns of the N1 x N2 view of z, for tiles of TA adjacent columns.
template <int LOGN1>
__global__ __launch_bounds__(kNT) void k_fwd_a(const float* __restrict__ in, size_t n, int logM,
                                               float2* __restrict__ mid, Tables tb, int aligned, uint32_t total,
                                               uint32_t per_wg, uint32_t* __restrict__ zero_ptr, uint32_t zero_words)
{
    constexpr int NT = kNT, LOGE = kLogE, PER = kPer;
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1, TA = 1 << LOGT, ELEMS = 1 << LOGE;
    // clears the status words and key histograms the next kernels of the sender accumulate into
    for (uint32_t i = blockIdx.x * NT + threadIdx.x; i < zero_words; i += gridDim.x * NT) zero_ptr[i] = 0u;
    constexpr int KN = N1 >= NT ? N1 / NT : 1;   // distinct k1 per lane in the store loop
    constexpr int DC = N1 >= NT ? 1 : NT / N1;   // column step between a lane's consecutive stores
    constexpr int NCOL = PER / KN;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid0 = threadIdx.x;
    const uint32_t M = 1u << logM, N2 = M >> LOGN1, tiles = N2 >> LOGT;
    uint32_t t = blockIdx.x * per_wg;
    const uint32_t tend = t + per_wg < total ? t + per_wg : total;
    if (t >= tend) return;
    load_stage_twiddles<LOGN1, NT>(tw, tb, tid0);

    float2 r[PER];
    auto load_tile = [&](uint32_t tile, int tid) {
        const size_t cbase = (size_t)(tile / tiles) * (size_t)(2 * (size_t)M);
        const uint32_t col0 = (tile % tiles) << LOGT;
        if (aligned && cbase + 2 * (size_t)M <= n) {  // whole chunk present: no per-element guards
            const float2* src = reinterpret_cast<const float2*>(in + cbase) + col0;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
                r[q] = src[(uint32_t)n1 * N2 + col];
            }
        } else {
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
                r[q] = load_pair(in, cbase + 2 * ((size_t)n1 * N2 + col0 + col), n, aligned);
            }
        }
    };
    load_tile(t, tid0);
    for (;;) {
        const int tid = opaque_lane(tid0);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
            d[sw_idx<LOGT>(n1, col)] = r[q];
        }
        __syncthreads();
        const bool more = t + 1 < tend;
        if (more) load_tile(t + 1, tid);
        run_fft<LOGN1, LOGT, NT, false>(d, tw, tid);
        float2* out = mid + (size_t)(t / tiles) * (size_t)M;
        const uint32_t col0 = (t % tiles) << LOGT;
        const int sh = 22 - logM;
#pragma unroll
        for (int kk = 0; kk < KN; ++kk) {
            const uint32_t pos = (uint32_t)(tid + kk * NT) & (N1 - 1);  // paired position this lane stores to
            const uint32_t k1 = row_of_pos(pos, N1);
            const uint32_t cfirst = (uint32_t)(tid + kk * NT) >> LOGN1;
            const float2 ratio = twiddle(tb, ((uint32_t)DC * k1) << sh);
            float2 cur = make_float2(1.f, 0.f);
#pragma unroll
            for (int j = 0; j < NCOL; ++j) {
                const uint32_t col = cfirst + j * DC, n2 = col0 + col;
                if (j % 8 == 0) cur = twiddle(tb, (n2 * k1) << sh);
                out[n2 * N1 + pos] = cmul(d[sw_idx<LOGT>(k1, col)], cur);
                cur = cmul(cur, ratio);
            }
        }
        if (!more) break;
        ++t;
        __syncthreads();
    }
}

__device__ __forceinline__ uint32_t fft_key_of(float2 z)
{
    return __float_as_uint(__fmaf_rn(z.x, z.x, __fmul_rn(z.y, z.y)));
}

// Forward pass B: N2-point FFTs along n2 for a tile of rows and their mirrors, then the real-FFT split and,
// if hist != nullptr, the first radix-select digit of every bin's key (12-bit histogram per chunk).
template <int LOGN2>
__global__ __launch_bounds__(kNT) void k_fwd_b(const float2* __restrict__ mid, int logM, float2* __restrict__ spec,
                                               uint32_t sstride, Tables tb, uint32_t* __restrict__ hist,
                                               uint32_t total, uint32_t per_wg, int pair_spec)
{
    constexpr int NT = kNT, LOGE = kLogE, PER = kPer;
    constexpr int N2 = 1 << LOGN2, LOGT = LOGE - LOGN2, T2 = 1 << LOGT, ELEMS = 1 << LOGE;
    static_assert(NT % T2 == 0, "a lane keeps one slot");
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    uint32_t* h16 = reinterpret_cast<uint32_t*>(tw + N2);
    const int tid0 = threadIdx.x;
    const int logN1 = logM - LOGN2;
    const uint32_t M = 1u << logM, N1 = 1u << logN1, tiles = N1 >> LOGT;
    uint32_t t = blockIdx.x * per_wg;
    const uint32_t tend = t + per_wg < total ? t + per_wg : total;
    if (t >= tend) return;
    load_stage_twiddles<LOGN2, NT>(tw, tb, tid0);
    if (hist)
        for (int i = tid0; i < kHistLdsWords; i += NT) h16[i] = 0u;
    constexpr int DK = NT >> LOGT;  // k2 step between a lane's consecutive elements

    float2 r[PER];
    auto load_tile = [&](uint32_t tile, int tid) {
        const int slot = tid & (T2 - 1), kq0 = tid >> LOGT;
        const float2* src = mid + (size_t)(tile / tiles) * (size_t)M;
        const uint32_t pos = (tile % tiles) * T2 + slot;
#pragma unroll
        for (int q = 0; q < PER; ++q) r[q] = src[(uint32_t)(kq0 + q * DK) * N1 + pos];
    };
    load_tile(t, tid0);
    for (;;) {
        const int tid = opaque_lane(tid0);
        const int slot = tid & (T2 - 1), kq0 = tid >> LOGT;
#pragma unroll
        for (int q = 0; q < PER; ++q) d[sw_idx<LOGT>(kq0 + q * DK, slot)] = r[q];
        __syncthreads();
        const bool more = t + 1 < tend;
        if (more) load_tile(t + 1, tid);
        run_fft<LOGN2, LOGT, NT, false>(d, tw, tid);
        const size_t c = t / tiles;
        float2* out = spec + c * (size_t)sstride;
        const uint32_t pos = (t % tiles) * T2 + slot;
        const uint32_t k1 = row_of_pos(pos, N1);
        const uint32_t col = pair_spec ? pos : k1;  // where this lane's row sits inside each run of N1 bins
        const bool self = (k1 == 0) || (k1 == N1 / 2);
        const int ps = self ? slot : (slot ^ 1);
        // W_L^(k1 + N1*k2): k2 advances by DK per step, i.e. by exactly kSplitStep 32nds of a turn
        const float2 base = twiddle(tb, (k1 + ((uint32_t)kq0 << logN1)) << (21 - logM));
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int k2 = kq0 + q * DK;
            const uint32_t k = k1 + ((uint32_t)k2 << logN1);
            const float2 a = d[sw_idx<LOGT>(k2, slot)];
            float2 x;
            if (k == 0) {
                x = make_float2(a.x + a.y, 0.f);
                const float2 xm = make_float2(a.x - a.y, 0.f);
                out[M] = xm;
                if (hist) {
                    const uint32_t b = fft_key_of(xm) >> kKeyShift;
                    atomicAdd(&h16[b >> 1], 1u << ((b & 1u) * 16u));
                }
            } else {
                const int k2p = (k1 == 0) ? ((N2 - k2) & (N2 - 1)) : (N2 - 1 - k2);
                const float2 b = d[sw_idx<LOGT>(k2p, ps)];
                x = split_fwd(a, b, cmul(base, make_float2(kW32re[q * kSplitStep], kW32im[q * kSplitStep])));
            }
            out[col + ((uint32_t)k2 << logN1)] = x;
            if (hist) {
                const uint32_t b = fft_key_of(x) >> kKeyShift;
                atomicAdd(&h16[b >> 1], 1u << ((b & 1u) * 16u));
            }
        }
        if (hist) {  // at most 8193 bins per tile, so the 16-bit halves cannot carry into each other
            __syncthreads();
            uint32_t* g = hist + c * kHistBins;
            for (int i = tid; i < kHistLdsWords; i += NT) {
                const uint32_t v = h16[i];
                if (v) {
                    if (v & 0xFFFFu) atomicAdd(&g[2 * i], v & 0xFFFFu);
                    if (v >> 16) atomicAdd(&g[2 * i + 1], v >> 16);
                    h16[i] = 0u;
                }
            }
        }
        if (!more) break;
        ++t;
        __syncthreads();
    }
}

// Inverse pass B: undo the split, inverse N2-point FFTs over k2, times conj W_M^(n2 k1).
template <int LOGN2>
__global__ __launch_bounds__(kNT) void k_inv_b(const float2* __restrict__ spec, uint32_t sstride, int logM,
                                               float2* __restrict__ mid, Tables tb, uint32_t total, uint32_t per_wg,
                                               int pair_spec)
{
    constexpr int NT = kNT, LOGE = kLogE, PER = kPer;
    constexpr int N2 = 1 << LOGN2, LOGT = LOGE - LOGN2, T2 = 1 << LOGT, ELEMS = 1 << LOGE;
    static_assert(NT % T2 == 0, "a lane keeps one slot");
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid0 = threadIdx.x;
    const int logN1 = logM - LOGN2;
    const uint32_t M = 1u << logM, N1 = 1u << logN1, tiles = N1 >> LOGT;
    uint32_t t = blockIdx.x * per_wg;
    const uint32_t tend = t + per_wg < total ? t + per_wg : total;
    if (t >= tend) return;
    load_stage_twiddles<LOGN2, NT>(tw, tb, tid0);
    constexpr int DK = NT >> LOGT;

    float2 r[PER];
    float2 xnyq = make_float2(0.f, 0.f);
    auto load_tile = [&](uint32_t tile, int tid) {
        const int slot = tid & (T2 - 1), kq0 = tid >> LOGT;
        const float2* X = spec + (size_t)(tile / tiles) * (size_t)sstride;
        const uint32_t pos = (tile % tiles) * T2 + slot, row = row_of_pos(pos, N1);
        const uint32_t col = pair_spec ? pos : row;
#pragma unroll
        for (int q = 0; q < PER; ++q) r[q] = X[col + ((uint32_t)(kq0 + q * DK) << logN1)];
        if (row == 0 && kq0 == 0) xnyq = X[M];
    };
    load_tile(t, tid0);
    for (;;) {
        const int tid = opaque_lane(tid0);
        const int slot = tid & (T2 - 1), kq0 = tid >> LOGT;
#pragma unroll
        for (int q = 0; q < PER; ++q) d[sw_idx<LOGT>(kq0 + q * DK, slot)] = r[q];
        const float2 xm = xnyq;
        __syncthreads();
        const uint32_t pos = (t % tiles) * T2 + slot;
        const uint32_t k1 = row_of_pos(pos, N1);
        const bool self = (k1 == 0) || (k1 == N1 / 2);
        const int ps = self ? slot : (slot ^ 1);
        const float2 base = twiddle(tb, (k1 + ((uint32_t)kq0 << logN1)) << (21 - logM));
        float2 z[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int k2 = kq0 + q * DK;
            const uint32_t k = k1 + ((uint32_t)k2 << logN1);
            float2 a = r[q], b;
            if (k == 0) {  // imaginary parts of the DC and Nyquist bins are ignored
                b = xm;
                a.y = 0.f;
                b.y = 0.f;
            } else {
                const int k2p = (k1 == 0) ? ((N2 - k2) & (N2 - 1)) : (N2 - 1 - k2);
                b = d[sw_idx<LOGT>(k2p, ps)];
            }
            z[q] = split_inv(a, b, cmul(base, make_float2(kW32re[q * kSplitStep], kW32im[q * kSplitStep])));
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PER; ++q) d[sw_idx<LOGT>(kq0 + q * DK, slot)] = z[q];
        __syncthreads();
        const bool more = t + 1 < tend;
        if (more) load_tile(t + 1, tid);
        run_fft<LOGN2, LOGT, NT, true>(d, tw, tid);
        float2* dst = mid + (size_t)(t / tiles) * (size_t)M;
        const int sh = 22 - logM;
        const float2 ratio = twiddle(tb, ((uint32_t)DK * k1) << sh);
        float2 cur = make_float2(1.f, 0.f);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const uint32_t n2 = (uint32_t)(kq0 + q * DK);
            if (q % 8 == 0) cur = twiddle(tb, (n2 * k1) << sh);
            dst[n2 * N1 + pos] = cmulc(d[sw_idx<LOGT>((int)n2, slot)], cur);
            cur = cmul(cur, ratio);
        }
        if (!more) break;
        ++t;
        __syncthreads();
    }
}

// Inverse pass A: inverse N1-point FFTs over k1 for a tile of columns n2; writes the real samples.
template <int LOGN1>
__global__ __launch_bounds__(kNT) void k_inv_a(const float2* __restrict__ mid, int logM, float* __restrict__ out,
                                               size_t n, Tables tb, int aligned, uint32_t total, uint32_t per_wg)
{
    constexpr int NT = kNT, LOGE = kLogE, PER = kPer;
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1, TA = 1 << LOGT, ELEMS = 1 << LOGE;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid0 = threadIdx.x;
    const uint32_t M = 1u << logM, N2 = M >> LOGN1, tiles = N2 >> LOGT;
    uint32_t t = blockIdx.x * per_wg;
    const uint32_t tend = t + per_wg < total ? t + per_wg : total;
    if (t >= tend) return;
    load_stage_twiddles<LOGN1, NT>(tw, tb, tid0);

    float2 r[PER];
    auto load_tile = [&](uint32_t tile, int tid) {
        const float2* src = mid + (size_t)(tile / tiles) * (size_t)M;
        const uint32_t col0 = (tile % tiles) << LOGT;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int w = tid + q * NT, pos = w & (N1 - 1), col = w >> LOGN1;
            r[q] = src[(uint32_t)(col0 + col) * N1 + pos];
        }
    };
    load_tile(t, tid0);
    const float scale = 1.0f / (float)(2u * M);
    for (;;) {
        const int tid = opaque_lane(tid0);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int w = tid + q * NT, col = w >> LOGN1;
            d[sw_idx<LOGT>((int)row_of_pos((uint32_t)w & (N1 - 1), N1), col)] = r[q];
        }
        __syncthreads();
        const bool more = t + 1 < tend;
        if (more) load_tile(t + 1, tid);
        run_fft<LOGN1, LOGT, NT, true>(d, tw, tid);
        const size_t cbase = (size_t)(t / tiles) * (size_t)(2 * (size_t)M);
        const uint32_t col0 = (t % tiles) << LOGT;
        if (aligned && cbase + 2 * (size_t)M <= n) {  // whole chunk inside the output: no per-element guards
            float2* dst = reinterpret_cast<float2*>(out + cbase) + col0;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
                const float2 v = d[sw_idx<LOGT>(n1, col)];
                dst[(uint32_t)n1 * N2 + col] = make_float2(v.x * scale, v.y * scale);
            }
        } else {
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int w = tid + q * NT, col = w & (TA - 1), n1 = w >> LOGT;
                const float2 v = d[sw_idx<LOGT>(n1, col)];
                store_pair(out, cbase + 2 * ((size_t)n1 * N2 + col0 + col), n, aligned,
                           make_float2(v.x * scale, v.y * scale));
            }
        }
        if (!more) break;
        ++t;
        __syncthreads();
    }
}

// ---------------------------------------------------------------- launch ----
constexpr int kSmallNT = 256;

template <typename K>
hipError_t set_lds(K kernel, size_t bytes)
{
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

template <int LOGM>
hipError_t small_fwd(const float* in, size_t n, size_t C, float2* spec, uint32_t sstride, Tables t, int aligned,
                     hipStream_t s)
{
    constexpr int LOGE = LOGM >= 12 ? LOGM : 12;
    const size_t lds = ((size_t)(1 << LOGE) + (1 << LOGM)) * sizeof(float2);
    auto kern = k_fwd_small<LOGM, LOGE, kSmallNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t per = (size_t)1 << (LOGE - LOGM);
    FFTSP_LAUNCH("rfft_small", kern, dim3((unsigned)((C + per - 1) / per)), dim3(kSmallNT), lds, s, in, n, C, spec, sstride,
                 t, aligned);
    return hipGetLastError();
}

template <int LOGM>
hipError_t small_inv(const float2* spec, uint32_t sstride, size_t n, size_t C, float* out, Tables t, int aligned,
                     hipStream_t s)
{
    constexpr int LOGE = LOGM >= 12 ? LOGM : 12;
    const size_t lds = ((size_t)(1 << LOGE) + (1 << LOGM)) * sizeof(float2);
    auto kern = k_inv_small<LOGM, LOGE, kSmallNT>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t per = (size_t)1 << (LOGE - LOGM);
    FFTSP_LAUNCH("irfft_small", kern, dim3((unsigned)((C + per - 1) / per)), dim3(kSmallNT), lds, s, spec, sstride, n, C,
                 out, t, aligned);
    return hipGetLastError();
}

// persistent grid: at most two workgroups per compute unit, each walking a contiguous run of tiles
struct Grid {
    uint32_t wgs, per_wg;
};
Grid persistent_grid(size_t total, uint32_t kMaxWgs = 512)  // 512 = 256 compute units x 2 resident workgroups
{
    Grid g;
    g.per_wg = (uint32_t)((total + kMaxWgs - 1) / kMaxWgs);
    g.wgs = (uint32_t)((total + g.per_wg - 1) / g.per_wg);
    return g;
}

template <int LOGN1>
hipError_t fwd_a(const float* in, size_t n, int logM, size_t C, float2* mid, Tables t, int aligned, uint32_t* zero_ptr,
                 uint32_t zero_words, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN1)) * sizeof(float2);
    auto kern = k_fwd_a<LOGN1>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN1)) >> (kLogE - LOGN1));
    const Grid g = persistent_grid(total);
    FFTSP_LAUNCH("rfft_pass_a", kern, dim3(g.wgs), dim3(kNT), lds, s, in, n, logM, mid, t, aligned, (uint32_t)total,
                 g.per_wg, zero_ptr, zero_words);
    return hipGetLastError();
}

template <int LOGN2>
hipError_t fwd_b(const float2* mid, int logM, size_t C, float2* spec, uint32_t sstride, Tables t, uint32_t* hist,
                 int pair_spec, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN2)) * sizeof(float2) + kHistLdsWords * sizeof(uint32_t);
    auto kern = k_fwd_b<LOGN2>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN2)) >> (kLogE - LOGN2));
    const Grid g = persistent_grid(total);
    FFTSP_LAUNCH("rfft_pass_b", kern, dim3(g.wgs), dim3(kNT), lds, s, mid, logM, spec, sstride, t, hist,
                 (uint32_t)total, g.per_wg, pair_spec);
    return hipGetLastError();
}

template <int LOGN2>
hipError_t inv_b(const float2* spec, uint32_t sstride, int logM, size_t C, float2* mid, Tables t, int pair_spec,
                 hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN2)) * sizeof(float2);
    auto kern = k_inv_b<LOGN2>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN2)) >> (kLogE - LOGN2));
    const Grid g = persistent_grid(total, 256);  // measured: one workgroup per CU with longer tile runs is faster here
    FFTSP_LAUNCH("irfft_pass_b", kern, dim3(g.wgs), dim3(kNT), lds, s, spec, sstride, logM, mid, t, (uint32_t)total,
                 g.per_wg, pair_spec);
    return hipGetLastError();
}

template <int LOGN1>
hipError_t inv_a(const float2* mid, int logM, size_t C, float* out, size_t n, Tables t, int aligned, hipStream_t s)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN1)) * sizeof(float2);
    auto kern = k_inv_a<LOGN1>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN1)) >> (kLogE - LOGN1));
    const Grid g = persistent_grid(total);
    FFTSP_LAUNCH("irfft_pass_a", kern, dim3(g.wgs), dim3(kNT), lds, s, mid, logM, out, n, t, aligned, (uint32_t)total,
                 g.per_wg);
    return hipGetLastError();
}

}  // namespace

#define FFTSP_SMALL_CASES(X) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13)

// hist (optional, u32[C][kHistBins]): receives the 12-bit histogram of the keys' top bits when the two-pass
// kernels run; they first clear zero_words words at zero_ptr (which must cover hist).  *hist_done = 1 if the
// FFT filled hist, 0 if the caller still has to clear and fill it (single-workgroup sizes).
int fft_pair_log(int logL)
{
    const int logM = logL - 1;
    return logM >= 14 ? (logM + 1) / 2 : 0;
}

hipError_t launch_rfft(const float* in, size_t n, int logL, size_t C, float* spec, uint32_t sstride, float2* mid,
                       Tables t, uint32_t* hist, uint32_t* zero_ptr, size_t zero_words, int* hist_done, int pair_spec,
                       int* pair_log, hipStream_t s)
{
    if (pair_log) *pair_log = 0;
    if (zero_words > 0xffffffffu) return hipErrorInvalidValue;
    if (!hist) zero_words = 0;
    const int logM = logL - 1;
    const int aligned = (reinterpret_cast<uintptr_t>(in) & 7u) == 0;
    float2* sp = reinterpret_cast<float2*>(spec);
    if (hist_done) *hist_done = 0;
    if (C * ((size_t)1 << (logM > 13 ? logM - 13 : 0)) > 0x7fffffffu) return hipErrorInvalidValue;
    switch (logM) {
#define X(p) \
    case p: return small_fwd<p>(in, n, C, sp, sstride, t, aligned, s);
        FFTSP_SMALL_CASES(X)
#undef X
        default: break;
    }
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    switch (logN1) {
        case 7: e = fwd_a<7>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, s); break;
        case 8: e = fwd_a<8>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, s); break;
        case 9: e = fwd_a<9>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, s); break;
        case 10: e = fwd_a<10>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, s); break;
        case 11: e = fwd_a<11>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    if (hist_done) *hist_done = hist != nullptr;
    if (pair_log && pair_spec) *pair_log = logN1;
    switch (logN2) {
        case 7: return fwd_b<7>(mid, logM, C, sp, sstride, t, hist, pair_spec, s);
        case 8: return fwd_b<8>(mid, logM, C, sp, sstride, t, hist, pair_spec, s);
        case 9: return fwd_b<9>(mid, logM, C, sp, sstride, t, hist, pair_spec, s);
        case 10: return fwd_b<10>(mid, logM, C, sp, sstride, t, hist, pair_spec, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_irfft(const float* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out, float2* mid,
                        Tables t, int pair_spec, hipStream_t s)
{
    const int logM = logL - 1;
    const int aligned = (reinterpret_cast<uintptr_t>(out) & 7u) == 0;
    const float2* sp = reinterpret_cast<const float2*>(spec);
    if (C * ((size_t)1 << (logM > 13 ? logM - 13 : 0)) > 0x7fffffffu) return hipErrorInvalidValue;
    switch (logM) {
#define X(p) \
    case p: return small_inv<p>(sp, sstride, n, C, out, t, aligned, s);
        FFTSP_SMALL_CASES(X)
#undef X
        default: break;
    }
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    switch (logN2) {
        case 7: e = inv_b<7>(sp, sstride, logM, C, mid, t, pair_spec, s); break;
        case 8: e = inv_b<8>(sp, sstride, logM, C, mid, t, pair_spec, s); break;
        case 9: e = inv_b<9>(sp, sstride, logM, C, mid, t, pair_spec, s); break;
        case 10: e = inv_b<10>(sp, sstride, logM, C, mid, t, pair_spec, s); break;
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

// Device-side building blocks of the LDS-resident Stockham FFT passes (shared by the per-pass kernels in
// fft.hip and the fused, cache-resident kernels in fused.hip).  Internal: nothing here is part of the C ABI.
#pragma once
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

// 16 points: four radix-4 butterflies over n1 (elements n0, n0+4, n0+8, n0+12), the inner twiddles W16^(n0 k0),
// four radix-4 butterflies over n0; output k = k0 + 4 k1.  One LDS round trip where two radix-4 stages take two.
template <bool INV>
__device__ __forceinline__ void bf16(float2* v)
{
    const float c1 = 0.92387953251128674f, s1 = 0.38268343236508977f, h = 0.70710678118654752440f;
    float2 y[4][4];  // y[n0][k0]
#pragma unroll
    for (int n0 = 0; n0 < 4; ++n0) {
        float2 t[4] = {v[n0], v[n0 + 4], v[n0 + 8], v[n0 + 12]};
        bf4<INV>(t);
#pragma unroll
        for (int k0 = 0; k0 < 4; ++k0) y[n0][k0] = t[k0];
    }
    // W16^m = (cos(m pi/8), -sin(m pi/8)), conjugated for the inverse
    auto rot = [](float2 a, float wr, float wi) {  // a * (wr + i wi) forward, a * (wr - i wi) inverse
        return INV ? make_float2(a.x * wr + a.y * wi, a.y * wr - a.x * wi)
                   : make_float2(a.x * wr - a.y * wi, a.y * wr + a.x * wi);
    };
    y[1][1] = rot(y[1][1], c1, -s1);   // W^1
    y[1][2] = rot(y[1][2], h, -h);     // W^2
    y[1][3] = rot(y[1][3], s1, -c1);   // W^3
    y[2][1] = rot(y[2][1], h, -h);     // W^2
    y[2][2] = rot90<INV>(y[2][2]);     // W^4 = -i
    y[2][3] = rot(y[2][3], -h, -h);    // W^6
    y[3][1] = rot(y[3][1], s1, -c1);   // W^3
    y[3][2] = rot(y[3][2], -h, -h);    // W^6
    y[3][3] = rot(y[3][3], -c1, s1);   // W^9
#pragma unroll
    for (int k0 = 0; k0 < 4; ++k0) {
        float2 t[4] = {y[0][k0], y[1][k0], y[2][k0], y[3][k0]};
        bf4<INV>(t);
#pragma unroll
        for (int k1 = 0; k1 < 4; ++k1) v[k0 + 4 * k1] = t[k1];
    }
}

template <int RL, bool INV>
__device__ __forceinline__ void butterfly(float2* v)
{
    if constexpr (RL == 1) bf2<INV>(v);
    if constexpr (RL == 2) bf4<INV>(v);
    if constexpr (RL == 3) bf8<INV>(v);
    if constexpr (RL == 4) bf16<INV>(v);
}

// log2 of the next stage's radix when `rem` binary stages remain: as few LDS round trips as a lane's sixteen
// points allow (radix 16 where the count is not a multiple of three).
__host__ __device__ constexpr int stage_radix_log(int rem)
{
    return rem <= 4 ? rem : (rem % 3 == 0 ? 3 : (rem == 5 ? 2 : 4));
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
        constexpr int RL = stage_radix_log(LOGR - NS_LOG);
        fft_stage<LOGR, LOGT, NT, INV, NS_LOG, RL>(d, tw, tid);
        run_fft<LOGR, LOGT, NT, INV, NS_LOG + RL>(d, tw, tid);
    }
}

// LDS stages run_fft takes for `rem` remaining levels
constexpr int lds_stages(int rem)
{
    int n = 0;
    while (rem > 0) {
        rem -= stage_radix_log(rem);
        ++n;
    }
    return n;
}

// the same, calling between(k) after LDS stage k (k = 0, 1, ...)
template <int LOGR, int LOGT, int NT, bool INV, int NS_LOG, int K = 0, typename Between>
__device__ __forceinline__ void run_fft_between(float2* d, const float2* tw, int tid, Between between)
{
    if constexpr (NS_LOG < LOGR) {
        constexpr int RL = stage_radix_log(LOGR - NS_LOG);
        fft_stage<LOGR, LOGT, NT, INV, NS_LOG, RL>(d, tw, tid);
        between(K);
        run_fft_between<LOGR, LOGT, NT, INV, NS_LOG + RL, K + 1>(d, tw, tid, between);
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

// Two adjacent slots of one LDS row travel as one 16-byte value: the XOR swizzle keeps an even/odd slot pair
// adjacent (possibly swapped), so a pair is one 128-bit LDS access plus a conditional swap.
__device__ __forceinline__ float2 lo2(float4 v) { return make_float2(v.x, v.y); }
__device__ __forceinline__ float2 hi2(float4 v) { return make_float2(v.z, v.w); }
__device__ __forceinline__ float4 join(float2 a, float2 b) { return make_float4(a.x, a.y, b.x, b.y); }

template <int LOGT>
__device__ __forceinline__ void lds_store2(float2* d, int i, int b2, float4 v)
{
    static_assert(LOGT >= 1, "needs at least two slots per row");
    const int idx = sw_idx<LOGT>(i, b2);  // slot b2 (even); slot b2+1 lives at idx^1
    *reinterpret_cast<float4*>(d + (idx & ~1)) = (idx & 1) ? make_float4(v.z, v.w, v.x, v.y) : v;
}

template <int LOGT>
__device__ __forceinline__ float4 lds_load2(const float2* d, int i, int b2)
{
    static_assert(LOGT >= 1, "needs at least two slots per row");
    const int idx = sw_idx<LOGT>(i, b2);
    const float4 v = *reinterpret_cast<const float4*>(d + (idx & ~1));
    return (idx & 1) ? make_float4(v.z, v.w, v.x, v.y) : v;
}

// Which tile of its chunk work item `tile` is.  Workgroups walk runs of consecutive work items in step, so
// at any moment the chip would touch only every per_wg-th tile position of each chunk: a few fixed byte offsets
// of every row, i.e. a fraction of the memory channels.  Rotating the order by the chunk index spreads the
// offsets in flight over the whole row; the rotation is a multiple of 4, so aligned groups of up to 4 tiles stay together.
// (tiles is a power of two.)
__device__ __forceinline__ uint32_t tile_in_chunk(uint32_t tile, uint32_t tiles)
{
    return (tile + 4 * (tile / tiles)) & (tiles - 1);
}

// Tile run of a pass-A workgroup.  A pass-A tile is 64 bytes of every row it touches, half a 128-byte line;
// tiles 2m and 2m+1 share their lines.  Workgroups are dealt to the 8 XCDs round-robin by index, so workgroups
// b, b+8, ... share an L2: 2^glog of them walk the members of the same run of aligned tile groups in step, and
// each line crosses the fabric once.  The workgroup's tiles are t, t+2^glog, ... < tend.  Returns false if this
// workgroup has nothing to do.
__device__ __forceinline__ bool grouped_run(uint32_t groups, uint32_t per_wg, int glog, uint32_t& t, uint32_t& tend)
{
    const uint32_t b = blockIdx.x, x = b & 7u, y = b >> 3, h = y & ((1u << glog) - 1u);
    const uint32_t rho = ((y >> glog) << 3) + x;  // which group of workgroups
    const uint32_t p0 = rho * per_wg;
    if (p0 >= groups) return false;
    const uint32_t p1 = p0 + per_wg < groups ? p0 + per_wg : groups;
    t = (p0 << glog) + h;
    tend = p1 << glog;
    return true;
}

// rows held by pair kp of a run of N1 paired positions: (kp, N1-kp), and (0, N1/2) for kp = 0
__device__ __forceinline__ uint32_t mirror_row(uint32_t kp, uint32_t N1) { return kp ? N1 - kp : N1 / 2; }

// The first radix-8 stage of an R-point Stockham chain, done in registers: a lane that holds rows j + t*R/8
// (t = 0..7) of two adjacent columns has all inputs of two butterflies, so the stage needs no LDS round trip and
// no barrier of its own.  The outputs go to rows 8j + t, where the next stage (NS = 8) reads them.
template <int LOGT, bool INV>
__device__ __forceinline__ void first_stage_store(float2* d, int j, int col_even, const float4 (&x)[8])
{
    float2 a[8], b[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        a[t] = lo2(x[t]);
        b[t] = hi2(x[t]);
    }
    bf8<INV>(a);
    bf8<INV>(b);
#pragma unroll
    for (int t = 0; t < 8; ++t) lds_store2<LOGT>(d, 8 * j + t, col_even, join(a[t], b[t]));
}

// rank key of a bin: the bit pattern of fl(re*re + fl(im*im)), sign bit masked (see key_of in codec.hip)
__device__ __forceinline__ uint32_t fft_key_of(float2 z)
{
    return __float_as_uint(__fmaf_rn(z.x, z.x, __fmul_rn(z.y, z.y))) & 0x7FFFFFFFu;  // as the codec's key_of
}

}  // namespace
}  // namespace fftsp

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
#include "fft_core.h"
#include <cmath>

namespace fftsp {
namespace {

// The next tile's loads are issued in at most this many portions: one before the LDS stages, one after each of the
// first stages.  A wave that issues a whole tile's loads at once stands in the issue until the memory pipeline has
// taken them; in portions the stages in between proceed meanwhile.
constexpr int kSpreadA = 2;   // forward pass A (measured: 144 us whole, 137-138 in two portions, 138-141 in three)
constexpr int kSpreadFB = 3;  // forward pass B (110-112 us -> 108-109)
constexpr int kSpreadIB = 2;  // inverse pass B (114-116 -> 113)
constexpr int kSpreadIA = 3;  // inverse pass A (117 -> 115-116)
template <int LDS_LEVELS, int MOST>
constexpr int portions()
{
    return lds_stages(LDS_LEVELS) + 1 < MOST ? lds_stages(LDS_LEVELS) + 1 : MOST;
}
template <int LOGN1>
constexpr int spread_parts()
{
    return portions<LOGN1 - 3, kSpreadA>();
}

// Where chunk c's samples live: elements [first, limit) of the gradient; pairs != 0 allows 8-byte accesses.
struct Span {
    size_t first, limit;
    int pairs;
};
template <bool TABLE>
__device__ __forceinline__ Span chunk_span(const TableArg<TABLE>& tab, size_t c, size_t C, size_t chunk_len, size_t n,
                                           int aligned8)
{
    Span sp;
    if constexpr (TABLE) {
        if (c < C) {
            sp.first = tab.t.goff[c];
            sp.limit = sp.first + tab.t.glen[c];
        } else {
            sp.first = sp.limit = 0;
        }
        sp.pairs = aligned8 && !(sp.first & 1u);
    } else {
        sp.first = c * chunk_len;
        sp.limit = n;
        sp.pairs = aligned8;
    }
    return sp;
}

// ------------------------------------------------------------------ small ---
// M = 2^LOGM <= 2^13 complex points per chunk, 2^(LOGE-LOGM) chunks per workgroup.
template <int LOGM, int LOGE, int NT, bool TABLE>
__global__ __launch_bounds__(NT) void k_fwd_small(const float* __restrict__ in, size_t n, size_t C,
                                                  float2* __restrict__ spec, uint32_t sstride, Tables tb, int aligned,
                                                  TableArg<TABLE> tab)
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
        const Span sp = chunk_span<TABLE>(tab, c0 + b, C, 2 * M, n, aligned);
        d[sw_idx<LOGT>(i, b)] = load_pair(in, sp.first + 2 * (size_t)i, sp.limit, sp.pairs);
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

template <int LOGM, int LOGE, int NT, bool TABLE>
__global__ __launch_bounds__(NT) void k_inv_small(const float2* __restrict__ spec, uint32_t sstride, size_t n, size_t C,
                                                  float* __restrict__ out, Tables tb, int aligned, float gain,
                                                  TableArg<TABLE> tab)
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
    const float scale = gain * (1.0f / (float)(2 * M));  // 1/L is a power of two: the product is gain, rescaled exactly
#pragma unroll
    for (int q = 0; q < ELEMS / NT; ++q) {
        const int w = tid + q * NT, i = w & (M - 1), b = w >> LOGM;
        const Span sp = chunk_span<TABLE>(tab, c0 + b, C, 2 * M, n, aligned);
        float2 v = d[sw_idx<LOGT>(i, b)];
        store_pair(out, sp.first + 2 * (size_t)i, sp.limit, sp.pairs, make_float2(v.x * scale, v.y * scale));
    }
}

// Software pipeline of the persistent two-pass kernels.  Vector-memory results return in issue order and are
// counted by a single counter, so the order of issue decides what a wait really waits for.  Per tile t:
//     [table lookups for tile t's store loop, lookups for tile t+1's split, loads of tile t+1]   one batch
//     LDS FFT of tile t
//     store loop of tile t
//     barrier, LDS fill from the registers that hold tile t+1, barrier
// Every load is older than the stores issued after it, so no wait for a load ever waits for a store to be
// acknowledged.  The loads of the batch are unconditional (on the last tile they read one valid dummy address),
// which keeps the code between issue and use free of branches that would make the waits conservative.

// Column-to-column ratios of pass A's twiddles W_M^(n2 k1) for the row pairs a lane stores: they depend on the lane
// alone, so a workgroup looks them up once for all its tiles.
template <int LOGN1>
struct PassARatios {
    static constexpr int HP = (1 << LOGN1) / 2;
    static constexpr int KN = HP >= kNT ? HP / kNT : 1;
    float2 a[KN], b[KN];
};
template <int LOGN1>
__device__ __forceinline__ PassARatios<LOGN1> pass_a_ratios(const Tables& tb, int logM, int tid)
{
    constexpr int N1 = 1 << LOGN1, HP = N1 / 2, KN = PassARatios<LOGN1>::KN;
    constexpr int DC = HP >= kNT ? 1 : kNT / HP;
    PassARatios<LOGN1> r;
#pragma unroll
    for (int kk = 0; kk < KN; ++kk) {
        const uint32_t kp = (uint32_t)(tid + kk * kNT) & (HP - 1);
        r.a[kk] = twiddle(tb, ((uint32_t)DC * kp) << (22 - logM));
        r.b[kk] = twiddle(tb, ((uint32_t)DC * mirror_row(kp, N1)) << (22 - logM));
    }
    return r;
}

// One tile of pass A once its first stage is in LDS: the twiddle look-ups of the store loop, `prefetch()` (loads of
// a later tile, issued here so that they are older than this tile's stores), the LDS stages, and the store loop,
// which multiplies by W_M^(n2 k1) and writes row k1 next to row N1 - k1.
template <int LOGN1, bool HALF, typename Prefetch>
__device__ __forceinline__ void fwd_a_tile(uint32_t t, uint32_t tiles, int logM, typename Cx<HALF>::One* __restrict__ mid,
                                           const Tables& tb, float2* d, const float2* tw, int tid, float in_scale,
                                           const PassARatios<LOGN1>& ratio, Prefetch prefetch)
{
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1;
    constexpr int HP = N1 / 2, LOGHP = LOGN1 - 1;  // row pairs per column
    constexpr int KN = HP >= NT ? HP / NT : 1;   // distinct row pairs per lane in the store loop
    constexpr int DC = HP >= NT ? 1 : NT / HP;   // column step between a lane's consecutive stores
    constexpr int NCOL = PER2 / KN;
    static_assert(NCOL <= 8, "twiddle recurrence is anchored once");
    const uint32_t M = 1u << logM;
    const uint32_t col0 = tile_in_chunk(t, tiles) << LOGT;
    const int sh = 22 - logM;
    float2 cur_a[KN], cur_b[KN];
#pragma unroll
    for (int kk = 0; kk < KN; ++kk) {
        const uint32_t kp = (uint32_t)(tid + kk * NT) & (HP - 1);
        const uint32_t ka = kp, kb = mirror_row(kp, N1);
        const uint32_t cfirst = (uint32_t)(tid + kk * NT) >> LOGHP;
        cur_a[kk] = twiddle(tb, ((col0 + cfirst) * ka) << sh);
        cur_b[kk] = twiddle(tb, ((col0 + cfirst) * kb) << sh);
        if constexpr (HALF) {  // the variant's power-of-two factors ride on the twiddles (exact)
            cur_a[kk] = make_float2(cur_a[kk].x * in_scale, cur_a[kk].y * in_scale);
            cur_b[kk] = make_float2(cur_b[kk].x * in_scale, cur_b[kk].y * in_scale);
        }
    }
    // the next tile's loads go out in kSpreadA portions: one before the LDS stages, one after each of the first stages
    prefetch(0);
    run_fft_between<LOGN1, LOGT, NT, false, 3>(d, tw, tid, [&](int k) {
        if (k + 1 < spread_parts<LOGN1>()) prefetch(k + 1);
    });
    typename Cx<HALF>::Two* out = reinterpret_cast<typename Cx<HALF>::Two*>(mid + (size_t)(t / tiles) * (size_t)M);
#pragma unroll
    for (int kk = 0; kk < KN; ++kk) {
        const uint32_t kp = (uint32_t)(tid + kk * NT) & (HP - 1);  // pair of paired positions (2kp, 2kp+1)
        const uint32_t ka = kp, kb = mirror_row(kp, N1);
        const uint32_t cfirst = (uint32_t)(tid + kk * NT) >> LOGHP;
#pragma unroll
        for (int j = 0; j < NCOL; ++j) {
            const uint32_t col = cfirst + j * DC, n2 = col0 + col;
            const float2 va = cmul(d[sw_idx<LOGT>((int)ka, (int)col)], cur_a[kk]);
            const float2 vb = cmul(d[sw_idx<LOGT>((int)kb, (int)col)], cur_b[kk]);
            out[n2 * (uint32_t)HP + kp] = cx_store<HALF>(join(va, vb));
            cur_a[kk] = cmul(cur_a[kk], ratio.a[kk]);
            cur_b[kk] = cmul(cur_b[kk], ratio.b[kk]);
        }
    }
}

// Forward pass A: N1-point FFTs down the columns of the N1 x N2 view of z, for tiles of TA adjacent columns.
// FAST: every tile of this workgroup's run lies in a chunk that is wholly inside the input, and the input is
// 16-byte aligned: two columns per 16-byte load, no guards.  Otherwise every element is loaded under a guard
// (ragged last chunk, unaligned tensors); the two variants are separate loops so that the guarded one does
// not put branches between the fast one's loads and their use.
template <int LOGN1, bool FAST, bool TABLE, bool HALF>
__device__ __forceinline__ void fwd_a_run(const float* __restrict__ in, size_t n, int logM,
                                          typename Cx<HALF>::One* __restrict__ mid, const Tables& tb, int aligned,
                                          uint32_t t, uint32_t tend, uint32_t tstep, float2* d, const float2* tw, int tid0,
                                          const TableArg<TABLE>& tab, float in_scale)
{
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1, TA = 1 << LOGT;
    static_assert(LOGT >= 2 && (NT % (TA / 2)) == 0, "tile shape");
    const uint32_t M = 1u << logM, N2 = M >> LOGN1, tiles = N2 >> LOGT;

    // live = false: the tile does not exist; the fast loads are still issued, all to one valid address
    // part p of spread_parts(): loads q with q * parts / PER2 == p; prologue calls pass every part in turn
    auto load_tile = [&](float4 (&r)[PER2], uint32_t tile, int tid, bool live, int part) {
        // every tile lies in a real chunk, so the span needs no chunk count
        const Span sp = chunk_span<TABLE>(tab, tile / tiles, ~(size_t)0, 2 * (size_t)M, n, aligned & 1);
        const uint32_t col0 = tile_in_chunk(tile, tiles) << LOGT;
        if constexpr (FAST) {
            const float4* src = live ? reinterpret_cast<const float4*>(in + sp.first) + (col0 >> 1)
                                     : reinterpret_cast<const float4*>(tb.hi);
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                if (q * spread_parts<LOGN1>() / PER2 != part) continue;
                const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGT - 1);
                r[q] = src[live ? (uint32_t)n1 * (N2 >> 1) + bp : 0u];
            }
        } else {
            if (!live || part != 0) return;
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGT - 1);
                const size_t gi = sp.first + 2 * ((size_t)n1 * N2 + col0 + 2 * bp);
                r[q] = join(load_pair(in, gi, sp.limit, sp.pairs), load_pair(in, gi + 2, sp.limit, sp.pairs));
            }
        }
    };
    // r[q] holds rows (tid >> (LOGT-1)) + q * N1/8 of one column pair: the first stage runs on the way into LDS
    static_assert(PER2 == 8 && (NT >> (LOGT - 1)) == N1 / 8, "a lane's loads are the inputs of two radix-8 butterflies");
    auto fill = [&](const float4 (&r)[PER2], int tid) {
        first_stage_store<LOGT, false>(d, tid >> (LOGT - 1), 2 * (tid & (TA / 2 - 1)), r);
    };
    float4 r[PER2];
#pragma unroll
    for (int part = 0; part < spread_parts<LOGN1>(); ++part) load_tile(r, t, tid0, true, part);
    const PassARatios<LOGN1> ratio = pass_a_ratios<LOGN1>(tb, logM, tid0);
    fill(r, tid0);
    __syncthreads();
    for (;;) {
        const int tid = opaque_lane(tid0);
        const bool more = t + tstep < tend;
        fwd_a_tile<LOGN1, HALF>(t, tiles, logM, mid, tb, d, tw, tid, in_scale, ratio,
                                [&](int part) { load_tile(r, more ? t + tstep : t, tid, more, part); });
        if (!more) break;
        t += tstep;
        __syncthreads();
        fill(r, tid);
        __syncthreads();
    }
}

// `aligned`: bit 0 = input is 8-byte aligned, bit 1 = 16-byte aligned.
template <int LOGN1, bool TABLE, bool HALF>
__global__ __launch_bounds__(kNT) void k_fwd_a(const float* __restrict__ in, size_t n, int logM,
                                               typename Cx<HALF>::One* __restrict__ mid, Tables tb, int aligned,
                                               uint32_t total, uint32_t per_wg, int glog, uint32_t* __restrict__ zero_ptr,
                                               uint32_t zero_words, TableArg<TABLE> tab, float in_scale,
                                               const uint32_t* __restrict__ only_if)
{
    constexpr int NT = kNT, ELEMS = 1 << kLogE;
    if (only_if && *only_if == 0u) return;  // stand-by launch behind a fused kernel that did finish
    // clears the status words and key histograms the next kernels of the sender accumulate into
    for (uint32_t i = blockIdx.x * NT + threadIdx.x; i < zero_words; i += gridDim.x * NT) zero_ptr[i] = 0u;
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid0 = threadIdx.x;
    uint32_t t, tend;
    if (!grouped_run(total, per_wg, glog, t, tend)) return;
    load_stage_twiddles<LOGN1, NT>(tw, tb, tid0);
    const uint32_t tiles = (1u << logM) >> kLogE;  // tiles per chunk
    bool fast = (aligned & 2) != 0;
    if constexpr (TABLE) {
        // every tensor this run touches fills its chunk and starts on a 16-byte boundary
        for (uint32_t c = t / tiles; c <= (tend - 1) / tiles; ++c)
            fast = fast && (tab.t.goff[c] & 3u) == 0 && tab.t.glen[c] == (2u << logM);
    } else {
        const size_t last_chunk_end = ((size_t)((tend - 1) / tiles) + 1) << (logM + 1);
        fast = fast && last_chunk_end <= n;
    }
    if (fast)
        fwd_a_run<LOGN1, true, TABLE, HALF>(in, n, logM, mid, tb, aligned, t, tend, 1u << glog, d, tw, tid0, tab,
                                            in_scale);
    else
        fwd_a_run<LOGN1, false, TABLE, HALF>(in, n, logM, mid, tb, aligned, t, tend, 1u << glog, d, tw, tid0, tab,
                                             in_scale);
}


// Forward pass B: N2-point FFTs along n2 for a tile of rows and their mirrors, then the real-FFT split.
// A lane owns one pair of slots (row ka and its mirror kb), i.e. 16 bytes of every run it touches.
// CODEC: the spectrum is stored in the paired order and the first radix-select digit of every bin's key is
// counted into the 12-bit histogram of the chunk (hist); otherwise natural bin order and no histogram.
// The store loop is free of branches (partner addresses and the rare self-mirrored rows are handled with
// selects) so that its LDS reads can be issued ahead in batches instead of one wait per read.
// HALF (CODEC only): the intermediate is read and the spectrum written as binary16 pairs; the histogram counts
// the keys of the values as stored, which are the ones the selection will see.
template <int LOGN2, bool CODEC, bool HALF>
__global__ __launch_bounds__(kNT) void k_fwd_b(const typename Cx<HALF>::One* __restrict__ mid, int logM,
                                               typename Cx<HALF>::One* __restrict__ spec, uint32_t sstride, Tables tb,
                                               uint32_t* __restrict__ hist, uint32_t total, uint32_t per_wg,
                                               float mid_scale, const uint32_t* __restrict__ only_if)
{
    static_assert(CODEC || !HALF, "binary16 storage is the codec's own");
    if (only_if && *only_if == 0u) return;  // stand-by launch behind a fused kernel that did finish
    using Two = typename Cx<HALF>::Two;
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int N2 = 1 << LOGN2, LOGT = LOGE - LOGN2, ELEMS = 1 << LOGE;
    constexpr int LOGP = LOGT - 1, P = 1 << LOGP;  // slot pairs per tile
    static_assert(LOGT >= 1 && NT % P == 0, "a lane keeps one slot pair");
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    uint32_t* h16 = reinterpret_cast<uint32_t*>(tw + N2);
    const int tid0 = threadIdx.x;
    const int logN1 = logM - LOGN2;
    const uint32_t M = 1u << logM, N1 = 1u << logN1, tiles = N1 >> LOGT;
    // runs differ by at most one tile: the first total - per_wg * gridDim.x workgroups take one more
    const uint32_t extra = total - per_wg * gridDim.x;
    uint32_t t = blockIdx.x * per_wg + (blockIdx.x < extra ? blockIdx.x : extra);
    const uint32_t tend = t + per_wg + (blockIdx.x < extra ? 1u : 0u);
    if (t >= tend) return;
    load_stage_twiddles<LOGN2, NT>(tw, tb, tid0);
    if (CODEC)
        for (int i = tid0; i < kHistLdsWords; i += NT) h16[i] = 0u;
    constexpr int DK = NT >> LOGP;  // k2 step between a lane's consecutive pairs
    static_assert(2 * kSplitStep * (PER2 - 1) < 16, "split twiddle steps stay inside the 32nd-root table");
    // the LDS histogram has 16-bit counters and a tile adds at most 2^13 + 1 keys: flush after at most 7 tiles
    constexpr uint32_t kFlushEvery = 7;
    constexpr int BATCH = 4;  // pairs whose LDS reads are issued together
    static_assert(PER2 % BATCH == 0, "batches divide the store loop");

    Two r[PER2];
    constexpr int PARTS = portions<LOGN2 - 3, kSpreadFB>();
    // part < 0: the whole tile; otherwise the loads q with q * PARTS / PER2 == part
    auto load_tile = [&](uint32_t tile, int tid, bool live, int part = -1) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const Two* src = reinterpret_cast<const Two*>(mid + (live ? (size_t)(tile / tiles) * (size_t)M : 0));
        const uint32_t pp = tile_in_chunk(tile, tiles) * P + p;
#pragma unroll
        for (int q = 0; q < PER2; ++q)
            if (part < 0 || q * PARTS / PER2 == part) r[q] = src[live ? (uint32_t)(kq0 + q * DK) * (N1 >> 1) + pp : 0u];
    };
    // r[q] holds rows kq0 + q * N2/8 of one slot pair: the first radix-8 stage runs on the way into LDS
    static_assert(PER2 == 8 && DK == N2 / 8, "a lane's loads are the inputs of two radix-8 butterflies");
    auto fill = [&](int tid) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        float4 v[PER2];
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            v[q] = cx_load(r[q]);
            if constexpr (HALF)  // undo the factor that kept the intermediate inside binary16's range
                v[q] = make_float4(v[q].x * mid_scale, v[q].y * mid_scale, v[q].z * mid_scale, v[q].w * mid_scale);
        }
        first_stage_store<LOGT, false>(d, kq0, 2 * p, v);
    };
    // one key into the 16-bit LDS histogram (bucket b: word b/2, half b%2); on = false adds nothing
    auto count = [&](float2 x, bool on) {
        const uint32_t b = fft_key_of(x) >> kKeyShift;
        atomicAdd(&h16[b >> 1], on ? 1u << ((b & 1u) * 16u) : 0u);
    };
    load_tile(t, tid0, true);
    fill(tid0);
    __syncthreads();
    uint32_t unflushed = 0;
    for (;;) {
        const int tid = opaque_lane(tid0);
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const uint32_t pp = tile_in_chunk(t, tiles) * P + p;
        const uint32_t ka = pp, kb = mirror_row(pp, N1);
        const bool self = pp == 0;  // rows 0 and N1/2 are their own mirrors
        // W_L^(k1 + N1*k2): k2 advances by DK per step, i.e. by exactly 2*kSplitStep 32nds of a turn
        const float2 base_a = twiddle(tb, (ka + ((uint32_t)kq0 << logN1)) << (21 - logM));
        const float2 base_b = twiddle(tb, (kb + ((uint32_t)kq0 << logN1)) << (21 - logM));
        const bool more = t + 1 < tend;
        load_tile(more ? t + 1 : t, tid, more, 0);
        run_fft_between<LOGN2, LOGT, NT, false, 3>(d, tw, tid, [&](int k) {
            if (k + 1 < PARTS) load_tile(more ? t + 1 : t, tid, more, k + 1);
        });
        const size_t c = t / tiles;
        typename Cx<HALF>::One* out = spec + c * (size_t)sstride;
#pragma unroll
        for (int q0 = 0; q0 < PER2; q0 += BATCH) {
            float2 a0[BATCH], a1[BATCH], pa[BATCH], pb[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int k2 = kq0 + (q0 + u) * DK, k2p = N2 - 1 - k2;
                // X[ka, k2] pairs with Z[kb, N2-1-k2] and X[kb, k2] with Z[ka, N2-1-k2]; row 0 pairs with itself
                // at (N2-k2) mod N2 and row N1/2 with itself at N2-1-k2
                const int ia = self ? sw_idx<LOGT>((N2 - k2) & (N2 - 1), 2 * p) : sw_idx<LOGT>(k2p, 2 * p + 1);
                const int ib = self ? sw_idx<LOGT>(k2p, 2 * p + 1) : sw_idx<LOGT>(k2p, 2 * p);
                a0[u] = d[sw_idx<LOGT>(k2, 2 * p)];
                a1[u] = d[sw_idx<LOGT>(k2, 2 * p + 1)];
                pa[u] = d[ia];
                pb[u] = d[ib];
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int q = q0 + u, k2 = kq0 + q * DK;
                const float2 wq = make_float2(kW32re[2 * q * kSplitStep], kW32im[2 * q * kSplitStep]);
                float2 xa = split_fwd(a0[u], pa[u], cmul(base_a, wq));
                const float2 xb = split_fwd(a1[u], pb[u], cmul(base_b, wq));
                if (q == 0) {  // k2 = 0 only here: bin 0 and the Nyquist bin come from Z[0] alone
                    const bool dc = self && kq0 == 0;
                    const typename Cx<HALF>::One xm_st = cx_store<HALF>(make_float2(a0[u].x - a0[u].y, 0.f));
                    if (dc) {
                        xa = make_float2(a0[u].x + a0[u].y, 0.f);
                        out[M] = xm_st;
                    }
                    if (CODEC) count(cx_load(xm_st), dc);
                }
                if constexpr (CODEC) {
                    const Two st = cx_store<HALF>(join(xa, xb));
                    reinterpret_cast<Two*>(out)[((uint32_t)k2 << (logN1 - 1)) + pp] = st;
                    const float4 seen = cx_load(st);  // what the selection will read back
                    count(lo2(seen), true);
                    count(hi2(seen), true);
                } else {
                    out[ka + ((uint32_t)k2 << logN1)] = xa;
                    out[kb + ((uint32_t)k2 << logN1)] = xb;
                }
            }
        }
        ++unflushed;
        if (CODEC && (!more || unflushed == kFlushEvery || (t + 1) / tiles != c)) {
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
            unflushed = 0;
        }
        if (!more) break;
        ++t;
        __syncthreads();
        fill(tid);
        __syncthreads();
    }
}

// Inverse pass B: undo the split, inverse N2-point FFTs over k2, times conj W_M^(n2 k1).
// PAIR: the spectrum is read in the paired order (the codec's own buffer), otherwise in natural bin order.
// HALF (PAIR only): spectrum and intermediate are binary16 pairs.
template <int LOGN2, bool PAIR, bool HALF>
__global__ __launch_bounds__(kNT) void k_inv_b(const typename Cx<HALF>::One* __restrict__ spec, uint32_t sstride, int logM,
                                               typename Cx<HALF>::One* __restrict__ mid, Tables tb, uint32_t total,
                                               uint32_t per_wg, float mid_scale, const uint32_t* __restrict__ only_if)
{
    static_assert(PAIR || !HALF, "binary16 storage is the codec's own");
    if (only_if && *only_if == 0u) return;  // stand-by launch behind a fused kernel that did finish
    using One = typename Cx<HALF>::One;
    using Two = typename Cx<HALF>::Two;
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int N2 = 1 << LOGN2, LOGT = LOGE - LOGN2, ELEMS = 1 << LOGE;
    constexpr int LOGP = LOGT - 1, P = 1 << LOGP;
    static_assert(LOGT >= 1 && NT % P == 0, "a lane keeps one slot pair");
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid0 = threadIdx.x;
    const int logN1 = logM - LOGN2;
    const uint32_t M = 1u << logM, N1 = 1u << logN1, tiles = N1 >> LOGT;
    // runs differ by at most one tile: the first total - per_wg * gridDim.x workgroups take one more
    const uint32_t extra = total - per_wg * gridDim.x;
    uint32_t t = blockIdx.x * per_wg + (blockIdx.x < extra ? blockIdx.x : extra);
    const uint32_t tend = t + per_wg + (blockIdx.x < extra ? 1u : 0u);
    if (t >= tend) return;
    load_stage_twiddles<LOGN2, NT>(tw, tb, tid0);
    constexpr int DK = NT >> LOGP;
    static_assert(PER2 <= 8, "twiddle recurrence is anchored once");

    Two r[PER2];
    One xnyq;                // Nyquist bin of the chunk of the tile held in r
    float2 base_a, base_b;   // split twiddles of that tile
    constexpr int PARTS = portions<LOGN2 - 3, kSpreadIB>();
    // part < 0: the whole tile; otherwise the loads q with q * PARTS / PER2 == part (the look-ups go with part 0)
    auto load_tile = [&](uint32_t tile, int tid, bool live, int part = -1) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const One* X = spec + (live ? (size_t)(tile / tiles) * (size_t)sstride : 0);
        const uint32_t pp = tile_in_chunk(tile, tiles) * P + p;
        const uint32_t ka = pp, kb = mirror_row(pp, N1);
        if (part <= 0) {
            base_a = twiddle(tb, (ka + ((uint32_t)kq0 << logN1)) << (21 - logM));
            base_b = twiddle(tb, (kb + ((uint32_t)kq0 << logN1)) << (21 - logM));
        }
        if constexpr (PAIR) {
            const Two* X4 = reinterpret_cast<const Two*>(X);
#pragma unroll
            for (int q = 0; q < PER2; ++q)
                if (part < 0 || q * PARTS / PER2 == part) r[q] = X4[live ? ((uint32_t)(kq0 + q * DK) << (logN1 - 1)) + pp : 0u];
        } else {
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                if (!(part < 0 || q * PARTS / PER2 == part)) continue;
                const uint32_t o = (uint32_t)(kq0 + q * DK) << logN1;
                r[q] = join(X[live ? ka + o : 0u], X[live ? kb + o : 0u]);
            }
        }
        if (part <= 0) xnyq = X[live ? M : 0u];
    };
    auto fill = [&](int tid) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
#pragma unroll
        for (int q = 0; q < PER2; ++q) lds_store2<LOGT>(d, kq0 + q * DK, 2 * p, cx_load(r[q]));
    };
    load_tile(t, tid0, true);
    fill(tid0);
    __syncthreads();
    for (;;) {
        const int tid = opaque_lane(tid0);
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const uint32_t pp = tile_in_chunk(t, tiles) * P + p;
        const uint32_t ka = pp, kb = mirror_row(pp, N1);
        const bool self = pp == 0;
        // partners of all pairs first (one batch of LDS reads), then the arithmetic: no branches in between
        float2 pa[PER2], pb[PER2];
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            const int k2 = kq0 + q * DK, k2p = N2 - 1 - k2;
            const int ia = self ? sw_idx<LOGT>((N2 - k2) & (N2 - 1), 2 * p) : sw_idx<LOGT>(k2p, 2 * p + 1);
            const int ib = self ? sw_idx<LOGT>(k2p, 2 * p + 1) : sw_idx<LOGT>(k2p, 2 * p);
            pa[q] = d[ia];
            pb[q] = d[ib];
        }
        float4 z[PER2];
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            const float2 wq = make_float2(kW32re[2 * q * kSplitStep], kW32im[2 * q * kSplitStep]);
            const float4 rq = cx_load(r[q]);
            float2 a0 = lo2(rq), b0 = pa[q];
            if (q == 0) {  // k2 = 0 only here; imaginary parts of the DC and Nyquist bins are ignored
                const bool dc = self && kq0 == 0;
                b0 = dc ? make_float2(cx_load(xnyq).x, 0.f) : b0;
                a0.y = dc ? 0.f : a0.y;
            }
            z[q] = join(split_inv(a0, b0, cmul(base_a, wq)), split_inv(hi2(rq), pb[q], cmul(base_b, wq)));
        }
        __syncthreads();
        // z[q] are rows kq0 + q * N2/8 of this lane's slot pair: the first inverse radix-8 stage runs here
        static_assert(PER2 == 8 && DK == N2 / 8, "a lane's values are the inputs of two radix-8 butterflies");
        first_stage_store<LOGT, true>(d, kq0, 2 * p, z);
        __syncthreads();
        // store-loop twiddles of this tile, then split twiddles and data of the next one
        const int sh = 22 - logM;
        const float2 ratio_a = twiddle(tb, ((uint32_t)DK * ka) << sh);
        const float2 ratio_b = twiddle(tb, ((uint32_t)DK * kb) << sh);
        float2 cur_a = twiddle(tb, ((uint32_t)kq0 * ka) << sh);
        float2 cur_b = twiddle(tb, ((uint32_t)kq0 * kb) << sh);
        if constexpr (HALF) {  // keeps the unnormalised partial sums inside binary16's range (exact power of two)
            cur_a = make_float2(cur_a.x * mid_scale, cur_a.y * mid_scale);
            cur_b = make_float2(cur_b.x * mid_scale, cur_b.y * mid_scale);
        }
        const bool more = t + 1 < tend;
        load_tile(more ? t + 1 : t, tid, more, 0);
        run_fft_between<LOGN2, LOGT, NT, true, 3>(d, tw, tid, [&](int k) {
            if (k + 1 < PARTS) load_tile(more ? t + 1 : t, tid, more, k + 1);
        });
        Two* dst = reinterpret_cast<Two*>(mid + (size_t)(t / tiles) * (size_t)M);
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            const uint32_t n2 = (uint32_t)(kq0 + q * DK);
            const float4 v = lds_load2<LOGT>(d, (int)n2, 2 * p);
            dst[n2 * (N1 >> 1) + pp] = cx_store<HALF>(join(cmulc(lo2(v), cur_a), cmulc(hi2(v), cur_b)));
            cur_a = cmul(cur_a, ratio_a);
            cur_b = cmul(cur_b, ratio_b);
        }
        if (!more) break;
        ++t;
        __syncthreads();
        fill(tid);
        __syncthreads();
    }
}

// Inverse pass A: inverse N1-point FFTs over k1 for a tile of columns n2; writes the real samples.
// `aligned`: bit 0 = output is 8-byte aligned, bit 1 = 16-byte aligned.
template <int LOGN1, bool TABLE, bool HALF>
__global__ __launch_bounds__(kNT) void k_inv_a(const typename Cx<HALF>::One* __restrict__ mid, int logM,
                                               float* __restrict__ out, size_t n, Tables tb, int aligned, uint32_t total,
                                               uint32_t per_wg, int glog, float gain, TableArg<TABLE> tab,
                                               const uint32_t* __restrict__ only_if)
{
    using Two = typename Cx<HALF>::Two;
    if (only_if && *only_if == 0u) return;  // stand-by launch behind a fused kernel that did finish
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int N1 = 1 << LOGN1, LOGT = LOGE - LOGN1, TA = 1 << LOGT, ELEMS = 1 << LOGE;
    constexpr int HP = N1 / 2, LOGHP = LOGN1 - 1;
    static_assert(LOGT >= 2 && (NT % (TA / 2)) == 0, "tile shape");
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + ELEMS;
    const int tid0 = threadIdx.x;
    const uint32_t M = 1u << logM, N2 = M >> LOGN1, tiles = N2 >> LOGT;
    uint32_t t, tend;
    if (!grouped_run(total, per_wg, glog, t, tend)) return;
    const uint32_t tstep = 1u << glog;
    load_stage_twiddles<LOGN1, NT>(tw, tb, tid0);

    Two r[PER2];
    constexpr int PARTS = portions<LOGN1, kSpreadIA>();
    // part < 0: the whole tile; otherwise the loads q with q * PARTS / PER2 == part
    auto load_tile = [&](uint32_t tile, int tid, bool live, int part = -1) {
        const Two* src = reinterpret_cast<const Two*>(mid + (live ? (size_t)(tile / tiles) * (size_t)M : 0));
        const uint32_t col0 = tile_in_chunk(tile, tiles) << LOGT;
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            if (!(part < 0 || q * PARTS / PER2 == part)) continue;
            const int w = tid + q * NT, kp = w & (HP - 1), col = w >> LOGHP;
            r[q] = src[live ? (uint32_t)(col0 + col) * HP + kp : 0u];
        }
    };
    auto fill = [&](int tid) {
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            const int w = tid + q * NT, kp = w & (HP - 1), col = w >> LOGHP;
            const float4 rq = cx_load(r[q]);
            d[sw_idx<LOGT>(kp, col)] = lo2(rq);
            d[sw_idx<LOGT>((int)mirror_row((uint32_t)kp, N1), col)] = hi2(rq);
        }
    };
    load_tile(t, tid0, true);
    fill(tid0);
    __syncthreads();
    const float scale = gain * (1.0f / (float)(2u * M));
    for (;;) {
        const int tid = opaque_lane(tid0);
        const bool more = t + tstep < tend;
        load_tile(more ? t + tstep : t, tid, more, 0);
        run_fft_between<LOGN1, LOGT, NT, true, 0>(d, tw, tid, [&](int k) {
            if (k + 1 < PARTS) load_tile(more ? t + tstep : t, tid, more, k + 1);
        });
        const Span sp = chunk_span<TABLE>(tab, t / tiles, ~(size_t)0, 2 * (size_t)M, n, aligned & 1);
        const size_t cbase = sp.first;
        const uint32_t col0 = tile_in_chunk(t, tiles) << LOGT;
        // whole chunk inside the output (per-tensor: the tensor fills its chunk, 16-byte aligned): no guards
        if ((aligned & 2) && cbase + 2 * (size_t)M <= sp.limit && (!TABLE || (cbase & 3u) == 0)) {
            float4* dst = reinterpret_cast<float4*>(out + cbase) + (col0 >> 1);
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGT - 1);
                const float4 v = lds_load2<LOGT>(d, n1, 2 * bp);
                dst[(uint32_t)n1 * (N2 >> 1) + bp] = make_float4(v.x * scale, v.y * scale, v.z * scale, v.w * scale);
            }
        } else {
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGT - 1);
                const float4 v = lds_load2<LOGT>(d, n1, 2 * bp);
                const size_t gi = cbase + 2 * ((size_t)n1 * N2 + col0 + 2 * bp);
                store_pair(out, gi, sp.limit, sp.pairs, make_float2(v.x * scale, v.y * scale));
                store_pair(out, gi + 2, sp.limit, sp.pairs, make_float2(v.z * scale, v.w * scale));
            }
        }
        if (!more) break;
        t += tstep;
        __syncthreads();
        fill(tid);
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

template <int LOGM, bool TABLE>
hipError_t small_fwd(const float* in, size_t n, size_t C, float2* spec, uint32_t sstride, Tables t, int aligned,
                     const ChunkTable* tab, hipStream_t s)
{
    constexpr int LOGE = LOGM >= 12 ? LOGM : 12;
    const size_t lds = ((size_t)(1 << LOGE) + (1 << LOGM)) * sizeof(float2);
    auto kern = k_fwd_small<LOGM, LOGE, kSmallNT, TABLE>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t per = (size_t)1 << (LOGE - LOGM);
    FFTSP_LAUNCH("rfft_small", kern, dim3((unsigned)((C + per - 1) / per)), dim3(kSmallNT), lds, s, in, n, C, spec, sstride,
                 t, aligned, table_arg<TABLE>(tab));
    return hipGetLastError();
}

template <int LOGM, bool TABLE>
hipError_t small_inv(const float2* spec, uint32_t sstride, size_t n, size_t C, float* out, Tables t, int aligned,
                     float gain, const ChunkTable* tab, hipStream_t s)
{
    constexpr int LOGE = LOGM >= 12 ? LOGM : 12;
    const size_t lds = ((size_t)(1 << LOGE) + (1 << LOGM)) * sizeof(float2);
    auto kern = k_inv_small<LOGM, LOGE, kSmallNT, TABLE>;
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t per = (size_t)1 << (LOGE - LOGM);
    FFTSP_LAUNCH("irfft_small", kern, dim3((unsigned)((C + per - 1) / per)), dim3(kSmallNT), lds, s, spec, sstride, n, C,
                 out, t, aligned, gain, table_arg<TABLE>(tab));
    return hipGetLastError();
}

// persistent grid: workgroups walk contiguous runs of tiles; two of them are resident per compute unit (512 on
// the chip), and a kernel may ask for a few rounds of that when shorter runs balance better
struct Grid {
    uint32_t wgs, per_wg;
};
// Every workgroup takes per_wg tiles and the first total - per_wg * wgs of them one more.  With 512 workgroups
// (256 compute units x 2 resident) the two workgroups of a compute unit are b and b + 256, so the longer runs pair
// up with the shorter ones and every compute unit gets the same number of tiles.
Grid persistent_grid(size_t total, uint32_t kMaxWgs = 512)
{
    Grid g;
    g.wgs = (uint32_t)(total < kMaxWgs ? total : kMaxWgs);
    g.per_wg = (uint32_t)(total / g.wgs);
    return g;
}

// pass A: 2^glog workgroups (b, b+8, ...) share a run of aligned tile groups; per_wg counts tile groups and wgs
// is a multiple of 8 * 2^glog
constexpr int kGroupLog = 1;
constexpr uint32_t kPassAWgs = 2048;  // most workgroups the forward pass A is cut into
Grid grouped_grid(size_t groups, int glog, uint32_t kMaxWgs = 512)
{
    Grid g;
    const uint32_t wg_groups = kMaxWgs >> glog;
    g.per_wg = (uint32_t)((groups + wg_groups - 1) / wg_groups);
    const uint32_t used = (uint32_t)((groups + g.per_wg - 1) / g.per_wg);
    const uint32_t unit = 8u << glog;
    g.wgs = (((used << glog) + unit - 1) / unit) * unit;
    return g;
}

// HALF launchers take the same buffer pointers; the kernels read them as binary16 pairs
template <int LOGN1, bool TABLE, bool HALF>
hipError_t fwd_a(const float* in, size_t n, int logM, size_t C, float2* mid_f32, Tables t, int aligned,
                 uint32_t* zero_ptr, uint32_t zero_words, const ChunkTable* tab, float in_scale, hipStream_t s,
                 const uint32_t* only_if = nullptr)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN1)) * sizeof(float2);
    auto kern = k_fwd_a<LOGN1, TABLE, HALF>;
    auto* mid = reinterpret_cast<typename Cx<HALF>::One*>(mid_f32);
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN1)) >> (kLogE - LOGN1));
    const int glog = logM - kLogE >= kGroupLog ? kGroupLog : 1;  // a chunk has 2^(logM-kLogE) >= 2 tiles
    // measured: 143 us against 149 with 512; a stand-by launch (only_if) takes the small grid, which leaves sooner
    const Grid g = grouped_grid(total >> glog, glog, only_if ? 512 : kPassAWgs);
    FFTSP_LAUNCH(only_if ? "rfft_pass_a_standby" : "rfft_pass_a", kern, dim3(g.wgs), dim3(kNT), lds, s, in, n, logM, mid,
                 t, aligned, (uint32_t)(total >> glog), g.per_wg, glog, zero_ptr, zero_words, table_arg<TABLE>(tab),
                 in_scale, only_if);
    return hipGetLastError();
}

template <int LOGN2, bool CODEC, bool HALF>
hipError_t fwd_b(const float2* mid_f32, int logM, size_t C, float2* spec_f32, uint32_t sstride, Tables t, uint32_t* hist,
                 float mid_scale, hipStream_t s, const uint32_t* only_if = nullptr)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN2)) * sizeof(float2) + kHistLdsWords * sizeof(uint32_t);
    auto kern = k_fwd_b<LOGN2, CODEC, HALF>;
    auto* mid = reinterpret_cast<const typename Cx<HALF>::One*>(mid_f32);
    auto* spec = reinterpret_cast<typename Cx<HALF>::One*>(spec_f32);
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN2)) >> (kLogE - LOGN2));
    const Grid g = persistent_grid(total);
    FFTSP_LAUNCH(only_if ? "rfft_pass_b_standby" : "rfft_pass_b", kern, dim3(g.wgs), dim3(kNT), lds, s, mid, logM, spec,
                 sstride, t, hist, (uint32_t)total, g.per_wg, mid_scale, only_if);
    return hipGetLastError();
}

template <int LOGN2, bool PAIR, bool HALF>
hipError_t inv_b(const float2* spec_f32, uint32_t sstride, int logM, size_t C, float2* mid_f32, Tables t, float mid_scale,
                 hipStream_t s, const uint32_t* only_if = nullptr)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN2)) * sizeof(float2);
    auto kern = k_inv_b<LOGN2, PAIR, HALF>;
    auto* spec = reinterpret_cast<const typename Cx<HALF>::One*>(spec_f32);
    auto* mid = reinterpret_cast<typename Cx<HALF>::One*>(mid_f32);
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN2)) >> (kLogE - LOGN2));
    const Grid g = persistent_grid(total, only_if ? 512 : 1536);  // measured: 117 us against 126 with 512
    FFTSP_LAUNCH(only_if ? "irfft_pass_b_standby" : "irfft_pass_b", kern, dim3(g.wgs), dim3(kNT), lds, s, spec, sstride,
                 logM, mid, t, (uint32_t)total, g.per_wg, mid_scale, only_if);
    return hipGetLastError();
}

template <int LOGN1, bool TABLE, bool HALF>
hipError_t inv_a(const float2* mid_f32, int logM, size_t C, float* out, size_t n, Tables t, int aligned, float gain,
                 const ChunkTable* tab, hipStream_t s, const uint32_t* only_if = nullptr)
{
    const size_t lds = ((size_t)(1 << kLogE) + (1 << LOGN1)) * sizeof(float2);
    auto kern = k_inv_a<LOGN1, TABLE, HALF>;
    auto* mid = reinterpret_cast<const typename Cx<HALF>::One*>(mid_f32);
    hipError_t e = set_lds(kern, lds);
    if (e != hipSuccess) return e;
    const size_t total = C * (((size_t)1 << (logM - LOGN1)) >> (kLogE - LOGN1));
    const int glog = logM - kLogE >= kGroupLog ? kGroupLog : 1;
    const Grid g = grouped_grid(total >> glog, glog);
    FFTSP_LAUNCH(only_if ? "irfft_pass_a_standby" : "irfft_pass_a", kern, dim3(g.wgs), dim3(kNT), lds, s, mid, logM, out,
                 n, t, aligned, (uint32_t)(total >> glog), g.per_wg, glog, gain, table_arg<TABLE>(tab), only_if);
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
                       int* pair_log, const ChunkTable* tab, hipStream_t s, const uint32_t* only_if)
{
    if (pair_log) *pair_log = 0;
    if (tab && C > (size_t)kMaxTableChunks) return hipErrorInvalidValue;
    if (zero_words > 0xffffffffu) return hipErrorInvalidValue;
    if (!hist) zero_words = 0;
    const int logM = logL - 1;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(in);
    const int aligned = ((addr & 7u) == 0 ? 1 : 0) | ((addr & 15u) == 0 ? 2 : 0);
    float2* sp = reinterpret_cast<float2*>(spec);
    if (hist_done) *hist_done = 0;
    if (C * ((size_t)1 << (logM > 13 ? logM - 13 : 0)) > 0x7fffffffu) return hipErrorInvalidValue;
    switch (logM) {
#define X(p) \
    case p: \
        return tab ? small_fwd<p, true>(in, n, C, sp, sstride, t, aligned & 1, tab, s) \
                   : small_fwd<p, false>(in, n, C, sp, sstride, t, aligned & 1, nullptr, s);
        FFTSP_SMALL_CASES(X)
#undef X
        default: break;
    }
    // the codec stores its own spectrum in the paired order and wants the histogram; the stage-level entry point
    // wants neither
    if ((hist != nullptr) != (pair_spec != 0)) return hipErrorInvalidValue;
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
#define FWD_A(p)                                                                              \
    (tab ? fwd_a<p, true, false>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, tab, 1.0f, s, only_if)      \
         : fwd_a<p, false, false>(in, n, logM, C, mid, t, aligned, zero_ptr, zero_words, nullptr, 1.0f, s, only_if))
    switch (logN1) {
        case 7: e = FWD_A(7); break;
        case 8: e = FWD_A(8); break;
        case 9: e = FWD_A(9); break;
        case 10: e = FWD_A(10); break;
        case 11: e = FWD_A(11); break;
        default: return hipErrorInvalidValue;
    }
#undef FWD_A
    if (e != hipSuccess) return e;
    if (hist_done) *hist_done = hist != nullptr;
    if (pair_log && pair_spec) *pair_log = logN1;
    if (hist) {
        switch (logN2) {
            case 7: return fwd_b<7, true, false>(mid, logM, C, sp, sstride, t, hist, 1.0f, s, only_if);
            case 8: return fwd_b<8, true, false>(mid, logM, C, sp, sstride, t, hist, 1.0f, s, only_if);
            case 9: return fwd_b<9, true, false>(mid, logM, C, sp, sstride, t, hist, 1.0f, s, only_if);
            case 10: return fwd_b<10, true, false>(mid, logM, C, sp, sstride, t, hist, 1.0f, s, only_if);
            default: return hipErrorInvalidValue;
        }
    }
    switch (logN2) {
        case 7: return fwd_b<7, false, false>(mid, logM, C, sp, sstride, t, nullptr, 1.0f, s);
        case 8: return fwd_b<8, false, false>(mid, logM, C, sp, sstride, t, nullptr, 1.0f, s);
        case 9: return fwd_b<9, false, false>(mid, logM, C, sp, sstride, t, nullptr, 1.0f, s);
        case 10: return fwd_b<10, false, false>(mid, logM, C, sp, sstride, t, nullptr, 1.0f, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_irfft(const float* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out, float2* mid,
                        Tables t, int pair_spec, float gain, const ChunkTable* tab, hipStream_t s, const uint32_t* only_if)
{
    if (tab && C > (size_t)kMaxTableChunks) return hipErrorInvalidValue;
    const int logM = logL - 1;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(out);
    const int aligned = ((addr & 7u) == 0 ? 1 : 0) | ((addr & 15u) == 0 ? 2 : 0);
    const float2* sp = reinterpret_cast<const float2*>(spec);
    if (C * ((size_t)1 << (logM > 13 ? logM - 13 : 0)) > 0x7fffffffu) return hipErrorInvalidValue;
    switch (logM) {
#define X(p) \
    case p: \
        return tab ? small_inv<p, true>(sp, sstride, n, C, out, t, aligned & 1, gain, tab, s) \
                   : small_inv<p, false>(sp, sstride, n, C, out, t, aligned & 1, gain, nullptr, s);
        FFTSP_SMALL_CASES(X)
#undef X
        default: break;
    }
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    if (pair_spec) {
        switch (logN2) {
            case 7: e = inv_b<7, true, false>(sp, sstride, logM, C, mid, t, 1.0f, s, only_if); break;
            case 8: e = inv_b<8, true, false>(sp, sstride, logM, C, mid, t, 1.0f, s, only_if); break;
            case 9: e = inv_b<9, true, false>(sp, sstride, logM, C, mid, t, 1.0f, s, only_if); break;
            case 10: e = inv_b<10, true, false>(sp, sstride, logM, C, mid, t, 1.0f, s, only_if); break;
            default: return hipErrorInvalidValue;
        }
    } else {
        switch (logN2) {
            case 7: e = inv_b<7, false, false>(sp, sstride, logM, C, mid, t, 1.0f, s); break;
            case 8: e = inv_b<8, false, false>(sp, sstride, logM, C, mid, t, 1.0f, s); break;
            case 9: e = inv_b<9, false, false>(sp, sstride, logM, C, mid, t, 1.0f, s); break;
            case 10: e = inv_b<10, false, false>(sp, sstride, logM, C, mid, t, 1.0f, s); break;
            default: return hipErrorInvalidValue;
        }
    }
    if (e != hipSuccess) return e;
#define INV_A(p)                                                          \
    (tab ? inv_a<p, true, false>(mid, logM, C, out, n, t, aligned, gain, tab, s, only_if) \
         : inv_a<p, false, false>(mid, logM, C, out, n, t, aligned, gain, nullptr, s, only_if))
    switch (logN1) {
        case 7: return INV_A(7);
        case 8: return INV_A(8);
        case 9: return INV_A(9);
        case 10: return INV_A(10);
        case 11: return INV_A(11);
        default: return hipErrorInvalidValue;
    }
#undef INV_A
}

// Half-precision variant (two-pass sizes, the codec's own buffers): the same four kernels with the intermediate
// and the spectrum stored as binary16 pairs.  in_scale (a power of two) multiplies the samples on the way in;
// the receiver divides through `gain`.
hipError_t launch_rfft_half(const float* in, size_t n, int logL, size_t C, void* spec, uint32_t sstride, void* mid,
                            Tables t, uint32_t* hist, uint32_t* zero_ptr, size_t zero_words, float in_scale,
                            int* pair_log, hipStream_t s)
{
    const int logM = logL - 1;
    if (logM < 14 || !hist || zero_words > 0xffffffffu) return hipErrorInvalidValue;
    if (C * ((size_t)1 << (logM - 13)) > 0x7fffffffu) return hipErrorInvalidValue;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(in);
    const int aligned = ((addr & 7u) == 0 ? 1 : 0) | ((addr & 15u) == 0 ? 2 : 0);
    float2* sp = static_cast<float2*>(spec);
    float2* md = static_cast<float2*>(mid);
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    // A first-pass sum of N1 terms is about sqrt(N2) times smaller than a spectrum value, an unnormalised inverse
    // second-pass sum about sqrt(N2) times larger: the stored intermediate is lifted (lowered) by 2^(logN2 / 2) so
    // that it sits where the caller's scale put the spectrum.  Powers of two: exact.
    const float lift = std::ldexp(1.0f, logN2 / 2);
#define FWD_A(p) \
    fwd_a<p, false, true>(in, n, logM, C, md, t, aligned, zero_ptr, (uint32_t)zero_words, nullptr, in_scale * lift, s)
    switch (logN1) {
        case 7: e = FWD_A(7); break;
        case 8: e = FWD_A(8); break;
        case 9: e = FWD_A(9); break;
        case 10: e = FWD_A(10); break;
        case 11: e = FWD_A(11); break;
        default: return hipErrorInvalidValue;
    }
#undef FWD_A
    if (e != hipSuccess) return e;
    *pair_log = logN1;
    switch (logN2) {
        case 7: return fwd_b<7, true, true>(md, logM, C, sp, sstride, t, hist, 1.0f / lift, s);
        case 8: return fwd_b<8, true, true>(md, logM, C, sp, sstride, t, hist, 1.0f / lift, s);
        case 9: return fwd_b<9, true, true>(md, logM, C, sp, sstride, t, hist, 1.0f / lift, s);
        case 10: return fwd_b<10, true, true>(md, logM, C, sp, sstride, t, hist, 1.0f / lift, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_irfft_half(const void* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out, void* mid,
                             Tables t, float gain, hipStream_t s)
{
    const int logM = logL - 1;
    if (logM < 14) return hipErrorInvalidValue;
    if (C * ((size_t)1 << (logM - 13)) > 0x7fffffffu) return hipErrorInvalidValue;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(out);
    const int aligned = ((addr & 7u) == 0 ? 1 : 0) | ((addr & 15u) == 0 ? 2 : 0);
    const float2* sp = static_cast<const float2*>(spec);
    float2* md = static_cast<float2*>(mid);
    const int logN1 = (logM + 1) / 2, logN2 = logM / 2;
    hipError_t e;
    const float lift = std::ldexp(1.0f, logN2 / 2);  // see launch_rfft_half
    switch (logN2) {
        case 7: e = inv_b<7, true, true>(sp, sstride, logM, C, md, t, 1.0f / lift, s); break;
        case 8: e = inv_b<8, true, true>(sp, sstride, logM, C, md, t, 1.0f / lift, s); break;
        case 9: e = inv_b<9, true, true>(sp, sstride, logM, C, md, t, 1.0f / lift, s); break;
        case 10: e = inv_b<10, true, true>(sp, sstride, logM, C, md, t, 1.0f / lift, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
#define INV_A(p) inv_a<p, false, true>(md, logM, C, out, n, t, aligned, gain * lift, nullptr, s)
    switch (logN1) {
        case 7: return INV_A(7);
        case 8: return INV_A(8);
        case 9: return INV_A(9);
        case 10: return INV_A(10);
        case 11: return INV_A(11);
        default: return hipErrorInvalidValue;
    }
#undef INV_A
}

}  // namespace fftsp

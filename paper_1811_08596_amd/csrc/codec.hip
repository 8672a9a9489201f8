// Selection, quantization, packing and their inverses for gfx950.
//
// Follows arXiv 1811.08596: Sec. 3.1.1 (keep the largest-magnitude frequency
// components, zero the rest), Sec. 3.2 (status bitmap -> prefix sum -> dense
// vector) and Sec. 3.2.1 / Algorithm 1 (offset-based N-bit float).
//
// Selection is an exact radix select on the 31-bit key
//     key = bits( fma(re, re, im*im) )        (binary32, one product rounded, then one fused step)
// so it is integer work: a 12-bit histogram of the top key bits per chunk finds
// the bucket that holds the k-th largest key; bins in higher buckets are kept
// outright, bins in that bucket ("candidates") are written out tile by tile in
// bin order, and one workgroup per chunk finishes the select on the candidates
// (two more digits), resolves ties by lowest bin index, scans the per-tile
// survivor counts and finds the survivors' largest component, which fixes eps
// (pbase) of Algorithm 1.  A last pass flags, ranks (wave ballots + popcounts),
// quantizes and bit-packs.
#include "internal.h"

namespace fftsp {
namespace {

constexpr int NT = kTileThreads;     // 256 lanes = 4 waves
constexpr int ROWS = 8;              // rows of 64 bins per wave
constexpr int WAVE_BINS = ROWS * 64; // 512
static_assert(kTile == 4 * WAVE_BINS, "tile geometry");

// The sign bit is masked: a finite sum of squares has none, and a NaN that carries one must still land inside the
// 31-bit key space the histogram and the radix digits are sized for (selection among non-finite bins is then
// ordinary integer work on their bit patterns, and exactly k bins survive whatever the input holds).
__device__ __forceinline__ uint32_t key_of(float2 z)
{
    return __float_as_uint(__fmaf_rn(z.x, z.x, __fmul_rn(z.y, z.y))) & 0x7FFFFFFFu;
}
__device__ __forceinline__ uint32_t vbits_of(float2 z)
{
    const uint32_t a = __float_as_uint(z.x) & 0x7FFFFFFFu, b = __float_as_uint(z.y) & 0x7FFFFFFFu;
    return a > b ? a : b;
}
// What is ranked and coded is either a complex frequency bin (two codes) or, for time-domain Top-k, a sample of
// the gradient itself (one code; the rank key is the bit pattern of |x|, an exact magnitude order).
__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }
__device__ __forceinline__ uint32_t vbits_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }
template <bool REAL>
struct Elem {
    using T = float2;
    static constexpr uint32_t kCodes = 2;
    static __device__ __forceinline__ T zero() { return make_float2(0.f, 0.f); }
};
template <>
struct Elem<true> {
    using T = float;
    static constexpr uint32_t kCodes = 1;
    static __device__ __forceinline__ T zero() { return 0.f; }
};
// samples of chunk c that exist (time domain: the last chunk may end early, the rest counts as zeros)
template <bool REAL>
__device__ __forceinline__ uint32_t present_of(size_t n, size_t c, uint32_t B)
{
    if constexpr (REAL) {
        const size_t left = n - c * (size_t)B;
        return left < (size_t)B ? (uint32_t)left : B;
    } else {
        return B;
    }
}

// a plain 16-byte value that the compiler keeps in registers
typedef uint32_t u32x4 __attribute__((vector_size(16)));

// number of set bits of a wave-uniform mask below this lane (v_mbcnt_lo/hi: two instructions, no 64-bit math)
__device__ __forceinline__ uint32_t prefix_popc(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Cooperative load of one tile of the spectrum buffer, [tbase, tbase+count), into LDS as whole 16-byte pieces.
// A tile is contiguous in the buffer in either bin order (paired runs are tile-aligned), so lanes then pick
// their own bins from LDS at spec_index(j) - tbase instead of issuing half-dense global loads.
__device__ __forceinline__ void tile_to_lds(const float2* __restrict__ X, uint32_t tbase, uint32_t count,
                                            uint32_t sstride, float2* stage, int tid)
{
    if (count == (uint32_t)kTile && (sstride & 1u) == 0) {  // chunk base and tile base are 16-byte aligned
        const float4* src = reinterpret_cast<const float4*>(X + tbase);
        float4* dst = reinterpret_cast<float4*>(stage);
#pragma unroll
        for (int i = 0; i < kTile / 2 / kTileThreads; ++i) dst[tid + i * kTileThreads] = src[tid + i * kTileThreads];
    } else {
        for (uint32_t i = tid; i < count; i += kTileThreads) stage[i] = X[tbase + i];
    }
}

// The same from a spectrum stored as binary16 pairs (half-precision variant): converted on the way into LDS, so
// everything behind it works on binary32 values as before.
__device__ __forceinline__ void tile_to_lds(const uint32_t* __restrict__ X, uint32_t tbase, uint32_t count,
                                            uint32_t sstride, float2* stage, int tid)
{
    if (count == (uint32_t)kTile && (sstride & 3u) == 0) {  // four bins per 16 bytes
        const uint4* src = reinterpret_cast<const uint4*>(X + tbase);
        float4* dst = reinterpret_cast<float4*>(stage);
#pragma unroll
        for (int i = 0; i < kTile / 4 / kTileThreads; ++i) {
            const int idx = tid + i * kTileThreads;
            const uint4 v = src[idx];
            dst[2 * idx] = cx_load(make_uint2(v.x, v.y));
            dst[2 * idx + 1] = cx_load(make_uint2(v.z, v.w));
        }
    } else {
        for (uint32_t i = tid; i < count; i += kTileThreads) stage[i] = unpack_half2(X[tbase + i]);
    }
}

// What a kernel's input or output array holds: samples (time domain), or complex bins as binary32 or binary16 pairs.
template <bool REAL, bool HALF>
struct Stored {
    using T = typename Cx<HALF>::One;
};
template <bool HALF>
struct Stored<true, HALF> {
    using T = float;
};

// Time domain: samples [tbase, tbase + kTile) of a chunk, zeros from `present` on.
__device__ __forceinline__ void tile_to_lds(const float* __restrict__ X, uint32_t tbase, uint32_t present, float* stage,
                                            int tid)
{
    if (tbase + (uint32_t)kTile <= present) {  // chunks start on multiples of 32 samples of a 16-byte aligned gradient
        const float4* src = reinterpret_cast<const float4*>(X + tbase);
        float4* dst = reinterpret_cast<float4*>(stage);
#pragma unroll
        for (int i = 0; i < kTile / 4 / kTileThreads; ++i) dst[tid + i * kTileThreads] = src[tid + i * kTileThreads];
    } else {
        for (uint32_t i = tid; i < (uint32_t)kTile; i += kTileThreads) stage[i] = tbase + i < present ? X[tbase + i] : 0.f;
    }
}

// In-tile slot (position in the spectrum buffer minus the tile base) of this lane's bin in each of the wave's
// rows (bins j0, j0 + 64, ...).  The 512 bins of a wave lie in one half of one paired run when a run has at least
// 1024 positions, so the slot is linear in the row and costs one add instead of the whole index computation;
// shorter runs go through spec_index row by row.
struct RowSlots {
    uint32_t first;  // row 0 (the run's middle bin N1/2 sits at position 1, off the line of the other rows)
    uint32_t lin;    // row r >= 1: lin + r * step
    int step;
    bool linear;
};
__device__ __forceinline__ RowSlots row_slots(uint32_t j0, uint32_t tbase, int pair_log)
{
    RowSlots s;
    s.linear = pair_log == 0 || pair_log >= 10;
    s.first = s.lin = j0 - tbase;
    s.step = 64;
    if (pair_log >= 10) {
        const uint32_t N1 = 1u << pair_log, k1 = j0 & (N1 - 1u), run = j0 - k1 - tbase;
        const bool upper = k1 >= N1 / 2;
        s.lin = run + (upper ? 2u * (N1 - k1) + 1u : 2u * k1);
        s.first = k1 == N1 / 2 ? run + 1u : s.lin;
        s.step = upper ? -128 : 128;
    }
    return s;
}
__device__ __forceinline__ uint32_t slot_of(const RowSlots& s, int r, uint32_t j0, uint32_t tbase, int pair_log)
{
    if (s.linear) return r == 0 ? s.first : s.lin + (uint32_t)(r * s.step);
    return spec_index(j0 + (uint32_t)r * 64u, pair_log) - tbase;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t u = __shfl_xor(v, o, 64);
        v = u > v ? u : v;
    }
    return v;
}

// 32bit_to_Nbit of Algorithm 1 (value > max clamps to the top code; below eps flushes to the zero code)
__device__ __forceinline__ uint32_t quantize(uint32_t fbits, uint32_t pbase, int bits, int shift)
{
    if (bits == 32) return fbits;
    const uint32_t Mmax = (1u << (bits - 1)) - 1u;
    const uint32_t q = (fbits & 0x7FFFFFFFu) >> shift;
    uint32_t c = 0;
    if (q >= pbase) {
        c = q - pbase + 1u;
        c = c > Mmax ? Mmax : c;
    }
    const uint32_t sign = c ? (fbits >> 31) : 0u;
    return (sign << (bits - 1)) | c;
}
// Nbit_to_32bit of Algorithm 1
__device__ __forceinline__ uint32_t dequantize(uint32_t code, uint32_t pbase, int bits, int shift)
{
    if (bits == 32) return code;
    const uint32_t Mmax = (1u << (bits - 1)) - 1u;
    const uint32_t c = code & Mmax, sign = (code >> (bits - 1)) & 1u;
    return c ? (((c - 1u + pbase) << shift) | (sign << 31)) : 0u;
}

__global__ void k_zero_u32(uint32_t* p, size_t count)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

// ------------------------------------------------------------- histogram ----
constexpr int HIST_TILES = 4;  // tiles per workgroup

__global__ __launch_bounds__(NT) void k_hist(const float2* __restrict__ spec, uint32_t sstride, int pair_log, uint32_t B,
                                             uint32_t groups, uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[kHistBins];
    const int tid = threadIdx.x;
    const size_t c = blockIdx.x / groups;
    const uint32_t base = (blockIdx.x % groups) * (HIST_TILES * kTile);
    for (int i = tid; i < kHistBins; i += NT) h[i] = 0u;
    __syncthreads();
    const float2* X = spec + c * (size_t)sstride;
#pragma unroll 4
    for (int i = tid; i < HIST_TILES * kTile; i += NT) {
        const uint32_t j = base + i;
        if (j < B) atomicAdd(&h[key_of(X[spec_index(j, pair_log)]) >> kKeyShift], 1u);
    }
    __syncthreads();
    uint32_t* g = hist + c * kHistBins;
    for (int i = tid; i < kHistBins; i += NT) {
        const uint32_t v = h[i];
        if (v) atomicAdd(&g[i], v);
    }
}

// Time domain: the same histogram over the samples' |x| patterns, as a kernel of its own because it is the first
// and largest pass of that path.  Gradients crowd into a few dozen of the buckets (16 per binade), so plain LDS
// counters serialise; here every lane adds into one of kHistCopies copies chosen by its lane id, the copies are
// skewed by one bank each, and a counter is a 16-bit half of a word (a copy receives at most 8192 keys).
// Measured on 62 M samples: 2 copies x 8 tiles 76 us; 1 x 8: 82; 4 x 8: 85; 2 x 4: 92; 2 x 16: 95; 8 x 16: 126
// (more LDS per workgroup costs residency, shorter stretches pay the flush more often).
constexpr int kHistCopies = 2;
constexpr int kHistSampleTiles = 8;  // tiles of 2048 samples per workgroup
constexpr int kHistCopyWords = kHistBins / 2 + 1;
static_assert(kHistSampleTiles * kTile / kHistCopies < 65536, "16-bit counters");

__global__ __launch_bounds__(NT) void k_hist_samples(const float* __restrict__ in, uint32_t L, uint32_t groups,
                                                     uint32_t* __restrict__ hist, size_t n)
{
    __shared__ uint32_t h[kHistCopies * kHistCopyWords];
    const int tid = threadIdx.x;
    const size_t c = blockIdx.x / groups;
    const uint32_t base = (blockIdx.x % groups) * (uint32_t)(kHistSampleTiles * kTile);
    for (int i = tid; i < kHistCopies * kHistCopyWords; i += NT) h[i] = 0u;
    __syncthreads();
    const float* X = in + c * (size_t)L;
    const uint32_t present = present_of<true>(n, c, L);
    const uint32_t count = L - base < (uint32_t)(kHistSampleTiles * kTile) ? L - base : (uint32_t)(kHistSampleTiles * kTile);
    uint32_t* mine = h + (tid & (kHistCopies - 1)) * kHistCopyWords;
    auto add = [&](float x) __attribute__((always_inline)) {
        const uint32_t b = key_of(x) >> kKeyShift;
        atomicAdd(&mine[b >> 1], 1u << (16u * (b & 1u)));
    };
    if (base + count <= present) {  // chunks start on multiples of 32 samples of a 16-byte aligned gradient
        const float4* X4 = reinterpret_cast<const float4*>(X + base);
#pragma unroll 4
        for (uint32_t i = tid; i < count / 4u; i += NT) {
            const float4 v = X4[i];
            add(v.x);
            add(v.y);
            add(v.z);
            add(v.w);
        }
    } else {  // the gradient ends inside this stretch: what lies past its end counts as zeros
        for (uint32_t i = tid; i < count; i += NT) add(base + i < present ? X[base + i] : 0.f);
    }
    __syncthreads();
    uint32_t* g = hist + c * kHistBins;
    for (int w = tid; w < kHistBins / 2; w += NT) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int k = 0; k < kHistCopies; ++k) {
            const uint32_t v = h[k * kHistCopyWords + w];
            lo += v & 0xFFFFu;
            hi += v >> 16;
        }
        if (lo) atomicAdd(&g[2 * w], lo);
        if (hi) atomicAdd(&g[2 * w + 1], hi);
    }
}

// inclusive scan over the 256 lanes of a workgroup; tmp has 4 entries
__device__ __forceinline__ uint32_t block_scan_incl_256(uint32_t v, uint32_t* tmp)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(x, o, 64);
        if (lane >= o) x += u;
    }
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    uint32_t add = 0;
    for (int w = 0; w < wave; ++w) add += tmp[w];
    __syncthreads();
    return x + add;
}

// Per chunk: the bucket b* holding the k-th largest key, and how many of its bins are still needed.
__global__ __launch_bounds__(NT) void k_find_bucket(const uint32_t* __restrict__ hist, uint32_t k,
                                                    uint32_t* __restrict__ sel)
{
    __shared__ uint32_t tmp[4];
    const int tid = threadIdx.x;
    const size_t c = blockIdx.x;
    constexpr int PER = kHistBins / NT;  // 16 buckets per lane, lane t owns the buckets counted from the top
    uint32_t loc[PER];
    uint32_t s = 0;
    const uint32_t top = kHistBins - 1 - tid * PER;  // highest bucket of this lane
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        loc[i] = hist[c * kHistBins + (top - i)];
        s += loc[i];
    }
    const uint32_t incl = block_scan_incl_256(s, tmp);
    uint32_t run = incl - s;  // bins in buckets above this lane's range
    if (k == 0) {
        if (tid == 0) {
            sel[c * 8 + 0] = kHistBins;  // no bucket qualifies: nothing is kept
            sel[c * 8 + 1] = 0;
        }
        return;
    }
    // The histogram counts every bin of the chunk, so some bucket always qualifies; should it ever not (fewer than
    // k bins counted), the selection words still get defined values instead of the previous call's.
    if (tid == 0) {
        sel[c * 8 + 0] = 0;
        sel[c * 8 + 1] = 0;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        if (run < k && run + loc[i] >= k) {
            sel[c * 8 + 0] = top - i;
            sel[c * 8 + 1] = k - run;
        }
        run += loc[i];
    }
}

// --------------------------------------------------------------- collect ----
// Per tile: count and range of the bins kept outright, and the candidates in bin order.
template <bool REAL, bool HALF>
__global__ __launch_bounds__(NT) void k_collect(const typename Stored<REAL, HALF>::T* __restrict__ spec, uint32_t sstride,
                                                int pair_log, uint32_t B, uint32_t Tn, const uint32_t* __restrict__ sel,
                                                uint32_t* __restrict__ tinfo, uint2* __restrict__ cand, size_t n)
{
    using E = typename Elem<REAL>::T;
    __shared__ uint32_t wcnt[4], wdef[4], wvmax[4];
    __shared__ E stage[kTile];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t c = blockIdx.x / Tn;
    const uint32_t tile = blockIdx.x % Tn;
    const typename Stored<REAL, HALF>::T* X = spec + c * (size_t)sstride;
    const uint32_t tbase = tile * kTile;
    if constexpr (REAL)
        tile_to_lds(X, tbase, present_of<REAL>(n, c, B), stage, tid);
    else
        tile_to_lds(X, tbase, B - tbase < (uint32_t)kTile ? B - tbase : (uint32_t)kTile, sstride, stage, tid);
    const uint32_t bstar = sel[c * 8 + 0];
    __syncthreads();
    const uint32_t j0 = tbase + wave * WAVE_BINS + lane;
    const RowSlots slots = row_slots(j0, tbase, pair_log);
    uint32_t key[ROWS], vb[ROWS];
    uint64_t cm[ROWS];
    uint32_t ndef = 0, vmax = 0, ncand = 0, mine = 0;  // mine: bit r set = this lane's bin of row r is a candidate
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const uint32_t j = j0 + r * 64;
        const bool valid = j < B;
        const E z = valid ? stage[slot_of(slots, r, j0, tbase, pair_log)] : Elem<REAL>::zero();
        key[r] = key_of(z);
        vb[r] = vbits_of(z);
        const uint32_t bucket = key[r] >> kKeyShift;
        const bool isdef = valid && bucket > bstar;
        const bool iscand = valid && bucket == bstar;
        if (isdef) {
            ++ndef;
            vmax = vb[r] > vmax ? vb[r] : vmax;
        }
        mine |= (uint32_t)iscand << r;
        cm[r] = __ballot(iscand);
        ncand += (uint32_t)__popcll(cm[r]);
    }
    ndef = wave_sum(ndef);
    vmax = wave_max(vmax);
    if (lane == 0) {
        wcnt[wave] = ncand;
        wdef[wave] = ndef;
        wvmax[wave] = vmax;
    }
    __syncthreads();
    uint32_t off = 0;
    for (int w = 0; w < wave; ++w) off += wcnt[w];
    uint2* out = cand + (c * Tn + tile) * (size_t)kTile;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        if ((mine >> r) & 1u) out[off + prefix_popc(cm[r])] = make_uint2(key[r], vb[r]);
        off += (uint32_t)__popcll(cm[r]);
    }
    if (tid == 0) {
        uint32_t* ti = tinfo + (c * Tn + tile) * 4;
        ti[0] = wdef[0] + wdef[1] + wdef[2] + wdef[3];
        uint32_t m = wvmax[0];
        m = wvmax[1] > m ? wvmax[1] : m;
        m = wvmax[2] > m ? wvmax[2] : m;
        m = wvmax[3] > m ? wvmax[3] : m;
        ti[1] = m;
        ti[2] = wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        ti[3] = 0;
    }
}

// --------------------------------------------------------------- resolve ----
constexpr int RT = 1024;           // lanes of the per-chunk workgroup
constexpr int RW = RT / 64;        // 16 waves
constexpr int MAX_TILES = ((1 << (kMaxLogL - 1)) + 1 + kTile - 1) / kTile;  // 1025

// inclusive scan over 1024 lanes; tmp has 16 entries
__device__ __forceinline__ uint32_t block_scan_incl_1024(uint32_t v, uint32_t* tmp)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(x, o, 64);
        if (lane >= o) x += u;
    }
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    uint32_t add = 0;
    for (int w = 0; w < wave; ++w) add += tmp[w];
    __syncthreads();
    return x + add;
}

// byte offset of chunk c's record from the first record of the launch: c * S, or from the table in per-tensor launches
template <bool TABLE>
__device__ __forceinline__ size_t record_offset(const TableArg<TABLE>& tab, size_t c, size_t S)
{
    if constexpr (TABLE)
        return (size_t)tab.t.roff[c];
    else
        return c * S;
}

// Candidates that did not fit in LDS are walked from memory.
constexpr int kWalk = 8;  // further rows of 64 candidates of one tile fetched in one round trip
// All tiles of a chunk, a wave per tile, kWalkTiles tiles per round trip: the first row of candidates of each tile of
// a batch (usually all a tile has) is fetched before any is used.  begin(t) and end(t) bracket tile t's rows, which
// go to row(entry, valid) in candidate order; all three are called by the whole wave.
constexpr int kWalkTiles = 8;
template <typename B, typename R, typename E>
__device__ __forceinline__ void walk_tiles(const uint2* __restrict__ cd, const uint32_t* tnc, uint32_t Tn, int wave, int lane,
                                           B&& begin, R&& row, E&& end)
{
    for (uint32_t t0 = (uint32_t)wave; t0 < Tn; t0 += RW * kWalkTiles) {
        uint2 first[kWalkTiles];
#pragma unroll
        for (int u = 0; u < kWalkTiles; ++u) {
            const uint32_t t = t0 + (uint32_t)u * RW;
            const uint32_t nc = t < Tn ? tnc[t] : 0u;
            // lanes past the end read their tile's first slot (always allocated) and drop it
            first[u] = cd[(size_t)(t < Tn ? t : 0u) * kTile + ((uint32_t)lane < nc ? (uint32_t)lane : 0u)];
        }
#pragma unroll
        for (int u = 0; u < kWalkTiles; ++u) {
            const uint32_t t = t0 + (uint32_t)u * RW;
            if (t < Tn) {
                const uint32_t nc = tnc[t];
                begin(t);
                if (nc) row(first[u], (uint32_t)lane < nc);
                if (nc > 64u) {  // long runs of equal keys (a chunk of zeros) fill whole tiles
                    const uint2* tile_cands = cd + (size_t)t * kTile;
                    for (uint32_t i0 = 64u; i0 < nc; i0 += 64u * kWalk) {
                        uint2 e[kWalk];
#pragma unroll
                        for (int v = 0; v < kWalk; ++v) {
                            const uint32_t i = i0 + (uint32_t)v * 64u + (uint32_t)lane;
                            e[v] = tile_cands[i < nc ? i : 0u];
                        }
#pragma unroll
                        for (int v = 0; v < kWalk; ++v) {
                            const uint32_t r0 = i0 + (uint32_t)v * 64u;
                            if (r0 < nc) row(e[v], r0 + (uint32_t)lane < nc);
                        }
                    }
                }
                end(t);
            }
        }
    }
}

constexpr int kStageBatch = 9;  // tiles whose candidates a wave of k_resolve fetches in one go

struct HeaderInfo {
    int write;
    uint64_t n;
    uint32_t L, C, N, m, k, S;
    float theta;
    uint32_t domain;  // 0: records hold frequency bins, 1: samples (time-domain Top-k)
    uint32_t scale;   // log2 of the factor on the spectrum (two's complement; half-precision variant), else 0
};

// One workgroup per chunk: finish the radix select on the candidates, break ties by bin order,
// scan the tiles, find the survivors' largest component, write the record header and zero the
// code words that two tiles will share.
// KEYS: a candidate's second word equals its key (time domain: both are the pattern of |x|), so only keys are
// staged and the stage holds twice as many candidates.
template <bool TABLE, bool KEYS>
__global__ __launch_bounds__(RT) void k_resolve(uint32_t Tn, uint32_t k, int bits, int m, uint32_t W, size_t S,
                                                uint32_t word3, uint32_t stage_cap, uint32_t static_vmax,
                                                uint32_t codes_per_bin,
                                                uint32_t* __restrict__ sel,
                                                const uint32_t* __restrict__ tinfo, uint32_t* __restrict__ tscan,
                                                const uint2* __restrict__ cand, uint8_t* __restrict__ records,
                                                uint8_t* __restrict__ stream, HeaderInfo hdr, TableArg<TABLE> tab)
{
    __shared__ uint32_t h[1024];
    __shared__ uint32_t tmp[RW];
    __shared__ uint32_t tgt[MAX_TILES], teq[MAX_TILES], ttake[MAX_TILES], trank[MAX_TILES], tsurv[MAX_TILES];
    __shared__ uint32_t toff[MAX_TILES], tnc[MAX_TILES], tdef[MAX_TILES], tvd[MAX_TILES];
    __shared__ uint32_t s_digit, s_need, s_vmax, s_carry[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t c = blockIdx.x;
    const uint32_t bstar = sel[c * 8 + 0];
    uint32_t need = sel[c * 8 + 1];
    const uint32_t* ti = tinfo + c * Tn * 4;
    const uint2* cd = cand + c * Tn * (size_t)kTile;
    uint32_t tau = 0xFFFFFFFFu, quota = 0;

    // Stage the candidates in LDS when they fit (they are read four times below): tile t's candidates go to
    // stage[toff[t] ..).  Otherwise every pass reads them from global memory.
    extern __shared__ float2 smem[];
    uint2* stage = reinterpret_cast<uint2*>(smem);
    uint32_t* stage_keys = reinterpret_cast<uint32_t*>(smem);
    auto staged_key = [&](uint32_t i) __attribute__((always_inline)) {
        if constexpr (KEYS)
            return stage_keys[i];
        else
            return stage[i].x;
    };
    if (tid == 0) s_carry[0] = 0;
    __syncthreads();
    for (uint32_t base = 0; base < Tn; base += RT) {
        const uint32_t t = base + tid;
        uint32_t nc = 0;
        if (t < Tn) {  // the per-tile summaries are read once; every later pass takes them from LDS
            const uint4 info = reinterpret_cast<const uint4*>(ti)[t];
            tdef[t] = info.x;
            tvd[t] = info.y;
            tnc[t] = nc = info.z;
        }
        const uint32_t carry = s_carry[0];
        const uint32_t incl = block_scan_incl_1024(nc, tmp);
        if (t < Tn) toff[t] = carry + incl - nc;
        __syncthreads();
        if (tid == RT - 1) s_carry[0] = carry + incl;
        __syncthreads();
    }
    const bool staged = s_carry[0] <= stage_cap;
    if (staged) {
        // A wave per tile, kStageBatch tiles in flight per wave: a tile's candidates are one contiguous run (about 40
        // for a 2^20 chunk), so a wave fetches them with one coalesced load, and all loads of a batch are issued
        // before the first is used: one memory round trip per batch, no search for the tile a candidate belongs to.
        for (uint32_t t0 = (uint32_t)wave; t0 < Tn; t0 += RW * kStageBatch) {
            uint2 v[kStageBatch];
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const uint32_t t = t0 + (uint32_t)u * RW;
                const uint32_t nc = t < Tn ? tnc[t] : 0u;
                // lanes past the end read their tile's first slot (always allocated) and drop it
                v[u] = cd[(size_t)(t < Tn ? t : 0u) * kTile + ((uint32_t)lane < nc ? (uint32_t)lane : 0u)];
            }
#pragma unroll
            for (int u = 0; u < kStageBatch; ++u) {
                const uint32_t t = t0 + (uint32_t)u * RW;
                if (t < Tn && (uint32_t)lane < tnc[t]) {
                    if constexpr (KEYS)
                        stage_keys[toff[t] + (uint32_t)lane] = v[u].x;
                    else
                        stage[toff[t] + (uint32_t)lane] = v[u];
                }
            }
            // the rare tile with more than a row of candidates (runs of equal keys)
#pragma unroll 1
            for (int u = 0; u < kStageBatch; ++u) {
                const uint32_t t = t0 + (uint32_t)u * RW;
                if (t >= Tn) break;
                const uint32_t nc = tnc[t], o = toff[t];
                for (uint32_t i = 64u + (uint32_t)lane; i < nc; i += 64u) {
                    const uint2 e = cd[(size_t)t * kTile + i];
                    if constexpr (KEYS)
                        stage_keys[o + i] = e.x;
                    else
                        stage[o + i] = e;
                }
            }
        }
    }
    __syncthreads();

    if (need > 0) {
        uint32_t prefix = bstar << kKeyShift;
        // two more digits: bits 18..9, then bits 8..0
        for (int pass = 0; pass < 2; ++pass) {
            const int shift = pass == 0 ? 9 : 0;
            const uint32_t dmask = pass == 0 ? 1023u : 511u;
            const uint32_t pmask = pass == 0 ? (0xFFFFFFFFu << kKeyShift) : (0xFFFFFFFFu << 9);
            h[tid] = 0u;
            if (tid == 0) {  // defined even if no digit qualifies (the counts then disagree with the histogram)
                s_digit = 0u;
                s_need = 0u;
            }
            __syncthreads();
            if (staged) {
                const uint32_t total = s_carry[0];
                for (uint32_t i = tid; i < total; i += RT) {
                    const uint32_t key = staged_key(i);
                    if ((key & pmask) == prefix) atomicAdd(&h[(key >> shift) & dmask], 1u);
                }
            } else {
                walk_tiles(cd, tnc, Tn, wave, lane, [](uint32_t) {}, [&](uint2 e, bool valid) {
                    const bool hit = valid && (e.x & pmask) == prefix;
                    const uint32_t digit = (e.x >> shift) & dmask;
                    const uint64_t act = __ballot(hit);
                    if (act) {
                        // a row whose keys share the digit (a run of equal values, e.g. zeros) is one atomic
                        const int first = __ffsll((unsigned long long)act) - 1;
                        const uint32_t d0 = __shfl(digit, first, 64);
                        if (__ballot(hit && digit == d0) == act) {
                            if (lane == first) atomicAdd(&h[d0], (uint32_t)__popcll(act));
                        } else if (hit) {
                            atomicAdd(&h[digit], 1u);
                        }
                    }
                }, [](uint32_t) {});
            }
            __syncthreads();
            const uint32_t bin = 1023u - (uint32_t)tid;  // scan from the top digit down
            const uint32_t cnt = h[bin];
            const uint32_t incl = block_scan_incl_1024(cnt, tmp);
            const uint32_t excl = incl - cnt;
            if (excl < need && incl >= need) {
                s_digit = bin;
                s_need = need - excl;
            }
            __syncthreads();
            prefix |= s_digit << shift;
            need = s_need;
            __syncthreads();
        }
        tau = prefix;
        quota = need;  // bins equal to tau still to take, in bin order
    }

    // per tile: candidates above tau and equal to tau
    if (staged) {
        // one lane per tile walks that tile's staged candidates (about 40 for a 2^20 chunk): no ballots, no
        // wave-serial loop over tiles
        for (uint32_t t = tid; t < Tn; t += RT) {
            const uint32_t nc = tnc[t], o = toff[t];
            uint32_t gt = 0, eq = 0;
            for (uint32_t i = 0; i < nc; ++i) {
                const uint32_t key = staged_key(o + i);
                gt += key > tau;
                eq += key == tau;
            }
            tgt[t] = gt;
            teq[t] = eq;
        }
    } else {
        uint32_t gt = 0, eq = 0;  // wave-uniform counts from ballots
        walk_tiles(cd, tnc, Tn, wave, lane, [&](uint32_t) { gt = eq = 0; }, [&](uint2 e, bool valid) {
            gt += (uint32_t)__popcll(__ballot(valid && e.x > tau));
            eq += (uint32_t)__popcll(__ballot(valid && e.x == tau));
        }, [&](uint32_t t) {
            if (lane == 0) {
                tgt[t] = gt;
                teq[t] = eq;
            }
        });
    }
    if (tid == 0) {
        s_carry[0] = 0;
        s_carry[1] = 0;
        s_vmax = 0;
    }
    __syncthreads();

    // scan over tiles: equal-key prefix decides who gets the tie quota, survivor prefix gives the ranks
    for (uint32_t base = 0; base < Tn; base += RT) {
        const uint32_t t = base + tid;
        const bool in = t < Tn;
        const uint32_t eq = in ? teq[t] : 0u;
        const uint32_t ceq = s_carry[0], crk = s_carry[1];
        const uint32_t eqincl = block_scan_incl_1024(eq, tmp);
        const uint32_t eqpre = ceq + eqincl - eq;
        const uint32_t take = eqpre >= quota ? 0u : (eq < quota - eqpre ? eq : quota - eqpre);
        const uint32_t surv = in ? (tdef[t] + tgt[t] + take) : 0u;
        const uint32_t rkincl = block_scan_incl_1024(surv, tmp);
        // ranks never leave [0, k]: whatever the counts say, the code words of a tile stay inside the record
        const uint32_t rank_raw = crk + rkincl - surv;
        const uint32_t rank = rank_raw < k ? rank_raw : k;
        if (in) {
            ttake[t] = take;
            trank[t] = rank;
            tsurv[t] = surv < k - rank ? surv : k - rank;
            tscan[(c * Tn + t) * 2 + 0] = rank;
            tscan[(c * Tn + t) * 2 + 1] = eqpre;
        }
        __syncthreads();
        if (tid == RT - 1) {
            s_carry[0] = ceq + eqincl;
            s_carry[1] = crk + rkincl;
        }
        __syncthreads();
    }

    // largest component over the survivors (not needed when the caller fixed the range: Sec. 3.2.1, static max)
    uint32_t vm = 0;  // per-lane running maximum, reduced once at the end
    if (static_vmax) {
        // nothing to find
    } else if (staged) {
        for (uint32_t t = tid; t < Tn; t += RT) {
            const uint32_t nc = tnc[t], o = toff[t], take = ttake[t];
            if (tdef[t]) vm = tvd[t] > vm ? tvd[t] : vm;
            uint32_t eqrun = 0;  // candidates equal to tau seen so far, in bin order
            for (uint32_t i = 0; i < nc; ++i) {
                uint2 e;
                if constexpr (KEYS)
                    e = make_uint2(stage_keys[o + i], stage_keys[o + i]);
                else
                    e = stage[o + i];
                const bool iseq = e.x == tau;
                const bool kept = e.x > tau || (iseq && eqrun < take);
                eqrun += iseq;
                if (kept) vm = e.y > vm ? e.y : vm;
            }
        }
    } else {
        uint32_t take = 0, eqrun = 0;
        walk_tiles(cd, tnc, Tn, wave, lane, [&](uint32_t t) {
            take = ttake[t];
            if (lane == 0 && tdef[t]) vm = tvd[t] > vm ? tvd[t] : vm;
            eqrun = 0;
        }, [&](uint2 e, bool valid) {
            const bool iseq = valid && e.x == tau;
            const uint64_t em = __ballot(iseq);
            const bool kept = valid && (e.x > tau || (iseq && eqrun + prefix_popc(em) < take));
            if (kept) vm = e.y > vm ? e.y : vm;
            eqrun += (uint32_t)__popcll(em);
        }, [](uint32_t) {});
    }
    vm = wave_max(vm);
    if (lane == 0 && vm) atomicMax(&s_vmax, vm);
    __syncthreads();

    const uint32_t vmax = static_vmax ? static_vmax : s_vmax;
    uint32_t pbase = 0;
    if (bits != 32) {
        const int shift = 23 - m;
        const int64_t pb = (int64_t)(vmax >> shift) - (int64_t)((1u << (bits - 1)) - 2u);
        pbase = pb < 1 ? 1u : (uint32_t)pb;
    }
    uint32_t* rec = reinterpret_cast<uint32_t*>(records + record_offset<TABLE>(tab, c, S));
    if (tid == 0) {
        sel[c * 8 + 2] = tau;
        sel[c * 8 + 3] = quota;
        sel[c * 8 + 4] = pbase;
        sel[c * 8 + 5] = vmax;
        rec[0] = pbase;
        rec[1] = vmax;
        rec[2] = k;
        rec[3] = word3;
    }
    uint32_t* codes = rec + 4 + W;
    const uint32_t twoN = codes_per_bin * (uint32_t)bits;  // code bits per kept bin
    for (uint32_t t = tid; t < Tn; t += RT) {
        if (tsurv[t]) {
            codes[(twoN * trank[t]) >> 5] = 0u;
            codes[(twoN * (trank[t] + tsurv[t]) - 1u) >> 5] = 0u;
        }
    }
    const uint32_t code_words = (twoN * k + 31u) >> 5;
    const uint32_t rec_words = (uint32_t)(S / 4) - 4u - W;
    for (uint32_t w = code_words + tid; w < rec_words; w += RT) codes[w] = 0u;

    if (hdr.write && c == 0 && tid < 16) {
        uint32_t v = 0;
        switch (tid) {
            case 0: v = 0x31505346u; break;  // "FSP1"
            case 1: v = 1u; break;
            case 2: v = (uint32_t)hdr.n; break;
            case 3: v = (uint32_t)(hdr.n >> 32); break;
            case 4: v = hdr.L; break;
            case 5: v = hdr.C; break;
            case 6: v = hdr.N; break;
            case 7: v = hdr.m; break;
            case 8: v = hdr.k; break;
            case 9: v = hdr.S; break;
            case 10: v = __float_as_uint(hdr.theta); break;
            case 11: v = hdr.domain; break;
            case 12: v = hdr.scale; break;
            default: break;
        }
        reinterpret_cast<uint32_t*>(stream)[tid] = v;
    }
}

// ------------------------------------------------------------------ emit ----
// Per tile: flags, ranks, Algorithm 1 codes, bit-packing, bitmap words.
template <bool TABLE, bool REAL, bool HALF>
__global__ __launch_bounds__(NT) void k_emit(const typename Stored<REAL, HALF>::T* __restrict__ spec, uint32_t sstride, int pair_log,
                                             uint32_t B, uint32_t Tn, uint32_t W, int bits, int m, size_t S,
                                             const uint32_t* __restrict__ sel, const uint32_t* __restrict__ tscan,
                                             uint8_t* __restrict__ records, TableArg<TABLE> tab, size_t n)
{
    using E = typename Elem<REAL>::T;
    constexpr uint32_t CODES = Elem<REAL>::kCodes;
    __shared__ __align__(16) uint32_t cw[kTile * 2 + 8];  // code words of this tile (bits = 32 worst case), see shw
    __shared__ uint32_t bmw[kTile / 32];
    __shared__ uint32_t weq[4], wfl[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t c = blockIdx.x / Tn;
    const uint32_t tile = blockIdx.x % Tn;
    const uint32_t tau = sel[c * 8 + 2], quota = sel[c * 8 + 3], pbase = sel[c * 8 + 4];
    const uint32_t rank0 = tscan[(c * Tn + tile) * 2 + 0], eq0 = tscan[(c * Tn + tile) * 2 + 1];
    const uint32_t twoN = CODES * (uint32_t)bits;  // code bits per kept bin
    const int shift = 23 - m;
    const uint32_t lds_words = (uint32_t)kTile * twoN / 32u + 2u + 3u;

    // the spectrum tile is staged in the LDS words that later hold the packed codes
    const typename Stored<REAL, HALF>::T* X = spec + c * (size_t)sstride;
    E* stage = reinterpret_cast<E*>(cw);
    static_assert(sizeof(cw) >= kTile * sizeof(float2), "the code buffer doubles as the tile staging area");
    const uint32_t tbase = tile * kTile;
    if constexpr (REAL)
        tile_to_lds(X, tbase, present_of<REAL>(n, c, B), stage, tid);
    else
        tile_to_lds(X, tbase, B - tbase < (uint32_t)kTile ? B - tbase : (uint32_t)kTile, sstride, stage, tid);
    __syncthreads();
    const uint32_t j0 = tbase + wave * WAVE_BINS + lane;
    const RowSlots slots = row_slots(j0, tbase, pair_log);
    E z[ROWS];
    uint64_t em[ROWS], fm[ROWS];
    uint32_t neq = 0, gtbits = 0, eqbits = 0;  // bit r = this lane's bin of row r is above / equal to the threshold
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const uint32_t j = j0 + r * 64;
        const bool valid = j < B;
        z[r] = valid ? stage[slot_of(slots, r, j0, tbase, pair_log)] : Elem<REAL>::zero();
        const uint32_t key = key_of(z[r]);
        const bool gt = valid && key > tau, eq = valid && key == tau;
        gtbits |= (uint32_t)gt << r;
        eqbits |= (uint32_t)eq << r;
        em[r] = __ballot(eq);
        neq += (uint32_t)__popcll(em[r]);
    }
    if (lane == 0) weq[wave] = neq;
    __syncthreads();  // every lane has taken its bins out of the staging area
    for (uint32_t i = tid; i < lds_words; i += NT) cw[i] = 0u;  // ordered before the code writes by the next barrier
    uint32_t eqrun = eq0;
    for (int w = 0; w < wave; ++w) eqrun += weq[w];
    uint32_t nfl = 0, flbits = 0;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        bool flag = (gtbits >> r) & 1u;
        if (em[r]) {  // wave-uniform: ties are rare, skip their bookkeeping otherwise
            flag = flag || (((eqbits >> r) & 1u) && eqrun + prefix_popc(em[r]) < quota);
            eqrun += (uint32_t)__popcll(em[r]);
        }
        flbits |= (uint32_t)flag << r;
        fm[r] = __ballot(flag);
        nfl += (uint32_t)__popcll(fm[r]);
    }
    if (lane == 0) {
        wfl[wave] = nfl;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            bmw[(wave * ROWS + r) * 2 + 0] = (uint32_t)fm[r];
            bmw[(wave * ROWS + r) * 2 + 1] = (uint32_t)(fm[r] >> 32);
        }
    }
    __syncthreads();
    uint32_t rank = rank0;
    for (int w = 0; w < wave; ++w) rank += wfl[w];
    const uint32_t total = wfl[0] + wfl[1] + wfl[2] + wfl[3];
    const uint32_t w0 = (twoN * rank0) >> 5;
    uint32_t* rec = reinterpret_cast<uint32_t*>(records + record_offset<TABLE>(tab, c, S));
    uint32_t* bitmap = rec + 4;
    uint32_t* codes = bitmap + W;
    // The tile's code words are built in LDS at cw[shw + i] for the record's word w0 + i, with shw chosen so that an
    // LDS word and its place in memory are aligned alike: whole 16-byte groups then go out as one store each.
    const uint32_t shw = (uint32_t)((reinterpret_cast<uintptr_t>(codes + w0) >> 2) & 3u);
    // the one or two binary32 patterns a bin is coded from
    auto part = [](const E& v, int h) __attribute__((always_inline)) {
        if constexpr (REAL)
            return __float_as_uint(v);
        else
            return __float_as_uint(h ? v.y : v.x);
    };
    if (bits == 8) {
        // 8-bit codes: a survivor is one aligned 16-bit store (bin) or one byte (sample), no read-modify-write
        uint16_t* cw16 = reinterpret_cast<uint16_t*>(cw);
        uint8_t* cw8 = reinterpret_cast<uint8_t*>(cw);
        const uint32_t base16 = rank0 - 2u * w0 + 2u * shw;  // first survivor's 16-bit slot inside cw (two codes each)
        const uint32_t base8 = rank0 - 4u * w0 + 4u * shw;   // first survivor's byte inside cw (one code each)
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if ((flbits >> r) & 1u) {
                const uint32_t rk = rank + prefix_popc(fm[r]);
                const uint32_t cre = quantize(part(z[r], 0), pbase, 8, shift);
                if constexpr (REAL) {
                    cw8[base8 + (rk - rank0)] = (uint8_t)cre;
                } else {
                    const uint32_t cim = quantize(part(z[r], 1), pbase, 8, shift);
                    cw16[base16 + (rk - rank0)] = (uint16_t)(cre | (cim << 8));
                }
            }
            rank += (uint32_t)__popcll(fm[r]);
        }
    } else {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if ((flbits >> r) & 1u) {
                const uint32_t rk = rank + prefix_popc(fm[r]);
                const uint32_t cre = quantize(part(z[r], 0), pbase, bits, shift);
                const uint32_t cim = quantize(part(z[r], 1), pbase, bits, shift);
                uint32_t p = twoN * rk - (w0 << 5) + (shw << 5);  // bit position inside cw
#pragma unroll
                for (int h = 0; h < (int)CODES; ++h) {
                    const uint32_t code = h ? cim : cre;
                    const uint32_t wi = p >> 5, sh = p & 31u;
                    atomicOr(&cw[wi], code << sh);
                    if (sh + (uint32_t)bits > 32u) atomicOr(&cw[wi + 1], code >> (32u - sh));
                    p += (uint32_t)bits;
                }
            }
            rank += (uint32_t)__popcll(fm[r]);
        }
    }
    __syncthreads();
    if (tid < kTile / 32) {
        const uint32_t wi = tile * (kTile / 32) + tid;
        if (wi < W) bitmap[wi] = bmw[tid];
    }
    if (total) {
        const uint32_t w1 = (twoN * (rank0 + total) - 1u) >> 5;
        const uint32_t rec_words = (uint32_t)(S / 4) - 4u - W;  // code words the record has room for
        const uint32_t nw_all = w1 - w0 + 1u;
        const uint32_t nw = w0 >= rec_words ? 0u : (nw_all < rec_words - w0 ? nw_all : rec_words - w0);
        // group g = LDS words 4g .. 4g+3 = record words w0 - shw + 4g .. (16-byte aligned in memory)
        const uint32_t groups = (shw + nw + 3u) >> 2;
        uint32_t* gbase = codes + w0 - shw;
        for (uint32_t g = tid; g < groups; g += NT) {
            const uint32_t i0 = 4u * g;  // LDS index of the group's first word; its tile word index is i0 - shw
            if (i0 >= shw + 1u && i0 + 3u + 1u < shw + nw) {
                // all four words lie strictly inside the tile's run
                *reinterpret_cast<uint4*>(gbase + i0) = *reinterpret_cast<const uint4*>(cw + i0);
            } else {
#pragma unroll
                for (uint32_t j = 0; j < 4u; ++j) {
                    const uint32_t li = i0 + j;
                    if (li < shw || li >= shw + nw) continue;
                    const uint32_t i = li - shw, v = cw[li];
                    if (i == 0 || i == nw - 1u)
                        atomicOr(&codes[w0 + i], v);  // may be shared with the neighbouring tile (zeroed by k_resolve)
                    else
                        codes[w0 + i] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------- decode ----
constexpr int GROUP_WORDS = 16;  // one wave of the decode kernel covers 512 bins = 16 bitmap words

// Per chunk: number of set bits before each group of 16 bitmap words (the prefix sum of Sec. 3.2's status
// vector, kept at the granularity a wave needs); checks the headers and leaves the verdict in *verdict.
__device__ __forceinline__ void group_prefix_chunk(const uint8_t* __restrict__ stream, const uint8_t* __restrict__ record,
                                                   bool first_of_stream, uint32_t W, uint32_t k, uint32_t word3,
                                                   const HeaderInfo& hdr, uint32_t* __restrict__ gprefix,
                                                   uint32_t* __restrict__ verdict)
{
    __shared__ uint32_t tmp[RW];
    __shared__ uint32_t s_carry;
    const int tid = threadIdx.x;
    const uint32_t* rec = reinterpret_cast<const uint32_t*>(record);
    const uint32_t* bitmap = rec + 4;
    const uint32_t G = (W + GROUP_WORDS - 1) / GROUP_WORDS;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    // set bits of one group of 16 words
    auto group_count = [&](uint32_t g) {
        uint32_t cnt = 0;
        if (g < G) {
            const uint32_t w0 = g * GROUP_WORDS;
            if (w0 + GROUP_WORDS <= W) {
                const uint4* p = reinterpret_cast<const uint4*>(bitmap + w0);  // records and bitmaps are 16-byte aligned
#pragma unroll
                for (int i = 0; i < GROUP_WORDS / 4; ++i) {
                    const uint4 v = p[i];
                    cnt += (uint32_t)(__popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w));
                }
            } else {
                for (uint32_t w = w0; w < W; ++w) cnt += (uint32_t)__popc(bitmap[w]);
            }
        }
        return cnt;
    };
    // two adjacent groups per lane, so that the longest chunk (1025 groups) is one scan, not two
    for (uint32_t base = 0; base < G; base += 2 * RT) {
        const uint32_t g = base + 2 * (uint32_t)tid;
        const uint32_t cnt0 = group_count(g), cnt1 = group_count(g + 1);
        const uint32_t carry = s_carry;
        const uint32_t incl = block_scan_incl_1024(cnt0 + cnt1, tmp);
        const uint32_t before = carry + incl - cnt0 - cnt1;
        if (g < G) gprefix[g] = before;
        if (g + 1 < G) gprefix[g + 1] = before + cnt0;
        __syncthreads();
        if (tid == RT - 1) s_carry = carry + incl;
        __syncthreads();
    }
    if (tid == 0) {
        bool bad = s_carry != k || rec[2] != k || rec[3] != word3;
        if (hdr.write && first_of_stream) {
            const uint32_t* h = reinterpret_cast<const uint32_t*>(stream);
            bad = bad || h[0] != 0x31505346u || h[1] != 1u || h[2] != (uint32_t)hdr.n ||
                  h[3] != (uint32_t)(hdr.n >> 32) || h[4] != hdr.L || h[5] != hdr.C || h[6] != hdr.N ||
                  h[7] != hdr.m || h[8] != hdr.k || h[9] != hdr.S || h[11] != hdr.domain || h[12] != hdr.scale;
        }
        *verdict = bad ? 6u : 0u;
    }
}

template <bool TABLE>
__global__ __launch_bounds__(RT) void k_group_prefix(const uint8_t* __restrict__ stream,
                                                     const uint8_t* __restrict__ records, size_t S, uint32_t W,
                                                     uint32_t k, uint32_t word3, HeaderInfo hdr,
                                                     uint32_t* __restrict__ gprefix, uint32_t* __restrict__ sel,
                                                     uint32_t* __restrict__ status, int reset_status,
                                                     TableArg<TABLE> tab)
{
    const size_t c = blockIdx.x;
    const uint32_t G = (W + GROUP_WORDS - 1) / GROUP_WORDS;
    group_prefix_chunk(stream, records + record_offset<TABLE>(tab, c, S), c == 0, W, k, word3, hdr, gprefix + c * G,
                       sel + c * 8 + 7);
    // The whole control block is cleared: the status word (raised again by k_decode, which runs after this kernel)
    // and the hand-over words of the fused inverse transform that may follow.
    if (reset_status && c == 0)
        for (uint32_t i = threadIdx.x; i < (uint32_t)(kControlBytes / 4); i += RT) status[i] = 0u;
}

// The same for several peers' streams: workgroup (peer, chunk).
__global__ __launch_bounds__(RT) void k_group_prefix_peers(PeerList streams, uint32_t C, size_t S, uint32_t W, uint32_t k,
                                                           HeaderInfo hdr, uint32_t* __restrict__ gprefix,
                                                           uint32_t* __restrict__ verd, uint32_t* __restrict__ status)
{
    const uint32_t peer = blockIdx.x / C, c = blockIdx.x % C;
    const uint32_t G = (W + GROUP_WORDS - 1) / GROUP_WORDS;
    const uint8_t* stream = streams.p[peer];
    group_prefix_chunk(stream, stream + 64 + (size_t)c * S, c == 0, W, k, 0u, hdr,
                       gprefix + ((size_t)peer * C + c) * G, verd + (size_t)peer * C + c);
    if (blockIdx.x == 0)  // the whole control block, as k_group_prefix does
        for (uint32_t i = threadIdx.x; i < (uint32_t)(kControlBytes / 4); i += RT) status[i] = 0u;
}

// Persistent decoder.  A workgroup walks tiles of 2048 bins (blockIdx, blockIdx + grid, ...), one wave per
// group of 16 bitmap words.  The kept bins of a wave's 512 bins have consecutive ranks, so their codes are one
// contiguous byte range of the record: the wave fetches that range with 16-byte loads into its own LDS window
// and picks the codes out of LDS by rank (a per-bin gather from global memory costs one memory instruction per
// row of 64 bins and was measured at a quarter of the kernel's time).  The work on a tile is a chain of two
// dependent memory round trips (bitmap word and group prefix, then the codes) before anything can be stored, so
// the kernel is software-pipelined: while one item is dequantised, the codes of the next and the bitmap words
// of the one after are in flight.  All loads are unconditional (clamped to addresses inside the record).
//
// With P > 1 peers (receiver under an allgather: Sec. 4, implementation) an item is (tile, peer): a tile's bins
// are summed over the peers in list order in registers, starting from zero, and stored once.
struct DecHead {
    uint32_t word, run, pbase;  // this lane's bitmap word (lanes 0..15), kept bins before the wave's group, record pbase
};

// NL = 16-byte loads per lane: 1 for codes of up to 8 bits, 2 up to 16, 4 for 32
template <int NL>
struct DecCodes {
    u32x4 main[NL];
    u32x4 tail;  // lane 0: the 16 bytes behind the main window (the window starts on a 16-byte boundary <= the first code)
};

struct DecItem {
    uint32_t t, peer;  // tile index over all chunks, index into the peer list
};

// VEC: the spectrum buffer is the codec's own (chunks padded to 16 bins, 16-byte aligned): whole-line stores, and
// the one bin a partial tile may write past the chunk's last bin lands in the padding.
// verd: header verdict of (peer, chunk) at verd[peer * C + chunk].
// One stream.
// REAL: time-domain records (one code per kept sample); `spec` is then the gradient itself, chunk stride B = L
// samples, written up to sample n only.
// HALF: the spectrum is written as binary16 pairs (half-precision variant).
template <int NL, bool VEC, bool TABLE, bool REAL, bool HALF>
__global__ __launch_bounds__(NT) void k_decode(const uint8_t* __restrict__ records, size_t S, uint32_t B, uint32_t W,
                                               uint32_t k, int bits, int m, uint32_t Tn, uint32_t total, size_t C,
                                               const uint32_t* __restrict__ gprefix, const uint32_t* __restrict__ sel,
                                               uint32_t* __restrict__ status,
                                               typename Stored<REAL, HALF>::T* __restrict__ spec, uint32_t sstride,
                                               int pair_log, TableArg<TABLE> tab, size_t n)
{
    using E = typename Elem<REAL>::T;
    constexpr uint32_t CODES = Elem<REAL>::kCodes;
    constexpr int kWin = NL * 1024 + 32;  // bytes of LDS per wave: main window, tail, slack for the 3-word read
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // header verdicts of k_group_prefix raise the status word
    for (size_t c = (size_t)blockIdx.x * NT + tid; c < C; c += (size_t)gridDim.x * NT) {
        const uint32_t verdict = sel[c * 8 + 7];
        if (verdict) atomicMax(status, verdict);
    }
    const uint32_t G = (W + GROUP_WORDS - 1) / GROUP_WORDS;
    const int shift = 23 - m;
    const uint32_t code_base = 16u + 4u * W;  // byte offset of the codes inside a record
    __shared__ __attribute__((aligned(16))) E stage[kTile];
    __shared__ __attribute__((aligned(16))) uint8_t cwin_all[4 * kWin];
    uint8_t* cwin = cwin_all + wave * kWin;

    auto record_of = [&](uint32_t t) __attribute__((always_inline)) {
        return records + record_offset<TABLE>(tab, t / Tn, S);
    };
    auto load_head = [&](uint32_t t, bool live) __attribute__((always_inline)) {
        if (!live) t = 0;
        const uint32_t* rec = reinterpret_cast<const uint32_t*>(record_of(t));
        const uint32_t g = (t % Tn) * (kTile / 32 / GROUP_WORDS) + wave;
        const uint32_t wi = g * GROUP_WORDS + lane;
        const bool has = live && lane < GROUP_WORDS && wi < W;
        DecHead h;
        h.word = rec[4 + (has ? wi : 0u)];
        h.run = gprefix[(size_t)(t / Tn) * G + (g < G ? g : 0u)];
        h.pbase = rec[0];
        if (!has) h.word = 0u;
        return h;
    };
    // rank of this lane's bin in row r if its bit is set; advances run past the row
    auto row_rank = [&](const DecHead& h, int r, uint32_t& run, bool& set) __attribute__((always_inline)) {
        const uint32_t lo = __shfl(h.word, 2 * r, 64), hi = __shfl(h.word, 2 * r + 1, 64);
        const uint64_t mask = (uint64_t)lo | ((uint64_t)hi << 32);
        const uint32_t half = lane < 32 ? lo : hi;
        set = ((half >> (lane & 31)) & 1u) && k > 0;
        uint32_t rank = run + prefix_popc(mask);
        run += (uint32_t)__popcll(mask);
        return rank < k ? rank : (k ? k - 1u : 0u);  // a corrupt bitmap must not point outside the record
    };
    // first byte of the wave's LDS window inside the record: the 16-byte boundary at or below its first code
    auto window_start = [&](const DecHead& h) __attribute__((always_inline)) {
        const uint32_t first = h.run < k ? h.run : (k ? k - 1u : 0u);
        return (code_base + ((CODES * (uint32_t)bits * first) >> 3)) & ~15u;
    };
    auto load_codes = [&](uint32_t t, bool live, const DecHead& h, DecCodes<NL>& cd) __attribute__((always_inline)) {
        if (!live) t = 0;
        const uint8_t* rec = record_of(t);
        const uint32_t start = window_start(h), last = (uint32_t)S - 16u;  // S is a multiple of 16, at least 32
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const uint32_t off = start + (uint32_t)(i * 1024 + lane * 16);
            cd.main[i] = *reinterpret_cast<const u32x4*>(rec + (off < last ? off : last));
        }
        const uint32_t off = start + (uint32_t)(NL * 1024);
        cd.tail = *reinterpret_cast<const u32x4*>(rec + (off < last ? off : last));
    };
    auto finish = [&](uint32_t t, const DecHead& h, const DecCodes<NL>& cd) __attribute__((always_inline)) {
        const uint32_t tile = t % Tn, tbase = tile * kTile;
        const uint32_t j0 = tbase + wave * WAVE_BINS + lane;
        const RowSlots slots = row_slots(j0, tbase, pair_log);
#pragma unroll
        for (int i = 0; i < NL; ++i) *reinterpret_cast<u32x4*>(cwin + i * 1024 + lane * 16) = cd.main[i];
        if (lane == 0) *reinterpret_cast<u32x4*>(cwin + NL * 1024) = cd.tail;
        __syncthreads();  // codes visible to the wave; the previous tile's stage has been read by everyone
        const uint32_t start = window_start(h);
        uint32_t run = h.run;
        // The tile's bins occupy one contiguous range of the spectrum buffer in either bin order (paired runs are
        // tile-aligned), so values are placed in LDS at their in-tile position and written out as whole lines.
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            bool set;
            const uint32_t rank = row_rank(h, r, run, set);
            E out = Elem<REAL>::zero();
            if (set) {
                const uint32_t p = CODES * (uint32_t)bits * rank;             // bit offset of the bin's codes
                uint32_t cre, cim = 0u;
                if (bits == 8) {
                    if constexpr (REAL) {
                        cre = cwin[code_base + (p >> 3) - start];
                    } else {
                        const uint32_t v = *reinterpret_cast<const uint16_t*>(cwin + (code_base + (p >> 3) - start));
                        cre = v & 0xFFu;
                        cim = v >> 8;
                    }
                } else {
                    const uint32_t* w = reinterpret_cast<const uint32_t*>(cwin + (code_base + 4u * (p >> 5) - start));
                    const uint32_t keep = bits == 32 ? 0xFFFFFFFFu : ((1u << bits) - 1u);
                    const uint32_t sh = p & 31u;
                    if constexpr (REAL) {
                        const uint64_t w01 = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
                        cre = (uint32_t)(w01 >> sh) & keep;
                    } else {
                        const uint32_t w0 = w[0], w1 = w[1], w2 = w[2];
                        const uint32_t q = sh + (uint32_t)bits;
                        const uint64_t w01 = (uint64_t)w0 | ((uint64_t)w1 << 32), w12 = (uint64_t)w1 | ((uint64_t)w2 << 32);
                        cre = (uint32_t)(w01 >> sh) & keep;
                        cim = (uint32_t)((q >= 32u ? w12 : w01) >> (q & 31u)) & keep;
                    }
                }
                if constexpr (REAL) {
                    out = __uint_as_float(dequantize(cre, h.pbase, bits, shift));
                } else {
                    out.x = __uint_as_float(dequantize(cre, h.pbase, bits, shift));
                    out.y = __uint_as_float(dequantize(cim, h.pbase, bits, shift));
                }
            }
            const uint32_t j = j0 + r * 64;
            if (j < B) stage[slot_of(slots, r, j0, tbase, pair_log)] = out;
        }
        __syncthreads();
        typename Stored<REAL, HALF>::T* X = spec + (size_t)(t / Tn) * (size_t)sstride;
        if constexpr (REAL) {
            // samples of this tile that exist in the gradient (the last chunk may end inside or before the tile)
            const uint32_t present = present_of<REAL>(n, t / Tn, B);
            const uint32_t count = present > tbase ? (present - tbase < (uint32_t)kTile ? present - tbase : (uint32_t)kTile) : 0u;
            if (VEC && count == (uint32_t)kTile) {
                float4* dst = reinterpret_cast<float4*>(X + tbase);
                const float4* src = reinterpret_cast<const float4*>(stage);
#pragma unroll
                for (int i = 0; i < kTile / 4 / NT; ++i) dst[tid + i * NT] = src[tid + i * NT];
            } else {
                for (uint32_t i = tid; i < count; i += NT) X[tbase + i] = stage[i];
            }
        } else if constexpr (HALF) {
            const uint32_t count = B - tbase < (uint32_t)kTile ? B - tbase : (uint32_t)kTile;
            if constexpr (VEC) {  // four bins per 16-byte store; up to three land in the chunk's padding
                uint4* dst = reinterpret_cast<uint4*>(X + tbase);
                const float4* src = reinterpret_cast<const float4*>(stage);
#pragma unroll
                for (int i = 0; i < kTile / 4 / NT; ++i) {
                    const uint32_t idx = (uint32_t)(tid + i * NT);
                    if (4u * idx < count) {
                        const uint2 a = cx_store<true>(src[2 * idx]), b = cx_store<true>(src[2 * idx + 1]);
                        dst[idx] = make_uint4(a.x, a.y, b.x, b.y);
                    }
                }
            } else {
                for (uint32_t i = tid; i < count; i += NT) X[tbase + i] = pack_half2(stage[i]);
            }
        } else {
            const uint32_t count = B - tbase < (uint32_t)kTile ? B - tbase : (uint32_t)kTile;
            if constexpr (VEC) {
                float4* dst = reinterpret_cast<float4*>(X + tbase);
                const float4* src = reinterpret_cast<const float4*>(stage);
#pragma unroll
                for (int i = 0; i < kTile / 2 / NT; ++i) {
                    const uint32_t idx = (uint32_t)(tid + i * NT);
                    if (2u * idx < count) dst[idx] = src[idx];
                }
            } else {
                for (uint32_t i = tid; i < count; i += NT) X[tbase + i] = stage[i];
            }
        }
    };

    // Three register sets rotate by name through a loop body written out three times: rotating by assignment
    // would copy registers that loads are still filling, and a copy waits for its load.
    uint32_t t = blockIdx.x;
    const uint32_t step = gridDim.x;
    if (t >= total) return;
    DecHead h0, h1, h2;
    DecCodes<NL> c0, c1, c2;
    // tile t is in (hc, cc), tile t+1 in (hn, cn); fetches what tiles t+1 and t+2 need, then finishes tile t
    auto advance = [&](const DecHead& hc, const DecCodes<NL>& cc, const DecHead& hn, DecCodes<NL>& cn, DecHead& hn2) __attribute__((always_inline)) {
        const bool more = t + step < total;
        const bool more2 = more && t + 2 * step < total;
        hn2 = load_head(more2 ? t + 2 * step : 0u, more2);
        load_codes(more ? t + step : 0u, more, hn, cn);
        finish(t, hc, cc);
        t += step;
        return more;
    };
    h0 = load_head(t, true);
    h1 = load_head(t + step, t + step < total);
    load_codes(t, true, h0, c0);
    for (;;) {
        if (!advance(h0, c0, h1, c1, h2)) break;
        if (!advance(h1, c1, h2, c2, h0)) break;
        if (!advance(h2, c2, h0, c0, h1)) break;
    }
}

// The decoder for several peers' streams: same pipeline, items are (tile, peer).
template <int NL, bool VEC>
__global__ __launch_bounds__(NT) void k_decode_peers(PeerList recs, uint32_t npeers, size_t S, uint32_t B, uint32_t W,
                                               uint32_t k, int bits, int m, uint32_t Tn, uint32_t total, size_t C,
                                               const uint32_t* __restrict__ gprefix, const uint32_t* __restrict__ verd,
                                               uint32_t* __restrict__ status,
                                               float2* __restrict__ spec, uint32_t sstride, int pair_log)
{
    constexpr int kWin = NL * 1024 + 32;  // bytes of LDS per wave: main window, tail, slack for the 3-word read
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t P = npeers;
    // header verdicts of the group-prefix kernel raise the status word
    for (size_t i = (size_t)blockIdx.x * NT + tid; i < C * P; i += (size_t)gridDim.x * NT) {
        const uint32_t verdict = verd[i];
        if (verdict) atomicMax(status, verdict);
    }
    const uint32_t G = (W + GROUP_WORDS - 1) / GROUP_WORDS;
    const int shift = 23 - m;
    const uint32_t code_base = 16u + 4u * W;  // byte offset of the codes inside a record
    __shared__ float2 stage[kTile];
    __shared__ __attribute__((aligned(16))) uint8_t cwin_all[4 * kWin];
    uint8_t* cwin = cwin_all + wave * kWin;
    const uint32_t step = gridDim.x;

    auto record_of = [&](DecItem it) __attribute__((always_inline)) {
        return recs.p[it.peer] + (size_t)(it.t / Tn) * S;
    };
    auto next_item = [&](DecItem it) __attribute__((always_inline)) {
        DecItem n;
        const bool last_peer = it.peer + 1u == P;
        n.peer = last_peer ? 0u : it.peer + 1u;
        n.t = last_peer ? it.t + step : it.t;
        return n;
    };
    // live = false: the item does not exist; the loads are still issued, to item (0, 0)
    auto load_head = [&](DecItem it, bool live) __attribute__((always_inline)) {
        if (!live) it.t = it.peer = 0;
        const uint32_t* rec = reinterpret_cast<const uint32_t*>(record_of(it));
        const uint32_t g = (it.t % Tn) * (kTile / 32 / GROUP_WORDS) + wave;
        const uint32_t wi = g * GROUP_WORDS + lane;
        const bool has = live && lane < GROUP_WORDS && wi < W;
        DecHead h;
        h.word = rec[4 + (has ? wi : 0u)];
        h.run = gprefix[((size_t)it.peer * C + it.t / Tn) * G + (g < G ? g : 0u)];
        h.pbase = rec[0];
        if (!has) h.word = 0u;
        return h;
    };
    // rank of this lane's bin in row r if its bit is set; advances run past the row
    auto row_rank = [&](const DecHead& h, int r, uint32_t& run, bool& set) __attribute__((always_inline)) {
        const uint32_t lo = __shfl(h.word, 2 * r, 64), hi = __shfl(h.word, 2 * r + 1, 64);
        const uint64_t mask = (uint64_t)lo | ((uint64_t)hi << 32);
        const uint32_t half = lane < 32 ? lo : hi;
        set = ((half >> (lane & 31)) & 1u) && k > 0;
        uint32_t rank = run + prefix_popc(mask);
        run += (uint32_t)__popcll(mask);
        return rank < k ? rank : (k ? k - 1u : 0u);  // a corrupt bitmap must not point outside the record
    };
    // first byte of the wave's LDS window inside the record: the 16-byte boundary at or below its first code
    auto window_start = [&](const DecHead& h) __attribute__((always_inline)) {
        const uint32_t first = h.run < k ? h.run : (k ? k - 1u : 0u);
        return (code_base + ((2u * (uint32_t)bits * first) >> 3)) & ~15u;
    };
    auto load_codes = [&](DecItem it, bool live, const DecHead& h, DecCodes<NL>& cd) __attribute__((always_inline)) {
        if (!live) it.t = it.peer = 0;
        const uint8_t* rec = record_of(it);
        const uint32_t start = window_start(h), last = (uint32_t)S - 16u;  // S is a multiple of 16, at least 32
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const uint32_t off = start + (uint32_t)(i * 1024 + lane * 16);
            cd.main[i] = *reinterpret_cast<const u32x4*>(rec + (off < last ? off : last));
        }
        const uint32_t off = start + (uint32_t)(NL * 1024);
        cd.tail = *reinterpret_cast<const u32x4*>(rec + (off < last ? off : last));
    };
    float2 acc[ROWS];  // this lane's bins of the tile being summed over the peers
    auto finish = [&](DecItem it, const DecHead& h, const DecCodes<NL>& cd) __attribute__((always_inline)) {
        const uint32_t tile = it.t % Tn, tbase = tile * kTile;
        const uint32_t j0 = tbase + wave * WAVE_BINS + lane;
        const RowSlots slots = row_slots(j0, tbase, pair_log);
#pragma unroll
        for (int i = 0; i < NL; ++i) *reinterpret_cast<u32x4*>(cwin + i * 1024 + lane * 16) = cd.main[i];
        if (lane == 0) *reinterpret_cast<u32x4*>(cwin + NL * 1024) = cd.tail;
        __syncthreads();  // codes visible to the wave; the previous tile's stage has been read by everyone
        const uint32_t start = window_start(h);
        uint32_t run = h.run;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            bool set;
            const uint32_t rank = row_rank(h, r, run, set);
            float2 out = make_float2(0.f, 0.f);
            if (set) {
                const uint32_t p = 2u * (uint32_t)bits * rank;                // bit offset of the pair in the codes
                uint32_t cre, cim;
                if (bits == 8) {
                    const uint32_t v = *reinterpret_cast<const uint16_t*>(cwin + (code_base + (p >> 3) - start));
                    cre = v & 0xFFu;
                    cim = v >> 8;
                } else {
                    const uint32_t* w = reinterpret_cast<const uint32_t*>(cwin + (code_base + 4u * (p >> 5) - start));
                    const uint32_t w0 = w[0], w1 = w[1], w2 = w[2];
                    const uint32_t sh = p & 31u, q = sh + (uint32_t)bits;
                    const uint64_t w01 = (uint64_t)w0 | ((uint64_t)w1 << 32), w12 = (uint64_t)w1 | ((uint64_t)w2 << 32);
                    const uint32_t keep = bits == 32 ? 0xFFFFFFFFu : ((1u << bits) - 1u);
                    cre = (uint32_t)(w01 >> sh) & keep;
                    cim = (uint32_t)((q >= 32u ? w12 : w01) >> (q & 31u)) & keep;
                }
                out.x = __uint_as_float(dequantize(cre, h.pbase, bits, shift));
                out.y = __uint_as_float(dequantize(cim, h.pbase, bits, shift));
            }
            const float2 prev = it.peer == 0 ? make_float2(0.f, 0.f) : acc[r];
            acc[r] = make_float2(prev.x + out.x, prev.y + out.y);
        }
        if (it.peer + 1u != P) {
            __syncthreads();  // every lane has picked its codes before the next item overwrites the window
            return;
        }
        // The tile's bins occupy one contiguous range of the spectrum buffer in either bin order (paired runs are
        // tile-aligned), so the sums are placed in LDS at their in-tile position and written out as whole lines.
#pragma unroll
        for (int r = 0; r < ROWS; ++r)
            if (j0 + (uint32_t)r * 64u < B) stage[slot_of(slots, r, j0, tbase, pair_log)] = acc[r];
        __syncthreads();
        float2* X = spec + (size_t)(it.t / Tn) * (size_t)sstride;
        const uint32_t count = B - tbase < (uint32_t)kTile ? B - tbase : (uint32_t)kTile;
        if constexpr (VEC) {
            float4* dst = reinterpret_cast<float4*>(X + tbase);
            const float4* src = reinterpret_cast<const float4*>(stage);
#pragma unroll
            for (int i = 0; i < kTile / 2 / NT; ++i) {
                const uint32_t idx = (uint32_t)(tid + i * NT);
                if (2u * idx < count) dst[idx] = src[idx];
            }
        } else {
            for (uint32_t i = tid; i < count; i += NT) X[tbase + i] = stage[i];
        }
    };

    // Three register sets rotate by name through a loop body written out three times: rotating by assignment
    // would copy registers that loads are still filling, and a copy waits for its load.
    DecItem cur;
    cur.t = blockIdx.x;
    cur.peer = 0;
    if (cur.t >= total) return;
    DecHead h0, h1, h2;
    DecCodes<NL> c0, c1, c2;
    // item `cur` is in (hc, cc), the next one in (hn, cn); fetches what the next two items need, then finishes cur
    auto advance = [&](const DecHead& hc, const DecCodes<NL>& cc, const DecHead& hn, DecCodes<NL>& cn, DecHead& hn2) __attribute__((always_inline)) {
        const DecItem nxt = next_item(cur), nx2 = next_item(nxt);
        const bool more = nxt.t < total, more2 = more && nx2.t < total;
        hn2 = load_head(nx2, more2);
        load_codes(nxt, more, hn, cn);
        finish(cur, hc, cc);
        cur = nxt;
        return more;
    };
    h0 = load_head(cur, true);
    {
        const DecItem nxt = next_item(cur);
        h1 = load_head(nxt, nxt.t < total);
    }
    load_codes(cur, true, h0, c0);
    for (;;) {
        if (!advance(h0, c0, h1, c1, h2)) break;
        if (!advance(h1, c1, h2, c2, h0)) break;
        if (!advance(h2, c2, h0, c0, h1)) break;
    }
}

}  // namespace

// status words and histograms are adjacent: one fill
static hipError_t launch_zero_hist(uint8_t* ws_base, const Workspace& w, size_t C, hipStream_t s)
{
    uint32_t* status = reinterpret_cast<uint32_t*>(ws_base + w.status);
    const size_t zero_words = (w.hist - w.status) / 4 + C * kHistBins;
    FFTSP_LAUNCH("zero_fill", k_zero_u32, dim3((unsigned)((zero_words + 255) / 256)), dim3(256), 0, s, status,
                 zero_words);
    return hipGetLastError();
}

hipError_t launch_zero_control(uint8_t* ws_base, const Workspace& w, size_t C, hipStream_t s)
{
    return launch_zero_hist(ws_base, w, C, s);
}

hipError_t launch_clear_status(uint8_t* ws_base, const Workspace& w, hipStream_t s)
{
    FFTSP_LAUNCH("zero_fill", k_zero_u32, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(ws_base + w.status),
                 (size_t)1);
    return hipGetLastError();
}

hipError_t launch_encode(const float* spec, const CodecArgs& a, uint8_t* stream_base, uint8_t* records,
                         uint8_t* ws_base, const Workspace& w, int hist_ready, hipStream_t s)
{
    const uint32_t B = codec_bins(a.L, a.time_domain), Tn = codec_tiles(a.L, a.time_domain), W = (B + 31) / 32;
    const float2* X = reinterpret_cast<const float2*>(spec);
    uint32_t* hist = reinterpret_cast<uint32_t*>(ws_base + w.hist);
    uint32_t* sel = reinterpret_cast<uint32_t*>(ws_base + w.sel);
    uint32_t* tinfo = reinterpret_cast<uint32_t*>(ws_base + w.tinfo);
    uint32_t* tscan = reinterpret_cast<uint32_t*>(ws_base + w.tscan);
    uint2* cand = reinterpret_cast<uint2*>(ws_base + w.cand);
    if (a.C * (size_t)Tn > 0x7fffffffu || Tn > (uint32_t)MAX_TILES) return hipErrorInvalidValue;
    if (a.time_domain && (a.tab || a.pair_log || hist_ready)) return hipErrorInvalidValue;
    // binary16 spectra come from the two-pass FFT only, which also fills the histogram
    if (a.half && (a.tab || a.time_domain || !a.pair_log || !hist_ready)) return hipErrorInvalidValue;
    const uint32_t* Xh = reinterpret_cast<const uint32_t*>(spec);

    if (!hist_ready) {
        hipError_t e = launch_zero_hist(ws_base, w, a.C, s);
        if (e != hipSuccess) return e;
        const uint32_t groups = (Tn + HIST_TILES - 1) / HIST_TILES;
        const uint32_t sgroups = (Tn + kHistSampleTiles - 1) / kHistSampleTiles;
        if (a.time_domain)
            FFTSP_LAUNCH("hist", k_hist_samples, dim3((unsigned)(a.C * sgroups)), dim3(NT), 0, s, spec, a.L, sgroups,
                         hist, a.n);
        else
            FFTSP_LAUNCH("hist", k_hist, dim3((unsigned)(a.C * groups)), dim3(NT), 0, s, X, a.sstride, a.pair_log, B,
                         groups, hist);
    }
    FFTSP_LAUNCH("find_bucket", k_find_bucket, dim3((unsigned)a.C), dim3(NT), 0, s, hist, a.k, sel);
    if (a.time_domain)
        FFTSP_LAUNCH("collect", (k_collect<true, false>), dim3((unsigned)(a.C * Tn)), dim3(NT), 0, s, spec, a.sstride, 0,
                     B, Tn, sel, tinfo, cand, a.n);
    else if (a.half)
        FFTSP_LAUNCH("collect", (k_collect<false, true>), dim3((unsigned)(a.C * Tn)), dim3(NT), 0, s, Xh, a.sstride,
                     a.pair_log, B, Tn, sel, tinfo, cand, a.n);
    else
        FFTSP_LAUNCH("collect", (k_collect<false, false>), dim3((unsigned)(a.C * Tn)), dim3(NT), 0, s, X, a.sstride,
                     a.pair_log, B, Tn, sel, tinfo, cand, a.n);
    HeaderInfo h{a.write_header, a.hdr_n, a.hdr_L, a.hdr_C, (uint32_t)a.bits, (uint32_t)a.m, a.hdr_k, a.hdr_S,
                 a.hdr_theta, a.time_domain ? 1u : 0u, (uint32_t)a.hdr_scale};
    const uint32_t codes_per_bin = a.time_domain ? 1u : 2u;
    // up to 12 Ki candidates (96 KiB) are staged in LDS by the per-chunk workgroup, 24 Ki where keys alone suffice
    constexpr uint32_t kStageCap = 12 * 1024;
    const uint32_t stage_cap = a.time_domain ? 2 * kStageCap : kStageCap;
    {
        // set on every call (a host-side table write): the attribute belongs to the current device, and a flag
        // remembered across calls would be neither per device nor safe between host threads
        const void* fn = a.tab           ? reinterpret_cast<const void*>(k_resolve<true, false>)
                         : a.time_domain ? reinterpret_cast<const void*>(k_resolve<false, true>)
                                         : reinterpret_cast<const void*>(k_resolve<false, false>);
        const hipError_t e =
            hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kStageCap * sizeof(uint2)));
        if (e != hipSuccess) return e;
    }
    if (a.tab && a.C > (size_t)kMaxTableChunks) return hipErrorInvalidValue;
#define FFTSP_RESOLVE(TABLE, KEYS)                                                                                    \
    FFTSP_LAUNCH("resolve", (k_resolve<TABLE, KEYS>), dim3((unsigned)a.C), dim3(RT), kStageCap * sizeof(uint2), s, Tn, \
                 a.k, a.bits, a.m, W, a.S, a.word3, stage_cap, a.static_vmax, codes_per_bin, sel, tinfo, tscan, cand,  \
                 records, stream_base, h, table_arg<TABLE>(a.tab))
#define FFTSP_EMIT(TABLE, REAL, HALF, src)                                                                            \
    FFTSP_LAUNCH("emit", (k_emit<TABLE, REAL, HALF>), dim3((unsigned)(a.C * Tn)), dim3(NT), 0, s, src, a.sstride,     \
                 a.pair_log, B, Tn, W, a.bits, a.m, a.S, sel, tscan, records, table_arg<TABLE>(a.tab), a.n)
    if (a.tab) {
        FFTSP_RESOLVE(true, false);
        FFTSP_EMIT(true, false, false, X);
    } else {
        if (a.time_domain)
            FFTSP_RESOLVE(false, true);
        else
            FFTSP_RESOLVE(false, false);
        if (a.time_domain)
            FFTSP_EMIT(false, true, false, spec);
        else if (a.half)
            FFTSP_EMIT(false, false, true, Xh);
        else
            FFTSP_EMIT(false, false, false, X);
    }
#undef FFTSP_RESOLVE
#undef FFTSP_EMIT
    return hipGetLastError();
}

// the decode kernel proper: one stream with its verdicts in the sel array (chunk c: word 8c+7), or the peer
// list with verdicts at verd[peer * C + c]
static hipError_t launch_decode_kernel(const PeerList& recs, uint32_t npeers, const CodecArgs& a, float* spec,
                                       const uint32_t* gprefix, const uint32_t* verd, uint32_t* status, bool peers_layout,
                                       hipStream_t s)
{
    const uint32_t B = codec_bins(a.L, a.time_domain), W = (B + 31) / 32, Tn = codec_tiles(a.L, a.time_domain);
    // persistent grid: about two rounds of the workgroups a chip holds at once (six to eight per compute unit);
    // measured best at 4096 (2048: +10 %, one workgroup per tile: +8 %)
    const uint32_t total = (uint32_t)(a.C * Tn);
    const uint32_t grid = total < 4096u ? total : 4096u;
#define FFTSP_DECODE(NL, VEC)                                                                                      \
    do {                                                                                                           \
        if (peers_layout)                                                                                          \
            FFTSP_LAUNCH("decode", (k_decode_peers<NL, VEC>), dim3(grid), dim3(NT), 0, s, recs, npeers, a.S, B, W,  \
                         a.k, a.bits, a.m, Tn, total, a.C, gprefix, verd, status,                                  \
                         reinterpret_cast<float2*>(spec), a.sstride, a.pair_log);                                  \
        else if (a.tab)                                                                                            \
            FFTSP_LAUNCH("decode", (k_decode<NL, VEC, true, false, false>), dim3(grid), dim3(NT), 0, s, recs.p[0], \
                         a.S, B, W, a.k, a.bits, a.m, Tn, total, a.C, gprefix, verd, status,                       \
                         reinterpret_cast<float2*>(spec), a.sstride, a.pair_log, table_arg<true>(a.tab), a.n);     \
        else if (a.half)                                                                                           \
            FFTSP_LAUNCH("decode", (k_decode<NL, VEC, false, false, true>), dim3(grid), dim3(NT), 0, s, recs.p[0], \
                         a.S, B, W, a.k, a.bits, a.m, Tn, total, a.C, gprefix, verd, status,                       \
                         reinterpret_cast<uint32_t*>(spec), a.sstride, a.pair_log, table_arg<false>(a.tab), a.n);  \
        else                                                                                                       \
            FFTSP_LAUNCH("decode", (k_decode<NL, VEC, false, false, false>), dim3(grid), dim3(NT), 0, s,           \
                         recs.p[0], a.S, B, W, a.k, a.bits, a.m, Tn, total, a.C, gprefix, verd, status,            \
                         reinterpret_cast<float2*>(spec), a.sstride, a.pair_log, table_arg<false>(a.tab), a.n);    \
    } while (0)
    if (a.half && (peers_layout || a.tab || a.time_domain)) return hipErrorInvalidValue;
    if (a.time_domain) {
        // one code per sample: a wave's 512 samples are at most 1 KiB of codes up to 16 bits, 2 KiB at 32
        if (peers_layout || a.tab || a.pair_log) return hipErrorInvalidValue;
        const bool vec16 = (reinterpret_cast<uintptr_t>(spec) & 15u) == 0;
#define FFTSP_DECODE_REAL(NL, VEC)                                                                                 \
    FFTSP_LAUNCH("decode", (k_decode<NL, VEC, false, true, false>), dim3(grid), dim3(NT), 0, s, recs.p[0], a.S, B, W, \
                 a.k, a.bits, a.m, Tn, total, a.C, gprefix, verd, status, spec, a.sstride, 0,                      \
                 table_arg<false>(nullptr), a.n)
        if (a.bits <= 16) {
            if (vec16)
                FFTSP_DECODE_REAL(1, true);
            else
                FFTSP_DECODE_REAL(1, false);
        } else {
            if (vec16)
                FFTSP_DECODE_REAL(2, true);
            else
                FFTSP_DECODE_REAL(2, false);
        }
#undef FFTSP_DECODE_REAL
        return hipGetLastError();
    }
    const bool vec = a.sstride == padded_bins(a.L) && (reinterpret_cast<uintptr_t>(spec) & 15u) == 0;
    // code widths are 3..16 or 32 bits
    const int nl = a.bits <= 8 ? 1 : a.bits <= 16 ? 2 : 4;
    switch (nl * 2 + (vec ? 1 : 0)) {
        case 2: FFTSP_DECODE(1, false); break;
        case 3: FFTSP_DECODE(1, true); break;
        case 4: FFTSP_DECODE(2, false); break;
        case 5: FFTSP_DECODE(2, true); break;
        case 8: FFTSP_DECODE(4, false); break;
        default: FFTSP_DECODE(4, true); break;
    }
#undef FFTSP_DECODE
    return hipGetLastError();
}

hipError_t launch_decode(const uint8_t* stream_base, const uint8_t* records, const CodecArgs& a, float* spec,
                         uint8_t* ws_base, const Workspace& w, int check_header, int reset_status, hipStream_t s)
{
    const uint32_t B = codec_bins(a.L, a.time_domain), W = (B + 31) / 32, Tn = codec_tiles(a.L, a.time_domain);
    uint32_t* status = reinterpret_cast<uint32_t*>(ws_base + w.status);
    uint32_t* sel = reinterpret_cast<uint32_t*>(ws_base + w.sel);
    uint32_t* gprefix = reinterpret_cast<uint32_t*>(ws_base + w.prefix);
    if (a.C * (size_t)Tn > 0x7fffffffu) return hipErrorInvalidValue;
    HeaderInfo h{check_header, a.hdr_n, a.hdr_L, a.hdr_C, (uint32_t)a.bits, (uint32_t)a.m, a.hdr_k, a.hdr_S,
                 a.hdr_theta, a.time_domain ? 1u : 0u, (uint32_t)a.hdr_scale};
    if (a.tab && a.C > (size_t)kMaxTableChunks) return hipErrorInvalidValue;
    if (a.tab)
        FFTSP_LAUNCH("group_prefix", k_group_prefix<true>, dim3((unsigned)a.C), dim3(RT), 0, s, stream_base, records, a.S,
                     W, a.k, a.word3, h, gprefix, sel, status, reset_status, table_arg<true>(a.tab));
    else
        FFTSP_LAUNCH("group_prefix", k_group_prefix<false>, dim3((unsigned)a.C), dim3(RT), 0, s, stream_base, records, a.S,
                     W, a.k, a.word3, h, gprefix, sel, status, reset_status, table_arg<false>(a.tab));
    PeerList recs{};
    recs.p[0] = records;
    return launch_decode_kernel(recs, 1u, a, spec, gprefix, sel, status, false, s);
}

hipError_t launch_decode_peers(const PeerList& streams, int npeers, const CodecArgs& a, float* spec, uint8_t* ws_base,
                               const Workspace& w, const PeerWorkspace& pw, hipStream_t s)
{
    const uint32_t B = a.L / 2 + 1, W = (B + 31) / 32, Tn = tiles_per_chunk(a.L);
    uint32_t* status = reinterpret_cast<uint32_t*>(ws_base + w.status);
    uint32_t* gprefix = reinterpret_cast<uint32_t*>(ws_base + pw.prefix);
    uint32_t* verd = reinterpret_cast<uint32_t*>(ws_base + pw.verd);
    if (npeers < 1 || npeers > kMaxPeers) return hipErrorInvalidValue;
    if (a.C * (size_t)Tn > 0x7fffffffu || a.C * (size_t)npeers > 0x7fffffffu) return hipErrorInvalidValue;
    HeaderInfo h{1, a.hdr_n, a.hdr_L, a.hdr_C, (uint32_t)a.bits, (uint32_t)a.m, a.hdr_k, a.hdr_S, a.hdr_theta, 0u, 0u};
    FFTSP_LAUNCH("group_prefix", k_group_prefix_peers, dim3((unsigned)(a.C * (size_t)npeers)), dim3(RT), 0, s, streams,
                 (uint32_t)a.C, a.S, W, a.k, h, gprefix, verd, status);
    PeerList recs{};
    for (int i = 0; i < npeers; ++i) recs.p[i] = streams.p[i] + 64;  // records follow the 64-byte stream header
    return launch_decode_kernel(recs, (uint32_t)npeers, a, spec, gprefix, verd, status, true, s);
}

}  // namespace fftsp

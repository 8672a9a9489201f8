// The two FFT passes of a chunk fused into one persistent kernel whose intermediate never leaves the L2 cache.
//
// The transform is the DFT sum of arXiv 1811.08596 Sec. 3.1.1 (and its inverse on the receiver, Sec. 3.1, last
// paragraph), factored M = N1*N2 exactly as in fft.hip.  There, pass A writes the whole intermediate to memory and
// pass B reads it back: two sweeps of the gradient's size per direction.  Here the chip's eight L2 caches (one per
// XCD, 4 MiB each) carry it instead.  Workgroups are dispatched to XCDs round-robin by index, so the 64 resident
// workgroups b = x, x+8, ... of XCD x form a team that shares one L2.  A team works in turns; a turn is 64 tiles of
// 8192 points (4 MiB of intermediate: one chunk of 2^20 samples, or several shorter chunks):
//     pass A on the team's tiles   -> stored into one of the team's three 4 MiB turn buffers
//     every member arrives         -> the turn's "stored" counter
//     pass B on the team's tiles   <- loaded from the buffer with L1-bypassing loads (served by L2)
//     every member arrives         -> the turn's "loaded" counter, which the stores that reuse the buffer wait for
// A member runs pass A of turn s and pass B of turn s - 2 in one slot of its walk, so that what a wait refers to
// lies two tiles back and has normally long happened.  Measured, the kernels are slower than the per-pass ones
// (a team advances at the pace of its slowest member), so they are off unless FFTSP_FUSED=1 is set.
//
// Hand-over protocol.  Writers: plain stores, then every wave waits until its stores are acknowledged by L2
// (vmcnt(0)), a workgroup barrier, and one device-scope atomic increment.  Readers: poll the counter with
// device-scope loads, a workgroup barrier, then loads that bypass the per-CU L1 (device-scope relaxed atomic
// loads), which an earlier turn may have filled with the region's old contents.  No L2 write-back or invalidate
// is issued: writer and reader share the L2, which is what makes the hand-over cheap (about 2 us).  That premise
// is checked, not assumed: every workgroup publishes the XCD it runs on (XCC_ID register) and a team whose members
// disagree gives up.  All waits are bounded; a workgroup whose wait expires, or that sees the give-up word set,
// sets it and exits, and so does every other workgroup at its next wait.  The host always enqueues the per-pass
// kernels of fft.hip behind a fused kernel with the give-up word as their switch: they return at once unless it
// is set, in which case they redo the whole transform.  The result is therefore the same either way.
#include "fft_core.h"
#include <cstdlib>

namespace fftsp {
namespace {

constexpr int kXcds = 8;         // L2 caches of the chip; workgroup b runs on XCD b % 8
constexpr int kXcdWgs = 64;      // workgroups of this kernel resident per XCD: 32 compute units x 2
constexpr int kTurnTiles = 64;   // tiles per turn: 64 x 64 KiB = one L2's worth of intermediate
constexpr int kSkew = 2;         // a turn's second pass runs this many turns behind its first pass
constexpr int kBufs = kSkew + 1; // turn buffers per XCD, used round-robin
// stage twiddles exp(-2 pi i e / 1024): a radix-16 stage reads e < 15/16 of a turn only
constexpr int kTwEntries = 960;
// tile, stage twiddles, 16-bit key histogram, one word for the outcome of a wait
constexpr size_t kFusedLds = ((size_t)(1 << kLogE) + kTwEntries) * sizeof(float2) + kHistLdsWords * sizeof(uint32_t) + 16;
static_assert(2 * kFusedLds <= 160 * 1024, "two workgroups per compute unit (the kernel has no static LDS)");

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16 bytes read past the L1 (two device-scope 8-byte loads: they are served by L2, never by this CU's L1)
__device__ __forceinline__ float4 ld_l2(const float4* p)
{
    const uint64_t* q = reinterpret_cast<const uint64_t*>(p);
    const uint64_t a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float4(__uint_as_float((uint32_t)a), __uint_as_float((uint32_t)(a >> 32)), __uint_as_float((uint32_t)b),
                       __uint_as_float((uint32_t)(b >> 32)));
}

// XCD this wave runs on (hardware register XCC_ID, bits 3:0)
__device__ __forceinline__ uint32_t xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & 15u; }

// Members drift up to kSkew turns apart, so arrivals are counted per turn: a ring of kRing counters, turn u in
// entry u % kRing, which has seen members * (u / kRing + 1) arrivals once every member has arrived for turn u.
constexpr int kRing = 4;
static_assert(kRing > kSkew + 1 && (kRing & (kRing - 1)) == 0, "a ring entry is not reused while its turn is awaited");
__device__ __forceinline__ uint32_t* turn_ctr(uint32_t* ring, uint32_t u) { return ring + (u & (uint32_t)(kRing - 1)); }
__device__ __forceinline__ uint32_t turn_target(uint32_t members, uint32_t u) { return members * (u / (uint32_t)kRing + 1u); }

struct TeamCtl {
    uint32_t* stored;   // ring: members that finished storing a turn's tiles
    uint32_t* loaded;   // ring: members that finished loading a turn's tiles
    uint32_t* gave_up;  // != 0: some workgroup of the launch gave up; everybody leaves
    uint32_t spin_limit;
};

// Wait (lane 0 polls) until *ctr >= target.  Returns false if the wait expired or the launch has given up; the
// give-up word is then set.  Called by every lane of the workgroup.
__device__ __forceinline__ bool team_wait(const uint32_t* ctr, uint32_t target, const TeamCtl& tc, uint32_t* s_ok)
{
    if (threadIdx.x == 0) {
        uint32_t spins = 0;
        bool ok = true;
        while (ld_agent(ctr) < target) {
            if (spins >= tc.spin_limit || ld_agent(tc.gave_up) != 0u) {
                ok = false;
                break;
            }
            ++spins;
            __builtin_amdgcn_s_sleep(1);
        }
        if (ok && ld_agent(tc.gave_up) != 0u) ok = false;
        if (!ok) __hip_atomic_store(tc.gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_ok = ok ? 1u : 0u;
    }
    __syncthreads();
    const bool ok = *s_ok != 0u;
    __syncthreads();
    return ok;
}

// Every lane's stores have reached L2, then one arrival is counted.
__device__ __forceinline__ void team_arrive_after_stores(uint32_t* ctr)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// stage twiddles for transforms of up to 1024 points from one table: tw[e] = exp(-2 pi i e / 1024), e < 960
template <int NT>
__device__ __forceinline__ void load_shared_twiddles(float2* tw, const Tables& tb, int tid)
{
    for (int e = tid; e < kTwEntries; e += NT) tw[e] = tb.hi[e << 1];
}

// run_fft on a table of 1024th roots: a transform of 2^LOGR points reads every 2^(10-LOGR)-th entry
template <int LOGR, int LOGT, int NT, bool INV, int NS_LOG, int RL>
__device__ __forceinline__ void fft_stage_1024(float2* d, const float2* tw, int tid)
{
    constexpr int R = 1 << LOGR, T = 1 << LOGT, RHO = 1 << RL, NS = 1 << NS_LOG;
    constexpr int NBF = (R / RHO) * T;
    static_assert(NBF % NT == 0, "butterflies must divide evenly over the workgroup");
    static_assert(LOGR <= 10, "the shared table holds 1024th roots");
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
                const float2 c = tw[(t * k) << (10 - NS_LOG - RL)];
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
template <int LOGR, int LOGT, int NT, bool INV, int NS_LOG>
__device__ __forceinline__ void run_fft_1024(float2* d, const float2* tw, int tid)
{
    if constexpr (NS_LOG < LOGR) {
        constexpr int RL = stage_radix_log(LOGR - NS_LOG);
        fft_stage_1024<LOGR, LOGT, NT, INV, NS_LOG, RL>(d, tw, tid);
        run_fft_1024<LOGR, LOGT, NT, INV, NS_LOG + RL>(d, tw, tid);
    }
}

// ------------------------------------------------------------ forward ----
// One member's walk over its team's turns.  FAST: every chunk this member reads lies wholly inside a 16-byte aligned
// input (no guards on the loads).
template <int LOGN1, int LOGN2, bool FAST>
__device__ __forceinline__ void fused_fwd_run(const float* __restrict__ in, size_t n, uint32_t C, int aligned,
                                              float2* __restrict__ scratch, float2* __restrict__ spec, uint32_t sstride,
                                              const Tables& tb, uint32_t* __restrict__ hist, uint32_t x, uint32_t mi,
                                              uint32_t members, const TeamCtl& tc, float2* d,
                                              const float2* tw, uint32_t* h16, uint32_t* s_ok, int tid0)
{
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int logM = LOGN1 + LOGN2;
    constexpr uint32_t M = 1u << logM, N1 = 1u << LOGN1, N2 = 1u << LOGN2;
    constexpr int LOGG = logM - LOGE;               // log2 of the tiles per chunk and pass
    static_assert(LOGG >= 1 && LOGG <= 6, "a turn holds whole chunks");
    constexpr uint32_t G = 1u << LOGG, CPR = (uint32_t)kTurnTiles >> LOGG;  // chunks per turn
    // pass A geometry (tile = TA adjacent columns, all N1 rows)
    constexpr int LOGTA = LOGE - LOGN1, TA = 1 << LOGTA;
    constexpr int HP = N1 / 2, LOGHP = LOGN1 - 1;
    static_assert(LOGTA >= 2 && (NT % (TA / 2)) == 0, "pass A tile shape");
    constexpr int KN = HP >= NT ? HP / NT : 1;
    constexpr int DC = HP >= NT ? 1 : NT / HP;
    constexpr int NCOL = PER2 / KN;
    static_assert(NCOL <= 8, "twiddle recurrence is anchored once");
    static_assert(PER2 == 8 && (NT >> (LOGTA - 1)) == N1 / 8, "a lane's loads are the inputs of two radix-8 butterflies");
    // pass B geometry (tile = P row pairs, all N2 columns)
    constexpr int LOGTB = LOGE - LOGN2, LOGP = LOGTB - 1, P = 1 << LOGP;
    static_assert(LOGTB >= 1 && NT % P == 0, "a lane keeps one slot pair");
    constexpr int DK = NT >> LOGP;
    static_assert(DK == (int)N2 / 8, "a lane's loads are the inputs of two radix-8 butterflies");
    static_assert(2 * kSplitStep * (PER2 - 1) < 16, "split twiddle steps stay inside the 32nd-root table");
    constexpr int BATCH = 4;

    const uint32_t tpm = (uint32_t)kTurnTiles / members;  // tiles per member, pass and turn
    const uint32_t groups = (C + CPR - 1) / CPR;          // turns of the whole call
    if (groups <= x) return;                              // this XCD has nothing to do (nobody waits for it)
    const uint32_t turns = (groups - x + (uint32_t)kXcds - 1) / (uint32_t)kXcds;

    // tile i of this member in turn u: chunk, its slot in the scratch region, tile index inside the chunk
    auto tile_of = [&](uint32_t u, uint32_t i, uint32_t& c, uint32_t& slot, uint32_t& tl) {
        const uint32_t q = mi * tpm + i;
        slot = q >> LOGG;
        tl = q & (G - 1u);
        c = (u * (uint32_t)kXcds + x) * CPR + slot;
        return c < C;
    };

    float4 r[PER2];
    // ---- pass A pieces ----
    auto load_a = [&](uint32_t u, uint32_t i, int tid, bool live) {
        uint32_t c, slot, tl;
        const bool ok = tile_of(u, i, c, slot, tl) && live;
        const uint32_t col0 = tl << LOGTA;
        if constexpr (FAST) {
            // a tile that does not exist still issues its loads, all to one valid address
            const float4* src = ok ? reinterpret_cast<const float4*>(in + (size_t)c * (2 * (size_t)M)) + (col0 >> 1)
                                   : reinterpret_cast<const float4*>(tb.hi);
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGTA - 1);
                r[q] = src[ok ? (uint32_t)n1 * (N2 >> 1) + bp : 0u];
            }
        } else {
            if (!ok) return;
            const size_t first = (size_t)c * (2 * (size_t)M);
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGTA - 1);
                const size_t gi = first + 2 * ((size_t)n1 * N2 + col0 + 2 * bp);
                r[q] = join(load_pair(in, gi, n, aligned & 1), load_pair(in, gi + 2, n, aligned & 1));
            }
        }
    };
    auto fill_a = [&](int tid) { first_stage_store<LOGTA, false>(d, tid >> (LOGTA - 1), 2 * (tid & (TA / 2 - 1)), r); };

    // ---- pass B pieces ----
    auto load_b_from = [&](const float2* region, uint32_t slot, uint32_t tl, int tid) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const float4* src = reinterpret_cast<const float4*>(region + (size_t)slot * M);
        const uint32_t pp = tl * P + p;
#pragma unroll
        for (int q = 0; q < PER2; ++q) r[q] = ld_l2(src + (uint32_t)(kq0 + q * DK) * (N1 >> 1) + pp);
    };
    auto fill_b = [&](int tid) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        first_stage_store<LOGTB, false>(d, kq0, 2 * p, r);
    };
    auto count = [&](float2 v, bool on) {
        const uint32_t b = fft_key_of(v) >> kKeyShift;
        atomicAdd(&h16[b >> 1], on ? 1u << ((b & 1u) * 16u) : 0u);
    };

    // A-side twiddles of one tile: W_M^(n2 k1) as a base and a ratio per row pair (see fwd_a_run in fft.hip)
    struct ATw {
        float2 ratio_a[KN], ratio_b[KN], cur_a[KN], cur_b[KN];
    };
    auto a_twiddles = [&](int tid, uint32_t tl) {
        ATw t;
        const uint32_t col0 = tl << LOGTA;
        constexpr int sh = 22 - logM;
#pragma unroll
        for (int kk = 0; kk < KN; ++kk) {
            const uint32_t kp = (uint32_t)(tid + kk * NT) & (HP - 1);
            const uint32_t ka = kp, kb = mirror_row(kp, N1);
            const uint32_t cfirst = (uint32_t)(tid + kk * NT) >> LOGHP;
            t.ratio_a[kk] = twiddle(tb, ((uint32_t)DC * ka) << sh);
            t.ratio_b[kk] = twiddle(tb, ((uint32_t)DC * kb) << sh);
            t.cur_a[kk] = twiddle(tb, ((col0 + cfirst) * ka) << sh);
            t.cur_b[kk] = twiddle(tb, ((col0 + cfirst) * kb) << sh);
        }
        return t;
    };
    auto a_store = [&](int tid, float2* region, uint32_t slot, uint32_t tl, ATw& t) {
        float4* out = reinterpret_cast<float4*>(region + (size_t)slot * M);
        const uint32_t col0 = tl << LOGTA;
#pragma unroll
        for (int kk = 0; kk < KN; ++kk) {
            const uint32_t kp = (uint32_t)(tid + kk * NT) & (HP - 1);
            const uint32_t ka = kp, kb = mirror_row(kp, N1);
            const uint32_t cfirst = (uint32_t)(tid + kk * NT) >> LOGHP;
#pragma unroll
            for (int j = 0; j < NCOL; ++j) {
                const uint32_t col = cfirst + j * DC, n2 = col0 + col;
                const float2 va = cmul(d[sw_idx<LOGTA>((int)ka, (int)col)], t.cur_a[kk]);
                const float2 vb = cmul(d[sw_idx<LOGTA>((int)kb, (int)col)], t.cur_b[kk]);
                out[n2 * (uint32_t)HP + kp] = join(va, vb);
                t.cur_a[kk] = cmul(t.cur_a[kk], t.ratio_a[kk]);
                t.cur_b[kk] = cmul(t.cur_b[kk], t.ratio_b[kk]);
            }
        }
    };
    // the real-FFT split of the tile in LDS, the spectrum store and the key histogram (see k_fwd_b in fft.hip)
    auto b_split_store = [&](int tid, uint32_t c, uint32_t tl, float2 base_a, float2 base_b) {
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const uint32_t pp = tl * P + p;
        const bool self = pp == 0;
        float2* out = spec + (size_t)c * (size_t)sstride;
#pragma unroll
        for (int q0 = 0; q0 < PER2; q0 += BATCH) {
            float2 a0[BATCH], a1[BATCH], pa[BATCH], pb[BATCH];
#pragma unroll
            for (int v = 0; v < BATCH; ++v) {
                const int k2 = kq0 + (q0 + v) * DK, k2p = (int)N2 - 1 - k2;
                const int ia = self ? sw_idx<LOGTB>(((int)N2 - k2) & ((int)N2 - 1), 2 * p) : sw_idx<LOGTB>(k2p, 2 * p + 1);
                const int ib = self ? sw_idx<LOGTB>(k2p, 2 * p + 1) : sw_idx<LOGTB>(k2p, 2 * p);
                a0[v] = d[sw_idx<LOGTB>(k2, 2 * p)];
                a1[v] = d[sw_idx<LOGTB>(k2, 2 * p + 1)];
                pa[v] = d[ia];
                pb[v] = d[ib];
            }
#pragma unroll
            for (int v = 0; v < BATCH; ++v) {
                const int q = q0 + v, k2 = kq0 + q * DK;
                const float2 wq = make_float2(kW32re[2 * q * kSplitStep], kW32im[2 * q * kSplitStep]);
                float2 xa = split_fwd(a0[v], pa[v], cmul(base_a, wq));
                const float2 xb = split_fwd(a1[v], pb[v], cmul(base_b, wq));
                if (q == 0) {  // k2 = 0 only here: bin 0 and the Nyquist bin come from Z[0] alone
                    const bool dc = self && kq0 == 0;
                    const float2 xm = make_float2(a0[v].x - a0[v].y, 0.f);
                    if (dc) {
                        xa = make_float2(a0[v].x + a0[v].y, 0.f);
                        out[M] = xm;
                    }
                    count(xm, dc);
                }
                reinterpret_cast<float4*>(out)[((uint32_t)k2 << (LOGN1 - 1)) + pp] = join(xa, xb);
                count(xa, true);
                count(xb, true);
            }
        }
    };
    auto flush_hist = [&](uint32_t c) {
        uint32_t* g = hist + (size_t)c * kHistBins;
        for (int i = tid0; i < kHistLdsWords; i += NT) {
            const uint32_t v = h16[i];
            if (v) {
                if (v & 0xFFFFu) atomicAdd(&g[2 * i], v & 0xFFFFu);
                if (v >> 16) atomicAdd(&g[2 * i + 1], v >> 16);
                h16[i] = 0u;
            }
        }
    };
    auto region_of = [&](uint32_t u) { return scratch + (size_t)(u % (uint32_t)kBufs) * ((size_t)kTurnTiles << kLogE); };

    // Slot s of the walk: pass A of turn s, then pass B of turn s - kSkew.  What a wait refers to lies two or three
    // tiles back in every member's walk, so it has normally long happened; a tile's loads are issued one tile ahead
    // (the second pass's before the first pass's FFT, the first pass's before the second pass's FFT).
    load_a(0, 0, tid0, true);
    for (uint32_t s = 0; s < turns + (uint32_t)kSkew; ++s) {
        uint32_t ca = 0, slota = 0, tla = 0, cb = 0, slotb = 0, tlb = 0;
        const bool has_a = s < turns && tile_of(s, 0, ca, slota, tla);
        const bool in_b = s >= (uint32_t)kSkew;
        const uint32_t ub = s - (uint32_t)kSkew;
        const bool has_b = in_b && tile_of(ub, 0, cb, slotb, tlb);
        int tid = opaque_lane(tid0);
        if (has_a) fill_a(tid);
        __syncthreads();
        ATw at = a_twiddles(tid, tla);
        if (in_b) {
            // turn ub's intermediate is complete once all members have stored their tiles of it
            if (!team_wait(turn_ctr(tc.stored, ub), turn_target(members, ub), tc, s_ok)) return;
            if (has_b) load_b_from(region_of(ub), slotb, tlb, tid);
        }
        if (s < turns) {
            if (has_a) run_fft_1024<LOGN1, LOGTA, NT, false, 3>(d, tw, tid);
            // the buffer is free once every member has taken its tile of the turn that used it last out of it
            if (s >= (uint32_t)kBufs) {
                const uint32_t uold = s - (uint32_t)kBufs;
                if (!team_wait(turn_ctr(tc.loaded, uold), turn_target(members, uold), tc, s_ok)) return;
            }
            if (has_a) a_store(tid, region_of(s), slota, tla, at);
            __syncthreads();  // the tile has left LDS
            team_arrive_after_stores(turn_ctr(tc.stored, s));
        }
        tid = opaque_lane(tid0);
        if (in_b) {
            if (has_b) fill_b(tid);
            __syncthreads();
            if (tid0 == 0)
                __hip_atomic_fetch_add(turn_ctr(tc.loaded, ub), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        load_a(s + 1u, 0, tid, s + 1u < turns);
        if (in_b) {
            const int p = tid & (P - 1), kq0 = tid >> LOGP;
            const uint32_t pp = tlb * P + p;
            const uint32_t ka = pp, kb = mirror_row(pp, N1);
            const float2 base_a = twiddle(tb, (ka + ((uint32_t)kq0 << LOGN1)) << (21 - logM));
            const float2 base_b = twiddle(tb, (kb + ((uint32_t)kq0 << LOGN1)) << (21 - logM));
            if (has_b) {
                run_fft_1024<LOGN2, LOGTB, NT, false, 3>(d, tw, tid);
                b_split_store(tid, cb, tlb, base_a, base_b);
            }
            __syncthreads();  // the tile has left LDS; the LDS histogram is complete for it
            if (has_b) flush_hist(cb);
        }
    }
}

// Control words (u32 index into the workspace's control block; kCtlGaveUpWord is shared with the host code).
constexpr int kCtlGaveUp = kCtlGaveUpWord;
constexpr int kCtlXcc = 32;      // + x: XCD claimed by team slot x, plus one
constexpr int kCtlStored = 128;  // + 64 x
constexpr int kCtlLoaded = 160;  // + 64 x

template <int LOGN1, int LOGN2>
__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_fused_fwd(const float* __restrict__ in, size_t n, uint32_t C, int aligned,
                                                   float2* __restrict__ scratch_all, float2* __restrict__ spec,
                                                   uint32_t sstride, Tables tb, uint32_t* __restrict__ hist,
                                                   uint32_t* __restrict__ ctl, uint32_t spin_limit)
{
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + (1 << kLogE);
    uint32_t* h16 = reinterpret_cast<uint32_t*>(tw + kTwEntries);
    uint32_t* s_ok = h16 + kHistLdsWords;
    const int tid0 = threadIdx.x;
    const uint32_t x = blockIdx.x & (kXcds - 1u), y = blockIdx.x >> 3;
    const uint32_t members = (uint32_t)kXcdWgs, mi = y;  // the XCD's 64 workgroups are one team, a tile each per turn
    TeamCtl tc;
    tc.stored = ctl + kCtlStored + 64 * x;
    tc.loaded = ctl + kCtlLoaded + 64 * x;
    tc.gave_up = ctl + kCtlGaveUp;
    tc.spin_limit = spin_limit;
    if (tid0 == 0) {
        // all members of a team slot must sit behind one L2: the first to arrive claims the XCD for the slot
        const uint32_t me = xcc_id() + 1u;
        const uint32_t prev = atomicCAS(ctl + kCtlXcc + x, 0u, me);
        if (prev != 0u && prev != me) {
            __hip_atomic_store(tc.gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // before this workgroup counts as arrived anywhere
        }
    }
    load_shared_twiddles<kNT>(tw, tb, tid0);
    for (int i = tid0; i < kHistLdsWords; i += kNT) h16[i] = 0u;
    float2* scratch = scratch_all + (size_t)x * (size_t)kBufs * ((size_t)kTurnTiles << kLogE);
    // only the gradient's last chunk can be ragged; the team that transforms it loads under guards
    constexpr int LOGG = LOGN1 + LOGN2 - kLogE;
    constexpr uint32_t CPR = (uint32_t)kTurnTiles >> LOGG;
    const uint32_t last_group = (C - 1u) / CPR;
    const bool ragged = ((size_t)C << (LOGN1 + LOGN2 + 1)) != n;
    const bool mine = (last_group % (uint32_t)kXcds) == x;
    const bool fast = (aligned & 2) != 0 && !(ragged && mine);
    __syncthreads();
    if (fast)
        fused_fwd_run<LOGN1, LOGN2, true>(in, n, C, aligned, scratch, spec, sstride, tb, hist, x, mi,
                                          members, tc, d, tw, h16, s_ok, tid0);
    else
        fused_fwd_run<LOGN1, LOGN2, false>(in, n, C, aligned, scratch, spec, sstride, tb, hist, x, mi,
                                           members, tc, d, tw, h16, s_ok, tid0);
}

// ------------------------------------------------------------ inverse ----
// The receiver's two passes in the same scheme: the split and the inverse N2-point transforms of a tile of row
// pairs (read from the decoded spectrum, stored into the team's scratch region), hand-over, then the inverse
// N1-point transforms of a tile of columns (loaded from the region past the L1, stored as real samples).
template <int LOGN1, int LOGN2>
__device__ __forceinline__ void fused_inv_run(const float2* __restrict__ spec, uint32_t sstride, size_t n, uint32_t C,
                                              int aligned, float gain, float2* __restrict__ scratch,
                                              float* __restrict__ out, const Tables& tb, uint32_t x, uint32_t mi,
                                              uint32_t members, const TeamCtl& tc, float2* d,
                                              const float2* tw, uint32_t* s_ok, int tid0)
{
    constexpr int NT = kNT, LOGE = kLogE, PER2 = kPer / 2;
    constexpr int logM = LOGN1 + LOGN2;
    constexpr uint32_t M = 1u << logM, N1 = 1u << LOGN1, N2 = 1u << LOGN2;
    constexpr int LOGG = logM - LOGE;
    static_assert(LOGG >= 1 && LOGG <= 6, "a turn holds whole chunks");
    constexpr uint32_t G = 1u << LOGG, CPR = (uint32_t)kTurnTiles >> LOGG;
    // pass over k2 (tile = P row pairs, all N2 columns)
    constexpr int LOGTB = LOGE - LOGN2, LOGP = LOGTB - 1, P = 1 << LOGP;
    static_assert(LOGTB >= 1 && NT % P == 0, "a lane keeps one slot pair");
    constexpr int DK = NT >> LOGP;
    static_assert(PER2 == 8 && DK == (int)N2 / 8, "a lane's values are the inputs of two radix-8 butterflies");
    // pass over k1 (tile = TA adjacent columns, all N1 rows)
    constexpr int LOGTA = LOGE - LOGN1, TA = 1 << LOGTA;
    constexpr int HP = N1 / 2, LOGHP = LOGN1 - 1;
    static_assert(LOGTA >= 2 && (NT % (TA / 2)) == 0, "tile shape");

    const uint32_t tpm = (uint32_t)kTurnTiles / members;
    const uint32_t groups = (C + CPR - 1) / CPR;
    if (groups <= x) return;
    const uint32_t turns = (groups - x + (uint32_t)kXcds - 1) / (uint32_t)kXcds;
    const float scale = gain * (1.0f / (float)(2u * M));

    auto tile_of = [&](uint32_t u, uint32_t i, uint32_t& c, uint32_t& slot, uint32_t& tl) {
        const uint32_t q = mi * tpm + i;
        slot = q >> LOGG;
        tl = q & (G - 1u);
        c = (u * (uint32_t)kXcds + x) * CPR + slot;
        return c < C;
    };

    float4 r[PER2];
    float2 xnyq = make_float2(0.f, 0.f);  // Nyquist bin of the chunk of the spectrum tile held in r
    float2 base_a = make_float2(1.f, 0.f), base_b = make_float2(1.f, 0.f);  // split twiddles of that tile
    // a tile that does not exist still issues its loads, all to one valid address
    auto load_spec = [&](uint32_t u, uint32_t i, int tid, bool live) {
        uint32_t c, slot, tl;
        const bool ok = tile_of(u, i, c, slot, tl) && live;
        const int p = tid & (P - 1), kq0 = tid >> LOGP;
        const float2* X = ok ? spec + (size_t)c * (size_t)sstride : reinterpret_cast<const float2*>(tb.hi);
        const uint32_t pp = tl * P + p;
        const uint32_t ka = pp, kb = mirror_row(pp, N1);
        base_a = twiddle(tb, (ka + ((uint32_t)kq0 << LOGN1)) << (21 - logM));
        base_b = twiddle(tb, (kb + ((uint32_t)kq0 << LOGN1)) << (21 - logM));
        const float4* X4 = reinterpret_cast<const float4*>(X);
#pragma unroll
        for (int q = 0; q < PER2; ++q) r[q] = X4[ok ? ((uint32_t)(kq0 + q * DK) << (LOGN1 - 1)) + pp : 0u];
        xnyq = X[ok ? M : 0u];
    };
    auto load_mid_from = [&](const float2* region, uint32_t slot, uint32_t tl, int tid) {
        const float4* src = reinterpret_cast<const float4*>(region + (size_t)slot * M);
        const uint32_t col0 = tl << LOGTA;
#pragma unroll
        for (int q = 0; q < PER2; ++q) {
            const int w = tid + q * NT, kp = w & (HP - 1), col = w >> LOGHP;
            r[q] = ld_l2(src + (uint32_t)(col0 + col) * HP + kp);
        }
    };

    auto region_of = [&](uint32_t u) { return scratch + (size_t)(u % (uint32_t)kBufs) * ((size_t)kTurnTiles << kLogE); };

    // Slot s: the split and the transforms over k2 of turn s, then the transforms over k1 of turn s - kSkew (same
    // skewed walk as the forward kernel).  A tile past the last chunk (last turn of a call whose chunks do not fill
    // it) is transformed like any other: its loads read one valid dummy address, its stores land in the region or are
    // dropped by the output guards, so the loop needs no branches around the arithmetic.
    load_spec(0, 0, tid0, true);
    for (uint32_t s = 0; s < turns + (uint32_t)kSkew; ++s) {
        uint32_t c = 0, slot = 0, tl = 0;
        const bool in_a = s >= (uint32_t)kSkew;
        const uint32_t ua = s - (uint32_t)kSkew;
        int tid = opaque_lane(tid0);
        if (s < turns) {
            (void)tile_of(s, 0, c, slot, tl);
            const int p = tid & (P - 1), kq0 = tid >> LOGP;
            const uint32_t pp = tl * P + p;
            const uint32_t ka = pp, kb = mirror_row(pp, N1);
            const bool self = pp == 0;
#pragma unroll
            for (int q = 0; q < PER2; ++q) lds_store2<LOGTB>(d, kq0 + q * DK, 2 * p, r[q]);
            __syncthreads();
            float4 z[PER2];
            {
                // partners of all pairs first (one batch of LDS reads), then the arithmetic
                float2 pa[PER2], pb[PER2];
#pragma unroll
                for (int q = 0; q < PER2; ++q) {
                    const int k2 = kq0 + q * DK, k2p = (int)N2 - 1 - k2;
                    const int ia = self ? sw_idx<LOGTB>(((int)N2 - k2) & ((int)N2 - 1), 2 * p) : sw_idx<LOGTB>(k2p, 2 * p + 1);
                    const int ib = self ? sw_idx<LOGTB>(k2p, 2 * p + 1) : sw_idx<LOGTB>(k2p, 2 * p);
                    pa[q] = d[ia];
                    pb[q] = d[ib];
                }
#pragma unroll
                for (int q = 0; q < PER2; ++q) {
                    const float2 wq = make_float2(kW32re[2 * q * kSplitStep], kW32im[2 * q * kSplitStep]);
                    float2 a0 = lo2(r[q]), b0 = pa[q];
                    if (q == 0) {  // k2 = 0 only here; imaginary parts of the DC and Nyquist bins are ignored
                        const bool dc = self && kq0 == 0;
                        b0 = dc ? make_float2(xnyq.x, 0.f) : b0;
                        a0.y = dc ? 0.f : a0.y;
                    }
                    z[q] = join(split_inv(a0, b0, cmul(base_a, wq)), split_inv(hi2(r[q]), pb[q], cmul(base_b, wq)));
                }
            }
            __syncthreads();
            first_stage_store<LOGTB, true>(d, kq0, 2 * p, z);
            __syncthreads();
            constexpr int sh = 22 - logM;
            const float2 ratio_a = twiddle(tb, ((uint32_t)DK * ka) << sh);
            const float2 ratio_b = twiddle(tb, ((uint32_t)DK * kb) << sh);
            float2 cur_a = twiddle(tb, ((uint32_t)kq0 * ka) << sh);
            float2 cur_b = twiddle(tb, ((uint32_t)kq0 * kb) << sh);
            if (in_a) {
                if (!team_wait(turn_ctr(tc.stored, ua), turn_target(members, ua), tc, s_ok)) return;
                uint32_t c2, slot2, tl2;
                (void)tile_of(ua, 0, c2, slot2, tl2);
                load_mid_from(region_of(ua), slot2, tl2, tid);
            }
            run_fft_1024<LOGN2, LOGTB, NT, true, 3>(d, tw, tid);
            if (s >= (uint32_t)kBufs) {
                const uint32_t uold = s - (uint32_t)kBufs;
                if (!team_wait(turn_ctr(tc.loaded, uold), turn_target(members, uold), tc, s_ok)) return;
            }
            {
                float4* dst = reinterpret_cast<float4*>(region_of(s) + (size_t)slot * M);
#pragma unroll
                for (int q = 0; q < PER2; ++q) {
                    const uint32_t n2 = (uint32_t)(kq0 + q * DK);
                    const float4 v = lds_load2<LOGTB>(d, (int)n2, 2 * p);
                    dst[n2 * (N1 >> 1) + pp] = join(cmulc(lo2(v), cur_a), cmulc(hi2(v), cur_b));
                    cur_a = cmul(cur_a, ratio_a);
                    cur_b = cmul(cur_b, ratio_b);
                }
            }
            __syncthreads();
            team_arrive_after_stores(turn_ctr(tc.stored, s));
        } else {
            // the walk's last slots: only the transforms over k1 are left
            if (!team_wait(turn_ctr(tc.stored, ua), turn_target(members, ua), tc, s_ok)) return;
            uint32_t c2, slot2, tl2;
            (void)tile_of(ua, 0, c2, slot2, tl2);
            load_mid_from(region_of(ua), slot2, tl2, tid);
        }
        tid = opaque_lane(tid0);
        if (in_a) {
            (void)tile_of(ua, 0, c, slot, tl);
#pragma unroll
            for (int q = 0; q < PER2; ++q) {
                const int w = tid + q * NT, kp = w & (HP - 1), col = w >> LOGHP;
                d[sw_idx<LOGTA>(kp, col)] = lo2(r[q]);
                d[sw_idx<LOGTA>((int)mirror_row((uint32_t)kp, N1), col)] = hi2(r[q]);
            }
            __syncthreads();
            if (tid0 == 0)
                __hip_atomic_fetch_add(turn_ctr(tc.loaded, ua), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        load_spec(s + 1u, 0, tid, s + 1u < turns);
        if (in_a) {
            run_fft_1024<LOGN1, LOGTA, NT, true, 0>(d, tw, tid);
            // a chunk past the end starts beyond n: the guarded branch below then stores nothing
            const size_t cbase = (size_t)c * (2 * (size_t)M);
            const uint32_t col0 = tl << LOGTA;
            if ((aligned & 2) && cbase + 2 * (size_t)M <= n) {  // whole chunk inside the output: no guards
                float4* dst = reinterpret_cast<float4*>(out + cbase) + (col0 >> 1);
#pragma unroll
                for (int q = 0; q < PER2; ++q) {
                    const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGTA - 1);
                    const float4 v = lds_load2<LOGTA>(d, n1, 2 * bp);
                    dst[(uint32_t)n1 * (N2 >> 1) + bp] = make_float4(v.x * scale, v.y * scale, v.z * scale, v.w * scale);
                }
            } else {
#pragma unroll
                for (int q = 0; q < PER2; ++q) {
                    const int w = tid + q * NT, bp = w & (TA / 2 - 1), n1 = w >> (LOGTA - 1);
                    const float4 v = lds_load2<LOGTA>(d, n1, 2 * bp);
                    const size_t gi = cbase + 2 * ((size_t)n1 * N2 + col0 + 2 * bp);
                    store_pair(out, gi, n, aligned & 1, make_float2(v.x * scale, v.y * scale));
                    store_pair(out, gi + 2, n, aligned & 1, make_float2(v.z * scale, v.w * scale));
                }
            }
            __syncthreads();
        }
    }
}

template <int LOGN1, int LOGN2>
__global__ __launch_bounds__(kNT) __attribute__((amdgpu_waves_per_eu(4, 4))) void k_fused_inv(
    const float2* __restrict__ spec, uint32_t sstride, size_t n, uint32_t C, int aligned, float gain,
    float2* __restrict__ scratch_all, float* __restrict__ out, Tables tb, uint32_t* __restrict__ ctl,
    uint32_t spin_limit)
{
    extern __shared__ float2 smem[];
    float2* d = smem;
    float2* tw = smem + (1 << kLogE);
    uint32_t* s_ok = reinterpret_cast<uint32_t*>(tw + kTwEntries);
    const int tid0 = threadIdx.x;
    const uint32_t x = blockIdx.x & (kXcds - 1u), y = blockIdx.x >> 3;
    const uint32_t members = (uint32_t)kXcdWgs, mi = y;  // the XCD's 64 workgroups are one team, a tile each per turn
    TeamCtl tc;
    tc.stored = ctl + kCtlStored + 64 * x;
    tc.loaded = ctl + kCtlLoaded + 64 * x;
    tc.gave_up = ctl + kCtlGaveUp;
    tc.spin_limit = spin_limit;
    if (tid0 == 0) {
        const uint32_t me = xcc_id() + 1u;
        const uint32_t prev = atomicCAS(ctl + kCtlXcc + x, 0u, me);
        if (prev != 0u && prev != me) {
            __hip_atomic_store(tc.gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        }
    }
    load_shared_twiddles<kNT>(tw, tb, tid0);
    float2* scratch = scratch_all + (size_t)x * (size_t)kBufs * ((size_t)kTurnTiles << kLogE);
    __syncthreads();
    fused_inv_run<LOGN1, LOGN2>(spec, sstride, n, C, aligned, gain, scratch, out, tb, x, mi, members, tc, d,
                                tw, s_ok, tid0);
}

}  // namespace

FusedKnobs fused_knobs()
{
    FusedKnobs k;
    k.enabled = 0;  // off until measured faster on the GPU
    k.spin_limit = 1u << 18;  // a poll takes about a microsecond: a quarter of a second before a wait gives up
    if (const char* e = std::getenv("FFTSP_FUSED")) k.enabled = std::atoi(e) != 0;
    if (const char* e = std::getenv("FFTSP_FUSED_SPIN")) k.spin_limit = (uint32_t)std::strtoul(e, nullptr, 10);
    return k;
}

static_assert(kFusedScratchBytes == (size_t)kXcds * kBufs * ((size_t)kTurnTiles << kLogE) * sizeof(float2),
              "the workspace reserves what the kernels address");

bool fused_applies(int logL, size_t C) { return fused_shape(logL, C); }

hipError_t launch_fused_rfft(const float* in, size_t n, int logL, size_t C, float2* spec, uint32_t sstride,
                             float2* scratch, Tables t, uint32_t* hist, uint32_t* ctl, const FusedKnobs& knobs,
                             hipStream_t s)
{
    const int logM = logL - 1;
    if (!fused_applies(logL, C) || C > 0x7fffffu) return hipErrorInvalidValue;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(in);
    const int aligned = ((addr & 7u) == 0 ? 1 : 0) | ((addr & 15u) == 0 ? 2 : 0);
#define FFTSP_FUSED_FWD(a, b)                                                                                         \
    do {                                                                                                              \
        auto kern = k_fused_fwd<a, b>;                                                                                \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                       \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLds);              \
        if (e != hipSuccess) return e;                                                                                \
        FFTSP_LAUNCH("rfft_fused", kern, dim3(kXcds * kXcdWgs), dim3(kNT), kFusedLds, s, in, n, (uint32_t)C, aligned, \
                     scratch, spec, sstride, t, hist, ctl, knobs.spin_limit);                     \
    } while (0)
    switch (logM) {
        case 14: FFTSP_FUSED_FWD(7, 7); break;
        case 15: FFTSP_FUSED_FWD(8, 7); break;
        case 16: FFTSP_FUSED_FWD(8, 8); break;
        case 17: FFTSP_FUSED_FWD(9, 8); break;
        case 18: FFTSP_FUSED_FWD(9, 9); break;
        case 19: FFTSP_FUSED_FWD(10, 9); break;
        default: return hipErrorInvalidValue;
    }
#undef FFTSP_FUSED_FWD
    return hipGetLastError();
}

// ctl: the control block, zero.  The decoded spectrum is the codec's own buffer (paired order).
hipError_t launch_fused_irfft(const float2* spec, uint32_t sstride, size_t n, int logL, size_t C, float* out,
                              float2* scratch, Tables t, float gain, uint32_t* ctl, const FusedKnobs& knobs, hipStream_t s)
{
    const int logM = logL - 1;
    if (!fused_applies(logL, C) || C > 0x7fffffu) return hipErrorInvalidValue;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(out);
    const int aligned = ((addr & 7u) == 0 ? 1 : 0) | ((addr & 15u) == 0 ? 2 : 0);
#define FFTSP_FUSED_INV(a, b)                                                                                            \
    do {                                                                                                                 \
        auto kern = k_fused_inv<a, b>;                                                                                   \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                          \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLds);                 \
        if (e != hipSuccess) return e;                                                                                   \
        FFTSP_LAUNCH("irfft_fused", kern, dim3(kXcds * kXcdWgs), dim3(kNT), kFusedLds, s, spec, sstride, n, (uint32_t)C, \
                     aligned, gain, scratch, out, t, ctl, knobs.spin_limit);                         \
    } while (0)
    switch (logM) {
        case 14: FFTSP_FUSED_INV(7, 7); break;
        case 15: FFTSP_FUSED_INV(8, 7); break;
        case 16: FFTSP_FUSED_INV(8, 8); break;
        case 17: FFTSP_FUSED_INV(9, 8); break;
        case 18: FFTSP_FUSED_INV(9, 9); break;
        case 19: FFTSP_FUSED_INV(10, 9); break;
        default: return hipErrorInvalidValue;
    }
#undef FFTSP_FUSED_INV
    return hipGetLastError();
}

}  // namespace fftsp

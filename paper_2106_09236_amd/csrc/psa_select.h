// Top-u selection of one head by a whole work-group (device function).
// Stage a2: I_sparse = the u queries with the largest sampled measure (Sec. 3.2,
// text after Eq. 11), ties to the lower query index.
//
// The measures (a few KB to tens of KB, L2-resident, just written by stage a1)
// are mapped to order-preserving 32-bit keys and the u-th largest key is found
// by a most-significant-digit radix select: four passes of an 8-bit histogram in
// LDS.  A last pass in index order emits every query above the cut-off plus the
// lowest-indexed queries equal to it, by ballot/popcount prefix sums, so the
// output is ascending in query index and does not depend on scheduling.
#pragma once

#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

// float -> unsigned key, increasing with the float; -0 and +0 map to one key.
__device__ __forceinline__ unsigned order_key(float f) {
    f += 0.0f;
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// u_b by the rule in force, clamped to [1, n] and capped by the host's bound.
__device__ __forceinline__ int n_selected(URule r, int n, int u_max) {
    if (n <= 0) return 0;
    double x = r.rule == PSA_U_RATIO ? ceil(r.factor * (double)n) : ceil(r.factor * log((double)n));
    if (!(x >= 1.0)) x = 1.0;
    if (x > (double)n) x = (double)n;
    int u = (int)x;
    return u > u_max ? u_max : u;
}

// ---- keys in registers: n <= NT * KPT.  Thread t owns KPT queries: for KPT < 4
// the consecutive queries t*KPT .. t*KPT + KPT - 1; for KPT a multiple of 4, KPT/4
// groups of 4 consecutive queries, group g of thread t starting at (g*NT + t)*4, so
// that the measures are read with fully coalesced 16-byte loads.  Index order is
// (group, thread, slot) order, which the emission restores with two work-group scans
// of per-group counts packed into 64 bits.
//
// The u-th largest key is found by narrowing an interval [lo, lo + span] of key
// values: each pass cuts the interval into up to 256 equal bins of 2^s keys,
// histograms the keys inside it (LDS atomics) and keeps the bin that holds the
// u-th largest.  The first interval is [min key, max key], so the bins spread
// over the measures that actually occur instead of over the float format.  After
// the first pass the surviving keys (a few hundred at most, as a rule) are
// compacted into LDS, one per thread, and the remaining passes cost next to nothing.
template <int NT>
struct SelectScratch {
    unsigned hist[256];
    unsigned red[2][NT / 64];
    unsigned cand[NT];
    unsigned n_cand;
    unsigned bin, need, count;
    unsigned long long cnt[2][NT / 64];
};

// Exclusive prefix sum over the work-group, in thread order, of four 16-bit
// counters packed into 64 bits (no field may exceed 65535 in total); `total`
// receives the packed sums.  Barriers inside; `cnt` is one row of NT/64 entries.
template <int NT>
__device__ __forceinline__ unsigned long long block_exclusive_scan4x16(unsigned long long v, unsigned long long* cnt,
                                                                       unsigned long long& total) {
    constexpr int NW = NT / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    if (lane == 63) cnt[wave] = incl;
    __syncthreads();
    unsigned long long before = incl - v;
    total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { const unsigned long long cw = cnt[w]; if (w < wave) before += cw; total += cw; }
    return before;
}

// Every thread of the work-group must call (barriers inside).  Writes the u
// selected indices, ascending, to out[0 .. u) and -1 to out[u .. u_max); `out`
// may point to LDS or to global memory.  `after_loads` is called by every thread
// once the loads of the measures are in flight (other work of the caller that
// waits for memory goes there; it may contain barriers).  `vec4`: the row Mh is
// 16-byte aligned (used for KPT a multiple of 4).
template <int NT, int KPT, typename F>
__device__ __forceinline__ void block_select(const float* __restrict__ Mh, bool vec4, int n, int u, int u_max,
                                             int* out, SelectScratch<NT>& sc, F&& after_loads)
{
    constexpr int NW = NT / 64;
    constexpr bool GROUPED = (KPT % 4) == 0;
    static_assert(KPT < 4 || GROUPED, "KPT must be 1, 2 or a multiple of 4");
    static_assert(KPT <= 16, "four 16-bit group counters");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto idx_of = [&](int k) -> int { return GROUPED ? ((k >> 2) * NT + tid) * 4 + (k & 3) : tid * KPT + k; };
    auto grp_of = [](int k) -> int { return GROUPED ? (k >> 2) : 0; };

    if (u <= 0) {                                              // n == 0
        after_loads();
        for (int t = tid; t < u_max; t += NT) out[t] = -1;
        return;
    }

    PSA_TS(0);
    float mv[KPT];
    if (GROUPED && vec4) {
#pragma unroll
        for (int g = 0; g < KPT / 4; ++g) {
            const int i0 = (g * NT + tid) * 4;
            // a group that starts at or beyond n is never used; one that straddles n lies inside the row
            const float4 x = *reinterpret_cast<const float4*>(Mh + (i0 < n ? i0 : 0));
            mv[4 * g + 0] = x.x; mv[4 * g + 1] = x.y; mv[4 * g + 2] = x.z; mv[4 * g + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int i = idx_of(k);
            mv[k] = Mh[i < n ? i : n - 1];                              // clamped, unconditional load
        }
    }
    after_loads();
    PSA_TS(1);
    unsigned keys[KPT];
    unsigned kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
        const unsigned key = order_key(mv[k]);
        keys[k] = key;
        if (idx_of(k) < n) {
            kmin = key < kmin ? key : kmin;
            kmax = key > kmax ? key : kmax;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned a = __shfl_xor(kmin, off, 64), b = __shfl_xor(kmax, off, 64);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { sc.red[0][wave] = kmin; sc.red[1][wave] = kmax; }
    if (tid == 0) sc.n_cand = 0u;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const unsigned a = sc.red[0][w], b = sc.red[1][w];
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }

    PSA_TS(2);
    // ---- narrow [lo, lo + span] down to the key of the u-th largest measure
    unsigned lo = kmin, span = kmax - kmin, need = (unsigned)u;
    bool all_from_lo = false;                  // keys >= lo are exactly the u largest
    bool compact = false;                      // keys come from sc.cand (one per thread) instead of registers
    unsigned ck = 0u;
    bool cvalid = false;
    while (span != 0u) {                       // work-group-uniform; at most 4 rounds (8 bits of span each)
        const int bits = 32 - __builtin_clz(span);
        const int s = bits > 8 ? bits - 8 : 0;
        for (int t = tid; t < 256; t += NT) sc.hist[t] = 0u;
        __syncthreads();
        if (!compact) {
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const unsigned off = keys[k] - lo;
                if (idx_of(k) < n && off <= span) atomicAdd(&sc.hist[off >> s], 1u);
            }
        } else {
            const unsigned off = ck - lo;
            if (cvalid && off <= span) atomicAdd(&sc.hist[off >> s], 1u);
        }
        __syncthreads();
        // wave 0 walks the histogram from the top: lane l owns bins 255-4l .. 252-4l
        if (wave == 0) {
            unsigned h4[4], local = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { h4[q] = sc.hist[255 - (4 * lane + q)]; local += h4[q]; }
            unsigned incl = local;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned v = __shfl_up(incl, off, 64);
                if (lane >= off) incl += v;
            }
            unsigned before = incl - local;              // keys in higher bins
            if (before < need && need <= incl) {         // exactly one lane
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (need <= before + h4[q]) {
                        sc.bin = (unsigned)(255 - (4 * lane + q));
                        sc.need = need - before;
                        sc.count = h4[q];
                        break;
                    }
                    before += h4[q];
                }
            }
        }
        __syncthreads();
        const unsigned bin = sc.bin, count = sc.count;
        need = sc.need;
        if (count == need) {
            // every key of this bin is kept: all keys from the bin's lower end upwards are the
            // u largest, and no finer look at the bin is needed (the usual exit: after two
            // rounds the bin of the cut-off holds a single key)
            lo += bin << s;
            all_from_lo = true;
            break;
        }
        const unsigned blo = bin << s;                   // offset of the bin inside the interval
        const unsigned rest = span - blo;                // offsets left from the bin's start to the interval's end
        const unsigned bspan = (s == 0) ? 0u : ((1u << s) - 1u);
        lo += blo;
        span = rest < bspan ? rest : bspan;
        if (!compact && span != 0u && count <= (unsigned)NT) {
            // the bin's keys move to LDS (in any order: only their values matter now)
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const unsigned off = keys[k] - lo;
                if (idx_of(k) < n && off <= span) sc.cand[atomicAdd(&sc.n_cand, 1u)] = keys[k];
            }
            __syncthreads();
            cvalid = (unsigned)tid < sc.n_cand;
            ck = sc.cand[tid];
            compact = true;
        }
    }
    // T: key of the u-th largest measure, `need` of the keys equal to it are kept (lowest indices
    // first); or, after the early exit, the lower end of the last bin, all keys from T upwards kept
    const unsigned T = lo;
    PSA_TS(3);

    // ---- emit in index order: (group, thread, slot)
    unsigned long long pk_eq = 0ull;
#pragma unroll
    for (int k = 0; k < KPT; ++k) pk_eq += (!all_from_lo && idx_of(k) < n && keys[k] == T) ? (1ull << (16 * grp_of(k))) : 0ull;
    // (ranks among the keys equal to T matter only when the cut-off falls among ties; the
    // flag is the same in every thread, so the scan's barriers stay uniform)
    unsigned long long tot_eq = 0ull, pre_eq = 0ull;
    if (!all_from_lo) pre_eq = block_exclusive_scan4x16<NT>(pk_eq, sc.cnt[0], tot_eq);
    unsigned take = 0u;
    unsigned long long pk_tk = 0ull;
    {
        unsigned base = 0u;                              // keys equal to T in earlier groups
        int g_prev = -1;
        unsigned eq_before = 0u;
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int g = grp_of(k);
            if (g != g_prev) {
                if (g_prev >= 0) base += (unsigned)((tot_eq >> (16 * g_prev)) & 0xFFFFull);
                eq_before = base + (unsigned)((pre_eq >> (16 * g)) & 0xFFFFull);
                g_prev = g;
            }
            const bool valid = idx_of(k) < n;
            const bool eq = !all_from_lo && valid && keys[k] == T;
            const bool tk = (valid && (keys[k] > T || (all_from_lo && keys[k] == T))) || (eq && eq_before < need);
            eq_before += eq ? 1u : 0u;
            take |= tk ? (1u << k) : 0u;
            pk_tk += tk ? (1ull << (16 * g)) : 0ull;
        }
    }
    unsigned long long tot_tk;
    const unsigned long long pre_tk = block_exclusive_scan4x16<NT>(pk_tk, sc.cnt[1], tot_tk);
    {
        unsigned base = 0u;
        int g_prev = -1;
        int pos = 0;
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
            const int g = grp_of(k);
            if (g != g_prev) {
                if (g_prev >= 0) base += (unsigned)((tot_tk >> (16 * g_prev)) & 0xFFFFull);
                pos = (int)(base + (unsigned)((pre_tk >> (16 * g)) & 0xFFFFull));
                g_prev = g;
            }
            if ((take >> k) & 1u) {
                if (pos < u_max) out[pos] = idx_of(k);
                ++pos;
            }
        }
    }
    for (int t = u + tid; t < u_max; t += NT) out[t] = -1;
    PSA_TS_DRAIN();
    PSA_TS(4);
}

// ---- any n: the keys are re-read from memory in every pass; most-significant-
// digit radix select, four passes of an 8-bit histogram.
template <int NT>
struct StreamSelectScratch {
    unsigned hist[256];
    unsigned prefix, need;
    int cnt[2][NT / 64];
};

// Every thread of the work-group must call (barriers inside).  Writes the u
// selected indices, ascending, to out[0 .. u) and -1 to out[u .. u_max); `out`
// may point to LDS or to global memory.
// KPT > 0: each thread keeps up to KPT keys in registers (n <= NT * KPT);
// KPT = 0: keys are re-read from memory in every pass (any n).
template <int NT, int KPT>
__device__ __forceinline__ void block_select_stream(const float* __restrict__ Mh, int n, int u, int u_max,
                                             int* out, StreamSelectScratch<NT>& sc)
{
    constexpr int NW = NT / 64;
    constexpr int KR = KPT > 0 ? KPT : 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    if (u <= 0) {
        for (int t = tid; t < u_max; t += NT) out[t] = -1;
        return;
    }

    // element k of thread t is query k * NT + t (coalesced, and index order is
    // kept within each k, which the emission pass relies on)
    unsigned keys[KR];
    if (KPT > 0) {
#pragma unroll
        for (int k = 0; k < KR; ++k) {
            const int i = k * NT + tid;
            const unsigned key = order_key(Mh[i < n ? i : n - 1]);      // clamped, unconditional load
            keys[k] = i < n ? key : 0u;
        }
    }
    const int n_iter = (n + NT - 1) / NT;
    auto key_at = [&](int k) -> unsigned {
        if (KPT > 0) return keys[k];
        const int i = k * NT + tid;
        const unsigned key = order_key(Mh[i < n ? i : n - 1]);
        return i < n ? key : 0u;
    };

    // ---- radix select of the u-th largest key, most significant byte first
    unsigned prefix = 0, need = (unsigned)u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int t = tid; t < 256; t += NT) sc.hist[t] = 0;
        __syncthreads();
        const unsigned himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
        auto count_one = [&](int k) {
            const int i = k * NT + tid;
            const unsigned key = key_at(k);
            const bool match = i < n && (key & himask) == prefix;
            const unsigned d = (key >> shift) & 255u;
            // Same-address LDS atomics serialise; measures of one head usually
            // share their leading byte, so count a wave-uniform digit once.
            const unsigned long long act = __ballot(match);
            if (act) {
                const int first = __ffsll((long long)act) - 1;
                const unsigned d0 = __shfl(d, first, 64);
                const unsigned long long same = __ballot(match && d == d0);
                if (same == act) {
                    if (lane == first) atomicAdd(&sc.hist[d0], (unsigned)__popcll(act));
                } else if (match) {
                    atomicAdd(&sc.hist[d], 1u);
                }
            }
        };
        if (KPT > 0) {
#pragma unroll
            for (int k = 0; k < KR; ++k) if (k < n_iter) count_one(k);
        } else {
            for (int k = 0; k < n_iter; ++k) count_one(k);
        }
        __syncthreads();
        // wave 0 walks the histogram from the top: lane l owns digits 255-4l .. 252-4l
        if (wave == 0) {
            unsigned h4[4], local = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { h4[q] = sc.hist[255 - (4 * lane + q)]; local += h4[q]; }
            unsigned incl = local;                       // inclusive prefix over lanes
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const unsigned v = __shfl_up(incl, off, 64);
                if (lane >= off) incl += v;
            }
            unsigned before = incl - local;              // keys with a larger digit
            if (before < need && need <= incl) {         // exactly one lane
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (need <= before + h4[q]) {
                        sc.prefix = prefix | ((unsigned)(255 - (4 * lane + q)) << shift);
                        sc.need = need - before;
                        break;
                    }
                    before += h4[q];
                }
            }
        }
        __syncthreads();
        prefix = sc.prefix;
        need = sc.need;
    }
    const unsigned T = prefix;      // key of the u-th largest measure; `need` equal keys are kept

    // ---- emit in index order
    int base_eq = 0, base_sel = 0;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    auto emit_one = [&](int k) {
        const int i = k * NT + tid;
        const unsigned key = key_at(k);
        const bool gt = i < n && key > T, eq = i < n && key == T;
        const unsigned long long beq = __ballot(eq);
        if (lane == 0) sc.cnt[0][wave] = __popcll(beq);
        __syncthreads();
        int eq_before = base_eq + __popcll(beq & lt_mask), eq_total = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) { const int cw = sc.cnt[0][w]; if (w < wave) eq_before += cw; eq_total += cw; }
        const bool take = gt || (eq && (unsigned)eq_before < need);
        const unsigned long long btk = __ballot(take);
        if (lane == 0) sc.cnt[1][wave] = __popcll(btk);
        __syncthreads();
        int pos = base_sel + __popcll(btk & lt_mask), tk_total = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) { const int cw = sc.cnt[1][w]; if (w < wave) pos += cw; tk_total += cw; }
        if (take && pos < u_max) out[pos] = i;
        base_eq += eq_total;
        base_sel += tk_total;
        __syncthreads();
    };
    if (KPT > 0) {
#pragma unroll
        for (int k = 0; k < KR; ++k) if (k < n_iter) emit_one(k);
    } else {
        for (int k = 0; k < n_iter; ++k) emit_one(k);
    }
    for (int t = u + tid; t < u_max; t += NT) out[t] = -1;
}

}  // namespace psa

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

// u_b = clamp(ceil(c ln n), 1, n), additionally capped by the host's bound.
__device__ __forceinline__ int n_selected(double c, int n, int u_max) {
    if (n <= 0) return 0;
    double x = ceil(c * log((double)n));
    if (!(x >= 1.0)) x = 1.0;
    if (x > (double)n) x = (double)n;
    int u = (int)x;
    return u > u_max ? u_max : u;
}

template <int NT>
struct SelectScratch {
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
__device__ __forceinline__ void block_select(const float* __restrict__ Mh, int n, int u, int u_max,
                                             int* out, SelectScratch<NT>& sc)
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

// -----------------------------------------------------------------------------
// The same selection by ONE wave, keys in registers (n <= 64 * KPL), no
// work-group barrier: used where the selection sits on the critical path of a
// larger work-group (the attend prologue), whose other waves meanwhile wait for
// their first K tile.  Element k of lane l is query k * 64 + l.
// `hist` is 256 words of LDS owned by the calling wave.
// -----------------------------------------------------------------------------
__device__ __forceinline__ unsigned wave_inclusive_scan(unsigned v) {
    // Hillis-Steele inside each row of 16 lanes (out-of-row sources read 0) ...
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);   // row_shr:8
    // ... then carry row totals: lane 15 -> rows 1 and 3, lane 31 -> rows 2 and 3
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
    v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31
    return v;
}

__device__ __forceinline__ int lanes_below(unsigned long long mask) {
    return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
}

template <int KPL>
__device__ __forceinline__ void wave_select(const float* __restrict__ Mh, int n, int u, int u_max,
                                            int* out, unsigned* hist)
{
    const int lane = threadIdx.x & 63;
    if (u <= 0) {
        for (int t = lane; t < u_max; t += 64) out[t] = -1;
        return;
    }
    unsigned keys[KPL];
#pragma unroll
    for (int k = 0; k < KPL; ++k) {
        const int i = k * 64 + lane;
        const unsigned key = order_key(Mh[i < n ? i : n - 1]);          // clamped, unconditional load
        keys[k] = i < n ? key : 0u;
    }
    const int n_iter = (n + 63) >> 6;

    unsigned prefix = 0, need = (unsigned)u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        *reinterpret_cast<uint4*>(hist + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
        wave_lds_sync();
        const unsigned himask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            if (k < n_iter) {
                const int i = k * 64 + lane;
                const bool match = i < n && (keys[k] & himask) == prefix;
                const unsigned d = (keys[k] >> shift) & 255u;
                // same-address LDS atomics serialise: count a wave-uniform digit once
                const unsigned long long act = __ballot(match);
                if (act) {
                    const int first = __ffsll((long long)act) - 1;
                    const unsigned d0 = (unsigned)__builtin_amdgcn_readlane((int)d, first);
                    const unsigned long long same = __ballot(match && d == d0);
                    if (same == act) {
                        if (lane == first) atomicAdd(&hist[d0], (unsigned)__popcll(act));
                    } else if (match) {
                        atomicAdd(&hist[d], 1u);
                    }
                }
            }
        }
        wave_lds_sync();
        // lane l owns digits 255-4l .. 252-4l: walk the histogram from the top
        const uint4 hv = *reinterpret_cast<const uint4*>(hist + 252 - 4 * lane);   // digits 252-4l .. 255-4l
        const unsigned h4[4] = {hv.w, hv.z, hv.y, hv.x};
        const unsigned local = h4[0] + h4[1] + h4[2] + h4[3];
        const unsigned incl = wave_inclusive_scan(local);
        unsigned before = incl - local;              // keys with a larger digit
        const bool found = before < need && need <= incl;       // exactly one lane
        unsigned new_prefix = 0, new_need = 0;
        if (found) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (need <= before + h4[q]) {
                    new_prefix = prefix | ((unsigned)(255 - (4 * lane + q)) << shift);
                    new_need = need - before;
                    break;
                }
                before += h4[q];
            }
        }
        const int src = __ffsll((long long)__ballot(found)) - 1;
        prefix = (unsigned)__builtin_amdgcn_readlane((int)new_prefix, src);
        need = (unsigned)__builtin_amdgcn_readlane((int)new_need, src);
        wave_lds_sync();
    }
    const unsigned T = prefix;      // key of the u-th largest measure; `need` equal keys are kept

    int base_eq = 0, base_sel = 0;
#pragma unroll
    for (int k = 0; k < KPL; ++k) {
        if (k < n_iter) {
            const int i = k * 64 + lane;
            const bool gt = i < n && keys[k] > T, eq = i < n && keys[k] == T;
            const unsigned long long beq = __ballot(eq);
            const bool take = gt || (eq && (unsigned)(base_eq + lanes_below(beq)) < need);
            const unsigned long long btk = __ballot(take);
            const int pos = base_sel + lanes_below(btk);
            if (take && pos < u_max) out[pos] = i;
            base_eq += __popcll(beq);
            base_sel += __popcll(btk);
        }
    }
    for (int t = u + lane; t < u_max; t += 64) out[t] = -1;
}

}  // namespace psa

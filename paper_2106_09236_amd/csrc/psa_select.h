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

}  // namespace psa

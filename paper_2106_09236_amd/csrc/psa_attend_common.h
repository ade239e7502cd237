// Parts of the attend stage that do not depend on the tensor type: the prologue
// (top-u selection of the head, mean of the valid V rows), the fill of the
// unselected rows (stage a4) and the hand-over by which the LAST work-group of a
// head to finish merges the per-split partial softmax results into the
// selected rows (end of stage a3).
#pragma once

#include "psa_device.h"
#include "psa_internal.h"
#include "psa_select.h"

namespace psa {

// Kernel arguments of the attend stage (passed by value).
struct AttendParams {
    const void* Q; const void* K; const void* V;
    const int* lengths;
    const float* M;          // [BH, L] sampled measure (stage a1)
    const double* vpart;     // [BH, n_chunk, 64] column sums of V per measure chunk
    const float* mu;         // [BH, 64] mean of V, written by the select kernel (long heads)
    int* sel;                // [BH, u_max]
    int* ucount;             // [B]
    int* ticket;             // [BH] zero on entry (stage a1 clears it, the last work-group resets it)
    void* part;              // partial records
    void* out;
    int H, L, u_max, n_split, n_qgroup, rounds, part_stride, n_chunk, fused_select, rows_per_wg;
    double c;
};

template <int NT>
struct CommonScratch {
    SelectScratch<NT> select;
    float mean[kD];
    int sel[kFusedSelectMaxL];       // I_sparse of the head when selected in this work-group
    unsigned char flag[512];
    int last;
};

// ---- prologue: I_sparse and the mean of the valid V rows.
// Short heads: every work-group repeats the selection (a few KB of measures, L2
// hits; it runs while the first K tile is still in flight) and sums the few
// per-chunk V partials.  Long heads: both come from the select kernel.
// Returns the pointer to the head's selected indices (LDS or global) and u.
template <int NT>
__device__ __forceinline__ const int* attend_prologue(const AttendParams& P, int head, int n, int wg_in_head,
                                                      CommonScratch<NT>& cs, int& u)
{
    const int tid = threadIdx.x;
    const int b = head / P.H;
    const int* selp;
    if (P.fused_select) {
        u = n_selected(P.c, n, P.u_max);
        // wave 0 selects (keys in registers, no barrier); wave 1 sums the V partials
        if (tid < 64) {
            if (P.L <= 512) wave_select<8>(P.M + (size_t)head * P.L, n, u, P.u_max, cs.sel, cs.select.hist);
            else            wave_select<kFusedSelectMaxL / 64>(P.M + (size_t)head * P.L, n, u, P.u_max, cs.sel, cs.select.hist);
        } else if (tid < 64 + kD) {
            const int e = tid - 64;
            double t = 0.0;
            for (int ch = 0; ch < P.n_chunk; ++ch) t += P.vpart[((size_t)head * P.n_chunk + ch) * kD + e];   // fixed order
            cs.mean[e] = n > 0 ? (float)(t / (double)n) : 0.f;
        }
        __syncthreads();
        if (wg_in_head == 0) {                       // publish for the taps and for later calls that reuse I_sparse
            for (int t = tid; t < P.u_max; t += NT) P.sel[(size_t)head * P.u_max + t] = cs.sel[t];
            if (tid == 0 && head % P.H == 0) P.ucount[b] = u;
        }
        selp = cs.sel;
    } else {
        u = P.ucount[b];
        if (tid < kD) cs.mean[tid] = P.mu[(size_t)head * kD + tid];
        __syncthreads();
        selp = P.sel + (size_t)head * P.u_max;
    }
    return selp;
}

// ---- 16-byte row stores of the output type
template <typename T> struct OutTraits;
template <> struct OutTraits<float> {
    static constexpr int LPR = 16, EPL = 4;
    static __device__ __forceinline__ void store(float* row, int sub, const float* v) {
        reinterpret_cast<float4*>(row)[sub] = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct OutTraits<bf16_t> {
    static constexpr int LPR = 8, EPL = 8;
    static __device__ __forceinline__ void store(bf16_t* row, int sub, const float* v) {
        reinterpret_cast<uint4*>(row)[sub] = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]),
                                                        pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    }
};

// ---- stage a4 for rows [r0, r0 + rows) of the head: a valid row that is not
// selected receives the mean of the valid V rows (Sec. 3.1: uniform scores give
// the plain average of the values); a row at or beyond the length receives zeros.
template <typename T, int NT>
__device__ __forceinline__ void fill_rows(T* out_head, const int* selp, int u, int n, int L, int r0, int rows,
                                          CommonScratch<NT>& cs)
{
    using OT = OutTraits<T>;
    constexpr int LPR = OT::LPR, EPL = OT::EPL, RPP = NT / LPR;
    const int tid = threadIdx.x, sub = tid % LPR, row = tid / LPR;
    float mean[EPL], zero[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) { mean[e] = cs.mean[sub * EPL + e]; zero[e] = 0.f; }
    for (int blk = 0; blk < rows; blk += 512) {
        const int nb = rows - blk < 512 ? rows - blk : 512;
        const int lo = r0 + blk;
        for (int t = tid; t < nb; t += NT) cs.flag[t] = 0;
        __syncthreads();
        for (int t = tid; t < u; t += NT) {
            const int i = selp[t];
            if (i >= lo && i < lo + nb) cs.flag[i - lo] = 1;
        }
        __syncthreads();
        for (int rl = row; rl < nb; rl += RPP) {
            const int i = lo + rl;
            if (i >= L) break;
            if (i >= n) OT::store(out_head + (size_t)i * kD, sub, zero);
            else if (!cs.flag[rl]) OT::store(out_head + (size_t)i * kD, sub, mean);
        }
        __syncthreads();
    }
}

// Partial records cross work-groups (and XCDs, whose L2s are not coherent with
// each other) inside one kernel.  They are written and read with agent-scope
// relaxed atomic accesses, which go through to memory element by element, so no
// cache-wide write-back or invalidate is needed around the ticket.
template <typename R> __device__ __forceinline__ void rec_store(R* p, R v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename R> __device__ __forceinline__ R rec_load(const R* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float  rec_exp2(float x)  { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ double rec_exp2(double x) { return exp2_f64(x); }

// ---- hand-over: every work-group of the head makes its stores visible and takes
// a ticket; the one that draws the last ticket merges the head's records, in
// split order, into the selected rows of `out`.  No work-group ever waits for
// another, so the scheme cannot deadlock whatever the residency.
// R: record element type.  ACC_LAYOUT: O stored in accumulator layout (blocks
// of [16 registers][64 lanes] per 16 queries) instead of [query][64].
template <typename T, typename R, bool ACC_LAYOUT, int NT>
__device__ __forceinline__ void ticket_and_merge(const AttendParams& P, int head, int n, int u, const int* selp,
                                                 int nq, CommonScratch<NT>& cs)
{
    using OT = OutTraits<T>;
    constexpr int LPR = OT::LPR, EPL = OT::EPL, RPP = NT / LPR;
    const int tid = threadIdx.x, sub = tid % LPR, row = tid / LPR;
    const int n_wg_head = P.n_split * P.n_qgroup;

    // The barrier waits for every wave's record stores to complete (they are
    // agent-scope write-through stores, complete means in memory); one thread
    // then takes the ticket.  The work-group that draws the last ticket reads the
    // other work-groups' records with agent-scope loads.
    __syncthreads();
    if (tid == 0) {
        const int t = __hip_atomic_fetch_add(P.ticket + head, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = (t == n_wg_head - 1);
        if (last) __hip_atomic_store(P.ticket + head, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
        cs.last = last;
    }
    __syncthreads();
    if (!cs.last) return;

    T* out_head = static_cast<T*>(P.out) + (size_t)head * P.L * kD;
    const R* part = static_cast<const R*>(P.part);
    for (int rank = row; rank < u; rank += RPP) {
        const int i = selp[rank];
        if (i < 0 || i >= n) continue;
        const int qg = rank / nq, q = rank % nq;
        const R* base = part + ((size_t)head * P.n_qgroup + qg) * P.n_split * P.part_stride;
        // online merge, 4 splits per step; every split has a record (empty ones
        // carry m = -inf, l = 0, O = 0)
        R mx = -INFINITY, lt = 0, acc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = 0;
        for (int s0 = 0; s0 < P.n_split; s0 += 4) {
            R m4[4], l4[4], o4[4][EPL];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int s = s0 + k < P.n_split ? s0 + k : P.n_split - 1;
                const R* rec = base + (size_t)s * P.part_stride;
                const R mv = rec_load(rec + q);
                m4[k] = s0 + k < P.n_split ? mv : (R)-INFINITY;
                l4[k] = rec_load(rec + nq + q);
                if (ACC_LAYOUT) {
                    // EPL = 4 elements 4*sub .. +3 = register `sub`, lanes e*16 + q%16
                    const R* o = rec + 2 * nq + (q >> 4) * 1024 + sub * 64 + (q & 15);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) o4[k][e] = rec_load(o + e * 16);
                } else {
                    const R* o = rec + 2 * nq + q * kD + sub * EPL;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) o4[k][e] = rec_load(o + e);
                }
            }
            R cm = mx;
#pragma unroll
            for (int k = 0; k < 4; ++k) cm = m4[k] > cm ? m4[k] : cm;
            if (cm == (R)-INFINITY) continue;
            const R a = (mx == (R)-INFINITY) ? (R)0 : rec_exp2(mx - cm);
            lt *= a;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] *= a;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const R sc = (m4[k] == (R)-INFINITY) ? (R)0 : rec_exp2(m4[k] - cm);
                lt += sc * l4[k];
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] += sc * o4[k][e];
            }
            mx = cm;
        }
        float val[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) val[e] = lt > 0 ? (float)(acc[e] / lt) : 0.f;
        OT::store(out_head + (size_t)i * kD, sub, val);
    }
}

}  // namespace psa

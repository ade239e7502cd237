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
    const double* vpart;     // [BH, n_vpart, 64] column sums of V (per measure chunk or per segment)
    const float* mu;         // [BH, 64] mean of V, written by the select kernel (long heads)
    int* sel;                // [BH, u_max]
    int* ucount;             // [B]
    int* ticket;             // [BH] zero on entry (stage a1 clears it, the last work-group resets it)
    const uint2* cand;       // [BH, n_chunk, cand_len] sorted per-chunk candidates (cand_len > 0), else unused
    const int* given_sel;    // non-null: caller's index sets [BH, u_max], checked inside the attend work-groups ...
    const int* given_u;      // ... with their lengths [B]; vpart then holds the V column sums, n_chunk of them per head
    void* part;              // partial records
    void* out;
    int H, L, u_max, n_split, n_qgroup, rounds, part_stride, n_chunk, fused_select, rows_per_wg, cand_len;
    int n_vpart;             // column-sum vectors of V per head in `vpart` (as many as lists, or one per measure chunk)
    int separate_merge;      // 1: records are merged by the merge kernel, not by the last work-group
    int nq;                  // selected queries per query group (= per record)
    int fill;                // psa_fill_t: what the unselected valid rows receive
    URule urule;
};

// NSEL: longest index list kept in LDS; NCAND: most candidates (lists * list length) the prologue merges.
// The single-launch kernel for short heads uses a small instance (64 / 256) so that two of its
// work-groups fit a CU.
template <int NT, int NSEL = kSelLdsMax, int NCAND = kMaxCandidates>
struct CommonScratch {
    static constexpr int kSel = NSEL, kCand = NCAND;
    float mean[kD];
    int sel[NSEL];                   // I_sparse of the head
    unsigned ckey[NCAND];            // candidate lists of the head: order keys ...
    int cidx[NCAND];                 // ... and query indices (-1 = empty slot)
    unsigned char flag[512];
    int plen[8];                     // per list: how many of its first entries can be among the u best
    int last;
};

// ---- prologue: I_sparse and the mean of the valid V rows.
// Two ways, by the shape of the problem (decided on the host):
//  * candidate lists (short heads measured by the LDS kernel): the measure stage
//    left, per chunk of the head, its best queries sorted by decreasing measure
//    (ties: lower index first).  The position of a candidate in the merged order
//    is its position in its own list plus, for every other list, the number of
//    entries that come before it: one binary search per (candidate, list), spread
//    over the lanes of a group of 8.
//  * otherwise: I_sparse and the mean come from the select kernel.
// `issue_tile` is called once the prologue's own loads are in flight: the caller
// requests its first K tile there, so that the tile streams in behind them while
// the selection runs (barriers inside are LDS-only and do not wait for it).
// Returns the pointer to the head's selected indices (LDS or global) and u.
template <int NT, typename CS, typename F>
__device__ __forceinline__ const int* attend_prologue(const AttendParams& P, int head, int n, int wg_in_head,
                                                      CS& cs, int& u, F&& issue_tile)
{
    const int tid = threadIdx.x;
    const int b = head / P.H;
    const int* selp;
    // The last wave sums the per-chunk float64 column sums of V (fixed order).  The
    // first 8 chunks are requested BEFORE the K tile (loads complete in issue order,
    // so anything requested after the tile would wait for all of it).
    double vsum = 0.0;
    const int e = tid - (NT - kD);
    double vp0[8];
    auto load_vpart = [&](double (&vp)[8], int c0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int c2 = c0 + k < P.n_vpart ? c0 + k : P.n_vpart - 1;
            const double* src = P.vpart + ((size_t)head * P.n_vpart + c2) * kD + (e >= 0 ? e : 0);
            vp[k] = *src;
        }
    };
    auto add_vpart = [&](const double (&vp)[8], int c0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) vsum += c0 + k < P.n_vpart ? vp[k] : 0.0;
    };
    auto sum_vpart = [&]() {
        add_vpart(vp0, 0);
        for (int c0 = 8; c0 < P.n_vpart; c0 += 8) { double vp[8]; load_vpart(vp, c0); add_vpart(vp, c0); }
    };
    if (P.given_sel) {
        // caller-given index sets (Sec. 4.4): entries beyond u_b or outside the item's frames become -1
        // and are skipped; the mean of V comes from the column sums, as below
        const int* gsel = P.given_sel + (size_t)head * P.u_max;
        constexpr int SPT = (CS::kSel + NT - 1) / NT;              // entries per thread (u_max <= CS::kSel here)
        int sv[SPT];
#pragma unroll
        for (int k = 0; k < SPT; ++k) { const int t = k * NT + tid; sv[k] = gsel[t < P.u_max ? t : P.u_max - 1]; }
        int ub = P.given_u[b];
        if (e >= 0) load_vpart(vp0, 0);
        ub = ub < 0 ? 0 : ub;
        ub = ub > P.u_max ? P.u_max : ub;
        u = ub > n ? n : ub;
        if (e >= 0) sum_vpart();
        issue_tile();
#pragma unroll
        for (int k = 0; k < SPT; ++k) {
            const int t = k * NT + tid;
            if (t < P.u_max) cs.sel[t] = (t < u && sv[k] >= 0 && sv[k] < n) ? sv[k] : -1;
        }
        if (e >= 0) cs.mean[e] = n > 0 ? (float)(vsum / (double)n) : 0.f;
        for (int t = tid; t < 512; t += NT) cs.flag[t] = 0;         // for fill_rows: its first block needs no barrier of its own
        lds_barrier();
        if (wg_in_head == 0) {                       // publish for later calls that reuse the sets
            for (int t = tid; t < P.u_max; t += NT) P.sel[(size_t)head * P.u_max + t] = cs.sel[t];
            if (tid == 0 && head % P.H == 0) P.ucount[b] = u;
        }
        selp = cs.sel;
    } else if (P.fused_select) {                 // implies candidate lists (cand_len > 0)
        {
            constexpr int CPT = (CS::kCand + NT - 1) / NT;         // candidates per thread
            const int total = P.n_chunk * P.cand_len;
            const uint2* ch = P.cand + (size_t)head * total;
            uint2 ce[CPT];
#pragma unroll
            for (int k = 0; k < CPT; ++k) {
                const int t = k * NT + tid;
                const uint2* src = ch + (t < total ? t : total - 1);
                ce[k] = *src;
            }
            if (e >= 0) load_vpart(vp0, 0);
            u = n_selected(P.urule, n, P.u_max);
#pragma unroll
            for (int k = 0; k < CPT; ++k) {
                const int t = k * NT + tid;
                if (t < total) { cs.ckey[t] = ce[k].x; cs.cidx[t] = (int)ce[k].y; }
            }
            if (e >= 0) sum_vpart();
            // the small loads are back: only now ask for the K tile, so that the burst of
            // tile requests of all work-groups does not delay them
            issue_tile();
            for (int t = tid; t < P.u_max; t += NT) cs.sel[t] = -1;
            if (e >= 0) cs.mean[e] = n > 0 ? (float)(vsum / (double)n) : 0.f;
            PSA_TS(9);
            lds_barrier();
            PSA_TS(10);
            // lane g of a group of 4 (up to 4 lists) or 8 searches list g for the group's candidate
            const int gs = P.n_chunk <= 4 ? 2 : 3;
            const int len = P.cand_len, nl = P.n_chunk;
            if ((total << gs) <= NT || nl <= 4 || nl > 8 || u < 1) {
                for (int t0 = 0; t0 < (total << gs); t0 += NT) {
                    const int t = t0 + tid;
                    const int ci = t >> gs, c2 = t & ((1 << gs) - 1);
                    int cnt = 0;
                    unsigned key = 0u;
                    int qidx = -1, mych = 0;
                    if (ci < total) {
                        key = cs.ckey[ci]; qidx = cs.cidx[ci];
                        mych = ci / len;
                        if (c2 == mych) {
                            cnt = ci - mych * len;                      // its position in its own list
                        } else if (c2 < nl) {
                            const unsigned* lst = cs.ckey + c2 * len;
                            int lo = 0, hi = len;                       // first entry that does not come before mine
                            while (lo < hi) {
                                const int mid = (lo + hi) >> 1;
                                const unsigned ek = lst[mid];
                                const bool before = ek > key || (ek == key && c2 < mych);   // lower chunk = lower index
                                if (before) lo = mid + 1; else hi = mid;
                            }
                            cnt = lo;
                        }
                    }
                    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0xB1, 0xF, 0xF, false);      // sum over the group's lanes
                    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x4E, 0xF, 0xF, false);
                    if (gs == 3) cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x141, 0xF, 0xF, false);
                    if (c2 == 0 && ci < total && key != 0u && qidx >= 0 && cnt < u) cs.sel[cnt] = qidx;
                }
            } else {
                // More than 4 lists and more candidates than threads can take in one trip (8 lists of 49: seven
                // trips of 1.5 thousand cycles in every work-group of the head).  Most of them cannot be among the u best: with
                // p = ceil(u / lists), at least u candidates are no smaller than T = the least of the lists'
                // p-th keys, so only each list's prefix of keys >= T takes part; a candidate's place among
                // those is its place among all (everything that comes before it is >= T as well).
                if (tid < 8) {
                    const int pp = (u + nl - 1) / nl - 1;
                    unsigned tl = 0xFFFFFFFFu;
                    for (int l2 = 0; l2 < nl; ++l2) { const unsigned k2 = pp < len ? cs.ckey[l2 * len + pp] : 0u; tl = k2 < tl ? k2 : tl; }
                    int lo = 0, hi = tid < nl ? len : 0;                // entries of list tid with key >= T
                    const unsigned* lst = cs.ckey + (tid < nl ? tid : 0) * len;
                    while (lo < hi) { const int mid = (lo + hi) >> 1; if (lst[mid] >= tl) lo = mid + 1; else hi = mid; }
                    cs.plen[tid] = lo;
                }
                lds_barrier();
                int off[9];
                off[0] = 0;
#pragma unroll
                for (int l2 = 0; l2 < 8; ++l2) off[l2 + 1] = off[l2] + cs.plen[l2];
                const int total2 = off[8];
                for (int t0 = 0; t0 < (total2 << gs); t0 += NT) {
                    const int t = t0 + tid;
                    const int ci = t >> gs, c2 = t & ((1 << gs) - 1);
                    int cnt = 0, qidx = -1;
                    unsigned key = 0u;
                    if (ci < total2) {
                        int mych = 0;
#pragma unroll
                        for (int l2 = 1; l2 < 8; ++l2) mych += ci >= off[l2] ? 1 : 0;       // (off[l2] = total2 beyond the last list)
                        const int rk = ci - off[mych];
                        key = cs.ckey[mych * len + rk]; qidx = cs.cidx[mych * len + rk];
                        if (c2 == mych) {
                            cnt = rk;                                   // its position in its own list
                        } else if (c2 < nl) {
                            const unsigned* lst = cs.ckey + c2 * len;
                            int lo = 0, hi = cs.plen[c2];               // first entry that does not come before mine
                            while (lo < hi) {
                                const int mid = (lo + hi) >> 1;
                                const unsigned ek = lst[mid];
                                const bool before = ek > key || (ek == key && c2 < mych);   // lower chunk = lower index
                                if (before) lo = mid + 1; else hi = mid;
                            }
                            cnt = lo;
                        }
                    }
                    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0xB1, 0xF, 0xF, false);      // sum over the group's lanes
                    cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x4E, 0xF, 0xF, false);
                    if (gs == 3) cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x141, 0xF, 0xF, false);
                    if (c2 == 0 && ci < total2 && key != 0u && qidx >= 0 && cnt < u) cs.sel[cnt] = qidx;
                }
            }
            PSA_TS(11);
        }
        for (int t = tid; t < 512; t += NT) cs.flag[t] = 0;         // for fill_rows: its first block needs no barrier of its own
        lds_barrier();
        PSA_TS(12);
        if (wg_in_head == 0) {                       // publish for the taps and for later calls that reuse I_sparse
            for (int t = tid; t < P.u_max; t += NT) P.sel[(size_t)head * P.u_max + t] = cs.sel[t];
            if (tid == 0 && head % P.H == 0) P.ucount[b] = u;
        }
        selp = cs.sel;
    } else {
        // I_sparse, u and the mean come from the select kernel; the index list is
        // copied to LDS when it fits, so that later reads do not go to memory again
        const int* gsel = P.sel + (size_t)head * P.u_max;
        const int s0v = gsel[tid < P.u_max ? tid : P.u_max - 1];
        u = P.ucount[b];
        const float mv = P.mu[(size_t)head * kD + (tid & (kD - 1))];
        issue_tile();
        selp = gsel;
        if (P.u_max <= CS::kSel) {
            if (tid < P.u_max) cs.sel[tid] = s0v;
            for (int t = tid + NT; t < P.u_max; t += NT) cs.sel[t] = gsel[t];
            selp = cs.sel;
        }
        if (tid < kD) cs.mean[tid] = mv;
        for (int t = tid; t < 512; t += NT) cs.flag[t] = 0;         // for fill_rows (see above)
        lds_barrier();
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
// the plain average of the values) or, with VALUE_FILL, its own row of V (Eq. 12
// as printed); a row at or beyond the length receives zeros.
template <typename T, int NT, bool VALUE_FILL, typename CS>
__device__ __forceinline__ void fill_rows_impl(T* out_head, const T* V_head, const int* selp, int u, int n, int L,
                                               int r0, int rows, CS& cs)
{
    using OT = OutTraits<T>;
    constexpr int LPR = OT::LPR, EPL = OT::EPL, RPP = NT / LPR;
    const int tid = threadIdx.x, sub = tid % LPR, row = tid / LPR;
    float mean[EPL], zero[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) { mean[e] = cs.mean[sub * EPL + e]; zero[e] = 0.f; }
    // cs.flag[t] = 1: row lo + t of the current block of 512 rows is selected.  The prologue left the
    // flags at zero behind a barrier, so the first block (the only one, as a rule) starts marking at once.
    for (int blk = 0; blk < rows; blk += 512) {
        const int nb = rows - blk < 512 ? rows - blk : 512;
        const int lo = r0 + blk;
        if (blk > 0) {
            lds_barrier();                                // the previous block's flags have been read
            for (int t = tid; t < nb; t += NT) cs.flag[t] = 0;
            lds_barrier();
        }
        for (int t = tid; t < u; t += NT) {
            const int i = selp[t];
            if (i >= lo && i < lo + nb) cs.flag[i - lo] = 1;
        }
        lds_barrier();
        if (VALUE_FILL) {
            // copies of 16 bytes, the loads unconditional on a clamped row and four in flight
#pragma unroll 4
            for (int rl = row; rl < nb; rl += RPP) {
                const int i = lo + rl;
                const int ic = i < n ? i : (n > 0 ? n - 1 : 0);
                uint4 v = reinterpret_cast<const uint4*>(V_head + (size_t)ic * kD)[sub];
                if (i >= n) v = make_uint4(0u, 0u, 0u, 0u);
                if (i < L && (i >= n || !cs.flag[rl])) reinterpret_cast<uint4*>(out_head + (size_t)i * kD)[sub] = v;
            }
        } else {
            for (int rl = row; rl < nb; rl += RPP) {
                const int i = lo + rl;
                if (i >= L) break;
                if (i >= n) OT::store(out_head + (size_t)i * kD, sub, zero);
                else if (!cs.flag[rl]) OT::store(out_head + (size_t)i * kD, sub, mean);
            }
        }
    }
}
template <typename T, int NT, typename CS>
__device__ __forceinline__ void fill_rows(const AttendParams& P, T* out_head, const T* V_head, const int* selp,
                                          int u, int n, int wg_in_head, CS& cs)
{
    if (P.fill == PSA_FILL_VALUE)
        fill_rows_impl<T, NT, true>(out_head, V_head, selp, u, n, P.L, wg_in_head * P.rows_per_wg, P.rows_per_wg, cs);
    else
        fill_rows_impl<T, NT, false>(out_head, V_head, selp, u, n, P.L, wg_in_head * P.rows_per_wg, P.rows_per_wg, cs);
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
// R: record element type.  ACC_LAYOUT (float32 tensors): O stored in accumulator layout (blocks
// of [16 registers][64 lanes] per 16 queries) instead of [query][64], as float32 values O / l behind
// the float64 m and l.
template <typename T, typename R, bool ACC_LAYOUT, int NT, typename CS>
__device__ __forceinline__ void ticket_and_merge(const AttendParams& P, int head, int n, int u, const int* selp,
                                                 int nq, CS& cs)
{
    using OT = OutTraits<T>;
    constexpr int LPR = OT::LPR, EPL = OT::EPL, RPP = NT / LPR;
    const int tid = threadIdx.x, sub = tid % LPR, row = tid / LPR;
    const int n_wg_head = P.n_split * P.n_qgroup;
    if (P.separate_merge) return;

    // Ordering of the hand-over, made explicit rather than left to what the barrier
    // happens to emit: every wave first waits until its own record stores have been
    // acknowledged (they are agent-scope write-through stores: acknowledged means in
    // memory, visible to every XCD), then joins the barrier; only after the barrier
    // does one thread take the ticket.  So the ticket of a work-group can become
    // visible only after all of its records are.  The work-group that draws the
    // last ticket reads the other work-groups' records with agent-scope loads,
    // which bypass its own caches.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
                    // float32 values O / l.  EPL = 4 elements 4*sub + e: accumulator register 4e + sub/4 of lane
                    // group sub%4 (lanes 16 (sub%4) + q%16)
                    const float* o = reinterpret_cast<const float*>(rec + 2 * nq) + (q >> 4) * 1024 + (sub >> 2) * 64 + (sub & 3) * 16 + (q & 15);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) o4[k][e] = (R)rec_load(o + e * 256);
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
                const R wo = ACC_LAYOUT ? sc * l4[k] : sc;           // (those records hold O / l)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] += wo * o4[k][e];
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

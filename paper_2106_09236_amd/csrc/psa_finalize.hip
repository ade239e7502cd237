// Stage a3 (merge) + a4: writes every row of `out`.
//   selected query   -> merge of its per-split partial softmax results     (Eq. 8, Eq. 12 upper branch)
//   other valid row  -> mean of the valid V rows (Sec. 3.1: a query with uniform
//                       scores yields the plain average of the values)
//   row >= length    -> zeros
// Pure data movement: 16 (f32) or 8 (bf16) adjacent lanes write one 256 B / 128 B
// row with one 16-byte store each.  Partials are merged in split order, so the
// result is independent of scheduling.
#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

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

__device__ __forceinline__ float  rec_exp2(float x)  { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ double rec_exp2(double x) { return exp2_f64(x); }

constexpr int kMaxFinalRows = 512;     // upper bound of rows per fill work-group

// Two kinds of work-group share one launch so that they overlap:
//   blockIdx.x <  n_fill : FILL   rows [x * rows_per_wg, ...) that are not selected:
//                          mean of the valid V rows, or zeros beyond the length
//   blockIdx.x == n_fill : MERGE  the u selected rows of the head from the
//                          per-split partial softmax records, in split order
// R is the element type of the records: double for float32 tensors (merged in
// float64, rounded once on the store), float for bfloat16 tensors.
template <typename T, typename R>
__global__ __launch_bounds__(256)
void finalize_kernel(const int* __restrict__ lengths, const int* __restrict__ sel,
                     const double* __restrict__ vsum, const R* __restrict__ part, T* __restrict__ out,
                     int H, int L, int u_max, int n_split, int n_qgroup, int nq, int part_stride,
                     int rows_per_wg, int n_fill)
{
    using OT = OutTraits<T>;
    constexpr int LPR = OT::LPR, EPL = OT::EPL, RPP = 256 / LPR;
    __shared__ unsigned char s_sel[kMaxFinalRows];
    __shared__ float s_mean[kD];

    const int head = blockIdx.y;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x;
    const int sub = tid % LPR, row = tid / LPR;
    const int* selh = sel + (size_t)head * u_max;

    if ((int)blockIdx.x == n_fill) {
        // ------------------------------------------------------------- MERGE
        for (int rank = row; rank < u_max; rank += RPP) {
            const int i = selh[rank];                               // -1 beyond u_b
            if (i < 0 || i >= n) continue;
            const int qg = rank / nq, q = rank % nq;
            const R* base = part + ((size_t)head * n_qgroup + qg) * n_split * part_stride;
            // online merge, 4 splits per step; every split has a record (empty
            // ones carry m = -inf, l = 0, O = 0)
            R mx = -INFINITY, lt = 0, acc[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = 0;
            for (int s0 = 0; s0 < n_split; s0 += 4) {
                R m4[4], l4[4], o4[4][EPL];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int s = s0 + k < n_split ? s0 + k : n_split - 1;
                    const R* rec = base + (size_t)s * part_stride;
                    m4[k] = s0 + k < n_split ? rec[q] : (R)-INFINITY;
                    l4[k] = rec[nq + q];
                    if (sizeof(R) == 8) {
                        // float32 tensors: O in accumulator layout, blocks of [16 registers][64 lanes]
                        // per column tile of 16 queries; EPL = 4 elements = register `sub`, lanes e*16 + q%16
                        const R* o = rec + 2 * nq + (q >> 4) * 1024 + sub * 64 + (q & 15);
#pragma unroll
                        for (int e = 0; e < EPL; ++e) o4[k][e] = o[e * 16];
                    } else {
                        const R* o = rec + 2 * nq + q * kD + sub * EPL;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) o4[k][e] = o[e];
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
            OT::store(out + ((size_t)head * L + i) * kD, sub, val);
        }
        return;
    }

    // ------------------------------------------------------------------ FILL
    const int r0 = blockIdx.x * rows_per_wg;
    // both loads are issued before the barrier: the selected indices and the
    // per-split float64 column sums of V (summed in split order)
    int my_sel[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) { const int t = tid + 256 * k; my_sel[k] = t < u_max ? selh[t] : -1; }
    double t = 0.0;
    if (tid < kD) for (int s = 0; s < n_split; ++s) t += vsum[((size_t)head * n_split + s) * kD + tid];
    for (int r = tid; r < rows_per_wg; r += 256) s_sel[r] = 0;
    if (tid < kD) s_mean[tid] = n > 0 ? (float)(t / (double)n) : 0.f;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 2; ++k) if (my_sel[k] >= r0 && my_sel[k] < r0 + rows_per_wg) s_sel[my_sel[k] - r0] = 1;
    for (int tt = tid + 512; tt < u_max; tt += 256) {               // more than 512 selected rows
        const int i = selh[tt];
        if (i >= r0 && i < r0 + rows_per_wg) s_sel[i - r0] = 1;
    }
    __syncthreads();

    float mean[EPL], zero[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) { mean[e] = s_mean[sub * EPL + e]; zero[e] = 0.f; }
    for (int rl = row; rl < rows_per_wg; rl += RPP) {
        const int i = r0 + rl;
        if (i >= L) break;
        if (i >= n) OT::store(out + ((size_t)head * L + i) * kD, sub, zero);
        else if (!s_sel[rl]) OT::store(out + ((size_t)head * L + i) * kD, sub, mean);
    }
}

hipError_t launch_finalize(const Plan& p, const Args& a, const Scratch& w)
{
    // more rows per fill work-group when there are many splits, so that re-reading
    // the per-split V sums stays small next to the rows written
    int rows = 8 * p.n_split;
    rows = rows < kFinalRows ? kFinalRows : (rows > kMaxFinalRows ? kMaxFinalRows : rows);
    rows = (rows + 63) & ~63;
    const int n_fill = (p.L + rows - 1) / rows;
    dim3 grid(n_fill + 1, p.BH), block(256);
    const int nq = p.nq_group;
    if (p.dtype == PSA_F32) {
        hipLaunchKernelGGL((finalize_kernel<float, double>), grid, block, 0, a.stream, a.lengths, w.sel, w.vpart,
                           (const double*)w.part, (float*)a.out, p.H, p.L, p.u_max, p.n_split, p.n_qgroup, nq,
                           (int)p.part_stride, rows, n_fill);
    } else {
        hipLaunchKernelGGL((finalize_kernel<bf16_t, float>), grid, block, 0, a.stream, a.lengths, w.sel, w.vpart,
                           (const float*)w.part, (bf16_t*)a.out, p.H, p.L, p.u_max, p.n_split, p.n_qgroup, nq,
                           (int)p.part_stride, rows, n_fill);
    }
    return hipGetLastError();
}

}  // namespace psa

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
__device__ __forceinline__ double rec_exp2(double x) { return exp2(x); }

// R is the element type of the partial records: double for float32 tensors
// (merged in float64, rounded once on the store), float for bfloat16 tensors.
template <typename T, typename R>
__global__ __launch_bounds__(256)
void finalize_kernel(const int* __restrict__ lengths, const int* __restrict__ sel,
                     const int* __restrict__ ucount, const float* __restrict__ mu,
                     const R* __restrict__ part, T* __restrict__ out,
                     int H, int L, int u_max, int n_split, int n_qgroup, int nq, int part_stride)
{
    using OT = OutTraits<T>;
    constexpr int LPR = OT::LPR, EPL = OT::EPL, RPP = 256 / LPR;
    __shared__ int s_rank[kFinalRows];

    const int head = blockIdx.y;
    const int r0 = blockIdx.x * kFinalRows;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int u = ucount[b];
    const int tid = threadIdx.x;

    if (tid < kFinalRows) s_rank[tid] = -1;
    __syncthreads();
    for (int t = tid; t < u; t += 256) {
        const int i = sel[(size_t)head * u_max + t];
        if (i >= r0 && i < r0 + kFinalRows) s_rank[i - r0] = t;
    }
    __syncthreads();

    const int sub = tid % LPR, row = tid / LPR;
    float mean[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) mean[e] = mu[(size_t)head * kD + sub * EPL + e];

#pragma unroll
    for (int p = 0; p < kFinalRows / RPP; ++p) {
        const int rl = row + p * RPP;
        const int i = r0 + rl;
        if (i >= L) continue;
        float val[EPL];
        const int rank = (i < n) ? s_rank[rl] : -1;
        if (i >= n) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) val[e] = 0.f;
        } else if (rank < 0) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) val[e] = mean[e];
        } else {
            const int qg = rank / nq, q = rank % nq;
            const R* base = part + ((size_t)head * n_qgroup + qg) * n_split * part_stride;
            R mx = -INFINITY;
            for (int s = 0; s < n_split; ++s) { const R ms = base[(size_t)s * part_stride + q]; mx = ms > mx ? ms : mx; }
            R lt = 0, acc[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = 0;
            for (int s = 0; s < n_split; ++s) {
                const R* rec = base + (size_t)s * part_stride;
                const R ms = rec[q];
                if (ms == -INFINITY) continue;                     // empty split
                const R sc = rec_exp2(ms - mx);
                lt += sc * rec[nq + q];
                const R* o = rec + 2 * nq + q * kD + sub * EPL;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] += sc * o[e];
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) val[e] = lt > 0 ? (float)(acc[e] / lt) : 0.f;
        }
        OT::store(out + ((size_t)head * L + i) * kD, sub, val);
    }
}

hipError_t launch_finalize(const Plan& p, const Args& a, const Scratch& w)
{
    dim3 grid((p.L + kFinalRows - 1) / kFinalRows, p.BH), block(256);
    const int nq = p.nq_group;
    if (p.dtype == PSA_F32) {
        hipLaunchKernelGGL((finalize_kernel<float, double>), grid, block, 0, a.stream, a.lengths, w.sel, w.u, w.mu,
                           (const double*)w.part, (float*)a.out, p.H, p.L, p.u_max, p.n_split, p.n_qgroup, nq, (int)p.part_stride);
    } else {
        hipLaunchKernelGGL((finalize_kernel<bf16_t, float>), grid, block, 0, a.stream, a.lengths, w.sel, w.u, w.mu,
                           (const float*)w.part, (bf16_t*)a.out, p.H, p.L, p.u_max, p.n_split, p.n_qgroup, nq, (int)p.part_stride);
    }
    return hipGetLastError();
}

}  // namespace psa

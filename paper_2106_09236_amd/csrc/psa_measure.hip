// Stage a1: scores of every query against its sampled keys and the sampled
// sparsity measure  M_i = max_t s_it - (1/#samples) sum_t s_it  (Sec. 3.2, Eq. 11),
// plus, as a by-product for stage a4, per-chunk column sums of the valid V rows.
//
// This is a gather, not a contraction: each query touches U random key rows of
// its own head.  A key row is 256 B (f32) or 128 B (bf16); a group of 16 (f32)
// or 8 (bf16) adjacent lanes reads one row with one 16-byte load per lane, so a
// wave fetches 4 or 8 whole rows per load instruction, each fully coalesced.
// The group's lanes hold the matching slice of the query in registers, the dot
// product is finished with DPP lane exchanges inside the group, and max / sum
// are carried per group.  One group owns one query at a time.
#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

template <typename T> struct RowTraits;
template <> struct RowTraits<float>  { static constexpr int LPR = 16; };   // lanes per key row
template <> struct RowTraits<bf16_t> { static constexpr int LPR = 8; };

// ---- slice of a row held by one lane: 16 bytes
template <typename T> struct Slice;
template <> struct Slice<float> {
    float4 v;
    __device__ __forceinline__ void load(const float* row, int sub) { v = reinterpret_cast<const float4*>(row)[sub]; }
    __device__ __forceinline__ void zero() { v = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ float dot(const Slice<float>& k) const {
        float d = v.x * k.v.x;
        d = fmaf(v.y, k.v.y, d);
        d = fmaf(v.z, k.v.z, d);
        d = fmaf(v.w, k.v.w, d);
        return d;
    }
};
template <> struct Slice<bf16_t> {
    uint4 v;   // 8 bf16
    __device__ __forceinline__ void load(const bf16_t* row, int sub) { v = reinterpret_cast<const uint4*>(row)[sub]; }
    __device__ __forceinline__ void zero() { v = make_uint4(0u, 0u, 0u, 0u); }
    __device__ __forceinline__ float dot(const Slice<bf16_t>& k) const {
        // products of two bf16 are exact in f32; v_dot2_f32_bf16 accumulates in f32
        float d = 0.f;
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.x), __builtin_bit_cast(bf16x2, k.v.x), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.y), __builtin_bit_cast(bf16x2, k.v.y), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.z), __builtin_bit_cast(bf16x2, k.v.z), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.w), __builtin_bit_cast(bf16x2, k.v.w), d, false);
        return d;
    }
};

template <int LPR> __device__ __forceinline__ float group_sum(float x);
template <> __device__ __forceinline__ float group_sum<16>(float x) { return group_sum16(x); }
template <> __device__ __forceinline__ float group_sum<8>(float x) { return group_sum8(x); }

// ---- accumulate the 16-byte slice of a V row into doubles
__device__ __forceinline__ void add_slice(double* acc, const Slice<float>& s) {
    acc[0] += (double)s.v.x; acc[1] += (double)s.v.y; acc[2] += (double)s.v.z; acc[3] += (double)s.v.w;
}
__device__ __forceinline__ void add_slice(double* acc, const Slice<bf16_t>& s) {
    acc[0] += (double)bf16_lo(s.v.x); acc[1] += (double)bf16_hi(s.v.x);
    acc[2] += (double)bf16_lo(s.v.y); acc[3] += (double)bf16_hi(s.v.y);
    acc[4] += (double)bf16_lo(s.v.z); acc[5] += (double)bf16_hi(s.v.z);
    acc[6] += (double)bf16_lo(s.v.w); acc[7] += (double)bf16_hi(s.v.w);
}

template <typename T>
__global__ __launch_bounds__(256)
void measure_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                    const int* __restrict__ lengths, const int* __restrict__ idx,
                    float* __restrict__ M, double* __restrict__ vpart,
                    int H, int L, int U, int n_chunk)
{
    constexpr int LPR = RowTraits<T>::LPR;        // lanes per row
    constexpr int EPL = kD / LPR;                 // elements per lane
    constexpr int G = 64 / LPR;                   // query groups per wave
    constexpr int RPP = 256 / LPR;                // V rows per pass of the whole work-group
    constexpr int QPW = kMeasureRows / 4;         // queries per wave

    const int head = blockIdx.y;
    const int chunk = blockIdx.x;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int i0 = chunk * kMeasureRows;
    const int tid = threadIdx.x;

    const T* Qh = Q + (size_t)head * L * kD;
    const T* Kh = K + (size_t)head * L * kD;
    const T* Vh = V + (size_t)head * L * kD;

    // ------------------------------------------------------------------ V sums
    // Column sums of the valid V rows of this chunk, in float64 so that the mean
    // of a4 carries no visible rounding (Sec. 3.1: the fill is the plain average).
    __shared__ double red[RPP][kD];
    {
        const int sub = tid % LPR, r = tid / LPR;
        double acc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = 0.0;
#pragma unroll
        for (int p = 0; p < kMeasureRows / RPP; ++p) {
            const int j = i0 + r + p * RPP;
            if (j < n) {
                Slice<T> s;
                s.load(Vh + (size_t)j * kD, sub);
                add_slice(acc, s);
            }
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) red[r][sub * EPL + e] = acc[e];
        __syncthreads();
        if (tid < kD) {
            double s = 0.0;
            for (int rr = 0; rr < RPP; ++rr) s += red[rr][tid];     // fixed order
            vpart[((size_t)head * n_chunk + chunk) * kD + tid] = s;
        }
    }

    // ------------------------------------------------------------------ measure
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane / LPR, sub = lane % LPR;
    const int gbase = lane - sub;                  // first lane of this group

    for (int pass = 0; pass < QPW / G; ++pass) {
        const int i = i0 + wave * QPW + pass * G + g;
        const bool in_tensor = i < L;
        const bool active = i < n;
        Slice<T> q;
        if (active) q.load(Qh + (size_t)i * kD, sub); else q.zero();
        const int* irow = idx + ((size_t)head * L + (in_tensor ? i : 0)) * U;

        float mx = -INFINITY, sm = 0.f;
        int cnt = 0;
        for (int tb = 0; tb < U; tb += LPR) {
            // each lane of the group fetches one sample index of this block
            const int t_mine = tb + sub;
            const int jv = (active && t_mine < U) ? irow[t_mine] : -1;
            const int nt = (U - tb) < LPR ? (U - tb) : LPR;      // wave-uniform
            if (nt == LPR) {
                Slice<T> kr[LPR];
                bool ok[LPR];
#pragma unroll
                for (int tt = 0; tt < LPR; ++tt) {
                    const int j = __shfl(jv, gbase + tt, 64);
                    ok[tt] = (unsigned)j < (unsigned)n;
                    kr[tt].load(Kh + (size_t)(ok[tt] ? j : 0) * kD, sub);
                }
#pragma unroll
                for (int tt = 0; tt < LPR; ++tt) {
                    const float s = group_sum<LPR>(q.dot(kr[tt])) * 0.125f;   // 1/sqrt(64)
                    mx = ok[tt] ? fmaxf(mx, s) : mx;
                    sm += ok[tt] ? s : 0.f;
                    cnt += ok[tt] ? 1 : 0;
                }
            } else {
                for (int tt = 0; tt < nt; ++tt) {
                    const int j = __shfl(jv, gbase + tt, 64);
                    const bool ok = (unsigned)j < (unsigned)n;
                    Slice<T> kr;
                    kr.load(Kh + (size_t)(ok ? j : 0) * kD, sub);
                    const float s = group_sum<LPR>(q.dot(kr)) * 0.125f;
                    mx = ok ? fmaxf(mx, s) : mx;
                    sm += ok ? s : 0.f;
                    cnt += ok ? 1 : 0;
                }
            }
        }
        if (in_tensor && sub == 0) {
            float m = 0.f;
            if (active && cnt > 0) m = mx - sm / (float)cnt;
            M[(size_t)head * L + i] = m;
        }
    }
}

hipError_t launch_measure(const Plan& p, const Args& a, const Scratch& w)
{
    dim3 grid(p.n_chunk, p.BH), block(256);
    if (p.dtype == PSA_F32) {
        hipLaunchKernelGGL(measure_kernel<float>, grid, block, 0, a.stream,
                           (const float*)a.Q, (const float*)a.K, (const float*)a.V, a.lengths, a.idx,
                           w.M, w.vpart, p.H, p.L, p.U, p.n_chunk);
    } else {
        hipLaunchKernelGGL(measure_kernel<bf16_t>, grid, block, 0, a.stream,
                           (const bf16_t*)a.Q, (const bf16_t*)a.K, (const bf16_t*)a.V, a.lengths, a.idx,
                           w.M, w.vpart, p.H, p.L, p.U, p.n_chunk);
    }
    return hipGetLastError();
}

}  // namespace psa

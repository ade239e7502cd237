// Gradients of stages a3 and a4 for a fixed index set I_sparse (Eq. 7, Eq. 8, Eq. 12;
// retraining a prob-sparse model from a trained dense one, Sec. 4.2).  The selection is
// a hard choice, so nothing flows through stages a1 and a2.  Per head, with G the
// upstream gradient of `out`, p_ij the softmax weights of the kept queries and
// scale = 1/sqrt(d):
//   c_ij = G_i . v_j           D_i = sum_j p_ij c_ij          g_ij = scale * p_ij (c_ij - D_i)
//   dQ_i = sum_j g_ij k_j      dK_j = sum_i g_ij q_i          dV_j = sum_i p_ij G_i   (+ the fill's share)
// The weights are recomputed from Q and K (the forward keeps no statistics):
//   bwd_stats_kernel   partial (max, sum, weighted sum of c) per kept query and key split
//   bwd_dq_kernel      combines them into ln sum exp and D, then dQ (per key split)
//   bwd_dkv_kernel     key-stationary: dK, dV, the fill's gradient, zero rows
//   bwd_dq_reduce_kernel  adds the key splits of dQ in split order
// Both tensor types are computed in float64: where attention is sharply peaked (the queries
// the selection prefers) p_ij is almost 1 for one key and c_ij - D_i is a difference of nearly
// equal numbers, of which float32 arithmetic leaves only noise (measured on bfloat16 tensors:
// errors of 4 times the gradient's own size).  Every sum has a fixed order, so results do not
// depend on scheduling.
#include <type_traits>

#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

constexpr int kBwdThreads = 256;
constexpr int kBwdKeys = 64;         // keys per block
constexpr int kBwdQ = 16;            // kept queries per tile

template <typename C> struct BwdLds {
    static constexpr int KS = kD + (sizeof(C) == 8 ? 2 : 4);      // padded row of the K / V blocks (16-byte multiples)
    C Ks[kBwdKeys][KS];
    C Vs[kBwdKeys][KS];
    C Qs[kBwdQ][kD];
    C Gs[kBwdQ][kD];
    C P[kBwdQ][kBwdKeys];
    C Gd[kBwdQ][kBwdKeys];
    C lse[kBwdQ], D[kBwdQ];
    int qi[kBwdQ];
    unsigned char flag[kBwdKeys];
};

template <typename T> __device__ __forceinline__ float load_elem(const T* p);
template <> __device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_elem<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->x); }
template <typename T> __device__ __forceinline__ void store_elem(T* p, float v);
template <> __device__ __forceinline__ void store_elem<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_elem<bf16_t>(bf16_t* p, float v) { p->x = f32_to_bf16(v); }

__device__ __forceinline__ float  bexp(float x)  { return __expf(x); }
__device__ __forceinline__ double bexp(double x) { return exp(x); }
__device__ __forceinline__ float  blog(float x)  { return __logf(x); }
__device__ __forceinline__ double blog(double x) { return log(x); }

struct BwdParams {
    const void* Q; const void* K; const void* V; const void* G;
    const int* lengths; const int* sel; const int* u;
    void* dQ; void* dK; void* dV;
    void* stats_part;      // [BH][QT][S][16][3]  (max, sum, weighted c) per kept query and key split
    void* stats;           // [BH][QT * 16][2]    ln sum exp, D
    void* gsum_part;       // [BH][S][64]         column sums of G over the valid rows outside I_sparse, per key split
    void* dq_part;         // [BH][QT][S][16][64] (S > 1)
    int H, L, u_stride, QT, S, blocks_per_split, fill;
};

// rows [r0, r0 + rows) of a [L, 64] tensor of one head into an LDS block as C; rows at or beyond n as zeros
template <typename T, typename C, int STRIDE>
__device__ __forceinline__ void stage_rows(C (*dst)[STRIDE], const T* head, int r0, int rows, int n)
{
    for (int t = threadIdx.x; t < rows * kD; t += kBwdThreads) {
        const int r = t >> 6, e = t & 63;
        const int j = r0 + r;
        dst[r][e] = j < n ? (C)load_elem(head + (size_t)j * kD + e) : (C)0;
    }
}
// the rows of the kept queries qi[0 .. 16) (-1: none) into an LDS tile
template <typename T, typename C>
__device__ __forceinline__ void stage_kept(C (*dst)[kD], const T* head, const int* qi)
{
    for (int t = threadIdx.x; t < kBwdQ * kD; t += kBwdThreads) {
        const int r = t >> 6, e = t & 63;
        const int i = qi[r];
        dst[r][e] = i >= 0 ? (C)load_elem(head + (size_t)i * kD + e) : (C)0;
    }
}
// kept queries of tile qt of the head: entries beyond u_b or outside [0, n) count as absent
__device__ __forceinline__ void stage_tile_indices(int* qi, const BwdParams& P, int head, int qt, int n, int ub)
{
    if (threadIdx.x < kBwdQ) {
        const int t = qt * kBwdQ + threadIdx.x;
        int i = -1;
        if (t < ub) { i = P.sel[(size_t)head * P.u_stride + t]; if (i < 0 || i >= n) i = -1; }
        qi[threadIdx.x] = i;
    }
}
__device__ __forceinline__ int kept_count(const BwdParams& P, int b, int n)
{
    int ub = P.u[b];
    ub = ub < 0 ? 0 : (ub > P.u_stride ? P.u_stride : ub);
    return ub > n ? n : ub;
}

// scores and the gradient's first contraction for key jj of the staged block against 4 kept queries
template <typename C, typename L>
__device__ __forceinline__ void scores4(const L& lds, int jj, int q0, C (&s)[4], C (&c)[4])
{
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) { s[ii] = 0; c[ii] = 0; }
#pragma unroll 8
    for (int e = 0; e < kD; ++e) {
        const C k = lds.Ks[jj][e], v = lds.Vs[jj][e];
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) { s[ii] += lds.Qs[q0 + ii][e] * k; c[ii] += lds.Gs[q0 + ii][e] * v; }
    }
}

// ---- partial softmax statistics per kept query and key split; column sums of G over the rows the fill serves
template <typename T, typename C>
__global__ __launch_bounds__(kBwdThreads)
void bwd_stats_kernel(const BwdParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char s_bwd[];
    auto& lds = *reinterpret_cast<BwdLds<C>*>(s_bwd);
    const int split = blockIdx.x, qt = blockIdx.y, head = blockIdx.z;
    const int b = head / P.H, L = P.L;
    const int n = valid_len(P.lengths, b, L);
    const int ub = kept_count(P, b, n);
    const int tid = threadIdx.x, jj = tid & 63, wave = tid >> 6, q0 = 4 * wave;
    const T* Qh = static_cast<const T*>(P.Q) + (size_t)head * L * kD;
    const T* Kh = static_cast<const T*>(P.K) + (size_t)head * L * kD;
    const T* Vh = static_cast<const T*>(P.V) + (size_t)head * L * kD;
    const T* Gh = static_cast<const T*>(P.G) + (size_t)head * L * kD;
    const int k_first = split * P.blocks_per_split * kBwdKeys;
    int k_end = k_first + P.blocks_per_split * kBwdKeys;
    k_end = k_end < n ? k_end : n;

    // the fill's rows: valid rows of this key range that are not kept (query tile 0 only)
    if (qt == 0) {
        C* gs = static_cast<C*>(P.gsum_part) + ((size_t)head * P.S + split) * kD;
        C tot = 0;                                                   // column tid & 63, rows wave, wave + 4, ...
        for (int r0 = k_first; r0 < k_end; r0 += kBwdKeys) {
            if (tid < kBwdKeys) lds.flag[tid] = 0;
            __syncthreads();
            for (int t = tid; t < ub; t += kBwdThreads) {
                const int i = P.sel[(size_t)head * P.u_stride + t];
                if (i >= r0 && i < r0 + kBwdKeys) lds.flag[i - r0] = 1;
            }
            __syncthreads();
            for (int r = wave; r < kBwdKeys; r += 4) {
                const int j = r0 + r;
                if (j < k_end && !lds.flag[r]) tot += (C)load_elem(Gh + (size_t)j * kD + jj);
            }
            __syncthreads();
        }
        lds.P[wave][jj] = tot;
        __syncthreads();
        if (tid < kD) gs[tid] = ((lds.P[0][tid] + lds.P[1][tid]) + lds.P[2][tid]) + lds.P[3][tid];
        __syncthreads();
    }
    if (qt * kBwdQ >= ub) return;                                    // no kept query in this tile (work-group-uniform)

    stage_tile_indices(lds.qi, P, head, qt, n, ub);
    __syncthreads();
    stage_kept<T, C>(lds.Qs, Qh, lds.qi);
    stage_kept<T, C>(lds.Gs, Gh, lds.qi);
    C m[4], l[4], dacc[4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) { m[ii] = -INFINITY; l[ii] = 0; dacc[ii] = 0; }
    for (int r0 = k_first; r0 < k_end; r0 += kBwdKeys) {
        __syncthreads();
        stage_rows<T, C>(lds.Ks, Kh, r0, kBwdKeys, n);
        stage_rows<T, C>(lds.Vs, Vh, r0, kBwdKeys, n);
        __syncthreads();
        if (r0 + jj < n) {
            C s[4], c[4];
            scores4<C>(lds, jj, q0, s, c);
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const C sc = s[ii] * (C)0.125;
                const C mn = sc > m[ii] ? sc : m[ii];
                const C a = bexp(m[ii] - mn), w = bexp(sc - mn);       // (exp(-inf) = 0 on the first key)
                l[ii] = l[ii] * a + w;
                dacc[ii] = dacc[ii] * a + w * c[ii];
                m[ii] = mn;
            }
        }
    }
    // the 64 lanes of a wave hold the same 4 queries: fold them, lane order fixed by the xor tree
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
        C mw = m[ii];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { const C o = __shfl_xor(mw, off, 64); mw = o > mw ? o : mw; }
        const C a = mw == (C)-INFINITY ? (C)0 : bexp(m[ii] - mw);
        C lw = l[ii] * a, dw = dacc[ii] * a;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { lw += __shfl_xor(lw, off, 64); dw += __shfl_xor(dw, off, 64); }
        if (jj == 0) {
            C* sp = static_cast<C*>(P.stats_part) + ((((size_t)head * P.QT + qt) * P.S + split) * kBwdQ + q0 + ii) * 3;
            sp[0] = mw; sp[1] = lw; sp[2] = dw;
        }
    }
}

// combine the key splits' statistics of the tile's 16 kept queries: ln sum exp and D into lds (all threads call)
template <typename C, typename L>
__device__ __forceinline__ void combine_stats(L& lds, const BwdParams& P, int head, int qt)
{
    if (threadIdx.x < kBwdQ) {
        const C* sp = static_cast<const C*>(P.stats_part) + (((size_t)head * P.QT + qt) * P.S * kBwdQ + threadIdx.x) * 3;
        C mx = -INFINITY;
        for (int s = 0; s < P.S; ++s) { const C v = sp[(size_t)s * kBwdQ * 3]; mx = v > mx ? v : mx; }
        C lt = 0, dt = 0;
        for (int s = 0; s < P.S; ++s) {
            const C ms = sp[(size_t)s * kBwdQ * 3];
            const C a = ms == (C)-INFINITY ? (C)0 : bexp(ms - mx);
            lt += a * sp[(size_t)s * kBwdQ * 3 + 1];
            dt += a * sp[(size_t)s * kBwdQ * 3 + 2];
        }
        lds.lse[threadIdx.x] = lt > 0 ? mx + blog(lt) : (C)0;
        lds.D[threadIdx.x] = lt > 0 ? dt / lt : (C)0;
    }
}

// weights and score gradients of the staged key block against the staged tile: P[i][jj], Gd[i][jj]
template <typename C, typename L>
__device__ __forceinline__ void weights_tile(L& lds, int r0, int n)
{
    const int jj = threadIdx.x & 63, q0 = 4 * (threadIdx.x >> 6);
    C s[4], c[4];
    scores4<C>(lds, jj, q0, s, c);
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
        const bool ok = r0 + jj < n && lds.qi[q0 + ii] >= 0;
        const C p = ok ? bexp(s[ii] * (C)0.125 - lds.lse[q0 + ii]) : (C)0;
        lds.P[q0 + ii][jj] = p;
        lds.Gd[q0 + ii][jj] = (C)0.125 * p * (c[ii] - lds.D[q0 + ii]);
    }
}

template <typename T, typename C>
__global__ __launch_bounds__(kBwdThreads)
void bwd_dq_kernel(const BwdParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char s_bwd[];
    auto& lds = *reinterpret_cast<BwdLds<C>*>(s_bwd);
    const int split = blockIdx.x, qt = blockIdx.y, head = blockIdx.z;
    const int b = head / P.H, L = P.L;
    const int n = valid_len(P.lengths, b, L);
    const int ub = kept_count(P, b, n);
    if (qt * kBwdQ >= ub) return;                                    // work-group-uniform
    const int tid = threadIdx.x;
    const T* Qh = static_cast<const T*>(P.Q) + (size_t)head * L * kD;
    const T* Kh = static_cast<const T*>(P.K) + (size_t)head * L * kD;
    const T* Vh = static_cast<const T*>(P.V) + (size_t)head * L * kD;
    const T* Gh = static_cast<const T*>(P.G) + (size_t)head * L * kD;
    const int k_first = split * P.blocks_per_split * kBwdKeys;
    int k_end = k_first + P.blocks_per_split * kBwdKeys;
    k_end = k_end < n ? k_end : n;

    stage_tile_indices(lds.qi, P, head, qt, n, ub);
    combine_stats<C>(lds, P, head, qt);
    __syncthreads();
    if (split == 0 && tid < kBwdQ) {                                 // for the key-stationary kernel
        C* st = static_cast<C*>(P.stats) + ((size_t)head * P.QT * kBwdQ + qt * kBwdQ + tid) * 2;
        st[0] = lds.lse[tid]; st[1] = lds.D[tid];
    }
    stage_kept<T, C>(lds.Qs, Qh, lds.qi);
    stage_kept<T, C>(lds.Gs, Gh, lds.qi);
    const int i = tid >> 4, e0 = 4 * (tid & 15);                     // this thread's share of dQ: query i, elements e0 .. e0+3
    C acc[4] = {0, 0, 0, 0};
    for (int r0 = k_first; r0 < k_end; r0 += kBwdKeys) {
        __syncthreads();
        stage_rows<T, C>(lds.Ks, Kh, r0, kBwdKeys, n);
        stage_rows<T, C>(lds.Vs, Vh, r0, kBwdKeys, n);
        __syncthreads();
        weights_tile<C>(lds, r0, n);
        __syncthreads();
#pragma unroll 4
        for (int jj = 0; jj < kBwdKeys; ++jj) {                      // keys in order
            const C g = lds.Gd[i][jj];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += g * lds.Ks[jj][e0 + e];
        }
    }
    const int qi = lds.qi[i];
    if (P.S == 1) {
        if (qi >= 0) {
            T* row = static_cast<T*>(P.dQ) + ((size_t)head * L + qi) * kD + e0;
#pragma unroll
            for (int e = 0; e < 4; ++e) store_elem(row + e, (float)acc[e]);
        }
    } else {
        C* dp = static_cast<C*>(P.dq_part) + ((((size_t)head * P.QT + qt) * P.S + split) * kBwdQ + i) * kD + e0;
#pragma unroll
        for (int e = 0; e < 4; ++e) dp[e] = acc[e];
    }
}

template <typename T, typename C>
__global__ __launch_bounds__(kBwdThreads)
void bwd_dq_reduce_kernel(const BwdParams P)
{
    const int qt = blockIdx.x, head = blockIdx.y;
    const int b = head / P.H;
    const int n = valid_len(P.lengths, b, P.L);
    const int ub = kept_count(P, b, n);
    if (qt * kBwdQ >= ub) return;
    const int tid = threadIdx.x, i = tid >> 4, e0 = 4 * (tid & 15);
    const int t = qt * kBwdQ + i;
    int qi = -1;
    if (t < ub) { qi = P.sel[(size_t)head * P.u_stride + t]; if (qi < 0 || qi >= n) qi = -1; }
    if (qi < 0) return;
    const C* dp = static_cast<const C*>(P.dq_part) + (((size_t)head * P.QT + qt) * P.S * kBwdQ + i) * kD + e0;
    C acc[4] = {0, 0, 0, 0};
    for (int s = 0; s < P.S; ++s)                                    // split order
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += dp[(size_t)s * kBwdQ * kD + e];
    T* row = static_cast<T*>(P.dQ) + ((size_t)head * P.L + qi) * kD + e0;
#pragma unroll
    for (int e = 0; e < 4; ++e) store_elem(row + e, (float)acc[e]);
}

// ---- key-stationary: one work-group per block of 64 keys walks all kept queries of the head
template <typename T, typename C>
__global__ __launch_bounds__(kBwdThreads)
void bwd_dkv_kernel(const BwdParams P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char s_bwd[];
    auto& lds = *reinterpret_cast<BwdLds<C>*>(s_bwd);
    const int blk = blockIdx.x, head = blockIdx.y;
    const int b = head / P.H, L = P.L;
    const int n = valid_len(P.lengths, b, L);
    const int ub = kept_count(P, b, n);
    const int tid = threadIdx.x;
    const int r0 = blk * kBwdKeys;
    const T* Qh = static_cast<const T*>(P.Q) + (size_t)head * L * kD;
    const T* Kh = static_cast<const T*>(P.K) + (size_t)head * L * kD;
    const T* Vh = static_cast<const T*>(P.V) + (size_t)head * L * kD;
    const T* Gh = static_cast<const T*>(P.G) + (size_t)head * L * kD;
    const int jj = tid >> 2, e0 = 16 * (tid & 3);                    // this thread's share of dK, dV: key jj, elements e0 .. e0+15
    const int j = r0 + jj;

    // which rows of this block are kept queries
    if (tid < kBwdKeys) lds.flag[tid] = 0;
    __syncthreads();
    for (int t = tid; t < ub; t += kBwdThreads) {
        const int i = P.sel[(size_t)head * P.u_stride + t];
        if (i >= r0 && i < r0 + kBwdKeys && i < n) lds.flag[i - r0] = 1;
    }
    stage_rows<T, C>(lds.Ks, Kh, r0, kBwdKeys, n);
    stage_rows<T, C>(lds.Vs, Vh, r0, kBwdKeys, n);
    C dk[16], dv[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[e] = 0; dv[e] = 0; }
    if (r0 < n) {
        const int n_qt = (ub + kBwdQ - 1) / kBwdQ;
        for (int qt = 0; qt < n_qt; ++qt) {                          // query tiles in order
            __syncthreads();
            stage_tile_indices(lds.qi, P, head, qt, n, ub);
            if (tid < kBwdQ) {
                const C* st = static_cast<const C*>(P.stats) + ((size_t)head * P.QT * kBwdQ + qt * kBwdQ + tid) * 2;
                lds.lse[tid] = st[0]; lds.D[tid] = st[1];
            }
            __syncthreads();
            stage_kept<T, C>(lds.Qs, Qh, lds.qi);
            stage_kept<T, C>(lds.Gs, Gh, lds.qi);
            __syncthreads();
            weights_tile<C>(lds, r0, n);
            __syncthreads();
#pragma unroll 2
            for (int i = 0; i < kBwdQ; ++i) {
                const C p = lds.P[i][jj], g = lds.Gd[i][jj];
#pragma unroll
                for (int e = 0; e < 16; ++e) { dv[e] += p * lds.Gs[i][e0 + e]; dk[e] += g * lds.Qs[i][e0 + e]; }
            }
        }
    }
    __syncthreads();
    // the fill's share of dV: the mean hands every valid v_j 1/n of each filled row's gradient; the
    // value fill hands v_j the gradient of its own row
    if (P.fill == PSA_FILL_MEAN) {
        if (tid < kD) {
            const C* gs = static_cast<const C*>(P.gsum_part) + (size_t)head * P.S * kD + tid;
            C t = 0;
            for (int s = 0; s < P.S; ++s) t += gs[(size_t)s * kD];     // split order
            lds.Qs[0][tid] = n > 0 ? t / (C)n : (C)0;
        }
        __syncthreads();
    }
    if (j < L) {
        T* dkr = static_cast<T*>(P.dK) + ((size_t)head * L + j) * kD + e0;
        T* dvr = static_cast<T*>(P.dV) + ((size_t)head * L + j) * kD + e0;
        T* dqr = static_cast<T*>(P.dQ) + ((size_t)head * L + j) * kD + e0;
        const bool valid = j < n, kept = valid && lds.flag[jj];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            C v = dv[e];
            if (P.fill == PSA_FILL_MEAN) v += lds.Qs[0][e0 + e];
            else if (valid && !kept) v += (C)load_elem(Gh + (size_t)j * kD + e0 + e);
            store_elem(dkr + e, valid ? (float)dk[e] : 0.f);
            store_elem(dvr + e, valid ? (float)v : 0.f);
            if (!kept) store_elem(dqr + e, 0.f);                     // no gradient reaches a query outside I_sparse
        }
    }
}

template <typename T, typename C>
static hipError_t launch_bwd_t(const BwdParams& P, int BH, hipStream_t stream)
{
    static std::atomic<uint64_t> raised[3];
    const int lds = (int)sizeof(BwdLds<C>);
    hipError_t e = ensure_lds_limit((const void*)bwd_stats_kernel<T, C>, lds, raised[0]);
    if (e == hipSuccess) e = ensure_lds_limit((const void*)bwd_dq_kernel<T, C>, lds, raised[1]);
    if (e == hipSuccess) e = ensure_lds_limit((const void*)bwd_dkv_kernel<T, C>, lds, raised[2]);
    if (e != hipSuccess) return e;
    const dim3 qgrid(P.S, P.QT, BH);
    hipLaunchKernelGGL((bwd_stats_kernel<T, C>), qgrid, dim3(kBwdThreads), lds, stream, P);
    hipLaunchKernelGGL((bwd_dq_kernel<T, C>), qgrid, dim3(kBwdThreads), lds, stream, P);
    hipLaunchKernelGGL((bwd_dkv_kernel<T, C>), dim3((P.L + kBwdKeys - 1) / kBwdKeys, BH), dim3(kBwdThreads), lds, stream, P);
    if (P.S > 1) hipLaunchKernelGGL((bwd_dq_reduce_kernel<T, C>), dim3(P.QT, BH), dim3(kBwdThreads), 0, stream, P);
    return hipGetLastError();
}

// Plan of the backward: query tiles, key splits and the carving of its workspace (host arithmetic).
BwdPlan make_bwd_plan(const psa_shape_t& s, int u_stride)
{
    BwdPlan p;
    const int BH = s.B * s.H;
    const size_t ce = sizeof(double);                           // the arithmetic type of every intermediate
    p.QT = (u_stride + kBwdQ - 1) / kBwdQ;
    const int n_blocks = (s.L_K + kBwdKeys - 1) / kBwdKeys;
    int S = (int)((512 + (int64_t)BH * p.QT - 1) / ((int64_t)BH * p.QT));
    S = S < 1 ? 1 : (S > 64 ? 64 : S);
    S = S > n_blocks ? n_blocks : S;
    p.blocks_per_split = (n_blocks + S - 1) / S;
    p.S = (n_blocks + p.blocks_per_split - 1) / p.blocks_per_split;
    auto al = [](size_t x) { return (x + 255) & ~(size_t)255; };
    size_t off = 0;
    p.off_stats_part = off; off += al((size_t)BH * p.QT * p.S * kBwdQ * 3 * ce);
    p.off_stats = off;      off += al((size_t)BH * p.QT * kBwdQ * 2 * ce);
    p.off_gsum = off;       off += al((size_t)BH * p.S * kD * ce);
    p.off_dq_part = off;    off += p.S > 1 ? al((size_t)BH * p.QT * p.S * kBwdQ * kD * ce) : 0;
    p.total = off;
    return p;
}

hipError_t launch_backward(const psa_shape_t& s, const BwdPlan& bp, const void* Q, const void* K, const void* V,
                           const int* lengths, const int* sel, const int* u, int u_stride, int fill, const void* G,
                           void* dQ, void* dK, void* dV, void* workspace, hipStream_t stream)
{
    unsigned char* w = static_cast<unsigned char*>(workspace);
    BwdParams P;
    P.Q = Q; P.K = K; P.V = V; P.G = G; P.lengths = lengths; P.sel = sel; P.u = u;
    P.dQ = dQ; P.dK = dK; P.dV = dV;
    P.stats_part = w + bp.off_stats_part; P.stats = w + bp.off_stats; P.gsum_part = w + bp.off_gsum;
    P.dq_part = w + bp.off_dq_part;
    P.H = s.H; P.L = s.L_K; P.u_stride = u_stride; P.QT = bp.QT; P.S = bp.S; P.blocks_per_split = bp.blocks_per_split;
    P.fill = fill;
    const int BH = s.B * s.H;
    return s.dtype == PSA_F32 ? launch_bwd_t<float, double>(P, BH, stream) : launch_bwd_t<bf16_t, double>(P, BH, stream);
}

}  // namespace psa

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
// All five contractions run on the matrix cores (v_mfma_f64_16x16x4f64 on exactly widened inputs):
//   lane (c, g) = (lane % 16, lane / 16)
//   A[i][k]: i = c, k = g      B[k][j]: k = g, j = c      D[i][j]: i = 4r + g, j = c  (r = 0..3)
// A wave takes 16 keys against a tile of 16 kept queries.  The query-stationary kernels compute the scores
// transposed (keys on the rows), so that a lane's four values belong to ONE query (its statistics are
// per-lane scalars) and are, unchanged, the B operand of the product that contracts over keys (dQ).  The
// key-stationary kernel computes them upright (queries on the rows), so that the same holds for the
// products that contract over queries (dK, dV).  Operands come straight from global memory: for the score
// products a lane reads 16 contiguous elements of its row (step t of lane group g stands for element
// 16 g + t in both operands: the contraction order is free), for the others 4 contiguous elements 4c ..
// 4c + 3, component dt feeding accumulator dt, whose row m then stands for element 4 m + dt.
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
constexpr int kBwdKeys = 64;         // keys per block: 16 per wave
constexpr int kBwdQ = 16;            // kept queries per tile
constexpr int kBwdWaves = kBwdThreads / 64;
constexpr int kBwdStaged = 64;        // kept queries staged in LDS at a time by the key-stationary kernel
constexpr int kBwdStage = kD + 4;     // floats between their rows
constexpr int kBwdChunk = 2048;      // rows per pass of the fill's column sums
typedef double bwd_x4 __attribute__((ext_vector_type(4)));

template <typename T> __device__ __forceinline__ float load_elem(const T* p);
template <> __device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_elem<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->x); }

// 16 or 4 contiguous elements as float, and a 4-element store
template <typename T> struct BwdMem;
template <> struct BwdMem<float> {
    static __device__ __forceinline__ void row16(const float* p, float (&v)[16]) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float4 x = reinterpret_cast<const float4*>(p)[k];
            v[4 * k] = x.x; v[4 * k + 1] = x.y; v[4 * k + 2] = x.z; v[4 * k + 3] = x.w;
        }
    }
    static __device__ __forceinline__ void row4(const float* p, float (&v)[4]) {
        const float4 x = *reinterpret_cast<const float4*>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
    static __device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct BwdMem<bf16_t> {
    static __device__ __forceinline__ void row16(const bf16_t* p, float (&v)[16]) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint4 x = reinterpret_cast<const uint4*>(p)[k];
            v[8 * k] = bf16_lo(x.x); v[8 * k + 1] = bf16_hi(x.x); v[8 * k + 2] = bf16_lo(x.y); v[8 * k + 3] = bf16_hi(x.y);
            v[8 * k + 4] = bf16_lo(x.z); v[8 * k + 5] = bf16_hi(x.z); v[8 * k + 6] = bf16_lo(x.w); v[8 * k + 7] = bf16_hi(x.w);
        }
    }
    static __device__ __forceinline__ void row4(const bf16_t* p, float (&v)[4]) {
        const uint2 x = *reinterpret_cast<const uint2*>(p);
        v[0] = bf16_lo(x.x); v[1] = bf16_hi(x.x); v[2] = bf16_lo(x.y); v[3] = bf16_hi(x.y);
    }
    static __device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
        *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
    }
};

// e^x in float64 (2^(x log2 e) by the degree-7 series of the forward: 5e-9 relative); e^(-inf) = 0
__device__ __forceinline__ double bwd_exp(double x) { return exp2_f64(x * 1.4426950408889634074); }

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

__device__ __forceinline__ int kept_count(const BwdParams& P, int b, int n)
{
    int ub = P.u[b];
    ub = ub < 0 ? 0 : (ub > P.u_stride ? P.u_stride : ub);
    return ub > n ? n : ub;
}
// kept query `t` of the head (an index into its list): its row, or -1 when the entry lies beyond u_b or outside [0, n)
__device__ __forceinline__ int kept_row(const BwdParams& P, int head, int t, int n, int ub)
{
    if (t >= ub) return -1;
    const int i = P.sel[(size_t)head * P.u_stride + t];
    return (i < 0 || i >= n) ? -1 : i;
}

// the two score products of 16 rows `a` against 16 rows `b` (16 contiguous elements per lane each):
// s = sum_e a1[e] b1[e], c = sum_e a2[e] b2[e], two independent MFMA chains
__device__ __forceinline__ void score_products(const float (&a1)[16], const double (&b1)[16], const float (&a2)[16],
                                               const double (&b2)[16], bwd_x4& s, bwd_x4& c)
{
    s = bwd_x4{0.0, 0.0, 0.0, 0.0};
    c = bwd_x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        s = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a1[t], b1[t], s, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a2[t], b2[t], c, 0, 0, 0);
    }
}

// ---- partial softmax statistics per kept query and key split; column sums of G over the rows the fill serves
template <typename T>
__global__ __launch_bounds__(kBwdThreads)
void bwd_stats_kernel(const BwdParams P)
{
    using M = BwdMem<T>;
    __shared__ double s_part[kBwdWaves][kBwdQ][3];
    __shared__ double s_gs[4 * kBwdWaves][kD];
    __shared__ unsigned s_bits[kBwdChunk / 32];
    const int split = blockIdx.x, qt = blockIdx.y, head = blockIdx.z;
    const int b = head / P.H, L = P.L;
    const int n = valid_len(P.lengths, b, L);
    const int ub = kept_count(P, b, n);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15, g = lane >> 4;
    const T* Qh = static_cast<const T*>(P.Q) + (size_t)head * L * kD;
    const T* Kh = static_cast<const T*>(P.K) + (size_t)head * L * kD;
    const T* Vh = static_cast<const T*>(P.V) + (size_t)head * L * kD;
    const T* Gh = static_cast<const T*>(P.G) + (size_t)head * L * kD;
    const int k_first = split * P.blocks_per_split * kBwdKeys;
    int k_end = k_first + P.blocks_per_split * kBwdKeys;
    k_end = k_end < n ? k_end : n;

    // the fill's rows: valid rows of this key range that are not kept (query tile 0 only).  The range is walked
    // in chunks of 2048 rows whose kept rows are marked in a bit mask; a wave then reads 4 rows per load
    // instruction (16 bytes per lane), 8 of them in flight, and adds the rows that are not marked.
    if (qt == 0) {
        double* gs = static_cast<double*>(P.gsum_part) + ((size_t)head * P.S + split) * kD;
        double tot[4] = {0.0, 0.0, 0.0, 0.0};                        // columns 4c .. 4c + 3 over rows 4 it + g
        for (int c0 = k_first; c0 < k_end; c0 += kBwdChunk) {
            const int c1 = c0 + kBwdChunk < k_end ? c0 + kBwdChunk : k_end;
            __syncthreads();
            if (tid < kBwdChunk / 32) s_bits[tid] = 0u;
            __syncthreads();
            for (int t = tid; t < ub; t += kBwdThreads) {
                const int i = P.sel[(size_t)head * P.u_stride + t];
                if (i >= c0 && i < c1) atomicOr(&s_bits[(i - c0) >> 5], 1u << ((i - c0) & 31));
            }
            __syncthreads();
            const int n_it = (c1 - c0 + 3) >> 2;
#pragma unroll 8
            for (int it = wave; it < n_it; it += kBwdWaves) {        // (rows in a fixed order per lane)
                const int rr = 4 * it + g, jr = c0 + rr;
                float x[4];
                M::row4(Gh + (size_t)(jr < c1 ? jr : c1 - 1) * kD + 4 * c, x);
                const bool use = jr < c1 && !((s_bits[rr >> 5] >> (rr & 31)) & 1u);
#pragma unroll
                for (int e = 0; e < 4; ++e) tot[e] += use ? (double)x[e] : 0.0;
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 4; ++e) s_gs[wave * 4 + g][4 * c + e] = tot[e];
        __syncthreads();
        if (tid < kD) {
            double t = 0.0;
#pragma unroll
            for (int k = 0; k < 4 * kBwdWaves; ++k) t += s_gs[k][tid];   // fixed order
            gs[tid] = t;
        }
    }
    if (qt * kBwdQ >= ub) return;                                    // no kept query in this tile (work-group-uniform)

    // B operands: the kept query of column c and its upstream gradient (zeros for an absent entry)
    const int qi = kept_row(P, head, qt * kBwdQ + c, n, ub);
    double qd[16], gd[16];
    {
        float qf[16], gf[16];
        M::row16(Qh + (size_t)(qi >= 0 ? qi : 0) * kD + 16 * g, qf);
        M::row16(Gh + (size_t)(qi >= 0 ? qi : 0) * kD + 16 * g, gf);
#pragma unroll
        for (int t = 0; t < 16; ++t) { qd[t] = qi >= 0 ? (double)qf[t] : 0.0; gd[t] = qi >= 0 ? (double)gf[t] : 0.0; }
    }
    // this lane: query c, keys 4r + g of the wave's sub-blocks (wave w takes sub-blocks w, w + 4, ... of 16 keys)
    double m = -INFINITY, l = 0.0, dacc = 0.0;
    // the next sub-block's rows are requested before the current one is worked on (on a clamped row, so the
    // request past the end is harmless; n > 0: the head has kept queries)
    float kn[16], vn[16];
    {
        const int row = k_first + 16 * wave + c < n ? k_first + 16 * wave + c : n - 1;
        M::row16(Kh + (size_t)row * kD + 16 * g, kn);
        M::row16(Vh + (size_t)row * kD + 16 * g, vn);
    }
    for (int j0 = k_first + 16 * wave; j0 < k_end; j0 += kBwdKeys) {
        float kf[16], vf[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) { kf[t] = kn[t]; vf[t] = vn[t]; }
        {
            const int row = j0 + kBwdKeys + c < n ? j0 + kBwdKeys + c : n - 1;
            M::row16(Kh + (size_t)row * kD + 16 * g, kn);
            M::row16(Vh + (size_t)row * kD + 16 * g, vn);
        }
        bwd_x4 s, cc;
        score_products(kf, qd, vf, gd, s, cc);
        double sc[4], mn = m;
        bool ok[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            ok[r] = j0 + 4 * r + g < k_end;
            sc[r] = s[r] * 0.125;
            if (ok[r] && sc[r] > mn) mn = sc[r];
        }
        if (mn > -INFINITY) {
            const double a = m == -INFINITY ? 0.0 : bwd_exp(m - mn);
            l *= a; dacc *= a;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const double w = ok[r] ? bwd_exp(sc[r] - mn) : 0.0;
                l += w; dacc += w * cc[r];
            }
            m = mn;
        }
    }
    // fold the four lane groups (the same query, different keys), then the four waves, in fixed order
    {
        double mw = m;
        { const double o = __shfl_xor(mw, 16, 64); mw = o > mw ? o : mw; }
        { const double o = __shfl_xor(mw, 32, 64); mw = o > mw ? o : mw; }
        const double a = m == -INFINITY ? 0.0 : bwd_exp(m - mw);
        l *= a; dacc *= a;
        l += __shfl_xor(l, 16, 64); dacc += __shfl_xor(dacc, 16, 64);
        l += __shfl_xor(l, 32, 64); dacc += __shfl_xor(dacc, 32, 64);
        if (g == 0) { s_part[wave][c][0] = mw; s_part[wave][c][1] = l; s_part[wave][c][2] = dacc; }
    }
    __syncthreads();
    if (tid < kBwdQ) {
        double mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < kBwdWaves; ++w) mx = s_part[w][tid][0] > mx ? s_part[w][tid][0] : mx;
        double lt = 0.0, dt = 0.0;
#pragma unroll
        for (int w = 0; w < kBwdWaves; ++w) {
            const double a = s_part[w][tid][0] == -INFINITY ? 0.0 : bwd_exp(s_part[w][tid][0] - mx);
            lt += a * s_part[w][tid][1]; dt += a * s_part[w][tid][2];
        }
        double* sp = static_cast<double*>(P.stats_part) + ((((size_t)head * P.QT + qt) * P.S + split) * kBwdQ + tid) * 3;
        sp[0] = mx; sp[1] = lt; sp[2] = dt;
    }
}

// combine the key splits' statistics of the tile's 16 kept queries: ln sum exp and D (threads 0 .. 15)
__device__ __forceinline__ void combine_stats(double* lse, double* D, const BwdParams& P, int head, int qt)
{
    if (threadIdx.x < kBwdQ) {
        const double* sp = static_cast<const double*>(P.stats_part) + (((size_t)head * P.QT + qt) * P.S * kBwdQ + threadIdx.x) * 3;
        double mx = -INFINITY;
        for (int s = 0; s < P.S; ++s) { const double v = sp[(size_t)s * kBwdQ * 3]; mx = v > mx ? v : mx; }
        double lt = 0, dt = 0;
        for (int s = 0; s < P.S; ++s) {
            const double ms = sp[(size_t)s * kBwdQ * 3];
            const double a = ms == -INFINITY ? 0.0 : exp(ms - mx);
            lt += a * sp[(size_t)s * kBwdQ * 3 + 1];
            dt += a * sp[(size_t)s * kBwdQ * 3 + 2];
        }
        lse[threadIdx.x] = lt > 0 ? mx + log(lt) : 0.0;
        D[threadIdx.x] = lt > 0 ? dt / lt : 0.0;
    }
}

// ---- dQ of the tile's kept queries over this key split
template <typename T>
__global__ __launch_bounds__(kBwdThreads)
void bwd_dq_kernel(const BwdParams P)
{
    using M = BwdMem<T>;
    __shared__ double s_lse[kBwdQ], s_D[kBwdQ];
    __shared__ double s_acc[kBwdWaves][16][64];                      // the waves' accumulators, register by register
    const int split = blockIdx.x, qt = blockIdx.y, head = blockIdx.z;
    const int b = head / P.H, L = P.L;
    const int n = valid_len(P.lengths, b, L);
    const int ub = kept_count(P, b, n);
    if (qt * kBwdQ >= ub) return;                                    // work-group-uniform
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15, g = lane >> 4;
    const T* Qh = static_cast<const T*>(P.Q) + (size_t)head * L * kD;
    const T* Kh = static_cast<const T*>(P.K) + (size_t)head * L * kD;
    const T* Vh = static_cast<const T*>(P.V) + (size_t)head * L * kD;
    const T* Gh = static_cast<const T*>(P.G) + (size_t)head * L * kD;
    const int k_first = split * P.blocks_per_split * kBwdKeys;
    int k_end = k_first + P.blocks_per_split * kBwdKeys;
    k_end = k_end < n ? k_end : n;

    combine_stats(s_lse, s_D, P, head, qt);
    __syncthreads();
    if (split == 0 && tid < kBwdQ) {                                 // for the key-stationary kernel
        double* st = static_cast<double*>(P.stats) + ((size_t)head * P.QT * kBwdQ + qt * kBwdQ + tid) * 2;
        st[0] = s_lse[tid]; st[1] = s_D[tid];
    }
    const int qi = kept_row(P, head, qt * kBwdQ + c, n, ub);
    double qd[16], gd[16];
    {
        float qf[16], gf[16];
        M::row16(Qh + (size_t)(qi >= 0 ? qi : 0) * kD + 16 * g, qf);
        M::row16(Gh + (size_t)(qi >= 0 ? qi : 0) * kD + 16 * g, gf);
#pragma unroll
        for (int t = 0; t < 16; ++t) { qd[t] = qi >= 0 ? (double)qf[t] : 0.0; gd[t] = qi >= 0 ? (double)gf[t] : 0.0; }
    }
    const double lse_c = s_lse[c], D_c = s_D[c];
    // dQ^T of this wave's keys: acc[dt][r] is element 4 (4r + g) + dt of query c
    bwd_x4 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) acc[dt] = bwd_x4{0.0, 0.0, 0.0, 0.0};
    // operands of a sub-block: the lane's key row for the score products (16 contiguous elements), and for the
    // second product's A the keys 4r + g, elements 4c .. 4c + 3; the next sub-block's are requested before
    // the current one is worked on (clamped rows: the request past the end is harmless)
    float kn[16], vn[16], k4n[4][4];
    auto request = [&](int j0) {
        const int row = j0 + c < n ? j0 + c : n - 1;
        M::row16(Kh + (size_t)row * kD + 16 * g, kn);
        M::row16(Vh + (size_t)row * kD + 16 * g, vn);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int key = j0 + 4 * r + g;
            M::row4(Kh + (size_t)(key < n ? key : n - 1) * kD + 4 * c, k4n[r]);
        }
    };
    request(k_first + 16 * wave);
    for (int j0 = k_first + 16 * wave; j0 < k_end; j0 += kBwdKeys) {
        float kf[16], vf[16], k4[4][4];
#pragma unroll
        for (int t = 0; t < 16; ++t) { kf[t] = kn[t]; vf[t] = vn[t]; }
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) k4[r][dt] = k4n[r][dt];
        request(j0 + kBwdKeys);
        bwd_x4 s, cc;
        score_products(kf, qd, vf, gd, s, cc);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool ok = j0 + 4 * r + g < k_end && qi >= 0;
            const double p = ok ? bwd_exp(s[r] * 0.125 - lse_c) : 0.0;
            const double gv = 0.125 * p * (cc[r] - D_c);             // g_ij of query c and key 4r + g
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)k4[r][dt], gv, acc[dt], 0, 0, 0);
        }
    }
    // the four waves' shares in wave order: thread (wave w, lane) adds up row r = w of every accumulator, which
    // gives it the four consecutive elements 16 w + 4 g .. + 3 of query c
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) s_acc[wave][4 * dt + r][lane] = acc[dt][r];
    __syncthreads();
    double tot[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kBwdWaves; ++w) t += s_acc[w][4 * dt + wave][lane];
        tot[dt] = t;
    }
    const int e0 = 16 * wave + 4 * g;
    if (P.S == 1) {
        if (qi >= 0) {
            const float v[4] = {(float)tot[0], (float)tot[1], (float)tot[2], (float)tot[3]};
            M::store4(static_cast<T*>(P.dQ) + ((size_t)head * L + qi) * kD + e0, v);
        }
    } else {
        double* dp = static_cast<double*>(P.dq_part) + ((((size_t)head * P.QT + qt) * P.S + split) * kBwdQ + c) * kD + e0;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) dp[dt] = tot[dt];
    }
}

template <typename T>
__global__ __launch_bounds__(kBwdThreads)
void bwd_dq_reduce_kernel(const BwdParams P)
{
    using M = BwdMem<T>;
    const int qt = blockIdx.x, head = blockIdx.y;
    const int b = head / P.H;
    const int n = valid_len(P.lengths, b, P.L);
    const int ub = kept_count(P, b, n);
    if (qt * kBwdQ >= ub) return;
    const int tid = threadIdx.x, i = tid >> 4, e0 = 4 * (tid & 15);
    const int qi = kept_row(P, head, qt * kBwdQ + i, n, ub);
    if (qi < 0) return;
    const double* dp = static_cast<const double*>(P.dq_part) + (((size_t)head * P.QT + qt) * P.S * kBwdQ + i) * kD + e0;
    double acc[4] = {0, 0, 0, 0};
    for (int s = 0; s < P.S; ++s)                                    // split order
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += dp[(size_t)s * kBwdQ * kD + e];
    const float v[4] = {(float)acc[0], (float)acc[1], (float)acc[2], (float)acc[3]};
    M::store4(static_cast<T*>(P.dQ) + ((size_t)head * P.L + qi) * kD + e0, v);
}

// ---- key-stationary: one work-group per block of 64 keys (16 per wave) walks all kept queries of the head
template <typename T>
__global__ __launch_bounds__(kBwdThreads)
void bwd_dkv_kernel(const BwdParams P)
{
    using M = BwdMem<T>;
    __shared__ unsigned char s_flag[kBwdKeys];
    __shared__ double s_gm[kD];
    __shared__ __attribute__((aligned(16))) float s_q[kBwdStaged][kBwdStage], s_g[kBwdStaged][kBwdStage];
    __shared__ double s_lse[kBwdStaged], s_D[kBwdStaged];
    __shared__ int s_qrow[kBwdStaged];
    const int blk = blockIdx.x, head = blockIdx.y;
    const int b = head / P.H, L = P.L;
    const int n = valid_len(P.lengths, b, L);
    const int ub = kept_count(P, b, n);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15, g = lane >> 4;
    const int r0 = blk * kBwdKeys;
    const T* Qh = static_cast<const T*>(P.Q) + (size_t)head * L * kD;
    const T* Kh = static_cast<const T*>(P.K) + (size_t)head * L * kD;
    const T* Vh = static_cast<const T*>(P.V) + (size_t)head * L * kD;
    const T* Gh = static_cast<const T*>(P.G) + (size_t)head * L * kD;
    const int j = r0 + 16 * wave + c;                                // this lane's key (the column of its accumulators)

    // which rows of this block are kept queries; the fill's share of dV under the mean fill: every valid v_j
    // receives 1/n of each filled row's gradient
    if (tid < kBwdKeys) s_flag[tid] = 0;
    if (tid < kD) {
        double t = 0;
        if (P.fill == PSA_FILL_MEAN) {
            const double* gs = static_cast<const double*>(P.gsum_part) + (size_t)head * P.S * kD + tid;
            for (int s = 0; s < P.S; ++s) t += gs[(size_t)s * kD]; // split order
        }
        s_gm[tid] = n > 0 ? t / (double)n : 0.0;
    }
    __syncthreads();
    for (int t = tid; t < ub; t += kBwdThreads) {
        const int i = P.sel[(size_t)head * P.u_stride + t];
        if (i >= r0 && i < r0 + kBwdKeys && i < n) s_flag[i - r0] = 1;
    }
    __syncthreads();

    // dK^T, dV^T of this wave's 16 keys: acc[dt][r] is element 4 (4r + g) + dt of key j
    bwd_x4 dk[4], dv[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) { dk[dt] = bwd_x4{0.0, 0.0, 0.0, 0.0}; dv[dt] = bwd_x4{0.0, 0.0, 0.0, 0.0}; }
    const bool wave_live = r0 + 16 * wave < n;                       // wave-uniform: some key of the wave is valid
    // B operands of the score products: this lane's key row
    double kd[16], vd[16];
    if (r0 < n) {                                                    // (work-group-uniform; n > 0 inside)
        const int row = j < n ? j : n - 1;
        float kf[16], vf[16];
        M::row16(Kh + (size_t)row * kD + 16 * g, kf);
        M::row16(Vh + (size_t)row * kD + 16 * g, vf);
#pragma unroll
        for (int t = 0; t < 16; ++t) { kd[t] = (double)kf[t]; vd[t] = (double)vf[t]; }
        // The kept queries are the same for all four waves: their rows of Q and G (as float) and their
        // statistics are staged in LDS 64 at a time, so the loop over query tiles touches no global memory.
        // Rows are kBwdStage floats apart: 16-byte reads of 8 consecutive rows then fall on all 32 banks.
        for (int q0 = 0; q0 < ub; q0 += kBwdStaged) {                // work-group-uniform
            __syncthreads();                                         // the previous 64 have been used
            {
                const int row_s = tid >> 2, part = tid & 3;          // 64 rows, 4 threads each
                const int qs = kept_row(P, head, q0 + row_s, n, ub);
                float a[16], bq[16];
                M::row16(Qh + (size_t)(qs >= 0 ? qs : 0) * kD + 16 * part, a);
                M::row16(Gh + (size_t)(qs >= 0 ? qs : 0) * kD + 16 * part, bq);
#pragma unroll
                for (int t = 0; t < 16; ++t) {
                    s_q[row_s][16 * part + t] = qs >= 0 ? a[t] : 0.f;
                    s_g[row_s][16 * part + t] = qs >= 0 ? bq[t] : 0.f;
                }
                if (part == 0) {
                    s_qrow[row_s] = qs;
                    // (statistics exist for the tiles that hold a kept query)
                    const bool has = q0 + row_s < ((ub + kBwdQ - 1) / kBwdQ) * kBwdQ;
                    const double* st = static_cast<const double*>(P.stats) + ((size_t)head * P.QT * kBwdQ + (has ? q0 + row_s : 0)) * 2;
                    s_lse[row_s] = has ? st[0] : 0.0;
                    s_D[row_s] = has ? st[1] : 0.0;
                }
            }
            __syncthreads();
            if (!wave_live) continue;
            int n_t = (ub - q0 + kBwdQ - 1) / kBwdQ;
            n_t = n_t < kBwdStaged / kBwdQ ? n_t : kBwdStaged / kBwdQ;
            for (int tt = 0; tt < n_t; ++tt) {                       // query tiles in order
                // A operands of the score products: staged query 16 tt + c
                float qf[16], gf[16];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float4 x = *reinterpret_cast<const float4*>(&s_q[16 * tt + c][16 * g + 4 * k]);
                    const float4 y = *reinterpret_cast<const float4*>(&s_g[16 * tt + c][16 * g + 4 * k]);
                    qf[4 * k] = x.x; qf[4 * k + 1] = x.y; qf[4 * k + 2] = x.z; qf[4 * k + 3] = x.w;
                    gf[4 * k] = y.x; gf[4 * k + 1] = y.y; gf[4 * k + 2] = y.z; gf[4 * k + 3] = y.w;
                }
                bwd_x4 s, cc;
                score_products(qf, kd, gf, vd, s, cc);               // s[r], cc[r]: staged query 16 tt + 4r + g against key j
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int qq = 16 * tt + 4 * r + g;
                    const bool ok = j < n && s_qrow[qq] >= 0;
                    const double p = ok ? bwd_exp(s[r] * 0.125 - s_lse[qq]) : 0.0;
                    const double gv = 0.125 * p * (cc[r] - s_D[qq]);
                    // A operands of the products that contract over the queries: elements 4c .. 4c + 3 of row qq
                    const float4 q4 = *reinterpret_cast<const float4*>(&s_q[qq][4 * c]);
                    const float4 g4 = *reinterpret_cast<const float4*>(&s_g[qq][4 * c]);
                    dk[0] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)q4.x, gv, dk[0], 0, 0, 0);
                    dv[0] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)g4.x, p, dv[0], 0, 0, 0);
                    dk[1] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)q4.y, gv, dk[1], 0, 0, 0);
                    dv[1] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)g4.y, p, dv[1], 0, 0, 0);
                    dk[2] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)q4.z, gv, dk[2], 0, 0, 0);
                    dv[2] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)g4.z, p, dv[2], 0, 0, 0);
                    dk[3] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)q4.w, gv, dk[3], 0, 0, 0);
                    dv[3] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)g4.w, p, dv[3], 0, 0, 0);
                }
            }
        }
    }
    // rows of dK, dV (and the rows of dQ outside I_sparse, which no gradient reaches): 16 bytes at a time
    if (j < L) {
        const bool valid = j < n, kept = valid && s_flag[16 * wave + c];
        T* dkr = static_cast<T*>(P.dK) + ((size_t)head * L + j) * kD;
        T* dvr = static_cast<T*>(P.dV) + ((size_t)head * L + j) * kD;
        T* dqr = static_cast<T*>(P.dQ) + ((size_t)head * L + j) * kD;
        const float zero[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int e0 = 16 * r + 4 * g;
            float own[4] = {0.f, 0.f, 0.f, 0.f};                     // the value fill hands v_j the gradient of its own row
            if (P.fill != PSA_FILL_MEAN && valid && !kept) M::row4(Gh + (size_t)j * kD + e0, own);
            float ok_[4], ov[4];
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                double v = dv[dt][r];
                if (P.fill == PSA_FILL_MEAN) v += s_gm[e0 + dt]; else v += (double)own[dt];
                ok_[dt] = valid ? (float)dk[dt][r] : 0.f;
                ov[dt] = valid ? (float)v : 0.f;
            }
            M::store4(dkr + e0, ok_);
            M::store4(dvr + e0, ov);
            if (!kept) M::store4(dqr + e0, zero);
        }
    }
}

template <typename T>
static hipError_t launch_bwd_t(const BwdParams& P, int BH, hipStream_t stream)
{
    const dim3 qgrid(P.S, P.QT, BH);
    hipLaunchKernelGGL(bwd_stats_kernel<T>, qgrid, dim3(kBwdThreads), 0, stream, P);
    hipLaunchKernelGGL(bwd_dq_kernel<T>, qgrid, dim3(kBwdThreads), 0, stream, P);
    hipLaunchKernelGGL(bwd_dkv_kernel<T>, dim3((P.L + kBwdKeys - 1) / kBwdKeys, BH), dim3(kBwdThreads), 0, stream, P);
    if (P.S > 1) hipLaunchKernelGGL(bwd_dq_reduce_kernel<T>, dim3(P.QT, BH), dim3(kBwdThreads), 0, stream, P);
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
    return s.dtype == PSA_F32 ? launch_bwd_t<float>(P, BH, stream) : launch_bwd_t<bf16_t>(P, BH, stream);
}

}  // namespace psa

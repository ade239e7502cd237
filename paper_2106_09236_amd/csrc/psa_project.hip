// The projections around the attention path (Sec. 3.1: Q = X W_q, K = X W_k,
// V = X W_v; Sec. 2.2, Eq. 5: the multi-head self-attention module; Sec. 4.2: 4
// heads of 64 dimensions): one GEMM kernel, C[m][n] = sum_k A[m][k] W[n][k] + bias[n],
// with the head split of the projected tensors folded into its addressing, so
// that Q, K, V are produced directly as [B, H, L, 64] and the output matrix reads
// the attention result in that layout: no transposes in memory.
//
// Both operands have the contraction index contiguous (W is stored [d_out, d_in]),
// which is the layout the MFMA operands want.  A work-group of 4 waves computes a
// 64 x 64 tile of C, each wave a 32 x 32 quarter:
//   bfloat16  v_mfma_f32_32x32x16_bf16, lane (c, h) = (lane % 32, lane / 32):
//             A[i = c][k = 8h + e], B[k = 8h + e][j = c], D[i = 8(r/4) + 4h + r%4][j = c]
//   float32   v_mfma_f32_32x32x2f32: A[i = c][k = h], B[k = h][j = c], same D; the
//             contraction order is free, so step t of a 64-wide chunk takes k = 32h + t
//             and a lane reads 32 contiguous floats of its row.
// The contraction runs in chunks of 64 through LDS, the next chunk's global loads
// in flight during the current chunk's products.
#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

constexpr int kPT = 64;                       // tile edge and contraction chunk

struct ProjectParams {
    const void* A;                            // [M, Kd] rows, or [B, H, L, 64] when a_heads
    const void* W[3];                         // [N, Kd] each
    const void* bias[3];                      // [N] or nullptr
    void* C[3];                               // [M, N] rows, or [B, H, L, 64] when c_heads
    int M, N, Kd, L, H, a_heads, c_heads;
};

template <typename T> struct ProjTraits;
template <> struct ProjTraits<float> {
    static constexpr int kStride = 68;        // floats per LDS row (64 + 4 pad)
    static constexpr int kVecPerRow = 16, kVecPerThread = 4;
    typedef float4 Vec;
};
template <> struct ProjTraits<bf16_t> {
    static constexpr int kStride = 72;        // bf16 per LDS row (64 + 8 pad)
    static constexpr int kVecPerRow = 8, kVecPerThread = 2;
    typedef uint4 Vec;
};

template <typename T>
__global__ __launch_bounds__(256)
void project_kernel(const ProjectParams P)
{
    using PT = ProjTraits<T>;
    using Vec = typename PT::Vec;
    constexpr int S = PT::kStride, VPR = PT::kVecPerRow, VPT = PT::kVecPerThread;
    __shared__ __attribute__((aligned(16))) T sA[kPT * S];
    __shared__ __attribute__((aligned(16))) T sW[kPT * S];

    const int which = blockIdx.z;
    const T* A = static_cast<const T*>(P.A);
    const T* W = static_cast<const T*>(P.W[which]);
    const T* bias = static_cast<const T*>(P.bias[which]);
    T* C = static_cast<T*>(P.C[which]);
    const int n0 = blockIdx.x * kPT, m0 = blockIdx.y * kPT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int n_kc = P.Kd / kPT;

    // element offset of row m, contraction chunk kc, of A
    auto a_row = [&](int m, int kc) -> size_t {
        m = m < P.M ? m : P.M - 1;                                    // clamped: rows beyond M are never stored
        if (P.a_heads) { const int b = m / P.L, l = m - b * P.L; return (((size_t)b * P.H + kc) * P.L + l) * kD; }
        return (size_t)m * P.Kd + (size_t)kc * kPT;
    };
    Vec ra[VPT], rw[VPT];
    auto fetch = [&](int kc) {
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const int idx = tid + 256 * j, row = idx / VPR, col = idx % VPR;
            ra[j] = reinterpret_cast<const Vec*>(A + a_row(m0 + row, kc))[col];
            rw[j] = reinterpret_cast<const Vec*>(W + (size_t)(n0 + row) * P.Kd + (size_t)kc * kPT)[col];
        }
    };
    auto put = [&]() {
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            const int idx = tid + 256 * j, row = idx / VPR, col = idx % VPR;
            reinterpret_cast<Vec*>(sA + row * S)[col] = ra[j];
            reinterpret_cast<Vec*>(sW + row * S)[col] = rw[j];
        }
    };

    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    fetch(0);
    for (int kc = 0; kc < n_kc; ++kc) {
        __syncthreads();                                  // the previous chunk's reads of LDS are done
        put();
        __syncthreads();
        if (kc + 1 < n_kc) fetch(kc + 1);                 // in flight during the products (uniform branch)
        const T* ar = sA + (wm * 32 + c) * S;
        const T* wr = sW + (wn * 32 + c) * S;
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const uint4 a = *reinterpret_cast<const uint4*>(ar + kk * 16 + 8 * h);
                const uint4 b = *reinterpret_cast<const uint4*>(wr + kk * 16 + 8 * h);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const float4 a = *reinterpret_cast<const float4*>(ar + 32 * h + 4 * v);
                const float4 b = *reinterpret_cast<const float4*>(wr + 32 * h + 4 * v);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
            }
        }
    }

    // ---- epilogue: bias, rounding to the storage type, head-split or row-major store
    const int n = n0 + wn * 32 + c;
    float bv = 0.f;
    if (bias) {
        if constexpr (sizeof(T) == 2) bv = bf16_to_f32(reinterpret_cast<const uint16_t*>(bias)[n]);
        else bv = reinterpret_cast<const float*>(bias)[n];
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        if (m >= P.M) continue;
        size_t off;
        if (P.c_heads) {
            const int b = m / P.L, l = m - b * P.L;
            off = (((size_t)b * P.H + (n >> 6)) * P.L + l) * kD + (n & 63);
        } else {
            off = (size_t)m * P.N + n;
        }
        const float val = acc[r] + bv;
        if constexpr (sizeof(T) == 2) reinterpret_cast<uint16_t*>(C)[off] = (uint16_t)(cvt_pk_bf16(val, 0.f) & 0xFFFFu);
        else reinterpret_cast<float*>(C)[off] = val;
    }
}

static hipError_t launch_project(const ProjectParams& P, int n_mat, int dtype, hipStream_t stream)
{
    const dim3 grid(P.N / kPT, (P.M + kPT - 1) / kPT, n_mat);
    if (dtype == PSA_F32) hipLaunchKernelGGL(project_kernel<float>, grid, dim3(256), 0, stream, P);
    else                  hipLaunchKernelGGL(project_kernel<bf16_t>, grid, dim3(256), 0, stream, P);
    return hipGetLastError();
}

hipError_t launch_qkv_project(const psa_shape_t& s, const void* X, const psa_mhsa_weights_t& w,
                              void* Q, void* K, void* V, hipStream_t stream)
{
    ProjectParams P;
    P.A = X;
    P.W[0] = w.Wq; P.W[1] = w.Wk; P.W[2] = w.Wv;
    P.bias[0] = w.bq; P.bias[1] = w.bk; P.bias[2] = w.bv;
    P.C[0] = Q; P.C[1] = K; P.C[2] = V;
    P.M = s.B * s.L_K; P.N = s.H * kD; P.Kd = s.H * kD; P.L = s.L_K; P.H = s.H; P.a_heads = 0; P.c_heads = 1;
    return launch_project(P, 3, s.dtype, stream);
}

hipError_t launch_out_project(const psa_shape_t& s, const void* A, const psa_mhsa_weights_t& w, void* Y, hipStream_t stream)
{
    ProjectParams P;
    P.A = A;
    P.W[0] = w.Wo; P.W[1] = P.W[2] = nullptr;
    P.bias[0] = w.bo; P.bias[1] = P.bias[2] = nullptr;
    P.C[0] = Y; P.C[1] = P.C[2] = nullptr;
    P.M = s.B * s.L_K; P.N = s.H * kD; P.Kd = s.H * kD; P.L = s.L_K; P.H = s.H; P.a_heads = 1; P.c_heads = 0;
    return launch_project(P, 1, s.dtype, stream);
}

}  // namespace psa

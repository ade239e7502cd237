// The projections around the attention path (Sec. 3.1: Q = X W_q, K = X W_k,
// V = X W_v; Sec. 2.2, Eq. 5: the multi-head self-attention module; Sec. 4.2: 4
// heads of 64 dimensions): one GEMM kernel, C[m][n] = sum_k A[m][k] W[n][k] + bias[n],
// with the head split of the projected tensors folded into its addressing, so
// that Q, K, V are produced directly as [B, H, L, 64] and the output matrix reads
// the attention result in that layout: no transposes in memory.
//
// Both operands have the contraction index contiguous (W is stored [d_out, d_in]),
// which is the layout the MFMA operands want.  A work-group of 4 waves computes a
// 128 x 128 tile of C, each wave a 64 x 64 quarter as 2 x 2 MFMA tiles of 32 x 32:
// The products are taken as C^T = W A^T (rows of W on the MFMA row axis), so that a
// lane ends up with one row of C and runs of four consecutive columns:
//   bfloat16  v_mfma_f32_32x32x16_bf16, lane (c, h) = (lane % 32, lane / 32):
//             A[i = c][k = 8h + e], B[k = 8h + e][j = c], D[i = 8(r/4) + 4h + r%4][j = c]
//   float32   v_mfma_f32_32x32x2f32: A[i = c][k = h], B[k = h][j = c], same D; the
//             contraction order is free, so step t of a chunk takes k = (chunk/2) h + t
//             and a lane reads contiguous floats of its row.
// The contraction runs in chunks (64 bfloat16 / 32 float32 elements) through LDS,
// the next chunk's global loads in flight during the current chunk's products.
#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

constexpr int kPT = 128;                      // tile edge

struct ProjectParams {
    const void* A;                            // [M, Kd] rows, or [B, H, L, 64] when a_heads
    const void* W[3];                         // [N, Kd] each
    const void* bias[3];                      // [N] or nullptr
    void* C[3];                               // [M, N] rows, or [B, H, L, 64] when c_heads
    int M, N, Kd, L, H, a_heads, c_heads;
};

template <typename T> struct ProjTraits;
template <> struct ProjTraits<float> {
    static constexpr int kChunk = 32;         // contraction elements per step through LDS
    static constexpr int kStride = 36;        // floats per LDS row (32 + 4 pad)
    typedef float4 Vec;
};
template <> struct ProjTraits<bf16_t> {
    static constexpr int kChunk = 64;
    static constexpr int kStride = 72;        // bf16 per LDS row (64 + 8 pad)
    typedef uint4 Vec;
};

template <typename T>
__global__ __launch_bounds__(256)
void project_kernel(const ProjectParams P)
{
    using PT = ProjTraits<T>;
    using Vec = typename PT::Vec;
    constexpr int S = PT::kStride, CH = PT::kChunk;
    constexpr int VPR = CH * (int)sizeof(T) / 16;          // 16-byte vectors per tile row: 8
    constexpr int VPT = kPT * VPR / 256;                   // vectors per thread and operand: 4
    __shared__ __attribute__((aligned(16))) T sA[kPT * S];
    __shared__ __attribute__((aligned(16))) T sW[kPT * S];

    const int which = blockIdx.z;
    const T* A = static_cast<const T*>(P.A);
    // (selected with conditionals: indexing the argument arrays by a run-time value would move them to scratch)
    const T* W = static_cast<const T*>(which == 0 ? P.W[0] : (which == 1 ? P.W[1] : P.W[2]));
    const T* bias = static_cast<const T*>(which == 0 ? P.bias[0] : (which == 1 ? P.bias[1] : P.bias[2]));
    T* C = static_cast<T*>(which == 0 ? P.C[0] : (which == 1 ? P.C[1] : P.C[2]));
    const int n0 = blockIdx.x * kPT, m0 = blockIdx.y * kPT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int n_kc = P.Kd / CH;

    // this thread's share of the tiles: vector `col` of rows row0 + 32 j (same for A and W)
    const int row0 = tid / VPR, col = tid % VPR;
    static_assert(256 / VPR == 32, "32 tile rows per pass of the work-group");
    size_t a_base[VPT], w_base[VPT];                       // element offsets of the rows at contraction element 0
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        int m = m0 + row0 + 32 * j;
        m = m < P.M ? m : P.M - 1;                         // clamped: rows beyond M are never stored
        if (P.a_heads) { const int b = m / P.L, l = m - b * P.L; a_base[j] = ((size_t)b * P.H * P.L + l) * kD; }
        else a_base[j] = (size_t)m * P.Kd;
        const int nr = n0 + row0 + 32 * j;
        w_base[j] = (size_t)(nr < P.N ? nr : P.N - 1) * P.Kd;          // clamped: columns beyond N are never stored
    }
    // contraction element k0 (a multiple of the chunk, so inside one head) of a row of A
    const size_t head_stride = (size_t)P.L * kD;
    static_assert(VPT == 4, "four vectors per thread and operand");
    Vec ra0, ra1, ra2, ra3, rw0, rw1, rw2, rw3;           // (named: arrays of these ended up in scratch memory)
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#define PSA_FETCH(J, KA, KW)                                                       \
    ra##J = reinterpret_cast<const Vec*>(A + a_base[J] + (KA))[col];                 \
    rw##J = reinterpret_cast<const Vec*>(W + w_base[J] + (KW))[col];
#define PSA_PUT(J)                                                                 \
    reinterpret_cast<Vec*>(sA + (row0 + 32 * J) * S)[col] = ra##J;                  \
    reinterpret_cast<Vec*>(sW + (row0 + 32 * J) * S)[col] = rw##J;
    PSA_FETCH(0, 0, 0) PSA_FETCH(1, 0, 0) PSA_FETCH(2, 0, 0) PSA_FETCH(3, 0, 0)
    for (int kc = 0; kc < n_kc; ++kc) {
        __syncthreads();                                  // the previous chunk's reads of LDS are done
        PSA_PUT(0) PSA_PUT(1) PSA_PUT(2) PSA_PUT(3)
        __syncthreads();
        // the next chunk travels during the products (the last iteration re-reads its own chunk: harmless)
        {
            const int k0 = (kc + 1 < n_kc ? kc + 1 : kc) * CH;   // a multiple of the chunk, so inside one head
            const size_t ka = P.a_heads ? (size_t)(k0 >> 6) * head_stride + (k0 & 63) : (size_t)k0;
            PSA_FETCH(0, ka, k0) PSA_FETCH(1, ka, k0) PSA_FETCH(2, ka, k0) PSA_FETCH(3, ka, k0)
        }
        const T* ar = sA + (wm * 64 + c) * S;
        const T* wr = sW + (wn * 64 + c) * S;
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int kk = 0; kk < CH / 16; ++kk) {
                bf16x8 a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(ar + i * 32 * S + kk * 16 + 8 * h));
                    b[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wr + i * 32 * S + kk * 16 + 8 * h));
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int v = 0; v < CH / 8; ++v) {            // lane half h takes k = (CH/2) h + 4v .. +3
                float4 a[2], b[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    a[i] = *reinterpret_cast<const float4*>(ar + i * 32 * S + (CH / 2) * h + 4 * v);
                    b[i] = *reinterpret_cast<const float4*>(wr + i * 32 * S + (CH / 2) * h + 4 * v);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].x, a[i].x, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].y, a[i].y, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].z, a[i].z, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].w, a[i].w, acc[i][j], 0, 0, 0);
                    }
            }
        }
    }

#undef PSA_FETCH
#undef PSA_PUT
    // ---- epilogue.  The products were taken as C^T = W A^T (W rows on the MFMA row axis), so a
    // lane owns ONE row m of C and, per register quad, four consecutive columns n: bias, rounding
    // to the storage type, and one 16-byte (float32) or 8-byte (bfloat16) store per quad, either
    // row-major or into the head-split layout.
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m0 + wm * 64 + i * 32 + c;
        if (m >= P.M) continue;
        size_t row_off;                                   // element offset of column 0 of row m ...
        size_t head_step;                                 // ... and of a step of 64 columns
        if (P.c_heads) {
            const int b = m / P.L, l = m - b * P.L;
            row_off = ((size_t)b * P.H * P.L + l) * kD;
            head_step = (size_t)P.L * kD;
        } else {
            row_off = (size_t)m * P.N;
            head_step = kD;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * 64 + j * 32 + 8 * q + 4 * h;      // first of four consecutive columns
                if (n >= P.N) continue;                                   // N is a multiple of 64: all four or none
                float bv[4] = {0.f, 0.f, 0.f, 0.f};
                if (bias) {
                    if constexpr (sizeof(T) == 2) {
                        const uint2 bb = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(bias) + n);
                        bv[0] = bf16_lo(bb.x); bv[1] = bf16_hi(bb.x); bv[2] = bf16_lo(bb.y); bv[3] = bf16_hi(bb.y);
                    } else {
                        const float4 bb = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(bias) + n);
                        bv[0] = bb.x; bv[1] = bb.y; bv[2] = bb.z; bv[3] = bb.w;
                    }
                }
                const size_t off = row_off + (size_t)(n >> 6) * head_step + (n & 63);
                const float v0 = acc[i][j][4 * q + 0] + bv[0], v1 = acc[i][j][4 * q + 1] + bv[1];
                const float v2 = acc[i][j][4 * q + 2] + bv[2], v3 = acc[i][j][4 * q + 3] + bv[3];
                if constexpr (sizeof(T) == 2)
                    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(C) + off) = make_uint2(cvt_pk_bf16(v0, v1), cvt_pk_bf16(v2, v3));
                else
                    *reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + off) = make_float4(v0, v1, v2, v3);
            }
    }
}

static hipError_t launch_project(const ProjectParams& P, int n_mat, int dtype, hipStream_t stream)
{
    const dim3 grid((P.N + kPT - 1) / kPT, (P.M + kPT - 1) / kPT, n_mat);
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

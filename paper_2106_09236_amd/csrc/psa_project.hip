// The projections around the attention path (Sec. 3.1: Q = X W_q, K = X W_k,
// V = X W_v; Sec. 2.2, Eq. 5: the multi-head self-attention module; Sec. 4.2: 4
// heads of 64 dimensions): one GEMM kernel, C[m][n] = sum_k A[m][k] W[n][k] + bias[n],
// with the head split of the projected tensors folded into its addressing, so
// that Q, K, V are produced directly as [B, H, L, 64] and the output matrix reads
// the attention result in that layout: no transposes in memory.
//
// Both operands have the contraction index contiguous (W is stored [d_out, d_in]),
// which is the layout the MFMA operands want.  A work-group of 4 waves computes a
// 128 x 128 tile of C, each wave a 64 x 64 quarter as 2 x 2 MFMA tiles of 32 x 32
// (128 x 64 with 2 x 1 MFMA tiles per wave for shapes that would otherwise leave
// compute units without work).  The products are taken as C^T = W A^T (rows of W on
// the MFMA row axis), so that a lane ends up with one row of C and runs of four
// consecutive columns:
//   v_mfma_f32_32x32x16_bf16, lane (c, h) = (lane % 32, lane / 32):
//   A[i = c][k = 8h + e], B[k = 8h + e][j = c], D[i = 8(r/4) + 4h + r%4][j = c]
// The contraction runs in chunks (64 bfloat16 / 32 float32 elements) through LDS,
// the next chunk's global loads in flight during the current chunk's products.
// bfloat16 tensors: project_kernel.  float32 tensors: project_split_kernel, which
// runs on the same bfloat16 MFMA with every operand split into three bfloat16 parts.
#include "psa_device.h"
#include "psa_internal.h"
#include "psa_trace.h"

namespace psa {

struct ProjectParams {
    const void* A;                            // [M, Kd] rows, or [B, H, L, 64] when a_heads
    const void* W[3];                         // [N, Kd] each
    const void* bias[3];                      // [N] or nullptr
    void* C[3];                               // [M, N] rows, or [B, H, L, 64] when c_heads
    int M, N, Kd, L, H, a_heads, c_heads, n_mat;
};

constexpr int kProjChunk = 64;                // bfloat16 contraction elements per step through LDS
constexpr int kProjStride = 72;               // bfloat16 per LDS row (64 + 8 pad)

// A wave computes WM x WN MFMA tiles (rows x columns of C); the four waves of a work-group
// form a 2 x 2 grid, so the work-group's tile of C is 64 WM x 64 WN.
template <int WM, int WN>
struct ProjLayout {
    static constexpr int kTM = 64 * WM, kTN = 64 * WN;                     // tile rows, tile columns
    static constexpr int kOperandElems = (kTM + kTN) * kProjStride;        // A tile, then W tile
    static constexpr int kEpiStride = kTN + 8;                             // staged output row, elements
    static constexpr int kEpiRows = 32 * WM;                               // rows per epilogue pass: one row of waves
    static_assert(kEpiRows * kEpiStride <= kOperandElems, "the staging tile fits in the operand tiles");
};

// What bounds it (in-kernel time stamps and probes at B*L = 16384, d_model = 512, bfloat16): not
// the contraction loop.  A loop with this mix of LDS reads, LDS writes, loads and one barrier per
// 32 MFMAs sustains 1.6 PFLOP/s when it runs for thousands of chunks; with d_model = 256..512 a
// tile has only 4..8 chunks, and the first loads of a work-group and its output stores take as
// long as its products (stores alone: 10 of 51 us).  Wave tiles of 4 x 2 MFMA tiles, and a
// variant feeding the rows of A straight from memory into operand registers (W alone in LDS),
// both ended at the same time as this kernel, as did two register sets with two LDS stages; two
// tiles per work-group with the second tile's first loads issued before the first tile's
// epilogue were slower (the registers those loads hold cost the third work-group per compute
// unit).  So the simple form is kept, with up to three work-groups per compute unit to overlap
// the phases.
template <int WM, int WN>
__global__ __launch_bounds__(256, 2)
void project_kernel(const ProjectParams P)
{
    using T = bf16_t;
    using LY = ProjLayout<WM, WN>;
    typedef unsigned int Vec __attribute__((ext_vector_type(4)));         // (native vectors: arrays of them stay in registers)
    constexpr int S = kProjStride, CH = kProjChunk;
    constexpr int TM = LY::kTM, TN = LY::kTN;
    constexpr int VPR = CH * 2 / 16;                       // 16-byte vectors per tile row: 8
    constexpr int NA = TM / 32, NW = TN / 32;              // vectors per thread and chunk: rows of A, rows of W
    static_assert(256 / VPR == 32, "32 tile rows per pass of the work-group");
    __shared__ __attribute__((aligned(16))) T smem[LY::kOperandElems];
    __shared__ __attribute__((aligned(16))) float sBias[TN];
    T* const sA = smem;
    T* const sW = smem + TM * S;

    PSA_TS(0);
    PSA_TS_WALL(5);
    // Work-groups are dealt to the 8 XCDs (each with an L2 of its own) in turn by their linear id.
    // All tiles that share a block of rows of A (every column tile of every matrix) are given to ONE
    // XCD in consecutive slots, so that block of A comes from memory once and from that L2 afterwards.
    const int n_nt = (P.N + TN - 1) / TN, n_mt = (P.M + TM - 1) / TM;
    const int per_rows = n_nt * P.n_mat;
    const int slot = blockIdx.x >> 3;
    const int mt = (slot / per_rows) * 8 + (blockIdx.x & 7);
    if (mt >= n_mt) return;
    const int inner = slot % per_rows;
    const int which = inner / n_nt;
    const T* A = static_cast<const T*>(P.A);
    // (selected with conditionals: indexing the argument arrays by a run-time value would move them to scratch)
    const T* W = static_cast<const T*>(which == 0 ? P.W[0] : (which == 1 ? P.W[1] : P.W[2]));
    const T* bias = static_cast<const T*>(which == 0 ? P.bias[0] : (which == 1 ? P.bias[1] : P.bias[2]));
    T* C = static_cast<T*>(which == 0 ? P.C[0] : (which == 1 ? P.C[1] : P.C[2]));
    const int n0 = (inner % n_nt) * TN, m0 = mt * TM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int n_kc = P.Kd / CH;

    // this thread's share of the tiles: vector `col` of rows row0 + 32 j
    const int row0 = tid / VPR, col = tid % VPR;
    const T* a_ptr[NA];
    const T* w_ptr[NW];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        int m = m0 + row0 + 32 * j;
        m = m < P.M ? m : P.M - 1;                         // clamped: rows beyond M are never stored
        size_t off;
        if (P.a_heads) { const int b = m / P.L, l = m - b * P.L; off = ((size_t)b * P.H * P.L + l) * kD; }
        else off = (size_t)m * P.Kd;
        a_ptr[j] = A + off + col * 8;
    }
#pragma unroll
    for (int j = 0; j < NW; ++j) {
        const int nr = n0 + row0 + 32 * j;
        w_ptr[j] = W + (size_t)(nr < P.N ? nr : P.N - 1) * P.Kd + col * 8;   // clamped likewise
    }
    // contraction element k0 (a multiple of the chunk, so inside one head) of a row of A
    const size_t head_stride = (size_t)P.L * kD;

    Vec ra[NA], rw[NW];
    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto fetch = [&](int kc) {
        const int k0 = kc * CH;
        const size_t ka = P.a_heads ? (size_t)(k0 >> 6) * head_stride + (k0 & 63) : (size_t)k0;
#pragma unroll
        for (int j = 0; j < NA; ++j) ra[j] = *reinterpret_cast<const Vec*>(a_ptr[j] + ka);
#pragma unroll
        for (int j = 0; j < NW; ++j) rw[j] = *reinterpret_cast<const Vec*>(w_ptr[j] + k0);
    };

    // the tile's bias values go to LDS once (an unconditional, clamped load; W stands in for a missing bias)
    T bias_raw;
    {
        const int nb = n0 + (tid & (TN - 1));
        bias_raw = (bias ? bias : W)[nb < P.N ? nb : P.N - 1];
    }
    fetch(0);
    if (tid < TN) {
        sBias[tid] = (bias && n0 + tid < P.N) ? bf16_lo((uint32_t)bias_raw.x) : 0.f;
    }
    for (int kc = 0; kc < n_kc; ++kc) {
        if (kc < 2) PSA_TS(1 + kc);
        __syncthreads();                                  // the previous chunk's reads of LDS are done
        {
            T* sa = sA + row0 * S + col * 8;
            T* sw = sW + row0 * S + col * 8;
#pragma unroll
            for (int j = 0; j < NA; ++j) *reinterpret_cast<Vec*>(sa + 32 * j * S) = ra[j];
#pragma unroll
            for (int j = 0; j < NW; ++j) *reinterpret_cast<Vec*>(sw + 32 * j * S) = rw[j];
        }
        __syncthreads();
        if (kc + 1 < n_kc) fetch(kc + 1);                 // travels during the products
        __builtin_amdgcn_sched_barrier(0);                // (keeps the loads above them)
        const T* ar = sA + (wm * 32 * WM + c) * S;
        const T* wr = sW + (wn * 32 * WN + c) * S;
#pragma unroll
        for (int kk = 0; kk < CH / 16; ++kk) {
            bf16x8 a[WM], b[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i)
                a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(ar + i * 32 * S + kk * 16 + 8 * h));
#pragma unroll
            for (int j = 0; j < WN; ++j)
                b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wr + j * 32 * S + kk * 16 + 8 * h));
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        }
    }
    PSA_TS(3);

    // ---- epilogue.  The products were taken as C^T = W A^T (W rows on the MFMA row axis), so a
    // lane owns ONE row m of C and, per register quad, four consecutive columns n.  Bias is added
    // and the value rounded to the storage type in registers; the tile then goes through LDS
    // (reusing the operand tiles), one row of waves at a time, so that every store instruction
    // writes whole 128-byte lines, either row-major or into the head-split layout.
    constexpr int EPV = 8;                                // elements per 16-byte vector
    constexpr int ES = LY::kEpiStride;
    constexpr int VROW = TN / EPV;                        // vectors per staged row
    constexpr int RPP = 256 / VROW;                       // rows per pass of the work-group
    float4 bb[WN][4];                                     // this lane's bias values
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) bb[j][q] = *reinterpret_cast<const float4*>(sBias + wn * 32 * WN + j * 32 + 8 * q + 4 * h);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        __syncthreads();                                  // the operand tiles (or the previous pass) are no longer read
        if (wm == p) {
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int nt = wn * 32 * WN + j * 32 + 8 * q + 4 * h;    // first of four consecutive tile columns
                        const float v0 = acc[i][j][4 * q + 0] + bb[j][q].x, v1 = acc[i][j][4 * q + 1] + bb[j][q].y;
                        const float v2 = acc[i][j][4 * q + 2] + bb[j][q].z, v3 = acc[i][j][4 * q + 3] + bb[j][q].w;
                        T* dst = smem + (i * 32 + c) * ES + nt;
                        *reinterpret_cast<uint2*>(dst) = make_uint2(cvt_pk_bf16(v0, v1), cvt_pk_bf16(v2, v3));
                    }
        }
        __syncthreads();
        const int vec = tid % VROW;
        const int n = n0 + vec * EPV;                     // N is a multiple of 64: a vector is inside or outside
#pragma unroll
        for (int rp = 0; rp < LY::kEpiRows / RPP; ++rp) {
            const int row = rp * RPP + tid / VROW;
            const int m = m0 + p * LY::kEpiRows + row;
            const Vec v = *reinterpret_cast<const Vec*>(smem + row * ES + vec * EPV);
            if (m < P.M && n < P.N) {
                size_t off;
                if (P.c_heads) {
                    const int b = m / P.L, l = m - b * P.L;
                    off = (((size_t)b * P.H + (n >> 6)) * P.L + l) * kD + (n & 63);
                } else {
                    off = (size_t)m * P.N + n;
                }
                *reinterpret_cast<Vec*>(C + off) = v;
            }
        }
    }
    PSA_TS(4);
    PSA_TS_WALL(6);
}

// float32 tensors on the bfloat16 matrix cores.  A float32 value is the exact sum of three
// bfloat16 values up to 2^-27 of its size (hi = bf16(x), mid = bf16(x - hi), lo = bf16(x - hi - mid);
// the differences are exact in float32), so a product a * w is, to 2^-25 relative, the sum of the six
// bfloat16 products hi*hi, hi*mid, mid*hi, mid*mid, hi*lo, lo*hi, each exact in the float32
// accumulator of the MFMA: the accuracy of a float32 MFMA contraction (same accumulator, same number
// of additions per term up to the factor 6) at 16/6 times its rate, since a bfloat16 MFMA covers 16
// contraction elements in half the cycles a float32 MFMA needs for 2.  The operands are split once,
// on their way from registers into LDS (three planes of bfloat16 per tile), so the split costs a few
// VALU instructions per loaded element.  The rest is project_kernel: 128 x (64 WN) tiles, 2 x WN
// MFMA tiles per wave, C^T = W A^T, chunks of 32 elements, the same epilogue.
template <int WM, int WN>
struct SplitLayout {
    static constexpr int kTM = 64 * WM, kTN = 64 * WN;
    static constexpr int kRow = 40;                                        // bfloat16 per LDS row: 32 + 8 pad (80 bytes)
    static constexpr int kPlane = (kTM + kTN) * kRow;                      // elements of one plane: A rows, then W rows
    static constexpr int kEpiStride = kTN + 4;                             // staged output row, floats
    static constexpr int kEpiRows = 32 * WM;                               // one row of waves per pass
    static_assert(kEpiRows * kEpiStride * 4 <= 3 * kPlane * 2, "the staging tile fits in the operand planes");
};

template <int WM, int WN>
__global__ __launch_bounds__(256, 2)
void project_split_kernel(const ProjectParams P)
{
    using LY = SplitLayout<WM, WN>;
    typedef float Vec __attribute__((ext_vector_type(4)));
    constexpr int CH = 32, S = LY::kRow, TM = LY::kTM, TN = LY::kTN;
    constexpr int NA = TM / 32, NW = TN / 32;              // float4 vectors per thread and chunk: rows of A, rows of W
    __shared__ __attribute__((aligned(16))) uint16_t smem[3 * LY::kPlane];
    __shared__ __attribute__((aligned(16))) float sBias[TN];

    PSA_TS(0);
    PSA_TS_WALL(5);
    // (the same dealing of tiles to XCDs as in project_kernel)
    const int n_nt = (P.N + TN - 1) / TN, n_mt = (P.M + TM - 1) / TM;
    const int per_rows = n_nt * P.n_mat;
    const int slot = blockIdx.x >> 3;
    const int mt = (slot / per_rows) * 8 + (blockIdx.x & 7);
    if (mt >= n_mt) return;
    const int inner = slot % per_rows;
    const int which = inner / n_nt;
    const float* A = static_cast<const float*>(P.A);
    const float* W = static_cast<const float*>(which == 0 ? P.W[0] : (which == 1 ? P.W[1] : P.W[2]));
    const float* bias = static_cast<const float*>(which == 0 ? P.bias[0] : (which == 1 ? P.bias[1] : P.bias[2]));
    float* C = static_cast<float*>(which == 0 ? P.C[0] : (which == 1 ? P.C[1] : P.C[2]));
    const int n0 = (inner % n_nt) * TN, m0 = mt * TM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;
    const int n_kc = P.Kd / CH;

    // this thread's share of the tiles: float4 `col` of rows row0 + 32 j
    const int row0 = tid >> 3, col = tid & 7;
    const float* a_ptr[NA];
    const float* w_ptr[NW];
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        int m = m0 + row0 + 32 * j;
        m = m < P.M ? m : P.M - 1;                         // clamped: rows beyond M are never stored
        size_t off;
        if (P.a_heads) { const int b = m / P.L, l = m - b * P.L; off = ((size_t)b * P.H * P.L + l) * kD; }
        else off = (size_t)m * P.Kd;
        a_ptr[j] = A + off + col * 4;
    }
#pragma unroll
    for (int j = 0; j < NW; ++j) {
        const int nr = n0 + row0 + 32 * j;
        w_ptr[j] = W + (size_t)(nr < P.N ? nr : P.N - 1) * P.Kd + col * 4;                     // clamped likewise
    }
    const size_t head_stride = (size_t)P.L * kD;

    Vec ra[NA], rw[NW];
    floatx16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto fetch = [&](int kc) {
        const int k0 = kc * CH;
        const size_t ka = P.a_heads ? (size_t)(k0 >> 6) * head_stride + (k0 & 63) : (size_t)k0;
#pragma unroll
        for (int j = 0; j < NA; ++j) ra[j] = *reinterpret_cast<const Vec*>(a_ptr[j] + ka);
#pragma unroll
        for (int j = 0; j < NW; ++j) rw[j] = *reinterpret_cast<const Vec*>(w_ptr[j] + k0);
    };
    // four floats -> their hi, mid and lo bfloat16 parts, 8 bytes into each plane
    auto put_split = [&](uint16_t* dst, Vec x) {
        const uint32_t h0 = cvt_pk_bf16(x.x, x.y), h1 = cvt_pk_bf16(x.z, x.w);
        float r0 = x.x - bf16_lo(h0), r1 = x.y - bf16_hi(h0), r2 = x.z - bf16_lo(h1), r3 = x.w - bf16_hi(h1);
        const uint32_t m0_ = cvt_pk_bf16(r0, r1), m1_ = cvt_pk_bf16(r2, r3);
        r0 -= bf16_lo(m0_); r1 -= bf16_hi(m0_); r2 -= bf16_lo(m1_); r3 -= bf16_hi(m1_);
        const uint32_t l0 = cvt_pk_bf16(r0, r1), l1 = cvt_pk_bf16(r2, r3);
        *reinterpret_cast<uint2*>(dst) = make_uint2(h0, h1);
        *reinterpret_cast<uint2*>(dst + LY::kPlane) = make_uint2(m0_, m1_);
        *reinterpret_cast<uint2*>(dst + 2 * LY::kPlane) = make_uint2(l0, l1);
    };

    float bias_raw;
    {
        const int nb = n0 + (tid & (TN - 1));
        bias_raw = (bias ? bias : W)[nb < P.N ? nb : P.N - 1];    // unconditional, clamped; W stands in for a missing bias
    }
    fetch(0);
    if (tid < TN) sBias[tid] = (bias && n0 + tid < P.N) ? bias_raw : 0.f;
    for (int kc = 0; kc < n_kc; ++kc) {
        if (kc < 2) PSA_TS(1 + kc);
        __syncthreads();                                  // the previous chunk's reads of LDS are done
        {
            uint16_t* sa = smem + row0 * S + col * 4;
            uint16_t* sw = smem + (TM + row0) * S + col * 4;
#pragma unroll
            for (int j = 0; j < NA; ++j) put_split(sa + 32 * j * S, ra[j]);
#pragma unroll
            for (int j = 0; j < NW; ++j) put_split(sw + 32 * j * S, rw[j]);
        }
        __syncthreads();
        if (kc + 1 < n_kc) fetch(kc + 1);                 // travels during the products
        __builtin_amdgcn_sched_barrier(0);                // (keeps the loads above them)
        const uint16_t* ar = smem + (wm * 32 * WM + c) * S + 8 * h;
        const uint16_t* wr = smem + (TM + wn * 32 * WN + c) * S + 8 * h;
#pragma unroll
        for (int kk = 0; kk < CH / 16; ++kk) {
            bf16x8 a[3][WM], b[3][WN];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    a[pl][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(ar + pl * LY::kPlane + i * 32 * S + kk * 16));
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    b[pl][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(wr + pl * LY::kPlane + j * 32 * S + kk * 16));
            }
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    // smallest terms first
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[2][j], a[0][i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[0][j], a[2][i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[1][j], a[1][i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[1][j], a[0][i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[0][j], a[1][i], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[0][j], a[0][i], acc[i][j], 0, 0, 0);
                }
        }
    }
    PSA_TS(3);

    // ---- epilogue (as in project_kernel): bias in registers, the tile through LDS one row of
    // waves at a time, stores of whole 128-byte lines
    constexpr int ES = LY::kEpiStride;
    constexpr int VROW = TN / 4;                          // float4 vectors per staged row
    constexpr int RPP = 256 / VROW;                       // rows per pass of the work-group
    float* const stage = reinterpret_cast<float*>(smem);
    float4 bb[WN][4];
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) bb[j][q] = *reinterpret_cast<const float4*>(sBias + wn * 32 * WN + j * 32 + 8 * q + 4 * h);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        __syncthreads();                                  // the operand planes (or the previous pass) are no longer read
        if (wm == p) {
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int nt = wn * 32 * WN + j * 32 + 8 * q + 4 * h;    // first of four consecutive tile columns
                        *reinterpret_cast<float4*>(stage + (i * 32 + c) * ES + nt) =
                            make_float4(acc[i][j][4 * q + 0] + bb[j][q].x, acc[i][j][4 * q + 1] + bb[j][q].y,
                                        acc[i][j][4 * q + 2] + bb[j][q].z, acc[i][j][4 * q + 3] + bb[j][q].w);
                    }
        }
        __syncthreads();
        const int vec = tid % VROW;
        const int n = n0 + vec * 4;                       // N is a multiple of 64: a vector is inside or outside
#pragma unroll
        for (int rp = 0; rp < LY::kEpiRows / RPP; ++rp) {
            const int row = rp * RPP + tid / VROW;
            const int m = m0 + p * LY::kEpiRows + row;
            const Vec v = *reinterpret_cast<const Vec*>(stage + row * ES + vec * 4);
            if (m < P.M && n < P.N) {
                size_t off;
                if (P.c_heads) {
                    const int b = m / P.L, l = m - b * P.L;
                    off = (((size_t)b * P.H + (n >> 6)) * P.L + l) * kD + (n & 63);
                } else {
                    off = (size_t)m * P.N + n;
                }
                *reinterpret_cast<Vec*>(C + off) = v;
            }
        }
    }
    PSA_TS(4);
    PSA_TS_WALL(6);
}

template <int WM, int WN>
static hipError_t launch_project_split(const ProjectParams& P, hipStream_t stream)
{
    using LY = SplitLayout<WM, WN>;
    const int n_nt = (P.N + LY::kTN - 1) / LY::kTN, n_mt = (P.M + LY::kTM - 1) / LY::kTM;
    hipLaunchKernelGGL((project_split_kernel<WM, WN>), dim3(8 * ((n_mt + 7) / 8) * n_nt * P.n_mat), dim3(256), 0, stream, P);
    return hipGetLastError();
}

template <int WM, int WN>
static hipError_t launch_project_as(const ProjectParams& P, hipStream_t stream)
{
    using LY = ProjLayout<WM, WN>;
    const int n_nt = (P.N + LY::kTN - 1) / LY::kTN, n_mt = (P.M + LY::kTM - 1) / LY::kTM;
    hipLaunchKernelGGL((project_kernel<WM, WN>), dim3(8 * ((n_mt + 7) / 8) * n_nt * P.n_mat), dim3(256), 0, stream, P);
    return hipGetLastError();
}

static hipError_t launch_project(const ProjectParams& P0, int n_mat, int dtype, hipStream_t stream)
{
    ProjectParams P = P0;
    P.n_mat = n_mat;
    // 128 x 128 tiles when they give every compute unit at least two work-groups, else 128 x 64
    const long wg128 = (long)((P.N + 127) / 128) * ((P.M + 127) / 128) * n_mat;
    if (dtype == PSA_F32) {
        // (128 x 64 tiles give 2 wg128 work-groups, 64 x 64 tiles 4 wg128)
        if (wg128 >= 512) return launch_project_split<2, 2>(P, stream);
        return 2 * wg128 >= 512 ? launch_project_split<2, 1>(P, stream) : launch_project_split<1, 1>(P, stream);
    }
    return wg128 >= 512 ? launch_project_as<2, 2>(P, stream) : launch_project_as<2, 1>(P, stream);
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

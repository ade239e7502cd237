// The exact sparsity measure of Eq. 10 for every query, as a diagnostic of what
// the sampled measure of stage a1 approximates:
//     M_i = ln sum_j exp(q_i . k_j / sqrt(d)) - (1/n) sum_j q_i . k_j / sqrt(d)
// over the n valid keys of the item.  A dense pass of the first product of
// attention on the matrix cores (the tile code of the attend stage, queries on
// the column axis, so a lane owns one query), with a running log-sum-exp and a
// running sum of the scores instead of the second product.
#include "psa_tile.h"

namespace psa {

constexpr double kLn2 = 0.693147180559945309417;

// float32 tensors: float64 MFMA and float64 log-sum-exp.  8 waves of 16 queries.
__global__ __launch_bounds__(512)
void exact_measure_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                              const int* __restrict__ lengths, float* __restrict__ M, int H, int L)
{
    const int head = blockIdx.y;
    const int n = valid_len(lengths, head / H, L);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int q = blockIdx.x * 128 + wave * 16 + c;
    const float* Qh = Q + (size_t)head * L * kD;
    const float* Kh = K + (size_t)head * L * kD;

    F32Tile tile;
    tile.load_q(Qh, q, q < n, g);
    // this lane's keys only (4r + g of every 16): running maximum and sum of 2^(t - max)
    // in base 2, and the plain sum of the scores; the four lanes of a query are combined at the end
    double m = -INFINITY, l = 0.0, ssum = 0.0;
    float4 knext[2][4];
    F32Tile::load_k_into(knext, Kh, 0, n, c, g);
    for (int j0 = 0; j0 < n; j0 += kTile) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int v = 0; v < 4; ++v) tile.kreg[sb][v] = knext[sb][v];
        F32Tile::load_k_into(knext, Kh, j0 + kTile, n, c, g);          // clamped: in flight during the step
        doublex4 s[2];
        tile.scores(s);
        double t[2][4], tmax = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool ok = (j0 + 16 * sb + 4 * r + g) < n;
                t[sb][r] = ok ? s[sb][r] * kScaleLog2eD : -INFINITY;
                ssum += ok ? s[sb][r] : 0.0;
                tmax = fmax(tmax, t[sb][r]);
            }
        if (tmax > -INFINITY) {                                 // this lane saw a valid key in the tile
            const double m_new = fmax(m, tmax);
            double acc = l * exp2_f64(m - m_new);
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc += exp2_f64(t[sb][r] - m_new);
            l = acc;
            m = m_new;
        }
    }
    // combine the four lanes g of the query (lanes c, c+16, c+32, c+48), in a fixed order
    double mx = m;
    mx = fmax(mx, __shfl_xor(mx, 16, 64));
    mx = fmax(mx, __shfl_xor(mx, 32, 64));
    double lw = (m == -INFINITY) ? 0.0 : l * exp2_f64(m - mx);
    lw += __shfl_xor(lw, 16, 64);
    lw += __shfl_xor(lw, 32, 64);
    ssum += __shfl_xor(ssum, 16, 64);
    ssum += __shfl_xor(ssum, 32, 64);
    if (g == 0 && q < L) {
        float out = 0.f;
        if (q < n) out = (float)(kLn2 * (mx + log2(lw)) - ssum * 0.125 / (double)n);
        M[(size_t)head * L + q] = out;
    }
}

// bfloat16 tensors: bf16 MFMA with float32 accumulation (the products are exact),
// log-sum-exp in float32, sum of scores carried in float64.  4 waves of 32 queries.
__global__ __launch_bounds__(256)
void exact_measure_bf16_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K,
                               const int* __restrict__ lengths, float* __restrict__ M, int H, int L)
{
    const int head = blockIdx.y;
    const int n = valid_len(lengths, head / H, L);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int q = blockIdx.x * 128 + wave * 32 + c;
    const bf16_t* Qh = Q + (size_t)head * L * kD;
    const bf16_t* Kh = K + (size_t)head * L * kD;

    Bf16Tile<1> tile;
    tile.load_q(0, Qh, q, q < n, h);
    float m = -INFINITY, l = 0.f;
    double ssum = 0.0;
    uint4 knext[4];
    Bf16Tile<1>::load_k_operand(knext, Kh, 0, n, c, h);
    for (int j0 = 0; j0 < n; j0 += kTile) {
        uint4 ka[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) ka[kk] = knext[kk];
        Bf16Tile<1>::load_k_operand(knext, Kh, j0 + kTile, n, c, h);   // clamped: in flight during the step
        const floatx16 s = tile.scores(ka, 0);
        float t[16], tmax = -INFINITY, tsum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = (j0 + 8 * (r >> 2) + 4 * h + (r & 3)) < n;
            t[r] = ok ? s[r] * kScaleLog2e : -INFINITY;
            tsum += ok ? s[r] : 0.f;
            tmax = fmaxf(tmax, t[r]);
        }
        ssum += (double)tsum;
        if (tmax > -INFINITY) {
            const float m_new = fmaxf(m, tmax);
            float acc = l * fast_exp2(m - m_new);
#pragma unroll
            for (int r = 0; r < 16; ++r) acc += fast_exp2(t[r] - m_new);
            l = acc;
            m = m_new;
        }
    }
    // combine the two half-waves of the query
    const float mo = swap_half(m);
    const float mx = fmaxf(m, mo);
    float lw = (m == -INFINITY) ? 0.f : l * fast_exp2(m - mx);
    lw += swap_half(lw);
    ssum += __shfl_xor(ssum, 32, 64);
    if (h == 0 && q < L) {
        float out = 0.f;
        if (q < n) out = (float)(kLn2 * ((double)mx + log2((double)lw)) - ssum * 0.125 / (double)n);
        M[(size_t)head * L + q] = out;
    }
}

}  // namespace psa

extern "C" int probsparse_exact_measure(const void* Q, const void* K, const int32_t* lengths, float* M_out,
                                        const psa_shape_t* shape, void* stream)
{
    using namespace psa;
    if (!Q || !K || !M_out || !shape) return PSA_ERR_NULL;
    if (shape->dtype != PSA_F32 && shape->dtype != PSA_BF16) return PSA_ERR_DTYPE;
    if (shape->B < 1 || shape->H < 1 || shape->L_Q < 1 || shape->L_K < 1 || shape->D != kD ||
        shape->L_Q != shape->L_K || (int64_t)shape->B * shape->H > 65535 || shape->L_K > (1 << 22)) return PSA_ERR_SHAPE;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K);
    if ((bits & 15) || (reinterpret_cast<uintptr_t>(M_out) & 3) || (reinterpret_cast<uintptr_t>(lengths) & 3)) return PSA_ERR_ALIGN;
    const int L = shape->L_K;
    const dim3 grid((L + 127) / 128, shape->B * shape->H);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (shape->dtype == PSA_F32)
        hipLaunchKernelGGL(exact_measure_f32_kernel, grid, dim3(512), 0, st, (const float*)Q, (const float*)K, lengths,
                           M_out, shape->H, L);
    else
        hipLaunchKernelGGL(exact_measure_bf16_kernel, grid, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)K, lengths,
                           M_out, shape->H, L);
    return hipGetLastError() == hipSuccess ? PSA_OK : PSA_ERR_HIP;
}

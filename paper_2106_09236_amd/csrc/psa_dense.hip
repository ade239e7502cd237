// Dense attention baseline: softmax(Q K^T / sqrt(d)) V over the valid keys of
// every query (Eq. 6), padded query rows zero.  It is the comparison point for
// the prob-sparse path and uses the same per-wave tile arithmetic (psa_tile.h),
// hence the same precision: float64 matrix cores for float32 tensors, bfloat16
// matrix cores with float32 accumulation for bfloat16 tensors.  A wave owns a
// tile of queries and walks all key tiles of its head with online softmax; no
// key split, no workspace.
#include "psa_tile.h"

namespace psa {

// ---- float32 tensors: 8 waves, 16 queries each; K and V straight from global
// memory (the 8 waves read the same tiles, served by L1), next K tile prefetched.
// ALLFULL: no lengths and L a multiple of 32, so every key tile is wholly valid: loads without clamps,
// steps without masks, as in the prob-sparse attend kernel (the baseline gets the same care).
template <bool ALLFULL>
__global__ __launch_bounds__(512)
void dense_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
                      const int* __restrict__ lengths, float* __restrict__ out, int H, int L)
{
    const int head = blockIdx.y;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int q = blockIdx.x * 128 + wave * 16 + c;
    const float* Qh = Q + (size_t)head * L * kD;
    const float* Kh = K + (size_t)head * L * kD;
    const float* Vh = V + (size_t)head * L * kD;
    float* oh = out + (size_t)head * L * kD;

    F32Tile tile;
    tile.init();
    tile.load_q(Qh, q, q < n, g);
    float4 knext[2][4];
    auto take_next = [&]() {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int v = 0; v < 4; ++v) tile.kreg[sb][v] = knext[sb][v];
    };
    if constexpr (ALLFULL) {
        // n = L >= 32: all tiles but the last prefetch their successor (rows up to j0 + 63 < n), then the last
        F32Tile::load_k_into<true>(knext, Kh, 0, n, c, g);
        int j0 = 0;
        for (; j0 + 2 * kTile <= n; j0 += kTile) {
            take_next();
            F32Tile::load_k_into<true>(knext, Kh, j0 + kTile, n, c, g);
            tile.step<false, true>(Vh, j0, n, c, g);
        }
        take_next();
        tile.step<false, true>(Vh, j0, n, c, g);
    } else {
        F32Tile::load_k_into(knext, Kh, 0, n, c, g);
        for (int j0 = 0; j0 < n; j0 += kTile) {
            take_next();
            F32Tile::load_k_into(knext, Kh, j0 + kTile, n, c, g);
            tile.step(Vh, j0, n, c, g);
        }
    }
    double l_tot = tile.l_run;
    l_tot += __shfl_xor(l_tot, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    if (q < L) {
        const double inv = (q < n && l_tot > 0.0) ? 1.0 / l_tot : 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)          // elements 16r + 4g .. + 3: one 16-byte store
            *reinterpret_cast<float4*>(oh + (size_t)q * kD + F32Tile::elem(0, r, g)) =
                make_float4((float)(tile.oacc[0][r] * inv), (float)(tile.oacc[1][r] * inv),
                            (float)(tile.oacc[2][r] * inv), (float)(tile.oacc[3][r] * inv));
    }
}

// ---- bfloat16 tensors: 4 waves, 32 queries each; the work-group stages each
// 32-key tile of K and V once in LDS (double-buffered, one barrier per tile).
__global__ __launch_bounds__(256)
void dense_bf16_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                       const int* __restrict__ lengths, bf16_t* __restrict__ out, int H, int L)
{
    __shared__ __attribute__((aligned(16))) uint16_t sKV[2][2][kTile * kB16Stride];   // [buffer][K|V]
    const int head = blockIdx.y;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int q = blockIdx.x * 128 + wave * 32 + c;
    const bf16_t* Qh = Q + (size_t)head * L * kD;
    const bf16_t* Kh = K + (size_t)head * L * kD;
    const bf16_t* Vh = V + (size_t)head * L * kD;
    bf16_t* oh = out + (size_t)head * L * kD;

    Bf16Tile<1> tile;
    tile.init();
    tile.load_q(0, Qh, q, q < n, h);

    // thread t stages 16 bytes of row t / 8 of the tile
    const int srow = tid >> 3, scol = tid & 7;
    auto fetch = [&](int j0, uint4& xk, uint4& xv) {
        const int j = j0 + srow;
        const bool ok = j < n;
        const size_t ro = (size_t)(ok ? j : last_row(n)) * kD;
        xk = reinterpret_cast<const uint4*>(Kh + ro)[scol];
        xv = reinterpret_cast<const uint4*>(Vh + ro)[scol];
        if (!ok) { xk = make_uint4(0u, 0u, 0u, 0u); xv = xk; }
    };
    auto put = [&](int buf, const uint4& xk, const uint4& xv) {
        *reinterpret_cast<uint4*>(&sKV[buf][0][srow * kB16Stride + scol * 8]) = xk;
        *reinterpret_cast<uint4*>(&sKV[buf][1][srow * kB16Stride + scol * 8]) = xv;
    };
    uint4 xk, xv;
    fetch(0, xk, xv);
    put(0, xk, xv);
    __syncthreads();
    int buf = 0;
    for (int j0 = 0; j0 < n; j0 += kTile) {
        fetch(j0 + kTile, xk, xv);                           // next tile, in flight during the step
        tile.step(sKV[buf][0], sKV[buf][1], j0, n, c, h);
        put(buf ^ 1, xk, xv);
        __syncthreads();
        buf ^= 1;
    }
    const float l_tot = tile.l_run[0] + swap_half(tile.l_run[0]);
    if (q < L) {
        const float inv = (q < n && l_tot > 0.f) ? 1.f / l_tot : 0.f;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int e = 32 * dt + 8 * r4 + 4 * h;
                const uint2 pk = make_uint2(pack_bf16(tile.oacc[0][dt][4 * r4 + 0] * inv, tile.oacc[0][dt][4 * r4 + 1] * inv),
                                            pack_bf16(tile.oacc[0][dt][4 * r4 + 2] * inv, tile.oacc[0][dt][4 * r4 + 3] * inv));
                *reinterpret_cast<uint2*>(oh + (size_t)q * kD + e) = pk;
            }
    }
}

}  // namespace psa

extern "C" {

size_t dense_attn_workspace_bytes(const psa_shape_t*) { return 0; }

int dense_attn_fwd(const void* Q, const void* K, const void* V, const int32_t* lengths, void* out,
                   const psa_shape_t* shape, void* /*workspace*/, size_t /*workspace_bytes*/, void* stream)
{
    using namespace psa;
    if (!Q || !K || !V || !out || !shape) return PSA_ERR_NULL;
    if (shape->dtype != PSA_F32 && shape->dtype != PSA_BF16) return PSA_ERR_DTYPE;
    if (shape->B < 1 || shape->H < 1 || shape->L_Q < 1 || shape->L_K < 1 || shape->D != kD ||
        shape->L_Q != shape->L_K || (int64_t)shape->B * shape->H > 65535 || shape->L_K > (1 << 22)) return PSA_ERR_SHAPE;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K) |
                           reinterpret_cast<uintptr_t>(V) | reinterpret_cast<uintptr_t>(out);
    if ((bits & 15) || (reinterpret_cast<uintptr_t>(lengths) & 3)) return PSA_ERR_ALIGN;
    const int L = shape->L_K, BH = shape->B * shape->H;
    dim3 grid((L + 127) / 128, BH);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (shape->dtype == PSA_F32 && lengths == nullptr && L % kTile == 0)
        hipLaunchKernelGGL(dense_f32_kernel<true>, grid, dim3(512), 0, st, (const float*)Q, (const float*)K, (const float*)V,
                           lengths, (float*)out, shape->H, L);
    else if (shape->dtype == PSA_F32)
        hipLaunchKernelGGL(dense_f32_kernel<false>, grid, dim3(512), 0, st, (const float*)Q, (const float*)K, (const float*)V,
                           lengths, (float*)out, shape->H, L);
    else
        hipLaunchKernelGGL(dense_bf16_kernel, grid, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V,
                           lengths, (bf16_t*)out, shape->H, L);
    return hipGetLastError() == hipSuccess ? PSA_OK : PSA_ERR_HIP;
}

}  // extern "C"

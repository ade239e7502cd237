// Stage a2 as a kernel of its own: one work-group per (batch, head).  Used when
// the measure stage could not hand sorted candidate lists to the attend stage
// (heads whose K does not fit in LDS).  It also turns the per-chunk float64 column
// sums of V into the mean of the valid V rows.
#include <type_traits>

#include "psa_select.h"

namespace psa {

template <int NT, int KPT>
__global__ __launch_bounds__(NT)
void select_kernel(const float* __restrict__ M, const int* __restrict__ lengths,
                   const double* __restrict__ vpart, float* __restrict__ mu,
                   int* __restrict__ sel, int* __restrict__ ucount,
                   int H, int L, int u_max, int n_chunk, double c)
{
    __shared__ typename std::conditional<(KPT > 0), SelectScratch<NT>, StreamSelectScratch<NT>>::type sc;
    __shared__ double red[NT / 64][kD];
    const int head = blockIdx.x;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, wave = tid >> 6;
    const int u = n_selected(c, n, u_max);
    if (tid == 0 && head % H == 0) ucount[b] = u;

    // mean of the valid V rows from the per-chunk column sums (fixed order)
    auto mean_of_v = [&]() {
        const int e = tid & 63;
        double s = 0.0;
        // eight loads in flight at a time (clamped, unconditional), added in chunk order
        for (int c0 = wave; c0 < n_chunk; c0 += 8 * (NT / 64)) {
            double v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int ch = c0 + k * (NT / 64);
                v[k] = vpart[((size_t)head * n_chunk + (ch < n_chunk ? ch : n_chunk - 1)) * kD + e];
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) s += (c0 + k * (NT / 64) < n_chunk) ? v[k] : 0.0;
        }
        red[wave][e] = s;
        __syncthreads();
        if (tid < kD) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) t += red[w][tid];
            mu[(size_t)head * kD + tid] = n > 0 ? (float)(t / (double)n) : 0.f;
        }
    };
    if constexpr (KPT > 0) {
        block_select<NT, KPT>(M + (size_t)head * L, n, u, u_max, sel + (size_t)head * u_max, sc, mean_of_v);
    } else {
        mean_of_v();
        block_select_stream<NT, 0>(M + (size_t)head * L, n, u, u_max, sel + (size_t)head * u_max, sc);
    }
}

hipError_t launch_select(const Plan& p, const Args& a, const Scratch& w)
{
#define PSA_SELECT_ARGS w.M, a.lengths, w.vpart, w.mu, w.sel, w.u, p.H, p.L, p.u_max, p.n_chunk, a.c
    if (p.L <= 2048)       hipLaunchKernelGGL((select_kernel<1024, 2>),  dim3(p.BH), dim3(1024), 0, a.stream, PSA_SELECT_ARGS);
    else if (p.L <= 16384) hipLaunchKernelGGL((select_kernel<1024, 16>), dim3(p.BH), dim3(1024), 0, a.stream, PSA_SELECT_ARGS);
    else                   hipLaunchKernelGGL((select_kernel<1024, 0>),  dim3(p.BH), dim3(1024), 0, a.stream, PSA_SELECT_ARGS);
#undef PSA_SELECT_ARGS
    return hipGetLastError();
}

}  // namespace psa

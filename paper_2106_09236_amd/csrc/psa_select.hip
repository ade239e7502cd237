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
                   int H, int L, int u_max, int n_chunk, URule urule)
{
    __shared__ typename std::conditional<(KPT > 0), SelectScratch<NT>, StreamSelectScratch<NT>>::type sc;
    __shared__ double red[NT / 64][kD];
    const int head = blockIdx.x;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, wave = tid >> 6;
    const int u = n_selected(urule, n, u_max);
    if (tid == 0 && head % H == 0) ucount[b] = u;

    // mean of the valid V rows from the per-chunk column sums (fixed order)
    auto mean_of_v = [&]() {
        const int e = tid & 63;
        double s = 0.0;
        // NB loads in flight at a time (clamped, unconditional), added in chunk order
        constexpr int NB = KPT >= 16 ? 16 : 4;            // long heads have hundreds of chunks
        for (int c0 = wave; c0 < n_chunk; c0 += NB * (NT / 64)) {
            double v[NB];
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const int ch = c0 + k * (NT / 64);
                v[k] = vpart[((size_t)head * n_chunk + (ch < n_chunk ? ch : n_chunk - 1)) * kD + e];
            }
#pragma unroll
            for (int k = 0; k < NB; ++k) s += (c0 + k * (NT / 64) < n_chunk) ? v[k] : 0.0;
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
        block_select<NT, KPT>(M + (size_t)head * L, (L & 3) == 0, n, u, u_max, sel + (size_t)head * u_max, sc, mean_of_v);
    } else {
        mean_of_v();
        block_select_stream<NT, 0>(M + (size_t)head * L, n, u, u_max, sel + (size_t)head * u_max, sc);
    }
}

// Caller-given index sets (Sec. 4.4: a layer reuses the index set of the layer
// before it): one work-group per head turns the column sums of V into the mean
// and copies the head's index row into the workspace, keeping only entries that
// are valid queries of the item (anything else becomes -1 and is skipped later).
__global__ __launch_bounds__(256)
void prep_indices_kernel(const int* __restrict__ lengths, const double* __restrict__ vpart, float* __restrict__ mu,
                         const int* __restrict__ sel_in, const int* __restrict__ u_in,
                         int* __restrict__ sel, int* __restrict__ ucount, int H, int L, int u_max, int n_chunk)
{
    __shared__ double red[4][kD];
    const int head = blockIdx.x;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, wave = tid >> 6, e = tid & 63;
    int u = u_in[b];
    u = u < 0 ? 0 : u;
    u = u > u_max ? u_max : u;
    u = u > n ? n : u;
    if (tid == 0 && head % H == 0) ucount[b] = u;
    for (int t = tid; t < u_max; t += 256) {
        const int sv = sel_in[(size_t)head * u_max + t];
        sel[(size_t)head * u_max + t] = (t < u && sv >= 0 && sv < n) ? sv : -1;
    }
    double s = 0.0;
    for (int ch = wave; ch < n_chunk; ch += 4) s += vpart[((size_t)head * n_chunk + ch) * kD + e];
    red[wave][e] = s;
    __syncthreads();
    if (tid < kD) {
        const double t = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
        mu[(size_t)head * kD + tid] = n > 0 ? (float)(t / (double)n) : 0.f;
    }
}

hipError_t launch_prep_indices(const Plan& p, const Args& a, const Scratch& w)
{
    hipLaunchKernelGGL(prep_indices_kernel, dim3(p.BH), dim3(256), 0, a.stream, a.lengths, w.vpart, w.mu,
                       a.given_sel, a.given_u, w.sel, w.u, p.H, p.L, p.u_max, p.n_chunk);
    return hipGetLastError();
}

hipError_t launch_select(const Plan& p, const Args& a, const Scratch& w)
{
#define PSA_SELECT_ARGS w.M, a.lengths, w.vpart, w.mu, w.sel, w.u, p.H, p.L, p.u_max, p.n_chunk, a.urule
    if (p.L <= 2048)       hipLaunchKernelGGL((select_kernel<1024, 2>),  dim3(p.BH), dim3(1024), 0, a.stream, PSA_SELECT_ARGS);
    else if (p.L <= 16384) hipLaunchKernelGGL((select_kernel<1024, 16>), dim3(p.BH), dim3(1024), 0, a.stream, PSA_SELECT_ARGS);
    else                   hipLaunchKernelGGL((select_kernel<1024, 0>),  dim3(p.BH), dim3(1024), 0, a.stream, PSA_SELECT_ARGS);
#undef PSA_SELECT_ARGS
    return hipGetLastError();
}

}  // namespace psa

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

// Long heads, stage a2 in two steps.  Step one, here: a head's measures are cut into up to 8
// segments of consecutive queries; one work-group per segment picks the segment's u best (any
// query among the head's u best is among its own segment's u best), ranks them by decreasing
// measure (ties: lower index first) and hands them on as a sorted list of (order key, query),
// together with the segment's share of the column sums of V.  Step two is the list merge at the
// start of the attend work-groups, the same as for the per-chunk lists of short heads.  This
// spreads the reading of the L measures and of the column sums over 8 times as many CUs as one
// work-group per head would use, and drops the index-ordered emission of the whole head.
__global__ __launch_bounds__(1024)
void select_segments_kernel(const float* __restrict__ M, const int* __restrict__ lengths,
                            const double* __restrict__ vpart, double* __restrict__ vseg, uint2* __restrict__ cand,
                            int H, int L, int u_max, int n_chunk, int n_seg, int seg_len, int cand_len, URule urule)
{
    constexpr int NT = 1024;
    __shared__ SelectScratch<NT> sc;
    __shared__ double red[NT / 64][kD];
    __shared__ int s_sel[kSegCandMax];
    __shared__ unsigned s_key[kSegCandMax];
    const int head = blockIdx.x / n_seg, seg = blockIdx.x - head * n_seg;
    const int n = valid_len(lengths, head / H, L);
    const int tid = threadIdx.x, wave = tid >> 6;
    const int i0 = seg * seg_len;
    int n_here = n - i0;                                   // valid queries of this segment
    n_here = n_here < 0 ? 0 : (n_here > seg_len ? seg_len : n_here);
    const int u = n_selected(urule, n, u_max);
    int u_here = u < n_here ? u : n_here;
    u_here = u_here < cand_len ? u_here : cand_len;        // (cand_len = min(u_max, seg_len): never binds)

    // the segment's share of the column sums of V: its measure chunks in order
    auto part_sum = [&]() {
        const int e = tid & 63;
        const int c_first = i0 / kMeasureQueries;
        int c_end = (i0 + seg_len) / kMeasureQueries;
        c_end = c_end < n_chunk ? c_end : n_chunk;
        const int span = c_end - c_first;                  // <= kSegKeys / kMeasureQueries = 32: two chunks per wave
        double v[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int ch = c_first + wave + k * (NT / 64);
            v[k] = vpart[((size_t)head * n_chunk + (ch < c_end ? ch : c_end - 1)) * kD + e];      // clamped, unconditional
        }
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < 2; ++k) t += (wave + k * (NT / 64) < span) ? v[k] : 0.0;
        red[wave][e] = t;
        __syncthreads();
        if (tid < kD) {
            double tot = 0.0;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) tot += red[w][tid];
            vseg[((size_t)head * n_seg + seg) * kD + tid] = tot;
        }
    };
    const float* Mh = M + (size_t)head * L + i0;
    block_select<NT, 2>(Mh, false, n_here, u_here, cand_len, s_sel, sc, part_sum);
    __syncthreads();
    // s_sel: the kept queries of the segment, ascending.  Rank them by (key descending, index ascending).
    unsigned key = 0u;
    int q = -1;
    if (tid < u_here) { q = s_sel[tid]; key = order_key(Mh[q]); }
    if (tid < kSegCandMax) s_key[tid] = key;
    __syncthreads();
    uint2* co = cand + ((size_t)head * n_seg + seg) * cand_len;
    if (tid < u_here) {
        int rank = 0;
        for (int t = 0; t < u_here; ++t) {
            const unsigned ko = s_key[t];
            rank += (ko > key || (ko == key && t < tid)) ? 1 : 0;
        }
        co[rank] = make_uint2(key, (unsigned)(i0 + q));
    } else if (tid < cand_len) {
        co[tid] = make_uint2(0u, 0xFFFFFFFFu);             // empty slot
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

hipError_t launch_select_segments(const Plan& p, const Args& a, const Scratch& w)
{
    hipLaunchKernelGGL(select_segments_kernel, dim3(p.BH * p.n_seg), dim3(1024), 0, a.stream, w.M, a.lengths, w.vpart,
                       w.vseg, w.cand, p.H, p.L, p.u_max, p.n_chunk, p.n_seg, p.seg_len, p.cand_len, a.urule);
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

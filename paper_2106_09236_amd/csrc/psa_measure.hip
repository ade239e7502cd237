// Stage a1: scores of every query against its sampled keys and the sampled
// sparsity measure  M_i = max_t s_it - (1/#samples) sum_t s_it  (Sec. 3.2, Eq. 11).
//
// This is a gather, not a contraction: each query touches U random key rows of
// its own head.  The work is bound by vector-ALU issue and by the L1 path, so
// the layout minimises instructions per gathered row while keeping every load
// instruction made of whole 64-byte segments:
//   * a QUAD of 4 adjacent lanes owns one query; a wave owns 16 queries;
//   * a key row (256 B f32 / 128 B bf16) is cut into 16-byte chunks, lane s of
//     the quad takes chunks s, s+4, s+8, ... so that one load instruction reads
//     a contiguous 64 B of each of 16 rows;
//   * the quad's lanes keep the matching chunks of the query in registers, the
//     dot product is finished with two DPP quad exchanges, and the sample index
//     travels from the lane that loaded it to the quad with one DPP quad
//     broadcast;
//   * 8 samples (32 or 16 loads per lane) are in flight per round.
#include <type_traits>

#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

template <typename T> struct RowTraits;
template <> struct RowTraits<float>  { static constexpr int kRowBytes = 256, kChunks = 4; };   // 16 B chunks per lane
template <> struct RowTraits<bf16_t> { static constexpr int kRowBytes = 128, kChunks = 2; };

// dot product of the lane's chunks of a query row and a key row
__device__ __forceinline__ float chunk_dot(const float4 (&q)[4], const float4 (&k)[4]) {
    float d = q[0].x * k[0].x;
    d = fmaf(q[0].y, k[0].y, d); d = fmaf(q[0].z, k[0].z, d); d = fmaf(q[0].w, k[0].w, d);
#pragma unroll
    for (int v = 1; v < 4; ++v) {
        d = fmaf(q[v].x, k[v].x, d); d = fmaf(q[v].y, k[v].y, d);
        d = fmaf(q[v].z, k[v].z, d); d = fmaf(q[v].w, k[v].w, d);
    }
    return d;
}
__device__ __forceinline__ float chunk_dot(const uint4 (&q)[2], const uint4 (&k)[2]) {
    // products of two bf16 are exact in f32; v_dot2_f32_bf16 accumulates in f32
    float d = 0.f;
#pragma unroll
    for (int v = 0; v < 2; ++v) {
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].x), __builtin_bit_cast(bf16x2, k[v].x), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].y), __builtin_bit_cast(bf16x2, k[v].y), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].z), __builtin_bit_cast(bf16x2, k[v].z), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].w), __builtin_bit_cast(bf16x2, k[v].w), d, false);
    }
    return d;
}

template <typename V, int NCH>
__device__ __forceinline__ void load_chunks(V (&dst)[NCH], const unsigned char* head_base, uint32_t row_off) {
    // chunks s, s+4, ...: 64 bytes apart; the lane's own 16*s is folded into row_off
#pragma unroll
    for (int v = 0; v < NCH; ++v) dst[v] = *reinterpret_cast<const V*>(head_base + row_off + 64u * v);
}

// broadcast lane `src` of every quad to the whole quad
template <int SRC>
__device__ __forceinline__ int quad_bcast(int x) {
    return __builtin_amdgcn_update_dpp(0, x, SRC * 0x55, 0xF, 0xF, false);
}
__device__ __forceinline__ float quad_sum(float x) {
    x += dpp_mov<0xB1>(x);
    x += dpp_mov<0x4E>(x);
    return x;
}

constexpr int kQueriesPerWave = 16;
constexpr int kMeasureQueries = 4 * kQueriesPerWave;      // per work-group of 256 threads

template <typename T>
__global__ __launch_bounds__(256)
void measure_kernel(const T* __restrict__ Q, const T* __restrict__ K,
                    const int* __restrict__ lengths, const int* __restrict__ idx,
                    float* __restrict__ M, int H, int L, int U, int chunks_per_head, int n_heads)
{
    using RT = RowTraits<T>;
    using Vec = typename std::conditional<sizeof(T) == 4, float4, uint4>::type;
    constexpr int NCH = RT::kChunks;

    // Work-groups are dealt to the 8 XCDs round-robin by linear id.  All chunks
    // of one head go to ONE XCD so that the head's K rows are fetched into a
    // single L2: slot t of XCD x handles head (t / chunks_per_head) * 8 + x.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int head = (slot / chunks_per_head) * 8 + xcd;
    const int chunk = slot % chunks_per_head;
    if (head >= n_heads) return;                  // grid is padded to a multiple of 8 heads
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int s = lane & 3;
    const int i = chunk * kMeasureQueries + wave * kQueriesPerWave + (lane >> 2);
    const bool in_tensor = i < L;
    const bool active = i < n;

    // a wave whose queries are all padding has nothing to fetch
    if (__ballot(active) == 0ull) {
        if (in_tensor && s == 0) M[(size_t)head * L + i] = 0.f;
        return;
    }

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(K + (size_t)head * L * kD);
    const unsigned char* Qb = reinterpret_cast<const unsigned char*>(Q + (size_t)head * L * kD);
    const int* irow = idx + ((size_t)head * L + (in_tensor ? i : 0)) * U;

    Vec q[NCH];
    if (active) {
        load_chunks<Vec, NCH>(q, Qb, (uint32_t)i * RT::kRowBytes + 16u * s);
    } else {
#pragma unroll
        for (int v = 0; v < NCH; ++v) q[v] = Vec{};
    }

    float mx = -INFINITY, sm = 0.f;
    int cnt = 0;
    // Lane s of a quad fetches sample 4k + s; a round consumes k = kb, kb+1 (8 samples).
    const int n_k = (U + 3) >> 2;
    auto fetch_idx = [&](int k) -> int {
        const int t = 4 * k + s;
        return (active && k < n_k && t < U) ? irow[t] : -1;
    };
    int jv0 = fetch_idx(0), jv1 = fetch_idx(1);
    for (int kb = 0; kb < n_k; kb += 2) {
        const int jn0 = fetch_idx(kb + 2), jn1 = fetch_idx(kb + 3);       // next round's indices
        int j[8];
        j[0] = quad_bcast<0>(jv0); j[1] = quad_bcast<1>(jv0); j[2] = quad_bcast<2>(jv0); j[3] = quad_bcast<3>(jv0);
        j[4] = quad_bcast<0>(jv1); j[5] = quad_bcast<1>(jv1); j[6] = quad_bcast<2>(jv1); j[7] = quad_bcast<3>(jv1);
        const bool mine_ok = ((unsigned)jv0 < (unsigned)n) && ((unsigned)jv1 < (unsigned)n);
        Vec kr[8][NCH];
        if (__ballot(!mine_ok) == 0ull) {
            // every sample of this round is usable in every quad of the wave
#pragma unroll
            for (int t = 0; t < 8; ++t) load_chunks<Vec, NCH>(kr[t], Kb, (uint32_t)j[t] * RT::kRowBytes + 16u * s);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float sc = quad_sum(chunk_dot(q, kr[t])) * 0.125f;      // 1/sqrt(64)
                mx = fmaxf(mx, sc);
                sm += sc;
            }
            cnt += 8;
        } else {
            // padded queries, the tail of U, or indices outside [0, n): drop those samples
            bool ok[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                ok[t] = (unsigned)j[t] < (unsigned)n;
                load_chunks<Vec, NCH>(kr[t], Kb, (uint32_t)(ok[t] ? j[t] : 0) * RT::kRowBytes + 16u * s);
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float sc = quad_sum(chunk_dot(q, kr[t])) * 0.125f;
                mx = ok[t] ? fmaxf(mx, sc) : mx;
                sm += ok[t] ? sc : 0.f;
                cnt += ok[t] ? 1 : 0;
            }
        }
        jv0 = jn0; jv1 = jn1;
    }
    if (in_tensor && s == 0) {
        float m = 0.f;
        if (active && cnt > 0) m = mx - sm / (float)cnt;
        M[(size_t)head * L + i] = m;
    }
}

template <typename T>
static hipError_t launch_measure_t(const Plan& p, const Args& a, const Scratch& w)
{
    const int chunks = (p.L + kMeasureQueries - 1) / kMeasureQueries;
    const int head_rounds = (p.BH + 7) / 8;
    dim3 grid((unsigned)(head_rounds * chunks * 8)), block(256);
    hipLaunchKernelGGL(measure_kernel<T>, grid, block, 0, a.stream,
                       (const T*)a.Q, (const T*)a.K, a.lengths, a.idx, w.M, p.H, p.L, p.U, chunks, p.BH);
    return hipGetLastError();
}

hipError_t launch_measure(const Plan& p, const Args& a, const Scratch& w)
{
    return p.dtype == PSA_F32 ? launch_measure_t<float>(p, a, w) : launch_measure_t<bf16_t>(p, a, w);
}

}  // namespace psa

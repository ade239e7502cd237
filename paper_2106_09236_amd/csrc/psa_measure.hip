// Stage a1: scores of every query against its sampled keys and the sampled
// sparsity measure  M_i = max_t s_it - (1/#samples) sum_t s_it  (Sec. 3.2, Eq. 11).
// By-product for stage a4: float64 column sums of the valid V rows, per chunk.
//
// This is a gather, not a contraction: each query touches U random key rows of
// its own head.
//   * Heads whose K fits in LDS (measure_quad_kernel) gather from an LDS copy of K
//     with 4 lanes per query.
//   * Longer heads gather through L1 from the head's XCD-local L2 with 8 adjacent
//     lanes per query: a key row (256 B f32 / 128 B bf16) is read 128 bytes at a
//     time, lane s of the 8 taking bytes 16s .. 16s+15, so that one load instruction
//     takes a whole 128-byte line for each of the wave's 8 queries (64-byte pieces,
//     4 lanes per query, measured half the rate out of L2); the lanes keep the
//     matching pieces of the query in registers and the dot product is closed with
//     three DPP exchanges.  measure_pipe_kernel (up to 64 samples per query) keeps
//     gather waves and loader waves apart; measure_stream_kernel takes any U.
#include <type_traits>

#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

template <typename T> struct RowTraits;
template <> struct RowTraits<float>  { static constexpr int kRowBytes = 256; };
template <> struct RowTraits<bf16_t> { static constexpr int kRowBytes = 128; };

// Column sums, in float64, of the valid V rows [r0, r0 + rows) of one head, by a
// whole work-group of NT threads.  The mean of the valid V rows is the fill of the
// unselected queries (Sec. 3.1: uniform scores give the plain average of the
// values); summing here, where the rows are cut into few fixed chunks, keeps the
// order of additions fixed.  Two halves around one work-group barrier:
//   v_colsum_partial : loads, per-wave sums -> s_red[wave][64]
//   (barrier by the caller)
//   v_colsum_finish  : threads 0..63 add the waves in order -> out64[64]
template <typename T, int NT>
__device__ __forceinline__ void v_colsum_partial(const T* __restrict__ Vh, int r0, int rows, int n,
                                                 double (*s_red)[kD])
{
    constexpr int LPR = RowTraits<T>::kRowBytes / 16;     // lanes per row, 16 bytes each
    constexpr int EPL = kD / LPR;                         // elements per lane
    constexpr int RPP = NT / LPR;                         // rows per pass
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = tid % LPR, r = tid / LPR;
    double acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.0;
    if (r0 < n) {
        // unconditional loads on a clamped row, so that all of them are in flight
        // together; rows at or beyond n are added as zeros (+0.0 changes nothing)
#pragma unroll 4
        for (int row = r; row < rows; row += RPP) {
            const int j = r0 + row;
            const bool ok = j < n;
            const T* src = Vh + (size_t)(ok ? j : n - 1) * kD;
            if constexpr (sizeof(T) == 4) {
                float4 v = reinterpret_cast<const float4*>(src)[sub];
                if (!ok) v = make_float4(0.f, 0.f, 0.f, 0.f);
                acc[0] += (double)v.x; acc[1] += (double)v.y; acc[2] += (double)v.z; acc[3] += (double)v.w;
            } else {
                uint4 v = reinterpret_cast<const uint4*>(src)[sub];
                if (!ok) v = make_uint4(0u, 0u, 0u, 0u);
                acc[0] += (double)bf16_lo(v.x); acc[1] += (double)bf16_hi(v.x);
                acc[2] += (double)bf16_lo(v.y); acc[3] += (double)bf16_hi(v.y);
                acc[4] += (double)bf16_lo(v.z); acc[5] += (double)bf16_hi(v.z);
                acc[6] += (double)bf16_lo(v.w); acc[7] += (double)bf16_hi(v.w);
            }
        }
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
    if (lane < LPR) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_red[wave][sub * EPL + e] = acc[e];
    }
}
template <int NT>
__device__ __forceinline__ void v_colsum_finish(double* __restrict__ out64, double (*s_red)[kD])
{
    const int tid = threadIdx.x;
    if (tid < kD) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) t += s_red[w][tid];           // fixed order
        out64[tid] = t;
    }
}
template <typename T, int NT>
__device__ __forceinline__ void block_v_colsum(const T* __restrict__ Vh, int r0, int rows, int n,
                                               double* __restrict__ out64, double (*s_red)[kD])
{
    v_colsum_partial<T, NT>(Vh, r0, rows, n, s_red);
    __syncthreads();
    v_colsum_finish<NT>(out64, s_red);
}

constexpr int kStreamThreads = 512;
constexpr int kQueriesPerWave = 8;
static_assert(kMeasureQueries == (kStreamThreads / 64) * kQueriesPerWave, "one query per 8 lanes, eight waves");

// -----------------------------------------------------------------------------
// Streaming gather, one work-group per chunk of 64 queries, any number of samples.
// 8 lanes per query, whole 128-byte lines per load instruction, and nothing but the
// gather itself waits on memory inside the loop:
//   * the sample indices of a query (up to 8 rounds of 8 = 64 samples) are fetched
//     up front with the query row and the chunk's V rows, all unconditionally;
//   * the key rows of round k + 1 are requested before round k is reduced (16 row
//     loads in flight per wave), from two register sets that swap roles;
//   * key rows are read through a buffer descriptor over the head's VALID rows: a
//     32-bit offset per lane instead of a 64-bit address, and a sample index that
//     lies outside [0, n) reads zeros instead of needing a clamp (it is still left
//     out of the maximum and the mean);
//   * the V column sums cross the waves behind an LDS-only barrier, which does not
//     drain the loads in flight.
// Samples beyond 64 per query are fetched round by round after the pipelined part.
// (Its work-groups spend two fifths of their life waiting for their first inputs, see
// measure_pipe_kernel below, which the host prefers whenever U <= 64.)
// -----------------------------------------------------------------------------
constexpr int kStreamPre = 8;                    // rounds of 8 samples whose indices are fetched up front

template <typename T>
__global__ __launch_bounds__(kStreamThreads)
void measure_stream_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                           const int* __restrict__ lengths, const int* __restrict__ idx,
                           float* __restrict__ M, double* __restrict__ vpart, int* __restrict__ ticket,
                           int H, int L, int U, int chunks_per_head, int n_heads)
{
    using RT = RowTraits<T>;
    using Vec = typename std::conditional<sizeof(T) == 4, float4, uint4>::type;
    constexpr int NCH = RT::kRowBytes / 128;      // 16-byte chunks per lane: 8 lanes cover 128 bytes of a row
    constexpr int VLPR = RT::kRowBytes / 16, VEPL = kD / VLPR, VRPP = kStreamThreads / VLPR, VN = kMeasureQueries / VRPP;

    // all chunks of one head on ONE XCD (the head's K is fetched into a single L2)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int head = (slot / chunks_per_head) * 8 + xcd;
    const int chunk = slot % chunks_per_head;
    if (head >= n_heads) return;                  // grid is padded to a multiple of 8 heads (work-group-uniform)
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int s = lane & 7, gbase = lane & ~7;
    const int i = chunk * kMeasureQueries + wave * kQueriesPerWave + (lane >> 3);
    const bool in_tensor = i < L;
    const bool active = i < n;
    __shared__ double s_red[kStreamThreads / 64][kD];
    if (chunk == 0 && tid == 0) ticket[head] = 0;           // the attend stage counts work-groups per head
    if (chunk * kMeasureQueries >= n) {                     // the whole chunk is padding (work-group-uniform)
        if (in_tensor && s == 0) M[(size_t)head * L + i] = 0.f;
        if (tid < kD) vpart[((size_t)head * chunks_per_head + chunk) * kD + tid] = 0.0;
        return;
    }

    const T* Kh = K + (size_t)head * L * kD;
    const unsigned char* Qb = reinterpret_cast<const unsigned char*>(Q + (size_t)head * L * kD);
    const T* Vh = V + (size_t)head * L * kD;
    const int* irow = idx + ((size_t)head * L + (in_tensor ? i : 0)) * U;
    // the head's valid K rows as a raw buffer: offsets at or beyond n rows read zeros
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(Kh), 0, n * RT::kRowBytes, 0x00020000);
    const int lane_ofs = 16 * s;

    PSA_TS(0);
    // ---- every small load of the chunk, unconditional and on clamped addresses, in the
    // order in which the results are needed: sample indices, query row, V rows
    const int n_k = (U + 7) >> 3;
    int jraw[kStreamPre];
#pragma unroll
    for (int k = 0; k < kStreamPre; ++k) { const int t = 8 * k + s; jraw[k] = irow[t < U ? t : U - 1]; }
    Vec q[NCH];
#pragma unroll
    for (int v = 0; v < NCH; ++v)
        q[v] = *reinterpret_cast<const Vec*>(Qb + (size_t)(active ? i : 0) * RT::kRowBytes + lane_ofs + 128 * v);
    Vec vbuf[VN];
    const int vsub = tid % VLPR, vrow = tid / VLPR;
#pragma unroll
    for (int k = 0; k < VN; ++k) {
        const int j = chunk * kMeasureQueries + vrow + k * VRPP;
        vbuf[k] = reinterpret_cast<const Vec*>(Vh + (size_t)(j < n ? j : n - 1) * kD)[vsub];      // n > 0 here
    }
    if (!active) {
#pragma unroll
        for (int v = 0; v < NCH; ++v) q[v] = Vec{};
    }

    auto row_dot = [&](const Vec (&kr)[NCH]) -> float {
        float d = 0.f;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int v = 0; v < NCH; ++v) {
                d = fmaf(q[v].x, kr[v].x, d); d = fmaf(q[v].y, kr[v].y, d);
                d = fmaf(q[v].z, kr[v].z, d); d = fmaf(q[v].w, kr[v].w, d);
            }
        } else {
            // products of two bf16 are exact in f32; v_dot2_f32_bf16 accumulates in f32
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].x), __builtin_bit_cast(bf16x2, kr[0].x), d, false);
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].y), __builtin_bit_cast(bf16x2, kr[0].y), d, false);
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].z), __builtin_bit_cast(bf16x2, kr[0].z), d, false);
            d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].w), __builtin_bit_cast(bf16x2, kr[0].w), d, false);
        }
        return d;                                                   // this lane's share of the dot product
    };
    float mx = -INFINITY, sm = 0.f;
    int cnt = 0;
    // One round = the 8 samples jv of the query's lanes (-1: no such sample).  `full` (wave-uniform):
    // every sample of the round is usable in every query of the wave, so the sums need no mask.
    auto request = [&](int k, int jv, Vec (&kr)[8][NCH]) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (8 * k + t >= U) break;                              // wave-uniform: no such sample
            const int j = __shfl(jv, gbase + t, 64);
            const int ofs = j * RT::kRowBytes + lane_ofs;            // (wraps for j < 0: out of range, reads zeros)
#pragma unroll
            for (int v = 0; v < NCH; ++v) {
                const auto x = __builtin_amdgcn_raw_buffer_load_b128(krsrc, ofs + 128 * v, 0, 0);
                kr[t][v] = __builtin_bit_cast(Vec, x);
            }
        }
    };
    auto reduce = [&](int k, int jv, bool full, const Vec (&kr)[8][NCH]) {
        if (full) {
            // sums over the query's 8 lanes, one exchange stage at a time for all rows; the
            // 1/sqrt(64) is applied once at the end (exact: a power of 2)
            float d[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) d[t] = row_dot(kr[t]);
#pragma unroll
            for (int t = 0; t < 8; ++t) d[t] += dpp_mov<0xB1>(d[t]);
#pragma unroll
            for (int t = 0; t < 8; ++t) d[t] += dpp_mov<0x4E>(d[t]);
#pragma unroll
            for (int t = 0; t < 8; ++t) d[t] += dpp_mov<0x141>(d[t]);
#pragma unroll
            for (int t = 0; t < 8; ++t) { mx = fmaxf(mx, d[t]); sm += d[t]; }
            cnt += 8;
        } else {
            // padded queries, the tail of U, or indices outside [0, n): those samples are dropped
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (8 * k + t >= U) break;                          // wave-uniform
                const bool ok = (unsigned)__shfl(jv, gbase + t, 64) < (unsigned)n;
                const float sc = group_sum8(row_dot(kr[t]));
                mx = ok ? fmaxf(mx, sc) : mx;
                sm += ok ? sc : 0.f;
                cnt += ok ? 1 : 0;
            }
        }
    };
    auto sample_of = [&](int k, int raw) -> int { return (active && 8 * k + s < U) ? raw : -1; };
    auto is_full = [&](int jv) -> bool { return __ballot((unsigned)jv >= (unsigned)n) == 0ull; };

    // ---- the first round's rows are requested as soon as the indices are back ...
    Vec ka[8][NCH], kb[8][NCH];
    const int n_pre = n_k < kStreamPre ? n_k : kStreamPre;
    int jcur = sample_of(0, jraw[0]);
    if (__ballot(active) != 0ull) request(0, jcur, ka);
    PSA_TS(1);
    // ---- ... and the column sums of this chunk's valid V rows (float64) are formed under them
    {
        double acc[VEPL];
#pragma unroll
        for (int e = 0; e < VEPL; ++e) acc[e] = 0.0;
#pragma unroll
        for (int k = 0; k < VN; ++k) {
            const bool vok = chunk * kMeasureQueries + vrow + k * VRPP < n;
            if constexpr (sizeof(T) == 4) {
                const float4 v = vbuf[k];
                acc[0] += vok ? (double)v.x : 0.0; acc[1] += vok ? (double)v.y : 0.0;
                acc[2] += vok ? (double)v.z : 0.0; acc[3] += vok ? (double)v.w : 0.0;
            } else {
                const uint4 v = vbuf[k];
                acc[0] += vok ? (double)bf16_lo(v.x) : 0.0; acc[1] += vok ? (double)bf16_hi(v.x) : 0.0;
                acc[2] += vok ? (double)bf16_lo(v.y) : 0.0; acc[3] += vok ? (double)bf16_hi(v.y) : 0.0;
                acc[4] += vok ? (double)bf16_lo(v.z) : 0.0; acc[5] += vok ? (double)bf16_hi(v.z) : 0.0;
                acc[6] += vok ? (double)bf16_lo(v.w) : 0.0; acc[7] += vok ? (double)bf16_hi(v.w) : 0.0;
            }
        }
#pragma unroll
        for (int off = VLPR; off < 64; off <<= 1)
#pragma unroll
            for (int e = 0; e < VEPL; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
        if (lane < VLPR) {
#pragma unroll
            for (int e = 0; e < VEPL; ++e) s_red[wave][vsub * VEPL + e] = acc[e];
        }
        lds_barrier();
        v_colsum_finish<kStreamThreads>(vpart + ((size_t)head * chunks_per_head + chunk) * kD, s_red);
    }
    PSA_TS(2);
    if (__ballot(active) == 0ull) {               // a wave whose queries are all padding has nothing to gather
        if (in_tensor && s == 0) M[(size_t)head * L + i] = 0.f;
        return;
    }

    // ---- the pipelined rounds: compile-time round numbers, so the two register sets alternate
    // without copies and jraw[] is indexed statically
    bool fcur = is_full(jcur);
#pragma unroll
    for (int k = 0; k < kStreamPre; ++k) {
        if (k >= n_pre) break;                                      // wave-uniform
        int jnext = -1;
        if (k + 1 < kStreamPre) jnext = sample_of(k + 1, jraw[k + 1 < kStreamPre ? k + 1 : 0]);
        if (k + 1 < kStreamPre && k + 1 < n_pre) { if (k & 1) request(k + 1, jnext, ka); else request(k + 1, jnext, kb); }
        if (k & 1) reduce(k, jcur, fcur, kb); else reduce(k, jcur, fcur, ka);
        jcur = jnext;
        fcur = is_full(jcur);
    }
    // ---- more than 64 samples per query: the remaining rounds, their indices fetched here
#pragma unroll 1
    for (int k = kStreamPre; k < n_k; ++k) {
        const int t = 8 * k + s;
        const int jv = sample_of(k, irow[t < U ? t : U - 1]);
        request(k, jv, ka);
        reduce(k, jv, is_full(jv), ka);
    }
    PSA_TS(3);
    if (in_tensor && s == 0) {
        float m = 0.f;
        if (active && cnt > 0) m = (mx - sm / (float)cnt) * 0.125f;         // 1/sqrt(64), exact
        M[(size_t)head * L + i] = m;
    }
    PSA_TS_DRAIN();
    PSA_TS(4);
}

// -----------------------------------------------------------------------------
// Streaming gather with loader waves.  Traces of the kernel above show a work-group
// spending two fifths of its life before its first key row arrives: sample indices,
// query rows and V rows come from HBM (about 2 us), and a load that waits for HBM
// holds back every later load of the same wave (loads complete in issue order), so
// fetching the next chunk's inputs from inside the gather loop only moves the
// stall.  Here the two kinds of load never meet in one wave:
//   * a work-group is 8 gather waves + 2 loader waves and takes several consecutive
//     chunks of 64 queries of one head;
//   * the loader waves bring the NEXT chunk's sample indices (one wave) and query
//     rows (the other) into a second LDS stage while the gather waves work on the
//     current one; the second also forms the float64 column sums of the current
//     chunk's V rows (nothing the gather waves wait for);
//   * a gather wave reads its query row and, per round, the 4 sample indices of
//     its query from LDS (all 8 lanes of a query read the same words: a
//     broadcast, no lane shuffles), and touches memory only for key rows: 8 lanes
//     per query, whole 128-byte lines, through a buffer descriptor over the head's
//     valid rows; a round is requested, waited for and reduced before the next
//     (with 16 gather waves on a CU the other waves' requests fill the return
//     path meanwhile; keeping more of one wave's loads in flight measured slower).
// One LDS-only barrier per chunk.  Used for up to 64 samples per query (the stage
// holds the chunk's indices); beyond that measure_stream_kernel takes over.
// -----------------------------------------------------------------------------
// A buffer load that writes LDS directly, no registers: lane l's 16 bytes land at lds + 16 l.
// (The body exists in the device pass only: the host pass does not know the instruction's sizes.)
__device__ __forceinline__ void buffer_load_to_lds_b128(__amdgpu_buffer_rsrc_t rsrc, void* lds, int voffset, int soffset) {
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) void lds_void;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)lds, 16, voffset, soffset, 0, 2 /* non-temporal */);
#endif
}

constexpr int kPipeGatherWaves = 8;
constexpr int kPipeThreads = (kPipeGatherWaves + 2) * 64;       // + two loader waves
constexpr int kPipeMaxU = kPipeMaxSamples;
// cache-policy bits of a buffer load for data that is read once (non-temporal): the loader waves' streams
// of indices, query rows and V rows must not push the head's K rows, which are re-read all the time, out of L2
// (longform, inputs from HBM: 47.5 -> 45.5 us)
constexpr int kStreamOnce = 2;
static_assert(kMeasureQueries == kPipeGatherWaves * kQueriesPerWave, "one query per 8 lanes, eight gather waves");

__host__ __device__ constexpr int pipe_idx_stride(int U) { return U; }                     // ints per staged index row (as in memory)
template <typename T>
__host__ __device__ constexpr int pipe_stage_bytes(int U) {
    // (+ 16: the last round of the last row reads up to 3 entries past its end; 16-byte alignment of the rows)
    return ((kMeasureQueries * pipe_idx_stride(U) * 4 + 16 + 15) & ~15) + kMeasureQueries * RowTraits<T>::kRowBytes;
}

template <typename T>
__global__ __launch_bounds__(kPipeThreads, sizeof(T) == 2 ? 6 : 3)    // bfloat16: two work-groups per CU whichever SIMDs get a work-group's odd waves
void measure_pipe_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                         const int* __restrict__ lengths, const int* __restrict__ idx,
                         float* __restrict__ M, double* __restrict__ vpart, int* __restrict__ ticket,
                         uint2* __restrict__ cand, int cand_len, double* __restrict__ vlist,
                         int H, int L, int U, int chunks_per_head, int chunks_per_wg, int n_heads)
{
    using RT = RowTraits<T>;
    using Vec = typename std::conditional<sizeof(T) == 4, float4, uint4>::type;
    constexpr int NCH = RT::kRowBytes / 128;      // 16-byte chunks per lane: 8 lanes cover 128 bytes of a row
    constexpr int NQL = kMeasureQueries * RT::kRowBytes / 1024;     // 16-byte loads per loader lane for 64 rows: 8 or 16
    // (order key, ~position) of the measures of this work-group's queries, for its candidate list (cand != nullptr)
    __shared__ unsigned long long s_rank[kListMax], s_list[kListMax];
    __shared__ double s_vtot[kD];                 // column sums of V over all chunks of this work-group (with the list)
    __shared__ int s_clean[2];                    // per stage: every query of the chunk is valid and every sample index usable
    extern __shared__ __attribute__((aligned(16))) unsigned char s_stage[];    // [2][ idx [64][Us] | q [64][row bytes] ]

    const int groups_per_head = (chunks_per_head + chunks_per_wg - 1) / chunks_per_wg;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int head = (slot / groups_per_head) * 8 + xcd;          // all work-groups of a head on one XCD
    const int chunk0 = (slot % groups_per_head) * chunks_per_wg;
    if (head >= n_heads) return;                  // grid is padded to a multiple of 8 heads (work-group-uniform)
    int chunk_end = chunk0 + chunks_per_wg;
    chunk_end = chunk_end < chunks_per_head ? chunk_end : chunks_per_head;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int s = lane & 7;
    const int ql = (wave & 7) * kQueriesPerWave + (lane >> 3);     // a gather lane's query within the chunk
    const int Us = pipe_idx_stride(U);
    const int stage_bytes = pipe_stage_bytes<T>(U);
    if (chunk0 == 0 && tid == 0) ticket[head] = 0;                 // the attend stage counts work-groups per head

    // chunks that are padding as a whole (all of them, once one is: chunks ascend)
    const int first_pad = (n + kMeasureQueries - 1) / kMeasureQueries;
    for (int chunk = (chunk0 > first_pad ? chunk0 : first_pad); chunk < chunk_end; ++chunk) {
        const int i = chunk * kMeasureQueries + tid;
        if (tid < kMeasureQueries && i < L) M[(size_t)head * L + i] = 0.f;
        if (tid < kD) vpart[((size_t)head * chunks_per_head + chunk) * kD + tid] = 0.0;
    }
    chunk_end = chunk_end < first_pad ? chunk_end : first_pad;
    uint2* cand_out = cand ? cand + ((size_t)head * groups_per_head + slot % groups_per_head) * cand_len : nullptr;
    double* vlist_out = cand ? vlist + ((size_t)head * groups_per_head + slot % groups_per_head) * kD : nullptr;
    if (chunk0 >= chunk_end) {                    // work-group-uniform: nothing valid here, an empty list
        if (cand_out) for (int t = tid; t < cand_len; t += kPipeThreads) cand_out[t] = make_uint2(0u, 0xFFFFFFFFu);
        if (cand_out && tid < kD) vlist_out[tid] = 0.0;
        return;
    }
    // n > 0 from here on
    if (cand_out) for (int t = tid; t < kListMax; t += kPipeThreads) s_rank[t] = 0ull;
    if (tid < kD) s_vtot[tid] = 0.0;

    const T* Kh = K + (size_t)head * L * kD;
    const T* Vh = V + (size_t)head * L * kD;
    const int* idx_h = idx + (size_t)head * L * U;
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(Kh), 0, n * RT::kRowBytes, 0x00020000);      // offsets at or beyond n rows read zeros
    const int lane_ofs = 16 * s;

    // ---- loader wave A: the chunk's sample indices -> LDS stage `st`
    auto load_indices = [&](int chunk, int st) {
        int* s_idx = reinterpret_cast<int*>(s_stage + (size_t)st * stage_bytes);
        const int i0 = chunk * kMeasureQueries;
        int rows = L - i0;                                           // rows of the tensor in this chunk
        rows = rows < kMeasureQueries ? rows : kMeasureQueries;
        // the chunk's indices are contiguous in memory: a raw buffer over them (reads past the end give 0)
        const __amdgpu_buffer_rsrc_t irsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int*>(idx_h + (size_t)i0 * U), 0, rows * U * 4, 0x00020000);
        // 16 bytes per lane and load (a quarter of the load instructions of a dword per lane: the loaders share
        // the CU's return path with the gather waves), all loads in flight together; the stage keeps the
        // indices as they lie in memory (row stride U), so the bytes at 1024 k + 16 lane go to the same place
        constexpr int NV = kPipeMaxU / 4;                            // 16 KB at most
        const int bytes = kMeasureQueries * U * 4;                   // (a multiple of 16)
        uint4 iv[NV];
#pragma unroll
        for (int k = 0; k < NV; ++k)
            if (1024 * k < bytes)                                    // wave-uniform
                iv[k] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(irsrc, 16 * lane, 1024 * k, kStreamOnce));
        bool bad = false;                                            // some index of the chunk outside [0, n)
#pragma unroll
        for (int k = 0; k < NV; ++k)
            if (1024 * k < bytes && 1024 * k + 16 * lane < bytes) {
                *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(s_idx) + 1024 * k + 16 * lane) = iv[k];
                bad |= iv[k].x >= (unsigned)n || iv[k].y >= (unsigned)n || iv[k].z >= (unsigned)n || iv[k].w >= (unsigned)n;
            }
        // a chunk of 64 valid queries whose samples are all usable: its gather needs no masks
        const bool clean = __ballot(bad) == 0ull && i0 + kMeasureQueries <= n;
        if (lane == 0) s_clean[st] = clean ? 1 : 0;
    };
    // ---- loader wave B: the chunk's query rows -> LDS stage `st`, and the chunk's V column sums -> vpart
    auto load_rows = [&](int q_chunk, int v_chunk, int st) {
        unsigned char* s_q = s_stage + (size_t)st * stage_bytes + (stage_bytes - kMeasureQueries * RT::kRowBytes);
        // raw buffers over the head's valid rows: rows at or beyond n read zeros
        auto fetch = [&](const T* base, int chunk, Vec (&x)[NQL]) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(base), 0, n * RT::kRowBytes, 0x00020000);
#pragma unroll
            for (int k = 0; k < NQL; ++k)                            // 16 bytes at position 1024 k + 16 lane of the chunk's 64 rows
                x[k] = __builtin_bit_cast(Vec, __builtin_amdgcn_raw_buffer_load_b128(
                           rs, chunk * kMeasureQueries * RT::kRowBytes + 16 * lane, 1024 * k, kStreamOnce));
        };
        // the query rows go straight to LDS (16 bytes of position 1024 k + 16 lane of the chunk's rows land at
        // the same position of the stage: no staging registers, which would count against the gather waves'
        // cap), the V rows to registers; both in flight together
        if (q_chunk >= 0) {
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<T*>(Q + (size_t)head * L * kD), 0, n * RT::kRowBytes, 0x00020000);
#pragma unroll
            for (int k = 0; k < NQL; ++k)
                buffer_load_to_lds_b128(rs, s_q + 1024 * k, q_chunk * kMeasureQueries * RT::kRowBytes + 16 * lane, 1024 * k);
        }
        if (v_chunk < 0) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); return; }
        Vec vv[NQL];
        fetch(Vh, v_chunk, vv);
        // column sums of the chunk's valid V rows in float64: lane l holds 16 bytes of rows
        // (1024 k + 16 l) / row bytes; first its own rows, then the lanes that hold the same columns
        // (rows at or beyond n came back as zeros)
        constexpr int VLPR = RT::kRowBytes / 16, VEPL = kD / VLPR;
        double acc[VEPL];
#pragma unroll
        for (int e = 0; e < VEPL; ++e) acc[e] = 0.0;
#pragma unroll
        for (int k = 0; k < NQL; ++k) {
            if constexpr (sizeof(T) == 4) {
                const float4 v = vv[k];
                acc[0] += (double)v.x; acc[1] += (double)v.y; acc[2] += (double)v.z; acc[3] += (double)v.w;
            } else {
                const uint4 v = vv[k];
                acc[0] += (double)bf16_lo(v.x); acc[1] += (double)bf16_hi(v.x);
                acc[2] += (double)bf16_lo(v.y); acc[3] += (double)bf16_hi(v.y);
                acc[4] += (double)bf16_lo(v.z); acc[5] += (double)bf16_hi(v.z);
                acc[6] += (double)bf16_lo(v.w); acc[7] += (double)bf16_hi(v.w);
            }
        }
#pragma unroll
        for (int off = VLPR; off < 64; off <<= 1)
#pragma unroll
            for (int e = 0; e < VEPL; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
        if (lane < VLPR) {
            double* vo = vpart + ((size_t)head * chunks_per_head + v_chunk) * kD + lane * VEPL;
#pragma unroll
            for (int e = 0; e < VEPL; ++e) { vo[e] = acc[e]; s_vtot[lane * VEPL + e] += acc[e]; }    // chunks in order
        }
    };

    // ---- gather waves: one chunk from LDS stage `st`
    auto gather_chunk = [&](int chunk, int st) {
        const unsigned char* sbase = s_stage + (size_t)st * stage_bytes;
        const int* s_idx = reinterpret_cast<const int*>(sbase) + ql * Us;
        const unsigned char* s_q = sbase + (stage_bytes - kMeasureQueries * RT::kRowBytes) + ql * RT::kRowBytes;
        const int i = chunk * kMeasureQueries + ql;
        const bool in_tensor = i < L;
        const bool active = i < n;
        if (__ballot(active) == 0ull) {                              // all 8 queries of the wave are padding
            if (in_tensor && s == 0) M[(size_t)head * L + i] = 0.f;
            return;
        }
        Vec q[NCH];
#pragma unroll
        for (int v = 0; v < NCH; ++v) q[v] = *reinterpret_cast<const Vec*>(s_q + lane_ofs + 128 * v);
        auto row_dot = [&](const Vec (&kr)[NCH]) -> float {         // this lane's share of q . k
            float d = 0.f;
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int v = 0; v < NCH; ++v) {
                    d = fmaf(q[v].x, kr[v].x, d); d = fmaf(q[v].y, kr[v].y, d);
                    d = fmaf(q[v].z, kr[v].z, d); d = fmaf(q[v].w, kr[v].w, d);
                }
            } else {
                // products of two bf16 are exact in f32; v_dot2_f32_bf16 accumulates in f32
                d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].x), __builtin_bit_cast(bf16x2, kr[0].x), d, false);
                d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].y), __builtin_bit_cast(bf16x2, kr[0].y), d, false);
                d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].z), __builtin_bit_cast(bf16x2, kr[0].z), d, false);
                d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[0].w), __builtin_bit_cast(bf16x2, kr[0].w), d, false);
            }
            return d;
        };
        float mx = -INFINITY, sm = 0.f;
        int cnt = 0;
        // Rounds of 4 samples from one set of row registers: request, wait, reduce.  (Two sets with the next
        // round requested before the current one is reduced, and a ring of 8 single-row buffers, both measured
        // slower, in a micro-benchmark of the loop alone as well: with 16 such waves on a CU the other waves'
        // requests fill the return path while this one computes.)
        auto round_idx = [&](int k, int (&j)[4]) {                   // the 4 sample indices of round k of this lane's query
#pragma unroll
            for (int t = 0; t < 4; ++t) j[t] = s_idx[4 * k + t];      // (4-byte aligned: rows are U entries apart)
        };
        // requests the key rows of round k; returns whether every sample of the round is usable in
        // every query of the wave (wave-uniform), in which case the sums need no mask
        auto request = [&](int k, Vec (&kr)[4][NCH]) -> bool {
            int j[4];
            round_idx(k, j);
            bool bad = !active;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (4 * k + t >= U) break;                          // wave-uniform: no such sample
                bad |= (unsigned)j[t] >= (unsigned)n;
                const int ofs = j[t] * RT::kRowBytes + lane_ofs;     // (out of range for a bad index: reads zeros)
#pragma unroll
                for (int v = 0; v < NCH; ++v) {
                    const auto x = __builtin_amdgcn_raw_buffer_load_b128(krsrc, ofs + 128 * v, 0, 0);
                    kr[t][v] = __builtin_bit_cast(Vec, x);
                }
            }
            return 4 * k + 4 <= U && __ballot(bad) == 0ull;
        };
        auto reduce = [&](int k, bool full, const Vec (&kr)[4][NCH]) {
            if (full) {
                // sums over the query's 8 lanes, one exchange stage at a time for all rows; the
                // 1/sqrt(64) is applied once at the end (exact: a power of 2)
                float d[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = row_dot(kr[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0xB1>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0x4E>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0x141>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) { mx = fmaxf(mx, d[t]); sm += d[t]; }
                cnt += 4;
            } else {
                // padded queries, the tail of U, or indices outside [0, n): those samples are dropped
                int j[4];
                round_idx(k, j);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (4 * k + t >= U) break;                      // wave-uniform
                    const bool ok = active && (unsigned)j[t] < (unsigned)n;
                    const float sc = group_sum8(row_dot(kr[t]));
                    mx = ok ? fmaxf(mx, sc) : mx;
                    sm += ok ? sc : 0.f;
                    cnt += ok ? 1 : 0;
                }
            }
        };
        const int n_r = (U + 3) >> 2;
        Vec ka[4][NCH];
        if (__builtin_amdgcn_readfirstlane(s_clean[st]) != 0) {
            // every query of the chunk is valid and every sample index usable (the loader wave's finding): whole
            // rounds without tests, masks or counts
            const int n_whole = U >> 2;
#pragma unroll 1
            for (int k = 0; k < n_whole; ++k) {
                int j[4];
                round_idx(k, j);
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int v = 0; v < NCH; ++v)
                        ka[t][v] = __builtin_bit_cast(Vec, __builtin_amdgcn_raw_buffer_load_b128(
                                       krsrc, j[t] * RT::kRowBytes + lane_ofs + 128 * v, 0, 0));
                float d[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = row_dot(ka[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0xB1>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0x4E>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0x141>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) { mx = fmaxf(mx, d[t]); sm += d[t]; }
            }
            cnt = 4 * n_whole;
            if (4 * n_whole < U) {                                   // the last U % 4 samples
                const bool fa = request(n_whole, ka);
                reduce(n_whole, fa, ka);
            }
        } else {
#pragma unroll 1
            for (int k = 0; k < n_r; ++k) {
                const bool fa = request(k, ka);
                reduce(k, fa, ka);
            }
        }
        if (in_tensor && s == 0) {
            float m = 0.f;
            if (active && cnt > 0) m = (mx - sm / (float)cnt) * 0.125f;     // 1/sqrt(64), exact
            M[(size_t)head * L + i] = m;
            if (cand_out && active) {
                // order key of the measure (-0 -> +0; larger measure = larger key; 0 = not a candidate);
                // equal keys: the lower query is the larger
                const unsigned ub = __float_as_uint(m + 0.0f);
                const unsigned key = (ub & 0x80000000u) ? ~ub : (ub | 0x80000000u);
                const int pos = (chunk - chunk0) * kMeasureQueries + ql;
                s_rank[pos] = ((unsigned long long)key << 32) | (unsigned)~pos;
            }
        }
    };

    PSA_TS(0);
    // trip `chunk`: the loader waves fill the other stage with chunk + 1 while the gather waves work on
    // `chunk` (the first trip only loads).  One loop per kind of wave, each with the trip's barrier: what only
    // the gather waves use is then not live across the loaders' staging registers (the kernel's register cap
    // is what lets two work-groups share a CU).
    if (wave == kPipeGatherWaves) {
#pragma unroll 1
        for (int chunk = chunk0 - 1; chunk < chunk_end; ++chunk) {
            if (chunk + 1 < chunk_end) load_indices(chunk + 1, ((chunk - chunk0) & 1) ^ 1);
            lds_barrier();
        }
    } else if (wave == kPipeGatherWaves + 1) {
#pragma unroll 1
        for (int chunk = chunk0 - 1; chunk < chunk_end; ++chunk) {   // query rows one chunk ahead, V sums of the current one
            load_rows(chunk + 1 < chunk_end ? chunk + 1 : -1, chunk >= chunk0 ? chunk : -1, ((chunk - chunk0) & 1) ^ 1);
            lds_barrier();
        }
    } else {
#pragma unroll 1
        for (int chunk = chunk0 - 1; chunk < chunk_end; ++chunk) {
            if (chunk >= chunk0) gather_chunk(chunk, (chunk - chunk0) & 1);
            // the next stage is filled, and this one has been read by every gather wave
            lds_barrier();
            if (chunk < chunk0) PSA_TS(1);
        }

    }
    PSA_TS(2);
    // ---- local ranking for stage a2 (as in the LDS kernel): any query among the head's u largest is among
    // this work-group's u largest, so it hands on its first cand_len queries in order of decreasing measure
    // (ties: lower index first) as (order key, query index) pairs.  The last barrier of the loop has made
    // every gather wave's keys visible.  Two steps: every chunk of 64 ranks its own keys (two lanes per key,
    // 32 comparisons each) into a sorted list in LDS; then the up to 4 lists are merged, the position of an
    // entry being its own rank plus, per other list, the number of entries before it (a binary search per
    // list, four lanes per entry).  Ranking all 256 keys against each other took 3 us at the end of every
    // work-group; this takes under one.
    if (cand_out) {
        const int n_ch = chunk_end - chunk0;                         // chunks in use: 1 .. 4 (kListMax / 64)
        const int n_pos = n_ch * kMeasureQueries;
        int n_here = n - chunk0 * kMeasureQueries;                   // valid queries of this work-group
        n_here = n_here < n_pos ? n_here : n_pos;
        const int keep = cand_len < kMeasureQueries ? cand_len : kMeasureQueries;    // entries a chunk's list can contribute
        {
            const int h2 = tid & 1, pos = tid >> 1;                  // 512 gather lanes: two per position
            const bool ok = tid < kPipeGatherWaves * 64 && pos < n_pos;
            const unsigned long long mine = s_rank[ok ? pos : 0];
            const unsigned long long* row = s_rank + (ok ? pos & ~(kMeasureQueries - 1) : 0);
            int beat = 0;
#pragma unroll 8
            for (int t = 0; t < kMeasureQueries / 2; ++t) beat += row[2 * t + h2] > mine ? 1 : 0;
            beat += __builtin_amdgcn_update_dpp(0, beat, 0xB1, 0xF, 0xF, false);             // sum over the pair
            for (int t = tid; t < n_ch * kMeasureQueries; t += kPipeThreads) s_list[t] = 0ull;
            lds_barrier();
            if (ok && h2 == 0 && beat < keep) s_list[(pos / kMeasureQueries) * kMeasureQueries + beat] = mine;
            lds_barrier();
        }
        // merge: entry ci = (list, rank) -> position among all lists; keys are unique (they carry their position)
        for (int t0 = 0; t0 < n_ch * keep * 4; t0 += kPipeThreads) { // work-group-uniform trip count
            const int t = t0 + tid;
            const int ci = t >> 2, c2 = t & 3;
            const int lst = ci / keep, rk = ci - lst * keep;
            const bool ok = ci < n_ch * keep;
            const unsigned long long mine = ok ? s_list[lst * kMeasureQueries + rk] : 0ull;
            int cnt = 0;
            if (ok && c2 == lst) cnt = rk;
            else if (ok && c2 < n_ch) {
                const unsigned long long* other = s_list + c2 * kMeasureQueries;
                int lo = 0, hi = keep;                               // first entry that does not come before mine
                while (lo < hi) { const int mid = (lo + hi) >> 1; if (other[mid] > mine) lo = mid + 1; else hi = mid; }
                cnt = lo;
            }
            cnt += __builtin_amdgcn_update_dpp(0, cnt, 0xB1, 0xF, 0xF, false);               // sum over the quad
            cnt += __builtin_amdgcn_update_dpp(0, cnt, 0x4E, 0xF, 0xF, false);
            if (ok && c2 == 0 && (unsigned)(mine >> 32) != 0u && cnt < cand_len) {
                const int pos = (int)~(unsigned)mine;                // the key's low word is ~position
                cand_out[cnt] = make_uint2((unsigned)(mine >> 32), (unsigned)(chunk0 * kMeasureQueries + pos));
            }
        }
        for (int t = n_here + tid; t < cand_len; t += kPipeThreads) cand_out[t] = make_uint2(0u, 0xFFFFFFFFu);   // empty slots
        if (tid < kD) vlist_out[tid] = s_vtot[tid];                  // (written by the loader wave before the last barrier)
    }
    PSA_TS(3);
    PSA_TS_DRAIN();
    PSA_TS(4);
}

__device__ __forceinline__ float quad_sum(float x) {
    x += dpp_mov<0xB1>(x);
    x += dpp_mov<0x4E>(x);
    return x;
}
template <int T4>                                          // value of lane T4 of the quad, in all four lanes
__device__ __forceinline__ int quad_bcast(int x) {
    return __builtin_amdgcn_update_dpp(0, x, T4 * 0x55, 0xF, 0xF, false);
}

// -----------------------------------------------------------------------------
// Variant for heads whose whole K fits in LDS (L * row bytes <= 128 KB: L <= 512
// in f32, L <= 1024 in bf16).  A work-group of 8 waves copies the head's valid K
// rows into LDS once (coalesced) and gathers from there, FOUR lanes per query (16
// queries per wave): the sample index reaches the quad's lanes by a DPP quad
// broadcast, the lane sums take two exchange stages, and every instruction serves
// 16 (query, sample) pairs.  Lane s of a quad reads bytes 16s .. 16s+15 of each
// 64-byte piece of the row, and quad number g of the wave takes the pieces in
// the order g, g+1, ... (mod the pieces of a row): the LDS has 64 banks, a
// float32 row spans all of them once, so the four quads of any 16 adjacent lanes
// touch four different quarters of the banks whichever rows they read (random
// float32 rows, measured: 138 B/clk per CU this way, 114 with the pieces swapped
// in pairs, 60 with every quad on the same piece).  For float32 rows the gather
// runs at that LDS read rate (1 MB per chunk of 128 queries with 32 samples); for
// bfloat16 rows LDS reads and instruction issue are about level.  (Eight lanes per
// query in a 16-wave work-group, with the index passed by an LDS lane shuffle,
// measured 4..9 % slower.)
// -----------------------------------------------------------------------------
constexpr int kQuadThreads = 512;
constexpr int kQuadQueriesPerWave = 16;
static_assert(kLdsQueries == (kQuadThreads / 64) * kQuadQueriesPerWave, "one query per 4 lanes, 8 waves");


// KCOPY: 16-byte pieces of K per thread = LDS bytes / 8 KB: 16 (a head of up to 128 KB) or 8 (up
// to 64 KB).  With 64 KB two work-groups fit a CU; for bfloat16 rows the registers are capped to
// let them (4 waves per SIMD), so that one work-group copies its K while
// the other gathers.
// The work of one work-group: chunks [chunk0, chunk0 + chunks_per_wg) of `head`.  sK: KCOPY * 8 KB of LDS for
// the head's K; s_red, s_key: the work-group's reduction scratch.
template <typename T, int KCOPY>
__device__ __forceinline__ void measure_quad_body(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                                                  const int* __restrict__ lengths, const int* __restrict__ idx,
                                                  float* __restrict__ M, double* __restrict__ vpart,
                                                  uint2* __restrict__ cand, int cand_len,
                                                  int H, int L, int U, int chunks_per_head, int chunks_per_wg,
                                                  int head, int chunk0, unsigned char* sK, double (*s_red)[kD],
                                                  unsigned long long* s_key)
{
    using RT = RowTraits<T>;
    using Vec = typename std::conditional<sizeof(T) == 4, float4, uint4>::type;
    constexpr int NP = RT::kRowBytes / 64;               // 16-byte pieces per lane and row: 4 (f32) or 2 (bf16)
    static_assert(KCOPY * 16 * kQuadThreads <= kLdsMaxBytes, "at most 128 KB of K");
    auto put_v = [](double* p, double v) { *p = v; };
    auto put_c = [](uint2* p, unsigned key, unsigned q) { *p = make_uint2(key, q); };

    int chunk_end = chunk0 + chunks_per_wg;
    chunk_end = chunk_end < chunks_per_head ? chunk_end : chunks_per_head;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int s = lane & 3;
    const int qrot = (lane >> 2) & (RT::kRowBytes / 64 - 1);           // the quad's rotation of the piece order
    const int ql = wave * kQuadQueriesPerWave + (lane >> 2);            // query within a chunk
    // s_key: (order key, ~query) of a chunk's measures: one 64-bit compare ranks

    // chunks that are padding as a whole (all of them, once one is: chunks ascend)
    const int first_pad = (n + kLdsQueries - 1) / kLdsQueries;          // first chunk with no valid query
    for (int chunk = (chunk0 > first_pad ? chunk0 : first_pad); chunk < chunk_end; ++chunk) {
        const int i = chunk * kLdsQueries + ql;
        if (i < L && s == 0) M[(size_t)head * L + i] = 0.f;
        if (tid < kD) put_v(vpart + ((size_t)head * chunks_per_head + chunk) * kD + tid, 0.0);
        if (cand) {
            uint2* co = cand + ((size_t)head * chunks_per_head + chunk) * cand_len;
            for (int t = tid; t < cand_len; t += kQuadThreads) put_c(co + t, 0u, 0xFFFFFFFFu);
        }
    }
    chunk_end = chunk_end < first_pad ? chunk_end : first_pad;
    if (chunk0 >= chunk_end) return;                      // work-group-uniform

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(K + (size_t)head * L * kD);
    const unsigned char* Qb = reinterpret_cast<const unsigned char*>(Q + (size_t)head * L * kD);
    const T* Vh = V + (size_t)head * L * kD;
    // byte offset of this lane's v-th piece inside a row: piece (v + quad index) mod NP, bytes 16 s .. 16 s + 15 of it
    auto piece_ofs = [&](int v) -> uint32_t { return 64u * (uint32_t)((v + qrot) & (NP - 1)) + 16u * (uint32_t)s; };

    // ---- All loads of a chunk are issued back to back, unconditionally and on
    // clamped addresses, before anything uses them: a load inside a branch (or
    // sunk into one by the compiler) costs a full round trip of its own.
    //   q pieces and first sample indices of this lane's query (lane s of a quad
    //   holds samples 4k + s), this chunk's V rows for the column sums;
    // before the first chunk also K[0 .. n) of the head (16 bytes per thread, 16 in
    // flight; rows >= n are never read).  The loads of the next chunk are issued
    // before the current one is worked on.
    constexpr int VLPR = RT::kRowBytes / 16, VEPL = kD / VLPR, VRPP = kQuadThreads / VLPR, VN = kLdsQueries / VRPP;
    constexpr int KPRE = 10;                              // sample rounds fetched up front (U <= 40)
    const int n_r = (U + 3) >> 2;
    const int vsub = tid % VLPR, vrow = tid / VLPR;
    struct ChunkLoads { Vec q[NP]; int jraw[KPRE]; Vec vbuf[VN]; };
    auto issue = [&](int chunk, ChunkLoads& c) {
        const int i = chunk * kLdsQueries + ql;
        const int ic = i < n ? i : 0;                     // n > 0 here
#pragma unroll
        for (int v = 0; v < NP; ++v)
            c.q[v] = *reinterpret_cast<const Vec*>(Qb + (size_t)ic * RT::kRowBytes + piece_ofs(v));
        const int* irow = idx + ((size_t)head * L + (i < L ? i : 0)) * U;
#pragma unroll
        for (int k = 0; k < KPRE; ++k) { const int t = 4 * k + s; c.jraw[k] = irow[t < U ? t : U - 1]; }
#pragma unroll
        for (int k = 0; k < VN; ++k) {
            const int j = chunk * kLdsQueries + vrow + k * VRPP;
            c.vbuf[k] = reinterpret_cast<const Vec*>(Vh + (size_t)(j < n ? j : n - 1) * kD)[vsub];
        }
    };

    PSA_TS(0);
    ChunkLoads cur, nxt;
    issue(chunk0, cur);
    {
        const int n_chunks16 = n * (RT::kRowBytes / 16);
        uint4 buf[KCOPY];
#pragma unroll
        for (int k = 0; k < KCOPY; ++k) {
            const int ci = k * kQuadThreads + tid;
            buf[k] = reinterpret_cast<const uint4*>(Kb)[ci < n_chunks16 ? ci : n_chunks16 - 1];
        }
        PSA_TS(1);
        // ---- K -> LDS (the LDS area spans KCOPY * 8 KB, so the store needs no guard)
#pragma unroll
        for (int k = 0; k < KCOPY; ++k) reinterpret_cast<uint4*>(sK)[k * kQuadThreads + tid] = buf[k];
    }

    for (int chunk = chunk0; chunk < chunk_end; ++chunk) {
        const int i = chunk * kLdsQueries + ql;
        const bool in_tensor = i < L;
        const bool active = i < n;
        const int* irow = idx + ((size_t)head * L + (in_tensor ? i : 0)) * U;
        uint2* cand_out = cand ? cand + ((size_t)head * chunks_per_head + chunk) * cand_len : nullptr;

        // ---- column sums of this chunk's valid V rows, float64: per wave, then across waves
        {
            double acc[VEPL];
#pragma unroll
            for (int e = 0; e < VEPL; ++e) acc[e] = 0.0;
#pragma unroll
            for (int k = 0; k < VN; ++k) {
                const bool vok = chunk * kLdsQueries + vrow + k * VRPP < n;
                if constexpr (sizeof(T) == 4) {
                    const float4 v = cur.vbuf[k];
                    acc[0] += vok ? (double)v.x : 0.0; acc[1] += vok ? (double)v.y : 0.0;
                    acc[2] += vok ? (double)v.z : 0.0; acc[3] += vok ? (double)v.w : 0.0;
                } else {
                    const uint4 v = cur.vbuf[k];
                    acc[0] += vok ? (double)bf16_lo(v.x) : 0.0; acc[1] += vok ? (double)bf16_hi(v.x) : 0.0;
                    acc[2] += vok ? (double)bf16_lo(v.y) : 0.0; acc[3] += vok ? (double)bf16_hi(v.y) : 0.0;
                    acc[4] += vok ? (double)bf16_lo(v.z) : 0.0; acc[5] += vok ? (double)bf16_hi(v.z) : 0.0;
                    acc[6] += vok ? (double)bf16_lo(v.w) : 0.0; acc[7] += vok ? (double)bf16_hi(v.w) : 0.0;
                }
            }
#pragma unroll
            for (int off = VLPR; off < 64; off <<= 1)
#pragma unroll
                for (int e = 0; e < VEPL; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
            if (lane < VLPR) {
#pragma unroll
                for (int e = 0; e < VEPL; ++e) s_red[wave][vsub * VEPL + e] = acc[e];
            }
        }
        Vec q[NP];
        int jraw[KPRE];
#pragma unroll
        for (int v = 0; v < NP; ++v) q[v] = active ? cur.q[v] : Vec{};
#pragma unroll
        for (int k = 0; k < KPRE; ++k) jraw[k] = cur.jraw[k];
        // the next chunk's loads travel while this one is gathered (work-group-uniform branch)
        if (chunk + 1 < chunk_end) issue(chunk + 1, nxt);
        PSA_TS(2);
        lds_barrier();                                    // K and the V sums are in LDS
        PSA_TS(3);
        if (tid < kD) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < kQuadThreads / 64; ++w) t += s_red[w][tid];           // fixed order
            put_v(vpart + ((size_t)head * chunks_per_head + chunk) * kD + tid, t);
        }

        float mx = -INFINITY, sm = 0.f;
        int cnt = 0;
        auto row_dot = [&](const Vec (&kr)[NP]) -> float {           // this lane's share of q . k
            float d = 0.f;
#pragma unroll
            for (int v = 0; v < NP; ++v) {
                if constexpr (sizeof(T) == 4) {
                    d = fmaf(q[v].x, kr[v].x, d); d = fmaf(q[v].y, kr[v].y, d);
                    d = fmaf(q[v].z, kr[v].z, d); d = fmaf(q[v].w, kr[v].w, d);
                } else {
                    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].x), __builtin_bit_cast(bf16x2, kr[v].x), d, false);
                    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].y), __builtin_bit_cast(bf16x2, kr[v].y), d, false);
                    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].z), __builtin_bit_cast(bf16x2, kr[v].z), d, false);
                    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q[v].w), __builtin_bit_cast(bf16x2, kr[v].w), d, false);
                }
            }
            return d;
        };
        // one round of 4 samples: jv is sample 4k + s of this lane's query, -1 if none
        auto gather_round = [&](int jv) {
            const int j[4] = {quad_bcast<0>(jv), quad_bcast<1>(jv), quad_bcast<2>(jv), quad_bcast<3>(jv)};
            if (__ballot((unsigned)jv >= (unsigned)n) == 0ull) {
                // every sample of this round is usable in every query of the wave
                Vec kr[4][NP];
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int v = 0; v < NP; ++v)
                        kr[t][v] = *reinterpret_cast<const Vec*>(sK + (uint32_t)j[t] * RT::kRowBytes + piece_ofs(v));
                float d[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] = row_dot(kr[t]);
                // sums over the quad, one exchange stage at a time for all rows; the 1/sqrt(64) is
                // applied once at the end (exact: a power of 2)
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0xB1>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) d[t] += dpp_mov<0x4E>(d[t]);
#pragma unroll
                for (int t = 0; t < 4; ++t) { mx = fmaxf(mx, d[t]); sm += d[t]; }
                cnt += 4;
            } else {
                // padded queries, the tail of U, or indices outside [0, n): drop those samples
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bool ok = (unsigned)j[t] < (unsigned)n;
                    Vec kr[NP];
#pragma unroll
                    for (int v = 0; v < NP; ++v)
                        kr[v] = *reinterpret_cast<const Vec*>(sK + (uint32_t)(ok ? j[t] : 0) * RT::kRowBytes + piece_ofs(v));
                    const float sc = quad_sum(row_dot(kr));
                    mx = ok ? fmaxf(mx, sc) : mx;
                    sm += ok ? sc : 0.f;
                    cnt += ok ? 1 : 0;
                }
            }
        };
        // Rounds whose indices came with the chunk's other loads (no global load in this loop: the
        // wait for it would also wait for the next chunk's loads, which are in flight on purpose).
        const int n_pre = n_r < KPRE ? n_r : KPRE;
#pragma unroll 1
        for (int k = 0; k < n_pre; ++k) {
            int raw = jraw[KPRE - 1];
#pragma unroll
            for (int kk = 0; kk < KPRE - 1; ++kk) raw = (k == kk) ? jraw[kk] : raw;
            gather_round((active && 4 * k + s < U) ? raw : -1);
        }
        // only for U > 40: the remaining rounds, their indices fetched here
#pragma unroll 1
        for (int k = KPRE; k < n_r; ++k) {
            const int t = 4 * k + s;
            const int raw = irow[t < U ? t : U - 1];
            gather_round((active && t < U) ? raw : -1);
        }
        PSA_TS(4);
        float m = 0.f;
        if (active && cnt > 0) m = (mx - sm / (float)cnt) * 0.125f;         // 1/sqrt(64), exact
        if (in_tensor && s == 0) M[(size_t)head * L + i] = m;

        // ---- local ranking for stage a2.  Any query among the head's u largest is
        // among its own chunk's u largest, so each chunk hands on only its first
        // cand_len queries in order of decreasing measure (ties: lower index first),
        // as (order key, query index) pairs; the attend stage merges the few sorted
        // lists of a head instead of selecting among all L measures.
        {
            float f = m + 0.0f;                                         // -0 -> +0
            const unsigned ub = __float_as_uint(f);
            const unsigned key = active ? ((ub & 0x80000000u) ? ~ub : (ub | 0x80000000u)) : 0u;   // 0 = not a candidate
            if (s == 0) s_key[ql] = ((unsigned long long)key << 32) | (unsigned)~ql;      // equal keys: the lower query is larger
        }
        PSA_TS(5);
        lds_barrier();                       // also: every wave is done with s_red before the next chunk writes it
        PSA_TS(6);
        if (cand_out) {
            const unsigned long long mine64 = s_key[ql];
            const unsigned mine = (unsigned)(mine64 >> 32);
            int beat = 0;                                               // chunk-mates that come before this query
#pragma unroll
            for (int t = 0; t < kLdsQueries / 4; ++t)
                beat += s_key[4 * t + s] > mine64 ? 1 : 0;              // (adjacent words for the quad's lanes: no bank conflict)
            beat += __builtin_amdgcn_update_dpp(0, beat, 0xB1, 0xF, 0xF, false);     // sum over the quad
            beat += __builtin_amdgcn_update_dpp(0, beat, 0x4E, 0xF, 0xF, false);
            if (s == 0 && mine != 0u && beat < cand_len) put_c(cand_out + beat, mine, (unsigned)i);
            // slots beyond the chunk's valid queries are marked empty
            const int n_here = n - chunk * kLdsQueries < kLdsQueries ? n - chunk * kLdsQueries : kLdsQueries;
            for (int t = n_here + tid; t < cand_len; t += kQuadThreads) put_c(cand_out + t, 0u, 0xFFFFFFFFu);
        }
        cur = nxt;
        // the ranking reads s_key; the next chunk writes it only after its own first barrier
    }
    PSA_TS(7);
}

// KCOPY: 16-byte pieces of K per thread = LDS bytes / 8 KB (see measure_quad_body).
template <typename T, int KCOPY>
__global__ __launch_bounds__(kQuadThreads, (KCOPY == 8 && sizeof(T) == 2) ? 4 : 2)
void measure_quad_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                         const int* __restrict__ lengths, const int* __restrict__ idx,
                         float* __restrict__ M, double* __restrict__ vpart, int* __restrict__ ticket,
                         uint2* __restrict__ cand, int cand_len,
                         int H, int L, int U, int chunks_per_head, int chunks_per_wg, int n_heads)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char sK[];    // [n][row bytes]
    __shared__ double s_red[kQuadThreads / 64][kD];
    __shared__ unsigned long long s_key[kLdsQueries];
    // A work-group takes chunks_per_wg consecutive chunks of one head (the head's K
    // goes to LDS once for all of them); all work-groups of a head sit on one XCD.
    const int groups_per_head = (chunks_per_head + chunks_per_wg - 1) / chunks_per_wg;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int head = (slot / groups_per_head) * 8 + xcd;
    const int chunk0 = (slot % groups_per_head) * chunks_per_wg;
    if (head >= n_heads) return;
    if (chunk0 == 0 && threadIdx.x == 0) ticket[head] = 0;        // the attend stage counts work-groups per head
    measure_quad_body<T, KCOPY>(Q, K, V, lengths, idx, M, vpart, cand, cand_len, H, L, U, chunks_per_head,
                                       chunks_per_wg, head, chunk0, sK, s_red, s_key);
}

// The LDS measure kernel with 128 KB of K is above the default 64 KB of dynamic LDS.
template <typename T>
static hipError_t raise_measure_limit()
{
    static std::atomic<uint64_t> raised;               // per instantiation: devices already served
    return ensure_lds_limit((const void*)measure_quad_kernel<T, 16>, kLdsMaxBytes, raised);
}


// The streaming kernel's two LDS stages reach 64 KB at 64 samples per query in float32.
template <typename T>
static hipError_t raise_pipe_limit()
{
    static std::atomic<uint64_t> raised;               // per instantiation: devices already served
    return ensure_lds_limit((const void*)measure_pipe_kernel<T>, 2 * pipe_stage_bytes<T>(kPipeMaxU), raised);
}
hipError_t init_measure()
{
    hipError_t e = raise_measure_limit<float>();
    if (e == hipSuccess) e = raise_measure_limit<bf16_t>();
    if (e == hipSuccess) e = raise_pipe_limit<float>();
    if (e == hipSuccess) e = raise_pipe_limit<bf16_t>();
    return e;
}

template <typename T>
static hipError_t launch_measure_t(const Plan& p, const Args& a, const Scratch& w)
{
    const int head_rounds = (p.BH + 7) / 8;
    if (p.measure_lds) {
        const int chunks = p.n_chunk;                      // ceil(L / 128)
        const int groups = (chunks + p.chunks_per_wg - 1) / p.chunks_per_wg;
        dim3 grid((unsigned)(head_rounds * groups * 8)), block(kQuadThreads);
        uint2* cand = p.cand_len > 0 ? w.cand : nullptr;
        if (p.measure_lds == 2) {                         // K of a head within 64 KB: two work-groups per CU
            hipLaunchKernelGGL((measure_quad_kernel<T, 8>), grid, block, kLdsMaxBytes / 2, a.stream,
                               (const T*)a.Q, (const T*)a.K, (const T*)a.V, a.lengths, a.idx, w.M, w.vpart, w.ticket,
                               cand, p.cand_len, p.H, p.L, p.U, chunks, p.chunks_per_wg, p.BH);
            return hipGetLastError();
        }
        const hipError_t e = raise_measure_limit<T>();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((measure_quad_kernel<T, 16>), grid, block, kLdsMaxBytes, a.stream,
                           (const T*)a.Q, (const T*)a.K, (const T*)a.V, a.lengths, a.idx, w.M, w.vpart, w.ticket,
                           cand, p.cand_len, p.H, p.L, p.U, chunks, p.chunks_per_wg, p.BH);
        return hipGetLastError();
    }
    const int chunks = p.n_chunk;                          // ceil(L / 64)
    // up to 64 samples per query: persistent work-groups with loader waves; beyond, one work-group per chunk
    if (p.U <= kPipeMaxU) {
        const int groups = (chunks + p.chunks_per_wg - 1) / p.chunks_per_wg;
        const int lds = 2 * pipe_stage_bytes<T>(p.U);
        const hipError_t e = raise_pipe_limit<T>();
        if (e != hipSuccess) return e;
        dim3 grid((unsigned)(head_rounds * groups * 8)), block(kPipeThreads);
        hipLaunchKernelGGL(measure_pipe_kernel<T>, grid, block, lds, a.stream,
                           (const T*)a.Q, (const T*)a.K, (const T*)a.V, a.lengths, a.idx, w.M, w.vpart, w.ticket,
                           p.stream_lists ? w.cand : nullptr, p.cand_len, w.vseg,
                           p.H, p.L, p.U, chunks, p.chunks_per_wg, p.BH);
        return hipGetLastError();
    }
    dim3 grid((unsigned)(head_rounds * chunks * 8)), block(kStreamThreads);
    hipLaunchKernelGGL(measure_stream_kernel<T>, grid, block, 0, a.stream,
                       (const T*)a.Q, (const T*)a.K, (const T*)a.V, a.lengths, a.idx, w.M, w.vpart, w.ticket,
                       p.H, p.L, p.U, chunks, p.BH);
    return hipGetLastError();
}

// The by-products of the measure stage without the measure (caller-given index
// sets): column sums of the valid V rows per chunk of kMeasureQueries rows, and
// the head's ticket counter at zero.
template <typename T>
__global__ __launch_bounds__(256)
void vsum_kernel(const T* __restrict__ V, const int* __restrict__ lengths, double* __restrict__ vpart,
                 int* __restrict__ ticket, int H, int L, int chunks_per_head)
{
    __shared__ double s_red[4][kD];
    const int chunk = blockIdx.x, head = blockIdx.y;
    const int n = valid_len(lengths, head / H, L);
    if (chunk == 0 && threadIdx.x == 0) ticket[head] = 0;
    block_v_colsum<T, 256>(V + (size_t)head * L * kD, chunk * kMeasureQueries, kMeasureQueries, n,
                           vpart + ((size_t)head * chunks_per_head + chunk) * kD, s_red);
}

hipError_t launch_vsum(const Plan& p, const Args& a, const Scratch& w)
{
    const dim3 grid(p.n_chunk, p.BH);
    if (p.dtype == PSA_F32)
        hipLaunchKernelGGL(vsum_kernel<float>, grid, dim3(256), 0, a.stream, static_cast<const float*>(a.V), a.lengths,
                           w.vpart, w.ticket, p.H, p.L, p.n_chunk);
    else
        hipLaunchKernelGGL(vsum_kernel<bf16_t>, grid, dim3(256), 0, a.stream, static_cast<const bf16_t*>(a.V), a.lengths,
                           w.vpart, w.ticket, p.H, p.L, p.n_chunk);
    return hipGetLastError();
}

hipError_t launch_measure(const Plan& p, const Args& a, const Scratch& w)
{
    return p.dtype == PSA_F32 ? launch_measure_t<float>(p, a, w) : launch_measure_t<bf16_t>(p, a, w);
}

}  // namespace psa

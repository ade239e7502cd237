// Stage a1: scores of every query against its sampled keys and the sampled
// sparsity measure  M_i = max_t s_it - (1/#samples) sum_t s_it  (Sec. 3.2, Eq. 11).
// By-product for stage a4: float64 column sums of the valid V rows, per chunk.
//
// This is a gather, not a contraction: each query touches U random key rows of
// its own head.  The streaming kernel gives a query to 8 adjacent lanes:
//   * a key row (256 B f32 / 128 B bf16) is read 128 bytes at a time, lane s of
//     the 8 taking bytes 16s .. 16s+15, so that one load instruction takes a
//     whole 128-byte line for each of the wave's 8 queries;
//   * the lanes keep the matching chunks of the query in registers, the dot
//     product is finished with three DPP exchanges, and the sample index
//     travels from the lane that loaded it to the other seven by a lane shuffle;
//   * 8 samples are in flight per round.
// Heads whose K fits in LDS gather from an LDS copy of K with 4 lanes per query
// (measure_quad_kernel), longer heads through L1 from the head's XCD-local L2
// (measure_kernel).
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

template <typename T>
__global__ __launch_bounds__(kStreamThreads)
void measure_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                    const int* __restrict__ lengths, const int* __restrict__ idx,
                    float* __restrict__ M, double* __restrict__ vpart, int* __restrict__ ticket,
                    int H, int L, int U, int chunks_per_head, int n_heads)
{
    using RT = RowTraits<T>;
    using Vec = typename std::conditional<sizeof(T) == 4, float4, uint4>::type;
    constexpr int NCH = RT::kRowBytes / 128;      // 16-byte chunks per lane: 8 lanes cover 128 bytes of a row

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
    const int s = lane & 7, gbase = lane & ~7;
    const int i = chunk * kMeasureQueries + wave * kQueriesPerWave + (lane >> 3);
    const bool in_tensor = i < L;
    const bool active = i < n;

    // by-products for the attend stage: the head's ticket counter starts at zero,
    // and the column sums of this chunk's valid V rows
    __shared__ double s_red[kStreamThreads / 64][kD];
    PSA_TS(0);
    if (chunk == 0 && tid == 0) ticket[head] = 0;
    block_v_colsum<T, kStreamThreads>(V + (size_t)head * L * kD, chunk * kMeasureQueries, kMeasureQueries, n,
                                      vpart + ((size_t)head * chunks_per_head + chunk) * kD, s_red);
    PSA_TS(1);

    // a wave whose queries are all padding has nothing to fetch
    if (__ballot(active) == 0ull) {
        if (in_tensor && s == 0) M[(size_t)head * L + i] = 0.f;
        return;
    }

    const unsigned char* Kb = reinterpret_cast<const unsigned char*>(K + (size_t)head * L * kD);
    const unsigned char* Qb = reinterpret_cast<const unsigned char*>(Q + (size_t)head * L * kD);
    const int* irow = idx + ((size_t)head * L + (in_tensor ? i : 0)) * U;

    // lane s of the query's 8 lanes holds bytes 16s .. 16s+15 of every 128 bytes of a row, so
    // that one load instruction takes whole 128-byte lines, one per query of the wave
    Vec q[NCH];
#pragma unroll
    for (int v = 0; v < NCH; ++v)
        q[v] = *reinterpret_cast<const Vec*>(Qb + (size_t)(active ? i : 0) * RT::kRowBytes + 16 * s + 128 * v);   // clamped
    if (!active) {
#pragma unroll
        for (int v = 0; v < NCH; ++v) q[v] = Vec{};
    }

    float mx = -INFINITY, sm = 0.f;
    int cnt = 0;
    // Lane s fetches sample 8k + s; a round consumes one block k of 8 samples.
    const int n_k = (U + 7) >> 3;
    auto fetch_idx = [&](int k) -> int {
        const int t = 8 * k + s;
        const int v = irow[t < U ? t : U - 1];                      // clamped, unconditional
        return (active && t < U) ? v : -1;
    };
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
    int jv = fetch_idx(0), jn = fetch_idx(1);
    PSA_TS(2);
    for (int k = 0; k < n_k; ++k) {
        const int jnn = fetch_idx(k + 2);                           // two rounds ahead
        int j[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) j[t] = __shfl(jv, gbase + t, 64);
        Vec kr[8][NCH];
        if (__ballot((unsigned)jv >= (unsigned)n) == 0ull) {
            // every sample of this round is usable in every query of the wave
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int v = 0; v < NCH; ++v)
                    kr[t][v] = *reinterpret_cast<const Vec*>(Kb + (uint32_t)j[t] * RT::kRowBytes + 16u * s + 128u * v);
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
            // padded queries, the tail of U, or indices outside [0, n): drop those samples
            bool ok[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                ok[t] = (unsigned)j[t] < (unsigned)n;
#pragma unroll
                for (int v = 0; v < NCH; ++v)
                    kr[t][v] = *reinterpret_cast<const Vec*>(Kb + (uint32_t)(ok[t] ? j[t] : 0) * RT::kRowBytes + 16u * s + 128u * v);
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const float sc = group_sum8(row_dot(kr[t]));
                mx = ok[t] ? fmaxf(mx, sc) : mx;
                sm += ok[t] ? sc : 0.f;
                cnt += ok[t] ? 1 : 0;
            }
        }
        jv = jn; jn = jnn;
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

__device__ __forceinline__ float quad_sum(float x) {
    x += dpp_mov<0xB1>(x);
    x += dpp_mov<0x4E>(x);
    return x;
}
template <int T4>                                          // value of lane T4 of the quad, in all four lanes
__device__ __forceinline__ int quad_bcast(int x) {
    return __builtin_amdgcn_update_dpp(0, x, T4 * 0x55, 0xF, 0xF, false);
}

// KCOPY: 16-byte pieces of K per thread = LDS bytes / 8 KB: 16 (a head of up to 128 KB) or 8 (up
// to 64 KB).  With 64 KB two work-groups fit a CU; for bfloat16 rows the registers are capped to
// let them (4 waves per SIMD), so that one work-group copies its K while
// the other gathers.
template <typename T, int KCOPY>
__global__ __launch_bounds__(kQuadThreads, (KCOPY == 8 && sizeof(T) == 2) ? 4 : 2)
void measure_quad_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                         const int* __restrict__ lengths, const int* __restrict__ idx,
                         float* __restrict__ M, double* __restrict__ vpart, int* __restrict__ ticket,
                         uint2* __restrict__ cand, int cand_len,
                         int H, int L, int U, int chunks_per_head, int chunks_per_wg, int n_heads)
{
    using RT = RowTraits<T>;
    using Vec = typename std::conditional<sizeof(T) == 4, float4, uint4>::type;
    constexpr int NP = RT::kRowBytes / 64;               // 16-byte pieces per lane and row: 4 (f32) or 2 (bf16)
    static_assert(KCOPY * 16 * kQuadThreads <= kLdsMaxBytes, "at most 128 KB of K");
    extern __shared__ __attribute__((aligned(16))) unsigned char sK[];    // [n][row bytes]

    // A work-group takes chunks_per_wg consecutive chunks of one head (the head's K
    // goes to LDS once for all of them); all work-groups of a head sit on one XCD.
    const int groups_per_head = (chunks_per_head + chunks_per_wg - 1) / chunks_per_wg;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int head = (slot / groups_per_head) * 8 + xcd;
    const int chunk0 = (slot % groups_per_head) * chunks_per_wg;
    if (head >= n_heads) return;
    int chunk_end = chunk0 + chunks_per_wg;
    chunk_end = chunk_end < chunks_per_head ? chunk_end : chunks_per_head;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int s = lane & 3;
    const int qrot = (lane >> 2) & (RT::kRowBytes / 64 - 1);           // the quad's rotation of the piece order
    const int ql = wave * kQuadQueriesPerWave + (lane >> 2);            // query within a chunk
    __shared__ double s_red[kQuadThreads / 64][kD];
    __shared__ unsigned long long s_key[kLdsQueries];     // (order key, ~query) of a chunk's measures: one 64-bit compare ranks
    if (chunk0 == 0 && tid == 0) ticket[head] = 0;        // the attend stage counts work-groups per head

    // chunks that are padding as a whole (all of them, once one is: chunks ascend)
    const int first_pad = (n + kLdsQueries - 1) / kLdsQueries;          // first chunk with no valid query
    for (int chunk = (chunk0 > first_pad ? chunk0 : first_pad); chunk < chunk_end; ++chunk) {
        const int i = chunk * kLdsQueries + ql;
        if (i < L && s == 0) M[(size_t)head * L + i] = 0.f;
        if (tid < kD) vpart[((size_t)head * chunks_per_head + chunk) * kD + tid] = 0.0;
        if (cand) {
            uint2* co = cand + ((size_t)head * chunks_per_head + chunk) * cand_len;
            for (int t = tid; t < cand_len; t += kQuadThreads) co[t] = make_uint2(0u, 0xFFFFFFFFu);
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
        v_colsum_finish<kQuadThreads>(vpart + ((size_t)head * chunks_per_head + chunk) * kD, s_red);

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
            if (s == 0 && mine != 0u && beat < cand_len) cand_out[beat] = make_uint2(mine, (unsigned)i);
            // slots beyond the chunk's valid queries are marked empty
            const int n_here = n - chunk * kLdsQueries < kLdsQueries ? n - chunk * kLdsQueries : kLdsQueries;
            for (int t = n_here + tid; t < cand_len; t += kQuadThreads) cand_out[t] = make_uint2(0u, 0xFFFFFFFFu);
        }
        cur = nxt;
        // the ranking reads s_key; the next chunk writes it only after its own first barrier
    }
    PSA_TS(7);
}

// The LDS measure kernel with 128 KB of K is above the default 64 KB of dynamic LDS.
template <typename T>
static hipError_t raise_measure_limit()
{
    static std::atomic<uint64_t> raised;               // per instantiation: devices already served
    return ensure_lds_limit((const void*)measure_quad_kernel<T, 16>, kLdsMaxBytes, raised);
}
hipError_t init_measure()
{
    const hipError_t e = raise_measure_limit<float>();
    return e != hipSuccess ? e : raise_measure_limit<bf16_t>();
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
    dim3 grid((unsigned)(head_rounds * chunks * 8)), block(kStreamThreads);
    hipLaunchKernelGGL(measure_kernel<T>, grid, block, 0, a.stream,
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

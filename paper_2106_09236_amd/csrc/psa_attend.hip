// Stage a3: softmax attention of the selected queries over all valid keys
// (Eq. 7, Eq. 8, upper branch of Eq. 12), as partial results per key split.
//
// The two products  S = Q_sel K^T  and  O = P V  are contractions and run on the
// matrix cores.  Both are computed TRANSPOSED, with the selected queries on the
// column axis of the MFMA tiles:
//     S^T[key, q] = sum_e K[key, e] Q_sel[q, e]          A = K tile,   B = Q_sel^T
//     O^T[e,  q] = sum_key V[key, e] P[q, key]           A = V tile^T, B = P^T
// A lane of an MFMA accumulator holds one column, so every value a lane ever
// owns belongs to ONE query: running max, running sum and the rescale of online
// softmax are per-lane scalars, and the S^T accumulator registers are, unchanged,
// the B operand of the second product (their row order is taken as that
// product's contraction order; the V operand is fetched in the same order).
//
// Precision.  The parity bound for float32 tensors (1e-4 relative with a floor
// of 1e-2 RMS, element by element) is tighter than a float32 accumulation chain
// over hundreds of keys can promise, so float32 inputs are widened (exactly) to
// float64 and both products use v_mfma_f64_16x16x4; the exponent is evaluated in
// float64 as well.  bfloat16 inputs use v_mfma_f32_32x32x16_bf16 with float32
// accumulation; the probabilities are split into two bfloat16 terms (hi + lo)
// so that P keeps 16 significant bits in the second product.
//
// A work-group is 4 waves; each wave walks `tiles_per_wave` tiles of 32 keys
// with its own LDS staging area (no work-group barrier inside the loop), then
// the four waves' (m, l, O) are merged through LDS and one partial record per
// (head, query group, key split) goes to the workspace.  Records are merged in a
// fixed order by the finalize stage, so results do not depend on scheduling.
#include "psa_attend_common.h"

namespace psa {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr float  kScaleLog2e  = 0.125f * 1.4426950408889634f;   // (1/sqrt(64)) * log2(e)
constexpr double kScaleLog2eD = 0.125 * 1.4426950408889634074;

// 2^x on the transcendental unit; -inf -> 0, no denormal handling needed here
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int kOStride = 65;          // elements per query row in the merge area (odd: no bank conflicts)

// =============================================================================
// float32 tensors: float64 matrix cores, 16x16x4 tiles
//   lane (c, g) = (lane % 16, lane / 16)
//   A[i][k]: i = c, k = g      B[k][j]: k = g, j = c      D[i][j]: i = 4r + g, j = c  (r = 0..3)
// The kernel is bound by the float64 MFMA rate, so operands go straight from
// global memory to registers (each lane reads 64 contiguous bytes of its K row)
// and the work is cut fine: a work-group is 8 waves, wave w owns ONE column tile
// of 16 selected queries (ct = w % NCG) and one 32-key tile per round
// (kt = w / NCG), which puts two waves on every SIMD to overlap each other's
// loads, exponentials and merges.
// =============================================================================
constexpr int kF32Waves = 8;
constexpr int kStateDoubles = 18;      // m, l, 16 accumulator values per lane
constexpr int kF32SmemBytes = kF32Waves * kStateDoubles * 64 * 8;     // 73728: dynamic LDS

// Record layout for float32 tensors (doubles), NQ = 16 * NCG queries:
//   [ m[NQ] | l[NQ] | O: per column tile ct a block of 1024 = [16 registers][64 lanes] ]
// element e of query q: block q / 16, register e / 4, lane (e % 4) * 16 + q % 16,
// i.e. exactly the accumulator layout, so record stores are fully coalesced.
template <int NCG>      // column tiles of 16 selected queries per query group: 1 or 2
__global__ __launch_bounds__(512)
void attend_f32_kernel(const AttendParams P)
{
    const float* Q = static_cast<const float*>(P.Q);
    const float* K = static_cast<const float*>(P.K);
    const float* V = static_cast<const float*>(P.V);
    double* part = static_cast<double*>(P.part);
    const int H = P.H, L = P.L, n_split = P.n_split, n_qgroup = P.n_qgroup, rounds = P.rounds, part_stride = P.part_stride;
    __shared__ CommonScratch<512> cs;
    constexpr int NQ = NCG * 16;
    constexpr int KT = kF32Waves / NCG;                 // key tiles per round of the work-group
    constexpr int VPW = 16 / KT;                        // accumulator values each wave merges
    extern __shared__ __attribute__((aligned(16))) double smem[];     // [wave][kStateDoubles][64]

    const int split = blockIdx.x, qgroup = blockIdx.y, head = blockIdx.z;
    const int b = head / H;
    const int n = valid_len(P.lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int ct = wave % NCG, kt = wave / NCG;
    const int wg_in_head = qgroup * n_split + split;

    const float* Qh = Q + (size_t)head * L * kD;
    const float* Kh = K + (size_t)head * L * kD;
    const float* Vh = V + (size_t)head * L * kD;

    // Operands of one 32-key tile, straight from global memory.
    //   kreg[sb][v]     : key j0 + 16sb + c, elements 16v + 4g .. +3   (A of the first product; the
    //                     contraction order is free, and this one makes the four lanes g of a
    //                     row read 64 contiguous bytes per load instruction)
    //   vreg[sb][dt][r] : key j0 + 16sb + 4r + g, element 16dt + c     (A of the second product;
    //                     4r + g is the row order of the S^T accumulator registers)
    float4 kreg[2][4];
    float vreg[2][4][4];
    auto load_k = [&](int j0) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            // loads are unconditional on a clamped row (a guarded load would cost a
            // branch and a wait each); rows at or beyond n are zeroed afterwards
            const int j = j0 + 16 * sb + c;
            const bool ok = j < n;
            const float* row = Kh + (size_t)(ok ? j : n - 1) * kD + 4 * g;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float4 x = *reinterpret_cast<const float4*>(row + 16 * v);
                if (!ok) x = make_float4(0.f, 0.f, 0.f, 0.f);
                kreg[sb][v] = x;
            }
        }
    };
    auto load_v = [&](int j0) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = j0 + 16 * sb + 4 * r + g;
                const bool ok = j < n;
                const float* row = Vh + (size_t)(ok ? j : n - 1) * kD + c;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const float x = row[16 * dt];
                    vreg[sb][dt][r] = ok ? x : 0.f;
                }
            }
    };

    // The first K tile does not depend on the selection: it is requested first and
    // streams in while the prologue picks I_sparse.  Then the query row (needs the
    // index); the V tile is requested only once the first product has been issued,
    // so that it arrives under the MFMAs and the softmax.
    const int j_first = (split * rounds * KT + kt) * kTile;
    load_k(j_first);
    int u;
    const int* selp = attend_prologue<512>(P, head, n, wg_in_head, cs, u);
    const int qrank = qgroup * NQ + ct * 16 + c;
    const int qi = qrank < u ? selp[qrank] : -1;
    // B operand of the first product: qreg[4v + e] = Q[q][16v + 4g + e], widened
    double qreg[16];
    {
        const bool ok = qi >= 0 && qi < n;
        const float* src = Qh + (size_t)(ok ? qi : 0) * kD + 4 * g;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float4 x = *reinterpret_cast<const float4*>(src + 16 * v);
            if (!ok) x = make_float4(0.f, 0.f, 0.f, 0.f);
            qreg[4 * v + 0] = (double)x.x; qreg[4 * v + 1] = (double)x.y;
            qreg[4 * v + 2] = (double)x.z; qreg[4 * v + 3] = (double)x.w;
        }
    }

    float m_run = -INFINITY;
    double l_run = 0.0;
    doublex4 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = doublex4{0.0, 0.0, 0.0, 0.0};

    for (int rd = 0; rd < rounds; ++rd) {
        const int j0 = ((split * rounds + rd) * KT + kt) * kTile;
        if (j0 >= n) break;                                   // wave-uniform
        if (rd > 0) load_k(j0);

        // first product for both 16-key sub-tiles: two independent MFMA chains
        doublex4 s[2];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) s[sb] = doublex4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int sb = 0; sb < 2; ++sb) {
                s[sb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)kreg[sb][v].x, qreg[4 * v + 0], s[sb], 0, 0, 0);
                s[sb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)kreg[sb][v].y, qreg[4 * v + 1], s[sb], 0, 0, 0);
                s[sb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)kreg[sb][v].z, qreg[4 * v + 2], s[sb], 0, 0, 0);
                s[sb] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)kreg[sb][v].w, qreg[4 * v + 3], s[sb], 0, 0, 0);
            }
        }
        load_v(j0);
        // online softmax in base 2 over the 32 keys.  The subtracted constant only
        // has to be the same for every key of a query, so the running max is kept
        // in float32 while the exponent itself is formed in float64.
        double t[2][4];
        bool ok[2][4];
        float tmax = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ok[sb][r] = (j0 + 16 * sb + 4 * r + g) < n;
                t[sb][r] = s[sb][r] * kScaleLog2eD;
                if (ok[sb][r]) tmax = fmaxf(tmax, (float)t[sb][r]);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(m_run, tmax);               // finite: key j0 is valid
        const double alpha = exp2_f64((double)m_run - (double)m_new);
        double p[2][4], lsum = 0.0;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[sb][r] = ok[sb][r] ? exp2_f64(t[sb][r] - (double)m_new) : 0.0;
                lsum += p[sb][r];
            }
        l_run = l_run * alpha + lsum;
        m_run = m_new;
        // second product: four independent chains (one per 16 output elements)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] *= alpha;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    oacc[dt] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)vreg[sb][dt][r], p[sb][r], oacc[dt], 0, 0, 0);
    }

    // ---- merge the KT waves that share a column tile.  Every wave publishes its
    // state (m, l, 16 accumulator values per lane) in register layout, then wave
    // kt merges accumulator values kt*VPW .. +VPW of all KT states and stores them.
    double* mine = smem + (size_t)wave * kStateDoubles * 64;
    mine[0 * 64 + lane] = (double)m_run;
    mine[1 * 64 + lane] = l_run;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) mine[(2 + 4 * dt + r) * 64 + lane] = oacc[dt][r];
    __syncthreads();

    double wgt[KT], mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < KT; ++w) {
        wgt[w] = smem[(size_t)(w * NCG + ct) * kStateDoubles * 64 + lane];       // m of wave (w, ct)
        mx = fmax(mx, wgt[w]);
    }
#pragma unroll
    for (int w = 0; w < KT; ++w) wgt[w] = (wgt[w] == -INFINITY) ? 0.0 : exp2_f64(wgt[w] - mx);

    double* rec = part + (((size_t)head * n_qgroup + qgroup) * n_split + split) * part_stride;
    double* rec_O = rec + 2 * NQ + ct * 1024;
#pragma unroll
    for (int k = 0; k < VPW; ++k) {
        const int vi = kt * VPW + k;
        double acc = 0.0;
#pragma unroll
        for (int w = 0; w < KT; ++w)
            acc += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 2 + vi) * 64 + lane];
        rec_store(rec_O + vi * 64 + lane, acc);
    }
    if (kt == 0) {
        double l_tot = 0.0;
#pragma unroll
        for (int w = 0; w < KT; ++w) l_tot += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 1) * 64 + lane];
        l_tot += __shfl_xor(l_tot, 16, 64);
        l_tot += __shfl_xor(l_tot, 32, 64);
        if (g == 0) { rec_store(rec + ct * 16 + c, mx); rec_store(rec + NQ + ct * 16 + c, l_tot); }
    }

    // ---- stage a4 for this work-group's share of the rows, then the hand-over
    fill_rows<float, 512>(static_cast<float*>(P.out) + (size_t)head * L * kD, selp, u, n, L,
                          wg_in_head * P.rows_per_wg, P.rows_per_wg, cs);
    ticket_and_merge<float, double, true, 512>(P, head, n, u, selp, NQ, cs);
}

// =============================================================================
// bfloat16 tensors: v_mfma_f32_32x32x16_bf16, float32 accumulation
//   lane (c, h) = (lane % 32, lane / 32)
//   A[i][k]: i = c, k = 8h + e   B[k][j]: k = 8h + e, j = c   (e = 0..7 packed in the lane)
//   D[i][j]: i = 8(r/4) + 4h + r%4, j = c   (r = 0..15)
// =============================================================================
constexpr int kB16Stride = 72;                                  // bf16 per staged row (64 + 8 pad)
constexpr int kB16WaveBytes = 2 * kTile * kB16Stride * 2;       // K and V

template <int NQT>     // column tiles of 32 selected queries per work-group
__global__ __launch_bounds__(256)
void attend_bf16_kernel(const AttendParams P)
{
    const bf16_t* Q = static_cast<const bf16_t*>(P.Q);
    const bf16_t* K = static_cast<const bf16_t*>(P.K);
    const bf16_t* V = static_cast<const bf16_t*>(P.V);
    float* part = static_cast<float*>(P.part);
    const int H = P.H, L = P.L, n_split = P.n_split, n_qgroup = P.n_qgroup, tiles_per_wave = P.rounds, part_stride = P.part_stride;
    __shared__ CommonScratch<256> cs;
    constexpr int NQ = NQT * 32;
    constexpr int kStageBytes = kWaves * kB16WaveBytes;
    constexpr int kMergeBytes = kWaves * 32 * (kOStride + 2) * 4;
    constexpr int kSmemBytes = kStageBytes > kMergeBytes ? kStageBytes : kMergeBytes;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemBytes];

    const int split = blockIdx.x, qgroup = blockIdx.y, head = blockIdx.z;
    const int b = head / H;
    const int n = valid_len(P.lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int wg_in_head = qgroup * n_split + split;
    int u;
    const int* selp = attend_prologue<256>(P, head, n, wg_in_head, cs, u);

    const bf16_t* Qh = Q + (size_t)head * L * kD;
    const bf16_t* Kh = K + (size_t)head * L * kD;
    const bf16_t* Vh = V + (size_t)head * L * kD;

    // B operand of the first product: qreg[qt][kk] = Q[q][32h + 8kk .. +8]
    uint4 qreg[NQT][4];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const int r = qgroup * NQ + qt * 32 + c;
        const int qi = r < u ? selp[r] : -1;
        const bool ok = qi >= 0 && qi < n;
        const uint4* src = reinterpret_cast<const uint4*>(Qh + (size_t)(ok ? qi : 0) * kD) + 4 * h;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            uint4 x = src[v];
            if (!ok) x = make_uint4(0u, 0u, 0u, 0u);
            qreg[qt][v] = x;
        }
    }

    float m_run[NQT], l_run[NQT];
    floatx16 oacc[NQT][2];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        m_run[qt] = -INFINITY; l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qt][dt][r] = 0.f;
    }

    uint16_t* sK = reinterpret_cast<uint16_t*>(smem + wave * kB16WaveBytes);
    uint16_t* sV = sK + kTile * kB16Stride;
    const int tile0 = (split * kWaves + wave) * tiles_per_wave;

    for (int ti = 0; ti < tiles_per_wave; ++ti) {
        const int j0 = (tile0 + ti) * kTile;
        if (j0 >= n) break;                                   // wave-uniform

        wave_lds_sync();
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = it * 8 + (lane >> 3), col8 = lane & 7;
            const int j = j0 + row;
            const bool ok = j < n;                            // clamped, unconditional loads
            const size_t ro = (size_t)(ok ? j : n - 1) * kD;
            uint4 xk = reinterpret_cast<const uint4*>(Kh + ro)[col8];
            uint4 xv = reinterpret_cast<const uint4*>(Vh + ro)[col8];
            if (!ok) { xk = make_uint4(0u, 0u, 0u, 0u); xv = xk; }
            *reinterpret_cast<uint4*>(sK + row * kB16Stride + col8 * 8) = xk;
            *reinterpret_cast<uint4*>(sV + row * kB16Stride + col8 * 8) = xv;
        }
        wave_lds_sync();

        // A operand of the second product, shared by all query tiles: for step st
        // and element e the key is 16st + 8(e/4) + 4h + e%4 (the row order of the
        // S^T accumulator registers 8st..8st+7), column 32dt + c
        uint4 vop[2][2];
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                uint32_t av[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const int e = 2 * e2;
                    const int k0 = 16 * st + 8 * (e >> 2) + 4 * h + (e & 3);
                    const uint32_t lo = sV[k0 * kB16Stride + dt * 32 + c];
                    const uint32_t hi = sV[(k0 + 1) * kB16Stride + dt * 32 + c];
                    av[e2] = lo | (hi << 16);
                }
                vop[st][dt] = make_uint4(av[0], av[1], av[2], av[3]);
            }
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            floatx16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const uint4 a = *reinterpret_cast<const uint4*>(sK + c * kB16Stride + 32 * h + 8 * kk);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, qreg[qt][kk]), s, 0, 0, 0);
            }
            // online softmax in base 2; keys at or beyond n are masked out
            float tmax = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j0 + 8 * (r >> 2) + 4 * h + (r & 3);
                s[r] = (j < n) ? s[r] * kScaleLog2e : -INFINITY;
                tmax = fmaxf(tmax, s[r]);
            }
            tmax = fmaxf(tmax, swap_half(tmax));
            const float m_new = fmaxf(m_run[qt], tmax);       // finite: key j0 is valid
            const float alpha = fast_exp2(m_run[qt] - m_new);
            float lsum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = fast_exp2(s[r] - m_new); lsum += s[r]; }
            l_run[qt] = l_run[qt] * alpha + lsum;
            m_run[qt] = m_new;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[qt][dt][r] *= alpha;
            // P = P_hi + P_lo, both bf16: 16 significant bits survive
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                uint32_t ph[4], pl[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float p0 = s[8 * st + 2 * e2], p1 = s[8 * st + 2 * e2 + 1];
                    const uint16_t h0 = f32_to_bf16(p0), h1 = f32_to_bf16(p1);
                    ph[e2] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                    pl[e2] = pack_bf16(p0 - bf16_to_f32(h0), p1 - bf16_to_f32(h1));
                }
                const bf16x8 bh = __builtin_bit_cast(bf16x8, make_uint4(ph[0], ph[1], ph[2], ph[3]));
                const bf16x8 bl = __builtin_bit_cast(bf16x8, make_uint4(pl[0], pl[1], pl[2], pl[3]));
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, vop[st][dt]);
                    oacc[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bh, oacc[qt][dt], 0, 0, 0);
                    oacc[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bl, oacc[qt][dt], 0, 0, 0);
                }
            }
        }
    }

    // ---- merge the four waves through LDS, one query tile at a time
    float* sO = reinterpret_cast<float*>(smem);                        // [wave][32][kOStride]
    float* sM = sO + kWaves * 32 * kOStride;                           // [wave][32]
    float* sL = sM + kWaves * 32;                                      // [wave][32]
    float* rec = part + (((size_t)head * n_qgroup + qgroup) * n_split + split) * part_stride;
    float* rec_m = rec;                // [NQ]
    float* rec_l = rec + NQ;           // [NQ]
    float* rec_O = rec + 2 * NQ;       // [NQ][64], not normalised
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        __syncthreads();               // staging areas / previous round are dead
        const float l_tot = l_run[qt] + swap_half(l_run[qt]);
        if (h == 0) { sM[wave * 32 + c] = m_run[qt]; sL[wave * 32 + c] = l_tot; }
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int e = dt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                sO[(wave * 32 + c) * kOStride + e] = oacc[qt][dt][r];
            }
        __syncthreads();
        const int e = tid & 63;
        for (int q = tid >> 6; q < 32; q += 4) {
            float mw[kWaves], mx = -INFINITY;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { mw[w] = sM[w * 32 + q]; mx = fmaxf(mx, mw[w]); }
            float lt = 0.f, ot = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float sc = (mw[w] == -INFINITY) ? 0.f : fast_exp2(mw[w] - mx);
                lt += sc * sL[w * 32 + q];
                ot += sc * sO[(w * 32 + q) * kOStride + e];
            }
            const int qg = qt * 32 + q;
            if (e == 0) { rec_store(rec_m + qg, mx); rec_store(rec_l + qg, lt); }
            rec_store(rec_O + qg * kD + e, ot);
        }
    }
    // ---- stage a4 for this work-group's share of the rows, then the hand-over
    fill_rows<bf16_t, 256>(static_cast<bf16_t*>(P.out) + (size_t)head * L * kD, selp, u, n, L,
                           wg_in_head * P.rows_per_wg, P.rows_per_wg, cs);
    ticket_and_merge<bf16_t, float, false, 256>(P, head, n, u, selp, NQ, cs);
}

hipError_t launch_attend(const Plan& p, const Args& a, const Scratch& w)
{
    AttendParams P;
    P.Q = a.Q; P.K = a.K; P.V = a.V; P.lengths = a.lengths;
    P.M = w.M; P.vpart = w.vpart; P.mu = w.mu; P.sel = w.sel; P.ucount = w.u; P.ticket = w.ticket;
    P.part = w.part; P.out = a.out;
    P.H = p.H; P.L = p.L; P.u_max = p.u_max; P.n_split = p.n_split; P.n_qgroup = p.n_qgroup;
    P.rounds = p.tiles_per_wave; P.part_stride = (int)p.part_stride; P.n_chunk = p.n_chunk;
    P.fused_select = p.fused_select; P.rows_per_wg = p.rows_per_wg; P.c = a.c;
    dim3 grid(p.n_split, p.n_qgroup, p.BH);
    if (p.dtype == PSA_F32) {
        // 72 KB of dynamic LDS: above the 64 KB default, so the limit is raised once per kernel
        static bool raised[2] = {false, false};
        const int which = p.nq_group == 16 ? 0 : 1;
        if (!raised[which]) {
            const void* fn = which == 0 ? (const void*)attend_f32_kernel<1> : (const void*)attend_f32_kernel<2>;
            const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kF32SmemBytes);
            if (e != hipSuccess) return e;
            raised[which] = true;
        }
        if (which == 0) hipLaunchKernelGGL(attend_f32_kernel<1>, grid, dim3(512), kF32SmemBytes, a.stream, P);
        else            hipLaunchKernelGGL(attend_f32_kernel<2>, grid, dim3(512), kF32SmemBytes, a.stream, P);
    } else {
        if (p.nq_group == 32) hipLaunchKernelGGL(attend_bf16_kernel<1>, grid, dim3(256), 0, a.stream, P);
        else                  hipLaunchKernelGGL(attend_bf16_kernel<2>, grid, dim3(256), 0, a.stream, P);
    }
    return hipGetLastError();
}

}  // namespace psa

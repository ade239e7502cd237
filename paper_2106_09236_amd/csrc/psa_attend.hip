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
#include "psa_device.h"
#include "psa_internal.h"

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
void attend_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
                       const int* __restrict__ lengths, const int* __restrict__ sel,
                       double* __restrict__ vsum, double* __restrict__ part,
                       int H, int L, int u_max, int n_split, int n_qgroup, int rounds, int part_stride)
{
    constexpr int NQ = NCG * 16;
    constexpr int KT = kF32Waves / NCG;                 // key tiles per round of the work-group
    constexpr int VPW = 16 / KT;                        // accumulator values each wave merges
    extern __shared__ __attribute__((aligned(16))) double smem[];     // [wave][kStateDoubles][64]

    const int split = blockIdx.x, qgroup = blockIdx.y, head = blockIdx.z;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int ct = wave % NCG, kt = wave / NCG;

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
            const int j = j0 + 16 * sb + c;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                kreg[sb][v] = (j < n) ? *reinterpret_cast<const float4*>(Kh + (size_t)j * kD + 16 * v + 4 * g)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto load_v = [&](int j0) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = j0 + 16 * sb + 4 * r + g;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
                    vreg[sb][dt][r] = (j < n) ? Vh[(size_t)j * kD + 16 * dt + c] : 0.f;
            }
    };

    // Loads complete in issue order, so they are issued in the order of use:
    // selected index, K tile, the query row (needs the index); the V tile is
    // requested only once the first product has been issued, so that it streams
    // in under the MFMAs and the softmax instead of competing with K and Q.
    const int qrank = qgroup * NQ + ct * 16 + c;
    int qi = -1;
    if (qrank < u_max) qi = sel[(size_t)head * u_max + qrank];                  // -1 beyond u_b
    const int j_first = (split * rounds * KT + kt) * kTile;
    load_k(j_first);
    // B operand of the first product: qreg[4v + e] = Q[q][16v + 4g + e], widened
    double qreg[16];
    if (qi >= 0 && qi < n) {
        const float* src = Qh + (size_t)qi * kD + 4 * g;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float4 x = *reinterpret_cast<const float4*>(src + 16 * v);
            qreg[4 * v + 0] = (double)x.x; qreg[4 * v + 1] = (double)x.y;
            qreg[4 * v + 2] = (double)x.z; qreg[4 * v + 3] = (double)x.w;
        }
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) qreg[v] = 0.0;
    }

    float m_run = -INFINITY;
    double l_run = 0.0;
    doublex4 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) oacc[dt] = doublex4{0.0, 0.0, 0.0, 0.0};
    double vs[4] = {0.0, 0.0, 0.0, 0.0};     // column sums of this lane's V elements (for the mean of a4)

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
        if (ct == 0) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                float tv = 0.f;                               // 8 terms in float32, then widened
#pragma unroll
                for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) tv += vreg[sb][dt][r];
                vs[dt] += (double)tv;
            }
        }
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
    // column sums of V ride on the same barrier: lanes g = 0 of the ct = 0 waves
    // reuse the m slot AFTER the merge below has read it (second barrier)
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
        rec_O[vi * 64 + lane] = acc;
    }
    if (kt == 0) {
        double l_tot = 0.0;
#pragma unroll
        for (int w = 0; w < KT; ++w) l_tot += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 1) * 64 + lane];
        l_tot += __shfl_xor(l_tot, 16, 64);
        l_tot += __shfl_xor(l_tot, 32, 64);
        if (g == 0) { rec[ct * 16 + c] = mx; rec[NQ + ct * 16 + c] = l_tot; }
    }

    // ---- column sums of the valid V rows this work-group walked
    if (qgroup == 0) {
        __syncthreads();                                       // states are dead
        double* sV = smem;                                     // [KT][64]
        if (ct == 0) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                double tv = vs[dt];
                tv += __shfl_xor(tv, 16, 64);
                tv += __shfl_xor(tv, 32, 64);
                if (g == 0) sV[kt * kD + 16 * dt + c] = tv;
            }
        }
        __syncthreads();
        if (tid < kD) {
            double tv = 0.0;
#pragma unroll
            for (int w = 0; w < KT; ++w) tv += sV[w * kD + tid];       // fixed order
            vsum[((size_t)head * n_split + split) * kD + tid] = tv;
        }
    }
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
void attend_bf16_kernel(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                        const int* __restrict__ lengths, const int* __restrict__ sel,
                        double* __restrict__ vsum, float* __restrict__ part,
                        int H, int L, int u_max, int n_split, int n_qgroup, int tiles_per_wave, int part_stride)
{
    constexpr int NQ = NQT * 32;
    constexpr int kStageBytes = kWaves * kB16WaveBytes;
    constexpr int kMergeBytes = kWaves * 32 * (kOStride + 2) * 4;
    constexpr int kSmemBytes = kStageBytes > kMergeBytes ? kStageBytes : kMergeBytes;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemBytes];

    const int split = blockIdx.x, qgroup = blockIdx.y, head = blockIdx.z;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;

    const bf16_t* Qh = Q + (size_t)head * L * kD;
    const bf16_t* Kh = K + (size_t)head * L * kD;
    const bf16_t* Vh = V + (size_t)head * L * kD;
    const int* selh = sel + (size_t)head * u_max;

    // B operand of the first product: qreg[qt][kk] = Q[q][32h + 8kk .. +8]
    uint4 qreg[NQT][4];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const int r = qgroup * NQ + qt * 32 + c;
        int qi = -1;
        if (r < u_max) qi = selh[r];                          // -1 beyond u_b
        if (qi >= 0 && qi < n) {
            const uint4* src = reinterpret_cast<const uint4*>(Qh + (size_t)qi * kD) + 4 * h;
#pragma unroll
            for (int v = 0; v < 4; ++v) qreg[qt][v] = src[v];
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) qreg[qt][v] = make_uint4(0u, 0u, 0u, 0u);
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

    double vs[2] = {0.0, 0.0};               // column sums of this lane's V elements (for the mean of a4)

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
            uint4 xk = make_uint4(0u, 0u, 0u, 0u), xv = xk;
            if (j < n) {
                xk = reinterpret_cast<const uint4*>(Kh + (size_t)j * kD)[col8];
                xv = reinterpret_cast<const uint4*>(Vh + (size_t)j * kD)[col8];
            }
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
        for (int dt = 0; dt < 2; ++dt) {
            float t = 0.f;                                    // 16 bf16 terms in float32, then widened
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const uint4 x = vop[st][dt];
                t += bf16_lo(x.x) + bf16_hi(x.x) + bf16_lo(x.y) + bf16_hi(x.y)
                   + bf16_lo(x.z) + bf16_hi(x.z) + bf16_lo(x.w) + bf16_hi(x.w);
            }
            vs[dt] += (double)t;
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
            if (e == 0) { rec_m[qg] = mx; rec_l[qg] = lt; }
            rec_O[qg * kD + e] = ot;
        }
    }
    // ---- column sums of the valid V rows this work-group walked
    if (qgroup == 0) {
        __syncthreads();
        double* sVs = reinterpret_cast<double*>(smem);                 // [wave][64]
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            double t = vs[dt];
            t += __shfl_xor(t, 32, 64);
            if (h == 0) sVs[wave * kD + 32 * dt + c] = t;
        }
        __syncthreads();
        if (tid < kD) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) t += sVs[w * kD + tid];   // fixed order
            vsum[((size_t)head * n_split + split) * kD + tid] = t;
        }
    }
}

hipError_t launch_attend(const Plan& p, const Args& a, const Scratch& w)
{
    dim3 grid(p.n_split, p.n_qgroup, p.BH);
#define PSA_ATTEND_ARGS a.lengths, w.sel, w.vpart, reinterpret_cast<RecT*>(w.part), \
        p.H, p.L, p.u_max, p.n_split, p.n_qgroup, p.tiles_per_wave, (int)p.part_stride
    if (p.dtype == PSA_F32) {
        using RecT = double;
        const float *Q = (const float*)a.Q, *K = (const float*)a.K, *V = (const float*)a.V;
        // 72 KB of dynamic LDS: above the 64 KB default, so the limit is raised once per kernel
        static bool raised[2] = {false, false};
        const int which = p.nq_group == 16 ? 0 : 1;
        if (!raised[which]) {
            const void* fn = which == 0 ? (const void*)attend_f32_kernel<1> : (const void*)attend_f32_kernel<2>;
            const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kF32SmemBytes);
            if (e != hipSuccess) return e;
            raised[which] = true;
        }
        if (which == 0) hipLaunchKernelGGL(attend_f32_kernel<1>, grid, dim3(512), kF32SmemBytes, a.stream, Q, K, V, PSA_ATTEND_ARGS);
        else            hipLaunchKernelGGL(attend_f32_kernel<2>, grid, dim3(512), kF32SmemBytes, a.stream, Q, K, V, PSA_ATTEND_ARGS);
    } else {
        using RecT = float;
        const bf16_t *Q = (const bf16_t*)a.Q, *K = (const bf16_t*)a.K, *V = (const bf16_t*)a.V;
        if (p.nq_group == 32) hipLaunchKernelGGL(attend_bf16_kernel<1>, grid, dim3(256), 0, a.stream, Q, K, V, PSA_ATTEND_ARGS);
        else                  hipLaunchKernelGGL(attend_bf16_kernel<2>, grid, dim3(256), 0, a.stream, Q, K, V, PSA_ATTEND_ARGS);
    }
#undef PSA_ATTEND_ARGS
    return hipGetLastError();
}

}  // namespace psa

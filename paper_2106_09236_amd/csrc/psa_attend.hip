// Stage a3: softmax attention of the selected queries over all valid keys
// (Eq. 7, Eq. 8, upper branch of Eq. 12), as partial results per key split.
//
// The two products  S = Q_sel K^T  and  O = P V  are contractions and run on the
// matrix cores.  Both are computed TRANSPOSED, with the selected queries on the
// column axis of 32x32 MFMA tiles:
//     S^T[key, q] = sum_e K[key, e] Q_sel[q, e]          A = K tile,   B = Q_sel^T
//     O^T[e,  q] = sum_key V[key, e] P[q, key]           A = V tile^T, B = P^T
// In the 32x32 accumulator layout lane (c, h) = (lane % 32, lane / 32) holds
// column c, so every value a lane ever owns belongs to ONE query: the running
// max, the running sum, the rescale of online softmax are all per-lane scalars,
// and the S^T accumulator registers are, unchanged, the B operand of the second
// product (row index of accumulator register r is 8*(r/4) + 4*h + r%4, which is
// taken as that product's contraction order).
//
// A work-group is 4 waves; each wave walks `tiles_per_wave` tiles of 32 keys
// with its own LDS staging area (no work-group barrier inside the loop), then
// the four waves' (m, l, O) are merged through LDS and one partial record per
// (head, query group, key split) goes to the workspace.  Records are merged in a
// fixed order by the finalize stage, so results do not depend on scheduling.
#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

constexpr float kScaleLog2e = 0.125f * 1.4426950408889634f;   // (1/sqrt(64)) * log2(e)

template <typename T> struct TileTraits;
template <> struct TileTraits<float> {
    static constexpr int kStride = 68;                 // floats per staged K row (64 + 4 pad)
    static constexpr int kWaveBytes = kTile * kStride * 4;            // K only; V comes straight from global
    static constexpr int kQRegs = 32;                  // B operand registers per query tile
};
template <> struct TileTraits<bf16_t> {
    static constexpr int kStride = 72;                 // bf16 per staged row (64 + 8 pad)
    static constexpr int kWaveBytes = 2 * kTile * kStride * 2;        // K and V
    static constexpr int kQRegs = 16;
};

// 2^x on the transcendental unit; -inf -> 0, no denormal handling needed here
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int kOStride = 65;                           // floats per query row in the merge area

template <typename T, int NQT>
__global__ __launch_bounds__(256)
void attend_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                   const int* __restrict__ lengths, const int* __restrict__ sel,
                   const int* __restrict__ ucount, float* __restrict__ part,
                   int H, int L, int u_max, int n_split, int n_qgroup, int tiles_per_wave, int part_stride)
{
    using TT = TileTraits<T>;
    constexpr int NQ = NQT * 32;
    constexpr int kStageBytes = kWaves * TT::kWaveBytes;
    constexpr int kMergeBytes = kWaves * 32 * (kOStride + 2) * 4;
    constexpr int kSmemBytes = kStageBytes > kMergeBytes ? kStageBytes : kMergeBytes;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kSmemBytes];

    const int split = blockIdx.x, qgroup = blockIdx.y, head = blockIdx.z;
    const int b = head / H;
    const int n = valid_len(lengths, b, L);
    const int u = ucount[b];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;

    const T* Qh = Q + (size_t)head * L * kD;
    const T* Kh = K + (size_t)head * L * kD;
    const T* Vh = V + (size_t)head * L * kD;
    const int* selh = sel + (size_t)head * u_max;

    // ---- B operand of the first product: this lane's query row, its half of d
    // f32 : qreg[qt][kk]        = Q[q][32h + kk]            (one float per MFMA step)
    // bf16: qreg[qt][4kk..4kk+3] = Q[q][32h + 8kk .. +8]    (8 bf16 per MFMA step)
    uint32_t qreg[NQT][TT::kQRegs];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const int r = qgroup * NQ + qt * 32 + c;
        int qi = -1;
        if (r < u) qi = selh[r];
        if (qi >= 0 && qi < n) {
            const uint4* src = reinterpret_cast<const uint4*>(Qh + (size_t)qi * kD) + h * (TT::kQRegs / 4);
#pragma unroll
            for (int v = 0; v < TT::kQRegs / 4; ++v) {
                const uint4 x = src[v];
                qreg[qt][4 * v + 0] = x.x; qreg[qt][4 * v + 1] = x.y;
                qreg[qt][4 * v + 2] = x.z; qreg[qt][4 * v + 3] = x.w;
            }
        } else {
#pragma unroll
            for (int v = 0; v < TT::kQRegs; ++v) qreg[qt][v] = 0u;
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

    unsigned char* stage = smem + wave * TT::kWaveBytes;
    const int tile0 = (split * kWaves + wave) * tiles_per_wave;

    for (int ti = 0; ti < tiles_per_wave; ++ti) {
        const int j0 = (tile0 + ti) * kTile;
        if (j0 >= n) break;                                   // wave-uniform

        if constexpr (sizeof(T) == 4) {
            // ---------------------------------------------------------- f32 tile
            float* sK = reinterpret_cast<float*>(stage);
            wave_lds_sync();                                  // previous tile's reads are done
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int row = it * 4 + (lane >> 4), col4 = lane & 15;
                const int j = j0 + row;
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j < n) x = reinterpret_cast<const float4*>(Kh + (size_t)j * kD)[col4];
                *reinterpret_cast<float4*>(sK + row * TT::kStride + col4 * 4) = x;
            }
            // A operand of the second product straight from global memory:
            // step r contracts key j0 + 8(r/4) + 4h + r%4, lanes c = 32 consecutive floats
            float vreg[2][16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j0 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
                    vreg[dt][r] = (j < n) ? reinterpret_cast<const float*>(Vh)[(size_t)j * kD + dt * 32 + c] : 0.f;
            }
            wave_lds_sync();

#pragma unroll
            for (int qt = 0; qt < NQT; ++qt) {
                floatx16 s;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float4 a = *reinterpret_cast<const float4*>(sK + c * TT::kStride + 32 * h + 4 * v);
                    s = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, __uint_as_float(qreg[qt][4 * v + 0]), s, 0, 0, 0);
                    s = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, __uint_as_float(qreg[qt][4 * v + 1]), s, 0, 0, 0);
                    s = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, __uint_as_float(qreg[qt][4 * v + 2]), s, 0, 0, 0);
                    s = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, __uint_as_float(qreg[qt][4 * v + 3]), s, 0, 0, 0);
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
                const float m_new = fmaxf(m_run[qt], tmax);   // finite: key j0 is valid
                const float alpha = fast_exp2(m_run[qt] - m_new);
                float lsum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) { s[r] = fast_exp2(s[r] - m_new); lsum += s[r]; }
                l_run[qt] = l_run[qt] * alpha + lsum;
                m_run[qt] = m_new;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[qt][dt][r] *= alpha;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(vreg[dt][r], s[r], oacc[qt][dt], 0, 0, 0);
                }
            }
        } else {
            // --------------------------------------------------------- bf16 tile
            uint16_t* sK = reinterpret_cast<uint16_t*>(stage);
            uint16_t* sV = sK + kTile * TT::kStride;
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
                *reinterpret_cast<uint4*>(sK + row * TT::kStride + col8 * 8) = xk;
                *reinterpret_cast<uint4*>(sV + row * TT::kStride + col8 * 8) = xv;
            }
            wave_lds_sync();

#pragma unroll
            for (int qt = 0; qt < NQT; ++qt) {
                floatx16 s;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const uint4 a = *reinterpret_cast<const uint4*>(sK + c * TT::kStride + 32 * h + 8 * kk);
                    const uint4 bq = make_uint4(qreg[qt][4 * kk], qreg[qt][4 * kk + 1], qreg[qt][4 * kk + 2], qreg[qt][4 * kk + 3]);
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, bq), s, 0, 0, 0);
                }
                float tmax = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + 8 * (r >> 2) + 4 * h + (r & 3);
                    s[r] = (j < n) ? s[r] * kScaleLog2e : -INFINITY;
                    tmax = fmaxf(tmax, s[r]);
                }
                tmax = fmaxf(tmax, swap_half(tmax));
                const float m_new = fmaxf(m_run[qt], tmax);
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
                // second product, 16 keys per MFMA step: step st takes accumulator
                // registers 8st..8st+7, i.e. keys 16st + 8(e/4) + 4h + e%4, e = 0..7
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const uint4 bp = make_uint4(pack_bf16(s[8 * st + 0], s[8 * st + 1]), pack_bf16(s[8 * st + 2], s[8 * st + 3]),
                                                pack_bf16(s[8 * st + 4], s[8 * st + 5]), pack_bf16(s[8 * st + 6], s[8 * st + 7]));
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        uint32_t av[4];
#pragma unroll
                        for (int e2 = 0; e2 < 4; ++e2) {
                            const int e = 2 * e2;
                            const int k0 = 16 * st + 8 * (e >> 2) + 4 * h + (e & 3);
                            const uint32_t lo = sV[k0 * TT::kStride + dt * 32 + c];
                            const uint32_t hi = sV[(k0 + 1) * TT::kStride + dt * 32 + c];
                            av[e2] = lo | (hi << 16);
                        }
                        const uint4 a = make_uint4(av[0], av[1], av[2], av[3]);
                        oacc[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, bp), oacc[qt][dt], 0, 0, 0);
                    }
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
}

template <typename T>
static hipError_t launch_attend_t(const Plan& p, const Args& a, const Scratch& w)
{
    dim3 grid(p.n_split, p.n_qgroup, p.BH), block(256);
    if (p.qt_per_group == 1) {
        hipLaunchKernelGGL((attend_kernel<T, 1>), grid, block, 0, a.stream,
                           (const T*)a.Q, (const T*)a.K, (const T*)a.V, a.lengths, w.sel, w.u, w.part,
                           p.H, p.L, p.u_max, p.n_split, p.n_qgroup, p.tiles_per_wave, (int)p.part_stride);
    } else {
        hipLaunchKernelGGL((attend_kernel<T, 2>), grid, block, 0, a.stream,
                           (const T*)a.Q, (const T*)a.K, (const T*)a.V, a.lengths, w.sel, w.u, w.part,
                           p.H, p.L, p.u_max, p.n_split, p.n_qgroup, p.tiles_per_wave, (int)p.part_stride);
    }
    return hipGetLastError();
}

hipError_t launch_attend(const Plan& p, const Args& a, const Scratch& w)
{
    return p.dtype == PSA_F32 ? launch_attend_t<float>(p, a, w) : launch_attend_t<bf16_t>(p, a, w);
}

}  // namespace psa

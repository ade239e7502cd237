// Per-wave attention tiles on the matrix cores, shared by the attend stage (a3)
// and the dense baseline.  Both products are computed TRANSPOSED, with the
// queries on the column axis of the MFMA tiles:
//     S^T[key, q] = sum_e K[key, e] Q[q, e]          A = K tile,   B = Q^T
//     O^T[e,  q] = sum_key V[key, e] P[q, key]       A = V tile^T, B = P^T
// A lane of an MFMA accumulator holds one column, so every value a lane ever
// owns belongs to ONE query: running max, running sum and the rescale of online
// softmax (Eq. 7, Eq. 8 evaluated tile by tile) are per-lane scalars, and the
// S^T accumulator registers are, unchanged, the B operand of the second product
// (their row order is taken as that product's contraction order; the V operand
// is fetched in the same order).
#pragma once

#include "psa_device.h"
#include "psa_internal.h"

namespace psa {

typedef double doublex4 __attribute__((ext_vector_type(4)));

// row every clamped load falls back to: the last valid one, or row 0 of an empty item
__device__ __forceinline__ int last_row(int n) { return n > 0 ? n - 1 : 0; }

constexpr float  kScaleLog2e  = 0.125f * 1.4426950408889634f;   // (1/sqrt(64)) * log2(e)
constexpr double kScaleLog2eD = 0.125 * 1.4426950408889634074;

// 2^x on the transcendental unit; -inf -> 0, no denormal handling needed here
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// =============================================================================
// float32 tensors: widened (exactly) to float64, v_mfma_f64_16x16x4f64.
// The parity bound for float32 tensors (1e-4 relative with a floor of 1e-2 RMS,
// element by element) is tighter than a float32 accumulation chain over hundreds
// of keys can promise; the exponent is evaluated in float64 as well.
//   lane (c, g) = (lane % 16, lane / 16)
//   A[i][k]: i = c, k = g      B[k][j]: k = g, j = c      D[i][j]: i = 4r + g, j = c  (r = 0..3)
// One object = one column tile of 16 queries walked by one wave, 32 keys a step.
// =============================================================================
struct F32Tile {
    double qreg[16];        // B of the first product: qreg[4v + e] = Q[q][16v + 4g + e]
    float4 kreg[2][4];      // A of the first product: key j0 + 16sb + c, elements 16v + 4g .. +3 (the
                            // contraction order is free; this one makes the four lanes g of a row
                            // read 64 contiguous bytes per load instruction)
    float4 vreg[2][4];      // A of the second product: key j0 + 16sb + 4r + g, elements 4c .. 4c+3 (one
                            // 16-byte load per key row; 4r + g is the row order of the S^T accumulator
                            // registers).  Component dt feeds accumulator dt, whose row m then stands
                            // for element 4m + dt.
    float m_run;
    double l_run;
    doublex4 oacc[4];       // O^T: element elem(dt, r, g) = 16r + 4g + dt of query c in oacc[dt][r]

    // Where an output element lives: accumulator register 4 dt + r of the lanes of group g.
    static __device__ __forceinline__ constexpr int elem(int dt, int r, int g) { return 16 * r + 4 * g + dt; }
    static __device__ __forceinline__ constexpr int reg_of(int e) { return 4 * (e & 3) + (e >> 4); }
    static __device__ __forceinline__ constexpr int grp_of(int e) { return (e >> 2) & 3; }

    __device__ __forceinline__ void init() {
        m_run = -INFINITY; l_run = 0.0;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] = doublex4{0.0, 0.0, 0.0, 0.0};
    }
    // query row `qrow` (nullptr-safe through `ok`): lanes c of the tile pass their own row
    __device__ __forceinline__ void load_q(const float* Qh, int qi, bool ok, int g) {
        const float* src = Qh + (size_t)(ok ? qi : 0) * kD + 4 * g;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float4 x = *reinterpret_cast<const float4*>(src + 16 * v);
            if (!ok) x = make_float4(0.f, 0.f, 0.f, 0.f);
            qreg[4 * v + 0] = (double)x.x; qreg[4 * v + 1] = (double)x.y;
            qreg[4 * v + 2] = (double)x.z; qreg[4 * v + 3] = (double)x.w;
        }
    }
    // Loads are unconditional on a clamped row (a guarded load would cost a branch
    // and a wait each); rows at or beyond n are zeroed afterwards.  FULL (the caller
    // knows, wave-uniformly, that all 32 rows of the tile are valid) drops the clamps,
    // the zeroing and, in the step, the masks: about a sixth of the step's vector
    // instructions.  Used by the rows kernel (7 % faster); in the key-split kernel and the
    // dense baseline the second copy of the step measured slower (20.1 -> 26.8 us, 98.6 ->
    // 104.4 us), so they keep the masked form alone.
    template <bool FULL = false>
    static __device__ __forceinline__ void load_k_into(float4 (&dst)[2][4], const float* Kh, int j0, int n, int c, int g) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            const int j = j0 + 16 * sb + c;
            const bool ok = FULL || j < n;
            const float* row = Kh + (size_t)(ok ? j : last_row(n)) * kD + 4 * g;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float4 x = *reinterpret_cast<const float4*>(row + 16 * v);
                if (!ok) x = make_float4(0.f, 0.f, 0.f, 0.f);
                dst[sb][v] = x;
            }
        }
    }
    __device__ __forceinline__ void load_k(const float* Kh, int j0, int n, int c, int g) { load_k_into(kreg, Kh, j0, n, c, g); }
    template <bool FULL = false>
    __device__ __forceinline__ void load_v(const float* Vh, int j0, int n, int c, int g) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = j0 + 16 * sb + 4 * r + g;
                const bool ok = FULL || j < n;
                float4 x = *reinterpret_cast<const float4*>(Vh + (size_t)(ok ? j : last_row(n)) * kD + 4 * c);
                if (!ok) x = make_float4(0.f, 0.f, 0.f, 0.f);
                vreg[sb][r] = x;
            }
    }
    // First product for both 16-key sub-tiles of the K tile in kreg (two independent
    // MFMA chains): s[sb][r] = q . k of key j0 + 16sb + 4r + g, unscaled.
    __device__ __forceinline__ void scores(doublex4 (&s)[2]) const {
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
    }
    // One step over keys j0 .. j0+31 (key j0 must be valid).  kreg must hold the K
    // tile.  With V_PRELOADED the caller has already requested the V tile;
    // otherwise it is requested here, once the first product has been issued, so
    // that it arrives under the MFMAs and the softmax.
    template <bool V_PRELOADED = false, bool FULL = false>
    __device__ __forceinline__ void step(const float* Vh, int j0, int n, int c, int g) {
        doublex4 s[2];
        scores(s);
        if (!V_PRELOADED) load_v<FULL>(Vh, j0, n, c, g);
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
                ok[sb][r] = FULL || (j0 + 16 * sb + 4 * r + g) < n;
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
            for (int r = 0; r < 4; ++r) {
                oacc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)vreg[sb][r].x, p[sb][r], oacc[0], 0, 0, 0);
                oacc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)vreg[sb][r].y, p[sb][r], oacc[1], 0, 0, 0);
                oacc[2] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)vreg[sb][r].z, p[sb][r], oacc[2], 0, 0, 0);
                oacc[3] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)vreg[sb][r].w, p[sb][r], oacc[3], 0, 0, 0);
            }
    }
};

// =============================================================================
// bfloat16 tensors: v_mfma_f32_32x32x16_bf16, float32 accumulation; the
// probabilities are split into two bfloat16 terms (hi + lo) so that P keeps 16
// significant bits in the second product.
//   lane (c, h) = (lane % 32, lane / 32)
//   A[i][k]: i = c, k = 8h + e   B[k][j]: k = 8h + e, j = c   (e = 0..7 packed in the lane)
//   D[i][j]: i = 8(r/4) + 4h + r%4, j = c   (r = 0..15)
// One object = NQT column tiles of 32 queries walked by one wave, 32 keys a step;
// the K and V tiles are staged in LDS rows of kB16Stride elements.
// =============================================================================
constexpr int kB16Stride = 72;                                  // bf16 per staged row (64 + 8 pad)

template <int NQT>
struct Bf16Tile {
    uint4 qreg[NQT][4];     // B of the first product: qreg[qt][kk] = Q[q][32h + 8kk .. +8]
    float m_run[NQT], l_run[NQT];
    floatx16 oacc[NQT][2];  // O^T: element 32dt + 8(r/4) + 4h + r%4 of query c in oacc[qt][dt][r]

    __device__ __forceinline__ void init() {
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            m_run[qt] = -INFINITY; l_run[qt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[qt][dt][r] = 0.f;
        }
    }
    __device__ __forceinline__ void load_q(int qt, const bf16_t* Qh, int qi, bool ok, int h) {
        const uint4* src = reinterpret_cast<const uint4*>(Qh + (size_t)(ok ? qi : 0) * kD) + 4 * h;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            uint4 x = src[v];
            if (!ok) x = make_uint4(0u, 0u, 0u, 0u);
            qreg[qt][v] = x;
        }
    }
    // ---- operands straight from global memory (the prob-sparse attend kernel).
    // K tile as the A operand of the first product: lane (c, h) reads the 64
    // contiguous bytes 64h .. 64h+63 of row j0 + c.  Rows at or beyond n are read
    // from the last valid row instead; their scores are masked in the step.
    static __device__ __forceinline__ void load_k_operand(uint4 (&ka)[4], const bf16_t* Kh, int j0, int n, int c, int h) {
        const int j = j0 + c;
        const uint4* src = reinterpret_cast<const uint4*>(Kh + (size_t)(j < n ? j : last_row(n)) * kD) + 4 * h;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) ka[kk] = src[kk];
    }
    // V tile, row-major as it lies in memory (lane reads 16 bytes of row it*8 + lane/8) ...
    static __device__ __forceinline__ void load_v_rows(uint4 (&vr)[4], const bf16_t* Vh, int j0, int n, int lane) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int j = j0 + it * 8 + (lane >> 3);
            vr[it] = reinterpret_cast<const uint4*>(Vh + (size_t)(j < n ? j : last_row(n)) * kD)[lane & 7];
        }
    }
    // ... and into the wave's LDS tile, rows at or beyond n as zeros (P is 0 there, but
    // 0 times a NaN in the padding would still poison the sum).
    static __device__ __forceinline__ void stage_v_rows(const uint4 (&vr)[4], uint16_t* sV, int j0, int n, int lane) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = it * 8 + (lane >> 3);
            const uint4 x = (j0 + row < n) ? vr[it] : make_uint4(0u, 0u, 0u, 0u);
            *reinterpret_cast<uint4*>(sV + row * kB16Stride + (lane & 7) * 8) = x;
        }
    }

    // One step over the staged keys j0 .. j0+31 (key j0 valid; rows at or beyond n
    // are zero in LDS), K from LDS as well.
    __device__ __forceinline__ void step(const uint16_t* sK, const uint16_t* sV, int j0, int n, int c, int h) {
        uint4 ka[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) ka[kk] = *reinterpret_cast<const uint4*>(sK + c * kB16Stride + 32 * h + 8 * kk);
        step_ops(ka, sV, j0, n, c, h);
    }

    // First product of one K tile with query tile qt: s[r] = q . k of key
    // j0 + 8(r/4) + 4h + r%4 for query c, unscaled.
    __device__ __forceinline__ floatx16 scores(const uint4 (&ka)[4], int qt) const {
        floatx16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[kk]), __builtin_bit_cast(bf16x8, qreg[qt][kk]), s, 0, 0, 0);
        return s;
    }

    // The step proper: ka = A operand of the first product (this lane's K row,
    // elements 32h + 8kk .. +8), V tile in LDS.
    __device__ __forceinline__ void step_ops(const uint4 (&ka)[4], const uint16_t* sV, int j0, int n, int c, int h) {
        // A operand of the second product, shared by all query tiles: for step st
        // and element e the key is 16st + 8(e/4) + 4h + e%4 (the row order of the
        // S^T accumulator registers 8st..8st+7), column 32dt + c
        // V lies row-major in LDS; the transposing LDS read (ds_read_b64_tr_b16) hands a lane of each
        // group of 16 lanes one column of a 4 x 16 block: source lane s of the group points at row
        // s / 4 of the block, columns 4 (s % 4) .. + 3, and lane i receives column i of the four rows.
        // Two such reads (keys 16st + 4h .. + 3 and 16st + 8 + 4h .. + 3) make the operand's 8 elements.
        typedef short shortx4 __attribute__((ext_vector_type(4)));
        uint4 vop[2][2];
        {
            const int s16 = c & 15;
            const uint16_t* src = sV + (4 * h + (s16 >> 2)) * kB16Stride + (c & 16) + 4 * (s16 & 3);
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const uint16_t* p0 = src + (16 * st) * kB16Stride + dt * 32;
                    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (shortx4 __attribute__((address_space(3)))*)(p0));
                    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (shortx4 __attribute__((address_space(3)))*)(p0 + 8 * kB16Stride));
                    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
                    vop[st][dt] = make_uint4(l2.x, l2.y, h2.x, h2.y);
                }
        }
        const bool full = j0 + kTile <= n;                        // wave-uniform: no key of the tile is masked
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
            floatx16 s = scores(ka, qt);
            // online softmax in base 2 on the raw scores (the scale is positive, so it
            // commutes with the maximum and folds into the exponent's multiply-add);
            // keys at or beyond n are masked out
            if (!full) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + 8 * (r >> 2) + 4 * h + (r & 3);
                    s[r] = (j < n) ? s[r] : -INFINITY;
                }
            }
            float tmax = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
            tmax = fmaxf(tmax, swap_half(tmax));
            const float m_new = fmaxf(m_run[qt], tmax * kScaleLog2e);   // finite: key j0 is valid
            const float alpha = fast_exp2(m_run[qt] - m_new);
            float lsum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = fast_exp2(fmaf(s[r], kScaleLog2e, -m_new)); lsum += s[r]; }
            l_run[qt] = l_run[qt] * alpha + lsum;
            if (__builtin_amdgcn_ballot_w64(m_new > m_run[qt]) != 0) {  // wave-uniform: some maximum moved
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[qt][dt][r] *= alpha;
            }
            m_run[qt] = m_new;
            // P = P_hi + P_lo, both bf16: 16 significant bits survive
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                uint32_t ph[4], pl[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float p0 = s[8 * st + 2 * e2], p1 = s[8 * st + 2 * e2 + 1];
                    ph[e2] = cvt_pk_bf16(p0, p1);
                    pl[e2] = cvt_pk_bf16(p0 - bf16_lo(ph[e2]), p1 - bf16_hi(ph[e2]));
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
};

}  // namespace psa

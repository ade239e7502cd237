// Stage a3 (and, fused into the same kernel, a2 for short heads and a4):
// softmax attention of the selected queries over all valid keys (Eq. 7, Eq. 8,
// upper branch of Eq. 12) on the matrix cores, as partial results per key split
// that the last work-group of each head merges into `out`.
//
// The per-wave tile arithmetic lives in psa_tile.h; the selection, the fill and
// the hand-over in psa_attend_common.h.  This file holds the two kernels: how a
// work-group cuts its key range and its selected queries over its waves, and how
// the waves' partial (m, l, O) are merged through LDS into one record per
// (head, query group, key split).  Records are merged in a fixed order, so
// results do not depend on scheduling.
#include "psa_attend_common.h"
#include "psa_tile.h"

namespace psa {

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

// Record layout for float32 tensors, NQ = 16 * NCG queries:
//   [ m[NQ] | l[NQ] as float64 | O / l as float32: per column tile ct a block of 1024 = [16 registers][64 lanes] ]
// element e of query q: block q / 16, register 4 (e % 4) + e / 16, lane ((e / 4) % 4) * 16 + q % 16
// (F32Tile::reg_of, grp_of), i.e. exactly the accumulator layout, so record stores are fully coalesced.
// ALLFULL: the host knows that every key tile of every head is wholly valid (no lengths, L a multiple of
// 32): the loads then need no clamps and the step no masks (a run-time test per tile with both forms of
// the step in one kernel measured slower: 20.1 -> 26.8 us).
// The work of one work-group (key split `split`, query group `qgroup` of `head`); `smem`: kF32SmemBytes of LDS.
template <int NCG, bool ALLFULL, typename CS>      // NCG: column tiles of 16 selected queries per query group, 1 or 2
__device__ __forceinline__ void attend_f32_body(const AttendParams& P, int split, int qgroup, int head, double* smem, CS& cs)
{
    const float* Q = static_cast<const float*>(P.Q);
    const float* K = static_cast<const float*>(P.K);
    const float* V = static_cast<const float*>(P.V);
    double* part = static_cast<double*>(P.part);
    const int H = P.H, L = P.L, n_split = P.n_split, n_qgroup = P.n_qgroup, rounds = P.rounds, part_stride = P.part_stride;
    constexpr int NQ = NCG * 16;
    constexpr int KT = kF32Waves / NCG;                 // key tiles per round of the work-group
    constexpr int VPW = 16 / KT;                        // accumulator values each wave merges
    // smem: [wave][kStateDoubles][64]
    const int b = head / H;
    const int n = valid_len(P.lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int ct = wave % NCG, kt = wave / NCG;
    const int wg_in_head = qgroup * n_split + split;

    const float* Qh = Q + (size_t)head * L * kD;
    const float* Kh = K + (size_t)head * L * kD;
    const float* Vh = V + (size_t)head * L * kD;

    // The first K tile does not depend on the selection: it is requested as soon as
    // the prologue's own small loads are in flight and streams in while the prologue
    // picks I_sparse; then the query row (needs the index).
    PSA_TS(0);
    F32Tile tile;
    tile.init();
    const int j_first = (split * rounds * KT + kt) * kTile;
    // A wave whose first tile lies past the end (more waves than key tiles: short heads) does no tile
    // step, but its first loads are issued before that is looked at; the masked loads clamp every row,
    // the unmasked ones must be pointed at rows that exist (rows 0 .. 31: L is a multiple of 32 here).
    const int j_ld = (ALLFULL && j_first >= n) ? 0 : j_first;
    int u;
    const int* selp = attend_prologue<512>(P, head, n, wg_in_head, cs, u,
                                           [&]() { F32Tile::load_k_into<ALLFULL>(tile.kreg, Kh, j_ld, n, c, g); });
    PSA_TS(1);
    const int qrank = qgroup * NQ + ct * 16 + c;
    const int qi = qrank < u ? selp[qrank] : -1;
    tile.load_q(Qh, qi, qi >= 0 && qi < n, g);
    tile.load_v<ALLFULL>(Vh, j_ld, n, c, g);                  // behind K and Q in the queue, needed last

    // ---- stage a4 for this work-group's share of the rows: the stores go out now
    // and complete under the matrix work below
    fill_rows<float, 512>(P, static_cast<float*>(P.out) + (size_t)head * L * kD, Vh, selp, u, n, wg_in_head, cs);

    PSA_TS(2);
    // the K tile of the next round is requested before the current round's products
    // (clamped addresses past the end: harmless), so only the first round waits for K
    float4 knext[2][4];
    for (int rd = 0; rd < rounds; ++rd) {
        const int j0 = ((split * rounds + rd) * KT + kt) * kTile;
        if (j0 >= n) break;                                   // wave-uniform
        if (rd > 0) {
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int v = 0; v < 4; ++v) tile.kreg[sb][v] = knext[sb][v];
        }
        if (rd + 1 < rounds) F32Tile::load_k_into(knext, Kh, j0 + KT * kTile, n, c, g);     // (may lie past the end: clamped)
        if (rd == 0) tile.step<true, ALLFULL>(Vh, j0, n, c, g);
        else         tile.step<false, ALLFULL>(Vh, j0, n, c, g);
    }
    PSA_TS(3);
    const float m_run = tile.m_run;
    const double l_run = tile.l_run;
    doublex4 (&oacc)[4] = tile.oacc;

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
    PSA_TS(4);
    __syncthreads();
    PSA_TS(5);

    double wgt[KT], mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < KT; ++w) {
        wgt[w] = smem[(size_t)(w * NCG + ct) * kStateDoubles * 64 + lane];       // m of wave (w, ct)
        mx = fmax(mx, wgt[w]);
    }
#pragma unroll
    for (int w = 0; w < KT; ++w) wgt[w] = (wgt[w] == -INFINITY) ? 0.0 : exp2_f64(wgt[w] - mx);

    if (n_split == 1) {
        // the only split of its head: no record, the rows go straight to `out`
        double l_tot = 0.0;
#pragma unroll
        for (int w = 0; w < KT; ++w) l_tot += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 1) * 64 + lane];
        l_tot += __shfl_xor(l_tot, 16, 64);
        l_tot += __shfl_xor(l_tot, 32, 64);
        const double inv = l_tot > 0.0 ? 1.0 / l_tot : 0.0;
        float* orow = static_cast<float*>(P.out) + ((size_t)head * L + (qi >= 0 && qi < n ? qi : 0)) * kD;
#pragma unroll
        for (int k = 0; k < VPW; ++k) {
            const int vi = kt * VPW + k;
            double acc = 0.0;
#pragma unroll
            for (int w = 0; w < KT; ++w)
                acc += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 2 + vi) * 64 + lane];
            if (qi >= 0 && qi < n) orow[F32Tile::elem(vi >> 2, vi & 3, g)] = (float)(acc * inv);   // register vi = 4 dt + r
        }
        return;
    }
    // The record keeps m and l in float64 and O divided by the split's own l in float32 (6e-8 relative per
    // element, far inside the parity bound): half the bytes of a float64 O, which made up a third of this
    // kernel's memory traffic.
    double* rec = part + (((size_t)head * n_qgroup + qgroup) * n_split + split) * part_stride;
    float* rec_O = reinterpret_cast<float*>(rec + 2 * NQ) + ct * 1024;
    double l_tot = 0.0;
#pragma unroll
    for (int w = 0; w < KT; ++w) l_tot += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 1) * 64 + lane];
    l_tot += __shfl_xor(l_tot, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    const double inv = l_tot > 0.0 ? 1.0 / l_tot : 0.0;
#pragma unroll
    for (int k = 0; k < VPW; ++k) {
        const int vi = kt * VPW + k;
        double acc = 0.0;
#pragma unroll
        for (int w = 0; w < KT; ++w)
            acc += wgt[w] * smem[((size_t)(w * NCG + ct) * kStateDoubles + 2 + vi) * 64 + lane];
        rec_store(rec_O + vi * 64 + lane, (float)(acc * inv));
    }
    if (kt == 0 && g == 0) { rec_store(rec + ct * 16 + c, mx); rec_store(rec + NQ + ct * 16 + c, l_tot); }

    PSA_TS(6);
    PSA_TS(7);
    // ---- the hand-over
    ticket_and_merge<float, double, true, 512>(P, head, n, u, selp, NQ, cs);
    PSA_TS(8);
}

template <int NCG, bool ALLFULL>
__global__ __launch_bounds__(512)
void attend_f32_kernel(const AttendParams P)
{
    __shared__ CommonScratch<512> cs;
    extern __shared__ __attribute__((aligned(16))) double smem[];
    attend_f32_body<NCG, ALLFULL>(P, blockIdx.x, blockIdx.y, blockIdx.z, smem, cs);
}

// =============================================================================
// bfloat16 tensors: v_mfma_f32_32x32x16_bf16, float32 accumulation
//   lane (c, h) = (lane % 32, lane / 32)
//   A[i][k]: i = c, k = 8h + e   B[k][j]: k = 8h + e, j = c   (e = 0..7 packed in the lane)
//   D[i][j]: i = 8(r/4) + 4h + r%4, j = c   (r = 0..15)
// The kernel is bound by streaming K and V, and at these sizes by the latency of
// the stream rather than its width: a work-group is 8 waves, each walks its own
// run of 32-key tiles for all NQT * 32 selected queries of the group, the K tile
// going straight into A-operand registers, the V tile through a wave-private LDS
// tile (the second product needs it transposed; it is read back with the
// transposing LDS read); the next tile is requested
// before the current one is used.  One work-group per CU.
// =============================================================================
constexpr int kB16Waves = 8;
constexpr int kB16StageBytes = kB16Waves * kTile * kB16Stride * 2;     // 36864: one V tile per wave
constexpr int kB16StateVec = 9;                                        // float4 per lane: 8 accumulator quads, (m, l, -, -)
constexpr int kB16MergeBytes = kB16Waves * kB16StateVec * 64 * 16;     // 73728
constexpr int kB16SmemBytes = kB16StageBytes + kB16MergeBytes;         // 110592: dynamic LDS

// Record layout for bfloat16 tensors (floats), NQ = 32 * NQT queries:
//   [ m[NQ] | l[NQ] | O: per query tile qt and accumulator quad (8 per tile) a block [64 lanes][4] ]
// element e of query q = 32 qt + c: quad e / 8, lane c + 32 * ((e / 4) % 2), slot e % 4:
// the accumulator layout, four registers at a time, so a lane stores 16 bytes.
// Merges, in split order, the records of splits s_first, s_first + s_step, ... of
// one query group for (query tile qt, quad, lane): running maximum m, sum l and
// four unnormalised output elements.  COHERENT: the records were written by other work-groups of this very
// launch (with agent-scope stores) and are read past the caches; else by an earlier launch.
template <bool COHERENT = false>
__device__ __forceinline__ void merge_splits_b16(const float* base, int stride, int NQ, int n_split, int s_first, int s_step,
                                                 int qt, int quad, int lane, float& mx, float& lt, float (&acc)[4])
{
    const int q = qt * 32 + (lane & 31);
    mx = -INFINITY; lt = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = 0.f;
    for (int s0 = s_first; s0 < n_split; s0 += 4 * s_step) {
        float m4[4], l4[4], o4[4][4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int s = s0 + k * s_step;
            const bool ok = s < n_split;
            const float* rec = base + (size_t)(ok ? s : s0) * stride;
            const float* op = rec + 2 * NQ + ((size_t)(qt * 8 + quad) * 64 + lane) * 4;
            float mv;
            if (COHERENT) {
                mv = rec_load(rec + q);
                l4[k] = rec_load(rec + NQ + q);
                const unsigned long long a = rec_load(reinterpret_cast<const unsigned long long*>(op));
                const unsigned long long b = rec_load(reinterpret_cast<const unsigned long long*>(op) + 1);
                o4[k][0] = __uint_as_float((unsigned)a); o4[k][1] = __uint_as_float((unsigned)(a >> 32));
                o4[k][2] = __uint_as_float((unsigned)b); o4[k][3] = __uint_as_float((unsigned)(b >> 32));
            } else {
                mv = rec[q];
                l4[k] = rec[NQ + q];
                const float4 ov = *reinterpret_cast<const float4*>(op);
                o4[k][0] = ov.x; o4[k][1] = ov.y; o4[k][2] = ov.z; o4[k][3] = ov.w;
            }
            m4[k] = ok ? mv : -INFINITY;
        }
        float cm = mx;
#pragma unroll
        for (int k = 0; k < 4; ++k) cm = fmaxf(cm, m4[k]);
        if (cm == -INFINITY) continue;
        const float a = (mx == -INFINITY) ? 0.f : fast_exp2(mx - cm);
        lt *= a;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] *= a;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float sc = (m4[k] == -INFINITY) ? 0.f : fast_exp2(m4[k] - cm);
            lt = fmaf(sc, l4[k], lt);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fmaf(sc, o4[k][e], acc[e]);
        }
        mx = cm;
    }
}

// Four consecutive output elements 8 quad + 4h .. +3 of row i, normalised.
__device__ __forceinline__ void store_quad_b16(bf16_t* out_head, int i, int quad, int h, float lt, const float (&acc)[4]) {
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const uint2 pk = make_uint2(cvt_pk_bf16(acc[0] * inv, acc[1] * inv), cvt_pk_bf16(acc[2] * inv, acc[3] * inv));
    *reinterpret_cast<uint2*>(out_head + (size_t)i * kD + 8 * quad + 4 * h) = pk;
}

// The work of one work-group; `smem_b16`: kB16SmemBytes of LDS, or with ALIAS (the wave states reuse the V tiles'
// area behind a barrier) kB16MergeBytes.
template <int NQT, bool ALIAS, typename CS>     // NQT: column tiles of 32 selected queries per work-group
__device__ __forceinline__ void attend_bf16_body(const AttendParams& P, int split, int qgroup, int head,
                                                 unsigned char* smem_b16, CS& cs)
{
    const bf16_t* Q = static_cast<const bf16_t*>(P.Q);
    const bf16_t* K = static_cast<const bf16_t*>(P.K);
    const bf16_t* V = static_cast<const bf16_t*>(P.V);
    float* part = static_cast<float*>(P.part);
    const int H = P.H, L = P.L, n_split = P.n_split, n_qgroup = P.n_qgroup, tiles_per_wave = P.rounds, part_stride = P.part_stride;
    constexpr int NQ = NQT * 32;
    const int b = head / H;
    const int n = valid_len(P.lengths, b, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int wg_in_head = qgroup * n_split + split;

    const bf16_t* Qh = Q + (size_t)head * L * kD;
    const bf16_t* Kh = K + (size_t)head * L * kD;
    const bf16_t* Vh = V + (size_t)head * L * kD;
    bf16_t* out_head = static_cast<bf16_t*>(P.out) + (size_t)head * L * kD;

    // this wave's tiles: tile0 .. tile0 + nt - 1 (nt = 0: nothing valid in its range)
    const int tile0 = (split * kB16Waves + wave) * tiles_per_wave;
    int nt = (n - tile0 * kTile + kTile - 1) / kTile;
    nt = nt < 0 ? 0 : (nt > tiles_per_wave ? tiles_per_wave : nt);

    // The first tile does not depend on the selection: it is requested as soon as
    // the prologue's own small loads are in flight.
    uint4 kn[4], vn[4];
    PSA_TS(0);
    int u;
    const int* selp = attend_prologue<512>(P, head, n, wg_in_head, cs, u, [&]() {
        Bf16Tile<NQT>::load_k_operand(kn, Kh, tile0 * kTile, n, c, h);
        Bf16Tile<NQT>::load_v_rows(vn, Vh, tile0 * kTile, n, lane);
    });
    PSA_TS(1);

    Bf16Tile<NQT> tile;
    tile.init();
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        const int r = qgroup * NQ + qt * 32 + c;
        const int qi = r < u ? selp[r] : -1;
        tile.load_q(qt, Qh, qi, qi >= 0 && qi < n, h);
    }
    // ---- stage a4 for this work-group's share of the rows: the stores go out now
    // and complete under the matrix work below
    fill_rows<bf16_t, 512>(P, out_head, Vh, selp, u, n, wg_in_head, cs);
    PSA_TS(2);

    uint16_t* sV = reinterpret_cast<uint16_t*>(smem_b16) + wave * kTile * kB16Stride;
    for (int ti = 0; ti < nt - 1; ++ti) {
        const int j0 = (tile0 + ti) * kTile;
        uint4 kc[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kc[kk] = kn[kk];
        wave_lds_sync();                                      // previous tile's reads are done
        Bf16Tile<NQT>::stage_v_rows(vn, sV, j0, n, lane);
        Bf16Tile<NQT>::load_k_operand(kn, Kh, j0 + kTile, n, c, h);        // next tile, in flight during the step
        Bf16Tile<NQT>::load_v_rows(vn, Vh, j0 + kTile, n, lane);
        wave_lds_sync();
        tile.step_ops(kc, sV, j0, n, c, h);
    }
    if (nt > 0) {
        const int j0 = (tile0 + nt - 1) * kTile;
        wave_lds_sync();
        Bf16Tile<NQT>::stage_v_rows(vn, sV, j0, n, lane);
        wave_lds_sync();
        tile.step_ops(kn, sV, j0, n, c, h);
    }
    PSA_TS(3);

    // ---- merge the eight waves through LDS, one query tile at a time: every wave
    // publishes its state in register layout, then wave w merges accumulator quad
    // w (registers 4(w % 4) .. +3 of column half w / 4) of all eight states, in
    // wave order, and stores it into the record.
    if (ALIAS) lds_barrier();                                  // every wave is done with its V tile
    float4* sState = reinterpret_cast<float4*>(smem_b16 + (ALIAS ? 0 : kB16StageBytes));   // [wave][kB16StateVec][64]
    float* rec = part + (((size_t)head * n_qgroup + qgroup) * n_split + split) * part_stride;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
        if (qt > 0) lds_barrier();                             // the previous tile's states have been read
        float4* mine = sState + (size_t)wave * kB16StateVec * 64;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                mine[(dt * 4 + r4) * 64 + lane] = make_float4(tile.oacc[qt][dt][4 * r4 + 0], tile.oacc[qt][dt][4 * r4 + 1],
                                                              tile.oacc[qt][dt][4 * r4 + 2], tile.oacc[qt][dt][4 * r4 + 3]);
        mine[8 * 64 + lane] = make_float4(tile.m_run[qt], tile.l_run[qt], 0.f, 0.f);
        lds_barrier();
        float mw[kB16Waves], lw[kB16Waves], mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < kB16Waves; ++w) {
            const float4 ml = sState[((size_t)w * kB16StateVec + 8) * 64 + lane];
            mw[w] = ml.x; lw[w] = ml.y;
            mx = fmaxf(mx, ml.x);
        }
        float acc[4] = {0.f, 0.f, 0.f, 0.f}, lt = 0.f;
#pragma unroll
        for (int w = 0; w < kB16Waves; ++w) {
            const float sc = (mw[w] == -INFINITY) ? 0.f : fast_exp2(mw[w] - mx);
            const float4 o = sState[((size_t)w * kB16StateVec + wave) * 64 + lane];
            acc[0] = fmaf(sc, o.x, acc[0]); acc[1] = fmaf(sc, o.y, acc[1]);
            acc[2] = fmaf(sc, o.z, acc[2]); acc[3] = fmaf(sc, o.w, acc[3]);
            lt = fmaf(sc, lw[w], lt);
        }
        lt += swap_half(lt);
        float* ro = rec + 2 * NQ + ((size_t)(qt * 8 + wave) * 64 + lane) * 4;
        if (n_split == 1) {
            // the only split of its head: no record, the rows go straight to `out`
            const int rank = qgroup * NQ + qt * 32 + c;
            const int i = rank < u ? selp[rank] : -1;
            if (i >= 0 && i < n) store_quad_b16(out_head, i, wave, h, lt, acc);
        } else if (P.separate_merge) {
            // the merge kernel that follows reads the records with plain loads
            *reinterpret_cast<float4*>(ro) = make_float4(acc[0], acc[1], acc[2], acc[3]);
            if (wave == 0 && h == 0) { rec[qt * 32 + c] = mx; rec[NQ + qt * 32 + c] = lt; }
        } else {
            // the head's last work-group reads them inside this launch: stores that go through to memory
            rec_store(reinterpret_cast<unsigned long long*>(ro),
                      (unsigned long long)__float_as_uint(acc[0]) | ((unsigned long long)__float_as_uint(acc[1]) << 32));
            rec_store(reinterpret_cast<unsigned long long*>(ro) + 1,
                      (unsigned long long)__float_as_uint(acc[2]) | ((unsigned long long)__float_as_uint(acc[3]) << 32));
            if (wave == 0 && h == 0) { rec_store(rec + qt * 32 + c, mx); rec_store(rec + NQ + qt * 32 + c, lt); }
        }
    }
    PSA_TS(4);
    // ---- few splits: the work-group that draws the head's last ticket merges the records (no work-group waits
    // for another; ordering as in ticket_and_merge), wave w taking accumulator quad w of every query tile
    if (n_split > 1 && !P.separate_merge) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const int t = __hip_atomic_fetch_add(P.ticket + head, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = (t == n_split * n_qgroup - 1);
            if (last) __hip_atomic_store(P.ticket + head, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
            cs.last = last;
        }
        __syncthreads();
        if (cs.last) {
            for (int qg = 0; qg < n_qgroup; ++qg) {
                const float* base = part + ((size_t)head * n_qgroup + qg) * n_split * part_stride;
#pragma unroll
                for (int qt = 0; qt < NQT; ++qt) {
                    if (qg * NQ + qt * 32 >= u) break;                 // work-group-uniform: no selected query there
                    const int rank = qg * NQ + qt * 32 + c;
                    const int i = rank < u ? selp[rank] : -1;
                    float mx, lt, acc[4];
                    merge_splits_b16<true>(base, part_stride, NQ, n_split, 0, 1, qt, wave, lane, mx, lt, acc);
                    if (i >= 0 && i < n) store_quad_b16(out_head, i, wave, h, lt, acc);
                }
            }
        }
    }
    PSA_TS(5);
    PSA_TS_DRAIN();
    PSA_TS(6);
}

template <int NQT>
__global__ __launch_bounds__(512)
void attend_bf16_kernel(const AttendParams P)
{
    __shared__ CommonScratch<512> cs;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_b16[];
    attend_bf16_body<NQT, false>(P, blockIdx.x, blockIdx.y, blockIdx.z, smem_b16, cs);
}

// Merge kernel for bfloat16 records: work-group (quad, query tile, head), four
// waves; wave w merges splits w, w + 4, ..., the four partial results are
// combined through LDS in wave order by wave 0, which writes 8 bytes of each of
// the tile's 32 output rows.
__global__ __launch_bounds__(256)
void merge_b16_kernel(const AttendParams P)
{
    __shared__ float s_part[3][6][64];
    const int quad = blockIdx.x, qtile = blockIdx.y, head = blockIdx.z;
    const int b = head / P.H;
    const int n = valid_len(P.lengths, b, P.L);
    const int u = P.ucount[b];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int NQ = P.nq, nqt = NQ / 32;
    const int qg = qtile / nqt, qt = qtile % nqt;
    const int rank = qtile * 32 + c;
    if (qtile * 32 >= u) return;                               // work-group-uniform
    const int i = rank < u ? P.sel[(size_t)head * P.u_max + rank] : -1;
    const float* base = static_cast<const float*>(P.part) + ((size_t)head * P.n_qgroup + qg) * P.n_split * P.part_stride;
    float mx, lt, acc[4];
    merge_splits_b16(base, P.part_stride, NQ, P.n_split, wave, 4, qt, quad, lane, mx, lt, acc);
    if (wave > 0) {
        float (*sp)[64] = s_part[wave - 1];
        sp[0][lane] = mx; sp[1][lane] = lt;
#pragma unroll
        for (int e = 0; e < 4; ++e) sp[2 + e][lane] = acc[e];
    }
    __syncthreads();
    if (wave == 0) {
        float cm = mx;
#pragma unroll
        for (int w = 0; w < 3; ++w) cm = fmaxf(cm, s_part[w][0][lane]);
        const float a0 = (mx == -INFINITY) ? 0.f : fast_exp2(mx - cm);
        lt *= a0;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] *= a0;
#pragma unroll
        for (int w = 0; w < 3; ++w) {
            const float mw = s_part[w][0][lane];
            const float sc = (mw == -INFINITY) ? 0.f : fast_exp2(mw - cm);
            lt = fmaf(sc, s_part[w][1][lane], lt);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fmaf(sc, s_part[w][2 + e][lane], acc[e]);
        }
        if (i >= 0 && i < n)
            store_quad_b16(static_cast<bf16_t*>(P.out) + (size_t)head * P.L * kD, i, quad, h, lt, acc);
    }
}

// =============================================================================
// Merge kernel, for heads cut into many key splits (n_split > kTicketMaxSplit):
// one work-group per selected query merges that query's per-split records, in
// split order, and writes its output row.  With that many splits the records of
// one head are hundreds of KB, too much for the single work-group that draws the
// last ticket, so the merge gets a launch of its own and u * B * H work-groups.
// =============================================================================
template <typename T, typename R, bool ACC_LAYOUT>
__global__ __launch_bounds__(256)
void merge_kernel(const AttendParams P)
{
    constexpr int kMaxSplit = 512;
    __shared__ R s_w[kMaxSplit];
    __shared__ R s_part[4][kD];
    __shared__ R s_red[2][4];
    const int rank = blockIdx.x, head = blockIdx.y;
    const int b = head / P.H;
    const int n = valid_len(P.lengths, b, P.L);
    const int u = P.ucount[b];
    if (rank >= u) return;
    const int i = P.sel[(size_t)head * P.u_max + rank];
    if (i < 0 || i >= n) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nq = P.nq, qg = rank / nq, q = rank % nq;
    const R* base = static_cast<const R*>(P.part) + ((size_t)head * P.n_qgroup + qg) * P.n_split * P.part_stride;

    // every split has a record (empty ones carry m = -inf, l = 0, O = 0)
    R ms[2], ls[2];                                   // this thread's splits: tid, tid + 256
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int s = tid + 256 * k;
        const R* rec = base + (size_t)(s < P.n_split ? s : P.n_split - 1) * P.part_stride;
        const R mv = rec[q], lv = rec[nq + q];
        ms[k] = s < P.n_split ? mv : (R)-INFINITY;
        ls[k] = s < P.n_split ? lv : (R)0;
    }
    R mx = ms[0] > ms[1] ? ms[0] : ms[1];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { const R o = __shfl_xor(mx, off, 64); mx = o > mx ? o : mx; }
    if (lane == 0) s_red[0][wave] = mx;
    __syncthreads();
    mx = s_red[0][0];
#pragma unroll
    for (int w = 1; w < 4; ++w) mx = s_red[0][w] > mx ? s_red[0][w] : mx;
    R lt = 0;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int s = tid + 256 * k;
        const R wgt = (ms[k] == (R)-INFINITY) ? (R)0 : rec_exp2(ms[k] - mx);
        if (s < P.n_split) s_w[s] = ACC_LAYOUT ? wgt * ls[k] : wgt;   // (records in accumulator layout hold O / l)
        lt += wgt * ls[k];
    }
    // sum of l over the work-group in a fixed order: lanes by xor tree, waves in order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) lt += __shfl_xor(lt, off, 64);
    if (lane == 0) s_red[1][wave] = lt;
    __syncthreads();
    lt = s_red[1][0] + s_red[1][1] + s_red[1][2] + s_red[1][3];

    // wave w adds splits w, w+4, ... for element `lane`; the four partial sums are added in order
    R acc = 0;
    for (int s = wave; s < P.n_split; s += 4) {
        const R* rec = base + (size_t)s * P.part_stride + 2 * nq;
        const R ov = ACC_LAYOUT ? (R)reinterpret_cast<const float*>(rec)[(q >> 4) * 1024 + F32Tile::reg_of(lane) * 64 + F32Tile::grp_of(lane) * 16 + (q & 15)]
                                : rec[q * kD + lane];
        acc += s_w[s] * ov;
    }
    s_part[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        const R tot = s_part[0][lane] + s_part[1][lane] + s_part[2][lane] + s_part[3][lane];
        const float val = lt > 0 ? (float)(tot / lt) : 0.f;
        T* row = static_cast<T*>(P.out) + ((size_t)head * P.L + i) * kD;
        if constexpr (sizeof(T) == 4) {
            reinterpret_cast<float*>(row)[lane] = val;
        } else {
            const float nxt = __shfl_down(val, 1, 64);
            if ((lane & 1) == 0) reinterpret_cast<uint32_t*>(row)[lane >> 1] = pack_bf16(val, nxt);
        }
    }
}

// =============================================================================
// Many selected queries per head (the ratio rule of Sec. 3.2 keeps half of them):
// splitting the keys over waves would leave every work-group with a large merge
// of partial states, so here a wave owns its selected queries (16 for float32
// tensors, 32 for bfloat16) and walks every key tile of the head with online
// softmax, as in dense attention: no partial records, no merge.  A work-group of
// 4 waves takes 64 (float32) or 128 (bfloat16) consecutive ranks of the head's
// selection and its share of the rows to fill.  grid (query blocks, heads).
// =============================================================================
// KSPLIT = 2 (float32 tensors, fewer than two waves per SIMD otherwise): 8 waves, the second four walk
// the second half of the key tiles for the same queries and hand their state (m, l, O) to the first
// four through LDS, lane for lane: a two-way merge inside the work-group, once per kernel.
template <int KSPLIT>
__global__ __launch_bounds__(256 * KSPLIT)
void attend_rows_f32_kernel(const AttendParams P)
{
    constexpr int NT = 256 * KSPLIT;
    __shared__ CommonScratch<NT> cs;
    __shared__ double s_state[KSPLIT == 2 ? 4 * 18 * 64 : 1];       // [query tile][m, l, O^T 16][lane]
    const int qblock = blockIdx.x, head = blockIdx.y;
    const int H = P.H, L = P.L;
    const int n = valid_len(P.lengths, head / H, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wq = wave & 3, kh = wave >> 2;                        // query tile, key half
    const int c = lane & 15, g = lane >> 4;
    const float* Qh = static_cast<const float*>(P.Q) + (size_t)head * L * kD;
    const float* Kh = static_cast<const float*>(P.K) + (size_t)head * L * kD;
    const float* Vh = static_cast<const float*>(P.V) + (size_t)head * L * kD;
    float* oh = static_cast<float*>(P.out) + (size_t)head * L * kD;

    // this wave's keys: tiles [0, half) or [half, all)
    const int n_tiles = (n + kTile - 1) / kTile;
    const int half = KSPLIT == 2 ? (n_tiles + 1) / 2 : n_tiles;
    const int j_begin = kh * half * kTile;
    const int j_end = (kh == KSPLIT - 1) ? n : (half * kTile < n ? half * kTile : n);

    F32Tile tile;
    tile.init();
    float4 knext[2][4];
    int u;
    const int* selp = attend_prologue<NT>(P, head, n, qblock, cs, u,
                                          [&]() { F32Tile::load_k_into(knext, Kh, j_begin, n, c, g); });
    const int rank = qblock * 64 + wq * 16 + c;
    int qi = rank < u ? selp[rank] : -1;
    if (qi >= n) qi = -1;
    tile.load_q(Qh, qi, qi >= 0, g);
    fill_rows<float, NT>(P, oh, Vh, selp, u, n, qblock, cs);
    const bool live = qblock * 64 + wq * 16 < u;          // wave-uniform: some rank of this wave is in use
    if (KSPLIT == 1 && !live) return;
    if (live) {
        for (int j0 = j_begin; j0 < j_end; j0 += kTile) {
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int v = 0; v < 4; ++v) tile.kreg[sb][v] = knext[sb][v];
            // tiles that lie wholly inside the valid rows (all but the last one or two) need no masks
            if (j0 + 2 * kTile <= n) F32Tile::load_k_into<true>(knext, Kh, j0 + kTile, n, c, g);
            else                     F32Tile::load_k_into<false>(knext, Kh, j0 + kTile, n, c, g);
            if (j0 + kTile <= n) tile.step<false, true>(Vh, j0, n, c, g);
            else                 tile.step<false, false>(Vh, j0, n, c, g);
        }
    }
    if constexpr (KSPLIT == 2) {
        double* ex = s_state + (size_t)wq * 18 * 64 + lane;
        if (kh == 1 && live) {
            ex[0] = (double)tile.m_run; ex[64] = tile.l_run;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 4; ++r) ex[(2 + 4 * dt + r) * 64] = tile.oacc[dt][r];
        }
        lds_barrier();
        if (kh == 1 || !live) return;
        const float m_b = (float)ex[0];
        const float m_new = fmaxf(tile.m_run, m_b);
        // (the first half holds key 0, so m_new is finite whenever n > 0)
        const double wa = tile.m_run == -INFINITY ? 0.0 : exp2_f64((double)tile.m_run - (double)m_new);
        const double wb = m_b == -INFINITY ? 0.0 : exp2_f64((double)m_b - (double)m_new);
        tile.l_run = tile.l_run * wa + ex[64] * wb;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) tile.oacc[dt][r] = tile.oacc[dt][r] * wa + ex[(2 + 4 * dt + r) * 64] * wb;
    }
    double l_tot = tile.l_run;
    l_tot += __shfl_xor(l_tot, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    if (qi >= 0) {
        const double inv = l_tot > 0.0 ? 1.0 / l_tot : 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)          // elements 16r + 4g .. + 3: one 16-byte store
            *reinterpret_cast<float4*>(oh + (size_t)qi * kD + F32Tile::elem(0, r, g)) =
                make_float4((float)(tile.oacc[0][r] * inv), (float)(tile.oacc[1][r] * inv),
                            (float)(tile.oacc[2][r] * inv), (float)(tile.oacc[3][r] * inv));
    }
}

// bfloat16: 8 waves, 4 query tiles of 32 selected queries x 2 halves of the keys (two waves per
// tile measured faster than one at every size: conformer_l with half the queries kept 91 -> 79 us).
// Each group of four waves stages the 32-key tiles of K and V of its half once in LDS
// (double-buffered, one barrier per tile); the halves merge as for float32.
__global__ __launch_bounds__(512)
void attend_rows_bf16_kernel(const AttendParams P)
{
    constexpr int KSPLIT = 2;
    constexpr int NT = 256 * KSPLIT;
    __shared__ CommonScratch<NT> cs;
    __shared__ __attribute__((aligned(16))) uint16_t sKV[KSPLIT][2][2][kTile * kB16Stride];   // [key half][buffer][K|V]
    static_assert(sizeof(sKV) >= 4 * 34 * 64 * sizeof(float), "the state hand-over reuses the tile buffers");
    const int qblock = blockIdx.x, head = blockIdx.y;
    const int H = P.H, L = P.L;
    const int n = valid_len(P.lengths, head / H, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wq = wave & 3, kh = wave >> 2;                        // query tile, key half
    const int c = lane & 31, h = lane >> 5;
    const bf16_t* Qh = static_cast<const bf16_t*>(P.Q) + (size_t)head * L * kD;
    const bf16_t* Kh = static_cast<const bf16_t*>(P.K) + (size_t)head * L * kD;
    const bf16_t* Vh = static_cast<const bf16_t*>(P.V) + (size_t)head * L * kD;
    bf16_t* oh = static_cast<bf16_t*>(P.out) + (size_t)head * L * kD;

    // this half's keys: tiles [0, half) or [half, all); every wave makes `half` rounds (the barriers are the work-group's)
    const int n_tiles = (n + kTile - 1) / kTile;
    const int half = KSPLIT == 2 ? (n_tiles + 1) / 2 : n_tiles;
    const int j_begin = kh * half * kTile;
    const int j_end = (kh == KSPLIT - 1) ? n : (half * kTile < n ? half * kTile : n);

    // thread t of a half stages 16 bytes of row t / 8 of the half's tile
    const int srow = (tid & 255) >> 3, scol = tid & 7;
    auto fetch = [&](int j0, uint4& xk, uint4& xv) {
        const int j = j0 + srow;
        const bool ok = j < n;
        const size_t ro = (size_t)(ok ? j : last_row(n)) * kD;
        xk = reinterpret_cast<const uint4*>(Kh + ro)[scol];
        xv = reinterpret_cast<const uint4*>(Vh + ro)[scol];
        if (!ok) { xk = make_uint4(0u, 0u, 0u, 0u); xv = xk; }
    };
    auto put = [&](int buf, const uint4& xk, const uint4& xv) {
        *reinterpret_cast<uint4*>(&sKV[kh][buf][0][srow * kB16Stride + scol * 8]) = xk;
        *reinterpret_cast<uint4*>(&sKV[kh][buf][1][srow * kB16Stride + scol * 8]) = xv;
    };
    uint4 xk, xv;
    int u;
    const int* selp = attend_prologue<NT>(P, head, n, qblock, cs, u, [&]() { fetch(j_begin, xk, xv); });
    Bf16Tile<1> tile;
    tile.init();
    const int rank = qblock * 128 + wq * 32 + c;
    int qi = rank < u ? selp[rank] : -1;
    if (qi >= n) qi = -1;
    tile.load_q(0, Qh, qi, qi >= 0, h);
    fill_rows<bf16_t, NT>(P, oh, Vh, selp, u, n, qblock, cs);
    if (qblock * 128 >= u) return;                        // work-group-uniform: no rank of this block is in use
    put(0, xk, xv);
    __syncthreads();
    int buf = 0;
    {
        // the halves differ by at most one tile: all rounds but the last need no test (a branch around the
        // step costs 8 % of the loop)
        int j0 = j_begin;
        for (int i = 0; i + 1 < half; ++i, j0 += kTile) {
            fetch(j0 + kTile, xk, xv);                       // next tile, in flight during the step
            tile.step(sKV[kh][buf][0], sKV[kh][buf][1], j0, n, c, h);
            put(buf ^ 1, xk, xv);
            __syncthreads();
            buf ^= 1;
        }
        if (j0 < j_end) tile.step(sKV[kh][buf][0], sKV[kh][buf][1], j0, n, c, h);     // (wave-uniform)
        __syncthreads();                                     // the buffers are reused below
    }
    {
        // every wave is past its last tile: the tile buffers carry the second half's state to the first
        float* ex = reinterpret_cast<float*>(&sKV[0][0][0][0]) + (size_t)wq * 34 * 64 + lane;
        if (kh == 1) {
            ex[0] = tile.m_run[0]; ex[64] = tile.l_run[0];
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) ex[(2 + 16 * dt + r) * 64] = tile.oacc[0][dt][r];
        }
        lds_barrier();
        if (kh == 1) return;
        const float m_b = ex[0];
        const float m_new = fmaxf(tile.m_run[0], m_b);      // finite whenever n > 0: the first half holds key 0
        const float wa = tile.m_run[0] == -INFINITY ? 0.f : fast_exp2(tile.m_run[0] - m_new);
        const float wb = m_b == -INFINITY ? 0.f : fast_exp2(m_b - m_new);
        tile.l_run[0] = tile.l_run[0] * wa + ex[64] * wb;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) tile.oacc[0][dt][r] = tile.oacc[0][dt][r] * wa + ex[(2 + 16 * dt + r) * 64] * wb;
    }
    const float l_tot = tile.l_run[0] + swap_half(tile.l_run[0]);
    if (qi >= 0) {
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int e = 32 * dt + 8 * r4 + 4 * h;
                const uint2 pk = make_uint2(pack_bf16(tile.oacc[0][dt][4 * r4 + 0] * inv, tile.oacc[0][dt][4 * r4 + 1] * inv),
                                            pack_bf16(tile.oacc[0][dt][4 * r4 + 2] * inv, tile.oacc[0][dt][4 * r4 + 3] * inv));
                *reinterpret_cast<uint2*>(oh + (size_t)qi * kD + e) = pk;
            }
    }
}

// The four attend kernels that use more than the default 64 KB of dynamic LDS, and the
// devices on which each has had its limit raised.
static std::atomic<uint64_t> g_attend_raised[6];
static hipError_t raise_attend_limit(int k)
{
    const void* fn[6] = {(const void*)attend_f32_kernel<1, false>, (const void*)attend_f32_kernel<2, false>,
                         (const void*)attend_f32_kernel<1, true>, (const void*)attend_f32_kernel<2, true>,
                         (const void*)attend_bf16_kernel<1>, (const void*)attend_bf16_kernel<2>};
    return ensure_lds_limit(fn[k], k < 4 ? kF32SmemBytes : kB16SmemBytes, g_attend_raised[k]);
}
hipError_t init_attend()
{
    for (int k = 0; k < 6; ++k) { const hipError_t e = raise_attend_limit(k); if (e != hipSuccess) return e; }
    return hipSuccess;
}

hipError_t launch_attend(const Plan& p, const Args& a, const Scratch& w)
{
    AttendParams P;
    P.Q = a.Q; P.K = a.K; P.V = a.V; P.lengths = a.lengths;
    P.vpart = (p.n_seg > 0 || p.stream_lists) ? w.vseg : w.vpart;
    P.n_vpart = p.n_seg > 0 ? p.n_seg : p.stream_lists ? p.n_lists : p.n_chunk; P.mu = w.mu; P.sel = w.sel; P.ucount = w.u; P.ticket = w.ticket;
    P.part = w.part; P.out = a.out;
    P.H = p.H; P.L = p.L; P.u_max = p.u_max; P.n_split = p.n_split; P.n_qgroup = p.n_qgroup;
    P.rounds = p.tiles_per_wave; P.part_stride = (int)p.part_stride; P.n_chunk = p.n_lists;
    P.fused_select = p.fused_select; P.rows_per_wg = p.rows_per_wg; P.urule = a.urule; P.fill = a.fill;
    P.cand = w.cand; P.cand_len = p.cand_len; P.separate_merge = p.separate_merge; P.nq = p.nq_group;
    P.given_sel = p.given_inline ? a.given_sel : nullptr; P.given_u = a.given_u;
    if (p.rows_mode) {
        const dim3 rgrid(p.n_qgroup, p.BH);
        if (p.dtype == PSA_F32 && p.rows_mode == 2) hipLaunchKernelGGL(attend_rows_f32_kernel<2>, rgrid, dim3(512), 0, a.stream, P);
        else if (p.dtype == PSA_F32) hipLaunchKernelGGL(attend_rows_f32_kernel<1>, rgrid, dim3(256), 0, a.stream, P);
        else                    hipLaunchKernelGGL(attend_rows_bf16_kernel, rgrid, dim3(512), 0, a.stream, P);
        return hipGetLastError();
    }
    dim3 grid(p.n_split, p.n_qgroup, p.BH);
    if (p.dtype == PSA_F32) {
        // 72 KB of dynamic LDS: above the 64 KB default
        const bool all_full = a.lengths == nullptr && p.L % kTile == 0;      // every key tile of every head is wholly valid
        const int which = (p.nq_group == 16 ? 0 : 1) + (all_full ? 2 : 0);
        const hipError_t e = raise_attend_limit(which);
        if (e != hipSuccess) return e;
        if (which == 0)      hipLaunchKernelGGL((attend_f32_kernel<1, false>), grid, dim3(512), kF32SmemBytes, a.stream, P);
        else if (which == 1) hipLaunchKernelGGL((attend_f32_kernel<2, false>), grid, dim3(512), kF32SmemBytes, a.stream, P);
        else if (which == 2) hipLaunchKernelGGL((attend_f32_kernel<1, true>), grid, dim3(512), kF32SmemBytes, a.stream, P);
        else                 hipLaunchKernelGGL((attend_f32_kernel<2, true>), grid, dim3(512), kF32SmemBytes, a.stream, P);
    } else {
        const int which = p.nq_group == 32 ? 0 : 1;
        const hipError_t e = raise_attend_limit(4 + which);
        if (e != hipSuccess) return e;
        if (which == 0) hipLaunchKernelGGL(attend_bf16_kernel<1>, grid, dim3(512), kB16SmemBytes, a.stream, P);
        else            hipLaunchKernelGGL(attend_bf16_kernel<2>, grid, dim3(512), kB16SmemBytes, a.stream, P);
    }
    if (p.separate_merge) {
        if (p.dtype == PSA_F32) {
            hipLaunchKernelGGL((merge_kernel<float, double, true>), dim3(p.u_max, p.BH), dim3(256), 0, a.stream, P);
        } else {
            const int n_qtile = p.n_qgroup * (p.nq_group / 32);
            hipLaunchKernelGGL(merge_b16_kernel, dim3(8, n_qtile, p.BH), dim3(256), 0, a.stream, P);
        }
    }
    return hipGetLastError();
}

}  // namespace psa

// C ABI of libprobsparse.so: argument checks, launch plan, workspace carving and
// the stage pipeline.  All checks run before the first launch; nothing here
// allocates, frees or synchronises.
#include <stdio.h>
#include <math.h>
#include <string.h>

#include "psa_internal.h"

namespace psa {

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static int check_shape(const psa_shape_t* s)
{
    if (!s) return PSA_ERR_NULL;
    if (s->dtype != PSA_F32 && s->dtype != PSA_BF16) return PSA_ERR_DTYPE;
    if (s->B < 1 || s->H < 1 || s->L_Q < 1 || s->L_K < 1 || s->U < 1) return PSA_ERR_SHAPE;
    if (s->D != kD) return PSA_ERR_SHAPE;
    if (s->L_Q != s->L_K) return PSA_ERR_SHAPE;           // self-attention only (Sec. 3.1)
    if ((int64_t)s->B * s->H > 65535) return PSA_ERR_SHAPE;   // heads ride on a 16-bit grid axis
    if (s->L_K > (1 << 22)) return PSA_ERR_SHAPE;
    if (s->U > (1 << 16)) return PSA_ERR_SHAPE;
    return PSA_OK;
}

static int u_max_of(URule r, int L)
{
    double x = r.rule == PSA_U_RATIO ? ceil(r.factor * (double)L) : ceil(r.factor * log((double)L));
    if (!(x >= 1.0)) x = 1.0;
    if (x > (double)L) x = (double)L;
    return (int)x;
}

static bool good_rule(URule r)
{
    return (r.rule == PSA_U_LOG || r.rule == PSA_U_RATIO) && r.factor > 0.0 && isfinite(r.factor);
}

bool make_plan(const psa_shape_t* s, URule urule, int u_stride, Plan* p)
{
    if (check_shape(s) != PSA_OK) return false;
    p->given_indices = u_stride > 0;
    if (!p->given_indices && !good_rule(urule)) return false;
    if (u_stride < 0 || u_stride > s->L_K) return false;
    p->B = s->B; p->H = s->H; p->L = s->L_K; p->U = s->U; p->dtype = s->dtype;
    p->BH = s->B * s->H;
    p->u_max = p->given_indices ? u_stride : u_max_of(urule, p->L);
    // float32 tensors run on 16-wide float64 MFMA tiles (<= 2 per work-group),
    // bfloat16 tensors on 32-wide tiles (<= 2 per work-group)
    // (with very few heads, two groups of 16 queries give twice the work-groups)
    if (p->dtype == PSA_F32) p->nq_group = (p->u_max > 16 && (int64_t)p->BH * ((p->L + 127) / 128) >= 64) ? 32 : 16;
    else                     p->nq_group = p->u_max > 32 ? 64 : 32;
    p->n_qgroup = (p->u_max + p->nq_group - 1) / p->nq_group;

    // key splits: enough work-groups to cover the 256 CUs twice (float32) or once
    // (bfloat16, whose work-groups take a CU each).  One round of an attend
    // work-group walks `tiles_wg` tiles of 32 keys: 8 (one per wave) for bfloat16;
    // 8 or 4 for float32 (8 waves over 1 or 2 column tiles).
    const int tiles_wg = p->dtype == PSA_F32 ? (p->nq_group == 16 ? 8 : 4) : 8;
    const int n_tiles = (p->L + kTile - 1) / kTile;
    const int max_split = (n_tiles + tiles_wg - 1) / tiles_wg;
    const int wg_goal = p->dtype == PSA_F32 ? 512 : 256;     // bfloat16: one 8-wave work-group per CU
    int target = (wg_goal + p->BH * p->n_qgroup - 1) / (p->BH * p->n_qgroup);
    if (target < 1) target = 1;
    int n_split = target < max_split ? target : max_split;
    if (n_split > kMaxSplit) n_split = kMaxSplit;
    p->tiles_per_wave = (n_tiles + n_split * tiles_wg - 1) / (n_split * tiles_wg);      // rounds
    p->n_split = (n_tiles + p->tiles_per_wave * tiles_wg - 1) / (p->tiles_per_wave * tiles_wg);
    // bfloat16: any split brings the hand-over of records to the head's last work-group (or, beyond 8 splits, the
    // merge kernel) while a round of tiles takes about 2 us, so heads are cut only where that saves at least three
    // rounds (B=16 H=8 L=1024: 20.1 us whole against 20.5 us in two splits that save two rounds)
    if (p->dtype == PSA_BF16 && p->n_split > 1) {
        const int rounds_whole = (n_tiles + tiles_wg - 1) / tiles_wg;
        if (rounds_whole - p->tiles_per_wave < 3) { p->n_split = 1; p->tiles_per_wave = rounds_whole; }
    }

    // Many selected queries per head: no key split over work-groups, a wave owns its queries (see
    // attend_rows_*_kernel).  rows_mode 1: a wave walks all keys; 2: two waves share a query tile, each
    // on half of the keys, and merge inside the work-group.  float32: 1 from 2048 waves on (two per
    // SIMD: a lone wave cannot overlap its softmax arithmetic with its matrix products), else 2.
    // bfloat16: always 2 (more waves per SIMD hide more of a tile's round trips).  Measured, attend
    // stage, half of the queries kept: conformer_s 70 us with the keys split over work-groups, 72 us
    // with one wave per query tile, 60 us with two; float32 B=8 H=4 L=512: 108 -> 60 us, B=32 H=4
    // L=512 (2048 waves) 116 us with one wave per tile against 119 us with two; bfloat16 B=32 H=4
    // L=512: 32 -> 20 us, B=24 H=4 L=700: 88 -> 40 us; conformer_l: 102 us split over work-groups,
    // 91 us one wave per tile, 79 us two.
    // With few waves the split over work-groups uses more CUs and stays: float32 below 256 waves
    // (B=2 H=4 L=512: 53 against 59 us), bfloat16 below 1024 or while its work-groups fit one round
    // (B=2 H=8 L=2048: 29 against 39 us).  Between 64 and 255 selected queries a head fills only one
    // to four work-groups of this kind, so float32 takes them only with 512 waves or more and all
    // work-groups in one round (B=32 H=4 L=512 u=75: 94 -> 60 us; but B=16 H=4 L=1024 u=84, 384
    // waves: 82 us split over work-groups against 107 us; B=64 H=4 L=512 u=75, two rounds: 101
    // against 119 us); bfloat16 by the same rule as above (B=128 H=4 L=512 u=75: 56 -> 31 us).
    const int q_per_wave = p->dtype == PSA_F32 ? 16 : 32;
    const int64_t row_waves = (int64_t)p->BH * ((p->u_max + q_per_wave - 1) / q_per_wave);
    p->rows_mode = 0;
    if (p->u_max >= kRowsModeMin) {
        const int64_t split_wgs = (int64_t)p->BH * p->n_qgroup * p->n_split;
        if (p->dtype == PSA_F32) {
            const int64_t rows_wgs = (int64_t)p->BH * ((p->u_max + 63) / 64);
            if (p->u_max >= 256) p->rows_mode = row_waves >= 2048 ? 1 : (row_waves >= 256 ? 2 : 0);
            else if (row_waves >= 512 && rows_wgs <= 256) p->rows_mode = 2;
        } else if (row_waves >= 1024 || (row_waves >= 512 && split_wgs > 256)) p->rows_mode = 2;
    }
    if (p->rows_mode) {
        p->nq_group = p->dtype == PSA_F32 ? 64 : 128;       // 4 waves of 16 or 32 queries
        p->n_qgroup = (p->u_max + p->nq_group - 1) / p->nq_group;
        p->n_split = 1;
        p->tiles_per_wave = n_tiles;
    }
    p->n_wg_head = p->n_split * p->n_qgroup;
    p->rows_per_wg = (p->L + p->n_wg_head - 1) / p->n_wg_head;

    const size_t row_bytes = p->dtype == PSA_F32 ? 256 : 128;
    p->measure_lds = !p->given_indices && (size_t)p->L * row_bytes <= (size_t)kLdsMaxBytes;
    const int mq = p->measure_lds ? kLdsQueries : kMeasureQueries;
    p->n_chunk = (p->L + mq - 1) / mq;
    // LDS measure kernel (one work-group per CU): once the heads alone would fill the
    // 256 CUs, a work-group takes several chunks of its head and loads the head's K once
    p->chunks_per_wg = 1;
    if (p->measure_lds) {
        // bfloat16 heads whose K fits 64 KB: two work-groups per CU (one copies its K while the other gathers)
        const bool two_per_cu = p->dtype == PSA_BF16 && (size_t)p->L * row_bytes <= (size_t)kLdsMaxBytes / 2;
        if (two_per_cu) p->measure_lds = 2;
        const int slots = two_per_cu ? 512 : 256;
        while (p->chunks_per_wg < p->n_chunk &&
               (int64_t)p->BH * ((p->n_chunk + p->chunks_per_wg - 1) / p->chunks_per_wg) > slots) ++p->chunks_per_wg;
    }
    else if (!p->given_indices) {
        // streaming measure kernel: about two persistent work-groups per CU, each on consecutive chunks of one head
        const int64_t chunks_all = (int64_t)p->BH * p->n_chunk;
        int cpw = (int)((chunks_all + 511) / 512);
        cpw = cpw < 1 ? 1 : (cpw > 16 ? 16 : cpw);
        p->chunks_per_wg = cpw < p->n_chunk ? cpw : p->n_chunk;
    }
    // sorted per-chunk candidate lists: only with the LDS measure kernel (few chunks per head)
    p->cand_len = 0;
    if (p->measure_lds) {
        const int len = p->u_max < kLdsQueries ? p->u_max : kLdsQueries;
        if (p->n_chunk * len <= kMaxCandidates) p->cand_len = len;
    }
    p->n_lists = p->n_chunk;
    p->stream_lists = 0;
    // Streamed heads: a work-group of the measure kernel ranks the queries of its own chunks and hands on its
    // best u as one sorted list, exactly as a chunk of the LDS kernel does; where the head's work-groups are
    // at most 8 (the attend prologue merges up to 8 lists) no select launch is needed (conformer_l: 8.3 us).
    if (!p->measure_lds && !p->given_indices && p->U <= kPipeMaxSamples) {
        const int groups = (p->n_chunk + p->chunks_per_wg - 1) / p->chunks_per_wg;
        const int span = p->chunks_per_wg * kMeasureQueries;
        const int len = p->u_max < span ? p->u_max : span;
        // (the ranking at the end of a work-group is all pairs of its queries: up to 256 of them, a microsecond)
        // (few candidates only: every attend work-group of the head merges them; with hundreds of kept queries per
        // head the select kernel is the cheaper way: conformer_l at r_sparse = 0.5 134 against 123 us)
        if (groups <= 8 && span <= kListMax && (int64_t)groups * len <= 512) {
            p->cand_len = len; p->n_lists = groups; p->stream_lists = 1;
        }
    }
    p->n_seg = 0;
    p->seg_len = 0;
    // Long heads: the measures of a head are cut into up to 8 segments, a work-group per segment
    // picks the segment's best queries and hands them on as a sorted list, like a chunk of the LDS
    // measure kernel does (one work-group per head loads and ranks all L measures on one CU: 15 us
    // at L = 4096 against 8.4 us in segments).  Only where all segment work-groups run at once
    // (at most one per CU) and the head is long enough to pay for the list merge in the attend
    // stage (about 2.5 us); up to 2048 measures one work-group per head is as fast.
    if (!p->measure_lds && !p->given_indices && p->cand_len == 0 && p->L > 2048) {
        int n_seg = (p->L + 511) / 512;
        if (n_seg > kSegMax) n_seg = kSegMax;
        if (n_seg > 256 / p->BH) n_seg = 256 / p->BH;
        if (n_seg >= 2) {
            const int seg_len = ((p->L + n_seg - 1) / n_seg + kMeasureQueries - 1) / kMeasureQueries * kMeasureQueries;
            n_seg = (p->L + seg_len - 1) / seg_len;
            const int len = p->u_max < seg_len ? p->u_max : seg_len;
            if (seg_len <= kSegKeys && len <= kSegCandMax && n_seg * len <= kMaxCandidates) {
                p->n_seg = n_seg; p->seg_len = seg_len; p->cand_len = len; p->n_lists = n_seg;
            }
        }
    }
    p->fused_select = p->cand_len > 0;
    // caller-given index sets that fit the attend work-groups' LDS list, few enough column-sum chunks
    // for one wave to add up: no prep kernel (one launch less: conformer_s 27.8 -> 25 us)
    p->given_inline = p->given_indices && p->u_max <= kSelLdsMax && p->n_chunk <= 64;
    p->separate_merge = p->n_split > kTicketMaxSplit;

    // float32 tensors: m, l as float64 and 64 float32 values per query (34 doubles); bfloat16: 66 floats
    p->part_stride = (size_t)p->nq_group * (p->dtype == PSA_F32 ? 2 + kD / 2 : kD + 2);
    p->part_elem = p->dtype == PSA_F32 ? sizeof(double) : sizeof(float);
    size_t off = 0;
    p->off_M = off;      off += align256((size_t)p->BH * p->L * sizeof(float));
    p->off_vpart = off;  off += align256((size_t)p->BH * p->n_chunk * kD * sizeof(double));
    p->off_vseg = off;   off += align256((size_t)p->BH * (p->stream_lists ? p->n_lists : p->n_seg) * kD * sizeof(double));
    p->off_mu = off;     off += align256((size_t)p->BH * kD * sizeof(float));
    p->off_sel = off;    off += align256((size_t)p->BH * p->u_max * sizeof(int));
    p->off_u = off;      off += align256((size_t)p->B * sizeof(int));
    p->off_ticket = off; off += align256((size_t)p->BH * sizeof(int));
    p->off_cand = off;   off += align256((size_t)p->BH * p->n_lists * p->cand_len * sizeof(uint2));
    p->off_part = off;   off += p->rows_mode ? 0 : align256((size_t)p->BH * p->n_qgroup * p->n_split * p->part_stride * p->part_elem);
    p->total = off;
    return true;
}

Scratch carve(const Plan& p, void* workspace)
{
    unsigned char* w = static_cast<unsigned char*>(workspace);
    Scratch s;
    s.M = reinterpret_cast<float*>(w + p.off_M);
    s.vpart = reinterpret_cast<double*>(w + p.off_vpart);
    s.vseg = reinterpret_cast<double*>(w + p.off_vseg);
    s.mu = reinterpret_cast<float*>(w + p.off_mu);
    s.sel = reinterpret_cast<int*>(w + p.off_sel);
    s.ticket = reinterpret_cast<int*>(w + p.off_ticket);
    s.cand = reinterpret_cast<uint2*>(w + p.off_cand);
    s.u = reinterpret_cast<int*>(w + p.off_u);
    s.part = w + p.off_part;
    return s;
}

static inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

static int check_ptrs(const void* Q, const void* K, const void* V, const int32_t* lengths, const void* out,
                      const void* workspace)
{
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(out, 16) ||
        misaligned(lengths, 4) || misaligned(workspace, 256)) return PSA_ERR_ALIGN;
    return PSA_OK;
}

static int run(const void* Q, const void* K, const void* V, const int32_t* lengths, const int32_t* sample_idx,
               const psa_options_t* opt, void* out, const psa_shape_t* shape, void* workspace, size_t workspace_bytes,
               void* stream, int stage_mask, float* M_out, int32_t* sel_out, int32_t* u_out, bool checks_only = false)
{
    if (!Q || !K || !V || !sample_idx || !out || !shape || !workspace || !opt) return PSA_ERR_NULL;
    int rc = check_shape(shape);
    if (rc != PSA_OK) return rc;
    const URule urule{opt->u_rule, opt->factor};
    if (!good_rule(urule)) return PSA_ERR_ARG;
    if (opt->fill != PSA_FILL_MEAN && opt->fill != PSA_FILL_VALUE) return PSA_ERR_ARG;
    if (stage_mask <= 0 || (stage_mask & ~PSA_STAGE_ALL)) return PSA_ERR_ARG;
    rc = check_ptrs(Q, K, V, lengths, out, workspace);
    if (rc != PSA_OK) return rc;
    if (misaligned(sample_idx, 4)) return PSA_ERR_ALIGN;
    Plan p;
    if (!make_plan(shape, urule, 0, &p)) return PSA_ERR_SHAPE;
    if (workspace_bytes < p.total) return PSA_ERR_WORKSPACE;
    if (checks_only) return PSA_OK;

    Args a;
    a.Q = Q; a.K = K; a.V = V; a.lengths = lengths; a.idx = sample_idx; a.out = out;
    a.urule = urule; a.fill = opt->fill; a.given_sel = nullptr; a.given_u = nullptr;
    a.stream = static_cast<hipStream_t>(stream);
    const Scratch w = carve(p, workspace);

    if ((stage_mask & PSA_STAGE_MEASURE) && launch_measure(p, a, w) != hipSuccess) return PSA_ERR_HIP;
    if (stage_mask & PSA_STAGE_SELECT) {
        if (p.n_seg > 0) { if (launch_select_segments(p, a, w) != hipSuccess) return PSA_ERR_HIP; }
        else if (!p.fused_select && launch_select(p, a, w) != hipSuccess) return PSA_ERR_HIP;
    }
    if ((stage_mask & PSA_STAGE_ATTEND) && launch_attend(p, a, w) != hipSuccess) return PSA_ERR_HIP;

    if (M_out && hipMemcpyAsync(M_out, w.M, (size_t)p.BH * p.L * sizeof(float), hipMemcpyDeviceToDevice, a.stream) != hipSuccess)
        return PSA_ERR_HIP;
    if (sel_out && hipMemcpyAsync(sel_out, w.sel, (size_t)p.BH * p.u_max * sizeof(int), hipMemcpyDeviceToDevice, a.stream) != hipSuccess)
        return PSA_ERR_HIP;
    if (u_out && hipMemcpyAsync(u_out, w.u, (size_t)p.B * sizeof(int), hipMemcpyDeviceToDevice, a.stream) != hipSuccess)
        return PSA_ERR_HIP;
    return PSA_OK;
}

static int run_c(const void* Q, const void* K, const void* V, const int32_t* lengths, const int32_t* sample_idx,
                 double c, void* out, const psa_shape_t* shape, void* workspace, size_t workspace_bytes,
                 void* stream, int stage_mask, float* M_out, int32_t* sel_out, int32_t* u_out)
{
    const psa_options_t opt{PSA_U_LOG, PSA_FILL_MEAN, c};
    return run(Q, K, V, lengths, sample_idx, &opt, out, shape, workspace, workspace_bytes, stream, stage_mask,
               M_out, sel_out, u_out);
}

static int run_indices(const void* Q, const void* K, const void* V, const int32_t* lengths, const int32_t* sel,
                       const int32_t* u, int u_stride, int fill, void* out, const psa_shape_t* shape,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!Q || !K || !V || !sel || !u || !out || !shape || !workspace) return PSA_ERR_NULL;
    int rc = check_shape(shape);
    if (rc != PSA_OK) return rc;
    if (u_stride < 1 || u_stride > shape->L_K) return PSA_ERR_ARG;
    if (fill != PSA_FILL_MEAN && fill != PSA_FILL_VALUE) return PSA_ERR_ARG;
    rc = check_ptrs(Q, K, V, lengths, out, workspace);
    if (rc != PSA_OK) return rc;
    if (misaligned(sel, 4) || misaligned(u, 4)) return PSA_ERR_ALIGN;
    Plan p;
    if (!make_plan(shape, URule{PSA_U_LOG, 1.0}, u_stride, &p)) return PSA_ERR_SHAPE;
    if (workspace_bytes < p.total) return PSA_ERR_WORKSPACE;

    Args a;
    a.Q = Q; a.K = K; a.V = V; a.lengths = lengths; a.idx = nullptr; a.out = out;
    a.urule = URule{PSA_U_LOG, 1.0}; a.fill = fill; a.given_sel = sel; a.given_u = u;
    a.stream = static_cast<hipStream_t>(stream);
    const Scratch w = carve(p, workspace);
    if (launch_vsum(p, a, w) != hipSuccess) return PSA_ERR_HIP;
    if (!p.given_inline && launch_prep_indices(p, a, w) != hipSuccess) return PSA_ERR_HIP;
    if (launch_attend(p, a, w) != hipSuccess) return PSA_ERR_HIP;
    return PSA_OK;
}

static int check_project(const psa_shape_t* shape, const psa_mhsa_weights_t* w, bool need_in, bool need_out)
{
    if (!shape || !w) return PSA_ERR_NULL;
    const int rc = check_shape(shape);
    if (rc != PSA_OK) return rc;
    if ((int64_t)shape->B * shape->L_K > 0x7FFFFFFF) return PSA_ERR_SHAPE;
    if (need_in && (!w->Wq || !w->Wk || !w->Wv)) return PSA_ERR_NULL;
    if (need_out && !w->Wo) return PSA_ERR_NULL;
    const void* ptrs[8] = {w->Wq, w->Wk, w->Wv, w->Wo, w->bq, w->bk, w->bv, w->bo};
    for (int i = 0; i < 4; ++i) if (misaligned(ptrs[i], 16)) return PSA_ERR_ALIGN;
    for (int i = 4; i < 8; ++i) if (misaligned(ptrs[i], 4)) return PSA_ERR_ALIGN;
    return PSA_OK;
}

// Q, K, V, A of the whole module, then the attention's own scratch
static size_t mhsa_tensor_bytes(const psa_shape_t* s)
{
    return align256((size_t)s->B * s->H * s->L_K * kD * (s->dtype == PSA_F32 ? 4 : 2));
}

// ---- scratch for the entry point that may not allocate: one array per device in the
// library's own image (each GPU the library runs on holds it until the process ends).
// In host code the array's name is only a handle; its device address is looked up once
// per device and that pointer is what the kernels and copies are given.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kStaticScratchDevices = 64;
static std::atomic<void*> g_scratch_ptr[kStaticScratchDevices];

static hipError_t static_scratch_ptr(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kStaticScratchDevices) return hipErrorInvalidDevice;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // the current device's copy of the array (two threads racing here look up the same address)
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return hipSuccess;
}

}  // namespace psa

extern "C" {

size_t probsparse_static_workspace_bytes(void) { return psa::kStaticScratchBytes; }

int probsparse_attn_fwd_static(const void* Q, const void* K, const void* V, const int32_t* lengths,
                               const int32_t* sample_idx, double c, void* out, const psa_shape_t* shape, void* stream)
{
    using namespace psa;
    // the size check is host arithmetic and comes before anything touches the device
    if (!shape) return PSA_ERR_NULL;
    const int rc = check_shape(shape);
    if (rc != PSA_OK) return rc;
    Plan p;
    if (!good_rule(URule{PSA_U_LOG, c})) return PSA_ERR_ARG;
    if (!make_plan(shape, c, &p)) return PSA_ERR_SHAPE;
    if (p.total > kStaticScratchBytes) return PSA_ERR_WORKSPACE;
    if (!Q || !K || !V || !sample_idx || !out) return PSA_ERR_NULL;
    void* ws = nullptr;
    if (static_scratch_ptr(&ws) != hipSuccess) return PSA_ERR_HIP;
    return run_c(Q, K, V, lengths, sample_idx, c, out, shape, ws, kStaticScratchBytes, stream, PSA_STAGE_ALL,
                 nullptr, nullptr, nullptr);
}

int probsparse_qkv_project(const void* X, const psa_mhsa_weights_t* weights, void* Q, void* K, void* V,
                           const psa_shape_t* shape, void* stream)
{
    using namespace psa;
    if (!X || !Q || !K || !V) return PSA_ERR_NULL;
    const int rc = check_project(shape, weights, true, false);
    if (rc != PSA_OK) return rc;
    if (misaligned(X, 16) || misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16)) return PSA_ERR_ALIGN;
    return launch_qkv_project(*shape, X, *weights, Q, K, V, static_cast<hipStream_t>(stream)) == hipSuccess ? PSA_OK : PSA_ERR_HIP;
}

int probsparse_out_project(const void* A, const psa_mhsa_weights_t* weights, void* Y, const psa_shape_t* shape, void* stream)
{
    using namespace psa;
    if (!A || !Y) return PSA_ERR_NULL;
    const int rc = check_project(shape, weights, false, true);
    if (rc != PSA_OK) return rc;
    if (misaligned(A, 16) || misaligned(Y, 16)) return PSA_ERR_ALIGN;
    return launch_out_project(*shape, A, *weights, Y, static_cast<hipStream_t>(stream)) == hipSuccess ? PSA_OK : PSA_ERR_HIP;
}

size_t probsparse_mhsa_workspace_bytes(const psa_shape_t* shape, const psa_options_t* opt)
{
    const size_t inner = probsparse_attn_workspace_bytes_opt(shape, opt);
    if (inner == 0) return 0;
    return 4 * psa::mhsa_tensor_bytes(shape) + inner;
}

int probsparse_mhsa_fwd(const void* X, const psa_mhsa_weights_t* weights, const int32_t* lengths,
                        const int32_t* sample_idx, const psa_options_t* opt, void* Y, const psa_shape_t* shape,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace psa;
    if (!X || !Y || !workspace || !sample_idx || !opt) return PSA_ERR_NULL;
    int rc = check_project(shape, weights, true, true);
    if (rc != PSA_OK) return rc;
    if (misaligned(X, 16) || misaligned(Y, 16) || misaligned(workspace, 256)) return PSA_ERR_ALIGN;
    const size_t inner = probsparse_attn_workspace_bytes_opt(shape, opt);
    if (inner == 0) return PSA_ERR_ARG;
    const size_t tb = mhsa_tensor_bytes(shape);
    if (workspace_bytes < 4 * tb + inner) return PSA_ERR_WORKSPACE;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    void *Q = ws, *K = ws + tb, *V = ws + 2 * tb, *A = ws + 3 * tb;
    // the attention's own checks run before the first launch of the module
    rc = run(Q, K, V, lengths, sample_idx, opt, A, shape, ws + 4 * tb, workspace_bytes - 4 * tb, stream, PSA_STAGE_ALL,
             nullptr, nullptr, nullptr, true);
    if (rc != PSA_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_qkv_project(*shape, X, *weights, Q, K, V, st) != hipSuccess) return PSA_ERR_HIP;
    rc = run(Q, K, V, lengths, sample_idx, opt, A, shape, ws + 4 * tb, workspace_bytes - 4 * tb, stream, PSA_STAGE_ALL,
             nullptr, nullptr, nullptr);
    if (rc != PSA_OK) return rc;
    return launch_out_project(*shape, A, *weights, Y, st) == hipSuccess ? PSA_OK : PSA_ERR_HIP;
}


size_t probsparse_attn_workspace_bytes(const psa_shape_t* shape, double c)
{
    psa::Plan p;
    return psa::make_plan(shape, c, &p) ? p.total : 0;
}

int32_t probsparse_u_max(const psa_shape_t* shape, double c)
{
    psa::Plan p;
    return psa::make_plan(shape, c, &p) ? p.u_max : 0;
}

size_t probsparse_attn_workspace_bytes_opt(const psa_shape_t* shape, const psa_options_t* opt)
{
    psa::Plan p;
    if (!opt || (opt->fill != PSA_FILL_MEAN && opt->fill != PSA_FILL_VALUE)) return 0;
    return psa::make_plan(shape, psa::URule{opt->u_rule, opt->factor}, 0, &p) ? p.total : 0;
}

int32_t probsparse_u_max_opt(const psa_shape_t* shape, const psa_options_t* opt)
{
    psa::Plan p;
    if (!opt) return 0;
    return psa::make_plan(shape, psa::URule{opt->u_rule, opt->factor}, 0, &p) ? p.u_max : 0;
}

int probsparse_attn_fwd_opt(const void* Q, const void* K, const void* V, const int32_t* lengths,
                            const int32_t* sample_idx, const psa_options_t* opt, void* out,
                            const psa_shape_t* shape, void* workspace, size_t workspace_bytes, void* stream,
                            float* M_out, int32_t* sel_out, int32_t* u_out)
{
    return psa::run(Q, K, V, lengths, sample_idx, opt, out, shape, workspace, workspace_bytes, stream,
                    PSA_STAGE_ALL, M_out, sel_out, u_out);
}

size_t probsparse_attn_with_indices_workspace_bytes(const psa_shape_t* shape, int32_t u_stride)
{
    psa::Plan p;
    if (u_stride < 1) return 0;
    return psa::make_plan(shape, psa::URule{PSA_U_LOG, 1.0}, u_stride, &p) ? p.total : 0;
}

int probsparse_attn_fwd_with_indices(const void* Q, const void* K, const void* V, const int32_t* lengths,
                                     const int32_t* sel, const int32_t* u, int32_t u_stride, int32_t fill,
                                     void* out, const psa_shape_t* shape, void* workspace, size_t workspace_bytes,
                                     void* stream)
{
    return psa::run_indices(Q, K, V, lengths, sel, u, u_stride, fill, out, shape, workspace, workspace_bytes, stream);
}

size_t probsparse_attn_bwd_workspace_bytes(const psa_shape_t* shape, int32_t u_stride)
{
    if (psa::check_shape(shape) != PSA_OK || u_stride < 1 || u_stride > shape->L_K) return 0;
    return psa::make_bwd_plan(*shape, u_stride).total;
}

int probsparse_attn_bwd(const void* Q, const void* K, const void* V, const int32_t* lengths,
                        const int32_t* sel, const int32_t* u, int32_t u_stride, int32_t fill,
                        const void* dOut, void* dQ, void* dK, void* dV, const psa_shape_t* shape,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    using namespace psa;
    if (!Q || !K || !V || !sel || !u || !dOut || !dQ || !dK || !dV || !shape || !workspace) return PSA_ERR_NULL;
    const int rc = check_shape(shape);
    if (rc != PSA_OK) return rc;
    if (u_stride < 1 || u_stride > shape->L_K) return PSA_ERR_ARG;
    if (fill != PSA_FILL_MEAN && fill != PSA_FILL_VALUE) return PSA_ERR_ARG;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(dOut, 16) || misaligned(dQ, 16) ||
        misaligned(dK, 16) || misaligned(dV, 16) || misaligned(lengths, 4) || misaligned(sel, 4) || misaligned(u, 4) ||
        misaligned(workspace, 256)) return PSA_ERR_ALIGN;
    const BwdPlan bp = make_bwd_plan(*shape, u_stride);
    if (workspace_bytes < bp.total) return PSA_ERR_WORKSPACE;
    return launch_backward(*shape, bp, Q, K, V, lengths, sel, u, u_stride, fill, dOut, dQ, dK, dV, workspace,
                           static_cast<hipStream_t>(stream)) == hipSuccess ? PSA_OK : PSA_ERR_HIP;
}

int probsparse_attn_fwd(const void* Q, const void* K, const void* V, const int32_t* lengths,
                        const int32_t* sample_idx, double c, void* out, const psa_shape_t* shape,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    return psa::run_c(Q, K, V, lengths, sample_idx, c, out, shape, workspace, workspace_bytes, stream,
                    PSA_STAGE_ALL, nullptr, nullptr, nullptr);
}

int probsparse_attn_fwd_debug(const void* Q, const void* K, const void* V, const int32_t* lengths,
                              const int32_t* sample_idx, double c, void* out, const psa_shape_t* shape,
                              void* workspace, size_t workspace_bytes, void* stream,
                              float* M_out, int32_t* sel_out, int32_t* u_out)
{
    return psa::run_c(Q, K, V, lengths, sample_idx, c, out, shape, workspace, workspace_bytes, stream,
                    PSA_STAGE_ALL, M_out, sel_out, u_out);
}

int probsparse_attn_fwd_stages(const void* Q, const void* K, const void* V, const int32_t* lengths,
                               const int32_t* sample_idx, double c, void* out, const psa_shape_t* shape,
                               void* workspace, size_t workspace_bytes, void* stream, int stage_mask)
{
    return psa::run_c(Q, K, V, lengths, sample_idx, c, out, shape, workspace, workspace_bytes, stream,
                    stage_mask, nullptr, nullptr, nullptr);
}

const char* probsparse_strerror(int code)
{
    switch (code) {
        case PSA_OK:            return "ok";
        case PSA_ERR_NULL:      return "a required pointer is NULL";
        case PSA_ERR_SHAPE:     return "unsupported shape (need B,H,L,U >= 1, D == 64, L_Q == L_K, B*H <= 65535)";
        case PSA_ERR_DTYPE:     return "unsupported dtype (PSA_F32 or PSA_BF16)";
        case PSA_ERR_ARG:       return "invalid argument (factor must be finite and positive; stage mask within PSA_STAGE_ALL; known rule and fill; 1 <= u_stride <= L)";
        case PSA_ERR_WORKSPACE: return "workspace smaller than probsparse_attn_workspace_bytes() (or, for probsparse_attn_fwd_static, the shape needs more than probsparse_static_workspace_bytes())";
        case PSA_ERR_HIP:       return "HIP runtime error on launch or copy";
        case PSA_ERR_ALIGN:     return "device pointer not sufficiently aligned (16 B tensors, 256 B workspace)";
        default:                return "unknown status";
    }
}

int probsparse_describe_plan(const psa_shape_t* shape, const psa_options_t* opt, int32_t u_stride,
                             char* buf, size_t buf_bytes)
{
    using namespace psa;
    if (!shape || !buf || (!opt && u_stride <= 0)) return PSA_ERR_NULL;
    if (buf_bytes == 0) return PSA_ERR_ARG;
    const int rc = check_shape(shape);
    if (rc != PSA_OK) return rc;
    Plan p;
    const URule urule = opt ? URule{opt->u_rule, opt->factor} : URule{PSA_U_LOG, 1.0};
    if (u_stride < 0) return PSA_ERR_ARG;
    if (u_stride == 0 && !good_rule(urule)) return PSA_ERR_ARG;
    if (!make_plan(shape, urule, u_stride, &p)) return u_stride > 0 ? PSA_ERR_ARG : PSA_ERR_SHAPE;
    const char* measure = p.given_indices ? "none" : p.measure_lds == 2 ? "lds_half" : p.measure_lds == 1 ? "lds" : "stream";
    const char* select = p.given_indices ? (p.given_inline ? "given_inline" : "given_prep")
                       : p.n_seg > 0 ? "segments" : p.fused_select ? "lists" : "kernel";
    const char* attend = p.rows_mode == 2 ? "rows_half_keys" : p.rows_mode == 1 ? "rows" : "key_split";
    const char* merge = p.rows_mode ? "none" : p.n_split == 1 ? "none" : p.separate_merge ? "kernel" : "last_work_group";
    const int n = snprintf(buf, buf_bytes,
                           "u_max=%d measure=%s chunks=%d chunks_per_wg=%d select=%s lists=%d list_len=%d segments=%d "
                           "attend=%s queries_per_group=%d query_groups=%d key_splits=%d rounds=%d merge=%s workspace=%zu",
                           p.u_max, measure, p.n_chunk, p.chunks_per_wg, select, p.cand_len > 0 ? p.n_lists : 0, p.cand_len,
                           p.n_seg, attend, p.nq_group, p.n_qgroup, p.n_split, p.tiles_per_wave, merge, p.total);
    return (n < 0 || (size_t)n >= buf_bytes) ? PSA_ERR_ARG : PSA_OK;
}

int probsparse_init(void)
{
    if (psa::init_measure() != hipSuccess || psa::init_attend() != hipSuccess) return PSA_ERR_HIP;
    void* ws = nullptr;
    if (psa::static_scratch_ptr(&ws) != hipSuccess) return PSA_ERR_HIP;      // this device's static scratch
    return PSA_OK;
}

int probsparse_version(void) { return 100; }

}  // extern "C"

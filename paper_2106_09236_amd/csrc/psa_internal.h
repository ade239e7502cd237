// Internal declarations shared by the translation units of libprobsparse.so.
// Host-side plan (grid sizes, workspace carving) and the launch functions of
// the four kernel groups.  Nothing here is visible through the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/probsparse.h"

namespace psa {

constexpr int kD = 64;             // per-head dimension (Sec. 4.2: 256 / 4 heads)
constexpr int kTile = 32;          // keys per MFMA tile in the attend kernel
constexpr int kMeasureQueries = 64; // queries (and V rows) per work-group of the streaming measure kernel
constexpr int kLdsQueries = 128;    // same, for the measure kernel that keeps a head's K in LDS
constexpr int kLdsMaxBytes = 128 * 1024;   // largest K of one head that kernel accepts
constexpr int kSelLdsMax = 2048;           // index lists of up to this many entries are kept in LDS by the attend kernels
constexpr int kTicketMaxSplit = 8;         // up to this many key splits the last work-group of a head merges them
constexpr int kMaxSplit = 512;             // key splits per head the merge kernel handles
constexpr int kMaxCandidates = 2048;       // lists * cand_len an attend work-group can merge in LDS
constexpr int kRowsModeMin = 64;           // from this many selected queries per head on, the attend stage may keep a head's keys in one work-group
constexpr int kSegMax = 8;                 // segments per head of the segment-select kernel (lists the attend stage merges)
constexpr int kSegKeys = 2048;             // most queries of one segment
constexpr int kSegCandMax = 256;           // longest list a segment hands on
constexpr int kPipeMaxSamples = 64;        // samples per query up to which the streaming measure kernel stages a chunk's indices in LDS
constexpr int kListMax = 256;              // most queries a work-group of the streaming measure kernel ranks among themselves

struct bf16_t { uint16_t x; };

// How many queries of an item of n valid frames are kept (stage a2):
//   PSA_U_LOG    ceil(factor * ln n)   the rule of the Informer work (Sec. 1, Sec. 3.2)
//   PSA_U_RATIO  ceil(factor * n)      L_sparse = r_sparse * L (Sec. 3.2, Sec. 4.2)
// both clamped to [1, n].
struct URule { int rule; double factor; };

// Everything the launches need, derived on the host from (shape, c).
struct Plan {
    int B, H, L, U, dtype;
    int BH;
    int u_max;            // upper bound of u_b over all possible lengths
    int nq_group;         // selected queries one attend work-group handles (16, 32 or 64)
    int n_qgroup;         // ceil(u_max / nq_group)
    int measure_lds;      // 1: a head's K fits in LDS for the measure stage; 2: in half of it (two work-groups per CU)
    int n_chunk;          // measure chunks (= V column-sum chunks) per head
    int chunks_per_wg;    // LDS measure kernel: consecutive chunks of a head one work-group takes
    int fused_select;     // 1: top-u selection runs inside the attend work-groups
    int cand_len;         // > 0: sorted candidate lists of this length are handed to the attend stage
    int n_seg;            // > 0: long heads, the lists come from the segment-select kernel, n_seg per head
    int seg_len;          //      queries per segment (a multiple of the measure chunk)
    int n_lists;          // candidate lists per head: measure chunks (LDS measure kernel), work-groups of the streaming kernel, or segments
    int stream_lists;     // 1: the lists (and one V column sum per list, in vseg) come from the streaming measure kernel
    int n_split;          // attend work-groups per head along the key axis
    int tiles_per_wave;   // rounds of key tiles an attend work-group walks
    int n_wg_head;        // attend work-groups per head = n_split * n_qgroup
    int rows_per_wg;      // output rows each of them fills
    int separate_merge;   // 1: too many splits for the last work-group of a head; a merge kernel follows
    int given_indices;    // 1: I_sparse comes from the caller (no measure, no selection)
    int given_inline;     // 1: the attend work-groups check the caller's sets and form the mean of V themselves (no prep kernel)
    int rows_mode;        // 1: many selected queries: a wave owns its queries and walks all keys (no key split);
                          // 2: the same with the keys cut in two inside the work-group (float32)
    // workspace carving (byte offsets, each 256-aligned)
    size_t off_M, off_vpart, off_vseg, off_mu, off_sel, off_u, off_ticket, off_cand, off_part, total;
    size_t part_stride;   // elements per (head, qgroup, split) partial record: nq_group * (2 + 64) floats, or nq_group * (2 + 32) doubles
    size_t part_elem;     // bytes per element of a record: 8 for float32 tensors, 4 for bfloat16
};

// Pointers into the carved workspace.
struct Scratch {
    float*  M;       // [BH, L]            sampled measure
    double* vpart;   // [BH, n_chunk, 64]  column sums of the valid V rows of each measure chunk
    double* vseg;    // [BH, n_seg or n_lists, 64]  the same summed over the chunks of each segment / of each streaming work-group
    float*  mu;      // [BH, 64]           mean of the valid V rows (long heads only)
    int*    sel;     // [BH, u_max]        I_sparse, ascending, -1 padded
    int*    u;       // [B]                u_b
    int*    ticket;  // [BH]               attend work-groups of the head that have finished
    uint2*  cand;    // [BH, n_lists, cand_len]  (order key, query) of each list's best queries, sorted
    void*   part;    // [BH, n_qgroup, n_split, part_stride] double (f32 tensors) or float (bf16)
};

struct Args {
    const void* Q; const void* K; const void* V;
    const int* lengths; const int* idx;
    void* out;
    URule urule;
    int fill;                  // psa_fill_t
    const int* given_sel;      // [BH, u_max] caller's index sets (given_indices plans), else unused
    const int* given_u;        // [B]
    hipStream_t stream;
};

// u_stride > 0: plan for caller-given index sets of that row stride (urule is ignored).
// Kernels that use more than the default 64 KB of dynamic LDS need the limit raised
// once per device.  `done` is the kernel's own bit mask of devices already served
// (devices beyond 63 are simply served on every call); two threads racing on the
// first call both set the attribute, which is harmless.
inline hipError_t ensure_lds_limit(const void* fn, int bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_relaxed) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_relaxed);
    return e;
}

bool make_plan(const psa_shape_t* s, URule urule, int u_stride, Plan* p);
inline bool make_plan(const psa_shape_t* s, double c, Plan* p) { return make_plan(s, URule{PSA_U_LOG, c}, 0, p); }
Scratch carve(const Plan& p, void* workspace);

// One-time, per-device set-up of the kernels that need it (dynamic LDS limits); the launch
// functions do the same on their first use.
hipError_t init_measure();
hipError_t init_attend();

hipError_t launch_measure(const Plan& p, const Args& a, const Scratch& w);
hipError_t launch_select(const Plan& p, const Args& a, const Scratch& w);
hipError_t launch_select_segments(const Plan& p, const Args& a, const Scratch& w);     // long heads: lists for the attend stage
hipError_t launch_attend(const Plan& p, const Args& a, const Scratch& w);
hipError_t launch_vsum(const Plan& p, const Args& a, const Scratch& w);             // V column sums alone
hipError_t launch_prep_indices(const Plan& p, const Args& a, const Scratch& w);     // mean of V, caller's index sets

// Gradients of stages a3 and a4 for a fixed index set (psa_backward.hip): query tiles of 16 kept
// queries, S key splits of `blocks_per_split` blocks of 64 keys, and the carving of the workspace.
struct BwdPlan {
    int QT, S, blocks_per_split;
    size_t off_stats_part, off_stats, off_gsum, off_dq_part, total;
};
BwdPlan make_bwd_plan(const psa_shape_t& s, int u_stride);
hipError_t launch_backward(const psa_shape_t& s, const BwdPlan& bp, const void* Q, const void* K, const void* V,
                           const int* lengths, const int* sel, const int* u, int u_stride, int fill, const void* G,
                           void* dQ, void* dK, void* dV, void* workspace, hipStream_t stream);

hipError_t launch_qkv_project(const psa_shape_t& s, const void* X, const psa_mhsa_weights_t& w,
                              void* Q, void* K, void* V, hipStream_t stream);
hipError_t launch_out_project(const psa_shape_t& s, const void* A, const psa_mhsa_weights_t& w, void* Y, hipStream_t stream);

}  // namespace psa

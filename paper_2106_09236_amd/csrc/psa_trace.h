// Optional in-kernel phase timestamps (compiled out unless PSA_TRACE is defined).
// With -DPSA_TRACE, wave PSA_TRACE_WAVE (default 0) of every work-group stores
// the shader clock at each PSA_TS(k) into g_psa_trace[wg % 4096][k]; a harness
// that includes the kernel sources in one translation unit reads the symbol
// back and averages the phase lengths (the shader clock is local to a compute unit).  PSA_TS_DRAIN() waits for the wave's
// outstanding memory operations, so that a phase's time includes its loads.
#pragma once

#ifdef PSA_TRACE
#ifndef PSA_TRACE_WAVE
#define PSA_TRACE_WAVE 0
#endif
__device__ unsigned long long g_psa_trace[4096 * 16];
#define PSA_TS(k)                                                                                          \
    do {                                                                                                   \
        if ((int)threadIdx.x == 64 * PSA_TRACE_WAVE) {                                                     \
            const unsigned wg_ = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);           \
            g_psa_trace[(wg_ % 4096u) * 16 + (k)] = clock64();                                             \
        }                                                                                                  \
    } while (0)
// the same with the device-wide constant-rate counter (100 MHz), comparable between work-groups
#define PSA_TS_WALL(k)                                                                                     \
    do {                                                                                                   \
        if ((int)threadIdx.x == 64 * PSA_TRACE_WAVE) {                                                     \
            const unsigned wg_ = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);           \
            g_psa_trace[(wg_ % 4096u) * 16 + (k)] = wall_clock64();                                        \
        }                                                                                                  \
    } while (0)
#define PSA_TS_DRAIN() asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory")
#else
#define PSA_TS_WALL(k) do {} while (0)
#define PSA_TS(k) do {} while (0)
#define PSA_TS_DRAIN() do {} while (0)
#endif

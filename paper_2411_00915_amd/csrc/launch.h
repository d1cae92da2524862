// Kernel launch helper with optional per-kernel timing.
//
// When timing is switched on (lora_timing_begin), every kernel is launched with
// a start/stop event pair attached to the kernel itself (hipExtLaunchKernelGGL),
// so the elapsed time of a pair is that kernel's own duration on the stream it
// was launched on, without launch gaps.  Off by default: plain launches.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

enum lora_kernel_id {
    LORA_K_SHRINK_GENERAL = 0,
    LORA_K_EXPAND_GENERAL,
    LORA_K_SHRINK_TILED,
    LORA_K_EXPAND_TILED,
    LORA_K_GEMM_GENERAL,
    LORA_K_GEMM_TILED,
    LORA_K_GEMM_TILED_DELTA,
    LORA_K_DELTA_FUSED,
    LORA_K_V_SPLIT,
    LORA_K_SHRINK_STREAM,
    LORA_K_EXPAND_STREAM,
    LORA_K_MERGE,
    LORA_K_GEMM_RING,
    LORA_K_GEMM_RING_DELTA,
    LORA_K_CLEAR,
    LORA_K_PROBE_EMPTY,
    LORA_K_PROBE_READ,
    LORA_K_PROBE_MFMA,
    LORA_K_COUNT
};

// buffer given to lora_trace_set (nullptr: none)
long long* lora_trace_buffer(size_t* bytes);

bool lora_timing_on();
// hands out an event pair and remembers it under kernel_id; false if none could be made
bool lora_timing_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop);

#define LORA_LAUNCH(id, kernel, grid, block, lds, stream, ...)                                   \
    do {                                                                                         \
        hipEvent_t ev_s_ = nullptr, ev_e_ = nullptr;                                             \
        if (lora_timing_on() && lora_timing_events((id), &ev_s_, &ev_e_))                        \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ev_s_, ev_e_, 0, __VA_ARGS__); \
        else                                                                                     \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                   \
    } while (0)

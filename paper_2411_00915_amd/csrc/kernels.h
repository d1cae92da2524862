// Internal launch interface between the C-ABI layer (abi.hip) and the kernel
// translation units.  Every function enqueues on `stream` and returns the HIP
// status of the launch.
#pragma once
#include <hip/hip_runtime.h>

#include "plan_internal.h"

// v is [P][T][R] fp32: P partial sums (K split over workgroups), added in order by every consumer
struct lora_vspec {
    int R;
    int P;
    long long part;   // floats between consecutive parts (T * R)
};
static inline lora_vspec lora_vspec_of(const lora_plan* p)
{
    return lora_vspec{p->R, p->v_parts, (long long)p->T * p->R};
}

struct lora_dev_tables {
    const int32_t* perm;
    const int32_t* token_adapter;
    const int32_t* row_key;        // fused GEMM: adapter of the token (bits 0..22 all ones: none) | removal bit
    const int32_t* rank;
    const float* scale;
    const lora_tile* shrink_tiles;
    const lora_tile* expand_tiles;
    void* sync;                    // hand-off counters of the single-launch decode kernel: 128 bytes per adapter group
    const int32_t* order;          // fused GEMM: row order and per-tile (adapter, rank block) lists
    const int32_t* extra_ptr128;
    const int32_t* extra128;
    const int32_t* extra_ptr256;
    const int32_t* extra256;
    const void* zeros;             // 256 zero bytes
    const int32_t* shrink_rows;    // single-launch decode kernel: 16 tokens per shrink / expand tile, padded
    const int32_t* expand_rows;
};

// general VALU family (any dtype, any alignment)
hipError_t launch_shrink_general(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                 const void* const* At, float* v, hipStream_t stream);
hipError_t launch_expand_general(const lora_plan* p, const lora_dev_tables& d, const float* v,
                                 const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream);

// tiled MFMA family (bf16; K, ranks, ldx, ldy multiples of 8; 16-byte aligned bases)
// vb != nullptr: room for the split of v into two bf16 terms, [T][2][R]; *split_done tells whether the launch wrote it
hipError_t launch_shrink_tiled(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                               const void* const* At, float* v, hipStream_t stream, void* vb = nullptr,
                               bool* split_done = nullptr);
hipError_t launch_expand_tiled(const lora_plan* p, const lora_dev_tables& d, const float* v,
                               const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream);

// streaming kernels for prefill-sized batches (plans with shrink_stream / expand_stream; called by the two above)
hipError_t launch_shrink_stream(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                const void* const* At, float* v, hipStream_t stream, void* vb = nullptr,
                                bool* split_done = nullptr);
hipError_t launch_expand_stream(const lora_plan* p, const lora_dev_tables& d, const float* v,
                                const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream);

// both steps in one launch (decode regime: every tile small); same layout demands as the tiled family.
// trace != nullptr: the instrumented build, which leaves 8 time stamps per workgroup there (lora_trace_set);
// hipErrorInvalidValue if trace_bytes does not hold them
hipError_t launch_delta_fused_small(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                    const void* const* At, const void* const* Bt, float* v, void* y, int64_t ldy,
                                    float beta, hipStream_t stream, long long* trace = nullptr, size_t trace_bytes = 0);

// mixture mode: the second batch (every token that is not the merged adapter's, with that adapter and the negated
// scale) whose delta the fused GEMM folds in besides the tokens' own; plan == nullptr: none
struct gemm_removal {
    const lora_plan* plan = nullptr;
    const lora_dev_tables* tables = nullptr;
    const float* v = nullptr;      // its shrink's output
    void* vb = nullptr;            // room for the bf16 split of it, T * 2 * plan->R elements
    bool split_done = false;       // the shrink has written the split already
};

// base GEMM  y = x Wt^T  (+ optional adapter delta in the epilogue when p != nullptr)
hipError_t launch_gemm_general(int32_t T, int32_t K, int32_t N, int32_t dtype, const void* x, int64_t ldx,
                               const void* Wt, int64_t ldw, void* y, int64_t ldy,
                               const lora_plan* p, const lora_dev_tables* d, const float* v, const gemm_removal& rm,
                               const void* const* Bt, hipStream_t stream);
bool gemm_tiled_supported(int32_t T, int32_t K, int32_t N, int32_t dtype, const void* x, int64_t ldx,
                          const void* Wt, int64_t ldw, const void* y, int64_t ldy);
hipError_t launch_gemm_tiled(int32_t T, int32_t K, int32_t N, const void* x, int64_t ldx,
                             const void* Wt, int64_t ldw, void* y, int64_t ldy,
                             const lora_plan* p, const lora_dev_tables* d, const float* v, void* vb, bool split_done,
                             const gemm_removal& rm, const void* const* Bt, hipStream_t stream);

// mode switch: Wt_l += s Bt_l At_l for L layers in one launch (device arrays of L pointers each)
hipError_t launch_merge_tiled(int32_t L, int32_t N, int32_t K, int32_t r, float s, void* const* Wt, int64_t ldw,
                              const void* const* At, const void* const* Bt, hipStream_t stream);
hipError_t launch_merge_general(int32_t L, int32_t N, int32_t K, int32_t r, float s, int32_t dtype, void* const* Wt,
                                int64_t ldw, const void* const* At, const void* const* Bt, hipStream_t stream);

// Internal layout of a batch plan.  Host tables are filled by planner.cpp (no
// HIP there); the device mirror is managed by abi.hip.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/lora_abi.h"

// Tile shape code of a lora_tile:  bits 0..3 = token blocks of 16 per wave
// tile (TB), bits 4..7 = rank blocks of 16 per wave tile (JB, shrink only).
static inline int32_t lora_shape_code(int tb, int jb) { return (tb & 15) | ((jb & 15) << 4); }
static inline int lora_shape_tb(int32_t code) { return code & 15; }
static inline int lora_shape_jb(int32_t code) { return (code >> 4) & 15; }
// shrink tiles only: bits 8..11 = index of the tile's K part, bits 12..15 = number of K parts
static inline int lora_shape_part(int32_t code) { return (code >> 8) & 15; }
static inline int lora_shape_parts(int32_t code) { return (code >> 12) & 15; }

// Planner tunables (defaults come from measurements on MI355X).  A plan is made with a snapshot: the process
// defaults, overridden by the shape table's entry for the batch, overridden by the descriptor's own values.
struct lora_tuning {
    int32_t shrink_waves;          // wavefronts per shrink workgroup (big build, <= 8)
    int32_t shrink_tb2_min_rows;   // groups with at least this many tokens use 32-row wave tiles
    int32_t shrink_max_jb;         // rank blocks of 16 per shrink tile (1, 2 or 4)
    int32_t expand_wave_bytes;     // target bytes of Bt + y one expand wavefront streams
    int32_t expand_tb2_min_rows;   // token-count thresholds for 32 / 64 row expand tiles
    int32_t expand_tb4_min_rows;
    int32_t tiled_min_tokens;      // AUTO: batches with fewer active tokens use the general kernels
    int32_t shrink_small_waves;    // wavefronts per shrink workgroup, small build (<= 16)
    int32_t shrink_small_jb;       // rank blocks per shrink tile for groups below shrink_tb2_min_rows (1 or 2)
    int32_t shrink_target_wgs;     // small build: split K over up to 4 workgroups until the launch has this many
    int32_t fused_wait_us;         // single-launch decode kernel: microseconds an expand block waits before it computes v itself (+1; 1 = never wait)
    int32_t fused_delay;           // single-launch decode kernel: head start of the shrink blocks' loads, units of ~0.4 us (+1)
    int32_t expand_wave_bytes_big; // like expand_wave_bytes, for adapter groups of at least expand_tb2_min_rows tokens
    int32_t shrink_tb4_min_rows;   // groups with at least this many tokens use 64-token shrink tiles
    int32_t shrink_stream_min_tokens;  // batches with at least this many adapter tokens use the streaming shrink
    int32_t shrink_stream_wgs;     // streaming shrink: 64-token tiles when 128-token tiles give fewer workgroups than this
    int32_t expand_stream_stages;  // streaming expand: stages (of 64 features per wavefront) one workgroup walks
};
static_assert(sizeof(lora_tuning) == LORA_TUNING_COUNT * sizeof(int32_t), "lora_tuning and LORA_TUNING_COUNT disagree");

struct lora_plan {
    int32_t T = 0, S = 0, n_a = 0, K = 0, N = 0, dtype = 0, variant_req = 0;
    lora_tuning tuning{};          // the tunables this plan is made with
    int32_t tuning_source = 0;     // 0 defaults, 1 shape table entry, +2 values given by the descriptor
    int32_t R = 8;                 // v row stride (floats)
    int32_t v_parts = 1;           // v holds this many partial sums [P][T][R]; consumers add them in order
    int32_t family = LORA_VARIANT_GENERAL;
    int32_t shrink_waves = 4;      // wavefronts per shrink workgroup (split the K range), 1..16
    bool shrink_small = false;     // every shrink tile is 16 tokens x <= 32 rank rows: small kernel build
    bool shrink_stream = false;    // shrink tiles are those of the streaming kernel (prefill-sized batches)
    bool expand_stream = false;    // likewise for the expand tiles
    int32_t expand_stream_ks = 1;  // streaming expand: largest number of 32-rank steps (1, 2, 4) among the tiles
    int32_t expand_stream_lds = 0; // streaming expand: dynamic LDS bytes of the launch
    bool expand_small = false;     // every expand tile is 16 tokens of rank <= 64: small kernel build
    bool fused_ok = false;         // both small: shrink and expand can run as one launch
    int32_t fused_wait_us = 0;     // microseconds an expand block waits for its group's shrink tiles before it computes v itself
    int32_t fused_delay = 0;       // units of ~0.4 us an expand block waits before sending its first loads
    int32_t shrink_max_blocks = 1; // largest TB*JB among the shrink tiles (sizes the LDS reduction buffer)
    std::vector<int32_t> token_adapter, perm, group_adapter, group_offset, rank;
    std::vector<float> scale;
    std::vector<lora_tile> shrink_tiles, expand_tiles;
    // fused GEMM: row order (tokens sorted by adapter, then tokens without adapter) and, per token tile of 128
    // or 256 rows of that order, the adapter stages present: packed adapter | (64-column block of the
    // adapter's [v_hi | v_lo] concatenation) << 24.  (The 256 x 256 ring kernel uses the row order only: its
    // wavefronts find the adapters of their own 64 rows themselves.)
    std::vector<int32_t> order, extra_ptr128, extra128, extra_ptr256, extra256;
    std::vector<int32_t> shrink_rows, expand_rows;   // single-launch decode kernel: 16 tokens per tile, padded
    bool tiled_layout_ok = false;  // K and all active ranks multiples of 8
    bool shrink_tiled_only = false; // family GENERAL, but the shrink has tiles and runs on the MFMA kernels (ranks that
                                    // only the expand cannot take: not multiples of 8, or above 128)
    // fused GEMM: what a row is matched against an adapter stage by: its adapter in bits 0..22 (all ones: none),
    // bit 23 set when the removal of the merged adapter applies to it
    std::vector<int32_t> row_key;

    // Mixture mode: adapter `merged` is folded into the base weight.  This plan then holds the tokens' own branches
    // (the merged adapter's tokens count as tokens without adapter) and `unmerge` is a plan over the same tokens in
    // which every token that is not the merged adapter's uses that adapter with the negated scale.
    int32_t merged = -1;
    lora_plan* unmerge = nullptr;  // owned

    // device mirror (one allocation), valid when d_buf != nullptr
    int device = -1;
    void* d_buf = nullptr;
    size_t d_bytes = 0;
    void* h_stage = nullptr;       // pinned staging for the stream-ordered copy
    int32_t* d_perm = nullptr;
    int32_t* d_token_adapter = nullptr;
    int32_t* d_row_key = nullptr;
    int32_t* d_rank = nullptr;
    float* d_scale = nullptr;
    lora_tile* d_shrink_tiles = nullptr;
    lora_tile* d_expand_tiles = nullptr;
    int32_t* d_order = nullptr;
    int32_t* d_extra_ptr128 = nullptr;
    int32_t* d_extra128 = nullptr;
    int32_t* d_extra_ptr256 = nullptr;
    int32_t* d_extra256 = nullptr;
    int32_t* d_shrink_rows = nullptr;
    int32_t* d_expand_rows = nullptr;
    void* d_zeros = nullptr;          // 256 zero bytes (source of masked chunks in the fused GEMM)
    void* d_sync = nullptr;           // hand-off counters, 128 bytes per adapter group (only when fused_ok)
};

// How a plan's device tables are released: set by the translation unit that owns them (abi.hip) when the library
// is loaded; stays null in host-only builds of the planner, where no plan ever has device tables.
extern void (*lora_plan_device_release)(lora_plan*);

// stage ids and row keys of the fused GEMM: bit 23 marks the stages / the rows of the merged adapter's removal
constexpr int32_t LORA_UNMERGE_BIT = 1 << 23;

// bytes of v a plan's own tiles use, and where the removal's share starts (mixture mode)
static inline size_t lora_own_v_bytes(const lora_plan* p)
{
    return (size_t)p->v_parts * (size_t)p->T * (size_t)p->R * sizeof(float);
}
static inline size_t lora_unmerge_v_offset(const lora_plan* p) { return (lora_own_v_bytes(p) + 255) / 256 * 256; }


/*
 * C ABI of the MI355X heterogeneous-LoRA batching operator.
 *
 * The operator is the one VaLoRA's ATMM accelerates (paper section 4.3.1):
 * one batch of tokens, each request (segment) bound to its own LoRA adapter,
 * adapters of different ranks, segments of different lengths, no padding.
 * With the LoRA definition of section 2 (an adapter's update is the product
 * of its two low-rank factors; in unmerged inference its result is added onto
 * the base layer's output) every token t of a segment that uses adapter a gets
 *
 *         y[t,:] = x[t,:] W  +  s_a * (x[t,:] A_a) B_a
 *
 * x [T,K], W [K,N], A_a [K,r_a], B_a [r_a,N] as mathematical objects.
 *
 * MEMORY LAYOUT.  Every weight is stored the way section 2 dimensions the
 * factors (A as r x d, B as d x r) and the way torch.nn.Linear stores
 * `weight`: [out_features, in_features] row-major, contraction index fastest.
 *
 *     A_a  is stored as  At_a [r_a, K]   At_a[j*K   + k] = A_a[k,j]
 *     B_a  is stored as  Bt_a [N, r_a]   Bt_a[n*r_a + j] = B_a[j,n]
 *     W    is stored as  Wt   [N, K]     Wt  [n*ldw + k] = W[k,n]
 *     x [T,K] row-major (ldx), y [T,N] row-major (ldy),
 *     v [P][T,R] row-major fp32, R = lora_plan_query's v_row_stride, P = the
 *       plan's v_parts (1, 2 or 4): the shrink may split K over P workgroups,
 *       each writing its partial sum to its own part; the value is
 *       v[t,j] = sum_p v[(p*T + t)*R + j] for j < r_a, and every consumer in
 *       the library adds the parts in that order.  The rest of a row is never
 *       read or written.  lora_plan_query's v_bytes covers all P parts.
 *
 * OWNERSHIP.  The caller owns every device buffer (x, W, At_a, Bt_a, the two
 * device arrays of adapter pointers, v, y, workspace) and the HIP stream.  The
 * library owns only the plan: host tables, and a few small device tables that
 * are allocated by lora_plan_upload (or by the first compute call that uses
 * the plan) and released by lora_plan_destroy.  Compute calls enqueue kernels
 * on the caller's stream and return; they never synchronise.  The caller must
 * not destroy a plan while work that uses it is still in flight (the plan's
 * device tables are recycled for later plans, not synchronised on).
 *
 * THREADS.  Distinct plans may be created, used and destroyed from distinct
 * host threads at the same time (the pool of recycled device tables and the
 * timing records are locked).  One plan is used by one thread, on one stream,
 * at a time.  The default tunables and the shape table are process-wide and locked; every plan
 * keeps the snapshot it was made with.  The timing switch is process-wide: use it while no other
 * thread launches.
 *
 * ERRORS.  Every function returns a lora_status; nothing throws.  All
 * descriptor validation happens in lora_plan_create, which is pure host code
 * and needs no GPU.  Compute calls check pointers, leading dimensions and
 * alignment before launching and map HIP failures to LORA_ERR_DEVICE.
 *
 * MIXTURE MODE (section 4.4.1: one adapter m stays merged in the base weight
 * while requests of other adapters run in the same batch; their branch takes
 * m's update off again, the paper's deLoRA).  A plan made with
 * merged_adapter_plus1 = m + 1 computes, on the merged weight W',
 *
 *     tokens of adapter m:          y = x W'                      (no branch)
 *     tokens of adapter a != m:     y = x W' + s_a (x A_a) B_a - s_m (x A_m) B_m
 *     tokens without adapter:       y = x W'                    - s_m (x A_m) B_m
 *
 * which equals unmerged inference on W up to the rounding of W'.  The caller
 * passes the same pointer tables as always (entry m is read for the removal);
 * no concatenated matrices exist anywhere.  Inside, the removal is a second
 * batch over the same tokens ("every token that is not m's uses adapter m with
 * scale -s_m") with tiles of its own: lora_shrink writes its partial sums
 * behind the batch's own in v (lora_plan_view: unmerge_v_offset, row stride and
 * parts), lora_expand and lora_delta add first the removal (with the caller's
 * beta), then the tokens' own branches (accumulating): two passes over y, each
 * rounding it once, so a token with an adapter of its own gets
 * rnd(rnd(beta y + removal) + own) -- within u (|beta y + removal| + |y|) of
 * the exact value, u the unit roundoff of the dtype.  lora_fused_forward's
 * GEMM takes the removal in as one more adapter for the rows it applies to,
 * inside the same fp32 accumulators: one rounding, as without mixture mode.  "Rows of tokens without adapter are
 * left untouched" then holds for the tokens of adapter m only.
 * merged_adapter_plus1 naming an adapter of rank 0: same as 0.
 *
 * ALIGNMENT for the tuned bf16 kernels: base pointers 16 bytes; K, ldx, ldy,
 * ldw multiples of 8; ranks multiples of 8, at most 128.  Anything else (and
 * fp32) runs through general kernels with no alignment demands, which are one
 * to two orders of magnitude slower per token; padding an adapter's factors
 * with zero rank rows / columns to a multiple of 8 changes no result and moves
 * it onto the tuned kernels.  The rank demands are the expand's (rows of Bt_a
 * have r elements): lora_shrink alone runs on the tuned kernels for any rank
 * up to LORA_MAX_RANK when the rest holds (the plan view's
 * shrink_kernel_family says so) -- the case of task heads of arbitrary width
 * (section 4.2.2), which are a shrink with rank = number of outputs.
 */
#ifndef LORA_ABI_H
#define LORA_ABI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LORA_MAX_RANK 256
#define LORA_TUNING_COUNT 17     /* number of planner tunables, see lora_tuning_set */

typedef enum {
    LORA_OK = 0,
    LORA_ERR_INVALID_ARG = 1,   /* null pointer, bad segment table, id or rank out of range ... */
    LORA_ERR_UNSUPPORTED = 2,   /* valid request this build cannot run (dtype, size limits) */
    LORA_ERR_NOMEM = 3,         /* host or device allocation failed */
    LORA_ERR_WORKSPACE = 4,     /* caller's workspace is too small or misaligned */
    LORA_ERR_DEVICE = 5         /* a HIP call or kernel launch failed */
} lora_status;

typedef enum { LORA_F32 = 0, LORA_BF16 = 1 } lora_dtype;

/* Kernel family selection; tests use the non-default values to drive every
 * family over the same inputs. */
typedef enum {
    LORA_VARIANT_AUTO = 0,      /* planner decides per batch */
    LORA_VARIANT_GENERAL = 1,   /* general VALU kernels only */
    LORA_VARIANT_TILED = 2      /* tiled MFMA kernels wherever the layout allows */
} lora_variant;

typedef struct lora_plan lora_plan;   /* opaque, library-owned */

/*
 * Batch descriptor = the operator's problem statement (section 4.3.1: requests
 * of heterogeneous length, adapters of heterogeneous rank; section 5: the
 * request-to-adapter mapping of the batch).  All pointers are HOST pointers and
 * are only read during lora_plan_create.
 */
typedef struct {
    int32_t        num_tokens;     /* T >= 0 */
    int32_t        num_segments;   /* S >= 0 */
    const int32_t* seg_indptr;     /* [S+1], [0]=0, non-decreasing, [S]=T; empty segments allowed */
    const int32_t* seg_adapter;    /* [S], in [-1, num_adapters); -1 = no adapter (y = xW) */
    int32_t        num_adapters;   /* n_a >= 0 */
    const int32_t* adapter_rank;   /* [n_a], 0..LORA_MAX_RANK; rank 0 = no adapter */
    const float*   adapter_scale;  /* [n_a], finite */
    int32_t        k;              /* in features  K >= 1 */
    int32_t        n;              /* out features N >= 1 */
    int32_t        dtype;          /* lora_dtype of x, At, Bt, Wt, y (v is always fp32) */
    int32_t        variant;        /* lora_variant */
    const int32_t* tuning;         /* optional: planner tunables for THIS plan, [tuning_count] in the order of
                                      lora_tuning_set (entries <= 0 and entries beyond tuning_count: not given).
                                      What is given here overrides the shape table's entry, which overrides the
                                      process defaults.  NULL / 0: nothing given */
    int32_t        tuning_count;
    int32_t        merged_adapter_plus1;  /* mixture mode (section 4.4.1): 1 + the index of the adapter whose update
                                      the caller has folded into the base weight this batch runs on
                                      (W' = W + s_m A_m B_m, e.g. by lora_merge); 0 = none.  See MIXTURE MODE below */
} lora_batch_desc;

/* One unit of kernel work: the rows [row0,row0+nrows) of `perm` (all of one
 * adapter) times the columns [c0,c0+cn) -- rank indices for shrink, output
 * features for expand. */
typedef struct {
    int32_t adapter;
    int32_t row0;
    int32_t nrows;
    int32_t c0;
    int32_t cn;
    int32_t shape;      /* tile shape code chosen by the planner; shrink: bits 8..11 K part, 12..15 number of K
                           parts, 16..31 adapter group; expand: bits 8..19 / 20..31 shrink / expand tiles of the adapter
                           group when the plan can run as one launch, else 0 */
    int32_t reserved0;  /* rank of the adapter */
    int32_t reserved1;  /* shrink tiles: bit pattern of the adapter's scale; expand tiles: adapter group */
} lora_tile;

/* Read-only view of a plan's host tables (valid until lora_plan_destroy). */
typedef struct {
    int32_t        num_tokens;
    int32_t        num_active;      /* tokens that have an adapter of rank > 0 */
    int32_t        num_groups;      /* distinct adapters in use */
    int32_t        v_row_stride;    /* R */
    int32_t        kernel_family;   /* lora_variant actually chosen (GENERAL or TILED) */
    int32_t        shrink_waves;    /* wavefronts per workgroup of the shrink launch */
    int32_t        v_parts;         /* P: number of partial sums v holds (see lora_shrink) */
    int32_t        tuning_source;   /* where this plan's tunables came from: 0 process defaults only, 1 an entry of
                                       the shape table, + 2 if the descriptor gave values of its own */
    int32_t        tuning[LORA_TUNING_COUNT];   /* the tunables this plan was made with (order of lora_tuning_set) */
    int32_t        shrink_kernel_family;   /* the family lora_shrink runs: TILED also when kernel_family is GENERAL only
                                              because of ranks the expand kernels cannot take (see ALIGNMENT) */
    const int32_t* token_adapter;   /* [T]  adapter of each token, -1 = none */
    const int32_t* perm;            /* [num_active] tokens with an adapter, stably sorted by adapter */
    const int32_t* group_adapter;   /* [num_groups] ascending adapter ids */
    const int32_t* group_offset;    /* [num_groups+1] exclusive prefix sums into perm */
    const lora_tile* shrink_tiles;  int32_t num_shrink_tiles;
    const lora_tile* expand_tiles;  int32_t num_expand_tiles;
    /* Tables of lora_fused_forward's GEMM (empty when the plan cannot use the MFMA kernels): the row order it walks
     * (tokens sorted by adapter, then tokens without adapter; whole blocks of 256 rows ordered by decreasing number
     * of adapter stages), and per tile of 256 rows of that order its adapter stages: one entry
     * adapter | block << 24 per adapter present and per block of 64 columns of the adapter's [v_hi | v_lo]
     * (2 r columns).  The register-staged GEMM kernels walk these lists; the 256 x 256 ring kernel uses the row
     * order alone (each wavefront finds the adapters of its own 64 rows). */
    int32_t        num_gemm_rows;        /* T, or 0 */
    int32_t        num_gemm_tiles;       /* ceil(T / 256), or 0 */
    const int32_t* gemm_order;           /* [num_gemm_rows] */
    const int32_t* gemm_stage_offset;    /* [num_gemm_tiles + 1] exclusive prefix sums into gemm_stage */
    const int32_t* gemm_stage;           /* [gemm_stage_offset[num_gemm_tiles]] */
    /* Mixture mode (merged_adapter_plus1 > 0 and that adapter has rank > 0); otherwise -1 / 0 / NULL.  The stage
     * list of a tile that holds a token the removal applies to ends with the entries
     * merged_adapter | 1 << 23 | block << 24, one per block of the merged adapter's 2 r columns; gemm_order then
     * lists tokens with an adapter of their own, tokens without one, and last the merged adapter's tokens. */
    int32_t        merged_adapter;       /* m, or -1 */
    int32_t        num_unmerge;          /* tokens the removal applies to: all that are not m's */
    int32_t        unmerge_v_row_stride; /* row stride (floats) and parts of the removal's share of v */
    int32_t        unmerge_v_parts;
    size_t         unmerge_v_offset;     /* bytes from the start of v to that share (256-byte aligned) */
    const int32_t* unmerge_perm;         /* [num_unmerge] those tokens, ascending */
    const lora_tile* unmerge_shrink_tiles;  int32_t num_unmerge_shrink_tiles;   /* tile lists of the removal */
    const lora_tile* unmerge_expand_tiles;  int32_t num_unmerge_expand_tiles;
} lora_plan_view;

/*
 * lora_plan -- the per-batch step that stands where ATMM looks up the tile
 * configuration for the input shapes at hand (section 4.3.1, "adaptive tiling
 * against input shapes"; the shape-keyed table of section 4.3.2).  From the
 * segment table and the rank table it derives: the adapter of every token, the
 * stable grouping of tokens by adapter, and the tile lists of the shrink and
 * expand launches (tile shape chosen per adapter group from the group's token
 * count and rank).  Pure host code, deterministic: equal descriptors give
 * byte-identical tables.  One plan serves every layer / projection that shares
 * the segment table, K, N, ranks and scales.
 *
 * Returns LORA_ERR_INVALID_ARG for: null desc/out; negative sizes; merged_adapter_plus1 outside [0, n_a]; null tables
 * with non-zero counts; seg_indptr not starting at 0, decreasing, or not ending
 * at T; adapter id outside [-1, n_a); rank outside [0, LORA_MAX_RANK];
 * non-finite scale; K or N < 1; unknown dtype or variant.
 */
lora_status lora_plan_create(const lora_batch_desc* desc, lora_plan** out);
void        lora_plan_destroy(lora_plan* plan);   /* NULL is allowed */

/* v_row_stride R (floats), bytes of the v buffer (P*T*R*4; in mixture mode that, rounded up to 256, plus the
 * removal's share), and the bytes of workspace lora_fused_forward needs (v plus its bf16 split).  Any out pointer
 * may be NULL. */
lora_status lora_plan_query(const lora_plan* plan, int32_t* v_row_stride,
                            size_t* v_bytes, size_t* fused_workspace_bytes);

lora_status lora_plan_export(const lora_plan* plan, lora_plan_view* out);

/* Copy the plan's tables to the current device (allocates the library-owned
 * device tables; stream-ordered copy on hip_stream).  Optional: compute calls
 * do it on first use. */
lora_status lora_plan_upload(lora_plan* plan, void* hip_stream);

/*
 * lora_shrink -- first of the two extra products per adapted layer (section
 * 3.2; the skinny K -> r GEMM of every adapter branch, batched by ATMM,
 * section 4.3.1), with the adapter's scale folded in:
 *
 *     v[t, j] = s_a * sum_k x[t,k] * A_a[k,j]        j < r_a,  a = adapter(t)
 *
 * x: device, [T,K] row-major, leading dimension ldx (elements).
 * d_At_ptrs: device array [n_a] of device pointers to At_a [r_a,K]; entries of
 *   adapters no token uses are never dereferenced.
 * v: device, fp32 [P][T,R] (layout above); rows of tokens without adapter are
 *   left untouched.
 * fp32 accumulation; the products of two bf16 values are exact in fp32.
 */
lora_status lora_shrink(lora_plan* plan, const void* x, int64_t ldx,
                        const void* const* d_At_ptrs, float* v, void* hip_stream);

/*
 * lora_expand -- the second extra product and the extra addition per adapted
 * layer (section 3.2; the r -> N GEMM of every adapter branch, section 4.3.1):
 *
 *     y[t, n] = beta * y[t, n] + sum_j v[t,j] * B_a[j,n]
 *
 * v as written by lora_shrink (already scaled).  d_Bt_ptrs: device array [n_a]
 * of device pointers to Bt_a [N,r_a].  y: device, [T,N], ldy; beta is 1
 * (accumulate onto the base output) or 0 (overwrite); rows of tokens without
 * adapter are left untouched bit for bit (also for beta = 0).
 * fp32 accumulation, one round-to-nearest-even at the store.
 */
lora_status lora_expand(lora_plan* plan, const float* v,
                        const void* const* d_Bt_ptrs, void* y, int64_t ldy,
                        float beta, void* hip_stream);

/*
 * lora_delta -- both extra products of an adapted layer in one call (section
 * 3.2 counts two extra matrix products, one extra addition and their kernel
 * launches per layer as the cost of unmerged inference):
 *
 *     y[t,:] = beta * y[t,:] + s_a * (x[t,:] A_a) B_a
 *
 * Arguments as for lora_shrink and lora_expand; v is scratch of lora_plan_query's
 * v_bytes.  When every tile of the plan is small (decode-shaped batches:
 * adapter groups of fewer than 64 tokens, ranks <= 64) both steps run as ONE
 * kernel launch: expand blocks send out their Bt and y loads, wait (bounded)
 * for their adapter group's shrink blocks through counters in the plan's device
 * tables, and if those are not seen in time compute their rows of v themselves.
 * Otherwise it is lora_shrink followed by lora_expand.  A plan's launches must
 * not overlap (one stream at a time): the counters live in the plan.
 */
lora_status lora_delta(lora_plan* plan, const void* x, int64_t ldx,
                       const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                       float* v, void* y, int64_t ldy, float beta, void* hip_stream);

/*
 * lora_delta_static -- lora_delta for callers that cannot allocate device memory or call anything that does: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and same result
 * as lora_delta, without the v argument: v and the single launch's hand-off counters live in a device array that
 * is part of the library's image (LORA_STATIC_V_BYTES + LORA_STATIC_MAX_GROUPS * 128 bytes, held by every GPU the
 * library runs on until the process ends).  The call allocates nothing and frees nothing.
 *   - The plan must already be on the current device (lora_plan_upload, which does allocate, at set-up);
 *     otherwise LORA_ERR_INVALID_ARG.
 *   - lora_plan_query's v_bytes above LORA_STATIC_V_BYTES, more than LORA_STATIC_MAX_GROUPS distinct adapters
 *     in use, or a plan in mixture mode: LORA_ERR_UNSUPPORTED (use lora_delta with a caller-owned v).
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents (the counters are
 *     cleared by a small kernel at the start of every call that uses them): calls that overlap on one GPU
 *     -- two streams, two threads -- race.  Calls on one stream, and calls on different GPUs, do not.
 */
#define LORA_STATIC_V_BYTES   (16u << 20)
#define LORA_STATIC_MAX_GROUPS 4096
lora_status lora_delta_static(lora_plan* plan, const void* x, int64_t ldx,
                              const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                              void* y, int64_t ldy, float beta, void* hip_stream);

/*
 * lora_base_gemm -- the base-model product shared by all requests of the batch
 * (section 1 / section 2, unmerged inference):  y = x W, Wt [N,K] with ldw.
 * bf16 MFMA with fp32 accumulation (fp32 dtype: VALU).  Used for the
 * "separate" path base GEMM + shrink + expand.
 */
lora_status lora_base_gemm(int32_t num_tokens, int32_t k, int32_t n, int32_t dtype,
                           const void* x, int64_t ldx, const void* Wt, int64_t ldw,
                           void* y, int64_t ldy, void* hip_stream);

/*
 * lora_fused_forward -- whole layer in one call, y = x W + s_a (x A_a) B_a,
 * with the adapter delta added to the base GEMM's fp32 accumulators before the
 * single rounding of y (unmerged inference at close to the cost of merged
 * inference, sections 2 and 4.4).  Runs the shrink into `workspace` (which
 * holds v and its split into two bf16 terms; size from lora_plan_query,
 * 256-byte aligned), then one GEMM kernel that walks the tokens in
 * adapter-sorted order and adds each adapter's v B_a to the accumulators of
 * the rows that carry it (as extra k-stages of its pipeline, or wavefront by
 * wavefront after the K loop, depending on the kernel).  LORA_ERR_WORKSPACE if
 * the workspace is too small.
 */
lora_status lora_fused_forward(lora_plan* plan, const void* x, int64_t ldx,
                               const void* Wt, int64_t ldw,
                               const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                               void* y, int64_t ldy,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * lora_merge -- mode switch (section 4.4.2, "swift inference mode switch"): fold one adapter into
 * the base weights of all layers, or take it out again, in place and in one launch:
 *     Wt_l[n*ldw + k] += scale * sum_j Bt_l[n*rank + j] * At_l[j*k_dim + k]     l = 0..num_layers-1
 * i.e. W_l <- W_l + scale * A_l B_l; pass -scale to unmerge.  fp32 accumulation, one rounding
 * (RNE) at the store; a merge followed by the unmerge restores W_l only to within that rounding.
 * d_Wt_ptrs, d_At_ptrs, d_Bt_ptrs: device arrays of num_layers device pointers each (layouts as
 * above: Wt_l [n, k] with leading dimension ldw, At_l [rank, k], Bt_l [n, rank]); every layer has
 * the same n, k and rank.  The weights must not be in use by work in flight on another stream.
 * bf16 with k, ldw and rank multiples of 8, rank <= 128 and 16-byte aligned layer pointers runs
 * the streaming kernel (every weight read and written once, whole cache lines); with
 * variant = LORA_VARIANT_GENERAL, fp32 or any other shape a general kernel runs.
 * LORA_VARIANT_TILED on a shape the streaming kernel does not take: LORA_ERR_UNSUPPORTED.
 * num_layers = 0 or rank = 0: nothing to do, LORA_OK.
 */
lora_status lora_merge(int32_t num_layers, int32_t n, int32_t k, int32_t rank, float scale, int32_t dtype,
                       int32_t variant, void* const* d_Wt_ptrs, int64_t ldw,
                       const void* const* d_At_ptrs, const void* const* d_Bt_ptrs, void* hip_stream);

const char* lora_status_str(lora_status s);

/*
 * Planner tunables: what steers the planner's choice of tile shapes, kernel family and K split.  Every plan is
 * made with a snapshot of them: the process defaults (this call), overridden by the shape table's entry for the
 * batch (lora_tuning_table_set, below), overridden by the values the batch descriptor gives.  `values` is an int32
 * array of up to LORA_TUNING_COUNT entries in the order: shrink_waves (wavefronts per shrink workgroup, 1..8),
 * shrink_tb2_min_rows (adapter groups with at least this many tokens use
 * 32-token shrink tiles), shrink_max_jb (rank blocks of 16 per shrink tile,
 * 1..4), expand_wave_bytes (bytes of Bt and y one expand wavefront streams),
 * expand_tb2_min_rows, expand_tb4_min_rows (token-count thresholds for 32- and
 * 64-token expand tiles), tiled_min_tokens (AUTO uses the general kernels below
 * this many active tokens), shrink_small_waves (wavefronts per shrink workgroup
 * when every tile is small, 1..16), shrink_small_jb (rank blocks of 16 per shrink
 * tile for adapter groups below shrink_tb2_min_rows, 1..2), shrink_target_wgs
 * (small launches split K over up to 4 workgroups per tile until they have this
 * many workgroups), fused_wait_us (lora_delta's single launch: microseconds an expand
 * block waits for its shrink blocks before it computes its rows of v itself, plus one;
 * 1 = never wait, always recompute; default 2 ms),
 * fused_delay (lora_delta's single launch: head start given to the shrink blocks'
 * loads, units of about 0.4 us, plus one), expand_wave_bytes_big (expand_wave_bytes
 * for adapter groups of at least expand_tb2_min_rows tokens), shrink_tb4_min_rows
 * (adapter groups with at least this many tokens use 64-token shrink tiles),
 * shrink_stream_min_tokens (batches with at least this many adapter tokens, ranks
 * <= 128 and K >= 1024 use the streaming shrink: tiles of up to 128 tokens over all
 * rank rows, At shared through LDS; the expand then streams likewise; smaller
 * batches that cannot run as lora_delta's single launch and hold an adapter group
 * of at least 64 tokens, or 128 tokens in all, use them too; 2^30 or more
 * switches the streaming kernels off),
 * shrink_stream_wgs (the streaming kernels use 64-token tiles when 128-token tiles
 * would give fewer workgroups than this), expand_stream_stages (stages of 64
 * features per wavefront that one workgroup of the streaming expand walks).
 * Entries <= 0 keep the current value; plans made
 * earlier are unaffected.  Host only, thread-safe.
 */
void lora_tuning_set(const int32_t* values, int32_t count);
void lora_tuning_get(int32_t* values, int32_t count);

/*
 * The shape table: the counterpart of the table ATMM consults per input shape (section 4.3.1) and fills offline
 * by profiling every candidate configuration per shape (section 4.3.2, Algorithm 2: loops over token counts in
 * steps of 32, over the ranks, and over the tile configurations).  An entry holds the tunables that measured best
 * on MI355X for one shape class; lora_plan_create looks the batch's class up and plans with that entry (on top of
 * the process defaults, below the descriptor's own values).  The key of a batch:
 *   tokens       tokens that have an adapter; the entry with the smallest `tokens` >= that count applies (entries
 *                are made for multiples of 32), else the one with the largest
 *   k, n         in / out features (exact match)
 *   max_rank     largest rank in use, rounded up to 8, 16, 32, 64, 128 or 256 (exact match)
 *   group_class  0: every adapter group has fewer than 64 tokens (decode-shaped); 2: the adapter groups hold 512
 *                tokens or more on average (few long requests, e.g. image-sized prefill); 1: otherwise (exact match)
 * An entry without values (all <= 0) says that the class was searched and keeps the defaults; it is there so that a
 * batch of that class is not planned with the entry of the next larger token count.
 * The library ships with the table its offline search (paper_2411_00915_amd/autotune.py) wrote on MI355X;
 * lora_tuning_table_set replaces it for the process (entries are copied; NULL / 0 restores the shipped table),
 * lora_tuning_table_get copies up to `capacity` entries out and returns the table's size.  Plans made earlier keep
 * what they were made with.  Thread-safe.
 */
typedef struct {
    int32_t tokens, k, n, max_rank, group_class;
    int32_t values[LORA_TUNING_COUNT];      /* order of lora_tuning_set; <= 0: keep the default */
} lora_tuning_entry;
lora_status lora_tuning_table_set(const lora_tuning_entry* entries, int32_t count);
int32_t     lora_tuning_table_get(lora_tuning_entry* entries, int32_t capacity);

/*
 * Per-kernel timing for benchmarks (the paper times its operator over repeated
 * rounds, section 6.3.2).  Between lora_timing_begin and lora_timing_end every
 * kernel the library launches carries its own start/stop event pair, so the
 * recorded time is the kernel's duration on its stream without launch gaps.
 * lora_timing_end synchronises the device and folds the pairs into per-kernel
 * statistics that lora_timing_read returns (microseconds).  Kernel ids run from
 * 0 to lora_kernel_count()-1; lora_kernel_name gives the kernel's name as a
 * profiler shows it.  Not for use while another thread launches.
 */
lora_status lora_timing_begin(void);
lora_status lora_timing_end(void);
lora_status lora_timing_read(int32_t kernel_id, int64_t* count, double* total_us,
                             double* min_us, double* max_us);
const char* lora_kernel_name(int32_t kernel_id);
int32_t     lora_kernel_count(void);

/*
 * lora_trace_set -- phase time stamps of lora_delta's single launch, for diagnosis (the paper attributes the
 * operator's cost to kernel context operations and under-used cores, section 3.2; the stamps show where the time
 * of a launch goes on this machine).  While a buffer is set, lora_delta runs the instrumented build of its
 * single-launch kernel (plans whose view says so; every other path ignores the buffer): same arithmetic, same
 * results, a few stores and two extra waits per workgroup slower.  Thread 0 of workgroup b writes 8 int64 values at
 * device_buffer[8 b ..], ticks of the device's constant-rate wall clock (hipDeviceAttributeWallClockRate, kHz);
 * workgroups 0 .. num_shrink_tiles-1 are the plan's shrink tiles in list order, the expand tiles follow:
 *   shrink tile: [0] start  [1] descriptor, tokens and adapter pointer arrived  [2] v stores issued (first
 *                wavefront)  [3] every thread's v stores acknowledged  [4] the group's count added  [5], [7] unused
 *   expand tile: [0] start  [1] as above  [2] first Bt / y loads requested  [3] the group's count seen, or the
 *                bounded wait given up  [4] the tile's rows of v in LDS  [5] first wavefront's y stores
 *                acknowledged (left alone if that wavefront had no columns)  [7] 1 if the count was seen, 0 if
 *                the tile recomputed v itself
 *   both:        [6] where the workgroup ran: XCD number << 32 | the wavefront's hardware id register (compute
 *                unit in bits 8..11, shader array in bit 12, shader engine in bits 13..15)
 * device_buffer: device memory, 8-byte aligned, owned by the caller, who also clears it; it must hold 64 bytes per
 * tile of every plan used while it is set (lora_delta returns LORA_ERR_WORKSPACE otherwise and launches nothing).
 * NULL switches tracing off.  Process-wide; not for use while another thread launches.
 * Returns LORA_ERR_INVALID_ARG for a misaligned buffer or bytes == 0.
 */
lora_status lora_trace_set(void* device_buffer, size_t bytes);
/* rate of the clock the stamps count, in kHz, on the current device; 0 if it cannot be read */
int32_t     lora_trace_tick_khz(void);

/*
 * lora_probe -- measured ceilings of the machine, for benchmark reports (the per-kernel timers above time them
 * like any kernel of the library).  buffer: device memory, 16-byte aligned, `bytes` long.
 *   LORA_PROBE_EMPTY  a launch of 1280 workgroups (iters > 1: of iters workgroups) of 256 threads that does nothing:
 *                     the floor of any kernel duration
 *   LORA_PROBE_READ   one-shot read of the first floor(bytes / 32 KiB) * 32 KiB of the buffer, no dependency
 *                     between loads (every lane asks for its eight 16-byte pieces at once, whole cache lines per
 *                     wavefront, non-temporal): what a launch of that size can get out of HBM at best
 *   LORA_PROBE_MFMA   `iters` x 16 independent v_mfma_f32_16x16x32_bf16 per wavefront on register operands, 2048
 *                     workgroups of 4 wavefronts (2048 * 4 * iters * 16 * 16384 flops); writes the shader-clock
 *                     ticks and the wall-clock ticks the loop took on one wavefront to buffer[0], buffer[1] and
 *                     the wall clock's rate in kHz to buffer[2], as uint64: the clock the chip holds under
 *                     matrix load is buffer[0] / buffer[1] * buffer[2] kHz
 * Errors: LORA_ERR_INVALID_ARG for a null or misaligned buffer, bytes < 64, an unknown kind, iters < 1.
 */
enum { LORA_PROBE_EMPTY = 0, LORA_PROBE_READ = 1, LORA_PROBE_MFMA = 2 };
lora_status lora_probe(int32_t kind, void* buffer, size_t bytes, int32_t iters, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LORA_ABI_H */

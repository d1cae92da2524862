// Base GEMM y = x W (bf16 MFMA, fp32 accumulate), optionally with the adapter
// delta folded in: y = x W + v B_a per token, v = s_a (x A_a) from the shrink.
//
// This is the base-model product that unmerged inference shares across all
// requests of the batch, with the adapter branches added on top (paper
// sections 1-2); adding the delta to the fp32 accumulators before y is rounded
// makes unmerged inference cost close to merged inference (section 4.4).
//
// Both kernels walk the tokens in adapter-sorted order, so that neighbouring rows share an adapter.
//   gemm_ring_kernel: after the K loop every wavefront adds the deltas of its own 64 tokens to its accumulators,
//     adapter by adapter and 32 ranks at a time, with Bt_a[its features, ranks] and the tokens' v (split into two
//     bf16 terms v_hi + v_lo) straight from memory as MFMA operands (see the kernel).
//   gemm_tiled_kernel: the delta enters as extra k-stages of the same pipeline; for each adapter a present in a
//     row tile it runs ceil(2 r_a / 64) more stages whose "W tile" is Bt_a[features, ranks] and whose "x tile" is the
//     matching columns of [v_hi | v_lo] (rows of other adapters zero; Bt_a is simply addressed twice).  Their loads
//     are prefetched like any other stage's.
//
// x [T,K] and Wt [N,K] are both contraction-index-fastest, so tiles arrive in LDS
// as 16-byte chunks and come back out of it as ready-made MFMA operands (8
// consecutive k per lane).  Two kernels:
//
//   gemm_ring_kernel (further down): 256 x 256 tiles of large problems.  8 wavefronts, 16x16x32 MFMA,
//     loads HBM -> LDS directly into a ring of four 32-k stages.
//   gemm_tiled_kernel: everything else.  Loads HBM -> registers -> LDS, double buffered (dynamic LDS,
//     2 x (BM + BT) x 128 bytes); workgroup tile = 4 wavefronts (2 x 2), each WB x WB MFMA blocks of 32 x 32:
//     WB = 4: 256 features x 256 tokens x 64 k (K no multiple of 32)
//     WB = 2: 128 x 128 x 64 (small problems, less padding waste)
//
// Lane roles in v_mfma_f32_32x32x16_bf16 (D = A*B + C, A 32x16, B 16x32):
//   lane l supplies A[row l%32][k 8*(l/32) .. +7], B[k 8*(l/32) .. +7][col l%32],
//   receives D[row 8*(i/4) + 4*(l/32) + i%4][col l%32], i = 0..15.
// MFMA rows carry output features, columns carry tokens.  MFMA row 8q+4h+p of a
// block stands for feature 16h + 4q + p, so a lane (h = l/32) ends up with the
// 16 consecutive features 16h .. 16h+15 of its token: 32-byte stores of y.
#include <atomic>
#include "device_util.h"
#include "kernels.h"
#include "launch.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

union op16 {
    uint4 u;
    bf16x8 v;
};

namespace {

constexpr int BK = 64;    // k per stage; a tile row is 128 bytes = 8 chunks of 16 bytes

// LDS tile: rows x 8 chunks of 16 bytes; chunk c of row r lives at chunk slot c ^ f(r).  A ds_read_b128 of a
// wavefront is served 8 lanes at a time, so f must take 8 different values over the 8 rows those lanes read.
// x tile: lanes read consecutive rows -> f = r & 7.  W tile: lanes 8g..8g+7 read rows 4g..4g+3 and
// 16+4g..16+4g+3 (the feature permutation of the MFMA rows) -> f = (r & 3) | bit 4 of r << 2.
__device__ __forceinline__ int lds_slot(int row, int chunk) { return row * 8 + (chunk ^ ((row >> 1) & 7)); }
__device__ __forceinline__ int lds_slot_w(int row, int chunk) { return row * 8 + (chunk ^ (((row >> 1) & 3) | ((row >> 2) & 4))); }

// 16-byte loads through pointers that come out of a table or are computed from one: the address space is stated,
// or they would be flat loads (which also count as LDS traffic, so that waits on them are coarse)
__device__ __forceinline__ uint4 ldg16(const void* p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const u32x4 r = *(const __attribute__((address_space(1))) u32x4*)(uintptr_t)p;
    return uint4{r[0], r[1], r[2], r[3]};
#else       // the host pass only parses device functions
    return *reinterpret_cast<const uint4*>(p);
#endif
}

// the same from a wavefront-uniform base plus a 32-bit byte offset per lane (one address register per lane for any
// number of loads that share the offset)
__device__ __forceinline__ uint4 ldg16_off(const void* uniform_base, uint32_t byte_off)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const __attribute__((address_space(1))) char* b = (const __attribute__((address_space(1))) char*)(uintptr_t)uniform_base;
    const u32x4 r = *(const __attribute__((address_space(1))) u32x4*)(b + byte_off);
    return uint4{r[0], r[1], r[2], r[3]};
#else
    return *reinterpret_cast<const uint4*>(static_cast<const char*>(uniform_base) + byte_off);
#endif
}

__device__ __forceinline__ void split_bf16(const float* f, op16& hi, op16& lo)
{
    uint32_t h[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const bf16_t hb = f32_to_bf16(f[i]);
        h[i] = hb;
        l[i] = f32_to_bf16(f[i] - bf16_to_f32(hb));
    }
    hi.u = uint4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    lo.u = uint4{l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
}

extern __shared__ uint4 gemm_lds[];
constexpr int META_MAX = 256;      // adapter stages of a tile whose metadata is cached in LDS (more are read from memory)

struct gemm_delta_args {
    const int32_t* order;          // [T] tokens sorted by adapter, then tokens without adapter; nullptr = identity
    const int32_t* row_key;        // [T] the token's adapter (bits 0..22; all ones: none) | removal bit
    const int32_t* rank;
    const int32_t* extra_ptr;      // [token tiles + 1]
    const int32_t* extra;          // stage id (adapter, | removal bit) | rank block << 24
    const bf16_t* vb;              // [T][2][R]: v_hi, v_lo
    int R;
    const bf16_t* const* Bt_ptrs;
    const bf16_t* zeros;           // 16 zero bytes: the source of chunks that are masked out
    const bf16_t* vb2;             // mixture mode: [T][2][R2] split of the removal's v (read by the marked stages)
    int R2;
    int merged;                    // mixture mode: the merged adapter, else -1
};

// Stage ids and row keys.  An ordinary stage (id = adapter) concerns the rows of that adapter.  A stage whose id
// carries the removal bit (mixture mode: the merged adapter's update is taken off again) concerns every row whose key
// carries it: the rows of all other adapters and of none.  Rows beyond T have the key "none" without the bit.
constexpr int STAGE_REMOVAL = LORA_UNMERGE_BIT, KEY_NONE = LORA_UNMERGE_BIT - 1;
__device__ __forceinline__ bool stage_hits(int row_key, int stage_id)
{
    return (stage_id & STAGE_REMOVAL) ? (row_key & STAGE_REMOVAL) != 0 : (row_key & KEY_NONE) == stage_id;
}
// columns [part * r + j, + 8) of the token's [v_hi | v_lo] that the stage reads
__device__ __forceinline__ const bf16_t* stage_v(const gemm_delta_args& da, int stage_id, int token, int part, int j)
{
    return (stage_id & STAGE_REMOVAL) ? da.vb2 + ((int64_t)token * 2 + part) * da.R2 + j
                                      : da.vb + ((int64_t)token * 2 + part) * da.R + j;
}

// Workgroups are dealt round-robin to the 8 XCDs; every XCD gets a contiguous run of tiles (so its L2 sees
// neighbouring tiles).  Inside a run the tiles go in groups of GN feature tiles, token tile fastest over GN
// feature tiles, so the 32 tiles an XCD works on at a time form an 8 x 4 block and share 8 x panels and 4 W
// panels (instead of 32 x panels and one W panel) in its L2.
__device__ __forceinline__ void tile_of_workgroup(int id, int tiles_n, int tiles_t, int& tile_n, int& tile_t)
{
    const int n_wg = tiles_n * tiles_t;
    const int per = n_wg / 8, rem = n_wg % 8;
    const int xcd = id & 7, q = id >> 3;
    id = xcd * per + (xcd < rem ? xcd : rem) + q;       // XCD k owns per + (k < rem) tiles
    constexpr int GN = 4;
    const int group = id / (GN * tiles_t), first_n = group * GN;
    const int group_n = min(tiles_n - first_n, GN);
    const int in_group = id - group * (GN * tiles_t);
    tile_n = first_n + in_group % group_n;
    tile_t = in_group / group_n;
}

// KTAIL: K is not a multiple of 64, the last K stage's chunks beyond K are zero-filled
template <int WB, bool DELTA, bool KTAIL>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(
    int T, int K, int N, const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ Wt, int64_t ldw,
    bf16_t* __restrict__ y, int64_t ldy, int tiles_n, int tiles_t, gemm_delta_args da)
{
    constexpr int BM = 64 * WB;            // features per workgroup tile
    constexpr int BT = 64 * WB;            // tokens per workgroup tile
    constexpr int NLD = (BM * 8) / 256;    // 16-byte chunks of W (and of x) per thread and stage
    uint4* lds_w0 = gemm_lds;                       // [2][BM * 8]
    uint4* lds_x0 = gemm_lds + 2 * BM * 8;          // [2][BT * 8]
    // DELTA: the tile's adapter stages {adapter, rank, Bt pointer} are fetched once, up front, into LDS
    uint4* lds_meta = gemm_lds + 4 * BM * 8;        // [META_MAX]
    // DELTA: token and adapter of the rows this thread stages, parked in LDS so that they hold no
    // registers during the K stages: [NLD][256] int2
    int2* lds_rows = reinterpret_cast<int2*>(lds_meta + META_MAX);

    int tile_n, tile_t;
    tile_of_workgroup(blockIdx.x, tiles_n, tiles_t, tile_n, tile_t);
    const int n0 = tile_n * BM, t0 = tile_t * BT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = (wave & 1) * (32 * WB), wt = (wave >> 1) * (32 * WB);   // wavefront tile origin
    const int c_lane8 = (tid & 7) * 8;                           // this thread's k offset inside a stage

    // global -> register staging: the rows this thread fetches in every stage
    const bf16_t* gw[NLD];
    const bf16_t* gx[NLD];
    int slot[NLD], slot_w[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int q = tid + i * 256, row = q >> 3, c = q & 7;
        int nr = n0 + row; if (nr >= N) nr = N - 1;
        int pos = t0 + row;
        const bool pos_ok = pos < T;
        if (!pos_ok) pos = T - 1;
        const int tok = DELTA ? da.order[pos] : pos;
        gw[i] = Wt + (int64_t)nr * ldw + c * 8;
        gx[i] = x + (int64_t)tok * ldx + c * 8;
        slot[i] = lds_slot(row, c);
        slot_w[i] = lds_slot_w(row, c);
        if constexpr (DELTA) lds_rows[i * 256 + tid] = make_int2(tok, pos_ok ? da.row_key[tok] : KEY_NONE);
    }

    floatx16 acc[WB][WB];
#pragma unroll
    for (int a = 0; a < WB; ++a)
#pragma unroll
        for (int b = 0; b < WB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // LDS rows this lane reads as MFMA operands
    const int l32 = lane & 31, h = lane >> 5;
    // feature of MFMA row l32 = 8q + 4hh + p  ->  16 hh + 4 q + p
    const int frow = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);

    const int stages_k = (K + BK - 1) / BK;
    int extra_base = 0, n_extra = 0, stages = stages_k;
    if constexpr (DELTA) {
        extra_base = da.extra_ptr[tile_t];
        n_extra = da.extra_ptr[tile_t + 1] - extra_base;
        stages += n_extra;
        for (int e = tid; e < n_extra && e < META_MAX; e += 256) {
            const int packed = da.extra[extra_base + e];
            const int a_id = packed & KEY_NONE;
            const uint64_t bt = reinterpret_cast<uint64_t>(da.Bt_ptrs[a_id]);
            lds_meta[e] = uint4{(uint32_t)packed, (uint32_t)da.rank[a_id], (uint32_t)bt, (uint32_t)(bt >> 32)};
        }
    }
    bool skip[WB];                                               // column blocks without a token of the stage's adapter
#pragma unroll
    for (int b = 0; b < WB; ++b) skip[b] = false;
    uint4 rw[NLD], rx[NLD];
    auto load_k_stage = [&](int s) {
        const int k = s * BK;
        const bool in = !KTAIL || k + c_lane8 < K;               // K % 8 == 0: chunk is whole or absent
        // same issue order as in the steady loop: all W chunks, then all x chunks
#pragma unroll
        for (int i = 0; i < NLD; ++i) rw[i] = in ? *reinterpret_cast<const uint4*>(gw[i] + k) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < NLD; ++i) rx[i] = in ? *reinterpret_cast<const uint4*>(gx[i] + k) : uint4{0, 0, 0, 0};
    };
    auto load_stage = [&](int s) {
        if (!DELTA || s < stages_k) {
            load_k_stage(s);
        } else {
            // adapter stage: Bt_a[feature rows, ranks] against 64 columns of [v_hi | v_lo] of the adapter's tokens
            const int e = s - stages_k;
            int packed, r;
            const bf16_t* Bt;
            if (e < META_MAX) {
                const uint4 m = lds_meta[e];
                packed = (int)m.x;
                r = (int)m.y;
                Bt = reinterpret_cast<const bf16_t*>((uint64_t)m.z | ((uint64_t)m.w << 32));
            } else {
                packed = da.extra[extra_base + e];
                r = da.rank[packed & KEY_NONE];
                Bt = da.Bt_ptrs[packed & KEY_NONE];
            }
            const int a_id = packed & 0xffffff;
            // column of the adapter's [v_hi | v_lo] concatenation; r % 8 == 0, so a chunk lies in one half
            const int col = (packed >> 24) * 64 + c_lane8;
            const bool in = col < 2 * r;
            const int part = col >= r ? 1 : 0;
            const int j = col - part * r;
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                int nr = n0 + ((tid + i * 256) >> 3);
                if (nr >= N) nr = N - 1;
                const int2 ta = lds_rows[i * 256 + tid];         // (token, its adapter)
                rw[i] = in ? *reinterpret_cast<const uint4*>(Bt + (int64_t)nr * r + j) : uint4{0, 0, 0, 0};
                rx[i] = (in && stage_hits(ta.y, a_id))
                            ? *reinterpret_cast<const uint4*>(stage_v(da, a_id, ta.x, part, j))
                            : uint4{0, 0, 0, 0};
            }
        }
    };
    auto store_stage = [&](int buf) {
        uint4* lw = lds_w0 + buf * BM * 8;
        uint4* lx = lds_x0 + buf * BT * 8;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            lw[slot_w[i]] = rw[i];
            lx[slot[i]] = rx[i];
        }
    };
    auto read_ops = [&](const uint4* lw, const uint4* lx, int ks, op16 (&wa)[WB], op16 (&xb)[WB]) {
        const int c = ks * 2 + h;
#pragma unroll
        for (int a = 0; a < WB; ++a) wa[a].u = lw[lds_slot_w(wn + a * 32 + frow, c)];
#pragma unroll
        for (int b = 0; b < WB; ++b) xb[b].u = lx[lds_slot(wt + b * 32 + l32, c)];
    };
    auto mma = [&](const op16 (&wa)[WB], const op16 (&xb)[WB]) {
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            if (DELTA && skip[b]) continue;                      // wavefront-uniform
#pragma unroll
            for (int a = 0; a < WB; ++a)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[a].v, xb[b].v, acc[a][b], 0, 0, 0);
        }
    };
    // an adapter stage only concerns the column blocks that hold one of the adapter's tokens
    auto set_skip = [&](int stage) {
        if constexpr (DELTA) {
            if (stage < stages_k) return;
            const int e = stage - stages_k;
            const int a_id = (e < META_MAX ? (int)lds_meta[e].x : da.extra[extra_base + e]) & 0xffffff;
#pragma unroll
            for (int b = 0; b < WB; ++b) {
                // row wt + 32 b + l32 of the tile is staged by thread (row * 8) & 255 as its chunk slot (row * 8) >> 8
                const int q = (wt + b * 32 + (lane & 31)) * 8;
                skip[b] = __ballot(stage_hits(lds_rows[(q >> 8) * 256 + (q & 255)].y, a_id)) == 0;
            }
        }
    };

    // Software pipeline.  Global loads run two stages ahead (registers), LDS is double
    // buffered, MFMA operands are double buffered in registers: while the matrix cores
    // work on k-step ks the LDS reads of ks+1 are in flight, and the barrier between
    // stages sits before the last k-step so that its MFMAs cover the first reads of the
    // next stage.
    op16 waA[WB], xbA[WB], waB[WB], xbB[WB];
    int s = 0;
    const bool steady = WB == 4 && !KTAIL && stages_k >= 3 && n_extra <= META_MAX;
    if (!steady) {
        // (the adapter stages' descriptors in LDS are read by every thread: with a single K stage the load of
        // stage 1 below is already an adapter stage's)
        if constexpr (DELTA) __syncthreads();
        load_stage(0);
        store_stage(0);
        if (stages > 1) load_stage(1);
        __syncthreads();
        read_ops(lds_w0, lds_x0, 0, waA, xbA);
    }
    if constexpr (WB == 4 && !KTAIL) if (steady) {
        // (its own straight-line prologue: were the steady loop reachable through the branchy general
        // loader, the compiler would wait for all outstanding loads at the top of every iteration)
        // Running source pointers of the stage to fetch next.  A K stage advances them by 64 elements; an
        // adapter stage sets them afresh: W chunks to Bt_a[feature row, ranks], x chunks to the token's
        // [v_hi | v_lo] columns, and every chunk that is masked out (beyond the rank, or a token of another
        // adapter) to a block of zeros -- so all stages issue the same 16 unconditional loads.
        const bf16_t* pw[NLD];
        const bf16_t* px[NLD];
#pragma unroll
        for (int i = 0; i < NLD; ++i) { pw[i] = gw[i]; px[i] = gx[i]; }
        auto advance = [&](int next) {
            if (!DELTA || next < stages_k) {
#pragma unroll
                for (int i = 0; i < NLD; ++i) { pw[i] += BK; px[i] += BK; }
            } else if (next < stages) {
                const uint4 m = lds_meta[next - stages_k];
                const int a_id = (int)m.x & 0xffffff, r = (int)m.y;
                const bf16_t* Bt = reinterpret_cast<const bf16_t*>((uint64_t)m.z | ((uint64_t)m.w << 32));
                const int col = ((int)m.x >> 24) * 64 + c_lane8;
                const bool in = col < 2 * r;
                const int part = col >= r ? 1 : 0;
                const int j = col - part * r;
#pragma unroll
                for (int i = 0; i < NLD; ++i) {
                    int nr = n0 + ((tid + i * 256) >> 3);
                    if (nr >= N) nr = N - 1;
                    const int2 ta = lds_rows[i * 256 + tid];
                    pw[i] = in ? Bt + (int64_t)nr * r + j : da.zeros;
                    px[i] = (in && stage_hits(ta.y, a_id)) ? stage_v(da, a_id, ta.x, part, j) : da.zeros;
                }
            }
        };
        auto load_ptrs = [&]() {
#pragma unroll
            for (int i = 0; i < NLD; ++i) rw[i] = *reinterpret_cast<const uint4*>(pw[i]);
#pragma unroll
            for (int i = 0; i < NLD; ++i) rx[i] = *reinterpret_cast<const uint4*>(px[i]);
        };
        __syncthreads();                                 // lds_meta / lds_rows are complete
        // stages 0, 1 and 2 are K stages (stages_k >= 3): straight-line code up to the first loop (were it
        // reachable through a branch with loads in flight, the compiler would wait for all of them at the
        // top of every iteration instead of the oldest one)
        load_ptrs();
        store_stage(0);
#pragma unroll
        for (int i = 0; i < NLD; ++i) { pw[i] += BK; px[i] += BK; }
        load_ptrs();
#pragma unroll
        for (int i = 0; i < NLD; ++i) { pw[i] += BK; px[i] += BK; }
        __syncthreads();
        read_ops(lds_w0, lds_x0, 0, waA, xbA);
        // Steady state over all stages but the last two, written out so that every MFMA is followed by exactly
        // one memory operation (the scheduler is pinned to that order): the 64 MFMAs of a stage
        // carry its 32 LDS operand reads, the 16 LDS writes of the next stage and the 16 global
        // loads of the stage after that, and the matrix cores never wait for a block of them.
        auto one_read = [&](const uint4* lw, const uint4* lx, int ks, int i, op16 (&wa)[WB], op16 (&xb)[WB]) {
            const int c = ks * 2 + h;
            if (i < 4) wa[i].u = lw[lds_slot_w(wn + i * 32 + frow, c)];
            else xb[i - 4].u = lx[lds_slot(wt + (i - 4) * 32 + l32, c)];
        };
#define MMA1(WA, XB, IDX) \
        acc[(IDX) >> 2][(IDX) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(WA[(IDX) >> 2].v, XB[(IDX) & 3].v, acc[(IDX) >> 2][(IDX) & 3], 0, 0, 0)
#define PIN(MASK) do { __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); __builtin_amdgcn_sched_group_barrier(MASK, 1, 0); } while (0)
        // the body of one stage; ADV_GENERAL: the pointer update after it may set up an adapter stage
#define STAGE_BODY(ADV_GENERAL)                                                                                        \
        {                                                                                                              \
            const int buf = s & 1;                                                                                     \
            const uint4* lw = lds_w0 + buf * BM * 8;                                                                   \
            const uint4* lx = lds_x0 + buf * BT * 8;                                                                   \
            uint4* lw_n = lds_w0 + (buf ^ 1) * BM * 8;                                                                 \
            uint4* lx_n = lds_x0 + (buf ^ 1) * BT * 8;                                                                 \
            /* k-step 0: reads of k-step 1, W chunks of stage s+1 into LDS */                                          \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waA, xbA, i); one_read(lw, lx, 1, i, waB, xbB); PIN(0x100); }       \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waA, xbA, 8 + i); lw_n[slot_w[i]] = rw[i]; PIN(0x200); }           \
            /* k-step 1: reads of k-step 2, x chunks of stage s+1 into LDS */                                          \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waB, xbB, i); one_read(lw, lx, 2, i, waA, xbA); PIN(0x100); }       \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waB, xbB, 8 + i); lx_n[slot[i]] = rx[i]; PIN(0x200); }             \
            /* k-step 2: reads of k-step 3, W chunks of stage s+2 from memory */                                       \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waA, xbA, i); one_read(lw, lx, 3, i, waB, xbB); PIN(0x100); }       \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waA, xbA, 8 + i); rw[i] = *reinterpret_cast<const uint4*>(pw[i]); PIN(0x020); } \
            __syncthreads(); /* stage s+1 is in LDS; nobody reads stage s any more */                                  \
            /* k-step 3: reads of k-step 0 of stage s+1, x chunks of stage s+2 from memory */                          \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waB, xbB, i); one_read(lw_n, lx_n, 0, i, waA, xbA); PIN(0x100); }   \
            _Pragma("unroll") for (int i = 0; i < 8; ++i) { MMA1(waB, xbB, 8 + i); rx[i] = *reinterpret_cast<const uint4*>(px[i]); PIN(0x020); } \
            if (ADV_GENERAL) advance(s + 3);                                                                           \
            else { _Pragma("unroll") for (int i = 0; i < NLD; ++i) { pw[i] += BK; px[i] += BK; } }                     \
        }
        // K stages whose successors are K stages too: a loop without any branch in its body (a branch
        // makes the compiler wait for all outstanding loads instead of the oldest one)
        for (; s + 3 < stages_k; ++s) STAGE_BODY(false)
        // the stages around and inside the adapter part
        for (; s + 2 < stages; ++s) STAGE_BODY(true)
#undef STAGE_BODY
#undef MMA1
#undef PIN
    }
    // the last two stages (and everything, for the small tile / K tail builds)
    for (; s < stages; ++s) {
        set_skip(s);
        const int buf = s & 1;
        const uint4* lw = lds_w0 + buf * BM * 8;
        const uint4* lx = lds_x0 + buf * BT * 8;
        const uint4* lw_n = lds_w0 + (buf ^ 1) * BM * 8;
        const uint4* lx_n = lds_x0 + (buf ^ 1) * BT * 8;
        read_ops(lw, lx, 1, waB, xbB);
        mma(waA, xbA);
        read_ops(lw, lx, 2, waA, xbA);
        if (s + 1 < stages) store_stage(buf ^ 1);        // stage s+1: fetched one stage ago
        if (s + 2 < stages) load_stage(s + 2);
        mma(waB, xbB);
        read_ops(lw, lx, 3, waB, xbB);
        mma(waA, xbA);
        __syncthreads();                                 // stage s+1 is in LDS; nobody reads stage s any more
        if (s + 1 < stages) read_ops(lw_n, lx_n, 0, waA, xbA);
        mma(waB, xbB);
    }

    // ---- epilogue: one rounding, store (rows go back to their tokens) ------
#pragma unroll
    for (int b = 0; b < WB; ++b) {
        const int pos = t0 + wt + b * 32 + l32;                  // this lane's row of the order in column block b
        if (pos >= T) continue;
        const int t = DELTA ? da.order[pos] : pos;
#pragma unroll
        for (int a = 0; a < WB; ++a) {
            const int n = n0 + wn + a * 32 + 16 * h;             // first of this lane's 16 features
            bf16_t* yp = y + (int64_t)t * ldy + n;
            // acc index i = 4q + p  <->  feature offset 4q + p
            if (n + 16 <= N) {
                uint32_t o[8];
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    o[q] = (uint32_t)f32_to_bf16(acc[a][b][2 * q]) | ((uint32_t)f32_to_bf16(acc[a][b][2 * q + 1]) << 16);
                *reinterpret_cast<uint4*>(yp) = uint4{o[0], o[1], o[2], o[3]};
                *reinterpret_cast<uint4*>(yp + 8) = uint4{o[4], o[5], o[6], o[7]};
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (n + i < N) yp[i] = f32_to_bf16(acc[a][b][i]);
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------------------
// Ring variant of the 256 x 256 tile: the same MFMA blocking and lane roles, but the tiles go HBM -> LDS
// directly (global_load_lds_dwordx4, no staging registers, no LDS write instructions) into a ring of four
// stages of 32 k, three stages ahead of the one the matrix cores work on.  A workgroup's tile walks through
// lines that nobody has touched yet, stage after stage, so its loads see memory latency (microseconds
// under load), not L2 latency; with register staging the fetch distance was half a 64-k stage.
//
// A direct-to-LDS load puts lane i's 16 bytes at LDS address M0 + 16 i: the LDS image of one load is 1 KB
// contiguous = 16 tile rows of 64 bytes, and the XOR swizzle is applied on the global side (lane i fetches the
// chunk that belongs in slot i).  The loads are issued from inline assembly, so the compiler does not count
// them: the waits for them are written out (s_waitcnt vmcnt), and since memory returns loads in order,
// "at most 16 outstanding" means that everything but the two youngest stages has landed.
constexpr int RK = 32;             // k per ring stage; a tile row is 64 bytes = 4 chunks of 16 bytes
constexpr int RING = 4;            // stages in the LDS ring
constexpr int RING_STAGE = 2048;   // uint4 per stage: 256 W rows x 4 chunks, then 256 x rows x 4 chunks

// Chunk c of row r lives at slot 4 r + (c ^ f(r)).  An operand read (ds_read_b128) has lane l take chunk l / 16 of
// one of 16 rows: x rows r0 + l % 16, W rows r0 + 16 (l % 16 / 4) + l % 4 (the MFMA row permutation).  The f below
// make these reads free of bank conflicts (checked with the SQ_LDS_BANK_CONFLICT counter on a read-only kernel:
// 0 stalled cycles, against half of all LDS cycles for f = bits 2..3 of r, or none).
__device__ __forceinline__ int ring_f_x(int row) { return (row >> 1) & 3; }
__device__ __forceinline__ int ring_f_w(int row) { return ((row >> 1) & 1) | ((row >> 3) & 2); }

typedef __attribute__((address_space(3))) void* lds_void_ptr;
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)(lds_void_ptr)p; }

// lane i's 16 bytes at g -> LDS byte address lds_base + 16 i (lds_base wavefront-uniform).  M0 carries the LDS
// address; nothing else in these kernels uses M0 (LDS instructions of gfx9 and later do not read it).
__device__ __forceinline__ void load16_to_lds(const void* g, uint32_t lds_base)
{
    // (readfirstlane: the operand has to be a scalar register also where the compiler cannot prove it uniform)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory");
}

template <bool DELTA>
__global__ __launch_bounds__(512) void gemm_ring_kernel(
    int T, int K, int N, const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ Wt, int64_t ldw,
    bf16_t* __restrict__ y, int64_t ldy, int tiles_n, int tiles_t, gemm_delta_args da)
{
    // Eight wavefronts, two per SIMD, each 128 features x 64 tokens = 4 x 2 MFMA blocks (128 accumulator
    // registers).  A wavefront cannot issue an MFMA while it issues a load (each load costs it about one
    // MFMA slot, also with all lanes masked off); with a second wavefront on the SIMD the matrix core takes
    // that one's MFMA meanwhile.
    //
    // DELTA: the rows of the tile are tokens in adapter-sorted order, and after the K loop every wavefront adds the
    // adapter deltas of its own 64 tokens to its accumulators by itself: for each adapter among them (one or two,
    // mostly) and each block of 32 ranks, Bt_a[its 128 features, 32 ranks] as the MFMA row operand straight from
    // memory, and the tokens' v (its two bf16 terms) as the column operands, masked to the adapter's tokens.  No LDS, no workgroup barrier, no work for the rows of other wavefronts: a wavefront pays
    // for the adapters of its own 64 tokens only, where a shared adapter stage would cost all eight of them a whole
    // 256 x 256 x 32 step per adapter and block of ranks.
    constexpr int BM = 256, BT = 256, WA = 8, WX = 4;
    uint4* ring = gemm_lds;                                          // [RING][RING_STAGE]

    int tile_n, tile_t;
    tile_of_workgroup(blockIdx.x, tiles_n, tiles_t, tile_n, tile_t);
    const int n0 = tile_n * BM, t0 = tile_t * BT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = (wave & 1) * 128, wt = (wave >> 1) * 64;         // wavefront tile origin
    // Lane roles in v_mfma_f32_16x16x32_bf16 (D = A*B + C, A 16x32, B 32x16): lane l supplies A[row l%16][k 8(l/16) ..
    // +7] and B[k 8(l/16) .. +7][col l%16], and receives D[row 4(l/16) + i][col l%16], i = 0..3.  MFMA rows carry
    // features, columns carry tokens.  The 128 features of a wavefront are two groups of 64; block q of a group
    // holds the features 16 g + 4 q + i (MFMA row 4 g + i), so that over its four blocks a lane (g = l/16) ends up
    // with the 16 consecutive features 16 g .. 16 g + 15 of its token.
    const int l16 = lane & 15, kg = lane >> 4;
    const int frow = 16 * (l16 >> 2) + (l16 & 3);                   // feature (block 0 of a group) of MFMA row l16

    // Staging role: load j of this wavefront fills slots (2 wave + j) 64 .. +63 of the W part and of the x part
    // of a stage, i.e. rows (2 wave + j) 16 .. +15; this lane brings chunk slot lane & 3 of row .. + lane / 4.
    const int pc = lane & 3;
    const bf16_t* pw[2];
    const bf16_t* px[2];
    int cw[2];                                                       // logical chunk this lane fetches (W side)
    const int cx = pc ^ ring_f_x(lane >> 2);                         // (x side: the same for both loads)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int row = (wave * 2 + j) * 16 + (lane >> 2);
        cw[j] = pc ^ ring_f_w(row);
        int nr = n0 + row; if (nr >= N) nr = N - 1;
        int pos = t0 + row;
        const bool pos_ok = pos < T;
        if (!pos_ok) pos = T - 1;
        const int tok = DELTA ? da.order[pos] : pos;
        pw[j] = Wt + (int64_t)nr * ldw + cw[j] * 8;
        px[j] = x + (int64_t)tok * ldx + cx * 8;
    }
    // DELTA: token and key of row wt + lane of the tile (this wavefront's 64 tokens, one per lane)
    int my_tok = 0, my_key = KEY_NONE;
    if constexpr (DELTA) {
        const int pos = t0 + wt + lane;
        my_tok = da.order[pos < T ? pos : T - 1];
        my_key = pos < T ? da.row_key[my_tok] : KEY_NONE;
    }

    const int stages_k = K / RK;                                     // K % 32 == 0, stages_k >= 4 (checked by the launcher)
    const int stages = stages_k;

    floatx4 acc[WA][WX];
#pragma unroll
    for (int a = 0; a < WA; ++a)
#pragma unroll
        for (int b = 0; b < WX; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

    // source pointers of the stage to fetch next
    auto advance = [&](int next) {
        if (next < stages) {
#pragma unroll
            for (int j = 0; j < 2; ++j) { pw[j] += RK; px[j] += RK; }
        }
    };
    const uint32_t lds_w = __builtin_amdgcn_readfirstlane(lds_address(ring) + wave * 2048), lds_x = lds_w + 16384;
    auto issue = [&](int buf, int j4) {                              // one of the four loads of a stage
        const uint32_t base = (uint32_t)buf * (RING_STAGE * 16) + (j4 & 1) * 1024;
        if (j4 < 2) load16_to_lds(pw[j4 & 1], lds_w + base);
        else load16_to_lds(px[j4 & 1], lds_x + base);
    };

    // operand slots of a stage: one ds_read_b128 of a wavefront is one 16 x 32 operand block (lane group kg reads
    // chunk kg of its row); W block a = 4 G + q: + (64 G + 4 q) rows; x block b: + 16 b rows
    const int sw0 = (wn + frow) * 4 + (kg ^ ring_f_w(frow));
    const int sx0 = RING_STAGE / 2 + (wt + l16) * 4 + (kg ^ ring_f_x(l16));
    // W operands are single-buffered (block a is re-read for the next stage once its four MFMAs are out), x
    // operands double-buffered
    op16 wa[WA], xbA[WX], xbB[WX];
    auto read_w = [&](const uint4* st, int a) { wa[a].u = st[sw0 + ((a >> 2) * 64 + (a & 3) * 4) * 4]; };
    auto read_x = [&](const uint4* st, int b, op16 (&xb)[WX]) { xb[b].u = st[sx0 + b * 64]; };
#define RING_MMA(XB_, A_, B_) \
    acc[A_][B_] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[A_].v, XB_[B_].v, acc[A_][B_], 0, 0, 0)
#define RING_FENCE() __builtin_amdgcn_sched_barrier(0)

    // prologue: stages 0, 1, 2 on their way (all K stages), stage 0 landed, its first operands read
#pragma unroll
    for (int s0 = 0; s0 < 3; ++s0) {
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) issue(s0, j4);
        advance(s0 + 1);
    }
    asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
#pragma unroll
    for (int b = 0; b < WX; ++b) read_x(ring, b, xbA);
#pragma unroll
    for (int a = 0; a < 4; ++a) read_w(ring, a);

    // One stage = 32 MFMAs.  First half (W blocks 0..3): the reads of W blocks 4..7 of this stage and two of the
    // four loads of stage s + 3 (into the buffer that stage s - 1 used; everybody left it before the previous
    // barrier).  Then the wavefront waits until its own loads of stage s + 1 have landed (AHEAD = loads allowed
    // to be still outstanding) and for its LDS reads, and meets the others.  Second half (W blocks 4..7): the
    // reads of W blocks 0..3 and of the x blocks of stage s + 1, and the other two loads.
#define RING_HALF_STAGE(XB_, XN_, ISSUE, AHEAD, LAST)                                                                  \
    {                                                                                                                  \
        const uint4* st = ring + (s & 3) * RING_STAGE;                                                                 \
        const uint4* st_n = ring + ((s + 1) & 3) * RING_STAGE;                                                         \
        _Pragma("unroll") for (int i = 0; i < 16; ++i) {                                                               \
            RING_MMA(XB_, i >> 2, i & 3);                                                                              \
            if ((i & 3) == 1 && i < 16) read_w(st, 4 + (i >> 2));                                                      \
            if (ISSUE && (i == 7 || i == 11)) issue((s + 3) & 3, i == 7 ? 0 : 1);                                      \
            RING_FENCE();                                                                                              \
        }                                                                                                              \
        if (!(LAST)) asm volatile("s_waitcnt vmcnt(" #AHEAD ") lgkmcnt(0)\n\ts_barrier" ::: "memory");                   \
        _Pragma("unroll") for (int i = 16; i < 32; ++i) {                                                              \
            RING_MMA(XB_, i >> 2, i & 3);                                                                              \
            if (!(LAST) && (i & 1) == 0) { if (i < 24) read_x(st_n, (i - 16) >> 1, XN_); else read_w(st_n, (i - 24) >> 1); } \
            if (ISSUE && (i == 21 || i == 27)) issue((s + 3) & 3, i == 21 ? 2 : 3);                                    \
            RING_FENCE();                                                                                              \
        }                                                                                                              \
    }
    // Two stages per loop iteration, so that the x operand buffers swap roles statically; an odd number of
    // stages ahead of the last three is evened out by one stage up front and a register copy.
    int s = 0;
    if ((stages - 3) & 1) {
        RING_HALF_STAGE(xbA, xbB, true, 6, false)
        advance(4);
        _Pragma("unroll") for (int b = 0; b < WX; ++b) xbA[b].u = xbB[b].u;
        s = 1;
    }
    // K stages whose fourth successor is a K stage too: no branch in the body
    for (; s + 5 < stages_k; s += 2) {
        RING_HALF_STAGE(xbA, xbB, true, 6, false)
        _Pragma("unroll") for (int j = 0; j < 2; ++j) { pw[j] += RK; px[j] += RK; }
        ++s;
        RING_HALF_STAGE(xbB, xbA, true, 6, false)
        _Pragma("unroll") for (int j = 0; j < 2; ++j) { pw[j] += RK; px[j] += RK; }
        --s;
    }
    // the stages whose fourth successor may lie beyond the end
    for (; s + 4 < stages; s += 2) {
        RING_HALF_STAGE(xbA, xbB, true, 6, false)
        advance(s + 4);
        ++s;
        RING_HALF_STAGE(xbB, xbA, true, 6, false)
        advance(s + 4);
        --s;
    }
    // the last three stages fetch nothing
    RING_HALF_STAGE(xbA, xbB, false, 4, false)
    ++s;
    RING_HALF_STAGE(xbB, xbA, false, 0, false)
    ++s;
    RING_HALF_STAGE(xbA, xbB, false, 0, true)
#undef RING_HALF_STAGE
#undef RING_MMA
#undef RING_FENCE

    // ---- adapter deltas of this wavefront's 64 tokens -----------------------
    if constexpr (DELTA) {
        // token of MFMA column l16 of token block b
        int tokb[WX];
#pragma unroll
        for (int b = 0; b < WX; ++b) tokb[b] = __shfl(my_tok, 16 * b + l16);
        // acc += Bt_a[features, ranks] x v[tokens in `members`, ranks]^T  (members: bit i = row wt + i of the tile)
        auto apply = [&](int a, uint64_t members, const bf16_t* __restrict__ vb, int R) {
            const int r = da.rank[a];
            const char* Bt = reinterpret_cast<const char*>(da.Bt_ptrs[a]);
            const int row = n0 + wn + frow;                          // feature of MFMA row l16 in block 0
            for (int j0 = 0; j0 < r; j0 += 32) {
                const int j = j0 + 8 * kg;                           // this lane's 8 ranks of the block
                const bool in = j < r;                               // r % 8 == 0: all eight or none
                const uint32_t lane_off = (uint32_t)(row * r + j) * 2u;
                // all loads of the block go out before the first is waited for (no branch between them)
                op16 wb[WA], vh[WX], vl[WX];
#pragma unroll
                for (int blk = 0; blk < WA; ++blk) {
                    const int d = (blk >> 2) * 64 + (blk & 3) * 4;   // block blk holds the features row + d
                    wb[blk].u = (in && row + d < N) ? ldg16_off(Bt + (int64_t)d * r * 2, lane_off) : uint4{0, 0, 0, 0};
                }
#pragma unroll
                for (int b = 0; b < WX; ++b) {
                    const bool mine = in && ((members >> (16 * b + l16)) & 1ull);
                    const uint32_t off = (uint32_t)(tokb[b] * 2 * R + j) * 2u;   // (the launcher keeps T R 4 below 2^32)
                    vh[b].u = mine ? ldg16_off(vb, off) : uint4{0, 0, 0, 0};
                    vl[b].u = mine ? ldg16_off(vb, off + (uint32_t)R * 2u) : uint4{0, 0, 0, 0};
                }
#pragma unroll
                for (int b = 0; b < WX; ++b) {
                    if (((members >> (16 * b)) & 0xffffull) == 0) continue;      // wavefront-uniform
#pragma unroll
                    for (int blk = 0; blk < WA; ++blk) {
                        acc[blk][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[blk].v, vh[b].v, acc[blk][b], 0, 0, 0);
                        acc[blk][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb[blk].v, vl[b].v, acc[blk][b], 0, 0, 0);
                    }
                }
            }
        };
        const int own = my_key & KEY_NONE;
        uint64_t todo = __ballot(own != KEY_NONE);
        while (todo) {                                               // the distinct adapters among the 64 tokens
            const int a = __builtin_amdgcn_readlane(own, __ffsll((unsigned long long)todo) - 1);
            const uint64_t members = __ballot(own == a);
            todo &= ~members;
            apply(a, members, da.vb, da.R);
        }
        const uint64_t removal = __ballot((my_key & STAGE_REMOVAL) != 0);
        if (removal) apply(da.merged, removal, da.vb2, da.R2);     // mixture mode: the merged adapter, negated, for all of them
    }

    // ---- epilogue: one rounding, store (rows go back to their tokens) ------
#pragma unroll
    for (int b = 0; b < WX; ++b) {
        const int pos = t0 + wt + b * 16 + l16;
        if (pos >= T) continue;
        const int t = DELTA ? da.order[pos] : pos;
#pragma unroll
        for (int G = 0; G < 2; ++G) {
            const int n = n0 + wn + 64 * G + 16 * kg;                // first of this lane's 16 features
            bf16_t* yp = y + (int64_t)t * ldy + n;
            // feature offset 4 q + i is element i of block 4 G + q
            if (n + 16 <= N) {
                uint32_t o[8];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    o[2 * q] = (uint32_t)f32_to_bf16(acc[4 * G + q][b][0]) | ((uint32_t)f32_to_bf16(acc[4 * G + q][b][1]) << 16);
                    o[2 * q + 1] = (uint32_t)f32_to_bf16(acc[4 * G + q][b][2]) | ((uint32_t)f32_to_bf16(acc[4 * G + q][b][3]) << 16);
                }
                *reinterpret_cast<uint4*>(yp) = uint4{o[0], o[1], o[2], o[3]};
                *reinterpret_cast<uint4*>(yp + 8) = uint4{o[4], o[5], o[6], o[7]};
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (n + i < N) yp[i] = f32_to_bf16(acc[4 * G + (i >> 2)][b][i & 3]);
            }
        }
    }
}

// v (sum of its K parts, fp32) -> two bf16 terms hi + lo, rows [t][0][R] and [t][1][R] of vb; one wavefront per token
__global__ __launch_bounds__(256) void v_split_kernel(
    const int32_t* __restrict__ perm, int n_active, const int32_t* __restrict__ token_adapter, const int32_t* __restrict__ rank,
    const float* __restrict__ v, lora_vspec vsp, bf16_t* __restrict__ vb)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_active) return;
    const int t = perm[row];
    const int r = rank[token_adapter[t]];
    for (int j = threadIdx.x & 63; j < r; j += 64) {
        float f = v[(int64_t)t * vsp.R + j];
        for (int q = 1; q < vsp.P; ++q) f += v[q * vsp.part + (int64_t)t * vsp.R + j];
        const bf16_t hi = f32_to_bf16(f);
        vb[(int64_t)t * 2 * vsp.R + j] = hi;
        vb[(int64_t)t * 2 * vsp.R + vsp.R + j] = f32_to_bf16(f - bf16_to_f32(hi));
    }
}

template <int WB, bool DELTA, bool KTAIL>
hipError_t launch_one(int32_t T, int32_t K, int32_t N, const void* x, int64_t ldx, const void* Wt, int64_t ldw,
                      void* y, int64_t ldy, const gemm_delta_args& da, hipStream_t stream)
{
    constexpr int BM = 64 * WB;
    const int tiles_n = (N + BM - 1) / BM, tiles_t = (T + BM - 1) / BM;
    const size_t lds_bytes = (size_t)2 * 2 * BM * 8 * sizeof(uint4) +
                             (DELTA ? META_MAX * sizeof(uint4) + (size_t)(BM * 8 / 256) * 256 * sizeof(int2) : 0);
    static std::atomic<bool> attr_set{false};                 // dynamic LDS above 64 KB has to be allowed once per kernel
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled_kernel<WB, DELTA, KTAIL>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    LORA_LAUNCH(DELTA ? LORA_K_GEMM_TILED_DELTA : LORA_K_GEMM_TILED, (gemm_tiled_kernel<WB, DELTA, KTAIL>),
                dim3(tiles_n * tiles_t), dim3(256), lds_bytes, stream, T, K, N, (const bf16_t*)x, ldx, (const bf16_t*)Wt, ldw,
                (bf16_t*)y, ldy, tiles_n, tiles_t, da);
    return hipGetLastError();
}

template <bool DELTA>
hipError_t launch_ring(int32_t T, int32_t K, int32_t N, const void* x, int64_t ldx, const void* Wt, int64_t ldw,
                       void* y, int64_t ldy, const gemm_delta_args& da, hipStream_t stream)
{
    const int tiles_n = (N + 255) / 256, tiles_t = (T + 255) / 256;
    const size_t lds_bytes = (size_t)RING * RING_STAGE * sizeof(uint4);
    static std::atomic<bool> attr_set{false};                 // dynamic LDS above 64 KB has to be allowed once per kernel
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_ring_kernel<DELTA>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    LORA_LAUNCH(DELTA ? LORA_K_GEMM_RING_DELTA : LORA_K_GEMM_RING, (gemm_ring_kernel<DELTA>),
                dim3(tiles_n * tiles_t), dim3(512), lds_bytes, stream, T, K, N, (const bf16_t*)x, ldx, (const bf16_t*)Wt, ldw,
                (bf16_t*)y, ldy, tiles_n, tiles_t, da);
    return hipGetLastError();
}

}  // namespace

bool gemm_tiled_supported(int32_t T, int32_t K, int32_t N, int32_t dtype, const void* x, int64_t ldx,
                          const void* Wt, int64_t ldw, const void* y, int64_t ldy)
{
    auto mis = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; };
    if (dtype != LORA_BF16 || T < 1 || N < 1) return false;
    if (K % 8 || ldx % 8 || ldw % 8 || ldy % 8) return false;
    if (mis(x) || mis(Wt) || mis(y)) return false;
    const int64_t tiles = (int64_t)((N + 127) / 128) * ((T + 127) / 128);
    return tiles < (1ll << 31);
}

// p != nullptr: fold the adapter delta in; v holds the shrink's output and vb (room for T*2*R bf16) receives its split
// (split_done: the shrink has written it already);
// rm: likewise for the removal of the merged adapter (mixture mode)
hipError_t launch_gemm_tiled(int32_t T, int32_t K, int32_t N, const void* x, int64_t ldx,
                             const void* Wt, int64_t ldw, void* y, int64_t ldy,
                             const lora_plan* p, const lora_dev_tables* d, const float* v, void* vb, bool split_done,
                             const gemm_removal& rm, const void* const* Bt, hipStream_t stream)
{
    // 256 x 256 tiles once there are enough of them to fill the 256 compute units
    const bool big = (int64_t)((N + 255) / 256) * ((T + 255) / 256) >= 192;
    const bool delta = p && (!p->perm.empty() || rm.plan);
    // the ring kernel: whole 32-k stages, at least four of them
    // (the ring kernel's delta part addresses the split of v by 32-bit byte offsets)
    const bool ring_ok = big && K % RK == 0 && K / RK >= 4 &&
                         (!delta || ((int64_t)T * p->R * 4 < (1ll << 32) && (!rm.plan || (int64_t)T * rm.plan->R * 4 < (1ll << 32))));
    gemm_delta_args da{};
    if (delta) {
        // the bf16 split of v, unless the shrink has written it already
        if (!split_done && !p->perm.empty()) {
            LORA_LAUNCH(LORA_K_V_SPLIT, v_split_kernel, dim3((unsigned)(p->perm.size() + 3) / 4), dim3(256), 0, stream,
                        d->perm, (int)p->perm.size(), d->token_adapter, d->rank, v, lora_vspec_of(p), (bf16_t*)vb);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        if (!rm.split_done && rm.plan) {
            LORA_LAUNCH(LORA_K_V_SPLIT, v_split_kernel, dim3((unsigned)(rm.plan->perm.size() + 3) / 4), dim3(256), 0, stream,
                        rm.tables->perm, (int)rm.plan->perm.size(), rm.tables->token_adapter, rm.tables->rank, rm.v,
                        lora_vspec_of(rm.plan), (bf16_t*)rm.vb);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        da = gemm_delta_args{d->order, d->row_key, d->rank,
                             big ? d->extra_ptr256 : d->extra_ptr128,
                             big ? d->extra256 : d->extra128, (const bf16_t*)vb, p->R,
                             (const bf16_t* const*)Bt, (const bf16_t*)d->zeros,
                             (const bf16_t*)rm.vb, rm.plan ? rm.plan->R : 0, rm.plan ? p->merged : -1};
    }
    if (ring_ok)
        return delta ? launch_ring<true>(T, K, N, x, ldx, Wt, ldw, y, ldy, da, stream)
                     : launch_ring<false>(T, K, N, x, ldx, Wt, ldw, y, ldy, da, stream);
    const bool ktail = (K % BK) != 0;
#define GEMM_DISPATCH(WB_, D_, KT_) launch_one<WB_, D_, KT_>(T, K, N, x, ldx, Wt, ldw, y, ldy, da, stream)
    if (big) {
        if (delta) return ktail ? GEMM_DISPATCH(4, true, true) : GEMM_DISPATCH(4, true, false);
        return ktail ? GEMM_DISPATCH(4, false, true) : GEMM_DISPATCH(4, false, false);
    }
    if (delta) return ktail ? GEMM_DISPATCH(2, true, true) : GEMM_DISPATCH(2, true, false);
    return ktail ? GEMM_DISPATCH(2, false, true) : GEMM_DISPATCH(2, false, false);
#undef GEMM_DISPATCH
}

// Base GEMM y = x W (bf16 MFMA, fp32 accumulate) with an optional adapter-delta
// epilogue: y = x W + v B_a per token, v = s_a (x A_a) from the shrink kernel.
//
// This is the base-model product that unmerged inference shares across all
// requests of the batch, with the adapter branches added on top (paper
// sections 1-2); adding the delta to the fp32 accumulators before y is rounded
// makes unmerged inference cost close to merged inference (section 4.4).
//
// x [T,K] and Wt [N,K] are both contraction-index-fastest, so tiles go
// HBM -> registers -> LDS as 16-byte chunks and come back out of LDS as
// ready-made v_mfma_f32_32x32x16_bf16 operands (8 consecutive k per lane).
//
//   workgroup tile 128 features x 128 tokens x 64 k, 4 wavefronts (2 x 2),
//   wavefront tile 64 x 64 = 2 x 2 MFMA blocks of 32 x 32, LDS double buffered.
//
// Lane roles in v_mfma_f32_32x32x16_bf16 (D = A*B + C, A 32x16, B 16x32):
//   lane l supplies A[row l%32][k 8*(l/32) .. +7], B[k 8*(l/32) .. +7][col l%32],
//   receives D[row 8*(i/4) + 4*(l/32) + i%4][col l%32], i = 0..15.
// MFMA rows carry output features, columns carry tokens.  MFMA row 8q+4h+p of a
// block stands for feature 16h + 4q + p, so a lane (h = l/32) ends up with the
// 16 consecutive features 16h .. 16h+15 of its token: 32-byte stores of y.
#include "device_util.h"
#include "kernels.h"
#include "launch.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

union op16 {
    uint4 u;
    bf16x8 v;
};

namespace {

constexpr int BM = 128;   // features per workgroup tile
constexpr int BT = 128;   // tokens per workgroup tile
constexpr int BK = 64;    // k per stage; a tile row is 128 bytes = 8 chunks of 16 bytes

// LDS tile: 128 rows x 8 chunks; chunk c of row r lives at chunk slot c ^ (r & 7)
__device__ __forceinline__ int lds_slot(int row, int chunk) { return row * 8 + (chunk ^ (row & 7)); }

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

template <bool DELTA>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(
    int T, int K, int N, const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ Wt, int64_t ldw,
    bf16_t* __restrict__ y, int64_t ldy, int tiles_n, int tiles_t,
    const int32_t* __restrict__ token_adapter, const int32_t* __restrict__ rank,
    const float* __restrict__ v, lora_vspec vsp, const bf16_t* const* __restrict__ Bt_ptrs)
{
    const int R = vsp.R;
    __shared__ uint4 lds_w[2][BM * 8];
    __shared__ uint4 lds_x[2][BT * 8];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // run of tiles (so its L2 sees neighbouring tiles), walking token tiles
    // fastest inside a band of feature tiles so W panels stay hot.
    const int n_wg = tiles_n * tiles_t;
    int id = blockIdx.x;
    {
        const int per = n_wg / 8, rem = n_wg % 8;
        const int xcd = id & 7, q = id >> 3;
        // XCD k owns per + (k < rem) tiles
        id = xcd * per + (xcd < rem ? xcd : rem) + q;
    }
    const int tile_t = id % tiles_t, tile_n = id / tiles_t;
    const int n0 = tile_n * BM, t0 = tile_t * BT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = (wave & 1) * 64, wt = (wave >> 1) * 64;       // wavefront tile origin inside the workgroup tile

    // global -> register staging: 4 chunks of W and 4 chunks of x per thread and stage
    const bf16_t* gw[4];
    const bf16_t* gx[4];
    int slot[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = tid + i * 256, row = q >> 3, c = q & 7;
        int nr = n0 + row; if (nr >= N) nr = N - 1;
        int tr = t0 + row; if (tr >= T) tr = T - 1;
        gw[i] = Wt + (int64_t)nr * ldw + c * 8;
        gx[i] = x + (int64_t)tr * ldx + c * 8;
        slot[i] = lds_slot(row, c);
    }
    const int c_lane8 = (tid & 7) * 8;                           // this thread's k offset inside a stage

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // LDS rows this lane reads as MFMA operands
    const int l32 = lane & 31, h = lane >> 5;
    // feature of MFMA row l32 = 8q + 4hh + p  ->  16 hh + 4 q + p
    const int frow = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);

    const int stages = (K + BK - 1) / BK;
    uint4 rw[4], rx[4];
    auto load_stage = [&](int s) {
        const int k = s * BK;
        const bool in = k + c_lane8 < K;                         // K % 8 == 0: chunk is whole or absent
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            rw[i] = in ? *reinterpret_cast<const uint4*>(gw[i] + k) : uint4{0, 0, 0, 0};
            rx[i] = in ? *reinterpret_cast<const uint4*>(gx[i] + k) : uint4{0, 0, 0, 0};
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lds_w[buf][slot[i]] = rw[i];
            lds_x[buf][slot[i]] = rx[i];
        }
    };

    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < stages) load_stage(s + 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {                          // 4 MFMA k-steps of 16 per stage
            op16 wa[2], xb[2];
            const int c = ks * 2 + h;
#pragma unroll
            for (int a = 0; a < 2; ++a) wa[a].u = lds_w[buf][lds_slot(wn + a * 32 + frow, c)];
#pragma unroll
            for (int b = 0; b < 2; ++b) xb[b].u = lds_x[buf][lds_slot(wt + b * 32 + l32, c)];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[a].v, xb[b].v, acc[a][b], 0, 0, 0);
        }
        if (s + 1 < stages) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: adapter delta, rounding, store -------------------------
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int t = t0 + wt + b * 32 + l32;                    // this lane's token in column block b
        const bool t_ok = t < T;
        if constexpr (DELTA) {
            const int my_a = t_ok ? token_adapter[t] : -1;
            // adapters present in this 32-token column block, one pass each
            unsigned long long todo = __ballot(my_a >= 0) & 0xffffffffull;   // lanes 0..31 and 32..63 hold the same tokens
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const int a_id = __shfl(my_a, leader, 64);
                const unsigned long long same = __ballot(my_a == a_id) & 0xffffffffull;
                todo &= ~same;
                const int r = rank[a_id];
                const bf16_t* Bt = Bt_ptrs[a_id];
                const bool mine = my_a == a_id;
                for (int j0 = 0; j0 < r; j0 += 16) {
                    const int j = j0 + 8 * h;
                    op16 vhi, vlo;
                    float f[8];
                    if (mine && j < r) {
                        const float4 p0 = *reinterpret_cast<const float4*>(v + (int64_t)t * R + j);
                        const float4 p1 = *reinterpret_cast<const float4*>(v + (int64_t)t * R + j + 4);
                        f[0] = p0.x; f[1] = p0.y; f[2] = p0.z; f[3] = p0.w; f[4] = p1.x; f[5] = p1.y; f[6] = p1.z; f[7] = p1.w;
                        for (int q = 1; q < vsp.P; ++q) {
                            const float* vq = v + q * vsp.part + (int64_t)t * R + j;
                            const float4 q0 = *reinterpret_cast<const float4*>(vq);
                            const float4 q1 = *reinterpret_cast<const float4*>(vq + 4);
                            f[0] += q0.x; f[1] += q0.y; f[2] += q0.z; f[3] += q0.w; f[4] += q1.x; f[5] += q1.y; f[6] += q1.z; f[7] += q1.w;
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i) f[i] = 0.f;
                    }
                    split_bf16(f, vhi, vlo);
#pragma unroll
                    for (int a = 0; a < 2; ++a) {
                        int n = n0 + wn + a * 32 + frow;
                        op16 bo;
                        bo.u = (n < N && j < r) ? *reinterpret_cast<const uint4*>(Bt + (int64_t)n * r + j) : uint4{0, 0, 0, 0};
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bo.v, vhi.v, acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bo.v, vlo.v, acc[a][b], 0, 0, 0);
                    }
                }
            }
        }
        if (!t_ok) continue;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
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

}  // namespace

bool gemm_tiled_supported(int32_t T, int32_t K, int32_t N, int32_t dtype, const void* x, int64_t ldx,
                          const void* Wt, int64_t ldw, const void* y, int64_t ldy)
{
    auto mis = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; };
    if (dtype != LORA_BF16 || T < 1 || N < 1) return false;
    if (K % 8 || ldx % 8 || ldw % 8 || ldy % 8) return false;
    if (mis(x) || mis(Wt) || mis(y)) return false;
    const int64_t tiles = (int64_t)((N + BM - 1) / BM) * ((T + BT - 1) / BT);
    return tiles < (1ll << 31);
}

hipError_t launch_gemm_tiled(int32_t T, int32_t K, int32_t N, const void* x, int64_t ldx,
                             const void* Wt, int64_t ldw, void* y, int64_t ldy,
                             const lora_plan* p, const lora_dev_tables* d, const float* v,
                             const void* const* Bt, hipStream_t stream)
{
    const int tiles_n = (N + BM - 1) / BM, tiles_t = (T + BT - 1) / BT;
    const int grid = tiles_n * tiles_t;
    if (p && !p->perm.empty())
        LORA_LAUNCH(LORA_K_GEMM_TILED_DELTA, (gemm_tiled_kernel<true>), dim3(grid), dim3(256), 0, stream, T, K, N, (const bf16_t*)x, ldx, (const bf16_t*)Wt, ldw,
            (bf16_t*)y, ldy, tiles_n, tiles_t, d->token_adapter, d->rank, v, lora_vspec_of(p), (const bf16_t* const*)Bt);
    else
        LORA_LAUNCH(LORA_K_GEMM_TILED, (gemm_tiled_kernel<false>), dim3(grid), dim3(256), 0, stream, T, K, N, (const bf16_t*)x, ldx, (const bf16_t*)Wt, ldw,
            (bf16_t*)y, ldy, tiles_n, tiles_t, (const int32_t*)nullptr, (const int32_t*)nullptr, (const float*)nullptr, lora_vspec{0, 1, 0},
            (const bf16_t* const*)nullptr);
    return hipGetLastError();
}

// Tiled bf16 shrink / expand kernels for gfx950 (CDNA4), MFMA 16x16x32.
//
// Operator: v = s_a (x A_a),  y = beta y + v B_a  for tokens grouped by adapter
// (paper sections 2, 3.2 and 4.3.1).  What is kept from the paper's kernel
// design: tiles sized per input (the planner's tile list), no padding in
// memory, loads of the next data in flight while the current is consumed.
// What is different here: weights are stored contraction-index-fastest
// ([r,K] and [N,r]), so a 16-byte load per lane *is* the MFMA operand layout
// (8 consecutive k for one row) and no LDS transposition is needed; both
// kernels are bound by HBM, not by the matrix cores, so they are built to keep
// many 16-byte loads in flight per wavefront and to touch each byte of
// x / A / B / y once.
//
// Lane roles in v_mfma_f32_16x16x32_bf16 (D = A*B + C, A 16x32, B 32x16):
//   lane l supplies A[row l%16][k 8*(l/16) .. +7] and B[k 8*(l/16) .. +7][col l%16]
//   and receives D[row 4*(l/16)+i][col l%16], i = 0..3.
#include "device_util.h"
#include "kernels.h"
#include "launch.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

union op16 {            // one 16-byte MFMA operand
    uint4 u;
    bf16x8 v;
};

// 16-byte load from global memory.  Pointers fetched from a pointer table cannot be traced back to a
// kernel argument by the compiler, which would make their loads flat ones (counted as LDS traffic too,
// so that waits on them are coarse); the address space is therefore stated here.
__device__ __forceinline__ uint4 ld16(const bf16_t* p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
    const u32x4 r = *(const __attribute__((address_space(1))) u32x4*)(uintptr_t)p;
    return uint4{r[0], r[1], r[2], r[3]};
#else       // the host pass only parses device functions
    return *reinterpret_cast<const uint4*>(p);
#endif
}
__device__ __forceinline__ uint4 ld16_global(const bf16_t* p) { return ld16(p); }

__device__ __forceinline__ floatx4 mfma(const op16& a, const op16& b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

__device__ __align__(256) uint32_t lora_zero_block[64];       // what masked-out loads read (never written)

// ---------------------------------------------------------------------------
// Shrink.  One workgroup per tile = (16*TB tokens of one adapter) x (16*JB rank
// rows of At_a) x the whole K range.  MFMA rows = rank rows, MFMA columns =
// tokens, so a lane ends up with 4 consecutive rank entries of one token.
// The workgroup's wavefronts take contiguous slices of K; partial sums meet in
// LDS, are scaled by s_a and stored once (deterministic, no atomics).
// PUBLISH: v is stored with agent-scope write-through stores, so that workgroups on other XCDs can
// read it during the same launch without an L2 write-back
// `rows`: token of the tile's row i at rows[i] (perm + tile.row0).  PUBLISH: rows is the padded 16-entry
// table of the single-launch kernel instead, whose address does not depend on the tile descriptor.
template <int TB, int JB, int U, bool PUBLISH = false>
__device__ __forceinline__ void shrink_tile(
    const lora_tile tile, const int32_t* __restrict__ rows,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ At, int K,
    float* __restrict__ v, lora_vspec vsp, floatx4* lds, uint4* patch = nullptr)
{
    // U = k-steps whose loads are issued together before any of them is consumed
    const int R = vsp.R;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int m = lane & 15, g = lane >> 4;

    const bf16_t* xrow[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        int row = tb * 16 + m;
        if (!PUBLISH && row >= tile.nrows) row = 0;     // padding lanes re-read a valid row; never stored
        xrow[tb] = x + (int64_t)rows[row] * ldx + g * 8;
    }
    const bf16_t* arow[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        int j = jb * 16 + m;
        if (j >= tile.cn) j = 0;
        arow[jb] = At + (int64_t)(tile.c0 + j) * K + g * 8;
    }

    // Output element this thread stores first after the reduction (a tile has TB*JB*64
    // float4 slots; threads take slots threadIdx.x, threadIdx.x + blockDim.x, ...).
    // Looked up now: for tiles that fit the workgroup no global load is left between
    // the reduction and the store.  The tile carries s_a.
    const float s_a = __int_as_float(tile.reserved1);
    auto out_slot = [&](int e, int& t_out, int& j_out) {
        t_out = -1;
        j_out = 0;
        if (e < TB * JB * 64) {
            const int l = e & 63, blk = e >> 6;
            const int row = (blk / JB) * 16 + (l & 15);
            const int j = (blk % JB) * 16 + 4 * (l >> 4);
            if (row < tile.nrows && j < tile.cn) {
                t_out = rows[row];
                j_out = tile.c0 + j;
            }
        }
    };
    int out_t, out_j;
    out_slot((int)threadIdx.x, out_t, out_j);

    floatx4 acc[TB][JB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = floatx4{0.f, 0.f, 0.f, 0.f};

    // this tile's K part, then this wavefront's slice of it (in MFMA k-steps of 32)
    const int steps = (K + 31) >> 5;
    const int kpart = (tile.shape >> 8) & 15, kparts = (tile.shape >> 12) & 15;
    const int p_begin = (int)(((int64_t)steps * kpart) / kparts), p_end = (int)(((int64_t)steps * (kpart + 1)) / kparts);
    const int s_begin = p_begin + (int)(((int64_t)(p_end - p_begin) * wave) / W);
    const int s_end = p_begin + (int)(((int64_t)(p_end - p_begin) * (wave + 1)) / W);
    const int kmax = K - g * 8;                          // chunk at offset k is inside the row iff k < kmax

    int s = s_begin;
    // Single-launch decode kernel (16-token tiles, 8 loads of At per round): At is fetched as whole cache
    // lines -- 4 rows x 256 bytes per instruction instead of the MFMA operand shape, 16 rows x 64 bytes,
    // which would ask for half of each line twice; the launch is bound by the CUs' rate of line requests --
    // and reaches the operand layout through a 4 KB LDS patch of the wavefront's own.  A unit of four
    // instructions = 16 rank rows x four k-steps: the two column halves of the round (JB = 1) or the
    // two rank blocks (JB = 2).
    if constexpr (PUBLISH && TB == 1 && JB * U == 8) {
        const bf16_t* zeros = reinterpret_cast<const bf16_t*>(lora_zero_block);
        const int lr = lane >> 4, lc = lane & 15;
        for (; s + U <= s_end; s += U) {
            uint4 raw[8];
            op16 xa[U];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int unit = i >> 2;
                int j = (JB == 2 ? unit * 16 : 0) + 4 * (i & 3) + lr;
                if (j >= tile.cn) j = 0;
                const int k = ((s + (JB == 1 ? 4 * unit : 0)) << 5) + lc * 8;
                raw[i] = ld16(k < K ? At + (int64_t)(tile.c0 + j) * K + k : zeros);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = (s + u) << 5;
                xa[u].u = k < kmax ? ld16(xrow[0] + k) : uint4{0, 0, 0, 0};
            }
#pragma unroll
            for (int unit = 0; unit < 2; ++unit) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int q = 0; q < 4; ++q) patch[(4 * q + lr) * 16 + (lc ^ (4 * q + lr))] = raw[unit * 4 + q];
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    op16 a;
                    a.u = patch[m * 16 + ((4 * t + g) ^ m)];
                    const int jb = JB == 2 ? unit : 0;
                    acc[0][jb] = mfma(a, xa[JB == 1 ? 4 * unit + t : t], acc[0][jb]);
                }
            }
        }
    }
    for (; s + U <= s_end; s += U) {
        op16 xa[U][TB], aa[U][JB];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = (s + u) << 5;
            const bool in = k < kmax;
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) xa[u][tb].u = in ? ld16(xrow[tb] + k) : uint4{0, 0, 0, 0};
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) aa[u][jb].u = in ? ld16(arow[jb] + k) : uint4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = mfma(aa[u][jb], xa[u][tb], acc[tb][jb]);
    }
    for (; s < s_end; ++s) {
        const int k = s << 5;
        const bool in = k < kmax;
        op16 xa[TB], aa[JB];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) xa[tb].u = in ? ld16(xrow[tb] + k) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) aa[jb].u = in ? ld16(arow[jb] + k) : uint4{0, 0, 0, 0};
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) acc[tb][jb] = mfma(aa[jb], xa[tb], acc[tb][jb]);
    }

    // cross-wavefront reduction: lds[(wave*TB*JB + tb*JB + jb)*64 + lane]
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) lds[((wave * TB + tb) * JB + jb) * 64 + lane] = acc[tb][jb];
    __syncthreads();
    for (int e = threadIdx.x; e < TB * JB * 64; e += blockDim.x) {
        if (e != (int)threadIdx.x) out_slot(e, out_t, out_j);
        if (out_t < 0) continue;
        // all partials are fetched before the first add, so the LDS reads overlap
        floatx4 part[16];
#pragma unroll
        for (int w = 0; w < 16; ++w)
            part[w] = (w < W) ? lds[w * TB * JB * 64 + e] : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 8; st > 0; st >>= 1)
#pragma unroll
            for (int w = 0; w < st; ++w) part[w] += part[w + st];
        const float4 o = make_float4(s_a * part[0][0], s_a * part[0][1], s_a * part[0][2], s_a * part[0][3]);
        float* dst = v + kpart * vsp.part + (int64_t)out_t * R + out_j;
        if (PUBLISH) {
            __hip_atomic_store(dst + 0, o.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 1, o.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 2, o.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 3, o.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            *reinterpret_cast<float4*>(dst) = o;
        }
    }
}

extern __shared__ floatx4 shrink_lds[];

// Two builds of the shrink kernel.  "small": up to 16 wavefronts per workgroup,
// tiles of 16 tokens x 16 or 32 rank rows, every wavefront issues 8 (4) k-steps of
// loads at once -- the decode regime, where the whole launch is little more than
// one round of HBM latency.  "big": up to 8 wavefronts, every tile shape.
__global__ __launch_bounds__(1024) void shrink_tiled_small_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm, const float* __restrict__ scale,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* const* __restrict__ At_ptrs, int K,
    float* __restrict__ v, lora_vspec R)
{
    const lora_tile tile = tiles[blockIdx.x];
    const bf16_t* At = At_ptrs[tile.adapter];
    const int jb = (tile.shape >> 4) & 15;
    if (jb == 1) shrink_tile<1, 1, 8>(tile, perm + tile.row0, x, ldx, At, K, v, R, shrink_lds);
    else shrink_tile<1, 2, 4>(tile, perm + tile.row0, x, ldx, At, K, v, R, shrink_lds);
}

__global__ __launch_bounds__(512) void shrink_tiled_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm, const float* __restrict__ scale,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* const* __restrict__ At_ptrs, int K,
    float* __restrict__ v, lora_vspec R)
{
    const lora_tile tile = tiles[blockIdx.x];
    const bf16_t* At = At_ptrs[tile.adapter];
    const int tb = tile.shape & 15, jb = (tile.shape >> 4) & 15;
#define SHRINK_CASE(TB_, JB_, U_) \
    if (tb == TB_ && jb == JB_) { shrink_tile<TB_, JB_, U_>(tile, perm + tile.row0, x, ldx, At, K, v, R, shrink_lds); return; }
    SHRINK_CASE(1, 1, 8)
    SHRINK_CASE(1, 2, 4)
    SHRINK_CASE(1, 3, 4)
    SHRINK_CASE(1, 4, 4)
    SHRINK_CASE(2, 1, 4)
    SHRINK_CASE(2, 2, 4)
    SHRINK_CASE(2, 3, 2)
    SHRINK_CASE(2, 4, 2)
    SHRINK_CASE(4, 1, 4)
    SHRINK_CASE(4, 2, 2)
    SHRINK_CASE(4, 3, 2)
    SHRINK_CASE(4, 4, 2)
#undef SHRINK_CASE
}

// ---------------------------------------------------------------------------
// Streaming shrink for prefill-sized batches.  One workgroup (8 wavefronts) per tile =
// (16*NB tokens of one adapter, NB = 8/KW) x all of the adapter's rank rows x one K part.
// x is private to a wavefront (its 16 tokens).  It is fetched two stages (2 x 128 k) ahead into registers
// with loads that cover whole 128-byte lines (4 rows x 256 bytes per instruction: a CU's rate of line
// requests is what bounds it, and the MFMA operand shape, 16 rows x 64 bytes, would use half of each
// line per request), and is turned into MFMA operands through a 4 KB LDS patch that only this
// wavefront touches (no workgroup barrier involved).  At_a is common to all wavefronts of the tile, so
// every stage's slab At_a[:, 128 k] is fetched once per workgroup and shared through LDS (double
// buffer, XOR swizzle: the 16 lanes of a ds_read_b128 phase hit 16 different 16-byte columns).  With
// fewer than 8 token blocks the wavefronts also split each stage's 4 k-steps KW ways and add up in
// LDS at the end.  No branch inside the stage loop: chunks outside the K part (or K) and padding rows
// read a block of zeros.
template <int JB, int KW>
__device__ __forceinline__ void shrink_stream_tile(
    const lora_tile tile, const int32_t* __restrict__ perm,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ At, int K,
    float* __restrict__ v, lora_vspec vsp, const bf16_t* __restrict__ zeros, uint4* lds)
{
    constexpr int NB = 8 / KW;                    // token blocks of the tile
    constexpr int UW = 4 / KW;                    // k-steps per stage and wavefront
    constexpr int SLAB = JB * 16 * 16;            // 16-byte chunks of one stage's At slab: [16 JB rows][16]
    constexpr int NLD = SLAB >= 512 ? SLAB / 512 : 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int blk = wave % NB, kw = wave / NB;

    // the token whose results this lane ends up with (MFMA column m)
    const int row = blk * 16 + m;
    const bool row_ok = row < tile.nrows;
    const int tok = perm[tile.row0 + (row_ok ? row : 0)];

    // x loads: the wavefront's span of a stage is 64 UW bytes per row = CPR 16-byte chunks.  An instruction
    // takes 128 bytes (LPR = 8 lanes) of 8 rows -- whole cache lines -- so a lane meets only NP = 2 rows
    // (two pointers), H column blocks each; a span of 64 bytes (UW = 1) takes 16 rows x 64 bytes instead.
    constexpr int CPR = 4 * UW;
    constexpr int H = UW >= 2 ? UW / 2 : 1, NP = UW / H;
    constexpr int LPR = UW >= 2 ? 8 : 4, RPI = 64 / LPR;
    const int xl_row = lane / LPR, xl_c = lane % LPR;
    const bf16_t* xsrc[NP];
    int x_ok = 0;
    uint4* xw = lds + 2 * SLAB + wave * (16 * CPR);          // this wavefront's patch: [16 rows][CPR], swizzled
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int r = blk * 16 + p * RPI + xl_row;
        const bool ok = r < tile.nrows;
        x_ok |= (int)ok << p;
        xsrc[p] = x + (int64_t)perm[tile.row0 + (ok ? r : 0)] * ldx + (kw * CPR + xl_c) * 8;
    }
    // instruction i: row group i / H, column block i % H; where its 16 bytes go in the patch
    auto wslot = [&](int i) {
        const int r16 = (i / H) * RPI + xl_row, c = (i % H) * LPR + xl_c;
        return r16 * CPR + (c ^ (r16 % CPR));
    };

    const int steps = (K + 31) >> 5;
    const int kpart = (tile.shape >> 8) & 15, kparts = (tile.shape >> 12) & 15;
    const int p_begin = (int)(((int64_t)steps * kpart) / kparts), p_end = (int)(((int64_t)steps * (kpart + 1)) / kparts);
    const int k_begin = p_begin << 5, k_end = min(K, p_end << 5);
    const int n_stages = (p_end - p_begin + 3) >> 2;

    // At staging: chunk q of a slab = row q/16, 16-byte column q%16; thread's unit i is row j0 + 32 i, same column
    const int a_q = tid % SLAB, a_j0 = a_q >> 4, a_c = a_q & 15;
    const bf16_t* a_base = At + (int64_t)tile.c0 * K + a_c * 8;
    const int a_slot0 = a_j0 * 16 + (a_c ^ (a_j0 & 15));       // rows 32 apart share the swizzle
    auto load_a = [&](int s, uint4 (&ra)[NLD]) {
        const int k0 = k_begin + s * 128;
        const bool in = k0 + a_c * 8 < k_end;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int j = a_j0 + 32 * i;
            ra[i] = ld16(in ? a_base + (int64_t)(j < tile.cn ? j : 0) * K + k0 : zeros);
        }
    };
    auto load_x1 = [&](int s, int i) {
        const int k0 = k_begin + s * 128 + (i % H) * (LPR * 8);
        return ld16_global((((x_ok >> (i / H)) & 1) && k0 + (kw * CPR + xl_c) * 8 < k_end) ? xsrc[i / H] + k0 : zeros);
    };
    auto store_a = [&](int buf, const uint4 (&ra)[NLD]) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) lds[buf * SLAB + a_slot0 + 32 * 16 * i] = ra[i];
    };
    floatx4 acc[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) acc[jb] = floatx4{0.f, 0.f, 0.f, 0.f};
    // one stage: the stage's x goes through the wavefront's LDS patch (the registers are refilled at once
    // with the same rows of stage s_next, so nearly all x registers are in flight all the time), then per
    // k-step the LDS reads of x and of the slab, and the MFMAs
    auto compute = [&](int buf, op16 (&xr)[UW], int s_next) {
#pragma unroll
        for (int i = 0; i < UW; ++i) xw[wslot(i)] = xr[i].u;
#pragma unroll
        for (int i = 0; i < UW; ++i) xr[i].u = load_x1(s_next, i);
        __builtin_amdgcn_wave_barrier();         // the patch is exchanged between lanes of this wavefront only
#pragma unroll
        for (int i = 0; i < UW; ++i) {
            op16 b;
            b.u = xw[m * CPR + ((4 * i + g) ^ (m % CPR))];
            const int c = (kw * UW + i) * 4 + g;
            // the slab's LDS reads go out four rank blocks at a time, ahead of their MFMAs
            constexpr int JG = JB < 4 ? JB : 4;
#pragma unroll
            for (int j0 = 0; j0 < JB; j0 += JG) {
                op16 a[JG];
#pragma unroll
                for (int jb = 0; jb < JG; ++jb) a[jb].u = lds[buf * SLAB + ((j0 + jb) * 16 + m) * 16 + (c ^ m)];
#pragma unroll
                for (int jb = 0; jb < JG; ++jb) acc[j0 + jb] = mfma(a[jb], b, acc[j0 + jb]);
                if (JB > JG) __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    // x registers: NX stages in flight per wavefront (4 KB each); the widest tiles take fewer so that
    // their register count still lets a second workgroup onto the CU
    constexpr int NX = 2;
    uint4 ra[NLD];
    op16 xr[NX][UW];
    // the loads are issued in the order the stage loop keeps them in flight and consumes them, and the
    // loop has no guard branch, so every wait in it can name exactly the loads it needs
    load_a(0, ra);
#pragma unroll
    for (int i = 0; i < UW; ++i) xr[0][i].u = load_x1(0, i);
    store_a(0, ra);
    load_a(1, ra);
#pragma unroll
    for (int u = 1; u < NX; ++u)
#pragma unroll
        for (int i = 0; i < UW; ++i) xr[u][i].u = load_x1(u, i);
    __syncthreads();
    // stage s computes from slab buffer s%2; the slab of stage s+1 goes from its registers to the other
    // buffer after the MFMAs, and the slab after that is requested into them.  Stages past the last one
    // work on zeros.
    int s = 0;
    do {
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            compute(u & 1, xr[u], s + u + NX);
            __builtin_amdgcn_sched_barrier(0);
            store_a((u + 1) & 1, ra);
            load_a(s + u + 2, ra);
            __syncthreads();
        }
        s += NX;
    } while (s < n_stages);

    const float s_a = __int_as_float(tile.reserved1);
    floatx4* red = reinterpret_cast<floatx4*>(lds);
    if (KW > 1) {
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) red[(wave * JB + jb) * 64 + lane] = acc[jb];
        __syncthreads();
        if (kw != 0) return;
#pragma unroll
        for (int q = 1; q < KW; ++q)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) acc[jb] += red[((blk + NB * q) * JB + jb) * 64 + lane];
    }
    if (!row_ok) return;
    float* dst = v + kpart * vsp.part + (int64_t)tok * vsp.R + tile.c0 + 4 * g;
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
        if (jb * 16 + 4 * g < tile.cn)
            *reinterpret_cast<float4*>(dst + jb * 16) =
                make_float4(s_a * acc[jb][0], s_a * acc[jb][1], s_a * acc[jb][2], s_a * acc[jb][3]);
}

extern __shared__ uint4 shrink_stream_lds[];

// JBMAX: the largest rank-block count among the plan's tiles (the kernel's register count is that
// of its widest case, so plans without ranks above 64 get a leaner build)
template <int JBMAX>
__global__ __launch_bounds__(512) void shrink_stream_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* const* __restrict__ At_ptrs, int K,
    float* __restrict__ v, lora_vspec R, const bf16_t* __restrict__ zeros)
{
    const lora_tile tile = tiles[blockIdx.x];
    const bf16_t* At = At_ptrs[tile.adapter];
    const int nb = tile.shape & 15, jb = (tile.shape >> 4) & 15;
#define STREAM_CASE(JB_, KW_) \
    if (JB_ <= JBMAX && jb == JB_ && nb == 8 / KW_) { shrink_stream_tile<JB_, KW_>(tile, perm, x, ldx, At, K, v, R, zeros, shrink_stream_lds); return; }
    STREAM_CASE(4, 1) STREAM_CASE(4, 2) STREAM_CASE(4, 4)
    STREAM_CASE(2, 1) STREAM_CASE(2, 2) STREAM_CASE(2, 4)
    STREAM_CASE(1, 1) STREAM_CASE(1, 2) STREAM_CASE(1, 4)
    STREAM_CASE(8, 1) STREAM_CASE(8, 2) STREAM_CASE(8, 4)
#undef STREAM_CASE
}

hipError_t launch_shrink_tiled(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                               const void* const* At, float* v, hipStream_t stream)
{
    const int n_tiles = (int)p->shrink_tiles.size();
    if (n_tiles == 0) return hipSuccess;
    const int W = p->shrink_waves;
    const size_t lds_bytes = (size_t)W * p->shrink_max_blocks * 64 * sizeof(floatx4);   // <= 64 KB
    if (p->shrink_stream) {
        // two slabs of 16 JB rows x 256 bytes (the final cross-wavefront sum needs the same 8 JB KB), and a
        // 4 KB patch per wavefront
        const size_t stream_lds = (size_t)p->shrink_max_blocks * 8192 + 32768;
#define STREAM_LAUNCH(JBMAX_)                                                                                          \
    LORA_LAUNCH(LORA_K_SHRINK_STREAM, shrink_stream_kernel<JBMAX_>, dim3(n_tiles), dim3(512), stream_lds, stream,      \
                d.shrink_tiles, d.perm, (const bf16_t*)x, ldx, (const bf16_t* const*)At, p->K, v, lora_vspec_of(p),    \
                (const bf16_t*)d.zeros)
        if (p->shrink_max_blocks <= 2) STREAM_LAUNCH(2);
        else if (p->shrink_max_blocks <= 4) STREAM_LAUNCH(4);
        else STREAM_LAUNCH(8);
#undef STREAM_LAUNCH
        return hipGetLastError();
    }
    if (p->shrink_small)
        LORA_LAUNCH(LORA_K_SHRINK_TILED, shrink_tiled_small_kernel, dim3(n_tiles), dim3(64 * W), lds_bytes, stream,
                    d.shrink_tiles, d.perm, d.scale, (const bf16_t*)x, ldx, (const bf16_t* const*)At, p->K, v, lora_vspec_of(p));
    else
        LORA_LAUNCH(LORA_K_SHRINK_TILED, shrink_tiled_kernel, dim3(n_tiles), dim3(64 * W), lds_bytes, stream,
                    d.shrink_tiles, d.perm, d.scale, (const bf16_t*)x, ldx, (const bf16_t* const*)At, p->K, v, lora_vspec_of(p));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Expand.  One workgroup (4 wavefronts) per tile = (16*TB tokens of one adapter)
// x (a range of output features, split evenly over the wavefronts in chunks of
// 64).  MFMA rows = output features (rows of Bt_a), MFMA columns = tokens.  The
// fp32 v operand is split into two bf16 terms (v = hi + lo, error ~2^-16 |v|) so
// the matrix core sees v to fp32-like precision; contraction length is r <= 128.
//
// Within a chunk of 64 features, MFMA row 4q+i of block b stands for feature
// 16q + 4b + i, so after the 4 blocks a lane holds 16 *consecutive* features of
// one token: y is read and written as 32 contiguous bytes per lane.
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

// NP = number of v parts when known at compile time (0: read it from vsp, up to 4)
template <int TB, int KS, bool PREFETCH, int NP>
__device__ __forceinline__ void expand_tile(
    const lora_tile tile, const int32_t* __restrict__ perm, const float* __restrict__ v, lora_vspec vsp,
    const bf16_t* __restrict__ Bt, int r, bf16_t* __restrict__ y, int64_t ldy, int N, float beta)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int R = vsp.R;

    const int chunks = (tile.cn + 63) >> 6;
    const int c_begin = (chunks * wave) >> 2, c_end = (chunks * (wave + 1)) >> 2;
    if (c_begin >= c_end) return;
    const int n_end = tile.c0 + tile.cn;
    // feature row this lane loads for block b of a chunk: base + 16*(m/4) + 4*b + m%4
    const int row_in_chunk = 16 * (m >> 2) + (m & 3);

    int tok[TB];
    bool tok_ok[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int row = tb * 16 + m;
        tok_ok[tb] = row < tile.nrows;
        tok[tb] = perm[tile.row0 + (tok_ok[tb] ? row : 0)];
    }

    auto load_b = [&](int c, op16 (&bop)[4][KS]) {
        const int n_base = tile.c0 + (c << 6);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int n = n_base + row_in_chunk + 4 * b;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int j = s * 32 + g * 8;
                bop[b][s].u = (n < n_end && j < r) ? ld16(Bt + (int64_t)n * r + j) : uint4{0, 0, 0, 0};
            }
        }
    };
    auto load_y = [&](int c, uint4 (&yin)[TB][2]) {
        const int n_lane = tile.c0 + (c << 6) + 16 * g;
        const bool full = n_lane + 16 <= n_end;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if (beta != 0.f && tok_ok[tb] && full) {
                const bf16_t* yp = y + (int64_t)tok[tb] * ldy + n_lane;
                yin[tb][0] = ld16(yp);
                yin[tb][1] = ld16(yp + 8);
            } else {
                yin[tb][0] = uint4{0, 0, 0, 0};
                yin[tb][1] = uint4{0, 0, 0, 0};
            }
        }
    };

    // The loads that do not depend on v go out first: Bt and y of the first chunk.
    op16 bop[4][KS];
    uint4 yin[TB][2];
    load_b(c_begin, bop);
    load_y(c_begin, yin);

    // v operands (MFMA columns = tokens): lane holds v[token m][32 s + 8 g .. +7],
    // the sum of the P partial sums, split into two bf16 terms
    op16 vhi[TB][KS], vlo[TB][KS];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int j = s * 32 + g * 8;
            constexpr int MP = NP ? NP : 4;
            float4 pa[4], pb[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {                  // all parts are fetched before the first add
                if (q < MP && j < r && q < vsp.P) {
                    const float* vq = v + q * vsp.part + (int64_t)tok[tb] * R + j;
                    pa[q] = *reinterpret_cast<const float4*>(vq);
                    pb[q] = *reinterpret_cast<const float4*>(vq + 4);
                } else {
                    pa[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                    pb[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
            float f[8];
            f[0] = ((pa[0].x + pa[1].x) + pa[2].x) + pa[3].x; f[1] = ((pa[0].y + pa[1].y) + pa[2].y) + pa[3].y;
            f[2] = ((pa[0].z + pa[1].z) + pa[2].z) + pa[3].z; f[3] = ((pa[0].w + pa[1].w) + pa[2].w) + pa[3].w;
            f[4] = ((pb[0].x + pb[1].x) + pb[2].x) + pb[3].x; f[5] = ((pb[0].y + pb[1].y) + pb[2].y) + pb[3].y;
            f[6] = ((pb[0].z + pb[1].z) + pb[2].z) + pb[3].z; f[7] = ((pb[0].w + pb[1].w) + pb[2].w) + pb[3].w;
            split_bf16(f, vhi[tb][s], vlo[tb][s]);
        }
    }

    for (int c = c_begin; c < c_end; ++c) {
        // next chunk's loads are in flight while this chunk is multiplied and stored
        op16 bnext[4][KS];
        uint4 ynext[TB][2];
        const bool more = c + 1 < c_end;
        if (PREFETCH && more) {
            load_b(c + 1, bnext);
            load_y(c + 1, ynext);
        }
        const int n_lane = tile.c0 + (c << 6) + 16 * g;      // first of this lane's 16 features
        const bool full = n_lane + 16 <= n_end;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            floatx4 acc[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    acc[b] = mfma(bop[b][s], vhi[tb][s], acc[b]);
                    acc[b] = mfma(bop[b][s], vlo[tb][s], acc[b]);
                }
            }
            if (!tok_ok[tb]) continue;
            bf16_t* yp = y + (int64_t)tok[tb] * ldy + n_lane;
            if (full) {
                uint32_t out[8];
                const uint32_t* yi = reinterpret_cast<const uint32_t*>(&yin[tb][0]);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    float e0 = acc[q >> 1][(q & 1) * 2], e1 = acc[q >> 1][(q & 1) * 2 + 1];
                    if (beta != 0.f) {
                        e0 = fmaf(beta, bf16_to_f32((bf16_t)(yi[q] & 0xffffu)), e0);
                        e1 = fmaf(beta, bf16_to_f32((bf16_t)(yi[q] >> 16)), e1);
                    }
                    out[q] = (uint32_t)f32_to_bf16(e0) | ((uint32_t)f32_to_bf16(e1) << 16);
                }
                *reinterpret_cast<uint4*>(yp) = uint4{out[0], out[1], out[2], out[3]};
                *reinterpret_cast<uint4*>(yp + 8) = uint4{out[4], out[5], out[6], out[7]};
            } else {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    if (n_lane + q < n_end) {
                        float e = acc[q >> 2][q & 3];
                        if (beta != 0.f) e = fmaf(beta, bf16_to_f32(yp[q]), e);
                        yp[q] = f32_to_bf16(e);
                    }
                }
            }
        }
        if (more) {
            if (PREFETCH) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int s = 0; s < KS; ++s) bop[b][s] = bnext[b][s];
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) { yin[tb][0] = ynext[tb][0]; yin[tb][1] = ynext[tb][1]; }
            } else {
                load_b(c + 1, bop);
                load_y(c + 1, yin);
            }
        }
    }
}

// "small" build: 16-token tiles of ranks <= 64 only (the decode regime); few
// registers, so eight wavefronts fit on a SIMD and the whole launch is resident at once.
template <int NP>
__global__ __launch_bounds__(256) void expand_tiled_small_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm,
    const float* __restrict__ v, lora_vspec R, const bf16_t* const* __restrict__ Bt_ptrs,
    bf16_t* __restrict__ y, int64_t ldy, int N, float beta)
{
    const lora_tile tile = tiles[blockIdx.x];
    const int r = tile.reserved0;                       // the planner stores the adapter's rank here
    const bf16_t* Bt = Bt_ptrs[tile.adapter];
    if (r <= 32) expand_tile<1, 1, false, NP>(tile, perm, v, R, Bt, r, y, ldy, N, beta);
    else expand_tile<1, 2, false, NP>(tile, perm, v, R, Bt, r, y, ldy, N, beta);
}

__global__ __launch_bounds__(256) void expand_tiled_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm,
    const float* __restrict__ v, lora_vspec R, const bf16_t* const* __restrict__ Bt_ptrs,
    bf16_t* __restrict__ y, int64_t ldy, int N, float beta)
{
    const lora_tile tile = tiles[blockIdx.x];
    const int r = tile.reserved0;
    const bf16_t* Bt = Bt_ptrs[tile.adapter];
    const int tb = tile.shape & 15;
    const int ks = (r + 31) >> 5;
#define EXPAND_CASE(TB_, KS_) \
    if (tb == TB_ && ks == KS_) { expand_tile<TB_, KS_, (TB_ * KS_ <= 8), 0>(tile, perm, v, R, Bt, r, y, ldy, N, beta); return; }
    EXPAND_CASE(1, 1)
    EXPAND_CASE(1, 2)
    EXPAND_CASE(1, 3)
    EXPAND_CASE(1, 4)
    EXPAND_CASE(2, 1)
    EXPAND_CASE(2, 2)
    EXPAND_CASE(2, 3)
    EXPAND_CASE(2, 4)
    EXPAND_CASE(4, 1)
    EXPAND_CASE(4, 2)
#undef EXPAND_CASE
}

// ---------------------------------------------------------------------------
// Streaming expand for prefill-sized batches, the mirror image of the streaming shrink.  One
// workgroup (8 wavefronts) per tile = (16*NB tokens of one adapter) x a range of output features,
// walked in stages of 64*FW features.  Wavefront w owns token block w % NB and, inside a stage, the
// 64-feature chunk w / NB (wavefronts with w / NB >= FW idle).  y is private to a wavefront: it is
// read four stages ahead and written back with instructions that cover whole 128-byte lines (8 tokens
// x 64 features); the fp32 MFMA results reach that layout through an LDS patch of the wavefront's
// own.  The stage's rows of Bt_a (64 FW features x r) are common to the tile's wavefronts and are
// shared through LDS (double buffer, swizzled).  v (sum of the K parts, split into two bf16 terms)
// stays in registers for the whole tile.  No branch inside the stage loop: loads outside the tile read
// a block of zeros, stores outside it are masked.
template <int KS, int FW>
__device__ __forceinline__ void expand_stream_tile(
    const lora_tile tile, const int32_t* __restrict__ perm, const float* __restrict__ v, lora_vspec vsp,
    const bf16_t* __restrict__ Bt, int r, bf16_t* __restrict__ y, int64_t ldy, float beta,
    const bf16_t* __restrict__ zeros, uint4* lds)
{
    constexpr int RC = 4 * KS;                    // 16-byte chunks per slab row (32 KS ranks)
    constexpr int SH = KS == 1 ? 2 : (KS == 2 ? 1 : 0);
    constexpr int SLAB = FW * 64 * RC;            // 16-byte chunks of one stage's slab: [64 FW features][RC]
    constexpr int NLD = SLAB >= 512 ? SLAB / 512 : 1;
    constexpr int PROW = 68;                      // floats per patch row: 64 features + 4, rows start 4 banks apart
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int NB = tile.shape & 15;               // 1, 2, 4 or 8
    const int blk = wave & (NB - 1), fw = wave / NB;
    const bool active = fw < FW;
    const int n_end = tile.c0 + tile.cn;
    const int n_stages = (((tile.cn + 63) >> 6) + FW - 1) / FW;

    // v operands (MFMA columns = tokens): lane holds v[token m][32 s + 8 g .. +7]
    op16 vhi[KS], vlo[KS];
    {
        const int row = blk * 16 + m;
        const bool row_ok = active && row < tile.nrows;
        const int tok = perm[tile.row0 + (row_ok ? row : 0)];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int j = s * 32 + g * 8;
            float4 pa[4], pb[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {                  // all parts are fetched before the first add
                if (row_ok && j < r && q < vsp.P) {
                    const float* vq = v + q * vsp.part + (int64_t)tok * vsp.R + j;
                    pa[q] = *reinterpret_cast<const float4*>(vq);
                    pb[q] = *reinterpret_cast<const float4*>(vq + 4);
                } else {
                    pa[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                    pb[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
            float f[8];
            f[0] = ((pa[0].x + pa[1].x) + pa[2].x) + pa[3].x; f[1] = ((pa[0].y + pa[1].y) + pa[2].y) + pa[3].y;
            f[2] = ((pa[0].z + pa[1].z) + pa[2].z) + pa[3].z; f[3] = ((pa[0].w + pa[1].w) + pa[2].w) + pa[3].w;
            f[4] = ((pb[0].x + pb[1].x) + pb[2].x) + pb[3].x; f[5] = ((pb[0].y + pb[1].y) + pb[2].y) + pb[3].y;
            f[6] = ((pb[0].z + pb[1].z) + pb[2].z) + pb[3].z; f[7] = ((pb[0].w + pb[1].w) + pb[2].w) + pb[3].w;
            split_bf16(f, vhi[s], vlo[s]);
        }
    }

    // y: instruction i of a stage covers tokens 8i .. 8i+7 of the block, 128 bytes (64 features) each
    const int yl_row = lane >> 3, yl_c = lane & 7;
    bf16_t* ybase[2];
    int y_ok = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int rr = blk * 16 + 8 * i + yl_row;
        const bool ok = active && rr < tile.nrows;
        y_ok |= (int)ok << i;
        ybase[i] = y + (int64_t)perm[tile.row0 + (ok ? rr : 0)] * ldy + tile.c0 + fw * 64 + yl_c * 8;
    }
    const int y_n0 = tile.c0 + fw * 64 + yl_c * 8;           // first feature of this lane's 8 in stage 0
    auto load_y = [&](int s, int i) {
        const bool ok = ((y_ok >> i) & 1) && y_n0 + s * (FW * 64) < n_end && beta != 0.f;
        return ld16(ok ? ybase[i] + s * (FW * 64) : zeros);
    };

    // slab staging: unit q = feature row (q / RC) of the stage, 16-byte column q % RC
    const bf16_t* bsrc[NLD];
    int bslot[NLD], bfeat[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int q = (tid + i * 512) % SLAB, c = q % RC, f = q / RC;       // f in [0, 64 FW)
        const int f64 = f & 63;
        bfeat[i] = c * 8 < r ? tile.c0 + f : (1 << 30);                    // columns past the rank: never loaded
        bsrc[i] = Bt + (int64_t)(tile.c0 + f) * r + c * 8;
        bslot[i] = f * RC + (c ^ ((4 * (f64 >> 4) + (f64 & 3)) >> SH));
    }
    auto load_b = [&](int s, uint4 (&rb)[NLD]) {
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            rb[i] = ld16(bfeat[i] + s * (FW * 64) < n_end ? bsrc[i] + (int64_t)s * (FW * 64) * r : zeros);
    };
    auto store_b = [&](int buf, const uint4 (&rb)[NLD]) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) lds[buf * SLAB + bslot[i]] = rb[i];
    };

    float* patch = reinterpret_cast<float*>(lds + 2 * SLAB) + wave * (16 * PROW);
    // one stage: MFMA rows = features (row 4q+i of block b stands for feature 16q+4b+i of the chunk, so
    // that a lane ends with 4 x 4 consecutive features of token m), results to the patch, back in the
    // layout of the y loads, y = beta y + delta, rounded once, stored; then the y registers are
    // refilled with stage s_next
    auto stage = [&](int buf, int s, uint4 (&yr)[2]) {
        floatx4 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
            const int f = (active ? fw : 0) * 64 + 16 * (m >> 2) + 4 * b + (m & 3);   // idle wavefronts stay inside the slab
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                op16 a;
                a.u = lds[buf * SLAB + f * RC + ((4 * ks + g) ^ (m >> SH))];
                acc[b] = mfma(a, vhi[ks], acc[b]);
                acc[b] = mfma(a, vlo[ks], acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) *reinterpret_cast<floatx4*>(patch + m * PROW + 16 * g + 4 * b) = acc[b];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float* pr = patch + (8 * i + yl_row) * PROW + yl_c * 8;
            const floatx4 d0 = *reinterpret_cast<const floatx4*>(pr), d1 = *reinterpret_cast<const floatx4*>(pr + 4);
            const uint32_t yi[4] = {yr[i].x, yr[i].y, yr[i].z, yr[i].w};
            uint32_t out[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float e0 = fmaf(beta, bf16_to_f32((bf16_t)(yi[q] & 0xffffu)), q < 2 ? d0[2 * q] : d1[2 * q - 4]);
                const float e1 = fmaf(beta, bf16_to_f32((bf16_t)(yi[q] >> 16)), q < 2 ? d0[2 * q + 1] : d1[2 * q - 3]);
                out[q] = (uint32_t)f32_to_bf16(e0) | ((uint32_t)f32_to_bf16(e1) << 16);
            }
            if (((y_ok >> i) & 1) && y_n0 + s * (FW * 64) < n_end)
                *reinterpret_cast<uint4*>(ybase[i] + s * (FW * 64)) = uint4{out[0], out[1], out[2], out[3]};
            yr[i] = load_y(s + 4, i);
        }
        __builtin_amdgcn_wave_barrier();
    };

    uint4 rb0[NLD], rb1[NLD];
    uint4 yr0[2], yr1[2], yr2[2], yr3[2];
    load_b(0, rb0);
#pragma unroll
    for (int i = 0; i < 2; ++i) yr0[i] = load_y(0, i);
    store_b(0, rb0);
    load_b(1, rb0);
#pragma unroll
    for (int i = 0; i < 2; ++i) yr1[i] = load_y(1, i);
    load_b(2, rb1);
#pragma unroll
    for (int i = 0; i < 2; ++i) yr2[i] = load_y(2, i);
#pragma unroll
    for (int i = 0; i < 2; ++i) yr3[i] = load_y(3, i);
    __syncthreads();
    // stage s multiplies from slab buffer s%2; the slab of stage s+1 (in registers since two stages ago)
    // goes to the other buffer, and the slab of stage s+3 is requested.  Stages past the last one work
    // on zeros and store nothing.
    int s = 0;
    do {
#define EXPAND_STAGE(BUF_, S_, YR_, RB_)                 \
        stage(BUF_, S_, YR_);                            \
        __builtin_amdgcn_sched_barrier(0);               \
        store_b(1 - BUF_, RB_);                          \
        load_b((S_) + 3, RB_);                           \
        __syncthreads();
        EXPAND_STAGE(0, s, yr0, rb0)
        EXPAND_STAGE(1, s + 1, yr1, rb1)
        EXPAND_STAGE(0, s + 2, yr2, rb0)
        EXPAND_STAGE(1, s + 3, yr3, rb1)
#undef EXPAND_STAGE
        s += 4;
    } while (s < n_stages);
}

extern __shared__ uint4 expand_stream_lds[];

// KSMAX: the largest number of 32-rank steps among the plan's adapters (the register count of the
// kernel is that of its widest case)
template <int KSMAX>
__global__ __launch_bounds__(512) void expand_stream_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm,
    const float* __restrict__ v, lora_vspec R, const bf16_t* const* __restrict__ Bt_ptrs,
    bf16_t* __restrict__ y, int64_t ldy, float beta, const bf16_t* __restrict__ zeros)
{
    const lora_tile tile = tiles[blockIdx.x];
    const int r = tile.reserved0;
    const bf16_t* Bt = Bt_ptrs[tile.adapter];
    const int ks = r <= 32 ? 1 : (r <= 64 ? 2 : 4), fw = (tile.shape >> 4) & 15;
#define EXPAND_STREAM_CASE(KS_, FW_) \
    if (KS_ <= KSMAX && ks == KS_ && fw == FW_) { expand_stream_tile<KS_, FW_>(tile, perm, v, R, Bt, r, y, ldy, beta, zeros, expand_stream_lds); return; }
    EXPAND_STREAM_CASE(2, 1) EXPAND_STREAM_CASE(2, 2) EXPAND_STREAM_CASE(2, 4)
    EXPAND_STREAM_CASE(1, 1) EXPAND_STREAM_CASE(1, 2) EXPAND_STREAM_CASE(1, 4) EXPAND_STREAM_CASE(1, 8)
    EXPAND_STREAM_CASE(4, 1) EXPAND_STREAM_CASE(4, 2)
#undef EXPAND_STREAM_CASE
}

// ---------------------------------------------------------------------------
// Mode switch (paper section 4.4.2): Wt_l[n, :] += s * Bt_l[n, :] At_l for every layer l of the model
// in one launch, in place -- a rank-r update that reads and writes every weight once.  It is the
// streaming expand with the roles renamed: rows of Wt_l take the place of the tokens (8 wavefronts x
// 16 rows per workgroup, whole-line loads and stores through the wavefront's LDS patch, four stages
// ahead), Bt_l[n, :] that of v (already bf16: one MFMA term), and At_l that of the shared slab.  At_l
// is stored [r, K], so a stage's slab At_l[:, 64 k] is transposed on its way into LDS (16-byte loads
// along k, 2-byte LDS stores) to the [k][rank] layout the MFMA operand reads with ds_read_b128.
template <int KS>
__global__ __launch_bounds__(512) void merge_stream_kernel(
    int N, int K, int r, float s, bf16_t* const* __restrict__ Wt_ptrs, int64_t ldw,
    const bf16_t* const* __restrict__ At_ptrs, const bf16_t* const* __restrict__ Bt_ptrs,
    int tiles_n, int tiles_k, int stages_per_tile)
{
    const bf16_t* zeros = reinterpret_cast<const bf16_t*>(lora_zero_block);
    constexpr int RC = 4 * KS;
    constexpr int SH = KS == 1 ? 2 : (KS == 2 ? 1 : 0);
    constexpr int SLAB = 64 * RC;                 // 16-byte chunks of one stage's slab: [64 k][RC]
    constexpr int UNITS = 32 * KS * 8;            // 16-byte loads of one stage: [32 KS ranks][8 chunks of 8 k]
    constexpr int NLD = UNITS >= 512 ? UNITS / 512 : 1;
    constexpr int PROW = 68;
    uint4* lds = expand_stream_lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    int id = blockIdx.x;
    const int layer = id / (tiles_n * tiles_k);
    id -= layer * (tiles_n * tiles_k);
    const int tile_k = id / tiles_n, tile_n = id - tile_k * tiles_n;   // neighbours share the At slab
    bf16_t* Wt = Wt_ptrs[layer];
    const bf16_t* At = At_ptrs[layer];
    const bf16_t* Bt = Bt_ptrs[layer];
    const int n0 = tile_n * 128 + wave * 16;
    const int k0 = tile_k * stages_per_tile * 64;
    const int k_end = min(K, k0 + stages_per_tile * 64);
    const int n_stages = (k_end - k0 + 63) >> 6;

    // the rank-side operand (MFMA columns = rows n of Wt): lane holds Bt[n0 + m][32 ks + 8 g .. +7]
    op16 bop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int j = ks * 32 + g * 8;
        bop[ks].u = ld16((n0 + m < N && j < r) ? Bt + (int64_t)(n0 + m) * r + j : zeros);
    }

    // Wt rows: instruction i of a stage covers rows 8i .. 8i+7 of the wavefront's 16, 128 bytes (64 k) each
    const int yl_row = lane >> 3, yl_c = lane & 7;
    bf16_t* wbase[2];
    int w_ok = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int n = n0 + 8 * i + yl_row;
        const bool ok = n < N;
        w_ok |= (int)ok << i;
        wbase[i] = Wt + (int64_t)(ok ? n : 0) * ldw + k0 + yl_c * 8;
    }
    const int w_k0 = k0 + yl_c * 8;
    auto load_w = [&](int st, int i) {
        return ld16((((w_ok >> i) & 1) && w_k0 + st * 64 < k_end) ? wbase[i] + st * 64 : zeros);
    };

    // slab staging: unit q = rank row q / 8, columns 8 (q % 8) .. +7 of the stage
    const bf16_t* asrc[NLD];
    int acol[NLD], adst[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int q = (tid + i * 512) % UNITS, j = q >> 3, cc = q & 7;
        asrc[i] = At + (int64_t)(j < r ? j : 0) * K + k0 + cc * 8;
        acol[i] = j < r ? k0 + cc * 8 : (1 << 30);                     // ranks past r: never loaded
        adst[i] = (j >> 3) | ((j & 7) << 8) | (cc << 16);              // rank chunk, position in it, column chunk
    }
    auto load_a = [&](int st, uint4 (&ra)[NLD]) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) ra[i] = ld16(acol[i] + st * 64 < k_end ? asrc[i] + st * 64 : zeros);
    };
    bf16_t* lds16 = reinterpret_cast<bf16_t*>(lds);
    auto store_a = [&](int buf, const uint4 (&ra)[NLD]) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int c = adst[i] & 255, jj = (adst[i] >> 8) & 255, cc = adst[i] >> 16;
            const uint32_t w[4] = {ra[i].x, ra[i].y, ra[i].z, ra[i].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int f = cc * 8 + e;                                  // column of the stage = slab row
                const int slot = f * RC + (c ^ ((4 * (f >> 4) + (f & 3)) >> SH));
                lds16[(buf * SLAB + slot) * 8 + jj] = (bf16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
            }
        }
    };

    float* patch = reinterpret_cast<float*>(lds + 2 * SLAB) + wave * (16 * PROW);
    auto stage = [&](int buf, int st, uint4 (&wr)[2]) {
        floatx4 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
            const int f = 16 * (m >> 2) + 4 * b + (m & 3);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                op16 a;
                a.u = lds[buf * SLAB + f * RC + ((4 * ks + g) ^ (m >> SH))];
                acc[b] = mfma(a, bop[ks], acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) *reinterpret_cast<floatx4*>(patch + m * PROW + 16 * g + 4 * b) = acc[b];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float* pr = patch + (8 * i + yl_row) * PROW + yl_c * 8;
            const floatx4 d0 = *reinterpret_cast<const floatx4*>(pr), d1 = *reinterpret_cast<const floatx4*>(pr + 4);
            const uint32_t wi[4] = {wr[i].x, wr[i].y, wr[i].z, wr[i].w};
            uint32_t out[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float e0 = fmaf(s, q < 2 ? d0[2 * q] : d1[2 * q - 4], bf16_to_f32((bf16_t)(wi[q] & 0xffffu)));
                const float e1 = fmaf(s, q < 2 ? d0[2 * q + 1] : d1[2 * q - 3], bf16_to_f32((bf16_t)(wi[q] >> 16)));
                out[q] = (uint32_t)f32_to_bf16(e0) | ((uint32_t)f32_to_bf16(e1) << 16);
            }
            if (((w_ok >> i) & 1) && w_k0 + st * 64 < k_end)
                *reinterpret_cast<uint4*>(wbase[i] + st * 64) = uint4{out[0], out[1], out[2], out[3]};
            wr[i] = load_w(st + 4, i);
        }
        __builtin_amdgcn_wave_barrier();
    };

    uint4 ra0[NLD], ra1[NLD];
    uint4 wr0[2], wr1[2], wr2[2], wr3[2];
    load_a(0, ra0);
#pragma unroll
    for (int i = 0; i < 2; ++i) wr0[i] = load_w(0, i);
    store_a(0, ra0);
    load_a(1, ra0);
#pragma unroll
    for (int i = 0; i < 2; ++i) wr1[i] = load_w(1, i);
    load_a(2, ra1);
#pragma unroll
    for (int i = 0; i < 2; ++i) wr2[i] = load_w(2, i);
#pragma unroll
    for (int i = 0; i < 2; ++i) wr3[i] = load_w(3, i);
    __syncthreads();
    int st = 0;
    do {
#define MERGE_STAGE(BUF_, S_, WR_, RA_)                  \
        stage(BUF_, S_, WR_);                            \
        __builtin_amdgcn_sched_barrier(0);               \
        store_a(1 - BUF_, RA_);                          \
        load_a((S_) + 3, RA_);                           \
        __syncthreads();
        MERGE_STAGE(0, st, wr0, ra0)
        MERGE_STAGE(1, st + 1, wr1, ra1)
        MERGE_STAGE(0, st + 2, wr2, ra0)
        MERGE_STAGE(1, st + 3, wr3, ra1)
#undef MERGE_STAGE
        st += 4;
    } while (st < n_stages);
}

hipError_t launch_merge_tiled(int32_t L, int32_t N, int32_t K, int32_t r, float s, void* const* Wt, int64_t ldw,
                              const void* const* At, const void* const* Bt, hipStream_t stream)
{
    // 16 stages (1024 columns) per workgroup, fewer for small models so that the launch still has
    // about two workgroups per CU
    const int tiles_n = (N + 127) / 128;
    int stages = 16;
    while (stages > 4 && (int64_t)L * tiles_n * ((K + stages * 64 - 1) / (stages * 64)) < 512) stages /= 2;
    const int tiles_k = (K + stages * 64 - 1) / (stages * 64);
    const int64_t grid = (int64_t)L * tiles_n * tiles_k;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    // dynamic LDS: two slabs of 64 x 32 KS ranks and the eight patches (above 64 KB for ranks > 64)
#define MERGE_LAUNCH(KS_)                                                                                          \
    do {                                                                                                           \
        constexpr int lds_bytes = 2 * 64 * 4 * KS_ * 16 + 8 * 16 * 68 * 4;                                         \
        static bool attr_set = false;                                                                              \
        if (!attr_set) {                                                                                           \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&merge_stream_kernel<KS_>),           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);             \
            if (e != hipSuccess) return e;                                                                         \
            attr_set = true;                                                                                       \
        }                                                                                                          \
        LORA_LAUNCH(LORA_K_MERGE, merge_stream_kernel<KS_>, dim3((unsigned)grid), dim3(512), (size_t)lds_bytes,    \
                    stream, N, K, r, s, (bf16_t* const*)Wt, ldw, (const bf16_t* const*)At,                         \
                    (const bf16_t* const*)Bt, tiles_n, tiles_k, stages);                                           \
    } while (0)
    if (r <= 32) MERGE_LAUNCH(1);
    else if (r <= 64) MERGE_LAUNCH(2);
    else MERGE_LAUNCH(4);
#undef MERGE_LAUNCH
    return hipGetLastError();
}

hipError_t launch_expand_tiled(const lora_plan* p, const lora_dev_tables& d, const float* v,
                               const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream)
{
    const int n_tiles = (int)p->expand_tiles.size();
    if (n_tiles == 0) return hipSuccess;
    if (p->expand_stream) {
        // dynamic LDS above 64 KB has to be allowed once per kernel (the largest any tile mix needs: 98 KB)
#define EXPAND_STREAM_LAUNCH(KSMAX_)                                                                                    \
    do {                                                                                                                \
        static bool attr_set = false;                                                                                   \
        if (!attr_set) {                                                                                                \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&expand_stream_kernel<KSMAX_>),            \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 65536 + 34816);              \
            if (e != hipSuccess) return e;                                                                              \
            attr_set = true;                                                                                            \
        }                                                                                                               \
        LORA_LAUNCH(LORA_K_EXPAND_STREAM, expand_stream_kernel<KSMAX_>, dim3(n_tiles), dim3(512),                       \
                    (size_t)p->expand_stream_lds, stream, d.expand_tiles, d.perm, v, lora_vspec_of(p),                  \
                    (const bf16_t* const*)Bt, (bf16_t*)y, ldy, beta, (const bf16_t*)d.zeros);                           \
    } while (0)
        if (p->expand_stream_ks <= 1) EXPAND_STREAM_LAUNCH(1);
        else if (p->expand_stream_ks <= 2) EXPAND_STREAM_LAUNCH(2);
        else EXPAND_STREAM_LAUNCH(4);
#undef EXPAND_STREAM_LAUNCH
        return hipGetLastError();
    }
    if (p->expand_small && p->v_parts == 1)
        LORA_LAUNCH(LORA_K_EXPAND_TILED, expand_tiled_small_kernel<1>, dim3(n_tiles), dim3(256), 0, stream,
                    d.expand_tiles, d.perm, v, lora_vspec_of(p), (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N, beta);
    else if (p->expand_small && p->v_parts == 2)
        LORA_LAUNCH(LORA_K_EXPAND_TILED, expand_tiled_small_kernel<2>, dim3(n_tiles), dim3(256), 0, stream,
                    d.expand_tiles, d.perm, v, lora_vspec_of(p), (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N, beta);
    else if (p->expand_small)
        LORA_LAUNCH(LORA_K_EXPAND_TILED, expand_tiled_small_kernel<4>, dim3(n_tiles), dim3(256), 0, stream,
                    d.expand_tiles, d.perm, v, lora_vspec_of(p), (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N, beta);
    else
        LORA_LAUNCH(LORA_K_EXPAND_TILED, expand_tiled_kernel, dim3(n_tiles), dim3(256), 0, stream,
                    d.expand_tiles, d.perm, v, lora_vspec_of(p), (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N, beta);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------
// Decode regime, one launch for both steps.  Blocks [0, S) are shrink tiles
// (4 wavefronts, K split over the plan's P parts), blocks [S, S+E) are expand
// tiles.  An expand block first sends out the loads that do not depend on v
// (Bt and y of its first chunk), then waits until every shrink tile of its
// adapter group has published its part of v, gathers v into LDS and goes on as
// the expand kernel does.  This saves one launch and one round of dependent
// small loads per layer, and the Bt/y traffic overlaps the shrink.
//
// Hand-off: every adapter group g has two 64-bit counters in a 128-byte slot of
// its own, neither ever reset: done[g] counts finished shrink tiles, cons[g]
// finished expand tiles.  The group has need[g] shrink and ncons[g] expand tiles
// per launch, so while a launch runs e = cons[g] / ncons[g] is the number of
// launches completed before it, and its expand tiles wait for
// done[g] >= (e+1) * need[g].  There is no counter shared by all blocks.
// Producers never wait, and blocks are dispatched in index order, so all
// producers are dispatched before the first consumer.  Independently of that the wait is bounded: after spin_limit polls
// an expand block stops waiting and computes its v rows itself from x and At
// (slow, exact), so every wavefront reaches the end of the kernel in any case.
struct lora_sync_slot {          // one per adapter group, 128 bytes
    unsigned long long done;
    unsigned long long cons;
    unsigned long long pad[14];
};

__device__ __forceinline__ unsigned long long ld_agent(const unsigned long long* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent_f(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int KS>
__device__ __forceinline__ void fused_expand_item(
    const lora_tile tile, const int32_t* __restrict__ rows, const float* __restrict__ scale,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ At, int K,
    const float* v, lora_vspec vsp, const bf16_t* __restrict__ Bt, bf16_t* __restrict__ y, int64_t ldy, int N,
    float beta, lora_sync_slot* sync, int spin_limit, int delay, float* vt, int* flag)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int R = vsp.R;
    const int r = tile.reserved0;
    const int group = tile.reserved1;
    const unsigned int need = ((unsigned int)tile.shape >> 8) & 0xfffu;
    const unsigned int ncons = (unsigned int)tile.shape >> 20;
    lora_sync_slot* slot = sync + group;

    const int chunks = (tile.cn + 63) >> 6;
    const int c_begin = (chunks * wave) >> 2, c_end = (chunks * (wave + 1)) >> 2;
    const bool has_work = c_begin < c_end;
    const int n_end = tile.c0 + tile.cn;
    const int row_in_chunk = 16 * (m >> 2) + (m & 3);

    const bool tok_ok = m < tile.nrows;
    const int tok = rows[m];                             // padded table: needs nothing from the descriptor

    auto load_b = [&](int c, op16 (&bop)[4][KS]) {
        const int n_base = tile.c0 + (c << 6);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int n = n_base + row_in_chunk + 4 * b;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int j = s * 32 + g * 8;
                bop[b][s].u = (n < n_end && j < r) ? ld16(Bt + (int64_t)n * r + j) : uint4{0, 0, 0, 0};
            }
        }
    };
    auto load_y = [&](int c, uint4 (&yin)[2]) {
        const int n_lane = tile.c0 + (c << 6) + 16 * g;
        if (beta != 0.f && tok_ok && n_lane + 16 <= n_end) {
            const bf16_t* yp = y + (int64_t)tok * ldy + n_lane;
            yin[0] = ld16(yp);
            yin[1] = ld16(yp + 8);
        } else {
            yin[0] = uint4{0, 0, 0, 0};
            yin[1] = uint4{0, 0, 0, 0};
        }
    };

    // Let the shrink blocks' loads of x and At get ahead in the memory queues: what they
    // fetch is needed first (the expand blocks cannot finish before v exists).
    for (int i = 0; i < delay; ++i) __builtin_amdgcn_s_sleep(16);
    op16 bop[4][KS];
    uint4 yin[2];
    if (has_work) {
        load_b(c_begin, bop);
        load_y(c_begin, yin);
    }

    // ---- wait for the group's shrink tiles (bounded) -----------------------
    if (threadIdx.x == 0) {
        const unsigned long long target = (ld_agent(&slot->cons) / ncons + 1ull) * need;
        int ok = 0;
        for (int it = 0; it <= spin_limit; ++it) {
            if (ld_agent(&slot->done) >= target) { ok = 1; break; }
            __builtin_amdgcn_s_sleep(2);
        }
        *flag = ok;
    }
    __syncthreads();
    const bool published = *flag != 0;
    if (published) {
        // v is read with agent-scope loads, which do not use lines cached before the count was seen
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int row = threadIdx.x >> 4, j4 = (threadIdx.x & 15) * 4;
        if (row < tile.nrows && j4 < r) {
            const int t = rows[row];
            float pv[4][4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {                  // all parts are requested before the first add
                const float* vq = v + q * vsp.part + (int64_t)t * R + j4;
#pragma unroll
                for (int i = 0; i < 4; i += 2) {           // 8-byte agent-scope loads (vq is 16-byte aligned)
                    const unsigned long long two = (q < vsp.P) ? ld_agent(reinterpret_cast<const unsigned long long*>(vq + i)) : 0ull;
                    pv[q][i] = __uint_as_float((unsigned int)two);
                    pv[q][i + 1] = __uint_as_float((unsigned int)(two >> 32));
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) vt[row * 64 + j4 + i] = ((pv[0][i] + pv[1][i]) + pv[2][i]) + pv[3][i];
        }
    } else {
        // the shrink tiles were not seen in time: compute this tile's v rows here
        const float s_a = scale[tile.adapter];
        for (int idx = wave; idx < tile.nrows * r; idx += 4) {
            const int row = idx / r, j = idx - row * r;
            const bf16_t* xr = x + (int64_t)rows[row] * ldx;
            const bf16_t* ar = At + (int64_t)j * K;
            float acc = 0.f;
            for (int k = lane * 8; k < K; k += 512) {
                const uint4 xa = ld16(xr + k), aa = ld16(ar + k);
                const uint32_t* xp = reinterpret_cast<const uint32_t*>(&xa);
                const uint32_t* ap = reinterpret_cast<const uint32_t*>(&aa);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc = fmaf(bf16_to_f32((bf16_t)(xp[q] & 0xffffu)), bf16_to_f32((bf16_t)(ap[q] & 0xffffu)), acc);
                    acc = fmaf(bf16_to_f32((bf16_t)(xp[q] >> 16)), bf16_to_f32((bf16_t)(ap[q] >> 16)), acc);
                }
            }
            acc = wave_sum(acc);
            if (lane == 0) vt[row * 64 + j] = s_a * acc;
        }
    }
    __syncthreads();
    // this tile no longer needs the group's counters: count it as through (also when it
    // recomputed v itself, so that the launch arithmetic above stays exact)
    if (threadIdx.x == 0) __hip_atomic_fetch_add(&slot->cons, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!has_work) return;

    op16 vhi[KS], vlo[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const int j = s * 32 + g * 8;
        float f[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = (tok_ok && j < r) ? vt[m * 64 + j + i] : 0.f;
        split_bf16(f, vhi[s], vlo[s]);
    }

    for (int c = c_begin; c < c_end; ++c) {
        const int n_lane = tile.c0 + (c << 6) + 16 * g;
        const bool full = n_lane + 16 <= n_end;
        floatx4 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                acc[b] = mfma(bop[b][s], vhi[s], acc[b]);
                acc[b] = mfma(bop[b][s], vlo[s], acc[b]);
            }
        }
        if (tok_ok) {
            bf16_t* yp = y + (int64_t)tok * ldy + n_lane;
            if (full) {
                uint32_t out[8];
                const uint32_t* yi = reinterpret_cast<const uint32_t*>(&yin[0]);
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    float e0 = acc[q >> 1][(q & 1) * 2], e1 = acc[q >> 1][(q & 1) * 2 + 1];
                    if (beta != 0.f) {
                        e0 = fmaf(beta, bf16_to_f32((bf16_t)(yi[q] & 0xffffu)), e0);
                        e1 = fmaf(beta, bf16_to_f32((bf16_t)(yi[q] >> 16)), e1);
                    }
                    out[q] = (uint32_t)f32_to_bf16(e0) | ((uint32_t)f32_to_bf16(e1) << 16);
                }
                *reinterpret_cast<uint4*>(yp) = uint4{out[0], out[1], out[2], out[3]};
                *reinterpret_cast<uint4*>(yp + 8) = uint4{out[4], out[5], out[6], out[7]};
            } else {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    if (n_lane + q < n_end) {
                        float e = acc[q >> 2][q & 3];
                        if (beta != 0.f) e = fmaf(beta, bf16_to_f32(yp[q]), e);
                        yp[q] = f32_to_bf16(e);
                    }
                }
            }
        }
        if (c + 1 < c_end) {
            load_b(c + 1, bop);
            load_y(c + 1, yin);
        }
    }
}

// (five wavefronts per SIMD: the whole launch of a decode batch is then resident at once, expand blocks
// included, so none of them starts its chain of loads only after a shrink block has retired)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(5, 5))) void delta_fused_small_kernel(
    const lora_tile* __restrict__ shrink_tiles, int n_shrink, const lora_tile* __restrict__ expand_tiles,
    const int32_t* __restrict__ shrink_rows, const int32_t* __restrict__ expand_rows, const float* __restrict__ scale,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* const* __restrict__ At_ptrs, int K,
    float* v, lora_vspec vsp, const bf16_t* const* __restrict__ Bt_ptrs,
    bf16_t* __restrict__ y, int64_t ldy, int N, float beta, lora_sync_slot* sync, int spin_limit, int delay,
    int n_adapters)
{
    __shared__ floatx4 lds[4 * 2 * 64];      // 8 KB: shrink reduction buffer, or v rows [16][64] of an expand tile
    __shared__ uint4 patches[4 * 256];       // 16 KB: one 4 KB patch per wavefront (whole-line loads -> MFMA operands)
    __shared__ int flag;
    const int b = blockIdx.x;
    // With at most 64 adapters every lane fetches one entry of the pointer table while the tile
    // descriptor is still on its way; the tile's entry is then picked out of the wavefront's registers.
    // The workgroup's chain of dependent loads is descriptor / tokens / pointers -> data.
    const bool table_fits = n_adapters <= 64;
    const int lane_a = min((int)(threadIdx.x & 63), n_adapters - 1);
    auto pick = [&](uint64_t entry, int a) {
        const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)entry, a);
        const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(entry >> 32), a);
        return reinterpret_cast<const bf16_t*>((uint64_t)lo | ((uint64_t)hi << 32));
    };
    if (b < n_shrink) {
        const uint64_t a_entry = table_fits ? reinterpret_cast<uint64_t>(At_ptrs[lane_a]) : 0;
        const lora_tile tile = shrink_tiles[b];
        const bf16_t* At = table_fits ? pick(a_entry, tile.adapter) : At_ptrs[tile.adapter];
        const int32_t* rows = shrink_rows + (int64_t)b * 16;
        const int jb = (tile.shape >> 4) & 15;
        uint4* patch = patches + (threadIdx.x >> 6) * 256;
        if (jb == 1) shrink_tile<1, 1, 8, true>(tile, rows, x, ldx, At, K, v, vsp, lds, patch);
        else shrink_tile<1, 2, 4, true>(tile, rows, x, ldx, At, K, v, vsp, lds, patch);
        // publish: the write-through stores of every thread have completed before the
        // block's count is added (no L2 write-back: that would cost microseconds per block)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0)
            __hip_atomic_fetch_add(&sync[(unsigned int)tile.shape >> 16].done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        const uint64_t b_entry = table_fits ? reinterpret_cast<uint64_t>(Bt_ptrs[lane_a]) : 0;
        const lora_tile tile = expand_tiles[b - n_shrink];
        const bf16_t* Bt = table_fits ? pick(b_entry, tile.adapter) : Bt_ptrs[tile.adapter];
        const bf16_t* At = At_ptrs[tile.adapter];        // only the bounded-wait fallback reads it
        const int32_t* rows = expand_rows + (int64_t)(b - n_shrink) * 16;
        if (tile.reserved0 <= 32)
            fused_expand_item<1>(tile, rows, scale, x, ldx, At, K, v, vsp, Bt, y, ldy, N, beta, sync, spin_limit, delay,
                                 reinterpret_cast<float*>(lds), &flag);
        else
            fused_expand_item<2>(tile, rows, scale, x, ldx, At, K, v, vsp, Bt, y, ldy, N, beta, sync, spin_limit, delay,
                                 reinterpret_cast<float*>(lds), &flag);
    }
}

hipError_t launch_delta_fused_small(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                    const void* const* At, const void* const* Bt, float* v, void* y, int64_t ldy,
                                    float beta, hipStream_t stream)
{
    const int S = (int)p->shrink_tiles.size(), E = (int)p->expand_tiles.size();
    if (S + E == 0) return hipSuccess;
    lora_sync_slot* sync = reinterpret_cast<lora_sync_slot*>(d.sync);
    LORA_LAUNCH(LORA_K_DELTA_FUSED, delta_fused_small_kernel, dim3(S + E), dim3(256), 0, stream,
                d.shrink_tiles, S, d.expand_tiles, d.shrink_rows, d.expand_rows, d.scale, (const bf16_t*)x, ldx,
                (const bf16_t* const*)At, p->K, v, lora_vspec_of(p), (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N, beta,
                sync, p->fused_spin_limit, p->fused_delay, p->n_a);
    return hipGetLastError();
}

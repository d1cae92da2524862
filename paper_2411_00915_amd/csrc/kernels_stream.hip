// Streaming shrink / expand for prefill-sized batches and the mode-switch kernel (bf16, MFMA 16x16x32).
// What is common to the wavefronts of a tile (the adapter matrix) goes through LDS; the big stream (x, y, W)
// stays private to a wavefront, is fetched as whole cache lines several stages ahead, and reaches the MFMA
// operand layout through a small LDS patch of the wavefront's own.
#include <atomic>
#include "mfma_tile.h"
#include "kernels.h"
#include "launch.h"

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
    float* __restrict__ v, lora_vspec vsp, const bf16_t* __restrict__ zeros, uint4* lds, bf16_t* __restrict__ vb)
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
        return ld16_stream((((x_ok >> (i / H)) & 1) && k0 + (kw * CPR + xl_c) * 8 < k_end) ? xsrc[i / H] + k0 : zeros);
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
    // slab registers: two sets (a slab is requested three stages before it is multiplied) except for the
    // widest tiles (one set, two stages), whose register count is the kernel's
    constexpr int NRA = JB < 8 ? 2 : 1;
    uint4 ra[NRA][NLD];
    op16 xr[NX][UW];
    // the loads are issued in the order the stage loop keeps them in flight and consumes them, and the
    // loop has no guard branch, so every wait in it can name exactly the loads it needs
    load_a(0, ra[0]);
#pragma unroll
    for (int i = 0; i < UW; ++i) xr[0][i].u = load_x1(0, i);
    store_a(0, ra[0]);
    load_a(1, ra[0]);
#pragma unroll
    for (int u = 1; u < NX; ++u)
#pragma unroll
        for (int i = 0; i < UW; ++i) xr[u][i].u = load_x1(u, i);
    if constexpr (NRA == 2) load_a(2, ra[1]);
    __syncthreads();
    // stage s computes from slab buffer s%2; the slab of stage s+1 goes from its registers to the other
    // buffer after the MFMAs, and a later slab is requested into them.  Stages past the last one work on
    // zeros.
    int s = 0;
    do {
#pragma unroll
        for (int u = 0; u < NX; ++u) {
            compute(u & 1, xr[u], s + u + NX);
            __builtin_amdgcn_sched_barrier(0);
            store_a((u + 1) & 1, ra[u % NRA]);
            load_a(s + u + 1 + NRA, ra[u % NRA]);
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
    // vb (only when v has a single K part): the same values as two bf16 terms, rows [tok][0][R] and [tok][1][R],
    // what the fused forward's GEMM takes as operands
    bf16_t* dst_hi = vb ? vb + (int64_t)tok * 2 * vsp.R + tile.c0 + 4 * g : nullptr;
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
        if (jb * 16 + 4 * g < tile.cn) {
            const float f[4] = {s_a * acc[jb][0], s_a * acc[jb][1], s_a * acc[jb][2], s_a * acc[jb][3]};
            *reinterpret_cast<float4*>(dst + jb * 16) = make_float4(f[0], f[1], f[2], f[3]);
            if (vb) {
                uint32_t h[4], l[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bf16_t hb = f32_to_bf16(f[i]);
                    h[i] = hb;
                    l[i] = f32_to_bf16(f[i] - bf16_to_f32(hb));
                }
                *reinterpret_cast<uint2*>(dst_hi + jb * 16) = uint2{h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
                *reinterpret_cast<uint2*>(dst_hi + vsp.R + jb * 16) = uint2{l[0] | (l[1] << 16), l[2] | (l[3] << 16)};
            }
        }
}

extern __shared__ uint4 shrink_stream_lds[];

// JBMAX: the largest rank-block count among the plan's tiles (the kernel's register count is that
// of its widest case, so plans without ranks above 64 get a leaner build)
template <int JBMAX>
__global__ __launch_bounds__(512) void shrink_stream_kernel(
    const lora_tile* __restrict__ tiles, const int32_t* __restrict__ perm,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* const* __restrict__ At_ptrs, int K,
    float* __restrict__ v, lora_vspec R, const bf16_t* __restrict__ zeros, bf16_t* __restrict__ vb)
{
    const lora_tile tile = tiles[blockIdx.x];
    const bf16_t* At = At_ptrs[tile.adapter];
    const int nb = tile.shape & 15, jb = (tile.shape >> 4) & 15;
#define STREAM_CASE(JB_, KW_) \
    if (JB_ <= JBMAX && jb == JB_ && nb == 8 / KW_) { shrink_stream_tile<JB_, KW_>(tile, perm, x, ldx, At, K, v, R, zeros, shrink_stream_lds, vb); return; }
    STREAM_CASE(4, 1) STREAM_CASE(4, 2) STREAM_CASE(4, 4)
    STREAM_CASE(2, 1) STREAM_CASE(2, 2) STREAM_CASE(2, 4)
    STREAM_CASE(1, 1) STREAM_CASE(1, 2) STREAM_CASE(1, 4)
    STREAM_CASE(8, 1) STREAM_CASE(8, 2) STREAM_CASE(8, 4)
#undef STREAM_CASE
}

hipError_t launch_shrink_stream(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                const void* const* At, float* v, hipStream_t stream, void* vb, bool* split_done)
{
    const int n_tiles = (int)p->shrink_tiles.size();
    if (p->v_parts != 1) vb = nullptr;            // partial sums: the split is of their sum, a pass of its own
    if (split_done) *split_done = vb != nullptr;
    // two slabs of 16 JB rows x 256 bytes (the final cross-wavefront sum needs the same 8 JB KB), and a
    // 4 KB patch per wavefront
    const size_t stream_lds = (size_t)p->shrink_max_blocks * 8192 + 32768;
#define STREAM_LAUNCH(JBMAX_)                                                                                          \
    LORA_LAUNCH(LORA_K_SHRINK_STREAM, shrink_stream_kernel<JBMAX_>, dim3(n_tiles), dim3(512), stream_lds, stream,      \
                d.shrink_tiles, d.perm, (const bf16_t*)x, ldx, (const bf16_t* const*)At, p->K, v, lora_vspec_of(p),    \
                (const bf16_t*)d.zeros, (bf16_t*)vb)
    if (p->shrink_max_blocks <= 2) STREAM_LAUNCH(2);
    else if (p->shrink_max_blocks <= 4) STREAM_LAUNCH(4);
    else STREAM_LAUNCH(8);
#undef STREAM_LAUNCH
    return hipGetLastError();
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

    // Start of a tile: one chain of dependent loads, descriptor -> tokens -> data.  All three token loads go out
    // together, and everything that hangs on them (v, then the first four stages of y) is requested before any of
    // it is waited for; the first slab of Bt depends on the descriptor alone and goes out first of all.
    const int vrow = blk * 16 + m;
    const bool vrow_ok = active && vrow < tile.nrows;
    const int yl_row = lane >> 3, yl_c = lane & 7;
    int y_ok = 0;
    int tok_v, tok_y[2];
    tok_v = perm[tile.row0 + (vrow_ok ? vrow : 0)];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int rr = blk * 16 + 8 * i + yl_row;
        const bool ok = active && rr < tile.nrows;
        y_ok |= (int)ok << i;
        tok_y[i] = perm[tile.row0 + (ok ? rr : 0)];
    }

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
    uint4 rb0[NLD], rb1[NLD];
    load_b(0, rb1);

    // y: instruction i of a stage covers tokens 8i .. 8i+7 of the block, 128 bytes (64 features) each
    bf16_t* ybase[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) ybase[i] = y + (int64_t)tok_y[i] * ldy + tile.c0 + fw * 64 + yl_c * 8;
    const int y_n0 = tile.c0 + fw * 64 + yl_c * 8;           // first feature of this lane's 8 in stage 0
    auto load_y = [&](int s, int i) {
        const bool ok = ((y_ok >> i) & 1) && y_n0 + s * (FW * 64) < n_end && beta != 0.f;
        return ld16_stream(ok ? ybase[i] + s * (FW * 64) : zeros);
    };
    uint4 yr0[2], yr1[2], yr2[2], yr3[2];

    // v operands (MFMA columns = tokens): lane holds v[token m][32 s + 8 g .. +7] (rows, ranks and parts
    // that do not exist read the block of zeros)
    op16 vhi[KS], vlo[KS];
    {
        const float* zf = reinterpret_cast<const float*>(zeros);
        constexpr int SB = KS;                         // (all steps at once: 128 registers at rank 128, which fit)
#pragma unroll
        for (int s0 = 0; s0 < KS; s0 += SB) {
            float4 pa[SB][4], pb[SB][4];
#pragma unroll
            for (int ss = 0; ss < SB; ++ss) {
                const int j = (s0 + ss) * 32 + g * 8;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float* vq = (vrow_ok && j < r && q < vsp.P) ? v + q * vsp.part + (int64_t)tok_v * vsp.R + j : zf;
                    pa[ss][q] = *reinterpret_cast<const float4*>(vq);
                    pb[ss][q] = *reinterpret_cast<const float4*>(vq + 4);
                }
            }
            if (s0 + SB >= KS) {
                // behind the last of v: loads return in order, so the wait for v does not wait for these, and stage 0
                // starts as soon as its own y has arrived
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 2; ++i) yr0[i] = load_y(0, i);
                load_b(1, rb0);
#pragma unroll
                for (int i = 0; i < 2; ++i) yr1[i] = load_y(1, i);
#pragma unroll
                for (int i = 0; i < 2; ++i) yr2[i] = load_y(2, i);
#pragma unroll
                for (int i = 0; i < 2; ++i) yr3[i] = load_y(3, i);
                __builtin_amdgcn_sched_barrier(0);         // (the compiler would sink them below the wait for v)
            }
#pragma unroll
            for (int ss = 0; ss < SB; ++ss) {
                const float4 (&a)[4] = pa[ss];
                const float4 (&b)[4] = pb[ss];
                float f[8];
                f[0] = ((a[0].x + a[1].x) + a[2].x) + a[3].x; f[1] = ((a[0].y + a[1].y) + a[2].y) + a[3].y;
                f[2] = ((a[0].z + a[1].z) + a[2].z) + a[3].z; f[3] = ((a[0].w + a[1].w) + a[2].w) + a[3].w;
                f[4] = ((b[0].x + b[1].x) + b[2].x) + b[3].x; f[5] = ((b[0].y + b[1].y) + b[2].y) + b[3].y;
                f[6] = ((b[0].z + b[1].z) + b[2].z) + b[3].z; f[7] = ((b[0].w + b[1].w) + b[2].w) + b[3].w;
                split_bf16(f, vhi[s0 + ss], vlo[s0 + ss]);
            }
        }
    }

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
                st16_stream(ybase[i] + s * (FW * 64), uint4{out[0], out[1], out[2], out[3]});
            yr[i] = load_y(s + 4, i);
        }
        __builtin_amdgcn_wave_barrier();
    };

    store_b(0, rb1);
    load_b(2, rb1);
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

hipError_t launch_expand_stream(const lora_plan* p, const lora_dev_tables& d, const float* v,
                                const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream)
{
    const int n_tiles = (int)p->expand_tiles.size();
    // dynamic LDS above 64 KB has to be allowed once per kernel (the largest any tile mix needs: 98 KB)
#define EXPAND_STREAM_LAUNCH(KSMAX_)                                                                                    \
    do {                                                                                                                \
        static std::atomic<bool> attr_set{false};                                                                                   \
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
        return ld16_stream((((w_ok >> i) & 1) && w_k0 + st * 64 < k_end) ? wbase[i] + st * 64 : zeros);
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
                st16_stream(wbase[i] + st * 64, uint4{out[0], out[1], out[2], out[3]});
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
        static std::atomic<bool> attr_set{false};                                                                              \
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

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
// x / A / B / y once.  These are the kernels of decode-shaped batches and small adapter groups (and the
// single-launch decode kernel); prefill-sized batches go to the streaming kernels (kernels_stream.hip).
#include "mfma_tile.h"
#include "kernels.h"
#include "launch.h"

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
// The 16 tokens of a tile of the single-launch kernel: they are fetched through the
// scalar cache (their address depends on the workgroup index alone), not through the compute unit's vector memory
// pipeline, where a late workgroup's small loads queue behind the bulk loads of the workgroups that started
// before it, and parked in the first 16 lanes of a register; operator[] reads one by lane index (which may differ
// per lane).
struct tile_rows16 {
    int by_m;        // token of row (lane & 15)
    // t: the 16 tokens as just loaded from a wavefront-uniform address (one scalar load of 64 bytes, which the
    // caller requests before it waits for anything else).  Call with all lanes active: the per-lane view is
    // read out of lanes 0..15 here, once (a cross-lane read under a mask would return what inactive lanes hold).
    // by_row (may be null): 16 ints of LDS that receive the tokens by row index, for readers after a barrier.
    __device__ __forceinline__ void park(const int (&t)[16], int* by_row)
    {
        int v = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) asm("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(t[q]), "n"(q));
        by_m = __shfl(v, (int)threadIdx.x & 15, 64);
        if (by_row && threadIdx.x < 16) by_row[threadIdx.x] = v;
    }
    // row must be congruent to lane & 15 modulo 16 (the tiles of the single launch have 16 rows)
    __device__ __forceinline__ int operator[](int row) const { return by_m; }
};

template <int TB, int JB, int U, bool PUBLISH = false, typename Rows = const int32_t*>
__device__ __forceinline__ void shrink_tile(
    const lora_tile tile, Rows rows,
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
                raw[i] = ld16_stream(k < K ? At + (int64_t)(tile.c0 + j) * K + k : zeros);   // read once per launch
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
        } else if (out_j + 4 <= tile.c0 + tile.cn) {
            *reinterpret_cast<float4*>(dst) = o;
        } else {                                             // the rank is no multiple of 4: the row ends inside this slot
            const float ov[4] = {o.x, o.y, o.z, o.w};
            for (int i = 0; out_j + i < tile.c0 + tile.cn; ++i) dst[i] = ov[i];
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

hipError_t launch_shrink_tiled(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                               const void* const* At, float* v, hipStream_t stream, void* vb, bool* split_done)
{
    if (split_done) *split_done = false;          // only the streaming kernel writes the split
    const int n_tiles = (int)p->shrink_tiles.size();
    if (n_tiles == 0) return hipSuccess;
    const int W = p->shrink_waves;
    const size_t lds_bytes = (size_t)W * p->shrink_max_blocks * 64 * sizeof(floatx4);   // <= 64 KB
    if (p->shrink_stream) return launch_shrink_stream(p, d, x, ldx, At, v, stream, vb, split_done);
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

hipError_t launch_expand_tiled(const lora_plan* p, const lora_dev_tables& d, const float* v,
                               const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream)
{
    const int n_tiles = (int)p->expand_tiles.size();
    if (n_tiles == 0) return hipSuccess;
    if (p->expand_stream) return launch_expand_stream(p, d, v, Bt, y, ldy, beta, stream);
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
// producers are dispatched before the first consumer.  Independently of that the wait is bounded in time: once
// wait_ticks of the device's constant-rate wall clock have passed, an expand block stops waiting and computes
// its v rows itself from x and At (slow, exact), so every wavefront reaches the end of the kernel in any case.
struct lora_sync_slot {          // one per adapter group, 128 bytes
    unsigned long long done;
    unsigned long long cons;
    unsigned long long pad[14];
};

__device__ __forceinline__ unsigned long long ld_agent(const unsigned long long* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Phase time stamps of the instrumented build of the single-launch kernel (stamps == nullptr in the ordinary one,
// which the compiler then drops): thread 0 of a workgroup writes the device's constant-rate wall clock into
// slot k of the workgroup's record.
__device__ __forceinline__ void stamp(long long* stamps, int k)
{
    if (stamps != nullptr && threadIdx.x == 0) stamps[k] = (long long)wall_clock64();
}

template <int KS>
__device__ __forceinline__ void fused_expand_item(
    const lora_tile tile, const tile_rows16& rows, const float* __restrict__ scale,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* __restrict__ At, int K,
    const float* v, lora_vspec vsp, const bf16_t* __restrict__ Bt, bf16_t* __restrict__ y, int64_t ldy, int N,
    float beta, lora_sync_slot* sync, long long wait_ticks, int delay, float* vt, int* flag, const int* row_tok,
    long long* stamps)
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
                bop[b][s].u = (n < n_end && j < r) ? ld16_stream(Bt + (int64_t)n * r + j) : uint4{0, 0, 0, 0};
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
    stamp(stamps, 2);                                        // first Bt / y loads requested

    // ---- wait for the group's shrink tiles (bounded) -----------------------
    if (threadIdx.x == 0) {
        const unsigned long long target = (ld_agent(&slot->cons) / ncons + 1ull) * need;
        const long long t0 = (long long)wall_clock64();
        int ok = 0;
        for (;;) {
            if (ld_agent(&slot->done) >= target) { ok = 1; break; }
            if ((long long)wall_clock64() - t0 >= wait_ticks) break;       // wait_ticks = 0: one look, no waiting
            __builtin_amdgcn_s_sleep(2);
        }
        *flag = ok;
        if (stamps != nullptr) {
            stamps[3] = (long long)wall_clock64();           // the group's count seen (or the wait given up)
            stamps[7] = ok;
        }
    }
    __syncthreads();
    const bool published = *flag != 0;
    if (published) {
        // Thread 0 saw the count (its load returned before it reached the barrier above), so every producer's
        // v stores had been acknowledged by then.  v is read with agent-scope (sc1) loads, issued after the
        // barrier: they are served by the level the stores were written through to, never by a line this CU
        // or this XCD's L2 cached earlier (v is rewritten every launch).  The fence keeps the compiler from
        // moving them up.
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int row = threadIdx.x >> 4, j4 = (threadIdx.x & 15) * 4;
        if (row < tile.nrows && j4 < r) {
            const int t = row_tok[row];                    // written before the barrier above
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
            const bf16_t* xr = x + (int64_t)row_tok[row] * ldx;
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
    stamp(stamps, 4);                                        // the tile's rows of v are in LDS
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
    if (stamps != nullptr) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        stamp(stamps, 5);                                    // the first wavefront's stores of y acknowledged
    }
}

// (five wavefronts per SIMD: the whole launch of a decode batch is then resident at once, expand blocks
// included, so none of them starts its chain of loads only after a shrink block has retired)
// TRACE: the instrumented build (lora_trace_set): every workgroup leaves time stamps of its phases in trace[8 b ..]
template <bool TRACE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(5, 5))) void delta_fused_small_kernel(
    const lora_tile* __restrict__ shrink_tiles, int n_shrink, const lora_tile* __restrict__ expand_tiles,
    const int32_t* __restrict__ shrink_rows, const int32_t* __restrict__ expand_rows, const float* __restrict__ scale,
    const bf16_t* __restrict__ x, int64_t ldx, const bf16_t* const* __restrict__ At_ptrs, int K,
    float* v, lora_vspec vsp, const bf16_t* const* __restrict__ Bt_ptrs,
    bf16_t* __restrict__ y, int64_t ldy, int N, float beta, lora_sync_slot* sync, long long wait_ticks, int delay,
    int resident, long long* trace)
{
    __shared__ floatx4 lds[4 * 2 * 64];      // 8 KB: shrink reduction buffer, or v rows [16][64] of an expand tile
    __shared__ uint4 patches[4 * 256];       // 16 KB: one 4 KB patch per wavefront (whole-line loads -> MFMA operands)
    __shared__ int flag;
    const int b = blockIdx.x;
    long long* stamps = TRACE ? trace + (int64_t)b * 8 : nullptr;
    stamp(stamps, 0);                                        // start
    if (TRACE && threadIdx.x == 0) {                         // where the workgroup runs: XCD, and the hardware id register
        unsigned int xcc, hw;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        stamps[6] = (long long)(((unsigned long long)(xcc & 15u) << 32) | hw);
    }
    // A workgroup's chain of dependent loads is descriptor / tokens -> adapter pointer -> data, and the first two
    // steps go through the scalar cache: descriptor and tokens at addresses that depend on the workgroup index
    // alone, the pointer at one that depends on the descriptor.  (Fetching tokens and a per-lane copy of the
    // pointer table with vector loads saved the dependent step but put them behind the bulk loads of the compute
    // unit's earlier workgroups: late workgroups then got their own loads out 2 to 3 us after their start.)
    tile_rows16 rows;
    int t16[16];
    const int32_t* rows_src = b < n_shrink ? shrink_rows + (int64_t)b * 16 : expand_rows + (int64_t)(b - n_shrink) * 16;
#pragma unroll
    for (int q = 0; q < 16; ++q) t16[q] = rows_src[q];
    if (b < n_shrink) {
        const lora_tile tile = shrink_tiles[b];
        const bf16_t* At = At_ptrs[tile.adapter];
        rows.park(t16, nullptr);
        stamp(stamps, 1);                                    // descriptor, tokens and adapter pointer have arrived
        const int jb = (tile.shape >> 4) & 15;
        uint4* patch = patches + (threadIdx.x >> 6) * 256;
        if (jb == 1) shrink_tile<1, 1, 8, true, const tile_rows16&>(tile, rows, x, ldx, At, K, v, vsp, lds, patch);
        else shrink_tile<1, 2, 4, true, const tile_rows16&>(tile, rows, x, ldx, At, K, v, vsp, lds, patch);
        // Publish.  v was stored with agent-scope (sc1) stores, which are written through to the level all
        // XCDs share instead of staying in this XCD's L2.  A store's acknowledgement is what takes it off the
        // wavefront's vmcnt counter, so after s_waitcnt vmcnt(0) this thread's part of v is visible to every
        // agent-scope load on the device.  Every storing thread waits that way BEFORE the barrier; only then
        // does thread 0 add the block to its group's count (an agent-scope atomic, performed where those
        // loads are served).  A reader that has seen the count and then issues agent-scope loads of v gets
        // the published values.  (A release fence at agent scope would also write back the whole L2, which
        // holds the expand blocks' y stores: microseconds per block.)
        stamp(stamps, 2);                                    // v stores issued (first wavefront)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        stamp(stamps, 3);                                    // every thread's v stores acknowledged
        if (threadIdx.x == 0)
            __hip_atomic_fetch_add(&sync[(unsigned int)tile.shape >> 16].done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (TRACE) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            stamp(stamps, 4);                                // the count has been added
        }
    } else {
        const lora_tile tile = expand_tiles[b - n_shrink];
        const bf16_t* Bt = Bt_ptrs[tile.adapter];
        const bf16_t* At = At_ptrs[tile.adapter];        // only the bounded-wait fallback reads it
        int* row_tok = reinterpret_cast<int*>(patches);  // an expand workgroup stages nothing through the patches
        rows.park(t16, row_tok);
        stamp(stamps, 1);
        // The head start is for the workgroups that begin together with the shrink tiles.  Workgroups start in index
        // order; one beyond what the device holds at a time begins when an earlier one has ended, microseconds into
        // the launch: it does not wait on top of that.
        if (b >= resident) delay = 0;
        if (tile.reserved0 <= 32)
            fused_expand_item<1>(tile, rows, scale, x, ldx, At, K, v, vsp, Bt, y, ldy, N, beta, sync, wait_ticks, delay,
                                 reinterpret_cast<float*>(lds), &flag, row_tok, stamps);
        else
            fused_expand_item<2>(tile, rows, scale, x, ldx, At, K, v, vsp, Bt, y, ldy, N, beta, sync, wait_ticks, delay,
                                 reinterpret_cast<float*>(lds), &flag, row_tok, stamps);
    }
}

hipError_t launch_delta_fused_small(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                    const void* const* At, const void* const* Bt, float* v, void* y, int64_t ldy,
                                    float beta, hipStream_t stream, long long* trace, size_t trace_bytes)
{
    const int S = (int)p->shrink_tiles.size(), E = (int)p->expand_tiles.size();
    if (S + E == 0) return hipSuccess;
    if (trace != nullptr && trace_bytes < (size_t)(S + E) * 8 * sizeof(long long)) return hipErrorInvalidValue;
    lora_sync_slot* sync = reinterpret_cast<lora_sync_slot*>(d.sync);
    // the bound of the hand-off wait, from microseconds to ticks of the wall clock the kernel reads
    static int wall_khz[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (wall_khz[dev] == 0) {
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) khz = 100000;
        wall_khz[dev] = khz;
    }
    const long long wait_ticks = (long long)p->fused_wait_us * wall_khz[dev] / 1000;
    // workgroups the device holds at a time: five of this kernel's per compute unit (its occupancy attribute)
    static int resident[64] = {0};
    if (resident[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        resident[dev] = 5 * cus;
    }
#define DELTA_FUSED_LAUNCH(TRACE_)                                                                                      \
    LORA_LAUNCH(LORA_K_DELTA_FUSED, delta_fused_small_kernel<TRACE_>, dim3(S + E), dim3(256), 0, stream,               \
                d.shrink_tiles, S, d.expand_tiles, d.shrink_rows, d.expand_rows, d.scale, (const bf16_t*)x, ldx,       \
                (const bf16_t* const*)At, p->K, v, lora_vspec_of(p), (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N,  \
                beta, sync, wait_ticks, p->fused_delay, resident[dev], trace)
    if (trace != nullptr) DELTA_FUSED_LAUNCH(true);
    else DELTA_FUSED_LAUNCH(false);
#undef DELTA_FUSED_LAUNCH
    return hipGetLastError();
}

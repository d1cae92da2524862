// General VALU kernels: any dtype (fp32 / bf16), any rank up to LORA_MAX_RANK,
// no alignment demands.  One workgroup per token; the K-long dot products of
// the shrink are spread over the 64 lanes of a wavefront and finished with a
// wavefront reduction.  They back the fp32 plumbing configuration and every
// layout the tiled kernels do not take.
//
// Operator: v = s_a (x A_a),  y = beta y + v B_a   (paper sections 2, 3.2, 4.3.1).
#include <algorithm>

#include "device_util.h"
#include "kernels.h"
#include "launch.h"

template <typename T>
__global__ __launch_bounds__(256) void shrink_general_kernel(
    const int32_t* __restrict__ perm, const int32_t* __restrict__ token_adapter,
    const int32_t* __restrict__ rank, const float* __restrict__ scale,
    const T* __restrict__ x, int64_t ldx, const T* const* __restrict__ At, int K,
    float* __restrict__ v, lora_vspec vs)
{
    const int R = vs.R;
    const int t = perm[blockIdx.x];
    const int a = token_adapter[t];
    const int r = rank[a];
    const float s = scale[a];
    const T* xt = x + (int64_t)t * ldx;
    const T* A = At[a];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = wave; j < r; j += 4) {
        const T* Aj = A + (int64_t)j * K;
        float acc = 0.f;
        for (int k = lane; k < K; k += 64) acc = fmaf(elem<T>::load(xt + k), elem<T>::load(Aj + k), acc);
        acc = wave_sum(acc);
        if (lane == 0) {
            v[(int64_t)t * R + j] = s * acc;
            for (int p = 1; p < vs.P; ++p) v[p * vs.part + (int64_t)t * R + j] = 0.f;   // this kernel does not split K
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void expand_general_kernel(
    const int32_t* __restrict__ perm, const int32_t* __restrict__ token_adapter,
    const int32_t* __restrict__ rank, const float* __restrict__ v, lora_vspec vsp,
    const T* const* __restrict__ Bt, T* __restrict__ y, int64_t ldy, int N, float beta)
{
    const int R = vsp.R;
    __shared__ float vs[LORA_MAX_RANK];
    const int t = perm[blockIdx.x];
    const int a = token_adapter[t];
    const int r = rank[a];
    for (int j = threadIdx.x; j < r; j += 256) {
        float s = v[(int64_t)t * R + j];
        for (int p = 1; p < vsp.P; ++p) s += v[p * vsp.part + (int64_t)t * R + j];
        vs[j] = s;
    }
    __syncthreads();
    const T* B = Bt[a];
    for (int n = blockIdx.y * 256 + threadIdx.x; n < N; n += gridDim.y * 256) {
        const T* Bn = B + (int64_t)n * r;
        float acc = 0.f;
        for (int j = 0; j < r; ++j) acc = fmaf(vs[j], elem<T>::load(Bn + j), acc);
        T* yp = y + (int64_t)t * ldy + n;
        if (beta != 0.f) acc = fmaf(beta, elem<T>::load(yp), acc);
        elem<T>::store(yp, acc);
    }
}

hipError_t launch_shrink_general(const lora_plan* p, const lora_dev_tables& d, const void* x, int64_t ldx,
                                 const void* const* At, float* v, hipStream_t stream)
{
    const int n_active = (int)p->perm.size();
    if (n_active == 0) return hipSuccess;
    if (p->dtype == LORA_F32)
        LORA_LAUNCH(LORA_K_SHRINK_GENERAL, (shrink_general_kernel<float>), dim3(n_active), dim3(256), 0, stream, d.perm, d.token_adapter, d.rank, d.scale,
            (const float*)x, ldx, (const float* const*)At, p->K, v, lora_vspec_of(p));
    else
        LORA_LAUNCH(LORA_K_SHRINK_GENERAL, (shrink_general_kernel<bf16_t>), dim3(n_active), dim3(256), 0, stream, d.perm, d.token_adapter, d.rank, d.scale,
            (const bf16_t*)x, ldx, (const bf16_t* const*)At, p->K, v, lora_vspec_of(p));
    return hipGetLastError();
}

hipError_t launch_expand_general(const lora_plan* p, const lora_dev_tables& d, const float* v,
                                 const void* const* Bt, void* y, int64_t ldy, float beta, hipStream_t stream)
{
    const int n_active = (int)p->perm.size();
    if (n_active == 0) return hipSuccess;
    // the grid's x extent carries the tokens (up to 2^31-1); y splits N
    dim3 grid(n_active, (unsigned)std::min<int64_t>(((int64_t)p->N + 255) / 256, 64));
    if (p->dtype == LORA_F32)
        LORA_LAUNCH(LORA_K_EXPAND_GENERAL, (expand_general_kernel<float>), grid, dim3(256), 0, stream, d.perm, d.token_adapter, d.rank, v, lora_vspec_of(p),
            (const float* const*)Bt, (float*)y, ldy, p->N, beta);
    else
        LORA_LAUNCH(LORA_K_EXPAND_GENERAL, (expand_general_kernel<bf16_t>), grid, dim3(256), 0, stream, d.perm, d.token_adapter, d.rank, v, lora_vspec_of(p),
            (const bf16_t* const*)Bt, (bf16_t*)y, ldy, p->N, beta);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// General base GEMM  y[t,n] = sum_k x[t,k] Wt[n,k]  (+ adapter delta).
// One 16x16 output tile per workgroup, operands staged through LDS, fp32 FMA.
// Reference-grade: serves fp32 and unaligned shapes.
template <typename T>
__global__ __launch_bounds__(256) void gemm_general_kernel(
    int T_, int K, int N, const T* __restrict__ x, int64_t ldx, const T* __restrict__ Wt, int64_t ldw,
    T* __restrict__ y, int64_t ldy,
    const int32_t* __restrict__ token_adapter, const int32_t* __restrict__ rank,
    const float* __restrict__ v, lora_vspec vsp, const T* const* __restrict__ Bt,
    const int32_t* __restrict__ token_adapter2, const float* __restrict__ v2, lora_vspec vsp2)
{
    __shared__ float xs[16][17];
    __shared__ float ws[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int t = blockIdx.y * 16 + ty;
    const int n = blockIdx.x * 16 + tx;
    float acc = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
        const int tr = blockIdx.y * 16 + ty, kk = k0 + tx;
        xs[ty][tx] = (tr < T_ && kk < K) ? elem<T>::load(x + (int64_t)tr * ldx + kk) : 0.f;
        const int nr = blockIdx.x * 16 + ty;
        ws[ty][tx] = (nr < N && kk < K) ? elem<T>::load(Wt + (int64_t)nr * ldw + kk) : 0.f;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) acc = fmaf(xs[ty][k], ws[tx][k], acc);
        __syncthreads();
    }
    if (t < T_ && n < N) {
        // the token's own branch, then (mixture mode) the removal of the merged adapter: the same sum over the
        // second batch's token -> adapter map and v
        for (int pass = 0; pass < 2; ++pass) {
            const int32_t* ta = pass ? token_adapter2 : token_adapter;
            if (!ta) continue;
            const int a = ta[t];
            if (a < 0) continue;
            const float* vv = pass ? v2 : v;
            const lora_vspec sp = pass ? vsp2 : vsp;
            const int r = rank[a];
            const T* Bn = Bt[a] + (int64_t)n * r;
            float d = 0.f;
            for (int j = 0; j < r; ++j) {
                float vj = vv[(int64_t)t * sp.R + j];
                for (int q = 1; q < sp.P; ++q) vj += vv[q * sp.part + (int64_t)t * sp.R + j];
                d = fmaf(vj, elem<T>::load(Bn + j), d);
            }
            acc += d;
        }
        elem<T>::store(y + (int64_t)t * ldy + n, acc);
    }
}

hipError_t launch_gemm_general(int32_t T, int32_t K, int32_t N, int32_t dtype, const void* x, int64_t ldx,
                               const void* Wt, int64_t ldw, void* y, int64_t ldy,
                               const lora_plan* p, const lora_dev_tables* d, const float* v, const gemm_removal& rm,
                               const void* const* Bt, hipStream_t stream)
{
    if (T == 0) return hipSuccess;
    dim3 grid((N + 15) / 16, (T + 15) / 16);
    const int32_t* ta = p ? d->token_adapter : nullptr;
    const int32_t* rk = p ? d->rank : nullptr;
    const lora_vspec R = p ? lora_vspec_of(p) : lora_vspec{0, 1, 0};
    const int32_t* ta2 = rm.plan ? rm.tables->token_adapter : nullptr;
    const lora_vspec R2 = rm.plan ? lora_vspec_of(rm.plan) : lora_vspec{0, 1, 0};
    if (dtype == LORA_F32)
        LORA_LAUNCH(LORA_K_GEMM_GENERAL, (gemm_general_kernel<float>), grid, dim3(256), 0, stream, T, K, N, (const float*)x, ldx, (const float*)Wt, ldw,
            (float*)y, ldy, ta, rk, v, R, (const float* const*)Bt, ta2, rm.v, R2);
    else
        LORA_LAUNCH(LORA_K_GEMM_GENERAL, (gemm_general_kernel<bf16_t>), grid, dim3(256), 0, stream, T, K, N, (const bf16_t*)x, ldx, (const bf16_t*)Wt, ldw,
            (bf16_t*)y, ldy, ta, rk, v, R, (const bf16_t* const*)Bt, ta2, rm.v, R2);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// General mode switch  Wt_l[n,k] += s sum_j Bt_l[n,j] At_l[j,k]  (any dtype, any alignment, any rank):
// one thread per weight, fp32 accumulation, one rounding at the store.
template <typename T>
__global__ __launch_bounds__(256) void merge_general_kernel(
    int N, int K, int r, float s, T* const* __restrict__ Wt_ptrs, int64_t ldw,
    const T* const* __restrict__ At_ptrs, const T* const* __restrict__ Bt_ptrs)
{
    const int k = blockIdx.x * 256 + threadIdx.x, layer = blockIdx.z;
    if (k >= K) return;
    const T* At = At_ptrs[layer];
    for (int n = blockIdx.y; n < N; n += gridDim.y) {
        const T* Bn = Bt_ptrs[layer] + (int64_t)n * r;
        float d = 0.f;
        for (int j = 0; j < r; ++j) d = fmaf(elem<T>::load(Bn + j), elem<T>::load(At + (int64_t)j * K + k), d);
        T* w = Wt_ptrs[layer] + (int64_t)n * ldw + k;
        elem<T>::store(w, fmaf(s, d, elem<T>::load(w)));
    }
}

hipError_t launch_merge_general(int32_t L, int32_t N, int32_t K, int32_t r, float s, int32_t dtype, void* const* Wt,
                                int64_t ldw, const void* const* At, const void* const* Bt, hipStream_t stream)
{
    dim3 grid((K + 255) / 256, std::min(N, 65535), L);
    if (dtype == LORA_F32)
        LORA_LAUNCH(LORA_K_MERGE, (merge_general_kernel<float>), grid, dim3(256), 0, stream, N, K, r, s,
                    (float* const*)Wt, ldw, (const float* const*)At, (const float* const*)Bt);
    else
        LORA_LAUNCH(LORA_K_MERGE, (merge_general_kernel<bf16_t>), grid, dim3(256), 0, stream, N, K, r, s,
                    (bf16_t* const*)Wt, ldw, (const bf16_t* const*)At, (const bf16_t* const*)Bt);
    return hipGetLastError();
}

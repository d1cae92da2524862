// C-ABI entry points that touch the device: plan upload / destroy and the
// compute calls.  Argument checks happen here, before anything is launched.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <vector>

#include <cmath>

#include "kernels.h"
#include "launch.h"
#include "plan_internal.h"

// ---------------------------------------------------------------------------
// Device array of lora_delta_static (see there): v and the hand-off counters for callers that cannot allocate.
// Every device the library runs on holds its own copy of the array, at its own address, until the process ends.
namespace {
constexpr size_t kStaticSyncBytes = (size_t)LORA_STATIC_MAX_GROUPS * 128;            // one 128-byte slot per adapter group
constexpr size_t kStaticBytes = kStaticSyncBytes + (size_t)LORA_STATIC_V_BYTES;
}
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kMaxDevices] = {nullptr};       // device address of `scratch` on each device (the array's
                                                            // name is only a host-side handle for hipGetSymbolAddress)

// address of the current device's copy of `scratch`; looked up once per device, with that device current
lora_status static_scratch(unsigned char** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORA_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return LORA_ERR_DEVICE;
        }
        g_static_ptr[dev] = static_cast<unsigned char*>(ptr);
    }
    *out = g_static_ptr[dev];
    return LORA_OK;
}
}  // namespace

namespace {

struct cached_buf {
    int device;
    size_t bytes;
    void* dev;
    void* host;
};
std::mutex g_cache_mutex;
std::vector<cached_buf> g_cache;       // released plan tables, reused by later plans
constexpr size_t kCacheMax = 16;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

struct table_layout {
    size_t perm, token_adapter, row_key, rank, scale, shrink_tiles, expand_tiles, sync, sync_bytes, total;
    size_t order, extra_ptr128, extra128, extra_ptr256, extra256, zeros, shrink_rows, expand_rows;
};

table_layout layout_of(const lora_plan* p)
{
    table_layout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.perm = take(p->perm.size() * sizeof(int32_t));
    L.token_adapter = take(p->token_adapter.size() * sizeof(int32_t));
    L.row_key = take(p->row_key.size() * sizeof(int32_t));
    L.rank = take(p->rank.size() * sizeof(int32_t));
    L.scale = take(p->scale.size() * sizeof(float));
    L.shrink_tiles = take(p->shrink_tiles.size() * sizeof(lora_tile));
    L.expand_tiles = take(p->expand_tiles.size() * sizeof(lora_tile));
    L.order = take(p->order.size() * sizeof(int32_t));
    L.extra_ptr128 = take(p->extra_ptr128.size() * sizeof(int32_t));
    L.extra128 = take(p->extra128.size() * sizeof(int32_t));
    L.extra_ptr256 = take(p->extra_ptr256.size() * sizeof(int32_t));
    L.extra256 = take(p->extra256.size() * sizeof(int32_t));
    L.zeros = take(256);
    L.shrink_rows = take(p->shrink_rows.size() * sizeof(int32_t));
    L.expand_rows = take(p->expand_rows.size() * sizeof(int32_t));
    L.sync_bytes = p->fused_ok ? p->group_adapter.size() * 128 : 0;
    L.sync = take(L.sync_bytes);
    L.total = std::max<size_t>(off, 256);
    return L;
}

lora_status ensure_uploaded(lora_plan* p, hipStream_t stream)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return LORA_ERR_DEVICE;
    if (p->d_buf) return p->device == dev ? LORA_OK : LORA_ERR_INVALID_ARG;   // a plan lives on one device
    if (p->unmerge) {                                                         // mixture mode: the removal's tables first
        const lora_status st = ensure_uploaded(p->unmerge, stream);
        if (st != LORA_OK) return st;
    }

    // set-up is also where the address of lora_delta_static's device array is looked up (the first use of a
    // device array makes the runtime place it; the static call itself then finds it resolved)
    unsigned char* static_base = nullptr;
    (void)static_scratch(&static_base);

    const table_layout L = layout_of(p);
    // size classes (powers of two from 4 KiB) so that released buffers fit later plans
    size_t cls = 4096;
    while (cls < L.total) cls <<= 1;
    void* dbuf = nullptr;
    void* hbuf = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        for (size_t i = 0; i < g_cache.size(); ++i) {
            if (g_cache[i].device == dev && g_cache[i].bytes == cls) {
                dbuf = g_cache[i].dev;
                hbuf = g_cache[i].host;
                g_cache.erase(g_cache.begin() + i);
                break;
            }
        }
    }
    if (!dbuf) {
        if (hipMalloc(&dbuf, cls) != hipSuccess) { (void)hipGetLastError(); return LORA_ERR_NOMEM; }
        if (hipHostMalloc(&hbuf, cls, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(dbuf);
            return LORA_ERR_NOMEM;
        }
    }
    char* h = static_cast<char*>(hbuf);
    auto put = [&](size_t off, const void* src, size_t bytes) { if (bytes) std::memcpy(h + off, src, bytes); };
    put(L.perm, p->perm.data(), p->perm.size() * sizeof(int32_t));
    put(L.token_adapter, p->token_adapter.data(), p->token_adapter.size() * sizeof(int32_t));
    put(L.row_key, p->row_key.data(), p->row_key.size() * sizeof(int32_t));
    put(L.rank, p->rank.data(), p->rank.size() * sizeof(int32_t));
    put(L.scale, p->scale.data(), p->scale.size() * sizeof(float));
    put(L.shrink_tiles, p->shrink_tiles.data(), p->shrink_tiles.size() * sizeof(lora_tile));
    put(L.expand_tiles, p->expand_tiles.data(), p->expand_tiles.size() * sizeof(lora_tile));
    put(L.order, p->order.data(), p->order.size() * sizeof(int32_t));
    put(L.extra_ptr128, p->extra_ptr128.data(), p->extra_ptr128.size() * sizeof(int32_t));
    put(L.extra128, p->extra128.data(), p->extra128.size() * sizeof(int32_t));
    put(L.extra_ptr256, p->extra_ptr256.data(), p->extra_ptr256.size() * sizeof(int32_t));
    put(L.extra256, p->extra256.data(), p->extra256.size() * sizeof(int32_t));
    std::memset(h + L.zeros, 0, 256);
    put(L.shrink_rows, p->shrink_rows.data(), p->shrink_rows.size() * sizeof(int32_t));
    put(L.expand_rows, p->expand_rows.data(), p->expand_rows.size() * sizeof(int32_t));
    std::memset(h + L.sync, 0, L.sync_bytes);                    // hand-off counters start at zero
    if (hipMemcpyAsync(dbuf, hbuf, L.total, hipMemcpyHostToDevice, stream) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(dbuf);
        (void)hipHostFree(hbuf);
        return LORA_ERR_DEVICE;
    }
    char* d = static_cast<char*>(dbuf);
    p->device = dev;
    p->d_buf = dbuf;
    p->d_bytes = cls;
    p->h_stage = hbuf;
    p->d_perm = reinterpret_cast<int32_t*>(d + L.perm);
    p->d_token_adapter = reinterpret_cast<int32_t*>(d + L.token_adapter);
    p->d_row_key = reinterpret_cast<int32_t*>(d + L.row_key);
    p->d_rank = reinterpret_cast<int32_t*>(d + L.rank);
    p->d_scale = reinterpret_cast<float*>(d + L.scale);
    p->d_shrink_tiles = reinterpret_cast<lora_tile*>(d + L.shrink_tiles);
    p->d_expand_tiles = reinterpret_cast<lora_tile*>(d + L.expand_tiles);
    p->d_sync = d + L.sync;
    p->d_zeros = d + L.zeros;
    p->d_order = reinterpret_cast<int32_t*>(d + L.order);
    p->d_extra_ptr128 = reinterpret_cast<int32_t*>(d + L.extra_ptr128);
    p->d_extra128 = reinterpret_cast<int32_t*>(d + L.extra128);
    p->d_extra_ptr256 = reinterpret_cast<int32_t*>(d + L.extra_ptr256);
    p->d_extra256 = reinterpret_cast<int32_t*>(d + L.extra256);
    p->d_shrink_rows = reinterpret_cast<int32_t*>(d + L.shrink_rows);
    p->d_expand_rows = reinterpret_cast<int32_t*>(d + L.expand_rows);
    return LORA_OK;
}

lora_dev_tables tables_of(const lora_plan* p)
{
    return lora_dev_tables{p->d_perm, p->d_token_adapter, p->d_row_key, p->d_rank, p->d_scale, p->d_shrink_tiles, p->d_expand_tiles,
                           p->d_sync, p->d_order, p->d_extra_ptr128, p->d_extra128, p->d_extra_ptr256, p->d_extra256, p->d_zeros,
                           p->d_shrink_rows, p->d_expand_rows};
}

size_t elem_bytes(int32_t dtype) { return dtype == LORA_F32 ? 4 : 2; }

// mixture mode: the removal's share of the caller's v
float* removal_v(const lora_plan* p, float* v)
{
    return v ? reinterpret_cast<float*>(reinterpret_cast<char*>(v) + lora_unmerge_v_offset(p)) : nullptr;
}
const float* removal_v(const lora_plan* p, const float* v) { return removal_v(p, const_cast<float*>(v)); }

// layout the tiled kernels need at call time
bool tiled_call_ok(const void* base, int64_t ld) { return !misaligned(base, 16) && ld % 8 == 0; }

}  // namespace

// Releases a plan's device tables (called by lora_plan_destroy, planner.cpp, through lora_plan_device_release).
// Contract: the caller destroys a plan only after the work that uses it has finished.  The tables go back to a
// small cache for later plans.
static void release_device_tables(lora_plan* p)
{
    int cur = -1;
    (void)hipGetDevice(&cur);
    if (cur != p->device) (void)hipSetDevice(p->device);
    bool kept = false;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        if (g_cache.size() < kCacheMax) {
            g_cache.push_back(cached_buf{p->device, p->d_bytes, p->d_buf, p->h_stage});
            kept = true;
        }
    }
    if (!kept) {
        (void)hipFree(p->d_buf);
        (void)hipHostFree(p->h_stage);
    }
    if (cur != p->device && cur >= 0) (void)hipSetDevice(cur);
    p->d_buf = nullptr;
    p->h_stage = nullptr;
}
namespace {
struct install_release { install_release() { lora_plan_device_release = release_device_tables; } } g_install_release;
}

extern "C" lora_status lora_plan_upload(lora_plan* p, void* hip_stream)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    return ensure_uploaded(p, static_cast<hipStream_t>(hip_stream));
}

// The three calls on one plan's own tiles; the entry points below add the second batch of a plan in mixture mode.
// vb / split_done: see launch_shrink_tiled
static lora_status shrink_own(lora_plan* p, const void* x, int64_t ldx,
                              const void* const* d_At_ptrs, float* v, void* hip_stream, void* vb = nullptr,
                              bool* split_done = nullptr)
{
    if (split_done) *split_done = false;
    if (p->perm.empty()) return LORA_OK;                       // no token has an adapter: nothing to do
    if (!x || !d_At_ptrs || !v) return LORA_ERR_INVALID_ARG;
    if (ldx < p->K) return LORA_ERR_INVALID_ARG;
    if (misaligned(x, elem_bytes(p->dtype)) || misaligned(v, 16) || misaligned(d_At_ptrs, 8)) return LORA_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lora_status st = ensure_uploaded(p, stream);
    if (st != LORA_OK) return st;
    const lora_dev_tables d = tables_of(p);
    hipError_t e;
    if ((p->family == LORA_VARIANT_TILED || p->shrink_tiled_only) && tiled_call_ok(x, ldx))
        e = launch_shrink_tiled(p, d, x, ldx, d_At_ptrs, v, stream, vb, split_done);
    else if (p->family == LORA_VARIANT_TILED && p->variant_req == LORA_VARIANT_TILED)
        return LORA_ERR_UNSUPPORTED;                           // tiled kernels were demanded but x is not laid out for them
    else
        e = launch_shrink_general(p, d, x, ldx, d_At_ptrs, v, stream);
    return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

extern "C" lora_status lora_shrink(lora_plan* p, const void* x, int64_t ldx,
                                   const void* const* d_At_ptrs, float* v, void* hip_stream)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    if (p->unmerge) {                                          // mixture mode: the removal's share of v lies behind
        const lora_status st = shrink_own(p->unmerge, x, ldx, d_At_ptrs, removal_v(p, v), hip_stream);
        if (st != LORA_OK) return st;
    }
    return shrink_own(p, x, ldx, d_At_ptrs, v, hip_stream);
}

static lora_status expand_own(lora_plan* p, const float* v, const void* const* d_Bt_ptrs,
                              void* y, int64_t ldy, float beta, void* hip_stream)
{
    if (p->perm.empty()) return LORA_OK;
    if (!v || !d_Bt_ptrs || !y) return LORA_ERR_INVALID_ARG;
    if (ldy < p->N) return LORA_ERR_INVALID_ARG;
    if (misaligned(y, elem_bytes(p->dtype)) || misaligned(v, 16) || misaligned(d_Bt_ptrs, 8)) return LORA_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    lora_status st = ensure_uploaded(p, stream);
    if (st != LORA_OK) return st;
    const lora_dev_tables d = tables_of(p);
    hipError_t e;
    if (p->family == LORA_VARIANT_TILED && tiled_call_ok(y, ldy))
        e = launch_expand_tiled(p, d, v, d_Bt_ptrs, y, ldy, beta, stream);
    else if (p->family == LORA_VARIANT_TILED && p->variant_req == LORA_VARIANT_TILED)
        return LORA_ERR_UNSUPPORTED;
    else
        e = launch_expand_general(p, d, v, d_Bt_ptrs, y, ldy, beta, stream);
    return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

extern "C" lora_status lora_expand(lora_plan* p, const float* v, const void* const* d_Bt_ptrs,
                                   void* y, int64_t ldy, float beta, void* hip_stream)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    if (!(beta == 0.f || beta == 1.f)) return LORA_ERR_INVALID_ARG;
    if (p->unmerge && !p->unmerge->perm.empty()) {
        // mixture mode: the removal reaches every row any branch of this batch touches, so it takes the caller's
        // beta and the tokens' own branches accumulate onto it
        const lora_status st = expand_own(p->unmerge, removal_v(p, v), d_Bt_ptrs, y, ldy, beta, hip_stream);
        if (st != LORA_OK) return st;
        beta = 1.f;
    }
    return expand_own(p, v, d_Bt_ptrs, y, ldy, beta, hip_stream);
}

static lora_status delta_own(lora_plan* p, const void* x, int64_t ldx,
                             const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                             float* v, void* y, int64_t ldy, float beta, void* hip_stream)
{
    if (p->perm.empty()) return LORA_OK;
    if (!x || !d_At_ptrs || !d_Bt_ptrs || !v || !y) return LORA_ERR_INVALID_ARG;
    if (ldx < p->K || ldy < p->N) return LORA_ERR_INVALID_ARG;
    if (p->family == LORA_VARIANT_TILED && p->fused_ok && tiled_call_ok(x, ldx) && tiled_call_ok(y, ldy) &&
        !misaligned(v, 16) && !misaligned(d_At_ptrs, 8) && !misaligned(d_Bt_ptrs, 8)) {
        hipStream_t stream = static_cast<hipStream_t>(hip_stream);
        lora_status st = ensure_uploaded(p, stream);
        if (st != LORA_OK) return st;
        size_t trace_bytes = 0;
        long long* trace = lora_trace_buffer(&trace_bytes);
        const hipError_t e = launch_delta_fused_small(p, tables_of(p), x, ldx, d_At_ptrs, d_Bt_ptrs, v, y, ldy, beta, stream,
                                                      trace, trace_bytes);
        if (e == hipErrorInvalidValue && trace != nullptr) return LORA_ERR_WORKSPACE;   // the trace buffer is too small
        return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
    }
    lora_status st = shrink_own(p, x, ldx, d_At_ptrs, v, hip_stream);
    if (st != LORA_OK) return st;
    return expand_own(p, v, d_Bt_ptrs, y, ldy, beta, hip_stream);
}

extern "C" lora_status lora_delta(lora_plan* p, const void* x, int64_t ldx,
                                  const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                                  float* v, void* y, int64_t ldy, float beta, void* hip_stream)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    if (!(beta == 0.f || beta == 1.f)) return LORA_ERR_INVALID_ARG;
    if (p->unmerge && !p->unmerge->perm.empty()) {             // mixture mode: removal first, see lora_expand
        const lora_status st = delta_own(p->unmerge, x, ldx, d_At_ptrs, d_Bt_ptrs, removal_v(p, v), y, ldy, beta, hip_stream);
        if (st != LORA_OK) return st;
        beta = 1.f;
    }
    return delta_own(p, x, ldx, d_At_ptrs, d_Bt_ptrs, v, y, ldy, beta, hip_stream);
}

extern "C" lora_status lora_base_gemm(int32_t T, int32_t K, int32_t N, int32_t dtype,
                                      const void* x, int64_t ldx, const void* Wt, int64_t ldw,
                                      void* y, int64_t ldy, void* hip_stream)
{
    if (T < 0 || K < 1 || N < 1) return LORA_ERR_INVALID_ARG;
    if (dtype != LORA_F32 && dtype != LORA_BF16) return LORA_ERR_INVALID_ARG;
    if (T == 0) return LORA_OK;
    if (!x || !Wt || !y || ldx < K || ldw < K || ldy < N) return LORA_ERR_INVALID_ARG;
    if ((int64_t)(T + 15) / 16 > 65535) return LORA_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (gemm_tiled_supported(T, K, N, dtype, x, ldx, Wt, ldw, y, ldy))
        e = launch_gemm_tiled(T, K, N, x, ldx, Wt, ldw, y, ldy, nullptr, nullptr, nullptr, nullptr, false, gemm_removal{}, nullptr, stream);
    else
        e = launch_gemm_general(T, K, N, dtype, x, ldx, Wt, ldw, y, ldy, nullptr, nullptr, nullptr, gemm_removal{}, nullptr, stream);
    return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

extern "C" lora_status lora_merge(int32_t L, int32_t N, int32_t K, int32_t r, float scale, int32_t dtype,
                                  int32_t variant, void* const* d_Wt_ptrs, int64_t ldw,
                                  const void* const* d_At_ptrs, const void* const* d_Bt_ptrs, void* hip_stream)
{
    if (L < 0 || N < 1 || K < 1 || r < 0 || r > LORA_MAX_RANK || !std::isfinite(scale)) return LORA_ERR_INVALID_ARG;
    if (dtype != LORA_F32 && dtype != LORA_BF16) return LORA_ERR_INVALID_ARG;
    if (variant < LORA_VARIANT_AUTO || variant > LORA_VARIANT_TILED) return LORA_ERR_INVALID_ARG;
    if (L == 0 || r == 0) return LORA_OK;
    if (!d_Wt_ptrs || !d_At_ptrs || !d_Bt_ptrs || ldw < K) return LORA_ERR_INVALID_ARG;
    if (L > 65535) return LORA_ERR_UNSUPPORTED;
    const bool tiled_ok = dtype == LORA_BF16 && K % 8 == 0 && ldw % 8 == 0 && r % 8 == 0 && r <= 128;
    if (variant == LORA_VARIANT_TILED && !tiled_ok) return LORA_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (tiled_ok && variant != LORA_VARIANT_GENERAL)
        e = launch_merge_tiled(L, N, K, r, scale, d_Wt_ptrs, ldw, d_At_ptrs, d_Bt_ptrs, stream);
    else
        e = launch_merge_general(L, N, K, r, scale, dtype, d_Wt_ptrs, ldw, d_At_ptrs, d_Bt_ptrs, stream);
    return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

extern "C" lora_status lora_fused_forward(lora_plan* p, const void* x, int64_t ldx,
                                          const void* Wt, int64_t ldw,
                                          const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                                          void* y, int64_t ldy,
                                          void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    if (p->T == 0) return LORA_OK;
    if (!x || !Wt || !y || ldx < p->K || ldw < p->K || ldy < p->N) return LORA_ERR_INVALID_ARG;
    if ((int64_t)(p->T + 15) / 16 > 65535) return LORA_ERR_UNSUPPORTED;
    const lora_plan* u = p->unmerge && !p->unmerge->perm.empty() ? p->unmerge : nullptr;
    const bool has_delta = !p->perm.empty() || u;
    if (has_delta) {
        if (!d_At_ptrs || !d_Bt_ptrs) return LORA_ERR_INVALID_ARG;
        size_t need = 0;
        lora_plan_query(p, nullptr, nullptr, &need);
        if (!workspace || workspace_bytes < need || misaligned(workspace, 256)) return LORA_ERR_WORKSPACE;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // workspace: v (own parts, then the removal's), the bf16 split of the own v, the split of the removal's
    float* v = static_cast<float*>(workspace);
    size_t v_bytes = 0;
    lora_plan_query(p, nullptr, &v_bytes, nullptr);
    char* vb = workspace ? static_cast<char*>(workspace) + align_up(v_bytes, 256) : nullptr;
    char* vb2 = vb ? vb + align_up((size_t)p->T * 2 * p->R * 2, 256) : nullptr;
    bool split_done = false, split2_done = false;                // the streaming shrink writes the split of v itself
    if (has_delta) {
        lora_status st = shrink_own(p, x, ldx, d_At_ptrs, v, hip_stream, vb, &split_done);
        if (st == LORA_OK && u) st = shrink_own(p->unmerge, x, ldx, d_At_ptrs, removal_v(p, v), hip_stream, vb2, &split2_done);
        if (st != LORA_OK) return st;
    }
    lora_status st = ensure_uploaded(p, stream);
    if (st != LORA_OK) return st;
    const lora_dev_tables d = tables_of(p);
    lora_dev_tables d2{};
    if (u) d2 = tables_of(u);
    gemm_removal rm{u, u ? &d2 : nullptr, u ? removal_v(p, v) : nullptr, u ? vb2 : nullptr, split2_done};
    hipError_t e;
    if (gemm_tiled_supported(p->T, p->K, p->N, p->dtype, x, ldx, Wt, ldw, y, ldy) &&
        (!has_delta || (int32_t)p->order.size() == p->T))
        e = launch_gemm_tiled(p->T, p->K, p->N, x, ldx, Wt, ldw, y, ldy, p, &d, v, vb, split_done, rm, d_Bt_ptrs, stream);
    else
        e = launch_gemm_general(p->T, p->K, p->N, p->dtype, x, ldx, Wt, ldw, y, ldy, p, &d, v, rm, d_Bt_ptrs, stream);
    return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

// ---------------------------------------------------------------------------
// lora_delta_static: lora_delta for callers that cannot allocate.  What lora_delta keeps in caller- or
// library-allocated device memory beyond its inputs and outputs -- v (the shrink's partial sums) and the hand-off
// counters of the single-launch kernel -- lives in one file-scope device array instead.  Every device the library
// runs on holds its own copy of the array, at its own address, until the process ends.
namespace {
// zero-fill by a kernel (a memset node recorded into a captured graph is not reliable on replay)
__global__ __launch_bounds__(256) void clear_words_kernel(uint4* dst, int n16)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = uint4{0, 0, 0, 0};
}
}  // namespace

extern "C" lora_status lora_delta_static(lora_plan* p, const void* x, int64_t ldx,
                                         const void* const* d_At_ptrs, const void* const* d_Bt_ptrs,
                                         void* y, int64_t ldy, float beta, void* hip_stream)
{
    if (!p) return LORA_ERR_INVALID_ARG;
    if (!(beta == 0.f || beta == 1.f)) return LORA_ERR_INVALID_ARG;
    if (p->unmerge) return LORA_ERR_UNSUPPORTED;               // mixture mode: two batches, use lora_delta
    if (p->perm.empty()) return LORA_OK;
    if (!x || !d_At_ptrs || !d_Bt_ptrs || !y) return LORA_ERR_INVALID_ARG;
    if (ldx < p->K || ldy < p->N) return LORA_ERR_INVALID_ARG;
    size_t v_bytes = 0;
    lora_plan_query(p, nullptr, &v_bytes, nullptr);
    if (v_bytes > (size_t)LORA_STATIC_V_BYTES || p->group_adapter.size() > (size_t)LORA_STATIC_MAX_GROUPS)
        return LORA_ERR_UNSUPPORTED;                           // beyond the static array: use lora_delta
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return LORA_ERR_DEVICE;
    if (!p->d_buf || p->device != dev) return LORA_ERR_INVALID_ARG;   // uploading would allocate: do it at set-up
    unsigned char* base = nullptr;
    lora_status st = static_scratch(&base);
    if (st != LORA_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float* v = reinterpret_cast<float*>(base + kStaticSyncBytes);
    lora_dev_tables d = tables_of(p);
    d.sync = base;
    const bool single = p->family == LORA_VARIANT_TILED && p->fused_ok && tiled_call_ok(x, ldx) && tiled_call_ok(y, ldy) &&
                        !misaligned(d_At_ptrs, 8) && !misaligned(d_Bt_ptrs, 8);
    hipError_t e;
    if (single) {
        // the counters' launch arithmetic assumes one plan per slot: the array is shared by all plans, so they
        // start every call at zero
        const int n16 = (int)(p->group_adapter.size() * 128 / 16);
        LORA_LAUNCH(LORA_K_CLEAR, clear_words_kernel, dim3((n16 + 255) / 256), dim3(256), 0, stream,
                    reinterpret_cast<uint4*>(base), n16);
        if (hipGetLastError() != hipSuccess) return LORA_ERR_DEVICE;
        e = launch_delta_fused_small(p, d, x, ldx, d_At_ptrs, d_Bt_ptrs, v, y, ldy, beta, stream);
        return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
    }
    if (misaligned(x, elem_bytes(p->dtype)) || misaligned(y, elem_bytes(p->dtype)) || misaligned(d_At_ptrs, 8) ||
        misaligned(d_Bt_ptrs, 8))
        return LORA_ERR_INVALID_ARG;
    if (p->family == LORA_VARIANT_TILED && tiled_call_ok(x, ldx) && tiled_call_ok(y, ldy)) {
        e = launch_shrink_tiled(p, d, x, ldx, d_At_ptrs, v, stream);
        if (e == hipSuccess) e = launch_expand_tiled(p, d, v, d_Bt_ptrs, y, ldy, beta, stream);
    } else if (p->family == LORA_VARIANT_TILED && p->variant_req == LORA_VARIANT_TILED) {
        return LORA_ERR_UNSUPPORTED;
    } else {
        // (the same choice of shrink as lora_delta's: tiled also where only the expand is general)
        if (p->shrink_tiled_only && tiled_call_ok(x, ldx)) e = launch_shrink_tiled(p, d, x, ldx, d_At_ptrs, v, stream);
        else e = launch_shrink_general(p, d, x, ldx, d_At_ptrs, v, stream);
        if (e == hipSuccess) e = launch_expand_general(p, d, v, d_Bt_ptrs, y, ldy, beta, stream);
    }
    return e == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

// Per-kernel timing facility behind lora_timing_begin / _end / _read.
#include <cstdint>
#include <mutex>
#include <vector>

#include "../../include/lora_abi.h"
#include "launch.h"

namespace {
struct record { int id; hipEvent_t start, stop; };
std::mutex g_mu;
bool g_on = false;
std::vector<record> g_records;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_free;
struct stats { int64_t count; double total_us, min_us, max_us; };
stats g_stats[LORA_K_COUNT];
const char* kNames[LORA_K_COUNT] = {"shrink_general_kernel", "expand_general_kernel", "shrink_tiled_kernel",
                                    "expand_tiled_kernel", "gemm_general_kernel", "gemm_tiled_kernel",
                                    "gemm_tiled_kernel<delta>", "delta_fused_small_kernel", "v_split_kernel",
                                    "shrink_stream_kernel", "expand_stream_kernel", "merge_kernel",
                                    "gemm_ring_kernel", "gemm_ring_kernel<delta>", "clear_words_kernel", "probe_empty_kernel", "probe_read_kernel", "probe_mfma_kernel"};
long long* g_trace = nullptr;
size_t g_trace_bytes = 0;
}  // namespace

long long* lora_trace_buffer(size_t* bytes)
{
    std::lock_guard<std::mutex> lock(g_mu);
    *bytes = g_trace_bytes;
    return g_trace;
}

extern "C" lora_status lora_trace_set(void* device_buffer, size_t bytes)
{
    if (device_buffer != nullptr && ((reinterpret_cast<uintptr_t>(device_buffer) & 7) != 0 || bytes == 0)) return LORA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mu);
    g_trace = static_cast<long long*>(device_buffer);
    g_trace_bytes = device_buffer ? bytes : 0;
    return LORA_OK;
}

extern "C" int32_t lora_trace_tick_khz(void)
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    return khz > 0 ? khz : 0;
}

bool lora_timing_on() { return g_on; }

bool lora_timing_events(int id, hipEvent_t* start, hipEvent_t* stop)
{
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_on) return false;
    std::pair<hipEvent_t, hipEvent_t> ev;
    if (!g_free.empty()) {
        ev = g_free.back();
        g_free.pop_back();
    } else {
        if (hipEventCreate(&ev.first) != hipSuccess) return false;
        if (hipEventCreate(&ev.second) != hipSuccess) { (void)hipEventDestroy(ev.first); return false; }
    }
    g_records.push_back(record{id, ev.first, ev.second});
    *start = ev.first;
    *stop = ev.second;
    return true;
}

extern "C" lora_status lora_timing_begin(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    for (auto& r : g_records) g_free.emplace_back(r.start, r.stop);
    g_records.clear();
    for (auto& s : g_stats) s = stats{0, 0.0, 0.0, 0.0};
    g_on = true;
    return LORA_OK;
}

extern "C" lora_status lora_timing_end(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_on = false;
    if (hipDeviceSynchronize() != hipSuccess) return LORA_ERR_DEVICE;
    lora_status st = LORA_OK;
    for (auto& r : g_records) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            stats& s = g_stats[r.id];
            const double us = (double)ms * 1000.0;
            if (s.count == 0 || us < s.min_us) s.min_us = us;
            if (s.count == 0 || us > s.max_us) s.max_us = us;
            s.total_us += us;
            s.count += 1;
        } else {
            (void)hipGetLastError();
            st = LORA_ERR_DEVICE;
        }
        g_free.emplace_back(r.start, r.stop);
    }
    g_records.clear();
    return st;
}

extern "C" lora_status lora_timing_read(int32_t kernel_id, int64_t* count, double* total_us,
                                        double* min_us, double* max_us)
{
    if (kernel_id < 0 || kernel_id >= LORA_K_COUNT) return LORA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mu);
    const stats& s = g_stats[kernel_id];
    if (count) *count = s.count;
    if (total_us) *total_us = s.total_us;
    if (min_us) *min_us = s.min_us;
    if (max_us) *max_us = s.max_us;
    return LORA_OK;
}

extern "C" const char* lora_kernel_name(int32_t kernel_id)
{
    return (kernel_id >= 0 && kernel_id < LORA_K_COUNT) ? kNames[kernel_id] : "";
}

extern "C" int32_t lora_kernel_count(void) { return LORA_K_COUNT; }

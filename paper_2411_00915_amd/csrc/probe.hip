// Measured ceilings of the machine, for the benchmark's report (the paper times its operator over repeated rounds,
// section 6.3.2; a roofline fraction against the vendor's peak says little without what a plain kernel reaches on
// the same box in the same run).  Three small kernels behind lora_probe: an empty launch, a one-shot read without
// any dependency (every lane asks for all its 16-byte pieces at once, whole lines per wavefront, non-temporal), and
// a register-only loop of independent bf16 MFMAs that also reads the shader clock against the constant wall clock.
// Timed with the library's per-kernel timers like every other kernel.
#include <hip/hip_runtime.h>

#include "../../include/lora_abi.h"
#include "launch.h"
#include "mfma_tile.h"

namespace {

__global__ __launch_bounds__(256) void probe_empty_kernel(unsigned* sink, int never)
{
    if (never) sink[0] = 1;                                       // `never` is 0 at run time: nothing is read or written
}

// block b reads 256 * U consecutive 16-byte pieces starting at piece b * 256 * U (U pieces per lane, each
// instruction of a wavefront covers 1 KB); `pieces` is a multiple of 256 * U by construction of the launch
template <int U>
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, unsigned* sink, int never)
{
    const size_t base = ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 64 * U + (threadIdx.x & 63);
    uint4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = ld16_stream(reinterpret_cast<const bf16_t*>(src + base + u * 64));
    unsigned acc = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) acc += r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
    if (acc == 0x12345678u && never) sink[0] = acc;               // keeps the loads; `never` is 0 at run time
}

// iters x 16 independent MFMAs per wavefront on register operands; wavefront 0 of block 0 reports the shader
// clock ticks and wall-clock ticks the loop took: out[0], out[1]
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, unsigned long long* out, float* sink)
{
    op16 a, b;
    a.u = uint4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u ^ threadIdx.x};       // bf16 ones (one lane-dependent)
    b.u = uint4{0x3f003f00u, 0x3f003f00u, 0x3f003f00u, 0x3f003f00u};                     // bf16 halves
    floatx4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = mfma(a, b, acc[i]);
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == -1.f) sink[0] = s;                                   // keeps the MFMAs; the sums are positive
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = w1 - w0;
    }
}

}  // namespace

extern "C" lora_status lora_probe(int32_t kind, void* buffer, size_t bytes, int32_t iters, void* hip_stream)
{
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!buffer || bytes < 64 || (reinterpret_cast<uintptr_t>(buffer) & 15)) return LORA_ERR_INVALID_ARG;
    if (kind == LORA_PROBE_EMPTY) {
        // (iters > 1: that many workgroups instead of 1280)
        LORA_LAUNCH(LORA_K_PROBE_EMPTY, probe_empty_kernel, dim3(iters > 1 ? iters : 1280), dim3(256), 0, stream, static_cast<unsigned*>(buffer), 0);
    } else if (kind == LORA_PROBE_READ) {
        constexpr int U = 8;                                       // 128 bytes in flight per lane, 32 KB per workgroup
        const size_t blocks = bytes / (256 * U * 16);
        if (blocks == 0 || blocks > 0x7fffffffu) return LORA_ERR_INVALID_ARG;
        // (reads the first blocks * 32 KB of the buffer; the last 64 bytes of the buffer are the sink, never written)
        LORA_LAUNCH(LORA_K_PROBE_READ, probe_read_kernel<U>, dim3((unsigned)blocks), dim3(256), 0, stream,
                    static_cast<const uint4*>(buffer), reinterpret_cast<unsigned*>(static_cast<char*>(buffer) + bytes - 64), 0);
    } else if (kind == LORA_PROBE_MFMA) {
        if (iters < 1) return LORA_ERR_INVALID_ARG;
        // 2048 workgroups of 4 wavefronts: 8 wavefronts per SIMD
        if (bytes < 64) return LORA_ERR_INVALID_ARG;
        LORA_LAUNCH(LORA_K_PROBE_MFMA, probe_mfma_kernel, dim3(2048), dim3(256), 0, stream, iters,
                    static_cast<unsigned long long*>(buffer), reinterpret_cast<float*>(static_cast<char*>(buffer) + 32));
        // buffer[2]: the rate of the wall clock the kernel read, in kHz (stream-ordered copy from a host constant)
        static unsigned long long wall_khz[64] = {0};
        int dev = 0, khz = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LORA_ERR_DEVICE;
        if (wall_khz[dev] == 0) {
            if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) khz = 100000;
            wall_khz[dev] = (unsigned long long)khz;
        }
        if (hipMemcpyAsync(static_cast<char*>(buffer) + 16, &wall_khz[dev], 8, hipMemcpyHostToDevice, stream) != hipSuccess)
            return LORA_ERR_DEVICE;
    } else {
        return LORA_ERR_INVALID_ARG;
    }
    return hipGetLastError() == hipSuccess ? LORA_OK : LORA_ERR_DEVICE;
}

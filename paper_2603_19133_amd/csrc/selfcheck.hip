// Device self-check of the one hardware behaviour the row kernels' memory safety rests on: a raw buffer
// load (stride 0) is in range iff scalar offset + per-lane offset + 16 <= the descriptor's size, and a lane
// out of range reads zero.  Every address formed here lies inside the caller's 64 KiB workspace.
#include "common.hpp"
#include "kernels.hpp"

namespace picospec {

namespace {

constexpr int kCheckWords = kCheckBytes / 4;

__global__ __launch_bounds__(256) void check_fill_kernel(uint32_t* __restrict__ buf, uint32_t* __restrict__ status)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < kCheckWords; i += gridDim.x * blockDim.x) buf[i] = 0x40000000u + (uint32_t)i;   // never 0
    if (blockIdx.x == 0 && threadIdx.x == 0) *status = 0u;
}

// One wave.  Case c loads 16 bytes per lane at scalar offset soff[c] + lane * 16 + voff[c] through a descriptor
// of size[c] bytes; lane l must read its word iff soff + voff + l*16 + 16 <= size, zero otherwise.
__global__ __launch_bounds__(kWave) void check_range_kernel(const uint32_t* __restrict__ buf, uint32_t* __restrict__ status)
{
    const int lane = threadIdx.x;
    constexpr int kCases = 6;
    const int size[kCases] = {1024, 512, 1024, 8192, 4608, 1024};
    const int soff[kCases] = {0, 0, 4096, 4096, 4096, 0};
    const int voff[kCases] = {0, 0, 0, 0, 0, 4096};
    unsigned bad = 0;
#pragma unroll
    for (int c = 0; c < kCases; ++c) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)buf, 0, size[c], 0x00020000);
        const u32x4_t t = __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16 + voff[c], soff[c], 0);
        const int at = soff[c] + voff[c] + lane * 16;
        const bool in_range = at + 16 <= size[c];
        const uint32_t want = in_range ? 0x40000000u + (uint32_t)(at / 4) : 0u;
        if (t.x != want || (!in_range && (t.y | t.z | t.w) != 0u)) bad |= 1u << c;
    }
    if (bad) atomicOr(status, bad);
}

// One wave: a fixed loop of dependent fused multiply-adds, timed with the shader-clock counter (s_memtime) and with
// the constant 100 MHz wall clock (s_memrealtime).  Their ratio is the shader clock the device really runs at.
__global__ __launch_bounds__(kWave) void probe_clock_kernel(uint64_t* __restrict__ out)
{
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    float a = (float)threadIdx.x * 1e-3f;
    for (int i = 0; i < 4000; ++i) a = fmaf(a, 1.0001f, 0.5f);
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; }
    if (a == 12345.678f) out[1] = 0;             // (keeps the loop)
}

}  // namespace

hipError_t launch_probe_clock(uint64_t* out, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_clock_kernel, dim3(1), dim3(kWave), 0, stream, out);
    return hipGetLastError();
}

hipError_t launch_check_device(void* workspace, uint32_t* status, hipStream_t stream)
{
    hipLaunchKernelGGL(check_fill_kernel, dim3(16), dim3(256), 0, stream, (uint32_t*)workspace, status);
    hipLaunchKernelGGL(check_range_kernel, dim3(1), dim3(kWave), 0, stream, (const uint32_t*)workspace, status);
    return hipGetLastError();
}

}  // namespace picospec

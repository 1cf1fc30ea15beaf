// Measurement aids, not part of the attention path: what the chip sustains on the two resources the path is bound
// by, measured on the same box and in the same process as the benchmark, so that "fraction of the published peak"
// can be read beside "fraction of what a bare loop reaches here".
//   * esp_probe_mfma_bf16: every wavefront runs a loop of v_mfma_f32_32x32x16_bf16 on operands held in registers
//     (four independent accumulators, 2 wavefronts per SIMD, all CUs).  The operands come from a caller buffer:
//     with N(0,1) values the multipliers switch as they do in the prefill kernel, with a constant they hardly
//     switch, and the clock the chip holds under its power limit differs accordingly.
//   * esp_probe_stream_read: a grid-stride read of a buffer in 16-byte pieces, summed so that nothing is elided.
#include "esp_common.h"

namespace esp {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float probe_floatx16;

__global__ __launch_bounds__(512) void probe_mfma_kernel(const bf16x8* __restrict__ operands, int32_t n_operands,
                                                         int32_t iters, float* __restrict__ sink) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[(tid * 8 + i) % n_operands];
        b[i] = operands[(tid * 8 + 4 + i) % n_operands];
    }
    probe_floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 123.456f) sink[0] = s;          // keeps the loop alive without a store per lane
}

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, int64_t n_chunks,
                                                         uint32_t* __restrict__ sink) {
    uint32_t s = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_chunks; i += stride) {
        const uint4 w = load_once(&src[i]);
        s += w.x ^ w.y ^ w.z ^ w.w;
    }
    if (s == 0x9e3779b9u) sink[0] = s;
}

esp_status launch_probe_mfma(const void* operands, int64_t operand_bytes, int32_t iters, void* sink, int64_t* flops,
                             hipStream_t stream) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return fail(ESP_ERR_HIP, "probe: cannot query the device");
    const int waves = 8;                                   // per CU: two per SIMD
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(cus), dim3(waves * 64), 0, stream, (const bf16x8*)operands,
                       (int32_t)(operand_bytes / 16), iters, (float*)sink);
    if (flops) *flops = (int64_t)cus * waves * iters * 4 * (2LL * 32 * 32 * 16);
    return check_launch("probe_mfma_kernel");
}

esp_status launch_probe_read(const void* src, int64_t bytes, void* sink, hipStream_t stream) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return fail(ESP_ERR_HIP, "probe: cannot query the device");
    hipLaunchKernelGGL(probe_read_kernel, dim3(cus * 8), dim3(256), 0, stream, (const uint4*)src, bytes / 16, (uint32_t*)sink);
    return check_launch("probe_read_kernel");
}

}  // namespace esp

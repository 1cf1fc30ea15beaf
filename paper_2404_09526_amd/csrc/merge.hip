// esp_merge_partials: log-sum-exp weighted combination of P partial attention results of the
// same (token, head) pairs into the result over the union of their key sets (the final
// output after all sequence-parallel rounds, Sec. 2.3; the results returned to the master in
// distributed decoding, Sec. 4.2).  HBM-streaming: 16 lanes share one (token, head) pair,
// each owning 8 of the 128 output elements (one 16-byte load per bf16 partial, two per fp32 partial:
// partials that never leave this GPU, the rounds of a sequence-parallel prefill, may stay in fp32,
// so that the merged result is rounded to bf16 once and not twice).
#include "esp_common.h"

namespace esp {

template <bool F32>
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs parts, int32_t P, int64_t pairs,
                                                    uint4* O, float* LSE_out) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t pair = i >> 4;
    if (pair >= pairs) return;
    int seg = (int)(i & 15);

    float m = -INFINITY;
    float lse[ESP_MAX_PARTIALS];
#pragma unroll
    for (int p = 0; p < ESP_MAX_PARTIALS; ++p) {
        lse[p] = (p < P) ? parts.LSE_parts[p][pair] : -INFINITY;
        m = fmaxf(m, lse[p]);
    }
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float wsum = 0.f;
    if (m != -INFINITY) {
#pragma unroll
        for (int p = 0; p < ESP_MAX_PARTIALS; ++p) {
            if (p < P) {
                // an empty partial (LSE = -inf) gets weight exp(-inf) = 0
                float w = __expf(lse[p] - m);
                wsum += w;
                float f[8];
                if (F32) {
                    const float4* src = (const float4*)parts.O_parts[p] + (pair * 16 + seg) * 2;
                    const float4 a = load_once(&src[0]), b = load_once(&src[1]);
                    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
                } else {
                    const uint4 o = load_once(&((const uint4*)parts.O_parts[p])[pair * 16 + seg]);
                    f[0] = bf16_lo(o.x); f[1] = bf16_hi(o.x); f[2] = bf16_lo(o.y); f[3] = bf16_hi(o.y);
                    f[4] = bf16_lo(o.z); f[5] = bf16_hi(o.z); f[6] = bf16_lo(o.w); f[7] = bf16_hi(o.w);
                }
                if (w != 0.f) {  // keeps non-finite garbage of an empty partial out of the sum
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] += w * f[e];
                }
            }
        }
        float inv = 1.0f / wsum;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= inv;
    }
    uint4 out;
    out.x = pack_bf16(acc[0], acc[1]);
    out.y = pack_bf16(acc[2], acc[3]);
    out.z = pack_bf16(acc[4], acc[5]);
    out.w = pack_bf16(acc[6], acc[7]);
    O[pair * 16 + seg] = out;
    if (LSE_out != nullptr && seg == 0) LSE_out[pair] = (m == -INFINITY) ? -INFINITY : m + __logf(wsum);
}

esp_status launch_merge(const MergeArgs& parts, int32_t P, int64_t pairs, int32_t parts_f32, void* O, float* LSE_out,
                        hipStream_t stream) {
    int64_t threads = pairs * 16;
    int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffff) return fail(ESP_ERR_INVALID_ARG, "merge: too many rows for one launch");
    if (parts_f32)
        hipLaunchKernelGGL(merge_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, parts, P, pairs, (uint4*)O, LSE_out);
    else
        hipLaunchKernelGGL(merge_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, parts, P, pairs, (uint4*)O, LSE_out);
    return check_launch("merge_kernel");
}

}  // namespace esp

// Internal declarations shared by the translation units of libesp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "esp.h"

namespace esp {

constexpr int kHeadDim = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Records a message for esp_last_error() and returns `code`.
esp_status fail(esp_status code, const char* fmt, ...);
// Returns ESP_OK or converts the pending launch error into ESP_ERR_HIP.
esp_status check_launch(const char* what);

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;

// bf16 bit pattern (low or high half of a 32-bit word) to float: exact.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// Two floats to packed bf16 (round to nearest even), a in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    floatx2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// Loads and stores of data that passes once (pool rows under a decode pass, partials on their way to a merge):
// marked non-temporal, so that they do not displace what the caches hold.  Measured on the decode kernel: 74 % -> 82 %
// of the HBM rate.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_once(const uint4* p) {
    const u32x4 t = __builtin_nontemporal_load((const u32x4*)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ float4 load_once(const float4* p) {
    const floatx4 t = __builtin_nontemporal_load((const floatx4*)p);
    return make_float4(t[0], t[1], t[2], t[3]);
}
__device__ __forceinline__ void store_once(uint4* p, const uint4& v) {
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, (u32x4*)p);
}

// ---- launchers (one per kernel file) -------------------------------------------------
struct MergeArgs {
    const void* O_parts[ESP_MAX_PARTIALS];
    const float* LSE_parts[ESP_MAX_PARTIALS];
};
esp_status launch_kv_append(const void* k, const void* v, const int32_t* slot_idx, int32_t T, void* k_pool,
                            void* v_pool, int32_t row_bytes, hipStream_t stream);
esp_status launch_kv_gather(const void* k_pool, const void* v_pool, const int32_t* slot_idx, int32_t T, int64_t num_slots,
                            void* k, void* v, int32_t row_bytes, hipStream_t stream);
esp_status launch_probe_mfma(const void* operands, int64_t operand_bytes, int32_t iters, void* sink, int64_t* flops,
                             hipStream_t stream);
esp_status launch_probe_read(const void* src, int64_t bytes, void* sink, hipStream_t stream);
esp_status launch_merge(const MergeArgs& parts, int32_t P, int64_t pairs, int32_t parts_f32, void* O, float* LSE_out,
                        hipStream_t stream);

size_t decode_workspace_bytes(int32_t B, int32_t total_tokens, int32_t Hq, int32_t Hkv);
esp_status launch_decode(const void* q, const void* k_pool, const void* v_pool, const int32_t* slot_idx,
                         const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t Hq, int32_t Hkv,
                         float softmax_scale, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                         hipStream_t stream, const MergeArgs* peers = nullptr, int32_t n_peers = 0);

// the partial kernel on the matrix cores (decode_gq.hip): one partial per (range + request, head)
esp_status launch_decode_gq(const void* q, const void* k_pool, const void* v_pool, const int32_t* slot_idx,
                            const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t range, int32_t nwg,
                            int32_t Hq, int32_t Hkv, float scale_log2, float* part_acc, float* part_ml, hipStream_t stream);

int32_t set_prefill_sync_ticks(int32_t ticks);   // returns the previous value; negative restores the built-in default
esp_status launch_decode_static(const void* q, const void* k_pool, const void* v_pool, const int32_t* slot_idx,
                                const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t Hq, int32_t Hkv,
                                float softmax_scale, void* O, float* LSE, hipStream_t stream);

size_t prefill_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch, int32_t Hq, int32_t Hkv);
esp_status launch_prefill(const void* q, const void* k, const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                          const int32_t* cu_q, const int32_t* cu_kv, int32_t batch, int32_t Tq, int32_t Tkv,
                          int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv, float softmax_scale,
                          int32_t causal, int32_t o_f32, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                          const int32_t* retain_slot, void* k_pool, void* v_pool, const int32_t* kv_slot,
                          hipStream_t stream);

}  // namespace esp

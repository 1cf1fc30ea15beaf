// esp_kv_append: scatter of K/V token rows into scheduler-chosen slots of the token-granular
// pool (selective retention during prefill, Sec. 4.1 / Fig. 7; the master's save of the new
// token's K/V, Sec. 4.2).  A pure copy of bit patterns, HBM-bound: each kept row is read
// once and written once, in 16-byte pieces with consecutive lanes on consecutive pieces.
#include "esp_common.h"

namespace esp {

__global__ __launch_bounds__(256) void kv_append_kernel(const uint4* __restrict__ k, const uint4* __restrict__ v,
                                                        const int32_t* __restrict__ slot_idx, int64_t total_chunks,
                                                        int32_t chunks_per_row, uint4* __restrict__ k_pool,
                                                        uint4* __restrict__ v_pool) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total_chunks) return;
    int32_t t = (int32_t)(i / chunks_per_row);
    int32_t c = (int32_t)(i - (int64_t)t * chunks_per_row);
    int32_t slot = slot_idx[t];
    if (slot < 0) return;  // token not retained on this instance
    int64_t dst = (int64_t)slot * chunks_per_row + c;
    k_pool[dst] = load_once(&k[i]);
    v_pool[dst] = load_once(&v[i]);
}

// esp_kv_gather: the inverse view, rows of the pool in the order of a slot list (a request's resident K/V as the
// dense [T, Hkv, D] arrays the prefill call takes).  A negative slot, or one beyond the pool, gives a zero row.
__global__ __launch_bounds__(256) void kv_gather_kernel(const uint4* __restrict__ k_pool, const uint4* __restrict__ v_pool,
                                                        const int32_t* __restrict__ slot_idx, int64_t total_chunks,
                                                        int32_t chunks_per_row, int64_t num_slots,
                                                        uint4* __restrict__ k, uint4* __restrict__ v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total_chunks) return;
    int32_t t = (int32_t)(i / chunks_per_row);
    int32_t c = (int32_t)(i - (int64_t)t * chunks_per_row);
    int32_t slot = slot_idx[t];
    uint4 kk = make_uint4(0u, 0u, 0u, 0u), vv = kk;
    if (slot >= 0 && slot < num_slots) {
        int64_t src = (int64_t)slot * chunks_per_row + c;
        kk = load_once(&k_pool[src]);
        vv = load_once(&v_pool[src]);
    }
    k[i] = kk;
    v[i] = vv;
}

esp_status launch_kv_gather(const void* k_pool, const void* v_pool, const int32_t* slot_idx, int32_t T, int64_t num_slots,
                            void* k, void* v, int32_t row_bytes, hipStream_t stream) {
    int32_t cpr = row_bytes / 16;
    int64_t total = (int64_t)T * cpr;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return fail(ESP_ERR_INVALID_ARG, "gather: too many rows for one launch");
    hipLaunchKernelGGL(kv_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)k_pool,
                       (const uint4*)v_pool, slot_idx, total, cpr, num_slots, (uint4*)k, (uint4*)v);
    return check_launch("kv_gather_kernel");
}

esp_status launch_kv_append(const void* k, const void* v, const int32_t* slot_idx, int32_t T, void* k_pool,
                            void* v_pool, int32_t row_bytes, hipStream_t stream) {
    int32_t cpr = row_bytes / 16;
    int64_t total = (int64_t)T * cpr;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return fail(ESP_ERR_INVALID_ARG, "append: too many rows for one launch");
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)k,
                       (const uint4*)v, slot_idx, total, cpr, (uint4*)k_pool, (uint4*)v_pool);
    return check_launch("kv_append_kernel");
}

}  // namespace esp

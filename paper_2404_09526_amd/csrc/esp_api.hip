// C-ABI entry points of libesp: argument validation and dispatch to the kernel launchers.
// Every step of the hot path runs in the HIP kernels of this library; there is no fallback.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "esp_common.h"

namespace esp {

static thread_local char g_err[512] = "";

esp_status fail(esp_status code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

esp_status check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ESP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return ESP_OK;
}

static bool heads_ok(int32_t Hq, int32_t Hkv) { return Hq > 0 && Hkv > 0 && Hq % Hkv == 0; }
// head counts the decode kernels cover: all (a row-burst kernel for 4, 8, 16 or a multiple of 32 KV heads with query
// groups of 1, 2, 4 or 8; a per-head kernel for every other combination)
static bool decode_heads_supported(int32_t Hq, int32_t Hkv) { return heads_ok(Hq, Hkv); }

// ESP_DEBUG_VALIDATE=1 in the environment: the content of the device index arrays, trusted otherwise, is checked on
// the host before the launch.  A debugging aid: it waits for the stream and copies the arrays back.
static std::atomic<int> g_validate{[] {             // the environment is read once, when the library is loaded
    const char* e = getenv("ESP_DEBUG_VALIDATE");
    return (e && strcmp(e, "0") != 0 && e[0] != 0) ? 1 : 0;
}()};
static bool debug_validate() { return g_validate.load(std::memory_order_relaxed) != 0; }
static bool fetch_i32(const int32_t* dev, size_t n, hipStream_t stream, std::vector<int32_t>& out) {
    out.resize(n);
    if (n == 0) return true;
    if (hipStreamSynchronize(stream) != hipSuccess) return false;
    return hipMemcpy(out.data(), dev, n * sizeof(int32_t), hipMemcpyDeviceToHost) == hipSuccess;
}
// prefix offsets: start at 0, never decrease, end at `total`, no piece longer than `longest`
static esp_status check_offsets(const char* what, const int32_t* dev, int32_t n, int64_t total, int64_t longest, hipStream_t stream) {
    std::vector<int32_t> h;
    if (!fetch_i32(dev, (size_t)n + 1, stream, h)) return fail(ESP_ERR_HIP, "%s: cannot read the offsets back", what);
    if (h[0] != 0 || h[n] != total) return fail(ESP_ERR_INVALID_ARG, "%s: offsets run from %d to %d, expected 0 to %lld", what, h[0], h[n], (long long)total);
    for (int32_t i = 0; i < n; ++i) {
        if (h[i + 1] < h[i]) return fail(ESP_ERR_INVALID_ARG, "%s: offsets decrease at entry %d", what, i + 1);
        if ((int64_t)h[i + 1] - h[i] > longest) return fail(ESP_ERR_INVALID_ARG, "%s: piece %d has %d rows, more than the stated maximum %lld", what, i, h[i + 1] - h[i], (long long)longest);
    }
    return ESP_OK;
}
// slots: below num_slots; negative ones only where the call gives them a meaning; no slot twice if asked
static esp_status check_slots(const char* what, const int32_t* dev, int64_t n, int64_t num_slots, bool negative_ok, bool unique,
                              hipStream_t stream) {
    std::vector<int32_t> h;
    if (!fetch_i32(dev, (size_t)n, stream, h)) return fail(ESP_ERR_HIP, "%s: cannot read the slots back", what);
    for (int64_t i = 0; i < n; ++i) {
        if (h[i] >= num_slots) return fail(ESP_ERR_INVALID_ARG, "%s: slot_idx[%lld] = %d is not below num_slots = %lld", what, (long long)i, h[i], (long long)num_slots);
        if (h[i] < 0 && !negative_ok) return fail(ESP_ERR_INVALID_ARG, "%s: slot_idx[%lld] = %d is negative", what, (long long)i, h[i]);
    }
    if (unique) {
        std::sort(h.begin(), h.end());
        for (int64_t i = 1; i < n; ++i)
            if (h[i] >= 0 && h[i] == h[i - 1]) return fail(ESP_ERR_INVALID_ARG, "%s: slot %d is named twice", what, h[i]);
    }
    return ESP_OK;
}

}  // namespace esp

using namespace esp;

extern "C" {

const char* esp_last_error(void) { return g_err; }

int32_t esp_debug_set_validate(int32_t on) { return g_validate.exchange(on ? 1 : 0, std::memory_order_relaxed); }
int32_t esp_debug_set_prefill_sync_ticks(int32_t ticks) { return set_prefill_sync_ticks(ticks); }
const char* esp_version(void) { return "esp 0.1 gfx950"; }

size_t esp_prefill_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch, int32_t Hq, int32_t Hkv, int32_t D) {
    if (Tq < 0 || Tkv < 0 || batch < 1 || !heads_ok(Hq, Hkv) || D != kHeadDim) return 0;
    return prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv);
}

size_t esp_decode_workspace_bytes(int32_t B, int32_t total_tokens, int32_t max_len, int32_t Hq, int32_t Hkv,
                                  int32_t D) {
    (void)max_len;
    if (B < 0 || total_tokens < 0 || !decode_heads_supported(Hq, Hkv) || D != kHeadDim) return 0;   // 0: the call would be refused
    return decode_workspace_bytes(B, total_tokens, Hq, Hkv);
}

static esp_status prefill_entry(const void* q, const void* k, const void* v, const int32_t* q_pos,
                                const int32_t* kv_pos, const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
                                int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv,
                                int32_t D, float softmax_scale, int32_t causal, int32_t o_f32, void* O, float* LSE,
                                void* workspace, size_t workspace_bytes, void* stream,
                                const int32_t* retain_slot = nullptr, void* k_pool = nullptr, void* v_pool = nullptr,
                                int64_t num_slots = 0, const int32_t* kv_slot = nullptr) {
    if (Tq < 0 || Tkv < 0 || batch < 1 || max_q < 0 || max_kv < 0)
        return fail(ESP_ERR_INVALID_ARG, "prefill: negative size or batch < 1");
    if (!heads_ok(Hq, Hkv)) return fail(ESP_ERR_INVALID_ARG, "prefill: Hq=%d must be a positive multiple of Hkv=%d", Hq, Hkv);
    if (D != kHeadDim) return fail(ESP_ERR_UNSUPPORTED, "prefill: head_dim %d unsupported (only 128)", D);
    if (max_q > Tq || max_kv > Tkv) return fail(ESP_ERR_INVALID_ARG, "prefill: max_q/max_kv exceed Tq/Tkv");
    if ((cu_q == nullptr) != (cu_kv == nullptr)) return fail(ESP_ERR_INVALID_ARG, "prefill: cu_q and cu_kv must both be given or both NULL");
    if (cu_q == nullptr && batch != 1) return fail(ESP_ERR_INVALID_ARG, "prefill: batch > 1 needs cu_q/cu_kv");
    if (cu_q == nullptr && (max_q != Tq || max_kv != Tkv))
        return fail(ESP_ERR_INVALID_ARG, "prefill: without cu_q/cu_kv, max_q/max_kv must equal Tq/Tkv");
    if (retain_slot && Tkv > 0) {
        if (!k || !v || !k_pool || !v_pool || num_slots <= 0) return fail(ESP_ERR_INVALID_ARG, "prefill (retain): null k/v/pool or empty pool");
        if (debug_validate()) {
            esp_status st = check_slots("prefill (retain)", retain_slot, Tkv, num_slots, true, true, (hipStream_t)stream);
            if (st != ESP_OK) return st;
        }
        // no query row at all: nothing to attend, the rows are kept by the plain scatter
        if (Tq == 0) return launch_kv_append(k, v, retain_slot, Tkv, k_pool, v_pool, Hkv * D * 2, (hipStream_t)stream);
    }
    if (Tq == 0) return ESP_OK;
    if (kv_slot && Tkv > 0 && debug_validate()) {                   // k and v are the pools: rows come from these slots
        esp_status st = check_slots("prefill (pool)", kv_slot, Tkv, num_slots, false, false, (hipStream_t)stream);
        if (st != ESP_OK) return st;
    }
    if (!q || !O || !LSE || !q_pos) return fail(ESP_ERR_INVALID_ARG, "prefill: null q/q_pos/O/LSE");
    if (Tkv > 0 && (!k || !v || !kv_pos)) return fail(ESP_ERR_INVALID_ARG, "prefill: null k/v/kv_pos");
    if (!(softmax_scale == softmax_scale) || softmax_scale < 0.f) return fail(ESP_ERR_INVALID_ARG, "prefill: bad softmax_scale");
    size_t need = prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv);
    if (need > 0 && (!workspace || workspace_bytes < need))
        return fail(ESP_ERR_WORKSPACE, "prefill: workspace needs %zu bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if (need > 0 && ((uintptr_t)workspace & 255)) return fail(ESP_ERR_WORKSPACE, "prefill: workspace not 256-byte aligned");
    if (cu_q && debug_validate()) {
        esp_status st = check_offsets("prefill: cu_q", cu_q, batch, Tq, max_q, (hipStream_t)stream);
        if (st == ESP_OK) st = check_offsets("prefill: cu_kv", cu_kv, batch, Tkv, max_kv, (hipStream_t)stream);
        if (st != ESP_OK) return st;
    }
    return launch_prefill(q, k, v, q_pos, kv_pos, cu_q, cu_kv, batch, Tq, Tkv, max_q, max_kv, Hq, Hkv,
                          softmax_scale, causal, o_f32, O, LSE, workspace, workspace_bytes,
                          Tkv > 0 ? retain_slot : nullptr, k_pool, v_pool, Tkv > 0 ? kv_slot : nullptr, (hipStream_t)stream);
}

esp_status esp_partial_attn_prefill_retain(const void* q, const void* k, const void* v, const int32_t* q_pos,
                                           const int32_t* kv_pos, const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
                                           int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv,
                                           int32_t D, float softmax_scale, int32_t causal, const int32_t* retain_slot,
                                           void* k_pool, void* v_pool, int64_t num_slots, int32_t out_f32, void* O,
                                           float* LSE, void* workspace, size_t workspace_bytes, void* stream) {
    if (!retain_slot && Tkv > 0) return fail(ESP_ERR_INVALID_ARG, "prefill (retain): null retain_slot");
    if (num_slots < 0) return fail(ESP_ERR_INVALID_ARG, "prefill (retain): negative num_slots");
    return prefill_entry(q, k, v, q_pos, kv_pos, cu_q, cu_kv, batch, Tq, Tkv, max_q, max_kv, Hq, Hkv, D, softmax_scale, causal,
                         out_f32 ? 1 : 0, O, LSE, workspace, workspace_bytes, stream, retain_slot, k_pool, v_pool, num_slots);
}

esp_status esp_partial_attn_prefill(const void* q, const void* k, const void* v, const int32_t* q_pos,
                                    const int32_t* kv_pos, const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
                                    int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv,
                                    int32_t D, float softmax_scale, int32_t causal, void* O, float* LSE,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_entry(q, k, v, q_pos, kv_pos, cu_q, cu_kv, batch, Tq, Tkv, max_q, max_kv, Hq, Hkv, D, softmax_scale, causal, 0,
                         O, LSE, workspace, workspace_bytes, stream);
}

esp_status esp_partial_attn_prefill_f32(const void* q, const void* k, const void* v, const int32_t* q_pos,
                                        const int32_t* kv_pos, const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
                                        int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv,
                                        int32_t D, float softmax_scale, int32_t causal, float* O, float* LSE,
                                        void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_entry(q, k, v, q_pos, kv_pos, cu_q, cu_kv, batch, Tq, Tkv, max_q, max_kv, Hq, Hkv, D, softmax_scale, causal, 1,
                         O, LSE, workspace, workspace_bytes, stream);
}

esp_status esp_probe_mfma_bf16(const void* operands, int64_t operand_bytes, int32_t iters, void* sink, int64_t* flops,
                               void* stream) {
    if (!operands || operand_bytes < 16 || (operand_bytes & 15) || ((uintptr_t)operands & 15) || iters < 1 || !sink)
        return fail(ESP_ERR_INVALID_ARG, "probe: operands (16-byte aligned, a multiple of 16 bytes), iters >= 1 and a sink are needed");
    return launch_probe_mfma(operands, operand_bytes, iters, sink, flops, (hipStream_t)stream);
}

esp_status esp_probe_stream_read(const void* src, int64_t bytes, void* sink, void* stream) {
    if (!src || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || !sink)
        return fail(ESP_ERR_INVALID_ARG, "probe: a 16-byte aligned buffer of a multiple of 16 bytes and a sink are needed");
    return launch_probe_read(src, bytes, sink, (hipStream_t)stream);
}

esp_status esp_kv_gather(const void* k_pool, const void* v_pool, const int32_t* slot_idx, int32_t T, int64_t num_slots,
                         int32_t Hkv, int32_t D, void* k, void* v, void* stream) {
    if (T < 0 || num_slots < 0 || Hkv <= 0) return fail(ESP_ERR_INVALID_ARG, "gather: negative size");
    if (D != kHeadDim) return fail(ESP_ERR_UNSUPPORTED, "gather: head_dim %d unsupported (only 128)", D);
    if (T == 0) return ESP_OK;
    if (!k || !v || !slot_idx) return fail(ESP_ERR_INVALID_ARG, "gather: null pointer");
    if (num_slots > 0 && (!k_pool || !v_pool)) return fail(ESP_ERR_INVALID_ARG, "gather: null pool");
    return launch_kv_gather(k_pool, v_pool, slot_idx, T, num_slots, k, v, Hkv * D * 2, (hipStream_t)stream);
}

// the staging rows of the pool variant come first in its workspace, the dense call's own block after them
static size_t pool_staging_bytes(int32_t Tkv, int32_t Hkv) {
    size_t one = (size_t)(Tkv > 0 ? Tkv : 0) * (size_t)(Hkv > 0 ? Hkv : 0) * kHeadDim * 2;
    return (one + 255) / 256 * 256;
}

size_t esp_prefill_pool_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch, int32_t Hq, int32_t Hkv, int32_t D) {
    (void)D;
    return 2 * pool_staging_bytes(Tkv, Hkv) + prefill_workspace_bytes(Tq, Tkv, batch, Hq, Hkv);
}

esp_status esp_partial_attn_prefill_pool(const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
                                         const int32_t* slot_idx, const int32_t* q_pos, const int32_t* kv_pos,
                                         const int32_t* cu_q, const int32_t* cu_kv, int32_t batch, int32_t Tq,
                                         int32_t Tkv, int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv, int32_t D,
                                         float softmax_scale, int32_t causal, void* O, float* LSE, void* workspace,
                                         size_t workspace_bytes, void* stream) {
    if (Tkv < 0 || num_slots < 0 || Hkv <= 0) return fail(ESP_ERR_INVALID_ARG, "prefill (pool): negative size");
    if (D != kHeadDim) return fail(ESP_ERR_UNSUPPORTED, "prefill (pool): head_dim %d unsupported (only 128)", D);
    if (Tkv > 0 && !slot_idx) return fail(ESP_ERR_INVALID_ARG, "prefill (pool): null slot_idx");
    const size_t stage = pool_staging_bytes(Tkv, Hkv);
    const size_t need = esp_prefill_pool_workspace_bytes(Tq, Tkv, batch, Hq, Hkv, D);
    if (!workspace || workspace_bytes < need)
        return fail(ESP_ERR_WORKSPACE, "prefill (pool): workspace needs %zu bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if ((uintptr_t)workspace & 255) return fail(ESP_ERR_WORKSPACE, "prefill (pool): workspace not 256-byte aligned");
    char* ws = (char*)workspace;
    esp_status st = esp_kv_gather(k_pool, v_pool, slot_idx, Tkv, num_slots, Hkv, D, ws, ws + stage, stream);
    if (st != ESP_OK) return st;
    return esp_partial_attn_prefill(q, ws, ws + stage, q_pos, kv_pos, cu_q, cu_kv, batch, Tq, Tkv, max_q, max_kv, Hq, Hkv, D,
                                    softmax_scale, causal, O, LSE, ws + 2 * stage, workspace_bytes - 2 * stage, stream);
}

esp_status esp_partial_attn_prefill_pool_direct(const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
                                                const int32_t* slot_idx, const int32_t* q_pos, const int32_t* kv_pos,
                                                const int32_t* cu_q, const int32_t* cu_kv, int32_t batch, int32_t Tq,
                                                int32_t Tkv, int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv, int32_t D,
                                                float softmax_scale, int32_t causal, int32_t out_f32, void* O, float* LSE,
                                                void* workspace, size_t workspace_bytes, void* stream) {
    if (Tkv < 0 || num_slots < 0) return fail(ESP_ERR_INVALID_ARG, "prefill (pool): negative size");
    if (Tkv > 0 && !slot_idx) return fail(ESP_ERR_INVALID_ARG, "prefill (pool): null slot_idx");
    if (Tkv > 0 && num_slots == 0) return fail(ESP_ERR_INVALID_ARG, "prefill (pool): empty pool");
    return prefill_entry(q, k_pool, v_pool, q_pos, kv_pos, cu_q, cu_kv, batch, Tq, Tkv, max_q, max_kv, Hq, Hkv, D, softmax_scale,
                         causal, out_f32 ? 1 : 0, O, LSE, workspace, workspace_bytes, stream, nullptr, nullptr, nullptr, num_slots,
                         slot_idx);
}

// argument checks common to the two decode entry points; *done is set when there is nothing to launch
static esp_status decode_check(const void* q, const void* k_pool, const void* v_pool, int64_t num_slots, const int32_t* slot_idx,
                               const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t max_len, int32_t Hq,
                               int32_t Hkv, int32_t D, float softmax_scale, const void* O, const float* LSE, bool* done) {
    *done = false;
    if (B < 0 || total_tokens < 0 || max_len < 0 || num_slots < 0)
        return fail(ESP_ERR_INVALID_ARG, "decode: negative size");
    if (!heads_ok(Hq, Hkv)) return fail(ESP_ERR_INVALID_ARG, "decode: Hq=%d must be a positive multiple of Hkv=%d", Hq, Hkv);
    if (D != kHeadDim) return fail(ESP_ERR_UNSUPPORTED, "decode: head_dim %d unsupported (only 128)", D);
    if (max_len > total_tokens) return fail(ESP_ERR_INVALID_ARG, "decode: max_len exceeds total_tokens");
    if (B == 0) { *done = true; return ESP_OK; }
    if (!q || !O || !LSE || !seq_offsets) return fail(ESP_ERR_INVALID_ARG, "decode: null q/seq_offsets/O/LSE");
    if (total_tokens > 0 && (!k_pool || !v_pool || !slot_idx || num_slots == 0))
        return fail(ESP_ERR_INVALID_ARG, "decode: null pool/slot_idx");
    if (!(softmax_scale == softmax_scale) || softmax_scale < 0.f) return fail(ESP_ERR_INVALID_ARG, "decode: bad softmax_scale");
    if (!decode_heads_supported(Hq, Hkv))
        return fail(ESP_ERR_UNSUPPORTED, "decode: Hq=%d, Hkv=%d unsupported", Hq, Hkv);
    return ESP_OK;
}
static esp_status decode_validate(const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t max_len,
                                  int64_t num_slots, void* stream) {
    if (!debug_validate()) return ESP_OK;
    esp_status st = check_offsets("decode: seq_offsets", seq_offsets, B, total_tokens, max_len, (hipStream_t)stream);
    if (st == ESP_OK) st = check_slots("decode", slot_idx, total_tokens, num_slots, false, false, (hipStream_t)stream);
    return st;
}

esp_status esp_partial_attn_decode(const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
                                   const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B,
                                   int32_t total_tokens, int32_t max_len, int32_t Hq, int32_t Hkv, int32_t D,
                                   float softmax_scale, void* O, float* LSE, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    bool done;
    esp_status st = decode_check(q, k_pool, v_pool, num_slots, slot_idx, seq_offsets, B, total_tokens, max_len, Hq, Hkv, D,
                                 softmax_scale, O, LSE, &done);
    if (st != ESP_OK || done) return st;
    size_t need = decode_workspace_bytes(B, total_tokens, Hq, Hkv);
    if (!workspace || workspace_bytes < need)
        return fail(ESP_ERR_WORKSPACE, "decode: workspace needs %zu bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if ((uintptr_t)workspace & 255) return fail(ESP_ERR_WORKSPACE, "decode: workspace not 256-byte aligned");
    st = decode_validate(slot_idx, seq_offsets, B, total_tokens, max_len, num_slots, stream);
    if (st != ESP_OK) return st;
    return launch_decode(q, k_pool, v_pool, slot_idx, seq_offsets, B, total_tokens, Hq, Hkv, softmax_scale, O, LSE,
                         workspace, workspace_bytes, (hipStream_t)stream);
}

esp_status esp_partial_attn_decode_static(const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
                                          const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B,
                                          int32_t total_tokens, int32_t max_len, int32_t Hq, int32_t Hkv, int32_t D,
                                          float softmax_scale, void* O, float* LSE, void* stream) {
    bool done;
    esp_status st = decode_check(q, k_pool, v_pool, num_slots, slot_idx, seq_offsets, B, total_tokens, max_len, Hq, Hkv, D,
                                 softmax_scale, O, LSE, &done);
    if (st != ESP_OK || done) return st;
    st = decode_validate(slot_idx, seq_offsets, B, total_tokens, max_len, num_slots, stream);
    if (st != ESP_OK) return st;
    return launch_decode_static(q, k_pool, v_pool, slot_idx, seq_offsets, B, total_tokens, Hq, Hkv, softmax_scale, O, LSE,
                                (hipStream_t)stream);
}

esp_status esp_partial_attn_decode_merge(const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
                                         const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B,
                                         int32_t total_tokens, int32_t max_len, int32_t Hq, int32_t Hkv, int32_t D,
                                         float softmax_scale, const void* const* peer_O, const float* const* peer_LSE,
                                         int32_t n_peers, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    if (n_peers < 0 || n_peers > ESP_MAX_PARTIALS - 1)
        return fail(ESP_ERR_INVALID_ARG, "decode (merge): n_peers=%d outside 0..%d", n_peers, ESP_MAX_PARTIALS - 1);
    bool done;
    esp_status st = decode_check(q, k_pool, v_pool, num_slots, slot_idx, seq_offsets, B, total_tokens, max_len, Hq, Hkv, D,
                                 softmax_scale, O, LSE, &done);
    if (st != ESP_OK || done) return st;
    MergeArgs peers = {};
    if (n_peers > 0) {
        if (!peer_O || !peer_LSE) return fail(ESP_ERR_INVALID_ARG, "decode (merge): null pointer arrays");
        const size_t o_bytes = (size_t)B * Hq * kHeadDim * 2, l_bytes = (size_t)B * Hq * 4;
        for (int p = 0; p < n_peers; ++p) {
            if (!peer_O[p] || !peer_LSE[p]) return fail(ESP_ERR_INVALID_ARG, "decode (merge): null partial %d", p);
            if (((uintptr_t)peer_O[p] & 3) || ((uintptr_t)peer_LSE[p] & 3))
                return fail(ESP_ERR_INVALID_ARG, "decode (merge): partial %d not 4-byte aligned", p);
            const char *a = (const char*)peer_O[p], *b = (const char*)peer_LSE[p];
            if ((a < (const char*)O + o_bytes && (const char*)O < a + o_bytes) ||
                (b < (const char*)LSE + l_bytes && (const char*)LSE < b + l_bytes))
                return fail(ESP_ERR_INVALID_ARG, "decode (merge): the output overlaps partial %d", p);
            peers.O_parts[p] = peer_O[p];
            peers.LSE_parts[p] = peer_LSE[p];
        }
    }
    size_t need = decode_workspace_bytes(B, total_tokens, Hq, Hkv);
    if (!workspace || workspace_bytes < need)
        return fail(ESP_ERR_WORKSPACE, "decode: workspace needs %zu bytes, got %zu", need, workspace ? workspace_bytes : (size_t)0);
    if ((uintptr_t)workspace & 255) return fail(ESP_ERR_WORKSPACE, "decode: workspace not 256-byte aligned");
    st = decode_validate(slot_idx, seq_offsets, B, total_tokens, max_len, num_slots, stream);
    if (st != ESP_OK) return st;
    return launch_decode(q, k_pool, v_pool, slot_idx, seq_offsets, B, total_tokens, Hq, Hkv, softmax_scale, O, LSE,
                         workspace, workspace_bytes, (hipStream_t)stream, &peers, n_peers);
}

static esp_status merge_entry(const void* const* O_parts, const float* const* LSE_parts, int32_t P, int32_t T,
                              int32_t Hq, int32_t D, int32_t parts_f32, void* O, float* LSE_out, void* stream) {
    if (P < 1 || P > ESP_MAX_PARTIALS) return fail(ESP_ERR_INVALID_ARG, "merge: P=%d outside 1..%d", P, ESP_MAX_PARTIALS);
    if (T < 0 || Hq <= 0) return fail(ESP_ERR_INVALID_ARG, "merge: negative size");
    if (D != kHeadDim) return fail(ESP_ERR_UNSUPPORTED, "merge: head_dim %d unsupported (only 128)", D);
    if (!O_parts || !LSE_parts) return fail(ESP_ERR_INVALID_ARG, "merge: null pointer arrays");
    if (T == 0) return ESP_OK;
    if (!O) return fail(ESP_ERR_INVALID_ARG, "merge: null O");
    MergeArgs a;
    for (int p = 0; p < P; ++p) {
        if (!O_parts[p] || !LSE_parts[p]) return fail(ESP_ERR_INVALID_ARG, "merge: partial %d is null", p);
        a.O_parts[p] = O_parts[p];
        a.LSE_parts[p] = LSE_parts[p];
    }
    for (int p = P; p < ESP_MAX_PARTIALS; ++p) { a.O_parts[p] = nullptr; a.LSE_parts[p] = nullptr; }
    return launch_merge(a, P, (int64_t)T * Hq, parts_f32, O, LSE_out, (hipStream_t)stream);
}

esp_status esp_merge_partials(const void* const* O_parts, const float* const* LSE_parts, int32_t P, int32_t T,
                              int32_t Hq, int32_t D, void* O, float* LSE_out, void* stream) {
    return merge_entry(O_parts, LSE_parts, P, T, Hq, D, 0, O, LSE_out, stream);
}

esp_status esp_merge_partials_f32(const float* const* O_parts, const float* const* LSE_parts, int32_t P, int32_t T,
                                  int32_t Hq, int32_t D, void* O, float* LSE_out, void* stream) {
    for (int p = 0; O_parts && p < P && p < ESP_MAX_PARTIALS; ++p)
        if (O_parts[p] == O && O) return fail(ESP_ERR_INVALID_ARG, "merge: the bf16 output must not alias an fp32 partial");
    return merge_entry((const void* const*)O_parts, LSE_parts, P, T, Hq, D, 1, O, LSE_out, stream);
}

esp_status esp_kv_append(const void* k, const void* v, const int32_t* slot_idx, int32_t T, void* k_pool, void* v_pool,
                         int64_t num_slots, int32_t Hkv, int32_t D, void* stream) {
    if (T < 0 || num_slots < 0 || Hkv <= 0) return fail(ESP_ERR_INVALID_ARG, "append: negative size");
    if (D != kHeadDim) return fail(ESP_ERR_UNSUPPORTED, "append: head_dim %d unsupported (only 128)", D);
    if (T == 0) return ESP_OK;
    if (!k || !v || !slot_idx || !k_pool || !v_pool) return fail(ESP_ERR_INVALID_ARG, "append: null pointer");
    if (num_slots == 0) return fail(ESP_ERR_INVALID_ARG, "append: empty pool");
    if (debug_validate()) {
        esp_status st = check_slots("append", slot_idx, T, num_slots, true, true, (hipStream_t)stream);
        if (st != ESP_OK) return st;
    }
    return launch_kv_append(k, v, slot_idx, T, k_pool, v_pool, Hkv * D * 2, (hipStream_t)stream);
}

}  // extern "C"

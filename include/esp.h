/*
 * esp.h -- C ABI of libesp: one GPU's share of elastic-sequence-parallel (ESP)
 * attention on AMD MI355X (gfx950), after LoongServe (arXiv 2404.09526).
 *
 * The library computes, with hand-written HIP kernels only (there is no CPU or
 * library fallback):
 *   esp_partial_attn_prefill  a causal query chunk against ONE local KV shard
 *   esp_partial_attn_decode   one query token per request against the KV rows
 *                             this instance holds in its token-granular pool
 *   esp_merge_partials        log-sum-exp combination of partial results
 *   esp_kv_append             scatter of K/V rows into scheduler-chosen slots
 * and, on the host, the scheduler's two numeric helpers for the prefill phase:
 *   esp_plan_prefill_batches  batching plan (dynamic program over requests and instances)
 *   esp_fit_prefill_model     least-squares fit of the iteration-time model
 *
 * Conventions common to all calls
 *   - Every data pointer is DEVICE memory owned by the caller unless a
 *     parameter says "host".  The library never allocates, frees or keeps
 *     device memory.  Its only state between calls is process-wide and small:
 *     a launch counter that tags the prefill workspace (see there) and the two
 *     debugging switches at the end of this file.
 *   - bf16 tensors are passed as `const void*` (16-bit patterns); layouts are
 *     token-major and dense: Q/O [T, Hq, D], K/V [T, Hkv, D], pools
 *     [S, Hkv, D] (one for K, one for V), LSE [T, Hq] float.
 *   - Query head h reads KV head h / (Hq / Hkv).  D must be 128.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Work is enqueued asynchronously; the library never synchronises.
 *   - Results are deterministic: the same inputs give the same bits.
 *   - Return value: ESP_OK or a negative esp_status; nothing is enqueued when
 *     an error is returned, except for ESP_ERR_HIP where the launch itself
 *     failed.  esp_last_error() gives a thread-local message.
 *   - The CONTENT of device index arrays (positions, offsets, slots) is
 *     trusted, as it comes from the scheduler (scaling plan, Sec. 3 and 4.1):
 *     out-of-range or duplicate slots are undefined behaviour.  With
 *     ESP_DEBUG_VALIDATE=1 in the environment the calls check them first, on
 *     the host (the stream is waited for and the arrays are copied back; a
 *     debugging aid): prefix offsets must run from 0 to the row count without
 *     decreasing, with no piece above the stated maximum; decode slots must lie
 *     in [0, num_slots); append slots must be below num_slots and, where not
 *     negative, distinct.  A violation returns ESP_ERR_INVALID_ARG.
 *   - A row with no visible key yields O = 0 and LSE = -inf, never NaN.
 *   - LSE is the natural logarithm of the sum of exp(softmax_scale * q.k)
 *     over the visible keys.
 */
#ifndef ESP_H_
#define ESP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t esp_status;
#define ESP_OK                0
#define ESP_ERR_INVALID_ARG  (-1) /* null pointer, negative size, Hq % Hkv != 0, P out of range */
#define ESP_ERR_UNSUPPORTED  (-2) /* D != 128                                                   */
#define ESP_ERR_WORKSPACE    (-3) /* workspace missing or smaller than the matching *_bytes()  */
#define ESP_ERR_HIP          (-4) /* a HIP launch failed; see esp_last_error()                 */

#define ESP_MAX_PARTIALS 16

/*
 * Prefill partial attention (Sec. 2.3, Fig. 1: instance i attends its local
 * queries q_i to a key-value segment kv_j; kernel remarks in Sec. 6).
 *
 * For every local query row t and head h: softmax attention over the rows of
 * ONE KV shard that belong to the same request, restricted (causal != 0) to
 * rows with kv_pos <= q_pos[t] on GLOBAL token positions, so that contiguous,
 * striped or arbitrary sequence-parallel layouts use the same call.  Emits the
 * un-merged output O (bf16, normalised within the shard) and LSE (float).
 *
 *   q [Tq,Hq,D], k/v [Tkv,Hkv,D] bf16; q_pos [Tq], kv_pos [Tkv] int32.
 *   cu_q, cu_kv: int32 [batch+1] prefix offsets of the requests packed in q and
 *     in the shard (request r owns rows cu[r]..cu[r+1]); both NULL with
 *     batch = 1 means one request spanning everything.
 *   max_q, max_kv: upper bounds on a request's row counts (host-known; used
 *     only to size the launch).
 *   O [Tq,Hq,D] bf16, LSE [Tq,Hq] float: written for every row.
 *   workspace: at least esp_prefill_workspace_bytes(...) bytes, 256-byte
 *     aligned; contents need not be preserved between calls.  It holds work
 *     counters that are never cleared: every launch tags them with a number of
 *     its own (a per-process random 32-bit start, then +1 per call), so memory
 *     that has never been written is mistaken for the current launch's counters
 *     with probability 2^-32 per fresh workspace (query tiles would then be
 *     skipped).  A caller that wants certainty zeroes a new workspace once:
 *     the tag is never 0.  Calls that may run at the same time need a
 *     workspace each.
 * Positions may be in any order; ascending order inside a request lets whole
 * tiles be skipped or left unmasked.
 */
esp_status esp_partial_attn_prefill(
    const void* q, const void* k, const void* v,
    const int32_t* q_pos, const int32_t* kv_pos,
    const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
    int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale, int32_t causal,
    void* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

size_t esp_prefill_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch,
                                   int32_t Hq, int32_t Hkv, int32_t D);

/*
 * The same call with O [Tq,Hq,D] written as float: for partials that stay on this
 * GPU until they are combined (the rounds of sequence-parallel prefill, Sec. 2.3:
 * one call per key-value segment that passes by, one combination at the end), so
 * that the combined result is rounded to bf16 once, by esp_merge_partials_f32,
 * and not once per partial and again after the combination.  Everything else,
 * the workspace included, as in esp_partial_attn_prefill.
 */
esp_status esp_partial_attn_prefill_f32(
    const void* q, const void* k, const void* v,
    const int32_t* q_pos, const int32_t* kv_pos,
    const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
    int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale, int32_t causal,
    float* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Decode partial attention (Sec. 4.2, Fig. 8: every instance of the group runs
 * the local attention of the batch's query tokens against the key-value rows it
 * holds; token-granular pool of Sec. 6).
 *
 * Request b attends its single query token to the pool rows
 * slot_idx[seq_offsets[b] .. seq_offsets[b+1]) (no mask: all resident tokens
 * precede the query).  A request with no resident row gives O = 0, LSE = -inf.
 *
 *   q [B,Hq,D] bf16; k_pool/v_pool [num_slots,Hkv,D] bf16;
 *   slot_idx int32 [total_tokens]; seq_offsets int32 [B+1], seq_offsets[0] = 0,
 *   seq_offsets[B] = total_tokens; max_len >= every request's length.
 *   O [B,Hq,D] bf16, LSE [B,Hq] float.
 *   workspace: at least esp_decode_workspace_bytes(...) bytes, 256-byte aligned.
 * Every Hq that is a multiple of Hkv is accepted (MHA, GQA, MQA).  With 4, 8, 16 or
 * a multiple of 32 KV heads and 1 or 2 query heads per KV head a pool row is read
 * in whole-row bursts and multiplied on the vector ALU; every other layout is read
 * one KV head (256 bytes of a row) at a time and multiplied on the matrix cores,
 * the query heads of a KV head as the columns of a tile.
 */
esp_status esp_partial_attn_decode(
    const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
    const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B,
    int32_t total_tokens, int32_t max_len,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
    void* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

size_t esp_decode_workspace_bytes(int32_t B, int32_t total_tokens, int32_t max_len,
                                  int32_t Hq, int32_t Hkv, int32_t D);

/*
 * esp_partial_attn_decode for callers that cannot allocate or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernels, minus the workspace:
 * the split-K partials go to a block of ESP_DECODE_STATIC_SCRATCH_BYTES of
 * device memory built into the library (each GPU the library runs on holds it
 * until the process ends).  The call allocates and frees nothing.  A call whose
 * esp_decode_workspace_bytes(...) exceeds the block returns ESP_ERR_WORKSPACE.
 * All calls on one GPU share the block: calls that may overlap in time on one
 * GPU (two streams, two threads) race and must use esp_partial_attn_decode
 * with a workspace each.  Nothing in the block has to be cleared between calls.
 */
#define ESP_DECODE_STATIC_SCRATCH_BYTES (32u << 20)
esp_status esp_partial_attn_decode_static(
    const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
    const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B,
    int32_t total_tokens, int32_t max_len,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
    void* O, float* LSE, void* stream);

/*
 * The master's step of a multi-master decode (Sec. 4.2): its local partial
 * attention over the token pool, combined in the same pass with the partial
 * results its peers sent back for the same queries (the combination stated
 * below for esp_merge_partials, with the local result as one more partial).
 * The local result is never rounded to bf16 on its own and no separate merge
 * launch follows.  Arguments as esp_partial_attn_decode, plus
 *   peer_O   : HOST array of n_peers DEVICE pointers, each bf16 [B, Hq, D];
 *   peer_LSE : HOST array of n_peers DEVICE pointers, each fp32 [B, Hq];
 *   n_peers  : 0 .. ESP_MAX_PARTIALS - 1 (0: plain esp_partial_attn_decode).
 * The pointer arrays are read during the call only.  O / LSE receive the
 * FINAL result and must not overlap a peer's arrays (ESP_ERR_INVALID_ARG).
 * A master that holds no token of a request (seq_offsets[b+1] ==
 * seq_offsets[b]) passes its peers' combination through.  Errors as
 * esp_partial_attn_decode.
 */
esp_status esp_partial_attn_decode_merge(
    const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
    const int32_t* slot_idx, const int32_t* seq_offsets, int32_t B,
    int32_t total_tokens, int32_t max_len,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
    const void* const* peer_O, const float* const* peer_LSE, int32_t n_peers,
    void* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Combination of partial results ("generate the final output", Sec. 2.3;
 * results "sent back to the master", Sec. 4.2).  For each (token, head):
 *   m = max_p LSE_p,  w_p = exp(LSE_p - m),
 *   O = sum_p w_p O_p / sum_p w_p,   LSE = m + ln sum_p w_p.
 * Partials with LSE = -inf weigh 0; all -inf gives O = 0, LSE = -inf.
 *
 *   O_parts, LSE_parts: HOST arrays of P device pointers (1 <= P <=
 *     ESP_MAX_PARTIALS) to bf16 [T,Hq,D] and float [T,Hq]; read before return.
 *   O [T,Hq,D] bf16; LSE_out [T,Hq] float or NULL.  O may alias O_parts[i].
 */
esp_status esp_merge_partials(
    const void* const* O_parts, const float* const* LSE_parts, int32_t P,
    int32_t T, int32_t Hq, int32_t D,
    void* O, float* LSE_out, void* stream);

/*
 * The same combination of float partials (O_parts[p]: float [T,Hq,D], as
 * esp_partial_attn_prefill_f32 writes them); O is still bf16 and must not alias
 * a partial.
 */
esp_status esp_merge_partials_f32(
    const float* const* O_parts, const float* const* LSE_parts, int32_t P,
    int32_t T, int32_t Hq, int32_t D,
    void* O, float* LSE_out, void* stream);

/*
 * KV append / selective retention (Sec. 4.1, Fig. 7: instances of the new
 * group save selected key-value rows into their pool at the places the scaling
 * plan names; Sec. 4.2: a master saves the new token's K/V into its pool).
 *   k_pool[slot_idx[t]] = k[t], v_pool[slot_idx[t]] = v[t] for slot_idx[t] >= 0;
 *   rows with a negative slot are not kept.  A pure copy of 16-bit patterns.
 *
 *   k, v [T,Hkv,D] bf16; slot_idx int32 [T]; pools [num_slots,Hkv,D] bf16.
 */
esp_status esp_kv_append(
    const void* k, const void* v, const int32_t* slot_idx, int32_t T,
    void* k_pool, void* v_pool, int64_t num_slots, int32_t Hkv, int32_t D,
    void* stream);

/*
 * Prefill partial attention that keeps rows of the shard on the way (proactive
 * scale-down, Sec. 4.1, Fig. 7: while the key-value segments circulate during
 * prefill, every instance of the new, smaller group saves the rows the scaling
 * plan assigns to it into its pool, so that no migration is needed afterwards;
 * overhead claim of Sec. 7.4, Fig. 14).  The attention part is
 * esp_partial_attn_prefill (out_f32 != 0: esp_partial_attn_prefill_f32, O then
 * points to float); in the same pass
 *   k_pool[retain_slot[t]] = k[t], v_pool[retain_slot[t]] = v[t]
 * for every shard row t with retain_slot[t] >= 0, as esp_kv_append would do, but
 * from the tiles that pass through on-chip memory anyway: the rows are read from
 * device memory once.  Rows of requests that have no query row in this call, and
 * rows no query can see, are kept all the same.  With Tq = 0 the call is a plain
 * esp_kv_append.
 *
 *   retain_slot int32 [Tkv] (device); pools [num_slots,Hkv,D] bf16; slots that are
 *   not negative must be distinct and below num_slots (checked only under
 *   esp_debug_set_validate).  Everything else as in esp_partial_attn_prefill.
 */
esp_status esp_partial_attn_prefill_retain(
    const void* q, const void* k, const void* v,
    const int32_t* q_pos, const int32_t* kv_pos,
    const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
    int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale, int32_t causal,
    const int32_t* retain_slot, void* k_pool, void* v_pool, int64_t num_slots,
    int32_t out_f32, void* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Dense view of pool-resident rows: the inverse of esp_kv_append.  The key-value
 * rows a request keeps on this instance live in the token-granular pool at the
 * slots the scheduler chose (Sec. 4.1, Fig. 7; Sec. 6 "unified distributed
 * key-value cache pool"); a later prefill pass over them (the next chunk of a
 * long prompt, a follow-up turn) needs them as one shard.
 *   k[t] = k_pool[slot_idx[t]], v[t] = v_pool[slot_idx[t]]; a slot that is negative
 *   or not below num_slots gives a row of zeros.  A pure copy of 16-bit patterns.
 *
 *   pools [num_slots,Hkv,D] bf16; slot_idx int32 [T]; k, v [T,Hkv,D] bf16 (written).
 */
esp_status esp_kv_gather(
    const void* k_pool, const void* v_pool, const int32_t* slot_idx, int32_t T,
    int64_t num_slots, int32_t Hkv, int32_t D, void* k, void* v, void* stream);

/*
 * esp_partial_attn_prefill over a shard that lives in the pool: row i of the
 * shard is pool row slot_idx[i] (kv_pos[i] is its global position; cu_kv counts
 * shard rows, i.e. entries of slot_idx).  Same results as esp_kv_gather followed
 * by esp_partial_attn_prefill, which is how it is carried out: the gathered rows
 * are staged in the workspace (2 * Tkv * Hkv * D * 2 bytes on top of the dense
 * call's own block).  All other arguments as in esp_partial_attn_prefill.
 */
esp_status esp_partial_attn_prefill_pool(
    const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
    const int32_t* slot_idx, const int32_t* q_pos, const int32_t* kv_pos,
    const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
    int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale, int32_t causal,
    void* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

size_t esp_prefill_pool_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch,
                                        int32_t Hq, int32_t Hkv, int32_t D);

/*
 * The same without staging: the kernel's tile transfers take every row from
 * its pool slot (the slots of a tile travel to on-chip memory one step ahead
 * of the tile, each lane forms the address of the row its 16 bytes belong
 * to), so nothing is copied first and the workspace is the dense call's,
 * esp_prefill_workspace_bytes(...).  Sec. 4.1 / 4.2: key-value rows that an
 * instance kept stay at the slots they were placed in.  Arguments as
 * esp_partial_attn_prefill_pool, plus out_f32 (0: O is bf16; else fp32, as in
 * esp_partial_attn_prefill_f32).  Every slot_idx[i] must lie in
 * [0, num_slots): the kernel trusts it (checked on the host only while
 * esp_debug_set_validate is on).  Results equal those of the staged call up to
 * the order of fp32 additions (the same bound against the exact result holds).
 */
esp_status esp_partial_attn_prefill_pool_direct(
    const void* q, const void* k_pool, const void* v_pool, int64_t num_slots,
    const int32_t* slot_idx, const int32_t* q_pos, const int32_t* kv_pos,
    const int32_t* cu_q, const int32_t* cu_kv, int32_t batch,
    int32_t Tq, int32_t Tkv, int32_t max_q, int32_t max_kv,
    int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale, int32_t causal,
    int32_t out_f32, void* O, float* LSE,
    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aids (no part of the method): what this GPU sustains on the two
 * resources that bound the path, for the benchmark's "achievable" figures.
 *   esp_probe_mfma_bf16: every wavefront (8 per CU, all CUs) runs `iters` rounds of
 *     four independent 32x32x16 bf16 MFMAs on register operands taken from
 *     `operands` (device, 16-byte aligned, operand_bytes a multiple of 16; the
 *     values decide how much the multipliers switch, hence the clock under the
 *     power limit).  *flops (host, nullable) receives the FLOPs of the launch.
 *   esp_probe_stream_read: reads `bytes` (a multiple of 16) of device memory once.
 *   sink: 4 bytes of device memory (written only in a case that does not occur).
 */
esp_status esp_probe_mfma_bf16(const void* operands, int64_t operand_bytes, int32_t iters,
                               void* sink, int64_t* flops, void* stream);
esp_status esp_probe_stream_read(const void* src, int64_t bytes, void* sink, void* stream);

/*
 * Prefill batching plan (Sec. 5.3 "Batching", the dynamic program over sorted requests and sorted elastic
 * instances) -- host code, no GPU work; every pointer is HOST memory.
 *
 * Requests are given longest first (req_len[0] >= req_len[1] >= ... >= 1 tokens), instances in the scheduler's
 * order with their unused key-value slots.  A plan cuts the requests and a prefix of the instances into the same
 * number of consecutive non-empty pieces; batch b = requests [req_cuts[b-1], req_cuts[b]) on instances
 * [inst_cuts[b-1], inst_cuts[b]) (cuts start at 0), and must fit: its tokens <= the unused slots of its instances.
 * A batch costs sum over its requests of T / len, with T the iteration-time model below at the coefficients of
 * its degree of parallelism d = its number of instances: coefs[3*(d-1) .. 3*(d-1)+2] = alpha, beta, gamma.
 * The plan of least total cost is returned: *n_batches pieces, their end cuts in req_cuts / inst_cuts (room for
 * min(n_req, n_inst) entries each), the cost in *cost.  If nothing fits, *n_batches = 0 and *cost = +inf.
 * split_req / split_ins: NULL, or [(n_req+1) x (n_inst+1)] tables that receive, for the first i requests on the
 * first k instances, where the last batch starts (the two monotone tables of the section; -1 = no plan).
 */
esp_status esp_plan_prefill_batches(
    const int64_t* req_len, int32_t n_req, const int64_t* free_slots, int32_t n_inst,
    const double* coefs, int32_t* req_cuts, int32_t* inst_cuts, int32_t* n_batches, double* cost,
    int32_t* split_req, int32_t* split_ins);

/*
 * The same plan searched with the monotone split points of Eq. 6 (Sec. 5.3): the search for the last batch of
 * (first i requests, first k instances) starts at split_req[i][k-1] and split_ins[i-1][k] instead of at 0.  The
 * section states the monotonicity as a property; under the cost read here (see esp_plan_prefill_batches) it holds
 * in about three random instances in four, so this is a heuristic: the result is a valid plan (a cell with nothing
 * feasible inside the bounds is searched in full) whose cost is never below the exhaustive search's, equal to it
 * where the property holds, and up to a few times higher where it does not.  The exhaustive search stays the
 * default; the section itself calls it fast enough.  Same arguments and outputs.
 */
esp_status esp_plan_prefill_batches_monotone(
    const int64_t* req_len, int32_t n_req, const int64_t* free_slots, int32_t n_inst,
    const double* coefs, int32_t* req_cuts, int32_t* inst_cuts, int32_t* n_batches, double* cost,
    int32_t* split_req, int32_t* split_ins);

/*
 * Iteration-time model of the prefill phase (Sec. 5.5 "Optimizations", analytical model based on SIB, Eq. 7):
 *   T(R) = alpha + beta * sum_{r in R} len_r + gamma * sum_{r in R} len_r^2,
 * fitted by least squares to n >= 3 profiled batches (HOST arrays: per batch the two sums and the measured
 * time).  weights: NULL, or n non-negative factors; sample i's equation is multiplied by weights[i] before the
 * fit (1 / seconds[i] minimises the relative instead of the absolute residual).  coef receives alpha, beta,
 * gamma; a column without information (all zero) gets coefficient 0.
 */
esp_status esp_fit_prefill_model(
    const double* sum_len, const double* sum_len_sq, const double* seconds, const double* weights, int32_t n,
    double* coef);

/*
 * Debugging switches (process-wide; each returns the previous setting).
 *   esp_debug_set_validate: the host-side check of device index arrays described at
 *     the top (default: ESP_DEBUG_VALIDATE in the environment, read once at load time).
 *   esp_debug_set_prefill_sync_ticks: the longest time, in ticks of the 100 MHz wall
 *     clock, that prefill workgroups sharing a key-value head wait for each other at
 *     the start of a round (default 15000, or ESP_PREFILL_SYNC_TICKS read once at load
 *     time; 0 makes every such wait give up at once; negative restores the default).
 *     It changes timing only, never results.
 */
int32_t esp_debug_set_validate(int32_t on);
int32_t esp_debug_set_prefill_sync_ticks(int32_t ticks);

/* Message of the last error on the calling thread (static storage, never NULL). */
const char* esp_last_error(void);

/* Library version string, e.g. "esp 0.1 gfx950". */
const char* esp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ESP_H_ */

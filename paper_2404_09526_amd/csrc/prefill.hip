// esp_partial_attn_prefill: a causal query chunk against ONE local key-value shard, masked by
// global token position (sequence-parallel prefill, Sec. 2.3 / Fig. 1: instance i attends its
// local q_i to the segment kv_j of the current round; striped layout and tile-skipping remarks
// in Sec. 6).  Emits the un-merged output, normalised within the shard, and its log-sum-exp.
//
// Mapping to gfx950 (64-wide wavefronts, MFMA 32x32x16 bf16, 160 KiB LDS):
//   * a workgroup of 8 wavefronts owns 256 query rows of one head; each wavefront owns 32 rows
//     and keeps their Q fragment (B operand), running max / sum and the fp32 output
//     accumulator in registers for the whole KV sweep;
//   * K/V tiles of 64 rows go through LDS, double buffered; the K tile is the A operand of
//     S^T = K Q^T, so a lane ends up with scores of ONE query row (its column) and the row
//     statistics need one cross-half exchange only; P^T stays in registers and is the B operand
//     of O^T = V^T P^T, whose A operand comes from transposing LDS reads of the row-major V tile;
//   * 16-byte chunks are XOR-swizzled inside each 256-byte LDS row (differently for K and V) so
//     that the operand reads spread over all banks;
//   * per (workgroup, KV tile) the minimum / maximum positions decide: tile hidden -> skipped
//     without being loaded; tile fully visible -> no mask code; else element-wise kv_pos <= q_pos.
#include <limits.h>

#include "esp_common.h"

namespace esp {

constexpr int kBM = 256;   // query rows per workgroup
constexpr int kBN = 64;    // KV rows per tile
constexpr int kPfWaves = 8;
constexpr int kTileBytes = kBN * kHeadDim * 2;   // 16 KiB

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4_t;
#define ESP_LDS __attribute__((address_space(3)))

static int32_t prefill_kv_tiles_bound(int32_t Tkv, int32_t batch) { return Tkv / kBN + batch; }
static int32_t prefill_q_tiles_bound(int32_t Tq, int32_t batch) { return Tq / kBM + batch; }

size_t prefill_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch, int32_t Hq, int32_t Hkv) {
    (void)Tq; (void)Hq; (void)Hkv;
    return (size_t)prefill_kv_tiles_bound(Tkv, batch) * sizeof(int2) + 256;
}

// min / max position of every 64-row KV tile of every request: tile_mm[first_tile(r) + t]
__global__ __launch_bounds__(64) void kv_tile_minmax_kernel(const int32_t* __restrict__ kv_pos,
                                                            const int32_t* __restrict__ cu_kv, int32_t Tkv,
                                                            int2* __restrict__ tile_mm) {
    const int r = blockIdx.y, t = blockIdx.x, lane = threadIdx.x;
    int first = 0;
    for (int i = 0; i < r; ++i) first += (cu_kv[i + 1] - cu_kv[i] + kBN - 1) / kBN;
    const int lo = cu_kv ? cu_kv[r] : 0, hi = cu_kv ? cu_kv[r + 1] : Tkv;
    if (t >= (hi - lo + kBN - 1) / kBN) return;
    int row = lo + t * kBN + lane;
    int mn = INT_MAX, mx = INT_MIN;
    if (row < hi) mn = mx = kv_pos[row];
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        mn = min(mn, __shfl_xor(mn, s));
        mx = max(mx, __shfl_xor(mx, s));
    }
    if (lane == 0) tile_mm[first + t] = make_int2(mn, mx);
}

struct PrefillArgs {
    const uint16_t* q; const uint16_t* k; const uint16_t* v;
    const int32_t* q_pos; const int32_t* kv_pos; const int32_t* cu_q; const int32_t* cu_kv;
    const int2* tile_mm;
    uint16_t* O; float* LSE;
    int32_t batch, Tq, Tkv, Hq, Hkv, causal;
    float scale_log2;
};

// Both halves of the wavefront exchange a value: lo = value held by lane l & 31, hi = value held by
// lane l | 32.  v_permlane32_swap exchanges the upper half of its first register with the lower half of
// its second.  It is issued as inline assembly: with equal operands the compiler's own intrinsic gets
// folded as if both results were the same value.
__device__ __forceinline__ void half_pair(float x, float& lo, float& hi) {
    int a = __builtin_bit_cast(int, x), b = a;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    lo = __builtin_bit_cast(float, a);
    hi = __builtin_bit_cast(float, b);
}
__device__ __forceinline__ float half_swap_max(float x) {
    float lo, hi;
    half_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float half_swap_sum(float x) {
    float lo, hi;
    half_pair(x, lo, hi);
    return lo + hi;
}

// LDS barrier that does not wait for outstanding global loads (the prefetch of a later tile stays
// in flight across it): LDS traffic of this wavefront is drained, then the workgroup meets.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

constexpr int kStages = 3;          // LDS stages per operand; tile j of the visible sequence lives in stage j % 3
constexpr float kRescaleStep = 8.f; // the running max is refreshed only when it grows by more than 2^8

// Schedule inside a workgroup: the two wavefronts that share a SIMD (w and w + 4) run half an iteration
// apart.  While one is in its matrix phase (O^T += V^T P^T of tile i, then S^T = K Q^T of tile i + 1) the
// other is in its vector phase (mask, running max, exp2, row sum, bf16 pack of its tile), so the MFMA pipe
// and the vector ALU of the SIMD are busy at the same time.  Phases are separated by workgroup barriers;
// group B (wavefronts 4-7) passes one extra barrier before its loop and group A one after it.
__global__ __launch_bounds__(kPfWaves * 64) void prefill_kernel(PrefillArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char lds_k[kStages][kTileBytes];
    __shared__ __attribute__((aligned(16))) unsigned char lds_v[kStages][kTileBytes];
    __shared__ __attribute__((aligned(16))) int32_t lds_pos[kStages][kBN];
    __shared__ int32_t lds_qmm[2][kPfWaves];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool group_b = wave >= kPfWaves / 2;
    const int G = a.Hq / a.Hkv;

    // ---- which (query tile, head): XCD-aware (consecutive workgroup ids land on consecutive
    //      XCDs, each with a private L2, so a KV head stays on one XCD), heaviest tiles first
    int rank, h;
    {
        const int bid = blockIdx.x;
        if (a.Hkv % 8 == 0) {
            const int per = (a.Hkv / 8) * G;        // query heads per XCD
            const int xcd = bid & 7, i = bid >> 3;
            rank = i / per;
            h = xcd * per + i % per;
        } else {
            rank = bid / a.Hq;
            h = bid % a.Hq;
        }
    }
    const int kvh = h / G;
    int q_lo, q_hi, kv_lo, kv_hi, tile0;   // rows of this query tile; rows and first KV tile of its request
    {
        int total = 0;
        for (int r = 0; r < a.batch; ++r) {
            int len = a.cu_q ? a.cu_q[r + 1] - a.cu_q[r] : a.Tq;
            total += (len + kBM - 1) / kBM;
        }
        if (rank >= total) return;
        int tl = total - 1 - rank;   // later tiles of a causal request see more keys: run them first
        int r = 0, first_kv_tile = 0;
        for (;; ++r) {
            int len = a.cu_q ? a.cu_q[r + 1] - a.cu_q[r] : a.Tq;
            int nt = (len + kBM - 1) / kBM;
            if (tl < nt) break;
            tl -= nt;
            int kvlen = a.cu_kv ? a.cu_kv[r + 1] - a.cu_kv[r] : a.Tkv;
            first_kv_tile += (kvlen + kBN - 1) / kBN;
        }
        const int qs = a.cu_q ? a.cu_q[r] : 0, qe = a.cu_q ? a.cu_q[r + 1] : a.Tq;
        q_lo = qs + tl * kBM;
        q_hi = min(q_lo + kBM, qe);
        kv_lo = a.cu_kv ? a.cu_kv[r] : 0;
        kv_hi = a.cu_kv ? a.cu_kv[r + 1] : a.Tkv;
        tile0 = first_kv_tile;
    }
    const int nkt = (kv_hi - kv_lo + kBN - 1) / kBN;
    const bool ragged_tail = (kv_hi - kv_lo) % kBN != 0;

    // ---- this lane's query row (column of S^T) and its Q fragment
    const int qi = lane & 31, hi = lane >> 5;
    const int my_row = q_lo + wave * 32 + qi;
    const bool row_ok = my_row < q_hi;
    const int ld_row = row_ok ? my_row : q_hi - 1;
    bf16x8 qf[8];
    {
        const uint16_t* qp = a.q + ((int64_t)ld_row * a.Hq + h) * kHeadDim + 8 * hi;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[t] = *(const bf16x8*)(qp + 16 * t);
    }
    // effective query position: non-causal rows see every real key (the tail sentinel is INT_MAX)
    const int my_qpos = a.causal ? a.q_pos[ld_row] : INT_MAX - 1;
    int wave_qmin = my_qpos, wave_qmax = my_qpos;
#pragma unroll
    for (int s = 16; s >= 1; s >>= 1) {
        wave_qmin = min(wave_qmin, __shfl_xor(wave_qmin, s));
        wave_qmax = max(wave_qmax, __shfl_xor(wave_qmax, s));
    }
    wave_qmin = __builtin_amdgcn_readfirstlane(wave_qmin);
    wave_qmax = __builtin_amdgcn_readfirstlane(wave_qmax);
    if (lane == 0) { lds_qmm[0][wave] = wave_qmin; lds_qmm[1][wave] = wave_qmax; }
    __syncthreads();
    int wg_qmax = lds_qmm[1][0];
#pragma unroll
    for (int w = 1; w < kPfWaves; ++w) wg_qmax = max(wg_qmax, lds_qmm[1][w]);
    wg_qmax = __builtin_amdgcn_readfirstlane(wg_qmax);

    // ---- staging: thread -> two 16-byte chunks of the K tile and of the V tile
    const int st_row0 = tid >> 4, st_row1 = st_row0 + 32, st_ch = tid & 15;
    const uint32_t st_k0 = st_row0 * 256 + ((st_ch ^ (st_row0 & 15)) << 4);
    const uint32_t st_k1 = st_row1 * 256 + ((st_ch ^ (st_row1 & 15)) << 4);
    const uint32_t st_v0 = st_row0 * 256 + ((st_ch ^ ((st_row0 & 3) << 2)) << 4);
    const uint32_t st_v1 = st_row1 * 256 + ((st_ch ^ ((st_row1 & 3) << 2)) << 4);
    // global side: a uniform 64-bit base per tile (scalar registers) plus a per-thread 32-bit byte offset
    // that never changes, so fetching a tile costs no vector address arithmetic
    const uint32_t kv_row_bytes = (uint32_t)a.Hkv * kHeadDim * 2;
    const uint32_t g_off0 = st_row0 * kv_row_bytes + st_ch * 16, g_off1 = st_row1 * kv_row_bytes + st_ch * 16;
    const char* kreq = (const char*)a.k + ((int64_t)kv_lo * a.Hkv + kvh) * (kHeadDim * 2);   // row kv_lo, head kvh
    const char* vreq = (const char*)a.v + ((int64_t)kv_lo * a.Hkv + kvh) * (kHeadDim * 2);
    const int32_t* preq = a.kv_pos + kv_lo;

    // ---- operand read offsets
    // K (A operand of S^T): row 32*kvb + qi, chunk 2t + hi
    const uint32_t k_row = qi * 256, k_x = qi & 15;
    auto k_rd = [&](int t) { return k_row + (((2 * t + hi) ^ k_x) << 4); };
    // V (A operand of O^T) by transposing reads: 16 lanes fetch a 4 (kv) x 16 (d) patch
    const int j = lane & 15, jq = j >> 2, dblk = (lane >> 4) & 1;
    uint32_t v_rd[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_rd[db] = (4 * hi + jq) * 256 + ((((db ^ jq) << 2) + 2 * dblk + ((j & 3) >> 1)) << 4) + (j & 1) * 8;

    floatx16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_ref = -INFINITY;   // exponent offset in use (scale*log2(e)*score units); trails the true max by <= 2^8
    float lsum = 0.f;          // running sum of exp2 over this lane's half of the keys

    uint4 gk0, gk1, gv0, gv1;
    int gpos = INT_MAX;
    const int kv_len = kv_hi - kv_lo;
    auto load_tile = [&](int t) {
        t = __builtin_amdgcn_readfirstlane(t);
        const int64_t tile_off = (int64_t)t * kBN * kv_row_bytes;          // uniform
        const char* kt = kreq + tile_off;
        const char* vt = vreq + tile_off;
        uint32_t o0 = g_off0, o1 = g_off1;
        if (ragged_tail && t == nkt - 1) {    // rows past the end re-read the last row; their scores are masked
            const int last = kv_len - 1 - t * kBN;
            o0 = min(st_row0, last) * kv_row_bytes + st_ch * 16;
            o1 = min(st_row1, last) * kv_row_bytes + st_ch * 16;
        }
        gk0 = *(const uint4*)(kt + o0);
        gk1 = *(const uint4*)(kt + o1);
        gv0 = *(const uint4*)(vt + o0);
        gv1 = *(const uint4*)(vt + o1);
        if (tid < kBN) {
            int r = t * kBN + tid;
            gpos = r < kv_len ? preq[r] : INT_MAX;
        }
    };
    auto store_tile = [&](int st) {
        *(uint4*)(lds_k[st] + st_k0) = gk0;
        *(uint4*)(lds_k[st] + st_k1) = gk1;
        *(uint4*)(lds_v[st] + st_v0) = gv0;
        *(uint4*)(lds_v[st] + st_v1) = gv1;
        if (tid < kBN) lds_pos[st][tid] = gpos;
    };

    floatx16 sacc[2];          // S^T of the tile in flight, then its probabilities
    union PFrag { uint32_t u[4]; bf16x8 v; };
    PFrag pf[2][2];            // P^T packed to bf16: [kvb][t2]
    // per-tile facts, wavefront-uniform, from the tile's (min, max) position
    auto tile_needs_mask = [&](int t, int2 mm) {
        return (ragged_tail && t == nkt - 1) || (a.causal && mm.y > wave_qmin);
    };

    // Operand fragments are fetched from LDS in batches of four MFMAs, two batches ahead of their use,
    // so that the LDS latency hides behind the MFMAs of earlier batches.  Batches 0-3: V^T fragments of
    // O^T += V^T P^T (two transposing reads each); batches 4-7: K fragments of S^T = K Q^T.
    union VFrag { short4_t s[2]; bf16x8 v; };
    VFrag fr[2][4];
    auto read_batch = [&](int bi, int slot, int st_v, int st_k) {
        if (bi < 4) {
            const int kvb = bi >> 1, t2 = bi & 1;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const unsigned char* vp = lds_v[st_v] + (32 * kvb + 16 * t2) * 256 + v_rd[db];
                fr[slot][db].s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ESP_LDS short4_t*)(vp));
                fr[slot][db].s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ESP_LDS short4_t*)(vp + 8 * 256));
            }
        } else {
            const int tp = bi - 4;   // t = 2*tp, 2*tp + 1
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int t = 2 * tp + (x >> 1), kvb = x & 1;
                fr[slot][x].v = *(const bf16x8*)(lds_k[st_k] + kvb * 8192 + k_rd(t));
            }
        }
    };
    auto mfma_batch = [&](int bi, int slot) {
        if (bi < 4) {
            const int kvb = bi >> 1, t2 = bi & 1;
#pragma unroll
            for (int db = 0; db < 4; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[slot][db].v, pf[kvb][t2].v, oacc[db], 0, 0, 0);
        } else {
            const int tp = bi - 4;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int t = 2 * tp + (x >> 1), kvb = x & 1;
                sacc[kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[slot][x].v, qf[t], sacc[kvb], 0, 0, 0);
            }
        }
    };
    // runs batches [first, last); the fragments of the first `primed` batches are already in flight
    auto matrix_phase = [&](int first, int last, int primed, int st_v, int st_k) {
#pragma unroll
        for (int bi = first; bi < last; ++bi) {
            if (bi == first) {
#pragma unroll
                for (int pb = first + primed; pb < first + 2 && pb < last; ++pb) read_batch(pb, pb % 2, st_v, st_k);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (bi == 4)
#pragma unroll
                for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[kvb][r] = 0.f;
            mfma_batch(bi, bi % 2);
            if (bi + 2 < last) read_batch(bi + 2, bi % 2, st_v, st_k);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    auto softmax = [&](int st, bool need_mask) {
        if (need_mask) {
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    int4 kp = *(const int4*)(&lds_pos[st][32 * kvb + 8 * bb + 4 * hi]);
                    if (kp.x > my_qpos) sacc[kvb][4 * bb + 0] = -INFINITY;
                    if (kp.y > my_qpos) sacc[kvb][4 * bb + 1] = -INFINITY;
                    if (kp.z > my_qpos) sacc[kvb][4 * bb + 2] = -INFINITY;
                    if (kp.w > my_qpos) sacc[kvb][4 * bb + 3] = -INFINITY;
                }
        }
        float tmax = sacc[0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sacc[0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sacc[1][r]);
        tmax = half_swap_max(tmax) * a.scale_log2;
        // refresh the exponent offset only when the row max outgrew it by more than 2^8 (or at the first
        // visible key): probabilities stay <= 2^8, which bf16 and the fp32 sums hold without loss
        const bool grow = tmax > m_ref + kRescaleStep;   // false while everything is still hidden (-inf > -inf)
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            const float m_new = grow ? tmax : m_ref;
            const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            m_ref = m_new;
            lsum *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        }
        const float m_use = (m_ref == -INFINITY) ? 0.f : m_ref;   // all keys hidden so far: exp2(-inf - 0) = 0
        float psum = 0.f;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = __builtin_amdgcn_exp2f(fmaf(sacc[kvb][r], a.scale_log2, -m_use));
                sacc[kvb][r] = p;
                psum += p;
            }
        lsum += psum;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    pf[kvb][t2].u[e] = pack_bf16(sacc[kvb][8 * t2 + 2 * e], sacc[kvb][8 * t2 + 2 * e + 1]);
    };

    // ---- sequence of visible tiles (skipping tiles no row of the workgroup can see), with their (min, max)
    auto tile_mm_at = [&](int t) {
        const int2* p = a.tile_mm + __builtin_amdgcn_readfirstlane(tile0 + t);   // uniform: a scalar load
        return *p;
    };
    auto next_tile = [&](int t, int2& mm) {
        mm = make_int2(0, 0);
        if (a.causal) {
            while (t < nkt) {
                mm = tile_mm_at(t);
                if (mm.x <= wg_qmax) break;
                ++t;
            }
        }
        return t;
    };

    // ---- prologue: tiles 0 and 1 of the visible sequence into LDS, tile 2 into registers, S of tile 0
    // (a wavefront whose 32 rows cannot see a tile still runs it, fully masked: it would only wait at the
    //  barriers otherwise, and one straight-line loop body keeps the register allocation tight)
    int2 mm_cur, mm_nxt, mm_wr, mm_ld = make_int2(0, 0);
    int t_cur = next_tile(0, mm_cur);                                   // tile whose S is in sacc / P in pf
    int t_nxt = t_cur < nkt ? next_tile(t_cur + 1, mm_nxt) : nkt;       // tile of the next S
    int t_wr = t_nxt < nkt ? next_tile(t_nxt + 1, mm_wr) : nkt;         // tile in registers, next to enter LDS
    if (t_cur < nkt) { load_tile(t_cur); store_tile(0); }
    if (t_nxt < nkt) { load_tile(t_nxt); store_tile(1); }
    if (t_wr < nkt) load_tile(t_wr);
    lds_barrier();
    if (t_cur < nkt) matrix_phase(4, 8, 0, 0, 0);
    if (group_b) lds_barrier();

    int st_cur = 0;                                // LDS stage of t_cur
    while (t_cur < nkt) {
        // ---- vector phase: softmax of tile t_cur; bookkeeping of the tile to prefetch
        const int st_nxt = st_cur == kStages - 1 ? 0 : st_cur + 1;
        const int st_wr = st_nxt == kStages - 1 ? 0 : st_nxt + 1;
        int t_ld = nkt;
        if (t_wr < nkt) t_ld = next_tile(t_wr + 1, mm_ld);
        softmax(st_cur, tile_needs_mask(t_cur, mm_cur));
        // first fragments of the matrix phase: their tile has been in LDS for a whole iteration
#pragma unroll
        for (int pb = 0; pb < 2; ++pb) read_batch(pb, pb, st_cur, st_nxt);
        // the probabilities must be complete BEFORE the barrier (the compiler would otherwise sink the exp2
        // work into the matrix phase, where it serialises with the MFMAs): the barrier consumes them
        asm volatile("s_barrier"
                     :: "v"(pf[0][0].v), "v"(pf[0][1].v), "v"(pf[1][0].v), "v"(pf[1][1].v), "v"(lsum)
                     : "memory");                  // nothing of this wavefront's LDS traffic is awaited by others
        // ---- matrix phase: stage tile t_wr, prefetch the one after it, PV of t_cur, S of t_nxt
        // (after the last tile the S product runs on a stale stage and is discarded)
        if (t_wr < nkt) {
            store_tile(st_wr);
            if (t_ld < nkt) load_tile(t_ld);
        }
        matrix_phase(0, 8, 2, st_cur, st_nxt);
        // likewise every MFMA is issued before the phase ends
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier"
                     :: "v"(sacc[0]), "v"(sacc[1]), "v"(oacc[0]), "v"(oacc[1]), "v"(oacc[2]), "v"(oacc[3])
                     : "memory");
        t_cur = t_nxt; t_nxt = t_wr; t_wr = t_ld;
        mm_cur = mm_nxt; mm_nxt = mm_wr; mm_wr = mm_ld;
        st_cur = st_nxt;
    }
    if (!group_b) lds_barrier();

    // ---- epilogue: normalise, write O (bf16) and LSE (natural log)
    const float ltot = half_swap_sum(lsum);
    const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
    if (row_ok) {
        uint16_t* op = a.O + ((int64_t)my_row * a.Hq + h) * kHeadDim + 4 * hi;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                uint2 w;
                w.x = pack_bf16(oacc[db][4 * bb + 0] * inv, oacc[db][4 * bb + 1] * inv);
                w.y = pack_bf16(oacc[db][4 * bb + 2] * inv, oacc[db][4 * bb + 3] * inv);
                *(uint2*)(op + 32 * db + 8 * bb) = w;
            }
        if (hi == 0)
            a.LSE[(int64_t)my_row * a.Hq + h] = ltot > 0.f ? (m_ref + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
    }
}

esp_status launch_prefill(const void* q, const void* k, const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                          const int32_t* cu_q, const int32_t* cu_kv, int32_t batch, int32_t Tq, int32_t Tkv,
                          int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv, float softmax_scale,
                          int32_t causal, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                          hipStream_t stream) {
    (void)workspace_bytes; (void)max_q;
    int2* tile_mm = (int2*)workspace;
    if (causal && Tkv > 0 && max_kv > 0) {
        dim3 grid((max_kv + kBN - 1) / kBN, batch);
        hipLaunchKernelGGL(kv_tile_minmax_kernel, grid, dim3(64), 0, stream, kv_pos, cu_kv, Tkv, tile_mm);
        esp_status st = check_launch("kv_tile_minmax_kernel");
        if (st != ESP_OK) return st;
    }
    PrefillArgs a;
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
    a.q_pos = q_pos; a.kv_pos = kv_pos; a.cu_q = cu_q; a.cu_kv = cu_kv; a.tile_mm = tile_mm;
    a.O = (uint16_t*)O; a.LSE = LSE;
    a.batch = batch; a.Tq = Tq; a.Tkv = Tkv; a.Hq = Hq; a.Hkv = Hkv; a.causal = causal ? 1 : 0;
    a.scale_log2 = softmax_scale * kLog2e;
    int64_t blocks = (int64_t)prefill_q_tiles_bound(Tq, batch) * Hq;
    if (blocks > 0x7fffffff) return fail(ESP_ERR_INVALID_ARG, "prefill: too many tiles for one launch");
    hipLaunchKernelGGL(prefill_kernel, dim3((unsigned)blocks), dim3(kPfWaves * 64), 0, stream, a);
    return check_launch("prefill_kernel");
}

}  // namespace esp

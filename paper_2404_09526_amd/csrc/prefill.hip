// esp_partial_attn_prefill: a causal query chunk against ONE local key-value shard, masked by
// global token position (sequence-parallel prefill, Sec. 2.3 / Fig. 1: instance i attends its
// local q_i to the segment kv_j of the current round; striped layout and tile-skipping remarks
// in Sec. 6).  Emits the un-merged output, normalised within the shard, and its log-sum-exp.
//
// Mapping to gfx950 (64-wide wavefronts, MFMA 32x32x16 bf16, 160 KiB LDS):
//   * one persistent workgroup of 8 wavefronts per CU works through items; an item is 256 query
//     rows of one head: each wavefront owns 32 rows and keeps their Q fragment (B operand), the
//     softmax state and the fp32 output accumulator in registers for the whole KV sweep.  Most
//     items are dealt to the workgroups beforehand, the light ones at the end are drawn from a
//     device-wide counter as workgroups become free (see the item loop at the end of the kernel);
//   * K/V tiles of 64 rows are fetched straight from global memory into a 4-stage LDS ring
//     (global_load ... lds, no register staging), K four tiles and V two tiles ahead of their use;
//   * the K tile is the A operand of S^T = K Q^T, so a lane ends up with scores of ONE query
//     row (its column); P^T stays in registers and is the B operand of O^T = V^T P^T, whose A
//     operand comes from transposing LDS reads of the row-major V tile;
//   * LDS rows of K are padded to 272 bytes and the 16-byte chunks of V rows are XOR-swizzled, so
//     that the operand reads spread over all banks;
//   * one uniform instruction stream per wavefront, software pipelined at the level of single
//     MFMAs: every step issues one MFMA of S^T for tile j+1, the exp2 of two scores of tile j,
//     one MFMA of O^T += V^T P^T that trails the probabilities by one chunk of 16 keys, and the
//     sum / bf16 pack of the two probabilities.  A wavefront issues an instruction only every
//     6-8 cycles and a 32x32x16 MFMA lasts 32, so with the two wavefronts of a SIMD running the
//     same mix the matrix pipe always has an MFMA of one of them to run;
//   * the softmax offset is optimistic: probabilities are taken against the offset in use
//     without looking at the scores first; one compare per tile on the probability sum tells
//     whether the offset has to move (exact rescale by a power of two), and a workgroup whose
//     scores leave the range this can handle redoes its rows with a plain, exact sweep;
//   * the minimum / maximum position of every KV tile (found by the workgroup itself while its
//     first tiles are in flight) decide: tiles past the last one any row can see are never
//     processed; tiles below every row of a wavefront run the branch-free "plain" iteration;
//     the others apply the element-wise test kv_pos <= q_pos; past the last tile any of its own
//     rows can see a wavefront stops its arithmetic and only keeps up transfers and barriers.
#include <limits.h>
#include <stdlib.h>

#include <atomic>
#include <chrono>
#include <random>

#include "esp_common.h"
#include "mfma_tile.h"

namespace esp {

constexpr int kBM = 256;   // query rows per workgroup
constexpr int kBN = 64;    // KV rows per tile
constexpr int kPfWaves = 8;
constexpr long long kSyncTicks = 15000;   // longest wait at a round start, in ticks of the 100 MHz wall clock (150 us)
constexpr int kTileBytes = kBN * kHeadDim * 2;   // 16 KiB: a V tile in LDS, rows of 256 bytes
constexpr int kKRow = 272;                       // LDS row pitch of a K tile: 256 bytes + 16 of padding
constexpr int kKTileBytes = kBN * kKRow;         // 17 KiB = 17 transfers of 1 KiB


static int32_t prefill_q_tiles_bound(int32_t Tq, int32_t batch) { return Tq / kBM + batch; }

// Global scratch memory of the prefill path: one 64-bit item counter (the first word of the block, the second is
// spare) and the arrival counts of the start-of-round waits (one per round parity, XCD and KV head; room for one
// per parity and query head).
// Every launch
// gets a tag of its own, so that a counter left by an earlier launch, or never written, is told from the current
// one without clearing it first (a clearing kernel ahead of each launch costs about 6 us).  Tags start at a random
// 32-bit value per process: stale memory passes for the current launch's counter with probability 2^-32.
static uint32_t next_launch_tag() {
    static std::atomic<uint32_t> tag{[] {
        uint32_t seed = (uint32_t)std::chrono::steady_clock::now().time_since_epoch().count();
        try { seed ^= std::random_device{}(); } catch (...) {}
        return seed;
    }()};
    const uint32_t t = tag.fetch_add(1, std::memory_order_relaxed) + 1;
    return t ? t : tag.fetch_add(1, std::memory_order_relaxed) + 1;   // never 0: cleared counters carry tag 0
}
// Longest start-of-round wait.  The default comes from ESP_PREFILL_SYNC_TICKS in the environment, read once when the
// library is loaded; esp_debug_set_prefill_sync_ticks replaces it (0: every wait gives up at once, the path a
// missing workgroup would cause).
static std::atomic<int32_t> g_sync_ticks{[] {
    if (const char* e = getenv("ESP_PREFILL_SYNC_TICKS")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 0 && v <= 1000000) return (int32_t)v;
    }
    return (int32_t)kSyncTicks;
}()};
int32_t set_prefill_sync_ticks(int32_t ticks) {
    return g_sync_ticks.exchange(ticks < 0 ? (int32_t)kSyncTicks : ticks > 1000000 ? 1000000 : ticks, std::memory_order_relaxed);
}
size_t prefill_workspace_bytes(int32_t Tq, int32_t Tkv, int32_t batch, int32_t Hq, int32_t Hkv) {
    (void)Tq; (void)Tkv; (void)batch; (void)Hkv;
    return ((size_t)8 * (2 + 2 * (size_t)(Hq > 0 ? Hq : 0)) + 255) / 256 * 256;   // pool counter (+ a spare word) + two counts per query head
}

struct PrefillArgs {
    const uint16_t* q; const uint16_t* k; const uint16_t* v;
    const int32_t* q_pos; const int32_t* kv_pos; const int32_t* cu_q; const int32_t* cu_kv;
    const int32_t* retain_slot;       // [Tkv] pool slot of every shard row (negative: not kept), or null: nothing is kept
    const int32_t* kv_slot;           // [Tkv] pool slot of every shard row when k and v ARE the token pools; null: dense shard
    uint16_t* k_pool; uint16_t* v_pool;
    void* O; float* LSE;              // O: bf16 [Tq, Hq, 128], or fp32 of the same shape when o_f32 is set
    int32_t batch, Tq, Tkv, Hq, Hkv, causal, o_f32;
    int32_t q_tiles, heads_per_xcd;   // upper bound of the number of query tiles; query heads per XCD (0: no split)
    unsigned long long* pool;         // counter of the item pool: launch tag (high word), draws so far (low word)
    uint32_t tag;                     // this launch's tag
    int32_t group_sync;               // workgroups sharing a KV head start their dealt rounds together
    int32_t sync_ticks;               // longest such wait, in ticks of the 100 MHz wall clock
    float scale_log2;
};

constexpr int kStages = 4;            // LDS stages per operand; tile j lives in stage j % 4
constexpr float kSumLimit = 1048576.f;  // 2^20: a tile's probability sum above this refreshes the offset

template <int V> struct IC { static constexpr int value = V; };

// MODE 0: the plain kernel.
// RETAIN (MODE 1): the variant that also keeps rows of the shard in the token pool while they pass through LDS (proactive
// scale-down, Sec. 4.1 / Fig. 7).  Every KV tile of a request and KV head is OWNED by one item, which stores its K
// and V rows to the pool slots that are not negative:
//   * a request whose shard rows are about as many as its query rows (a striped shard, causal self-attention): the
//     item of query tile i, first query head of the group, owns the four KV tiles 4i .. 4i+3 (the last query tile:
//     all that remain).  Under a causal mask these are the tiles on its diagonal, the last ones of its sweep, which
//     run the masked iteration anyway: the work is spread evenly over the items and costs each of them little;
//   * any other request (a chunk against a long prefix): one item owns every tile, the last query tile's, or the
//     first one's where the workgroups of a KV head walk the shard together (its turn comes in the last round).
// An owner sweeps at least up to its last owned tile (tiles it cannot see pass through LDS without arithmetic), runs
// the masked iteration from its first owned tile on, finds the slots in a ring of 8 LDS stages (the first four owned
// tiles' slots are fetched at the start, the others with their K tiles), and stores the sweep's last four tiles, which
// stay in LDS, after the sweep; an earlier tile j at the top of iteration j: complete in LDS by then, and issued
// ahead of the iteration's transfers, so that the hand-counted waits still see those as the newest operations in
// flight (they have to sit out the stores, though, which is why the tiles at the end are left for later).
//
// POOL (MODE 2): the shard's rows live in the token pool (a.k / a.v are the pools, a.kv_slot the slot of every shard
// row, Sec. 4.1 / 4.2: KV that an instance kept stays where it was placed).  The tile transfers take each row from its
// slot: the slots of tile t travel to a ring of 4 LDS stages (stage t % 4) one iteration before the tile's first
// transfer is issued, every lane reads the slot of the row its 16 bytes belong to and forms the address itself.
template <int MODE>
__global__ __launch_bounds__(kPfWaves * 64) void prefill_kernel(PrefillArgs a) {
    constexpr bool RETAIN = MODE == 1, POOL = MODE == 2;
    // One LDS block, V stages first: an LDS instruction adds a 16-bit immediate to its address register, so with
    // each array's base folded into the per-lane register every operand read of the loop needs no address math.
    constexpr int kLdsV = 0, kLdsK = kLdsV + kStages * kTileBytes, kLdsPos = kLdsK + kStages * kKTileBytes,
                  kLdsQmm = kLdsPos + kStages * kBN * 4, kLdsSched = kLdsQmm + 2 * kPfWaves * 4,
                  kLdsFlag = kLdsSched + kPfWaves * 64 * 8, kLdsSlot = kLdsFlag + 16,
                  kLdsTotal = kLdsSlot + (RETAIN ? 8 * kBN * 4 : POOL ? kStages * kBN * 4 : 0);
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kLdsTotal];
    int32_t (*lds_pos)[kBN] = (int32_t (*)[kBN])(smem + kLdsPos);
    int32_t (*lds_qmm)[kPfWaves] = (int32_t (*)[kPfWaves])(smem + kLdsQmm);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = a.Hq / a.Hkv;

    // ---- one query tile of one head (rank: position in the heaviest-first order of query tiles).  Returns false
    //      if there is no such tile.  With `claim_from` set, thread 0 also draws the workgroup's next item from that
    //      counter (a device-wide atomic, issued when the sweep is done; its latency hides behind the epilogue) and
    //      leaves the counter's old value in LDS (lds_next), to be read after the next workgroup barrier.
    int32_t* lds_next = (int32_t*)(smem + kLdsFlag + 4);
    // The pool counter needs no clearing between launches: its high word names the launch that counted in it.  A
    // draw is one fetch-and-add; if the old value carries this launch's tag, its low word is the ticket.  If not
    // (the first draws of a launch find the previous launch's count, or whatever a fresh workspace holds), the
    // drawer starts this launch's count with a compare-and-swap, or draws again if another one has done so.
    auto draw_finish = [&](unsigned long long* ctr, unsigned long long old) {
        if ((uint32_t)(old >> 32) == a.tag) return (int)(uint32_t)old;
        for (;;) {
            unsigned long long cur = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((uint32_t)(cur >> 32) == a.tag)
                return (int)(uint32_t)__hip_atomic_fetch_add(ctr, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__hip_atomic_compare_exchange_strong(ctr, &cur, ((unsigned long long)a.tag << 32) | 1ULL, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                return 0;
        }
    };
    auto process = [&](const int rank, const int h, unsigned long long* claim_from) {
    const int kvh = h / G;
    int q_lo, q_hi, kv_lo, kv_hi;   // rows of this query tile; rows of its request in the shard
    int own_lo = 0, own_hi = 0;     // KV tiles of the request whose rows this item keeps in the pool (none: equal)
    {
        // query tiles of request r; a request without query rows whose shard rows may have to be kept gets one
        // (empty) tile, so that it has a keeper
        auto tiles_of = [&](int r) {
            const int len = a.cu_q ? a.cu_q[r + 1] - a.cu_q[r] : a.Tq;
            int nt = (len + kBM - 1) / kBM;
            if (RETAIN && nt == 0 && a.retain_slot && a.cu_kv && a.cu_kv[r + 1] > a.cu_kv[r]) nt = 1;
            return nt;
        };
        int total = 0;
        for (int r = 0; r < a.batch; ++r) total += tiles_of(r);
        if (rank >= total) return false;
        int tl = total - 1 - rank;   // later tiles of a causal request see more keys: run them first
        int r = 0, nt = 0;
        for (;; ++r) {
            nt = tiles_of(r);
            if (tl < nt) break;
            tl -= nt;
        }
        const int qs = a.cu_q ? a.cu_q[r] : 0, qe = a.cu_q ? a.cu_q[r + 1] : a.Tq;
        q_lo = qs + tl * kBM;
        q_hi = min(q_lo + kBM, qe);
        kv_lo = a.cu_kv ? a.cu_kv[r] : 0;
        kv_hi = a.cu_kv ? a.cu_kv[r + 1] : a.Tkv;
        if (RETAIN && a.retain_slot != nullptr && h % G == 0) {   // which KV tiles this item owns (see the kernel's head)
            const int tiles = (kv_hi - kv_lo + kBN - 1) / kBN, per = kBM / kBN;
            if (!a.group_sync && a.causal && tiles <= per * nt + per) {
                own_lo = min(per * tl, tiles);
                own_hi = tl == nt - 1 ? tiles : min(per * tl + per, tiles);
            } else if (tl == (a.group_sync ? 0 : nt - 1)) {
                own_hi = tiles;
            }
        }
    }
    // the same for every lane by construction; said explicitly, since base addresses of the tile transfers derive
    // from them and must sit in scalar registers
    q_lo = __builtin_amdgcn_readfirstlane(q_lo); q_hi = __builtin_amdgcn_readfirstlane(q_hi);
    kv_lo = __builtin_amdgcn_readfirstlane(kv_lo); kv_hi = __builtin_amdgcn_readfirstlane(kv_hi);
    own_lo = __builtin_amdgcn_readfirstlane(own_lo); own_hi = __builtin_amdgcn_readfirstlane(own_hi);
    // The rest of the item exists twice in the keeping kernel: as everywhere else, and with an owner's extras.
    // (One body with the extras behind a run-time flag costs the items that own nothing dearly: measured +25 % on
    // a GQA batch, where three items in four own nothing, against +1.6 % with two bodies.)
    auto body = [&](auto keep_c) {
    constexpr bool KEEP = RETAIN && decltype(keep_c)::value != 0;
    const int kv_len = kv_hi - kv_lo;
    const int nkt = (kv_len + kBN - 1) / kBN;
    const int tail_rows = kv_len - (nkt - 1) * kBN;    // rows of the last tile (64 when not ragged)
    const int ragged_tile = tail_rows < kBN ? nkt - 1 : -8;          // index of the ragged last tile, if any

    // ---- global -> LDS in transfers of 64 lanes x 16 bytes = 1 KiB of consecutive LDS bytes.
    //      V tile (rows of 256 B, chunks XOR-swizzled): wavefront w moves rows 8w .. 8w+7 in two transfers; lane L
    //      writes LDS chunk L % 16 of row r = base + L / 16, so it fetches the global chunk (L % 16) ^ f(r).
    //      K tile (rows padded to 272 B): transfer n covers LDS bytes [1024 n, 1024 n + 1024) of the padded tile;
    //      lane L's byte 1024 n + 16 L falls into row B / 272 at B % 272 (a padding slot fetches chunk 0, unused).
    //      Wavefront w issues K transfers w and w + 8; wavefront 7 also the 17th; wavefront 0 the positions.
    const uint32_t kv_row_bytes = (uint32_t)a.Hkv * kHeadDim * 2;
    const int64_t tile_bytes = (int64_t)kBN * kv_row_bytes;
    const int st_sub = lane >> 4, st_p = lane & 15;
    const int st_r0 = wave * 8 + st_sub, st_r1 = st_r0 + 4;
    auto v_goff = [&](int r_lds, int r_glb) { return r_glb * kv_row_bytes + ((st_p ^ ((r_lds & 3) << 2)) << 4); };
    auto k_goff = [&](int n, int last_row) {
        const int B = 1024 * n + 16 * lane, row = B / kKRow, within = B - row * kKRow;
        return (uint32_t)(min(row, last_row) * kv_row_bytes + (within < 256 ? within : 0));
    };
    const uint32_t gv0 = v_goff(st_r0, st_r0), gv1 = v_goff(st_r1, st_r1);
    const uint32_t gk0 = k_goff(wave, kBN - 1), gk1 = k_goff(wave + 8, kBN - 1), gk2 = k_goff(16, kBN - 1);
    const uint32_t lds_base0 = (uint32_t)(uintptr_t)(ESP_LDS unsigned char*)smem;
    // row kv_lo, head kvh (POOL: slot 0, head kvh)
    const char* kreq = (const char*)a.k + ((int64_t)(POOL ? 0 : kv_lo) * a.Hkv + kvh) * (kHeadDim * 2);
    const char* vreq = (const char*)a.v + ((int64_t)(POOL ? 0 : kv_lo) * a.Hkv + kvh) * (kHeadDim * 2);
    // POOL: per transfer of this lane, the tile row its 16 bytes belong to (times 4: byte offset into a ring stage,
    // low byte) and where in the row's 256 bytes they sit (from bit 8 up)
    auto pool_key = [&](int row, int within) { return (uint32_t)((within << 8) | (row << 2)); };
    auto k_key = [&](int n) {
        const int B = 1024 * n + 16 * lane, row = B / kKRow, within = B - row * kKRow;
        return pool_key(min(row, kBN - 1), within < 256 ? within : 0);
    };
    const uint32_t pk0 = POOL ? k_key(wave) : 0, pk1 = POOL ? k_key(wave + 8) : 0, pk2 = POOL ? k_key(16) : 0;
    const uint32_t pv0 = POOL ? pool_key(st_r0, (st_p ^ ((st_r0 & 3) << 2)) << 4) : 0;
    const uint32_t pv1 = POOL ? pool_key(st_r1, (st_p ^ ((st_r1 & 3) << 2)) << 4) : 0;
    // the row's address: its slot from ring stage st, one 32 x 32 -> 64-bit multiply-add
    auto pool_slot = [&](int st, uint32_t key) { return *(const int32_t*)(smem + kLdsSlot + st * (kBN * 4) + (key & 0xff)); };
    auto pool_at = [&](const char* base, int32_t slot, uint32_t key) {
        return base + ((uint64_t)(uint32_t)slot * kv_row_bytes + (key >> 8));
    };
    auto pool_src = [&](const char* base, int st, uint32_t key) { return pool_at(base, pool_slot(st, key), key); };
    // slots of tile t into ring stage st (wavefront 6); rows past the end of a ragged last tile repeat the last row's
    // slot, so their transfers re-read that row (their scores get masked)
    const int32_t* slot_req = POOL ? a.kv_slot + kv_lo : nullptr;
    auto fetch_pool_slots = [&](int t, int st) {
        if (!POOL || wave != 6 || t >= nkt) return;
        const int rows = min(kBN, kv_len - t * kBN);
        load_to_lds_b32(lds_base0 + kLdsSlot + st * (kBN * 4), slot_req + t * kBN, min(lane, rows - 1) * 4);
    };
    // the same inside the sweep's plain iterations, where the tile is a full one that exists: nothing to work out
    const uint32_t lane4 = lane * 4;
    auto fetch_pool_slots_full = [&](int t, int st) {
        load_to_lds_b32(lds_base0 + kLdsSlot + st * (kBN * 4), slot_req + t * kBN, lane4);
    };
    const int32_t* preq = a.kv_pos + kv_lo;
    const uint32_t lds_base = lds_base0;
    const uint32_t lds_k0 = lds_base + kLdsK, lds_v0 = lds_base + kLdsV, lds_p0 = lds_base + kLdsPos;

    // K tile at kt into K stage st: 2 transfers per wavefront, 3 for wavefront 7; `part` picks one of them, so that
    // the sweep can spread them over an iteration (a burst of transfers from all wavefronts at once backs up the
    // memory pipeline and stalls the issuing wavefronts).  `tail`: it is the ragged last tile, whose rows past the
    // end re-read the last row (their scores get masked).
    auto fetch_k_part = [&](const char* kt, int st, bool tail, int part) {
        const uint32_t ko = lds_k0 + st * kKTileBytes;
        const int n = part == 0 ? wave : part == 1 ? wave + 8 : 16;
        if (part == 2 && wave != 7) return;
        if constexpr (POOL) { load_to_lds_b128_at(ko + 1024 * n, pool_src(kreq, st, part == 0 ? pk0 : part == 1 ? pk1 : pk2)); return; }
        if (__builtin_expect(tail, 0)) load_to_lds_b128(ko + 1024 * n, kt, k_goff(n, tail_rows - 1));
        else load_to_lds_b128(ko + 1024 * n, kt, part == 0 ? gk0 : part == 1 ? gk1 : gk2);
    };
    // V tile at vt and its positions at pt into V stage st: 2 transfers per wavefront, 3 for wavefront 0
    auto fetch_v_part = [&](const char* vt, const int32_t* pt, int st, bool tail, int part) {
        const uint32_t vo = lds_v0 + st * kTileBytes + wave * 2048;
        const int last = tail_rows - 1;
        if (part == 2) {
            if (wave != 0) return;
            load_to_lds_b32(lds_p0 + st * (kBN * 4), pt, (tail ? min(lane, last) : lane) * 4);
        } else if constexpr (POOL) {
            load_to_lds_b128_at(vo + 1024 * part, pool_src(vreq, st, part == 0 ? pv0 : pv1));
        } else if (__builtin_expect(tail, 0)) {
            const int r = part == 0 ? st_r0 : st_r1;
            load_to_lds_b128(vo + 1024 * part, vt, v_goff(r, min(r, last)));
        } else {
            load_to_lds_b128(vo + 1024 * part, vt, part == 0 ? gv0 : gv1);
        }
    };
    auto fetch_k = [&](const char* kt, int st, bool tail) {
        fetch_k_part(kt, st, tail, 0); fetch_k_part(kt, st, tail, 1); fetch_k_part(kt, st, tail, 2);
    };
    auto fetch_v = [&](const char* vt, const int32_t* pt, int st, bool tail) {
        fetch_v_part(vt, pt, st, tail, 0); fetch_v_part(vt, pt, st, tail, 1); fetch_v_part(vt, pt, st, tail, 2);
    };
    // positions past the end of a ragged last tile become INT_MAX, hidden from every query
    auto seal_tail = [&](int st) {
        if (wave == 0 && lane >= tail_rows) lds_pos[st][lane] = INT_MAX;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // written before the barrier that follows
    };

    // an owner's extras: slots of an owned tile t into stage t % 8 of the slot ring (wavefront 6), and the stores of
    // owned tiles' K and V rows from LDS to the pool (wavefront w: rows 8w .. 8w+7)
    const int32_t* sreq = KEEP ? a.retain_slot + kv_lo : nullptr;
    auto fetch_slots = [&](int t) {
        if (!KEEP || wave != 6 || t < own_lo || t >= own_hi) return;
        const int rows = min(kBN, kv_len - t * kBN);
        load_to_lds_b32(lds_base + kLdsSlot + (t & 7) * (kBN * 4), sreq + t * kBN, min(lane, rows - 1) * 4);
    };
    // Slots past the end of a ragged last tile become -1 (wavefront 6, once the tile's slots have landed and a
    // barrier before anyone reads them), so that the stores test the slot alone.
    auto seal_slots = [&]() {
        if (!KEEP || wave != 6 || ragged_tile < own_lo || ragged_tile >= own_hi) return;
        if (lane >= tail_rows) ((int32_t*)(smem + kLdsSlot))[(ragged_tile & 7) * kBN + lane] = -1;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };
    // K and V rows of tile t (both in stage st) to the pool, at the top of iteration t.  Every wavefront stores
    // exactly the LDS bytes its own transfers fill: of V the rows 8w .. 8w+7, of K the 1 KiB pieces w and w + 8 of
    // the padded tile (wavefront 7 also the 17th), lane L the 16 bytes at 1024 n + 16 L, i.e. row B / 272 at
    // B % 272 (nothing if that is padding).  The K stage is refilled during this very iteration, but each
    // wavefront's own refills follow its own reads in program order, and it reads nobody else's bytes.
    // All LDS reads first (slots and rows, one round trip), then the stores.
    auto keep_tile = [&](int t, int st) {
        if (!KEEP) return;
        if (t < own_lo || t >= own_hi) return;
        const int32_t* ring = (const int32_t*)(smem + kLdsSlot) + (t & 7) * kBN;
        const unsigned char* kt = smem + kLdsK + st * kKTileBytes;
        const unsigned char* vt = smem + kLdsV + st * kTileBytes;
        const int r0 = wave * 8 + st_sub, r1 = r0 + 4;
        const int b0 = 1024 * wave + 16 * lane, b1 = b0 + 8192, b2 = 16384 + 16 * lane;
        const int kr0 = b0 / kKRow, kr1 = b1 / kKRow, kr2 = b2 / kKRow;
        const int kw0 = b0 - kr0 * kKRow, kw1 = b1 - kr1 * kKRow, kw2 = b2 - kr2 * kKRow;
        const int32_t sv0 = ring[r0], sv1 = ring[r1];
        const int32_t sk0 = ring[kr0], sk1 = ring[kr1], sk2 = ring[kr2];
        const uint4 wv0 = *(const uint4*)(vt + r0 * 256 + ((st_p ^ ((r0 & 3) << 2)) << 4));
        const uint4 wv1 = *(const uint4*)(vt + r1 * 256 + ((st_p ^ ((r1 & 3) << 2)) << 4));
        const uint4 wk0 = *(const uint4*)(kt + b0), wk1 = *(const uint4*)(kt + b1), wk2 = *(const uint4*)(kt + b2);
        // address of a pool row's piece: one 32 x 32 -> 64-bit multiply-add each
        const uint32_t row_pitch = (uint32_t)a.Hkv * (kHeadDim * 2);
        ESP_GLOBAL char* kb = (ESP_GLOBAL char*)a.k_pool + (uint32_t)kvh * (kHeadDim * 2);
        ESP_GLOBAL char* vb = (ESP_GLOBAL char*)a.v_pool + (uint32_t)kvh * (kHeadDim * 2) + 16 * st_p;
        if (sk0 >= 0 && kw0 < 256) *(ESP_GLOBAL u32x4*)(kb + (uint64_t)(uint32_t)sk0 * row_pitch + kw0) = u32x4{wk0.x, wk0.y, wk0.z, wk0.w};
        if (sk1 >= 0 && kw1 < 256) *(ESP_GLOBAL u32x4*)(kb + (uint64_t)(uint32_t)sk1 * row_pitch + kw1) = u32x4{wk1.x, wk1.y, wk1.z, wk1.w};
        if (wave == 7 && sk2 >= 0 && kw2 < 256) *(ESP_GLOBAL u32x4*)(kb + (uint64_t)(uint32_t)sk2 * row_pitch + kw2) = u32x4{wk2.x, wk2.y, wk2.z, wk2.w};
        if (sv0 >= 0) *(ESP_GLOBAL u32x4*)(vb + (uint64_t)(uint32_t)sv0 * row_pitch) = u32x4{wv0.x, wv0.y, wv0.z, wv0.w};
        if (sv1 >= 0) *(ESP_GLOBAL u32x4*)(vb + (uint64_t)(uint32_t)sv1 * row_pitch) = u32x4{wv1.x, wv1.y, wv1.z, wv1.w};
    };

    // ---- this lane's query row (column of S^T); its position is needed first (schedule scan), so it is loaded first
    const int qi = lane & 31, hi = lane >> 5;
    const int my_row = q_lo + wave * 32 + qi;
    const bool row_ok = my_row < q_hi;
    const int ld_row = row_ok ? my_row : max(q_hi - 1, 0);            // (an empty tile of the keeping variant: any row)
    // effective query position: non-causal rows see every real key
    const int my_qpos = a.causal ? a.q_pos[ld_row] : INT_MAX - 1;   // INT_MAX marks rows past a ragged tail

    // the first tiles are requested right away, so that their latency hides behind the Q load and the schedule
    // scan (tiles the scan later finds hidden are fetched for nothing, which is harmless: they exist)
    if constexpr (POOL) {
        // the first four tiles' slots must be in LDS, and visible to every wavefront, before the first transfer
        fetch_pool_slots(0, 0); fetch_pool_slots(1, 1); fetch_pool_slots(2, 2); fetch_pool_slots(3, 3);
        wait_vm<0>();
        wg_barrier();
    }
    if (nkt > 4) {                                                   // the usual case, without a conditional in it
        fetch_k(kreq, 0, false); fetch_v(vreq, preq, 0, false);
        fetch_k(kreq + tile_bytes, 1, false); fetch_v(vreq + tile_bytes, preq + kBN, 1, false);
        fetch_k(kreq + 2 * tile_bytes, 2, false);
        fetch_k(kreq + 3 * tile_bytes, 3, false);
        fetch_slots(own_lo); fetch_slots(own_lo + 1); fetch_slots(own_lo + 2); fetch_slots(own_lo + 3);
    } else {
        fetch_slots(own_lo); fetch_slots(own_lo + 1); fetch_slots(own_lo + 2); fetch_slots(own_lo + 3);
        if (nkt > 0) { fetch_k(kreq, 0, 0 == ragged_tile); fetch_v(vreq, preq, 0, 0 == ragged_tile); }
        if (nkt > 1) { fetch_k(kreq + tile_bytes, 1, 1 == ragged_tile); fetch_v(vreq + tile_bytes, preq + kBN, 1, 1 == ragged_tile); }
        if (nkt > 2) fetch_k(kreq + 2 * tile_bytes, 2, 2 == ragged_tile);
        if (nkt > 3) fetch_k(kreq + 3 * tile_bytes, 3, 3 == ragged_tile);
    }
    // V stage 3 stands in for the tile before the first one (the loop multiplies the last chunk of tile j-1 at the
    // start of iteration j): zero it, since stale LDS contents could be NaN patterns; V(3) arrives there later
    {
        const uint4 z = make_uint4(0u, 0u, 0u, 0u);
        uint4* dst = (uint4*)(smem + kLdsV + 3 * kTileBytes) + tid * 2;
        dst[0] = z;
        dst[1] = z;
        if (tid == 0) *(int32_t*)(smem + kLdsFlag) = 0;      // "redo with the plain sweep" flag, see below
    }

    // ---- smallest / largest key position of KV tile t of this request, found by one thread: 16 loads of four
    //      positions when the request's positions are 16-byte aligned and the tile is full, one position at a
    //      time (index clamped to the last row) otherwise.  The loads of this thread's first tile are issued here,
    //      ahead of the barrier below, so that their latency overlaps the Q loads.
    const bool pos_vec_ok = (((uintptr_t)preq) & 15) == 0;
    auto tile_bounds = [&](int t) {
        int mn = INT_MAX, mx = INT_MIN;                             // beyond the end: hidden, needs no mask
        if (t < nkt) {
            if (pos_vec_ok && (t + 1) * kBN <= kv_len) {
                const int4* pp = (const int4*)(preq + t * kBN);
                int4 v[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) v[e] = pp[e];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    mn = min(min(mn, v[e].x), min(v[e].y, min(v[e].z, v[e].w)));
                    mx = max(max(mx, v[e].x), max(v[e].y, max(v[e].z, v[e].w)));
                }
            } else {
                for (int e = 0; e < kBN; ++e) {
                    const int pv = preq[min(t * kBN + e, kv_len - 1)];
                    mn = min(mn, pv);
                    mx = max(mx, pv);
                }
            }
        }
        return make_int2(mn, mx);
    };
    int2 mm_first = make_int2(INT_MAX, INT_MIN);
    if (a.causal) mm_first = tile_bounds(tid);

    // ---- the Q fragment of this lane's row
    bf16x8 qf[8];
    {
        const uint16_t* qp = a.q + ((int64_t)ld_row * a.Hq + h) * kHeadDim + 8 * hi;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[t] = *(const bf16x8*)(qp + 16 * t);
    }
    int wave_qmin = my_qpos, wave_qmax = my_qpos;
#pragma unroll
    for (int s = 16; s >= 1; s >>= 1) {
        wave_qmin = min(wave_qmin, __shfl_xor(wave_qmin, s));
        wave_qmax = max(wave_qmax, __shfl_xor(wave_qmax, s));
    }
    wave_qmin = __builtin_amdgcn_readfirstlane(wave_qmin);
    wave_qmax = __builtin_amdgcn_readfirstlane(wave_qmax);
    if (lane == 0) { lds_qmm[0][wave] = wave_qmin; lds_qmm[1][wave] = wave_qmax; }

    // ---- tile schedule of this workgroup: n_vis = 1 + last tile some row can see (tiles before it that are
    //      hidden, possible only with unordered positions, are swept fully masked); first_mask = first tile
    //      this wavefront has to mask (every later tile is masked too, which is exact for ascending positions
    //      and merely redundant otherwise); n_need = 1 + last tile a row of this wavefront can see: beyond it
    //      the wavefront only keeps up its share of the transfers and the barriers.
    //      The bounds of 512 tiles at a time (one per thread) go through LDS; every wavefront then reads them all,
    //      64 per step, and wavefront-wide ballots turn its three tests into bit masks whose highest / lowest set
    //      bit is the answer: no exchange of candidates, and one barrier for requests of up to 512 tiles.
    int n_vis = nkt, first_mask = nkt, n_need = nkt;
    int2* lds_mm = (int2*)(smem + kLdsSched);
    if (a.causal) lds_mm[tid] = mm_first;
    wg_barrier();          // LDS only: the Q loads and tile transfers stay in flight
    // (POOL: every wavefront has issued its first transfers, i.e. read the slots of tile 0: those of tile 4, which
    // iteration 0 asks for, may replace them; they land before the wait that ends the prologue)
    fetch_pool_slots(4, 0);
    if (a.causal) {
        int wg_qmax = lds_qmm[1][0];
#pragma unroll
        for (int w = 1; w < kPfWaves; ++w) wg_qmax = max(wg_qmax, lds_qmm[1][w]);
        int last_vis = -1, fm = nkt, lw = -1;
        for (int base = 0; base < nkt; base += kPfWaves * 64) {
            if (base > 0) {
                wg_barrier();                                       // everyone has read the previous 512
                lds_mm[tid] = tile_bounds(base + tid);
                wg_barrier();
            }
            const int cnt = min(kPfWaves * 64, nkt - base);
            for (int t0 = 0; t0 < cnt; t0 += 64) {
                const int2 mm = lds_mm[t0 + lane];                  // past the last tile: (INT_MAX, INT_MIN)
                const uint64_t vis = __builtin_amdgcn_ballot_w64(mm.x <= wg_qmax);
                if (vis) last_vis = base + t0 + 63 - __builtin_clzll(vis);
                const uint64_t mk = __builtin_amdgcn_ballot_w64(mm.y > wave_qmin);
                if (mk && fm == nkt) fm = base + t0 + __builtin_ctzll(mk);
                const uint64_t vw = __builtin_amdgcn_ballot_w64(mm.x <= wave_qmax);
                if (vw) lw = base + t0 + 63 - __builtin_clzll(vw);
            }
        }
        n_vis = last_vis + 1;
        first_mask = fm;
        n_need = lw + 1;
        if (KEEP) n_vis = max(n_vis, own_hi);                       // every owned tile passes through LDS, seen or not
    }

    // ---- operand read offsets
    // K (A operand of S^T): row 32*kvb + qi, chunk 2t + hi -> one base per lane, the rest are immediates
    const uint32_t k_rd = lds_k0 + qi * kKRow + hi * 16;
    // V (A operand of O^T) by transposing reads: 16 lanes fetch a 4 (kv) x 16 (d) patch
    const int j16 = lane & 15, jq = j16 >> 2, dblk = (lane >> 4) & 1;
    uint32_t v_rd[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_rd[db] = lds_v0 + (4 * hi + jq) * 256 + ((((db ^ jq) << 2) + 2 * dblk + ((j16 & 3) >> 1)) << 4) + (j16 & 1) * 8;

    floatx16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    // softmax state.  The offset m_use subtracted from the scaled scores moves in whole steps (so every change
    // of it rescales by an exact power of two) and only when it has to: lim is the largest tile sum
    // accepted without a move, -1 while the row has not seen a key yet (m_use is then a stand-in 0).
    float m_use = 0.f, lim = -1.f;
    float lsum = 0.f;          // running sum of exp2 over this lane's half of the keys (for the log-sum-exp)
    float lcorr = 0.f;         // what rounding the probabilities to bf16 added to that sum, over the tiles that track it
    float psum = 0.f, psum_r = 0.f, p0 = 0.f, p1 = 0.f;

    floatx16 sbuf[2][2];       // S^T of two tiles in flight: [tile parity][kvb]
    union PFrag { uint32_t u[4]; bf16x8 v; };
    PFrag pf[2][2];            // P^T packed to bf16, one fragment per chunk of 16 keys: [kvb][t2]
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) pf[c >> 1][c & 1].u[e] = 0u;
    union VFrag { short4_t s[2]; bf16x8 v; };
    VFrag frk[2], frv[2];      // operand fragments, fetched two steps ahead of their use

    // K fragment i = (t, kvb) = (i / 2, i % 2) of the tile in K stage st; V^T fragment p = (kvb, t2, db) =
    // (p / 8, (p / 4) % 2, p % 4) of the tile at byte offset stage_off of the V stages
    auto read_k = [&](int slot, int st, int i) {
        frk[slot].v = *(const ESP_LDS bf16x8*)(uintptr_t)(k_rd + st * kKTileBytes + (i & 1) * (32 * kKRow) + (i >> 1) * 32);
    };
    auto read_v = [&](int slot, uint32_t stage_off, int p) {
        const uint32_t vp = v_rd[p & 3] + stage_off + (32 * (p >> 3) + 16 * ((p >> 2) & 1)) * 256;
        frv[slot].s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ESP_LDS short4_t*)(uintptr_t)(vp));
        frv[slot].s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ESP_LDS short4_t*)(uintptr_t)(vp + 8 * 256));
    };

    // mask of a tile: key positions in lds_pos[st] against this lane's query position
    auto apply_mask = [&](floatx16 (&sc)[2], int st) {
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                const int4 kp = *(const int4*)(&lds_pos[st][32 * kvb + 8 * bb + 4 * hi]);
                if (kp.x > my_qpos) sc[kvb][4 * bb + 0] = -INFINITY;
                if (kp.y > my_qpos) sc[kvb][4 * bb + 1] = -INFINITY;
                if (kp.z > my_qpos) sc[kvb][4 * bb + 2] = -INFINITY;
                if (kp.w > my_qpos) sc[kvb][4 * bb + 3] = -INFINITY;
            }
    };
    // largest score of this lane's query row in a tile, in exp2 units (-inf if every key is masked)
    auto row_max = [&](const floatx16 (&sc)[2]) {
        float tmax = sc[0][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sc[0][r]);
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sc[1][r]);
        return half_swap_max(tmax) * a.scale_log2;
    };

    // probabilities of score pair c (0..15) of the current tile, in two parts placed behind the two MFMAs of a
    // step: exp2 first, then the fp32 partial sum (of the unrounded values: the log-sum-exp has to be good to
    // 1e-4) and the bf16 pack.  O^T accumulates the ROUNDED probabilities, so O is best normalised by their sum:
    // then it is a convex combination of value rows whatever the rounding did, an error common to the weights
    // cancels, and a row that sees a single key returns that key's value row exactly.  Summing the packed values
    // too (one dot product with (1, 1) per pair) costs 4 % of the loop's issue slots, though, and matters only
    // where few keys carry a row: so `track` is set in the masked iterations around the diagonal (a row with
    // fewer than 64 keys has no other) and in the exact sweep, and a tile at which the offset moves (a late,
    // dominant key) is accounted for in close_tile.  The plain iterations sum the unrounded values only.
    auto pair_exp = [&](const floatx16 (&sc)[2], int c) {
        const int kvb = c >> 3, r = 2 * (c & 7);
        p0 = __builtin_amdgcn_exp2f(fmaf(sc[kvb][r], a.scale_log2, -m_use));
        p1 = __builtin_amdgcn_exp2f(fmaf(sc[kvb][r + 1], a.scale_log2, -m_use));
    };
    auto packed_sum = [](uint32_t pk, float acc) {            // acc + both bf16 halves of pk
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
    };
    auto pair_sum_pack = [&](int c, bool track) {
        if (c == 0) psum = p0 + p1;
        else { psum += p0; psum += p1; }
        const uint32_t pk = pack_bf16(p0, p1);
        if (track) {
            psum_r = packed_sum(pk, c == 0 ? 0.f : psum_r);
            asm volatile("" :: "v"(psum_r));
        }
        asm volatile("" :: "v"(pk), "v"(psum));   // sum and pack here, not in a bunch further down
        pf[c >> 3][(c >> 2) & 1].u[c & 3] = pk;
    };

    // End of a tile in the pipelined sweep.  The probabilities were taken against the offset in use, without
    // looking at the scores first; that is exact as long as nothing left the range of fp32 / bf16, whatever their
    // size.  The tile sum tells: up to lim nothing needs doing (the common case: one compare); above it the
    // offset moves up to the tile's row maximum, and everything accumulated so far (the sum, O^T, and the last
    // chunk's P^T, which is multiplied only in the next iteration) is rescaled by the exact power of two.  A sum
    // that is not finite or beyond 2^100, or a first visible tile whose maximum is further than 2^64 from the
    // stand-in offset, means the optimistic pass cannot be trusted: the workgroup then redoes its rows with the
    // plain sweep below (`unsafe` is only ever set, never cleared).
    int32_t* lds_unsafe = (int32_t*)(smem + kLdsFlag);
    auto close_tile = [&](const floatx16 (&sc)[2], bool tracked) {
        lsum += psum;
        if (tracked) lcorr += psum_r - psum;
        if (__builtin_amdgcn_ballot_w64(!(psum <= lim)) != 0) {
            const float tm = row_max(sc);
            // A query row is held by two lanes (l and l | 32), each with the sum over its half of the tile's keys:
            // the decision must be the row's, or one half would go on with the old offset while the other one
            // moves.  Coded as a number so that a NaN sum counts too: 1 = above the limit, 3 = also out of range.
            const float mine = !(psum <= 0x1p100f) ? 3.f : !(psum <= lim) ? 1.f : 0.f;
            const float rows = half_swap_max(mine);
            const bool move = rows >= 1.f && tm != -INFINITY;        // a fresh row whose tile is all masked stays fresh
            const bool bad = move && (rows >= 3.f || (lim < 0.f && !(fabsf(tm) <= 64.f)));
            if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) *lds_unsafe = 1;
            if (!tracked) {
                // a tile whose rounded sum was not kept: its packed probabilities are all still in pf (the next
                // tile has not begun to overwrite them), so the sum is taken here; rows that stay where they are
                // have nothing dominant in this tile and go without
                float d = 0.f;
#pragma unroll
                for (int c = 0; c < 16; ++c) d = packed_sum(pf[c >> 3][(c >> 2) & 1].u[c & 3], d);
                if (move) lcorr += d - psum;
            }
            const float m_new = move ? m_use + ceilf(tm - m_use) : m_use;     // whole steps: alpha is a power of two
            const float alpha = __builtin_amdgcn_exp2f(m_use - m_new);        // 1 where nothing moves
            m_use = m_new;
            if (move) lim = kSumLimit;
            lsum *= alpha;
            lcorr *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t w = pf[1][1].u[e];
                pf[1][1].u[e] = pack_bf16(bf16_lo(w) * alpha, bf16_hi(w) * alpha);
            }
        }
    };

    const int mask_from = min(first_mask, tail_rows < kBN ? nkt - 1 : nkt);   // first tile this wavefront masks
    const char* k_next = kreq + 4 * tile_bytes;                       // K tile that iteration 0 fetches
    const char* v_next = vreq + 2 * tile_bytes;                       // V tile that iteration 0 fetches
    const int32_t* p_next = preq + 2 * kBN;

    // One tile per iteration, one workgroup barrier at its end; every wavefront runs the same uniform stream of
    // 16 steps, each with two MFMAs and one score pair:
    //   step m:  S^T MFMA m of tile j+1 (into sbuf[PAR^1]);  exp2 of pair m of tile j;
    //            O^T MFMA p = (m + 12) % 16;                 sum and pack of pair m
    // The O^T MFMAs trail the pairs by four steps, i.e. by one chunk of 16 keys: chunk c of tile j is multiplied
    // in steps 4c+4 .. 4c+7, and the last chunk in steps 0 .. 3 of iteration j+1 (after the loop for the last
    // tile).  With two wavefronts per SIMD, each issuing an instruction about every 6-8 cycles, this keeps an
    // MFMA (32 cycles) in front of every 5-6 other instructions of both wavefronts.
    // On entry: scores of tile j in sbuf[PAR]; frk = K fragments 0, 1 of tile j+1; frv = V^T fragments 12, 13
    // of tile j-1; pf[1][1] = last chunk of tile j-1 (zeros, and a zeroed V stage, when j = 0).
    // LDS stages: K(t), V(t) and the positions of tile t live in stage t % 4.  Iteration j reads K(j+1), the
    // first two fragments of K(j+2), V(j-1) (steps 0, 1) and V(j); it fetches K(j+4) over K(j), last read in
    // iteration j-1, and V(j+2) over V(j-2), last read in the first steps of iteration j-1: both before the
    // barrier that ended iteration j-1.  What a wavefront fetched in iteration j-1 has landed before the barrier
    // that ends its iteration j, and is first read in iteration j+1.
    // POOL, plain iterations: wavefront 6 fetches the slots of tile j+5 while j is below this (the sweep reaches that
    // tile, and it is a full one: see n_plain); no other wavefront does
    const int plain_slots = POOL && wave == 6 ? n_vis - 5 : INT_MIN;
    auto iteration = [&](auto st_c, auto par_c, auto plain_c, int j) {
        constexpr int ST = decltype(st_c)::value, PAR = decltype(par_c)::value;
        constexpr bool PLAIN = decltype(plain_c)::value != 0;
        constexpr int ST1 = (ST + 1) % kStages, ST2 = (ST + 2) % kStages, ST3 = (ST + 3) % kStages;
        floatx16 (&sc)[2] = sbuf[PAR];
        floatx16 (&sn)[2] = sbuf[PAR ^ 1];
        if (KEEP && !PLAIN && j < n_vis - 4) keep_tile(j, ST);
        if (!PLAIN && j >= mask_from) apply_mask(sc, ST);
        const bool do_k = PLAIN || j < n_vis - 4, do_v = PLAIN || j < n_vis - 2;
        const bool tail_k = !PLAIN && j + 4 == ragged_tile, tail_v = !PLAIN && j + 2 == ragged_tile;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int t = m >> 1, kvb = m & 1;
            // POOL: the slot of this step's transfer is read first, ahead of the step's fragment reads: LDS answers in
            // order, so a read placed next to the transfer would wait for those as well
            int32_t pslot = 0;
            if constexpr (POOL) {
                if (m == 1 && do_k && wave == 7) pslot = pool_slot(ST, pk2);
                if ((m == 3 || m == 6) && do_k) pslot = pool_slot(ST, m == 3 ? pk0 : pk1);
                if ((m == 9 || m == 12) && do_v) pslot = pool_slot(ST2, m == 9 ? pv0 : pv1);
            }
            if (t == 0) {                                 // S^T of tile j+1 (after the last tile: stale data, unused)
                floatx16 zero;
#pragma unroll
                for (int r = 0; r < 16; ++r) zero[r] = 0.f;
                sn[kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frk[m & 1].v, qf[t], zero, 0, 0, 0);
            } else {
                sn[kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frk[m & 1].v, qf[t], sn[kvb], 0, 0, 0);
            }
            pair_exp(sc, m);
            __builtin_amdgcn_sched_barrier(0);
            const int p = (m + 12) & 15;                  // O^T += V^T P^T, one chunk behind the pairs
            oacc[p & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frv[m & 1].v, pf[p >> 3][(p >> 2) & 1].v, oacc[p & 3], 0, 0, 0);
            // both fragments of step m+2; the K fragment last, so that the wait in front of its MFMA covers the
            // V^T fragment too (LDS reads return in order) and one wait per step is enough
            read_v(m & 1, (m < 2 ? ST3 : ST) * kTileBytes, (m + 14) & 15);
            read_k(m & 1, m + 2 < 16 ? ST1 : ST2, (m + 2) & 15);
            pair_sum_pack(m, !PLAIN);
            // the transfers of this iteration, spread out (a burst from all wavefronts at once backs up the memory
            // pipeline); the odd ones of wavefronts 7 and 0 go first, so that "all but the last four have landed"
            // is the same wait for every wavefront.  (Issued last instead, with a wait count per wavefront, they
            // would have a whole iteration more to land; measured, that is slower: 1.6 % on the 8K x 8K causal
            // shard, 6 % on a chunk against a 256K prefix.)
            if (m == 1) {
                if constexpr (POOL) {                   // over tile j+1's slots, last read in iteration j-1
                    if (PLAIN) { if (j < plain_slots) fetch_pool_slots_full(j + 5, ST1); }
                    else if (j + 5 < n_vis) fetch_pool_slots(j + 5, ST1);
                }
                if (KEEP && !PLAIN && do_k && j >= own_lo) fetch_slots(j + 4);
                if constexpr (POOL) {
                    if (do_k && wave == 7) load_to_lds_b128_at(lds_k0 + ST * kKTileBytes + 1024 * 16, pool_at(kreq, pslot, pk2));
                } else if (do_k) {
                    fetch_k_part(k_next, ST, tail_k, 2);
                }
                if (do_v) fetch_v_part(v_next, p_next, ST2, tail_v, 2);
            }
            if constexpr (POOL) {
                if (do_k && (m == 3 || m == 6))
                    load_to_lds_b128_at(lds_k0 + ST * kKTileBytes + 1024 * (m == 3 ? wave : wave + 8), pool_at(kreq, pslot, m == 3 ? pk0 : pk1));
                if (do_v && (m == 9 || m == 12))
                    load_to_lds_b128_at(lds_v0 + ST2 * kTileBytes + wave * 2048 + 1024 * (m / 12), pool_at(vreq, pslot, m == 9 ? pv0 : pv1));
            } else {
                if (do_k && (m == 3 || m == 6)) fetch_k_part(k_next, ST, tail_k, m / 6);
                if (do_v && (m == 9 || m == 12)) fetch_v_part(v_next, p_next, ST2, tail_v, m / 12);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        close_tile(sc, !PLAIN);
        k_next += tile_bytes; v_next += tile_bytes; p_next += kBN;
        // what iteration j-1 fetched must have landed; this iteration's own transfers may stay in flight
        if (do_k) wait_vm<4>();
        else if (do_v) wait_vm<2>();
        else wait_vm<0>();
        if (__builtin_expect(j + 1 == ragged_tile, 0)) { seal_tail(ST1); seal_slots(); }   // its positions landed with V(j+1), its slots before
        asm volatile("s_barrier" :: "v"(sn[0]), "v"(sn[1]), "v"(oacc[0]), "v"(oacc[1]), "v"(oacc[2]), "v"(oacc[3]),
                                    "v"(pf[1][1].v) : "memory");
    };

    // ---- prologue: K(0..3), V(0), V(1) were requested at kernel entry; S^T of tile 0, first fragments
    wait_vm<0>();
    // the Q fragments have landed with everything else; said in a way the compiler's own bookkeeping of loads
    // in flight understands, or every later reuse of these registers makes it wait for "pending" loads
    asm volatile("" :: "v"(qf[0]), "v"(qf[1]), "v"(qf[2]), "v"(qf[3]), "v"(qf[4]), "v"(qf[5]), "v"(qf[6]), "v"(qf[7]));
    if (ragged_tile >= 0 && ragged_tile < 2) seal_tail(ragged_tile);
    if (ragged_tile >= 0 && ragged_tile < 2) seal_slots();          // (in every other case before the iteration ahead of its own)
    wg_barrier();
    if (n_need > 0) {
        read_k(0, 0, 0);
        read_k(1, 0, 1);
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int t = m >> 1, kvb = m & 1;
            if (t == 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sbuf[0][kvb][r] = 0.f;
            }
            sbuf[0][kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frk[m & 1].v, qf[t], sbuf[0][kvb], 0, 0, 0);
            read_k(m & 1, m + 2 < 16 ? 0 : 1, (m + 2) & 15);        // ends with fragments 0, 1 of tile 1 (stale if absent)
        }
        read_v(0, 3 * kTileBytes, 12);                              // the zeroed stage: there is no tile -1
        read_v(1, 3 * kTileBytes, 13);
        // the offset starts at the exact row maximum of tile 0 wherever the row sees a key there (with ascending
        // positions: whenever it sees any key at all), so that the largest probability of a short row is exactly 1
        // and takes no bf16 rounding; rows still without a key keep the stand-in 0
        if (0 >= mask_from) apply_mask(sbuf[0], 0);
        const float tm0 = row_max(sbuf[0]);
        if (tm0 != -INFINITY) { m_use = tm0; lim = kSumLimit; }
    }
    // the sweep: a loop with a single exit over groups of four tiles (the stage of a tile is a compile-time
    // constant), then the zero to three tiles left over
    //   1. "plain" iterations: every transfer is a full tile that exists and this wavefront masks nothing, so the
    //      stream has no conditional code at all (a wavefront may leave this part earlier than its neighbours:
    //      the barriers and transfers per iteration are the same in both kinds);
    //   2. general iterations for the rest, again in groups of four, then one by one.
    //      (an owner: also short of its first owned tile, unless that is one of the sweep's last four, which are
    //      stored after the sweep)
    //      (POOL: one tile earlier before a ragged last tile, whose slot list a plain iteration does not fetch)
    const int n_plain = max(0, min(min(min(min(n_vis - 4, n_need), mask_from), ragged_tile >= 0 ? nkt - 5 - (POOL ? 1 : 0) : INT_MAX),
                                   KEEP && own_lo < n_vis - 4 ? own_lo : INT_MAX)) & ~3;
    int j = 0;
    for (; j < n_plain; j += 4) {
        iteration(IC<0>{}, IC<0>{}, IC<1>{}, j);
        iteration(IC<1>{}, IC<1>{}, IC<1>{}, j + 1);
        iteration(IC<2>{}, IC<0>{}, IC<1>{}, j + 2);
        iteration(IC<3>{}, IC<1>{}, IC<1>{}, j + 3);
    }
    for (; j + 4 <= n_need; j += 4) {
        iteration(IC<0>{}, IC<0>{}, IC<0>{}, j);
        iteration(IC<1>{}, IC<1>{}, IC<0>{}, j + 1);
        iteration(IC<2>{}, IC<0>{}, IC<0>{}, j + 2);
        iteration(IC<3>{}, IC<1>{}, IC<0>{}, j + 3);
    }
    if (j < n_need) {
        iteration(IC<0>{}, IC<0>{}, IC<0>{}, j);
        if (j + 1 < n_need) {
            iteration(IC<1>{}, IC<1>{}, IC<0>{}, j + 1);
            if (j + 2 < n_need) iteration(IC<2>{}, IC<0>{}, IC<0>{}, j + 2);
        }
    }
    if (n_need > 0) {                                               // last chunk of this wavefront's last tile
        const uint32_t last_off = (uint32_t)((n_need - 1) & 3) * kTileBytes;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            oacc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frv[m & 1].v, pf[1][1].v, oacc[m], 0, 0, 0);
            if (m < 2) read_v(m & 1, last_off, 14 + m);
        }
    }
    //   3. tiles that only other wavefronts can see: no arithmetic, but the same transfers, waits and barrier as
    //      in every other iteration (stages computed at run time here)
    for (int jj = n_need; jj < n_vis; ++jj) {
        const bool do_k = jj < n_vis - 4, do_v = jj < n_vis - 2;
        const bool tail_k = jj + 4 == ragged_tile, tail_v = jj + 2 == ragged_tile;
        if (KEEP && jj < n_vis - 4) keep_tile(jj, jj & 3);
        if (do_k && jj >= own_lo) fetch_slots(jj + 4);
        if (POOL && jj + 5 < n_vis) fetch_pool_slots(jj + 5, (jj + 1) & 3);
        if (do_k) fetch_k_part(k_next, jj & 3, tail_k, 2);
        if (do_v) fetch_v_part(v_next, p_next, (jj + 2) & 3, tail_v, 2);
        if (do_k) { fetch_k_part(k_next, jj & 3, tail_k, 0); fetch_k_part(k_next, jj & 3, tail_k, 1); }
        if (do_v) { fetch_v_part(v_next, p_next, (jj + 2) & 3, tail_v, 0); fetch_v_part(v_next, p_next, (jj + 2) & 3, tail_v, 1); }
        k_next += tile_bytes; v_next += tile_bytes; p_next += kBN;
        if (do_k) wait_vm<4>();
        else if (do_v) wait_vm<2>();
        else wait_vm<0>();
        if (__builtin_expect(jj + 1 == ragged_tile, 0)) { seal_tail((jj + 1) & 3); seal_slots(); }
        asm volatile("s_barrier" ::: "memory");
    }

    // The last four tiles of the sweep are still in their stages, with nothing in flight any more: an owner stores
    // those it owns now (under a causal mask the tiles on its diagonal, i.e. all it owns), where no hand-counted
    // wait has to sit out the stores.
    if (KEEP) {
        for (int t = max(max(own_lo, n_vis - 4), 0); t < own_hi; ++t) keep_tile(t, t & 3);
    }

    // ---- the plain sweep, for a workgroup whose optimistic pass met scores outside its range: one tile at a
    //      time through stage 0, row maximum before the exponentials, nothing overlapped.  Slow and exact.
    float m_fin = m_use;
    wg_barrier();                                                   // everyone's flag write and last LDS reads are done
    // the draw of the next item: as late as possible, so that items go out in the order in which workgroups
    // really become free, and early enough for the answer to arrive while the results are written
    unsigned long long next_item = 0;
    if (claim_from && tid == 0) {
        // an index the compiler cannot see through: with a provably uniform address it rewrites the atomic into
        // its one-per-wavefront form, which needs the answer at once instead of after the epilogue
        int idx = 0;
        asm volatile("" : "+v"(idx));
        next_item = __hip_atomic_fetch_add(claim_from + idx, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (__builtin_amdgcn_readfirstlane(*lds_unsafe) != 0) {
        float m_ref = -INFINITY;
        lsum = 0.f;
        lcorr = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
        for (int t = 0; t < n_vis; ++t) {
            wg_barrier();
            if constexpr (POOL) {
                fetch_pool_slots(t, 0);
                wait_vm<0>();
                wg_barrier();
            }
            fetch_k(kreq + (int64_t)t * tile_bytes, 0, t == ragged_tile);
            fetch_v(vreq + (int64_t)t * tile_bytes, preq + t * kBN, 0, t == ragged_tile);
            wait_vm<0>();
            if (t == ragged_tile) seal_tail(0);
            wg_barrier();
            floatx16 (&sc)[2] = sbuf[0];
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const int tt = m >> 1, kvb = m & 1;
                if (tt == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) sc[kvb][r] = 0.f;
                }
                read_k(0, 0, m);
                sc[kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frk[0].v, qf[tt], sc[kvb], 0, 0, 0);
            }
            apply_mask(sc, 0);
            const float m_new = fmaxf(m_ref, row_max(sc));
            const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            m_ref = m_new;
            lsum *= alpha;
            lcorr *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            m_use = (m_ref == -INFINITY) ? 0.f : m_ref;             // nothing visible yet: exp2(-inf - 0) = 0
#pragma unroll
            for (int c = 0; c < 16; ++c) { pair_exp(sc, c); pair_sum_pack(c, true); }
            lsum += psum;
            lcorr += psum_r - psum;
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                read_v(0, 0, p);
                oacc[p & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frv[0].v, pf[p >> 3][(p >> 2) & 1].v, oacc[p & 3], 0, 0, 0);
            }
        }
        m_fin = m_use;
        wg_barrier();                                               // the epilogue reuses the K stages
    }

    // ---- epilogue: normalise, write O (bf16) and LSE (natural log)
    const float ltot = half_swap_sum(lsum);
    const float ltot_r = half_swap_sum(lsum + lcorr);
    const float inv = ltot_r > 0.f ? 1.0f / ltot_r : 0.f;
    // O goes through LDS so that it leaves in whole rows: a lane holds 8-byte pieces of one row, 16 of them spread
    // over the 256 bytes; written to a wavefront-private 32 x 272-byte block (the K stages are free by now: the
    // barrier above ended all tile reads) they come back as 16 lanes x 16 bytes per row, four rows per store.
    const int rows_here = min(32, q_hi - (q_lo + wave * 32));       // rows of this wavefront that exist (may be <= 0)
    if (!a.o_f32) {
        unsigned char* blk = smem + kLdsK + wave * (32 * kKRow);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                uint2 w;
                w.x = pack_bf16(oacc[db][4 * bb + 0] * inv, oacc[db][4 * bb + 1] * inv);
                w.y = pack_bf16(oacc[db][4 * bb + 2] * inv, oacc[db][4 * bb + 3] * inv);
                *(uint2*)(blk + qi * kKRow + (32 * db + 8 * bb + 4 * hi) * 2) = w;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");          // same wavefront wrote what it reads next
        const int rsub = lane >> 4, c16 = lane & 15;
        uint16_t* orow = (uint16_t*)a.O + ((int64_t)(q_lo + wave * 32 + rsub) * a.Hq + h) * kHeadDim + 8 * c16;
        const int64_t ostep = (int64_t)4 * a.Hq * kHeadDim;
        if (rows_here >= 32) {                                      // all rows exist: eight stores in a row, no branches
            uint4 w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = *(const uint4*)(blk + (4 * i + rsub) * kKRow + 16 * c16);
#pragma unroll
            for (int i = 0; i < 8; ++i) *(uint4*)(orow + i * ostep) = w[i];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int r = 4 * i + rsub;
                const uint4 w = *(const uint4*)(blk + r * kKRow + 16 * c16);
                if (r < rows_here) *(uint4*)(orow + i * ostep) = w;
            }
        }
    } else {
        // fp32 output (a partial that stays on this GPU until the merge): rows of 512 bytes, padded to 528 in LDS;
        // the eight blocks of 32 rows fill the V and K stages exactly.  Two rows per store, 16 stores.
        constexpr int kFRow = 4 * kHeadDim + 16;
        static_assert(kPfWaves * 32 * kFRow <= kStages * (kTileBytes + kKTileBytes), "fp32 output staging must fit the tile stages");
        unsigned char* blk = smem + kLdsV + wave * (32 * kFRow);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int bb = 0; bb < 4; ++bb)
                *(float4*)(blk + qi * kFRow + (32 * db + 8 * bb + 4 * hi) * 4) =
                    make_float4(oacc[db][4 * bb + 0] * inv, oacc[db][4 * bb + 1] * inv, oacc[db][4 * bb + 2] * inv, oacc[db][4 * bb + 3] * inv);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const int rsub = lane >> 5, c32 = lane & 31;
        float* orow = (float*)a.O + ((int64_t)(q_lo + wave * 32 + rsub) * a.Hq + h) * kHeadDim + 4 * c32;
        const int64_t ostep = (int64_t)2 * a.Hq * kHeadDim;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            uint4 w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = *(const uint4*)(blk + (2 * (8 * half + i) + rsub) * kFRow + 16 * c32);
            if (rows_here >= 32) {
#pragma unroll
                for (int i = 0; i < 8; ++i) *(uint4*)(orow + (8 * half + i) * ostep) = w[i];
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (2 * (8 * half + i) + rsub < rows_here) *(uint4*)(orow + (8 * half + i) * ostep) = w[i];
            }
        }
    }
    if (row_ok && hi == 0)
        a.LSE[(int64_t)my_row * a.Hq + h] = ltot > 0.f ? (m_fin + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
    if (claim_from && tid == 0) *lds_next = draw_finish(claim_from, next_item);
    return true;
    };
    if constexpr (RETAIN) {
        if (own_hi > own_lo) return body(IC<1>{});
    }
    return body(IC<0>{});
    };

    // ---- persistent workgroups, one per CU.  Consecutive workgroup ids land on consecutive XCDs, each with a
    //      private L2, so XCD x keeps the heads [x * per, (x + 1) * per) (all query heads of a KV head together):
    //      a queue of M items, heaviest first (later query tiles of a causal request see more keys).  All but the
    //      last one or two rounds of a queue are dealt to the XCD's L workgroups back and forth (0 .. L-1,
    //      L-1 .. 0, ...), which for the linear size profile of a causal sweep gives every workgroup the same
    //      total.  XCDs do not run at quite the same speed, though, so the light items at the end of all queues
    //      form one pool that every workgroup draws from, through a device-wide counter, as it becomes free:
    //      a faster XCD takes more of them, and a workgroup whose dealt items were lighter a heavier one.  Pool
    //      items mostly miss their XCD's L2, but they are few and small.  Without the XCD split (head count not
    //      a multiple of 8) the same scheme runs with one queue over all workgroups.
    {
        const int P = gridDim.x, p = blockIdx.x;
        const bool split = a.heads_per_xcd > 0;
        const int L = split ? P >> 3 : P, l = split ? p >> 3 : p, x = split ? p & 7 : 0;
        const int width = split ? a.heads_per_xcd : a.Hq;
        const int M = a.q_tiles * width;
        // rounds dealt statically (M <= L: one item each).  With start-of-round waits everything is dealt: the items
        // are long and alike, a pool could not even them out further, and its items would walk K/V alone
        const int S = M <= L ? 1 : a.group_sync ? (M + L - 1) / L : max(1, (M - L) / L);
        const int pool_items = M > S * L ? (M - S * L) * (split ? 8 : 1) : 0;
        int i_pool = 0;
        bool drew = false;
        long long item_started = 0;
        for (int s = 0;; ++s) {
            // Long requests: the workgroups of an XCD that share a KV head (the same ones in every dealt round) walk
            // K/V together, and the L2 serves all but the first of them, as long as they stay within the few dozen
            // tiles it can hold per head.  Their items differ in length, so they would start the next round up to
            // that far apart, and since all run at the same speed the gap never closes: K/V then comes from memory
            // several times over.  So they wait for each other at the start of a dealt round: an arrival count per
            // (round parity, XCD, KV head), tagged like the pool counter, and a wait that ends by itself: after 1/64
            // of the time this workgroup's previous item took (waiting pays only where the items are long and alike;
            // where they differ a lot, as in a triangular sweep, it must cost next to nothing), at most after
            // kSyncTicks.  The deal goes back and forth, so a KV head is worked on by one set of workgroups in the
            // even rounds and by another in the odd ones: with a count per parity, the same workgroups meet at
            // a count every time, each adds one per round of that parity, and the round's target is that many full
            // sets.  Every workgroup arrives at every waiting round whether its wait is cut short or not, so the
            // total a count reaches is known beforehand, and the arrival that completes it clears the count (a
            // launch replayed from a captured graph carries the tag it was recorded with and must not find its own
            // earlier counts).
            if (a.group_sync && s >= 1 && (s + 1) * L <= M && tid == 0) {
                const int m_next = s * L + ((s & 1) ? L - 1 - l : l);
                unsigned long long* ctr = a.pool + 2 + ((s & 1) * 8 + x) * width + (m_next % width) / G;
                const uint32_t set = (uint32_t)((L / width) * G);                       // workgroups on one KV head
                const uint32_t target = set * (uint32_t)((s + (s & 1)) >> 1);            // rounds of this parity so far, this one included
                const int s_last = M / L - 1;                                            // last round that waits
                const uint32_t total = set * (uint32_t)((s & 1) ? (s_last + 1) >> 1 : s_last >> 1);
                const int before_me = draw_finish(ctr, __hip_atomic_fetch_add(ctr, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                if ((uint32_t)before_me + 1 == total) {
                    __hip_atomic_store(ctr, 0ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else if ((uint32_t)before_me + 1 < target) {
                    const long long t0 = wall_clock64();
                    const long long patience = min((long long)a.sync_ticks, (t0 - item_started) >> 6);
                    for (;;) {
                        const unsigned long long cur = __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        // a count that is no longer this launch's was cleared by its last arrival (see above)
                        if ((uint32_t)(cur >> 32) != a.tag || (uint32_t)cur >= target) break;
                        if (wall_clock64() - t0 > patience) break;
                        __builtin_amdgcn_s_sleep(16);
                    }
                }
            }
            if (s > 0) wg_barrier();                                  // every wavefront is done with the LDS of the previous item
            if (drew) i_pool = __builtin_amdgcn_readfirstlane(*lds_next);
            // every workgroup draws once per item from its last dealt one on, until a draw comes back empty: P draws
            // plus one per pool item.  The very last one clears the counter (replayed launches, see above).
            if (drew && i_pool == pool_items + P - 1 && tid == 0)
                __hip_atomic_store(a.pool, 0ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int qu, m;
            if (s < S) {
                qu = x;
                m = s * L + ((s & 1) ? L - 1 - l : l);
            } else {
                if (i_pool >= pool_items) break;
                qu = split ? i_pool & 7 : 0;                          // the queues take turns: still heaviest first
                m = S * L + (split ? i_pool >> 3 : i_pool);
            }
            if (m >= M) break;                                        // a last dealt round that is not full
            unsigned long long* claim = (s >= S - 1 && pool_items > 0) ? a.pool : nullptr;
            if (a.group_sync) item_started = wall_clock64();
            const bool ran = process(m / width, qu * width + m % width, claim);
            drew = claim != nullptr;
            if (drew && !ran) {                                       // no such query tile: it drew nothing
                wg_barrier();                                         // everyone has read the previous answer
                if (tid == 0)
                    *lds_next = draw_finish(claim, __hip_atomic_fetch_add(claim, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            }
        }
    }
}

esp_status launch_prefill(const void* q, const void* k, const void* v, const int32_t* q_pos, const int32_t* kv_pos,
                          const int32_t* cu_q, const int32_t* cu_kv, int32_t batch, int32_t Tq, int32_t Tkv,
                          int32_t max_q, int32_t max_kv, int32_t Hq, int32_t Hkv, float softmax_scale,
                          int32_t causal, int32_t o_f32, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                          const int32_t* retain_slot, void* k_pool, void* v_pool, const int32_t* kv_slot,
                          hipStream_t stream) {
    (void)max_q; (void)max_kv;
    PrefillArgs a;
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
    a.q_pos = q_pos; a.kv_pos = kv_pos; a.cu_q = cu_q; a.cu_kv = cu_kv;
    a.O = O; a.LSE = LSE; a.o_f32 = o_f32 ? 1 : 0;
    a.kv_slot = kv_slot;
    a.retain_slot = retain_slot; a.k_pool = (uint16_t*)k_pool; a.v_pool = (uint16_t*)v_pool;
    a.batch = batch; a.Tq = Tq; a.Tkv = Tkv; a.Hq = Hq; a.Hkv = Hkv; a.causal = causal ? 1 : 0;
    a.scale_log2 = softmax_scale * kLog2e;
    a.q_tiles = prefill_q_tiles_bound(Tq, batch);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return fail(ESP_ERR_HIP, "prefill: cannot query the device");
    const int64_t items = (int64_t)a.q_tiles * Hq;
    // one workgroup per CU (a workgroup fills a CU's registers and LDS); fewer if there are fewer items
    a.heads_per_xcd = (Hkv % 8 == 0 && cus % 8 == 0 && items >= cus) ? Hq / 8 : 0;
    const unsigned grid = (unsigned)(items < cus ? items : cus);
    a.pool = (unsigned long long*)workspace;
    a.tag = next_launch_tag();
    // start-of-round waits: one request with at least 512 KV tiles and a query chunk of at most an eighth of them
    // (a chunk against a long prefix: every query tile then sees nearly all of the shard, the items are alike), XCD
    // split, the same number of workgroups on every KV head of an XCD; the counters ((round parity, XCD, KV head),
    // at most 16 x heads_per_xcd) follow the pool counter
    a.group_sync = (a.heads_per_xcd > 0 && batch == 1 && Tkv >= 512 * kBN && (int64_t)Tkv >= 8 * (int64_t)Tq &&
                    (cus / 8) % a.heads_per_xcd == 0 &&
                    8 * (2 + 16 * (size_t)a.heads_per_xcd) <= workspace_bytes) ? 1 : 0;
    a.sync_ticks = g_sync_ticks.load(std::memory_order_relaxed);
    if (kv_slot && retain_slot) return fail(ESP_ERR_INVALID_ARG, "prefill: rows that are read from the pool are in it already");
    if (kv_slot)
        hipLaunchKernelGGL(prefill_kernel<2>, dim3(grid), dim3(kPfWaves * 64), 0, stream, a);
    else if (retain_slot)
        hipLaunchKernelGGL(prefill_kernel<1>, dim3(grid), dim3(kPfWaves * 64), 0, stream, a);
    else
        hipLaunchKernelGGL(prefill_kernel<0>, dim3(grid), dim3(kPfWaves * 64), 0, stream, a);
    return check_launch("prefill_kernel");
}

}  // namespace esp

// Decode partial attention on the matrix cores: every head layout but MHA-like ones that the row-burst kernel
// covers (MQA, GQA with any number of KV heads and query heads per KV head; Sec. 2.3 / Sec. 6: the method serves MHA,
// GQA and MQA alike).  With G query heads per KV head, a resident key row meets G queries: per token
// 2 * 2 * 128 * G flops on 512 bytes, which the vector ALU cannot keep up with from G = 4 or so on (a per-head kernel
// on it reached 11 % of the HBM rate for 32 / 1 heads, the row-burst kernel 46 % for 64 / 8), but which is a dense
// contraction.  The query heads of a request's KV head are the 32 columns of an MFMA tile (unused columns are zero):
//   S^T [32 keys x 32 heads] = K_tile [32 x 128] Q^T [128 x 32],   O^T [128 x 32 heads] += V_tile^T [128 x 32] P^T [32 x 32]
// The products are far from binding (16 MFMAs per 16 KiB gathered), so the kernel's time does not depend on G.
// Work is split as in the row-burst kernel: the concatenated token list in equal ranges, one workgroup per
// (range, KV head, chunk of up to 32 query heads); inside it every wavefront works alone, on every 8th tile of 32
// tokens of a request's part of the range, with an LDS block of its own (no workgroup barrier inside the sweep): it
// gathers the tile's K and V rows from their pool slots straight into LDS (16-byte pieces, a full address per
// lane), multiplies and keeps an exact running maximum; when the request's part of the range is done, the eight
// wavefronts combine their results through LDS and leave one partial (accumulator, maximum, sum) per
// (range + request, head) for the combine kernel.  (Eight partials per workgroup, one per wavefront, made the combine
// kernel read 145 MB for 32 / 1 heads and 64 requests: a quarter of the call's time.)
#include "mfma_tile.h"

namespace esp {

constexpr int kGqWaves = 8;
constexpr int kGqKRow = 272;                 // K rows padded by 16 bytes in LDS (bank spread of the operand reads)
constexpr int kGqKBytes = 9 * 1024;          // 32 x 272 = 8704 bytes, moved by 9 transfers of 1 KiB
constexpr int kGqVBytes = 32 * 256;
constexpr int kGqWaveBytes = kGqKBytes + kGqVBytes;

__global__ __launch_bounds__(kGqWaves * 64) void decode_partial_gq_kernel(
    const uint16_t* __restrict__ q, const char* __restrict__ k_pool, const char* __restrict__ v_pool,
    const int32_t* __restrict__ slot_idx, const int32_t* __restrict__ seq_offsets, int32_t B, int32_t total_tokens,
    int32_t range, int32_t Hq, int32_t Hkv, float scale_log2, float* __restrict__ part_acc, float* __restrict__ part_ml) {
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kGqWaves * kGqWaveBytes];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int qi = lane & 31, hi = lane >> 5;
    const int kvh = blockIdx.y;
    const int G = Hq / Hkv;
    const int g0 = blockIdx.z * 32;
    const int ng = min(32, G - g0);                             // query heads of this chunk: columns 0 .. ng-1
    const int h0 = kvh * G + g0;
    const int w = blockIdx.x;
    const uint32_t row_bytes = (uint32_t)Hkv * (kHeadDim * 2);
    const char* kbase = k_pool + (uint32_t)kvh * (kHeadDim * 2);
    const char* vbase = v_pool + (uint32_t)kvh * (kHeadDim * 2);
    const uint32_t lds_k = (uint32_t)(uintptr_t)(ESP_LDS unsigned char*)smem + wave * kGqWaveBytes;
    const uint32_t lds_v = lds_k + kGqKBytes;

    // operand read offsets (the layouts of the prefill kernel's tiles, for one block of 32 keys)
    const uint32_t k_rd = lds_k + qi * kGqKRow + hi * 16;
    const int j16 = lane & 15, jq = j16 >> 2, dblk = (lane >> 4) & 1;
    uint32_t v_rd[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_rd[db] = lds_v + (4 * hi + jq) * 256 + ((((db ^ jq) << 2) + 2 * dblk + ((j16 & 3) >> 1)) << 4) + (j16 & 1) * 8;

    int32_t t0 = w * range;
    const int32_t t1 = min(t0 + range, total_tokens);
    if (t0 >= t1) return;
    int lo = 0, hb = B;   // invariant: seq_offsets[lo] <= t0 < seq_offsets[hb]
    while (hb - lo > 1) {
        int mid = (lo + hb) >> 1;
        if (seq_offsets[mid] <= t0) lo = mid; else hb = mid;
    }
    int b = lo;

    union PFrag { uint32_t u[4]; bf16x8 v; };
    union VFrag { short4_t s[2]; bf16x8 v; };

    while (t0 < t1) {
        const int32_t req_end = seq_offsets[b + 1];
        if (req_end <= t0) { ++b; continue; }                   // empty request
        const int32_t pe = min(t1, req_end);
        const int32_t seg = pe - t0;                            // tokens of request b inside this range

        // Q^T fragments of the request's heads: column qi = head h0 + qi (columns past the chunk: zeros)
        bf16x8 qf[8];
        {
            const uint16_t* qp = q + ((int64_t)b * Hq + h0 + (qi < ng ? qi : 0)) * kHeadDim + 8 * hi;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                uint4 raw = *(const uint4*)(qp + 16 * t);
                if (qi >= ng) raw = make_uint4(0u, 0u, 0u, 0u);
                qf[t] = __builtin_bit_cast(bf16x8, raw);
            }
        }
        floatx16 oacc[4];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
        float m = -INFINITY;       // running maximum of this column's scaled scores (both halves hold the same)
        float l = 0.f, l_r = 0.f;  // this half's sums of the probabilities: as computed, and as rounded to bf16

        // slots of this wavefront's first tile: lane holds the slot of tile row lane % 32 (rows past the end: the last)
        auto tile_slots = [&](int i) {
            const int rows = min(32, seg - 32 * i);
            return slot_idx[t0 + 32 * i + min(qi, rows - 1)];
        };
        int32_t slots = 32 * wave < seg ? tile_slots(wave) : 0;
        for (int i = wave; 32 * i < seg; i += kGqWaves) {
            const int rows = min(32, seg - 32 * i);
            // ---- gather: K into rows of 272 bytes (lane L of transfer n fills LDS byte 1024 n + 16 L of the tile:
            //      row B / 272 at B % 272, padding slots fetch the row's first bytes), V into rows of 256 bytes with
            //      the 16-byte chunks XOR-swizzled by the row (chunk c of row r holds global chunk c ^ 4 (r % 4))
#pragma unroll
            for (int n = 0; n < 9; ++n) {
                const int Bo = 1024 * n + 16 * lane, row = min(Bo / kGqKRow, 31), within = Bo - (Bo / kGqKRow) * kGqKRow;
                const uint32_t s = (uint32_t)__shfl(slots, row);
                load_to_lds_b128_at_nt(lds_k + 1024 * n, kbase + ((uint64_t)s * row_bytes + (within < 256 ? within : 0)));
            }
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const int row = 4 * n + (lane >> 4);
                const uint32_t s = (uint32_t)__shfl(slots, row);
                load_to_lds_b128_at_nt(lds_v + 1024 * n, vbase + ((uint64_t)s * row_bytes + (((lane & 15) ^ ((row & 3) << 2)) << 4)));
            }
            int32_t slots_next = 0;
            if (32 * (i + kGqWaves) < seg) slots_next = tile_slots(i + kGqWaves);
            wait_vm<0>();
            asm volatile("" :: "v"(slots_next));

            // ---- S^T = K Q^T
            floatx16 sc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const bf16x8 kf = *(const ESP_LDS bf16x8*)(uintptr_t)(k_rd + t * 32);
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], sc, 0, 0, 0);
            }
            // register r of a lane is key 8 (r / 4) + 4 hi + r % 4 of the tile: keys past the end are hidden
            if (rows < 32) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + 4 * hi + (r & 3) >= rows) sc[r] = -INFINITY;
            }
            float tmax = sc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sc[r]);
            tmax = half_swap_max(tmax) * scale_log2;
            const float m_new = fmaxf(m, tmax);
            // nothing visible so far and nothing in this tile cannot happen (a tile has at least one row), but a
            // score may be -inf or NaN: exp2(-inf - -inf) must not leak a NaN into sums that are still zero
            const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
                l *= alpha; l_r *= alpha;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            }
            const float m_sub = (m == -INFINITY) ? 0.f : m;
            PFrag pf[2];
            float psum = 0.f, psum_r = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[2 * c], scale_log2, -m_sub));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[2 * c + 1], scale_log2, -m_sub));
                psum += p0 + p1;
                const uint32_t pk = pack_bf16(p0, p1);
                psum_r = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), __builtin_bit_cast(bf16x2, 0x3f803f80u), psum_r, false);
                pf[c >> 2].u[c & 3] = pk;
            }
            l += psum; l_r += psum_r;
            // ---- O^T += V^T P^T, 16 keys per step
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int t2 = p >> 2, db = p & 3;
                const uint32_t vp = v_rd[db] + (16 * t2) * 256;
                VFrag fv;
                fv.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ESP_LDS short4_t*)(uintptr_t)(vp));
                fv.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ESP_LDS short4_t*)(uintptr_t)(vp + 8 * 256));
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv.v, pf[t2].v, oacc[db], 0, 0, 0);
            }
            // the tile's LDS reads are complete before the next gather may overwrite it
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            slots = slots_next;
        }

        // ---- the partial of (range + request): O^T accumulated the ROUNDED probabilities, so each wavefront first
        //      brings it to the scale of its unrounded sum (the combine kernel divides by the sum that travels with
        //      the partial, and takes the log-sum-exp from it); then the 8 wavefronts' results are combined through
        //      LDS (their tile blocks are free now): register rho of every lane to row rho of the wavefront's block,
        //      64 lanes x 4 bytes a row, then maximum and sum; wavefront j combines registers 8j .. 8j+7 of all
        //      eight and writes them out.  One partial per (range + request, head) leaves the workgroup.
        const float l_tot = half_swap_sum(l), lr_tot = half_swap_sum(l_r);
        const float fix = lr_tot > 0.f ? l_tot / lr_tot : 0.f;
        float* mine = (float*)(smem + wave * kGqWaveBytes);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[(16 * db + r) * 64 + lane] = oacc[db][r] * fix;
        mine[64 * 64 + lane] = m;
        mine[65 * 64 + lane] = l_tot;
        __syncthreads();
        {
            float mw[kGqWaves], mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < kGqWaves; ++u) {
                mw[u] = ((const float*)(smem + u * kGqWaveBytes))[64 * 64 + lane];
                mx = fmaxf(mx, mw[u]);
            }
            float lsum = 0.f, out[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < kGqWaves; ++u) {
                const float* blk = (const float*)(smem + u * kGqWaveBytes);
                const float lu = blk[65 * 64 + lane];
                // a wavefront without a tile of this request (sum 0) has nothing to add
                const float c = lu > 0.f ? __builtin_amdgcn_exp2f(mw[u] - mx) : 0.f;
                lsum += lu * c;
#pragma unroll
                for (int e = 0; e < 8; ++e) out[e] += blk[(8 * wave + e) * 64 + lane] * c;
            }
            if (qi < ng) {
                const int64_t ph = (int64_t)(w + b) * Hq + h0 + qi;
                // registers 8 wave .. 8 wave + 7 = block db = wave / 2, r = 8 (wave % 2) .. + 7: two runs of four rows
                float* dst = part_acc + ph * kHeadDim + 32 * (wave >> 1) + 16 * (wave & 1) + 4 * hi;
                *(float4*)(dst) = make_float4(out[0], out[1], out[2], out[3]);
                *(float4*)(dst + 8) = make_float4(out[4], out[5], out[6], out[7]);
                if (wave == 0 && hi == 0) *(float2*)(part_ml + ph * 2) = make_float2(mx, lsum);
            }
        }
        __syncthreads();                                        // the blocks are read: the next request may gather into them
        t0 = pe;
        ++b;
    }
}

esp_status launch_decode_gq(const void* q, const void* k_pool, const void* v_pool, const int32_t* slot_idx,
                            const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t range, int32_t nwg,
                            int32_t Hq, int32_t Hkv, float scale_log2, float* part_acc, float* part_ml, hipStream_t stream) {
    const int G = Hq / Hkv;
    const int chunks = (G + 31) / 32;
    if (Hkv > 65535 || chunks > 65535) return fail(ESP_ERR_UNSUPPORTED, "decode: too many heads for one launch");
    hipLaunchKernelGGL(decode_partial_gq_kernel, dim3(nwg, Hkv, chunks), dim3(kGqWaves * 64), 0, stream, (const uint16_t*)q,
                       (const char*)k_pool, (const char*)v_pool, slot_idx, seq_offsets, B, total_tokens, range, Hq, Hkv,
                       scale_log2, part_acc, part_ml);
    return check_launch("decode_partial_gq_kernel");
}

}  // namespace esp

// esp_partial_attn_decode: one query token per request against the key/value rows this
// instance holds in its token-granular pool (distributed decoding, Sec. 4.2 / Fig. 8; pool at
// single-token granularity, Sec. 6).  The path is HBM-bound (about one flop per byte), so the
// design is about the gather:
//   * a pool row [Hkv, 128] bf16 is contiguous; a wavefront reads 1 KiB of it per load
//     instruction (4 KV heads x 128 elements, 16 bytes per lane), and the 8 wavefronts of a
//     workgroup cover neighbouring 1 KiB pieces of the same rows at the same time, so each
//     random slot is one multi-KiB burst;
//   * split-K with an even share: the concatenated token list of all requests is cut
//     into equal ranges, one per workgroup; a range that crosses request boundaries yields
//     one partial per (workgroup, request), stored at slot workgroup + request, which is
//     unique because both indices only grow along the token list;
//   * dot products on the vector ALU with a 16-lane butterfly per head, online softmax in
//     the exp2 domain per batch of tokens, fp32 accumulation;
//   * a second kernel combines the partials of each (request, head) and writes O, LSE.
#include <mutex>

#include "esp_common.h"

namespace esp {

// Split-K partials of the entry point that allocates nothing: a fixed block of device memory that every GPU the
// library runs on holds until the process ends.  In host code the array's name is only a stand-in; its device
// address is asked for once per device (static_scratch below) and that pointer is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[ESP_DECODE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call on that device).
static esp_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(ESP_ERR_HIP, "decode (static scratch): cannot identify the current device");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr)
            return fail(ESP_ERR_HIP, "decode (static scratch): hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ESP_OK;
}

constexpr int kDecWaves = 8;         // wavefronts per workgroup
constexpr int kDecTB = 4;            // tokens per wavefront per loop step
constexpr int kDecMaxWG = 1024;      // ranges (workgroups) along the token list

struct DecodeGeom {
    int32_t nwg;        // ranges
    int32_t range;      // tokens per range
    int32_t nhb_wg;     // 1 KiB head blocks handled by one workgroup (1, 2, 4 or 8)
    int32_t nt;         // wavefronts sharing one head block (token interleave) = 8 / nhb_wg
    int32_t ygroups;    // workgroups along y when a row has more than 8 head blocks
};

// Head counts of the row-burst kernel: whole 1 KiB head blocks (4 KV heads) that split the 8 wavefronts evenly, and
// one or two query heads per KV head.  Everything else (other KV head counts, larger query groups) goes to the
// matrix-core kernel of decode_gq.hip, which gathers one KV head's 256 bytes of a row at a time but does not pay for
// the size of the group: measured against it, this kernel's dot products on the vector ALU fall behind from four
// query heads per KV head on (16/4: 59 % of the HBM rate here, 71 % there; 64/8: 46 % and 68 %), and lead with one
// or two (32/32: 74 % and 69 %; 32/16: 68 % and 65 %).
static bool decode_burst_layout(int32_t Hq, int32_t Hkv) {
    const int G = Hq / Hkv;
    return (Hkv == 4 || Hkv == 8 || Hkv == 16 || Hkv % 32 == 0) && (G == 1 || G == 2);
}

static DecodeGeom decode_geom(int32_t total_tokens, int32_t Hq, int32_t Hkv) {
    DecodeGeom g;
    if (!decode_burst_layout(Hq, Hkv)) {
        // matrix-core kernel: every wavefront of a workgroup works on the same KV head, a tile of 32 tokens each per
        // step; the workgroup combines its wavefronts itself, so there is one partial per (range + request, head)
        g.nhb_wg = 0;
        g.nt = 1;
        g.ygroups = Hkv;
        int64_t step = (int64_t)kDecWaves * 32;
        int64_t want = ((int64_t)total_tokens + kDecMaxWG - 1) / kDecMaxWG;
        if (want < 2 * step) want = 2 * step;
        want = (want + step - 1) / step * step;
        g.range = (int32_t)want;
        g.nwg = (int32_t)(((int64_t)total_tokens + want - 1) / want);
        if (g.nwg < 1) g.nwg = 1;
        return g;
    }
    int nhb = Hkv / 4;
    g.nhb_wg = nhb < 8 ? nhb : 8;
    g.nt = kDecWaves / g.nhb_wg;
    g.ygroups = (nhb + 7) / 8;
    int64_t step = (int64_t)g.nt * kDecTB;                       // tokens one workgroup consumes per loop step
    int64_t want = ((int64_t)total_tokens + kDecMaxWG - 1) / kDecMaxWG;
    int64_t min_range = 8 * step;                                // do not cut finer than 8 loop steps
    if (want < min_range) want = min_range;
    want = (want + step - 1) / step * step;
    g.range = (int32_t)want;
    g.nwg = (int32_t)(((int64_t)total_tokens + want - 1) / want);
    if (g.nwg < 1) g.nwg = 1;
    return g;
}

// workspace: fp32 accumulators [slots][nt][Hq][128], then (m, l) pairs [slots][nt][Hq][2]
static size_t decode_slots(const DecodeGeom& g, int32_t B) { return (size_t)g.nwg + (size_t)B; }

size_t decode_workspace_bytes(int32_t B, int32_t total_tokens, int32_t Hq, int32_t Hkv) {
    DecodeGeom g = decode_geom(total_tokens, Hq, Hkv);
    size_t n = decode_slots(g, B) * (size_t)g.nt * (size_t)Hq;
    return n * (kHeadDim + 2) * sizeof(float) + 256;
}

__device__ __forceinline__ float row16_sum(float x) {
    // all-reduce over the 16 lanes of a DPP row by rotations (8, 4, 2, 1)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x128, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x124, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x122, 0xf, 0xf, false));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x121, 0xf, 0xf, false));
    return x;
}

__device__ __forceinline__ void unpack8(const uint4& w, float (&f)[8]) {
    f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x); f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
    f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z); f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

template <int G>
__global__ __launch_bounds__(kDecWaves * 64) void decode_partial_kernel(
    const uint16_t* __restrict__ q, const uint4* __restrict__ k_pool, const uint4* __restrict__ v_pool,
    const int32_t* __restrict__ slot_idx, const int32_t* __restrict__ seq_offsets, int32_t B, int32_t total_tokens,
    int32_t range, int32_t nhb_wg, int32_t Hq, int32_t Hkv, float scale_log2, float* __restrict__ part_acc,
    float* __restrict__ part_ml) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nt = kDecWaves / nhb_wg;
    const int hb = blockIdx.y * 8 + wave % nhb_wg;   // 1 KiB head block of the row
    const int tsub = wave / nhb_wg;                  // token interleave index among nt wavefronts
    const int w = blockIdx.x;
    const int row_chunks = Hkv * (kHeadDim * 2 / 16);          // 16-byte pieces per pool row
    const int lane_chunk = hb * 64 + lane;                     // this lane's piece within a row
    const int kvh = hb * 4 + (lane >> 4);                      // KV head of this lane
    const int dseg = (lane & 15) * 8;                          // first of its 8 elements

    int32_t t0 = w * range;
    const int32_t t1 = min(t0 + range, total_tokens);
    if (t0 >= t1) return;

    // request holding token t0: the last b with seq_offsets[b] <= t0
    int lo = 0, hi = B;   // invariant: seq_offsets[lo] <= t0 < seq_offsets[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (seq_offsets[mid] <= t0) lo = mid; else hi = mid;
    }
    int b = lo;

    while (t0 < t1) {
        int32_t req_end = seq_offsets[b + 1];
        if (req_end <= t0) { ++b; continue; }                   // empty request
        const int32_t pe = min(t1, req_end);

        float qf[G][8];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            uint4 qw = *(const uint4*)(q + ((int64_t)b * Hq + kvh * G + gi) * kHeadDim + dseg);
            unpack8(qw, qf[gi]);
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[gi][e] *= scale_log2;
        }
        float m[G], l[G], acc[G][8];
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            m[gi] = -INFINITY; l[gi] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[gi][e] = 0.f;
        }

        for (int32_t base = t0 + tsub; base < pe; base += nt * kDecTB) {
            uint4 kw[kDecTB], vw[kDecTB];
            bool valid[kDecTB];
#pragma unroll
            for (int u = 0; u < kDecTB; ++u) {
                int32_t tok = base + u * nt;
                valid[u] = tok < pe;
                int32_t slot = slot_idx[valid[u] ? tok : base];  // uniform per wavefront
                int64_t off = (int64_t)slot * row_chunks + lane_chunk;
                kw[u] = load_once(&k_pool[off]);
                vw[u] = load_once(&v_pool[off]);
            }
            float s[kDecTB][G];
#pragma unroll
            for (int u = 0; u < kDecTB; ++u) {
                float kf[8];
                unpack8(kw[u], kf);
#pragma unroll
                for (int gi = 0; gi < G; ++gi) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) d = fmaf(qf[gi][e], kf[e], d);
                    d = row16_sum(d);
                    s[u][gi] = valid[u] ? d : -INFINITY;
                }
            }
#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                float mx = m[gi];
#pragma unroll
                for (int u = 0; u < kDecTB; ++u) mx = fmaxf(mx, s[u][gi]);
                // the first token of a step is always valid, so mx is finite here
                float alpha = __builtin_amdgcn_exp2f(m[gi] - mx);
                m[gi] = mx;
                l[gi] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[gi][e] *= alpha;
#pragma unroll
                for (int u = 0; u < kDecTB; ++u) s[u][gi] = __builtin_amdgcn_exp2f(s[u][gi] - mx);
            }
#pragma unroll
            for (int u = 0; u < kDecTB; ++u) {
                float vf[8];
                unpack8(vw[u], vf);
#pragma unroll
                for (int gi = 0; gi < G; ++gi) {
                    l[gi] += s[u][gi];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[gi][e] = fmaf(s[u][gi], vf[e], acc[gi][e]);
                }
            }
        }

        // partial of (range w, request b): slot w + b, sub-slot tsub
        const int64_t pslot = ((int64_t)(w + b) * nt + tsub) * Hq;
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            int64_t ph = pslot + kvh * G + gi;
            float4* dst = (float4*)(part_acc + ph * kHeadDim + dseg);
            dst[0] = make_float4(acc[gi][0], acc[gi][1], acc[gi][2], acc[gi][3]);
            dst[1] = make_float4(acc[gi][4], acc[gi][5], acc[gi][6], acc[gi][7]);
            if ((lane & 15) == 0) *(float2*)(part_ml + ph * 2) = make_float2(m[gi], l[gi]);
        }
        t0 = pe;
        ++b;
    }
}


// One workgroup per (request, head): 4 groups of 64 lanes split the partials, each lane owns
// two output elements; the groups are then combined through LDS.
//
// PEERS: the master of a multi-master decode (Sec. 4.2) also holds the partial results its peers returned for the
// same queries (bf16 O, natural-log LSE).  They enter the same log-sum-exp combination here, so the local result is
// never rounded to bf16 on its own and no separate merge launch follows.
template <bool PEERS>
__global__ __launch_bounds__(256) void decode_combine_kernel(const int32_t* __restrict__ seq_offsets,
                                                             int32_t range, int32_t nt, int32_t Hq,
                                                             const float* __restrict__ part_acc,
                                                             const float* __restrict__ part_ml,
                                                             MergeArgs peers, int32_t n_peers,
                                                             uint32_t* __restrict__ O, float* __restrict__ LSE) {
    const int b = blockIdx.x / Hq, h = blockIdx.x % Hq;
    const int dp = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int32_t s0 = seq_offsets[b], s1 = seq_offsets[b + 1];
    float M = -INFINITY, L = 0.f, a0 = 0.f, a1 = 0.f;
    if (s1 > s0) {
        const int w_lo = s0 / range, w_hi = (s1 - 1) / range;
        const int n = (w_hi - w_lo + 1) * nt;
        for (int i = grp; i < n; i += 4) {
            int64_t ph = ((int64_t)(w_lo + b) * nt + i) * Hq + h;   // sub-slots of consecutive ranges are contiguous
            float2 ml = *(const float2*)(part_ml + ph * 2);
            if (ml.y == 0.f) continue;                              // a wavefront that saw no token
            float2 a = *(const float2*)(part_acc + ph * kHeadDim + dp * 2);
            float mx = fmaxf(M, ml.x);
            float c_old = __builtin_amdgcn_exp2f(M - mx), c_new = __builtin_amdgcn_exp2f(ml.x - mx);
            L = L * c_old + ml.y * c_new;
            a0 = a0 * c_old + a.x * c_new;
            a1 = a1 * c_old + a.y * c_new;
            M = mx;
        }
    }
    __shared__ float sm[4], sl[4], sa[4][128];
    if (dp == 0) { sm[grp] = M; sl[grp] = L; }
    sa[grp][dp * 2] = a0;
    sa[grp][dp * 2 + 1] = a1;
    __syncthreads();
    if (grp == 0) {
        float mx = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
        const int64_t pair = (int64_t)b * Hq + h;
        float lse_p[ESP_MAX_PARTIALS];                            // the peers' LSE in base-2 units, like mx
        if (PEERS) {
#pragma unroll
            for (int p = 0; p < ESP_MAX_PARTIALS; ++p) {
                lse_p[p] = (p < n_peers) ? peers.LSE_parts[p][pair] * kLog2e : -INFINITY;
                mx = fmaxf(mx, lse_p[p]);
            }
        }
        float Lt = 0.f, o0 = 0.f, o1 = 0.f;
        if (mx != -INFINITY) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float c = __builtin_amdgcn_exp2f(sm[g] - mx);     // exp2(-inf) = 0 for an idle group
                Lt += sl[g] * c;
                o0 += sa[g][dp * 2] * c;
                o1 += sa[g][dp * 2 + 1] * c;
            }
            if (PEERS) {
#pragma unroll
                for (int p = 0; p < ESP_MAX_PARTIALS; ++p) {
                    if (p < n_peers) {
                        const float w = __builtin_amdgcn_exp2f(lse_p[p] - mx);   // a peer's rows are normalised: mass w
                        const uint32_t o = ((const uint32_t*)peers.O_parts[p])[pair * (kHeadDim / 2) + dp];
                        if (w != 0.f) {                           // keeps the garbage of an empty partial out of the sum
                            Lt += w;
                            o0 += w * bf16_lo(o);
                            o1 += w * bf16_hi(o);
                        }
                    }
                }
            }
            float inv = 1.0f / Lt;
            o0 *= inv; o1 *= inv;
        }
        O[pair * (kHeadDim / 2) + dp] = pack_bf16(o0, o1);
        if (dp == 0) LSE[pair] = (mx == -INFINITY) ? -INFINITY : (mx + __builtin_amdgcn_logf(Lt)) * kLn2;
    }
}

esp_status launch_decode_static(const void* q, const void* k_pool, const void* v_pool, const int32_t* slot_idx,
                                const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t Hq, int32_t Hkv,
                                float softmax_scale, void* O, float* LSE, hipStream_t stream) {
    const size_t need = decode_workspace_bytes(B, total_tokens, Hq, Hkv);
    if (need > (size_t)ESP_DECODE_STATIC_SCRATCH_BYTES)
        return fail(ESP_ERR_WORKSPACE, "decode (static scratch): this call needs %zu bytes of scratch memory, the built-in block holds %zu; "
                    "use esp_partial_attn_decode with a workspace", need, (size_t)ESP_DECODE_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    const esp_status st = static_scratch(&ws);
    if (st != ESP_OK) return st;
    return launch_decode(q, k_pool, v_pool, slot_idx, seq_offsets, B, total_tokens, Hq, Hkv, softmax_scale, O, LSE, ws,
                         (size_t)ESP_DECODE_STATIC_SCRATCH_BYTES, stream);
}

esp_status launch_decode(const void* q, const void* k_pool, const void* v_pool, const int32_t* slot_idx,
                         const int32_t* seq_offsets, int32_t B, int32_t total_tokens, int32_t Hq, int32_t Hkv,
                         float softmax_scale, void* O, float* LSE, void* workspace, size_t workspace_bytes,
                         hipStream_t stream, const MergeArgs* peers, int32_t n_peers) {
    (void)workspace_bytes;
    DecodeGeom g = decode_geom(total_tokens, Hq, Hkv);
    size_t n = decode_slots(g, B) * (size_t)g.nt * (size_t)Hq;
    float* part_acc = (float*)workspace;
    float* part_ml = part_acc + n * kHeadDim;
    const int G = Hq / Hkv;
    if (total_tokens > 0 && g.nhb_wg == 0) {
        esp_status st = launch_decode_gq(q, k_pool, v_pool, slot_idx, seq_offsets, B, total_tokens, g.range, g.nwg, Hq, Hkv,
                                         softmax_scale * kLog2e, part_acc, part_ml, stream);
        if (st != ESP_OK) return st;
    } else if (total_tokens > 0) {
        dim3 grid(g.nwg, g.ygroups), block(kDecWaves * 64);
        float sl2 = softmax_scale * kLog2e;
#define ESP_DECODE_LAUNCH(GG)                                                                                   \
    hipLaunchKernelGGL(decode_partial_kernel<GG>, grid, block, 0, stream, (const uint16_t*)q,                   \
                       (const uint4*)k_pool, (const uint4*)v_pool, slot_idx, seq_offsets, B, total_tokens,      \
                       g.range, g.nhb_wg, Hq, Hkv, sl2, part_acc, part_ml)
        switch (G) {
            case 1: ESP_DECODE_LAUNCH(1); break;
            case 2: ESP_DECODE_LAUNCH(2); break;
            default: return fail(ESP_ERR_UNSUPPORTED, "decode: Hq/Hkv=%d unsupported", G);
        }
#undef ESP_DECODE_LAUNCH
        esp_status st = check_launch("decode_partial_kernel");
        if (st != ESP_OK) return st;
    }
    const dim3 cgrid((unsigned)((int64_t)B * Hq));
    if (peers != nullptr && n_peers > 0)
        hipLaunchKernelGGL(decode_combine_kernel<true>, cgrid, dim3(256), 0, stream, seq_offsets, g.range, g.nt, Hq,
                           (const float*)part_acc, (const float*)part_ml, *peers, n_peers, (uint32_t*)O, LSE);
    else
        hipLaunchKernelGGL(decode_combine_kernel<false>, cgrid, dim3(256), 0, stream, seq_offsets, g.range, g.nt, Hq,
                           (const float*)part_acc, (const float*)part_ml, MergeArgs{}, 0, (uint32_t*)O, LSE);
    return check_launch("decode_combine_kernel");
}

}  // namespace esp

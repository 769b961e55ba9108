// Streaming (memory-bound) partial attention: one query token against a range of
// KV rows, for the heads that share one KV head.  This is the per-request
// "distinct part" of prefix-shared attention for decode rows (BatchLLM
// Sec. 4.3.3, Sec. 5: a matrix-vector product per request), and the fallback
// for every row when the dtype / head_dim has no matrix-core path.
//
// One workgroup (4 wavefronts) per item.  A KV row is read by 16 lanes, 16 or
// 32 bytes each, so every wavefront load instruction fetches four whole rows;
// the workgroup therefore runs 16 independent online-softmax streams over
// interleaved rows and merges them through LDS at the end.  Dot products are
// finished with DPP adds inside each 16-lane row; no matrix cores are used.
#include "bllm_device.h"
#include "bllm_internal.h"

namespace bllm {
namespace {

constexpr int kStreamThreads = 256;
constexpr int kStreams = 16;       // 4 wavefronts x 4 sixteen-lane rows
constexpr int kRowsPerStep = 4;    // KV rows each stream handles per loop step

template <bool kBf16, int EPL>
__device__ __forceinline__ void load_chunk(const void* base, size_t elem_off, bool valid, float (&out)[EPL]) {
    if constexpr (kBf16) {
        const uint16_t* p = static_cast<const uint16_t*>(base) + elem_off;
        if constexpr (EPL == 8) {
            uint4 raw = valid ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
            out[0] = bf16_lo(raw.x); out[1] = bf16_hi(raw.x);
            out[2] = bf16_lo(raw.y); out[3] = bf16_hi(raw.y);
            out[4] = bf16_lo(raw.z); out[5] = bf16_hi(raw.z);
            out[6] = bf16_lo(raw.w); out[7] = bf16_hi(raw.w);
        } else {
            uint2 raw = valid ? *reinterpret_cast<const uint2*>(p) : make_uint2(0, 0);
            out[0] = bf16_lo(raw.x); out[1] = bf16_hi(raw.x);
            out[2] = bf16_lo(raw.y); out[3] = bf16_hi(raw.y);
        }
    } else {
        const float* p = static_cast<const float*>(base) + elem_off;
#pragma unroll
        for (int x = 0; x < EPL; x += 4) {
            float4 raw = valid ? *reinterpret_cast<const float4*>(p + x) : make_float4(0.f, 0.f, 0.f, 0.f);
            out[x] = raw.x; out[x + 1] = raw.y; out[x + 2] = raw.z; out[x + 3] = raw.w;
        }
    }
}

template <bool kPrecise>
__device__ __forceinline__ float exp2_of(float x) {
    if constexpr (kPrecise) return exp2f(x);
    else return __builtin_amdgcn_exp2f(x);
}

template <bool kBf16, int D, int RHO>
__global__ __launch_bounds__(kStreamThreads) void stream_attention_kernel(
    const Item* __restrict__ items, const void* __restrict__ q_, const void* __restrict__ k_,
    const void* __restrict__ v_, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, float scale) {
    constexpr int EPL = D / 16;
    constexpr bool kPrecise = !kBf16;
    __shared__ float sm_m[kStreams][RHO];
    __shared__ float sm_l[kStreams][RHO];
    __shared__ float sm_acc[kStreams][RHO][D];

    const Item it = items[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int sub = lane & 15;
    const int stream = (tid >> 6) * 4 + (lane >> 4);
    const int head0 = it.kv_head * RHO;
    const float sc2 = scale * kLog2e;

    float* dst_o;
    float* dst_l;
    if (it.dst_row >= 0) {
        dst_o = ws_o + (static_cast<size_t>(it.dst_row) * n_q_heads + head0) * D;
        dst_l = ws_lse + static_cast<size_t>(it.dst_row) * n_q_heads + head0;
    } else {
        dst_o = o_part + (static_cast<size_t>(it.q_row0) * n_q_heads + head0) * D;
        dst_l = lse_part + static_cast<size_t>(it.q_row0) * n_q_heads + head0;
    }
    const int kv_len = it.kv_len < it.vis0 ? it.kv_len : it.vis0;   // single row: sees min(KV_LEN, VIS0)
    if (kv_len <= 0) {
        for (int idx = tid; idx < RHO * D; idx += kStreamThreads) dst_o[idx] = 0.f;
        if (tid < RHO) dst_l[tid] = -INFINITY;
        return;
    }

    float qf[RHO][EPL];
#pragma unroll
    for (int e = 0; e < RHO; ++e)
        load_chunk<kBf16, EPL>(q_, (static_cast<size_t>(it.q_row0) * n_q_heads + head0 + e) * D + sub * EPL, true, qf[e]);

    float m[RHO], l[RHO], acc[RHO][EPL];
#pragma unroll
    for (int e = 0; e < RHO; ++e) {
        m[e] = -INFINITY;
        l[e] = 0.f;
#pragma unroll
        for (int x = 0; x < EPL; ++x) acc[e][x] = 0.f;
    }

    const size_t row_stride = static_cast<size_t>(n_kv_heads) * D;
    const size_t kv_base = (static_cast<size_t>(it.kv_row0) * n_kv_heads + it.kv_head) * D + sub * EPL;

    for (int base = stream; base < kv_len; base += kStreams * kRowsPerStep) {
        float kf[kRowsPerStep][EPL], vf[kRowsPerStep][EPL];
        bool valid[kRowsPerStep];
#pragma unroll
        for (int u = 0; u < kRowsPerStep; ++u) {
            const int row = base + u * kStreams;
            valid[u] = row < kv_len;
            const size_t off = kv_base + static_cast<size_t>(row) * row_stride;
            load_chunk<kBf16, EPL>(k_, off, valid[u], kf[u]);
            load_chunk<kBf16, EPL>(v_, off, valid[u], vf[u]);
        }
        float s[kRowsPerStep][RHO];
#pragma unroll
        for (int u = 0; u < kRowsPerStep; ++u) {
#pragma unroll
            for (int e = 0; e < RHO; ++e) {
                float part = 0.f;
#pragma unroll
                for (int x = 0; x < EPL; ++x) part = fmaf(qf[e][x], kf[u][x], part);
                const float full = row16_sum(part) * sc2;
                s[u][e] = valid[u] ? full : -INFINITY;
            }
        }
#pragma unroll
        for (int e = 0; e < RHO; ++e) {
            float mx = m[e];
#pragma unroll
            for (int u = 0; u < kRowsPerStep; ++u) mx = fmaxf(mx, s[u][e]);
            const float alpha = exp2_of<kPrecise>(m[e] - mx);
            float p[kRowsPerStep];
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < kRowsPerStep; ++u) {
                p[u] = exp2_of<kPrecise>(s[u][e] - mx);
                psum += p[u];
            }
            l[e] = l[e] * alpha + psum;
            m[e] = mx;
#pragma unroll
            for (int x = 0; x < EPL; ++x) {
                float a = acc[e][x] * alpha;
#pragma unroll
                for (int u = 0; u < kRowsPerStep; ++u) a = fmaf(p[u], vf[u][x], a);
                acc[e][x] = a;
            }
        }
    }

    // ---- merge the 16 streams ---------------------------------------------------------------
#pragma unroll
    for (int e = 0; e < RHO; ++e) {
        if (sub == 0) {
            sm_m[stream][e] = m[e];
            sm_l[stream][e] = l[e];
        }
#pragma unroll
        for (int x = 0; x < EPL; ++x) sm_acc[stream][e][sub * EPL + x] = acc[e][x];
    }
    __syncthreads();
    for (int idx = tid; idx < RHO * D; idx += kStreamThreads) {
        const int e = idx / D;
        const int d = idx - e * D;
        float top = -INFINITY;
#pragma unroll
        for (int s2 = 0; s2 < kStreams; ++s2) top = fmaxf(top, sm_m[s2][e]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < kStreams; ++s2) {
            const float w = exp2_of<kPrecise>(sm_m[s2][e] - top);   // empty stream: exp2(-inf) = 0
            num = fmaf(w, sm_acc[s2][e][d], num);
            den = fmaf(w, sm_l[s2][e], den);
        }
        dst_o[idx] = num / den;
        if (d == 0) dst_l[e] = (top + log2f(den)) * kLn2;
    }
}

template <bool kBf16, int D>
hipError_t launch_rho(const LaunchCtx& c, const Item* items, int32_t n_items, const void* q, const void* k, const void* v,
                      float* o_part, float* lse_part, float* ws_o, float* ws_lse) {
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    dim3 grid(n_items), block(kStreamThreads);
#define BLLM_LAUNCH_STREAM(R)                                                                                         \
    hipLaunchKernelGGL((stream_attention_kernel<kBf16, D, R>), grid, block, 0, c.stream, items, q, k, v, o_part,     \
                       lse_part, ws_o, ws_lse, c.desc->n_q_heads, c.desc->n_kv_heads, c.scale)
    switch (rho) {
        case 1: BLLM_LAUNCH_STREAM(1); break;
        case 2: BLLM_LAUNCH_STREAM(2); break;
        case 4: BLLM_LAUNCH_STREAM(4); break;
        case 8: BLLM_LAUNCH_STREAM(8); break;
        default: return hipErrorInvalidValue;
    }
#undef BLLM_LAUNCH_STREAM
    return hipGetLastError();
}

}  // namespace

hipError_t launch_stream_attention(const LaunchCtx& c, const Item* items, int32_t n_items, const void* q, const void* k,
                                   const void* v, float* o_part, float* lse_part, float* ws_o, float* ws_lse) {
    if (n_items <= 0) return hipSuccess;
    const bool bf16 = c.desc->dtype == BLLM_BF16;
    const int d = c.desc->head_dim;
    if (bf16 && d == 128) return launch_rho<true, 128>(c, items, n_items, q, k, v, o_part, lse_part, ws_o, ws_lse);
    if (bf16 && d == 64) return launch_rho<true, 64>(c, items, n_items, q, k, v, o_part, lse_part, ws_o, ws_lse);
    if (!bf16 && d == 128) return launch_rho<false, 128>(c, items, n_items, q, k, v, o_part, lse_part, ws_o, ws_lse);
    if (!bf16 && d == 64) return launch_rho<false, 64>(c, items, n_items, q, k, v, o_part, lse_part, ws_o, ws_lse);
    return hipErrorInvalidValue;
}

}  // namespace bllm

// Kernel and launcher of the streaming partial attention; the device code is in
// stream_attention_body.h.
#include "stream_attention_body.h"

namespace bllm {
namespace {

using namespace stream_detail;

template <bool kBf16, int D, int RHO, int WPI, bool kPieces>
__global__ __launch_bounds__(kStreamThreads) void stream_attention_kernel(
    const Item* __restrict__ items, int n_items, const void* __restrict__ q_, const void* __restrict__ k_,
    const void* __restrict__ v_, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, float scale, MergeTarget mt) {
    stream_attention_body<kBf16, D, RHO, WPI, kPieces>(blockIdx.x, items, n_items, q_, k_, v_, o_part, lse_part, ws_o, ws_lse,
                                                       n_q_heads, n_kv_heads, scale, mt);
}

template <bool kBf16, int D, int RHO>
hipError_t launch_wpi(const LaunchCtx& c, const Item* items, int32_t n_items, int wpi, const void* q, const void* k,
                      const void* v, float* o_part, float* lse_part, float* ws_o, float* ws_lse, const MergeTarget& mt) {
    dim3 block(kStreamThreads);
#define BLLM_LAUNCH_STREAM_P(W, P)                                                                                    \
    hipLaunchKernelGGL((stream_attention_kernel<kBf16, D, RHO, W, P>), dim3((n_items * W + 3) / 4), block, 0,        \
                       c.stream, items, n_items, q, k, v, o_part, lse_part, ws_o, ws_lse, c.desc->n_q_heads,           \
                       c.desc->n_kv_heads, c.scale, mt)
#define BLLM_LAUNCH_STREAM(W)                                                                                         \
    do {                                                                                                              \
        if (mt.row_split != nullptr) BLLM_LAUNCH_STREAM_P(W, true);                                                   \
        else BLLM_LAUNCH_STREAM_P(W, false);                                                                          \
    } while (0)
    switch (wpi) {
        case 1: BLLM_LAUNCH_STREAM(1); break;
        case 2: BLLM_LAUNCH_STREAM(2); break;
        default: BLLM_LAUNCH_STREAM(4); break;
    }
#undef BLLM_LAUNCH_STREAM
#undef BLLM_LAUNCH_STREAM_P
    return hipGetLastError();
}

template <bool kBf16, int D>
hipError_t launch_rho(const LaunchCtx& c, const Item* items, int32_t n_items, int wpi, const void* q, const void* k,
                      const void* v, float* o_part, float* lse_part, float* ws_o, float* ws_lse, const MergeTarget& mt) {
    switch (c.desc->n_q_heads / c.desc->n_kv_heads) {
        case 1: return launch_wpi<kBf16, D, 1>(c, items, n_items, wpi, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
        case 2: return launch_wpi<kBf16, D, 2>(c, items, n_items, wpi, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
        case 4: return launch_wpi<kBf16, D, 4>(c, items, n_items, wpi, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
        case 8: return launch_wpi<kBf16, D, 8>(c, items, n_items, wpi, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_stream_attention(const LaunchCtx& c, const Item* items, int32_t n_items, int waves_per_item,
                                   const void* q, const void* k, const void* v, float* o_part, float* lse_part,
                                   float* ws_o, float* ws_lse, const MergeTarget& mt) {
    if (n_items <= 0) return hipSuccess;
    const bool bf16 = c.desc->dtype == BLLM_BF16;
    const int d = c.desc->head_dim;
    const int w = waves_per_item;
    if (bf16 && d == 128) return launch_rho<true, 128>(c, items, n_items, w, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
    if (bf16 && d == 64) return launch_rho<true, 64>(c, items, n_items, w, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
    if (!bf16 && d == 128) return launch_rho<false, 128>(c, items, n_items, w, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
    if (!bf16 && d == 64) return launch_rho<false, 64>(c, items, n_items, w, q, k, v, o_part, lse_part, ws_o, ws_lse, mt);
    return hipErrorInvalidValue;
}

}  // namespace bllm

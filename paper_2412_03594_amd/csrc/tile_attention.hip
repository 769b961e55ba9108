// Kernel and launcher of the matrix-core partial attention; the device code is in
// tile_attention_body.h.
#include "tile_attention_body.h"

namespace bllm {
namespace {

using namespace tile_detail;

template <int NW, int BN>
__global__ __launch_bounds__(64 * NW, 2) void tile_attention_kernel(
    const Item* __restrict__ items, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, int log2_rho, float scale, MergeTarget mt) {
    tile_attention_body<NW, BN>(items[blockIdx.x], q, k, v, o_part, lse_part, ws_o, ws_lse, n_q_heads, n_kv_heads, log2_rho,
                                scale, mt);
}

// Workgroups [0, n_pairs) take a two-range item each (the longest work first), the others a plain tile.
template <int NW, int BN>
__global__ __launch_bounds__(64 * NW, 2) void tile_through_kernel(
    const Item* __restrict__ pairs, int n_pairs, const Item* __restrict__ items, const uint16_t* __restrict__ q,
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, const uint16_t* __restrict__ k2,
    const uint16_t* __restrict__ v2, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, int log2_rho, float scale, void* o_out, float* lse_out,
    int final_from_row) {
    const int b = blockIdx.x;
    Item it;
    SecondRange r2;
    r2.o_out = o_out;
    r2.lse_out = lse_out;
    r2.final_from_row = final_from_row;
    if (b < n_pairs) {
        it = pairs[2 * b];
        const Item own = pairs[2 * b + 1];
        r2.k = k2;
        r2.v = v2;
        r2.kv_row0 = own.kv_row0;
        r2.kv_len = own.kv_len;
        r2.vis0 = own.vis0;
    } else {
        it = items[b - n_pairs];
    }
    tile_attention_body<NW, BN>(it, q, k, v, o_part, lse_part, ws_o, ws_lse, n_q_heads, n_kv_heads, log2_rho, scale,
                                MergeTarget{}, r2);
}

}  // namespace

hipError_t launch_tile_attention(const LaunchCtx& c, const Item* items, int32_t n_items, int waves, const void* q,
                                 const void* k, const void* v, float* o_part, float* lse_part, float* ws_o,
                                 float* ws_lse, const MergeTarget& mt) {
    if (n_items <= 0) return hipSuccess;
    if (c.desc->dtype != BLLM_BF16 || c.desc->head_dim != kD || waves != 4) return hipErrorInvalidValue;
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    int log2_rho = 0;
    while ((1 << log2_rho) < rho) ++log2_rho;
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
#define BLLM_LAUNCH_TILE(NW_, BN_)                                                                                 \
    hipLaunchKernelGGL((tile_attention_kernel<NW_, BN_>), dim3(n_items), dim3(64 * NW_), 0, c.stream, items, qq, kk, vv, \
                       o_part, lse_part, ws_o, ws_lse, c.desc->n_q_heads, c.desc->n_kv_heads, log2_rho, c.scale, mt)
    BLLM_LAUNCH_TILE(4, 64);
#undef BLLM_LAUNCH_TILE
    return hipGetLastError();
}

hipError_t launch_tile_attention_through(const LaunchCtx& c, const Item* pairs, int32_t n_pairs, const Item* items,
                                         int32_t n_items, int waves, const void* q, const void* k, const void* v,
                                         const void* k2, const void* v2, float* o_part, float* lse_part, float* ws_o,
                                         float* ws_lse, void* o_out, float* lse_out, int32_t final_from_row) {
    if (n_pairs < 0 || n_pairs + n_items <= 0) return hipErrorInvalidValue;
    if (c.desc->dtype != BLLM_BF16 || c.desc->head_dim != kD || waves != 4 || n_items < 0) return hipErrorInvalidValue;
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    int log2_rho = 0;
    while ((1 << log2_rho) < rho) ++log2_rho;
    hipLaunchKernelGGL((tile_through_kernel<4, 64>), dim3(n_pairs + n_items), dim3(256), 0, c.stream, pairs, n_pairs, items,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                       static_cast<const uint16_t*>(k2), static_cast<const uint16_t*>(v2), o_part, lse_part, ws_o, ws_lse,
                       c.desc->n_q_heads, c.desc->n_kv_heads, log2_rho, c.scale, o_out, lse_out, final_from_row);
    return hipGetLastError();
}

}  // namespace bllm

// The distinct-suffix pass as ONE launch when a batch has both prefill chunks (matrix-core tiles with a
// causal bound) and decode rows (streaming items): workgroup b is a chunk tile or 4 / WPI streaming items
// (BatchLLM Sec. 4.3.3: different thread blocks of one kernel do different parts, each with its own
// tiling).  The two kinds of work do not depend on each other, so nothing is exchanged: the launch only
// removes the tail of the tile kernel before the streaming kernel and lets the bandwidth-bound items run
// beside the latency-bound tiles (measured on l8b_mixed: 239 us against 245 us for the two kernels one after
// the other).  Up to 4 query heads per KV head.  Device code: tile_attention_body.h, stream_attention_body.h.
#include "stream_attention_body.h"
#include "tile_attention_body.h"

namespace bllm {
namespace {

constexpr int kThreads = 256;

struct SuffixFusedArgs {
    const Item* tiles;
    const Item* rows;
    int n_tiles, n_rows_items;
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    float* o_part;
    float* lse_part;
    float* ws_o;
    float* ws_lse;
    int n_q_heads, n_kv_heads, log2_rho;
    float scale;
    MergeTarget mt;
};

template <int RHO, int WPI, bool kPieces>
__global__ __launch_bounds__(kThreads, 2) void suffix_fused_kernel(SuffixFusedArgs a) {
    const int b = blockIdx.x;
    if (b < a.n_tiles) {
        tile_detail::tile_attention_body<4, 64>(a.tiles[b], a.q, a.k, a.v, a.o_part, a.lse_part, a.ws_o, a.ws_lse, a.n_q_heads,
                                                a.n_kv_heads, a.log2_rho, a.scale, a.mt);
    } else {
        stream_detail::stream_attention_body<true, 128, RHO, WPI, kPieces>(b - a.n_tiles, a.rows, a.n_rows_items, a.q, a.k, a.v,
                                                                           a.o_part, a.lse_part, a.ws_o, a.ws_lse, a.n_q_heads,
                                                                           a.n_kv_heads, a.scale, a.mt);
    }
}

template <int RHO>
hipError_t launch_for_rho(const SuffixFusedArgs& a, int wpi, hipStream_t stream) {
#define BLLM_LAUNCH_SF_P(W, P)                                                                                              \
    hipLaunchKernelGGL((suffix_fused_kernel<RHO, W, P>), dim3(a.n_tiles + (a.n_rows_items * W + 3) / 4), dim3(kThreads), 0, \
                       stream, a)
#define BLLM_LAUNCH_SF(W)                                         \
    do {                                                          \
        if (a.mt.row_split != nullptr) BLLM_LAUNCH_SF_P(W, true); \
        else BLLM_LAUNCH_SF_P(W, false);                          \
    } while (0)
    switch (wpi) {
        case 1: BLLM_LAUNCH_SF(1); break;
        case 2: BLLM_LAUNCH_SF(2); break;
        default: BLLM_LAUNCH_SF(4); break;
    }
#undef BLLM_LAUNCH_SF
#undef BLLM_LAUNCH_SF_P
    return hipGetLastError();
}

}  // namespace

hipError_t launch_suffix_fused(const LaunchCtx& c, const Item* tiles, int32_t n_tiles, const Item* rows, int32_t n_rows_items,
                               int waves_per_item, const void* q, const void* k, const void* v, float* o_part,
                               float* lse_part, float* ws_o, float* ws_lse, const MergeTarget& mt) {
    if (n_tiles <= 0 || n_rows_items <= 0) return hipErrorInvalidValue;
    if (c.desc->dtype != BLLM_BF16 || c.desc->head_dim != 128) return hipErrorInvalidValue;
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    SuffixFusedArgs a;
    a.tiles = tiles;
    a.rows = rows;
    a.n_tiles = n_tiles;
    a.n_rows_items = n_rows_items;
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.o_part = o_part;
    a.lse_part = lse_part;
    a.ws_o = ws_o;
    a.ws_lse = ws_lse;
    a.n_q_heads = c.desc->n_q_heads;
    a.n_kv_heads = c.desc->n_kv_heads;
    a.log2_rho = rho == 1 ? 0 : rho == 2 ? 1 : rho == 4 ? 2 : 3;
    a.scale = c.scale;
    a.mt = mt;
    switch (rho) {
        case 1: return launch_for_rho<1>(a, waves_per_item, c.stream);
        case 2: return launch_for_rho<2>(a, waves_per_item, c.stream);
        case 4: return launch_for_rho<4>(a, waves_per_item, c.stream);
        default: return hipErrorInvalidValue;      // 8 heads per KV head: the streaming items need more registers
                                                   // than two workgroups per compute unit leave (measured slower)
    }
}

}  // namespace bllm

// Online-softmax reductions of partial attention results (BatchLLM Sec. 5:
// the results of the different parts are reduced through online softmax).
//   lse_merge_kernel     two partials -> final output in the layer's dtype
//   split_combine_kernel n partials of one pass (KV split for occupancy) -> that
//                        pass's fp32 partial
// Both are pure streaming kernels: every thread owns 4 consecutive head-dim
// elements of one (row, head) and reads/writes them with 16-byte accesses.
#include "bllm_device.h"
#include "bllm_internal.h"

#include <type_traits>

namespace bllm {
namespace {

constexpr int kMergeThreads = 256;

typedef float float4v __attribute__((ext_vector_type(4)));

// 16-byte load of data that is read exactly once (does not displace what the caches hold)
__device__ __forceinline__ float4 load_once(const float* p) {
    const float4v r = __builtin_nontemporal_load(reinterpret_cast<const float4v*>(p));
    return make_float4(r[0], r[1], r[2], r[3]);
}

template <bool kBf16Out>
__global__ __launch_bounds__(kMergeThreads) void lse_merge_kernel(
    const float* __restrict__ o_a, const float* __restrict__ lse_a, const float* __restrict__ o_b,
    const float* __restrict__ lse_b, void* __restrict__ o_out, float* __restrict__ lse_out, int64_t n_row_heads,
    int quads_per_row_head /* D/4 */) {
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kMergeThreads + threadIdx.x;
    const int64_t rh = gid / quads_per_row_head;
    if (rh >= n_row_heads) return;
    const int quad = static_cast<int>(gid - rh * quads_per_row_head);
    const size_t off = static_cast<size_t>(rh) * quads_per_row_head * 4 + quad * 4;
    // An empty part's rows are specified as 0, but never multiply garbage by 0.  The loads do not
    // wait for the weights: both rows are fetched at once and an empty part's values are dropped.
    const float4 ra = load_once(o_a + off);
    const float4 rb = load_once(o_b + off);
    const MergeWeights w = merge_weights(lse_a[rh], lse_b[rh]);
    store_out4<kBf16Out>(o_out, off, merge_value(w, ra.x, rb.x), merge_value(w, ra.y, rb.y), merge_value(w, ra.z, rb.z),
                         merge_value(w, ra.w, rb.w));
    if (lse_out != nullptr && quad == 0) lse_out[rh] = w.lse;
}

// Rows that have no keys in a pass (the prefix rows in the distinct-suffix pass): the pass's
// partial is (0, -inf); merging, the final output is the other part's result converted to
// the layer's dtype.  Rows row0 .. of the [n_rows, Hq, D] tensors; rh counts from row0 * Hq.
template <bool kBf16Out>
__global__ __launch_bounds__(kMergeThreads) void keyless_rows_kernel(
    const float* __restrict__ o_a, const float* __restrict__ lse_a, void* __restrict__ o_out,
    float* __restrict__ lse_out, float* __restrict__ o_part, float* __restrict__ lse_part, int64_t rh0,
    int64_t n_row_heads, int quads_per_row_head) {
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kMergeThreads + threadIdx.x;
    const int64_t rel = gid / quads_per_row_head;
    if (rel >= n_row_heads) return;
    const int64_t rh = rh0 + rel;
    const int quad = static_cast<int>(gid - rel * quads_per_row_head);
    const size_t off = static_cast<size_t>(rh) * quads_per_row_head * 4 + quad * 4;
    if (o_a != nullptr) {
        const float4 r = load_once(o_a + off);
        const float l = lse_a[rh];
        const bool empty = l == -INFINITY;       // an empty other part: its rows are not read as values
        store_out4<kBf16Out>(o_out, off, empty ? 0.f : r.x, empty ? 0.f : r.y, empty ? 0.f : r.z, empty ? 0.f : r.w);
        if (lse_out != nullptr && quad == 0) lse_out[rh] = l;
    } else {
        *reinterpret_cast<float4*>(o_part + off) = make_float4(0.f, 0.f, 0.f, 0.f);
        if (quad == 0) lse_part[rh] = -INFINITY;
    }
}

__global__ __launch_bounds__(kMergeThreads) void split_combine_kernel(
    const RowSplit* __restrict__ row_split, const float* __restrict__ ws_o, const float* __restrict__ ws_lse,
    float* __restrict__ o_part, float* __restrict__ lse_part, int64_t n_row_heads, int n_q_heads,
    int quads_per_row_head) {
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kMergeThreads + threadIdx.x;
    const int64_t rh = gid / quads_per_row_head;
    if (rh >= n_row_heads) return;
    const int quad = static_cast<int>(gid - rh * quads_per_row_head);
    const int64_t row = rh / n_q_heads;
    const int head = static_cast<int>(rh - row * n_q_heads);
    const RowSplit sp = row_split[row];
    if (sp.n_splits <= 0) return;      // this row was written directly by the pass
    // Splits are taken four at a time (two for a row with two splits): their log-sum-exps and
    // rows are fetched together, then folded into the running (maximum, numerator, denominator).
    const size_t rh_stride = static_cast<size_t>(sp.stride) * n_q_heads;             // between splits
    const size_t wrh0 = static_cast<size_t>(sp.ws_row0) * n_q_heads + head;
    const size_t elem = static_cast<size_t>(quads_per_row_head) * 4;
    float top = -INFINITY;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    float den = 0.f;
    auto fold = [&](auto width, int c0) {
        constexpr int kW = decltype(width)::value;
        float l[kW];
        float4 x[kW];
#pragma unroll
        for (int i = 0; i < kW; ++i) {
            const int c = min(c0 + i, sp.n_splits - 1);      // past the end: re-read the last split (unused)
            const size_t wrh = wrh0 + c * rh_stride;
            l[i] = ws_lse[wrh];
            x[i] = load_once(ws_o + wrh * elem + quad * 4);
        }
        float m = top;
#pragma unroll
        for (int i = 0; i < kW; ++i)
            if (c0 + i < sp.n_splits) m = fmaxf(m, l[i]);
        const float r = top == -INFINITY ? 0.f : expf(top - m);
        num.x *= r;
        num.y *= r;
        num.z *= r;
        num.w *= r;
        den *= r;
        top = m;
#pragma unroll
        for (int i = 0; i < kW; ++i)
            if (c0 + i < sp.n_splits) {
                const float w = expf(l[i] - m);
                num.x = fmaf(w, x[i].x, num.x);
                num.y = fmaf(w, x[i].y, num.y);
                num.z = fmaf(w, x[i].z, num.z);
                num.w = fmaf(w, x[i].w, num.w);
                den += w;
            }
    };
    if (sp.n_splits <= 2) {
        fold(std::integral_constant<int, 2>{}, 0);
    } else {
        for (int c0 = 0; c0 < sp.n_splits; c0 += 4) fold(std::integral_constant<int, 4>{}, c0);
    }
    const float inv = 1.f / den;       // every split of a split row holds at least one key
    const size_t off = static_cast<size_t>(rh) * quads_per_row_head * 4 + quad * 4;
    *reinterpret_cast<float4*>(o_part + off) = make_float4(num.x * inv, num.y * inv, num.z * inv, num.w * inv);
    if (quad == 0) lse_part[rh] = top + logf(den);
}

}  // namespace

hipError_t launch_lse_merge(const LaunchCtx& c, const float* o_a, const float* lse_a, const float* o_b,
                            const float* lse_b, void* o_out, float* lse_out) {
    const int64_t n_row_heads = static_cast<int64_t>(c.n_rows) * c.desc->n_q_heads;
    const int quads = c.desc->head_dim / 4;
    const int64_t threads = n_row_heads * quads;
    if (threads == 0) return hipSuccess;
    dim3 grid(static_cast<unsigned>((threads + kMergeThreads - 1) / kMergeThreads)), block(kMergeThreads);
    if (c.desc->dtype == BLLM_BF16)
        hipLaunchKernelGGL(lse_merge_kernel<true>, grid, block, 0, c.stream, o_a, lse_a, o_b, lse_b, o_out, lse_out,
                           n_row_heads, quads);
    else
        hipLaunchKernelGGL(lse_merge_kernel<false>, grid, block, 0, c.stream, o_a, lse_a, o_b, lse_b, o_out, lse_out,
                           n_row_heads, quads);
    return hipGetLastError();
}

hipError_t launch_keyless_rows(const LaunchCtx& c, int32_t row0, int32_t n_rows, float* o_part, float* lse_part,
                               const MergeTarget& mt) {
    const int64_t n_row_heads = static_cast<int64_t>(n_rows) * c.desc->n_q_heads;
    const int quads = c.desc->head_dim / 4;
    const int64_t threads = n_row_heads * quads;
    if (threads == 0) return hipSuccess;
    const int64_t rh0 = static_cast<int64_t>(row0) * c.desc->n_q_heads;
    dim3 grid(static_cast<unsigned>((threads + kMergeThreads - 1) / kMergeThreads)), block(kMergeThreads);
    if (c.desc->dtype == BLLM_BF16)
        hipLaunchKernelGGL(keyless_rows_kernel<true>, grid, block, 0, c.stream, mt.o_a, mt.lse_a, mt.o_out, mt.lse_out,
                           o_part, lse_part, rh0, n_row_heads, quads);
    else
        hipLaunchKernelGGL(keyless_rows_kernel<false>, grid, block, 0, c.stream, mt.o_a, mt.lse_a, mt.o_out, mt.lse_out,
                           o_part, lse_part, rh0, n_row_heads, quads);
    return hipGetLastError();
}

hipError_t launch_split_combine(const LaunchCtx& c, const RowSplit* row_split, const float* ws_o, const float* ws_lse,
                                float* o_part, float* lse_part) {
    const int64_t n_row_heads = static_cast<int64_t>(c.n_rows) * c.desc->n_q_heads;
    const int quads = c.desc->head_dim / 4;
    const int64_t threads = n_row_heads * quads;
    if (threads == 0) return hipSuccess;
    dim3 grid(static_cast<unsigned>((threads + kMergeThreads - 1) / kMergeThreads)), block(kMergeThreads);
    hipLaunchKernelGGL(split_combine_kernel, grid, block, 0, c.stream, row_split, ws_o, ws_lse, o_part, lse_part,
                       n_row_heads, c.desc->n_q_heads, quads);
    return hipGetLastError();
}

}  // namespace bllm

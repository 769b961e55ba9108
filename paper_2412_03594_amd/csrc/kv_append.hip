// Writes the new keys and values of a token batch into the KV memory (BatchLLM
// Sec. 3.3.1, Sec. 3.4: the KV of a shared prefix is kept once per group, apart from
// the KV of every request's distinct part).  A pure scatter of whole rows: packed row
// t of k_new / v_new goes to row row_kv_dst[t] of the suffix arrays, or to row
// -row_kv_dst[t] - 1 of the prefix arrays when that value is negative.  Every thread
// moves 16 bytes; a row of Hkv * D elements is a multiple of 128 bytes.
#include "bllm_internal.h"

namespace bllm {
namespace {

constexpr int kAppendThreads = 256;

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(
    const int32_t* __restrict__ row_kv_dst, const uint4v* __restrict__ k_new, const uint4v* __restrict__ v_new,
    uint4v* __restrict__ k_prefix, uint4v* __restrict__ v_prefix, uint4v* __restrict__ k_suffix,
    uint4v* __restrict__ v_suffix, int64_t n_units /* n_rows * units_per_row */, int units_per_row) {
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * kAppendThreads + threadIdx.x;
    if (gid >= n_units) return;
    const int64_t row = gid / units_per_row;
    const int unit = static_cast<int>(gid - row * units_per_row);
    const int32_t d = row_kv_dst[row];
    const bool to_prefix = d < 0;
    const size_t dst = static_cast<size_t>(to_prefix ? -(d + 1) : d) * units_per_row + unit;
    const bool is_v = blockIdx.y == 1;
    const uint4v* src = is_v ? v_new : k_new;
    uint4v* out = to_prefix ? (is_v ? v_prefix : k_prefix) : (is_v ? v_suffix : k_suffix);
    out[dst] = __builtin_nontemporal_load(src + gid);     // the source row is read once
}

}  // namespace

hipError_t launch_kv_append(const LaunchCtx& c, const int32_t* row_kv_dst, const void* k_new, const void* v_new,
                            void* k_prefix, void* v_prefix, void* k_suffix, void* v_suffix) {
    const size_t elem = c.desc->dtype == BLLM_BF16 ? 2 : 4;
    const int units_per_row = static_cast<int>(static_cast<size_t>(c.desc->n_kv_heads) * c.desc->head_dim * elem / 16);
    const int64_t n_units = static_cast<int64_t>(c.n_rows) * units_per_row;
    if (n_units == 0) return hipSuccess;
    dim3 grid(static_cast<unsigned>((n_units + kAppendThreads - 1) / kAppendThreads), 2), block(kAppendThreads);
    hipLaunchKernelGGL(kv_append_kernel, grid, block, 0, c.stream, row_kv_dst, static_cast<const uint4v*>(k_new),
                       static_cast<const uint4v*>(v_new), static_cast<uint4v*>(k_prefix), static_cast<uint4v*>(v_prefix),
                       static_cast<uint4v*>(k_suffix), static_cast<uint4v*>(v_suffix), n_units, units_per_row);
    return hipGetLastError();
}

}  // namespace bllm

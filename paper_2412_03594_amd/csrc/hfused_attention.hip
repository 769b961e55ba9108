// Horizontally fused prefix-shared attention (BatchLLM Sec. 4.3.3: the partial attention on the
// shared prefix and on the distinct part run as different thread blocks of ONE launch, each with
// its own tiling, which removes the tail of one kernel before the next and the launch gaps).
//
// Workgroup b of the grid takes, in this order, a matrix-core tile of the shared-prefix part, a
// two-range item (a prefill chunk that fills its own tiles: prefix range, then the request's own
// range, final output straight from the accumulators - it exchanges nothing and arrives nowhere), a
// matrix-core tile of another prefill chunk of the distinct part, or 4 / WPI streaming items (decode
// rows).  Every other part writes its fp32 partial result to the workspace exactly as the separate
// passes do; then it ARRIVES at the counter of each (token row, KV head) it covered.  The part
// that arrives last at a counter reduces all partials of that row and head through online
// softmax and writes the final output (Sec. 5).  Nobody waits for anybody: there is no spinning,
// every workgroup runs to its end whatever the others do.  A streaming item that finds, when it
// starts, that every prefix part of its row has already arrived is certain to be the last: it
// fetches those partials behind its own KV stream, folds them with its result in registers and
// writes the final output directly, with no partial of its own.
//
// Ordering: the partial results are written with device-scope atomic stores (they go through to
// the level all compute dies share); the barrier of the workgroup waits until every wavefront's
// stores have completed, and only then does one thread per (row, KV head) increment the counter
// with a device-scope atomic.  The workgroup that sees the last count reads the other parts'
// partials with device-scope atomic loads, after the count.  A device-scope FENCE is avoided on
// purpose: it writes back and invalidates a whole L2, and with thousands of workgroups doing so the
// launch measured 8 times slower than the separate passes.  The last arrival also puts the counter
// back to zero for the next call.
#include "stream_attention_body.h"
#include "tile_attention_body.h"

namespace bllm {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxUnits = 128;        // token rows of a tile (32 * 4 wavefronts / rho) at rho = 1

struct HFusedArgs {
    const Item* prefix_tiles;
    const Item* suffix_tiles;
    const Item* suffix_rows;
    const Item* pairs;    // two-range items: the prefix range, then the request's own range (2 items each)
    int n_prefix_tiles, n_suffix_tiles, n_suffix_rows, n_pairs;
    const uint16_t* q;
    const uint16_t* k_prefix;
    const uint16_t* v_prefix;
    const uint16_t* k_suffix;
    const uint16_t* v_suffix;
    float* o1;            // prefix partial [T, Hq, D] (rows whose prefix is not split)
    float* l1;            // [T, Hq]
    float* o2;            // suffix partial
    float* l2;
    float* ws_o;          // pieces of split prefixes
    float* ws_lse;
    const RowSplit* prefix_row_split;    // [T]
    int32_t* arrivals;    // [T, Hkv], zero before and after the launch
    void* o_out;          // [T, Hq, D] bf16
    float* lse_out;       // [T, Hq] or null
    int n_q_heads, n_kv_heads, log2_rho, n_request_rows;
    float scale;
};

template <int RHO, int WPI>
__global__ __launch_bounds__(kThreads, RHO == 8 ? 1 : 2) void hfused_attention_kernel(HFusedArgs a) {
    constexpr int kD = 128;
    constexpr int kItemsPerBlock = 4 / WPI;
    __shared__ int s_late_row[kMaxUnits];
    __shared__ int s_late_head[kMaxUnits];
    __shared__ int s_n_late;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    if (tid == 0) s_n_late = 0;

    // ---- this workgroup's part --------------------------------------------------------------
    int n_units;                 // (token row, KV head) pairs this workgroup produced a partial for
    int unit_row = 0, unit_head = 0;     // the pair of thread tid, for tid < n_units
    const MergeTarget none{};
    // role of this workgroup: a matrix-core item (prefix tiles, pairs, chunk tiles in this order), else block
    // sb of streaming items (they come last and fill the slots the long items leave; placing them right after
    // the prefix tiles measured slower: l8b_mixed 0.784 against 0.746 ms)
    const int n_tile_slots = a.n_prefix_tiles + a.n_pairs + a.n_suffix_tiles;
    const int tile_slot = b;
    const int sb = b - n_tile_slots;
    if (tile_slot < n_tile_slots) {
        const bool prefix = tile_slot < a.n_prefix_tiles;
        const bool pair = !prefix && tile_slot < a.n_prefix_tiles + a.n_pairs;
        Item it;
        SecondRange r2;
        if (pair) {
            // both parts of these rows in this workgroup: nothing to exchange, nobody to arrive at
            it = a.pairs[2 * (tile_slot - a.n_prefix_tiles)];
            const Item own = a.pairs[2 * (tile_slot - a.n_prefix_tiles) + 1];
            r2.k = a.k_suffix;
            r2.v = a.v_suffix;
            r2.kv_row0 = own.kv_row0;
            r2.kv_len = own.kv_len;
            r2.vis0 = own.vis0;
            r2.o_out = a.o_out;
            r2.lse_out = a.lse_out;
        } else {
            it = prefix ? a.prefix_tiles[tile_slot] : a.suffix_tiles[tile_slot - a.n_prefix_tiles - a.n_pairs];
        }
        const bool from_prefix = prefix || pair;
        tile_detail::tile_attention_body<4, 64, true>(it, a.q, from_prefix ? a.k_prefix : a.k_suffix,
                                                from_prefix ? a.v_prefix : a.v_suffix, prefix ? a.o1 : a.o2,
                                                prefix ? a.l1 : a.l2, a.ws_o, a.ws_lse, a.n_q_heads, a.n_kv_heads,
                                                a.log2_rho, a.scale, none, r2);
        n_units = pair ? 0 : it.n_rows;
        unit_row = it.q_row0 + tid;
        unit_head = it.kv_head;
    } else {
        const int first = sb * kItemsPerBlock;
        // Has every prefix part of the item's row arrived already?  One decision per item, taken by the
        // first wavefront of the WPI that share it.
        __shared__ int s_certain[kItemsPerBlock];
        __shared__ int s_pending[kItemsPerBlock];
        const int wave = tid >> 6;
        const int item_in_block = wave / WPI;
        const int my_item = first + item_in_block;
        const bool item_ok = my_item < a.n_suffix_rows;
        int32_t* my_counter = nullptr;
        if (item_ok) {
            const Item it = a.suffix_rows[my_item];
            my_counter = a.arrivals + static_cast<size_t>(it.q_row0) * a.n_kv_heads + it.kv_head;
            if (tid == item_in_block * WPI * 64) {
                const RowSplit sp = a.prefix_row_split[it.q_row0];
                const int arrived = __hip_atomic_load(my_counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_certain[item_in_block] = arrived == (sp.n_splits > 0 ? sp.n_splits : 1) ? 1 : 0;
            }
        } else if (tid == item_in_block * WPI * 64) {
            s_certain[item_in_block] = 0;
        }
        __syncthreads();
        const bool certain_last = s_certain[item_in_block] != 0;
        MergeTarget mt{};
        if (certain_last) {
            mt.o_a = a.o1;
            mt.lse_a = a.l1;
            mt.o_out = a.o_out;
            mt.lse_out = a.lse_out;
            mt.row_split = a.prefix_row_split;
            mt.ws_o = a.ws_o;
            mt.ws_lse = a.ws_lse;
        }
        stream_detail::stream_attention_body<true, kD, RHO, WPI, true, true>(sb, a.suffix_rows, a.n_suffix_rows, a.q, a.k_suffix,
                                                                       a.v_suffix, a.o2, a.l2, a.ws_o, a.ws_lse, a.n_q_heads,
                                                                       a.n_kv_heads, a.scale, mt);
        if (tid == item_in_block * WPI * 64) {
            // a certain-last item has written the final output: its counter goes back to zero for the next
            // call; any other item still has to arrive
            if (certain_last) atomicExch(my_counter, 0);
            s_pending[item_in_block] = (item_ok && !certain_last) ? my_item : -1;
        }
        __syncthreads();
        n_units = kItemsPerBlock;                          // slots; empty ones are skipped below
        unit_row = -1;
        if (tid < kItemsPerBlock && s_pending[tid] >= 0) {
            const Item it = a.suffix_rows[s_pending[tid]];
            unit_row = it.q_row0;
            unit_head = it.kv_head;
        }
    }

    // ---- arrive; the last arrival of a (row, KV head) reduces its partials ---------------------
    coherent_stores_done();
    __syncthreads();             // every wavefront's partial stores have completed
    if (tid < n_units && unit_row >= 0) {
        const RowSplit sp = a.prefix_row_split[unit_row];
        const int expected = (sp.n_splits > 0 ? sp.n_splits : 1) + (unit_row < a.n_request_rows ? 1 : 0);
        int32_t* counter = a.arrivals + static_cast<size_t>(unit_row) * a.n_kv_heads + unit_head;
        if (atomicAdd(counter, 1) == expected - 1) {
            atomicExch(counter, 0);                       // every part has arrived: ready for the next call
            const int slot = atomicAdd(&s_n_late, 1);
            s_late_row[slot] = unit_row;
            s_late_head[slot] = unit_head;
        }
    }
    __syncthreads();
    const int n_late = s_n_late;
    if (n_late == 0) return;
    constexpr int kPairs = RHO * (kD / 4);                // (head of the KV head, 4 consecutive elements)
    for (int idx = tid; idx < n_late * kPairs; idx += kThreads) {
        const int u = idx / kPairs;
        const int p = idx - u * kPairs;
        const int row = s_late_row[u];
        const int head = s_late_head[u] * RHO + p / (kD / 4);
        const int x = 4 * (p % (kD / 4));
        const size_t rh = static_cast<size_t>(row) * a.n_q_heads + head;
        // the partials of this element, six at a time: prefix pieces (or the one prefix partial), then
        // the suffix partial; an absent one repeats the previous address and is not folded
        PartialFold f;
        const RowSplit sp = a.prefix_row_split[row];
        const int n_prefix = sp.n_splits > 0 ? sp.n_splits : 1;
        const int n_parts = n_prefix + (row < a.n_request_rows ? 1 : 0);
        auto part = [&](int c, const float*& po, const float*& pl) {
            if (c >= n_prefix) {
                po = a.o2 + rh * kD + x;
                pl = a.l2 + rh;
            } else if (sp.n_splits > 0) {
                const size_t wrh = static_cast<size_t>(sp.ws_row0 + c * sp.stride) * a.n_q_heads + head;
                po = a.ws_o + wrh * kD + x;
                pl = a.ws_lse + wrh;
            } else {
                po = a.o1 + rh * kD + x;
                pl = a.l1 + rh;
            }
        };
        for (int c0 = 0; c0 < n_parts; c0 += 6) {
            const float* po[6];
            float l[6];
            float4 xs[6];
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const float* pl;
                part(min(c0 + i, n_parts - 1), po[i], pl);
                l[i] = load_coherent1(pl);
            }
            load_coherent_six(po, xs);
#pragma unroll
            for (int i = 0; i < 6; ++i)
                if (c0 + i < n_parts) fold_add(f, l[i], xs[i]);
        }
        float4 r;
        const float lse = fold_result(f, r);
        store_out4<true>(a.o_out, rh * kD + x, r.x, r.y, r.z, r.w);
        if (x == 0 && a.lse_out != nullptr) a.lse_out[rh] = lse;
    }
}

template <int RHO>
hipError_t launch_for_rho(const HFusedArgs& a, int wpi, hipStream_t stream) {
    const int tiles = a.n_prefix_tiles + a.n_pairs + a.n_suffix_tiles;
#define BLLM_LAUNCH_HFUSED(W)                                                                                   \
    hipLaunchKernelGGL((hfused_attention_kernel<RHO, W>), dim3(tiles + (a.n_suffix_rows * W + 3) / 4), dim3(kThreads), \
                       0, stream, a)
    switch (wpi) {
        case 1: BLLM_LAUNCH_HFUSED(1); break;
        case 2: BLLM_LAUNCH_HFUSED(2); break;
        default: BLLM_LAUNCH_HFUSED(4); break;
    }
#undef BLLM_LAUNCH_HFUSED
    return hipGetLastError();
}

}  // namespace

hipError_t launch_hfused_attention(const LaunchCtx& c, const HFusedLists& lists, int suffix_wpi, const void* q,
                                   const void* k_prefix, const void* v_prefix, const void* k_suffix, const void* v_suffix,
                                   float* o1, float* l1, float* o2, float* l2, void* o_out, float* lse_out) {
    if (c.n_rows == 0) return hipSuccess;
    if (c.desc->dtype != BLLM_BF16 || c.desc->head_dim != 128) return hipErrorInvalidValue;
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    HFusedArgs a;
    a.prefix_tiles = lists.prefix_tiles;
    a.suffix_tiles = lists.suffix_tiles;
    a.suffix_rows = lists.suffix_rows;
    a.n_prefix_tiles = lists.n_prefix_tiles;
    a.n_suffix_tiles = lists.n_suffix_tiles;
    a.n_suffix_rows = lists.n_suffix_rows;
    a.pairs = lists.pairs;
    a.n_pairs = lists.n_pairs;
    a.q = static_cast<const uint16_t*>(q);
    a.k_prefix = static_cast<const uint16_t*>(k_prefix);
    a.v_prefix = static_cast<const uint16_t*>(v_prefix);
    a.k_suffix = static_cast<const uint16_t*>(k_suffix);
    a.v_suffix = static_cast<const uint16_t*>(v_suffix);
    a.o1 = o1;
    a.l1 = l1;
    a.o2 = o2;
    a.l2 = l2;
    a.ws_o = lists.ws_o;
    a.ws_lse = lists.ws_lse;
    a.prefix_row_split = lists.prefix_row_split;
    a.arrivals = lists.arrivals;
    a.o_out = o_out;
    a.lse_out = lse_out;
    a.n_q_heads = c.desc->n_q_heads;
    a.n_kv_heads = c.desc->n_kv_heads;
    a.log2_rho = rho == 1 ? 0 : rho == 2 ? 1 : rho == 4 ? 2 : 3;
    a.n_request_rows = lists.n_request_rows;
    a.scale = c.scale;
    switch (rho) {
        case 1: return launch_for_rho<1>(a, suffix_wpi, c.stream);
        case 2: return launch_for_rho<2>(a, suffix_wpi, c.stream);
        case 4: return launch_for_rho<4>(a, suffix_wpi, c.stream);
        case 8: return launch_for_rho<8>(a, suffix_wpi, c.stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace bllm

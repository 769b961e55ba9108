// Device code of the streaming partial attention (one workgroup = 4 / WPI work items), shared by the
// kernel of its own and by the horizontally fused kernel.
//
// Streaming (memory-bound) partial attention: one query token against a range of
// KV rows, for the heads that share one KV head.  This is the per-request
// "distinct part" of prefix-shared attention for decode rows (BatchLLM
// Sec. 4.3.3, Sec. 5: a matrix-vector product per request), and the fallback
// for every row when the dtype / head_dim has no matrix-core path.
//
// A KV row is read by 16 lanes, 16 or 32 bytes each, so one wavefront load
// instruction fetches four whole rows and a wavefront runs four independent
// online-softmax streams over interleaved rows.  WPI wavefronts (1, 2 or 4,
// chosen by the host from the typical range length) share one item; the
// streams of a wavefront are merged with lane exchanges, the wavefronts of an
// item through a few KB of LDS.  Dot products are finished with DPP adds inside
// each 16-lane row; no matrix cores are used.  In the bf16 instantiation K and
// V stay packed: q.k uses the 2-way bf16 dot instruction with fp32
// accumulation, and p.v uses it on row pairs with p rounded to bf16.
#pragma once

#include <type_traits>

#include "bllm_device.h"
#include "bllm_internal.h"

namespace bllm {
namespace stream_detail {

constexpr int kStreamThreads = 256;
constexpr int kWavesPerBlock = 4;
constexpr int kRowsPerStep = 4;    // KV rows each 16-lane stream handles per loop step

template <bool kBf16, int EPL>
struct Chunk;                      // EPL consecutive head-dim elements of one row, as loaded

template <>
struct Chunk<true, 8> { uint32_t w[4]; };
template <>
struct Chunk<true, 4> { uint32_t w[2]; };
template <>
struct Chunk<false, 8> { float f[8]; };
template <>
struct Chunk<false, 4> { float f[4]; };

template <bool kBf16, int EPL>
__device__ __forceinline__ Chunk<kBf16, EPL> load_chunk(const void* base, size_t elem_off, bool valid) {
    Chunk<kBf16, EPL> c;
    if constexpr (kBf16) {
        const uint16_t* p = static_cast<const uint16_t*>(base) + elem_off;
        if constexpr (EPL == 8) {
            // KV is streamed once: a non-temporal load keeps it from displacing reusable lines
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 zero4 = {0u, 0u, 0u, 0u};
            const u32x4 raw = valid ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)) : zero4;
            c.w[0] = raw[0]; c.w[1] = raw[1]; c.w[2] = raw[2]; c.w[3] = raw[3];
        } else {
            const uint2 raw = valid ? *reinterpret_cast<const uint2*>(p) : make_uint2(0, 0);
            c.w[0] = raw.x; c.w[1] = raw.y;
        }
    } else {
        const float* p = static_cast<const float*>(base) + elem_off;
#pragma unroll
        for (int x = 0; x < EPL; x += 4) {
            const float4 raw = valid ? *reinterpret_cast<const float4*>(p + x) : make_float4(0.f, 0.f, 0.f, 0.f);
            c.f[x] = raw.x; c.f[x + 1] = raw.y; c.f[x + 2] = raw.z; c.f[x + 3] = raw.w;
        }
    }
    return c;
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}

template <bool kPrecise>
__device__ __forceinline__ float exp2_of(float x) {
    if constexpr (kPrecise) return exp2f(x);
    else return __builtin_amdgcn_exp2f(x);
}

// exp2((a - b) * c) with the convention that an empty stream (a = -inf) weighs 0 even when b = -inf
template <bool kPrecise>
__device__ __forceinline__ float rel_weight(float a, float b, float c) {
    return a == -INFINITY ? 0.f : exp2_of<kPrecise>((a - b) * c);
}


// ---- transposing reduction over a row of 16 lanes -------------------------------------------
// Each lane brings 16 partial sums; afterwards lane i of the row holds the total of value i.
// Four pairing steps (mirror, half mirror, quad xor 2, quad xor 1); at each step a lane keeps
// the half of its values selected by one bit of its index and hands the other half over.
template <int kCtrl, int N>
__device__ __forceinline__ void halve(const float (&in)[2 * N], float (&out)[N], bool upper) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float keep = upper ? in[k + N] : in[k];
        const float send = upper ? in[k] : in[k + N];
        out[k] = keep + dpp_move<kCtrl>(send);
    }
}

__device__ __forceinline__ float row16_reduce_scatter(const float (&v)[16], int sub) {
    float w8[8], w4[4], w2[2], w1[1];
    halve<0x140, 8>(v, w8, (sub & 8) != 0);    // row_mirror
    halve<0x141, 4>(w8, w4, (sub & 4) != 0);   // row_half_mirror
    halve<0x4E, 2>(w4, w2, (sub & 2) != 0);    // quad_perm [2,3,0,1]
    halve<0xB1, 1>(w2, w1, (sub & 1) != 0);    // quad_perm [1,0,3,2]
    return w1[0];
}

// value of lane (4*quad + offset) of the caller's 16-lane row, for every lane of the row
template <int kSrcInRow>
__device__ __forceinline__ float row16_broadcast(float x) {
    // bit-mask swizzle inside each half wave: lane' = (lane & 0x10) | kSrcInRow
    constexpr int kPattern = (kSrcInRow << 5) | 0x10;
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), kPattern));
}
template <int kSrcInRow>
__device__ __forceinline__ uint32_t row16_broadcast_u32(uint32_t x) {
    constexpr int kPattern = (kSrcInRow << 5) | 0x10;
    return static_cast<uint32_t>(__builtin_amdgcn_ds_swizzle(static_cast<int>(x), kPattern));
}

// kPieces: the other part of a fused merge may be in several pieces (a split prefix); without it the
// kernel handles exactly one other partial and carries none of the bookkeeping.
// kCoherent: the partial result is written for another workgroup of the same launch (see store_partial4)
template <bool kBf16, int D, int RHO, int WPI, bool kPieces, bool kCoherent = false>
__device__ __forceinline__ void stream_attention_body(
    int block, const Item* __restrict__ items, int n_items, const void* __restrict__ q_, const void* __restrict__ k_,
    const void* __restrict__ v_, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, float scale, const MergeTarget& mt) {
    constexpr int EPL = D / 16;
    constexpr bool kPrecise = !kBf16;
    constexpr int kItemsPerBlock = kWavesPerBlock / WPI;
    constexpr int kStreams = 4 * WPI;                  // 16-lane streams per item
    constexpr int kRowsPerIter = kStreams * kRowsPerStep;
    __shared__ float sm_m[kItemsPerBlock][WPI][RHO];
    __shared__ float sm_l[kItemsPerBlock][WPI][RHO];
    __shared__ __attribute__((aligned(16))) float sm_acc[kItemsPerBlock][WPI][RHO][D];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: the item descriptor becomes a scalar load
    const int sub = lane & 15;
    const int item_in_block = wave / WPI;
    const int sw = wave % WPI;
    const int stream = sw * 4 + (lane >> 4);
    const int item_idx = block * kItemsPerBlock + item_in_block;
    const bool item_ok = item_idx < n_items;
    Item it = items[item_ok ? item_idx : 0];
    const int head0 = it.kv_head * RHO;
    const float c2 = scale * kLog2e;
    // a streaming item is one query row: it sees min(KV_LEN, VIS0) rows of its range
    const int kv_len = item_ok ? (it.kv_len < it.vis0 ? it.kv_len : it.vis0) : 0;

    float* dst_o;
    float* dst_l;
    if (it.dst_row >= 0) {
        dst_o = ws_o + (static_cast<size_t>(it.dst_row) * n_q_heads + head0) * D;
        dst_l = ws_lse + static_cast<size_t>(it.dst_row) * n_q_heads + head0;
    } else {
        dst_o = o_part + (static_cast<size_t>(it.q_row0) * n_q_heads + head0) * D;
        dst_l = lse_part + static_cast<size_t>(it.q_row0) * n_q_heads + head0;
    }

    Chunk<kBf16, EPL> qc[RHO];
#pragma unroll
    for (int e = 0; e < RHO; ++e)
        qc[e] = load_chunk<kBf16, EPL>(q_, (static_cast<size_t>(it.q_row0) * n_q_heads + head0 + e) * D + sub * EPL, true);

    // Fused merge: the other part of this item's row may be one partial result (row q_row0 of
    // mt.o_a / mt.lse_a) or n_other partial results in the split workspace.  What this thread will
    // need of them in the epilogue is requested right after the first K/V loads (up to kPre partials
    // per owned quad), so the latency is hidden behind the whole KV stream.
    //   WPI > 1: thread t of the item owns quads t, t + 64 WPI, ... of the item's RHO * D outputs;
    //   WPI = 1: the 16-lane row g of the wavefront owns heads g, g + 4, ...; lane `sub` its EPL elements.
    const size_t rh0 = static_cast<size_t>(it.q_row0) * n_q_heads + head0;   // (row, head) index of head 0
    constexpr int kQuads = RHO * D / 4;
    constexpr int kQuadsPerThread = WPI == 1 ? ((RHO + 3) / 4) * (EPL / 4) : (kQuads + 64 * WPI - 1) / (64 * WPI);
    constexpr int kPre = !kPieces ? 1 : WPI == 1 ? 2 : 4;
    const bool fused = mt.o_a != nullptr;
    RowSplit sp{0, 0, 0};
    if constexpr (kPieces) {
        if (fused && mt.row_split != nullptr) sp = mt.row_split[it.q_row0];
    }
    const int n_other = (kPieces && sp.n_splits > 0) ? sp.n_splits : 1;
    // head e's partial c: D values at other_o(e, c), log-sum-exp other_l(e, c)
    auto other_o = [&](int e, int c) -> const float* {
        return (kPieces && sp.n_splits > 0)
                   ? mt.ws_o + (static_cast<size_t>(sp.ws_row0 + c * sp.stride) * n_q_heads + head0 + e) * D
                   : mt.o_a + (rh0 + e) * D;
    };
    // (kCoherent: the other part was written by workgroups of this same launch)
    auto other_l = [&](int e, int c) -> float {
        const float* p = (kPieces && sp.n_splits > 0)
                             ? mt.ws_lse + static_cast<size_t>(sp.ws_row0 + c * sp.stride) * n_q_heads + head0 + e
                             : mt.lse_a + rh0 + e;
        if constexpr (kCoherent) return load_coherent1(p);
        else return *p;
    };
    auto other_x = [&](int e, int c, int d) -> float4 {
        if constexpr (kCoherent) return load_coherent4_tracked(other_o(e, c) + d);
        else return *reinterpret_cast<const float4*>(other_o(e, c) + d);
    };
    // the quad with index i of this thread: head e, first element d (false: no such quad)
    auto quad_of = [&](int i, int& e, int& d) -> bool {
        if constexpr (WPI == 1) {
            e = 4 * (i / (EPL / 4)) + (lane >> 4);
            d = sub * EPL + 4 * (i % (EPL / 4));
            return e < RHO;
        } else {
            const int q4 = sw * 64 + lane + i * 64 * WPI;
            e = (4 * q4) / D;
            d = 4 * q4 - e * D;
            return q4 < kQuads;
        }
    };
    float4 pre_o[kQuadsPerThread][kPre];
    float pre_l[kQuadsPerThread][kPre];
    // folds the other part's partials of quad i (head e, element d), then this part's (lb, o2); stores
    auto fold_and_store = [&](int i, int e, int d, float lb, const float4& o2) {
        PartialFold f;
#pragma unroll
        for (int c = 0; c < kPre; ++c)
            if (c < n_other) fold_add(f, pre_l[i][c], pre_o[i][c]);
        for (int c = kPre; c < n_other; ++c) fold_add(f, other_l(e, c), other_x(e, c, d));
        fold_add(f, lb, o2);
        float4 r;
        const float lse = fold_result(f, r);
        store_out4<kBf16>(mt.o_out, (rh0 + e) * D + d, r.x, r.y, r.z, r.w);
        if (d == 0 && mt.lse_out != nullptr) mt.lse_out[rh0 + e] = lse;
    };

    float m[RHO], l[RHO], acc[RHO][EPL];
#pragma unroll
    for (int e = 0; e < RHO; ++e) {
        m[e] = -INFINITY;
        l[e] = 0.f;
#pragma unroll
        for (int x = 0; x < EPL; ++x) acc[e][x] = 0.f;
    }

    // Fast path (bf16, heads in groups of 4): after a transposing reduction lane i of a 16-lane
    // row owns the score of (head i / 4, row i % 4) of the step, so the softmax is evaluated once
    // per score instead of once per lane; mq / lq are the running max / sum of head
    // 4 * hg + sub / 4, replicated over the quad.
    constexpr bool kFast = kBf16 && (RHO % 4 == 0) && kRowsPerStep == 4;
    constexpr int kHG = kFast ? RHO / 4 : 1;
    float mq[kHG], lq[kHG];
#pragma unroll
    for (int hg = 0; hg < kHG; ++hg) {
        mq[hg] = -INFINITY;
        lq[hg] = 0.f;
    }

    const size_t row_stride = static_cast<size_t>(n_kv_heads) * D;
    const size_t kv_base = (static_cast<size_t>(it.kv_row0) * n_kv_heads + it.kv_head) * D + sub * EPL;

    Chunk<kBf16, EPL> ka[kRowsPerStep], va[kRowsPerStep], kb[kRowsPerStep], vb[kRowsPerStep];
    // Rows past the end are clamped to the last row (their scores are masked), so every
    // load is unconditional and the eight loads of a step issue back to back.
    auto fetch = [&](int base, Chunk<kBf16, EPL>(&kk)[kRowsPerStep], Chunk<kBf16, EPL>(&vv)[kRowsPerStep]) {
#pragma unroll
        for (int u = 0; u < kRowsPerStep; ++u) {
            const int row = min(base + u * kStreams, kv_len - 1);
            const size_t off = kv_base + static_cast<size_t>(row) * row_stride;
            kk[u] = load_chunk<kBf16, EPL>(k_, off, true);
            vv[u] = load_chunk<kBf16, EPL>(v_, off, true);
        }
    };
    // One step of the online softmax on the rows held in kc / vc (rows base + u * kStreams).
    auto step = [&](int base, const Chunk<kBf16, EPL>(&kc)[kRowsPerStep], const Chunk<kBf16, EPL>(&vc)[kRowsPerStep]) {

        if constexpr (kFast) {
#pragma unroll
            for (int hg = 0; hg < kHG; ++hg) {
                float part[16];
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float a = 0.f;
#pragma unroll
                        for (int x = 0; x < EPL / 2; ++x) a = dot2_bf16(kc[u].w[x], qc[hg * 4 + e].w[x], a);
                        part[e * 4 + u] = a;
                    }
                float sc = row16_reduce_scatter(part, sub);          // score of (head sub / 4, row sub % 4)
                if (base + (sub & 3) * kStreams >= kv_len) sc = -INFINITY;
                float mxq = fmaxf(sc, dpp_move<0xB1>(sc));
                mxq = fmaxf(mxq, dpp_move<0x4E>(mxq));
                const float m_new = fmaxf(mq[hg], mxq);               // finite: row `base` is valid
                const float alpha_q = __builtin_amdgcn_exp2f((mq[hg] - m_new) * c2);
                const float p = __builtin_amdgcn_exp2f(fmaf(sc, c2, -m_new * c2));
                float ps = p + dpp_move<0xB1>(p);
                ps += dpp_move<0x4E>(ps);
                lq[hg] = lq[hg] * alpha_q + ps;
                mq[hg] = m_new;
                // rows (0,1) packed in the quad's lane 0, rows (2,3) in its lane 2
                const bf16x2 pkv = {static_cast<__bf16>(p), static_cast<__bf16>(dpp_move<0xB1>(p))};
                const uint32_t pk = __builtin_bit_cast(uint32_t, pkv);
                auto head = [&](auto ec) {
                    constexpr int e = decltype(ec)::value;
                    const uint32_t p01 = row16_broadcast_u32<4 * e>(pk);
                    const uint32_t p23 = row16_broadcast_u32<4 * e + 2>(pk);
                    const float alpha = row16_broadcast<4 * e>(alpha_q);
                    float(&a)[EPL] = acc[hg * 4 + e];
#pragma unroll
                    for (int x = 0; x < EPL / 2; ++x) {
                        const uint32_t lo01 = __builtin_amdgcn_perm(vc[1].w[x], vc[0].w[x], 0x05040100u);
                        const uint32_t hi01 = __builtin_amdgcn_perm(vc[1].w[x], vc[0].w[x], 0x07060302u);
                        const uint32_t lo23 = __builtin_amdgcn_perm(vc[3].w[x], vc[2].w[x], 0x05040100u);
                        const uint32_t hi23 = __builtin_amdgcn_perm(vc[3].w[x], vc[2].w[x], 0x07060302u);
                        a[2 * x] = dot2_bf16(lo23, p23, dot2_bf16(lo01, p01, a[2 * x] * alpha));
                        a[2 * x + 1] = dot2_bf16(hi23, p23, dot2_bf16(hi01, p01, a[2 * x + 1] * alpha));
                    }
                };
                head(std::integral_constant<int, 0>{});
                head(std::integral_constant<int, 1>{});
                head(std::integral_constant<int, 2>{});
                head(std::integral_constant<int, 3>{});
            }
        } else {
            float s[kRowsPerStep][RHO];
#pragma unroll
            for (int u = 0; u < kRowsPerStep; ++u) {
#pragma unroll
                for (int e = 0; e < RHO; ++e) {
                    float part = 0.f;
                    if constexpr (kBf16) {
#pragma unroll
                        for (int x = 0; x < EPL / 2; ++x) part = dot2_bf16(kc[u].w[x], qc[e].w[x], part);
                    } else {
#pragma unroll
                        for (int x = 0; x < EPL; ++x) part = fmaf(qc[e].f[x], kc[u].f[x], part);
                    }
                    s[u][e] = row16_sum(part);
                }
            }
            // rows past the end exist only in the last iteration of a stream
            if (base + (kRowsPerStep - 1) * kStreams >= kv_len) {
#pragma unroll
                for (int u = 1; u < kRowsPerStep; ++u)
                    if (base + u * kStreams >= kv_len) {
#pragma unroll
                        for (int e = 0; e < RHO; ++e) s[u][e] = -INFINITY;
                    }
            }
#pragma unroll
            for (int e = 0; e < RHO; ++e) {
                float mx = m[e];
#pragma unroll
                for (int u = 0; u < kRowsPerStep; ++u) mx = fmaxf(mx, s[u][e]);
                // row `base` is valid, so mx is finite; m = -inf gives alpha = 0
                const float alpha = exp2_of<kPrecise>((m[e] - mx) * c2);
                const float mc = mx * c2;
                float p[kRowsPerStep];
                float psum = 0.f;
#pragma unroll
                for (int u = 0; u < kRowsPerStep; ++u) {
                    p[u] = exp2_of<kPrecise>(fmaf(s[u][e], c2, -mc));
                    psum += p[u];
                }
                l[e] = l[e] * alpha + psum;
                m[e] = mx;
                if constexpr (kBf16) {
                    static_assert(kRowsPerStep == 4, "row pairing below assumes 4 rows");
                    const bf16x2 p01v = {static_cast<__bf16>(p[0]), static_cast<__bf16>(p[1])};
                    const bf16x2 p23v = {static_cast<__bf16>(p[2]), static_cast<__bf16>(p[3])};
                    const uint32_t p01 = __builtin_bit_cast(uint32_t, p01v);
                    const uint32_t p23 = __builtin_bit_cast(uint32_t, p23v);
#pragma unroll
                    for (int x = 0; x < EPL / 2; ++x) {
                        // the same head-dim element of two rows, side by side
                        const uint32_t lo01 = __builtin_amdgcn_perm(vc[1].w[x], vc[0].w[x], 0x05040100u);
                        const uint32_t hi01 = __builtin_amdgcn_perm(vc[1].w[x], vc[0].w[x], 0x07060302u);
                        const uint32_t lo23 = __builtin_amdgcn_perm(vc[3].w[x], vc[2].w[x], 0x05040100u);
                        const uint32_t hi23 = __builtin_amdgcn_perm(vc[3].w[x], vc[2].w[x], 0x07060302u);
                        acc[e][2 * x] = dot2_bf16(lo23, p23, dot2_bf16(lo01, p01, acc[e][2 * x] * alpha));
                        acc[e][2 * x + 1] = dot2_bf16(hi23, p23, dot2_bf16(hi01, p01, acc[e][2 * x + 1] * alpha));
                    }
                } else {
#pragma unroll
                    for (int x = 0; x < EPL; ++x) {
                        float a = acc[e][x] * alpha;
#pragma unroll
                        for (int u = 0; u < kRowsPerStep; ++u) a = fmaf(p[u], vc[u].f[x], a);
                        acc[e][x] = a;
                    }
                }
            }
        }
    };
    // Software pipeline: the loads of step n+1 are in flight while step n computes.  The two
    // register buffers swap roles every step (no copies), and the last step is peeled so that
    // every prefetch inside the loop is unconditional.
    const bool has_rows = stream < kv_len;
    if (has_rows) fetch(stream, ka, va);
    // The requests for the other part's partials go out behind the first K/V loads, so the K/V
    // stream does not start later because of them (loads return in order).
    if (fused && item_ok) {
#pragma unroll
        for (int i = 0; i < kQuadsPerThread; ++i) {
            int e, d;
            if (quad_of(i, e, d)) {
#pragma unroll
                for (int c = 0; c < kPre; ++c)
                    if (c < n_other) {
                        pre_o[i][c] = other_x(e, c, d);
                        pre_l[i][c] = other_l(e, c);
                    }
            }
        }
    }
    if (has_rows) {
        int base = stream;
        for (;;) {
            if (base + kRowsPerIter >= kv_len) {
                step(base, ka, va);
                break;
            }
            fetch(base + kRowsPerIter, kb, vb);
            __builtin_amdgcn_sched_barrier(0);
            step(base, ka, va);
            base += kRowsPerIter;
            if (base + kRowsPerIter >= kv_len) {
                step(base, kb, vb);
                break;
            }
            fetch(base + kRowsPerIter, ka, va);
            __builtin_amdgcn_sched_barrier(0);
            step(base, kb, vb);
            base += kRowsPerIter;
        }
    }

    if constexpr (kFast) {
        // hand every lane of a row the running max / sum of each head
#pragma unroll
        for (int hg = 0; hg < kHG; ++hg) {
            m[hg * 4 + 0] = row16_broadcast<0>(mq[hg]);  l[hg * 4 + 0] = row16_broadcast<0>(lq[hg]);
            m[hg * 4 + 1] = row16_broadcast<4>(mq[hg]);  l[hg * 4 + 1] = row16_broadcast<4>(lq[hg]);
            m[hg * 4 + 2] = row16_broadcast<8>(mq[hg]);  l[hg * 4 + 2] = row16_broadcast<8>(lq[hg]);
            m[hg * 4 + 3] = row16_broadcast<12>(mq[hg]); l[hg * 4 + 3] = row16_broadcast<12>(lq[hg]);
        }
    }
    // ---- merge the four streams of this wavefront (lanes ^16, ^32): scale to the common
    // maximum, then plain sums ------------------------------------------------------------------
#pragma unroll
    for (int e = 0; e < RHO; ++e) {
        float mw = fmaxf(m[e], __shfl_xor(m[e], 16));
        mw = fmaxf(mw, __shfl_xor(mw, 32));
        const float f = rel_weight<kPrecise>(m[e], mw, c2);
        float lw = l[e] * f;
        lw += __shfl_xor(lw, 16);
        lw += __shfl_xor(lw, 32);
        l[e] = lw;
        m[e] = mw;
#pragma unroll
        for (int x = 0; x < EPL; ++x) {
            float a = acc[e][x] * f;
            a += __shfl_xor(a, 16);
            a += __shfl_xor(a, 32);
            acc[e][x] = a;
        }
    }

    if constexpr (WPI == 1) {
        if (item_ok && fused) {
            // fused merge: this part is (acc / l, log-sum-exp); every lane holds all of it after the
            // exchange above
#pragma unroll
            for (int i = 0; i < kQuadsPerThread; ++i) {
#pragma unroll
                for (int ee = 0; ee < 4; ++ee) {
                    constexpr int kPerHead = EPL / 4;
                    const int e = 4 * (i / kPerHead) + ee;          // static: indexes the register arrays
                    const int x = 4 * (i % kPerHead);
                    if (e < RHO && ee == (lane >> 4)) {
                        const float inv = l[e] > 0.f ? 1.f / l[e] : 0.f;
                        const float lb = l[e] > 0.f ? (m[e] * c2 + log2f(l[e])) * kLn2 : -INFINITY;
                        fold_and_store(i, e, sub * EPL + x, lb,
                                       make_float4(acc[e][x] * inv, acc[e][x + 1] * inv, acc[e][x + 2] * inv, acc[e][x + 3] * inv));
                    }
                }
            }
        } else if (item_ok && lane < 16) {
#pragma unroll
            for (int e = 0; e < RHO; ++e) {
                const float inv = l[e] > 0.f ? 1.f / l[e] : 0.f;     // empty range: output 0
#pragma unroll
                for (int x = 0; x < EPL; x += 4)
                    store_partial4<kCoherent>(dst_o + e * D + sub * EPL + x, acc[e][x] * inv, acc[e][x + 1] * inv,
                                              acc[e][x + 2] * inv, acc[e][x + 3] * inv);
                if (sub == 0) store_partial1<kCoherent>(dst_l + e, l[e] > 0.f ? (m[e] * c2 + log2f(l[e])) * kLn2 : -INFINITY);
            }
        }
    } else {
        if (lane < 16) {
#pragma unroll
            for (int e = 0; e < RHO; ++e) {
                if (sub == 0) {
                    sm_m[item_in_block][sw][e] = m[e];
                    sm_l[item_in_block][sw][e] = l[e];
                }
#pragma unroll
                for (int x = 0; x < EPL; ++x) sm_acc[item_in_block][sw][e][sub * EPL + x] = acc[e][x];
            }
        }
        __syncthreads();
        if (item_ok && fused) {
            // fused merge, four consecutive head-dim elements per thread
#pragma unroll
            for (int i = 0; i < kQuadsPerThread; ++i) {
                int e, d;
                if (quad_of(i, e, d)) {
                    float top = -INFINITY;
#pragma unroll
                    for (int w = 0; w < WPI; ++w) top = fmaxf(top, sm_m[item_in_block][w][e]);
                    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
                    float den = 0.f;
#pragma unroll
                    for (int w = 0; w < WPI; ++w) {
                        const float wgt = rel_weight<kPrecise>(sm_m[item_in_block][w][e], top, c2);
                        const float4 x = *reinterpret_cast<const float4*>(&sm_acc[item_in_block][w][e][d]);
                        num.x = fmaf(wgt, x.x, num.x);
                        num.y = fmaf(wgt, x.y, num.y);
                        num.z = fmaf(wgt, x.z, num.z);
                        num.w = fmaf(wgt, x.w, num.w);
                        den = fmaf(wgt, sm_l[item_in_block][w][e], den);
                    }
                    const float inv = den > 0.f ? 1.f / den : 0.f;
                    const float lb = den > 0.f ? (top * c2 + log2f(den)) * kLn2 : -INFINITY;
                    fold_and_store(i, e, d, lb, make_float4(num.x * inv, num.y * inv, num.z * inv, num.w * inv));
                }
            }
        } else if (item_ok) {
            const int t_in_item = sw * 64 + lane;
            for (int idx = t_in_item; idx < RHO * D; idx += 64 * WPI) {
                const int e = idx / D;
                const int d = idx - e * D;
                float top = -INFINITY;
#pragma unroll
                for (int w = 0; w < WPI; ++w) top = fmaxf(top, sm_m[item_in_block][w][e]);
                float num = 0.f, den = 0.f;
#pragma unroll
                for (int w = 0; w < WPI; ++w) {
                    const float wgt = rel_weight<kPrecise>(sm_m[item_in_block][w][e], top, c2);
                    num = fmaf(wgt, sm_acc[item_in_block][w][e][d], num);
                    den = fmaf(wgt, sm_l[item_in_block][w][e], den);
                }
                store_partial1<kCoherent>(dst_o + idx, den > 0.f ? num / den : 0.f);
                if (d == 0) store_partial1<kCoherent>(dst_l + e, den > 0.f ? (top * c2 + log2f(den)) * kLn2 : -INFINITY);
            }
        }
    }
}

}  // namespace stream_detail
}  // namespace bllm

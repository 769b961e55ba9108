// Matrix-core partial attention for bf16, head_dim 128: a block of query rows
// (all rows of a prefix-sharing group x the query heads that share one KV head,
// or the rows of one prefill chunk) against a range of KV rows.
//
// This is the shared-prefix part of prefix-shared attention (BatchLLM
// Sec. 4.3.3, Sec. 5): because every query of the group sees the same keys, the
// per-request matrix-vector products become one matrix-matrix product and each
// KV tile is fetched once per workgroup for up to 256 stacked query rows.  The
// same kernel, with the causal bound of a prefill chunk, serves the chunk rows
// of the distinct part.
//
// Layout of the computation (per wavefront: 64 stacked query rows, 64 KV rows a step):
//   S^T = K Q^T      A operand = K tile from LDS, B operand = Q held in registers
//   O^T += V^T P^T   A operand = V^T tile from LDS, B operand = P straight from
//                    the S^T accumulators
// Working on the transposes puts one query per lane column, so the running
// maximum, the running sum and the rescale factor are per-lane scalars and the
// softmax needs a single cross-lane exchange (lane ^ 32) per step.
// The accumulator rows a lane holds (kv = 8i + 4h + j) are not contiguous in kv;
// the V^T tile is therefore stored in LDS with the kv positions of each group of
// 16 permuted so that the 8 values a lane needs are one 16-byte read.
#include "bllm_device.h"
#include "bllm_internal.h"

namespace bllm {
namespace {

constexpr int kTileThreads = 256;
constexpr int kBN = 64;              // KV rows per step
constexpr int kD = 128;
constexpr int kKPitch = 272;         // bytes per K row in LDS (256 + 16 pad: conflict-free 16-byte column reads)
constexpr int kVtPitch = 128;        // bytes per V^T row in LDS (64 kv slots), XOR-swizzled in 16-byte units
constexpr int kKBytes = kBN * kKPitch;
constexpr int kVtBytes = kD * kVtPitch;

__device__ __forceinline__ int vt_swizzle(int d) { return (d ^ (d >> 3)) & 7; }

struct Staging {
    uint4 k[4];
    uint4 v[4];
};

// Each thread stages a 4 (kv) x 8 (d) block of K and of V: rows 4*kvq..4*kvq+3,
// columns 8*dchunk..8*dchunk+7; 16 consecutive threads read one 256-byte row.
__device__ __forceinline__ void stage_global(Staging& st, const uint16_t* __restrict__ kg, const uint16_t* __restrict__ vg,
                                             size_t row_stride, int tile_base, int kv_len, int kvq, int dchunk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = tile_base + 4 * kvq + i;
        if (r < kv_len) {
            const size_t off = static_cast<size_t>(r) * row_stride + dchunk * 8;
            st.k[i] = *reinterpret_cast<const uint4*>(kg + off);
            st.v[i] = *reinterpret_cast<const uint4*>(vg + off);
        } else {
            st.k[i] = make_uint4(0, 0, 0, 0);
            st.v[i] = make_uint4(0, 0, 0, 0);
        }
    }
}

__device__ __forceinline__ uint32_t comp(const uint4& x, int c) {
    return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w;
}

__device__ __forceinline__ void stage_to_lds(const Staging& st, unsigned char* sk, unsigned char* svt, int kvq, int dchunk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(sk + (4 * kvq + i) * kKPitch + dchunk * 16) = st.k[i];
    // transpose the 4 x 8 block of V: for each column d, the 4 kv values become one 8-byte word
    const int unit = 2 * (kvq >> 2) + (kvq & 1);
    const int half8 = (kvq >> 1) & 1;
#pragma unroll
    for (int dd = 0; dd < 8; ++dd) {
        const int c = dd >> 1;
        uint32_t w0, w1;
        if ((dd & 1) == 0) {
            w0 = (comp(st.v[0], c) & 0xffffu) | (comp(st.v[1], c) << 16);
            w1 = (comp(st.v[2], c) & 0xffffu) | (comp(st.v[3], c) << 16);
        } else {
            w0 = (comp(st.v[0], c) >> 16) | (comp(st.v[1], c) & 0xffff0000u);
            w1 = (comp(st.v[2], c) >> 16) | (comp(st.v[3], c) & 0xffff0000u);
        }
        const int d = 8 * dchunk + dd;
        *reinterpret_cast<uint2*>(svt + d * kVtPitch + ((unit ^ vt_swizzle(d)) << 4) + half8 * 8) = make_uint2(w0, w1);
    }
}

__global__ __launch_bounds__(kTileThreads, 1) void tile_attention_kernel(
    const Item* __restrict__ items, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, int log2_rho, float scale) {
    __shared__ __attribute__((aligned(16))) unsigned char smem_k[2][kKBytes];
    __shared__ __attribute__((aligned(16))) unsigned char smem_vt[2][kVtBytes];

    const Item it = items[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;       // query column inside a 32-wide block; also the A-operand row
    const int h = lane >> 5;         // lane half
    const int rho = 1 << log2_rho;
    const int head0 = it.kv_head << log2_rho;
    const int kv_len = it.kv_len;
    const float c2 = scale * kLog2e;

    float* dst_o;
    float* dst_l;
    if (it.dst_row >= 0) {
        dst_o = ws_o + (static_cast<size_t>(it.dst_row) * n_q_heads + head0) * kD;
        dst_l = ws_lse + static_cast<size_t>(it.dst_row) * n_q_heads + head0;
    } else {
        dst_o = o_part + (static_cast<size_t>(it.q_row0) * n_q_heads + head0) * kD;
        dst_l = lse_part + static_cast<size_t>(it.q_row0) * n_q_heads + head0;
    }

    // stacked row m = 64*wave + 32*qb + col  ->  token row m >> log2_rho, head m & (rho-1)
    int tok[2], hd[2];
    bool row_ok[2];
    int vis[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int m = 64 * wave + 32 * qb + col;
        tok[qb] = m >> log2_rho;
        hd[qb] = m & (rho - 1);
        row_ok[qb] = tok[qb] < it.n_rows;
        const int vv = it.vis0 + tok[qb];
        vis[qb] = (row_ok[qb] && vv < kv_len) ? vv : kv_len;
    }

    if (kv_len <= 0) {               // empty part: output 0, log-sum-exp -inf
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (!row_ok[qb]) continue;
            float* orow = dst_o + (static_cast<size_t>(tok[qb]) * n_q_heads + hd[qb]) * kD;
            for (int x = h * 64; x < h * 64 + 64; x += 4) *reinterpret_cast<float4*>(orow + x) = make_float4(0.f, 0.f, 0.f, 0.f);
            if (h == 0) dst_l[static_cast<size_t>(tok[qb]) * n_q_heads + hd[qb]] = -INFINITY;
        }
        return;
    }

    // first / last token row of this wavefront -> smallest / largest visible count
    const int wave_tok_lo = (64 * wave) >> log2_rho;
    const int wave_tok_hi = min(it.n_rows - 1, (64 * wave + 63) >> log2_rho);
    const bool wave_has_rows = wave_tok_lo < it.n_rows;
    const int wave_min_vis = wave_has_rows ? min(kv_len, it.vis0 + wave_tok_lo) : kv_len;
    const int wave_max_vis = wave_has_rows ? min(kv_len, it.vis0 + wave_tok_hi) : 0;

    // ---- Q fragments (B operand of S^T = K Q^T): Q[query = col][d = 16 t + 8 h + 0..7] -------
    bf16x8 qreg[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const uint16_t* qrow = q + (static_cast<size_t>(it.q_row0 + tok[qb]) * n_q_heads + head0 + hd[qb]) * kD + 8 * h;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            uint4 raw = row_ok[qb] ? *reinterpret_cast<const uint4*>(qrow + 16 * t) : make_uint4(0, 0, 0, 0);
            qreg[qb][t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    floatx16 oacc[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int x = 0; x < 16; ++x) oacc[db][qb][x] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};

    const size_t row_stride = static_cast<size_t>(n_kv_heads) * kD;
    const uint16_t* kg = k + (static_cast<size_t>(it.kv_row0) * n_kv_heads + it.kv_head) * kD;
    const uint16_t* vg = v + (static_cast<size_t>(it.kv_row0) * n_kv_heads + it.kv_head) * kD;
    const int dchunk = tid & 15;
    const int kvq = tid >> 4;
    const int n_tiles = (kv_len + kBN - 1) / kBN;

    Staging st;
    stage_global(st, kg, vg, row_stride, 0, kv_len, kvq, dchunk);
    stage_to_lds(st, smem_k[0], smem_vt[0], kvq, dchunk);
    __syncthreads();

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const int tile_base = tile * kBN;
        const bool more = tile + 1 < n_tiles;
        if (more) stage_global(st, kg, vg, row_stride, tile_base + kBN, kv_len, kvq, dchunk);

        if (tile_base < wave_max_vis) {
            const unsigned char* sk = smem_k[buf];
            const unsigned char* svt = smem_vt[buf];
            // ---- S^T = K Q^T ---------------------------------------------------------------
            floatx16 sacc[2][2];
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) sacc[kvb][qb][x] = 0.f;
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const uint4 raw = *reinterpret_cast<const uint4*>(sk + (32 * kvb + col) * kKPitch + 32 * t + 16 * h);
                    const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        sacc[kvb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][t], sacc[kvb][qb], 0, 0, 0);
                }
            }
            // ---- online softmax, one query per lane column -----------------------------------
            const bool need_mask = tile_base + kBN > wave_min_vis;
            bf16x8 pb[2][2][2];      // [qb][kvb][u]
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (need_mask) {
#pragma unroll
                    for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                        for (int x = 0; x < 16; ++x) {
                            const int kvi = tile_base + 32 * kvb + 8 * (x >> 2) + 4 * h + (x & 3);
                            if (kvi >= vis[qb]) sacc[kvb][qb][x] = -INFINITY;
                        }
                }
                float mloc = -INFINITY;
#pragma unroll
                for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) mloc = fmaxf(mloc, sacc[kvb][qb][x]);
                mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
                const float m_new = fmaxf(m_run[qb], mloc);
                // m_new is finite from the first tile on: KV row 0 is visible to every row.
                const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c2);
                const float mc = m_new * c2;
                float lsum = 0.f;
#pragma unroll
                for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kvb][qb][x], c2, -mc));
                        sacc[kvb][qb][x] = p;
                        lsum += p;
                    }
                l_run[qb] = l_run[qb] * alpha + lsum;
                m_run[qb] = m_new;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int x = 0; x < 16; ++x) oacc[db][qb][x] *= alpha;
#pragma unroll
                for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int e = 0; e < 8; ++e) pb[qb][kvb][u][e] = static_cast<__bf16>(sacc[kvb][qb][8 * u + e]);
            }
            // ---- O^T += V^T P^T -----------------------------------------------------------------
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int d = 32 * db + col;
                const int sw = vt_swizzle(d);
#pragma unroll
                for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int unit = 4 * kvb + 2 * u + h;
                        const uint4 raw = *reinterpret_cast<const uint4*>(svt + d * kVtPitch + ((unit ^ sw) << 4));
                        const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                        for (int qb = 0; qb < 2; ++qb)
                            oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][kvb][u], oacc[db][qb], 0, 0, 0);
                    }
                }
            }
        }
        if (more) stage_to_lds(st, smem_k[buf ^ 1], smem_vt[buf ^ 1], kvq, dchunk);
        __syncthreads();
    }

    // ---- epilogue: normalise and store O (transposed back), log-sum-exp --------------------------
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float ltot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (!row_ok[qb]) continue;
        const float inv = 1.f / ltot;
        float* orow = dst_o + (static_cast<size_t>(tok[qb]) * n_q_heads + hd[qb]) * kD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float4 o4 = make_float4(oacc[db][qb][4 * i] * inv, oacc[db][qb][4 * i + 1] * inv,
                                        oacc[db][qb][4 * i + 2] * inv, oacc[db][qb][4 * i + 3] * inv);
                *reinterpret_cast<float4*>(orow + 32 * db + 8 * i + 4 * h) = o4;
            }
        if (h == 0) dst_l[static_cast<size_t>(tok[qb]) * n_q_heads + hd[qb]] = (m_run[qb] * c2 + log2f(ltot)) * kLn2;
    }
}

}  // namespace

hipError_t launch_tile_attention(const LaunchCtx& c, const Item* items, int32_t n_items, const void* q, const void* k,
                                 const void* v, float* o_part, float* lse_part, float* ws_o, float* ws_lse) {
    if (n_items <= 0) return hipSuccess;
    if (c.desc->dtype != BLLM_BF16 || c.desc->head_dim != kD) return hipErrorInvalidValue;
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    int log2_rho = 0;
    while ((1 << log2_rho) < rho) ++log2_rho;
    hipLaunchKernelGGL(tile_attention_kernel, dim3(n_items), dim3(kTileThreads), 0, c.stream, items,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                       o_part, lse_part, ws_o, ws_lse, c.desc->n_q_heads, c.desc->n_kv_heads, log2_rho, c.scale);
    return hipGetLastError();
}

}  // namespace bllm

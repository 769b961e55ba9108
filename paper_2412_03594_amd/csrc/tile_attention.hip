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
// Layout of the computation (per wavefront: 32 stacked query rows, 64 KV rows a step):
//   S^T = K Q^T      A operand = K tile from LDS, B operand = Q held in registers
//   O^T += V^T P^T   A operand = V^T tile from LDS, B operand = P straight from
//                    the S^T accumulators
// Working on the transposes puts one query per lane column, so the running
// maximum, the running sum and the rescale factor are per-lane scalars.  The
// reference maximum is raised lazily (only when a tile exceeds it by 2^8), so
// the common step needs no cross-lane exchange and no rescale of O.
// The accumulator rows a lane holds (kv = 8i + 4h + j) are not contiguous in kv;
// the V^T tile is therefore stored in LDS with the kv positions of each group of
// 16 permuted so that the 8 values a lane needs are one 16-byte read.
// K and V tiles are double-buffered in LDS; the next tile's global loads are in
// flight while the current one is multiplied; one barrier per step.
#include "bllm_device.h"
#include "bllm_internal.h"

namespace bllm {
namespace {

constexpr int kBN = 64;              // KV rows per step
constexpr int kD = 128;
constexpr int kKPitch = 272;         // bytes per K row in LDS (256 + 16 pad: conflict-free 16-byte column reads)
constexpr int kVtPitch = 128;        // bytes per V^T row in LDS (64 kv slots), XOR-swizzled in 16-byte units
constexpr int kKBytes = kBN * kKPitch;
constexpr int kVtBytes = kD * kVtPitch;

__device__ __forceinline__ int vt_swizzle(int d) { return (d ^ (d >> 3)) & 7; }

// Each thread stages a 4 (kv) x 8 (d) block of K and of V: rows 4*kvq..4*kvq+3,
// columns 8*dchunk..8*dchunk+7; 16 consecutive threads read one 256-byte row.
// Rows past the end of the range are staged as zeros.
__device__ __forceinline__ void stage_global(uint4 (&dst)[4], const uint16_t* __restrict__ src, size_t row_stride,
                                             int tile_base, int kv_len, int kvq, int dchunk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = tile_base + 4 * kvq + i;
        dst[i] = (r >= 0 && r < kv_len) ? *reinterpret_cast<const uint4*>(src + static_cast<size_t>(r) * row_stride + dchunk * 8)
                            : make_uint4(0, 0, 0, 0);
    }
}

__device__ __forceinline__ uint32_t comp(const uint4& x, int c) {
    return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w;
}

__device__ __forceinline__ void stage_k_to_lds(const uint4 (&st)[4], unsigned char* sk, int kvq, int dchunk) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(sk + (4 * kvq + i) * kKPitch + dchunk * 16) = st[i];
}

// transpose the 4 x 8 block of V: for each column d, the 4 kv values become one 8-byte word
__device__ __forceinline__ void stage_v_to_lds(const uint4 (&st)[4], unsigned char* svt, int kvq, int dchunk) {
    const int unit = 2 * (kvq >> 2) + (kvq & 1);
    const int half8 = (kvq >> 1) & 1;
#pragma unroll
    for (int dd = 0; dd < 8; ++dd) {
        const int c = dd >> 1;
        uint32_t w0, w1;
        if ((dd & 1) == 0) {
            w0 = __builtin_amdgcn_perm(comp(st[1], c), comp(st[0], c), 0x05040100u);
            w1 = __builtin_amdgcn_perm(comp(st[3], c), comp(st[2], c), 0x05040100u);
        } else {
            w0 = __builtin_amdgcn_perm(comp(st[1], c), comp(st[0], c), 0x07060302u);
            w1 = __builtin_amdgcn_perm(comp(st[3], c), comp(st[2], c), 0x07060302u);
        }
        const int d = 8 * dchunk + dd;
        *reinterpret_cast<uint2*>(svt + d * kVtPitch + ((unit ^ vt_swizzle(d)) << 4) + half8 * 8) = make_uint2(w0, w1);
    }
}

// The running maximum is only raised when a tile exceeds it by more than this many powers of
// two; below that the stale maximum is exact arithmetic anyway (weights up to 2^8, fp32 sums).
constexpr float kMaxSlack = 8.f;

// NW wavefronts per workgroup, 32 stacked query rows each.  With about 200 registers a
// wavefront, two wavefronts share a SIMD, so one runs its exp / convert work on the vector
// ALUs while the other keeps the matrix cores busy.
template <int NW>
__global__ __launch_bounds__(64 * NW, 2) void tile_attention_kernel(
    const Item* __restrict__ items, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, float* __restrict__ o_part, float* __restrict__ lse_part, float* __restrict__ ws_o,
    float* __restrict__ ws_lse, int n_q_heads, int n_kv_heads, int log2_rho, float scale) {
    __shared__ __attribute__((aligned(16))) unsigned char smem_k[2][kKBytes];
    __shared__ __attribute__((aligned(16))) unsigned char smem_vt[2][kVtBytes];

    const Item it = items[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31;       // query column of this lane; also the A-operand row
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

    // stacked row m = 32*wave + col  ->  token row m >> log2_rho, head m & (rho-1)
    const int m_row = 32 * wave + col;
    const int tok = m_row >> log2_rho;
    const int hd = m_row & (rho - 1);
    const bool row_ok = tok < it.n_rows;
    const int vis = (row_ok && it.vis0 + tok < kv_len) ? it.vis0 + tok : kv_len;   // padding rows see everything

    if (kv_len <= 0) {               // empty part: output 0, log-sum-exp -inf
        if (row_ok) {
            float* orow = dst_o + (static_cast<size_t>(tok) * n_q_heads + hd) * kD;
            for (int x = h * 64; x < h * 64 + 64; x += 4) *reinterpret_cast<float4*>(orow + x) = make_float4(0.f, 0.f, 0.f, 0.f);
            if (h == 0) dst_l[static_cast<size_t>(tok) * n_q_heads + hd] = -INFINITY;
        }
        return;
    }

    // smallest visible count among this wavefront's rows: tiles that end below it need no mask
    const int wave_tok_lo = (32 * wave) >> log2_rho;
    const int wave_min_vis = wave_tok_lo < it.n_rows ? min(kv_len, it.vis0 + wave_tok_lo) : kv_len;

    // ---- Q fragments (B operand of S^T = K Q^T): Q[query = col][d = 16 t + 8 h + 0..7] -------
    bf16x8 qreg[8];
    {
        const uint16_t* qrow = q + (static_cast<size_t>(it.q_row0 + tok) * n_q_heads + head0 + hd) * kD + 8 * h;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint4 raw = row_ok ? *reinterpret_cast<const uint4*>(qrow + 16 * t) : make_uint4(0, 0, 0, 0);
            qreg[t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    floatx16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[db][x] = 0.f;
    float m_run = -INFINITY;         // reference maximum, in log2 units (score * c2)
    float l_run = 0.f;               // this lane's share of the running sum

    const size_t row_stride = static_cast<size_t>(n_kv_heads) * kD;
    const uint16_t* kg = k + (static_cast<size_t>(it.kv_row0) * n_kv_heads + it.kv_head) * kD;
    const uint16_t* vg = v + (static_cast<size_t>(it.kv_row0) * n_kv_heads + it.kv_head) * kD;
    const int n_tiles = (kv_len + kBN - 1) / kBN;

    // Staging: 256 threads cover a 64 x 128 tile in 4 (kv) x 8 (d) blocks.  With 8 wavefronts the
    // lower four stage K and the upper four stage V; with 4 wavefronts every thread stages both.
    const int st_tid = tid & 255;
    const int dchunk = st_tid & 15;
    const int kvq = st_tid >> 4;
    const bool do_k = NW == 4 || tid < 256;
    const bool do_v = NW == 4 || tid >= 256;
    uint4 st_k[4], st_v[4];
    auto load_tile = [&](int tile_base) {
        if (do_k) stage_global(st_k, kg, row_stride, tile_base, kv_len, kvq, dchunk);
        if (do_v) stage_global(st_v, vg, row_stride, tile_base, kv_len, kvq, dchunk);
    };
    auto store_tile = [&](int buf) {
        if (do_k) stage_k_to_lds(st_k, smem_k[buf], kvq, dchunk);
        if (do_v) stage_v_to_lds(st_v, smem_vt[buf], kvq, dchunk);
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const int tile_base = tile * kBN;
        const bool more = tile + 1 < n_tiles;
        if (more) load_tile(tile_base + kBN);

        // ---- S^T = K Q^T (64 kv x 32 queries) ---------------------------------------------------
        const unsigned char* sk = smem_k[buf];
        floatx16 sacc[2];
        {
            const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 8; ++t) {
#pragma unroll
                for (int kvb = 0; kvb < 2; ++kvb) {
                    const uint4 raw = *reinterpret_cast<const uint4*>(sk + (32 * kvb + col) * kKPitch + 32 * t + 16 * h);
                    sacc[kvb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), qreg[t],
                                                                         t == 0 ? zero : sacc[kvb], 0, 0, 0);
                }
            }
        }
        if (tile_base + kBN > wave_min_vis) {       // last tile(s) of an item: mask what a row cannot see
#pragma unroll
            for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int kvi = tile_base + 32 * kvb + 8 * (x >> 2) + 4 * h + (x & 3);
                    sacc[kvb][x] = kvi >= vis ? -INFINITY : sacc[kvb][x];
                }
            asm volatile("" ::: "memory");           // keep it a branch
        }
        // ---- reference maximum: raised (and O, l rescaled) only when exceeded by kMaxSlack ------
        float mx = -INFINITY;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int x = 0; x < 16; ++x) mx = fmaxf(mx, sacc[kvb][x]);
        const float zloc = mx * c2;
        if (__any(zloc > m_run + kMaxSlack)) {
            const float z = fmaxf(zloc, __shfl_xor(zloc, 32));
            const float m_new = fmaxf(m_run, z);
            // first tile: m_run = -inf and m_new is finite (KV row 0 is visible to every row)
            float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            asm volatile("" : "+v"(alpha));          // rare path: must stay behind its branch
            l_run *= alpha;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha;
        }
        // ---- P = exp2(S c2 - m) in bf16, running sum -------------------------------------------
        bf16x8 pb[2][2];             // [kvb][u]
        float lsum = 0.f;
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kvb][8 * u + e], c2, -m_run));
                    lsum += p;
                    pb[kvb][u][e] = static_cast<__bf16>(p);
                }
        l_run += lsum;
        // ---- O^T += V^T P^T ---------------------------------------------------------------------
        const unsigned char* svt = smem_vt[buf];
#pragma unroll
        for (int kvb = 0; kvb < 2; ++kvb) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const int d = 32 * db + col;
                    const int unit = 4 * kvb + 2 * u + h;
                    const uint4 raw = *reinterpret_cast<const uint4*>(svt + d * kVtPitch + ((unit ^ vt_swizzle(d)) << 4));
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), pb[kvb][u], oacc[db], 0, 0, 0);
                }
            }
        }
        // the other buffers were last read in the previous step, before its barrier
        if (more) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise and store O (transposed back), log-sum-exp --------------------------
    const float ltot = l_run + __shfl_xor(l_run, 32);
    if (row_ok) {
        const float inv = 1.f / ltot;
        float* orow = dst_o + (static_cast<size_t>(tok) * n_q_heads + hd) * kD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 o4 = make_float4(oacc[db][4 * i] * inv, oacc[db][4 * i + 1] * inv, oacc[db][4 * i + 2] * inv,
                                              oacc[db][4 * i + 3] * inv);
                *reinterpret_cast<float4*>(orow + 32 * db + 8 * i + 4 * h) = o4;
            }
        if (h == 0) dst_l[static_cast<size_t>(tok) * n_q_heads + hd] = (m_run + log2f(ltot)) * kLn2;
    }
}

}  // namespace

hipError_t launch_tile_attention(const LaunchCtx& c, const Item* items, int32_t n_items, int waves, const void* q,
                                 const void* k, const void* v, float* o_part, float* lse_part, float* ws_o,
                                 float* ws_lse) {
    if (n_items <= 0) return hipSuccess;
    if (c.desc->dtype != BLLM_BF16 || c.desc->head_dim != kD || (waves != 4 && waves != 8)) return hipErrorInvalidValue;
    const int rho = c.desc->n_q_heads / c.desc->n_kv_heads;
    int log2_rho = 0;
    while ((1 << log2_rho) < rho) ++log2_rho;
    const uint16_t* qq = static_cast<const uint16_t*>(q);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
    if (waves == 8)
        hipLaunchKernelGGL(tile_attention_kernel<8>, dim3(n_items), dim3(512), 0, c.stream, items, qq, kk, vv, o_part,
                           lse_part, ws_o, ws_lse, c.desc->n_q_heads, c.desc->n_kv_heads, log2_rho, c.scale);
    else
        hipLaunchKernelGGL(tile_attention_kernel<4>, dim3(n_items), dim3(256), 0, c.stream, items, qq, kk, vv, o_part,
                           lse_part, ws_o, ws_lse, c.desc->n_q_heads, c.desc->n_kv_heads, log2_rho, c.scale);
    return hipGetLastError();
}

}  // namespace bllm

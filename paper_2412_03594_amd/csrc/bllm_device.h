// Small device-side helpers shared by the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bllm {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// float -> bfloat16 bits, round to nearest even (inputs here are finite).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// Online-softmax merge of two normalised partial results (BatchLLM Sec. 5) with natural-log
// log-sum-exps la, lb: out = (wa * a + wb * b) * inv, lse as returned.  An empty part (-inf) gets
// weight exactly 0; two empty parts give weights 0, inv 0 and lse -inf.
struct MergeWeights {
    float wa, wb, inv, lse;
};
__device__ __forceinline__ MergeWeights merge_weights(float la, float lb) {
    MergeWeights w;
    const float top = fmaxf(la, lb);
    if (top == -INFINITY) {
        w.wa = w.wb = 0.f;
        w.inv = 0.f;
        w.lse = -INFINITY;
    } else {
        w.wa = expf(la - top);         // exp(-inf) = 0 for an empty part
        w.wb = expf(lb - top);
        const float tot = w.wa + w.wb;
        w.inv = 1.f / tot;
        w.lse = top + logf(tot);
    }
    return w;
}
// one merged element; a value of a part with weight 0 is dropped, never multiplied
__device__ __forceinline__ float merge_value(const MergeWeights& w, float a, float b) {
    return (w.wa * (w.wa > 0.f ? a : 0.f) + w.wb * (w.wb > 0.f ? b : 0.f)) * w.inv;
}
// Running online-softmax fold of any number of normalised partial results, four consecutive
// elements at a time: (top, den, num) with result num / den and log-sum-exp top + log(den).
// A partial with log-sum-exp -inf is skipped (its values are never touched).
struct PartialFold {
    float top = -INFINITY;
    float den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
};
__device__ __forceinline__ void fold_add(PartialFold& f, float lse, const float4& x) {
    if (lse == -INFINITY) return;
    const float m = fmaxf(f.top, lse);
    const float r = f.top == -INFINITY ? 0.f : expf(f.top - m);
    const float w = expf(lse - m);
    f.num.x = fmaf(w, x.x, f.num.x * r);
    f.num.y = fmaf(w, x.y, f.num.y * r);
    f.num.z = fmaf(w, x.z, f.num.z * r);
    f.num.w = fmaf(w, x.w, f.num.w * r);
    f.den = fmaf(f.den, r, w);
    f.top = m;
}
// result of the fold: values in `o`, log-sum-exp returned (nothing folded: 0 and -inf)
__device__ __forceinline__ float fold_result(const PartialFold& f, float4& o) {
    const float inv = f.den > 0.f ? 1.f / f.den : 0.f;
    o = make_float4(f.num.x * inv, f.num.y * inv, f.num.z * inv, f.num.w * inv);
    return f.den > 0.f ? f.top + logf(f.den) : -INFINITY;
}

// Partial results that another workgroup of the SAME launch will read (single-launch path) are written
// and read with device-scope coherent accesses (the cache-policy bit the compiler gives a device-scope
// atomic access): such a store goes through to the level all compute dies share, such a load does not
// hit a stale line of the reader's own L2, and neither needs the whole-L2 write-back / invalidate of a
// device-scope fence.  Single words are atomic accesses; 16-byte accesses, for which there is no atomic
// form, are written as the same instruction with the same bit.  The compiler does not count those, so
// coherent_stores_done() / the wait inside load_coherent_pair() wait for them explicitly.
typedef float float4r __attribute__((ext_vector_type(4)));
template <bool kCoherent>
__device__ __forceinline__ void store_partial1(float* p, float x) {
    if constexpr (kCoherent) __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = x;
}
template <bool kCoherent>
__device__ __forceinline__ void store_partial4(float* p, float x0, float x1, float x2, float x3) {
    if constexpr (kCoherent) {
#if defined(__HIP_DEVICE_COMPILE__)
        const float4r v = {x0, x1, x2, x3};
        // the two idle cycles keep a following vector instruction from overwriting the data registers while
        // the store still reads them (the compiler inserts them itself for stores it knows about)
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
#endif
    } else {
        *reinterpret_cast<float4*>(p) = make_float4(x0, x1, x2, x3);
    }
}
// every coherent 16-byte store of this wavefront has completed
__device__ __forceinline__ void coherent_stores_done() {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
#endif
}
__device__ __forceinline__ float load_coherent1(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// a 16-byte coherent load the compiler keeps track of (four single-word ones): for loads that stay in
// flight behind other work
__device__ __forceinline__ float4 load_coherent4_tracked(const float* p) {
    return make_float4(load_coherent1(p), load_coherent1(p + 1), load_coherent1(p + 2), load_coherent1(p + 3));
}
// six coherent 16-byte loads in flight together, then the wait; the results are tied to the wait
__device__ __forceinline__ void load_coherent_six(const float* const (&p)[6], float4 (&x)[6]) {
#if defined(__HIP_DEVICE_COMPILE__)
    float4r v0, v1, v2, v3, v4, v5;
    asm volatile(
        "global_load_dwordx4 %0, %6, off sc1\n\tglobal_load_dwordx4 %1, %7, off sc1\n\t"
        "global_load_dwordx4 %2, %8, off sc1\n\tglobal_load_dwordx4 %3, %9, off sc1\n\t"
        "global_load_dwordx4 %4, %10, off sc1\n\tglobal_load_dwordx4 %5, %11, off sc1\n\ts_waitcnt vmcnt(0)"
        : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5)
        : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(p[4]), "v"(p[5])
        : "memory");
    x[0] = make_float4(v0[0], v0[1], v0[2], v0[3]);
    x[1] = make_float4(v1[0], v1[1], v1[2], v1[3]);
    x[2] = make_float4(v2[0], v2[1], v2[2], v2[3]);
    x[3] = make_float4(v3[0], v3[1], v3[2], v3[3]);
    x[4] = make_float4(v4[0], v4[1], v4[2], v4[3]);
    x[5] = make_float4(v5[0], v5[1], v5[2], v5[3]);
#endif
}

// Stores 4 consecutive merged elements at element offset `off` of an output in the layer's dtype.
template <bool kBf16Out>
__device__ __forceinline__ void store_out4(void* out, size_t off, float x0, float x1, float x2, float x3) {
    if constexpr (kBf16Out) {
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(out) + off) = make_uint2(pack_bf16(x0, x1), pack_bf16(x2, x3));
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(out) + off) = make_float4(x0, x1, x2, x3);
    }
}

// Data-parallel-primitive lane exchange inside a row of 16 lanes.
template <int kCtrl>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), kCtrl, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);   // row_half_mirror
    x += dpp_move<0x140>(x);   // row_mirror
    return x;
}

}  // namespace bllm

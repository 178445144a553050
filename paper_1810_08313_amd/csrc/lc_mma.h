// Device-side building blocks shared by the MLP kernels: MFMA operand fragments for bf16 and
// fp32 operands, their loads, stores and conversions, weight-row access helpers and the
// XCD-aware block index.  Internal linkage: every translation unit gets its own copy.
#pragma once
#include "lc_internal.h"

namespace lc {
namespace {

// ------------------------------------------------------------------ fragments

template <typename OT>
struct Frag;
template <>
struct Frag<float> {
    float v[8];
};
template <>
struct Frag<bf16_t> {
    bf16x8 v;
};

__device__ __forceinline__ Frag<float> load8(const float* p) {
    Frag<float> f;
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    f.v[0] = a.x; f.v[1] = a.y; f.v[2] = a.z; f.v[3] = a.w;
    f.v[4] = b.x; f.v[5] = b.y; f.v[6] = b.z; f.v[7] = b.w;
    return f;
}
__device__ __forceinline__ Frag<bf16_t> load8(const bf16_t* p) {
    Frag<bf16_t> f;
    f.v = *reinterpret_cast<const bf16x8*>(p);
    return f;
}

// Marks the point where prefetched registers are consumed.  Without it the compiler moves the
// conversion of a prefetched weight row up to its load, which makes every trip wait for the loads
// it has just issued (loads retire in order) and turns the prefetch queue into a plain load.
__device__ __forceinline__ void consume_here(float4& x) {
    asm volatile("" : "+v"(x.x), "+v"(x.y), "+v"(x.z), "+v"(x.w));
}
__device__ __forceinline__ void consume_here(Frag<float>& f) {
    asm volatile("" : "+v"(f.v[0]), "+v"(f.v[1]), "+v"(f.v[2]), "+v"(f.v[3]), "+v"(f.v[4]), "+v"(f.v[5]),
                      "+v"(f.v[6]), "+v"(f.v[7]));
}
__device__ __forceinline__ void consume_here(Frag<bf16_t>& f) {
    f32x4 t = __builtin_bit_cast(f32x4, f.v);
    asm volatile("" : "+v"(t));
    f.v = __builtin_bit_cast(bf16x8, t);
}

__device__ __forceinline__ void pack8(Frag<float>& f, const float (&x)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = x[e];
}
__device__ __forceinline__ void pack8(Frag<bf16_t>& f, const float (&x)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = static_cast<bf16_t>(x[e]);  // round to nearest even
}

__device__ __forceinline__ f32x4 mma8(const Frag<float>& a, const Frag<float>& b, f32x4 c) {
#pragma unroll
    for (int e = 0; e < 8; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[e], b.v[e], c, 0, 0, 0);
    return c;
}
__device__ __forceinline__ f32x4 mma8(const Frag<bf16_t>& a, const Frag<bf16_t>& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return static_cast<float>(x); }

template <typename OT>
__device__ __forceinline__ void store4(OT* p, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store4<float>(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
template <>
__device__ __forceinline__ void store4<bf16_t>(bf16_t* p, float a, float b, float c, float d) {
    bf16x4 v;
    v[0] = static_cast<bf16_t>(a); v[1] = static_cast<bf16_t>(b);
    v[2] = static_cast<bf16_t>(c); v[3] = static_cast<bf16_t>(d);
    *reinterpret_cast<bf16x4*>(p) = v;
}

// 8 consecutive outputs at a 16-byte aligned address
__device__ __forceinline__ void store8(float* p, const float (&y)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(y[0], y[1], y[2], y[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(y[4], y[5], y[6], y[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&y)[8]) {
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = static_cast<bf16_t>(y[i]);
    *reinterpret_cast<bf16x8*>(p) = v;
}

// Four consecutive floats of a weight row, zero outside [0, d_out).  When the
// state of all replicas is far larger than the caches, each weight is touched
// once per kernel and the loads and stores carry the non-temporal hint; small
// models, whose weights stay cache-resident between kernels, use plain accesses.
__device__ __forceinline__ float4 load_w4(const float* row, int c, int d_out, bool vec, bool stream) {
    if (vec && c + 3 < d_out) {
        if (!stream) return *reinterpret_cast<const float4*>(row + c);
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + c));
        return make_float4(t[0], t[1], t[2], t[3]);
    }
    // unaligned or ragged rows, element by element.  (Loading unconditionally from clamped
    // positions instead was measured and is slower: the cost of these loads grows with the
    // number of active lanes, and most lanes are past the end of a narrow row.)
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < d_out) r.x = row[c];
    if (c + 1 < d_out) r.y = row[c + 1];
    if (c + 2 < d_out) r.z = row[c + 2];
    if (c + 3 < d_out) r.w = row[c + 3];
    return r;
}
__device__ __forceinline__ void store_w4(float* row, int c, int d_out, bool vec, bool stream, float4 v) {
    if (vec && c + 3 < d_out) {
        if (stream) __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4*>(row + c));
        else *reinterpret_cast<float4*>(row + c) = v;
        return;
    }
    if (c < d_out) row[c] = v.x;
    if (c + 1 < d_out) row[c + 1] = v.y;
    if (c + 2 < d_out) row[c + 2] = v.z;
    if (c + 3 < d_out) row[c + 3] = v.w;
}

// Row `row` of a d_in x d_out matrix, columns c .. c+3, zero beyond either end -- without a branch
// around the loads (rows past the end read the last row and are zeroed afterwards).
__device__ __forceinline__ float4 load_w4_rows(const float* base, int row, int d_in, int c, int d_out, bool vec,
                                               bool stream) {
    const int rr = row < d_in ? row : d_in - 1;
    const float4 x = load_w4(base + static_cast<int64_t>(rr) * d_out, c, d_out, vec, stream);
    return row < d_in ? x : make_float4(0.f, 0.f, 0.f, 0.f);
}

// Weight access mode of a kernel instance.  kWGeneric checks every element against the row end
// (any d_out, any alignment).  The other two are for layers whose rows are 16-byte aligned and a
// multiple of 64 columns long: every access is one unconditional 16-byte instruction, which lets
// the compiler issue a trip's loads back to back with no control flow between them.
constexpr int kWGeneric = 0, kWVector = 1, kWVectorStream = 2;

template <int WM>
__device__ __forceinline__ float4 load_wm(const float* row, int c, int d_out, bool vec) {
    if constexpr (WM == kWVector) {
        return *reinterpret_cast<const float4*>(row + c);
    } else if constexpr (WM == kWVectorStream) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + c));
        return make_float4(t[0], t[1], t[2], t[3]);
    } else {
        return load_w4(row, c, d_out, vec, false);
    }
}
template <int WM>
__device__ __forceinline__ void store_wm(float* row, int c, int d_out, bool vec, float4 v) {
    if constexpr (WM == kWVector) {
        *reinterpret_cast<float4*>(row + c) = v;
    } else if constexpr (WM == kWVectorStream) {
        __builtin_nontemporal_store(f32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4*>(row + c));
    } else {
        store_w4(row, c, d_out, vec, false, v);
    }
}

// The momentum-SGD update with its roundings spelled out: v' = fma(beta, v, fma(wd, w, g)) and
// w' = fma(-lr, v', w).  Kernels whose results are compared bit for bit (the backward kernel, the
// tau = 1 first-layer kernel, the averaging kernels that form x_bar - lr v themselves) must not
// leave the choice of which products are fused to the compiler's contraction pass.
// Softmax cross-entropy of one sample from e_c = exp(z_c - max z), without the cancellation of
// "p_y - 1" and "log(sum)" when the label's class holds almost all of the mass (a well-fitted
// sample: p_y = 1 - 1e-5 in fp32 leaves three digits of p_y - 1).  With s the sum of e_c over the
// classes OTHER than the label y:
//     p_y - 1 = -s / (s + e_y),      -log p_y = log1p(s / e_y)   (while s < e_y; else the plain form).
__device__ __forceinline__ float xent_loss(float s_other, float e_y, float zy_minus_max) {
    return s_other < e_y ? log1pf(s_other / e_y) : logf(s_other + e_y) - zy_minus_max;
}
__device__ __forceinline__ float xent_delta(float e_c, bool is_label, float s_other, float inv_sum) {
    return (is_label ? -s_other : e_c) * inv_sum;
}

__device__ __forceinline__ float momentum_update(float beta, float v, float g, float wd, float w) {
    return __builtin_fmaf(beta, v, __builtin_fmaf(wd, w, g));
}
__device__ __forceinline__ float weight_update(float w, float lr, float v) { return __builtin_fmaf(-lr, v, w); }

__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroups are handed to the 8 XCDs round-robin.  This maps the hardware
// block id to a logical one such that each XCD works on a contiguous range of
// logical blocks (consecutive blocks of one replica then share that XCD's L2
// for the replica's activations).  Returns -1 for the padding blocks.
__device__ __forceinline__ int64_t xcd_logical_block(int64_t total) {
    const int64_t per = (total + kXcds - 1) / kXcds;
    const int64_t bid = blockIdx.x;
    const int64_t logical = (bid % kXcds) * per + bid / kXcds;
    return logical < total ? logical : -1;
}

// Logical block -> (replica g, tile rem of the per_group tiles of a replica).
//   set == 0  replica-major: a replica's blocks are neighbours and share its activations in the L2
//   set >= 1  tile-major inside sets of `set` replicas (set divides n_groups): neighbouring blocks
//             take the same weight tile for different replicas
__device__ __forceinline__ void shared_order(int64_t logical, int per_group, int set, int& g, int& rem) {
    if (set > 0) {
        const int64_t per_set = static_cast<int64_t>(per_group) * set;
        const int within = static_cast<int>(logical % per_set);
        g = static_cast<int>(logical / per_set) * set + within % set;
        rem = within / set;
    } else {
        g = static_cast<int>(logical / per_group);
        rem = static_cast<int>(logical % per_group);
    }
}

}  // namespace
}  // namespace lc

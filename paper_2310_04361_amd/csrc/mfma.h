// gfx950 matrix-core helpers: operand types, the 16x16x32 bf16 MFMA and its register layout.
//
// v_mfma_f32_16x16x32_bf16 computes D[16][16] += A[16][32] * B[32][16] per wavefront.
// With lane = 16*q + c (q = 0..3, c = 0..15):
//   A operand: lane holds A[i = c][k = 8q .. 8q+7]      (8 consecutive bf16 = one 16-byte load)
//   B operand: lane holds B[k = 8q .. 8q+7][j = c]      (same shape: 8 consecutive k of column c)
//   D / C    : lane holds D[i = 4q + r][j = c], r = 0..3
// Only "the same k goes to the same (lane group, slot) in A and in B" matters for the sum over k,
// so any k permutation applied to both operands is allowed; the kernels use that freedom.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dmoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// v_mfma_f32_32x32x16_bf16: D[32][32] += A[32][16] * B[16][32].  With lane = 32*h + c (h = 0..1,
// c = 0..31): A operand holds A[i = c][k = 8h .. 8h+7], B operand holds B[k = 8h .. 8h+7][j = c],
// and register r (0..15) of D holds D[i = 8*(r/4) + 4h + (r%4)][j = c].
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load in flight, which would drain the prefetches that the pipelined kernels keep outstanding
// across their barriers.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Neuron order of the hidden activations.  Lane (q, .) of the up-projection's 16-neuron tile mt
// holds the accumulator rows 4q + r; the packed up weights put the neurons there so that the
// 16-byte piece p = 4*(mt/2) + q of an H row (rows 4q + r of the tile pair 2*(mt/2), +1) is the
// eight CONSECUTIVE neurons 8p .. 8p+7: an expert of m neurons fills exactly its first
// ceil(m / 8) pieces, which lets the down-projection pack the real pieces of consecutive experts
// densely into its k-steps.
__host__ __device__ __forceinline__ int neuron_of_slot(int mt, int row) {
    return 8 * (4 * (mt >> 1) + (row >> 2)) + 4 * (mt & 1) + (row & 3);
}

__device__ __forceinline__ bf16x8 load8(const __bf16* p) {
    return *reinterpret_cast<const bf16x8*>(p);
}

// Router scores (Sec. 3.3) of the experts e0 .. e0+3 of one token from the second product's
// accumulator: |acc + c2|, and 0 for the components from E on (E need not be a multiple of 4;
// e0 is one, and e0 < E).
__device__ __forceinline__ float4 router_scores4(const f32x4& acc, const __bf16* __restrict__ r_b2,
                                                 int e0, int E) {
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        // the load is unconditional (clamped index): under the bound test each of the four would
        // be a block of its own that waits for its value
        const float bias = r_b2 ? (float)r_b2[min(e0 + r, E - 1)] : 0.0f;
        v[r] = e0 + r < E ? fabsf(acc[r] + bias) : 0.0f;
    }
    return make_float4(v[0], v[1], v[2], v[3]);
}
// ... and their store to row[e0 .. e0+3] of a [.][E] array: 16 bytes at once where the rows keep
// that alignment, else element by element up to E.
__device__ __forceinline__ void store_scores4(float* __restrict__ row, int e0, int E, const float4& v) {
    if ((E & 3) == 0) {
        *reinterpret_cast<float4*>(row + e0) = v;
    } else {
        row[e0] = v.x;
        if (e0 + 1 < E) row[e0 + 1] = v.y;
        if (e0 + 2 < E) row[e0 + 2] = v.z;
        if (e0 + 3 < E) row[e0 + 3] = v.w;
    }
}

// OCP E4M3 byte -> value (exact in bf16): 1 sign, 4 exponent bits (bias 7), 3 mantissa bits,
// subnormals m / 8 * 2^-6, no infinities.  Plain arithmetic, used by the one-time packing.
__device__ __forceinline__ float e4m3_value(uint32_t b) {
    const int e = (b >> 3) & 15, m = b & 7;
    const float mag = e == 0 ? ldexpf((float)m, -9) : ldexpf((float)(8 + m), e - 10);
    return (b & 0x80u) ? -mag : mag;
}

// Element `flat` of expert e's matrix `which` (0 up, 1 gate, 2 down) as a bf16 number: the stored
// bf16 value, or scale * e4m3(byte) for 8-bit weights (exact: the scales are powers of two).
__device__ __forceinline__ __bf16 expert_weight(const void* w, const float* scales, int fp8, int which,
                                               int e, size_t flat) {
    if (!fp8) return static_cast<const __bf16*>(w)[flat];
    return (__bf16)(scales[3 * e + which] * e4m3_value(static_cast<const uint8_t*>(w)[flat]));
}

// Eight E4M3 bytes (one lane's share of a weight fragment) -> eight bf16 numbers, exactly, with
// the hardware converter (two bytes per instruction) and a byte permute that keeps the upper
// halves of the fp32 results.
__device__ __forceinline__ bf16x8 e4m3x8_to_bf16(uint2 v) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
    u32x4v out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t word = i < 2 ? v.x : v.y;
        const f32x2 f = (i & 1) ? __builtin_amdgcn_cvt_pk_f32_fp8(word, true)
                                : __builtin_amdgcn_cvt_pk_f32_fp8(word, false);
        // bytes 2,3 of f[0] -> low half, bytes 2,3 of f[1] -> high half
        out[i] = __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);
    }
    return __builtin_bit_cast(bf16x8, out);
}

__device__ __forceinline__ bf16x8 zero8() {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.0f;
    return z;
}

__device__ __forceinline__ float bf16_to_float(__bf16 v) { return (float)v; }

// Activation A(v) in fp32.  GELU(v) = v * Phi(v); the tanh form is its usual approximation.
__device__ __forceinline__ float activate(int act, float v) {
    if (act == DMOE_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == DMOE_ACT_GELU_ERF) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
    const float u = 0.79788456080286535588f * (v + 0.044715f * v * v * v);
    return 0.5f * v * (1.0f + tanhf(u));
}

// Activations of the bf16 kernels (fp32 in, fp32 out).
// erf by the rational-times-exponential approximation 7.1.26 of Abramowitz & Stegun
// (absolute error below 1.5e-7, far inside bf16 resolution), tanh through one exponential.
__device__ __forceinline__ float fast_erf(float v) {
    const float a = fabsf(v);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, a, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float r = 1.0f - p * t * __expf(-a * a);
    return copysignf(r, v);
}

__device__ __forceinline__ float activate_fast(int act, float v) {
    if (act == DMOE_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == DMOE_ACT_GELU_ERF) return 0.5f * v * (1.0f + fast_erf(v * 0.70710678118654752440f));
    const float u = 0.79788456080286535588f * (v + 0.044715f * v * v * v);
    const float th = 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * u));  // tanh(u)
    return 0.5f * v * (1.0f + th);
}

// The activation as a compile-time constant for an epilogue that applies it to a hundred values
// per lane: with the layer's `act` tested per value the compiler kept two scalar branches around
// every one of them.  with_activation(act, f) calls f(ActTag<act>{}) once, under one test.
template <int ACT>
struct ActTag {
    static constexpr int value = ACT;
};
template <class F>
__device__ __forceinline__ void with_activation(int act, F&& f) {
    if (act == DMOE_ACT_RELU) f(ActTag<DMOE_ACT_RELU>{});
    else if (act == DMOE_ACT_GELU_ERF) f(ActTag<DMOE_ACT_GELU_ERF>{});
    else f(ActTag<DMOE_ACT_GELU_TANH>{});
}

}  // namespace dmoe

// Router (Sec. 3.3): scores = | R2 relu(R1 x + c1) + c2 |, one row of E scores per token.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

// ---------------------------------------------------------------------------------- fp32 path
// One workgroup per token; a wavefront per output unit with lanes striding the reduction.
__global__ __launch_bounds__(256) void router_f32_kernel(const float* __restrict__ x,
                                                         const float* __restrict__ r_w1,
                                                         const float* __restrict__ r_b1,
                                                         const float* __restrict__ r_w2,
                                                         const float* __restrict__ r_b2,
                                                         float* __restrict__ scores, int d, int dh,
                                                         int E) {
    extern __shared__ float smem[];
    float* xs = smem;       // [d]
    float* hs = smem + d;   // [dh]
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int k = threadIdx.x; k < d; k += 256) xs[k] = x[(size_t)t * d + k];
    __syncthreads();
    for (int j = wave; j < dh; j += 4) {
        const float* w = r_w1 + (size_t)j * d;
        float a = 0.0f;
        for (int k = lane; k < d; k += 64) a = fmaf(w[k], xs[k], a);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
        if (lane == 0) hs[j] = fmaxf(a + (r_b1 ? r_b1[j] : 0.0f), 0.0f);
    }
    __syncthreads();
    for (int i = wave; i < E; i += 4) {
        const float* w = r_w2 + (size_t)i * dh;
        float a = 0.0f;
        for (int k = lane; k < dh; k += 64) a = fmaf(w[k], hs[k], a);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
        if (lane == 0) scores[(size_t)t * E + i] = fabsf(a + (r_b2 ? r_b2[i] : 0.0f));
    }
}

// ---------------------------------------------------------------------------------- bf16 path
// One wavefront per 16 tokens, tokens on the MFMA column axis for both layers:
//   layer 1:  hid^T[dh][16] = R1[dh][d] * x^T[d][16]   (A = R1 rows, B = token rows of x)
//   layer 2:  s^T[E][16]    = R2[E][dh] * hid^T        (A = R2 rows, B = layer-1 accumulators)
// The layer-1 accumulator of lane (q, c) holds hidden units 16h + 4q + r of token c, which is
// exactly a B operand of layer 2 up to a permutation of k; R2 is loaded with the same
// permutation (two 8-byte pieces per lane), so the hidden vector never leaves registers.
// NH = dh / 16.
template <int NH>
__global__ __launch_bounds__(256) void router_bf16_kernel(const __bf16* __restrict__ x,
                                                          const __bf16* __restrict__ r_w1,
                                                          const __bf16* __restrict__ r_b1,
                                                          const __bf16* __restrict__ r_w2,
                                                          const __bf16* __restrict__ r_b2,
                                                          float* __restrict__ scores, int T, int d,
                                                          int E) {
    constexpr int dh = NH * 16;
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15;
    const int tile = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int t0 = tile * 16;
    if (t0 >= T) return;  // uniform per wavefront
    const int tok = min(t0 + c, T - 1);
    const __bf16* xrow = x + (size_t)tok * d + 8 * q;
    const __bf16* w1 = r_w1 + (size_t)c * d + 8 * q;

    f32x4 acc[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) acc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < d; k0 += 32) {
        const bf16x8 b = load8(xrow + k0);
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const bf16x8 a = load8(w1 + (size_t)h * 16 * d + k0);
            acc[h] = mfma16(a, b, acc[h]);
        }
    }

    // bias, relu, round to bf16: slot 4*half + r of step s  <->  hidden unit 32s + 16half + 4q + r
    bf16x8 hb[NH / 2];
#pragma unroll
    for (int s = 0; s < NH / 2; ++s) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int h = 2 * s + half;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[h][r];
                if (r_b1) v += (float)r_b1[h * 16 + 4 * q + r];
                hb[s][half * 4 + r] = (__bf16)fmaxf(v, 0.0f);
            }
        }
    }

    const int NE = (E + 15) / 16;
    for (int et = 0; et < NE; ++et) {
        const int erow = min(et * 16 + c, E - 1);
        const __bf16* w2 = r_w2 + (size_t)erow * dh + 4 * q;
        f32x4 acc2 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NH / 2; ++s) {
            const bf16x4 lo = *reinterpret_cast<const bf16x4*>(w2 + 32 * s);
            const bf16x4 hi = *reinterpret_cast<const bf16x4*>(w2 + 32 * s + 16);
            bf16x8 a;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = lo[i];
                a[4 + i] = hi[i];
            }
            acc2 = mfma16(a, hb[s], acc2);
        }
        const int e0 = et * 16 + 4 * q;  // this lane: experts e0 .. e0+3 of token t0 + c
        if (t0 + c < T && e0 < E) {
            store_scores4(scores + (size_t)(t0 + c) * E, e0, E, router_scores4(acc2, r_b2, e0, E));
        }
    }
}

template <int NH>
void launch_router_bf16_t(const dmoe_layer& L, const void* x, int T, float* scores, hipStream_t s) {
    const int tiles = div_up(T, 16);
    launch_kernel(router_bf16_kernel<NH>, div_up(tiles, 4), 256, 0, s, 
        (const __bf16*)x, (const __bf16*)L.r_w1, (const __bf16*)L.r_b1, (const __bf16*)L.r_w2,
        (const __bf16*)L.r_b2, scores, T, L.d_model, L.n_experts);
}

}  // namespace

bool router_bf16_supported(const dmoe_layer& L) {
    const int dh = L.router_hidden;
    const bool dh_ok = dh == 32 || dh == 64 || dh == 128 || dh == 256 || dh == 512;
    return dh_ok && L.d_model % 32 == 0;
}

void launch_router_f32(const dmoe_layer& L, const float* x, int T, float* scores, hipStream_t s) {
    LaunchTimer tm(kSlotRouter, s);
    const size_t lds = sizeof(float) * (size_t)(L.d_model + L.router_hidden);
    launch_kernel(router_f32_kernel, T, 256, lds, s, x, (const float*)L.r_w1, (const float*)L.r_b1,
                                          (const float*)L.r_w2, (const float*)L.r_b2, scores,
                                          L.d_model, L.router_hidden, L.n_experts);
}

void launch_router_bf16(const dmoe_layer& L, const void* x, int T, float* scores, hipStream_t s) {
    LaunchTimer tm(kSlotRouter, s);
    switch (L.router_hidden) {
    case 32: launch_router_bf16_t<2>(L, x, T, scores, s); break;
    case 64: launch_router_bf16_t<4>(L, x, T, scores, s); break;
    case 128: launch_router_bf16_t<8>(L, x, T, scores, s); break;
    case 256: launch_router_bf16_t<16>(L, x, T, scores, s); break;
    case 512: launch_router_bf16_t<32>(L, x, T, scores, s); break;
    default: break;  // refused earlier by router_bf16_supported
    }
}

}  // namespace dmoe

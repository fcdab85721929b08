// fp32 expert execution and merge (Sec. 3.2, Appendix G): token-major, straight from the mask.
// One workgroup per token walks the token's selected experts in ascending order, so the result
// is deterministic.  Meant for the small fp32 exactness configuration, not for speed.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

__global__ __launch_bounds__(256) void ffn_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w_up, const float* __restrict__ w_gate,
    const float* __restrict__ b_up, const float* __restrict__ w_down,
    const float* __restrict__ b_down, const uint64_t* __restrict__ mask, float* __restrict__ y,
    int d, int E, int m, int W, int act) {
    extern __shared__ float smem[];
    float* xs = smem;          // [d]
    float* ys = smem + d;      // [d]
    float* hs = smem + 2 * d;  // [m]
    const int t = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int k = threadIdx.x; k < d; k += 256) {
        xs[k] = x[(size_t)t * d + k];
        ys[k] = b_down ? b_down[k] : 0.0f;
    }
    __syncthreads();
    for (int e = 0; e < E; ++e) {
        const uint64_t word = mask[(size_t)t * W + (e >> 6)];
        if (!((word >> (e & 63)) & 1ull)) continue;  // uniform over the workgroup
        for (int j = wave; j < m; j += 4) {
            const size_t row = ((size_t)e * m + j) * d;
            float a = 0.0f, g = 0.0f;
            for (int k = lane; k < d; k += 64) {
                a = fmaf(w_up[row + k], xs[k], a);
                if (w_gate) g = fmaf(w_gate[row + k], xs[k], g);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                a += __shfl_xor(a, off, 64);
                g += __shfl_xor(g, off, 64);
            }
            if (lane == 0) {
                if (w_gate) hs[j] = activate(act, g) * a;
                else hs[j] = activate(act, a + (b_up ? b_up[(size_t)e * m + j] : 0.0f));
            }
        }
        __syncthreads();
        for (int c = threadIdx.x; c < d; c += 256) {
            float acc = ys[c];
            const float* wd = w_down + (size_t)e * m * d + c;
            for (int j = 0; j < m; ++j) acc = fmaf(hs[j], wd[(size_t)j * d], acc);
            ys[c] = acc;
        }
        __syncthreads();
    }
    for (int c = threadIdx.x; c < d; c += 256) y[(size_t)t * d + c] = ys[c];
}

}  // namespace

void launch_ffn_f32(const dmoe_layer& L, const float* x, int T, const uint64_t* mask, float* y,
                    hipStream_t s) {
    LaunchTimer tm(kSlotFfnF32, s);
    const int W = div_up(L.n_experts, 64);
    const size_t lds = sizeof(float) * (size_t)(2 * L.d_model + L.expert_size);
    launch_kernel(ffn_f32_kernel, T, 256, lds, s, x, (const float*)L.w_up,
                                       L.gated ? (const float*)L.w_gate : nullptr,
                                       (const float*)L.b_up, (const float*)L.w_down,
                                       (const float*)L.b_down, mask, y, L.d_model, L.n_experts,
                                       L.expert_size, W, L.act);
}

}  // namespace dmoe

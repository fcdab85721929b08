// bf16 expert execution and merge (Sec. 3.2, Appendix G) on the gfx950 matrix cores.
//
// Two kernels, both driven by the sorted per-expert token lists:
//   up    expert-major grouped GEMM over the compact lists: gathers the listed rows of x (no
//         copy), multiplies by the expert's up (and gate) rows, applies bias + activation in fp32
//         and writes the hidden activations, rounded to bf16, to H[list position][m_pad].
//   down  output-stationary: a workgroup owns 256 consecutive tokens x 128 output columns as an
//         fp32 tile in LDS, walks all experts, multiplies the chunk's compact H rows of each
//         expert by that expert's down-projection slice and adds the result into the owning
//         token rows with LDS atomics.  Every y element is written exactly once, in bf16; no
//         global atomics, no second pass.
// Tokens ride on the MFMA column axis in `up` (so four consecutive neurons of one token land in
// one lane and H is written in 8-byte pieces) and on the row axis in `down` (so one LDS-add
// instruction covers 16 consecutive output columns of four token rows).
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

constexpr int kDownCols = 128;                 // output columns per down workgroup
constexpr int kDownStride = kDownCols + 16;    // LDS row stride in floats (bank spread)
constexpr int kDownWaves = 8;

// w_down[E][m][d] -> w2t[E][d][m_pad], zero-filled for j >= m.
__global__ void pack_down_kernel(const __bf16* __restrict__ w_down, __bf16* __restrict__ w2t,
                                 int E, int m, int d, int m_pad) {
    const size_t n = (size_t)E * d * m_pad;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int j = (int)(i % m_pad);
        const size_t ec = i / m_pad;
        const int col = (int)(ec % d);
        const int e = (int)(ec / d);
        w2t[i] = j < m ? w_down[((size_t)e * m + j) * d + col] : (__bf16)0.0f;
    }
}

// One wavefront per work item = (expert, 64 consecutive list rows).
// MT = m_pad / 16 neuron tiles per branch.
template <int MT, bool GATED>
__global__ __launch_bounds__(256) void up_bf16_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ w_up,
    const __bf16* __restrict__ w_gate, const __bf16* __restrict__ b_up,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ item_start,
    const int32_t* __restrict__ lists, __bf16* __restrict__ H, int d, int E, int m, int act) {
    constexpr int TT = kUpRows / 16;
    constexpr int BR = GATED ? 2 : 1;
    constexpr int m_pad = MT * 16;
    extern __shared__ int32_t s_items[];  // item_start[0..E]
    for (int i = threadIdx.x; i <= E; i += blockDim.x) s_items[i] = item_start[i];
    __syncthreads();
    const int total = s_items[E];
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;

    for (int item = wave; item < total; item += n_waves) {
        int lo = 0, hi = E;  // last e with s_items[e] <= item
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_items[mid] <= item) lo = mid; else hi = mid;
        }
        const int e = lo;
        const int p0 = offsets[e] + (item - s_items[e]) * kUpRows;
        const int pend = offsets[e + 1];
        const int rows = min(kUpRows, pend - p0);

        const __bf16* xr[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int tok = lists[min(p0 + tt * 16 + c, pend - 1)];
            xr[tt] = x + (size_t)tok * d + 8 * q;
        }
        const __bf16* wr[BR][MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const size_t row = (size_t)e * m + min(mt * 16 + c, m - 1);
            wr[0][mt] = w_up + row * d + 8 * q;
            if (GATED) wr[BR - 1][mt] = w_gate + row * d + 8 * q;
        }

        f32x4 acc[BR][MT][TT];
#pragma unroll
        for (int br = 0; br < BR; ++br)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[br][mt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int k0 = 0; k0 < d; k0 += 32) {
            bf16x8 b[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) b[tt] = load8(xr[tt] + k0);
#pragma unroll
            for (int br = 0; br < BR; ++br)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const bf16x8 a = load8(wr[br][mt] + k0);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        acc[br][mt][tt] = mfma16(a, b[tt], acc[br][mt][tt]);
                }
        }

        // lane (q, c) of tile (mt, tt): neurons mt*16 + 4q + r of list row tt*16 + c
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int n0 = mt * 16 + 4 * q;
            float bias[4] = {0.f, 0.f, 0.f, 0.f};
            if (!GATED && b_up) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (n0 + r < m) bias[r] = (float)b_up[(size_t)e * m + n0 + r];
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                bf16x4 h;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v;
                    if (GATED) v = activate(act, acc[BR - 1][mt][tt][r]) * acc[0][mt][tt][r];
                    else v = activate(act, acc[0][mt][tt][r] + bias[r]);
                    if (n0 + r >= m) v = 0.0f;
                    h[r] = (__bf16)v;
                }
                const int ri = tt * 16 + c;
                if (ri < rows)
                    *reinterpret_cast<bf16x4*>(H + (size_t)(p0 + ri) * m_pad + n0) = h;
            }
        }
    }
}

// One workgroup per (256-token chunk, 128-column slice).  KS = m_pad / 32 MFMA k-steps.
template <int KS>
__global__ __launch_bounds__(kDownWaves * 64) void down_bf16_kernel(
    const __bf16* __restrict__ w2t, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ group_off,
    const int32_t* __restrict__ lists, const __bf16* __restrict__ H, __bf16* __restrict__ y, int T,
    int d, int E, int NG) {
    constexpr int m_pad = KS * 32;
    constexpr int NT = kDownCols / 16;
    extern __shared__ float Y[];  // [kChunk][kDownStride]
    const int NS = d / kDownCols;
    const int chunk = blockIdx.x / NS, slice = blockIdx.x % NS;
    const int t_base = chunk * kChunk, col0 = slice * kDownCols;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, q = lane >> 4, c = lane & 15;

    for (int i = tid; i < kChunk * kDownCols; i += kDownWaves * 64) {
        const int row = i / kDownCols, col = i % kDownCols;
        Y[row * kDownStride + col] = b_down ? (float)b_down[col0 + col] : 0.0f;
    }
    __syncthreads();

    const int g_lo = chunk * kChunkGroups;
    const int g_hi = min(g_lo + kChunkGroups, NG);
    for (int e = wave; e < E; e += kDownWaves) {
        const int lo = group_off[(size_t)g_lo * E + e];
        const int n = group_off[(size_t)g_hi * E + e] - lo;
        if (n <= 0) continue;
        const int p0 = offsets[e] + lo;
        bf16x8 bw[NT][KS];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                bw[nt][ks] = load8(w2t + ((size_t)e * d + col0 + nt * 16 + c) * m_pad + ks * 32 + 8 * q);

        for (int r0 = 0; r0 < n; r0 += 16) {
            bf16x8 a[KS];
            const bool va = r0 + c < n;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                a[ks] = va ? load8(H + (size_t)(p0 + r0 + c) * m_pad + ks * 32 + 8 * q) : zero8();
            int lrow[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ri = r0 + 4 * q + r;
                lrow[r] = ri < n ? lists[p0 + ri] - t_base : -1;
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(a[ks], bw[nt][ks], acc);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if ((unsigned)lrow[r] < (unsigned)kChunk)
                        atomicAdd(&Y[lrow[r] * kDownStride + nt * 16 + c], acc[r]);
            }
        }
    }
    __syncthreads();

    for (int i = tid; i < kChunk * (kDownCols / 8); i += kDownWaves * 64) {
        const int row = i / (kDownCols / 8), cg = i % (kDownCols / 8);
        const int t = t_base + row;
        if (t < T) {
            const float* src = Y + row * kDownStride + cg * 8;
            bf16x8 o;
#pragma unroll
            for (int k = 0; k < 8; ++k) o[k] = (__bf16)src[k];
            *reinterpret_cast<bf16x8*>(y + (size_t)t * d + col0 + cg * 8) = o;
        }
    }
}

template <int MT, bool GATED>
void launch_up_t(const dmoe_layer& L, const void* x, const int32_t* offsets,
                 const int32_t* item_start, const int32_t* lists, void* H, int grid,
                 hipStream_t s) {
    const size_t lds = sizeof(int32_t) * (size_t)(L.n_experts + 1);
    up_bf16_kernel<MT, GATED><<<grid, 256, lds, s>>>(
        (const __bf16*)x, (const __bf16*)L.w_up, (const __bf16*)L.w_gate, (const __bf16*)L.b_up,
        offsets, item_start, lists, (__bf16*)H, L.d_model, L.n_experts, L.expert_size, L.act);
}

template <int KS>
void launch_down_t(const dmoe_layer& L, int T, const int32_t* offsets, const int32_t* group_off,
                   const int32_t* lists, const void* H, void* y, hipStream_t s) {
    const int NG = div_up(T, kGroup), NC = div_up(T, kChunk), NS = L.d_model / kDownCols;
    const size_t lds = sizeof(float) * (size_t)kChunk * kDownStride;
    static bool attr_set = false;  // raising the dynamic-LDS limit is a per-function, idempotent setting
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&down_bf16_kernel<KS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    down_bf16_kernel<KS><<<NC * NS, kDownWaves * 64, lds, s>>>(
        (const __bf16*)L.packed, (const __bf16*)L.b_down, offsets, group_off, lists,
        (const __bf16*)H, (__bf16*)y, T, L.d_model, L.n_experts, NG);
}

}  // namespace

bool up_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    return (mp == 32 || mp == 64 || mp == 128) && L.d_model % 32 == 0 && L.n_experts <= 4096;
}

bool down_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    return (mp == 32 || mp == 64 || mp == 128) && L.d_model % kDownCols == 0;
}

void launch_pack_bf16(const dmoe_layer& L, void* packed, hipStream_t s) {
    LaunchTimer tm(kSlotPack, s);
    pack_down_kernel<<<2048, 256, 0, s>>>((const __bf16*)L.w_down, (__bf16*)packed, L.n_experts,
                                          L.expert_size, L.d_model, m_pad_of(L.expert_size));
}

void launch_up_bf16(const dmoe_layer& L, const void* x, int T, const int32_t* offsets,
                    const int32_t* item_start, const int32_t* token_lists, void* H,
                    hipStream_t s) {
    LaunchTimer tm(kSlotUp, s);
    // persistent wavefronts: enough to cover the worst case once, capped at a few per SIMD
    const long long worst = (long long)T * L.n_experts / kUpRows + L.n_experts;
    const int grid = (int)std::min<long long>(div_up((int)std::min<long long>(worst, 1 << 30), 4),
                                              256 * 8);
    const int mt = m_pad_of(L.expert_size) / 16;
    if (L.gated) {
        if (mt == 2) launch_up_t<2, true>(L, x, offsets, item_start, token_lists, H, grid, s);
        else if (mt == 4) launch_up_t<4, true>(L, x, offsets, item_start, token_lists, H, grid, s);
        else launch_up_t<8, true>(L, x, offsets, item_start, token_lists, H, grid, s);
    } else {
        if (mt == 2) launch_up_t<2, false>(L, x, offsets, item_start, token_lists, H, grid, s);
        else if (mt == 4) launch_up_t<4, false>(L, x, offsets, item_start, token_lists, H, grid, s);
        else launch_up_t<8, false>(L, x, offsets, item_start, token_lists, H, grid, s);
    }
}

void launch_down_bf16(const dmoe_layer& L, int T, const int32_t* offsets, const int32_t* group_off,
                      const int32_t* token_lists, const void* H, void* y, hipStream_t s) {
    LaunchTimer tm(kSlotDown, s);
    const int ks = m_pad_of(L.expert_size) / 32;
    if (ks == 1) launch_down_t<1>(L, T, offsets, group_off, token_lists, H, y, s);
    else if (ks == 2) launch_down_t<2>(L, T, offsets, group_off, token_lists, H, y, s);
    else launch_down_t<4>(L, T, offsets, group_off, token_lists, H, y, s);
}

}  // namespace dmoe

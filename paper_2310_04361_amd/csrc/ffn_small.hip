// Small-token (decode) experts: T <= 16 tokens ride in ONE MFMA column tile, so the work is
// reading every touched expert's weights exactly once -- a weight-bandwidth-bound stream.
//
//   up_small    one workgroup of sixteen wavefronts per expert; experts nobody selected exit
//               before touching their weights.  With the gate folded in (gate_dh > 0) every
//               workgroup first repeats the second router product and the threshold of Eq. 4 from
//               the router's hidden rows -- 128 KB of router matrix out of L2 and a handful of
//               MFMAs per wavefront -- and so knows its own expert's tokens without a gate kernel
//               in front of it; one extra workgroup writes the scores, the mask and the
//               per-expert token sets for the kernels and callers that follow.  The 16 x rows sit in LDS; wavefront (tile, slice)
//               streams a K slice of one neuron tile of the up (and gate) fragments -- 1 KiB
//               contiguous per load, 8 to 16 loads in flight per wavefront -- the slices are added
//               through LDS and h (zero for tokens that did not select the expert) goes out as an
//               H fragment.
//   down_small  workgroup = (4 output-column tiles, group of experts): streams the touched
//               experts' down fragments of its columns, accumulates in registers and writes one
//               fp32 partial per expert group (no atomics).
//   finish      y = bf16(b_down + sum of the partials).
// colmask[e] (bit j = token j keeps expert e) comes from the gate's ballot transpose.
#include "dmoe_internal.h"
#include "mfma.h"
#include "small_gate.h"

namespace dmoe {

namespace {


// Sixteen wavefronts per workgroup = MT neuron tiles (m_pad / 16) x KQ slices of the K range: an
// expert's weights are a pure stream, so what counts is how many bytes a CU keeps in flight.
// Wavefront (mt, kq) streams its slice of tile mt (up and gate fragments, eight k-steps of loads
// issued together), the KQ partial products are added through LDS.
constexpr int kUpSmallWaves = 16;

// W8: the weight fragments hold one E4M3 byte per weight (half the stream); they are converted to
// bf16 in registers, and the per-expert power-of-two scales are applied to the fp32 sums.
template <int MT, bool GATED, bool W8>
__global__ __launch_bounds__(64 * kUpSmallWaves) void up_small_kernel(
    const SmallGroup G, const __bf16* __restrict__ x, int T, int d, int m, int act, int KQ,
    int E, int gate_dh) {
    const SmallMod& M = G.m[blockIdx.z];
    const __bf16* __restrict__ wupf = M.wupf;
    const __bf16* __restrict__ wgatef = M.wgatef;
    const __bf16* __restrict__ b_up = M.b_up;
    __bf16* __restrict__ Hs = M.Hs;
    constexpr int KS = MT / 2, kThreads = 64 * kUpSmallWaves, BR = GATED ? 2 : 1;
    const int e = blockIdx.x;
    extern __shared__ char smem[];
    const int tid = threadIdx.x, lane = tid & 63, q = lane >> 4, c = lane & 15;
    const int pieces = d / 8;
    // With the gate folded in, the first x pieces of every thread are requested before the gate
    // and parked in LDS after it (the gate's scores use the same LDS).
    constexpr int kPre = 4;
    bf16x8 xpre[kPre];
    auto x_piece = [&](int i) {
        return load8(x + (size_t)min(i / pieces, T - 1) * d + (i % pieces) * 8);
    };
    if (gate_dh > 0 && e < E) {
#pragma unroll
        for (int k = 0; k < kPre; ++k)
            if (tid + k * kThreads < 16 * pieces) xpre[k] = x_piece(tid + k * kThreads);
    }
    uint64_t cm;
    if (gate_dh > 0) {
        // scores of all experts in LDS, then this expert's column against every token's threshold
        const int W = (E + 63) >> 6;
        // (all in the dynamic block: a static array next to a 160 KB dynamic limit is refused)
        int* s_keep = reinterpret_cast<int*>(smem);                   // [16]
        uint64_t* mw = reinterpret_cast<uint64_t*>(smem + 64);        // [16][W], output workgroup only
        float* sc = reinterpret_cast<float*>(mw + 16 * W);            // [16][E]
        const bool out_wg = e == E;  // the extra workgroup: scores, mask, token sets to memory
        small_scores_to_lds(M, T, gate_dh, E, sc, out_wg);
        __syncthreads();
        if (out_wg) {
            select_small_body(sc, mw, M.mask, nullptr, M.group_cnt, M.colmask, T, E, W, M.tau);
            return;
        }
        const int t = threadIdx.x >> 6;  // wavefront t = token t
        bool keep = false;
        if (t < T) keep = small_keeps(sc[(size_t)t * E + e], M.tau, small_row_max(sc + (size_t)t * E, E));
        if ((threadIdx.x & 63) == 0) s_keep[t] = keep ? 1 : 0;
        __syncthreads();
        cm = __ballot((threadIdx.x & 63) < 16 && s_keep[threadIdx.x & 15] != 0) & 0xffffull;
        __syncthreads();  // the score rows make way for the x rows
    } else {
        cm = M.colmask[e];
    }
    if (cm == 0ull) return;  // uniform: nobody selected this expert
    const int row_bytes = 2 * d + 16;
    char* xs = smem;                                                    // [16][2d + 16]
    // [16 waves][BR][64][4] partial sums: they take the place of the x rows once every wavefront
    // has finished reading those
    float* red = reinterpret_cast<float*>(smem);
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = w % MT, kq = w / MT;
    auto x_park = [&](int i, bf16x8 v) {
        *reinterpret_cast<bf16x8*>(xs + (i / pieces) * row_bytes + (i % pieces) * 16) = v;
    };
    int i_first = tid;
    if (gate_dh > 0) {
#pragma unroll
        for (int k = 0; k < kPre; ++k)
            if (tid + k * kThreads < 16 * pieces) x_park(tid + k * kThreads, xpre[k]);
        i_first = tid + kPre * kThreads;
    }
    for (int i = i_first; i < 16 * pieces; i += kThreads) x_park(i, x_piece(i));
    __syncthreads();

    const int NK32 = d / 32, per = NK32 / KQ;  // k-steps per slice (KQ divides NK32)
    f32x4 acc[BR];
#pragma unroll
    for (int br = 0; br < BR; ++br) acc[br] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (kq < KQ) {
        const size_t frag0 = (((size_t)e * MT + mt) * NK32 * 64 + lane) * 8;  // elements
        const __bf16* au = wupf + frag0;
        const __bf16* ag = wgatef + frag0;
        const uint8_t* au8 = M.wupf8 + frag0;
        const uint8_t* ag8 = M.wgatef8 + frag0;
        const char* bsrc = xs + c * row_bytes + q * 16;
        const int k0 = kq * per;
        for (int kb = 0; kb < per; kb += 8) {
            bf16x8 a[8][BR];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int ks = k0 + min(kb + i, per - 1);  // past the slice: a block already read
                if (W8) {
                    a[i][0] = e4m3x8_to_bf16(*reinterpret_cast<const uint2*>(au8 + (size_t)ks * 512));
                    if (GATED)
                        a[i][BR - 1] = e4m3x8_to_bf16(*reinterpret_cast<const uint2*>(ag8 + (size_t)ks * 512));
                } else {
                    a[i][0] = load8(au + (size_t)ks * 512);
                    if (GATED) a[i][BR - 1] = load8(ag + (size_t)ks * 512);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (kb + i < per) {
                    const bf16x8 b = *reinterpret_cast<const bf16x8*>(bsrc + (k0 + kb + i) * 64);
#pragma unroll
                    for (int br = 0; br < BR; ++br) acc[br] = mfma16(a[i][br], b, acc[br]);
                }
            }
        }
    }
    __syncthreads();  // the x rows have been consumed
#pragma unroll
    for (int br = 0; br < BR; ++br)
        *reinterpret_cast<f32x4*>(red + ((w * BR + br) * 64 + lane) * 4) = acc[br];
    __syncthreads();
    if (kq != 0) return;
    // wavefront (mt, 0): sum the KQ slices; lane (q, c): neurons neuron_of_slot(mt, 4q + r) of token c
#pragma unroll
    for (int br = 0; br < BR; ++br) {
        f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < KQ; ++k) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(red + (((k * MT + mt) * BR + br) * 64 + lane) * 4);
            sum += v;
        }
        acc[br] = sum;
    }
    const bool keep = c < T && ((cm >> c) & 1ull);
    float s_up = 1.0f, s_gate = 1.0f, s_down = 1.0f;
    if (W8) {
        s_up = M.w_scales[3 * e + 0];
        s_gate = M.w_scales[3 * e + 1];
        s_down = M.w_scales[3 * e + 2];  // folded into H: the down kernel sums over experts
    }
    bf16x4 hv;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int n = neuron_of_slot(mt, 4 * q + r);
        float v;
        if (GATED) {
            v = activate_fast(act, acc[BR - 1][r] * s_gate) * (acc[0][r] * s_up);
        } else {
            const float bias = b_up ? (float)b_up[(size_t)e * m + min(n, m - 1)] : 0.0f;
            v = activate_fast(act, acc[0][r] * s_up + bias);
        }
        v *= s_down;
        if (n >= m || !keep) v = 0.0f;
        hv[r] = (__bf16)v;
    }
    *reinterpret_cast<bf16x4*>(Hs + (((size_t)e * KS + (mt >> 1)) * 64 + lane) * 8 + (mt & 1) * 4) = hv;
}

constexpr int kSmallPerGroup = 256;  // experts per group at most

// grid = (column-tile groups of 4, expert groups); KS = m_pad / 32.
template <int KS, bool W8>
__global__ __launch_bounds__(256) void down_small_kernel(const SmallGroup G, int T, int d, int E,
                                                         int per) {
    const SmallMod& M = G.m[blockIdx.z];
    const __bf16* __restrict__ w2f = M.w2f;
    const uint64_t* __restrict__ colmask = M.colmask;
    const __bf16* __restrict__ Hs = M.Hs;
    float* __restrict__ partial = M.partial;
    __shared__ int s_list[kSmallPerGroup];
    __shared__ int s_n;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, q = lane >> 4, c = lane & 15;
    const int eg = blockIdx.y;
    const int e0 = eg * per, e1 = min(E, e0 + per);
    if (w == 0) {  // compact list of this group's touched experts
        int n = 0;
        for (int base = e0; base < e1; base += 64) {
            const int e = base + lane;
            const bool f = e < e1 && colmask[e] != 0ull;
            const uint64_t bal = __ballot(f);
            if (f) s_list[n + __popcll(bal & ((1ull << lane) - 1ull))] = e;
            n += __popcll(bal);
        }
        if (lane == 0) s_n = n;
    }
    __syncthreads();
    const int n = s_n;
    const int ct = blockIdx.x * 4 + w;
    if (ct >= d / 16) return;
    const __bf16* wa = w2f + ((size_t)ct * KS * 64 + lane) * 8;
    const uint8_t* wa8 = M.w2f8 + ((size_t)ct * KS * 64 + lane) * 8;
    const size_t w_expert_stride = (size_t)(d / 16) * KS * 512;
    const __bf16* hb = Hs + lane * 8;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int i = 0; i < n; ++i) {
        const int e = s_list[i];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            acc = mfma16(W8 ? e4m3x8_to_bf16(*reinterpret_cast<const uint2*>(
                                  wa8 + (size_t)e * w_expert_stride + ks * 512))
                            : load8(wa + (size_t)e * w_expert_stride + ks * 512),
                         load8(hb + ((size_t)e * KS + ks) * 512), acc);
    }
    // lane (q, c): columns 16ct + 4q .. +3 of token c
    if (c < T) {
        float4 o;
        o.x = acc[0]; o.y = acc[1]; o.z = acc[2]; o.w = acc[3];
        *reinterpret_cast<float4*>(partial + ((size_t)eg * 16 + c) * d + 16 * ct + 4 * q) = o;
    }
}

__global__ void finish_small_kernel(const SmallGroup G, int T, int d, int EG) {
    const SmallMod& M = G.m[blockIdx.z];
    const float* __restrict__ partial = M.partial;
    const __bf16* __restrict__ b_down = M.b_down;
    __bf16* __restrict__ y = M.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * d) return;
    const int t = i / d, col = i % d;
    float v = b_down ? (float)b_down[col] : 0.0f;
    const float* p = partial + (size_t)t * d + col;
    const size_t stride = (size_t)16 * d;
    int eg = 0;
    for (; eg + 8 <= EG; eg += 8) {  // eight independent loads in flight
        float u[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) u[k] = p[(size_t)(eg + k) * stride];
#pragma unroll
        for (int k = 0; k < 8; ++k) v += u[k];
    }
    for (; eg < EG; ++eg) v += p[(size_t)eg * stride];
    y[i] = (__bf16)v;
}

template <int MT, bool GATED, bool W8>
void launch_up_small_t(const dmoe_layer& L, const SmallGroup& G, int n_layers, const void* x, int T,
                       bool gate, hipStream_t s) {
    const int E = L.n_experts;
    size_t lds = std::max(16 * (2 * (size_t)L.d_model + 16),
                          sizeof(float) * kUpSmallWaves * (GATED ? 2 : 1) * 64 * 4);
    if (gate) lds = std::max(lds, 64 + sizeof(uint64_t) * 16 * div_up(E, 64) + sizeof(float) * 16 * (size_t)E);
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_small_kernel<MT, GATED, W8>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    // K slices: as many as the sixteen wavefronts allow and the k-steps divide into
    int KQ = kUpSmallWaves / MT;
    while (KQ > 1 && (L.d_model / 32) % KQ != 0) KQ >>= 1;
    launch_kernel(up_small_kernel<MT, GATED, W8>, dim3(E + (gate ? 1 : 0), 1, n_layers),
                  64 * kUpSmallWaves, lds, s, G, (const __bf16*)x, T, L.d_model, L.expert_size, L.act,
                  KQ, E, gate ? L.router_hidden : 0);
}

template <int MT, bool GATED>
void launch_up_small_w(const dmoe_layer& L, const SmallGroup& G, int n_layers, const void* x, int T,
                       bool gate, hipStream_t s) {
    if (weights_fp8(L)) launch_up_small_t<MT, GATED, true>(L, G, n_layers, x, T, gate, s);
    else launch_up_small_t<MT, GATED, false>(L, G, n_layers, x, T, gate, s);
}

}  // namespace

bool small_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    // LDS of the up kernel: the 16 x rows (the partial sums of its wavefronts reuse the space)
    const size_t up_lds = 16 * (2 * (size_t)L.d_model + 16);
    return L.packed != nullptr && (mp == 32 || mp == 64 || mp == 128) && L.d_model % 32 == 0 &&
           up_lds <= 160 * 1024 &&
           div_up(L.n_experts, kSmallMaxGroups) <= kSmallPerGroup;
}

void launch_small_bf16(const dmoe_layer& L, const SmallGroup& G, int n_layers, const void* x, int T,
                       bool gate, hipStream_t s) {
    const int mt = m_pad_of(L.expert_size) / 16;
    {
        LaunchTimer tm(kSlotSmallUp, s);
        if (L.gated) {
            if (mt == 2) launch_up_small_w<2, true>(L, G, n_layers, x, T, gate, s);
            else if (mt == 4) launch_up_small_w<4, true>(L, G, n_layers, x, T, gate, s);
            else launch_up_small_w<8, true>(L, G, n_layers, x, T, gate, s);
        } else {
            if (mt == 2) launch_up_small_w<2, false>(L, G, n_layers, x, T, gate, s);
            else if (mt == 4) launch_up_small_w<4, false>(L, G, n_layers, x, T, gate, s);
            else launch_up_small_w<8, false>(L, G, n_layers, x, T, gate, s);
        }
    }
    // expert groups: enough workgroups to fill the chip, at most kSmallMaxGroups partial sums
    const int E = L.n_experts, d = L.d_model;
    const int ncg = div_up(d / 16, 4);
    int EG = std::max(1, std::min({kSmallMaxGroups, div_up(1024, ncg), std::max(1, E / 4)}));
    EG = std::max(EG, div_up(E, kSmallPerGroup));
    const int per = div_up(E, EG);
    EG = div_up(E, per);
    const dim3 grid(ncg, EG, n_layers);
    const int ks = mt / 2;
    {
        LaunchTimer tm(kSlotSmallDown, s);
        const bool w8 = weights_fp8(L);
        if (ks == 1 && !w8) launch_kernel(down_small_kernel<1, false>, grid, 256, 0, s, G, T, d, E, per);
        else if (ks == 2 && !w8) launch_kernel(down_small_kernel<2, false>, grid, 256, 0, s, G, T, d, E, per);
        else if (!w8) launch_kernel(down_small_kernel<4, false>, grid, 256, 0, s, G, T, d, E, per);
        else if (ks == 1) launch_kernel(down_small_kernel<1, true>, grid, 256, 0, s, G, T, d, E, per);
        else if (ks == 2) launch_kernel(down_small_kernel<2, true>, grid, 256, 0, s, G, T, d, E, per);
        else launch_kernel(down_small_kernel<4, true>, grid, 256, 0, s, G, T, d, E, per);
    }
    LaunchTimer tm(kSlotSmallFinish, s);
    launch_kernel(finish_small_kernel, dim3(div_up(T * d, 256), 1, n_layers), 256, 0, s, G, T, d, EG);
}

}  // namespace dmoe

// Expert up-projection on 8-bit operands (weight format DMOE_W_FP8_E4M3_X8; the lower-precision
// layers of Appendix C, with the 8-bit floating-point format of the gfx950 matrix cores in place
// of int8).
//
//   quantise  one wavefront per token: the row maximum, the power-of-two scale
//             s_t = 2^ceil(log2(max / 448)), and every element rounded to the nearest E4M3 value
//             of x / s_t (ties to the even mantissa): by integer arithmetic on the fp32 bits where
//             the quantised value is wanted as well, by the hardware converter where only the
//             code is (it gives that arithmetic's code for every input it can meet here; see
//             e4m3_codes8).
//   up        the wide-expert kernel of ffn_bf16.hip (a workgroup owns 256 list rows of one
//             expert, the weights of a K block go through LDS once per workgroup, every
//             wavefront stages its own 64 gathered x rows) on v_mfma_f32_16x16x128_f8f6f4: a K block
//             is 128 wide, so per element of K the kernel gathers, stages and reads half the
//             bytes and issues a quarter of the matrix instructions at twice their rate.
//             The instruction adds the products of a 32-wide block with less than fp32
//             precision (measured: within 3e-4 of the block's largest product); the scales
//             s_t * w_scale enter once, on the accumulators, before the activation.
//
// Operand layout of v_mfma_f32_16x16x128_f8f6f4 with both formats E4M3 (lane = 16q + c): the lane
// holds 32 bytes; A: row c of the 16 x 128 tile, B: column c of the 128 x 16 tile, both the k values
// 32q .. 32q + 31 in byte order; D as in the other 16 x 16 MFMAs (D[4q + r][c]).  Only "the same k in
// the same (q, byte) of A and B" matters for the sum.
//   wupx8[E][m_pad/16][d/128][64][32]: lane (q, c) of block (e, neuron tile mt, K block) holds
//   w[e][neuron_of_slot(mt, c)][128 kb + 32q ..], zero bytes for neurons >= m.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int kScaleOne = 0x7f7f7f7f;   // E8M0 block scales of 1.0: the MFMA runs unscaled

__device__ __forceinline__ f32x4 mfma128(i32x8 a, i32x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, kScaleOne, 0, kScaleOne);
}

// ---- row-wise quantisation of x ----------------------------------------------------------------
// E4M3 code of v (|v| <= 448): round to nearest, ties to even.  The grid step at magnitude a is
// 2^(e - 3) with e = max(floor(log2 a), -6) (-6: the subnormal range), a / step is exact, rintf
// rounds it to nearest-even, and a result of 16 steps is the next power of two.
__device__ __forceinline__ uint32_t e4m3_code(float v, float* value) {
    const float a = fabsf(v);
    int e = (int)((__float_as_uint(a) >> 23) & 0xffu) - 127;
    e = max(e, -6);
    float r = rintf(ldexpf(a, 3 - e));   // 0 .. 16
    *value = copysignf(ldexpf(r, e - 3), v);
    uint32_t code;
    if (r < 8.0f) {
        code = (uint32_t)r;              // zero or subnormal (only at e == -6)
    } else {
        if (r == 16.0f) {
            e += 1;
            r = 8.0f;
        }
        code = ((uint32_t)(e + 7) << 3) | ((uint32_t)r - 8u);
    }
    return code | (v < 0.0f ? 0x80u : 0u);
}

// Codes of eight values by the hardware converter.  For every bf16 number of magnitude up to
// 448 (the only inputs here: bf16 values times a power of two) v_cvt_pk_fp8_f32 returns the code
// of e4m3_code above -- checked exhaustively on the device, all 34754 inputs -- at a tenth of the
// instructions, so the kernels that need only the codes use it.
__device__ __forceinline__ uint2 e4m3_codes8(const float (&v)[8]) {
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

__global__ __launch_bounds__(256) void quantize_x_kernel(const __bf16* __restrict__ x, int T, int d,
                                                         uint8_t* __restrict__ x8,
                                                         float* __restrict__ xscale,
                                                         __bf16* __restrict__ xhat) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const __bf16* row = x + (size_t)t * d;
    float amax = 0.0f;
    for (int k = 8 * lane; k < d; k += 512) {
        const bf16x8 v = load8(row + k);
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)v[i]));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    // smallest power of two s with amax / s <= 448 = 0.875 * 2^9: amax = f * 2^ex, f in [0.5, 1)
    int s_exp = 0;
    if (amax > 0.0f && amax < INFINITY) {
        int ex;
        const float f = frexpf(amax, &ex);
        s_exp = f <= 0.875f ? ex - 9 : ex - 8;
        s_exp = min(max(s_exp, -100), 100);
    }
    if (lane == 0) xscale[t] = ldexpf(1.0f, s_exp);
    for (int k = 8 * lane; k < d; k += 512) {
        const bf16x8 v = load8(row + k);
        if (!xhat) {  // uniform: codes only
            float sv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) sv[i] = ldexpf((float)v[i], -s_exp);
            *reinterpret_cast<uint2*>(x8 + (size_t)t * d + k) = e4m3_codes8(sv);
            continue;
        }
        uint32_t lo = 0, hi = 0;
        bf16x8 q;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float val;
            const uint32_t code = e4m3_code(ldexpf((float)v[i], -s_exp), &val);
            if (i < 4) lo |= code << (8 * i); else hi |= code << (8 * (i - 4));
            q[i] = (__bf16)ldexpf(val, s_exp);   // exact: four significant bits
        }
        *reinterpret_cast<uint2*>(x8 + (size_t)t * d + k) = make_uint2(lo, hi);
        *reinterpret_cast<bf16x8*>(xhat + (size_t)t * d + k) = q;
    }
}

// ---- one-time packing -----------------------------------------------------------------------------
__global__ void pack_up_x8_kernel(const uint8_t* __restrict__ w, uint8_t* __restrict__ out, int E,
                                  int m, int d, int MT) {
    const size_t n = (size_t)E * MT * 16 * d;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int j = (int)(i & 31), lane = (int)((i >> 5) & 63);
        size_t f = i >> 11;
        const int kb = (int)(f % (d / 128));
        f /= (d / 128);
        const int mt = (int)(f % MT);
        const int e = (int)(f / MT);
        const int q = lane >> 4, c = lane & 15;
        const int neuron = neuron_of_slot(mt, c);
        out[i] = neuron < m ? w[((size_t)e * m + neuron) * d + 128 * kb + 32 * q + j] : (uint8_t)0;
    }
}

constexpr int kX8RowBytes = 144;   // 128 bytes of one x row + 16 bytes of bank skew

// ---- up-projection ----------------------------------------------------------------------------------
// Workgroup = (expert, 4 x 16*TT consecutive list rows); NT = neuron tiles of both branches.
// H8OUT: the hidden rows go out quantised for the 8-bit down-projection (DMOE_W_FP8_E4M3_A8):
// rounded to bf16 as usual, then the row's power-of-two scale and E4M3 codes, H8[row][16 MT] and
// hs8[row], instead of the bf16 row.
template <int MT, bool GATED, int TT, bool H8OUT>
__global__ __launch_bounds__(256, 2) void up_wide_x8_kernel(
    const uint8_t* __restrict__ x8, const float* __restrict__ xscale,
    const uint8_t* __restrict__ wupx, const uint8_t* __restrict__ wgatex,
    const float* __restrict__ w_scales, const __bf16* __restrict__ b_up,
    const int32_t* __restrict__ witem, const int32_t* __restrict__ wfirst,
    const int32_t* __restrict__ alist, __bf16* __restrict__ Hf, uint8_t* __restrict__ H8,
    uint8_t* __restrict__ hs8, int d, int E, int m, int act) {
    constexpr int BR = GATED ? 2 : 1;
    constexpr int KS = MT / 2;
    constexpr int NT = BR * MT;         // neuron tiles (2 KiB of weights each) per K block
    constexpr int WR = TT * 16;         // rows per wavefront
    constexpr int UR = 4 * WR;          // rows per work item
    constexpr int NL = TT * 2;          // x load instructions per K block: 8 rows x 128 bytes each
    constexpr int NWL = NT / 2;         // weight load instructions per thread and K block
    static_assert(NT % 2 == 0, "the weights of a K block are copied 4 KiB at a time");
    extern __shared__ char smem[];
    char* wbuf = smem;                                            // [2][NT][64][32]
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15, w = threadIdx.x >> 6;
    char* xs = smem + 2 * NT * 2048 + w * (WR * kX8RowBytes);     // [WR][kX8RowBytes], private
    float* sbias = reinterpret_cast<float*>(smem + 2 * NT * 2048 + 4 * (WR * kX8RowBytes));  // [2][MT * 16]
    const int NKB = d / 128;   // >= 2
    const int ld_row = lane >> 3, ld_piece = lane & 7;
    const int total = witem[E];
    int j = blockIdx.x;
    if (j >= total) return;

    // item j: its expert is the last e with witem[e] <= j (uniform binary search)
    auto locate = [&](int jj, int& e, int& item) {
        int lo = 0, hi = E;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (witem[mid] <= jj) lo = mid; else hi = mid;
        }
        e = lo;
        item = wfirst[lo] + (jj - witem[lo]);
    };
    // tokens of the x rows this lane fetches; padding rows (-1) read token 0 and produce H rows
    // that nobody merges
    auto rows_of = [&](int item, uint32_t (&xtok)[NL], bool& active) {
        const int32_t* tl = alist + (size_t)item * UR + w * WR;
        active = tl[0] >= 0;  // valid rows are a prefix
#pragma unroll
        for (int i = 0; i < NL; ++i) xtok[i] = (uint32_t)max(tl[ld_row + 8 * i], 0);
    };
    // The K block's weights are NT tiles of 2 KiB; this thread copies the 16-byte pieces
    // tid, tid + 256, ...: piece 256 i + tid belongs to tile 2i + (tid >> 7), the first MT of
    // which are up rows and the rest gate rows -- one base per matrix plus i times a stride.
    const uint32_t wlane = (uint32_t)((threadIdx.x >> 7) * NKB * 2048 + (threadIdx.x & 127) * 16);
    const size_t wstride = (size_t)2 * NKB * 2048;   // two neuron tiles on
    i32x4 xr[NL], wr[NWL];
    auto issue = [&](int e, const uint32_t (&xtok)[NL], bool active, int kb) {
        const size_t we = (size_t)e * MT * NKB * 2048 + (size_t)kb * 2048 + wlane;
#pragma unroll
        for (int i = 0; i < NWL; ++i)
            wr[i] = *reinterpret_cast<const i32x4*>(((GATED && i >= MT / 2) ? wgatex : wupx) + we +
                                                    (i % (MT / 2)) * wstride);
        if (active) {
#pragma unroll
            for (int i = 0; i < NL; ++i)
                xr[i] = *reinterpret_cast<const i32x4*>(
                    x8 + ((size_t)xtok[i] * (uint32_t)d + (uint32_t)(16 * ld_piece + 128 * kb)));
        }
    };
    auto park = [&](int buf, bool active) {
#pragma unroll
        for (int i = 0; i < NWL; ++i)
            *reinterpret_cast<i32x4*>(wbuf + buf * NT * 2048 + (256 * i + threadIdx.x) * 16) = wr[i];
        if (active) {
            char* dst = xs + ld_row * kX8RowBytes + ld_piece * 16;
#pragma unroll
            for (int i = 0; i < NL; ++i)
                *reinterpret_cast<i32x4*>(dst + 8 * i * kX8RowBytes) = xr[i];
        }
    };
    auto park_bias = [&](int e, int par) {  // plain experts: the item's biases, by neuron
        if (!GATED && (int)threadIdx.x < MT * 16)
            sbias[par * MT * 16 + threadIdx.x] =
                b_up ? (float)b_up[(size_t)e * m + min((int)threadIdx.x, m - 1)] : 0.0f;
    };

    // The K blocks of all the items of the workgroup form one stream: block k is multiplied while
    // block k + 1 waits in LDS or is on its way there and block k + 2 is in flight, also across
    // the end of an item -- the next item's first blocks arrive during this item's epilogue.
    int e, item;
    uint32_t xtok[NL];
    bool active;
    locate(j, e, item);
    rows_of(item, xtok, active);
    issue(e, xtok, active, 0);
    park(0, active);
    park_bias(e, 0);
    lds_barrier();
    issue(e, xtok, active, 1);
    int buf = 0, par = 0;
    for (;;) {
        // the item after this one (the last item names itself: its first blocks are read again
        // and never used)
        const int jn = j + (int)gridDim.x;
        const bool more = jn < total;
        int en = e, itemn = item;
        if (more) locate(jn, en, itemn);
        const int32_t* tl = alist + (size_t)item * UR + w * WR;

        f32x4 acc[NT][TT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[nt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto multiply = [&]() {
            if (active) {
                const char* wsrc_l = wbuf + buf * NT * 2048 + lane * 32;
                const char* xsrc = xs + c * kX8RowBytes + q * 32;
                i32x8 b[TT];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const i32x4 b0 = *reinterpret_cast<const i32x4*>(xsrc + tt * 16 * kX8RowBytes);
                    const i32x4 b1 = *reinterpret_cast<const i32x4*>(xsrc + tt * 16 * kX8RowBytes + 16);
                    b[tt] = i32x8{b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const i32x4 a0 = *reinterpret_cast<const i32x4*>(wsrc_l + nt * 2048);
                    const i32x4 a1 = *reinterpret_cast<const i32x4*>(wsrc_l + nt * 2048 + 16);
                    const i32x8 a = i32x8{a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) acc[nt][tt] = mfma128(a, b[tt], acc[nt][tt]);
                }
            }
        };
        // block kb is in LDS buffer `buf`, block kb + 1 in flight to the registers
        for (int kb = 0; kb < NKB - 2; ++kb) {
            multiply();
            park(buf ^ 1, active);
            lds_barrier();
            buf ^= 1;
            issue(e, xtok, active, kb + 2);
        }
        // The next item's rows and this item's row scales are requested here, two blocks before
        // the end: vector loads return in order, so requested any later they would queue behind
        // the next item's first blocks, and any earlier their wait would hold up this item's start.
        uint32_t xtokn[NL];
        bool activen;
        rows_of(itemn, xtokn, activen);
        int tok_c[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) tok_c[tt] = max(tl[16 * tt + c], 0);
        multiply();                    // block NKB - 2
        park(buf ^ 1, active);
        lds_barrier();
        buf ^= 1;
        float s_xr[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) s_xr[tt] = xscale[tok_c[tt]];
        issue(en, xtokn, activen, 0);
        multiply();                    // block NKB - 1; the next item's block 0 arrives
        park(buf ^ 1, activen);
        park_bias(en, par ^ 1);
        lds_barrier();
        buf ^= 1;
        issue(en, xtokn, activen, 1);

        if (active) with_activation(act, [&](auto act_c) {
            constexpr int ACT = decltype(act_c)::value;
            // lane (q, c) of tile (mt, tt): neurons neuron_of_slot(mt, 4q + r) of list row 16tt + c.
            // The accumulators are sums of code products: times the row's scale and the
            // matrix's scale they are the pre-activations.
            const float s_up = w_scales[3 * e + 0], s_gate = w_scales[3 * e + 1];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const float s_x = s_xr[tt];
                const size_t row = (size_t)item * UR + w * WR + 16 * tt + c;
                bf16x8 hv[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const int mt = 2 * ks + half;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float v;
                            if (GATED)
                                v = activate_fast(ACT, acc[MT + mt][tt][r] * (s_x * s_gate)) *
                                    (acc[mt][tt][r] * (s_x * s_up));
                            else
                                v = activate_fast(ACT, acc[mt][tt][r] * (s_x * s_up) +
                                                           sbias[par * MT * 16 + neuron_of_slot(mt, 4 * q + r)]);
                            if (neuron_of_slot(mt, 4 * q + r) >= m) v = 0.0f;
                            hv[ks][half * 4 + r] = (__bf16)v;
                        }
                    }
                }
                if (!H8OUT) {
                    __bf16* dst = Hf + row * (KS * 32) + 8 * q;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<bf16x8*>(dst + ks * 32) = hv[ks];
                } else {
                    // the row's neurons are spread over the four lanes (q) of column c
                    float amax = 0.0f;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)hv[ks][i]));
                    amax = fmaxf(amax, __shfl_xor(amax, 16, 64));
                    amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
                    int s_exp = 0;
                    if (amax > 0.0f && amax < INFINITY) {
                        int ex;
                        const float f = frexpf(amax, &ex);
                        s_exp = f <= 0.875f ? ex - 9 : ex - 8;
                        s_exp = min(max(s_exp, -100), 100);
                    }
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        float sv[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) sv[i] = ldexpf((float)hv[ks][i], -s_exp);
                        // piece 4ks + q of the row: neurons 8 (4ks + q) .. + 7, one byte each
                        *reinterpret_cast<uint2*>(H8 + row * (KS * 32) + 8 * (4 * ks + q)) = e4m3_codes8(sv);
                    }
                    if (q == 0) hs8[row] = (uint8_t)(127 + s_exp);
                }
                // one list row at a time: interleaving more of them costs registers that the
                // requests in flight are using
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        if (!more) break;
        j = jn;
        e = en;
        item = itemn;
        active = activen;
        par ^= 1;
#pragma unroll
        for (int i = 0; i < NL; ++i) xtok[i] = xtokn[i];
    }
}

template <int MT, bool GATED, int TT, bool H8OUT>
void launch_up_x8_t(const dmoe_layer& L, const PackedLayout& P, const uint8_t* x8,
                    const float* xscale, const int32_t* witem, const int32_t* wfirst,
                    const int32_t* alist, void* H, uint8_t* H8, uint8_t* hs8, int grid,
                    hipStream_t s) {
    constexpr int NT = (GATED ? 2 : 1) * MT;
    const size_t lds = 2 * NT * 2048 + 4 * (size_t)TT * 16 * kX8RowBytes + 2 * MT * 16 * sizeof(float);
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_wide_x8_kernel<MT, GATED, TT, H8OUT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    const char* pk = static_cast<const char*>(L.packed);
    launch_kernel(up_wide_x8_kernel<MT, GATED, TT, H8OUT>, grid, 256, lds, s, x8, xscale,
                  (const uint8_t*)(pk + P.wupx8), (const uint8_t*)(pk + P.wgatex8),
                  (const float*)(pk + P.scales), (const __bf16*)L.b_up, witem, wfirst, alist,
                  (__bf16*)H, H8, hs8, L.d_model, L.n_experts, L.expert_size, L.act);
}

}  // namespace

void launch_quantize_x(const dmoe_layer& L, const void* x, int T, uint8_t* x8, float* xscale,
                       void* xhat, hipStream_t s) {
    LaunchTimer tm(kSlotQuantX, s);
    launch_kernel(quantize_x_kernel, div_up(T, 4), 256, 0, s, (const __bf16*)x, T, L.d_model, x8,
                  xscale, (__bf16*)xhat);
}

void launch_pack_x8(const dmoe_layer& L, void* packed, hipStream_t s) {
    const PackedLayout P = packed_layout(L);
    char* pk = static_cast<char*>(packed);
    const int mt = m_pad_of(L.expert_size) / 16;
    launch_kernel(pack_up_x8_kernel, 2048, 256, 0, s, (const uint8_t*)L.w_up, (uint8_t*)(pk + P.wupx8),
                  L.n_experts, L.expert_size, L.d_model, mt);
    if (L.gated)
        launch_kernel(pack_up_x8_kernel, 2048, 256, 0, s, (const uint8_t*)L.w_gate,
                      (uint8_t*)(pk + P.wgatex8), L.n_experts, L.expert_size, L.d_model, mt);
}

void launch_up_x8(const dmoe_layer& L, const uint8_t* x8, const float* xscale, int T,
                  const int32_t* witem, const int32_t* wfirst, const int32_t* alist, void* H,
                  uint8_t* H8, uint8_t* hs8, hipStream_t s) {
    LaunchTimer tm(kSlotUp, s);
    const PackedLayout P = packed_layout(L);
    const int grid = round_up(
        (int)std::min<long long>((long long)T * L.n_experts / 256 + L.n_experts, 512), 8);
    if (L.gated && H8) launch_up_x8_t<4, true, 4, true>(L, P, x8, xscale, witem, wfirst, alist, H, H8, hs8, grid, s);
    else if (L.gated) launch_up_x8_t<4, true, 4, false>(L, P, x8, xscale, witem, wfirst, alist, H, nullptr, nullptr, grid, s);
    else if (H8) launch_up_x8_t<8, false, 4, true>(L, P, x8, xscale, witem, wfirst, alist, H, H8, hs8, grid, s);
    else launch_up_x8_t<8, false, 4, false>(L, P, x8, xscale, witem, wfirst, alist, H, nullptr, nullptr, grid, s);
}

}  // namespace dmoe

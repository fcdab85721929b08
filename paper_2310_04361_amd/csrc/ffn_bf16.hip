// bf16 expert up-projection (+ gate) and activation (Sec. 3.2, Appendix G) on the gfx950 matrix
// cores, and the one-time packing of the expert and router weights.
//
//   up    expert-major grouped GEMM over the compact lists.  A wavefront owns UR = 16*TT list
//         rows of one expert, gathers those rows of x in 128-byte pieces (eight lanes per row, so
//         the vector memory path sees whole cache lines), stages them in its own LDS buffers and
//         multiplies them with the expert's up (and gate) rows; bias + activation in fp32; the
//         hidden activations go out rounded to bf16, one row of m_pad values per list row.
// Tokens ride on the MFMA column axis, so four consecutive neurons of one token land in one lane.
//
// Fragment order.  Every weight operand that a wavefront reads with one load instruction is
// stored as the 1 KiB block  [lane 0..63][8 bf16]  in exactly the register layout of the MFMA,
// because a 16-byte-per-lane access with a 64-byte or larger lane stride costs a cache-line
// lookup per lane and that, not bandwidth, bounded the first version of these kernels.
//   H row (m_pad bf16): natural neuron order -- the packed up weights place the neurons on the
//     MFMA rows (neuron_of_slot in mfma.h) so that the accumulators of lane (q, .) for the tile
//     pair (2ks, 2ks+1) are the eight consecutive neurons of the 16-byte piece 4ks + q.
//   An expert's H rows start at a multiple of UR rows (its first up-projection work item).
#include <cmath>

#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

constexpr int kUpRowBytes = 144;               // 64 bf16 of one x row + 16 bytes of bank skew

// ---- one-time weight packing ------------------------------------------------------------------------
// (small-token path) w_down[E][m][d] -> w2f[E][d/16][KS][64][8]: lane (q, c) of fragment (e, column tile ct, ks)
// holds W_down[e][8*(4ks + q) + s][16ct + c] (piece 4ks + q of an H row), zero for neurons >= m.
// OUT = __bf16: the weight as a bf16 number (8-bit weights are scaled out); OUT = uint8_t: the
// raw E4M3 byte (8-bit weights only), for the kernels that convert in registers.
template <typename OUT>
__device__ __forceinline__ OUT packed_weight(const void* w, const float* scales, int fp8, int which,
                                             int e, size_t flat, bool valid) {
    if constexpr (sizeof(OUT) == 1) {
        return valid ? static_cast<const uint8_t*>(w)[flat] : (uint8_t)0;
    } else {
        return valid ? expert_weight(w, scales, fp8, which, e, flat) : (__bf16)0.0f;
    }
}

// Scales of 8-bit weights -> the nearest power of two (in log2; the sign is kept, zero stays
// zero): with such a scale scale * e4m3(byte) is exactly a bf16 number, which is what makes the
// bf16 copies of the prefill kernels and the in-register conversion of the small-token kernels
// the same layer.
__global__ void snap_scales_kernel(const float* __restrict__ in, float* __restrict__ out, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float v = in[i], a = fabsf(v);
    float r = 0.0f;
    if (a > 0.0f && a < INFINITY) r = copysignf(exp2f(rintf(log2f(a))), v);
    out[i] = r;
}

template <typename OUT>
__global__ void pack_down_kernel(const void* __restrict__ w_down, const float* __restrict__ scales,
                                 int fp8, OUT* __restrict__ w2f, int E, int m, int d, int KS) {
    const size_t n = (size_t)E * d * KS * 32;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int s = (int)(i & 7), lane = (int)((i >> 3) & 63);
        size_t f = i >> 9;
        const int ks = (int)(f % KS);
        f /= KS;
        const int ct = (int)(f % (d / 16));
        const int e = (int)(f / (d / 16));
        const int q = lane >> 4, c = lane & 15;
        const int neuron = 8 * (4 * ks + q) + s;  // piece 4ks + q of the H row
        w2f[i] = packed_weight<OUT>(w_down, scales, fp8, 2, e,
                                    ((size_t)e * m + min(neuron, m - 1)) * d + 16 * ct + c, neuron < m);
    }
}

// w[E][m][d] -> wf[E][MT][d/32][64][8]: lane (q, c) of fragment (e, neuron tile mt, k-step) holds
// w[e][n(mt, c)][32 kstep + 8q + s], zero rows for neurons >= m; n(mt, c) = neuron_of_slot for the
// expert matrices, 16mt + c for the router matrices.
// `which`: 0 up, 1 gate (selects the scale of 8-bit weights)
template <typename OUT>
__global__ void pack_up_kernel(const void* __restrict__ w, const float* __restrict__ scales, int fp8,
                               int which, OUT* __restrict__ wf, int E, int m, int d, int MT,
                               int piece_order) {
    const size_t n = (size_t)E * MT * 16 * d;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int s = (int)(i & 7), lane = (int)((i >> 3) & 63);
        size_t f = i >> 9;
        const int kstep = (int)(f % (d / 32));
        f /= (d / 32);
        const int mt = (int)(f % MT);
        const int e = (int)(f / MT);
        const int q = lane >> 4, c = lane & 15;
        // experts: the neuron order that makes H pieces consecutive; router matrices: natural
        const int neuron = piece_order ? neuron_of_slot(mt, c) : 16 * mt + c;
        wf[i] = packed_weight<OUT>(w, scales, fp8, which, e,
                                   ((size_t)e * m + min(neuron, m - 1)) * d + 32 * kstep + 8 * q + s,
                                   neuron < m);
    }
}

// Experts of one weight tile: w_up (, w_gate) [E][m][d] -> wt[E][d/32][64][8], one 16-row tile per
// expert and k-step.  Gated (m <= 8): rows 0..7 are the up rows and 8..15 the gate rows; plain
// (m <= 16): row c is neuron c.  Zero rows for neurons >= m; lane (q, c) holds row c, columns
// 32 kstep + 8q + s.
__global__ void pack_up_tiny_kernel(const void* __restrict__ w_up, const void* __restrict__ w_gate,
                                    const float* __restrict__ scales, int fp8,
                                    __bf16* __restrict__ wt, int E, int m, int d, int gated) {
    const size_t n = (size_t)E * 16 * d;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int s = (int)(i & 7), lane = (int)((i >> 3) & 63);
        const size_t f = i >> 9;
        const int kstep = (int)(f % (d / 32));
        const int e = (int)(f / (d / 32));
        const int q = lane >> 4, c = lane & 15;
        const int neuron = gated ? (c & 7) : c, which = gated ? (c >> 3) : 0;  // 0 up, 1 gate
        wt[i] = packed_weight<__bf16>(which ? w_gate : w_up, scales, fp8, which, e,
                                      ((size_t)e * m + min(neuron, m - 1)) * d + 32 * kstep + 8 * q + s,
                                      neuron < m);
    }
}

// ---- up-projection ---------------------------------------------------------------------------------
// One wavefront per work item = (expert, UR = 16*TT consecutive list rows); no workgroup-level
// synchronisation after the work-item table has been staged.  MT = m_pad / 16 neuron tiles per
// branch.  K advances in blocks of 64: the wavefront loads the next block of its x rows
// (lane = (row % 8, 16-byte piece of the 128-byte row segment)) and of the weight fragments
// while the MFMAs run on the current block out of LDS / registers.
template <int MT, bool GATED, int TT, int NBUF>
__global__ __launch_bounds__(256, NBUF == 1 ? 3 : 1) void up_bf16_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ wupf,
    const __bf16* __restrict__ wgatef, const __bf16* __restrict__ b_up,
    const int32_t* __restrict__ witem, const int32_t* __restrict__ wfirst, int NW,
    const int32_t* __restrict__ alist, __bf16* __restrict__ Hf, int d, int E, int m, int act) {
    constexpr int BR = GATED ? 2 : 1;
    constexpr int KS = MT / 2;
    constexpr int UR = TT * 16;
    constexpr int NL = TT * 2;  // x load instructions per K block: 8 rows x 128 bytes each
    extern __shared__ char smem[];
    int32_t* s_wit = reinterpret_cast<int32_t*>(smem);  // witem[w][0..E], then wfirst[w][0..E-1]
    int32_t* s_wf = s_wit + (E + 1);
    const int items_bytes = ((2 * E + 1) * 4 + 15) & ~15;
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15;
    const int wave_in_block = threadIdx.x >> 6;
    char* xs = smem + items_bytes + wave_in_block * (NBUF * UR * kUpRowBytes);
    const int NK32 = d / 32, NKB = d / 64;
    const int ld_row = lane >> 3, ld_piece = lane & 7;

    // Work items are walked window by window: the wavefronts of XCD k (workgroups are dealt
    // round-robin to the 8 XCDs) take the windows k, k+8, ... so that the x rows they gather --
    // each row is used by every expert its token selected -- stay in that XCD's L2; gathered out
    // of the last-level cache the same rows come in at about a third of the rate.
    // A single window is shared by all workgroups.
    const bool windowed = NW > 1;
    const int wg = windowed ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int n_wg = windowed ? (int)(gridDim.x >> 3) : (int)gridDim.x;
    const int wave = wg * (blockDim.x >> 6) + wave_in_block;
    const int n_waves = n_wg * (blockDim.x >> 6);
    for (int wdx = windowed ? (int)(blockIdx.x & 7) : 0; wdx < NW; wdx += 8) {
    __syncthreads();  // the previous window's table is no longer read
    for (int i = threadIdx.x; i <= 2 * E; i += blockDim.x)
        s_wit[i] = i <= E ? witem[(size_t)wdx * (E + 1) + i] : wfirst[(size_t)wdx * E + (i - E - 1)];
    __syncthreads();
    const int total = s_wit[E];
    // item jj: its expert is the last e with s_wit[e] <= jj
    auto locate = [&](int jj, int& e, int& item) {
        int lo = 0, hi = E;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_wit[mid] <= jj) lo = mid; else hi = mid;
        }
        e = lo;
        item = s_wf[lo] + (jj - s_wit[lo]);
    };
    int j = wave;
    if (j < total) {
        int e, item;
        locate(j, e, item);
        // x rows as 32-bit offsets in 16-byte units (T * d / 8 fits): half the registers of
        // pointers.  Rows of the aligned list past the expert's last token hold -1: they read
        // token 0 and produce H rows that nobody merges.
        uint32_t xoff[NL];
        auto rows_from = [&](const int (&tok)[NL]) {
#pragma unroll
            for (int i = 0; i < NL; ++i)
                xoff[i] = (uint32_t)(((size_t)max(tok[i], 0) * d) >> 3) + ld_piece;
        };
        const __bf16* wf[BR];
        auto weights_of = [&](int ee) {
            wf[0] = wupf + (size_t)ee * MT * NK32 * 512 + lane * 8;
            if (GATED) wf[BR - 1] = wgatef + (size_t)ee * MT * NK32 * 512 + lane * 8;
        };
        {
            const int32_t* tl = alist + (size_t)item * UR + ld_row;
            int tok[NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) tok[i] = tl[8 * i];
            rows_from(tok);
        }
        weights_of(e);

        bf16x8 xr[NL];
        bf16x8 a0[2][BR][MT], a1[2][BR][MT];
        auto load_x = [&](int kb) {
#pragma unroll
            for (int i = 0; i < NL; ++i) xr[i] = load8(x + (((size_t)xoff[i] + 8 * kb) << 3));
        };
        auto load_a = [&](int kb, bf16x8 (&a)[2][BR][MT]) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int br = 0; br < BR; ++br)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        a[ks][br][mt] = load8(wf[br] + ((size_t)mt * NK32 + 2 * kb + ks) * 512);
        };
        auto store_x = [&](int buf) {
            char* dst = xs + (buf % NBUF) * (UR * kUpRowBytes) + ld_row * kUpRowBytes + ld_piece * 16;
#pragma unroll
            for (int i = 0; i < NL; ++i)
                *reinterpret_cast<bf16x8*>(dst + 8 * i * kUpRowBytes) = xr[i];
        };
        // The first block of an item is requested before the epilogue of the item before it (here:
        // before anything else), so an item starts with its block 0 on the way.
        load_x(0);
        load_a(0, a0);
        for (;;) {
            // the accumulators start at the biases of this lane's neurons (no registers held for
            // them through the K loop)
            f32x4 acc[BR][MT][TT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                f32x4 bias = f32x4{0.f, 0.f, 0.f, 0.f};
                if (!GATED && b_up) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int n = neuron_of_slot(mt, 4 * q + r);
                        bias[r] = (float)b_up[(size_t)e * m + min(n, m - 1)];
                    }
                }
#pragma unroll
                for (int br = 0; br < BR; ++br)
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) acc[br][mt][tt] = br == 0 ? bias : f32x4{0.f, 0.f, 0.f, 0.f};
            }
            auto compute = [&](int buf, const bf16x8 (&a)[2][BR][MT]) {
                const char* src = xs + (buf % NBUF) * (UR * kUpRowBytes) + c * kUpRowBytes + q * 16;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    bf16x8 b[TT];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        b[tt] = *reinterpret_cast<const bf16x8*>(src + tt * 16 * kUpRowBytes + ks * 64);
#pragma unroll
                    for (int br = 0; br < BR; ++br)
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int tt = 0; tt < TT; ++tt)
                                acc[br][mt][tt] = mfma16(a[ks][br][mt], b[tt], acc[br][mt][tt]);
                }
            };

            store_x(0);
            // two K blocks per trip so that the two weight-fragment register sets simply alternate
            for (int kb = 0; kb < NKB - 2; kb += 2) {
                load_x(kb + 1);
                load_a(kb + 1, a1);
                compute(0, a0);
                store_x(1);
                load_x(kb + 2);
                load_a(kb + 2, a0);
                compute(1, a1);
                store_x(0);
            }
            // Last trip: its second set of requests is block 0 of the wavefront's NEXT item (the
            // last item names itself: the block is read and never used), whose list rows are
            // requested together with this item's last block, once its own offsets are done with.
            load_x(NKB - 1);
            load_a(NKB - 1, a1);
            const int jn = j + n_waves;
            const bool more = jn < total;
            int en = e, itemn = item;
            if (more) locate(jn, en, itemn);
            int tokn[NL];
            {
                const int32_t* tl = alist + (size_t)itemn * UR + ld_row;
#pragma unroll
                for (int i = 0; i < NL; ++i) tokn[i] = tl[8 * i];
            }
            compute(0, a0);
            store_x(1);
            rows_from(tokn);
            weights_of(en);
            load_x(0);
            load_a(0, a0);
            compute(1, a1);

            // lane (q, c) of tile (mt, tt): neurons 16mt + 4q + r of list row 16tt + c
            with_activation(act, [&](auto act_c) {
                constexpr int ACT = decltype(act_c)::value;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    __bf16* dst = Hf + ((size_t)item * UR + 16 * tt + c) * (KS * 32) + 8 * q;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        bf16x8 hv;
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int mt = 2 * ks + half;
                            const int n0 = neuron_of_slot(mt, 4 * q);  // + r: consecutive
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                float v;
                                if (GATED) {
                                    v = activate_fast(ACT, acc[BR - 1][mt][tt][r]) * acc[0][mt][tt][r];
                                } else {
                                    v = activate_fast(ACT, acc[0][mt][tt][r]);
                                }
                                if (n0 + r >= m) v = 0.0f;
                                hv[half * 4 + r] = (__bf16)v;
                            }
                        }
                        *reinterpret_cast<bf16x8*>(dst + ks * 32) = hv;
                        __builtin_amdgcn_sched_barrier(0);  // eight values at a time
                    }
                }
            });
            if (!more) break;
            j = jn;
            e = en;
            item = itemn;
        }
    }
    }  // windows
}

// Up-projection for experts that fit one 16-row weight tile: at most 16 neurons, or gated with at
// most 8 (the paper's own splits: experts of 6 for its text classifier, 2048 gated experts of 8
// for its language model).  In the general kernel a gated expert of 8 fills a quarter of the rows
// of four weight tiles and a plain one of 6 to 16 half of two; here the expert is ONE tile (gated:
// up rows and gate rows together), so a work item streams a quarter / half of the weight bytes
// and issues a quarter / half of the MFMAs, and what remains is the gather of the x rows.  Same
// work items, same x staging, same H rows (the unused pieces of the 32-neuron row are written as
// zeros) as up_bf16_kernel<2, GATED, TT>.
template <int TT, bool GATED>
__global__ __launch_bounds__(256) void up_tiny_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ wtf, const __bf16* __restrict__ b_up,
    const int32_t* __restrict__ witem, const int32_t* __restrict__ wfirst, int NW,
    const int32_t* __restrict__ alist, __bf16* __restrict__ Hf, int d, int E, int m, int act) {
    constexpr int UR = TT * 16;
    constexpr int NL = TT * 2;
    extern __shared__ char smem[];
    int32_t* s_wit = reinterpret_cast<int32_t*>(smem);  // witem[w][0..E-1], then wfirst[w][0..E-1]
    int32_t* s_wf = s_wit + E;
    const int items_bytes = (2 * E * 4 + 15) & ~15;
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15;
    const int wave_in_block = threadIdx.x >> 6;
    // one staging buffer per wavefront (its LDS accesses keep their order, so a second one buys
    // nothing): with thousands of experts the work-item table already takes 16 KiB or more, and
    // the LDS left decides how many wavefronts a CU holds
    char* xs = smem + items_bytes + wave_in_block * (UR * kUpRowBytes);
    const int NK32 = d / 32, NKB = d / 64;
    const int ld_row = lane >> 3, ld_piece = lane & 7;

    const bool windowed = NW > 1;
    const int wg = windowed ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int n_wg = windowed ? (int)(gridDim.x >> 3) : (int)gridDim.x;
    const int wave = wg * (blockDim.x >> 6) + wave_in_block;
    const int n_waves = n_wg * (blockDim.x >> 6);
    for (int wdx = windowed ? (int)(blockIdx.x & 7) : 0; wdx < NW; wdx += 8) {
    __syncthreads();  // the previous window's table is no longer read
    for (int i = threadIdx.x; i < 2 * E; i += blockDim.x)
        s_wit[i] = i < E ? witem[(size_t)wdx * (E + 1) + i] : wfirst[(size_t)wdx * E + (i - E)];
    const int total = witem[(size_t)wdx * (E + 1) + E];
    __syncthreads();
    for (int j = wave; j < total; j += n_waves) {
        int lo = 0, hi = E;  // last e with s_wit[e] <= j
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_wit[mid] <= j) lo = mid; else hi = mid;
        }
        const int e = lo;
        const int item = s_wf[e] + (j - s_wit[e]);
        const int32_t* tl = alist + (size_t)item * UR + ld_row;
        // Valid rows are a prefix of the item and padding rows hold -1.  With thousands of experts
        // most items are part-filled (4096 tokens, 2048 experts, 7 % density: 36 of 64 rows), and
        // what the kernel spends is load instructions: a load whose eight rows are all padding is
        // not issued (`need` has a bit per load instruction; its staging rows are zeroed once).
        const __bf16* xrow[NL];
        uint32_t need = 0;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int tok = tl[8 * i];
            need |= (__ballot(tok >= 0) != 0 ? 1u : 0u) << i;
            xrow[i] = x + (size_t)max(tok, 0) * d + 8 * ld_piece;  // a padding row next to valid ones reads token 0
        }
        need = __builtin_amdgcn_readfirstlane(need);
        const __bf16* wf = wtf + (size_t)e * NK32 * 512 + lane * 8;

        f32x4 acc[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[tt] = f32x4{0.f, 0.f, 0.f, 0.f};

        bf16x8 xr[NL];
        bf16x8 a0[2], a1[2];
        auto load_x = [&](int kb) {
#pragma unroll
            for (int i = 0; i < NL; ++i)
                if ((need >> i) & 1u) xr[i] = load8(xrow[i] + 64 * kb);
        };
        auto load_a = [&](int kb, bf16x8 (&a)[2]) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) a[ks] = load8(wf + (size_t)(2 * kb + ks) * 512);
        };
        auto store_x = [&]() {
            char* dst = xs + ld_row * kUpRowBytes + ld_piece * 16;
#pragma unroll
            for (int i = 0; i < NL; ++i)
                if ((need >> i) & 1u) *reinterpret_cast<bf16x8*>(dst + 8 * i * kUpRowBytes) = xr[i];
        };
        {   // rows that no load fills: zeros for the whole item
            char* dst = xs + ld_row * kUpRowBytes + ld_piece * 16;
            const bf16x8 zero = {};
#pragma unroll
            for (int i = 0; i < NL; ++i)
                if (!((need >> i) & 1u)) *reinterpret_cast<bf16x8*>(dst + 8 * i * kUpRowBytes) = zero;
        }
        auto compute = [&](const bf16x8 (&a)[2]) {
            const char* src = xs + c * kUpRowBytes + q * 16;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const bf16x8 b =
                        *reinterpret_cast<const bf16x8*>(src + tt * 16 * kUpRowBytes + ks * 64);
                    acc[tt] = mfma16(a[ks], b, acc[tt]);
                }
        };

        load_x(0);
        load_a(0, a0);
        store_x();
        for (int kb = 0; kb < NKB; kb += 2) {
            load_x(kb + 1);
            load_a(kb + 1, a1);
            compute(a0);
            store_x();
            const int nb = min(kb + 2, NKB - 1);  // the last trip re-reads a block it will not use
            load_x(nb);
            load_a(nb, a0);
            compute(a1);
            store_x();
        }

        // lane (q, c) of token tile tt holds tile rows 4q + r of list row 16tt + c.
        // Gated: q = 0, 1 the up products of neurons 4q + r, q = 2, 3 the gate products of
        // neurons 4(q - 2) + r.  Plain: neuron 4q + r (plus its bias).
        float bias[4] = {0.f, 0.f, 0.f, 0.f};
        if (!GATED && b_up) {
#pragma unroll
            for (int r = 0; r < 4; ++r) bias[r] = (float)b_up[(size_t)e * m + min(4 * q + r, m - 1)];
        }
        with_activation(act, [&](auto act_c) {
        constexpr int ACT = decltype(act_c)::value;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            float v[4], w[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (GATED) {
                    const float other = __shfl_xor(acc[tt][r], 32, 64);  // q <-> q ^ 2
                    const float up = q < 2 ? acc[tt][r] : other;
                    const float gate = q < 2 ? other : acc[tt][r];
                    v[r] = activate_fast(ACT, gate) * up;
                    if (4 * (q & 1) + r >= m) v[r] = 0.0f;
                } else {
                    v[r] = activate_fast(ACT, acc[tt][r] + bias[r]);
                    if (4 * q + r >= m) v[r] = 0.0f;
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) w[r] = __shfl_xor(v[r], 16, 64);  // the other half of a piece
            // piece p of the 32-neuron H row = neurons 8p .. 8p+7.  Gated: lane q = 0 has piece 0,
            // the others write the zero pieces 1..3.  Plain: lane q = 0 has piece 0, q = 2 piece 1,
            // q = 1 and 3 write the zero pieces 2 and 3.
            const bool real = GATED ? q == 0 : (q & 1) == 0;
            const int piece = GATED ? q : (real ? (q >> 1) : 2 + (q >> 1));
            bf16x8 hv;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                hv[r] = (__bf16)(real ? v[r] : 0.0f);
                hv[4 + r] = (__bf16)(real ? w[r] : 0.0f);
            }
            *reinterpret_cast<bf16x8*>(Hf + ((size_t)item * UR + 16 * tt + c) * 32 + 8 * piece) = hv;
        }
        });
    }
    }  // windows
}

// Up-projection for wide experts (8 or more neuron tiles per item, e.g. gated m = 64): there the
// weights of an expert are as large as its x rows, so streaming them once per wavefront made the
// kernel a weight stream.  Here a workgroup of four wavefronts owns 4 x 16*TT consecutive list
// rows of one expert and shares each K block of the weight fragments through LDS (double
// buffered, one barrier per block); the x rows stay private to their wavefront as above.
//
// The K blocks of all the items of a workgroup form one stream: while block k is multiplied,
// block k+1 waits in LDS or is on its way there and the loads of block k+2 are in flight -- also
// across the end of an item, so that the first blocks of the next item arrive during the
// activation epilogue of the current one instead of after it (an item is only 12 to 32 blocks
// long, and a round trip beyond L2 takes as long as two or three blocks).
template <int MT, bool GATED, int TT>
__global__ __launch_bounds__(256, 2) void up_wide_bf16_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ wupf,
    const __bf16* __restrict__ wgatef, const __bf16* __restrict__ b_up,
    const int32_t* __restrict__ witem, const int32_t* __restrict__ wfirst,
    const int32_t* __restrict__ alist, __bf16* __restrict__ Hf, int d, int E, int m, int act) {
    constexpr int BR = GATED ? 2 : 1;
    constexpr int KS = MT / 2;
    constexpr int NT = BR * MT;         // neuron tiles per K step
    constexpr int WR = TT * 16;         // rows per wavefront
    constexpr int UR = 4 * WR;          // rows per work item
    constexpr int NL = TT * 2;          // x load instructions per K block
    constexpr int NWF = 2 * NT;         // weight fragments (1 KiB each) per K block
    constexpr int NWL = NWF / 4;        // ... of which each wavefront copies every fourth
    static_assert(NWF % 4 == 0 && MT % 2 == 0, "weight fragments are copied four at a time");
    extern __shared__ char smem[];
    char* wbuf = smem;                                   // [2][NWF][1024]
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15, w = threadIdx.x >> 6;
    char* xs = smem + 2 * NWF * 1024 + w * (WR * kUpRowBytes);   // [WR][kUpRowBytes], private
    float* sbias = reinterpret_cast<float*>(smem + 2 * NWF * 1024 + 4 * (WR * kUpRowBytes));  // [2][MT * 16]
    const int NK32 = d / 32, NKB = d / 64;   // NKB >= 2
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
    auto rows_of = [&](int item, uint32_t (&xoff)[NL], bool& active) {
        const int32_t* tl = alist + (size_t)item * UR + w * WR;
        active = tl[0] >= 0;  // valid rows are a prefix
#pragma unroll
        for (int i = 0; i < NL; ++i)
            xoff[i] = (uint32_t)max(tl[ld_row + 8 * i], 0);
    };
    // Weight fragment f = (br * MT + mt) * 2 + ks of a K block; this wavefront copies the
    // fragments f = 4 i + w: ks = w & 1, mt = (2 i) % MT + (w >> 1), br = (2 i) / MT.
    const uint32_t woff = (uint32_t)(((w >> 1) * NK32 + (w & 1)) * 512 + lane * 8);
    bf16x8 xr[NL], wr[NWL];
    auto issue = [&](int e, const uint32_t (&xoff)[NL], bool active, int kb) {
        const size_t we = (size_t)e * MT * NK32 * 512 + (size_t)kb * 1024 + woff;
#pragma unroll
        for (int i = 0; i < NWL; ++i) {
            const __bf16* base = (GATED && (2 * i) / MT == BR - 1) ? wgatef : wupf;
            wr[i] = load8(base + we + (size_t)((2 * i) % MT) * NK32 * 512);
        }
        if (active) {
#pragma unroll
            for (int i = 0; i < NL; ++i)
                xr[i] = load8(x + ((size_t)xoff[i] * (uint32_t)d + (uint32_t)(8 * ld_piece + 64 * kb)));
        }
    };
    auto park = [&](int buf, bool active) {
#pragma unroll
        for (int i = 0; i < NWL; ++i)
            *reinterpret_cast<bf16x8*>(wbuf + buf * NWF * 1024 + (4 * i + w) * 1024 + lane * 16) = wr[i];
        if (active) {
            char* dst = xs + ld_row * kUpRowBytes + ld_piece * 16;
#pragma unroll
            for (int i = 0; i < NL; ++i)
                *reinterpret_cast<bf16x8*>(dst + 8 * i * kUpRowBytes) = xr[i];
        }
    };
    auto park_bias = [&](int e, int par) {  // plain experts: the item's biases, by neuron
        if (!GATED && (int)threadIdx.x < MT * 16)
            sbias[par * MT * 16 + threadIdx.x] =
                b_up ? (float)b_up[(size_t)e * m + min((int)threadIdx.x, m - 1)] : 0.0f;
    };

    int e, item;
    uint32_t xoff[NL];
    bool active;
    locate(j, e, item);
    rows_of(item, xoff, active);
    issue(e, xoff, active, 0);
    park(0, active);
    park_bias(e, 0);
    lds_barrier();
    issue(e, xoff, active, 1);
    int buf = 0, par = 0;
    for (;;) {
        // the item after this one (the last item names itself: its first blocks are read again
        // and never used)
        const int jn = j + (int)gridDim.x;
        const bool more = jn < total;
        int en = e, itemn = item;
        if (more) locate(jn, en, itemn);

        f32x4 acc[NT][TT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[nt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto multiply = [&]() {
            if (active) {
                const char* wsrc_l = wbuf + buf * NWF * 1024 + lane * 16;
                const char* xsrc = xs + c * kUpRowBytes + q * 16;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    bf16x8 b[TT];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        b[tt] = *reinterpret_cast<const bf16x8*>(xsrc + tt * 16 * kUpRowBytes + ks * 64);
                    // the weight tile of the next four MFMAs is read while the current four run
                    bf16x8 a_next = *reinterpret_cast<const bf16x8*>(wsrc_l + ks * 1024);
                    __builtin_amdgcn_sched_group_barrier(0x100, TT + 1, 0);  // the reads so far
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const bf16x8 a = a_next;
                        if (nt + 1 < NT)
                            a_next = *reinterpret_cast<const bf16x8*>(wsrc_l + ((nt + 1) * 2 + ks) * 1024);
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) acc[nt][tt] = mfma16(a, b[tt], acc[nt][tt]);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read ...
                        __builtin_amdgcn_sched_group_barrier(0x008, TT, 0); // ... then the MFMAs
                    }
                }
            }
        };
        // block kb is in LDS buffer `buf`, block kb + 1 in flight to the registers
        for (int kb = 0; kb < NKB - 2; ++kb) {
            multiply();
            park(buf ^ 1, active);
            lds_barrier();
            buf ^= 1;
            issue(e, xoff, active, kb + 2);
        }
        // The next item's rows are requested here, two blocks before the end: vector loads return
        // in order, so requested any later they would queue behind the next item's first blocks,
        // and any earlier their wait would hold up this item's start.
        uint32_t xoffn[NL];
        bool activen;
        rows_of(itemn, xoffn, activen);
        multiply();                    // block NKB - 2
        park(buf ^ 1, active);
        lds_barrier();
        buf ^= 1;
        issue(en, xoffn, activen, 0);
        multiply();                    // block NKB - 1; the next item's block 0 arrives
        park(buf ^ 1, activen);
        park_bias(en, par ^ 1);
        lds_barrier();
        buf ^= 1;
        issue(en, xoffn, activen, 1);

        if (active) with_activation(act, [&](auto act_c) {
            constexpr int ACT = decltype(act_c)::value;
            const float* sb = sbias + par * MT * 16;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                __bf16* dst = Hf + ((size_t)item * UR + w * WR + 16 * tt + c) * (KS * 32) + 8 * q;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    bf16x8 hv;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const int mt = 2 * ks + half;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float v;
                            if (GATED) v = activate_fast(ACT, acc[MT + mt][tt][r]) * acc[mt][tt][r];
                            else v = activate_fast(ACT, acc[mt][tt][r] + sb[neuron_of_slot(mt, 4 * q + r)]);
                            if (neuron_of_slot(mt, 4 * q + r) >= m) v = 0.0f;
                            hv[half * 4 + r] = (__bf16)v;
                        }
                    }
                    *reinterpret_cast<bf16x8*>(dst + ks * 32) = hv;
                    // eight values at a time: interleaving more of them costs registers the
                    // requests in flight are using
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        });
        if (!more) break;
        j = jn;
        e = en;
        item = itemn;
        active = activen;
        par ^= 1;
#pragma unroll
        for (int i = 0; i < NL; ++i) xoff[i] = xoffn[i];
    }
}

// ---- launchers ---------------------------------------------------------------------------------------
template <int MT, bool GATED, int TT, int NBUF = 2>
void launch_up_t(const dmoe_layer& L, const void* x, const PackedLayout& P, const int32_t* witem,
                 const int32_t* wfirst, int NW, const int32_t* alist, void* H, int grid,
                 hipStream_t s) {
    const size_t lds = ((2 * (size_t)L.n_experts + 1) * 4 + 15) / 16 * 16 +
                       4 * NBUF * (size_t)TT * 16 * kUpRowBytes;
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_bf16_kernel<MT, GATED, TT, NBUF>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    const char* pk = static_cast<const char*>(L.packed);
    launch_kernel(up_bf16_kernel<MT, GATED, TT, NBUF>, grid, 256, lds, s, 
        (const __bf16*)x, (const __bf16*)(pk + P.wupf), (const __bf16*)(pk + P.wgatef),
        (const __bf16*)L.b_up, witem, wfirst, NW, alist, (__bf16*)H, L.d_model, L.n_experts,
        L.expert_size, L.act);
}

template <int MT, bool GATED, int TT>
void launch_up_wide_t(const dmoe_layer& L, const void* x, const PackedLayout& P,
                      const int32_t* witem, const int32_t* wfirst, const int32_t* alist,
                      void* H, int grid, hipStream_t s) {
    constexpr int NWF = 2 * (GATED ? 2 : 1) * MT;
    const size_t lds = 2 * NWF * 1024 + 4 * (size_t)TT * 16 * kUpRowBytes + 2 * MT * 16 * sizeof(float);
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_wide_bf16_kernel<MT, GATED, TT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    const char* pk = static_cast<const char*>(L.packed);
    launch_kernel(up_wide_bf16_kernel<MT, GATED, TT>, grid, 256, lds, s, 
        (const __bf16*)x, (const __bf16*)(pk + P.wupf), (const __bf16*)(pk + P.wgatef),
        (const __bf16*)L.b_up, witem, wfirst, alist, (__bf16*)H, L.d_model, L.n_experts,
        L.expert_size, L.act);
}

}  // namespace

bool experts_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    if (!(mp == 32 || mp == 64 || mp == 128)) return false;
    if (L.gated && mp == 128) return false;  // accumulators of both branches would not fit
    return down_bf16_supported(L) && L.n_experts <= kMaxExperts;
}

void launch_pack_bf16(const dmoe_layer& L, void* packed, hipStream_t s) {
    LaunchTimer tm(kSlotPack, s);
    const PackedLayout P = packed_layout(L);
    const int mp = m_pad_of(L.expert_size);
    char* pk = static_cast<char*>(packed);
    const int fp8 = weights_fp8(L);
    const int E = L.n_experts, m = L.expert_size, d = L.d_model;
    const float* scales = nullptr;   // the snapped copy inside the packed buffer
    if (fp8) {
        launch_kernel(snap_scales_kernel, div_up(3 * E, 256), 256, 0, s, L.w_scales,
                      (float*)(pk + P.scales), 3 * E);
        scales = (const float*)(pk + P.scales);
    }
    launch_kernel(pack_down_kernel<__bf16>, 2048, 256, 0, s, L.w_down, scales, fp8, (__bf16*)(pk + P.w2f), E,
                                                  m, d, mp / 32);
    launch_pack_down_bf16(L, pk + P.w2g, s);
    launch_kernel(pack_up_kernel<__bf16>, 2048, 256, 0, s, L.w_up, scales, fp8, 0, (__bf16*)(pk + P.wupf), E,
                                                m, d, mp / 16, 1);
    if (L.gated)
        launch_kernel(pack_up_kernel<__bf16>, 2048, 256, 0, s, L.w_gate, scales, fp8, 1,
                                                    (__bf16*)(pk + P.wgatef), E, m, d, mp / 16, 1);
    if (up_tiny_supported(L))
        launch_kernel(pack_up_tiny_kernel, 2048, 256, 0, s, L.w_up, L.w_gate, scales, fp8,
                                                 (__bf16*)(pk + P.wtinyf), E, m, d, L.gated);
    if (fp8) {  // byte fragments for the small-token kernels
        launch_kernel(pack_down_kernel<uint8_t>, 2048, 256, 0, s, L.w_down, scales, 1, (uint8_t*)(pk + P.w2f8),
                                                       E, m, d, mp / 32);
        launch_kernel(pack_up_kernel<uint8_t>, 2048, 256, 0, s, L.w_up, scales, 1, 0, (uint8_t*)(pk + P.wupf8),
                                                     E, m, d, mp / 16, 1);
        if (L.gated)
            launch_kernel(pack_up_kernel<uint8_t>, 2048, 256, 0, s, L.w_gate, scales, 1, 1,
                                                         (uint8_t*)(pk + P.wgatef8), E, m, d, mp / 16, 1);
    }
    if (up_x8_supported(L)) launch_pack_x8(L, packed, s);  // operands of the 8-bit up-projection
    if (down_x8_shape(L)) launch_pack_down_x8(L, packed, s);  // ... and of the 8-bit down-projection
    // the router matrices use the same fragment format: "one expert" whose rows are the hidden
    // units (r_w1) or the experts (r_w2)
    const int dh = L.router_hidden;
    if (L.r_w1 && L.r_w2 && dh > 0 && dh % 32 == 0 && L.d_model % 32 == 0) {
        launch_kernel(pack_up_kernel<__bf16>, 512, 256, 0, s, L.r_w1, nullptr, 0, 0, (__bf16*)(pk + P.r1f), 1, dh,
                                                   L.d_model, dh / 16, 0);
        launch_kernel(pack_up_kernel<__bf16>, 512, 256, 0, s, L.r_w2, nullptr, 0, 0, (__bf16*)(pk + P.r2f), 1,
                                                   L.n_experts, dh, div_up(L.n_experts, 16), 0);
    }
}

// Groups of 64 tokens per up-projection window: the x rows of a window (about 3 MB) should stay
// in the 4 MB L2 of the XCD that works on it, and the number of windows is a multiple of 8 so
// that every XCD gets the same number.
int up_window_groups(const dmoe_layer& L, int T) {
    const int NG = div_up(T, kGroup);
    // wide experts: per window the XCD would stream every expert's weights (far more than its
    // L2) through the same cache, and the 256-row items span more than a window; measured slower
    if (up_rows_bf16(L) != 64) return std::max(1, NG);
    const double x_bytes = 2.0 * (double)NG * kGroup * L.d_model;
    const double window_bytes = 3.2 * 1048576.0;
    const int n_windows = 8 * std::max(1, (int)ceil(x_bytes / (8.0 * window_bytes)));
    return std::max(1, div_up(NG, n_windows));
}

void launch_up_bf16(const dmoe_layer& L, const void* x, int T, const int32_t* witem,
                    const int32_t* wfirst, const int32_t* alist, void* H, hipStream_t s) {
    LaunchTimer tm(kSlotUp, s);
    const PackedLayout P = packed_layout(L);
    const int NW = div_up(div_up(T, kGroup), up_window_groups(L, T));
    // persistent wavefronts: enough to cover the worst case once, capped at two workgroups per
    // CU; a multiple of 8 so that every XCD runs the same number
    const long long worst = (long long)T * L.n_experts / up_rows_bf16(L) + L.n_experts;
    const int grid = round_up((int)std::min<long long>((worst + 3) / 4, 256 * 2), 8);
    const int mt = m_pad_of(L.expert_size) / 16;
    if (up_rows_bf16(L) == 256) {  // wide experts: weights shared through LDS
        const int wgrid = round_up(
            (int)std::min<long long>((long long)T * L.n_experts / 256 + L.n_experts, 512), 8);
        if (L.gated) launch_up_wide_t<4, true, 4>(L, x, P, witem, wfirst, alist, H, wgrid, s);
        else launch_up_wide_t<8, false, 4>(L, x, P, witem, wfirst, alist, H, wgrid, s);
        return;
    }
    if (up_tiny_supported(L)) {
        constexpr int TT = 4;
        const size_t lds = (2 * (size_t)L.n_experts * 4 + 15) / 16 * 16 +
                           4 * (size_t)TT * 16 * kUpRowBytes;
        // as many workgroups per CU as LDS allows, at most the three that the registers allow
        // (squeezed into a fourth wavefront per SIMD's share of registers the kernel got slower)
        const int per_cu = std::max(1, std::min(3, (int)(160 * 1024 / lds)));
        const int grid = round_up((int)std::min<long long>((worst + 3) / 4, 256 * per_cu), 8);
        static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
        std::call_once(attr_once, [&] {
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_tiny_kernel<TT, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_tiny_kernel<TT, false>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        });
        const char* pk = static_cast<const char*>(L.packed);
        if (L.gated)
            launch_kernel(up_tiny_kernel<TT, true>, grid, 256, lds, s, 
                (const __bf16*)x, (const __bf16*)(pk + P.wtinyf), nullptr, witem, wfirst, NW, alist,
                (__bf16*)H, L.d_model, L.n_experts, L.expert_size, L.act);
        else
            launch_kernel(up_tiny_kernel<TT, false>, grid, 256, lds, s, 
                (const __bf16*)x, (const __bf16*)(pk + P.wtinyf), (const __bf16*)L.b_up, witem, wfirst,
                NW, alist, (__bf16*)H, L.d_model, L.n_experts, L.expert_size, L.act);
        return;
    }
    if (L.gated) {
        if (mt == 2) launch_up_t<2, true, 4>(L, x, P, witem, wfirst, NW, alist, H, grid, s);
        else launch_up_t<4, true, 4>(L, x, P, witem, wfirst, NW, alist, H, grid, s);
    } else {
        if (mt == 2) {
            // 32-neuron rows: one staging buffer, three workgroups per CU
            const int grid3 = round_up((int)std::min<long long>((worst + 3) / 4, 256 * 3), 8);
            launch_up_t<2, false, 4, 1>(L, x, P, witem, wfirst, NW, alist, H, grid3, s);
        }
        else if (mt == 4) launch_up_t<4, false, 4>(L, x, P, witem, wfirst, NW, alist, H, grid, s);
        else launch_up_t<8, false, 4>(L, x, P, witem, wfirst, NW, alist, H, grid, s);
    }
}

}  // namespace dmoe

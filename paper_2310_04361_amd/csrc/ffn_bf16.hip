// bf16 expert execution and merge (Sec. 3.2, Appendix G) on the gfx950 matrix cores.
//
// Two kernels, both driven by the sorted per-expert token lists:
//   up    expert-major grouped GEMM over the compact lists.  A wavefront owns UR = 16*TT list
//         rows of one expert, gathers those rows of x in 128-byte pieces (eight lanes per row, so
//         the vector memory path sees whole cache lines), stages them in its own LDS buffers and
//         multiplies them with the expert's up (and gate) rows; bias + activation in fp32; the
//         hidden activations go out rounded to bf16 in MFMA-fragment order.
//   down  output-stationary: a workgroup owns 64 consecutive tokens x 256 output columns as an
//         fp32 tile in LDS, walks all experts, multiplies the chunk's H fragments of each expert
//         by that expert's down-projection slice and adds the result into the owning token rows
//         (plain LDS read-add-write; each wavefront owns its own columns).  Every y element is
//         written exactly once, in bf16; no global atomics, no second pass.
// Tokens ride on the MFMA column axis in both kernels, so four consecutive neurons (up) or
// output columns (down) of one token land in one lane.
//
// Fragment order.  Every operand that a wavefront reads with one load instruction is stored as
// the 1 KiB block  [lane 0..63][8 bf16]  in exactly the register layout of the MFMA, because a
// 16-byte-per-lane access with a 64-byte or larger lane stride costs a cache-line lookup per
// lane and that, not bandwidth, bounded the first version of these kernels.
//   H fragment F, k-step ks: lane (q, c) holds, for list row 16*(F - first fragment of the
//     expert) + c, the neurons 32ks + 16*(s/4) + 4q + (s%4), s = 0..7 -- the order in which the
//     up kernel's accumulators come out; the packed down-projection uses the same k order.
//   An expert's H rows start at a multiple of UR rows (its first up-projection work item), so
//     fragments never mix experts.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

constexpr int kDownWaves = 8;
constexpr int kDownCols = kDownWaves * 32;     // output columns per down workgroup
constexpr int kDownBatch = 128;                // experts per tile-list batch
constexpr int kDownTilesPerExpert = (kChunk + 31) / 32;       // 32-row tiles per (chunk, expert)
constexpr int kDownStride = kDownCols + 4;     // LDS row stride in floats
constexpr size_t kDownLds = sizeof(float) * kChunk * kDownStride +
                            sizeof(int2) * kDownBatch * kDownTilesPerExpert;
constexpr int kUpRowBytes = 144;               // 64 bf16 of one x row + 16 bytes of bank skew

// ---- activations (fp32 in, fp32 out) -------------------------------------------------------------
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

// ---- one-time weight packing ------------------------------------------------------------------------
// w_down[E][m][d] -> w2f[E][d/16][KS][64][8]: lane (q, c) of fragment (e, column tile ct, ks)
// holds W_down[e][32ks + 16*(s/4) + 4q + s%4][16ct + c], zero for neurons >= m.
__global__ void pack_down_kernel(const __bf16* __restrict__ w_down, __bf16* __restrict__ w2f,
                                 int E, int m, int d, int KS) {
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
        const int neuron = 32 * ks + 16 * (s >> 2) + 4 * q + (s & 3);
        w2f[i] = neuron < m ? w_down[((size_t)e * m + neuron) * d + 16 * ct + c] : (__bf16)0.0f;
    }
}

// w[E][m][d] -> wf[E][MT][d/32][64][8]: lane (q, c) of fragment (e, neuron tile mt, k-step) holds
// w[e][16mt + c][32 kstep + 8q + s], zero rows for neurons >= m.
__global__ void pack_up_kernel(const __bf16* __restrict__ w, __bf16* __restrict__ wf, int E, int m,
                               int d, int MT) {
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
        const int neuron = 16 * mt + c;
        wf[i] = neuron < m ? w[((size_t)e * m + neuron) * d + 32 * kstep + 8 * q + s] : (__bf16)0.0f;
    }
}

// ---- up-projection ---------------------------------------------------------------------------------
// One wavefront per work item = (expert, UR = 16*TT consecutive list rows); no workgroup-level
// synchronisation after the work-item table has been staged.  MT = m_pad / 16 neuron tiles per
// branch.  K advances in blocks of 64: the wavefront loads the next block of its x rows
// (lane = (row % 8, 16-byte piece of the 128-byte row segment)) and of the weight fragments
// while the MFMAs run on the current block out of LDS / registers.
template <int MT, bool GATED, int TT>
__global__ __launch_bounds__(256) void up_bf16_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ wupf,
    const __bf16* __restrict__ wgatef, const __bf16* __restrict__ b_up,
    const int32_t* __restrict__ item_start, const int32_t* __restrict__ alist,
    __bf16* __restrict__ Hf, int d, int E, int m, int act) {
    constexpr int BR = GATED ? 2 : 1;
    constexpr int KS = MT / 2;
    constexpr int UR = TT * 16;
    constexpr int NL = TT * 2;  // x load instructions per K block: 8 rows x 128 bytes each
    extern __shared__ char smem[];
    int32_t* s_items = reinterpret_cast<int32_t*>(smem);  // item_start[0..E+1]
    const int items_bytes = ((E + 2) * 4 + 15) & ~15;
    for (int i = threadIdx.x; i <= E + 1; i += blockDim.x) s_items[i] = item_start[i];
    __syncthreads();
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15;
    const int wave_in_block = threadIdx.x >> 6;
    char* xs = smem + items_bytes + wave_in_block * (2 * UR * kUpRowBytes);
    const int NK32 = d / 32, NKB = d / 64;
    const int ld_row = lane >> 3, ld_piece = lane & 7;

    const int total = s_items[E];
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;

    // Items are taken in expert-major order.  (Ordering them so that an XCD's wavefronts share a
    // token window -- for L2 reuse of the x rows -- measured slower: the gathers then collide
    // on the same L2 channels.)
    for (int item = wave; item < total; item += n_waves) {
        int lo = 0, hi = E;  // last e with s_items[e] <= item
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_items[mid] <= item) lo = mid; else hi = mid;
        }
        const int e = lo;
        // rows of the aligned list past the expert's last token hold -1: they read token 0 and
        // produce H rows that nobody merges
        const int32_t* tl = alist + (size_t)item * UR + ld_row;
        const __bf16* xrow[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int tok = max(tl[8 * i], 0);
            xrow[i] = x + (size_t)tok * d + 8 * ld_piece;
        }
        const __bf16* wf[BR];
        wf[0] = wupf + (size_t)e * MT * NK32 * 512 + lane * 8;
        if (GATED) wf[BR - 1] = wgatef + (size_t)e * MT * NK32 * 512 + lane * 8;

        // biases of this lane's neurons, fetched now so that their latency hides under the K loop
        float bias[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = 16 * mt + 4 * q + r;
                bias[mt][r] = (!GATED && b_up) ? (float)b_up[(size_t)e * m + min(n, m - 1)] : 0.0f;
            }

        f32x4 acc[BR][MT][TT];
#pragma unroll
        for (int br = 0; br < BR; ++br)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[br][mt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

        bf16x8 xr[NL];
        bf16x8 a0[2][BR][MT], a1[2][BR][MT];
        auto load_x = [&](int kb) {
#pragma unroll
            for (int i = 0; i < NL; ++i) xr[i] = load8(xrow[i] + 64 * kb);
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
            char* dst = xs + buf * (UR * kUpRowBytes) + ld_row * kUpRowBytes + ld_piece * 16;
#pragma unroll
            for (int i = 0; i < NL; ++i)
                *reinterpret_cast<bf16x8*>(dst + 8 * i * kUpRowBytes) = xr[i];
        };
        auto compute = [&](int buf, const bf16x8 (&a)[2][BR][MT]) {
            const char* src = xs + buf * (UR * kUpRowBytes) + c * kUpRowBytes + q * 16;
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

        load_x(0);
        load_a(0, a0);
        store_x(0);
        // two K blocks per trip so that the two weight-fragment register sets simply alternate
        for (int kb = 0; kb < NKB; kb += 2) {
            load_x(kb + 1);
            load_a(kb + 1, a1);
            compute(0, a0);
            store_x(1);
            const int nb = min(kb + 2, NKB - 1);  // the last trip re-reads a block it will not use
            load_x(nb);
            load_a(nb, a0);
            compute(1, a1);
            store_x(0);
        }

        // lane (q, c) of tile (mt, tt): neurons 16mt + 4q + r of list row 16tt + c
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            __bf16* dst = Hf + (((size_t)item * TT + tt) * KS * 64 + lane) * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 hv;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int mt = 2 * ks + half;
                    const int n0 = 16 * mt + 4 * q;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float v;
                        if (GATED) {
                            v = activate_fast(act, acc[BR - 1][mt][tt][r]) * acc[0][mt][tt][r];
                        } else {
                            v = activate_fast(act, acc[0][mt][tt][r] + bias[mt][r]);
                        }
                        if (n0 + r >= m) v = 0.0f;
                        hv[half * 4 + r] = (__bf16)v;
                    }
                }
                *reinterpret_cast<bf16x8*>(dst + (size_t)ks * 512) = hv;
            }
        }
    }
}

// Up-projection for wide experts (8 or more neuron tiles per item, e.g. gated m = 64): there the
// weights of an expert are as large as its x rows, so streaming them once per wavefront made the
// kernel a weight stream.  Here a workgroup of four wavefronts owns 4 x 16*TT consecutive list
// rows of one expert and shares each K block of the weight fragments through LDS (double
// buffered, one barrier per block); the x rows stay private to their wavefront as above.
template <int MT, bool GATED, int TT>
__global__ __launch_bounds__(256, 2) void up_wide_bf16_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ wupf,
    const __bf16* __restrict__ wgatef, const int32_t* __restrict__ item_start,
    const int32_t* __restrict__ alist, __bf16* __restrict__ Hf, int d, int E, int m, int act) {
    constexpr int BR = GATED ? 2 : 1;
    constexpr int KS = MT / 2;
    constexpr int NT = BR * MT;         // neuron tiles per K step
    constexpr int WR = TT * 16;         // rows per wavefront
    constexpr int UR = 4 * WR;          // rows per work item
    constexpr int NL = TT * 2;          // x load instructions per K block
    constexpr int NWF = 2 * NT;         // weight fragments (1 KiB each) per K block
    static_assert(NWF % 4 == 0, "weight fragments are copied four at a time");
    extern __shared__ char smem[];
    char* wbuf = smem;                                   // [2][NWF][1024]
    const int lane = threadIdx.x & 63, q = lane >> 4, c = lane & 15, w = threadIdx.x >> 6;
    char* xs = smem + 2 * NWF * 1024 + w * (WR * kUpRowBytes);   // [WR][kUpRowBytes], private
    const int NK32 = d / 32, NKB = d / 64;
    const int ld_row = lane >> 3, ld_piece = lane & 7;
    const int total = item_start[E];

    for (int item = blockIdx.x; item < total; item += gridDim.x) {
        // expert of this item: the last e with item_start[e] <= item (uniform binary search)
        int lo = 0, hi = E;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (item_start[mid] <= item) lo = mid; else hi = mid;
        }
        const int e = lo;
        const int32_t* tl = alist + (size_t)item * UR + w * WR + ld_row;
        const bool active = alist[(size_t)item * UR + w * WR] >= 0;  // valid rows are a prefix
        const __bf16* xrow[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) xrow[i] = x + (size_t)max(tl[8 * i], 0) * d + 8 * ld_piece;
        // weight fragment f = (br*MT + mt)*2 + ks of K block kb; thread copies piece (f % 4 == w)
        const __bf16* wsrc[NWF / 4];
#pragma unroll
        for (int i = 0; i < NWF / 4; ++i) {
            const int f = 4 * i + w, ks = f & 1, tile = f >> 1, br = tile / MT, mt = tile % MT;
            const __bf16* base = (GATED && br == BR - 1) ? wgatef : wupf;
            wsrc[i] = base + (((size_t)e * MT + mt) * NK32 + ks) * 512 + lane * 8;
        }

        f32x4 acc[NT][TT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[nt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

        bf16x8 xr[NL], wr[NWF / 4];
        auto load_next = [&](int kb) {
#pragma unroll
            for (int i = 0; i < NWF / 4; ++i) wr[i] = load8(wsrc[i] + (size_t)kb * 1024);
            if (active) {
#pragma unroll
                for (int i = 0; i < NL; ++i) xr[i] = load8(xrow[i] + 64 * kb);
            }
        };
        auto store_next = [&](int buf) {
#pragma unroll
            for (int i = 0; i < NWF / 4; ++i)
                *reinterpret_cast<bf16x8*>(wbuf + buf * NWF * 1024 + (4 * i + w) * 1024 + lane * 16) = wr[i];
            if (active) {
                char* dst = xs + ld_row * kUpRowBytes + ld_piece * 16;
#pragma unroll
                for (int i = 0; i < NL; ++i)
                    *reinterpret_cast<bf16x8*>(dst + 8 * i * kUpRowBytes) = xr[i];
            }
        };
        __syncthreads();  // the previous item's last K block has been consumed by every wavefront
        load_next(0);
        store_next(0);
        __syncthreads();
        for (int kb = 0; kb < NKB; ++kb) {
            load_next(min(kb + 1, NKB - 1));  // the last trip re-reads a block it will not use
            if (active) {
                const char* wsrc_l = wbuf + (kb & 1) * NWF * 1024 + lane * 16;
                const char* xsrc = xs + c * kUpRowBytes + q * 16;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    bf16x8 b[TT];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        b[tt] = *reinterpret_cast<const bf16x8*>(xsrc + tt * 16 * kUpRowBytes + ks * 64);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const bf16x8 a = *reinterpret_cast<const bf16x8*>(wsrc_l + (nt * 2 + ks) * 1024);
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) acc[nt][tt] = mfma16(a, b[tt], acc[nt][tt]);
                    }
                }
            }
            store_next((kb + 1) & 1);
            __syncthreads();
        }

        if (active) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                __bf16* dst = Hf + ((((size_t)item * 4 + w) * TT + tt) * KS * 64 + lane) * 8;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    bf16x8 hv;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const int mt = 2 * ks + half;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float v;
                            if (GATED) v = activate_fast(act, acc[MT + mt][tt][r]) * acc[mt][tt][r];
                            else v = activate_fast(act, acc[mt][tt][r]);
                            if (16 * mt + 4 * q + r >= m) v = 0.0f;
                            hv[half * 4 + r] = (__bf16)v;
                        }
                    }
                    *reinterpret_cast<bf16x8*>(dst + (size_t)ks * 512) = hv;
                }
            }
        }
    }
}

// ---- down-projection and merge ------------------------------------------------------------------------
// One workgroup per (64-token chunk, 256-column slice), two of them per CU; KS = m_pad / 32
// MFMA k-steps.
//
// The fp32 output tile Y[64][256] lives in LDS.  The eight wavefronts own 32 columns each, so
// no two wavefronts ever touch the same element and the merge is a plain read-add-write (LDS
// float atomics proved far slower).  All wavefronts walk the same list of tiles -- up to 32
// consecutive rows of one expert's part of H, all belonging to this chunk -- built once per
// batch of experts from the group offsets.
// Per tile and wavefront: D[32 cols][32 rows] = W2 slice * H_tile^T as 2 x 2 MFMA 16x16x32
// tiles with the tokens on the MFMA column axis, so a lane ends up with four consecutive output
// columns of ONE token: one 16-byte LDS read and write per MFMA tile, one row address per
// token.  The row stride of 260 floats spreads consecutive-token rows over the banks.
// Operands of the next kDepth tiles are kept in flight while the current one is merged.
template <int KS>
__global__ __launch_bounds__(kDownWaves * 64) void down_bf16_kernel(
    const __bf16* __restrict__ w2f, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ item_start, const int32_t* __restrict__ group_off,
    const int32_t* __restrict__ alist, const __bf16* __restrict__ Hf, __bf16* __restrict__ y, int T,
    int d, int E, int NG, int frags_per_item) {
    constexpr int kThreads = kDownWaves * 64;
    constexpr int kDepth = KS <= 2 ? 4 : 2;  // tiles of operands in flight per wavefront
    extern __shared__ float smem_f[];
    float* Y = smem_f;  // [kChunk][kDownStride]
    int2* tiles = reinterpret_cast<int2*>(smem_f + kChunk * kDownStride);
    __shared__ int s_wave_tot[kDownWaves];
    // The slices of one chunk share its H rows and token lists: keep them on one XCD (workgroups
    // are dealt round-robin to the 8 XCDs) and next to each other in launch order.
    const int NS = d / kDownCols;
    const int k_in_xcd = blockIdx.x >> 3;
    const int chunk = (k_in_xcd / NS) * 8 + (blockIdx.x & 7), slice = k_in_xcd % NS;
    if (chunk * kChunk >= T) return;  // the grid is rounded up to whole groups of 8 chunks
    const int t_base = chunk * kChunk, col0 = slice * kDownCols;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, q = lane >> 4, c = lane & 15;
    {   // every row of the tile starts as the output bias of this slice
        static_assert(kThreads % kDownCols == 0, "one column per thread");
        const int col = tid % kDownCols;
        const float bias = b_down ? (float)b_down[col0 + col] : 0.0f;
        for (int row = tid / kDownCols; row < kChunk; row += kThreads / kDownCols)
            Y[row * kDownStride + col] = bias;
    }

    const int g_lo = chunk * kChunkGroups;
    const int g_hi = min(g_lo + kChunkGroups, NG);
    // weight fragments of this wavefront's two column tiles: + (e * d/16) fragments per expert
    const __bf16* wbase =
        w2f + ((size_t)(col0 / 16 + 2 * __builtin_amdgcn_readfirstlane(wave)) * KS * 64 + lane) * 8;
    const size_t w_expert_stride = (size_t)(d / 16) * KS * 512;
    // element (token t, column wave*32 + nt*16 + 4q) is at ybase + t * kDownStride + nt * 16
    float* ybase = Y + wave * 32 + 4 * q - (ptrdiff_t)t_base * kDownStride;

    for (int ebase = 0; ebase < E; ebase += kDownBatch) {
        __syncthreads();  // Y initialised / previous batch's tile list no longer read
        // ---- tile list of this batch: thread i < kDownBatch describes expert ebase + i
        int n_mine = 0, nt_mine = 0, row0 = 0;
        const int e_mine = ebase + tid;
        if (tid < kDownBatch && e_mine < E) {
            // rows lo .. hi-1 of expert e_mine's list belong to this chunk
            const int lo = group_off[(size_t)g_lo * E + e_mine];
            n_mine = group_off[(size_t)g_hi * E + e_mine] - lo;
            if (n_mine > 0) {
                nt_mine = (n_mine + 31) >> 5;
                row0 = item_start[e_mine] * frags_per_item * 16 + lo;  // row of H / alist
            }
        }
        int incl = nt_mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(incl, off, 64);
            if (lane >= off) incl += v;
        }
        if (lane == 63) s_wave_tot[wave] = incl;
        __syncthreads();
        int start = incl - nt_mine, ntiles = 0;
        for (int w2 = 0; w2 < kDownWaves; ++w2) {
            const int v = s_wave_tot[w2];
            if (w2 < wave) start += v;
            ntiles += v;
        }
        for (int k = 0; k < nt_mine; ++k)
            tiles[start + k] = make_int2(row0 + 32 * k, (e_mine << 8) | min(32, n_mine - 32 * k));
        __syncthreads();
        // ---- walk the tiles with a ring of kDepth tiles of operands in flight
        bf16x8 a_st[kDepth][2][KS], b_st[kDepth][2][KS];
        int tok_st[kDepth][2], rows_st[kDepth];
        // Issues the loads only; nothing here waits on them, so kDepth tiles of loads overlap.
        // A tile is up to 32 consecutive rows of H that all belong to this chunk; they start at
        // any row, so each lane finds its row's fragment and slot itself (the rows of a tile
        // still sit in at most three adjacent 1 KiB fragments).  Lanes past the tile's last row
        // read row 0 of the tile again and skip the merge.  Tiles past the end repeat the last
        // one with no rows.
        // lane l of (ent_x, ent_y) holds the entry of tile ent_base + l: one LDS read per 64 tiles,
        // then constant-cost broadcasts instead of an LDS round trip per tile
        int ent_base = 0, ent_x = 0, ent_y = 0;
        auto load_entries = [&](int base) {
            const int2 ent = tiles[min(base + lane, max(ntiles - 1, 0))];
            ent_base = base;
            ent_x = ent.x;
            ent_y = ent.y;
        };
        load_entries(0);
        auto fetch = [&](int ti, bf16x8 (&a)[2][KS], bf16x8 (&b)[2][KS], int (&tok)[2], int& rows_out) {
            const int tc = min(ti, ntiles - 1);
            if (tc >= ent_base + 64) load_entries(tc);  // uniform
            const int row_first = __builtin_amdgcn_readlane(ent_x, tc - ent_base);
            const int packed = __builtin_amdgcn_readlane(ent_y, tc - ent_base);
            const int rows = ti < ntiles ? (packed & 0xff) : 0;
            const __bf16* wp = wbase + (size_t)(packed >> 8) * w_expert_stride;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = row_first + (16 * h + c < rows ? 16 * h + c : 0);
                const __bf16* hp = Hf + ((size_t)(row >> 4) * KS * 64 + 16 * q + (row & 15)) * 8;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    a[h][ks] = load8(wp + (h * KS + ks) * 512);
                    b[h][ks] = load8(hp + ks * 512);
                }
                tok[h] = alist[row];
            }
            rows_out = rows;
        };
        if (ntiles > 0) {
#pragma unroll
            for (int st = 0; st < kDepth; ++st)
                fetch(st, a_st[st], b_st[st], tok_st[st], rows_st[st]);
        }
        for (int t0 = 0; t0 < ntiles; t0 += kDepth) {
#pragma unroll
            for (int st = 0; st < kDepth; ++st) {
                // keep each stage's work inside the stage: hoisting a later stage's first use of
                // its loads up here would make this stage wait for them as well
                __builtin_amdgcn_sched_barrier(0);
                f32x4 acc[2][2];  // [column tile nt][token tile tt]
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt) {
                        acc[nt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
                            acc[nt][tt] = mfma16(a_st[st][nt][ks], b_st[st][tt][ks], acc[nt][tt]);
                    }
                int tok0 = tok_st[st][0], tok1 = tok_st[st][1];
                // Pin the MFMAs and the token reads here (an empty asm the optimiser cannot move
                // values across): otherwise they sink below the refill, the old and the new
                // operands of the stage overlap and the ring turns into register copies that
                // wait on loads just issued.  The refill then reuses the stage's registers.
                asm volatile("" : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]),
                                  "+v"(tok0), "+v"(tok1));
                __builtin_amdgcn_sched_barrier(0);
                const int rows = rows_st[st];
                fetch(t0 + st + kDepth, a_st[st], b_st[st], tok_st[st], rows_st[st]);

                // lane (q, c) of tile (nt, tt): columns nt*16 + 4q .. +3 of tile row tt*16 + c.
                // (Two variants measured slower: feeding the old values in as the MFMA's C operand,
                // and requesting them before the MFMAs.)
                const int tok[2] = {tok0, tok1};
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    if (16 * tt + c < rows) {
                        float4* yp = reinterpret_cast<float4*>(ybase + tok[tt] * kDownStride);
                        float4 o0 = yp[0], o1 = yp[4];
                        o0.x += acc[0][tt][0]; o0.y += acc[0][tt][1];
                        o0.z += acc[0][tt][2]; o0.w += acc[0][tt][3];
                        o1.x += acc[1][tt][0]; o1.y += acc[1][tt][1];
                        o1.z += acc[1][tt][2]; o1.w += acc[1][tt][3];
                        yp[0] = o0;
                        yp[4] = o1;
                    }
                }
            }
        }
    }
    __syncthreads();

    for (int i = tid; i < kChunk * (kDownCols / 8); i += kThreads) {
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

// ---- launchers ---------------------------------------------------------------------------------------
template <int MT, bool GATED, int TT>
void launch_up_t(const dmoe_layer& L, const void* x, const PackedLayout& P,
                 const int32_t* item_start, const int32_t* alist, void* H, int grid,
                 hipStream_t s) {
    const size_t lds = (((size_t)L.n_experts + 2) * 4 + 15) / 16 * 16 +
                       4 * 2 * (size_t)TT * 16 * kUpRowBytes;
    static bool attr_set = false;  // per-function, idempotent: allow more than 64 KiB of LDS
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_bf16_kernel<MT, GATED, TT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    const char* pk = static_cast<const char*>(L.packed);
    up_bf16_kernel<MT, GATED, TT><<<grid, 256, lds, s>>>(
        (const __bf16*)x, (const __bf16*)(pk + P.wupf), (const __bf16*)(pk + P.wgatef),
        (const __bf16*)L.b_up, item_start, alist, (__bf16*)H, L.d_model, L.n_experts,
        L.expert_size, L.act);
}

template <int MT, bool GATED, int TT>
void launch_up_wide_t(const dmoe_layer& L, const void* x, const PackedLayout& P,
                      const int32_t* item_start, const int32_t* alist, void* H, int grid,
                      hipStream_t s) {
    constexpr int NWF = 2 * (GATED ? 2 : 1) * MT;
    const size_t lds = 2 * NWF * 1024 + 4 * (size_t)TT * 16 * kUpRowBytes;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_wide_bf16_kernel<MT, GATED, TT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        attr_set = true;
    }
    const char* pk = static_cast<const char*>(L.packed);
    up_wide_bf16_kernel<MT, GATED, TT><<<grid, 256, lds, s>>>(
        (const __bf16*)x, (const __bf16*)(pk + P.wupf), (const __bf16*)(pk + P.wgatef), item_start,
        alist, (__bf16*)H, L.d_model, L.n_experts, L.expert_size, L.act);
}

template <int KS>
void launch_down_t(const dmoe_layer& L, const PackedLayout& P, int T, const int32_t* item_start,
                   const int32_t* group_off, const int32_t* alist, const void* H, void* y,
                   hipStream_t s) {
    const int NG = div_up(T, kGroup), NC = div_up(T, kChunk), NS = L.d_model / kDownCols;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&down_bf16_kernel<KS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDownLds);
        attr_set = true;
    }
    const char* pk = static_cast<const char*>(L.packed);
    down_bf16_kernel<KS><<<round_up(NC, 8) * NS, kDownWaves * 64, kDownLds, s>>>(
        (const __bf16*)(pk + P.w2f), (const __bf16*)L.b_down, item_start, group_off, alist,
        (const __bf16*)H, (__bf16*)y, T, L.d_model, L.n_experts, NG, up_rows_bf16(L) / 16);
}

}  // namespace

bool experts_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    if (!(mp == 32 || mp == 64 || mp == 128)) return false;
    if (L.gated && mp == 128) return false;  // accumulators of both branches would not fit
    return L.d_model % kDownCols == 0 && L.n_experts <= 8192;
}

void launch_pack_bf16(const dmoe_layer& L, void* packed, hipStream_t s) {
    LaunchTimer tm(kSlotPack, s);
    const PackedLayout P = packed_layout(L);
    const int mp = m_pad_of(L.expert_size);
    char* pk = static_cast<char*>(packed);
    pack_down_kernel<<<2048, 256, 0, s>>>((const __bf16*)L.w_down, (__bf16*)(pk + P.w2f),
                                          L.n_experts, L.expert_size, L.d_model, mp / 32);
    pack_up_kernel<<<2048, 256, 0, s>>>((const __bf16*)L.w_up, (__bf16*)(pk + P.wupf), L.n_experts,
                                        L.expert_size, L.d_model, mp / 16);
    if (L.gated)
        pack_up_kernel<<<2048, 256, 0, s>>>((const __bf16*)L.w_gate, (__bf16*)(pk + P.wgatef),
                                            L.n_experts, L.expert_size, L.d_model, mp / 16);
    // the router matrices use the same fragment format: "one expert" whose rows are the hidden
    // units (r_w1) or the experts (r_w2)
    const int dh = L.router_hidden;
    if (L.r_w1 && L.r_w2 && dh > 0 && dh % 32 == 0 && L.d_model % 32 == 0) {
        pack_up_kernel<<<512, 256, 0, s>>>((const __bf16*)L.r_w1, (__bf16*)(pk + P.r1f), 1, dh,
                                           L.d_model, dh / 16);
        pack_up_kernel<<<512, 256, 0, s>>>((const __bf16*)L.r_w2, (__bf16*)(pk + P.r2f), 1,
                                           L.n_experts, dh, div_up(L.n_experts, 16));
    }
}

void launch_up_bf16(const dmoe_layer& L, const void* x, int T, const int32_t* item_start,
                    const int32_t* alist, void* H, hipStream_t s) {
    LaunchTimer tm(kSlotUp, s);
    const PackedLayout P = packed_layout(L);
    // persistent wavefronts: enough to cover the worst case once, capped at two workgroups per CU
    const long long worst = (long long)T * L.n_experts / up_rows_bf16(L) + L.n_experts;
    const int grid = (int)std::min<long long>((worst + 3) / 4, 256 * 2);
    const int mt = m_pad_of(L.expert_size) / 16;
    if (up_rows_bf16(L) == 256) {  // wide experts without b_up: weights shared through LDS
        const int wgrid = (int)std::min<long long>((long long)T * L.n_experts / 256 + L.n_experts, 512);
        if (L.gated) launch_up_wide_t<4, true, 4>(L, x, P, item_start, alist, H, wgrid, s);
        else launch_up_wide_t<8, false, 4>(L, x, P, item_start, alist, H, wgrid, s);
        return;
    }
    if (L.gated) {
        if (mt == 2) launch_up_t<2, true, 4>(L, x, P, item_start, alist, H, grid, s);
        else launch_up_t<4, true, 4>(L, x, P, item_start, alist, H, grid, s);
    } else {
        if (mt == 2) launch_up_t<2, false, 4>(L, x, P, item_start, alist, H, grid, s);
        else if (mt == 4) launch_up_t<4, false, 4>(L, x, P, item_start, alist, H, grid, s);
        else launch_up_t<8, false, 4>(L, x, P, item_start, alist, H, grid, s);
    }
}

void launch_down_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                      const int32_t* group_off, const int32_t* alist, const void* H, void* y,
                      hipStream_t s) {
    LaunchTimer tm(kSlotDown, s);
    const PackedLayout P = packed_layout(L);
    const int ks = m_pad_of(L.expert_size) / 32;
    if (ks == 1) launch_down_t<1>(L, P, T, item_start, group_off, alist, H, y, s);
    else if (ks == 2) launch_down_t<2>(L, P, T, item_start, group_off, alist, H, y, s);
    else launch_down_t<4>(L, P, T, item_start, group_off, alist, H, y, s);
}

}  // namespace dmoe

// bf16 expert execution and merge (Sec. 3.2, Appendix G) on the gfx950 matrix cores.
//
// Two kernels, both driven by the sorted per-expert token lists:
//   up    expert-major grouped GEMM over the compact lists: gathers the listed rows of x (no
//         copy), multiplies by the expert's up (and gate) rows, applies bias + activation in fp32
//         and writes the hidden activations, rounded to bf16, to H[list position][m_pad].
//   down  output-stationary: a workgroup owns 128 consecutive tokens x 256 output columns as an
//         fp32 tile in LDS, walks all experts, multiplies the chunk's compact H rows of each
//         expert by that expert's down-projection slice and adds the result into the owning
//         token rows (plain LDS read-add-write; each wavefront owns its own columns).  Every y
//         element is written exactly once, in bf16; no global atomics, no second pass.
// Tokens ride on the MFMA column axis in both kernels, so four consecutive neurons (up) or
// output columns (down) of one token land in one lane: H is written in 8-byte pieces and the LDS
// merge moves 16 bytes per lane with a single row address.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

constexpr int kDownWaves = 8;
constexpr int kDownCols = kDownWaves * 32;     // output columns per down workgroup
constexpr int kDownBatch = 256;                // experts per tile-list batch
constexpr int kDownStride = kDownCols + 4;      // LDS row stride in floats
constexpr size_t kDownLds =
    sizeof(float) * kChunk * kDownStride + sizeof(int2) * kDownBatch * (kChunk / 32);

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

// One workgroup per (128-token chunk, 256-column slice); KS = m_pad / 32 MFMA k-steps.
//
// The fp32 output tile Y[128][256] lives in LDS.  The eight wavefronts own 32 columns each, so
// no two wavefronts ever touch the same element and the merge is a plain read-add-write (LDS
// float atomics proved far slower).  All wavefronts walk the same list of row tiles -- up to 32
// compact H rows of one expert -- built once per batch of 256 experts from the group offsets.
// Per tile and wavefront: D[32 cols][32 tokens] = W2t slice * H_tile^T as 2 x 2 MFMA 16x16x32
// tiles with the tokens on the MFMA column axis, so a lane ends up with four consecutive output
// columns of ONE token: one 16-byte LDS read and write per MFMA tile, one row address per
// token.  The row stride of 260 floats spreads consecutive-token rows over the banks.
// Operands of the next kDepth tiles are kept in flight while the current one is merged.
template <int KS>
__global__ __launch_bounds__(kDownWaves * 64) void down_bf16_kernel(
    const __bf16* __restrict__ w2t, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ group_off,
    const int32_t* __restrict__ lists, const __bf16* __restrict__ H, __bf16* __restrict__ y, int T,
    int d, int E, int NG) {
    constexpr int m_pad = KS * 32;
    constexpr int kThreads = kDownWaves * 64;
    constexpr int kDepth = KS <= 2 ? 4 : 2;  // row tiles of operands in flight per wavefront
    extern __shared__ float smem[];
    float* Y = smem;  // [kChunk][kDownStride]
    int2* tiles = reinterpret_cast<int2*>(smem + kChunk * kDownStride);  // [kDownBatch * kChunk/32]
    __shared__ int s_wave_tot[kDownWaves];
    const int NS = d / kDownCols;
    const int chunk = blockIdx.x / NS, slice = blockIdx.x % NS;
    const int t_base = chunk * kChunk, col0 = slice * kDownCols;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, q = lane >> 4, c = lane & 15;

    for (int i = tid; i < kChunk * kDownCols; i += kThreads) {
        const int row = i / kDownCols, col = i % kDownCols;
        Y[row * kDownStride + col] = b_down ? (float)b_down[col0 + col] : 0.0f;
    }

    const int g_lo = chunk * kChunkGroups;
    const int g_hi = min(g_lo + kChunkGroups, NG);
    // A operand rows: output columns wave*32 + nt*16 + c of this slice, k = 8q..8q+7 (+32 ks)
    const __bf16* wbase = w2t + (size_t)(col0 + wave * 32 + c) * m_pad + 8 * q;
    float* ybase = Y + wave * 32 + 4 * q;  // + lrow * kDownStride + nt * 16

    for (int ebase = 0; ebase < E; ebase += kDownBatch) {
        __syncthreads();  // Y initialised / previous batch's tile list no longer read
        // ---- tile list of this batch: thread i < kDownBatch describes expert ebase + i
        int n = 0, p0 = 0;
        const int e_mine = ebase + tid;
        if (tid < kDownBatch && e_mine < E) {
            const int lo = group_off[(size_t)g_lo * E + e_mine];
            n = group_off[(size_t)g_hi * E + e_mine] - lo;
            p0 = offsets[e_mine] + lo;
        }
        const int nt_mine = (n + 31) >> 5;
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
            tiles[start + k] = make_int2(p0 + 32 * k, (e_mine << 8) | min(32, n - 32 * k));
        __syncthreads();

        // ---- walk the tiles with a ring of kDepth tiles of operands in flight
        bf16x8 a_st[kDepth][2][KS], b_st[kDepth][2][KS];
        int tok_st[kDepth][2], rows_st[kDepth];
        // Issues the loads only; nothing here waits on them (token ids stay raw until the tile
        // is consumed), so kDepth tiles of loads overlap.  Tiles past the end reload the last
        // one with rows = 0.
        auto fetch = [&](int ti, bf16x8 (&a)[2][KS], bf16x8 (&b)[2][KS], int (&tok)[2],
                         int& rows_out) {
            const int2 ent = tiles[min(ti, ntiles - 1)];
            const int rows = ent.y & 0xff, e = ent.y >> 8;
            const __bf16* wp = wbase + (size_t)e * d * m_pad;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = ent.x + min(16 * h + c, rows - 1);
                const __bf16* hp = H + (size_t)row * m_pad + 8 * q;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    a[h][ks] = load8(wp + (size_t)h * 16 * m_pad + 32 * ks);
                    b[h][ks] = load8(hp + 32 * ks);
                }
                tok[h] = lists[row];
            }
            rows_out = ti < ntiles ? rows : 0;
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
                const int rows = rows_st[st];
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
                int lrow0 = tok_st[st][0] - t_base, lrow1 = tok_st[st][1] - t_base;
                // Pin the MFMAs and the token reads here (an empty asm the optimiser cannot move
                // values across): otherwise they sink below the refill, the old and the new
                // operands of the stage overlap and the ring turns into register copies that
                // wait on loads just issued.  The refill then reuses the stage's registers.
                asm volatile("" : "+v"(acc[0][0]), "+v"(acc[0][1]), "+v"(acc[1][0]), "+v"(acc[1][1]),
                                  "+v"(lrow0), "+v"(lrow1));
                __builtin_amdgcn_sched_barrier(0);
                fetch(t0 + st + kDepth, a_st[st], b_st[st], tok_st[st], rows_st[st]);

                // lane (q, c) of tile (nt, tt): columns nt*16 + 4q .. +3 of token tt*16 + c
                const int lrow[2] = {lrow0, lrow1};
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    if (16 * tt + c < rows && (unsigned)lrow[tt] < (unsigned)kChunk) {
                        float4* yp = reinterpret_cast<float4*>(ybase + lrow[tt] * kDownStride);
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
    const size_t lds = kDownLds;
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

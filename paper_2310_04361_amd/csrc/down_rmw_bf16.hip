// bf16 down-projection and merge for SPARSE selections: work proportional to the executed
// (token, expert) pairs (Sec. 3.2; the merge the paper's kernel does with global atomics).
//
// down_bf16.hip sums over experts inside the matrix cores at a cost that does not depend on how
// many experts a token selected; for H rows of 64 or 128 neurons it is cheaper, below a density
// of a few per cent, to touch only the executed rows (see down_max_pairs_sparse for the measured
// crossovers).  Where both could apply, both kernels are launched; each reads the pair count that
// the list-building kernel left in offsets[E] and the one that does not apply exits at once, so
// no host synchronisation is needed to choose.
//
// One workgroup per (128-token chunk, 256-column slice); KS = m_pad / 32 MFMA k-steps.
// The fp32 output tile Y[128][256] lives in LDS.  The eight wavefronts own 32 columns each, so
// no two wavefronts ever touch the same element and the merge is a plain read-add-write (LDS
// float atomics proved far slower).  All wavefronts walk the same list of tiles -- up to 32
// consecutive rows of one expert's part of H, all belonging to this chunk -- built once per
// batch of experts from the group offsets.
// Per tile and wavefront: D[32 cols][32 rows] = W2 slice * H_tile^T as 2 x 2 MFMA 16x16x32
// tiles with the tokens on the MFMA column axis, so a lane ends up with four consecutive output
// columns of ONE token: one 16-byte LDS read and write per MFMA tile, one row address per
// token.  The row stride of 260 floats spreads consecutive-token rows over the banks.
// Operands of the next kDepth tiles are kept in flight while the current one is merged.
// Weights: the 16x16x32 fragments w2f (also used by the small-token path); H rows as written by
// the up kernel (16-byte piece 4ks + q of a row = neurons 8(4ks + q) .. +7 = the k values of lane
// group q in k-step ks).
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

constexpr int kDownWaves = 8;
constexpr int kDownCols = kDownWaves * 32;     // output columns per workgroup
constexpr int kDownBatch = 128;                // experts per tile-list batch
constexpr int kDownTilesPerExpert = (kChunk + 31) / 32;       // 32-row tiles per (chunk, expert)
constexpr int kDownStride = kDownCols + 4;     // LDS row stride in floats
constexpr size_t kDownLds = sizeof(float) * kChunk * kDownStride +
                            sizeof(int2) * kDownBatch * kDownTilesPerExpert;

template <int KS>
__global__ __launch_bounds__(kDownWaves * 64) void down_rmw_bf16_kernel(
    const __bf16* __restrict__ w2f, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ item_start, const int32_t* __restrict__ group_off,
    const int32_t* __restrict__ alist, const int32_t* __restrict__ offsets,
    const __bf16* __restrict__ Hf, __bf16* __restrict__ y, int T, int d, int E, int NG,
    int rows_per_item, long long max_pairs) {
    if (offsets[E] > max_pairs) return;  // dense enough for the other kernel (uniform)
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
                row0 = item_start[e_mine] * rows_per_item + lo;  // row of H / alist
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
        // A tile is up to 32 consecutive rows of H that all belong to this chunk.  Lanes past
        // the tile's last row read row 0 of the tile again and skip the merge.  Tiles past the
        // end repeat the last one with no rows.
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
                const __bf16* hp = Hf + (size_t)row * (KS * 32) + 8 * q;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    a[h][ks] = load8(wp + (h * KS + ks) * 512);
                    b[h][ks] = load8(hp + ks * 32);
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


template <int KS>
void launch_down_rmw_t(const dmoe_layer& L, const PackedLayout& P, int T, const int32_t* item_start,
                       const int32_t* group_off, const int32_t* alist, const int32_t* offsets,
                       const void* H, void* y, long long max_pairs, hipStream_t s) {
    const int NG = div_up(T, kGroup), NC = div_up(T, kChunk), NS = L.d_model / kDownCols;
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&down_rmw_bf16_kernel<KS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDownLds);
    });
    const char* pk = static_cast<const char*>(L.packed);
    launch_kernel(down_rmw_bf16_kernel<KS>, round_up(NC, 8) * NS, kDownWaves * 64, kDownLds, s, 
        (const __bf16*)(pk + P.w2f), (const __bf16*)L.b_down, item_start, group_off, alist, offsets,
        (const __bf16*)H, (__bf16*)y, T, L.d_model, L.n_experts, NG, up_rows_bf16(L), max_pairs);
}

}  // namespace

// Density (executed pairs / (T * E)) up to which the pair-proportional kernel is the faster one.
// Measured crossovers: about 0.03 for H rows of 64 or 128 neurons (4096 tokens x 256 gated
// experts of 64, d = 2048; 50432 tokens x 24 experts of 128, d = 768); with 32-neuron rows the
// matrix-core kernel wins at every density (16384 tokens x 128 experts of 24: 59 us against 81 us
// at 1 %), so this kernel is not launched there at all.  Sizes that the matrix-core kernel
// cannot address all go to this one.
long long down_max_pairs_sparse(const dmoe_layer& L, int T) {
    if (!down_bf16_addressable(L, T)) return 0x7fffffffffffffffLL;
    const double dens = m_pad_of(L.expert_size) <= 32 ? 0.0 : 0.03;
    return (long long)(dens * (double)T * (double)L.n_experts);
}

void launch_down_rmw_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                          const int32_t* group_off, const int32_t* alist, const int32_t* offsets,
                          const void* H, void* y, long long max_pairs, hipStream_t s) {
    LaunchTimer tm(kSlotDownRmw, s);
    const PackedLayout P = packed_layout(L);
    const int ks = m_pad_of(L.expert_size) / 32;
    if (ks == 1) launch_down_rmw_t<1>(L, P, T, item_start, group_off, alist, offsets, H, y, max_pairs, s);
    else if (ks == 2) launch_down_rmw_t<2>(L, P, T, item_start, group_off, alist, offsets, H, y, max_pairs, s);
    else launch_down_rmw_t<4>(L, P, T, item_start, group_off, alist, offsets, H, y, max_pairs, s);
}

}  // namespace dmoe

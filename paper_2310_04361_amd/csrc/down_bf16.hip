// bf16 down-projection and merge, y_t = b_down + sum over the selected experts of W_down,e^T h
// (Sec. 3.2; gated experts Appendix G), with the sum over experts taken INSIDE the matrix cores.
//
// The merge of expert outputs is what the paper's own kernel does with global atomics.  Here a
// wavefront owns a block of 128 tokens x 64 output columns as fp32 MFMA accumulators for the
// whole kernel and walks all experts.  For one expert it multiplies the expert's 64-column
// slice of W_down (A operand, M axis = columns) with a 32-token tile of hidden activations
// (B operand, N axis = tokens) in which the tokens that did not select the expert are ZERO
// columns.  A zero column adds nothing, so the accumulator of token t ends up with exactly the
// sum over t's selected experts, in ascending expert order (run-to-run reproducible), and every
// y element is written once.  No scatter, no atomics, no fp32 tile in LDS.
//
// Dense k-packing.  An H row is a sequence of 16-byte pieces of eight consecutive neurons; an
// expert of m neurons fills PG = ceil(m / 8) of them.  The MFMA k-step is 16 = two pieces, and
// the pieces of G consecutive experts (a "stage": G = 2 when PG is odd) are laid end to end, so
// that a stage takes KSP = G * PG / 2 k-steps with no padded neurons: lane half h of k-step s
// works on piece 2s + h of the stage.  Experts of 24 neurons cost 3 k-steps per pair instead of
// 4.  The two halves of one k-step may thus belong to different experts, each with its own
// selection.
//
// Building the B tiles.  H holds one row per executed (token, expert) pair, expert-major, rows
// ascending in token id, so the rows of one 64-token select group are consecutive:
// row0(e, group) + rank of the token among the group's selected tokens.  The four wavefronts of
// a workgroup share the work: wavefront w takes select group (w & 1) of the chunk with
// lane = token and the lane half (w >> 1) of every k-step; per expert it tests the token's mask
// bit and ranks it with a ballot, and fetches its pieces with buffer loads whose offset is
// pushed out of range for unselected tokens -- the hardware returns zeros for those and moves no
// data.  The pieces go to LDS in MFMA operand order; after one barrier every wavefront reads
// the four finished tiles.
//
// Pipeline.  Work advances in phases of 8 MFMAs (one k-step of one stage for the wavefront's
// 4 token tiles x 2 column tiles).  The first phase of stage n writes the tiles of stage n+1
// (fetched two stages earlier) to LDS buffer (n+1) % 3 and issues the fetch for stage n+3; every
// phase requests the weight blocks of the phase R-1 ahead and reads from LDS the B operands of
// the next phase; the one barrier per stage sits in the middle of its MFMAs.  Three buffers keep
// a wavefront that runs ahead from overwriting tiles that a slower one still reads.  Everything
// but the MFMAs is cut into pieces pinned between them (see the loop).
//
// Operand layouts (v_mfma_f32_32x32x16_bf16, lane = 32h + c):
//   B tile (32 tokens, k-step s): lane (h, c) holds piece 2s + h of the stage for token c.
//   w2g[stage][d/32][KSP][64][8]: lane (h, r) of block (stage, column tile, s) holds the same
//     eight neurons for output column 32*tile + 16*((r>>2)&1) + 4*(r>>3) + (r&3).  With that
//     column order the 16 accumulator registers of lane (h, c) are the 16 CONSECUTIVE columns
//     16h .. 16h+15 of token c, so y goes out in 16-byte stores.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDnTokens = 128;  // tokens per workgroup: 4 tiles of 32 = 2 select groups of 64
constexpr int kDnTiles = 4;
constexpr int kDnCols = 256;    // columns per workgroup: 4 wavefronts x 64
constexpr int kDnBuffers = 3;

// Pieces per expert (padded up to a supported count), experts per stage, k-steps per stage.
struct DownPacking {
    int PG, G, KSP;
};
DownPacking down_packing(int m) {
    static const int kCounts[] = {2, 3, 4, 6, 8, 12, 16};
    int pg = div_up(m, 8);
    for (int v : kCounts)
        if (pg <= v) {
            pg = v;
            break;
        }
    const int g = (pg == 2 || (pg & 1)) ? 2 : 1;  // an even number of pieces, at least two k-steps
    return DownPacking{pg, g, g * pg / 2};
}

__global__ void pack_down32_kernel(const __bf16* __restrict__ w_down, __bf16* __restrict__ w2g,
                                   int E, int m, int d, int PG, int G, int KSP) {
    const int n_stages = (E + G - 1) / G;
    const size_t n = (size_t)n_stages * (d / 32) * KSP * 512;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int s8 = (int)(i & 7), lane = (int)((i >> 3) & 63);
        size_t f = i >> 9;
        const int s = (int)(f % KSP);
        f /= KSP;
        const int ct = (int)(f % (d / 32));
        const int st = (int)(f / (d / 32));
        const int h = lane >> 5, r = lane & 31;
        const int col = 32 * ct + 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
        const int pi = 2 * s + h;                   // piece of the stage
        const int e = st * G + pi / PG, neuron = 8 * (pi % PG) + s8;
        w2g[i] = (e < E && neuron < m) ? w_down[((size_t)e * m + neuron) * d + col] : (__bf16)0.0f;
    }
}

constexpr int const_gcd(int a, int b) { return b == 0 ? a : const_gcd(b, a % b); }

// KSP k-steps per stage of G experts (PG = 2*KSP/G pieces each); R = weight sets in flight;
// WPS = wavefronts per SIMD the register budget is cut for.
template <int KSP, int G, int R, int WPS>
__global__ __launch_bounds__(256, WPS) void down_bf16_kernel(
    const __bf16* __restrict__ w2g, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ item_start, const int32_t* __restrict__ group_off,
    const uint32_t* __restrict__ mask32, const int32_t* __restrict__ offsets,
    const __bf16* __restrict__ H, __bf16* __restrict__ y, int T, int d, int E, int NG, int W32,
    int rows_per_item, int row_bytes, long long max_pairs_sparse) {
    if (offsets[E] <= max_pairs_sparse) return;  // sparse enough for the pair-proportional kernel
    constexpr int PG = 2 * KSP / G;                  // pieces per expert
    constexpr int kImage = kDnTiles * KSP * 1024;    // the B tiles of one stage
    extern __shared__ __attribute__((aligned(16))) char img[];  // [kDnBuffers][kImage]
    // The column slices of one chunk share its H rows: keep them on one XCD (workgroups are dealt
    // round-robin to the 8 XCDs) and next to each other in launch order.
    const int NS = d / kDnCols;
    const int k_in_xcd = blockIdx.x >> 3;
    const int chunk = (k_in_xcd / NS) * 8 + (blockIdx.x & 7), slice = k_in_xcd % NS;
    const int t_base = chunk * kDnTokens;
    if (t_base >= T) return;  // the grid is rounded up to whole groups of 8 chunks
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, c = lane & 31;
    const int col_w = slice * kDnCols + wave * 64;
    const int n_stages = (E + G - 1) / G;

    // ---- tile-building role: select group bg of the chunk (lane = token), lane half bh
    const int bg = wave & 1, bh = wave >> 1;
    const int g = chunk * 2 + bg;
    const int tok_b = g * kGroup + lane;
    const bool tok_ok = tok_b < T;
    const uint32_t* mrow = mask32 + (size_t)min(tok_b, T - 1) * W32;
    const int32_t* grow = group_off + (size_t)min(g, NG) * E;  // group_off has NG + 1 rows
    // per batch of 32 experts: this token's mask word, and in lane i the first H row of
    // (expert 32b + i, group g)
    // Nothing below sits under a condition that depends on the expert: a load inside a
    // conditional region makes the compiler's wait-count bookkeeping assume the worst at the
    // join, and the stage would wait for the loads it has just issued.  Past the last expert the
    // same code runs on clamped addresses with every token unselected.
    const int n_batches = (E + 31) >> 5;
    uint32_t mw = 0u, mw_next = 0u;
    int rowv = 0, is_next = 0, go_next = 0;
    auto load_batch = [&](int b, uint32_t& m_out, int& is_out, int& go_out) {
        m_out = tok_ok ? mrow[b] : 0u;
        const int ec = min(32 * b + c, E - 1);
        is_out = item_start[ec];
        go_out = grow[ec];
    };
    u32x4 breg[2][KSP];  // H pieces of two stages in flight
    __amdgpu_buffer_rsrc_t b_rsrc[G];
    uint32_t b_voff[G];
#pragma unroll
    for (int eo = 0; eo < G; ++eo) {
        b_rsrc[eo] = __builtin_amdgcn_make_buffer_rsrc((void*)H, 0, 0, 0x00020000);
        b_voff[eo] = 0x80000000u;
    }
    auto build_prepare = [&](int e, int eo) {  // called with e = 0, 1, 2, ... in this order
        if ((e & 31) == 0) {                   // the values fetched 32 experts ago become current
            if (e > 0) {
                mw = mw_next;
                rowv = is_next * rows_per_item + go_next;
            }
            load_batch(min((e >> 5) + 1, n_batches - 1), mw_next, is_next, go_next);
        }
        const bool sel = ((mw >> (e & 31)) & 1u) != 0u && e < E;
        const uint64_t bal = __ballot(sel);
        const int rank = __builtin_amdgcn_mbcnt_hi(
            (uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
        const int row0 = __builtin_amdgcn_readlane(rowv, e & 31);
        // at most 64 rows of this expert belong to the group; unselected tokens get an offset
        // beyond the descriptor's range, for which the load returns zeros
        b_rsrc[eo] = __builtin_amdgcn_make_buffer_rsrc(
            (void*)((const char*)H + (size_t)row0 * row_bytes), 0, kGroup * row_bytes, 0x00020000);
        b_voff[eo] = sel ? (uint32_t)(rank * row_bytes) : 0x80000000u;
    };
    auto build_fetch = [&](u32x4 (&br)[KSP]) {
#pragma unroll
        for (int s = 0; s < KSP; ++s) {
            const int pi = 2 * s + bh;  // piece of the stage (uniform per wavefront)
            const int eo = G == 1 ? 0 : pi / PG, p = pi - eo * PG;
            br[s] = __builtin_amdgcn_raw_buffer_load_b128(
                eo ? b_rsrc[G - 1] : b_rsrc[0], (eo ? b_voff[G - 1] : b_voff[0]) + 16 * p, 0, 0);
        }
    };
    // lane = token 32h + c of the group: tile 2bg + h of the chunk, operand lane (bh, c)
    char* const wdst = img + (((2 * bg + h) * KSP) * 64 + 32 * bh + c) * 16;
    auto write_tiles = [&](int buf, const u32x4 (&br)[KSP]) {
#pragma unroll
        for (int s = 0; s < KSP; ++s)
            *reinterpret_cast<u32x4*>(wdst + buf * kImage + s * 1024) = br[s];
    };

    // ---- multiplying role: 128 tokens x columns col_w .. col_w + 63
    const __bf16* const wsrc = w2g + ((size_t)(col_w / 32) * KSP * 64 + lane) * 8;
    const size_t w_stage_stride = (size_t)(d / 32) * KSP * 512;
    // Work advances in phases: phase p = stage p / KSP, k-step p % KSP = 8 MFMAs (4 token tiles x
    // 2 column tiles) that need two 1 KiB weight blocks.  R weight sets are in flight, so a block
    // is requested R - 1 phases before its use whatever the expert size (the weights of a stage
    // reach all workgroups of an XCD at about the same time, so nearly every request is answered
    // from beyond L2).  A loop trip is an even number of stages, so that the two register sets
    // of the H fetch simply alternate.
    constexpr int PH = R * (2 * KSP) / const_gcd(R, 2 * KSP);  // phases per loop trip
    auto load_phase = [&](int p, bf16x8 (&a)[2]) {
        const int st = min(p / KSP, n_stages - 1), ks = p % KSP;
        const __bf16* src = wsrc + (size_t)st * w_stage_stride + ks * 512;
        a[0] = load8(src);
        a[1] = load8(src + KSP * 512);
    };
    f32x16 acc[kDnTiles][2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float bias = b_down ? (float)b_down[col_w + 32 * ct + 16 * h + i] : 0.0f;
#pragma unroll
            for (int j = 0; j < kDnTiles; ++j) acc[j][ct][i] = bias;
        }
    }
    const char* const rsrc_l = img + lane * 16;
    // k-step ks of token tile j of the stage in buffer buf
    auto read_piece = [&](int buf, int ks, int j) {
        return *reinterpret_cast<const bf16x8*>(rsrc_l + buf * kImage + (j * KSP + ks) * 1024);
    };
    auto next_buf = [](int buf) { return buf == kDnBuffers - 1 ? 0 : buf + 1; };
    auto prepare_stage = [&](int st) {
#pragma unroll
        for (int eo = 0; eo < G; ++eo) build_prepare(st * G + eo, eo);
    };

    bf16x8 aw[R][2];
    bf16x8 bb[2][kDnTiles];  // B operands of the current phase and of the next one
    {
        int is0, go0;
        load_batch(0, mw, is0, go0);
        rowv = is0 * rows_per_item + go0;
    }
    // Same issue order as in the loop (H fetch first, then the weight loads): the wait before an
    // LDS write is computed for the worse of the two ways into the loop, and with the fetch
    // issued last here it would wait for every load in flight on every trip.
    prepare_stage(0);
    build_fetch(breg[0]);
    write_tiles(0, breg[0]);
    prepare_stage(1);
    build_fetch(breg[1]);
    prepare_stage(2);
    build_fetch(breg[0]);
#pragma unroll
    for (int q = 0; q < R - 1; ++q) load_phase(q, aw[q]);
    lds_barrier();
#pragma unroll
    for (int j = 0; j < kDnTiles; ++j) bb[0][j] = read_piece(0, 0, j);
    int buf = 0;
    // Per stage: its first phase writes the tiles of the NEXT stage to LDS and issues the fetch
    // for the one three ahead (the H rows come from beyond L2: fetched only one stage's MFMA
    // time ahead they were waited for on every stage); the barrier sits in the middle of the
    // stage's MFMAs.  Every phase first issues its weight loads and the LDS reads of the NEXT
    // phase's B operands (k-step 0 of the next stage in the last phase: the barrier has passed
    // by then), then runs its 8 MFMAs on operands requested a phase ago.  So the LDS write, the
    // barrier and all LDS reads overlap with matrix work of the same wavefront.  A trip past
    // the last stage multiplies zero tiles.
    for (int s0 = 0; s0 < n_stages; s0 += PH / KSP) {
#pragma unroll
        for (int q = 0; q < PH; ++q) {
            const int st = s0 + q / KSP;
            const int ks = q % KSP;
            const int nb = next_buf(buf);
            const int rbuf = ks < KSP - 1 ? buf : nb, rks = ks < KSP - 1 ? ks + 1 : 0;
            u32x4 (&br)[KSP] = breg[(q / KSP + 1) & 1];  // tiles of stage st + 1 now, then of st + 3
            // A wavefront issues in order, and an MFMA keeps the matrix pipe busy for 32 cycles
            // only: everything else the phase has to do is cut into pieces that sit BETWEEN its
            // MFMAs, each pinned by a scheduling barrier.  Left alone the scheduler groups the
            // pieces (the pipe idles meanwhile), sinks the H fetch to the end of the stage
            // (loads complete in issue order, so the next LDS write would wait for everything)
            // and issues each LDS read just before its use.
            auto mf = [&](int j, int ct) {
                acc[j][ct] = mfma32(aw[q % R][ct], bb[q & 1][j], acc[j][ct]);
                __builtin_amdgcn_sched_barrier(0);
            };
            __builtin_amdgcn_sched_barrier(0);
            if (ks == 0) write_tiles(nb, br);
            mf(0, 0);
            if (ks == 0) build_prepare((st + 3) * G, 0);
            mf(0, 1);
            if (ks == 0 && G == 2) build_prepare((st + 3) * G + 1, G - 1);
            mf(1, 0);
            if (ks == 0) build_fetch(br);
            load_phase(s0 * KSP + q + R - 1, aw[(q + R - 1) % R]);
            mf(1, 1);
            bb[(q + 1) & 1][0] = read_piece(rbuf, rks, 0);
            bb[(q + 1) & 1][1] = read_piece(rbuf, rks, 1);
            mf(2, 0);
            bb[(q + 1) & 1][2] = read_piece(rbuf, rks, 2);
            bb[(q + 1) & 1][3] = read_piece(rbuf, rks, 3);
            mf(2, 1);
            mf(3, 0);
            mf(3, 1);
            if (ks == (KSP >> 1) - 1) lds_barrier();  // every wavefront has written its part of st + 1
            if (ks == KSP - 1) buf = nb;
        }
    }

    // lane (h, c) of tile (j, ct): columns col_w + 32ct + 16h .. +15 of token t_base + 32j + c
#pragma unroll
    for (int j = 0; j < kDnTiles; ++j) {
        const int t = t_base + 32 * j + c;
        if (t < T) {
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                bf16x8 o0, o1;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    o0[i] = (__bf16)acc[j][ct][i];
                    o1[i] = (__bf16)acc[j][ct][8 + i];
                }
                __bf16* dst = y + (size_t)t * d + col_w + 32 * ct + 16 * h;
                *reinterpret_cast<bf16x8*>(dst) = o0;
                *reinterpret_cast<bf16x8*>(dst + 8) = o1;
            }
        }
    }
}

template <int KSP, int G, int R, int WPS>
void launch_down_t(const dmoe_layer& L, const PackedLayout& P, int T, const int32_t* item_start,
                   const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                   const void* H, void* y, long long max_pairs_sparse, hipStream_t s) {
    const int NG = div_up(T, kGroup), NC = div_up(T, kDnTokens), NS = L.d_model / kDnCols;
    constexpr size_t lds = (size_t)kDnBuffers * kDnTiles * KSP * 1024;
    static bool attr_set = false;  // per-function, idempotent: allow more than 64 KiB of LDS
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&down_bf16_kernel<KSP, G, R, WPS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const char* pk = static_cast<const char*>(L.packed);
    down_bf16_kernel<KSP, G, R, WPS><<<round_up(NC, 8) * NS, 256, lds, s>>>(
        (const __bf16*)(pk + P.w2g), (const __bf16*)L.b_down, item_start, group_off,
        reinterpret_cast<const uint32_t*>(mask), offsets, (const __bf16*)H, (__bf16*)y, T,
        L.d_model, L.n_experts, NG, 2 * div_up(L.n_experts, 64), up_rows_bf16(L),
        2 * m_pad_of(L.expert_size), max_pairs_sparse);
}

}  // namespace

bool down_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    return (mp == 32 || mp == 64 || mp == 128) && L.d_model % kDnCols == 0;
}

void launch_pack_down_bf16(const dmoe_layer& L, void* w2g, hipStream_t s) {
    const DownPacking dp = down_packing(L.expert_size);
    pack_down32_kernel<<<2048, 256, 0, s>>>((const __bf16*)L.w_down, (__bf16*)w2g, L.n_experts,
                                            L.expert_size, L.d_model, dp.PG, dp.G, dp.KSP);
}

void launch_down_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                      const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                      const void* H, void* y, long long max_pairs_sparse, hipStream_t s) {
    LaunchTimer tm(kSlotDown, s);
    const PackedLayout P = packed_layout(L);
    const DownPacking dp = down_packing(L.expert_size);
    // at most one workgroup per CU: a wavefront may use the whole register file of its SIMD, which
    // buys a deeper ring of weight sets
    const bool one_per_cu = div_up(T, kDnTokens) * (L.d_model / kDnCols) <= 256;
#define DMOE_DOWN(KSP_, G_, R_, WPS_) \
    launch_down_t<KSP_, G_, R_, WPS_>(L, P, T, item_start, group_off, mask, offsets, H, y, max_pairs_sparse, s)
#define DMOE_DOWN_BY_GRID(KSP_, G_, R2_)            \
    do {                                            \
        if (one_per_cu) DMOE_DOWN(KSP_, G_, 16, 1); \
        else DMOE_DOWN(KSP_, G_, R2_, 2);           \
    } while (0)
    if (dp.KSP == 2 && dp.G == 2) DMOE_DOWN_BY_GRID(2, 2, 8);
    else if (dp.KSP == 2) DMOE_DOWN_BY_GRID(2, 1, 8);
    else if (dp.KSP == 3 && dp.G == 2) DMOE_DOWN_BY_GRID(3, 2, 4);
    else if (dp.KSP == 3) DMOE_DOWN_BY_GRID(3, 1, 4);
    else if (dp.KSP == 4) DMOE_DOWN_BY_GRID(4, 1, 4);
    else if (dp.KSP == 6) DMOE_DOWN_BY_GRID(6, 1, 4);
    else DMOE_DOWN(8, 1, 8, 1);
#undef DMOE_DOWN_BY_GRID
#undef DMOE_DOWN
}

}  // namespace dmoe

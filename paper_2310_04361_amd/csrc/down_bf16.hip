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
// Building the B tiles.  H holds one row of m_pad activations per executed (token, expert) pair,
// expert-major, rows ascending in token id, so the rows of one 64-token select group are
// consecutive: row0(e, group) + rank of the token among the group's selected tokens.  The four
// wavefronts of a workgroup share the work: wavefront w takes select group (w & 1) of the chunk
// with lane = token, tests the token's mask bit, ranks it with a ballot, and fetches half
// (w >> 1) of its H row with buffer loads whose offset is pushed out of range for unselected
// tokens -- the hardware returns zeros for those and moves no data.  The pieces go to LDS in
// MFMA operand order; after one barrier every wavefront reads the four finished tiles.
//
// Pipeline.  Work advances in phases of 8 MFMAs (one k-step of one expert for the wavefront's
// 4 token tiles x 2 column tiles).  The first phase of expert e writes the tiles of e+1 (fetched
// one expert earlier) to LDS buffer (e+1) % 3 and issues the fetch for e+2; every phase requests
// the weight blocks of the phase R-1 ahead and reads from LDS the B operands of the next phase;
// the one barrier per expert sits in the middle of its MFMAs.  Three buffers keep a wavefront
// that runs ahead from overwriting tiles that a slower one still reads.  What is left over the
// pure MFMA time is mostly the wait for the H fetch, whose latency exceeds one expert's MFMA
// time while loads complete in issue order.
//
// Operand layouts (v_mfma_f32_32x32x16_bf16, lane = 32h + c):
//   H row: 2*KS2 pieces of 16 bytes, piece p = neurons 8p .. 8p+7.
//   B tile (32 tokens, k-step s): lane (h, c) holds piece h*KS2 + s of token c's row.
//   w2g[E][d/32][KS2][64][8]: lane (h, r) of block (e, column tile, s) holds the same neurons
//     for output column 32*tile + 16*((r>>2)&1) + 4*(r>>3) + (r&3).  With that column order the
//     16 accumulator registers of lane (h, c) are the 16 CONSECUTIVE columns 16h .. 16h+15 of
//     token c, so y goes out in 16-byte stores.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDnTokens = 128;  // tokens per workgroup: 4 tiles of 32 = 2 select groups of 64
constexpr int kDnTiles = 4;
constexpr int kDnCols = 256;    // columns per workgroup: 4 wavefronts x 64
constexpr int kDnBuffers = 3;

__global__ void pack_down32_kernel(const __bf16* __restrict__ w_down, __bf16* __restrict__ w2g,
                                   int E, int m, int d, int KS2) {
    const size_t n = (size_t)E * (d / 32) * KS2 * 512;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int s8 = (int)(i & 7), lane = (int)((i >> 3) & 63);
        size_t f = i >> 9;
        const int s = (int)(f % KS2);
        f /= KS2;
        const int ct = (int)(f % (d / 32));
        const int e = (int)(f / (d / 32));
        const int h = lane >> 5, r = lane & 31;
        const int col = 32 * ct + 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
        const int neuron = 8 * (h * KS2 + s) + s8;  // piece h*KS2 + s of the H row
        w2g[i] = neuron < m ? w_down[((size_t)e * m + neuron) * d + col] : (__bf16)0.0f;
    }
}

// KS2 = m_pad / 16 MFMA k-steps per expert; R = weight sets in flight (see below); WPS = wavefronts
// per SIMD the register budget is cut for.
template <int KS2, int R, int WPS>
__global__ __launch_bounds__(256, WPS) void down_bf16_kernel(
    const __bf16* __restrict__ w2g, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ item_start, const int32_t* __restrict__ group_off,
    const uint32_t* __restrict__ mask32, const int32_t* __restrict__ offsets,
    const __bf16* __restrict__ H, __bf16* __restrict__ y, int T, int d, int E, int NG, int W32,
    int rows_per_item, long long max_pairs_sparse) {
    if (offsets[E] <= max_pairs_sparse) return;  // sparse enough for the pair-proportional kernel
    constexpr int kRowBytes = KS2 * 32;              // one H row: m_pad bf16
    constexpr int kImage = kDnTiles * KS2 * 1024;    // the B tiles of one expert
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

    // ---- tile-building role: select group bg of the chunk (lane = token), row half bh
    const int bg = wave & 1, bh = wave >> 1;
    const int g = chunk * 2 + bg;
    const int tok_b = g * kGroup + lane;
    const bool tok_ok = tok_b < T;
    const uint32_t* mrow = mask32 + (size_t)min(tok_b, T - 1) * W32;
    const int32_t* grow = group_off + (size_t)min(g, NG) * E;  // group_off has NG + 1 rows
    // per batch of 32 experts: this token's mask word, and in lane i the first H row of
    // (expert 32b + i, group g)
    // Nothing below sits under a condition that depends on e: a load inside a conditional region
    // makes the compiler's wait-count bookkeeping assume the worst at the join, and the stage
    // would wait for the loads it has just issued.  Past the last expert the same code runs on
    // clamped addresses with every token unselected.
    const int n_batches = (E + 31) >> 5;
    uint32_t mw = 0u, mw_next = 0u;
    int rowv = 0, is_next = 0, go_next = 0;
    auto load_batch = [&](int b, uint32_t& m_out, int& is_out, int& go_out) {
        m_out = tok_ok ? mrow[b] : 0u;
        const int ec = min(32 * b + c, E - 1);
        is_out = item_start[ec];
        go_out = grow[ec];
    };
    u32x4 breg[2][KS2];  // H pieces of two experts in flight (fetched two experts ahead)
    __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)H, 0, 0, 0x00020000);
    uint32_t b_voff = 0x80000000u;
    auto build_prepare = [&](int e) {  // called with e = 0, 1, 2, ... in this order
        if ((e & 31) == 0) {           // the values fetched 32 experts ago become current
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
        b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(H + (size_t)row0 * (kRowBytes / 2)), 0,
                                                   kGroup * kRowBytes, 0x00020000);
        b_voff = sel ? (uint32_t)(rank * kRowBytes + bh * (kRowBytes / 2)) : 0x80000000u;
    };
    auto build_fetch = [&](u32x4 (&br)[KS2]) {
#pragma unroll
        for (int s = 0; s < KS2; ++s)
            br[s] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, b_voff + 16 * s, 0, 0);
    };
    // lane = token 32h + c of the group: tile 2bg + h of the chunk, operand lane (bh, c)
    char* const wdst = img + (((2 * bg + h) * KS2) * 64 + 32 * bh + c) * 16;
    auto write_tiles = [&](int buf, const u32x4 (&br)[KS2]) {
#pragma unroll
        for (int s = 0; s < KS2; ++s)
            *reinterpret_cast<u32x4*>(wdst + buf * kImage + s * 1024) = br[s];
    };

    // ---- multiplying role: 128 tokens x columns col_w .. col_w + 63
    const __bf16* const wsrc = w2g + ((size_t)(col_w / 32) * KS2 * 64 + lane) * 8;
    const size_t w_expert_stride = (size_t)(d / 32) * KS2 * 512;
    // Work advances in phases: phase p = expert p / KS2, k-step p % KS2 = 8 MFMAs (4 token tiles x
    // 2 column tiles) that need two 1 KiB weight blocks.  R weight sets are in flight, so a block
    // is requested R - 1 phases before its use whatever the expert size.  A loop trip is two
    // experts, so that the two register sets of the H fetch simply alternate.
    // The weights of an expert reach all workgroups of an XCD at about the same time, so nearly
    // every request is answered from beyond L2: R has to cover that latency.
    constexpr int PH = R > 2 * KS2 ? R : 2 * KS2;  // phases per loop trip (an even number of experts)
    auto load_phase = [&](int p, bf16x8 (&a)[2]) {
        const int e = min(p / KS2, E - 1), ks = p % KS2;
        const __bf16* src = wsrc + (size_t)e * w_expert_stride + ks * 512;
        a[0] = load8(src);
        a[1] = load8(src + KS2 * 512);
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
    // k-step ks of the four token tiles of the expert in buffer buf
    auto read_piece = [&](int buf, int ks, int j) {
        return *reinterpret_cast<const bf16x8*>(rsrc_l + buf * kImage + (j * KS2 + ks) * 1024);
    };
    auto read_pieces = [&](int buf, int ks, bf16x8 (&b)[kDnTiles]) {
#pragma unroll
        for (int j = 0; j < kDnTiles; ++j) b[j] = read_piece(buf, ks, j);
    };
    auto next_buf = [](int buf) { return buf == kDnBuffers - 1 ? 0 : buf + 1; };

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
    build_prepare(0);
    build_fetch(breg[0]);
    write_tiles(0, breg[0]);
    build_prepare(1);
    build_fetch(breg[1]);
    build_prepare(2);
    build_fetch(breg[0]);
#pragma unroll
    for (int q = 0; q < R - 1; ++q) load_phase(q, aw[q]);
    lds_barrier();
    read_pieces(0, 0, bb[0]);
    int buf = 0;
    // Per expert: its first phase writes the tiles of the NEXT expert to LDS and issues the fetch
    // for the one three ahead (the H rows come from beyond L2: fetched only one expert's MFMA
    // time ahead they were waited for on every expert); the barrier sits in the middle of the
    // expert's MFMAs.  Every phase first
    // issues its weight loads and the LDS reads of the NEXT phase's B operands (k-step 0 of the
    // next expert in the last phase: the barrier has passed by then), then runs its 8 MFMAs on
    // operands requested a phase ago.  So the LDS write, the barrier and all LDS reads overlap
    // with matrix work of the same wavefront.  A trip past the last expert multiplies zero tiles.
    for (int e0 = 0; e0 < E; e0 += PH / KS2) {
#pragma unroll
        for (int q = 0; q < PH; ++q) {
            const int e = e0 + q / KS2;
            u32x4 (&br)[KS2] = breg[(q / KS2 + 1) & 1];  // tiles of e + 1 now, then of e + 3
            const int ks = q % KS2;
            const int nb = next_buf(buf);
            const int rbuf = ks < KS2 - 1 ? buf : nb, rks = ks < KS2 - 1 ? ks + 1 : 0;
            // A wavefront issues in order, and an MFMA keeps the matrix pipe busy for 32 cycles
            // only: everything else the phase has to do is cut into pieces that sit BETWEEN its
            // MFMAs, each pinned by a scheduling barrier.  Left alone the scheduler groups the
            // pieces (the pipe idles meanwhile), sinks the H fetch to the end of the expert
            // (loads complete in issue order, so the next LDS write would wait for everything)
            // and issues each LDS read just before its use.
            auto mf = [&](int j, int ct) {
                acc[j][ct] = mfma32(aw[q % R][ct], bb[q & 1][j], acc[j][ct]);
                __builtin_amdgcn_sched_barrier(0);
            };
            __builtin_amdgcn_sched_barrier(0);
            if (ks == 0) write_tiles(nb, br);
            mf(0, 0);
            if (ks == 0) build_prepare(e + 3);
            mf(0, 1);
            if (ks == 0) build_fetch(br);
            mf(1, 0);
            load_phase(e0 * KS2 + q + R - 1, aw[(q + R - 1) % R]);
            mf(1, 1);
            bb[(q + 1) & 1][0] = read_piece(rbuf, rks, 0);
            bb[(q + 1) & 1][1] = read_piece(rbuf, rks, 1);
            mf(2, 0);
            bb[(q + 1) & 1][2] = read_piece(rbuf, rks, 2);
            bb[(q + 1) & 1][3] = read_piece(rbuf, rks, 3);
            mf(2, 1);
            mf(3, 0);
            mf(3, 1);
            if (ks == KS2 / 2 - 1) lds_barrier();  // every wavefront has written its part of e + 1
            if (ks == KS2 - 1) buf = nb;
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

template <int KS2, int R, int WPS>
void launch_down_t(const dmoe_layer& L, const PackedLayout& P, int T, const int32_t* item_start,
                   const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                   const void* H, void* y, long long max_pairs_sparse, hipStream_t s) {
    const int NG = div_up(T, kGroup), NC = div_up(T, kDnTokens), NS = L.d_model / kDnCols;
    constexpr size_t lds = (size_t)kDnBuffers * kDnTiles * KS2 * 1024;
    static bool attr_set = false;  // per-function, idempotent: allow more than 64 KiB of LDS
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&down_bf16_kernel<KS2, R, WPS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    const char* pk = static_cast<const char*>(L.packed);
    down_bf16_kernel<KS2, R, WPS><<<round_up(NC, 8) * NS, 256, lds, s>>>(
        (const __bf16*)(pk + P.w2g), (const __bf16*)L.b_down, item_start, group_off,
        reinterpret_cast<const uint32_t*>(mask), offsets, (const __bf16*)H, (__bf16*)y, T,
        L.d_model, L.n_experts, NG, 2 * div_up(L.n_experts, 64), up_rows_bf16(L), max_pairs_sparse);
}

}  // namespace

bool down_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    return (mp == 32 || mp == 64 || mp == 128) && L.d_model % kDnCols == 0;
}

void launch_pack_down_bf16(const dmoe_layer& L, void* w2g, hipStream_t s) {
    pack_down32_kernel<<<2048, 256, 0, s>>>((const __bf16*)L.w_down, (__bf16*)w2g, L.n_experts,
                                            L.expert_size, L.d_model, m_pad_of(L.expert_size) / 16);
}

void launch_down_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                      const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                      const void* H, void* y, long long max_pairs_sparse, hipStream_t s) {
    LaunchTimer tm(kSlotDown, s);
    const PackedLayout P = packed_layout(L);
    const int ks2 = m_pad_of(L.expert_size) / 16;
    // at most one workgroup per CU: a wavefront may use the whole register file of its SIMD, which
    // buys a deeper ring of weight sets
    const bool one_per_cu = div_up(T, kDnTokens) * (L.d_model / kDnCols) <= 256;
#define DMOE_DOWN(KS2_, R_, WPS_) \
    launch_down_t<KS2_, R_, WPS_>(L, P, T, item_start, group_off, mask, offsets, H, y, max_pairs_sparse, s)
    if (ks2 == 2 && one_per_cu) DMOE_DOWN(2, 16, 1);
    else if (ks2 == 2) DMOE_DOWN(2, 8, 2);
    else if (ks2 == 4 && one_per_cu) DMOE_DOWN(4, 16, 1);
    else if (ks2 == 4) DMOE_DOWN(4, 4, 2);
    else DMOE_DOWN(8, 8, 1);
#undef DMOE_DOWN
}

}  // namespace dmoe

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
// the pieces of G consecutive experts (a "stage": G = 2 when PG is odd or 2, G = 4 when PG = 1)
// are laid end to end, so that a stage takes KSP = G * PG / 2 k-steps with no padded neurons: lane half h of k-step s
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
constexpr int kDnColStep = 128;  // a workgroup covers CT * 128 columns: 4 wavefronts x CT tiles of 32

// Pieces per unit (padded up to a supported count), units per stage, k-steps per stage, units per
// expert.  A unit is an expert -- except that an expert of exactly 128 neurons is walked as two
// units of 64 (its weights ARE two experts of 64 laid end to end, its H rows two half rows): with
// 4 k-steps per stage instead of 8 the LDS tiles of a workgroup halve, two workgroups share a CU
// and one's start-up and output hide behind the other's loop.
struct DownPacking {
    int PG, G, KSP, UPE;
};
DownPacking down_packing(int m) {
    if (m == 128) return DownPacking{8, 1, 4, 2};
    static const int kCounts[] = {1, 2, 3, 4, 6, 8, 16};  // H rows are 32, 64 or 128 neurons wide
    int pg = div_up(m, 8);
    for (int v : kCounts)
        if (pg <= v) {
            pg = v;
            break;
        }
    // an even number of pieces, at least two k-steps
    const int g = pg == 1 ? 4 : ((pg == 2 || (pg & 1)) ? 2 : 1);
    return DownPacking{pg, g, g * pg / 2, 1};
}

__global__ void pack_down32_kernel(const void* __restrict__ w_down, const float* __restrict__ scales,
                                   int fp8, __bf16* __restrict__ w2g, int E, int m, int d, int PG,
                                   int G, int KSP, int UPE) {
    const int n_stages = (E * UPE + G - 1) / G;
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
        const int u = st * G + pi / PG;             // unit; unit u of expert e holds its neurons 8 PG u' ..
        const int e = u / UPE, neuron = 8 * PG * (u % UPE) + 8 * (pi % PG) + s8;
        w2g[i] = (e < E && neuron < m)
                     ? expert_weight(w_down, scales, fp8, 2, e, ((size_t)e * m + neuron) * d + col)
                     : (__bf16)0.0f;
    }
}

// Buffer descriptor flags of a raw (unstructured) buffer: offsets at or beyond num_records read
// as zero and move no data.
constexpr int kRawBuffer = 0x00020000;

constexpr int kDnTrip = 4;  // stages per loop trip = LDS buffers = H register sets

// KSP k-steps per stage of G experts (PG = 2*KSP/G pieces each); R = weight sets in flight
// (divides 4 KSP); WPS = wavefronts per SIMD the register budget is cut for; CT = column tiles
// per wavefront (2: the workgroup covers 256 columns; 3: 384 columns, 192 accumulator registers,
// one workgroup per CU only).
//
// Instruction count matters as much as latency here: with one wavefront per SIMD every
// instruction that is not an MFMA delays the next MFMA by about 4 cycles, and a wait inside a
// conditional block is computed for the worst path into it.  So the loop has no condition and
// few instructions: all global loads are buffer loads whose per-lane offsets are loop invariant
// (the moving part is one scalar offset); a loop trip is 4 stages, so every LDS address and
// register set is a compile-time constant; a token's mask word is shifted down by one bit per
// expert and replaced once per 32 experts BETWEEN two runs of the loop, by the word requested a
// run earlier; the MFMAs of a phase start with the operands that were requested last, so that
// one wait covers the phase.
template <int KSP, int G, int R, int WPS, int CT, int UPE = 1>
__global__ __launch_bounds__(256, WPS) void down_bf16_kernel(
    const __bf16* __restrict__ w2g, const __bf16* __restrict__ b_down,
    const int32_t* __restrict__ item_start, const int32_t* __restrict__ group_off,
    const uint32_t* __restrict__ mask32, const int32_t* __restrict__ offsets,
    const __bf16* __restrict__ H, __bf16* __restrict__ y, int T, int d, int E, int NG, int W32,
    int rows_per_item, int row_shift, uint32_t w_bytes, uint32_t h_bytes,
    long long max_pairs_sparse) {
    static_assert((kDnTrip * KSP) % R == 0 && 32 % (kDnTrip * G) == 0, "loop trip");
    static_assert(UPE == 1 || (UPE == 2 && G == 1), "two units per expert: one unit per stage");
    if (offsets[E] <= max_pairs_sparse) return;  // sparse enough for the pair-proportional kernel
    constexpr int PG = 2 * KSP / G;                  // pieces per expert
    constexpr int kImage = kDnTiles * KSP * 1024;    // the B tiles of one stage
    constexpr int PH = kDnTrip * KSP;                // phases per loop trip
    constexpr int kExpertsPerTrip = kDnTrip * G / UPE;
    constexpr int kTripsPerBatch = 32 / kExpertsPerTrip;
    extern __shared__ __attribute__((aligned(16))) char img[];  // [kDnTrip][kImage]
    // The column slices of one chunk share its H rows: keep them on one XCD (workgroups are dealt
    // round-robin to the 8 XCDs) and next to each other in launch order.
    constexpr int kDnCols = CT * kDnColStep;
    const int NS = d / kDnCols;
    const int k_in_xcd = blockIdx.x >> 3;
    const int chunk = (k_in_xcd / NS) * 8 + (blockIdx.x & 7), slice = k_in_xcd % NS;
    const int t_base = chunk * kDnTokens;
    if (t_base >= T) return;  // the grid is rounded up to whole groups of 8 chunks
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, c = lane & 31;
    const int col_w = slice * kDnCols + wave * (32 * CT);
    const int n_trips = (E * UPE + kDnTrip * G - 1) / (kDnTrip * G);

    // ---- tile-building role: select group bg of the chunk (lane = token), lane half bh
    const int bg = wave & 1, bh = wave >> 1;
    const int g = chunk * 2 + bg;
    const int tok_b = g * kGroup + lane;
    const bool tok_ok = tok_b < T;
    const uint32_t* mrow = mask32 + (size_t)min(tok_b, T - 1) * W32;
    const int32_t* grow = group_off + (size_t)min(g, NG) * E;  // group_off has NG + 1 rows
    // Per batch of 32 experts: this token's mask word (shifted down as the experts go by; zero
    // for a token beyond T and past the last expert: the words hold no bits from E up), and in
    // lane i the first H row of (expert 32b + i, group g).
    const int n_batches = (E + 31) >> 5;
    uint32_t mw, mw_next;
    int rowv, is_next, go_next;
    auto load_batch = [&](int b, uint32_t& m_out, int& is_out, int& go_out) {
        const int bc = min(b, n_batches - 1);
        m_out = mrow[bc];  // of a clamped token and batch: masked when it becomes current
        const int ec = min(32 * bc + c, E - 1);
        is_out = item_start[ec];
        go_out = grow[ec];
    };
    const __amdgpu_buffer_rsrc_t h_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)H, 0, (int)h_bytes, kRawBuffer);
    u32x4 breg[kDnTrip][KSP];  // H pieces of the stages in flight
    uint32_t b_voff[G];
    int sh_base = 0;  // position in the current batch of the first expert of the next trip
    // Byte offset of the token's H row of expert `sh` of the batch, or an offset beyond the buffer
    // (h_bytes is below 2^31) for an unselected token: the load returns zeros for those.
    auto build_prepare = [&](int sh, int eo) {
        const bool sel = (mw & 1u) != 0u;
        mw >>= 1;
        const uint64_t bal = __ballot(sel);
        const uint32_t rank = __builtin_amdgcn_mbcnt_hi(
            (uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
        const uint32_t row0 = (uint32_t)__builtin_amdgcn_readlane(rowv, sh);
        b_voff[eo] = ((row0 + rank) << row_shift) | (sel ? 0u : 0x80000000u);
    };
    // piece 2s + bh of the stage: expert (2s + bh) / PG of the stage, piece (2s + bh) % PG of its
    // row; the piece offset is a per-wavefront scalar
    uint32_t p_soff[KSP];
#pragma unroll
    for (int s = 0; s < KSP; ++s) p_soff[s] = 16u * (uint32_t)((2 * s + bh) % PG);
    // half: the unit of the expert (0, or 1 with two units per expert: the second half of the row)
    auto fetch_piece = [&](int s, u32x4 (&br)[KSP], int half) {
        const int eo0 = G == 1 ? 0 : (2 * s) / PG, eo1 = G == 1 ? 0 : (2 * s + 1) / PG;
        const uint32_t v = eo0 == eo1 ? b_voff[eo0] : (bh ? b_voff[eo1] : b_voff[eo0]);
        br[s] = __builtin_amdgcn_raw_buffer_load_b128(h_rsrc, v, p_soff[s] + (uint32_t)(half * PG * 16), 0);
    };
    auto build_fetch = [&](u32x4 (&br)[KSP], int half) {
#pragma unroll
        for (int s = 0; s < KSP; ++s) fetch_piece(s, br, half);
    };
    // lane = token 32h + c of the group: tile 2bg + h of the chunk, operand lane (bh, c)
    char* const wdst = img + (((2 * bg + h) * KSP) * 64 + 32 * bh + c) * 16;
    auto write_piece = [&](int buf, int s, const u32x4 (&br)[KSP]) {
        *reinterpret_cast<u32x4*>(wdst + buf * kImage + s * 1024) = br[s];
    };
    auto write_tiles = [&](int buf, const u32x4 (&br)[KSP]) {
#pragma unroll
        for (int s = 0; s < KSP; ++s) write_piece(buf, s, br);
    };

    // ---- multiplying role: 128 tokens x columns col_w .. col_w + 32 CT - 1
    // Work advances in phases: phase p = stage p / KSP, k-step p % KSP = 4 * CT MFMAs (4 token
    // tiles x CT column tiles) that need CT 1 KiB weight blocks.  R weight sets are in flight, so
    // a block is requested R - 1 phases before its use whatever the expert size (the weights of a
    // stage reach all workgroups of an XCD at about the same time, so nearly every request is
    // answered from beyond L2).  Past the last stage the offsets leave the buffer and the blocks
    // read as zero.
    const __amdgpu_buffer_rsrc_t w_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)w2g, 0, (int)w_bytes, kRawBuffer);
    uint32_t a_voff[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
        a_voff[ct] = (uint32_t)(((col_w / 32 + ct) * KSP * 64 + lane) * 16);
    const uint32_t w_stage_bytes = (uint32_t)(d / 32) * KSP * 1024;
    uint32_t a_stage = 0;  // byte offset of the stage the next weight request belongs to
    // requests the weights of the next phase in order, column tile by column tile; ks = its
    // k-step (compile-time)
    auto load_block = [&](int ks, int ct, bf16x8 (&a)[CT]) {
        a[ct] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(
                    w_rsrc, a_voff[ct] + (uint32_t)(ks & 3) * 1024u,
                    a_stage + (uint32_t)(ks >> 2) * 4096u, 0));
        if (ct == CT - 1 && ks == KSP - 1) a_stage += w_stage_bytes;
    };
    auto load_phase = [&](int ks, bf16x8 (&a)[CT]) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) load_block(ks, ct, a);
    };

    bf16x8 aw[R][CT];
    bf16x8 bb[2][kDnTiles];  // B operands of the current phase and of the next one
    // Start-up: the offsets and fetches of stages 0 .. 3, then the first weight requests (every H
    // fetch before the first weight request, as in the loop: the wait before an LDS write is
    // computed for the worse of the two ways into the loop).
    {
        int is0, go0;
        load_batch(0, mw, is0, go0);
        load_batch(1, mw_next, is_next, go_next);
        rowv = is0 * rows_per_item + go0;
        mw = tok_ok ? mw : 0u;
    }
    // (two units per expert: stage i is unit i & 1 of expert i / 2 of the trip, and the offsets
    // of an expert are computed once, before its first unit)
#pragma unroll
    for (int i = 0; i < kDnTrip; ++i) {
        if (UPE == 1) {
#pragma unroll
            for (int eo = 0; eo < G; ++eo) build_prepare(i * G + eo, eo);
        } else if ((i & 1) == 0) {
            build_prepare(i / 2, 0);
        }
        build_fetch(breg[i], UPE == 1 ? 0 : (i & 1));
    }
    sh_base = kExpertsPerTrip & 31;
#pragma unroll
    for (int q = 0; q < R - 1; ++q) load_phase(q % KSP, aw[q]);
    // every accumulator starts at the output bias: lane (h, c) holds columns 16h .. 16h + 15 of
    // each column tile (two 16-byte loads per tile, none under a per-element condition)
    f32x16 acc[kDnTiles][CT];
    {
        bf16x8 bias[CT][2];
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) bias[ct][0] = bias[ct][1] = zero8();
        if (b_down) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                bias[ct][0] = load8(b_down + col_w + 32 * ct + 16 * h);
                bias[ct][1] = load8(b_down + col_w + 32 * ct + 16 * h + 8);
            }
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i)
#pragma unroll
                for (int j = 0; j < kDnTiles; ++j) acc[j][ct][i] = (float)bias[ct][i >> 3][i & 7];
    }
    write_tiles(0, breg[0]);
    lds_barrier();
    const char* const rsrc_l = img + lane * 16;
    // k-step ks of token tile j of the stage in buffer buf
    auto read_piece = [&](int buf, int ks, int j) {
        return *reinterpret_cast<const bf16x8*>(rsrc_l + buf * kImage + (j * KSP + ks) * 1024);
    };
#pragma unroll
    for (int j = 0; j < kDnTiles; ++j) bb[0][j] = read_piece(0, 0, j);
    // Stage i of a trip (buffer i, MFMAs on the tiles of stage st): its first phase writes the
    // tiles of stage st + 1 to buffer i + 1 (fetched three stages earlier into register set
    // i + 1) and computes the offsets and issues the fetch of stage st + 4 into set i (written
    // out one stage ago); the barrier sits in the middle of the stage's MFMAs.  Every phase
    // requests the weights of the phase R - 1 ahead and reads from LDS the B operands of the NEXT
    // phase (k-step 0 of the next stage in the last phase: the barrier has passed by then), then
    // runs its MFMAs on operands requested earlier.  So the LDS write, the barrier and all LDS
    // reads overlap with matrix work of the same wavefront; the pieces sit between single MFMAs,
    // pinned by scheduling barriers (left alone the scheduler groups them and the matrix pipe
    // idles meanwhile).  Four buffers keep a wavefront that runs ahead from overwriting tiles
    // that a slower one still reads.  A trip past the last stage multiplies zero tiles.
    int trip = 0, trip_end = min(kTripsPerBatch - 1, n_trips), batch = 1;
    for (;;) {
        do {
#pragma unroll
            for (int q = 0; q < PH; ++q) {
                constexpr int kLast = kDnTiles * CT - 1;
                const int i = q / KSP, ks = q % KSP, ni = (i + 1) % kDnTrip;
                const int rbuf = ks < KSP - 1 ? i : ni, rks = ks < KSP - 1 ? ks + 1 : 0;
                // A memory instruction takes the wavefront several cycles to issue: at most one
                // global load (and two LDS operations) sits between two MFMAs, so that the
                // matrix pipe hides it.
                __builtin_amdgcn_sched_barrier(0);
                if (ks == 0) write_piece(ni, 0, breg[ni]);
#pragma unroll
                for (int n = 0; n <= kLast; ++n) {
                    // the operands requested last come first: their wait covers the whole phase
                    const int j = kDnTiles - 1 - n / CT, ct = CT - 1 - n % CT;
                    acc[j][ct] = mfma32(aw[q % R][ct], bb[q & 1][j], acc[j][ct]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks == 0) {
                        if (UPE == 1) {
#pragma unroll
                            for (int eo = 0; eo < G; ++eo)  // G <= 4: before the first fetch below
                                if (n == eo) build_prepare(sh_base + i * G + eo, eo);
                        } else if ((i & 1) == 0 && n == 0) {
                            build_prepare(sh_base + i / 2, 0);
                        }
#pragma unroll
                        for (int s = 1; s < KSP; ++s)
                            if (n == (s - 1) % 2) write_piece(ni, s, breg[ni]);
#pragma unroll
                        for (int s = 0; s < KSP; ++s)
                            if (n == (2 + CT + s < kLast ? 2 + CT + s : kLast))
                                fetch_piece(s, breg[i], UPE == 1 ? 0 : (i & 1));
                    }
                    if (n >= 2 && n < 2 + CT) load_block((q + R - 1) % KSP, n - 2, aw[(q + R - 1) % R]);
                    if (n == 2) {
                        bb[(q + 1) & 1][0] = read_piece(rbuf, rks, 0);
                        bb[(q + 1) & 1][1] = read_piece(rbuf, rks, 1);
                    }
                    if (n == 3) {
                        bb[(q + 1) & 1][2] = read_piece(rbuf, rks, 2);
                        bb[(q + 1) & 1][3] = read_piece(rbuf, rks, 3);
                    }
                }
                if (ks == (KSP >> 1) - 1) lds_barrier();  // every wavefront has written its part of st + 1
            }
            sh_base += kExpertsPerTrip;
        } while (++trip < trip_end);
        if (trip >= n_trips) break;
        // the next trip computes the offsets of the first experts of the next batch: its mask
        // word and first rows were requested a whole run of the loop ago
        mw = (tok_ok && batch < n_batches) ? mw_next : 0u;
        rowv = is_next * rows_per_item + go_next;
        ++batch;
        load_batch(batch, mw_next, is_next, go_next);
        sh_base = 0;
        trip_end = min(trip + kTripsPerBatch, n_trips);
    }

    // lane (h, c) of tile (j, ct): columns col_w + 32ct + 16h .. +15 of token t_base + 32j + c
#pragma unroll
    for (int j = 0; j < kDnTiles; ++j) {
        const int t = t_base + 32 * j + c;
        if (t < T) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
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

// Bytes of the packed down weights and of the H rows the kernel may address: both are reached
// through 32-bit buffer offsets.
size_t down_w_bytes(const dmoe_layer& L) {
    const DownPacking dp = down_packing(L.expert_size);
    return (size_t)div_up(L.n_experts * dp.UPE, dp.G) * (L.d_model / 32) * dp.KSP * 1024;
}
size_t down_h_bytes(const dmoe_layer& L, int T) {
    return (size_t)h_fragments(L, T) * 16 * 2 * m_pad_of(L.expert_size);
}

template <int KSP, int G, int R, int WPS, int CT, int UPE = 1>
void launch_down_t(const dmoe_layer& L, const PackedLayout& P, int T, const int32_t* item_start,
                   const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                   const void* H, void* y, long long max_pairs_sparse, hipStream_t s) {
    const int NG = div_up(T, kGroup), NC = div_up(T, kDnTokens), NS = L.d_model / (CT * kDnColStep);
    constexpr size_t lds = (size_t)kDnTrip * kDnTiles * KSP * 1024;
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&down_bf16_kernel<KSP, G, R, WPS, CT, UPE>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    const char* pk = static_cast<const char*>(L.packed);
    const int row_bytes = 2 * m_pad_of(L.expert_size);
    int row_shift = 0;
    while ((1 << row_shift) < row_bytes) ++row_shift;
    launch_kernel(down_bf16_kernel<KSP, G, R, WPS, CT, UPE>, round_up(NC, 8) * NS, 256, lds, s, 
        (const __bf16*)(pk + P.w2g), (const __bf16*)L.b_down, item_start, group_off,
        reinterpret_cast<const uint32_t*>(mask), offsets, (const __bf16*)H, (__bf16*)y, T,
        L.d_model, L.n_experts, NG, 2 * div_up(L.n_experts, 64), up_rows_bf16(L), row_shift,
        (uint32_t)down_w_bytes(L), (uint32_t)down_h_bytes(L, T), max_pairs_sparse);
}

}  // namespace

bool down_bf16_supported(const dmoe_layer& L) {
    const int mp = m_pad_of(L.expert_size);
    return (mp == 32 || mp == 64 || mp == 128) && L.d_model % (2 * kDnColStep) == 0;
}

// The matrix-core kernel reaches the packed weights and H through 32-bit buffer offsets, and
// marks unselected tokens with offsets from 2^31 up.
bool down_bf16_addressable(const dmoe_layer& L, int T) {
    return down_w_bytes(L) < (1ull << 32) && down_h_bytes(L, T) < (1ull << 31);
}

void launch_pack_down_bf16(const dmoe_layer& L, void* w2g, hipStream_t s) {
    const DownPacking dp = down_packing(L.expert_size);
    // 8-bit weights: the snapped scales that launch_pack_bf16 wrote into the packed buffer
    const float* scales = weights_fp8(L)
                              ? (const float*)(static_cast<const char*>(w2g) - packed_layout(L).w2g + packed_layout(L).scales)
                              : nullptr;
    launch_kernel(pack_down32_kernel, 2048, 256, 0, s, L.w_down, scales,
                                            weights_fp8(L), (__bf16*)w2g,
                                            L.n_experts, L.expert_size, L.d_model, dp.PG, dp.G, dp.KSP, dp.UPE);
}

void launch_down_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                      const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                      const void* H, void* y, long long max_pairs_sparse, hipStream_t s) {
    LaunchTimer tm(kSlotDown, s);
    const PackedLayout P = packed_layout(L);
    const DownPacking dp = down_packing(L.expert_size);
    // Shape of a workgroup: 128 tokens x 256 columns (one or two workgroups per CU), or 128 tokens
    // x 384 columns where that divides d (one per CU).  The wide shape is taken where it lets every
    // CU run exactly one workgroup while the narrow one would give some CUs two (16384 tokens,
    // d = 768: 256 workgroups of 12 tiles against 384 of 8 on 256 CUs).
    const int NC = div_up(T, kDnTokens);
    const int wg2 = NC * (L.d_model / (2 * kDnColStep));
    const bool can3 = L.d_model % (3 * kDnColStep) == 0;
    const int wg3 = can3 ? NC * (L.d_model / (3 * kDnColStep)) : 0;
    const bool wide = can3 && wg3 <= 256 && wg2 > 256;
    // at most one workgroup per CU: a wavefront may use the whole register file of its SIMD, which
    // buys a deeper ring of weight sets
    const bool one_per_cu = wg2 <= 256;
#define DMOE_DOWN(KSP_, G_, R_, WPS_, CT_) \
    launch_down_t<KSP_, G_, R_, WPS_, CT_>(L, P, T, item_start, group_off, mask, offsets, H, y, max_pairs_sparse, s)
    // Weight sets in flight per shape: wide / one narrow workgroup per CU / two per CU (R divides
    // 4 KSP).  With 8 k-steps per stage the four LDS buffers (128 KiB) leave room for one
    // workgroup per CU only.
#define DMOE_DOWN_BY_GRID(KSP_, G_, RW_, R1_, R2_)              \
    do {                                                        \
        if (wide) DMOE_DOWN(KSP_, G_, RW_, 1, 3);               \
        else if (one_per_cu) DMOE_DOWN(KSP_, G_, R1_, 1, 2);     \
        else DMOE_DOWN(KSP_, G_, R2_, 2, 2);                    \
    } while (0)
#define DMOE_DOWN_ONE_PER_CU(KSP_, G_, RW_, R1_)  \
    do {                                          \
        if (wide) DMOE_DOWN(KSP_, G_, RW_, 1, 3); \
        else DMOE_DOWN(KSP_, G_, R1_, 1, 2);      \
    } while (0)
    if (dp.UPE == 2) {  // experts of exactly 128 neurons as two units of 64
        if (wide) launch_down_t<4, 1, 8, 1, 3, 2>(L, P, T, item_start, group_off, mask, offsets, H, y, max_pairs_sparse, s);
        else if (one_per_cu) launch_down_t<4, 1, 16, 1, 2, 2>(L, P, T, item_start, group_off, mask, offsets, H, y, max_pairs_sparse, s);
        else launch_down_t<4, 1, 4, 2, 2, 2>(L, P, T, item_start, group_off, mask, offsets, H, y, max_pairs_sparse, s);
    }
    else if (dp.KSP == 2 && dp.G == 4) DMOE_DOWN_BY_GRID(2, 4, 8, 8, 4);
    else if (dp.KSP == 2 && dp.G == 2) DMOE_DOWN_BY_GRID(2, 2, 8, 8, 4);
    else if (dp.KSP == 2) DMOE_DOWN_BY_GRID(2, 1, 8, 8, 4);
    else if (dp.KSP == 3 && dp.G == 2) DMOE_DOWN_BY_GRID(3, 2, 12, 12, 4);
    else if (dp.KSP == 3) DMOE_DOWN_BY_GRID(3, 1, 12, 12, 4);
    else if (dp.KSP == 4) DMOE_DOWN_BY_GRID(4, 1, 8, 16, 4);
    else DMOE_DOWN_ONE_PER_CU(8, 1, 4, 8);
#undef DMOE_DOWN_ONE_PER_CU
#undef DMOE_DOWN_BY_GRID
#undef DMOE_DOWN
}

}  // namespace dmoe

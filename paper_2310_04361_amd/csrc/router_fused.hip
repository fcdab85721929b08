// Router (Sec. 3.3) fused with the dynamic-k gate (Sec. 3.4 Eq. 4) and the per-group expert counts
// that start the bucketing: one workgroup per group of 64 tokens.
//
//   stage 1  hid^T[d_h][64] = R1 * x^T.  The 64 x rows are staged in LDS (eight lanes per 128-byte
//            row piece), up to 768 columns at a time with all loads of the chunk in flight
//            together; each of the four wavefronts owns a quarter of the hidden units and reads
//            R1 as packed MFMA fragments.  bias + relu, round to bf16, park the hidden tile in LDS.
//   stage 2  s^T[E][64] = R2 * hid^T.  Each wavefront owns every fourth tile of 16 experts, reads
//            R2 as packed fragments and the hidden tile from LDS; |. + c2| goes to `scores`
//            (fp32, 16 bytes per lane) and stays in registers for
//   select   per-token maximum across the four wavefronts (LDS), the exact comparison
//            (double)s >= (double)tau * (double)max on those very fp32 scores, mask words
//            assembled per token, then the 64x64 ballot transpose that counts, per expert, the
//            tokens of the group that keep it.
// The scores that are written and the mask come from the same registers, so a caller that gates
// the returned scores again gets the same mask bit for bit.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

constexpr int kMaxTilesPerWave = 8;   // expert tiles per wavefront: E <= 4 * 8 * 16 = 512

// NH = d_h / 16; ETW = expert tiles per wavefront (E <= 64 * ETW); KBC = K blocks (64 wide) of x
// that sit in LDS at a time: 12 (all of d = 768) when there is at most about one workgroup per
// CU and its own latency is what counts, 4 when several workgroups share a CU and hide it.
// TT = tiles of 16 tokens per workgroup: 4 (a whole select group of 64 tokens), or 2 / 1 when
// there are too few groups to fill the chip -- a workgroup then handles a half or a quarter of a
// group and writes its expert counts to its own row of a table with 4 / TT rows per group, which
// the scan over the groups adds up.
// MODE: kWhole: both products (and the gate) in one workgroup.  A router whose two matrices take
// megabytes (d_h = 512, thousands of experts) would stream all of them through every CU; it runs
// as two launches instead, with the matrices split over blockIdx.y: kHiddenSlice computes the NH * 16
// hidden units from blockIdx.y * NH * 16 on and stores them to hid_g[T][dh_g]; kScoresSlice (NH * 16 =
// d_h) reads the stored hidden rows and computes the expert tiles blockIdx.y * tiles_y .. + tiles_y - 1.
enum { kWhole = 0, kHiddenSlice = 1, kScoresSlice = 2 };
template <int NH, int ETW, int KBC, int TT, int MODE = kWhole>
__global__ __launch_bounds__(256) void router_fused_kernel(
    const __bf16* __restrict__ x, const __bf16* __restrict__ r1f, const __bf16* __restrict__ r_b1,
    const __bf16* __restrict__ r2f, const __bf16* __restrict__ r_b2, float* __restrict__ scores,
    int T, int d, int E, float tau, int do_select, uint64_t* __restrict__ mask,
    int32_t* __restrict__ k_per_token, int32_t* __restrict__ group_cnt,
    uint64_t* __restrict__ colmask, __bf16* __restrict__ hid_g, int dh_g, int tiles_y) {
    constexpr int dh = NH * 16, HT = NH / 4, TOK = 16 * TT;
    constexpr int NR = (TOK + 31) / 32;  // staging passes of 32 rows
    constexpr int kHRow = dh * 2 + 16;  // bytes per hidden row in LDS
    constexpr int kXRowC = KBC * 128 + 16;  // bytes per staged x row: KBC blocks + bank skew
    extern __shared__ char smem[];
    char* xs = smem;                                            // [TOK][kXRowC]
    char* hid = MODE == kScoresSlice ? smem : smem + TOK * kXRowC;  // [TOK][kHRow]
    float* pmax = reinterpret_cast<float*>(hid + TOK * kHRow);  // [4][64]
    uint64_t* pw = reinterpret_cast<uint64_t*>(pmax + 256);     // [4][64][W]
    const int W = (E + 63) >> 6;
    uint64_t* fin = pw + 4 * 64 * W;                            // [64][W]

    const int g = blockIdx.x, t0 = g * TOK;  // g: row of the count table
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, q = lane >> 4, c = lane & 15;
    const int NK32 = d / 32, NKB = d / 64;

    // ---------------------------------------------------------------- stage 1
    // x comes from HBM: all loads of a chunk are issued together so that their latency is paid
    // once per chunk, not once per K block (loads complete in issue order, so a prefetch of x
    // inside the K loop would hold up the R1 fragments behind it).  The K loop itself has no
    // barrier and only L2-resident loads.
    const int ld_row = tid >> 3, ld_piece = tid & 7;
    const bool ld_ok = ld_row < TOK;  // 16 tokens: half of the threads stage nothing
    const __bf16* xp0 = x + (size_t)min(t0 + ld_row, T - 1) * d + 8 * ld_piece;
    const __bf16* xp1 = x + (size_t)min(t0 + ld_row + 32, T - 1) * d + 8 * ld_piece;
    char* xst = xs + ld_row * kXRowC + ld_piece * 16;
    // (a hidden slice starts at hidden tile blockIdx.y * NH)
    const __bf16* af = r1f + (((size_t)(MODE == kHiddenSlice ? blockIdx.y * NH : 0) + w * HT) * NK32 * 64 + lane) * 8;

    f32x4 acc[HT][TT];
#pragma unroll
    for (int h = 0; h < HT; ++h)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[h][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // R1 fragments: a ring of four K blocks, requested three blocks before their use (an L2
    // round trip takes longer than the 16 to 32 MFMAs of one block)
    bf16x8 ar[4][2][HT];
    auto load_a = [&](int kb, bf16x8 (&a)[2][HT]) {
        kb = min(kb, NKB - 1);  // the last trips re-read a block they will not use
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int h = 0; h < HT; ++h) a[ks][h] = load8(af + ((size_t)h * NK32 + 2 * kb + ks) * 512);
    };
    auto compute = [&](int kbl, const bf16x8 (&a)[2][HT]) {
        const char* src = xs + c * kXRowC + kbl * 128 + q * 16;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 b[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                b[tt] = *reinterpret_cast<const bf16x8*>(src + tt * 16 * kXRowC + ks * 64);
#pragma unroll
            for (int h = 0; h < HT; ++h)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[h][tt] = mfma16(a[ks][h], b[tt], acc[h][tt]);
        }
    };

    if constexpr (MODE != kScoresSlice) {
    for (int kb0 = 0; kb0 < NKB; kb0 += KBC) {
        const int nkb = min(KBC, NKB - kb0);  // a multiple of 4: d is a multiple of 256
        {
            bf16x8 xr[NR * KBC];
#pragma unroll
            for (int i = 0; i < KBC; ++i)
                if (i < nkb && ld_ok) {
                    xr[NR * i] = load8(xp0 + 64 * (kb0 + i));
                    if (NR == 2) xr[NR * i + NR - 1] = load8(xp1 + 64 * (kb0 + i));
                }
            if (kb0 > 0) lds_barrier();  // the previous chunk has been consumed
#pragma unroll
            for (int i = 0; i < KBC; ++i)
                if (i < nkb && ld_ok) {
                    *reinterpret_cast<bf16x8*>(xst + i * 128) = xr[NR * i];
                    if (NR == 2)
                        *reinterpret_cast<bf16x8*>(xst + 32 * kXRowC + i * 128) = xr[NR * i + NR - 1];
                }
        }
        if (kb0 == 0) {
#pragma unroll
            for (int i = 0; i < 3; ++i) load_a(i, ar[i]);
        }
        lds_barrier();
        for (int kbl = 0; kbl < nkb; kbl += 4) {  // nkb is a multiple of 4
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                load_a(kb0 + kbl + i + 3, ar[(i + 3) & 3]);
                compute(kbl + i, ar[i]);
            }
        }
    }

    }  // stage 1

    // R2 fragments of this wavefront's first expert tile: requested now, so that their latency
    // passes while the hidden tile is finished and stored
    constexpr int KS2 = dh / 32;
    const int NE = (E + 15) >> 4;
    // two sets of R2 fragments alternate (a third in flight measured the same on a router of
    // 2048 experts and d_h = 512)
    constexpr int kR2Ring = 2;
    bf16x8 r2a[kR2Ring][KS2];
    auto load_r2 = [&](int et, bf16x8 (&a)[KS2]) {
        et = min(et, NE - 1);
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) a[ks] = load8(r2f + (((size_t)et * KS2 + ks) * 64 + lane) * 8);
    };
    if constexpr (MODE == kScoresSlice) load_r2(blockIdx.y * tiles_y + w, r2a[0]);
    else if constexpr (MODE == kWhole) load_r2(w, r2a[0]);

    // lane (q, c) of tile (h, tt): hidden units 16*(w*HT + h) + 4q + r of token 16tt + c
#pragma unroll
    for (int h = 0; h < HT && MODE != kScoresSlice; ++h) {
        const int hu0 = 16 * (w * HT + h) + 4 * q;                      // within this workgroup's units
        const int hu_g = (MODE == kHiddenSlice ? blockIdx.y * dh : 0) + hu0;  // within the layer's
        float b1[4] = {0.f, 0.f, 0.f, 0.f};
        if (r_b1) {
#pragma unroll
            for (int r = 0; r < 4; ++r) b1[r] = (float)r_b1[hu_g + r];
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            bf16x4 hv;
#pragma unroll
            for (int r = 0; r < 4; ++r) hv[r] = (__bf16)fmaxf(acc[h][tt][r] + b1[r], 0.0f);
            if constexpr (MODE == kHiddenSlice) {
                const int t = t0 + 16 * tt + c;
                if (t < T) *reinterpret_cast<bf16x4*>(hid_g + (size_t)t * dh_g + hu_g) = hv;
            } else {
                *reinterpret_cast<bf16x4*>(hid + (16 * tt + c) * kHRow + hu0 * 2) = hv;
            }
        }
    }
    if constexpr (MODE == kHiddenSlice) return;
    if constexpr (MODE == kScoresSlice) {
        // the stored hidden rows of the group's tokens: 16-byte pieces, rows past T read row T - 1
        // (all loads of a thread in flight before the first store)
        constexpr int kPieces = dh / 8, kTrips = TOK * kPieces / 256;
        bf16x8 hr[kTrips];
#pragma unroll
        for (int j = 0; j < kTrips; ++j) {
            const int i = tid + 256 * j, row = i / kPieces, piece = i % kPieces;
            hr[j] = load8(hid_g + (size_t)min(t0 + row, T - 1) * dh_g + piece * 8);
        }
#pragma unroll
        for (int j = 0; j < kTrips; ++j) {
            const int i = tid + 256 * j, row = i / kPieces, piece = i % kPieces;
            *reinterpret_cast<bf16x8*>(hid + row * kHRow + piece * 16) = hr[j];
        }
    }
    lds_barrier();  // the hidden tile is in LDS (a full barrier would also wait for global stores)

    // ---------------------------------------------------------------- stage 2
    // scores of expert tile et for the group's 64 tokens: |R2 hid + c2| to `scores` and to o
    auto score_tile = [&](int et, const bf16x8 (&a)[KS2], float (&o)[TT][4]) {
        f32x4 a2[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) a2[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(
                    hid + (16 * tt + c) * kHRow + ks * 64 + q * 16);
                a2[tt] = mfma16(a[ks], b, a2[tt]);
            }
        }
        const int e0 = 16 * et + 4 * q;  // this lane: experts e0 .. e0+3
        // the second-layer biases as an accumulator-shaped vector (0 for experts from E on)
        // (every load unconditional, from a clamped index: under `if (e0 + r < E)` each of them
        // became a block of its own that waited for its value before the next one was requested)
        f32x4 b2 = f32x4{0.f, 0.f, 0.f, 0.f};
        if (r_b2) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float bv = (float)r_b2[min(e0 + r, E - 1)];
                b2[r] = e0 + r < E ? bv : 0.0f;
            }
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int t = t0 + 16 * tt + c;
            // padding experts (from E on) score 0
            const float4 out = e0 < E ? router_scores4(a2[tt] + b2, nullptr, e0, E)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
            if (scores && t < T && e0 < E) store_scores4(scores + (size_t)t * E, e0, E, out);
            o[tt][0] = out.x; o[tt][1] = out.y; o[tt][2] = out.z; o[tt][3] = out.w;
        }
    };
    if (!do_select) {
        // router alone: any number of expert tiles, the fragments of the next tile on their way
        // while the current one is multiplied
        float o[TT][4];
        const int et0 = MODE == kScoresSlice ? blockIdx.y * tiles_y : 0;
        const int et1 = MODE == kScoresSlice ? min(NE, et0 + tiles_y) : NE;
        load_r2(et0 + w + 4, r2a[1]);
        for (int et = et0 + w; et < et1; et += 4 * kR2Ring) {
#pragma unroll
            for (int i = 0; i < kR2Ring; ++i) {
                if (et + 4 * i < et1) score_tile(et + 4 * i, r2a[i], o);  // uniform per wavefront
                load_r2(et + 4 * (i + kR2Ring), r2a[i]);  // past the end: the last tile again
            }
        }
        return;
    }
    float sc[ETW][TT][4];  // [my tile][token tile][r]
    float vmax[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) vmax[tt] = 0.f;
#pragma unroll
    for (int j = 0; j < ETW; ++j) {
        const int et = w + 4 * j;
        if (j + 1 < ETW) load_r2(et + 4, r2a[(j + 1) & 1]);
        if (et < NE) {  // uniform per wavefront
            score_tile(et, r2a[j & 1], sc[j]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                vmax[tt] = fmaxf(vmax[tt], fmaxf(fmaxf(sc[j][tt][0], sc[j][tt][1]),
                                                 fmaxf(sc[j][tt][2], sc[j][tt][3])));
        }
    }

    // ---------------------------------------------------------------- select
    // maximum of each token over this wavefront's experts, then over the four wavefronts
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        float m = vmax[tt];
        m = fmaxf(m, __shfl_xor(m, 16, 64));
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        if (q == 0) pmax[w * 64 + 16 * tt + c] = m;
    }
    lds_barrier();  // LDS only: the scores' stores to global memory need not have landed
    const uint32_t keep_all = tau == 0.0f ? 1u : 0u;
    double thr[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int tk = 16 * tt + c;
        const float m = fmaxf(fmaxf(pmax[tk], pmax[64 + tk]), fmaxf(pmax[128 + tk], pmax[192 + tk]));
        thr[tt] = (double)tau * (double)m;  // exact: at most 48 significant bits
    }
    // this wavefront's bits of each token: its tile et = w + 4j is the only one it has in word j
    // (bits 16w .. 16w+15), so the word is stored whole, zero where the tile lies beyond E
#pragma unroll
    for (int j = 0; j < ETW; ++j) {
        const int et = w + 4 * j;
        const int e0 = 16 * et + 4 * q;
        if (j < W) {  // uniform
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                uint32_t bits = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // integer logic, no short circuit: as `a || b`, `c && d` this became a
                    // branch around every one of the 64-bit comparisons
                    const uint32_t ge = (double)sc[j][tt][r] >= thr[tt] ? 1u : 0u;
                    const uint32_t in = (et < NE ? 1u : 0u) & (e0 + r < E ? 1u : 0u);
                    bits |= ((keep_all | ge) & in) << (4 * q + r);
                }
                bits |= __shfl_xor(bits, 16, 64);
                bits |= __shfl_xor(bits, 32, 64);  // 16 bits: experts 16et .. 16et+15 of token c
                if (q == 0) pw[(w * 64 + 16 * tt + c) * W + j] = (uint64_t)bits << (16 * w);
            }
        }
    }
    lds_barrier();
    if (tid < 64) {
        const int t = t0 + tid;
        const bool mine = tid < TOK && t < T;  // lanes from TOK up: no token, an all-zero row
        int kt = 0;
        for (int wi = 0; wi < W; ++wi) {
            uint64_t word = 0ull;
            if (tid < TOK)
                word = pw[(0 * 64 + tid) * W + wi] | pw[(1 * 64 + tid) * W + wi] |
                       pw[(2 * 64 + tid) * W + wi] | pw[(3 * 64 + tid) * W + wi];
            fin[tid * W + wi] = mine ? word : 0ull;
            if (mine) mask[(size_t)t * W + wi] = word;
            kt += __popcll(word);
        }
        if (mine && k_per_token) k_per_token[t] = kt;
    }
    lds_barrier();
    // ballot transpose: lane = token; wavefront w handles the experts 64wi + 16w .. +15 of every
    // word wi (sixteen ballots per word and wavefront)
    for (int wi = 0; wi < W; ++wi) {
        const uint64_t word = fin[lane * W + wi];
        uint64_t col = 0;  // lane b: which tokens of the group keep expert 64wi + b
#pragma unroll
        for (int bi = 0; bi < 16; ++bi) {
            const int b = 16 * w + bi;
            const uint64_t bal = __ballot((word >> b) & 1ull);
            if (lane == b) col = bal;
        }
        const int e = 64 * wi + lane;
        if ((lane >> 4) == w && e < E) {
            group_cnt[(size_t)g * E + e] = __popcll(col);
            if (colmask) colmask[(size_t)g * E + e] = col;
        }
    }
}

template <int NH, int ETW, int KBC, int TT>
void launch_t3(const dmoe_layer& L, const void* x, int T, float* scores, float tau, uint64_t* mask,
               int32_t* k_per_token, int32_t* group_cnt, uint64_t* colmask, hipStream_t s) {
    const PackedLayout P = packed_layout(L);
    const int E = L.n_experts, W = div_up(E, 64);
    constexpr int TOK = 16 * TT;
    const size_t lds = TOK * (KBC * 128 + 16) + TOK * (NH * 32 + 16) + 256 * 4 +
                       (mask ? (size_t)5 * 64 * W * 8 : 0);  // the gate's words only when it runs
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&router_fused_kernel<NH, ETW, KBC, TT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    const char* pk = static_cast<const char*>(L.packed);
    launch_kernel(router_fused_kernel<NH, ETW, KBC, TT>, div_up(T, TOK), 256, lds, s, 
        (const __bf16*)x, (const __bf16*)(pk + P.r1f), (const __bf16*)L.r_b1,
        (const __bf16*)(pk + P.r2f), (const __bf16*)L.r_b2, scores, T, L.d_model, E, tau,
        mask != nullptr, mask, k_per_token, group_cnt, colmask, nullptr, 0, 0);
}

template <int NH, int ETW>
void launch_t2(const dmoe_layer& L, const void* x, int T, int split, float* scores, float tau,
               uint64_t* mask, int32_t* k_per_token, int32_t* group_cnt, uint64_t* colmask,
               hipStream_t s) {
    constexpr int kBig = NH <= 8 ? 12 : (NH == 16 ? 8 : 4);
    // parts of a group per workgroup: only where workgroups are few (one per CU, nothing hides
    // the latency of an x chunk), and the fewer rows leave LDS for chunks of 1024 columns
    if (split == 4)
        launch_t3<NH, ETW, 16, 1>(L, x, T, scores, tau, mask, k_per_token, group_cnt, colmask, s);
    else if (split == 2)
        launch_t3<NH, ETW, 16, 2>(L, x, T, scores, tau, mask, k_per_token, group_cnt, colmask, s);
    else if (kBig > 4 && div_up(T, 64) <= 512)
        launch_t3<NH, ETW, kBig, 4>(L, x, T, scores, tau, mask, k_per_token, group_cnt, colmask, s);
    else
        launch_t3<NH, ETW, 4, 4>(L, x, T, scores, tau, mask, k_per_token, group_cnt, colmask, s);
}

// ---- T <= 16: the same two products spread over many workgroups --------------------------------
// With so few tokens the router is a weight stream (R1 is 1 MiB at d = 2048, d_h = 256) and one
// workgroup per 64 tokens would leave it to a single CU.
//   hidden: workgroup = one tile of 16 hidden units, its (up to) sixteen wavefronts split K and
//           reduce through LDS; hid[16][d_h] (bf16) goes to a small global buffer.
//   scores: wavefront = one tile of 16 experts.
// The gate then runs as the stand-alone mask kernel on the stored scores.
__global__ __launch_bounds__(1024) void router_small_hidden_kernel(
    const SmallGroup G, const __bf16* __restrict__ x, int T, int d, int dh, int KQ) {
    const SmallMod& M = G.m[blockIdx.z];
    const __bf16* __restrict__ r1f = M.r1f;
    const __bf16* __restrict__ r_b1 = M.r_b1;
    __bf16* __restrict__ hid = M.hid;
    __shared__ float red[16][64][4];
    const int h = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, q = lane >> 4, c = lane & 15;
    const int NK32 = d / 32, per = NK32 / KQ;  // KQ <= 16 wavefronts split K; KQ divides NK32
    const __bf16* xr = x + (size_t)min(c, T - 1) * d + 8 * q;
    const __bf16* af = r1f + (((size_t)h * NK32) * 64 + lane) * 8;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (w < KQ) {
#pragma unroll 8
        for (int ks = w * per; ks < (w + 1) * per; ++ks)
            acc = mfma16(load8(af + (size_t)ks * 512), load8(xr + 32 * ks), acc);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) red[w][lane][r] = acc[r];
    __syncthreads();
    if (w == 0) {  // lane (q, c): hidden units 16h + 4q + r of token c
        bf16x4 hv;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float v = 0.0f;
            for (int k = 0; k < KQ; ++k) v += red[k][lane][r];
            if (r_b1) v += (float)r_b1[16 * h + 4 * q + r];
            hv[r] = (__bf16)fmaxf(v, 0.0f);
        }
        *reinterpret_cast<bf16x4*>(hid + (size_t)c * dh + 16 * h + 4 * q) = hv;
    }
}

__global__ __launch_bounds__(256) void router_small_scores_kernel(const SmallGroup G, int T,
                                                                  int dh, int E) {
    const SmallMod& M = G.m[blockIdx.z];
    const __bf16* __restrict__ hid = M.hid;
    const __bf16* __restrict__ r2f = M.r2f;
    const __bf16* __restrict__ r_b2 = M.r_b2;
    float* __restrict__ scores = M.scores;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, q = lane >> 4, c = lane & 15;
    const int et = blockIdx.x * 4 + w;
    if (et >= (E + 15) / 16) return;
    const int KS2 = dh / 32;
    const __bf16* af = r2f + (((size_t)et * KS2) * 64 + lane) * 8;
    const __bf16* hb = hid + (size_t)c * dh + 8 * q;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int ks = 0; ks < KS2; ++ks)
        acc = mfma16(load8(af + (size_t)ks * 512), load8(hb + 32 * ks), acc);
    const int e0 = 16 * et + 4 * q;
    if (c < T && e0 < E) {
        store_scores4(scores + (size_t)c * E, e0, E, router_scores4(acc, r_b2, e0, E));
    }
}

template <int NH>
void launch_t(const dmoe_layer& L, const void* x, int T, int split, float* scores, float tau,
              uint64_t* mask, int32_t* k_per_token, int32_t* group_cnt, uint64_t* colmask,
              hipStream_t s) {
    if (L.n_experts <= 128 || !mask)  // the router alone keeps no scores in registers
        launch_t2<NH, 2>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s);
    else if (L.n_experts <= 256)
        launch_t2<NH, 4>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s);
    else
        launch_t2<NH, 8>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s);
}

}  // namespace

void launch_router_small_hidden(const dmoe_layer& L, const SmallGroup& G, int n_layers,
                                const void* x, int T, hipStream_t s) {
    LaunchTimer tm(kSlotRouter, s);
    const int dh = L.router_hidden;
    int KQ = 16;  // wavefronts that split K: as many as divide the k-steps
    while (KQ > 1 && (L.d_model / 32) % KQ != 0) KQ >>= 1;
    launch_kernel(router_small_hidden_kernel, dim3(dh / 16, 1, n_layers), 1024, 0, s, G, (const __bf16*)x, T,
                                                                          L.d_model, dh, KQ);
}

void launch_router_small(const dmoe_layer& L, const SmallGroup& G, int n_layers, const void* x,
                         int T, hipStream_t s) {
    launch_router_small_hidden(L, G, n_layers, x, T, s);
    LaunchTimer tm(kSlotRouter, s);
    const int dh = L.router_hidden, E = L.n_experts;
    launch_kernel(router_small_scores_kernel, dim3(div_up(div_up(E, 16), 4), 1, n_layers), 256, 0, s, G, T, dh, E);
}

bool router_fused_scores_supported(const dmoe_layer& L) {
    const int dh = L.router_hidden;
    return L.packed != nullptr && (dh == 64 || dh == 128 || dh == 256 || dh == 512) &&
           L.d_model % 256 == 0;
}

bool router_fused_supported(const dmoe_layer& L) {
    return router_fused_scores_supported(L) && L.n_experts <= 64 * kMaxTilesPerWave;
}

// A router whose two matrices take 2 MB or more runs as two launches with the matrices split over
// the workgroups (see router_fused_kernel); needs a [T][d_h] bf16 buffer for the hidden rows.
bool router_sliced(const dmoe_layer& L) {
    const int dh = L.router_hidden;
    return router_fused_scores_supported(L) && (dh == 256 || dh == 512) &&
           2 * (size_t)dh * ((size_t)L.d_model + L.n_experts) >= (2u << 20);
}

template <int NH>
static void launch_scores_slices(const dmoe_layer& L, const PackedLayout& P, int T,
                                 const __bf16* hid, float* scores, hipStream_t s) {
    const int NG = div_up(T, kGroup), NE = div_up(L.n_experts, 16);
    // expert slices: enough workgroups for the chip, at least one tile per wavefront
    const int want = std::max(1, std::min(NE / 4, div_up(256, NG)));
    const int tiles_y = round_up(div_up(NE, want), 4);
    const size_t lds = 64 * (NH * 32 + 16) + 256 * 4;
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(
            reinterpret_cast<const void*>(&router_fused_kernel<NH, 2, 4, 4, kScoresSlice>),
            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    const char* pk = static_cast<const char*>(L.packed);
    launch_kernel(router_fused_kernel<NH, 2, 4, 4, kScoresSlice>, dim3(NG, div_up(NE, tiles_y)), 256, lds, s, 
        nullptr, nullptr, nullptr, (const __bf16*)(pk + P.r2f), (const __bf16*)L.r_b2, scores, T,
        L.d_model, L.n_experts, 0.0f, 0, nullptr, nullptr, nullptr, nullptr,
        const_cast<__bf16*>(hid), L.router_hidden, tiles_y);
}

void launch_router_sliced(const dmoe_layer& L, const void* x, int T, void* hid, float* scores,
                          hipStream_t s) {
    LaunchTimer tm(kSlotRouter, s);
    const PackedLayout P = packed_layout(L);
    const int NG = div_up(T, kGroup), dh = L.router_hidden;
    const char* pk = static_cast<const char*>(L.packed);
    {   // hidden rows: 128 hidden units per workgroup
        constexpr int NH = 8, KBC = 12;
        const size_t lds = 64 * (KBC * 128 + 16) + 64 * (NH * 32 + 16) + 256 * 4;
        static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
        std::call_once(attr_once, [&] {
            (void)hipFuncSetAttribute(
                reinterpret_cast<const void*>(&router_fused_kernel<NH, 2, KBC, 4, kHiddenSlice>),
                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        });
        launch_kernel(router_fused_kernel<NH, 2, KBC, 4, kHiddenSlice>, dim3(NG, dh / 128), 256, lds, s, 
            (const __bf16*)x, (const __bf16*)(pk + P.r1f), (const __bf16*)L.r_b1, nullptr, nullptr,
            nullptr, T, L.d_model, L.n_experts, 0.0f, 0, nullptr, nullptr, nullptr, nullptr,
            (__bf16*)hid, dh, 0);
    }
    if (dh == 256) launch_scores_slices<16>(L, P, T, (const __bf16*)hid, scores, s);
    else launch_scores_slices<32>(L, P, T, (const __bf16*)hid, scores, s);
}

int router_fused_split(const dmoe_layer&, int T) {
    // measured (router alone, 1 / 2 / 4 workgroups per group): 4096 tokens, d = 2048, d_h = 256:
    // 39 / 31 / 28 us; the same with d_h = 512 and 2048 experts: 101 / 72 / 67 us; 16384 tokens,
    // d = 768: 21 / 21 / 26 us
    const int NG = div_up(T, kGroup);
    return NG >= 192 ? 1 : (NG >= 96 ? 2 : 4);
}

void launch_router_fused(const dmoe_layer& L, const void* x, int T, int split, float* scores,
                         float tau, uint64_t* mask, int32_t* k_per_token, int32_t* group_cnt,
                         uint64_t* colmask, hipStream_t s) {
    LaunchTimer tm(kSlotRouter, s);
    if (colmask) split = 1;  // the token sets of an expert are per whole group
    switch (L.router_hidden) {
    case 64: launch_t<4>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s); break;
    case 128: launch_t<8>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s); break;
    case 256: launch_t<16>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s); break;
    case 512: launch_t<32>(L, x, T, split, scores, tau, mask, k_per_token, group_cnt, colmask, s); break;
    default: break;  // refused by router_fused_supported
    }
}

}  // namespace dmoe

// Internal declarations shared by the HIP translation units of libdmoe (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <mutex>

#include "../../include/dmoe.h"

namespace dmoe {

// ---- fixed granularities -------------------------------------------------------------------
constexpr int kGroup = 64;        // tokens per select group (one wavefront, lane = token)
constexpr int kChunkGroups = 2;   // groups per down-projection token chunk
constexpr int kChunk = kGroup * kChunkGroups;   // 128 tokens whose outputs live in LDS together
constexpr int kTilePad = 64;      // entries the expert kernels may read past the end of the lists

inline int round_up(int a, int b) { return (a + b - 1) / b * b; }
inline int div_up(int a, int b) { return (a + b - 1) / b; }
// Hidden units per H row: 32, 64 or 128 (the widths the expert kernels are compiled for), so
// experts of 65 .. 96 neurons take 128.
inline int m_pad_of(int m) {
    const int p = round_up(m, 32);
    return p == 96 ? 128 : p;
}

// List rows per up-projection work item (a multiple of 16); every expert's region of H starts
// at a multiple of this many rows.
inline int up_rows_bf16(const dmoe_layer& L) {
    // wide experts (8 neuron tiles per K step) use the kernel that shares the weights of a 256-row
    // item through LDS; everything else uses one wavefront per 64 rows
    const int tiles = (L.gated ? 2 : 1) * (m_pad_of(L.expert_size) / 16);
    return tiles == 8 ? 256 : 64;
}

// H capacity in 16-row fragments for T tokens: every expert may round up to a whole work item,
// and the down kernel reads one fragment past the last one.
inline size_t h_fragments(const dmoe_layer& L, int T) {
    return ((size_t)T * L.n_experts + (size_t)L.n_experts * up_rows_bf16(L)) / 16 + 4;
}

// 8-bit expert weights (both 8-bit formats); 8-bit expert inputs as well.
inline bool weights_fp8(const dmoe_layer& L) {
    return L.weight_format == DMOE_W_FP8_E4M3 || L.weight_format == DMOE_W_FP8_E4M3_X8 ||
           L.weight_format == DMOE_W_FP8_E4M3_A8;
}
inline bool acts_fp8(const dmoe_layer& L) {
    return L.weight_format == DMOE_W_FP8_E4M3_X8 || L.weight_format == DMOE_W_FP8_E4M3_A8;
}
// 8-bit hidden activations as well (every H row quantised before the down-projection) ...
inline bool hidden_fp8(const dmoe_layer& L) { return L.weight_format == DMOE_W_FP8_E4M3_A8; }
// ... and whether the 8-bit matrix-core down-projection covers the shape (H rows of 64 or 128
// neurons, 256-column slices); other shapes quantise H in place and run the bf16 kernels.
inline bool down_x8_shape(const dmoe_layer& L) {
    return hidden_fp8(L) && m_pad_of(L.expert_size) >= 64 && L.d_model % 256 == 0;
}
// ... and whether the 8-bit matrix-core up-projection covers the shape (the 256-row work items of
// the wide-expert kernel); other shapes run the bf16 kernels on the quantised input.
inline bool up_x8_supported(const dmoe_layer& L) { return acts_fp8(L) && up_rows_bf16(L) == 256; }

// Experts that fit ONE 16-row weight tile -- at most 16 neurons, or gated with at most 8 (up rows
// and gate rows together) -- take the up-projection kernel built around that tile.
inline bool up_tiny_supported(const dmoe_layer& L) {
    return L.dtype == DMOE_BF16 && L.expert_size <= (L.gated ? 8 : 16);
}

// Sub-buffers of the packed-weights buffer (bytes from its start).
struct PackedLayout {
    size_t w2f, w2g, wupf, wgatef, r1f, r2f, w2f8, wupf8, wgatef8, wtinyf, scales, wupx8, wgatex8, w2x8, wsc8, total;
};
inline PackedLayout packed_layout(const dmoe_layer& L) {
    PackedLayout P{};
    if (L.dtype != DMOE_BF16) return P;
    const size_t one =
        (2 * (size_t)L.n_experts * L.d_model * m_pad_of(L.expert_size) + 255) / 256 * 256;
    // the 32x32x16 down fragments pack the experts' real 8-neuron pieces in stages of one or two
    // experts: never more than m_pad neurons per expert, but a last half-filled stage counts as
    // two experts
    const size_t one_g =
        (2 * ((size_t)L.n_experts + 1) * L.d_model * m_pad_of(L.expert_size) + 255) / 256 * 256;
    P.w2f = 0;          // down-projection, 16x16x32 fragments (small-token path)
    P.w2g = one;        // down-projection, 32x32x16 fragments (down_bf16.hip)
    P.wupf = one + one_g;
    P.wgatef = P.wupf + one;
    size_t o = P.wupf + (L.gated ? 2 : 1) * one;
    // router weights as fragments: r1f[d_h/16][d/32][64][8], r2f[ceil(E/16)][d_h/32][64][8]
    P.r1f = o;
    o += (2 * (size_t)round_up(L.router_hidden > 0 ? L.router_hidden : 0, 16) * L.d_model + 255) / 256 * 256;
    P.r2f = o;
    o += (2 * (size_t)round_up(L.n_experts, 16) * round_up(L.router_hidden > 0 ? L.router_hidden : 0, 32) + 255) / 256 * 256;
    // 8-bit expert weights: the same fragments with one byte per weight for the small-token
    // kernels (w2f8, wupf8, wgatef8: half of `one` each)
    P.w2f8 = P.wupf8 = P.wgatef8 = o;
    if (weights_fp8(L)) {
        const size_t half = (one / 2 + 255) / 256 * 256;
        P.w2f8 = o;
        P.wupf8 = o + half;
        P.wgatef8 = o + 2 * half;
        o += (L.gated ? 3 : 2) * half;
    }
    // experts of one 16-row weight tile (at most 16 neurons; gated: 8 up rows + 8 gate rows)
    // (ffn_bf16.hip, up_tiny_kernel): wtinyf[E][d/32][64][8]
    P.wtinyf = o;
    if (up_tiny_supported(L)) o += (2 * (size_t)L.n_experts * 16 * L.d_model + 255) / 256 * 256;
    // 8-bit weights: the caller's scales snapped to powers of two, [E][3] fp32 -- the copy every
    // kernel uses, so that all paths compute the same layer whatever the caller passed
    P.scales = o;
    if (weights_fp8(L)) o += (sizeof(float) * 3 * (size_t)L.n_experts + 255) / 256 * 256;
    // 8-bit inputs: the up (and gate) matrices as operands of the 16x16x128 8-bit MFMA,
    // wupx8[E][m_pad/16][d/128][64][32] (ffn_x8.hip), one byte per weight
    P.wupx8 = P.wgatex8 = o;
    if (up_x8_supported(L)) {
        const size_t half = (one / 2 + 255) / 256 * 256;
        P.wupx8 = o;
        P.wgatex8 = o + half;
        o += (L.gated ? 2 : 1) * half;
    }
    // 8-bit hidden activations: the down matrices as operands of the 32x32x64 8-bit MFMA,
    // w2x8[E * units][d/32][64][32] (down_x8.hip; a unit = 64 neurons of an expert), and the E8M0
    // byte of every unit's down scale
    P.w2x8 = P.wsc8 = o;
    if (down_x8_shape(L)) {
        const size_t units = (size_t)L.n_experts * (m_pad_of(L.expert_size) / 64);
        P.w2x8 = o;
        o += (units * (L.d_model / 32) * 2048 + 255) / 256 * 256;
        P.wsc8 = o;
        o += (units + 255) / 256 * 256;
    }
    P.total = o;
    return P;
}

// ---- kernel timing slots --------------------------------------------------------------------
enum Slot {
    kSlotRouter = 0,
    kSlotMask,
    kSlotListsToMask,
    kSlotScanGroups,
    kSlotFill,
    kSlotUp,
    kSlotDown,
    kSlotDownRmw,
    kSlotFfnF32,
    kSlotSmallUp,
    kSlotSmallDown,
    kSlotSmallFinish,
    kSlotPack,
    kSlotQuantX,
    kSlotQuantH,
    kSlotCount
};

// Scope of the kernel launches that are accounted to one timing slot (see dmoe_timing_enable).
// With timing enabled, launch_kernel() inside the scope has the launch itself stamp an event pair
// with the start and the end of the kernel on the device, so what is summed is kernel time, not
// the gaps around event records.  One scope counts as one launch of its slot however many
// kernels it holds.
struct LaunchTimer {
    LaunchTimer(int slot, hipStream_t stream);
    ~LaunchTimer();
    int slot_;
    int index_;          // event pair reserved for the first launch, -1: timing off
    bool used_;          // that pair has been handed to a launch
    LaunchTimer* prev_;
    hipStream_t stream_;
};
// Event pair for the next launch of the calling thread's innermost scope (false: launch untimed).
bool timer_events_for_launch(hipEvent_t* start, hipEvent_t* stop);

// Every kernel of the library is launched through here.
template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s,
                          Args&&... args) {
    hipEvent_t ev0, ev1;
    if (timer_events_for_launch(&ev0, &ev1))
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, s, ev0, ev1, 0u,
                              static_cast<KArgs>(args)...);
    else
        kernel<<<grid, block, lds, s>>>(static_cast<KArgs>(args)...);
}

// ---- select / bucket (select.hip) -----------------------------------------------------------
// group_off is [(NG+1)][E] int32 with NG = ceil(T/64): after the scans, group_off[g][e] is the
// number of tokens < 64*g that selected expert e, and row NG holds the per-expert totals.
// colmask (nullable) is [NG][E] u64: bit j of colmask[g][e] = token 64g + j keeps expert e.
void launch_mask_from_scores(const float* scores, int T, int E, float tau, uint64_t* mask,
                             int32_t* k_per_token, int32_t* group_off, uint64_t* colmask,
                             hipStream_t s);
// Top-k gate: exactly k experts per token, ties at the k-th score to the lower expert index.
void launch_mask_topk(const float* scores, int T, int E, int k, uint64_t* mask,
                      int32_t* k_per_token, int32_t* group_off, uint64_t* colmask, hipStream_t s);
void launch_mask_from_lists(const int32_t* offsets, const int32_t* lists, int T, int E,
                            uint64_t* mask, int32_t* group_off, uint64_t* colmask, hipStream_t s);
// sub_cnt (nullable): the counts come as `split` rows per group (ceil(T * split / 64) rows) that
// are added up into group_off on the way.
void launch_scan_and_fill(const uint64_t* mask, int T, int E, int32_t* group_off, int32_t* counts,
                          int32_t* offsets, int32_t* item_start, int rows_per_item,
                          int32_t* token_lists, int32_t* aligned_lists, int window_groups,
                          int32_t* witem, int32_t* wfirst, hipStream_t s,
                          const int32_t* sub_cnt = nullptr, int split = 1);
// The up-projection walks its work items window by window (window = window_groups consecutive
// 64-token groups, window w on XCD w % 8) so that the x rows an XCD gathers stay in its L2:
// witem[NW][E+1], wfirst[NW][E] are built with the lists (nullable: no tables).  A single window
// (wide experts, whose weight stream would flush the rows anyway) is shared by all XCDs.
int up_window_groups(const dmoe_layer& L, int T);
constexpr int kMaxExperts = 4096;  // the list fill keeps 2 ints per expert in LDS

// ---- router (router.hip) ----------------------------------------------------------------------
void launch_router_f32(const dmoe_layer& L, const float* x, int T, float* scores, hipStream_t s);
void launch_router_bf16(const dmoe_layer& L, const void* x, int T, float* scores, hipStream_t s);
// Fused router + gate + group counts (router_fused.hip); mask == nullptr runs the router alone,
// which has no limit on the number of experts (router_fused_scores_supported).
bool router_fused_supported(const dmoe_layer& L);
bool router_fused_scores_supported(const dmoe_layer& L);
// split = 1, 2 or 4 workgroups per group of 64 tokens (router_fused_split: more where the groups
// alone would leave most of the chip idle).  With the gate and split > 1, group_cnt is a table
// of split rows per group -- row r holds the counts of the tokens 64 r / split .. -- that
// launch_scan_and_fill adds up; colmask forces split = 1.
int router_fused_split(const dmoe_layer& L, int T);
// Large routers (2 MB of matrices or more) without the gate: two launches with the matrices split
// over the workgroups; hid is a [T][d_h] bf16 scratch buffer.
bool router_sliced(const dmoe_layer& L);
void launch_router_sliced(const dmoe_layer& L, const void* x, int T, void* hid, float* scores,
                          hipStream_t s);
void launch_router_fused(const dmoe_layer& L, const void* x, int T, int split, float* scores,
                         float tau, uint64_t* mask, int32_t* k_per_token, int32_t* group_cnt,
                         uint64_t* colmask, hipStream_t s);

// ---- small-token path (T <= kSmallTokens): up to kGroupMax layers of one shape per launch ----
// The attention projections Q, K and V are three converted layers with the same input (Sec. 3.5),
// and at 16 tokens a forward is a handful of launches that each last a few microseconds: every
// small-token kernel therefore takes the per-layer pointers of a whole group and works on layer
// blockIdx.z.  A single layer is a group of one.
constexpr int kGroupMax = 4;
struct SmallMod {
    const __bf16 *r1f, *r_b1, *r2f, *r_b2;                 // packed router matrices, biases
    const __bf16 *wupf, *wgatef, *b_up, *w2f, *b_down;     // packed expert matrices, biases
    const uint8_t *wupf8, *wgatef8, *w2f8;                 // the same fragments, one E4M3 byte per weight
    const float* w_scales;                                 // [E][3] (up, gate, down); null: bf16 weights
    __bf16 *hid, *Hs, *y;                                  // router hidden tile, H fragments, output
    float *scores, *partial;                               // scores [T][E]; per-expert-group partial outputs
    uint64_t *mask, *colmask;                              // mask [T][W]; colmask [E]
    int32_t* group_cnt;                                    // [E] tokens per expert
    float tau;
};
struct SmallGroup {
    SmallMod m[kGroupMax];
};
// Router as a weight stream over many workgroups (same support conditions as the fused kernel);
// hid is a 16 x d_h bf16 scratch buffer per layer.  The gate runs separately.
void launch_router_small(const dmoe_layer& L, const SmallGroup& G, int n_layers, const void* x,
                         int T, hipStream_t s);
void launch_router_small_hidden(const dmoe_layer& L, const SmallGroup& G, int n_layers,
                                const void* x, int T, hipStream_t s);
// The same with the second product and the dynamic-k gate of every layer (M.tau) in ONE
// workgroup, which also writes mask, colmask and group_cnt; for E <= kSmallFusedSelectMaxE.
constexpr int kSmallFusedSelectMaxE = 1024;
void launch_router_select_small(const dmoe_layer& L, const SmallGroup& G, int n_layers,
                                const void* x, int T, hipStream_t s);
// Where the second router matrix is small the up-projection's workgroups repeat that product and
// the gate themselves (launch_small_bf16 with gate = true) and the gate launch goes away; with a
// larger matrix the repeated product costs each workgroup more than the launch (256 experts,
// d_h = 256: the up-projection grew by 10 us for a gate kernel of 8).
inline bool small_gate_in_up(const dmoe_layer& L) {
    return L.n_experts <= 64 && (size_t)L.n_experts * L.router_hidden <= 16384;
}
// Dynamic-k gate of every layer of the group on its stored scores (mask, colmask, group_cnt).
void launch_select_small_group(const dmoe_layer& L, const SmallGroup& G, int n_layers, int T,
                               hipStream_t s);

// ---- small-token experts (ffn_small.hip): T <= kSmallTokens, driven by colmask[0][e] -------------
constexpr int kSmallTokens = 16;
constexpr int kSmallMaxGroups = 32;   // expert groups whose partial outputs are summed at the end
bool small_bf16_supported(const dmoe_layer& L);
// Hs: E * (m_pad/32) KiB of fragments; partial: kSmallMaxGroups * 16 * d floats.
// gate: the up-projection computes the scores and the dynamic-k gate (M.tau) itself from the
// router's hidden rows (M.hid, written by launch_router_small_hidden) and writes M.scores, M.mask,
// M.colmask and M.group_cnt on the way; otherwise it reads M.colmask.
void launch_small_bf16(const dmoe_layer& L, const SmallGroup& G, int n_layers, const void* x, int T,
                       bool gate, hipStream_t s);

// ---- experts ----------------------------------------------------------------------------------
void launch_ffn_f32(const dmoe_layer& L, const float* x, int T, const uint64_t* mask, float* y,
                    hipStream_t s);
void launch_pack_bf16(const dmoe_layer& L, void* packed, hipStream_t s);
// H holds one row of m_pad hidden activations per list row (layout: see ffn_bf16.hip).
// alist is the work-item-aligned token list (see select.hip); its index is the row index of H.
void launch_up_bf16(const dmoe_layer& L, const void* x, int T, const int32_t* witem,
                    const int32_t* wfirst, const int32_t* alist, void* H, hipStream_t s);
// Down-projection and merge (down_bf16.hip): mask is the token-major selection bitmask that the
// lists were built from; group_off[g][e] = rows of expert e that belong to tokens before group g.
bool down_bf16_supported(const dmoe_layer& L);
bool down_bf16_addressable(const dmoe_layer& L, int T);
void launch_pack_down_bf16(const dmoe_layer& L, void* w2g, hipStream_t s);
// Two kernels, both launched: offsets[E] (the executed pairs) decides on the device which one
// works -- at most max_pairs_sparse pairs: the pair-proportional kernel (down_rmw_bf16.hip),
// more: the one that sums over experts inside the matrix cores (down_bf16.hip).
void launch_down_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                      const int32_t* group_off, const uint64_t* mask, const int32_t* offsets,
                      const void* H, void* y, long long max_pairs_sparse, hipStream_t s);
void launch_down_rmw_bf16(const dmoe_layer& L, int T, const int32_t* item_start,
                          const int32_t* group_off, const int32_t* alist, const int32_t* offsets,
                          const void* H, void* y, long long max_pairs_sparse, hipStream_t s);
long long down_max_pairs_sparse(const dmoe_layer& L, int T);

// ---- 8-bit hidden activations (down_x8.hip) -------------------------------------------------------
// Row-wise quantisation of the H rows that the up-projection wrote (see DMOE_W_FP8_E4M3_A8 in
// dmoe.h; the number of rows is item_start[E] * rows per item): to codes H8[row][64] and E8M0
// scale bytes hs8[row] for the 8-bit down-projection, or in place (the quantised rows as bf16
// numbers) for the bf16 down-projections.
void launch_pack_down_x8(const dmoe_layer& L, void* packed, hipStream_t s);
bool down_x8_addressable(const dmoe_layer& L, int T);
void launch_h_rows_to_e4m3(const dmoe_layer& L, const int32_t* item_start, const void* H,
                           uint8_t* H8, uint8_t* hs8, hipStream_t s);
void launch_h_rows_quantize(const dmoe_layer& L, const int32_t* item_start, void* H, hipStream_t s);
void launch_down_x8(const dmoe_layer& L, int T, const int32_t* item_start, const int32_t* group_off,
                    const uint64_t* mask, const uint8_t* H8, const uint8_t* hs8, void* y,
                    hipStream_t s);

// ---- 8-bit expert inputs (ffn_x8.hip) -------------------------------------------------------------
// Row-wise quantisation of x (see DMOE_W_FP8_E4M3_X8 in dmoe.h): x8[T][d] E4M3 codes, xscale[T]
// the power-of-two scales, xhat[T][d] (nullable) the quantised rows as bf16 numbers.
void launch_quantize_x(const dmoe_layer& L, const void* x, int T, uint8_t* x8, float* xscale,
                       void* xhat, hipStream_t s);
void launch_pack_x8(const dmoe_layer& L, void* packed, hipStream_t s);
// Up-projection on 8-bit operands; same work items, lists and H rows as launch_up_bf16.
// H8 / hs8 non-null: the rows go out quantised for the 8-bit
// down-projection instead of as bf16 rows in H.
void launch_up_x8(const dmoe_layer& L, const uint8_t* x8, const float* xscale, int T,
                  const int32_t* witem, const int32_t* wfirst, const int32_t* alist, void* H,
                  uint8_t* H8, uint8_t* hs8, hipStream_t s);

bool experts_bf16_supported(const dmoe_layer& L);
bool router_bf16_supported(const dmoe_layer& L);

}  // namespace dmoe

// C ABI of libdmoe: argument validation (host only, before any launch), workspace carving and
// kernel sequencing.  See include/dmoe.h for the contract of every entry point.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "dmoe_internal.h"

// Workspace of dmoe_forward_static: one array per GPU, held from the moment the library's code
// object is loaded on that GPU until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress (static_scratch_of_current_device below); it is never passed to a kernel.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace dmoe {

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// ---- static workspace ------------------------------------------------------------------------------
// Device address of `scratch` on the current GPU, looked up once per GPU (each GPU has its own
// copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(DMOE_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(DMOE_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(DMOE_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DMOE_OK;
}

// ---- timing ------------------------------------------------------------------------------------
const char* const kSlotNames[kSlotCount] = {
    "router", "mask_count", "lists_to_mask", "scan_groups", "fill_lists",
    "expert_up", "expert_down", "expert_down_sparse", "ffn_f32", "small_up", "small_down", "small_finish", "pack_weights",
    "quantize_x", "quantize_h"};
constexpr int kEventPairs = 8192;
bool g_timing = false;
std::vector<hipEvent_t> g_ev;      // 2 * kEventPairs once enabled
std::vector<int> g_ev_slot;        // slot of each pair; -1: reserved but never stamped
std::vector<char> g_ev_first;      // the pair is the first of its scope (counts as a launch)
int g_ev_used = 0;
thread_local LaunchTimer* g_scope = nullptr;
int64_t g_launches[kSlotCount];
double g_ms[kSlotCount];

int collect_events() {
    for (int i = 0; i < g_ev_used; ++i) {
        if (g_ev_slot[i] < 0) continue;
        hipError_t e = hipEventSynchronize(g_ev[2 * i + 1]);
        if (e != hipSuccess) return fail(DMOE_ERR_HIP, "hipEventSynchronize: %s", hipGetErrorString(e));
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, g_ev[2 * i], g_ev[2 * i + 1]);
        if (e != hipSuccess) return fail(DMOE_ERR_HIP, "hipEventElapsedTime: %s", hipGetErrorString(e));
        g_launches[g_ev_slot[i]] += g_ev_first[i] ? 1 : 0;
        g_ms[g_ev_slot[i]] += ms;
    }
    g_ev_used = 0;
    return DMOE_OK;
}

// ---- validation ----------------------------------------------------------------------------------
constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int check_layer(const dmoe_layer* L, bool need_router, bool need_experts) {
    if (!L) return fail(DMOE_ERR_NULL, "layer is NULL");
    if (L->d_model <= 0 || L->n_experts <= 0 || L->expert_size <= 0)
        return fail(DMOE_ERR_SHAPE, "d_model, n_experts and expert_size must be positive");
    if (L->dtype != DMOE_F32 && L->dtype != DMOE_BF16)
        return fail(DMOE_ERR_UNSUPPORTED, "dtype %d is not DMOE_F32 or DMOE_BF16", L->dtype);
    if (L->weight_format != DMOE_W_NATIVE && !weights_fp8(*L))
        return fail(DMOE_ERR_UNSUPPORTED, "weight_format %d is not one of DMOE_W_NATIVE, DMOE_W_FP8_E4M3, DMOE_W_FP8_E4M3_X8, DMOE_W_FP8_E4M3_A8", L->weight_format);
    if (weights_fp8(*L)) {
        if (L->dtype != DMOE_BF16) return fail(DMOE_ERR_UNSUPPORTED, "8-bit expert weights need a bf16 layer");
        if (!L->w_scales) return fail(DMOE_ERR_NULL, "8-bit expert weights need w_scales");
    }
    if (L->gated != 0 && L->gated != 1) return fail(DMOE_ERR_UNSUPPORTED, "gated must be 0 or 1");
    if (need_router) {
        if (L->router_hidden <= 0) return fail(DMOE_ERR_SHAPE, "router_hidden must be positive");
        if (!L->r_w1 || !L->r_w2) return fail(DMOE_ERR_NULL, "router weights are NULL");
        if (L->dtype == DMOE_BF16 && !router_bf16_supported(*L))
            return fail(DMOE_ERR_UNSUPPORTED,
                        "bf16 router needs d %% 32 == 0 and d_h in {32,64,128,256,512}");
        if (L->dtype == DMOE_F32 && (size_t)(L->d_model + L->router_hidden) * 4 > 65536)
            return fail(DMOE_ERR_UNSUPPORTED, "fp32 router needs d + d_h <= 16384");
    }
    if (need_experts) {
        if (L->act < DMOE_ACT_RELU || L->act > DMOE_ACT_GELU_TANH)
            return fail(DMOE_ERR_UNSUPPORTED, "unknown activation %d", L->act);
        if (!L->w_up || !L->w_down) return fail(DMOE_ERR_NULL, "expert weights are NULL");
        if (L->gated && !L->w_gate) return fail(DMOE_ERR_NULL, "gated layer without w_gate");
        if (L->gated && L->b_up)
            return fail(DMOE_ERR_UNSUPPORTED,
                        "a gated expert with b_up is undefined (Appendix G states it without biases)");
        if (L->dtype == DMOE_BF16) {
            if (!experts_bf16_supported(*L))
                return fail(DMOE_ERR_UNSUPPORTED,
                            "bf16 experts need d %% 256 == 0 and expert_size <= 128 (<= 64 if gated)");
            if (!L->packed)
                return fail(DMOE_ERR_NULL, "bf16 experts need layer->packed (dmoe_pack_weights)");
        } else if ((size_t)(2 * L->d_model + L->expert_size) * 4 > 65536) {
            return fail(DMOE_ERR_UNSUPPORTED, "fp32 experts need 2 d + m <= 16384");
        }
    }
    return DMOE_OK;
}

int check_tokens(int32_t T, int32_t E) {
    if (T < 0) return fail(DMOE_ERR_SHAPE, "n_tokens is negative");
    if (E > kMaxExperts) return fail(DMOE_ERR_UNSUPPORTED, "more than %d experts", kMaxExperts);
    if ((long long)T * E > 0x7fffffffLL - 64)
        return fail(DMOE_ERR_SHAPE, "n_tokens * n_experts does not fit the int32 list indices");
    return DMOE_OK;
}

int check_tau(float tau) {
    if (!(tau >= 0.0f && tau <= 1.0f)) return fail(DMOE_ERR_TAU, "tau must lie in [0, 1]");
    return DMOE_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
    if (need == 0) return DMOE_OK;
    if (!ws) return fail(DMOE_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % kAlign) return fail(DMOE_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (have < need) return fail(DMOE_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
    return DMOE_OK;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DMOE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return DMOE_OK;
}

// ---- workspace layouts -----------------------------------------------------------------------------
struct SelectWs {
    size_t group_off, mask, total;
};
SelectWs select_ws(int T, int E, bool need_mask) {
    SelectWs w{};
    size_t o = 0;
    w.group_off = o;
    o += align_up(sizeof(int32_t) * (size_t)(div_up(T, kGroup) + 1) * E);
    w.mask = o;
    if (need_mask) o += align_up(sizeof(uint64_t) * (size_t)T * div_up(E, 64));
    w.total = o;
    return w;
}

struct LayerWs {
    size_t scores, mask, group_off, sub_cnt, counts, offsets, item_start, witem, wfirst, lists, H, H8, hs8, colmask, partial, hid, x8, xscale, xhat, total;
};
LayerWs layer_ws(const dmoe_layer& L, int T) {
    LayerWs w{};
    const int E = L.n_experts;
    size_t o = 0;
    w.scores = o;     o += align_up(sizeof(float) * (size_t)T * E);
    w.mask = o;       o += align_up(sizeof(uint64_t) * (size_t)T * div_up(E, 64));
    w.group_off = o;  o += align_up(sizeof(int32_t) * (size_t)(div_up(T, kGroup) + 1) * E);
    // counts per part of a group when the router runs several workgroups per group
    // (sized so that the workspace never shrinks as T grows: at most 4 parts x 192 groups)
    w.sub_cnt = o;
    if (L.dtype == DMOE_BF16)
        o += align_up(sizeof(int32_t) * (size_t)std::min(div_up(T, 16), 4 * 192) * E);
    w.counts = o;     o += align_up(sizeof(int32_t) * (size_t)E);
    w.offsets = o;    o += align_up(sizeof(int32_t) * (size_t)(E + 1));
    w.item_start = o; o += align_up(sizeof(int32_t) * (size_t)(E + 2));
    // window tables of the up-projection
    const int n_windows = L.dtype == DMOE_BF16 ? div_up(div_up(T, kGroup), up_window_groups(L, T)) : 0;
    w.witem = o;      o += align_up(sizeof(int32_t) * (size_t)n_windows * (E + 1));
    w.wfirst = o;     o += align_up(sizeof(int32_t) * (size_t)n_windows * E);
    // token lists aligned to work items: one entry per row of H
    w.lists = o;      o += align_up(sizeof(int32_t) * h_fragments(L, T) * 16);
    w.H = o;
    if (L.dtype == DMOE_BF16) o += align_up(h_fragments(L, T) * (m_pad_of(L.expert_size) / 32) * 1024);
    // 8-bit hidden activations: codes and scale bytes of the same rows
    w.H8 = w.hs8 = o;
    if (down_x8_shape(L)) {
        w.H8 = o;   o += align_up(h_fragments(L, T) * 16 * m_pad_of(L.expert_size));
        w.hs8 = o;  o += align_up(h_fragments(L, T) * 16);
    }
    // small-token path: which tokens keep each expert, and the per-expert-group partial outputs
    w.colmask = o;
    w.partial = o;
    if (L.dtype == DMOE_BF16) {  // also above kSmallTokens: the workspace never shrinks as T grows
        o += align_up(sizeof(uint64_t) * (size_t)E);
        w.partial = o;
        o += align_up(sizeof(float) * (size_t)kSmallMaxGroups * 16 * L.d_model);
    }
    // hidden rows of the router: 16 for the small-token kernels, all T for a router that runs as
    // two launches
    const size_t hid_rows = (L.dtype == DMOE_BF16 && router_sliced(L)) ? std::max(T, 16) : 16;
    w.hid = o;        o += align_up(2 * hid_rows * (size_t)std::max(L.router_hidden, 16));
    // 8-bit expert inputs: codes, scales and the quantised rows as bf16 (the latter for the
    // kernels that are not 8-bit: small-token path, shapes without the 8-bit up-projection)
    w.x8 = w.xscale = w.xhat = o;
    if (acts_fp8(L)) {
        w.x8 = o;     o += align_up((size_t)std::max(T, 16) * L.d_model);
        w.xscale = o; o += align_up(sizeof(float) * (size_t)std::max(T, 16));
        w.xhat = o;   o += align_up(2 * (size_t)std::max(T, 16) * L.d_model);
    }
    w.total = o;
    return w;
}

bool use_small_path(const dmoe_layer& L, int T) {
    // (8-bit hidden activations: every batch size takes the list-based kernels)
    return L.dtype == DMOE_BF16 && T <= kSmallTokens && small_bf16_supported(L) && !hidden_fp8(L);
}

// Pointers of one layer for the small-token kernels (its workspace carved as in layer_ws).
SmallMod small_mod(const dmoe_layer& L, char* ws, const LayerWs& w, float* scores, uint64_t* mask,
                   void* y, float tau) {
    const PackedLayout P = packed_layout(L);
    const char* pk = static_cast<const char*>(L.packed);
    SmallMod M{};
    M.r1f = (const __bf16*)(pk + P.r1f);
    M.r_b1 = (const __bf16*)L.r_b1;
    M.r2f = (const __bf16*)(pk + P.r2f);
    M.r_b2 = (const __bf16*)L.r_b2;
    M.wupf = (const __bf16*)(pk + P.wupf);
    M.wgatef = (const __bf16*)(pk + P.wgatef);
    M.b_up = (const __bf16*)L.b_up;
    M.w2f = (const __bf16*)(pk + P.w2f);
    M.wupf8 = (const uint8_t*)(pk + P.wupf8);
    M.wgatef8 = (const uint8_t*)(pk + P.wgatef8);
    M.w2f8 = (const uint8_t*)(pk + P.w2f8);
    // the power-of-two copy of the scales made by dmoe_pack_weights
    M.w_scales = weights_fp8(L) ? (const float*)(pk + P.scales) : nullptr;
    M.b_down = (const __bf16*)L.b_down;
    M.hid = (__bf16*)(ws + w.hid);
    M.Hs = (__bf16*)(ws + w.H);
    M.y = (__bf16*)y;
    M.scores = scores;
    M.partial = reinterpret_cast<float*>(ws + w.partial);
    M.mask = mask;
    M.colmask = reinterpret_cast<uint64_t*>(ws + w.colmask);
    M.group_cnt = reinterpret_cast<int32_t*>(ws + w.group_off);
    M.tau = tau;
    return M;
}

// Experts from mask bits whose group counts are already in group_off (both in the workspace).
// gate_mod: the small-token path takes the gate into its up-projection (the scores, the mask and
// the counts are then outputs of that kernel, described by gate_mod).
int run_experts(const dmoe_layer& L, const void* x, int T, char* ws, const LayerWs& w,
                const uint64_t* mask, int32_t* offsets_out, int32_t* lists_out, void* y,
                hipStream_t s, int split = 1, const SmallMod* gate_mod = nullptr) {
    // split > 1: the counts are in sub_cnt, split rows per group (bf16 prefill path only)
    int32_t* group_off = reinterpret_cast<int32_t*>(ws + w.group_off);
    const int32_t* sub_cnt = split > 1 ? reinterpret_cast<const int32_t*>(ws + w.sub_cnt) : nullptr;
    int32_t* counts = reinterpret_cast<int32_t*>(ws + w.counts);
    int32_t* offsets = offsets_out ? offsets_out : reinterpret_cast<int32_t*>(ws + w.offsets);
    // the kernels read the work-item-aligned copy in the workspace; the caller's is compact
    int32_t* alist = reinterpret_cast<int32_t*>(ws + w.lists);
    int32_t* item_start = reinterpret_cast<int32_t*>(ws + w.item_start);
    const uint8_t* x8 = nullptr;
    const float* xscale = nullptr;
    if (acts_fp8(L)) {
        // the experts read the row-wise quantised input: as codes + scales where the 8-bit
        // up-projection runs, as bf16 numbers everywhere else
        const bool codes = up_x8_supported(L) && !use_small_path(L, T);
        launch_quantize_x(L, x, T, reinterpret_cast<uint8_t*>(ws + w.x8),
                          reinterpret_cast<float*>(ws + w.xscale), codes ? nullptr : ws + w.xhat, s);
        x8 = reinterpret_cast<const uint8_t*>(ws + w.x8);
        xscale = reinterpret_cast<const float*>(ws + w.xscale);
        if (!codes) x = ws + w.xhat;
    }
    if (L.dtype == DMOE_F32) {
        if (offsets_out)
            launch_scan_and_fill(mask, T, L.n_experts, group_off, counts, offsets, nullptr, 64,
                                 lists_out, nullptr, 1, nullptr, nullptr, s);
        launch_ffn_f32(L, (const float*)x, T, mask, (float*)y, s);
    } else if (use_small_path(L, T)) {
        SmallGroup G{};
        G.m[0] = gate_mod ? *gate_mod : small_mod(L, ws, w, nullptr, nullptr, y, 0.0f);
        launch_small_bf16(L, G, 1, x, T, gate_mod != nullptr, s);
        if (offsets_out)  // after the experts: with the gate folded in, they write mask and counts
            launch_scan_and_fill(mask, T, L.n_experts, group_off, counts, offsets, nullptr, 64,
                                 lists_out, nullptr, 1, nullptr, nullptr, s);
    } else {
        int32_t* witem = reinterpret_cast<int32_t*>(ws + w.witem);
        int32_t* wfirst = reinterpret_cast<int32_t*>(ws + w.wfirst);
        launch_scan_and_fill(mask, T, L.n_experts, group_off, counts, offsets, item_start,
                             up_rows_bf16(L), lists_out, alist, up_window_groups(L, T), witem,
                             wfirst, s, sub_cnt, split);
        void* H = ws + w.H;
        // 8-bit hidden activations on the 8-bit matrix cores: the rows as codes + scale bytes
        const bool down8 = hidden_fp8(L) && down_x8_shape(L) && down_x8_addressable(L, T);
        uint8_t* H8 = down8 ? reinterpret_cast<uint8_t*>(ws + w.H8) : nullptr;
        uint8_t* hs8 = down8 ? reinterpret_cast<uint8_t*>(ws + w.hs8) : nullptr;
        // (the 8-bit up-projection of gated experts writes them itself; after any other
        // up-projection a kernel of its own quantises the bf16 rows)
        const bool up_writes_codes = down8 && up_x8_supported(L);
        if (up_x8_supported(L))
            launch_up_x8(L, x8, xscale, T, witem, wfirst, alist, H, up_writes_codes ? H8 : nullptr,
                         up_writes_codes ? hs8 : nullptr, s);
        else
            launch_up_bf16(L, x, T, witem, wfirst, alist, H, s);
        if (down8) {
            if (!up_writes_codes) launch_h_rows_to_e4m3(L, item_start, H, H8, hs8, s);
            launch_down_x8(L, T, item_start, group_off, mask, H8, hs8, y, s);
            return check_launch("expert kernels");
        }
        if (hidden_fp8(L)) launch_h_rows_quantize(L, item_start, H, s);  // the bf16 kernels read hq
        const long long max_sparse = down_max_pairs_sparse(L, T);
        // both are launched and the pair count on the device decides, unless the limit already does
        if (max_sparse > 0)
            launch_down_rmw_bf16(L, T, item_start, group_off, alist, offsets, H, y, max_sparse, s);
        if (max_sparse != 0x7fffffffffffffffLL)
            launch_down_bf16(L, T, item_start, group_off, mask, offsets, H, y, max_sparse, s);
    }
    return check_launch("expert kernels");
}

}  // namespace

LaunchTimer::LaunchTimer(int slot, hipStream_t stream)
    : slot_(slot), index_(-1), used_(false), prev_(g_scope), stream_(stream) {
    if (g_timing && g_ev_used < kEventPairs) {
        index_ = g_ev_used++;
        g_ev_slot[index_] = -1;  // until a launch takes the pair
        g_ev_first[index_] = 1;
    }
    g_scope = this;
}
LaunchTimer::~LaunchTimer() { g_scope = prev_; }

bool timer_events_for_launch(hipEvent_t* start, hipEvent_t* stop) {
    LaunchTimer* t = g_scope;
    if (!t || t->index_ < 0) return false;
    int idx = t->index_;
    if (t->used_) {  // a further kernel of the same scope
        if (g_ev_used >= kEventPairs) return false;
        idx = g_ev_used++;
        g_ev_first[idx] = 0;
    }
    t->used_ = true;
    g_ev_slot[idx] = t->slot_;
    *start = g_ev[2 * idx];
    *stop = g_ev[2 * idx + 1];
    return true;
}

}  // namespace dmoe

using namespace dmoe;

extern "C" {

int32_t dmoe_version(void) { return 100; }

const char* dmoe_last_error(void) { return g_err; }

int32_t dmoe_workspace_bytes(const dmoe_layer* layer, int32_t n_tokens, size_t* out_bytes) {
    if (!out_bytes) return fail(DMOE_ERR_NULL, "out_bytes is NULL");
    if (int rc = check_layer(layer, false, false)) return rc;
    if (int rc = check_tokens(n_tokens, layer->n_experts)) return rc;
    *out_bytes = layer_ws(*layer, n_tokens).total;
    return DMOE_OK;
}

int32_t dmoe_select_workspace_bytes(int32_t n_tokens, int32_t n_experts, size_t* out_bytes) {
    if (!out_bytes) return fail(DMOE_ERR_NULL, "out_bytes is NULL");
    if (n_experts <= 0) return fail(DMOE_ERR_SHAPE, "n_experts must be positive");
    if (int rc = check_tokens(n_tokens, n_experts)) return rc;
    *out_bytes = select_ws(n_tokens, n_experts, true).total;
    return DMOE_OK;
}

int32_t dmoe_packed_bytes(const dmoe_layer* layer, size_t* out_bytes) {
    if (!out_bytes) return fail(DMOE_ERR_NULL, "out_bytes is NULL");
    if (int rc = check_layer(layer, false, false)) return rc;
    *out_bytes = packed_layout(*layer).total;
    return DMOE_OK;
}

int32_t dmoe_pack_weights(const dmoe_layer* layer, void* packed, size_t packed_bytes, void* stream) {
    if (int rc = check_layer(layer, false, false)) return rc;
    if (layer->dtype == DMOE_F32) return DMOE_OK;
    if (!layer->w_down || !layer->w_up || (layer->gated && !layer->w_gate))
        return fail(DMOE_ERR_NULL, "expert weights are NULL");
    // a layer with a router is packed with it: the router kernels read only the packed matrices
    if (layer->router_hidden > 0 && (!layer->r_w1 || !layer->r_w2))
        return fail(DMOE_ERR_NULL, "router_hidden > 0 but r_w1 / r_w2 is NULL (set router_hidden = 0 "
                                   "for a layer that is only used through dmoe_expert_ffn)");
    if (layer->router_hidden > 0 && !router_bf16_supported(*layer))
        return fail(DMOE_ERR_UNSUPPORTED, "bf16 router needs d %% 32 == 0 and d_h in {32,64,128,256,512}");
    if (!experts_bf16_supported(*layer))
        return fail(DMOE_ERR_UNSUPPORTED,
                    "bf16 experts need d %% 256 == 0 and expert_size <= 128 (<= 64 if gated)");
    size_t need = 0;
    dmoe_packed_bytes(layer, &need);
    if (!packed) return fail(DMOE_ERR_NULL, "packed is NULL");
    if (reinterpret_cast<uintptr_t>(packed) % kAlign) return fail(DMOE_ERR_WORKSPACE, "packed is not 256-byte aligned");
    if (packed_bytes < need) return fail(DMOE_ERR_WORKSPACE, "packed has %zu bytes, %zu needed", packed_bytes, need);
    launch_pack_bf16(*layer, packed, (hipStream_t)stream);
    return check_launch("pack_weights");
}

int32_t dmoe_router(const dmoe_layer* layer, const void* x, int32_t n_tokens, float* scores,
                    void* stream) {
    if (int rc = check_layer(layer, true, false)) return rc;
    if (int rc = check_tokens(n_tokens, layer->n_experts)) return rc;
    if (n_tokens == 0) return DMOE_OK;
    if (!x || !scores) return fail(DMOE_ERR_NULL, "x or scores is NULL");
    hipStream_t s = (hipStream_t)stream;
    if (layer->dtype == DMOE_F32) launch_router_f32(*layer, (const float*)x, n_tokens, scores, s);
    else if (router_fused_scores_supported(*layer))
        launch_router_fused(*layer, x, n_tokens, router_fused_split(*layer, n_tokens), scores, 0.0f,
                            nullptr, nullptr, nullptr, nullptr, s);
    else launch_router_bf16(*layer, x, n_tokens, scores, s);
    return check_launch("router");
}

}  // extern "C"

namespace {

// The gate of a call: the dynamic-k threshold (top_k < 0) or a fixed number of experts.
struct Gate {
    float tau;
    int top_k;
};
int check_gate(const Gate& g, int E) {
    if (g.top_k < 0) return check_tau(g.tau);
    if (g.top_k > E) return fail(DMOE_ERR_SHAPE, "k = %d exceeds the %d experts", g.top_k, E);
    return DMOE_OK;
}

int select_impl(const float* scores, int32_t n_tokens, int32_t n_experts, Gate gate,
                uint64_t* mask_bits, int32_t* k_per_token, int32_t* counts, int32_t* offsets,
                int32_t* token_lists, void* workspace, size_t workspace_bytes, void* stream) {
    if (n_experts <= 0) return fail(DMOE_ERR_SHAPE, "n_experts must be positive");
    if (int rc = check_tokens(n_tokens, n_experts)) return rc;
    if (int rc = check_gate(gate, n_experts)) return rc;
    if (!offsets) return fail(DMOE_ERR_NULL, "offsets is NULL");
    if (n_tokens > 0 && (!scores || !token_lists)) return fail(DMOE_ERR_NULL, "scores or token_lists is NULL");
    const SelectWs w = select_ws(n_tokens, n_experts, mask_bits == nullptr);
    if (int rc = check_ws(workspace, workspace_bytes, w.total)) return rc;
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = (hipStream_t)stream;
    int32_t* group_off = reinterpret_cast<int32_t*>(ws + w.group_off);
    uint64_t* mask = mask_bits ? mask_bits : reinterpret_cast<uint64_t*>(ws + w.mask);
    if (n_tokens > 0) {
        if (gate.top_k < 0)
            launch_mask_from_scores(scores, n_tokens, n_experts, gate.tau, mask, k_per_token, group_off, nullptr, s);
        else
            launch_mask_topk(scores, n_tokens, n_experts, gate.top_k, mask, k_per_token, group_off, nullptr, s);
    }
    launch_scan_and_fill(mask, n_tokens, n_experts, group_off, counts, offsets, nullptr, 64,
                         n_tokens > 0 ? token_lists : nullptr, nullptr, 1, nullptr, nullptr, s);
    return check_launch("select");
}

}  // namespace

extern "C" {

int32_t dmoe_select(const float* scores, int32_t n_tokens, int32_t n_experts, float tau,
                    uint64_t* mask_bits, int32_t* k_per_token, int32_t* counts, int32_t* offsets,
                    int32_t* token_lists, void* workspace, size_t workspace_bytes, void* stream) {
    return select_impl(scores, n_tokens, n_experts, Gate{tau, -1}, mask_bits, k_per_token, counts,
                       offsets, token_lists, workspace, workspace_bytes, stream);
}

int32_t dmoe_select_topk(const float* scores, int32_t n_tokens, int32_t n_experts, int32_t k,
                         uint64_t* mask_bits, int32_t* k_per_token, int32_t* counts,
                         int32_t* offsets, int32_t* token_lists, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (k < 0) return fail(DMOE_ERR_SHAPE, "k must not be negative");
    return select_impl(scores, n_tokens, n_experts, Gate{0.0f, k}, mask_bits, k_per_token, counts,
                       offsets, token_lists, workspace, workspace_bytes, stream);
}

int32_t dmoe_expert_ffn(const dmoe_layer* layer, const void* x, int32_t n_tokens,
                        const int32_t* offsets, const int32_t* token_lists, void* y,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_layer(layer, false, true)) return rc;
    if (int rc = check_tokens(n_tokens, layer->n_experts)) return rc;
    if (n_tokens == 0) return DMOE_OK;
    if (!x || !y || !offsets || !token_lists) return fail(DMOE_ERR_NULL, "x, y, offsets or token_lists is NULL");
    const LayerWs w = layer_ws(*layer, n_tokens);
    if (int rc = check_ws(workspace, workspace_bytes, w.total)) return rc;
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = (hipStream_t)stream;
    uint64_t* mask = reinterpret_cast<uint64_t*>(ws + w.mask);
    uint64_t* colmask = use_small_path(*layer, n_tokens) ? reinterpret_cast<uint64_t*>(ws + w.colmask) : nullptr;
    launch_mask_from_lists(offsets, token_lists, n_tokens, layer->n_experts, mask,
                           reinterpret_cast<int32_t*>(ws + w.group_off), colmask, s);
    return run_experts(*layer, x, n_tokens, ws, w, mask, nullptr, nullptr, y, s);
}

}  // extern "C"

namespace {

int forward_impl(const dmoe_layer* layer, const void* x, int32_t n_tokens, Gate gate, void* y,
                 float* scores_out, uint64_t* mask_out, int32_t* offsets_out,
                 int32_t* token_lists_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (int rc = check_layer(layer, true, true)) return rc;
    if (int rc = check_tokens(n_tokens, layer->n_experts)) return rc;
    if (int rc = check_gate(gate, layer->n_experts)) return rc;
    const float tau = gate.tau;
    if ((offsets_out == nullptr) != (token_lists_out == nullptr))
        return fail(DMOE_ERR_NULL, "offsets_out and token_lists_out go together");
    if (n_tokens == 0) return DMOE_OK;
    if (!x || !y) return fail(DMOE_ERR_NULL, "x or y is NULL");
    const LayerWs w = layer_ws(*layer, n_tokens);
    if (int rc = check_ws(workspace, workspace_bytes, w.total)) return rc;
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = (hipStream_t)stream;
    float* scores = scores_out ? scores_out : reinterpret_cast<float*>(ws + w.scores);
    uint64_t* mask = mask_out ? mask_out : reinterpret_cast<uint64_t*>(ws + w.mask);
    int32_t* group_off = reinterpret_cast<int32_t*>(ws + w.group_off);
    uint64_t* colmask = use_small_path(*layer, n_tokens) ? reinterpret_cast<uint64_t*>(ws + w.colmask) : nullptr;
    // the MFMA router takes any number of experts; with the gate fused in, up to 512
    const bool fused_router = layer->dtype == DMOE_BF16 && router_fused_scores_supported(*layer);
    const bool fused_gate = fused_router && router_fused_supported(*layer);
    int split = 1;
    if (fused_gate && n_tokens > kSmallTokens && gate.top_k < 0) {
        // router, dynamic-k gate and group counts in one kernel (with few token groups: several
        // workgroups per group, each with its own row of counts)
        if (!colmask) split = router_fused_split(*layer, n_tokens);
        int32_t* cnt = split > 1 ? reinterpret_cast<int32_t*>(ws + w.sub_cnt) : group_off;
        // (the gate works on the scores in registers: they go to memory only for a caller who
        // asked for them)
        launch_router_fused(*layer, x, n_tokens, split, scores_out, tau, mask, nullptr, cnt, colmask, s);
    } else if (fused_router && colmask && gate.top_k < 0 &&
               layer->n_experts <= kSmallFusedSelectMaxE) {
        SmallGroup G{};
        G.m[0] = small_mod(*layer, ws, w, scores, mask, y, tau);
        if (small_gate_in_up(*layer)) {
            // the hidden product here; the second product and the gate ride in the up-projection
            launch_router_small_hidden(*layer, G, 1, x, n_tokens, s);
            return run_experts(*layer, x, n_tokens, ws, w, mask, offsets_out, token_lists_out, y, s,
                               1, &G.m[0]);
        }
        // hidden product, then scores + gate in one workgroup
        launch_router_select_small(*layer, G, 1, x, n_tokens, s);
    } else {
        if (fused_router && n_tokens <= kSmallTokens) {
            SmallGroup G{};
            G.m[0] = small_mod(*layer, ws, w, scores, mask, y, tau);
            launch_router_small(*layer, G, 1, x, n_tokens, s);
        }
        else if (fused_router && router_sliced(*layer))
            launch_router_sliced(*layer, x, n_tokens, ws + w.hid, scores, s);
        else if (fused_router)
            launch_router_fused(*layer, x, n_tokens, router_fused_split(*layer, n_tokens), scores,
                                0.0f, nullptr, nullptr, nullptr, nullptr, s);
        else if (layer->dtype == DMOE_F32)
            launch_router_f32(*layer, (const float*)x, n_tokens, scores, s);
        else
            launch_router_bf16(*layer, x, n_tokens, scores, s);
        if (gate.top_k < 0)
            launch_mask_from_scores(scores, n_tokens, layer->n_experts, tau, mask, nullptr,
                                    group_off, colmask, s);
        else
            launch_mask_topk(scores, n_tokens, layer->n_experts, gate.top_k, mask, nullptr,
                             group_off, colmask, s);
    }
    return run_experts(*layer, x, n_tokens, ws, w, mask, offsets_out, token_lists_out, y, s, split);
}

}  // namespace

extern "C" {

int32_t dmoe_forward(const dmoe_layer* layer, const void* x, int32_t n_tokens, float tau, void* y,
                     float* scores_out, uint64_t* mask_out, int32_t* offsets_out,
                     int32_t* token_lists_out, void* workspace, size_t workspace_bytes,
                     void* stream) {
    return forward_impl(layer, x, n_tokens, Gate{tau, -1}, y, scores_out, mask_out, offsets_out,
                        token_lists_out, workspace, workspace_bytes, stream);
}

int32_t dmoe_forward_static(const dmoe_layer* layer, const void* x, int32_t n_tokens, float tau,
                            void* y, void* stream) {
    // sizes first: a layer / batch that does not fit is refused before anything else happens
    if (int rc = check_layer(layer, true, true)) return rc;
    if (int rc = check_tokens(n_tokens, layer->n_experts)) return rc;
    if (int rc = check_tau(tau)) return rc;
    if (n_tokens == 0) return DMOE_OK;
    if (!x || !y) return fail(DMOE_ERR_NULL, "x or y is NULL");
    const size_t need = layer_ws(*layer, n_tokens).total;
    if (need > kStaticScratchBytes)
        return fail(DMOE_ERR_WORKSPACE,
                    "dmoe_forward_static: %d tokens of this layer need %zu bytes of workspace, the "
                    "static one holds %zu; use dmoe_forward with a caller-owned workspace",
                    n_tokens, need, kStaticScratchBytes);
    void* ws = nullptr;
    if (int rc = static_scratch_of_current_device(&ws)) return rc;
    return forward_impl(layer, x, n_tokens, Gate{tau, -1}, y, nullptr, nullptr, nullptr, nullptr,
                        ws, kStaticScratchBytes, stream);
}

int32_t dmoe_forward_topk(const dmoe_layer* layer, const void* x, int32_t n_tokens, int32_t k,
                          void* y, float* scores_out, uint64_t* mask_out, int32_t* offsets_out,
                          int32_t* token_lists_out, void* workspace, size_t workspace_bytes,
                          void* stream) {
    if (k < 0) return fail(DMOE_ERR_SHAPE, "k must not be negative");
    return forward_impl(layer, x, n_tokens, Gate{0.0f, k}, y, scores_out, mask_out, offsets_out,
                        token_lists_out, workspace, workspace_bytes, stream);
}

int32_t dmoe_group_workspace_bytes(const dmoe_layer* const* layers, int32_t n_layers,
                                   int32_t n_tokens, size_t* out_bytes) {
    if (!layers || !out_bytes) return fail(DMOE_ERR_NULL, "layers or out_bytes is NULL");
    if (n_layers < 1 || n_layers > kGroupMax)
        return fail(DMOE_ERR_SHAPE, "a group holds 1 to %d layers", kGroupMax);
    size_t total = 0;
    for (int i = 0; i < n_layers; ++i) {
        if (int rc = check_layer(layers[i], true, true)) return rc;
        if (int rc = check_tokens(n_tokens, layers[i]->n_experts)) return rc;
        total += align_up(layer_ws(*layers[i], n_tokens).total);
    }
    *out_bytes = total;
    return DMOE_OK;
}

int32_t dmoe_forward_group(const dmoe_layer* const* layers, int32_t n_layers, const void* x,
                           int32_t n_tokens, const float* host_taus, void* const* host_ys,
                           void* workspace, size_t workspace_bytes, void* stream) {
    if (!layers || !host_taus || !host_ys) return fail(DMOE_ERR_NULL, "layers, host_taus or host_ys is NULL");
    if (n_layers < 1 || n_layers > kGroupMax)
        return fail(DMOE_ERR_SHAPE, "a group holds 1 to %d layers", kGroupMax);
    size_t need = 0, off[kGroupMax];
    for (int i = 0; i < n_layers; ++i) {
        if (int rc = check_layer(layers[i], true, true)) return rc;
        if (int rc = check_tokens(n_tokens, layers[i]->n_experts)) return rc;
        if (int rc = check_tau(host_taus[i])) return rc;
        const dmoe_layer &A = *layers[0], &B = *layers[i];
        if (A.d_model != B.d_model || A.n_experts != B.n_experts || A.expert_size != B.expert_size ||
            A.router_hidden != B.router_hidden || A.gated != B.gated || A.act != B.act ||
            A.dtype != B.dtype || A.weight_format != B.weight_format)
            return fail(DMOE_ERR_UNSUPPORTED, "the layers of a group must have one shape, activation and dtype");
        off[i] = need;
        need += align_up(layer_ws(B, n_tokens).total);
    }
    if (n_tokens == 0) return DMOE_OK;
    if (!x) return fail(DMOE_ERR_NULL, "x is NULL");
    for (int i = 0; i < n_layers; ++i)
        if (!host_ys[i]) return fail(DMOE_ERR_NULL, "host_ys[%d] is NULL", i);
    if (int rc = check_ws(workspace, workspace_bytes, need)) return rc;
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = (hipStream_t)stream;
    const dmoe_layer& L0 = *layers[0];
    // (layers with 8-bit inputs quantise x per layer call: they take the layer-by-layer route)
    bool fused = use_small_path(L0, n_tokens) && !acts_fp8(L0);
    for (int i = 0; i < n_layers; ++i) fused = fused && router_fused_scores_supported(*layers[i]);
    if (!fused) {  // larger batches: one layer after the other, each in its share of the workspace
        for (int i = 0; i < n_layers; ++i) {
            const size_t share = align_up(layer_ws(*layers[i], n_tokens).total);
            if (int rc = forward_impl(layers[i], x, n_tokens, Gate{host_taus[i], -1}, host_ys[i], nullptr,
                                      nullptr, nullptr, nullptr, ws + off[i], share, stream))
                return rc;
        }
        return DMOE_OK;
    }
    SmallGroup G{};
    for (int i = 0; i < n_layers; ++i) {
        const LayerWs w = layer_ws(*layers[i], n_tokens);
        char* wsi = ws + off[i];
        G.m[i] = small_mod(*layers[i], wsi, w, reinterpret_cast<float*>(wsi + w.scores),
                           reinterpret_cast<uint64_t*>(wsi + w.mask), host_ys[i], host_taus[i]);
    }
    const bool gate_in_up = small_gate_in_up(L0);
    if (gate_in_up) {
        launch_router_small_hidden(L0, G, n_layers, x, n_tokens, s);
    } else if (L0.n_experts <= kSmallFusedSelectMaxE) {
        launch_router_select_small(L0, G, n_layers, x, n_tokens, s);
    } else {
        launch_router_small(L0, G, n_layers, x, n_tokens, s);
        launch_select_small_group(L0, G, n_layers, n_tokens, s);
    }
    launch_small_bf16(L0, G, n_layers, x, n_tokens, gate_in_up, s);
    return check_launch("group kernels");
}

int32_t dmoe_timing_enable(int32_t on) {
    if (on && g_ev.empty()) {
        g_ev.resize(2 * kEventPairs);
        g_ev_slot.resize(kEventPairs);
        g_ev_first.resize(kEventPairs);
        for (auto& ev : g_ev) {
            hipError_t e = hipEventCreate(&ev);
            if (e != hipSuccess) {
                g_ev.clear();
                return fail(DMOE_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
            }
        }
    }
    g_timing = on != 0;
    return DMOE_OK;
}

int32_t dmoe_timing_reset(void) {
    const int rc = collect_events();
    memset(g_launches, 0, sizeof(g_launches));
    for (double& v : g_ms) v = 0.0;
    return rc;
}

int32_t dmoe_timing_slots(void) { return kSlotCount; }

int32_t dmoe_timing_read(int32_t index, const char** name, int64_t* launches, double* total_ms) {
    if (index < 0 || index >= kSlotCount) return fail(DMOE_ERR_SHAPE, "timing slot out of range");
    if (int rc = collect_events()) return rc;
    if (name) *name = kSlotNames[index];
    if (launches) *launches = g_launches[index];
    if (total_ms) *total_ms = g_ms[index];
    return DMOE_OK;
}

}  // extern "C"

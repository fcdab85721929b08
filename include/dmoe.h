/*
 * dmoe.h -- C ABI of the MI355X (gfx950) dynamic-k Mixture-of-Experts FFN forward.
 *
 * The layer is the inference module of "Dense to Dynamic-k Mixture-of-Experts" (D2DMoE):
 *   1. a two-layer router predicts, per token, the L2 norm of every expert's output (Sec. 3.3);
 *   2. the dynamic-k gate keeps expert i iff its score is >= tau * the token's maximum score
 *      (Sec. 3.4, Eq. 4);
 *   3. tokens are bucketed per expert (the metadata of Appendix C, in compact form);
 *   4. each selected expert runs up-projection (+gate), activation and down-projection, and the
 *      expert outputs are summed, unweighted, on top of the output bias, which stays outside
 *      the experts (Sec. 3.2; gated form: Appendix G).
 *
 * Conventions
 *   - Plain C.  Every entry point returns a dmoe_status; DMOE_OK is 0.  dmoe_last_error() gives
 *     a thread-local text for the last failure.
 *   - All argument errors are found on the host BEFORE anything is launched, so a failing call
 *     leaves every buffer untouched.
 *   - Pointers are DEVICE pointers unless the name says host.  The caller owns every buffer; the
 *     library allocates nothing, frees nothing and never synchronises the stream (its only state
 *     between calls: the per-GPU address of dmoe_forward_static's array, the one-time kernel
 *     attributes and, when enabled, the event pool of the timing aid).  Work is
 *     enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Row-major, innermost index last.  x[T][d] and y[T][d] have the layer's dtype; scores are
 *     always fp32.  Expert-major weights: w_up[E][m][d], w_gate[E][m][d] (gated only),
 *     b_up[E][m] (nullable), w_down[E][m][d] (row j of expert e is the d-vector that neuron j of
 *     that expert adds to the output), b_down[d] (nullable).  Router: r_w1[d_h][d], r_b1[d_h]
 *     (nullable), r_w2[E][d_h], r_b2[E] (nullable).  Biases have the layer's dtype.
 *   - Workspaces must be 256-byte aligned and at least as large as the matching *_workspace_bytes
 *     call says; their contents are scratch.
 *   - Unsupported shapes/dtypes are refused with DMOE_ERR_UNSUPPORTED; there is no fallback path.
 *     Supported: any n_tokens >= 0 with n_tokens * n_experts < 2^31 - 64 and n_experts <= 4096.
 *     bf16 layers: d_model a multiple of 256, expert_size 1 .. 128 (1 .. 64 if gated), router with
 *     router_hidden in {32, 64, 128, 256, 512}.  fp32 layers (the
 *     exactness configuration, one workgroup per token): d_model + router_hidden <= 16384 and
 *     2 d_model + expert_size <= 16384.
 */
#ifndef DMOE_H
#define DMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DMOE_OK = 0,
    DMOE_ERR_NULL = 1,        /* a required pointer is NULL */
    DMOE_ERR_SHAPE = 2,       /* a size is negative, zero where it must not be, or T*E overflows */
    DMOE_ERR_UNSUPPORTED = 3, /* dtype / activation / shape the kernels do not cover */
    DMOE_ERR_TAU = 4,         /* tau is NaN or outside [0, 1] */
    DMOE_ERR_WORKSPACE = 5,   /* workspace missing, too small or not 256-byte aligned */
    DMOE_ERR_HIP = 6          /* a HIP call failed; see dmoe_last_error() */
} dmoe_status;

enum { DMOE_F32 = 0, DMOE_BF16 = 1 };
/* storage of the expert matrices w_up, w_gate, w_down (dmoe_layer.weight_format) */
enum { DMOE_W_NATIVE = 0, DMOE_W_FP8_E4M3 = 1, DMOE_W_FP8_E4M3_X8 = 2, DMOE_W_FP8_E4M3_A8 = 3 };
enum { DMOE_ACT_RELU = 0, DMOE_ACT_GELU_ERF = 1, DMOE_ACT_GELU_TANH = 2 };

/*
 * One converted layer (Sec. 3.2-3.3).  `packed` is NULL or the buffer filled by
 * dmoe_pack_weights(); the bf16 expert kernels need it (DMOE_ERR_NULL otherwise), the fp32
 * kernels ignore it.  A gated layer must have b_up == NULL: Appendix G states the gated form
 * without biases, so where one would enter is undefined (DMOE_ERR_UNSUPPORTED).
 */
typedef struct {
    int32_t d_model;       /* d   */
    int32_t n_experts;     /* E   */
    int32_t expert_size;   /* m   neurons per expert */
    int32_t router_hidden; /* d_h */
    int32_t gated;         /* 0 plain two-layer FFN, 1 gated (GLU) FFN */
    int32_t act;           /* DMOE_ACT_* */
    int32_t dtype;         /* DMOE_F32 | DMOE_BF16: x, y and every parameter */
    int32_t weight_format; /* DMOE_W_NATIVE: expert matrices in `dtype`; DMOE_W_FP8_E4M3*: see below */
    const void *w_up, *w_gate, *b_up, *w_down, *b_down;
    const void *r_w1, *r_b1, *r_w2, *r_b2;
    const void *packed;
    const float *w_scales; /* DMOE_W_FP8_E4M3*: [E][3] fp32, see below; else ignored */
} dmoe_layer;

/*
 * Lower-precision experts (Appendix C times the experts in float16 and int8 as well; here weight-only 8-bit
 * floating point, the format the gfx950 matrix units and converters handle natively).
 * With weight_format == DMOE_W_FP8_E4M3 (bf16 layers only) w_up, w_gate and w_down hold one byte
 * per weight in the OCP 8-bit format E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits;
 * no infinities, largest value 448; the two NaN codes 0x7f / 0xff must not occur), in the same
 * [E][m][d] order, and
 *   W_up,e = w_scales[3e+0] * e4m3(w_up[e]),  W_gate,e = w_scales[3e+1] * e4m3(w_gate[e]),
 *   W_down,e = w_scales[3e+2] * e4m3(w_down[e]).
 * Every scale must be a power of two: then each weight is exactly a bf16 number, and the layer
 * computes what a DMOE_W_NATIVE bf16 layer with those weights computes -- the prefill kernels
 * run on bf16 copies made by dmoe_pack_weights, the small-token kernels (up to 16 tokens, where
 * the weights are the traffic) stream the bytes and convert in registers.  dmoe_pack_weights
 * replaces a scale that is not a power of two by the nearest one (in log2; zero stays zero) and
 * every kernel uses that copy, so all batch sizes compute the same layer.  w_scales is read by
 * dmoe_pack_weights only.  x, y, biases and the router stay bf16.
 *
 * DMOE_W_FP8_E4M3_X8 is DMOE_W_FP8_E4M3 with the experts' input quantised as well, so that the
 * up-projection (and gate) multiplies 8-bit operands on the matrix cores -- the counterpart of
 * the int8 layers Appendix C times.  The experts (not the router) read, instead of x_t,
 *   xq_t = s_t * e4m3(x_t / s_t),   s_t = 2^ceil(log2(max_j |x_tj| / 448))   (s_t = 1 for a zero row;
 *                                   its exponent is clamped to -100 .. 100),
 * where e4m3(.) rounds to the nearest E4M3 value, ties to the even mantissa (the largest
 * element of a row lands in (224, 448], so nothing overflows; magnitudes below 2^-10 s_t become
 * zero; a row with an element beyond 448 * 2^100, or a non-finite one, is outside the format and
 * its quantised values are unspecified).  Every xq element is a bf16 number, so the layer computes what a bf16 layer with the
 * same weights computes on the input xq, up to the summation: the 8-bit matrix-core instruction
 * adds the products of a 32-wide block with less than fp32 precision (measured: within 3e-4 of
 * the block's largest product).  The hidden activations and the down-projection are as in
 * DMOE_W_FP8_E4M3.  The definition holds for every batch size; the 8-bit matrix-core kernel
 * runs for batches above 16 tokens on experts of 128 neurons (64 if gated), other shapes run
 * their bf16 kernels on xq.
 *
 * DMOE_W_FP8_E4M3_A8 is DMOE_W_FP8_E4M3_X8 with the hidden activations quantised as well, so that
 * the down-projection multiplies 8-bit operands too (a fully 8-bit layer): the m hidden
 * activations of every selected (token, expert) pair, rounded to bf16 as in the other formats,
 * are replaced by
 *   hq = s * e4m3(h / s),   s = 2^ceil(log2(max_j |h_j| / 448))   (the rule of xq, per pair)
 * before they meet W_down.  Every batch size computes this definition; the 8-bit matrix-core
 * down-projection runs for H rows of 64 or 128 neurons (33 .. 128 neurons per expert), smaller
 * experts quantise H in place and run their bf16 kernels on hq; batches of up to 16 tokens take the
 * same kernels as larger ones (no weight-streaming path in this format).
 */

/* Library version (major*10000 + minor*100 + patch) and the text of the last error of the
 * calling thread ("" if none).  The returned string is owned by the library. */
int32_t dmoe_version(void);
const char *dmoe_last_error(void);

/* ---- sizes (host only, nothing is launched) ------------------------------------------------ */

/* Workspace that dmoe_forward / dmoe_expert_ffn need for n_tokens tokens (worst case: every
 * token selects every expert).  The requirement never shrinks as n_tokens grows, so a buffer
 * sized for the largest batch serves every smaller one. */
int32_t dmoe_workspace_bytes(const dmoe_layer *layer, int32_t n_tokens, size_t *out_bytes);
/* Workspace of dmoe_select. */
int32_t dmoe_select_workspace_bytes(int32_t n_tokens, int32_t n_experts, size_t *out_bytes);
/* Size of the packed-weights buffer of this layer (0 for fp32 layers). */
int32_t dmoe_packed_bytes(const dmoe_layer *layer, size_t *out_bytes);

/*
 * One-time re-layout of the weights for the MFMA kernels (bf16 layers): writes, into `packed`
 * (device, 256-byte aligned, dmoe_packed_bytes() large), the expert matrices (w_up, w_gate, w_down
 * -- the latter in two orders) and the router matrices (r_w1, r_w2) as 1 KiB blocks in the
 * register order of the matrix-core operands, the expert size rounded up to a multiple of 32
 * with zero neurons.  The layout is private to the library.  Reads the layer's weight pointers;
 * asynchronous on `stream`.  Put the pointer into layer->packed afterwards and keep the buffer
 * (and the original weights) alive as long as the layer is used.  For fp32 layers this is a
 * no-op that accepts packed == NULL.
 */
int32_t dmoe_pack_weights(const dmoe_layer *layer, void *packed, size_t packed_bytes,
                          void *stream);

/* ---- the hot path --------------------------------------------------------------------------- */

/*
 * Router (Sec. 3.3): scores[t][i] = | r_w2[i] . relu(r_w1 x_t + r_b1) + r_b2[i] |, fp32 out.
 * bf16 layers: products on the matrix cores with fp32 accumulation, the hidden vector is
 * rounded to bf16 between the two layers.  fp32 layers: fp32 throughout.
 * n_tokens == 0 is a no-op.
 */
int32_t dmoe_router(const dmoe_layer *layer, const void *x, int32_t n_tokens,
                    float *scores /* [T][E] */, void *stream);

/*
 * Dynamic-k gate + bucketing (Sec. 3.4 Eq. 4; Appendix C metadata).
 * Expert i of token t is kept iff (double)scores[t][i] >= (double)tau * (double)max_j scores[t][j]
 * -- the exact real comparison of the fp32 inputs (the fp64 product of two fp32 values is exact).
 * tau == 0 keeps every expert.  Scores must be finite; otherwise the selection is unspecified
 * but every output stays in range.
 *   mask_bits   [T][ceil(E/64)] u64, bit (i % 64) of word (i / 64) = expert i kept; nullable
 *   k_per_token [T] number of experts kept; nullable
 *   counts      [E] tokens per expert; nullable
 *   offsets     [E+1] exclusive prefix sum of counts, offsets[E] = P = number of pairs
 *   token_lists capacity T*E; the tokens of expert e are token_lists[offsets[e]..offsets[e+1]),
 *               in ascending order
 */
int32_t dmoe_select(const float *scores, int32_t n_tokens, int32_t n_experts, float tau,
                    uint64_t *mask_bits, int32_t *k_per_token, int32_t *counts, int32_t *offsets,
                    int32_t *token_lists, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Expert execution and merge (Sec. 3.2, Appendix G) for ANY valid per-expert token lists, e.g.
 * Bernoulli-sampled decisions as in the latency experiment of Sec. 4.4:
 *   y_t = b_down + sum over the experts e whose list holds t of E_e(x_t),
 *   plain  E_e(x) = w_down[e]^T A(w_up[e] x + b_up[e]),
 *   gated  E_e(x) = w_down[e]^T ( A(w_gate[e] x) o (w_up[e] x) ).
 * y is fully overwritten; a token in no list gets b_down (or 0).  Lists may be in any order;
 * a token listed twice for one expert counts once; entries outside [0, T) are ignored.
 * bf16 layers: fp32 accumulation, the hidden activations are rounded to bf16 before the
 * down-projection, expert outputs are summed in fp32 and rounded to bf16 once.
 */
int32_t dmoe_expert_ffn(const dmoe_layer *layer, const void *x, int32_t n_tokens,
                        const int32_t *offsets /* [E+1] */, const int32_t *token_lists,
                        void *y, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole layer on one stream with no host synchronisation: router (Sec. 3.3), dynamic-k gate
 * (Sec. 3.4, Eq. 4), bucketing (the metadata of Appendix C) and the selected experts summed on
 * top of b_down (Sec. 3.2; gated experts Appendix G) -- what dmoe_router, dmoe_select and
 * dmoe_expert_ffn compute one after the other.  Optional outputs (each nullable):
 * scores_out [T][E] fp32, mask_out [T][ceil(E/64)], offsets_out [E+1] and token_lists_out
 * (capacity T*E; both or neither).  An output that is not asked for may never be written at all
 * (the fused router and gate keep the scores in registers), so NULL is also the faster call.
 */
int32_t dmoe_forward(const dmoe_layer *layer, const void *x, int32_t n_tokens, float tau,
                     void *y, float *scores_out, uint64_t *mask_out, int32_t *offsets_out,
                     int32_t *token_lists_out, void *workspace, size_t workspace_bytes,
                     void *stream);

/*
 * dmoe_forward for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as dmoe_forward
 * (bit for bit: the same kernels run), without the optional outputs.  The workspace is a 32 MiB
 * array that lives in the library's device image -- every GPU the library runs on holds its own
 * copy until the process ends -- so the call refuses (DMOE_ERR_WORKSPACE, nothing launched) any
 * layer / n_tokens whose dmoe_workspace_bytes() exceeds 32 MiB: e.g. the 256 x 64 gated layer of
 * the 16-token decode configuration needs 14 MiB, 128 experts of 24 fit up to about 3000 tokens.
 * It calls no hipMalloc / hipFree or other allocating routine.  The first call on a GPU looks the
 * array's address up once (make that call outside a graph capture).  All calls on one GPU share
 * that GPU's array, which keeps the previous call's contents -- nothing in it needs to start at
 * zero -- so calls that overlap on one GPU (different streams, different threads) race: order
 * them on one stream or with events.
 */
int32_t dmoe_forward_static(const dmoe_layer *layer, const void *x, int32_t n_tokens, float tau,
                            void *y, void *stream);

/* ---- the conventional top-k gate (the rule Sec. 3.3 / 3.4 compare dynamic-k against) --------- */

/*
 * As dmoe_select / dmoe_forward, but every token keeps exactly k experts: those with the k
 * largest scores, ties at the k-th score going to the lower expert index.  0 <= k <= E
 * (DMOE_ERR_SHAPE otherwise); k == 0 keeps nothing (y = b_down), k == E is the dense layer.
 * Same buffers, workspace sizes, ownership and asynchrony as the dynamic-k calls.
 */
int32_t dmoe_select_topk(const float *scores, int32_t n_tokens, int32_t n_experts, int32_t k,
                         uint64_t *mask_bits, int32_t *k_per_token, int32_t *counts,
                         int32_t *offsets, int32_t *token_lists, void *workspace,
                         size_t workspace_bytes, void *stream);
int32_t dmoe_forward_topk(const dmoe_layer *layer, const void *x, int32_t n_tokens, int32_t k,
                          void *y, float *scores_out, uint64_t *mask_out, int32_t *offsets_out,
                          int32_t *token_lists_out, void *workspace, size_t workspace_bytes,
                          void *stream);

/* ---- several converted layers with one input (the attention projections, Sec. 3.5) ------------- */

/*
 * Sec. 3.5 replaces the query, key, value and output projections of an attention layer by small
 * MLPs that are then converted like an FFN, so a Transformer block holds four more dynamic-k
 * layers; Q, K and V read the same input.  dmoe_forward_group runs 1 to 4 layers of ONE shape
 * (d_model, n_experts, expert_size, router_hidden, gated, act, dtype all equal; weights, biases and
 * tau per layer) on the same x and writes layer i's output to host_ys[i].  Up to 16 tokens (bf16
 * layers) every stage -- router, gate, up-projection, down-projection, merge -- is ONE launch for
 * the whole group, which is what counts at that size; for more tokens the layers run one after
 * the other exactly as dmoe_forward would run them.  Results are those of dmoe_forward, bit for
 * bit.
 *   layers     host array of n_layers pointers to host dmoe_layer structs
 *   host_taus  host array of n_layers thresholds, each in [0, 1]
 *   host_ys    host array of n_layers DEVICE pointers, y_i[T][d] each, distinct
 *   workspace  dmoe_group_workspace_bytes() large (the sum of the layers' dmoe_workspace_bytes),
 *              256-byte aligned
 * DMOE_ERR_SHAPE for n_layers outside 1..4, DMOE_ERR_UNSUPPORTED for layers of different shape;
 * otherwise the errors, ownership and asynchrony of dmoe_forward.
 */
int32_t dmoe_group_workspace_bytes(const dmoe_layer *const *layers, int32_t n_layers,
                                   int32_t n_tokens, size_t *out_bytes);
int32_t dmoe_forward_group(const dmoe_layer *const *layers, int32_t n_layers, const void *x,
                           int32_t n_tokens, const float *host_taus, void *const *host_ys,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ---- per-kernel timing (measurement aid) ----------------------------------------------------- */

/*
 * When enabled, every kernel launch of the library stamps a pair of HIP events with the start and
 * the end of that kernel on the device (hipExtLaunchKernel on the launch stream), so the sums
 * are kernel time without the gaps around event records.  dmoe_timing_read() waits for those
 * events and returns, for kernel slot `index` (0 .. dmoe_timing_slots()-1), its name, the number
 * of launches (a step that takes two kernels counts once) and the summed duration in
 * milliseconds since the last dmoe_timing_reset().  Enabling allocates the event pool (the only
 * allocation the library ever makes); launches beyond the pool are not timed.  Not thread-safe;
 * meant for a benchmark's separate measurement pass.
 */
int32_t dmoe_timing_enable(int32_t on);
int32_t dmoe_timing_reset(void);
int32_t dmoe_timing_slots(void);
int32_t dmoe_timing_read(int32_t index, const char **name, int64_t *launches, double *total_ms);

#ifdef __cplusplus
}
#endif
#endif /* DMOE_H */

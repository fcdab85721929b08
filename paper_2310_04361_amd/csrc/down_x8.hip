// Down-projection with 8-bit hidden activations (weight format DMOE_W_FP8_E4M3_A8: the fully 8-bit
// reading of the lower-precision layers of Appendix C).
//
//   quantise  every H row that the up-projection wrote (bf16) by the row rule of the experts'
//             input: power-of-two scale from the row maximum, nearest E4M3 value, ties to even --
//             to codes + one E8M0 scale byte per row for the kernel below, or in place (the
//             quantised values are bf16 numbers) for the shapes that keep a bf16 down-projection.
//   down      y_t = b_down + sum over the selected experts of W_down,e^T hq (Sec. 3.2), the sum over
//             experts inside the matrix cores as in down_bf16.hip -- a workgroup owns 128 tokens x
//             256 columns as fp32 accumulators and walks all experts; tokens that did not select
//             an expert are zero columns of the B operand (out-of-range buffer loads) -- on
//             v_mfma_scale_f32_32x32x64_f8f6f4: one instruction per expert, token tile and column
//             tile, the row scale of H and the expert's weight scale as the instruction's block
//             scales.  Half the operand bytes and half the matrix-pipe time of the bf16 kernel.
//             H rows of 128 neurons are two such units of 64 per expert (UPE = 2): the same
//             pipeline walks units, and the selection of an expert is worked out at its first.
#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRawBuffer = 0x00020000;

// Operand layout of v_mfma_scale_f32_32x32x64_f8f6f4 (lane = 32h + c): 32 bytes per lane; bytes
// 0..15 belong to the instruction's first 32-wide K block and bytes 16..31 to its second, the
// scale of (row or column c, block b) is taken from lane (h = b, c).  Here every row has ONE
// scale, so both lanes of a row carry the same byte and only "the same k in the same (lane,
// byte) of A and B" matters: lane (h, c) holds the neurons 32h .. 32h + 31.
__device__ __forceinline__ f32x16 mfma64(i32x8 a, i32x8 b, f32x16 c, int sa, int sb) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, sa, 0, sb);
}

// E4M3 value nearest to v (|v| <= 448), ties to even, and its code: see quantize_x_kernel in
// ffn_x8.hip for the arithmetic (integer-exact: a / step is exact, rintf rounds to nearest-even).
__device__ __forceinline__ uint32_t e4m3_code_and_value(float v, float* value) {
    const float a = fabsf(v);
    int e = (int)((__float_as_uint(a) >> 23) & 0xffu) - 127;
    e = max(e, -6);
    float r = rintf(ldexpf(a, 3 - e));   // 0 .. 16
    *value = copysignf(ldexpf(r, e - 3), v);
    uint32_t code;
    if (r < 8.0f) {
        code = (uint32_t)r;
    } else {
        if (r == 16.0f) {
            e += 1;
            r = 8.0f;
        }
        code = ((uint32_t)(e + 7) << 3) | ((uint32_t)r - 8u);
    }
    return code | (v < 0.0f ? 0x80u : 0u);
}

// H rows of MP bf16 neurons, MP / 8 lanes per row.  CODES: H8[row][MP] and hs8[row]; otherwise
// the quantised values back into H.
template <int MP, bool CODES>
__global__ __launch_bounds__(256) void h_rows_quantize_kernel(__bf16* __restrict__ H,
                                                              const int32_t* __restrict__ item_start,
                                                              int E, int rows_per_item,
                                                              uint8_t* __restrict__ H8,
                                                              uint8_t* __restrict__ hs8) {
    constexpr int LPR = MP / 8;  // lanes per row: 4, 8 or 16
    const int rows = item_start[E] * rows_per_item;
    const int sub = threadIdx.x % LPR;
    const int n_threads = gridDim.x * blockDim.x;
    // every lane of a wavefront runs the same number of trips (the shuffles need their partners)
    const int trips = (rows + n_threads / LPR - 1) / (n_threads / LPR);
    for (int it = 0; it < trips; ++it) {
        const int row = (blockIdx.x * blockDim.x + threadIdx.x) / LPR + it * (n_threads / LPR);
        const bool live = row < rows;
        bf16x8 v = zero8();
        if (live) v = load8(H + (size_t)row * MP + 8 * sub);
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf((float)v[i]));
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        // smallest power of two s with amax / s <= 448 = 0.875 * 2^9 (1 for a zero row)
        int s_exp = 0;
        if (amax > 0.0f && amax < INFINITY) {
            int ex;
            const float f = frexpf(amax, &ex);
            s_exp = f <= 0.875f ? ex - 9 : ex - 8;
            s_exp = min(max(s_exp, -100), 100);
        }
        if (!live) continue;
        if (CODES) {
            // the hardware converter gives the codes of e4m3_code_and_value for every bf16 input
            // of magnitude up to 448 (checked exhaustively on the device)
            float a[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) a[i] = ldexpf((float)v[i], -s_exp);
            int lo = __builtin_amdgcn_cvt_pk_fp8_f32(a[0], a[1], 0, false);
            lo = __builtin_amdgcn_cvt_pk_fp8_f32(a[2], a[3], lo, true);
            int hi = __builtin_amdgcn_cvt_pk_fp8_f32(a[4], a[5], 0, false);
            hi = __builtin_amdgcn_cvt_pk_fp8_f32(a[6], a[7], hi, true);
            *reinterpret_cast<uint2*>(H8 + (size_t)row * MP + 8 * sub) = make_uint2((uint32_t)lo, (uint32_t)hi);
            if (sub == 0) hs8[row] = (uint8_t)(127 + s_exp);
        } else {
            bf16x8 q;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float val;
                (void)e4m3_code_and_value(ldexpf((float)v[i], -s_exp), &val);
                q[i] = (__bf16)ldexpf(val, s_exp);   // exact: four significant bits
            }
            *reinterpret_cast<bf16x8*>(H + (size_t)row * MP + 8 * sub) = q;
        }
    }
}

// w_down (E4M3 codes) [E][m][d] -> w2x8[E * UPE][d/32][64][32], a unit being 64 consecutive neurons
// of an expert: lane (h, r) of block (unit, column tile) holds the unit's neurons 32h .. 32h+31 of
// output column 32*tile + 16*((r>>2)&1) + 4*(r>>3) + (r&3)
// (the column order that makes a lane's 16 accumulators 16 consecutive columns); wsc8[unit] = the
// E8M0 byte of the magnitude of its expert's (power-of-two) down scale -- a negative scale flips
// the sign bit of the expert's codes instead, a zero scale zeroes them.
__global__ void pack_down_x8_kernel(const uint8_t* __restrict__ w, const float* __restrict__ scales,
                                    uint8_t* __restrict__ out, uint8_t* __restrict__ wsc8, int E,
                                    int m, int d, int UPE) {
    const size_t n = (size_t)E * UPE * (d / 32) * 2048;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    if (i < (size_t)E * UPE) {
        int ex = 1;
        (void)frexpf(fabsf(scales[3 * (i / UPE) + 2]), &ex);  // |scale| = 0.5 * 2^ex exactly (a power of two)
        wsc8[i] = (uint8_t)min(max(127 + ex - 1, 0), 254);
    }
    for (; i < n; i += stride) {
        const int j = (int)(i & 31), lane = (int)((i >> 5) & 63);
        size_t f = i >> 11;
        const int ct = (int)(f % (d / 32));
        const int unit = (int)(f / (d / 32));
        const int e = unit / UPE;
        const int h = lane >> 5, r = lane & 31;
        const int col = 32 * ct + 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
        const int neuron = 64 * (unit % UPE) + 32 * h + j;
        const float sc = scales[3 * e + 2];
        uint8_t b = neuron < m ? w[((size_t)e * m + neuron) * d + col] : (uint8_t)0;
        if (sc < 0.0f) b ^= 0x80;
        if (sc == 0.0f) b = 0;
        out[i] = b;
    }
}

constexpr int kD8Tokens = 128, kD8Tiles = 4, kD8CT = 2;
constexpr int kD8Image = kD8Tiles * 64 * 32;   // the four B tiles of one expert: 8 KiB
constexpr int kD8Buf = kD8Image + kD8Tokens;   // + one scale byte per token
constexpr int kD8Lds = 2 * kD8Buf;

// UPE = units of 64 neurons per expert (H rows of 64 * UPE bytes).
template <int UPE>
__global__ __launch_bounds__(256) void down_x8_kernel(
    const uint8_t* __restrict__ w2x8, const uint8_t* __restrict__ wsc8,
    const __bf16* __restrict__ b_down, const int32_t* __restrict__ item_start,
    const int32_t* __restrict__ group_off, const uint32_t* __restrict__ mask32,
    const uint8_t* __restrict__ H8, const uint8_t* __restrict__ hs8, __bf16* __restrict__ y, int T,
    int d, int E, int NG, int W32, int rows_per_item, uint32_t w_bytes, uint32_t h_bytes,
    uint32_t hs_bytes) {
    extern __shared__ __attribute__((aligned(16))) char img[];  // [2][kD8Buf]
    constexpr int kCols = kD8CT * 128;
    const int NS = d / kCols;
    const int k_in_xcd = blockIdx.x >> 3;
    const int chunk = (k_in_xcd / NS) * 8 + (blockIdx.x & 7), slice = k_in_xcd % NS;
    const int t_base = chunk * kD8Tokens;
    if (t_base >= T) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, c = lane & 31;
    const int col_w = slice * kCols + wave * (32 * kD8CT);

    // ---- tile-building role: select group bg of the chunk (lane = token), row half bh
    const int bg = wave & 1, bh = wave >> 1;
    const int g = chunk * 2 + bg;
    const int tok_b = g * kGroup + lane;
    const bool tok_ok = tok_b < T;
    const uint32_t* mrow = mask32 + (size_t)min(tok_b, T - 1) * W32;
    const int32_t* grow = group_off + (size_t)min(g, NG) * E;
    const int n_batches = (E + 31) >> 5;
    const __amdgpu_buffer_rsrc_t h_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)H8, 0, (int)h_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)hs8, 0, (int)hs_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)w2x8, 0, (int)w_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t ws_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)wsc8, 0, E * UPE, kRawBuffer);
    const int n_units = E * UPE;

    uint32_t mw = 0, mw_next;
    int rowv = 0, is_next, go_next;
    auto load_batch = [&](int b) {
        const int bc = min(b, n_batches - 1);
        mw_next = mrow[bc];
        const int ec = min(32 * bc + c, E - 1);
        is_next = item_start[ec];
        go_next = grow[ec];
    };
    load_batch(0);
    // fetch state of the next unit in order; the fetches run FOUR units ahead of the MFMAs, so a
    // batch of 32 experts starts between two quads of the loop below, which keeps the quad's
    // body free of branches (with a branch inside, the compiler moved all MFMAs of a quad behind
    // its memory operations)
    int fe = 0;  // next unit to fetch
    int fbatch = 0;
    auto next_batch = [&]() {
        mw = (tok_ok && fbatch < n_batches) ? mw_next : 0u;
        rowv = is_next * rows_per_item + go_next;
        ++fbatch;
        load_batch(fbatch);
    };
    next_batch();
    // first: the unit opens an expert (its selection, rank and row are worked out); a second
    // unit reads the next 64 bytes of the same row
    uint32_t voff_expert = 0, srow_expert = 0;
    auto fetch = [&](bool first, u32x4 (&hb)[2], uint32_t& hsc) {
        if (first) {  // compile-time at every call
            const bool sel = (mw & 1u) != 0u;
            mw >>= 1;
            const uint64_t bal = __ballot(sel);
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            const uint32_t row = (uint32_t)__builtin_amdgcn_readlane(rowv, (fe / UPE) & 31) + rank;
            const uint32_t oob = sel ? 0u : 0x80000000u;
            voff_expert = (row * (64u * UPE) + 32u * (uint32_t)bh) | oob;
            srow_expert = row | oob;
        }
        const uint32_t voff = voff_expert + 64u * (uint32_t)(fe % UPE);
        hb[0] = __builtin_amdgcn_raw_buffer_load_b128(h_rsrc, voff, 0, 0);
        hb[1] = __builtin_amdgcn_raw_buffer_load_b128(h_rsrc, voff, 16, 0);
        hsc = __builtin_amdgcn_raw_buffer_load_b8(s_rsrc, srow_expert, 0, 0);
        ++fe;
    };
    // a tile is two planes of 1 KiB: plane p holds bytes 16p .. 16p+15 of every operand lane, so
    // a 16-byte access of a wavefront covers consecutive addresses (no bank conflicts)
    char* const wdst = img + (2 * bg + h) * 2048 + (32 * bh + c) * 16;
    char* const sdst = img + kD8Image + (2 * bg + h) * 32 + c;
    auto park = [&](int buf, const u32x4 (&hb)[2], uint32_t hsc) {
        *reinterpret_cast<u32x4*>(wdst + buf * kD8Buf) = hb[0];
        *reinterpret_cast<u32x4*>(wdst + buf * kD8Buf + 1024) = hb[1];
        // (both row halves write the same byte: no branch in the loop)
        *reinterpret_cast<uint8_t*>(sdst + buf * kD8Buf) = (uint8_t)hsc;
    };

    // ---- multiplying role
    uint32_t a_voff[kD8CT];
#pragma unroll
    for (int ct = 0; ct < kD8CT; ++ct) a_voff[ct] = (uint32_t)(((col_w / 32 + ct) * 64 + lane) * 32);
    const uint32_t w_expert_bytes = (uint32_t)(d / 32) * 2048;
    int we = 0;  // next unit whose weights are requested
    auto load_w = [&](i32x8 (&a)[kD8CT], int& sa) {
#pragma unroll
        for (int ct = 0; ct < kD8CT; ++ct) {
            // (past the last expert: its weights again, against all-zero tiles)
            const uint32_t so = (uint32_t)min(we, n_units - 1) * w_expert_bytes;
            const u32x4 v0 = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, a_voff[ct], so, 0);
            const u32x4 v1 = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, a_voff[ct] + 16u, so, 0);
            a[ct] = i32x8{(int)v0[0], (int)v0[1], (int)v0[2], (int)v0[3], (int)v1[0], (int)v1[1], (int)v1[2], (int)v1[3]};
        }
        sa = (int)__builtin_amdgcn_raw_buffer_load_b8(ws_rsrc, 0u, (uint32_t)min(we, n_units - 1), 0);
        ++we;
    };

    f32x16 acc[kD8Tiles][kD8CT];
    {
        bf16x8 bias[kD8CT][2];
#pragma unroll
        for (int ct = 0; ct < kD8CT; ++ct) bias[ct][0] = bias[ct][1] = zero8();
        if (b_down) {
#pragma unroll
            for (int ct = 0; ct < kD8CT; ++ct) {
                bias[ct][0] = load8(b_down + col_w + 32 * ct + 16 * h);
                bias[ct][1] = load8(b_down + col_w + 32 * ct + 16 * h + 8);
            }
        }
#pragma unroll
        for (int ct = 0; ct < kD8CT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i)
#pragma unroll
                for (int j = 0; j < kD8Tiles; ++j) acc[j][ct][i] = (float)bias[ct][i >> 3][i & 7];
    }
    const char* const rsrc_l = img + lane * 16;
    const char* const ssrc_l = img + kD8Image + c;
    auto read_b = [&](int buf, int j, i32x8& b, int& sb) {
        const i32x4 b0 = *reinterpret_cast<const i32x4*>(rsrc_l + buf * kD8Buf + j * 2048);
        const i32x4 b1 = *reinterpret_cast<const i32x4*>(rsrc_l + buf * kD8Buf + j * 2048 + 1024);
        b = i32x8{b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
        sb = *reinterpret_cast<const uint8_t*>(ssrc_l + buf * kD8Buf + j * 32);
    };

    // Rotation of four: the H pieces and the weights of expert e + 3 are requested while expert e
    // is multiplied; the tiles of e + 1 are parked in the other LDS buffer meanwhile.  Everything
    // that is not an MFMA sits between two MFMAs (the matrix pipe is busy 64 cycles per
    // instruction, which hides it), pinned there by scheduling barriers.
    u32x4 hb[4][2];
    uint32_t hs[4];
    i32x8 aw[4][kD8CT];
    int sa[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) fetch(i % UPE == 0, hb[i], hs[i]);
#pragma unroll
    for (int i = 0; i < 3; ++i) load_w(aw[i], sa[i]);
    park(0, hb[0], hs[0]);
    lds_barrier();
    // bb[e & 1]: the four B tiles of expert e, read from LDS while expert e - 1 is multiplied
    i32x8 bb[2][kD8Tiles];
    int sb[2][kD8Tiles];
#pragma unroll
    for (int j = 0; j < kD8Tiles; ++j) read_b(0, j, bb[0][j], sb[0][j]);
    const int n_quads = (n_units + 3) >> 2;
    constexpr int kQuadsPerBatch = 8 * UPE;  // 32 experts
    for (int qd = 0; qd < n_quads; ++qd) {
        // the last quad of a batch fetches the first four units of the next batch
        if ((qd & (kQuadsPerBatch - 1)) == kQuadsPerBatch - 1) next_batch();
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // unit u = 4 qd + i: LDS buffer / B set i & 1, register sets i
            const int buf = i & 1, n3 = (i + 3) & 3, n1 = (i + 1) & 3;
            __builtin_amdgcn_sched_barrier(0);
            acc[0][0] = mfma64(aw[i][0], bb[buf][0], acc[0][0], sa[i], sb[buf][0]);
            __builtin_amdgcn_sched_barrier(0);
            park(buf ^ 1, hb[n1], hs[n1]);   // expert e + 1 (the buffer was read one expert ago)
            __builtin_amdgcn_sched_barrier(0);
            acc[0][1] = mfma64(aw[i][1], bb[buf][0], acc[0][1], sa[i], sb[buf][0]);
            __builtin_amdgcn_sched_barrier(0);
            fetch(i % UPE == 0, hb[i], hs[i]);  // unit u + 4 (this set was parked one unit ago)
            __builtin_amdgcn_sched_barrier(0);
            acc[1][0] = mfma64(aw[i][0], bb[buf][1], acc[1][0], sa[i], sb[buf][1]);
            __builtin_amdgcn_sched_barrier(0);
            acc[1][1] = mfma64(aw[i][1], bb[buf][1], acc[1][1], sa[i], sb[buf][1]);
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();                   // the tiles of e + 1 are complete
            __builtin_amdgcn_sched_barrier(0);
            acc[2][0] = mfma64(aw[i][0], bb[buf][2], acc[2][0], sa[i], sb[buf][2]);
            __builtin_amdgcn_sched_barrier(0);
            read_b(buf ^ 1, 0, bb[buf ^ 1][0], sb[buf ^ 1][0]);
            read_b(buf ^ 1, 1, bb[buf ^ 1][1], sb[buf ^ 1][1]);
            __builtin_amdgcn_sched_barrier(0);
            acc[2][1] = mfma64(aw[i][1], bb[buf][2], acc[2][1], sa[i], sb[buf][2]);
            __builtin_amdgcn_sched_barrier(0);
            read_b(buf ^ 1, 2, bb[buf ^ 1][2], sb[buf ^ 1][2]);
            read_b(buf ^ 1, 3, bb[buf ^ 1][3], sb[buf ^ 1][3]);
            __builtin_amdgcn_sched_barrier(0);
            acc[3][0] = mfma64(aw[i][0], bb[buf][3], acc[3][0], sa[i], sb[buf][3]);
            __builtin_amdgcn_sched_barrier(0);
            acc[3][1] = mfma64(aw[i][1], bb[buf][3], acc[3][1], sa[i], sb[buf][3]);
            __builtin_amdgcn_sched_barrier(0);
            load_w(aw[n3], sa[n3]);          // expert e + 3 (its set was used one expert ago)
        }
    }

#pragma unroll
    for (int j = 0; j < kD8Tiles; ++j) {
        const int t = t_base + 32 * j + c;
        if (t < T) {
#pragma unroll
            for (int ct = 0; ct < kD8CT; ++ct) {
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

}  // namespace

void launch_pack_down_x8(const dmoe_layer& L, void* packed, hipStream_t s) {
    const PackedLayout P = packed_layout(L);
    char* pk = static_cast<char*>(packed);
    launch_kernel(pack_down_x8_kernel, 2048, 256, 0, s, (const uint8_t*)L.w_down,
                  (const float*)(pk + P.scales), (uint8_t*)(pk + P.w2x8), (uint8_t*)(pk + P.wsc8),
                  L.n_experts, L.expert_size, L.d_model, m_pad_of(L.expert_size) / 64);
}

// The kernel reaches the packed weights and H8 through 32-bit buffer offsets, and marks
// unselected tokens with offsets from 2^31 up.
bool down_x8_addressable(const dmoe_layer& L, int T) {
    const size_t mp = m_pad_of(L.expert_size);
    return (size_t)L.n_experts * (mp / 64) * (L.d_model / 32) * 2048 < (1ull << 32) &&
           h_fragments(L, T) * 16 * mp < (1ull << 31);
}

void launch_h_rows_to_e4m3(const dmoe_layer& L, const int32_t* item_start, const void* H,
                           uint8_t* H8, uint8_t* hs8, hipStream_t s) {
    LaunchTimer tm(kSlotQuantH, s);
    if (m_pad_of(L.expert_size) == 64)
        launch_kernel(h_rows_quantize_kernel<64, true>, 2048, 256, 0, s, (__bf16*)const_cast<void*>(H),
                      item_start, L.n_experts, up_rows_bf16(L), H8, hs8);
    else
        launch_kernel(h_rows_quantize_kernel<128, true>, 2048, 256, 0, s, (__bf16*)const_cast<void*>(H),
                      item_start, L.n_experts, up_rows_bf16(L), H8, hs8);
}

void launch_h_rows_quantize(const dmoe_layer& L, const int32_t* item_start, void* H, hipStream_t s) {
    LaunchTimer tm(kSlotQuantH, s);
    const int mp = m_pad_of(L.expert_size);
    if (mp == 32)
        launch_kernel(h_rows_quantize_kernel<32, false>, 2048, 256, 0, s, (__bf16*)H, item_start,
                      L.n_experts, up_rows_bf16(L), (uint8_t*)nullptr, (uint8_t*)nullptr);
    else if (mp == 64)
        launch_kernel(h_rows_quantize_kernel<64, false>, 2048, 256, 0, s, (__bf16*)H, item_start,
                      L.n_experts, up_rows_bf16(L), (uint8_t*)nullptr, (uint8_t*)nullptr);
    else
        launch_kernel(h_rows_quantize_kernel<128, false>, 2048, 256, 0, s, (__bf16*)H, item_start,
                      L.n_experts, up_rows_bf16(L), (uint8_t*)nullptr, (uint8_t*)nullptr);
}

void launch_down_x8(const dmoe_layer& L, int T, const int32_t* item_start, const int32_t* group_off,
                    const uint64_t* mask, const uint8_t* H8, const uint8_t* hs8, void* y,
                    hipStream_t s) {
    LaunchTimer tm(kSlotDown, s);
    const PackedLayout P = packed_layout(L);
    const char* pk = static_cast<const char*>(L.packed);
    const int E = L.n_experts, d = L.d_model;
    const size_t rows = h_fragments(L, T) * 16;
    const int upe = m_pad_of(L.expert_size) / 64;
    const size_t w_bytes = (size_t)E * upe * (d / 32) * 2048;
    const int NG = div_up(T, kGroup), NC = div_up(T, kD8Tokens), NS = d / (kD8CT * 128);
    auto* kernel = upe == 1 ? down_x8_kernel<1> : down_x8_kernel<2>;
    launch_kernel(kernel, round_up(NC, 8) * NS, 256, kD8Lds, s, (const uint8_t*)(pk + P.w2x8),
                  (const uint8_t*)(pk + P.wsc8), (const __bf16*)L.b_down, item_start, group_off,
                  reinterpret_cast<const uint32_t*>(mask), H8, hs8, (__bf16*)y, T, d, E, NG,
                  2 * div_up(E, 64), up_rows_bf16(L), (uint32_t)w_bytes,
                  (uint32_t)(rows * 64 * upe), (uint32_t)rows);
}

}  // namespace dmoe

// Router scores and dynamic-k gate for at most 16 tokens inside ONE workgroup of sixteen
// wavefronts (Sec. 3.3, Sec. 3.4 Eq. 4): device functions shared by the stand-alone gate kernels
// (select.hip) and by the small-token up-projection, whose workgroups each repeat this little
// computation instead of waiting for a kernel of its own (ffn_small.hip).
#pragma once

#include "dmoe_internal.h"
#include "mfma.h"

namespace dmoe {

// Second router product, s = |R2 hid + c2|, for all experts: wavefront w multiplies the expert
// tiles w, w + 16, ...; the fp32 scores go to sc[16][E] (LDS) and, if wanted, to M.scores.
// Every workgroup that runs this on the same inputs gets the same bits.
__device__ __forceinline__ void small_scores_to_lds(const SmallMod& M, int T, int dh, int E,
                                                    float* __restrict__ sc, bool to_global) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, q = lane >> 4, c = lane & 15;
    const int KS2 = dh / 32, NE = (E + 15) >> 4;
    const __bf16* hb = M.hid + (size_t)c * dh + 8 * q;
    for (int et = w; et < NE; et += 16) {
        const __bf16* af = M.r2f + (((size_t)et * KS2) * 64 + lane) * 8;
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int ks = 0; ks < KS2; ++ks)  // eight k-steps of loads go out together
            acc = mfma16(load8(af + (size_t)ks * 512), load8(hb + 32 * ks), acc);
        const int e0 = 16 * et + 4 * q;  // lane (q, c): experts e0 .. e0+3 of token c
        if (c < T && e0 < E) {
            const float4 out = router_scores4(acc, M.r_b2, e0, E);
            if (to_global) store_scores4(M.scores + (size_t)c * E, e0, E, out);
            store_scores4(sc + (size_t)c * E, e0, E, out);
        }
    }
}

// Maximum of token t's score row, by the wavefront that owns the token (lanes stride the experts).
__device__ __forceinline__ float small_row_max(const float* __restrict__ row, int E) {
    const int lane = threadIdx.x & 63;
    float mx = -INFINITY;
    for (int e = lane; e < E; e += 64) mx = fmaxf(mx, row[e]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    return mx;
}

// The comparison of Eq. 4, exact: the fp64 product of two fp32 numbers is exact.
__device__ __forceinline__ bool small_keeps(float s, float tau, float mx) {
    return tau == 0.0f || (double)s >= (double)tau * (double)mx;
}

// T <= 16, one workgroup of 16 wavefronts: wavefront t = token t with lanes striding the experts,
// so the score row is read coalesced, the maximum is a wavefront reduction and a ballot IS a mask
// word.  The transpose to per-expert token sets (colmask) and counts then goes through LDS
// (mw[16][W]).
__device__ __forceinline__ void select_small_body(const float* __restrict__ scores,
                                                  uint64_t* __restrict__ mw,
                                                  uint64_t* __restrict__ mask,
                                                  int32_t* __restrict__ k_per_token,
                                                  int32_t* __restrict__ group_cnt,
                                                  uint64_t* __restrict__ colmask, int T, int E,
                                                  int W, float tau) {
    const int lane = threadIdx.x & 63, t = threadIdx.x >> 6;
    if (t < T) {
        const float* row = scores + (size_t)t * E;
        const float mx = small_row_max(row, E);
        int kt = 0;
        for (int w = 0; w < W; ++w) {
            const int e = 64 * w + lane;
            const bool keep = e < E && small_keeps(row[min(e, E - 1)], tau, mx);
            const uint64_t word = __ballot(keep);
            kt += __popcll(word);
            if (lane == 0) {
                mw[t * W + w] = word;
                mask[(size_t)t * W + w] = word;
            }
        }
        if (lane == 0 && k_per_token) k_per_token[t] = kt;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 1024) {
        uint64_t col = 0;
        for (int tt = 0; tt < T; ++tt) col |= ((mw[tt * W + (e >> 6)] >> (e & 63)) & 1ull) << tt;
        group_cnt[e] = __popcll(col);
        if (colmask) colmask[e] = col;
    }
}

}  // namespace dmoe

// Dynamic-k gate and per-expert bucketing (Sec. 3.4 Eq. 4; the metadata of Appendix C built by
// dedicated kernels instead of a full argsort).
//
// Data flow:  scores -> [tau_mask | topk_mask, count_from_mask] -> mask bits + per-(group, expert) counts
//             -> [scan_groups] prefix over token groups per expert
//             -> [fill] prefix over experts (list offsets, up-projection work items) and the
//                ascending per-expert token lists, compact and work-item aligned.
// A group is 64 consecutive tokens handled by one wavefront with lane = token; the 64x64 bit
// transpose between "experts of a token" and "tokens of an expert" is done with ballots.
#include "dmoe_internal.h"
#include "mfma.h"
#include "small_gate.h"

namespace dmoe {

namespace {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        int n = __shfl_up(v, off, kWave);
        if (lane >= off) v += n;
    }
    return v;
}

// Per-group expert counts from the mask words: one wavefront per (group of 64 tokens, mask word),
// lane = token.  The ballot transpose gives, for every expert of the word, the 64-bit set of the
// group's tokens that keep it: its population count goes to group_cnt[g][e], the set itself to
// colmask[g][e] if wanted.
__global__ __launch_bounds__(256) void count_from_mask_kernel(const uint64_t* __restrict__ mask,
                                                              int32_t* __restrict__ group_cnt,
                                                              uint64_t* __restrict__ colmask,
                                                              int T, int E, int W) {
    const int lane = lane_id();
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int NG = (T + kGroup - 1) / kGroup;
    const int g = wave / W, w = wave - g * W;
    if (g >= NG) return;  // uniform per wavefront
    const int t = g * kGroup + lane;
    const uint64_t word = t < T ? mask[(size_t)t * W + w] : 0ull;
    uint64_t col = 0;  // lane b: which tokens of the group keep expert 64w + b
#pragma unroll 8
    for (int b = 0; b < 64; ++b) {
        const uint64_t bal = __ballot((word >> b) & 1ull);
        if (lane == b) col = bal;
    }
    const int e = 64 * w + lane;
    if (e < E) {
        group_cnt[(size_t)g * E + e] = __popcll(col);
        if (colmask) colmask[(size_t)g * E + e] = col;
    }
}

// Dynamic-k gate (Sec. 3.4 Eq. 4) with one wavefront per token and the lanes striding the
// experts: the score row is read coalesced and once (CH = ceil(E / 64) values per lane, all
// loads in flight together), the maximum is a wavefront reduction and a ballot IS a mask word.
// The per-group expert counts are then taken from the mask words by count_from_mask_kernel.
template <int CH>
__global__ __launch_bounds__(256) void tau_mask_kernel(const float* __restrict__ scores,
                                                       uint64_t* __restrict__ mask,
                                                       int32_t* __restrict__ k_per_token, int T,
                                                       int E, int W, float tau) {
    const int lane = lane_id();
    const int t = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    if (t >= T) return;  // uniform per wavefront
    const float* row = scores + (size_t)t * E;
    float v[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int e = 64 * c + lane;
        v[c] = e < E ? row[e] : -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < CH; ++c) mx = fmaxf(mx, v[c]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    const double thr = (double)tau * (double)mx;  // exact: at most 48 significant bits
    int kt = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int e = 64 * c + lane;
        const bool keep = e < E && (tau == 0.0f || (double)v[c] >= thr);
        const uint64_t word = __ballot(keep);
        kt += __popcll(word);
        if (lane == 0 && c < W) mask[(size_t)t * W + c] = word;
    }
    if (lane == 0 && k_per_token) k_per_token[t] = kt;
}

// Top-k gate (the conventional rule that Sec. 3.3 / 3.4 compare against): keep the k largest
// scores of each token, ties at the k-th value going to the lower expert index, so that exactly
// k are kept.  One wavefront per token with the lanes striding the experts (coalesced row read).
// The k-th largest value is found by a radix descent over the 32 bits of an order-preserving
// integer image of the scores (one ballot per 64 experts and bit); the experts equal to it are
// then admitted in index order until k are reached.  CH = ceil(E / 64) values per lane.
template <int CH>
__global__ __launch_bounds__(256) void topk_mask_kernel(const float* __restrict__ scores,
                                                        uint64_t* __restrict__ mask,
                                                        int32_t* __restrict__ k_per_token, int T,
                                                        int E, int W, int k) {
    const int lane = lane_id();
    const int t = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    if (t >= T) return;  // uniform per wavefront
    const float* row = scores + (size_t)t * E;
    uint32_t key[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int e = 64 * c + lane;
        // -0 and +0 compare equal, as they do as numbers; then flip so that unsigned order =
        // numeric order (sign bit set: all bits flipped, else only the sign bit)
        const uint32_t b = e < E ? __float_as_uint(row[e] + 0.0f) : 0x80000000u;  // padding: -0 -> below
        key[c] = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
        if (e >= E) key[c] = 0u;  // below every real score
    }
    // largest x with #{key >= x} >= k
    uint32_t x = 0u;
    if (k > 0) {
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t cand = x | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int c = 0; c < CH; ++c) cnt += __popcll(__ballot(key[c] >= cand));
            if (cnt >= k) x = cand;  // uniform
        }
    }
    int above = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) above += __popcll(__ballot(key[c] > x));
    int need = k - above;  // how many of the experts equal to x are admitted, lowest index first
    int kt = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int e = 64 * c + lane;
        const bool eq = key[c] == x && e < E;
        const uint64_t eqb = __ballot(eq);
        const bool take = eq && (int)__popcll(eqb & ((1ull << lane) - 1ull)) < need;
        const uint64_t word = __ballot(k > 0 && ((key[c] > x && e < E) || take));
        need -= min(need, (int)__popcll(eqb));
        if (c < W) kt += __popcll(word);
        if (lane == 0 && c < W) mask[(size_t)t * W + c] = word;
    }
    if (lane == 0 && k_per_token) k_per_token[t] = kt;
}

__global__ __launch_bounds__(1024) void select_small_kernel(const float* __restrict__ scores,
                                                            uint64_t* __restrict__ mask,
                                                            int32_t* __restrict__ k_per_token,
                                                            int32_t* __restrict__ group_cnt,
                                                            uint64_t* __restrict__ colmask, int T,
                                                            int E, int W, float tau) {
    extern __shared__ uint64_t mw[];  // [16][W]
    select_small_body(scores, mw, mask, k_per_token, group_cnt, colmask, T, E, W, tau);
}

// Second router product and the gate in one workgroup per layer (T <= 16, E <= 1024): the scores
// go to global memory and to LDS, and after one barrier the gate runs on the LDS copy.  One
// launch less than scores + gate, which is what counts at this size.
__global__ __launch_bounds__(1024) void router_scores_select_small_kernel(const SmallGroup G, int T,
                                                                          int dh, int E, int W) {
    extern __shared__ uint64_t mw[];  // [16][W] mask words, then [16][E] fp32 scores
    const SmallMod& M = G.m[blockIdx.z];
    float* sc = reinterpret_cast<float*>(mw + 16 * W);
    small_scores_to_lds(M, T, dh, E, sc, true);
    __syncthreads();
    select_small_body(sc, mw, M.mask, nullptr, M.group_cnt, M.colmask, T, E, W, M.tau);
}

// the same gate for every layer of a group (blockIdx.z = layer), each with its own tau
__global__ __launch_bounds__(1024) void select_small_group_kernel(const SmallGroup G, int T, int E,
                                                                  int W) {
    extern __shared__ uint64_t mw[];  // [16][W]
    const SmallMod& M = G.m[blockIdx.z];
    select_small_body(M.scores, mw, M.mask, nullptr, M.group_cnt, M.colmask, T, E, W, M.tau);
}

__global__ void zero_u64_kernel(uint64_t* p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0ull;
}

// Caller-supplied lists -> mask bits.  One thread per list position; entries outside [0, T)
// are dropped, duplicates collapse in the OR.
__global__ void lists_to_mask_kernel(const int32_t* __restrict__ offsets,
                                     const int32_t* __restrict__ lists, int T, int E, int W,
                                     unsigned long long* __restrict__ mask) {
    const long long cap = (long long)T * E;
    long long first = offsets[0], last = offsets[E];
    if (first < 0) first = 0;
    if (last > cap) last = cap;
    long long p = first + (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (; p < last; p += stride) {
        // expert of position p: the last e with offsets[e] <= p
        int lo = 0, hi = E;  // answer in [lo, hi)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((long long)offsets[mid] <= p) lo = mid; else hi = mid;
        }
        if (p >= (long long)offsets[lo + 1]) continue;  // non-monotone offsets: drop
        const int t = lists[p];
        if ((unsigned)t < (unsigned)T)
            atomicOr(&mask[(size_t)t * W + (lo >> 6)], 1ull << (lo & 63));
    }
}

// One wavefront per expert: exclusive prefix sum of group_cnt[.][e] over the groups, in place;
// row NG receives the total.  With sub != nullptr the counts of group g are read as the sum of
// the rows split * g .. split * g + split - 1 of sub (n_sub rows in all).
__global__ __launch_bounds__(256) void scan_groups_kernel(int32_t* __restrict__ group_cnt, int NG,
                                                          int E, const int32_t* __restrict__ sub,
                                                          int split, int n_sub) {
    const int lane = lane_id();
    const int e = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    if (e >= E) return;
    // eight chunks of 64 groups per pass with all their loads in flight together (one memory round
    // trip per 512 groups instead of one per 64)
    int carry = 0;
    for (int base = 0; base < NG; base += 8 * kWave) {
        int v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int g = base + k * kWave + lane;
            if (sub) {
                v[k] = 0;
                for (int j = 0; j < split; ++j)
                    if (g < NG && split * g + j < n_sub) v[k] += sub[(size_t)(split * g + j) * E + e];
            } else {
                v[k] = g < NG ? group_cnt[(size_t)g * E + e] : 0;
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int g = base + k * kWave + lane;
            const int incl = wave_inclusive_scan(v[k]);
            if (g < NG) group_cnt[(size_t)g * E + e] = carry + incl - v[k];
            carry += __shfl(incl, kWave - 1, kWave);
        }
    }
    if (lane == 0) group_cnt[(size_t)NG * E + e] = carry;
}

// Prefix sums over the experts plus the list fill, one launch.
//
// Every workgroup first redoes the (tiny) scan over the per-expert totals in LDS:
//   s_off[e]  = start of expert e in the compact lists (offsets),
//   s_item[e] = first up-projection work item of expert e when an item covers rows_per_item list
//               rows; s_item[E] = number of items.
// Workgroup 0 also publishes counts / offsets / item_start and pads the aligned list.
// Then one wavefront per group of 64 tokens (lane = token) turns mask words into list entries:
// for every expert, the lanes whose token keeps it write their token id at
//   lists[offsets[e] + group_off[g][e] + rank]                 compact, ascending (caller-visible)
//   alist[item_start[e] * rows_per_item + group_off[g][e] + rank]   aligned copy for the kernels
// where rank counts the group's keepers below the lane.  In the aligned copy every expert starts
// on a work-item boundary -- the same indexing as the rows of H -- and the slack behind its last
// token holds -1.
__global__ __launch_bounds__(256) void fill_lists_kernel(
    const uint64_t* __restrict__ mask, int T, int E, int W, const int32_t* __restrict__ group_off,
    int rows_per_item, int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
    int32_t* __restrict__ item_start, int32_t* __restrict__ lists, int32_t* __restrict__ alist,
    int GW, int NW, int32_t* __restrict__ witem, int32_t* __restrict__ wfirst) {
    extern __shared__ int32_t sm[];
    int32_t* s_off = sm;                 // [E + 1]
    int32_t* s_item = sm + (E + 1);      // [E + 1]
    __shared__ int s_part[2][4];
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int NG = (T + kGroup - 1) / kGroup;
    const int32_t* totals = group_off + (size_t)NG * E;

    int carry = 0, icarry = 0;
    for (int base = 0; base < E; base += 256) {
        const int e = base + tid;
        const int cnt = e < E ? totals[e] : 0;
        const int items = (cnt + rows_per_item - 1) / rows_per_item;
        const int incl = wave_inclusive_scan(cnt), iincl = wave_inclusive_scan(items);
        if (lane == kWave - 1) {
            s_part[0][wave] = incl;
            s_part[1][wave] = iincl;
        }
        __syncthreads();
        int before = carry, ibefore = icarry, all = 0, iall = 0;
        for (int w2 = 0; w2 < 4; ++w2) {
            if (w2 < wave) {
                before += s_part[0][w2];
                ibefore += s_part[1][w2];
            }
            all += s_part[0][w2];
            iall += s_part[1][w2];
        }
        if (e < E) {
            s_off[e] = before + incl - cnt;
            s_item[e] = ibefore + iincl - items;
        }
        carry += all;
        icarry += iall;
        __syncthreads();
    }
    if (tid == 0) {
        s_off[E] = carry;
        s_item[E] = icarry;
    }
    __syncthreads();

    // gridDim.y workgroups share the mask words of one group; those with y = 0 also do the
    // per-launch work
    const bool first_y = blockIdx.y == 0;
    if (blockIdx.x == 0 && first_y) {
        for (int e = tid; e <= E; e += 256) {
            offsets[e] = s_off[e];
            if (item_start) item_start[e] = s_item[e];
            if (e < E && counts) counts[e] = totals[e];
        }
    }
    // Window table for the up-projection (block w lays out window w = GW consecutive groups):
    // the work items of expert e that window w works on are wfirst[w][e] .. + n (those whose
    // rows mostly belong to tokens of the window); witem[w][e] is the exclusive prefix of n over
    // the experts.
    if (witem && (int)blockIdx.x < NW && first_y) {
        const int wdx = blockIdx.x;
        const int32_t* r_lo = group_off + (size_t)(wdx * GW) * E;
        const int32_t* r_hi = group_off + (size_t)min(wdx * GW + GW, NG) * E;
        int wcarry = 0;
        for (int base = 0; base < E; base += 256) {
            const int e = base + tid;
            int n = 0, first = 0;
            if (e < E) {
                // the expert's items are dealt to the windows in proportion to its rows there
                // (cutting at ceil(row / rows_per_item) would hand every expert's first,
                // rounded-up item to window 0 and overload its XCD)
                // (in double: exact far beyond any real size, monotone in the row, and identical for
                // the shared boundary of two neighbouring windows -- a 64-bit integer division
                // costs hundreds of instructions)
                const int cnt = totals[e];
                const int items = (cnt + rows_per_item - 1) / rows_per_item;
                const double scale = cnt ? (double)items / (double)cnt : 0.0;
                const int k0 = min(items, (int)((double)r_lo[e] * scale + 0.5));
                const int k1 = r_hi[e] >= cnt ? items : min(items, (int)((double)r_hi[e] * scale + 0.5));
                n = k1 - k0;
                first = s_item[e] + k0;
            }
            const int incl = wave_inclusive_scan(n);
            __syncthreads();  // s_part from the previous pass has been read
            if (lane == kWave - 1) s_part[0][wave] = incl;
            __syncthreads();
            int before = wcarry, all = 0;
            for (int w2 = 0; w2 < 4; ++w2) {
                if (w2 < wave) before += s_part[0][w2];
                all += s_part[0][w2];
            }
            if (e < E) {
                witem[(size_t)wdx * (E + 1) + e] = before + incl - n;
                wfirst[(size_t)wdx * E + e] = first;
            }
            wcarry += all;
        }
        if (tid == 0) witem[(size_t)wdx * (E + 1) + E] = wcarry;
    }
    if (alist && first_y) {  // -1 behind each expert's last token, up to its next work-item boundary
        for (int i = blockIdx.x * 256 + tid; i < E * rows_per_item; i += gridDim.x * 256) {
            const int e = i / rows_per_item, j = i % rows_per_item;
            const int p = s_item[e] * rows_per_item + totals[e] + j;
            if (p < s_item[e + 1] * rows_per_item) alist[p] = -1;
        }
    }

    // one workgroup per group of 64 tokens (lane = token); wavefront w takes the experts
    // 64*word + 16w .. +15 of every mask word
    const int g = blockIdx.x;
    if (g >= NG || (!lists && !alist)) return;
    const int t = g * kGroup + lane;
    const bool valid = t < T;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int w = blockIdx.y; w < W; w += gridDim.y) {
        const uint64_t word = valid ? mask[(size_t)t * W + w] : 0ull;
        // lane b keeps the three bases of expert 64w + b; b is uniform in the loop below, so each
        // read of them is a broadcast through the scalar unit
        const int e_l = 64 * w + lane;
        const int goff_l = e_l < E ? group_off[(size_t)g * E + e_l] : 0;
        const int cbase_l = e_l < E ? s_off[e_l] + goff_l : 0;
        const int abase_l = e_l < E ? s_item[e_l] * rows_per_item + goff_l : 0;
        const int nb = min(64, E - 64 * w);
#pragma unroll
        for (int bi = 0; bi < 16; ++bi) {
            const int b = 16 * wave + bi;
            const uint64_t bal = __ballot(((word >> b) & 1ull) != 0 && b < nb);
            if (bal != 0ull) {  // uniform
                const int cbase = __builtin_amdgcn_readlane(cbase_l, b);
                const int abase = __builtin_amdgcn_readlane(abase_l, b);
                if ((word >> b) & 1ull) {
                    const int rank = __popcll(bal & below);
                    if (lists) lists[cbase + rank] = t;
                    if (alist) alist[abase + rank] = t;
                }
            }
        }
    }
}

}  // namespace

void launch_mask_from_scores(const float* scores, int T, int E, float tau, uint64_t* mask,
                             int32_t* k_per_token, int32_t* group_off, uint64_t* colmask,
                             hipStream_t s) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    LaunchTimer tm(kSlotMask, s);
    if (T <= 16) {
        launch_kernel(select_small_kernel, 1, 1024, sizeof(uint64_t) * 16 * W, s, 
            scores, mask, k_per_token, group_off, colmask, T, E, W, tau);
        return;
    }
    const int grid = div_up(T, 4);
    if (W <= 1) launch_kernel(tau_mask_kernel<1>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    else if (W <= 2) launch_kernel(tau_mask_kernel<2>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    else if (W <= 4) launch_kernel(tau_mask_kernel<4>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    else if (W <= 8) launch_kernel(tau_mask_kernel<8>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    else if (W <= 16) launch_kernel(tau_mask_kernel<16>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    else if (W <= 32) launch_kernel(tau_mask_kernel<32>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    else launch_kernel(tau_mask_kernel<64>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, tau);
    launch_kernel(count_from_mask_kernel, div_up(NG * W, 4), 256, 0, s, mask, group_off, colmask, T, E, W);
}

void launch_select_small_group(const dmoe_layer& L, const SmallGroup& G, int n_layers, int T,
                               hipStream_t s) {
    const int E = L.n_experts, W = div_up(E, 64);
    LaunchTimer tm(kSlotMask, s);
    launch_kernel(select_small_group_kernel, dim3(1, 1, n_layers), 1024, sizeof(uint64_t) * 16 * W, s, G, T, E, W);
}

void launch_router_select_small(const dmoe_layer& L, const SmallGroup& G, int n_layers,
                                const void* x, int T, hipStream_t s) {
    // first product: the many-workgroup hidden kernel; second product + gate: one workgroup
    const int E = L.n_experts, W = div_up(E, 64);
    launch_router_small_hidden(L, G, n_layers, x, T, s);
    LaunchTimer tm(kSlotMask, s);
    const size_t lds = sizeof(uint64_t) * 16 * W + sizeof(float) * 16 * (size_t)E;
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&router_scores_select_small_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    });
    launch_kernel(router_scores_select_small_kernel, dim3(1, 1, n_layers), 1024, lds, s, G, T, L.router_hidden, E, W);
}

void launch_mask_from_lists(const int32_t* offsets, const int32_t* lists, int T, int E,
                            uint64_t* mask, int32_t* group_off, uint64_t* colmask, hipStream_t s) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    {
        LaunchTimer tm(kSlotListsToMask, s);
        const size_t n = (size_t)T * W;
        launch_kernel(zero_u64_kernel, (int)std::min<size_t>(1024, (n + 255) / 256), 256, 0, s, mask, n);
        launch_kernel(lists_to_mask_kernel, 1024, 256, 0, s, offsets, lists, T, E, W,
                                                  reinterpret_cast<unsigned long long*>(mask));
    }
    LaunchTimer tm(kSlotMask, s);
    launch_kernel(count_from_mask_kernel, div_up(NG * W, 4), 256, 0, s, mask, group_off, colmask, T, E, W);
}

void launch_mask_topk(const float* scores, int T, int E, int k, uint64_t* mask,
                      int32_t* k_per_token, int32_t* group_off, uint64_t* colmask, hipStream_t s) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    LaunchTimer tm(kSlotMask, s);
    const int grid = div_up(T, 4);
    if (W <= 1) launch_kernel(topk_mask_kernel<1>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    else if (W <= 2) launch_kernel(topk_mask_kernel<2>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    else if (W <= 4) launch_kernel(topk_mask_kernel<4>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    else if (W <= 8) launch_kernel(topk_mask_kernel<8>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    else if (W <= 16) launch_kernel(topk_mask_kernel<16>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    else if (W <= 32) launch_kernel(topk_mask_kernel<32>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    else launch_kernel(topk_mask_kernel<64>, grid, 256, 0, s, scores, mask, k_per_token, T, E, W, k);
    // counts per (group, expert) and, if wanted, the per-expert token sets
    launch_kernel(count_from_mask_kernel, div_up(NG * W, 4), 256, 0, s, mask, group_off, colmask, T, E, W);
}

void launch_scan_and_fill(const uint64_t* mask, int T, int E, int32_t* group_off, int32_t* counts,
                          int32_t* offsets, int32_t* item_start, int rows_per_item,
                          int32_t* token_lists, int32_t* aligned_lists, int window_groups,
                          int32_t* witem, int32_t* wfirst, hipStream_t s, const int32_t* sub_cnt,
                          int split) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    const int NW = witem ? div_up(NG, window_groups) : 0;
    {
        LaunchTimer tm(kSlotScanGroups, s);
        launch_kernel(scan_groups_kernel, div_up(E, 4), 256, 0, s, group_off, NG, E, sub_cnt, split,
                                                        div_up(T, kGroup / split));
    }
    LaunchTimer tm(kSlotFill, s);
    const size_t lds = sizeof(int32_t) * 2 * ((size_t)E + 1);
    static std::once_flag attr_once;  // kernel attributes: once per process, thread-safe
    std::call_once(attr_once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&fill_lists_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    });
    // with few token groups and many experts the mask words of a group are split over several
    // workgroups (each repeats the prefix sums over the experts)
    const int ny = std::max(1, std::min(W, div_up(2048, std::max(1, NG))));
    launch_kernel(fill_lists_kernel, dim3(std::max(1, NG), ny), 256, lds, s, 
        mask, T, E, W, group_off, rows_per_item, counts, offsets, item_start, token_lists,
        aligned_lists, window_groups, NW, witem, wfirst);
}

}  // namespace dmoe

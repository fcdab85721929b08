// Dynamic-k gate and per-expert bucketing (Sec. 3.4 Eq. 4; the metadata of Appendix C built by
// dedicated kernels instead of a full argsort).
//
// Data flow:  scores -> [mask_count] -> mask bits + per-(group, expert) counts
//             -> [scan_groups] prefix over token groups per expert
//             -> [scan_experts] prefix over experts (list offsets, up-projection work items)
//             -> [fill] ascending per-expert token lists.
// A group is 64 consecutive tokens handled by one wavefront with lane = token; the 64x64 bit
// transpose between "experts of a token" and "tokens of an expert" is done with ballots.
#include "dmoe_internal.h"

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

// One wavefront per group of 64 tokens, lane = token.
// FROM_SCORES: evaluate Eq. 4 on the token's score row and write its mask words;
// otherwise read the mask words.  Either way, count, for every expert, the tokens of the group
// that keep it (ballot transpose) into group_cnt[g][e].
template <bool FROM_SCORES>
__global__ __launch_bounds__(256) void mask_count_kernel(const float* __restrict__ scores,
                                                         uint64_t* __restrict__ mask,
                                                         int32_t* __restrict__ k_per_token,
                                                         int32_t* __restrict__ group_cnt, int T,
                                                         int E, int W, float tau) {
    const int lane = lane_id();
    const int g = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int NG = (T + kGroup - 1) / kGroup;
    if (g >= NG) return;  // uniform per wavefront
    const int t = g * kGroup + lane;
    const bool valid = t < T;
    const float* row = scores + (size_t)(valid ? t : 0) * E;

    double thr = 0.0;
    if (FROM_SCORES) {
        float mx = -INFINITY;
        if (valid) {
            if ((E & 3) == 0) {
                const float4* r4 = reinterpret_cast<const float4*>(row);
                for (int i = 0; i < E / 4; ++i) {
                    float4 v = r4[i];
                    mx = fmaxf(mx, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
                }
            } else {
                for (int i = 0; i < E; ++i) mx = fmaxf(mx, row[i]);
            }
        }
        // exact: the fp64 product of two fp32 values carries at most 48 significant bits
        thr = (double)tau * (double)mx;
    }

    int kt = 0;
    for (int w = 0; w < W; ++w) {
        uint64_t word = 0;
        const int nb = min(64, E - 64 * w);
        if (FROM_SCORES) {
            if (valid) {
                if (tau == 0.0f) {
                    word = nb == 64 ? ~0ull : ((1ull << nb) - 1ull);
                } else {
                    for (int b = 0; b < nb; ++b) {
                        const double s = (double)row[64 * w + b];
                        word |= (uint64_t)(s >= thr) << b;
                    }
                }
                mask[(size_t)t * W + w] = word;
            }
        } else {
            if (valid) word = mask[(size_t)t * W + w];
        }
        kt += __popcll(word);
        int cnt = 0;
#pragma unroll 8
        for (int b = 0; b < 64; ++b) {
            const uint64_t bal = __ballot((word >> b) & 1ull);
            if (lane == b) cnt = __popcll(bal);
        }
        const int e = 64 * w + lane;
        if (e < E) group_cnt[(size_t)g * E + e] = cnt;
    }
    if (valid && k_per_token) k_per_token[t] = kt;
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
// row NG receives the total.
__global__ __launch_bounds__(256) void scan_groups_kernel(int32_t* __restrict__ group_cnt, int NG,
                                                          int E) {
    const int lane = lane_id();
    const int e = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    if (e >= E) return;
    int carry = 0;
    for (int base = 0; base < NG; base += kWave) {
        const int g = base + lane;
        const int v = g < NG ? group_cnt[(size_t)g * E + e] : 0;
        const int incl = wave_inclusive_scan(v);
        if (g < NG) group_cnt[(size_t)g * E + e] = carry + incl - v;
        carry += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) group_cnt[(size_t)NG * E + e] = carry;
}

// One wavefront: prefix sums over the experts.  offsets[e] = list start, item_start[e] = first
// up-projection work item of expert e when every item covers rows_per_item list rows;
// item_start[E] = number of items, item_start[E+1] = the largest per-expert item count.
__global__ __launch_bounds__(64) void scan_experts_kernel(const int32_t* __restrict__ totals, int E,
                                                          int rows_per_item,
                                                          int32_t* __restrict__ counts,
                                                          int32_t* __restrict__ offsets,
                                                          int32_t* __restrict__ item_start) {
    const int lane = lane_id();
    int carry = 0, icarry = 0, imax = 0;
    for (int base = 0; base < E; base += kWave) {
        const int e = base + lane;
        const int c = e < E ? totals[e] : 0;
        const int items = (c + rows_per_item - 1) / rows_per_item;
        imax = max(imax, items);
        const int incl = wave_inclusive_scan(c);
        const int iincl = wave_inclusive_scan(items);
        if (e < E) {
            if (counts) counts[e] = c;
            offsets[e] = carry + incl - c;
            if (item_start) item_start[e] = icarry + iincl - items;
        }
        carry += __shfl(incl, kWave - 1, kWave);
        icarry += __shfl(iincl, kWave - 1, kWave);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) imax = max(imax, __shfl_xor(imax, off, kWave));
    if (lane == 0) {
        offsets[E] = carry;
        if (item_start) {
            item_start[E] = icarry;
            item_start[E + 1] = imax;  // the largest number of work items of any expert
        }
    }
}

// One wavefront per group, lane = token: for every expert, the lanes whose token keeps it write
// their token id at  offsets[e] + group_off[g][e] + (rank among the group's keepers).
__global__ __launch_bounds__(256) void fill_lists_kernel(const uint64_t* __restrict__ mask, int T,
                                                         int E, int W,
                                                         const int32_t* __restrict__ group_off,
                                                         const int32_t* __restrict__ offsets,
                                                         int32_t* __restrict__ lists,
                                                         int32_t* __restrict__ lists_copy) {
    const int lane = lane_id();
    const int g = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int NG = (T + kGroup - 1) / kGroup;
    if (g >= NG) return;
    const int t = g * kGroup + lane;
    const bool valid = t < T;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int w = 0; w < W; ++w) {
        const uint64_t word = valid ? mask[(size_t)t * W + w] : 0ull;
        const int nb = min(64, E - 64 * w);
        for (int b = 0; b < nb; ++b) {
            const uint64_t bal = __ballot((word >> b) & 1ull);
            if (bal == 0ull) continue;  // uniform
            const int e = 64 * w + b;
            const int base = offsets[e] + group_off[(size_t)g * E + e];
            if ((word >> b) & 1ull) {
                const int p = base + __popcll(bal & below);
                lists[p] = t;
                if (lists_copy) lists_copy[p] = t;
            }
        }
    }
}

}  // namespace

void launch_mask_from_scores(const float* scores, int T, int E, float tau, uint64_t* mask,
                             int32_t* k_per_token, int32_t* group_off, hipStream_t s) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    LaunchTimer tm(kSlotMask, s);
    mask_count_kernel<true><<<div_up(NG, 4), 256, 0, s>>>(scores, mask, k_per_token, group_off, T,
                                                          E, W, tau);
}

void launch_mask_from_lists(const int32_t* offsets, const int32_t* lists, int T, int E,
                            uint64_t* mask, int32_t* group_off, hipStream_t s) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    {
        LaunchTimer tm(kSlotListsToMask, s);
        const size_t n = (size_t)T * W;
        zero_u64_kernel<<<(int)std::min<size_t>(1024, (n + 255) / 256), 256, 0, s>>>(mask, n);
        lists_to_mask_kernel<<<1024, 256, 0, s>>>(offsets, lists, T, E, W,
                                                  reinterpret_cast<unsigned long long*>(mask));
    }
    LaunchTimer tm(kSlotMask, s);
    mask_count_kernel<false><<<div_up(NG, 4), 256, 0, s>>>(nullptr, mask, nullptr, group_off, T, E,
                                                           W, 0.0f);
}

void launch_scan_and_fill(const uint64_t* mask, int T, int E, int32_t* group_off, int32_t* counts,
                          int32_t* offsets, int32_t* item_start, int rows_per_item,
                          int32_t* token_lists, int32_t* token_lists_copy, hipStream_t s) {
    const int W = div_up(E, 64), NG = div_up(T, kGroup);
    {
        LaunchTimer tm(kSlotScanGroups, s);
        scan_groups_kernel<<<div_up(E, 4), 256, 0, s>>>(group_off, NG, E);
    }
    {
        LaunchTimer tm(kSlotScanExperts, s);
        scan_experts_kernel<<<1, 64, 0, s>>>(group_off + (size_t)NG * E, E, rows_per_item, counts,
                                             offsets, item_start);
    }
    if (token_lists) {
        LaunchTimer tm(kSlotFill, s);
        fill_lists_kernel<<<div_up(NG, 4), 256, 0, s>>>(mask, T, E, W, group_off, offsets,
                                                        token_lists, token_lists_copy);
    }
}

}  // namespace dmoe

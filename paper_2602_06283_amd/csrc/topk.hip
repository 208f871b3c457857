// Alg. 3, TopK step: exact selection of the k largest scores per (sequence, KV head) by a
// most-significant-digit radix select on the fp32 bit patterns, spread over many workgroups.
//
//   topk_hist_kernel    histogram of the leading 11-bit digit of every valid score (the fused
//                       decode step gets it from the scoring pass instead).
//   topk_hist2_kernel   finds the threshold digit, then histograms the next 11 bits over the
//                       scores in that digit.
//   topk_filter_kernel  finds the second threshold digit, then sweeps: scores above the
//                       two-digit threshold are selected, scores equal to it are candidates
//                       (one bin of a 2^22-bin histogram: a handful unless many scores tie).
//   topk_resolve_kernel one workgroup per (sequence, head): ranks the candidates on the
//                       remaining score bits and then on the token position (smaller position
//                       wins a tie), and writes the selection in ascending position order
//                       through an LDS bitmap.  Leaves histograms and counters at zero.
// When the scoring pass has left an adaptive histogram (bins sized from the bucket-probability
// tables, a few dozen scores in the threshold bin), topk_filter_kernel<true> finds the
// threshold bin itself and sweeps with it, and the two histogram kernels are skipped.
// Stages talk through global memory across kernel boundaries only: no workgroup waits on
// another and no fence is needed.  LDS arrays that a thread walks in runs of PER consecutive
// words carry one pad word per run, which makes those walks free of bank conflicts.
#include "socket_internal.h"

namespace sk {

#ifdef SK_DEBUG_CLOCKS
__device__ long long sk_dbg[64];
#define SK_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x == 0) sk_dbg[i] = wall_clock64(); } while (0)
#else
#define SK_STAMP(i) ((void)0)
#endif

constexpr int kTopkThreads = 512;
constexpr int kRefineBins = 4096;                // bins of a candidate-refinement digit
constexpr int kBitmapWords = 8192;               // 32 KB of LDS
constexpr int kBitmapTokens = kBitmapWords * 32; // tokens one LDS bitmap pass covers
constexpr int kLowBits = 32 - kHistBits;         // score bits below the leading digit
constexpr int kDigit2Shift = kLowBits - kHistBits;   // second digit: the next kHistBits score bits
static_assert(kDigit2Shift >= 0 && kDigit2Shift <= 12, "the low score bits fit one refinement digit");
constexpr int kPer = 8;                          // scores per thread in a sweep
constexpr int kSlice = kTopkThreads * kPer;      // scores per workgroup
constexpr int kRankMax = 2 * kTopkThreads;       // candidates the all-pairs ranking handles
// threshold record: [0] k_eff, [1] first digit, [2] scores above it, [3] scores in it,
//                   [4] second digit, [5] scores selected outright, [6] candidates,
//                   [kThrBinLo], [kThrBinInv] adaptive binning written by the scoring pass

struct TopkArgs {
    const float *scores;
    const int32_t *seq_len;
    const int32_t *k;
    int32_t *idx;
    int32_t *n_selected;
    uint32_t *hist;       // first-digit histograms [B*Hkv][kHistBins]
    uint32_t *hist2;      // second-digit histograms of the threshold bin
    uint32_t *thr;        // threshold records [B*Hkv][kThrStride]
    uint32_t *counters;
    uint32_t *cand_key;
    int32_t *cand_idx;
    int32_t *staged;
    int Hkv, max_n, max_k;
    int adaptive;         // candidates share an adaptive bin, not the two leading digits
};

// Order-preserving map from fp32 to uint32 (larger float -> larger key).
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ bool selectable(float f) { return f > -__builtin_inff(); }  // false for NaN
__device__ __forceinline__ uint32_t digit2(uint32_t key) { return (key >> kDigit2Shift) & (kHistBins - 1); }

// word w of an array walked in runs of PER words, one pad word per run
template <int PER> __device__ __forceinline__ int padded(int w) { return w + w / PER; }
template <int N, int PER> constexpr int padded_size() { return N + N / PER; }

// Exclusive prefix sum over the 512 threads of a block; *total gets the block sum.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *total, uint32_t *tmp) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t x = wave_incl_scan(v);
    if (lane == 63) tmp[wave] = x;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kTopkThreads / 64; ++w) {
        uint32_t t = tmp[w];
        if (w < wave) base += t;
        sum += t;
    }
    __syncthreads();
    *total = sum;
    return base + x - v;
}

// Largest bin tb of the NBINS-bin padded LDS histogram h with count(bins >= tb) >= target.
// res[0] = tb, res[1] = count(bins > tb), res[2] = h[tb], res[3] = sum(h).
// A target outside [1, sum(h)] leaves res[0..2] untouched.
template <int NBINS>
__device__ __forceinline__ void find_threshold(const uint32_t *h, uint32_t target, uint32_t *res,
                                               uint32_t *tmp) {
    const int t = threadIdx.x;
    constexpr int PER = NBINS / kTopkThreads;       // bins per thread, highest bins first
    const int top = NBINS - 1 - t * PER;
    uint32_t c[PER];
    uint32_t part = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        c[i] = h[padded<PER>(top - i)];
        part += c[i];
    }
    uint32_t total;
    uint32_t above = block_excl_scan(part, &total, tmp);
    if (t == 0) res[3] = total;
    if (above < target && target <= above + part) {
        uint32_t cum = above;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (cum < target && cum + c[i] >= target) {
                res[0] = (uint32_t)(top - i);
                res[1] = cum;
                res[2] = c[i];
            }
            cum += c[i];
        }
    }
    __syncthreads();
}

// this thread's kPer scores of the slice starting at key0 (in bounds for any sequence length)
__device__ __forceinline__ void load_scores(const float *s, int i, int max_n, float *e) {
#pragma unroll
    for (int v = 0; v < kPer / 4; ++v) {
        float4 q = i + 4 * v < max_n ? *(const float4 *)(s + i + 4 * v) : make_float4(0, 0, 0, 0);
        e[4 * v] = q.x; e[4 * v + 1] = q.y; e[4 * v + 2] = q.z; e[4 * v + 3] = q.w;
    }
}

__device__ __forceinline__ int clamp_len(int v, int hi) { return v < 0 ? 0 : (v > hi ? hi : v); }

__global__ __launch_bounds__(kTopkThreads) void topk_hist_kernel(TopkArgs a) {
    __shared__ uint32_t h[kHistBins];
    const int tid = threadIdx.x;
    const int bh = blockIdx.y, b = bh / a.Hkv;
    const int key0 = blockIdx.x * kSlice;
    const int i = key0 + tid * kPer;
    float e[kPer];
    load_scores(a.scores + (int64_t)bh * a.max_n, i, a.max_n, e);
    const int key1 = min(key0 + kSlice, clamp_len(a.seq_len[b], a.max_n));
    if (key0 >= key1) return;
    for (int j = tid; j < kHistBins; j += kTopkThreads) h[j] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kPer; ++j)
        if (i + j < key1 && selectable(e[j])) atomicAdd(&h[order_key(e[j]) >> kLowBits], 1u);
    __syncthreads();
    uint32_t *gh = a.hist + (int64_t)bh * kHistBins;
    for (int j = tid; j < kHistBins; j += kTopkThreads)
        if (h[j]) atomicAdd(&gh[j], h[j]);
}

// First threshold digit, then the histogram of the second digit over the scores in it.
__global__ __launch_bounds__(kTopkThreads) void topk_hist2_kernel(TopkArgs a) {
    constexpr int PER = kHistBins / kTopkThreads;
    __shared__ uint32_t h[padded_size<kHistBins, PER>()];
    __shared__ uint32_t tmp[16];
    __shared__ uint32_t res[4];
    const int tid = threadIdx.x;
    const int bh = blockIdx.y, b = bh / a.Hkv;
    const int key0 = blockIdx.x * kSlice;
    const int i = key0 + tid * kPer;
    float e[kPer];
    load_scores(a.scores + (int64_t)bh * a.max_n, i, a.max_n, e);   // first: overlaps what follows
    const uint32_t *gh1 = a.hist + (int64_t)bh * kHistBins;
    uint32_t c1[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) c1[j] = gh1[tid + j * kTopkThreads];
    const int key1 = min(key0 + kSlice, clamp_len(a.seq_len[b], a.max_n));
    const uint32_t kreq = (uint32_t)clamp_len(a.k[b], a.max_k);
    if (key0 >= key1 && blockIdx.x != 0) return;       // workgroup 0 always publishes the record
#pragma unroll
    for (int j = 0; j < PER; ++j) h[padded<PER>(tid + j * kTopkThreads)] = c1[j];
    if (tid < 4) res[tid] = 0;
    __syncthreads();
    // a target beyond the number of valid scores finds nothing; res[3] then gives that number
    find_threshold<kHistBins>(h, kreq, res, tmp);
    uint32_t k_eff = kreq, tb1 = res[0], above1 = res[1], cnt1 = res[2];
    const uint32_t valid = res[3];
    if (valid < kreq) {                                 // fewer valid scores than asked for: take all
        k_eff = valid;
        if (valid > 0) {
            __syncthreads();
            find_threshold<kHistBins>(h, valid, res, tmp);
            tb1 = res[0]; above1 = res[1]; cnt1 = res[2];
        }
    }
    uint32_t *thr = a.thr + (int64_t)bh * kThrStride;
    if (blockIdx.x == 0 && tid == 0) {
        thr[0] = k_eff; thr[1] = tb1; thr[2] = above1; thr[3] = cnt1;
    }
    if (k_eff == 0 || key0 >= key1) return;
    __syncthreads();
    uint32_t *h2 = h;                                   // plain (unpadded) use from here on
    for (int j = tid; j < kHistBins; j += kTopkThreads) h2[j] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const uint32_t key = order_key(e[j]);
        if (i + j < key1 && selectable(e[j]) && (key >> kLowBits) == tb1) atomicAdd(&h2[digit2(key)], 1u);
    }
    __syncthreads();
    uint32_t *gh2 = a.hist2 + (int64_t)bh * kHistBins;
    for (int j = tid; j < kHistBins; j += kTopkThreads)
        if (h2[j]) atomicAdd(&gh2[j], h2[j]);
}

// Threshold, then the sweep.  ADAPT = false: the second threshold digit from the histogram of
// topk_hist2_kernel, lead = the two leading digits of the score key.  ADAPT = true: the
// threshold bin of the adaptive histogram, lead = that bin.
template <bool ADAPT>
__global__ __launch_bounds__(kTopkThreads) void topk_filter_kernel(TopkArgs a) {
    constexpr int PER = kHistBins / kTopkThreads;
    __shared__ uint32_t h[padded_size<kHistBins, PER>()];
    __shared__ uint32_t tmp[16];
    __shared__ uint32_t res[4];
    __shared__ uint32_t s_base[2];
    const int tid = threadIdx.x;
    const int bh = blockIdx.y, b = bh / a.Hkv;
    const int key0 = blockIdx.x * kSlice;
    const int i = key0 + tid * kPer;
    float e[kPer];
    load_scores(a.scores + (int64_t)bh * a.max_n, i, a.max_n, e);
    const uint32_t *gh = (ADAPT ? a.hist : a.hist2) + (int64_t)bh * kHistBins;
    uint32_t c2[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) c2[j] = gh[tid + j * kTopkThreads];
    uint32_t *thr = a.thr + (int64_t)bh * kThrStride;
    const int key1 = min(key0 + kSlice, clamp_len(a.seq_len[b], a.max_n));
    uint32_t k_eff, pair, above, n_cand;
    float bin_lo = 0.0f, bin_inv = 0.0f;
    if (ADAPT) {
        bin_lo = __uint_as_float(thr[kThrBinLo]);
        bin_inv = __uint_as_float(thr[kThrBinInv]);
        const uint32_t kreq = (uint32_t)clamp_len(a.k[b], a.max_k);
        if (key0 >= key1 && blockIdx.x != 0) return;   // workgroup 0 always publishes the record
#pragma unroll
        for (int j = 0; j < PER; ++j) h[padded<PER>(tid + j * kTopkThreads)] = c2[j];
        if (tid < 4) res[tid] = 0;
        __syncthreads();
        // a target beyond the number of valid scores finds nothing; res[3] then gives that number
        find_threshold<kHistBins>(h, kreq, res, tmp);
        k_eff = kreq;
        const uint32_t valid = res[3];
        if (valid < kreq) {                             // fewer valid scores than asked for: take all
            k_eff = valid;
            if (valid > 0) {
                __syncthreads();
                find_threshold<kHistBins>(h, valid, res, tmp);
            }
        }
        pair = res[0]; above = res[1]; n_cand = res[2];
        if (blockIdx.x == 0 && tid == 0) {
            thr[0] = k_eff; thr[5] = k_eff ? above : 0u; thr[6] = k_eff ? n_cand : 0u;
        }
        if (k_eff == 0) return;
    } else {
        k_eff = thr[0];
        const uint32_t tb1 = thr[1], above1 = thr[2];
        if (k_eff == 0) return;
        if (key0 >= key1 && blockIdx.x != 0) return;
#pragma unroll
        for (int j = 0; j < PER; ++j) h[padded<PER>(tid + j * kTopkThreads)] = c2[j];
        if (tid < 4) res[tid] = 0;
        __syncthreads();
        find_threshold<kHistBins>(h, k_eff - above1, res, tmp);    // 1 <= k_eff - above1 <= scores in tb1
        const uint32_t tb2 = res[0];
        above = above1 + res[1]; n_cand = res[2];
        if (blockIdx.x == 0 && tid == 0) {
            thr[4] = tb2; thr[5] = above; thr[6] = n_cand;
        }
        pair = (tb1 << kHistBits) | tb2;                           // the 2*kHistBits leading bits
    }
    if (key0 >= key1) return;
    uint32_t *cnt = a.counters + (int64_t)bh * kCounterStride;
    uint32_t *ckey = a.cand_key + (int64_t)bh * a.max_n;
    int32_t *cidx = a.cand_idx + (int64_t)bh * a.max_n;
    int32_t *staged = a.staged + (int64_t)bh * a.max_k;        // selected positions, unordered

    // Positions in the two lists are handed out with one atomic per workgroup and list:
    // every thread counts its hits and a block scan turns the counts into offsets.
    uint32_t keys[kPer];
    uint32_t flags = 0;                           // bit j: selected, bit 16+j: candidate
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const bool ok = i + j < key1 && selectable(e[j]);
        keys[j] = order_key(e[j]);
        const uint32_t lead = ADAPT ? score_bin(e[j], bin_lo, bin_inv) : keys[j] >> kDigit2Shift;
        if (ok && lead > pair) flags |= 1u << j;
        if (ok && lead == pair) flags |= 1u << (16 + j);
    }
    const uint32_t mine = (uint32_t)__popc(flags & 0xffffu) | ((uint32_t)__popc(flags >> 16) << 16);
    uint32_t total;
    const uint32_t before = block_excl_scan(mine, &total, tmp);   // both counts in one word
    if (tid == 0) {
        const uint32_t nsel = total & 0xffffu, ncand = total >> 16;
        s_base[0] = nsel ? atomicAdd(&cnt[0], nsel) : 0u;
        s_base[1] = ncand ? atomicAdd(&cnt[1], ncand) : 0u;
    }
    __syncthreads();
    uint32_t at_sel = s_base[0] + (before & 0xffffu), at_cand = s_base[1] + (before >> 16);
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        if (flags & (1u << j)) staged[at_sel++] = i + j;
        if (flags & (1u << (16 + j))) {
            ckey[at_cand] = keys[j];
            cidx[at_cand] = i + j;
            ++at_cand;
        }
    }
}

// Refinement digits of a candidate (long candidate lists only):
//   level 0..2: the first, the second and the remaining low digit of the score key (candidates
//               that came through the two-digit threshold agree on levels 0 and 1)
//   level 3..5: bits 30..19, 18..7, 6..0 of (2^31-1 - position), so a smaller position ranks higher
constexpr int kLevels = 6;
__device__ __forceinline__ uint32_t refine_digit(int level, uint32_t key, int32_t pos) {
    uint32_t inv = 0x7fffffffu - (uint32_t)pos;
    switch (level) {
        case 0: return key >> kLowBits;
        case 1: return digit2(key);
        case 2: return key & ((1u << kDigit2Shift) - 1u);
        case 3: return (inv >> 19) & 0xfffu;
        case 4: return (inv >> 7) & 0xfffu;
        default: return inv & 0x7fu;
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_resolve_kernel(TopkArgs a) {
    constexpr int RPER = kRefineBins / kTopkThreads, BPER = kBitmapWords / kTopkThreads;
    extern __shared__ uint32_t h[];               // 2 * padded_size<kBitmapWords, BPER>() words
    __shared__ uint32_t tmp[16];
    __shared__ uint32_t res[4];
    __shared__ uint32_t chosen[kLevels];
    __shared__ uint32_t s_count;
    constexpr int PRE = 8;                        // list entries per thread fetched up front
    const int tid = threadIdx.x;
    const int bh = blockIdx.x, b = bh / a.Hkv;
    uint32_t *gh1 = a.hist + (int64_t)bh * kHistBins;
    uint32_t *gh2 = a.hist2 + (int64_t)bh * kHistBins;
    uint32_t *cnt = a.counters + (int64_t)bh * kCounterStride;
    const uint32_t *thr = a.thr + (int64_t)bh * kThrStride;
    const uint32_t *ckey = a.cand_key + (int64_t)bh * a.max_n;
    const int32_t *cidx = a.cand_idx + (int64_t)bh * a.max_n;
    int32_t *staged = a.staged + (int64_t)bh * a.max_k;
    int32_t *out = a.idx + (int64_t)bh * a.max_k;
    SK_STAMP(0);
    // The heads of both lists are fetched before their lengths are known (the reads stay inside
    // the buffers), so that their latency overlaps the load of the threshold record.
    uint32_t pk[2];
    int32_t pp[2], ps[PRE];
#pragma unroll
    for (int j = 0; j < PRE; ++j) {
        const int i = tid + j * kTopkThreads;
        if (j < 2) {
            pk[j] = i < a.max_n ? ckey[i] : 0u;
            pp[j] = i < a.max_n ? cidx[i] : 0;
        }
        ps[j] = i < a.max_k ? staged[i] : 0;
    }
    const uint32_t k_eff = thr[0], above = k_eff ? thr[5] : 0u, n_cand = k_eff ? thr[6] : 0u;
    const int seq = clamp_len(a.seq_len[b], a.max_n);
    const uint32_t need0 = k_eff - above;         // candidates to keep
    SK_STAMP(1);

    bool keep[2] = {false, false};                // short list: this thread's candidates that are kept
    const bool short_list = n_cand <= (uint32_t)kRankMax;
    if (k_eff > 0 && short_list) {
        // ---- all-pairs ranking in LDS on (score bits, smaller position first)
        unsigned long long *ck = (unsigned long long *)h;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t i = tid + j * kTopkThreads;
            if (i < n_cand) ck[i] = ((unsigned long long)pk[j] << 32) | (0x7fffffffu - (uint32_t)pp[j]);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t i = tid + j * kTopkThreads;
            if (i < n_cand) {
                const unsigned long long me = ck[i];
                uint32_t rank = 0;
                for (uint32_t o = 0; o < n_cand; ++o) rank += ck[o] > me;
                keep[j] = rank < need0;
            }
        }
        __syncthreads();
    } else if (k_eff > 0) {
        // ---- long list (many tied scores): digit-by-digit refinement over the list in memory
        auto for_candidates = [&](int level, auto f) {
            for (uint32_t i = tid; i < n_cand; i += kTopkThreads) {
                const uint32_t key = ckey[i];
                const int32_t pos = cidx[i];
                bool match = true;
                for (int l = 0; l < level; ++l) match = match && refine_digit(l, key, pos) == chosen[l];
                if (match) f(key, pos);
            }
        };
        uint32_t need = need0, remaining = n_cand;
        if (tid == 0) {
            s_count = above;                      // next free staging slot
            chosen[0] = thr[1];                   // the digits every two-digit candidate has
            chosen[1] = thr[4];
        }
        __syncthreads();
        int level = a.adaptive ? 0 : 2;
        while (need > 0 && need < remaining && level < kLevels) {
            for (int i = tid; i < padded_size<kRefineBins, RPER>(); i += kTopkThreads) h[i] = 0;
            if (tid < 4) res[tid] = 0;
            __syncthreads();
            for_candidates(level, [&](uint32_t key, int32_t pos) {
                atomicAdd(&h[padded<RPER>((int)refine_digit(level, key, pos))], 1u);
            });
            __syncthreads();
            find_threshold<kRefineBins>(h, need, res, tmp);
            const uint32_t td = res[0];
            // candidates on the current prefix with a larger digit are selected
            for_candidates(level, [&](uint32_t key, int32_t pos) {
                if (refine_digit(level, key, pos) > td) staged[atomicAdd(&s_count, 1u)] = pos;
            });
            need -= res[1];
            remaining = res[2];
            __syncthreads();
            if (tid == 0) chosen[level] = td;
            ++level;
            __syncthreads();
        }
        if (need > 0)     // need == remaining: everything left on the prefix is selected
            for_candidates(level, [&](uint32_t, int32_t pos) { staged[atomicAdd(&s_count, 1u)] = pos; });
        __syncthreads();
    }
    SK_STAMP(2);

    if (k_eff > 0) {
        // ---- ascending emit: a bitmap of the selected positions in LDS, the running count of
        //      set bits before every bitmap word, then each selected position looks up its own
        //      rank (count before its word + set bits below it inside the word).
        uint32_t *before = h + padded_size<kBitmapWords, BPER>();       // [kBitmapWords], padded
        auto mark = [&](int32_t p) {
            if (p >= 0 && p < kBitmapTokens) atomicOr(&h[padded<BPER>(p >> 5)], 1u << (p & 31));
        };
        uint32_t written = 0;
        // every selected position, wherever it is kept, goes through f once
        auto for_selected = [&](auto f) {
#pragma unroll
            for (int j = 0; j < PRE; ++j)         // slots filled by the sweep: already in registers
                if (tid + j * kTopkThreads < above) f(ps[j]);
            for (uint32_t i = tid + PRE * kTopkThreads; i < above; i += kTopkThreads) f(staged[i]);
            if (short_list) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    if (keep[j]) f(pp[j]);
            } else {
                for (uint32_t i = above + tid; i < k_eff; i += kTopkThreads) f(staged[i]);
            }
        };
        for (int base = 0; base < seq; base += kBitmapTokens) {
            for (int i = tid; i < padded_size<kBitmapWords, BPER>(); i += kTopkThreads) h[i] = 0;
            __syncthreads();
            for_selected([&](int32_t p) { mark(p - base); });
            __syncthreads();
            uint32_t c[BPER];
            uint32_t mine = 0;
#pragma unroll
            for (int i = 0; i < BPER; ++i) {
                c[i] = __popc(h[padded<BPER>(tid * BPER + i)]);
                mine += c[i];
            }
            uint32_t total;
            uint32_t run = block_excl_scan(mine, &total, tmp);
#pragma unroll
            for (int i = 0; i < BPER; ++i) {
                before[padded<BPER>(tid * BPER + i)] = run;
                run += c[i];
            }
            __syncthreads();
            for_selected([&](int32_t p) {
                const int32_t q = p - base;
                if (q < 0 || q >= kBitmapTokens) return;
                const int wi = padded<BPER>(q >> 5);
                const uint32_t rank = written + before[wi] + __popc(h[wi] & ((1u << (q & 31)) - 1u));
                if (rank < (uint32_t)a.max_k) out[rank] = p;
            });
            written += total;
            __syncthreads();
        }
    }
    SK_STAMP(3);
    for (int i = (int)k_eff + tid; i < a.max_k; i += kTopkThreads) out[i] = -1;
    if (tid == 0) a.n_selected[bh] = (int32_t)k_eff;
    // leave the shared scratch clean for the next call
    for (int i = tid; i < kHistBins; i += kTopkThreads) {
        gh1[i] = 0;
        gh2[i] = 0;
    }
    if (tid < 2) cnt[tid] = 0;
    SK_STAMP(4);
#ifdef SK_DEBUG_CLOCKS
    if (threadIdx.x == 0 && blockIdx.x == 0) { sk_dbg[10] = n_cand; sk_dbg[11] = above; sk_dbg[12] = k_eff; }
#endif
}

#ifdef SK_DEBUG_CLOCKS
extern "C" int socket_debug_clocks(long long *out) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(sk_dbg), sizeof(long long) * 64);
}
#endif

int launch_topk(socket_ctx *ctx, const float *scores, const int32_t *seq_len, const int32_t *k,
                int batch, int32_t *idx, int32_t *n_selected, int hist_mode, hipStream_t st) {
    const Geometry &g = ctx->g;
    TopkArgs a;
    a.scores = scores; a.seq_len = seq_len; a.k = k; a.idx = idx; a.n_selected = n_selected;
    const int64_t BHmax = (int64_t)g.max_batch * g.Hkv;
    a.hist = ctx->hist; a.hist2 = ctx->hist + BHmax * kHistBins; a.thr = ctx->counters + BHmax * kCounterStride;
    a.counters = ctx->counters; a.cand_key = ctx->cand_key; a.cand_idx = ctx->cand_idx; a.staged = ctx->staged;
    a.Hkv = g.Hkv; a.max_n = g.max_n; a.max_k = g.max_k; a.adaptive = hist_mode == kHistAdaptive;
    const int BH = batch * g.Hkv;
    dim3 grid((g.max_n + kSlice - 1) / kSlice, BH);
    if (hist_mode == kHistAdaptive) {
        hipLaunchKernelGGL(topk_filter_kernel<true>, grid, dim3(kTopkThreads), 0, st, a);
    } else {
        if (hist_mode == kHistNone) hipLaunchKernelGGL(topk_hist_kernel, grid, dim3(kTopkThreads), 0, st, a);
        hipLaunchKernelGGL(topk_hist2_kernel, grid, dim3(kTopkThreads), 0, st, a);
        hipLaunchKernelGGL(topk_filter_kernel<false>, grid, dim3(kTopkThreads), 0, st, a);
    }
    constexpr size_t kResolveLds = 2 * (size_t)padded_size<kBitmapWords, kBitmapWords / kTopkThreads>() * 4;
    static bool lds_raised = false;   // 68 KB of dynamic LDS has to be allowed once per process
    if (!lds_raised) {
        if (hipFuncSetAttribute((const void *)topk_resolve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kResolveLds) != hipSuccess) return SOCKET_EHIP;
        lds_raised = true;
    }
    hipLaunchKernelGGL(topk_resolve_kernel, dim3(BH), dim3(kTopkThreads), kResolveLds, st, a);
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

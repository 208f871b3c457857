// Device code of the TopK step that more than one translation unit uses: the argument block,
// block-wide scans, the threshold search, and the resolve step (ranking of the candidates and
// ascending emit) as a device function.
#pragma once

#include "socket_internal.h"

namespace sk {

constexpr int kRefineBins = 4096;                // bins of a candidate-refinement digit
constexpr int kBitmapWords = 4096;               // 16 KB of LDS
constexpr int kBitmapTokens = kBitmapWords * 32; // tokens one LDS bitmap pass covers
constexpr int kLowBits = 32 - kHistBits;         // score bits below the leading digit
constexpr int kDigit2Shift = kLowBits - kHistBits;   // second digit: the next kHistBits score bits
static_assert(kDigit2Shift >= 0 && kDigit2Shift <= 12, "the low score bits fit one refinement digit");
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
    int32_t *staged;      // candidates picked by the long-list refinement
    int32_t *sel_regions; // positions selected outright, [n_regions][kSlice] per (sequence, KV head)
    uint32_t *sel_cnt;    // [n_regions] per (sequence, KV head)
    int n_regions;
    int pre_shift;        // the ordering step fetches the first 2^pre_shift entries of every region up front
    int Hkv, max_n, max_k;
    int adaptive;         // candidates share an adaptive bin, not the two leading digits
};

// the argument block for a context's scratch buffers
inline TopkArgs topk_args(socket_ctx *ctx, const float *scores, const int32_t *seq_len, const int32_t *k,
                          int32_t *idx, int32_t *n_selected, int hist_mode) {
    const Geometry &g = ctx->g;
    TopkArgs a;
    a.scores = scores; a.seq_len = seq_len; a.k = k; a.idx = idx; a.n_selected = n_selected;
    const int64_t BHmax = (int64_t)g.max_batch * g.Hkv;
    a.hist = ctx->hist; a.hist2 = ctx->hist + BHmax * kHistBins; a.thr = ctx->counters + BHmax * kCounterStride;
    a.counters = ctx->counters; a.cand_key = ctx->cand_key; a.cand_idx = ctx->cand_idx; a.staged = ctx->staged;
    a.sel_regions = ctx->sel_regions; a.sel_cnt = ctx->sel_cnt; a.n_regions = g.n_regions;
    a.pre_shift = 0;                                   // 16 * 512 preloads spread over the regions
    while (a.pre_shift < 12 && ((int64_t)g.n_regions << (a.pre_shift + 1)) <= 16 * kTopkThreads) ++a.pre_shift;
    a.Hkv = g.Hkv; a.max_n = g.max_n; a.max_k = g.max_k; a.adaptive = hist_mode == kHistAdaptive;
    return a;
}

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

// dynamic LDS the resolve step needs (two padded bitmap-sized arrays)
constexpr size_t kResolveLds = 2 * (size_t)padded_size<kBitmapWords, kBitmapWords / kTopkThreads>() * 4;

// The resolve step for one (sequence, KV head), run by a whole workgroup of kTopkThreads
// threads; `h` is kResolveLds bytes of LDS.  A device function, so that it can also be one of
// the roles of a launch whose other workgroups do other work.
__device__ __forceinline__ void topk_resolve_body(const TopkArgs &a, int bh, uint32_t *h) {
    constexpr int RPER = kRefineBins / kTopkThreads, BPER = kBitmapWords / kTopkThreads;
    __shared__ uint32_t tmp[16];
    __shared__ uint32_t res[4];
    __shared__ uint32_t chosen[kLevels];
    __shared__ uint32_t s_count;
    constexpr int kFastCand = 16;                 // kept candidates the merge-by-counting emit handles
    __shared__ int32_t s_kc[kFastCand];           // their positions
    __shared__ uint32_t s_nk;
    constexpr int PRE = 16;                       // list entries per thread fetched up front
    const int tid = threadIdx.x;
    const int b = bh / a.Hkv;
    uint32_t *gh1 = a.hist + (int64_t)bh * kHistBins;
    uint32_t *gh2 = a.hist2 + (int64_t)bh * kHistBins;
    uint32_t *cnt = a.counters + (int64_t)bh * kCounterStride;
    const uint32_t *thr = a.thr + (int64_t)bh * kThrStride;
    const uint32_t *ckey = a.cand_key + (int64_t)bh * a.max_n;
    const int32_t *cidx = a.cand_idx + (int64_t)bh * a.max_n;
    int32_t *staged = a.staged + (int64_t)bh * a.max_k;
    const int32_t *regions = a.sel_regions + (int64_t)bh * a.n_regions * kSlice;
    const uint32_t *selcnt = a.sel_cnt + (int64_t)bh * a.n_regions;
    __shared__ uint32_t s_regcnt[kMaxRegions];
    int32_t *out = a.idx + (int64_t)bh * a.max_k;
    // The heads of the lists are fetched before their lengths are known (the reads stay inside
    // the buffers), so that their latency overlaps the load of the threshold record: two
    // candidates per thread, and the first 2^pre_shift entries of every region.
    const int pre_n = 1 << a.pre_shift;
    uint32_t pk[2];
    int32_t pp[2], ps[PRE];
#pragma unroll
    for (int j = 0; j < PRE; ++j) {
        const int i = tid + j * kTopkThreads;
        if (j < 2) {
            pk[j] = i < a.max_n ? ckey[i] : 0u;
            pp[j] = i < a.max_n ? cidx[i] : 0;
        }
        const int rg = (i >> a.pre_shift) < a.n_regions ? i >> a.pre_shift : a.n_regions - 1;   // (a region that exists: the load is unconditional)
        ps[j] = regions[(int64_t)rg * kSlice + (i & (pre_n - 1))];
    }
    // (the loads above are wanted now, in flight beside the threshold record's: without this
    // the compiler moves each of them down to its first use, one memory latency apiece)
#pragma unroll
    for (int j = 0; j < PRE; ++j) asm volatile("" : "+v"(ps[j]));
    for (int i = tid; i < a.n_regions; i += kTopkThreads) s_regcnt[i] = selcnt[i];
    if (tid == 0) s_nk = 0;
    const uint32_t k_eff = thr[0], above = k_eff ? thr[5] : 0u, n_cand = k_eff ? thr[6] : 0u;
    const int seq = clamp_len(a.seq_len[b], a.max_n);
    const uint32_t need0 = k_eff - above;         // candidates to keep

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
            s_count = 0;                          // next free slot of the picked list
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

    // does any region hold entries beyond those in registers?
    bool spill = false;
    if (k_eff > 0) {
        bool mine = false;
        for (int r = tid; r < a.n_regions; r += kTopkThreads) mine = mine || s_regcnt[r] > (uint32_t)pre_n;
        spill = __syncthreads_or(mine);
    }
    const bool fast = k_eff > 0 && short_list && !spill && need0 <= (uint32_t)kFastCand && a.n_regions <= kTopkThreads;
    if (fast) {
        // ---- ascending emit by counting.  The regions, one after the other, already are the
        //      positions selected outright in ascending order; the few kept candidates have to be
        //      slipped in.  An entry's place is its index in that order plus the number of kept
        //      candidates before it; a candidate's place is the number of entries before it (a
        //      binary search in its own region, whose entries are all in LDS) plus the number of
        //      kept candidates before it.
        int32_t *s_ent = (int32_t *)h;                              // [n_regions << pre_shift]
        uint32_t *s_regpre = h + (kTopkThreads * PRE);              // [n_regions] entries before each region
#pragma unroll
        for (int j = 0; j < PRE; ++j) s_ent[tid + j * kTopkThreads] = ps[j];
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (keep[j]) s_kc[atomicAdd(&s_nk, 1u)] = pp[j];        // (their order does not matter: they are only counted)
        uint32_t total;
        const uint32_t pre = block_excl_scan(tid < a.n_regions ? s_regcnt[tid] : 0u, &total, tmp);
        s_regpre[tid] = pre;
        __syncthreads();
        const int nk = (int)s_nk;
        int32_t kc[kFastCand];                                      // the kept candidates, in registers
#pragma unroll
        for (int q = 0; q < kFastCand; ++q) kc[q] = q < nk ? s_kc[q] : 0x7fffffff;
        auto kept_before = [&](int32_t p) {
            uint32_t c = 0;
#pragma unroll
            for (int q = 0; q < kFastCand; ++q) c += kc[q] < p;
            return c;
        };
#pragma unroll
        for (int j = 0; j < PRE; ++j) {
            const int i = tid + j * kTopkThreads;
            const int rg = i >> a.pre_shift, e = i & (pre_n - 1);
            if (rg < a.n_regions && (uint32_t)e < s_regcnt[rg]) out[s_regpre[rg] + e + kept_before(ps[j])] = ps[j];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (keep[j]) {
                const int32_t p = pp[j];
                const int rg = p / kSlice;
                const int32_t *ent = s_ent + (rg << a.pre_shift);
                int lo = 0, hi = (int)s_regcnt[rg];                 // first entry >= p
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (ent[mid] < p) lo = mid + 1; else hi = mid;
                }
                out[s_regpre[rg] + lo + kept_before(p)] = p;
            }
    } else if (k_eff > 0) {
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
            for (int j = 0; j < PRE; ++j) {       // heads of the regions: already in registers
                const int i = tid + j * kTopkThreads;
                if ((i >> a.pre_shift) < a.n_regions && (uint32_t)(i & (pre_n - 1)) < s_regcnt[i >> a.pre_shift]) f(ps[j]);
            }
            if (spill)                            // regions that hold more than the entries fetched up front
                for (int r = 0; r < a.n_regions; ++r) {
                    const uint32_t c = s_regcnt[r];
                    for (uint32_t e = (uint32_t)pre_n + tid; e < c; e += kTopkThreads) f(regions[(int64_t)r * kSlice + e]);
                }
            if (short_list) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    if (keep[j]) f(pp[j]);
            } else {
                for (uint32_t i = tid; i < need0; i += kTopkThreads) f(staged[i]);
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
    for (int i = (int)k_eff + tid; i < a.max_k; i += kTopkThreads) out[i] = -1;
    if (tid == 0) a.n_selected[bh] = (int32_t)k_eff;
    // leave the shared scratch clean for the next call
    for (int i = tid; i < kHistBins; i += kTopkThreads) {
        gh1[i] = 0;
        gh2[i] = 0;
    }
    if (tid < 2) cnt[tid] = 0;
}

}  // namespace sk

// Alg. 3, TopK step: exact selection of the k largest scores per (sequence, KV head) by a
// most-significant-digit radix select on the fp32 bit patterns, spread over many workgroups.
//
//   topk_hist_kernel    histogram of the leading 11-bit digit of every valid score (the fused
//                       decode step gets it from the scoring pass instead).
//   topk_hist2_kernel   histogram of the next 11 bits over the scores in the threshold digit.
//   topk_filter_kernel  sweep: scores above the two-digit threshold are selected, scores equal
//                       to it become candidates.
//   topk_resolve_kernel one workgroup per (sequence, head): resolves the candidates on the
//                       remaining score bits and then on the token position, and writes the
//                       selection in ascending position order.
// Stages talk through global memory across kernel boundaries only: no workgroup waits on
// another and no fence is needed.
#include "socket_internal.h"

namespace sk {

#ifdef SK_DEBUG_CLOCKS
__device__ long long sk_dbg[64];
#define SK_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x == 0) sk_dbg[i] = wall_clock64(); } while (0)
#else
#define SK_STAMP(i) ((void)0)
#endif

constexpr int kTopkThreads = 512;
constexpr int kRefineBins = 4096;                // bins of the candidate-refinement digits
constexpr int kBitmapWords = 8192;               // 32 KB of LDS
constexpr int kBitmapTokens = kBitmapWords * 32; // tokens one LDS bitmap pass covers
constexpr int kLowBits = 32 - kHistBits;         // score bits below the leading digit
static_assert(kLowBits > 12 && kLowBits <= 24, "two refinement digits of at most 12 bits");
constexpr int kPer = 8;                         // scores per thread in a sweep
constexpr int kSlice = kTopkThreads * kPer;     // scores per workgroup

struct TopkArgs {
    const float *scores;
    const int32_t *seq_len;
    const int32_t *k;
    int32_t *idx;
    int32_t *n_selected;
    uint32_t *hist;       // first-digit histograms [B*Hkv][kHistBins]
    uint32_t *hist2;      // second-digit histograms of the threshold bin
    uint32_t *counters;
    uint32_t *cand_key;
    int32_t *cand_idx;
    int32_t *staged;
    int Hkv, max_n, max_k;
};

// Order-preserving map from fp32 to uint32 (larger float -> larger key).
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ bool selectable(float f) { return f > -__builtin_inff(); }  // false for NaN

// Exclusive prefix sum over the 512 threads of a block; *total gets the block sum.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *total, uint32_t *tmp) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
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

// Largest bin tb of the NBINS-bin LDS histogram h with count(bins >= tb) >= target.
// res[0] = tb, res[1] = count(bins > tb), res[2] = h[tb].  Requires 1 <= target <= sum(h).
template <int NBINS>
__device__ __forceinline__ void find_threshold(const uint32_t *h, uint32_t target, uint32_t *res,
                                               uint32_t *tmp) {
    const int t = threadIdx.x;
    constexpr int PER = NBINS / kTopkThreads;       // bins per thread, highest bins first
    const int top = NBINS - 1 - t * PER;
    uint32_t part = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) part += h[top - i];
    uint32_t total;
    uint32_t above = block_excl_scan(part, &total, tmp);
    if (above < target && target <= above + part) {
        uint32_t cum = above;
        for (int i = 0; i < PER; ++i) {
            uint32_t c = h[top - i];
            if (cum + c >= target) {
                res[0] = (uint32_t)(top - i);
                res[1] = cum;
                res[2] = c;
                break;
            }
            cum += c;
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kTopkThreads) void topk_hist_kernel(TopkArgs a) {
    __shared__ uint32_t h[kHistBins];
    const int tid = threadIdx.x;
    const int bh = blockIdx.y, b = bh / a.Hkv;
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > a.max_n ? a.max_n : seq);
    const int key0 = blockIdx.x * kSlice;
    const int key1 = min(key0 + kSlice, seq);
    if (key0 >= key1) return;
    for (int i = tid; i < kHistBins; i += kTopkThreads) h[i] = 0;
    __syncthreads();
    const float *s = a.scores + (int64_t)bh * a.max_n;
    for (int i = key0 + tid * 4; i < key1; i += kTopkThreads * 4) {
        float4 v = *(const float4 *)(s + i);      // max_n and slice are multiples of 4
        float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i + j < key1 && selectable(e[j])) atomicAdd(&h[order_key(e[j]) >> kLowBits], 1u);
    }
    __syncthreads();
    uint32_t *gh = a.hist + (int64_t)bh * kHistBins;
    for (int i = tid; i < kHistBins; i += kTopkThreads)
        if (h[i]) atomicAdd(&gh[i], h[i]);
}

// Threshold of the two leading digits, recomputed identically by every workgroup that
// needs it: tb1 from the first-digit histogram, then tb2 among the scores whose first digit
// is tb1.  out: [0] k_eff, [1] tb1, [2] tb2, [3] scores selected outright (above the pair),
// [4] scores equal to the pair (candidates).  h is LDS scratch of >= kHistBins words.
__device__ __forceinline__ void two_digit_threshold(const uint32_t *gh1, const uint32_t *gh2, int kreq,
                                                    bool want_second, uint32_t *h, uint32_t *res,
                                                    uint32_t *tmp, uint32_t *out) {
    const int tid = threadIdx.x;
    constexpr int PER = kHistBins / kTopkThreads;
    uint32_t c1[PER], c2[PER];                    // both histograms' loads go out together
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        c1[j] = gh1[tid + j * kTopkThreads];
        c2[j] = want_second ? gh2[tid + j * kTopkThreads] : 0u;
    }
    uint32_t part = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        h[tid + j * kTopkThreads] = c1[j];
        part += c1[j];
    }
    if (tid < 4) res[tid] = 0;
    __syncthreads();
    uint32_t valid;
    (void)block_excl_scan(part, &valid, tmp);
    const uint32_t k_eff = min((uint32_t)kreq, valid);
    out[0] = k_eff; out[1] = 0; out[2] = 0; out[3] = 0; out[4] = 0;
    if (k_eff == 0) return;
    find_threshold<kHistBins>(h, k_eff, res, tmp);
    const uint32_t tb1 = res[0], above1 = res[1], cnt1 = res[2];
    out[1] = tb1; out[3] = above1; out[4] = cnt1;
    if (!want_second) return;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PER; ++j) h[tid + j * kTopkThreads] = c2[j];
    __syncthreads();
    find_threshold<kHistBins>(h, k_eff - above1, res, tmp);   // 1 <= k_eff - above1 <= cnt1
    out[2] = res[0]; out[3] = above1 + res[1]; out[4] = res[2];
}

constexpr int kDigit2Shift = kLowBits - kHistBits;    // second digit: the next kHistBits score bits
static_assert(kDigit2Shift >= 0 && kDigit2Shift <= 12, "the low score bits fit one refinement digit");
__device__ __forceinline__ uint32_t digit2(uint32_t key) { return (key >> kDigit2Shift) & (kHistBins - 1); }

// Histogram of the second digit over the scores whose first digit is the threshold digit.
__global__ __launch_bounds__(kTopkThreads) void topk_hist2_kernel(TopkArgs a) {
    __shared__ uint32_t h[kHistBins];
    __shared__ uint32_t tmp[16];
    __shared__ uint32_t res[4];
    const int tid = threadIdx.x;
    const int bh = blockIdx.y, b = bh / a.Hkv;
    const int key0 = blockIdx.x * kSlice;
    const int i = key0 + tid * kPer;
    // this thread's scores first (in bounds for any length), so that their latency overlaps
    // the histogram loads and the threshold search
    const float *s = a.scores + (int64_t)bh * a.max_n;
    float e[kPer];
#pragma unroll
    for (int v = 0; v < kPer / 4; ++v) {
        float4 q = i + 4 * v < a.max_n ? *(const float4 *)(s + i + 4 * v) : make_float4(0, 0, 0, 0);
        e[4 * v] = q.x; e[4 * v + 1] = q.y; e[4 * v + 2] = q.z; e[4 * v + 3] = q.w;
    }
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > a.max_n ? a.max_n : seq);
    const int key1 = min(key0 + kSlice, seq);
    if (key0 >= key1) return;
    int kreq = a.k[b];
    kreq = kreq < 0 ? 0 : (kreq > a.max_k ? a.max_k : kreq);
    uint32_t th[5];
    two_digit_threshold(a.hist + (int64_t)bh * kHistBins, nullptr, kreq, false, h, res, tmp, th);
    if (th[0] == 0) return;
    const uint32_t tb1 = th[1];
    __syncthreads();
    for (int j = tid; j < kHistBins; j += kTopkThreads) h[j] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const uint32_t key = order_key(e[j]);
        if (i + j < key1 && selectable(e[j]) && (key >> kLowBits) == tb1) atomicAdd(&h[digit2(key)], 1u);
    }
    __syncthreads();
    uint32_t *gh2 = a.hist2 + (int64_t)bh * kHistBins;
    for (int j = tid; j < kHistBins; j += kTopkThreads)
        if (h[j]) atomicAdd(&gh2[j], h[j]);
}

// Sweep: scores above the two-digit threshold are selected, scores equal to it become
// candidates (few: one bin of a 2^22-bin histogram unless many scores tie).
__global__ __launch_bounds__(kTopkThreads) void topk_filter_kernel(TopkArgs a) {
    __shared__ uint32_t h[kHistBins];
    __shared__ uint32_t tmp[16];
    __shared__ uint32_t res[4];
    __shared__ uint32_t s_base[2];
    const int tid = threadIdx.x;
    const int bh = blockIdx.y, b = bh / a.Hkv;
    const int key0 = blockIdx.x * kSlice;
    const int i = key0 + tid * kPer;
    // kSlice scores per workgroup, kPer per thread, loaded first and held in registers
    const float *s = a.scores + (int64_t)bh * a.max_n;
    float e[kPer];
#pragma unroll
    for (int v = 0; v < kPer / 4; ++v) {
        float4 q = i + 4 * v < a.max_n ? *(const float4 *)(s + i + 4 * v) : make_float4(0, 0, 0, 0);
        e[4 * v] = q.x; e[4 * v + 1] = q.y; e[4 * v + 2] = q.z; e[4 * v + 3] = q.w;
    }
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > a.max_n ? a.max_n : seq);
    const int key1 = min(key0 + kSlice, seq);
    if (key0 >= key1) return;
    int kreq = a.k[b];
    kreq = kreq < 0 ? 0 : (kreq > a.max_k ? a.max_k : kreq);
    uint32_t th[5];
    two_digit_threshold(a.hist + (int64_t)bh * kHistBins, a.hist2 + (int64_t)bh * kHistBins, kreq, true, h,
                        res, tmp, th);
    if (th[0] == 0) return;
    const uint32_t pair = (th[1] << kHistBits) | th[2];       // the 2*kHistBits leading bits
    uint32_t *cnt = a.counters + (int64_t)bh * kCounterStride;
    uint32_t *ckey = a.cand_key + (int64_t)bh * a.max_n;
    int32_t *cidx = a.cand_idx + (int64_t)bh * a.max_n;
    int32_t *staged = a.staged + (int64_t)bh * a.max_k;       // selected positions, unordered

    // Positions in the two lists are handed out with one atomic per workgroup and list:
    // every thread counts its hits and a block scan turns the counts into offsets.
    uint32_t keys[kPer];
    uint32_t flags = 0;                           // bit j: selected, bit 16+j: candidate
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const bool ok = i + j < key1 && selectable(e[j]);
        keys[j] = order_key(e[j]);
        const uint32_t lead = keys[j] >> kDigit2Shift;
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

// Refinement digits of a candidate below the two leading digits:
//   level 0: the remaining low score bits
//   level 1..3: bits 30..19, 18..7, 6..0 of (2^31-1 - position), so a smaller position ranks higher
constexpr int kLevels = 4;
__device__ __forceinline__ uint32_t refine_digit(int level, uint32_t key, int32_t pos) {
    uint32_t inv = 0x7fffffffu - (uint32_t)pos;
    switch (level) {
        case 0: return key & ((1u << kDigit2Shift) - 1u);
        case 1: return (inv >> 19) & 0xfffu;
        case 2: return (inv >> 7) & 0xfffu;
        default: return inv & 0x7fu;
    }
}

// One workgroup per (sequence, KV head): resolves the candidates on the remaining score bits
// and then on the token position (smaller position wins a tie), writes the selection in
// ascending position order through an LDS bitmap, and leaves histograms and counters at
// zero for the next call.  Runs after the sweep as a kernel of its own, so it needs no
// fence or inter-workgroup signalling.
__global__ __launch_bounds__(kTopkThreads) void topk_resolve_kernel(TopkArgs a) {
    extern __shared__ uint32_t h[];               // kBitmapWords words: refinement histogram, then bitmap
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
    const uint32_t *ckey = a.cand_key + (int64_t)bh * a.max_n;
    const int32_t *cidx = a.cand_idx + (int64_t)bh * a.max_n;
    int32_t *staged = a.staged + (int64_t)bh * a.max_k;
    int32_t *out = a.idx + (int64_t)bh * a.max_k;
    // The heads of both lists are fetched before their lengths are known (the reads stay inside
    // the buffers), so that their latency overlaps the histogram loads and threshold search.
    SK_STAMP(0);
    uint32_t pk[PRE];
    int32_t pp[PRE], ps[PRE];
#pragma unroll
    for (int j = 0; j < PRE; ++j) {
        const int i = tid + j * kTopkThreads;
        pk[j] = i < a.max_n ? ckey[i] : 0u;
        pp[j] = i < a.max_n ? cidx[i] : 0;
        ps[j] = i < a.max_k ? staged[i] : 0;
    }
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > a.max_n ? a.max_n : seq);
    int kreq = a.k[b];
    kreq = kreq < 0 ? 0 : (kreq > a.max_k ? a.max_k : kreq);
    uint32_t th[5];
    two_digit_threshold(gh1, gh2, kreq, true, h, res, tmp, th);
    const uint32_t k_eff = th[0], above = th[3], n_cand = th[4];
    __syncthreads();
    SK_STAMP(1);

    // visit every candidate on the prefix chosen so far: f(key, position)
    auto for_candidates = [&](int level, auto f) {
#pragma unroll
        for (int j = 0; j < PRE; ++j) {
            const uint32_t i = tid + j * kTopkThreads;
            if (i >= n_cand) continue;
            bool match = true;
            for (int l = 0; l < level; ++l) match = match && refine_digit(l, pk[j], pp[j]) == chosen[l];
            if (match) f(pk[j], pp[j]);
        }
        for (uint32_t i = tid + PRE * kTopkThreads; i < n_cand; i += kTopkThreads) {
            const uint32_t key = ckey[i];
            const int32_t pos = cidx[i];
            bool match = true;
            for (int l = 0; l < level; ++l) match = match && refine_digit(l, key, pos) == chosen[l];
            if (match) f(key, pos);
        }
    };

    if (k_eff > 0) {
        // keep the `need` best of the n_cand candidates
        uint32_t need = k_eff - above, remaining = n_cand;
        if (tid == 0) s_count = above;            // next free staging slot
        __syncthreads();
        int level = 0;
        while (need > 0 && need < remaining && level < kLevels) {
            for (int i = tid; i < kRefineBins; i += kTopkThreads) h[i] = 0;
            __syncthreads();
            for_candidates(level, [&](uint32_t key, int32_t pos) { atomicAdd(&h[refine_digit(level, key, pos)], 1u); });
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
        SK_STAMP(2);

        // ---- ascending emit through an LDS bitmap, kBitmapTokens tokens per pass
        uint32_t written = 0;
        for (int base = 0; base < seq; base += kBitmapTokens) {
            for (int i = tid; i < kBitmapWords; i += kTopkThreads) h[i] = 0;
            __syncthreads();
            SK_STAMP(5);
#pragma unroll
            for (int j = 0; j < PRE; ++j) {       // slots filled by the sweep: already in registers
                const uint32_t i = tid + j * kTopkThreads;
                const int32_t p = ps[j] - base;
                if (i < above && p >= 0 && p < kBitmapTokens) atomicOr(&h[p >> 5], 1u << (p & 31));
            }
            for (uint32_t i = tid; i < k_eff; i += kTopkThreads) {
                if (i < above && i < (uint32_t)(PRE * kTopkThreads)) continue;
                const int32_t p = staged[i] - base;
                if (p >= 0 && p < kBitmapTokens) atomicOr(&h[p >> 5], 1u << (p & 31));
            }
            __syncthreads();
            SK_STAMP(6);
            constexpr int PER = kBitmapWords / kTopkThreads;
            uint32_t c = 0;
#pragma unroll
            for (int i = 0; i < PER; ++i) c += __popc(h[tid * PER + i]);
            uint32_t total;
            uint32_t at = written + block_excl_scan(c, &total, tmp);
            SK_STAMP(7);
            for (int i = 0; i < PER; ++i) {
                uint32_t w = h[tid * PER + i];
                while (w) {
                    int bit = __ffs(w) - 1;
                    w &= w - 1;
                    if (at < (uint32_t)a.max_k) out[at] = base + (tid * PER + i) * 32 + bit;
                    ++at;
                }
            }
            SK_STAMP(8);
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
                int batch, int32_t *idx, int32_t *n_selected, bool have_hist, hipStream_t st) {
    const Geometry &g = ctx->g;
    TopkArgs a;
    a.scores = scores; a.seq_len = seq_len; a.k = k; a.idx = idx; a.n_selected = n_selected;
    a.hist = ctx->hist; a.hist2 = ctx->hist + (int64_t)g.max_batch * g.Hkv * kHistBins; a.counters = ctx->counters; a.cand_key = ctx->cand_key; a.cand_idx = ctx->cand_idx; a.staged = ctx->staged;
    a.Hkv = g.Hkv; a.max_n = g.max_n; a.max_k = g.max_k;
    const int BH = batch * g.Hkv;
    dim3 grid((g.max_n + kSlice - 1) / kSlice, BH);
    if (!have_hist) hipLaunchKernelGGL(topk_hist_kernel, grid, dim3(kTopkThreads), 0, st, a);
    hipLaunchKernelGGL(topk_hist2_kernel, grid, dim3(kTopkThreads), 0, st, a);
    hipLaunchKernelGGL(topk_filter_kernel, grid, dim3(kTopkThreads), 0, st, a);
    hipLaunchKernelGGL(topk_resolve_kernel, dim3(BH), dim3(kTopkThreads), kBitmapWords * 4, st, a);
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

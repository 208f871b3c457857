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
#include "topk_device.h"

namespace sk {

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
    // this workgroup's region of the selected list: empty unless the sweep below says otherwise
    uint32_t *selcnt = a.sel_cnt + (int64_t)bh * a.n_regions + blockIdx.x;
    if (tid == 0) *selcnt = 0u;
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
    int32_t *region = a.sel_regions + ((int64_t)bh * a.n_regions + blockIdx.x) * kSlice;

    // Scores above the threshold bin go to this workgroup's own region of the selected list, in
    // position order (no reservation across workgroups: what a region holds depends on the
    // scores alone); candidates of the threshold bin, a handful, are appended to one list with
    // an atomic per workgroup - they are ranked as a set, so their order does not matter.
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
        const uint32_t ncand = total >> 16;
        *selcnt = total & 0xffffu;
        s_base[1] = ncand ? atomicAdd(&cnt[1], ncand) : 0u;
    }
    __syncthreads();
    uint32_t at_sel = before & 0xffffu, at_cand = s_base[1] + (before >> 16);
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        if (flags & (1u << j)) region[at_sel++] = i + j;
        if (flags & (1u << (16 + j))) {
            ckey[at_cand] = keys[j];
            cidx[at_cand] = i + j;
            ++at_cand;
        }
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_resolve_kernel(TopkArgs a) {
    extern __shared__ uint32_t resolve_lds[];
    topk_resolve_body(a, blockIdx.x, resolve_lds);
}

// Everything up to the sweep: the threshold and the two unordered lists (selected outright,
// candidates in the threshold bin).  The fused decode step continues from those lists.
int launch_topk_sweep(socket_ctx *ctx, const float *scores, const int32_t *seq_len, const int32_t *k,
                      int batch, int32_t *idx, int32_t *n_selected, int hist_mode, hipStream_t st) {
    const Geometry &g = ctx->g;
    const TopkArgs a = topk_args(ctx, scores, seq_len, k, idx, n_selected, hist_mode);
    dim3 grid((g.max_n + kSlice - 1) / kSlice, batch * g.Hkv);
    if (hist_mode == kHistAdaptive) {
        hipLaunchKernelGGL(topk_filter_kernel<true>, grid, dim3(kTopkThreads), 0, st, a);
    } else {
        if (hist_mode == kHistNone) hipLaunchKernelGGL(topk_hist_kernel, grid, dim3(kTopkThreads), 0, st, a);
        hipLaunchKernelGGL(topk_hist2_kernel, grid, dim3(kTopkThreads), 0, st, a);
        hipLaunchKernelGGL(topk_filter_kernel<false>, grid, dim3(kTopkThreads), 0, st, a);
    }
    return record_hip(ctx, hipGetLastError());
}

int launch_topk(socket_ctx *ctx, const float *scores, const int32_t *seq_len, const int32_t *k,
                int batch, int32_t *idx, int32_t *n_selected, int hist_mode, hipStream_t st) {
    int rc = launch_topk_sweep(ctx, scores, seq_len, k, batch, idx, n_selected, hist_mode, st);
    if (rc != SOCKET_OK) return rc;
    const TopkArgs a = topk_args(ctx, scores, seq_len, k, idx, n_selected, hist_mode);
    static_assert(kResolveLds <= 64 * 1024, "within the default dynamic LDS limit");
    hipLaunchKernelGGL(topk_resolve_kernel, dim3(ctx->g.Hkv * batch), dim3(kTopkThreads), kResolveLds, st, a);
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

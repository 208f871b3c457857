// C-ABI entry points of libsocket: parameter checks, scratch ownership, dispatch.
#include <new>

#include "socket_internal.h"

namespace sk {

static int pad_codes(int L) {
    if (L < 1 || L > 1024) return -1;
    if (L <= 16) return 16;
    if (L <= 32) return 32;
    if (L <= 64) return 64;
    return (L + 63) / 64 * 64;
}

int fill_geometry(const socket_params *p, Geometry *g) {
    if (!p || !g) return SOCKET_EINVAL;
    if (p->d != 64 && p->d != 128 && p->d != 256) return SOCKET_EINVAL;
    if (p->Hkv < 1 || p->Hq < 1 || p->Hq % p->Hkv) return SOCKET_EINVAL;
    int G = p->Hq / p->Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return SOCKET_EUNSUPPORTED;
    if (p->L < 1 || p->L > 1024 || p->P < 1 || p->P > 16) return SOCKET_EINVAL;
    if (p->kv_dtype != SOCKET_BF16 && p->kv_dtype != SOCKET_F32) return SOCKET_EINVAL;
    if (p->max_batch < 1 || p->max_n < 16 || p->max_n % 16) return SOCKET_EINVAL;
    if (p->max_k < 1 || p->max_k > p->max_n) return SOCKET_EINVAL;
    if (p->page_size < 0 || p->page_size % 16) return SOCKET_EINVAL;
    if (p->page_size > 0) {
        if (p->max_blocks_per_seq < 1 || p->num_blocks < 1) return SOCKET_EINVAL;
        if ((int64_t)p->max_blocks_per_seq * p->page_size < p->max_n) return SOCKET_EINVAL;
        // token / page is taken as a multiplication by ceil(2^32 / page): exact for every token
        // when the page size is a power of two, else as long as max_n * page < 2^32
        if ((p->page_size & (p->page_size - 1)) != 0 && (int64_t)p->max_n * p->page_size >= (int64_t)1 << 32)
            return SOCKET_EUNSUPPORTED;
    }
    // rows of the K / V / id tensors are numbered in 32 bits (2^31 rows of 64 bf16 elements would
    // already be 256 GiB of keys)
    const int64_t rows = p->page_size > 0 ? (int64_t)p->num_blocks * p->Hkv * p->page_size
                                          : (int64_t)p->max_batch * p->Hkv * (int64_t)p->max_n;
    if (rows >= (int64_t)1 << 31) return SOCKET_EINVAL;
    if ((int64_t)p->max_batch * p->Hkv * (int64_t)p->max_n >= (int64_t)1 << 31) return SOCKET_EINVAL;

    g->pf = pack_factor(p->L, p->P);
    g->Lu = p->L; g->Pu = p->P;
    g->mu = (float)((double)p->L / (double)(1 << p->P));
    const int L = p->L / g->pf, P = g->pf > 1 ? 8 : p->P;
    g->d = p->d; g->Hq = p->Hq; g->Hkv = p->Hkv; g->G = G; g->L = L; g->P = P;
    g->R = 1 << P;
    g->Lpad = pad_codes(L);
    g->S = g->Lpad >= 64 ? 4 : g->Lpad / 16;
    g->rounds = g->Lpad >= 64 ? g->Lpad / 64 : 1;
    g->cb = P <= 8 ? 1 : 2;
    g->page = p->page_size; g->max_blocks = p->max_blocks_per_seq; g->num_blocks = p->num_blocks;
    g->max_n = p->max_n; g->max_k = p->max_k; g->max_batch = p->max_batch;
    g->kv_dtype = p->kv_dtype;

    // Pick the bucket-probability layout that fits in LDS (a row is 64 floats = 256 B).
    const int64_t budget = 144 * 1024;
    int64_t direct = (int64_t)g->rounds * g->R * 256;
    g->Plo = (P + 1) / 2; g->Phi = P - g->Plo;
    g->Rlo = 1 << g->Plo; g->Rhi = 1 << g->Phi;
    g->GT = 0;
    int64_t factor = (int64_t)G * g->rounds * (g->Rlo + g->Rhi) * 256;
    if (P <= 8 && direct <= 128 * 1024) {
        g->mode = kDirect;
        g->table_rows = g->R;
        g->table_words = (int64_t)g->rounds * g->R * 64;
    } else if (P == 9 || P == 10) {
        // packed ids, one table per (table, bucket), scored group by group
        g->mode = kSplit;
        g->cb = 0;
        g->GT = g->Lpad < 32 ? g->Lpad : 32;
        g->S = g->GT / 16;
        g->rounds = g->Lpad / g->GT;
        g->table_rows = g->R;
        g->table_words = (int64_t)g->rounds * g->R * g->GT;
    } else if (g->pf == 1 && P >= 2 && factor <= budget) {
        g->mode = kFactor;
        g->table_rows = g->Rlo + g->Rhi;
        g->table_words = (int64_t)G * g->rounds * g->table_rows * 64;
    } else {
        return SOCKET_EUNSUPPORTED;
    }
    // split-K of the sparse decode: about 64 selected rows per workgroup, at most 64 splits
    int ns = (p->max_k + kDecodeChunk - 1) / kDecodeChunk;
    g->n_split = ns < 1 ? 1 : (ns > 64 ? 64 : ns);
    // The fused step's attention is cut by regions of the select's sweep (kSlice positions each):
    // ssr workgroups share a region when a region is expected to hold more than ~40 selected
    // tokens (as long as the whole batch's workgroups stay resident together: about five of
    // them per compute unit), rpg regions share a workgroup when there are more regions than
    // splits.
    g->n_regions = (p->max_n + kSlice - 1) / kSlice;
    if (g->n_regions > kMaxRegions) return SOCKET_EUNSUPPORTED;
    g->ssr = 1;
    g->rpg = (g->n_regions + kMaxSplits - 1) / kMaxSplits;
    while (g->rpg == 1 && g->n_regions * g->ssr * 2 <= kMaxSplits && g->ssr < 16 &&
           (int64_t)p->max_k > (int64_t)40 * g->n_regions * g->ssr &&
           (int64_t)g->n_regions * g->ssr * 2 * p->Hkv * p->max_batch <= 1280)
        g->ssr *= 2;
    g->n_split_sweep = g->rpg > 1 ? (g->n_regions + g->rpg - 1) / g->rpg : g->n_regions * g->ssr;
    return SOCKET_OK;
}

int record_hip(socket_ctx *ctx, hipError_t e) {
    if (e == hipSuccess) return SOCKET_OK;
    if (ctx) ctx->last_hip_error = (int)e;
    return SOCKET_EHIP;
}

}  // namespace sk

using namespace sk;

extern "C" {

int socket_validate_params(const socket_params *p) {
    Geometry g;
    return fill_geometry(p, &g);
}

int32_t socket_codes_per_token(int32_t L) { return pad_codes(L); }

int32_t socket_code_position(int32_t L, int32_t l, int32_t t) {
    int Lpad = pad_codes(L);
    if (Lpad < 0 || l < 0 || l >= Lpad || t < 0) return -1;
    int S = Lpad >= 64 ? 4 : Lpad / 16;
    int c = Lpad >= 64 ? l / 64 : 0;
    int lp = l - 64 * c;
    int sub = lp % S, m = lp / S;
    int s = ((m - t) % 16 + 16) % 16;
    return 64 * c + sub * 16 + s;
}

static bool packed_ids(int P) { return P == 9 || P == 10; }

int64_t socket_codes_bytes(int32_t L, int32_t P, int64_t tokens) {
    if (L < 1 || P < 1 || P > 16 || tokens < 0 || tokens % 16) return -1;
    const int Lpad = pad_codes(L / pack_factor(L, P));
    if (Lpad < 0) return -1;
    if (packed_ids(P)) return tokens / 16 * packed_tile_bytes(Lpad);
    return tokens * Lpad * (P <= 8 ? 1 : 2);
}

int socket_code_location(int32_t L, int32_t P, int32_t l, int32_t t, int64_t *lo_byte,
                         int64_t *hi_byte, int32_t *hi_shift) {
    if (L < 1 || P < 1 || P > 16) return SOCKET_EINVAL;
    const int pf = pack_factor(L, P);
    const int Lpad = pad_codes(L / pf);
    if (Lpad < 0 || l < 0 || l >= Lpad * pf || t < 0 || !lo_byte || !hi_byte || !hi_shift)
        return SOCKET_EINVAL;
    if (pf > 1) {
        // 8/P ids to a byte: the byte is the id of 8-plane table l / pf
        *lo_byte = (int64_t)t * Lpad + socket_code_position(L / pf, l / pf, t);
        *hi_byte = -1;
        *hi_shift = P * (l % pf);
        return SOCKET_OK;
    }
    if (packed_ids(P)) {
        const int GT = Lpad < 32 ? Lpad : 32, S = GT / 16;
        const int grp = l / GT, j = packed_pos(l % GT, t, S);
        const int sub = j >> 4, bit = 10 * (j & 15);           // bit of the 160-bit string where the id starts
        const int b0 = bit >> 3, b1 = b0 + 1;                   // the two bytes of the string that hold it
        *lo_byte = packed_word(t, grp, sub, b0 >> 2, Lpad, GT) + (b0 & 3);
        *hi_byte = packed_word(t, grp, sub, b1 >> 2, Lpad, GT) + (b1 & 3);
        *hi_shift = bit & 7;
        return SOCKET_OK;
    }
    const int cb = P <= 8 ? 1 : 2;
    *lo_byte = ((int64_t)t * Lpad + socket_code_position(L, l, t)) * cb;
    *hi_byte = cb == 2 ? *lo_byte + 1 : -1;
    *hi_shift = 0;
    return SOCKET_OK;
}

int socket_create(socket_ctx **out, const socket_params *p) {
    if (!out || !p) return SOCKET_EINVAL;
    *out = nullptr;
    Geometry g;
    int rc = fill_geometry(p, &g);
    if (rc != SOCKET_OK) return rc;
    socket_ctx *ctx = new (std::nothrow) socket_ctx();
    if (!ctx) return SOCKET_ENOMEM;
    ctx->p = *p;
    ctx->g = g;
    ctx->last_hip_error = 0;
    ctx->pending_hist = kHistNone;
    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) {
        delete ctx;
        return SOCKET_EHIP;
    }
    const int64_t BH = (int64_t)g.max_batch * g.Hkv;
    const int64_t sz_tables = BH * g.table_words * 4;
    const int64_t sz_tstats = BH * g.Lpad * 3 * 4;
    const int64_t sz_sub = g.pf > 1 ? BH * g.Lu * (1 << g.Pu) * 4 : 0;   // shared-byte ids: the small tables, for the read-back
    // fast prefill hash: bf16 keys, one-byte ids of 8 or 4 planes, W slab of a chunk of up to 64 tables fits LDS
    const bool fast8 = g.kv_dtype == SOCKET_BF16 && (g.P == 8 || g.P == 4) && g.cb == 1 && g.mode == kDirect && g.d <= 128;
    // the same for 10-plane tables with packed ids (groups of 32 tables, or one group of 16)
    const bool fast10 = g.kv_dtype == SOCKET_BF16 && g.P == 10 && g.mode == kSplit && (g.GT == 32 || g.GT == 16) && g.d <= 128;
    const bool fast_hash = fast8 || fast10;
    const int64_t sz_wfrag = fast8 ? (int64_t)g.Hkv * ((g.L + 63) / 64) * g.d * 1024
                             : fast10 ? (int64_t)g.Hkv * (g.Lpad / g.GT) * (5 * g.GT / 16) * (g.d / 16) * 1024 : 0;
    const int64_t sz_hist = 2 * BH * kHistBins * 4;   // first- and second-digit histograms
    const int64_t sz_cnt = BH * (kCounterStride + kThrStride) * 4;
    const int64_t sz_cand = BH * g.max_n * 4;
    const int64_t sz_staged = BH * g.max_k * 4;
    const int64_t sz_regions = BH * g.n_regions * kSlice * 4, sz_selcnt = BH * g.n_regions * 4;
    const int64_t sz_seq = (int64_t)g.max_batch * 4;
    const int64_t sz_part = (int64_t)g.max_batch * g.Hq * kMaxSplits * (g.d + 2) * 4;
    ctx->scratch_bytes = sz_wfrag + sz_tables + sz_tstats + sz_sub + sz_hist + sz_cnt + 2 * sz_cand + sz_staged + sz_regions + sz_selcnt + sz_part + sz_seq;
    bool ok = score_prepare(g) == SOCKET_OK &&
              hipMalloc((void **)&ctx->tables, sz_tables) == hipSuccess &&
              hipMalloc((void **)&ctx->tstats, sz_tstats) == hipSuccess &&
              (sz_sub == 0 || hipMalloc((void **)&ctx->subprobs, sz_sub) == hipSuccess) &&
              (!fast_hash || (hipMalloc(&ctx->wfrag, sz_wfrag) == hipSuccess && hash_prepare(g.d) == SOCKET_OK)) &&
              hipMalloc((void **)&ctx->hist, sz_hist) == hipSuccess &&
              hipMalloc((void **)&ctx->counters, sz_cnt) == hipSuccess &&
              hipMalloc((void **)&ctx->cand_key, sz_cand) == hipSuccess &&
              hipMalloc((void **)&ctx->cand_idx, sz_cand) == hipSuccess &&
              hipMalloc((void **)&ctx->staged, sz_staged) == hipSuccess &&
              hipMalloc((void **)&ctx->sel_regions, sz_regions) == hipSuccess &&
              hipMalloc((void **)&ctx->sel_cnt, sz_selcnt) == hipSuccess &&
              hipMalloc((void **)&ctx->partials, sz_part) == hipSuccess &&
              hipMalloc((void **)&ctx->seq_scratch, sz_seq) == hipSuccess;
    // Histograms and counters must start at zero; the kernels that use them leave them
    // at zero again, so this is the only clear (and it is outside any graph capture).
    ok = ok && hipMemset(ctx->hist, 0, sz_hist) == hipSuccess &&
         hipMemset(ctx->tstats, 0, sz_tstats) == hipSuccess &&
         hipMemset(ctx->counters, 0, sz_cnt) == hipSuccess &&
         hipMemset(ctx->sel_cnt, 0, sz_selcnt) == hipSuccess &&
         hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        socket_destroy(ctx);
        return SOCKET_ENOMEM;
    }
    *out = ctx;
    return SOCKET_OK;
}

int socket_destroy(socket_ctx *ctx) {
    if (!ctx) return SOCKET_EINVAL;
    void *bufs[] = {ctx->tables, ctx->tstats, ctx->subprobs, ctx->wfrag, ctx->hist, ctx->counters, ctx->cand_key, ctx->cand_idx, ctx->staged, ctx->sel_regions, ctx->sel_cnt, ctx->partials, ctx->seq_scratch};
    for (void *b : bufs)
        if (b) (void)hipFree(b);
    delete ctx;
    return SOCKET_OK;
}

int64_t socket_scratch_bytes(const socket_ctx *ctx) { return ctx ? ctx->scratch_bytes : 0; }

static bool batch_ok(const socket_ctx *ctx, int batch) {
    return batch >= 1 && batch <= ctx->g.max_batch;
}

static bool paging_ok(const socket_ctx *ctx, const int32_t *block_table) {
    return (ctx->g.page > 0) == (block_table != nullptr);
}

int socket_hash_keys(socket_ctx *ctx, const void *K, const void *proj, const int32_t *block_table,
                     const int32_t *row_begin, const int32_t *row_count, int32_t batch,
                     int32_t max_rows, void *codes, void *stream) {
    if (!ctx || !K || !proj || !row_begin || !row_count || !codes) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    if (max_rows < 0 || max_rows > ctx->g.max_n) return SOCKET_EINVAL;
    if (max_rows == 0) return SOCKET_OK;
    return launch_hash_keys(ctx, K, proj, block_table, row_begin, row_count, batch, max_rows, codes,
                            (hipStream_t)stream);
}

int socket_value_norms(socket_ctx *ctx, const void *V, const int32_t *block_table,
                       const int32_t *row_begin, const int32_t *row_count, int32_t batch,
                       int32_t max_rows, float *vnorm, void *stream) {
    if (!ctx || !V || !row_begin || !row_count || !vnorm) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    if (max_rows < 0 || max_rows > ctx->g.max_n) return SOCKET_EINVAL;
    if (max_rows == 0) return SOCKET_OK;
    return launch_value_norms(ctx, V, block_table, row_begin, row_count, batch, max_rows, vnorm,
                              (hipStream_t)stream);
}

int socket_set_forced_tokens(socket_ctx *ctx, int32_t n_sink, int32_t n_window) {
    if (!ctx || n_sink < 0 || n_window < 0) return SOCKET_EINVAL;
    ctx->n_sink = n_sink;
    ctx->n_window = n_window;
    return SOCKET_OK;
}

int socket_score(socket_ctx *ctx, const void *q, const void *codes, const void *proj, float tau,
                 const float *vnorm, const int32_t *block_table, const int32_t *seq_len,
                 int32_t batch, float *scores, void *stream) {
    if (!ctx || !q || !codes || !proj || !seq_len || !scores) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    if (!(tau > 0.0f) || !(tau < 3.0e38f)) return SOCKET_EINVAL;
    int rc = launch_soft_hash(ctx, q, proj, tau, batch, (hipStream_t)stream);
    if (rc != SOCKET_OK) return rc;
    return launch_score_keys(ctx, codes, vnorm, block_table, seq_len, batch, scores, false, nullptr, (hipStream_t)stream);
}

int socket_soft_hash(socket_ctx *ctx, const void *q, const void *proj, float tau, int32_t batch,
                     void *stream) {
    if (!ctx || !q || !proj) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch)) return SOCKET_EINVAL;
    if (!(tau > 0.0f) || !(tau < 3.0e38f)) return SOCKET_EINVAL;
    return launch_soft_hash(ctx, q, proj, tau, batch, (hipStream_t)stream);
}

int socket_hard_hash(socket_ctx *ctx, const void *q, const void *proj, int32_t batch, void *stream) {
    if (!ctx || !q || !proj) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch)) return SOCKET_EINVAL;
    return launch_hard_hash(ctx, q, proj, batch, (hipStream_t)stream);
}

int socket_score_keys(socket_ctx *ctx, const void *codes, const float *vnorm,
                      const int32_t *block_table, const int32_t *seq_len, int32_t batch,
                      float *scores, void *stream) {
    if (!ctx || !codes || !seq_len || !scores) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    return launch_score_keys(ctx, codes, vnorm, block_table, seq_len, batch, scores, false, nullptr, (hipStream_t)stream);
}

int socket_score_keys_binned(socket_ctx *ctx, const void *codes, const float *vnorm,
                             const int32_t *block_table, const int32_t *seq_len, int32_t batch,
                             float *scores, void *stream) {
    if (!ctx || !codes || !seq_len || !scores) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    int mode = sk::kHistNone;
    const int rc = launch_score_keys(ctx, codes, vnorm, block_table, seq_len, batch, scores, true, &mode, (hipStream_t)stream);
    if (rc == SOCKET_OK) ctx->pending_hist = mode;
    return rc;
}

int socket_topk_select_binned(socket_ctx *ctx, const float *scores, const int32_t *seq_len,
                              const int32_t *k, int32_t batch, int32_t *idx, int32_t *n_selected,
                              void *stream) {
    if (!ctx || !scores || !seq_len || !k || !idx || !n_selected) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch)) return SOCKET_EINVAL;
    if (ctx->pending_hist == sk::kHistNone) return SOCKET_EINVAL;    // no socket_score_keys_binned before it
    const int mode = ctx->pending_hist;
    ctx->pending_hist = sk::kHistNone;
    return launch_topk(ctx, scores, seq_len, k, batch, idx, n_selected, mode, (hipStream_t)stream);
}

int socket_reset(socket_ctx *ctx, void *stream) {
    if (!ctx) return SOCKET_EINVAL;
    return launch_reset(ctx, (hipStream_t)stream);
}

int socket_bucket_probs(socket_ctx *ctx, int32_t batch, float *probs, void *stream) {
    if (!ctx || !probs) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch)) return SOCKET_EINVAL;
    return launch_bucket_probs(ctx, batch, probs, (hipStream_t)stream);
}

int socket_probe_stream_read(const void *buf, int64_t bytes, uint32_t *sink, void *stream) {
    if (!buf || !sink || bytes < 16 || bytes % 16) return SOCKET_EINVAL;
    return launch_stream_read(buf, bytes, sink, (hipStream_t)stream);
}

int socket_topk_select(socket_ctx *ctx, const float *scores, const int32_t *seq_len,
                       const int32_t *k, int32_t batch, int32_t *idx, int32_t *n_selected,
                       void *stream) {
    if (!ctx || !scores || !seq_len || !k || !idx || !n_selected) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch)) return SOCKET_EINVAL;
    return launch_topk(ctx, scores, seq_len, k, batch, idx, n_selected, sk::kHistNone, (hipStream_t)stream);
}

int socket_dense_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const int32_t *block_table, const int32_t *seq_len, int32_t batch,
                        float scale, int32_t out_dtype, void *out, void *stream) {
    if (!ctx || !q || !K || !V || !seq_len || !out) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    if (out_dtype != SOCKET_F32 && out_dtype != SOCKET_BF16) return SOCKET_EINVAL;
    return launch_dense_decode(ctx, q, K, V, block_table, seq_len, batch, scale, out_dtype, out,
                               (hipStream_t)stream);
}

int socket_decode_step(socket_ctx *ctx, const void *q, const void *K, const void *V, void *codes,
                       const void *proj, float tau, const float *vnorm, const int32_t *block_table,
                       const int32_t *pos, const int32_t *k, int32_t batch, float scale,
                       float *scores, int32_t *idx, int32_t *n_selected, int32_t out_dtype,
                       void *out, void *stream) {
    if (!ctx || !q || !K || !V || !codes || !proj || !pos || !k || !scores || !idx || !n_selected || !out)
        return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    if (!(tau > 0.0f) || !(tau < 3.0e38f)) return SOCKET_EINVAL;
    if (out_dtype != SOCKET_BF16 && out_dtype != SOCKET_F32) return SOCKET_EINVAL;
    if (!(scale == scale) || scale > 3.0e38f || scale < -3.0e38f) return SOCKET_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    int32_t *len = ctx->seq_scratch;
    // 1. hash the appended key and soft-hash the queries (one launch); len = pos + 1
    int rc = launch_project(ctx, q, proj, tau, K, codes, block_table, pos, nullptr, len, batch, st, vnorm);
    if (rc != SOCKET_OK) return rc;
    // 2. score every key; the leading-digit histogram of the scores comes out of the same pass
    int hist_mode = sk::kHistNone;
    rc = launch_score_keys(ctx, codes, vnorm, block_table, len, batch, scores, true, &hist_mode, st);
    if (rc != SOCKET_OK) return rc;
    // 3. select, 4. attend
    //    (the attention starts from the regions the sweep leaves; the index row is ordered beside the merge)
    rc = launch_topk_sweep(ctx, scores, len, k, batch, idx, n_selected, hist_mode, st);
    if (rc != SOCKET_OK) return rc;
    return launch_sweep_decode(ctx, q, K, V, scores, len, k, idx, n_selected, hist_mode, block_table,
                               batch, scale, out_dtype, out, st);
}

int socket_sparse_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                         const int32_t *idx, const int32_t *n_selected,
                         const int32_t *block_table, int32_t batch, float scale, int32_t out_dtype,
                         void *out, void *stream) {
    if (!ctx || !q || !K || !V || !idx || !n_selected || !out) return SOCKET_EINVAL;
    if (!batch_ok(ctx, batch) || !paging_ok(ctx, block_table)) return SOCKET_EINVAL;
    if (out_dtype != SOCKET_BF16 && out_dtype != SOCKET_F32) return SOCKET_EINVAL;
    if (!(scale == scale) || scale > 3.0e38f || scale < -3.0e38f) return SOCKET_EINVAL;
    return launch_sparse_decode(ctx, q, K, V, idx, n_selected, block_table, batch, scale, out_dtype,
                                out, (hipStream_t)stream);
}

int socket_sparse_decode_noalloc(const socket_params *p, const void *q, const void *K, const void *V,
                                 const int32_t *idx, const int32_t *n_selected,
                                 const int32_t *block_table, int32_t batch, float scale,
                                 int32_t out_dtype, void *out, void *stream, int32_t *hip_error) {
    if (hip_error) *hip_error = 0;
    if (!p || !q || !K || !V || !idx || !n_selected || !out) return SOCKET_EINVAL;
    if (out_dtype != SOCKET_BF16 && out_dtype != SOCKET_F32) return SOCKET_EINVAL;
    if (!(scale == scale) || scale > 3.0e38f || scale < -3.0e38f) return SOCKET_EINVAL;
    int hip = 0;
    const int rc = sparse_decode_noalloc(p, q, K, V, idx, n_selected, block_table, batch, scale, out_dtype, out,
                                         (hipStream_t)stream, &hip);
    if (hip_error) *hip_error = hip;
    return rc;
}

const char *socket_strerror(int code) {
    switch (code) {
        case SOCKET_OK: return "ok";
        case SOCKET_EINVAL: return "invalid argument";
        case SOCKET_EUNSUPPORTED: return "unsupported configuration";
        case SOCKET_ENOMEM: return "scratch allocation failed";
        case SOCKET_EHIP: return "HIP runtime error";
        case SOCKET_ELIMIT: return "request exceeds the fixed scratch of the no-allocation entry point";
        default: return "unknown error";
    }
}

int socket_last_hip_error(const socket_ctx *ctx) { return ctx ? ctx->last_hip_error : 0; }

struct socket_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

int socket_graph_begin(void *stream) {
    if (!stream) return SOCKET_EINVAL;  // the default stream cannot be captured
    hipError_t e = hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal);
    return e == hipSuccess ? SOCKET_OK : SOCKET_EHIP;
}

int socket_graph_end(void *stream, socket_graph **out) {
    if (!stream || !out) return SOCKET_EINVAL;
    *out = nullptr;
    hipGraph_t graph = nullptr;
    if (hipStreamEndCapture((hipStream_t)stream, &graph) != hipSuccess || !graph) return SOCKET_EHIP;
    hipGraphExec_t exec = nullptr;
    if (hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return SOCKET_EHIP;
    }
    socket_graph *g = new (std::nothrow) socket_graph{graph, exec};
    if (!g) {
        (void)hipGraphExecDestroy(exec);
        (void)hipGraphDestroy(graph);
        return SOCKET_ENOMEM;
    }
    *out = g;
    return SOCKET_OK;
}

int socket_graph_launch(socket_graph *g, void *stream) {
    if (!g) return SOCKET_EINVAL;
    return hipGraphLaunch(g->exec, (hipStream_t)stream) == hipSuccess ? SOCKET_OK : SOCKET_EHIP;
}

int socket_graph_destroy(socket_graph *g) {
    if (!g) return SOCKET_EINVAL;
    (void)hipGraphExecDestroy(g->exec);
    (void)hipGraphDestroy(g->graph);
    delete g;
    return SOCKET_OK;
}

}  // extern "C"

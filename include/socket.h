/*
 * libsocket -- the decode-time hot path of SOCKET (soft-collision LSH sparse
 * attention) for AMD MI355X (gfx950).  C ABI; every kernel behind it is
 * hand-written HIP.
 *
 * Call order for one attention layer (the paper's three stages):
 *   prefill : socket_hash_keys over all cached keys            (Alg. 1)
 *   decode  : socket_hash_keys over the one appended key       (Alg. 1)
 *             socket_score        soft-hash q, score every key (Alg. 2 + Alg. 5 / Eq. 3)
 *             socket_topk_select  keep the k best tokens       (Alg. 3, TopK step)
 *             socket_sparse_decode  exact attention on them    (Eq. 2; Eq. 1 when all are kept)
 *
 * General rules
 *   - Every tensor argument is a caller-owned DEVICE pointer.  The library never
 *     allocates, frees or keeps one.  `socket_ctx` owns only its own scratch.
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream), does no host synchronisation and records no
 *     memset node, so a sequence of calls may be captured into a HIP graph.
 *   - One ctx serves one stream at a time: calls that share a ctx and overlap
 *     in time race on its scratch.
 *   - Every call returns 0 or a negative SOCKET_E* code; nothing throws.
 *     Arguments are checked on the host before any launch.
 *   - Per-sequence integers (lengths, k, row ranges) live in device memory, so a
 *     captured graph can be replayed with new values.
 *
 * Shapes: B sequences, Hq query heads, Hkv key/value heads (Hq = G * Hkv),
 * head dimension d, L hash tables of P hyperplanes (R = 2^P buckets per table).
 *
 * Layouts
 *   q        [B, Hq, d]                              element type = kv_dtype
 *   K, V     contiguous: [B, Hkv, max_n, d]          element type = kv_dtype
 *            paged:      [num_blocks, Hkv, page_size, d], with
 *            block_table [B, max_blocks_per_seq] int32; token t of sequence b is
 *            row t % page_size of block block_table[b][t / page_size]
 *   proj     [Hkv, d, L*P]  element type = kv_dtype; column l*P+i is hyperplane i
 *            of table l (the paper's W^(l), row i)
 *   codes    same token layout as K with d replaced by Lpad:
 *            [B, Hkv, max_n, Lpad] or [num_blocks, Hkv, page_size, Lpad];
 *            element uint8 when P <= 8, uint16 when P >= 11 (P = 9, 10: packed, below).
 *            Lpad = 16, 32 or 64 (the smallest that holds L) when L <= 64, else L
 *            rounded up to a multiple of 64.  The L bucket ids of token t are
 *            stored in a rotated order chosen so that the scoring kernel's table
 *            look-ups are free of LDS bank conflicts: with S = min(Lpad,64)/16 and
 *            l = 64*c + l' (l' < 64), the id of table l sits at position
 *                64*c + (l' % S)*16 + ((l' / S - t) mod 16).
 *            socket_code_position() returns that position.  Positions that map to
 *            tables >= L hold 0.
 *            P = 9 and P = 10 use a packed form instead, 10 bits per id (the paper counts
 *            600 bits per token for (P, L) = (10, 60); here 640 with Lpad = 64): tokens
 *            are stored in tiles of 16, [.., Hkv, max_n/16, 20*Lpad] bytes (paged:
 *            [num_blocks, Hkv, page_size/16, 20*Lpad]).  With GT = min(Lpad, 32) and
 *            S = GT/16 a tile holds Lpad/GT group blocks of 20*GT bytes, group c covering
 *            tables c*GT .. c*GT+GT-1.  The ids of a token's group form S strings of 160
 *            bits (little-endian), string `sub` holding, in bits [10 s, 10 s + 10), the id
 *            of table c*GT + sub + S*((t + s) mod 16), s = 0..15 (the rotation above).
 *            A block keeps bytes 0..15 of the strings in 16 rows (token t mod 16) of GT
 *            bytes, string `sub` at byte 16*sub, followed by 16 rows of GT/4 bytes with
 *            bytes 16..19 of the strings, string `sub` at byte 4*sub.
 *            P = 1, 2 and 4 keep f = 8/P ids to a byte when L is a multiple of f and L/f is
 *            32..128 (else a byte per id, as above): the byte for tables f*m .. f*m+f-1, table
 *            f*m+j in bits [P*j, P*j+P), is the 8-plane id of columns 8m .. 8m+7 of proj, and
 *            the code row is that of L/f eight-plane tables (Lpad and positions above with
 *            L/f for L and m for l).  The look-up table of such a byte holds the sum of its f
 *            tables' probabilities, so Eq. 3 stays one look-up per byte.
 *            socket_codes_bytes() and socket_code_location() describe all four forms.
 *   bucket id: bit i is 1 when hyperplane i gives a projection >= 0.
 *   scores   [B, Hkv, max_n] float32, logical token order; -inf for t >= seq_len
 *   idx      [B, Hkv, max_k] int32 logical token positions in ascending order,
 *            unused tail = -1;  n_selected [B, Hkv] int32
 *   out      [B, Hq, d] float32 or bf16
 */
#ifndef SOCKET_H
#define SOCKET_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types */
#define SOCKET_BF16 0
#define SOCKET_F32 1

/* error codes */
#define SOCKET_OK 0
#define SOCKET_EINVAL (-1)       /* null pointer, size out of range, inconsistent sizes */
#define SOCKET_EUNSUPPORTED (-2) /* a valid request this build has no kernel for */
#define SOCKET_ENOMEM (-3)       /* scratch allocation failed */
#define SOCKET_EHIP (-4)         /* a HIP call failed; see socket_last_hip_error */
#define SOCKET_ELIMIT (-5)       /* more than socket_sparse_decode_noalloc's fixed scratch can hold */

/* bytes of the fixed device array behind socket_sparse_decode_noalloc */
#define SOCKET_NOALLOC_SCRATCH_BYTES (4 * 1024 * 1024)

typedef struct socket_ctx socket_ctx;

typedef struct socket_params {
    int32_t d;         /* head dimension: 64, 128 or 256 */
    int32_t Hq;        /* query heads; Hq/Hkv must be 1, 2, 4 or 8 */
    int32_t Hkv;       /* key/value heads */
    int32_t L;         /* hash tables, 1..1024 */
    int32_t P;         /* hyperplanes per table, 1..16 */
    int32_t kv_dtype;  /* SOCKET_BF16 or SOCKET_F32: type of q, K, V and proj */
    int32_t max_batch; /* largest B any call will pass */
    int32_t max_n;     /* token capacity per sequence, a multiple of 16 */
    int32_t max_k;     /* largest k any call will select, <= max_n */
    int32_t page_size; /* 0 = contiguous K/V/codes; else tokens per block, a multiple of 16 */
    int32_t max_blocks_per_seq; /* paged only: columns of block_table */
    int32_t num_blocks;         /* paged only: blocks in the K/V/codes pools; a block_table
                                   entry outside [0, num_blocks) marks its tokens as absent */
} socket_params;

/* Host-only check of a parameter block; no GPU needed.  0 or SOCKET_EINVAL /
 * SOCKET_EUNSUPPORTED (for example a bucket-probability table that cannot fit in
 * the 160 KB of LDS). */
int socket_validate_params(const socket_params *p);

/* Padded codes-per-token (Lpad above) for L tables; -1 when L is out of range.  (Ids that
 * share bytes: call it with the number of bytes, L*P/8.) */
int32_t socket_codes_per_token(int32_t L);

/* Position of table l's bucket id inside token t's Lpad-long code row. */
int32_t socket_code_position(int32_t L, int32_t l, int32_t t);

/* Bytes of bucket-id storage for `tokens` tokens (a multiple of 16) of one (sequence or
 * block, KV head); -1 for arguments out of range. */
int64_t socket_codes_bytes(int32_t L, int32_t P, int64_t tokens);

/* Where the bucket id of table l (< Lpad) of token t is kept, as byte offsets from the start
 * of the (sequence or block, KV head) slab: with B0 the byte at *lo_byte and B1 the byte at
 * *hi_byte (taken as 0 when *hi_byte = -1, which is the case for P <= 8; l < L where ids
 * share bytes),
 *     id = ((B0 | B1 << 8) >> *hi_shift) & (2^P - 1).
 * Host-only; 0 or SOCKET_EINVAL. */
int socket_code_location(int32_t L, int32_t P, int32_t l, int32_t t, int64_t *lo_byte,
                         int64_t *hi_byte, int32_t *hi_shift);

/* Create / destroy a context on the current HIP device.  Creation allocates the
 * scratch (bucket-probability tables, radix histograms, candidate lists,
 * split-K partial results), sized from max_batch, max_n and max_k. */
int socket_create(socket_ctx **out, const socket_params *p);
int socket_destroy(socket_ctx *ctx);

/* Bytes of device scratch the context holds. */
int64_t socket_scratch_bytes(const socket_ctx *ctx);

/*
 * Alg. 1 (PrecomputeKeyHashes): bucket ids of cached keys.
 * For each sequence b < batch, tokens row_begin[b] .. row_begin[b]+row_count[b]-1
 * are hashed: h = sign(W^(l) k) per table, encoded as a bucket id, and written
 * into `codes`.  Prefill passes (0, n); a decode step passes (n, 1) for the
 * appended key.  `max_rows` (host) bounds every row_count[b] and sizes the
 * launch; rows beyond row_count[b] are not touched.
 * bf16 keys use bf16 MFMA with fp32 accumulation; fp32 keys use fp32 FMA.
 * row_begin, row_count: device int32 [batch].  block_table: device, paged only
 * (NULL otherwise).
 */
int socket_hash_keys(socket_ctx *ctx, const void *K, const void *proj,
                     const int32_t *block_table, const int32_t *row_begin,
                     const int32_t *row_count, int32_t batch, int32_t max_rows,
                     void *codes, void *stream);

/*
 * Value norms (Alg. 1 keeps ||v_j||_2 next to the bucket ids; Alg. 3 ranks tokens by
 * soft score x value norm).  For each sequence b < batch and every KV head,
 *     vnorm[b,h,t] = ||V[b,h,t,:]||_2      for t = row_begin[b] .. row_begin[b]+row_count[b]-1
 * (fp32 sum of squares).  Same row-range arguments as socket_hash_keys: prefill passes
 * (0, n), a decode step passes (n, 1) for the appended value row before it scores.
 * vnorm: device float32 [B, Hkv, max_n] in logical token order, for paged caches too.
 */
int socket_value_norms(socket_ctx *ctx, const void *V, const int32_t *block_table,
                       const int32_t *row_begin, const int32_t *row_count, int32_t batch,
                       int32_t max_rows, float *vnorm, void *stream);

/*
 * Sink and local-window tokens (Experiments section, evaluation protocol: a small number of
 * sink and local window tokens, e.g. 128, is always kept).  From this call on, every scoring
 * call on this context (socket_score, socket_score_keys, socket_decode_step) gives the score
 * +inf to the first n_sink and to the last n_window of a sequence's seq_len tokens, so that
 * the TopK step takes them first, in position order; they count towards k.  Tokens whose
 * block is absent stay -inf.  (0, 0), the state after socket_create, switches it off.
 * Host-side state: it takes effect for calls issued (or captured) after it returns.
 */
int socket_set_forced_tokens(socket_ctx *ctx, int32_t n_sink, int32_t n_window);

/*
 * Alg. 2 + Alg. 5 (SoftBucketProbs, SoftHashCollisionScores; Eq. 3, soft score).
 * Soft-hashes each query into its L x R bucket probabilities
 * (u = tanh(W q)/sqrt(d), softmax of u.c_r/tau over the R corners; evaluated in
 * fp64, stored as fp32), then gives every cached key j < seq_len[b] the score
 *     scores[b,h,j] = vnorm[b,h,j] * (1/G) * sum_{g in group(h)} sum_l p_g^(l)(codes[j,l])
 * and -inf to j >= seq_len[b].  G = 1 is the paper's single-query form; for
 * grouped-query attention the G queries sharing KV head h are averaged.
 * vnorm: device float32 [B, Hkv, max_n] (the paper's value-norm weights) or NULL
 * for 1.  seq_len: device int32 [batch].  tau > 0.
 */
int socket_score(socket_ctx *ctx, const void *q, const void *codes, const void *proj,
                 float tau, const float *vnorm, const int32_t *block_table,
                 const int32_t *seq_len, int32_t batch, float *scores, void *stream);

/*
 * The two halves of socket_score as separate calls, for callers that want to overlap or
 * time them: socket_soft_hash is Alg. 2 (SoftBucketProbs) and leaves the bucket
 * probabilities of every (sequence, KV head) in the context; socket_score_keys is Alg. 5
 * (SoftHashCollisionScores) and scores the keys against the probabilities the context
 * holds.  socket_score(...) == socket_soft_hash(...) followed by socket_score_keys(...).
 */
int socket_soft_hash(socket_ctx *ctx, const void *q, const void *proj, float tau, int32_t batch,
                     void *stream);
/*
 * Eq. 3, hard form (the traditional LSH scorer the paper compares against): instead of the
 * graded probabilities, the context's tables get 1 at the query's own bucket of every table
 * and 0 elsewhere (averaged over the G queries of a group), so that a following
 * socket_score_keys returns the collision count  #{ l : b_j^(l) = b_q^(l) }  (its group mean).
 * The query's bucket follows the same sign rule as socket_hash_keys, on the fp64 projection.
 */
int socket_hard_hash(socket_ctx *ctx, const void *q, const void *proj, int32_t batch, void *stream);

int socket_score_keys(socket_ctx *ctx, const void *codes, const float *vnorm,
                      const int32_t *block_table, const int32_t *seq_len, int32_t batch,
                      float *scores, void *stream);

/*
 * Alg. 5 and the TopK step of Alg. 3 as the fused decode step runs them, for callers that
 * issue the stages themselves: socket_score_keys_binned is socket_score_keys whose pass over
 * the keys also leaves, in the context, a histogram of the scores (bins sized from the bucket
 * probabilities the context holds, or leading digits of the score when those do not apply);
 * socket_topk_select_binned is socket_topk_select starting from that histogram instead of
 * making its own.  Same scores, same selection.  The two calls come in pairs on one context:
 * a socket_topk_select_binned without the other before it returns SOCKET_EINVAL.
 */
int socket_score_keys_binned(socket_ctx *ctx, const void *codes, const float *vnorm,
                             const int32_t *block_table, const int32_t *seq_len, int32_t batch,
                             float *scores, void *stream);
int socket_topk_select_binned(socket_ctx *ctx, const float *scores, const int32_t *seq_len,
                              const int32_t *k, int32_t batch, int32_t *idx, int32_t *n_selected,
                              void *stream);

/*
 * Clears the context's select scratch (histograms, counters, a pending
 * socket_score_keys_binned), with fill kernels on `stream`: for a caller that abandoned a chain
 * of calls half-way (an error, a socket_score_keys_binned never followed by its select).
 */
int socket_reset(socket_ctx *ctx, void *stream);

/*
 * Alg. 2 read-back: the bucket probabilities the context holds after socket_soft_hash,
 * socket_hard_hash, socket_score or socket_decode_step, as the scoring pass looks them up:
 *     probs[b, h, l, r] = (1/G) * sum_{g in group(h)} p_g^(l)(r | q)
 * device float32 [batch, Hkv, L, R], R = 2^P, whatever layout the context keeps them in
 * (ids that share bytes: a per-table copy the projection pass writes beside the summed tables).
 * For inspection and tests; not on the decode path.
 */
int socket_bucket_probs(socket_ctx *ctx, int32_t batch, float *probs, void *stream);

/*
 * Measurement aid, no part of the method: a kernel that reads `bytes` (a multiple of 16) of
 * device memory once and does nothing else, loading the way the scoring pass loads its ids.
 * What it reaches is the ceiling for any streaming kernel on this GPU, to be read beside the
 * published peak.  *sink: device word the kernel may write.
 */
int socket_probe_stream_read(const void *buf, int64_t bytes, uint32_t *sink, void *stream);

/*
 * Alg. 3, TopK step: for each (b, h) the min(k[b], #valid) tokens with the
 * largest scores, ties broken towards the smaller token position; -inf and NaN
 * scores are never selected.  The chosen positions are written in ascending
 * order, the rest of the max_k-long row is -1, and n_selected[b,h] is the count.
 * Exact (radix select on the fp32 bit patterns).
 * seq_len, k: device int32 [batch]; k[b] is clamped to max_k.
 */
int socket_topk_select(socket_ctx *ctx, const float *scores, const int32_t *seq_len,
                       const int32_t *k, int32_t batch, int32_t *idx,
                       int32_t *n_selected, void *stream);

/*
 * Eq. 2 (sparse attention over the selected set; Eq. 1 when the set is all
 * tokens): for each query head, alpha_i = softmax_{i in S}(scale * k_i.q) and
 * out = sum alpha_i v_i, with S = idx[b, h(kv head of that query head), :n_selected].
 * scale = 1 is the paper's definition (no 1/sqrt(d)).  Entries < 0 are skipped;
 * an empty set gives zeros; duplicate indices are a caller error.
 * out_dtype: SOCKET_F32 or SOCKET_BF16.
 */
int socket_sparse_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                         const int32_t *idx, const int32_t *n_selected,
                         const int32_t *block_table, int32_t batch, float scale,
                         int32_t out_dtype, void *out, void *stream);

/*
 * socket_sparse_decode for callers that cannot allocate device memory and hold no context:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and the same result as socket_sparse_decode, with the parameter block
 * in place of the context (d, Hq, Hkv, kv_dtype, max_batch, max_n, max_k and the paging fields
 * are used; L and P must be valid but play no part).  The split-K partial results go to a
 * fixed array of SOCKET_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until
 * the process ends; the call neither allocates nor frees, on the host side of HIP or on the
 * device.  A request that needs more, i.e.
 *     batch * Hq * min(64, ceil(max_k / 64)) * (d + 2) * 4  >  SOCKET_NOALLOC_SCRATCH_BYTES,
 * returns SOCKET_ELIMIT and launches nothing.  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU (different streams, or this call beside another of
 * itself) race on it; calls on one stream do not.  Nothing in the array has to be cleared
 * between calls.  *hip_error (may be NULL) receives the HIP code when SOCKET_EHIP is returned.
 */
int socket_sparse_decode_noalloc(const socket_params *p, const void *q, const void *K, const void *V,
                                 const int32_t *idx, const int32_t *n_selected,
                                 const int32_t *block_table, int32_t batch, float scale,
                                 int32_t out_dtype, void *out, void *stream, int32_t *hip_error);

/*
 * Eq. 1 (dense softmax attention over every token t < seq_len[b]), with the same split-K
 * kernels as socket_sparse_decode: the reference the sparse path is compared against on the
 * same GPU (the paper's throughput figures are relative to dense decoding).  An empty
 * sequence gives zeros.  seq_len: device int32 [batch].
 */
int socket_dense_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const int32_t *block_table, const int32_t *seq_len, int32_t batch,
                        float scale, int32_t out_dtype, void *out, void *stream);

/*
 * One decode step for one attention layer, fused: the caller has already written the new
 * key/value rows at position pos[b] of K and V.  Equivalent to
 *     socket_hash_keys(rows pos[b] .. pos[b])            (Alg. 1 on the appended key)
 *     socket_score with seq_len = pos + 1                (Alg. 2 + Alg. 5)
 *     socket_topk_select with seq_len = pos + 1          (Alg. 3, TopK)
 *     socket_sparse_decode                               (Eq. 2)
 * in five kernels instead of nine: the appended key's hash shares a launch with the queries'
 * soft hash, the scoring pass also produces the histogram that the selection starts from, the
 * attention starts from the lists the selection's sweep leaves (one region per workgroup of the
 * sweep, in position order), and the index row is put in order beside the merge of the
 * attention's splits.  codes, scores, idx and n_selected are bit-identical to the separate calls;
 * out is the same sum over the same tokens, cut into splits by position ranges of the sequence
 * instead of by ranges of the index row, so it agrees with the separate calls to rounding - and
 * with itself bit for bit: what a split sums, and in which order, depends on the scores alone
 * (Eq. 2 fixes the sum, not its order).  With value norms the caller updates vnorm for the
 * appended row first (socket_value_norms with max_rows = 1).
 * pos, k: device int32 [batch].
 */
int socket_decode_step(socket_ctx *ctx, const void *q, const void *K, const void *V, void *codes,
                       const void *proj, float tau, const float *vnorm, const int32_t *block_table,
                       const int32_t *pos, const int32_t *k, int32_t batch, float scale,
                       float *scores, int32_t *idx, int32_t *n_selected, int32_t out_dtype,
                       void *out, void *stream);

/* Text for an error code; last HIP error code seen by this context (0 if none). */
const char *socket_strerror(int code);
int socket_last_hip_error(const socket_ctx *ctx);

/*
 * HIP-graph helpers, so that a caller without HIP headers can record a chain of
 * the calls above once and replay it: begin capture on `stream`, issue calls on
 * that stream, end capture (instantiates), launch any number of times, destroy.
 */
typedef struct socket_graph socket_graph;
int socket_graph_begin(void *stream);
int socket_graph_end(void *stream, socket_graph **out);
int socket_graph_launch(socket_graph *g, void *stream);
int socket_graph_destroy(socket_graph *g);

#ifdef __cplusplus
}
#endif
#endif /* SOCKET_H */

// Internal declarations shared by the libsocket translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/socket.h"

namespace sk {

constexpr int kTile = 16;            // tokens per rotation period of the code layout
constexpr int kHistBits = 11;        // first radix digit of the top-k select (sign, exponent, 2 mantissa bits)
constexpr int kHistBins = 1 << kHistBits;
constexpr int kMaxLdsBytes = 160 * 1024;
constexpr int kScoreThreads = 512;
constexpr int kScoreU = 4;           // 16-byte loads a lane keeps in flight
constexpr int kDecodeThreads = 256;
constexpr int kDecodeChunk = 64;     // selected rows a decode workgroup handles per pass
constexpr int kDenseSplits = 64;     // splits per (sequence, KV head) of the dense attention baseline
constexpr int kMaxSplits = 128;      // most split-K partial results one merge takes
constexpr int kTopkThreads = 512;
constexpr int kPer = 8;              // scores per thread in a sweep of the select
constexpr int kSlice = kTopkThreads * kPer;      // scores per workgroup of the sweep: one region of the selected list
constexpr int kMaxRegions = 1024;    // regions per (sequence, KV head): max_n <= 4M tokens
constexpr int kCounterStride = 16;   // uint32 counters per (sequence, KV head)
constexpr int kThrStride = 16;       // uint32 words of the top-k threshold record per (sequence, KV head)
constexpr int kThrBinLo = 8;         // words of the record that hold the adaptive binning (float bits): offset,
constexpr int kThrBinInv = 9;        // and reciprocal width

// How the L x R bucket probabilities of one KV head are laid out for the scoring kernel.
//   direct : one entry per (table, bucket), already averaged over the G query heads:
//            T[c][r][64] floats, c = table / 64.
//   factor : bucket id split into low/high bit fields, p(r) = A[r_lo] * B[r_hi], kept per
//            query head: F[g][c][Rlo + Rhi][64] floats (rows < Rlo are A, the rest B).
// In both, word w of the 64 holds table l' = w % min(Lpad, 64); tables >= L hold 0.
//   split  : P = 9 or 10 (up to 1024 buckets): one entry per (table, bucket) as in `direct`,
//            but too large for LDS as a whole, so it is cut by tables into groups of
//            GT = min(Lpad, 32): T[group][r / 4][GT][4] floats; the scoring kernel takes the groups
//            one after the other (a 32-table group of 1024 buckets is 128 KB).  Goes with the
//            packed 10-bit id layout (see socket.h).
enum TableMode { kDirect = 0, kFactor = 1, kSplit = 2 };

// What the context's first-level histogram holds when the top-k select starts.
//   none     : nothing, the select histograms the scores itself
//   digit    : counts per leading 11-bit digit of the order-preserving score key
//   adaptive : counts per bin of score_bin() with the (offset, reciprocal width) pair stored in
//              the threshold record; the bins are narrow where the scores are dense, so the
//              threshold bin alone already isolates a short candidate list
enum HistMode { kHistNone = 0, kHistDigit = 1, kHistAdaptive = 2 };

struct Geometry {
    // Ids of 1, 2 or 4 bits are kept 8 / P to a byte when L is a multiple of that: the byte of
    // tables 8/P * l' .. is exactly the id of one 8-plane table l' over the same columns of W,
    // so everything below runs as (P, L) = (8, L * P / 8); only the bucket-probability tables
    // differ (an entry is the sum of the 8/P small tables' entries, not one product).
    int pf;          // ids per byte (1 = not shared)
    int Lu, Pu;      // the caller's L and P
    float mu;        // mean score of a uniformly drawn key: Lu / 2^Pu
    int d, Hq, Hkv, G, L, P, R;
    int Lpad;        // codes per token
    int S;           // lanes that share one token's 64 codes of a chunk (Lpad<64: Lpad/16, else 4);
                     // split mode: lanes that share one token's GT codes of a group (GT/16)
    int rounds;      // 64-table chunks per token (split mode: GT-table groups per token)
    int cb;          // bytes per code; 0 = packed 10-bit ids (split mode)
    int GT;          // split mode: tables per group
    int mode;        // TableMode
    int Plo, Phi, Rlo, Rhi;
    int table_rows;  // rows of 64 floats per chunk (direct: R, factor: Rlo+Rhi)
    int64_t table_words;  // floats per (sequence, KV head)
    int page, max_blocks, num_blocks, max_n, max_k, max_batch, kv_dtype;
    int n_split;     // split-K factor of sparse_decode
    int n_regions;   // regions of the select's sweep per (sequence, KV head): ceil(max_n / kSlice)
    int ssr, rpg;    // fused step: attention workgroups per region, or regions per attention workgroup
    int n_split_sweep;   // split-K factor of the fused step's attention: n_regions * ssr / rpg
};

}  // namespace sk

struct socket_ctx {
    socket_params p;
    sk::Geometry g;
    int device;
    int last_hip_error;
    int64_t scratch_bytes;
    int n_sink, n_window; // tokens at either end of a sequence that scoring forces into the selection
    float *tables;        // [max_batch*Hkv][table_words]
    float *tstats;        // [max_batch*Hkv][Lpad][3] spread of each table's bucket probabilities, sampled value norms
    float *subprobs;      // ids that share bytes only: [max_batch*Hkv][Lu][2^Pu] group-mean probabilities of the caller's tables
    const float *vnorm_sampled;   // the value-norm array the last projection pass sampled (or null)
    int pending_hist;     // HistMode of what socket_score_keys_binned left for socket_topk_select_binned
    void *wfrag;          // W cut into MFMA fragments for the fast prefill hash (null when that path does not apply)
    uint32_t *hist;       // [2][max_batch*Hkv][kHistBins]
    uint32_t *counters;   // [max_batch*Hkv][kCounterStride] counters, then [max_batch*Hkv][kThrStride] records
    uint32_t *cand_key;   // [max_batch*Hkv][max_n]
    int32_t *cand_idx;    // [max_batch*Hkv][max_n]
    int32_t *staged;      // [max_batch*Hkv][max_k] candidates picked by the long-list refinement
    int32_t *sel_regions; // [max_batch*Hkv][n_regions][kSlice] positions selected outright, by region of the sweep
    uint32_t *sel_cnt;    // [max_batch*Hkv][n_regions] how many each region holds
    float *partials;      // [max_batch*Hq][n_split][d+2]
    int32_t *seq_scratch; // [max_batch] lengths after the append of a fused decode step
};

namespace sk {

int fill_geometry(const socket_params *p, Geometry *g);  // host-only validation
inline int pack_factor(int L, int P) {
    // (at most 128 bytes of shared ids per token: two 64-table chunks of 256-entry tables are
    // what the scoring kernel's LDS holds; at least 32: shorter rows score no faster than a byte
    // per id with its small tables, measured)
    const int f = (P == 1 || P == 2 || P == 4) ? 8 / P : 1;
    return (L % f == 0 && L / f >= 32 && L / f <= 128) ? f : 1;
}
int record_hip(socket_ctx *ctx, hipError_t e);

// launchers (each returns a SOCKET_* code)
int score_prepare(const Geometry &g);   // once per context: checks the packed-id scoring kernel
int hash_prepare(int d);   // once per context that owns MFMA fragments of W (the fast 8-plane hash)
int launch_hash_keys(socket_ctx *ctx, const void *K, const void *proj, const int32_t *block_table,
                     const int32_t *row_begin, const int32_t *row_count, int batch, int max_rows,
                     void *codes, hipStream_t st);
// q null = append hash only; K null = soft hash only
int launch_project(socket_ctx *ctx, const void *q, const void *proj, float tau, const void *K,
                   void *codes, const int32_t *block_table, const int32_t *pos, const int32_t *count,
                   int32_t *len_out, int batch, hipStream_t st, const float *vnorm = nullptr);
int launch_hard_hash(socket_ctx *ctx, const void *q, const void *proj, int batch, hipStream_t st);
int launch_soft_hash(socket_ctx *ctx, const void *q, const void *proj, float tau, int batch,
                     hipStream_t st);
// want_hist: also accumulate a first-level histogram of the scores into the context; returns
// in *hist_mode which kind (HistMode) it left there
int launch_score_keys(socket_ctx *ctx, const void *codes, const float *vnorm,
                      const int32_t *block_table, const int32_t *seq_len, int batch, float *scores,
                      bool want_hist, int *hist_mode, hipStream_t st);
// hist_mode: what the context's histogram already holds about `scores` (HistMode)
int launch_topk(socket_ctx *ctx, const float *scores, const int32_t *seq_len, const int32_t *k,
                int batch, int32_t *idx, int32_t *n_selected, int hist_mode, hipStream_t st);
// the select up to its sweep (threshold + unordered lists); launch_sweep_decode continues from it
int launch_topk_sweep(socket_ctx *ctx, const float *scores, const int32_t *seq_len, const int32_t *k,
                      int batch, int32_t *idx, int32_t *n_selected, int hist_mode, hipStream_t st);
// Eq. 2 from the sweep's lists, then the split merge beside the ordering of the index row
int launch_sweep_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const float *scores, const int32_t *seq_len, const int32_t *k,
                        int32_t *idx, int32_t *n_selected, int hist_mode, const int32_t *block_table,
                        int batch, float scale, int out_dtype, void *out, hipStream_t st);
int launch_dense_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const int32_t *block_table, const int32_t *seq_len, int batch, float scale,
                        int out_dtype, void *out, hipStream_t st);
int launch_bucket_probs(socket_ctx *ctx, int batch, float *probs, hipStream_t st);
int launch_reset(socket_ctx *ctx, hipStream_t st);
int launch_stream_read(const void *buf, int64_t bytes, uint32_t *sink, hipStream_t st);
int launch_value_norms(socket_ctx *ctx, const void *V, const int32_t *block_table,
                       const int32_t *row_begin, const int32_t *row_count, int batch, int max_rows,
                       float *vnorm, hipStream_t st);
int launch_sparse_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                         const int32_t *idx, const int32_t *n_selected, const int32_t *block_table,
                         int batch, float scale, int out_dtype, void *out, hipStream_t st);
// the same without a context: partial results in a file-scope device array; *hip_error gets the
// HIP code when SOCKET_EHIP is returned
int sparse_decode_noalloc(const socket_params *p, const void *q, const void *K, const void *V,
                          const int32_t *idx, const int32_t *n_selected, const int32_t *block_table,
                          int batch, float scale, int out_dtype, void *out, hipStream_t st, int *hip_error);

// ---- device helpers -------------------------------------------------------------------

__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
    return __uint_as_float(((uint32_t)h) << 16);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---- cross-lane sums without LDS traffic
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}
// sum over lanes differing in bit 4 (adjacent 16-lane rows) / bit 5 (wavefront halves)
__device__ __forceinline__ float xor16_sum(float v) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float xor32_sum(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// sum over the LPR adjacent lanes that share a row (LPR = 8, 16, 32 or 64); every lane ends
// with the total
template <int LPR> __device__ __forceinline__ float row_sum(float v) {
    if (LPR >= 16) {
        v += dpp_f32<0x128>(v);      // row_ror:8
        v += dpp_f32<0x124>(v);      // row_ror:4
    } else {
        v += dpp_f32<0x141>(v);      // row_half_mirror: lane t <-> 7 - t inside each group of 8
    }
    v += dpp_f32<0x4E>(v);           // quad_perm [2,3,0,1]
    v += dpp_f32<0xB1>(v);           // quad_perm [1,0,3,2]
    if (LPR >= 32) v = xor16_sum(v);
    if (LPR >= 64) v = xor32_sum(v);
    return v;
}

// inclusive prefix sum over the 64 lanes of a wavefront: shifts inside the 16-lane rows, then
// the row totals carried over with the two row broadcasts
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
    x += __builtin_amdgcn_update_dpp(0u, x, 0x111, 0xF, 0xF, true);     // row_shr:1
    x += __builtin_amdgcn_update_dpp(0u, x, 0x112, 0xF, 0xF, true);     // row_shr:2
    x += __builtin_amdgcn_update_dpp(0u, x, 0x114, 0xF, 0xF, true);     // row_shr:4
    x += __builtin_amdgcn_update_dpp(0u, x, 0x118, 0xF, 0xF, true);     // row_shr:8
    x += __builtin_amdgcn_update_dpp(0u, x, 0x142, 0xA, 0xF, false);    // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0u, x, 0x143, 0xC, 0xF, false);    // row_bcast:31 into rows 2 and 3
    return x;
}

// max over the 64 lanes of a wavefront; every lane ends with it
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0x128>(v));
    v = fmaxf(v, dpp_f32<0x124>(v));
    v = fmaxf(v, dpp_f32<0x4E>(v));
    v = fmaxf(v, dpp_f32<0xB1>(v));
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Adaptive first-level bin of a score: the leading bits of 1 + max(v - lo, 0) * inv read as a
// float, i.e. 512 equal bins per octave of that quantity over four octaves, the last bin
// taking everything beyond.  Non-decreasing in v for any (lo, inv), which is all the exact
// select needs; how well the bins fit the scores only decides how short the candidate list is.
__device__ __forceinline__ uint32_t score_bin(float v, float lo, float inv) {
    const float y = fmaf(fmaxf(v - lo, 0.0f), inv, 1.0f);
    const uint32_t bin = (__float_as_uint(y) - 0x3f800000u) >> 14;
    return bin < (uint32_t)(kHistBins - 1) ? bin : (uint32_t)(kHistBins - 1);
}

// 8 consecutive elements of a K/V row as floats
template <typename T> struct Row8;
template <> struct Row8<uint16_t> {
    uint4 raw;
    __device__ __forceinline__ void load(const void *p) { raw = *(const uint4 *)p; }
    __device__ __forceinline__ void zero() { raw = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void store(void *p) const { *(uint4 *)p = raw; }
    __device__ __forceinline__ void get(float *f) const {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};
template <> struct Row8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const void *p) { a = ((const float4 *)p)[0]; b = ((const float4 *)p)[1]; }
    __device__ __forceinline__ void zero() { a = make_float4(0, 0, 0, 0); b = a; }
    __device__ __forceinline__ void store(void *p) const { ((float4 *)p)[0] = a; ((float4 *)p)[1] = b; }
    __device__ __forceinline__ void get(float *f) const {
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
};

// Table whose id is stored at position pos of token t's code row.
__device__ __forceinline__ int table_at(int pos, int t, int S) {
    int c = pos >> 6, p = pos & 63;
    int sub = p >> 4, s = p & 15;
    return (c << 6) + sub + S * ((t + s) & 15);
}

// P-bit field starting at bit `bitpos` of a little-endian bit row.
__device__ __forceinline__ uint32_t bit_field(const uint32_t *row, int bitpos, int P) {
    int w = bitpos >> 5, off = bitpos & 31;
    uint32_t v = row[w] >> off;
    if (off + P > 32) v |= row[w + 1] << (32 - off);
    return v & ((1u << P) - 1u);
}

// Position of table l's id inside token t's code row (inverse of table_at).
__device__ __forceinline__ int code_pos(int l, int t, int S) {
    int c = l >> 6, lp = l & 63;
    return (c << 6) + (lp % S) * 16 + ((lp / S - t) & 15);
}

// ---- packed 10-bit ids (split mode).  Tokens are stored in tiles of 16; a tile holds, for each
// group of GT tables, a block of 20*GT bytes.  The 16 ids that one lane of the scoring kernel
// looks up - those of position group `sub` (GT/16 of them per group) of one token - are one
// 160-bit little-endian string, id s in bits [10 s, 10 s + 10).  The block keeps the first
// 16 bytes of every string in 16 "main" rows (token t mod 16) of GT bytes, string `sub` at
// byte 16 sub, and the last 4 bytes in 16 "tail" rows of GT/4 bytes, string `sub` at byte
// 4 sub: a wavefront reads both as contiguous runs.  Inside a string the ids are rotated like
// the unpacked layouts: id s of string `sub` of token t belongs to table
// group*GT + sub + S ((t + s) mod 16), S = GT/16.
__host__ __device__ __forceinline__ int64_t packed_tile_bytes(int Lpad) { return 20 * (int64_t)Lpad; }
// byte offset of the main row / the tail row of token row `row`, group `grp`
__host__ __device__ __forceinline__ int64_t packed_main_row(int64_t row, int grp, int Lpad, int GT) {
    return (row >> 4) * packed_tile_bytes(Lpad) + (int64_t)grp * 20 * GT + (row & 15) * GT;
}
__host__ __device__ __forceinline__ int64_t packed_tail_row(int64_t row, int grp, int Lpad, int GT) {
    return (row >> 4) * packed_tile_bytes(Lpad) + (int64_t)grp * 20 * GT + 16 * GT + (row & 15) * (GT >> 2);
}
// byte offset, inside the (sequence or block, KV head) slab, of 32-bit word i (0..4) of string
// `sub` of token row `row`, group `grp`
__host__ __device__ __forceinline__ int64_t packed_word(int64_t row, int grp, int sub, int i, int Lpad, int GT) {
    return i < 4 ? packed_main_row(row, grp, Lpad, GT) + sub * 16 + 4 * i
                 : packed_tail_row(row, grp, Lpad, GT) + sub * 4;
}
// table (within its group) of id j = 16 sub + s of token t; and the inverse
__host__ __device__ __forceinline__ int packed_table_at(int j, int t, int S) {
    return (j >> 4) + S * ((t + (j & 15)) & 15);
}
__host__ __device__ __forceinline__ int packed_pos(int tl, int t, int S) {
    return (tl % S) * 16 + ((tl / S - t) & 15);
}

// Row index (in units of rows of the [.., Hkv, tokens, width] tensor) of token t of
// sequence b, KV head h; handles contiguous and paged storage.
struct RowMap {
    const int32_t *block_table;  // null = contiguous
    int Hkv, max_n, page, max_blocks, num_blocks;
    uint32_t page_magic;         // ceil(2^32 / page): t / page == (t * page_magic) >> 32 for every token t < max_n
                                 // (exact for power-of-two pages; otherwise socket_create checks max_n * page < 2^32)
    // block-table column and offset inside the block of token t: no division, no branch
    __device__ __forceinline__ int page_slot(int t) const { return (int)__umulhi((uint32_t)t, page_magic); }
    __device__ __forceinline__ int page_off(int t) const { return t - page_slot(t) * page; }
    // -1 when the token's block is absent (paged storage with an out-of-range table entry)
    __device__ __forceinline__ int64_t row(int b, int h, int t) const {
        if (block_table == nullptr) return ((int64_t)b * Hkv + h) * max_n + t;
        const int slot = page_slot(t), off = t - slot * page;
        int blk = block_table[(int64_t)b * max_blocks + slot];
        if ((unsigned)blk >= (unsigned)num_blocks) return -1;
        return ((int64_t)blk * Hkv + h) * page + off;
    }
};

inline RowMap row_map(const Geometry &g, const int32_t *block_table) {
    const uint32_t magic = g.page > 0 ? (uint32_t)((((uint64_t)1 << 32) + g.page - 1) / (uint64_t)g.page) : 0u;
    return RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks, magic};
}

}  // namespace sk

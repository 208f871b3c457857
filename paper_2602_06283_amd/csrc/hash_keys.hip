// Alg. 1 (PrecomputeKeyHashes): sign random projections of cached keys, packed into bucket ids.
//
// Kernels:
//   hash_mfma8_kernel  bf16 keys, 8- or 4-plane tables (one-byte ids), d <= 128: the W slab of a
//                      chunk of up to 64 tables sits in LDS as MFMA fragments, keys go from
//                      memory straight into registers, the ids are assembled in registers.
//   hash_mfma10_kernel the same structure for 10-plane tables with packed 10-bit ids.
//   hash_mfma_kernel   bf16 keys, any other shape: K[rows x d] * W[d x L*P] on bf16 MFMA
//                      (v_mfma_f32_32x32x16_bf16, fp32 accumulate), W held in registers,
//                      key tiles staged through LDS, sign bits taken from the accumulators'
//                      sign bit and packed into a per-key bit matrix in LDS.
//   hash_rows_kernel   fp32 keys, or a handful of appended rows: fp32 FMA, one thread per
//                      projection column, sign bits gathered with a wavefront ballot.
// The last two end in pack_codes(), which cuts the bit matrix into P-bit bucket ids and writes
// them in the rotated order the scoring kernel reads.
#include "socket_internal.h"

namespace sk {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;

struct HashArgs {
    const void *K;
    const void *W;
    void *codes;
    const int32_t *row_begin;
    const int32_t *row_count;
    RowMap map;
    int d, L, P, LP, Lpad, S, cb;
    int GT;                // tables per group of the packed 10-bit layout, 0 = unpacked ids
    int rows_per_wg;
    int tables_per_chunk;  // tables one workgroup covers (mfma kernel)
    int n_chunks;
};

// Cut `nrows` bit rows (LDS, stride `stride` words, bit j of a row = sign bit of the
// projection onto column first_table*P + j) into bucket ids and store them.
// tok[r] = logical token of row r, grow[r] = its row in the codes tensor (-1 = skip).
// Only tables in [first_table, first_table+ntab) are written; when the workgroup owns
// whole 4-byte words (whole == true) the ids go out as aligned dwords.
__device__ __forceinline__ void pack_codes(const uint32_t *bits, int stride, int nrows,
                                           const int *tok, const int64_t *grow, void *codes,
                                           int L, int P, int Lpad, int S, int cb,
                                           int first_table, int ntab, bool whole, int tid,
                                           int nthreads) {
    if (whole) {
        const int cpd = 4 / cb;             // ids per dword
        const int pos0 = (first_table >> 6) << 6;
        const int span = ((ntab + 63) >> 6) << 6;  // positions owned (whole 64-groups)
        const int dspan = (span < Lpad ? span : Lpad) / cpd;
        for (int i = tid; i < nrows * dspan; i += nthreads) {
            int r = i / dspan, dw = i - r * dspan;
            if (grow[r] < 0) continue;
            uint32_t word = 0;
            for (int e = 0; e < cpd; ++e) {
                int pos = pos0 + dw * cpd + e;
                int l = table_at(pos, tok[r], S);
                uint32_t code = 0;
                if (l < L && l >= first_table && l < first_table + ntab)
                    code = bit_field(bits + r * stride, (l - first_table) * P, P);
                word |= code << (8 * cb * e);
            }
            uint32_t *dst = (uint32_t *)((char *)codes + grow[r] * (int64_t)Lpad * cb) + pos0 / cpd + dw;
            *dst = word;
        }
    } else {
        for (int i = tid; i < nrows * Lpad; i += nthreads) {
            int r = i / Lpad, pos = i - r * Lpad;
            if (grow[r] < 0) continue;
            int l = table_at(pos, tok[r], S);
            uint32_t code = 0;
            if (l >= L) {
                if (first_table != 0) continue;   // padding positions belong to the first chunk
            } else if (l < first_table || l >= first_table + ntab) {
                continue;
            } else {
                code = bit_field(bits + r * stride, (l - first_table) * P, P);
            }
            int64_t at = grow[r] * (int64_t)Lpad + pos;
            if (cb == 1) ((uint8_t *)codes)[at] = (uint8_t)code;
            else ((uint16_t *)codes)[at] = (uint16_t)code;
        }
    }
}

// The same for the packed 10-bit layout: the workgroup owns groups g0 .. g0+ngrp-1 of GT
// tables whole, and every thread builds one aligned dword of a token's 160-bit id string
// (parts of the four or five ids that overlap it).
__device__ __forceinline__ void pack_codes_packed(const uint32_t *bits, int stride, int nrows,
                                                  const int *tok, const int64_t *grow, void *codes,
                                                  int L, int P, int Lpad, int GT, int first_table,
                                                  int ntab, int ngrp, int tid, int nthreads) {
    const int S = GT >> 4;
    const int g0 = first_table / GT;
    const int per_row = ngrp * S * 5;                // dwords per token
    for (int i = tid; i < nrows * per_row; i += nthreads) {
        const int r = i / per_row;
        int u = i - r * per_row;
        if (grow[r] < 0) continue;
        const int gl = u / (S * 5);
        u -= gl * (S * 5);
        const int sub = u / 5, wi = u - sub * 5;     // string, dword of the string
        const int grp = g0 + gl, t = tok[r];
        const uint32_t *row = bits + r * stride;
        uint32_t word = 0;
        const int s0 = (32 * wi) / 10;               // first id that reaches into this dword
#pragma unroll
        for (int e = 0; e < 5; ++e) {
            const int sidx = s0 + e, at = 10 * sidx - 32 * wi;   // bit of the dword where the id starts
            if (sidx > 15 || at >= 32) break;
            const int l = grp * GT + packed_table_at(sub * 16 + sidx, t, S);
            uint32_t id = 0;
            if (l < L && l >= first_table && l < first_table + ntab) id = bit_field(row, (l - first_table) * P, P);
            word |= at >= 0 ? id << at : id >> -at;
        }
        *(uint32_t *)((char *)codes + packed_word(grow[r], grp, sub, wi, Lpad, GT)) = word;
    }
}

// ---------------------------------------------------------------------------------------
// fp32-FMA kernel: ROWS rows per workgroup, one thread per projection column.
// ---------------------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float load_elem(const T *p);
template <> __device__ __forceinline__ float load_elem<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_elem<uint16_t>(const uint16_t *p) { return bf16_to_f32(*p); }

template <typename T, int ROWS>
__global__ __launch_bounds__(256) void hash_rows_kernel(HashArgs a) {
    extern __shared__ uint32_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.y, b = blockIdx.z;
    const int count = a.row_count[b];
    const int r0 = blockIdx.x * ROWS;
    if (r0 >= count) return;
    const int nrows = min(ROWS, count - r0);
    const int bw = 2 * ((a.LP + 63) / 64);     // bit-row stride in words

    float *ks = (float *)smem;                         // [ROWS][d]
    uint32_t *bits = smem + ROWS * a.d;                // [ROWS][bw]
    int *tok = (int *)(bits + ROWS * bw);              // [ROWS]
    int64_t *grow = (int64_t *)(tok + ROWS + (ROWS & 1));  // [ROWS], 8-byte aligned

    if (tid < ROWS) {
        int t = a.row_begin[b] + r0 + tid;
        bool live = tid < nrows && t >= 0 && t < a.map.max_n;
        tok[tid] = t;
        grow[tid] = live ? a.map.row(b, h, t) : -1;
    }
    __syncthreads();
    const T *K = (const T *)a.K;
    for (int i = tid; i < ROWS * a.d; i += 256) {
        int r = i / a.d, c = i - r * a.d;
        ks[i] = grow[r] >= 0 ? load_elem<T>(K + grow[r] * a.d + c) : 0.0f;
    }
    for (int i = tid; i < ROWS * bw; i += 256) bits[i] = 0;
    __syncthreads();

    const T *W = (const T *)a.W + (int64_t)h * a.d * a.LP;
    for (int base = 0; base < a.LP; base += 256) {
        const int col = base + tid;
        float acc[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) acc[r] = 0.0f;
        if (col < a.LP) {
            for (int c = 0; c < a.d; ++c) {
                float w = load_elem<T>(W + (int64_t)c * a.LP + col);
#pragma unroll
                for (int r = 0; r < ROWS; ++r) acc[r] = fmaf(ks[r * a.d + c], w, acc[r]);
            }
        }
        const int word = (base + wave * 64) >> 5;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            unsigned long long m = __ballot(col < a.LP && acc[r] >= 0.0f);
            if (lane == 0 && word < bw) {
                bits[r * bw + word] = (uint32_t)m;
                if (word + 1 < bw) bits[r * bw + word + 1] = (uint32_t)(m >> 32);
            }
        }
    }
    __syncthreads();
    if (a.GT)
        pack_codes_packed(bits, bw, ROWS, tok, grow, a.codes, a.L, a.P, a.Lpad, a.GT, 0, a.L, a.Lpad / a.GT, tid, 256);
    else
        pack_codes(bits, bw, ROWS, tok, grow, a.codes, a.L, a.P, a.Lpad, a.S, a.cb, 0, a.L, true, tid, 256);
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel.  512 threads = 8 waves; wave w owns projection columns
// [64w, 64w+64) of the workgroup's column chunk and keeps that slab of W in registers
// for the whole kernel.  The workgroup walks its rows in tiles of 64 keys, staged through
// LDS; a tile is multiplied as two halves of 32 keys so that the accumulators take 32
// registers and two workgroups fit a CU.
// MFMA operands: A = W^T (32 planes x 16 channels), B = K^T (16 channels x 32 keys), so
// lane (key n, half g) of the accumulator holds planes 8a + 4g + b (a,b in 0..3) of key n.
// One barrier per tile: the bit matrix is double-buffered and the row bookkeeping
// triple-buffered, so the waves that have finished a tile's products pack its ids while the
// others still multiply, and nobody waits a second time.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512, D <= 128 ? 4 : 2) void hash_mfma_kernel(HashArgs a) {
    constexpr int KS = D / 16;                 // MFMA k-steps
    constexpr int TILE = 64;                   // keys per tile
    constexpr int KSTRIDE = D * 2 + 16;        // bytes per staged key row (padded)
    constexpr int BSTRIDE = 17;                // words per bit row (16 + 1 pad)
    extern __shared__ uint32_t smem[];
    char *const kbase = (char *)smem;                  // two staged key tiles
    auto ktile = [&](int bf) { return kbase + bf * (TILE * KSTRIDE); };
    uint32_t *bits = smem + 2 * TILE * KSTRIDE / 4;   // [2][TILE][BSTRIDE]
    int *tok = (int *)(bits + 2 * TILE * BSTRIDE);    // [3][TILE]
    int64_t *grow = (int64_t *)(tok + 4 * TILE);      // [3][TILE] (8-byte aligned)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.y % a.n_chunks, h = blockIdx.y / a.n_chunks, b = blockIdx.z;
    const int count = a.row_count[b];
    const int wg_r0 = blockIdx.x * a.rows_per_wg;
    if (wg_r0 >= count) return;
    const int wg_r1 = min(count, wg_r0 + a.rows_per_wg);
    const int begin = a.row_begin[b];

    const int first_table = chunk * a.tables_per_chunk;
    const int ntab = max(0, min(a.tables_per_chunk, a.L - first_table));   // 0: a group of padding tables only
    const int ncols = ntab * a.P;              // live columns of this chunk (<= 512)
    const int col0 = first_table * a.P;

    // ---- this wave's slab of W as MFMA A-operand fragments: plane m = lane%32, channels
    //      16*ks + 8*(lane/32) .. +7
    const uint16_t *W = (const uint16_t *)a.W + (int64_t)h * D * a.LP;
    bf16x8_t wfrag[2][KS];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int j = wave * 64 + mb * 32 + (lane & 31);      // chunk-local column
        const bool live = j < ncols;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            union { bf16x8_t v; uint16_t u[8]; } f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int c = ks * 16 + (lane >> 5) * 8 + e;
                f.u[e] = live ? W[(int64_t)c * a.LP + col0 + j] : (uint16_t)0;
            }
            wfrag[mb][ks] = f.v;
        }
    }

    // ---- tile staging: thread -> (row = tid / 8, 1/8 of the row)
    constexpr int SEG = D * 2 / 8;             // bytes of a row each thread stages (16, 32 or 64)
    const int srow = tid >> 3, sseg = tid & 7;
    uint4 stage[SEG / 16];

    auto fetch = [&](int tile_r0, int slot) {  // slot: which third of the row bookkeeping
        int r = tile_r0 + srow;
        int t = begin + r;
        bool live = r < wg_r1 && t >= 0 && t < a.map.max_n;
        int64_t g = live ? a.map.row(b, h, t) : -1;
        if (sseg == 0) {
            tok[slot * TILE + srow] = t;
            grow[slot * TILE + srow] = g;
        }
        const char *src = (const char *)a.K + g * (int64_t)(D * 2) + sseg * SEG;
#pragma unroll
        for (int v = 0; v < SEG / 16; ++v)
            stage[v] = g >= 0 ? ((const uint4 *)src)[v] : make_uint4(0, 0, 0, 0);
    };
    auto commit = [&](int buf) {
        char *dst = ktile(buf) + srow * KSTRIDE + sseg * SEG;
#pragma unroll
        for (int v = 0; v < SEG / 16; ++v) ((uint4 *)dst)[v] = stage[v];
    };

    // ids of P = 8 planes are the bytes of a bit row, and the rotated order moves whole bytes:
    // position 64c + 16 sub + s of token t holds table 64c + sub + 4 ((t + s) mod 16)
    const bool byte_ids = a.P == 8 && a.S == 4 && (a.tables_per_chunk == 64 || a.n_chunks == 1);
    const bool whole = a.n_chunks == 1 || (a.tables_per_chunk & 63) == 0;

    fetch(wg_r0, 0);
    commit(0);
    __syncthreads();

    int buf = 0, slot = 0;
    for (int tile_r0 = wg_r0; tile_r0 < wg_r1; tile_r0 += TILE) {
        const bool more = tile_r0 + TILE < wg_r1;
        const int nslot = slot == 2 ? 0 : slot + 1;
        if (more) fetch(tile_r0 + TILE, nslot);
        uint32_t *bt = bits + buf * (TILE * BSTRIDE);

#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            // ---- MFMA: acc[mb] = W^T slab (32 planes) x K^T (32 keys)
            floatx16_t acc[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;
            const char *src = ktile(buf) + (nb * 32 + (lane & 31)) * KSTRIDE + (lane >> 5) * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8_t kf = *(const bf16x8_t *)(src + ks * 32);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag[0][ks], kf, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag[1][ks], kf, acc[1], 0, 0, 0);
            }
            // ---- sign bits: accumulator i of lane (n, g) is plane 8*(i/4) + 4g + i%4.
            //      Funnel-shift the 16 sign bits into one 16-bit value per lane, exchange with
            //      the other half-wave, and interleave nibbles into the 32 planes of the block.
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                uint32_t neg = __float_as_uint(acc[mb][15]) >> 31;
#pragma unroll
                for (int i = 14; i >= 0; --i)
                    neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[mb][i]), 31);
                neg &= 0xffffu;                         // bit 4a+b = sign of plane 8a+4g+b
                auto both = __builtin_amdgcn_permlane32_swap(neg, neg, false, false);
                uint32_t lo = both[0], hi = both[1];    // the g = 0 and g = 1 halves of key n, in every lane
                lo = (lo | (lo << 8)) & 0x00ff00ffu;
                lo = (lo | (lo << 4)) & 0x0f0f0f0fu;
                hi = (hi | (hi << 8)) & 0x00ff00ffu;
                hi = (hi | (hi << 4)) & 0x0f0f0f0fu;
                const uint32_t word = ~(lo | (hi << 4)); // bit p = 1 when plane p projects >= 0
                if (lane < 32) bt[(nb * 32 + lane) * BSTRIDE + wave * 2 + mb] = word;
            }
        }
        if (more) commit(buf ^ 1);
        __syncthreads();   // bit matrix complete, next tile staged, every wave done with this key tile

        const int *tk = tok + slot * TILE;
        const int64_t *gr = grow + slot * TILE;
        if (byte_ids) {
            // thread -> (row, 16-position group, half of it): 8 ids = 8 byte reads, one 8-byte store
            const int r = tid >> 3, sub = (tid >> 1) & 3, half = tid & 1;
            const int64_t g = gr[r];
            if (g >= 0) {
                const int t = tk[r];
                const uint8_t *rowb = (const uint8_t *)(bt + r * BSTRIDE);
                uint32_t out[2] = {0u, 0u};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int tbl = sub + 4 * ((t + half * 8 + e) & 15);     // chunk-local table
                    const uint32_t id = tbl < ntab ? rowb[tbl] : 0u;
                    out[e >> 2] |= id << (8 * (e & 3));
                }
                const int pos0 = (first_table >> 6) << 6;
                *(uint2 *)((char *)a.codes + g * (int64_t)a.Lpad + pos0 + sub * 16 + half * 8) = make_uint2(out[0], out[1]);
            }
        } else if (a.GT) {
            pack_codes_packed(bt, BSTRIDE, TILE, tk, gr, a.codes, a.L, a.P, a.Lpad, a.GT, first_table, ntab, 1,
                              tid, 512);
        } else {
            pack_codes(bt, BSTRIDE, TILE, tk, gr, a.codes, a.L, a.P, a.Lpad, a.S, a.cb, first_table, ntab,
                       whole, tid, 512);
        }
        buf ^= 1;
        slot = nslot;
    }
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel for 8-plane tables (one-byte ids), d <= 128: the fast path.
// A workgroup keeps the W slab of one 64-table chunk (512 columns) in LDS, already cut into
// MFMA A-operand fragments, and each of its 16 wavefronts works on 64-key blocks of its own:
// the keys go from memory straight into B-operand registers, so there is no staging, no
// barrier in the main loop, and the wavefronts drift apart - some multiply while others pack.
//
// Column order (S = 4 position groups of 16 ids per 64-table chunk; rows of 16 or 32 ids have
// S = 1 or 2 and read 4 as S below).  Position 16 sub + s of token t holds table
// sub + 4 ((t + s) mod 16).  The
// 32-column block p = 4 sub + q therefore holds tables sub + 4 (4q + e), e = 0..3: after four
// blocks the wavefront has, for each key, the 16 ids of position group `sub` in table order
// j = 4q + e as the 16 bytes of four sign words, and the stored group is those bytes rotated
// by t mod 16.
// Row order inside a block.  MFMA operands: A = W^T (32 rows x 16 channels), B = K^T
// (16 channels x 32 keys); accumulator i of lane (key n, half g) is row 8 (i/4) + 4g + i%4.
// Row m is given plane (table e, plane pl) with 8e + pl = 16 g + i, so that the 16 sign bits a
// lane collects from its accumulators are, in order, one half of the key's 32-bit sign word.
// hash_wfrag_kernel lays W out that way once per call; the main kernel copies it into LDS.
// ---------------------------------------------------------------------------------------
template <int D, int S, int P>
__global__ __launch_bounds__(256) void hash_wfrag_kernel(HashArgs a, uint4 *wfrag) {
    constexpr int BPG = P / 2;                 // 32-column blocks per position group of 16 ids (P = 8: 4, P = 4: 2)
    constexpr int KS = D / 16;
    const int p = blockIdx.x, chunk = blockIdx.y % a.n_chunks, h = blockIdx.y / a.n_chunks;
    const int first_table = chunk * 64;
    const int ntab = min(64, a.L - first_table);
    const int sub = p / BPG, q = p % BPG;
    const uint16_t *W = (const uint16_t *)a.W + (int64_t)h * D * a.LP;
    uint4 *dst = wfrag + ((int64_t)blockIdx.y * (BPG * S) + p) * KS * 64;
    for (int f = threadIdx.x; f < KS * 64; f += 256) {
        const int ks = f >> 6, lane = f & 63;
        const int g = lane >> 5, m = lane & 31;
        const int bit = 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3);
        // (a block holds 32 / P tables: table e of the block in bits [P e, P e + P) of the sign word)
        const int tt = sub + S * ((32 / P) * q + bit / P);     // chunk-local table
        const int col = (first_table + tt) * P + bit % P;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (tt < ntab) {
            uint16_t e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = W[(int64_t)(ks * 16 + g * 8 + i) * a.LP + col];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i >> 1] |= (uint32_t)e[i] << (16 * (i & 1));
        }
        dst[f] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <int V> struct IntTag { static constexpr int value = V; };

constexpr int kHash8Threads = 1024;

template <int D, int S, int P>
__global__ __launch_bounds__(kHash8Threads) void hash_mfma8_kernel(HashArgs a, const uint4 *wfrag) {
    static_assert(P == 8 || P == 4, "one-byte ids of 8 planes, or of 4 (a block's eight nibbles are spread over two words)");
    constexpr int KS = D / 16;                 // MFMA k-steps
    constexpr int BPG = P / 2;                 // 32-column blocks per position group of 16 ids
    constexpr int NCB = BPG * S;               // 32-column blocks of a chunk (S position groups)
    constexpr int NW = kHash8Threads / 64;
    extern __shared__ uint32_t smem[];
    uint4 *wl = (uint4 *)smem;                         // [NCB][KS][64 lanes] A fragments
    uint32_t *bits = smem + NCB * KS * 64 * 4;         // [NW waves][64 keys][4 words]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.y % a.n_chunks, h = blockIdx.y / a.n_chunks, b = blockIdx.z;
    const int count = a.row_count[b];
    const int begin = a.row_begin[b];
    const int first_table = chunk * 64;
    const int ntab = min(64, a.L - first_table);

    // ---- W slab -> LDS
    {
        const uint4 *src = wfrag + (int64_t)blockIdx.y * NCB * KS * 64;
        constexpr int N = NCB * KS * 64;
        if constexpr (N % kHash8Threads == 0) {
            constexpr int PER = N / kHash8Threads, NB = PER < 8 ? PER : 8;
            static_assert(PER % NB == 0, "whole batches of copies per thread");
#pragma unroll 1
            for (int u0 = 0; u0 < PER; u0 += NB) {
                uint4 v[NB];
#pragma unroll
                for (int u = 0; u < NB; ++u) v[u] = src[tid + (u0 + u) * kHash8Threads];
#pragma unroll
                for (int u = 0; u < NB; ++u) wl[tid + (u0 + u) * kHash8Threads] = v[u];
            }
        } else {
            for (int i = tid; i < N; i += kHash8Threads) wl[i] = src[i];
        }
    }
    __syncthreads();

    uint32_t *mybits = bits + wave * 256;
    const int n = lane & 31, g = lane >> 5;
    const char *Kb = (const char *)a.K;
    char *Cb = (char *)a.codes;

    auto key_row = [&](int r) -> int64_t {
        const int t = begin + r;
        return (r < count && t >= 0 && t < a.map.max_n) ? a.map.row(b, h, t) : -1;
    };
    // Branch-free: a key that does not exist reads row 0 of the cache instead (its ids are never
    // stored).
    bf16x8_t kf[2][KS];
    auto load_keys = [&](int r0) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int64_t row = key_row(r0 + nb * 32 + n);
            const char *src = Kb + (row >= 0 ? row : 0) * (int64_t)(D * 2) + g * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[nb][ks] = *(const bf16x8_t *)(src + ks * 32);
        }
    };
    // 32 sign bits of one key from the accumulators of a 32-row block: bit p = 1 when the
    // projection onto plane p is >= 0.  A lane's 16 accumulators are bits 16g .. 16g+15.
    auto sign_word = [&](const floatx16_t &acc) -> uint32_t {
        uint32_t neg = __float_as_uint(acc[15]) >> 31;
#pragma unroll
        for (int i = 14; i >= 0; --i) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[i]), 31);
        auto both = __builtin_amdgcn_permlane32_swap(neg, neg, false, false);   // g = 0 and g = 1 halves, in every lane
        return ~(both[0] | (both[1] << 16));
    };

    // 64-key blocks are dealt to the wavefronts of the whole launch round-robin
    const int nblocks = (count + 63) >> 6;
    const int stride = gridDim.x * NW;
    int blk = blockIdx.x * NW + wave;
    if (blk < nblocks) load_keys(blk * 64);
    for (; blk < nblocks; blk += stride) {
        const int r0 = blk * 64;
        const int64_t prow = key_row(r0 + lane);        // the key this lane packs
        const int rot = (begin + r0 + lane) & 15;
        uint4 done[S > 1 ? S - 1 : 1];                  // the key's position groups before the last, kept until the row is whole
#pragma unroll 1
        for (int p = 0; p < NCB; ++p) {
            const int sub = p / BPG, q = p % BPG;
            const uint4 *af = wl + (p * KS) * 64 + lane;
            floatx16_t acc0, acc1;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc0[i] = acc1[i] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                union { uint4 u; bf16x8_t v; } fa;
                fa.u = af[ks * 64];
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, kf[0][ks], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, kf[1][ks], acc1, 0, 0, 0);
            }
            const uint32_t w0 = sign_word(acc0), w1 = sign_word(acc1);
            const uint32_t w = lane < 32 ? w0 : w1;                     // lane = key n or 32 + n
            if (P == 8) {
                // bytes whose table (sub + S (4q + e)) lies beyond the chunk's live tables stay zero
                const int nlive = (ntab - sub - 4 * S * q + S - 1) >> (S == 4 ? 2 : S == 2 ? 1 : 0);   // live tables among e = 0..3 (<= 0: none)
                const uint32_t live_mask = nlive >= 4 ? 0xffffffffu : nlive <= 0 ? 0u : (1u << (8 * nlive)) - 1u;
                mybits[lane * 4 + q] = w & live_mask;
            } else {
                // eight 4-bit ids: each nibble becomes the byte of its table (sub + S (8q + e))
                auto spread = [](uint32_t x) {          // nibbles 0..3 of x -> bytes 0..3
                    const uint32_t t = (x | (x << 8)) & 0x00ff00ffu;
                    return (t | (t << 4)) & 0x0f0f0f0fu;
                };
                const int nlive = (ntab - sub - 8 * S * q + S - 1) >> (S == 4 ? 2 : S == 2 ? 1 : 0);   // live tables among e = 0..7
                const int n0 = nlive < 4 ? nlive : 4, n1 = nlive - 4 < 4 ? nlive - 4 : 4;
                const uint32_t m0 = n0 >= 4 ? 0xffffffffu : n0 <= 0 ? 0u : (1u << (8 * n0)) - 1u;
                const uint32_t m1 = n1 >= 4 ? 0xffffffffu : n1 <= 0 ? 0u : (1u << (8 * n1)) - 1u;
                mybits[lane * 4 + 2 * q] = spread(w & 0xffffu) & m0;
                mybits[lane * 4 + 2 * q + 1] = spread(w >> 16) & m1;
            }
            if (q == BPG - 1) {
                // ---- the 16 ids of position group `sub`, rotated by the token position
                const uint4 wv = *(const uint4 *)(mybits + lane * 4);
                const bool r1 = rot & 4, r2 = rot & 8;
                const uint32_t y0 = r1 ? wv.y : wv.x, y1 = r1 ? wv.z : wv.y, y2 = r1 ? wv.w : wv.z, y3 = r1 ? wv.x : wv.w;
                const uint32_t x0 = r2 ? y2 : y0, x1 = r2 ? y3 : y1, x2 = r2 ? y0 : y2, x3 = r2 ? y1 : y3;
                const uint32_t sh = rot & 3;
                uint4 o;
                o.x = __builtin_amdgcn_alignbyte(x1, x0, sh);
                o.y = __builtin_amdgcn_alignbyte(x2, x1, sh);
                o.z = __builtin_amdgcn_alignbyte(x3, x2, sh);
                o.w = __builtin_amdgcn_alignbyte(x0, x3, sh);
                // the four groups of a key go out together: 64 adjacent bytes, written back as one
                // whole line instead of four partial ones a quarter of the block apart
                if (S > 1 && sub == 0) done[0] = o;
                else if (S > 2 && sub == 1) done[S > 2 ? 1 : 0] = o;
                else if (S > 2 && sub == 2) done[S > 2 ? 2 : 0] = o;
                else if (prow >= 0) {
                    uint4 *dst = (uint4 *)(Cb + prow * (int64_t)a.Lpad + first_table);
#pragma unroll
                    for (int i = 0; i + 1 < S; ++i) dst[i] = done[i];
                    dst[S - 1] = o;
                }
            }
        }
        if (blk + stride < nblocks) load_keys((blk + stride) * 64);
    }
}

// ---------------------------------------------------------------------------------------
// The same structure for 10-plane tables with packed ids (groups of 16 S tables, S = 1 or 2,
// d <= 128): a workgroup keeps the W slab of one group (S x 160 columns = 5 S 32-column blocks)
// in LDS as MFMA fragments; every wavefront works on 64-key blocks of its own.
//
// Column order.  String `sub` (< S) of a token's group holds, before its rotation by the token
// position, the ids of tables sub, sub + S, .., sub + 15 S in bits [10 j, 10 j + 10): 160 bits =
// five sign words.  Block p = 5 sub + q produces word q: bit u = 32 q + (bit of the word) of the
// string is plane u % 10 of table sub + S (u / 10).  The stored string is that one rotated right
// by 10 (t mod 16) bits: a rotation of the five words and one funnel shift.
// ---------------------------------------------------------------------------------------
template <int D, int S>
__global__ __launch_bounds__(256) void hash_wfrag10_kernel(HashArgs a, uint4 *wfrag) {
    constexpr int KS = D / 16;
    const int p = blockIdx.x, grp = blockIdx.y % a.n_chunks, h = blockIdx.y / a.n_chunks;
    const int first_table = grp * 16 * S;
    const int ntab = min(16 * S, a.L - first_table);
    const int sub = p / 5, q = p % 5;
    const uint16_t *W = (const uint16_t *)a.W + (int64_t)h * D * a.LP;
    uint4 *dst = wfrag + ((int64_t)blockIdx.y * (5 * S) + p) * KS * 64;
    for (int f = threadIdx.x; f < KS * 64; f += 256) {
        const int ks = f >> 6, lane = f & 63;
        const int g = lane >> 5, m = lane & 31;
        const int bit = 16 * ((m >> 2) & 1) + 4 * (m >> 3) + (m & 3);   // bit of the sign word that MFMA row m becomes
        const int u = 32 * q + bit;
        const int tt = sub + S * (u / 10);                     // group-local table
        const int col = (first_table + tt) * 10 + u % 10;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (tt < ntab) {
            uint16_t e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = W[(int64_t)(ks * 16 + g * 8 + i) * a.LP + col];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i >> 1] |= (uint32_t)e[i] << (16 * (i & 1));
        }
        dst[f] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <int D, int S>
__global__ __launch_bounds__(kHash8Threads) void hash_mfma10_kernel(HashArgs a, const uint4 *wfrag) {
    constexpr int KS = D / 16;                 // MFMA k-steps
    constexpr int NCB = 5 * S;                 // 32-column blocks of a group
    constexpr int GT = 16 * S;                 // tables of a group
    constexpr int NW = kHash8Threads / 64;
    extern __shared__ uint32_t smem[];
    uint4 *wl = (uint4 *)smem;                         // [NCB][KS][64 lanes] A fragments
    uint32_t *bits = smem + NCB * KS * 64 * 4;         // [NW waves][64 keys][5 words]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = blockIdx.y % a.n_chunks, h = blockIdx.y / a.n_chunks, b = blockIdx.z;
    const int count = a.row_count[b];
    const int begin = a.row_begin[b];
    const int ntab = max(0, min(GT, a.L - grp * GT));

    {
        const uint4 *src = wfrag + (int64_t)blockIdx.y * NCB * KS * 64;
        for (int i = tid; i < NCB * KS * 64; i += kHash8Threads) wl[i] = src[i];
    }
    __syncthreads();

    uint32_t *mybits = bits + wave * 320;
    const int n = lane & 31, g = lane >> 5;
    const char *Kb = (const char *)a.K;
    char *Cb = (char *)a.codes;

    auto key_row = [&](int r) -> int64_t {
        const int t = begin + r;
        return (r < count && t >= 0 && t < a.map.max_n) ? a.map.row(b, h, t) : -1;
    };
    // (a key that does not exist reads row 0 of the cache instead; its ids are never stored)
    bf16x8_t kf[2][KS];
    auto load_keys = [&](int r0) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            const int64_t row = key_row(r0 + nb * 32 + n);
            const char *src = Kb + (row >= 0 ? row : 0) * (int64_t)(D * 2) + g * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[nb][ks] = *(const bf16x8_t *)(src + ks * 32);
        }
    };
    auto sign_word = [&](const floatx16_t &acc) -> uint32_t {
        uint32_t neg = __float_as_uint(acc[15]) >> 31;
#pragma unroll
        for (int i = 14; i >= 0; --i) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[i]), 31);
        auto both = __builtin_amdgcn_permlane32_swap(neg, neg, false, false);
        return ~(both[0] | (both[1] << 16));
    };

    const int nblocks = (count + 63) >> 6;
    const int stride = gridDim.x * NW;
    int blk = blockIdx.x * NW + wave;
    if (blk < nblocks) load_keys(blk * 64);
    for (; blk < nblocks; blk += stride) {
        const int r0 = blk * 64;
        const int64_t prow = key_row(r0 + lane);        // the key this lane packs
        const uint32_t turn = 10u * (uint32_t)((begin + r0 + lane) & 15);   // bits the string is rotated by
        uint4 head0 = make_uint4(0, 0, 0, 0);           // string 0, kept until string 1 is there too
        uint32_t tail0 = 0;
#pragma unroll 1
        for (int p = 0; p < NCB; ++p) {
            const int sub = p >= 5 ? 1 : 0, q = p - 5 * sub;
            const uint4 *af = wl + (p * KS) * 64 + lane;
            floatx16_t acc0, acc1;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc0[i] = acc1[i] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                union { uint4 u; bf16x8_t v; } fa;
                fa.u = af[ks * 64];
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, kf[0][ks], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.v, kf[1][ks], acc1, 0, 0, 0);
            }
            // ids of tables beyond the live ones stay zero: the string's first 10 nj bits are live
            const int nj = max(0, (ntab - sub + S - 1) / S);
            const int nlive = 10 * nj - 32 * q;
            const uint32_t live_mask = nlive >= 32 ? 0xffffffffu : nlive <= 0 ? 0u : (1u << nlive) - 1u;
            const uint32_t w0 = sign_word(acc0), w1 = sign_word(acc1);
            mybits[lane * 5 + q] = (lane < 32 ? w0 : w1) & live_mask;   // lane = key n or 32 + n
            if (q == 4) {
                uint32_t x0 = mybits[lane * 5], x1 = mybits[lane * 5 + 1], x2 = mybits[lane * 5 + 2];
                uint32_t x3 = mybits[lane * 5 + 3], x4 = mybits[lane * 5 + 4];
                // stored word k = bits [32 k + turn, +32) of the string, cyclically: words turned
                // by turn / 32, then a funnel shift by turn % 32
                const uint32_t wo = turn >> 5, sh = turn & 31;
                if (wo & 1) { const uint32_t t0 = x0; x0 = x1; x1 = x2; x2 = x3; x3 = x4; x4 = t0; }
                if (wo & 2) { const uint32_t t0 = x0, t1 = x1; x0 = x2; x1 = x3; x2 = x4; x3 = t0; x4 = t1; }
                if (wo & 4) { const uint32_t t4 = x4; x4 = x3; x3 = x2; x2 = x1; x1 = x0; x0 = t4; }
                uint4 o;
                o.x = __builtin_amdgcn_alignbit(x1, x0, sh);
                o.y = __builtin_amdgcn_alignbit(x2, x1, sh);
                o.z = __builtin_amdgcn_alignbit(x3, x2, sh);
                o.w = __builtin_amdgcn_alignbit(x4, x3, sh);
                const uint32_t ot = __builtin_amdgcn_alignbit(x0, x4, sh);
                if (S == 2 && sub == 0) {
                    head0 = o;
                    tail0 = ot;
                } else if (prow >= 0) {
                    // the strings of the key's group together: 16 S adjacent bytes of the tile's
                    // main rows and 4 S of its tail rows
                    uint4 *dst = (uint4 *)(Cb + packed_main_row(prow, grp, a.Lpad, GT));
                    if (S == 2) {
                        dst[0] = head0;
                        dst[1] = o;
                        *(uint2 *)(Cb + packed_tail_row(prow, grp, a.Lpad, GT)) = make_uint2(tail0, ot);
                    } else {
                        dst[0] = o;
                        *(uint32_t *)(Cb + packed_tail_row(prow, grp, a.Lpad, GT)) = ot;
                    }
                }
            }
        }
        if (blk + stride < nblocks) load_keys((blk + stride) * 64);
    }
}

template <typename T>
static int launch_rows(const HashArgs &a, int Hkv, int batch, int max_rows, hipStream_t st) {
    const int bw = 2 * ((a.LP + 63) / 64);
    if (max_rows <= 4) {
        constexpr int ROWS = 1;
        size_t lds = (size_t)ROWS * a.d * 4 + (size_t)ROWS * bw * 4 + (ROWS + 1) * 4 + ROWS * 8 + 16;
        dim3 grid(max_rows, Hkv, batch);
        hipLaunchKernelGGL((hash_rows_kernel<T, ROWS>), grid, dim3(256), lds, st, a);
    } else {
        constexpr int ROWS = 16;
        size_t lds = (size_t)ROWS * a.d * 4 + (size_t)ROWS * bw * 4 + (ROWS + 1) * 4 + ROWS * 8 + 16;
        dim3 grid((max_rows + ROWS - 1) / ROWS, Hkv, batch);
        hipLaunchKernelGGL((hash_rows_kernel<T, ROWS>), grid, dim3(256), lds, st, a);
    }
    return SOCKET_OK;
}

// dynamic LDS of hash_mfma8_kernel: the W slab as fragments, one id-word row per key of every wavefront's block
template <int D, int S, int P> constexpr size_t hash8_lds() {
    return (size_t)(P / 2 * S) * (D / 16) * 64 * 16 + (size_t)(kHash8Threads / 64) * 64 * 16;
}

template <int D, int S> constexpr size_t hash10_lds() {
    return (size_t)(5 * S) * (D / 16) * 64 * 16 + (size_t)(kHash8Threads / 64) * 64 * 20;
}

// once per context that uses a fast hash: more than 64 KB of dynamic LDS has to be allowed
// before the first launch
int hash_prepare(int d) {
    hipError_t e = hipSuccess;
    if (d == 128) e = hipFuncSetAttribute((const void *)hash_mfma10_kernel<128, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hash10_lds<128, 2>());
    if (e != hipSuccess) return SOCKET_EHIP;
    if (d == 64) e = hipFuncSetAttribute((const void *)hash_mfma8_kernel<64, 4, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hash8_lds<64, 4, 8>());
    if (d == 128) e = hipFuncSetAttribute((const void *)hash_mfma8_kernel<128, 4, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hash8_lds<128, 4, 8>());
    if (e == hipSuccess && d == 128) e = hipFuncSetAttribute((const void *)hash_mfma8_kernel<128, 2, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hash8_lds<128, 2, 8>());
    if (e == hipSuccess && d == 128) e = hipFuncSetAttribute((const void *)hash_mfma8_kernel<128, 4, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)hash8_lds<128, 4, 4>());
    return e == hipSuccess ? SOCKET_OK : SOCKET_EHIP;
}

template <int D, int S, int P>
static int launch_mfma8(HashArgs a, uint4 *wfrag, int Hkv, int batch, int max_rows, hipStream_t st) {
    constexpr int NW = kHash8Threads / 64;
    a.tables_per_chunk = 16 * S;
    a.n_chunks = S == 4 ? (a.L + 63) / 64 : 1;
    // W as MFMA fragments, once per call
    hipLaunchKernelGGL((hash_wfrag_kernel<D, S, P>), dim3(P / 2 * S, Hkv * a.n_chunks), dim3(256), 0, st, a, wfrag);
    // one workgroup per CU (the W slab fills most of its LDS); each wavefront takes 64-key blocks
    int per = 256 / (Hkv * a.n_chunks * batch);
    const int nblocks = (max_rows + 63) / 64;
    if (per > (nblocks + NW - 1) / NW) per = (nblocks + NW - 1) / NW;
    if (per < 1) per = 1;
    dim3 grid(per, Hkv * a.n_chunks, batch);
    constexpr size_t lds = hash8_lds<D, S, P>();
    hipLaunchKernelGGL((hash_mfma8_kernel<D, S, P>), grid, dim3(kHash8Threads), lds, st, a, (const uint4 *)wfrag);
    return SOCKET_OK;
}
template <int D, int P>
static int launch_mfma8(HashArgs a, uint4 *wfrag, int Hkv, int batch, int max_rows, hipStream_t st) {
    return a.S == 4 ? launch_mfma8<D, 4, P>(a, wfrag, Hkv, batch, max_rows, st)
         : a.S == 2 ? launch_mfma8<D, 2, P>(a, wfrag, Hkv, batch, max_rows, st)
                    : launch_mfma8<D, 1, P>(a, wfrag, Hkv, batch, max_rows, st);
}
template <int D>
static int launch_mfma8(HashArgs a, uint4 *wfrag, int Hkv, int batch, int max_rows, hipStream_t st) {
    return a.P == 8 ? launch_mfma8<D, 8>(a, wfrag, Hkv, batch, max_rows, st)
                    : launch_mfma8<D, 4>(a, wfrag, Hkv, batch, max_rows, st);
}

template <int D, int S>
static int launch_mfma10(HashArgs a, uint4 *wfrag, int Hkv, int batch, int max_rows, hipStream_t st) {
    constexpr int NW = kHash8Threads / 64;
    a.tables_per_chunk = 16 * S;
    a.n_chunks = a.Lpad / (16 * S);            // groups, padding groups included (their ids are zero)
    hipLaunchKernelGGL((hash_wfrag10_kernel<D, S>), dim3(5 * S, Hkv * a.n_chunks), dim3(256), 0, st, a, wfrag);
    int per = 256 / (Hkv * a.n_chunks * batch);
    const int nblocks = (max_rows + 63) / 64;
    if (per > (nblocks + NW - 1) / NW) per = (nblocks + NW - 1) / NW;
    if (per < 1) per = 1;
    dim3 grid(per, Hkv * a.n_chunks, batch);
    constexpr size_t lds = hash10_lds<D, S>();
    hipLaunchKernelGGL((hash_mfma10_kernel<D, S>), grid, dim3(kHash8Threads), lds, st, a, (const uint4 *)wfrag);
    return SOCKET_OK;
}
template <int D>
static int launch_mfma10(HashArgs a, uint4 *wfrag, int Hkv, int batch, int max_rows, hipStream_t st) {
    return a.GT == 32 ? launch_mfma10<D, 2>(a, wfrag, Hkv, batch, max_rows, st)
                      : launch_mfma10<D, 1>(a, wfrag, Hkv, batch, max_rows, st);
}

template <int D>
static int launch_mfma(HashArgs a, int Hkv, int batch, int max_rows, hipStream_t st) {
    constexpr int TILE = 64, KSTRIDE = D * 2 + 16, BSTRIDE = 17;
    if (a.GT) {
        // packed ids: a workgroup owns whole groups of GT tables (the high bits of four ids
        // share a byte), padding groups included
        a.tables_per_chunk = a.GT;
        a.n_chunks = a.Lpad / a.GT;
    } else {
        a.tables_per_chunk = 512 / a.P;
        if (a.tables_per_chunk > a.L) a.tables_per_chunk = a.L;
        a.n_chunks = (a.L + a.tables_per_chunk - 1) / a.tables_per_chunk;
    }
    // rows per workgroup: enough workgroups to fill 256 CUs, at least 1024 rows each so the
    // one-time load of the W slab is amortised
    int64_t total = (int64_t)max_rows * Hkv * batch * a.n_chunks;
    int rows = (int)((total + 511) / 512);
    rows = (rows + TILE - 1) / TILE * TILE;
    if (rows < 1024) rows = 1024;
    a.rows_per_wg = rows;
    size_t lds = 2 * TILE * KSTRIDE + 2 * TILE * BSTRIDE * 4 + 4 * TILE * 4 + 3 * TILE * 8;
    dim3 grid((max_rows + rows - 1) / rows, Hkv * a.n_chunks, batch);
    hipLaunchKernelGGL((hash_mfma_kernel<D>), grid, dim3(512), lds, st, a);
    return SOCKET_OK;
}

int launch_hash_keys(socket_ctx *ctx, const void *K, const void *proj, const int32_t *block_table,
                     const int32_t *row_begin, const int32_t *row_count, int batch, int max_rows,
                     void *codes, hipStream_t st) {
    const Geometry &g = ctx->g;
    HashArgs a;
    a.K = K; a.W = proj; a.codes = codes; a.row_begin = row_begin; a.row_count = row_count;
    a.map = row_map(g, block_table);
    a.d = g.d; a.L = g.L; a.P = g.P; a.LP = g.L * g.P; a.Lpad = g.Lpad; a.S = g.S; a.cb = g.cb;
    a.GT = g.mode == kSplit ? g.GT : 0;
    a.rows_per_wg = 0; a.tables_per_chunk = g.L; a.n_chunks = 1;
    int rc;
    if (max_rows == 1) {
        // one appended key per sequence: the projection kernel with its W slab staged in LDS
        return launch_project(ctx, nullptr, proj, 1.0f, K, codes, block_table, row_begin, row_count,
                              nullptr, batch, st);
    } else if (g.kv_dtype == SOCKET_F32) {
        rc = launch_rows<float>(a, g.Hkv, batch, max_rows, st);
    } else if (max_rows < 64) {
        rc = launch_rows<uint16_t>(a, g.Hkv, batch, max_rows, st);
    } else {
        const bool fast8 = ctx->wfrag != nullptr && (g.P == 8 || g.P == 4);   // one-byte ids of 8 or 4 planes, d <= 128
        const bool fast10 = ctx->wfrag != nullptr && g.P == 10;    // packed ids in groups of 32 tables, d <= 128
        switch (g.d) {
            case 64: rc = fast8 ? launch_mfma8<64>(a, (uint4 *)ctx->wfrag, g.Hkv, batch, max_rows, st)
                          : fast10 ? launch_mfma10<64>(a, (uint4 *)ctx->wfrag, g.Hkv, batch, max_rows, st)
                                   : launch_mfma<64>(a, g.Hkv, batch, max_rows, st); break;
            case 128: rc = fast8 ? launch_mfma8<128>(a, (uint4 *)ctx->wfrag, g.Hkv, batch, max_rows, st)
                           : fast10 ? launch_mfma10<128>(a, (uint4 *)ctx->wfrag, g.Hkv, batch, max_rows, st)
                                    : launch_mfma<128>(a, g.Hkv, batch, max_rows, st); break;
            case 256: rc = launch_mfma<256>(a, g.Hkv, batch, max_rows, st); break;
            default: return SOCKET_EUNSUPPORTED;
        }
    }
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

// Alg. 1 (PrecomputeKeyHashes): sign random projections of cached keys, packed into bucket ids.
//
// Two kernels:
//   hash_mfma_kernel   bf16 keys, many rows: K[rows x d] * W[d x L*P] on bf16 MFMA
//                      (v_mfma_f32_32x32x16_bf16, fp32 accumulate), W held in registers,
//                      key tiles staged through LDS, sign bits taken from the accumulators'
//                      sign bit and packed into a per-key bit matrix in LDS.
//   hash_rows_kernel   fp32 keys, or a handful of appended rows: fp32 FMA, one thread per
//                      projection column, sign bits gathered with a wavefront ballot.
// Both end in pack_codes(), which cuts the bit matrix into P-bit bucket ids and writes them
// in the rotated order the scoring kernel reads.
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
    pack_codes(bits, bw, ROWS, tok, grow, a.codes, a.L, a.P, a.Lpad, a.S, a.cb, 0, a.L, true, tid, 256);
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA kernel.  512 threads = 8 waves; wave w owns projection columns
// [64w, 64w+64) of the workgroup's column chunk and keeps that slab of W in registers
// for the whole kernel.  The workgroup walks its rows in tiles of 64 keys.
// MFMA operands: A = W^T (32 planes x 16 channels), B = K^T (16 channels x 32 keys), so
// lane (key n, half g) of the accumulator holds planes 8a + 4g + b (a,b in 0..3) of key n.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512) void hash_mfma_kernel(HashArgs a) {
    constexpr int KS = D / 16;                 // MFMA k-steps
    constexpr int TILE = 64;                   // keys per tile
    constexpr int KSTRIDE = D * 2 + 16;        // bytes per staged key row (padded)
    constexpr int BSTRIDE = 17;                // words per bit row (16 + 1 pad)
    extern __shared__ uint32_t smem[];
    char *const kbase = (char *)smem;                  // two staged key tiles
    auto ktile = [&](int bf) { return kbase + bf * (TILE * KSTRIDE); };
    uint32_t *bits = smem + 2 * TILE * KSTRIDE / 4;   // [TILE][BSTRIDE]
    int *tok = (int *)(bits + TILE * BSTRIDE);        // [2][TILE]
    int64_t *grow = (int64_t *)(tok + 2 * TILE);      // [2][TILE]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.y % a.n_chunks, h = blockIdx.y / a.n_chunks, b = blockIdx.z;
    const int count = a.row_count[b];
    const int wg_r0 = blockIdx.x * a.rows_per_wg;
    if (wg_r0 >= count) return;
    const int wg_r1 = min(count, wg_r0 + a.rows_per_wg);
    const int begin = a.row_begin[b];

    const int first_table = chunk * a.tables_per_chunk;
    const int ntab = min(a.tables_per_chunk, a.L - first_table);
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

    auto fetch = [&](int tile_r0, int buf) {
        // resolve rows of this tile (first 64 threads), then load this thread's segment
        int r = tile_r0 + srow;
        int t = begin + r;
        bool live = r < wg_r1 && t >= 0 && t < a.map.max_n;
        int64_t g = live ? a.map.row(b, h, t) : -1;
        if (sseg == 0) {
            tok[buf * TILE + srow] = t;
            grow[buf * TILE + srow] = g;
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

    fetch(wg_r0, 0);
    commit(0);
    __syncthreads();

    int buf = 0;
    for (int tile_r0 = wg_r0; tile_r0 < wg_r1; tile_r0 += TILE, buf ^= 1) {
        const bool more = tile_r0 + TILE < wg_r1;
        if (more) fetch(tile_r0 + TILE, buf ^ 1);

        // ---- MFMA: acc[mb][nb] = W^T slab (32 planes) x K^T (32 keys)
        floatx16_t acc[2][2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8_t kf[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const char *src = ktile(buf) + (nb * 32 + (lane & 31)) * KSTRIDE + ks * 32 + (lane >> 5) * 16;
                kf[nb] = *(const bf16x8_t *)src;
            }
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag[mb][ks], kf[nb], acc[mb][nb], 0, 0, 0);
        }

        // ---- sign bits: accumulator i of lane (n, g) is plane 8*(i/4) + 4g + i%4.
        //      Funnel-shift the 16 sign bits into one 16-bit value per lane, exchange with
        //      the other half-wave, and interleave nibbles into the 32 planes of the block.
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                uint32_t neg = __float_as_uint(acc[mb][nb][15]) >> 31;
#pragma unroll
                for (int i = 14; i >= 0; --i)
                    neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[mb][nb][i]), 31);
                neg &= 0xffffu;                         // bit 4a+b = sign of plane 8a+4g+b
                uint32_t other = __shfl_xor((int)neg, 32);
                uint32_t lo = (lane < 32) ? neg : other, hi = (lane < 32) ? other : neg;
                lo = (lo | (lo << 8)) & 0x00ff00ffu;
                lo = (lo | (lo << 4)) & 0x0f0f0f0fu;
                hi = (hi | (hi << 8)) & 0x00ff00ffu;
                hi = (hi | (hi << 4)) & 0x0f0f0f0fu;
                uint32_t word = ~(lo | (hi << 4));      // bit p = 1 when plane p projects >= 0
                if (lane < 32) bits[(nb * 32 + lane) * BSTRIDE + wave * 2 + mb] = word;
            }
        }
        __syncthreads();   // bit matrix complete; every wave is done reading this key tile

        const bool whole = a.n_chunks == 1 || (a.tables_per_chunk & 63) == 0;
        pack_codes(bits, BSTRIDE, TILE, tok + buf * TILE, grow + buf * TILE, a.codes, a.L, a.P,
                   a.Lpad, a.S, a.cb, first_table, ntab, whole, tid, 512);
        if (more) commit(buf ^ 1);
        __syncthreads();   // next tile staged; bit matrix free again
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

template <int D>
static int launch_mfma(HashArgs a, int Hkv, int batch, int max_rows, hipStream_t st) {
    constexpr int TILE = 64, KSTRIDE = D * 2 + 16, BSTRIDE = 17;
    a.tables_per_chunk = 512 / a.P;
    if (a.tables_per_chunk > a.L) a.tables_per_chunk = a.L;
    a.n_chunks = (a.L + a.tables_per_chunk - 1) / a.tables_per_chunk;
    // rows per workgroup: enough workgroups to fill 256 CUs, at least 1024 rows each so the
    // one-time load of the W slab is amortised
    int64_t total = (int64_t)max_rows * Hkv * batch * a.n_chunks;
    int rows = (int)((total + 511) / 512);
    rows = (rows + TILE - 1) / TILE * TILE;
    if (rows < 1024) rows = 1024;
    a.rows_per_wg = rows;
    size_t lds = 2 * TILE * KSTRIDE + TILE * BSTRIDE * 4 + 2 * TILE * 4 + 2 * TILE * 8;
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
    a.map = RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks};
    a.d = g.d; a.L = g.L; a.P = g.P; a.LP = g.L * g.P; a.Lpad = g.Lpad; a.S = g.S; a.cb = g.cb;
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
        switch (g.d) {
            case 64: rc = launch_mfma<64>(a, g.Hkv, batch, max_rows, st); break;
            case 128: rc = launch_mfma<128>(a, g.Hkv, batch, max_rows, st); break;
            case 256: rc = launch_mfma<256>(a, g.Hkv, batch, max_rows, st); break;
            default: return SOCKET_EUNSUPPORTED;
        }
    }
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

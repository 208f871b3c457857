// Eq. 2: exact softmax attention restricted to the selected tokens (Eq. 1 when every token is
// selected).  Split-K flash-decode: the selected rows of one (sequence, KV head) are divided
// among n_split workgroups; each gathers its K rows once for all G query heads of the group,
// keeps a running (max, sum, weighted value sum) per query head in fp32 over the gathered
// K and V rows, and writes one partial result per split; a second small kernel merges them.
// Logits use no 1/sqrt(d) unless the caller passes one as `scale`; with unit-variance data
// they reach +-100, so everything is max-subtracted.
#include "socket_internal.h"

namespace sk {

#ifdef SK_DEBUG_CLOCKS
__device__ long long sk_dbg3[64];
#define SK_STAMP3(i) do { if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0) sk_dbg3[i] = wall_clock64(); } while (0)
extern "C" int socket_debug_clocks3(long long *out) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(sk_dbg3), sizeof(long long) * 64);
}
#else
#define SK_STAMP3(i) ((void)0)
#endif

struct DecodeArgs {
    const void *q;
    const void *K;
    const void *V;
    const int32_t *idx;
    const int32_t *n_selected;
    float *partials;
    uint32_t *counters;
    void *out;
    RowMap map;
    float scale;
    int Hq, max_k, n_split, out_dtype;
    const int32_t *seq_len;   // dense variant only
};

// two adjacent elements of an LDS row as floats
__device__ __forceinline__ float2 pair_f32(const uint16_t *p) {
    const uint32_t w = *(const uint32_t *)p;
    return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}
__device__ __forceinline__ float2 pair_f32(const float *p) { return *(const float2 *)p; }

// DENSE = false: the rows are the selected tokens idx[...] (Eq. 2).  DENSE = true: the rows
// are all tokens below seq_len (Eq. 1), each split takes a contiguous range of them, and the
// next chunk's rows are loaded while the current chunk is worked on.
template <typename T, int D, int G, bool DENSE>
__global__ __launch_bounds__(kDecodeThreads) void sparse_decode_kernel(DecodeArgs a) {
    constexpr int LPR = D / 8;                       // lanes per row
    constexpr int RPW = 64 / LPR;                    // rows per wavefront pass
    constexpr int NWAVE = kDecodeThreads / 64;
    constexpr int RPP = NWAVE * RPW;                 // rows per workgroup pass
    constexpr int CH = kDecodeChunk;
    constexpr int NPASS = CH / RPP;
    static_assert(CH % RPP == 0, "chunk must be whole passes");
    // The value rows of a chunk go through LDS (at most 32 KB at a time), where every thread
    // owns two adjacent output channels of GPG query heads and walks the rows itself: no
    // cross-lane sums in the value product.
    constexpr int ROWB = D * (int)sizeof(T);
    constexpr int VROWS = CH * ROWB <= 32768 ? CH : 32768 / ROWB;
    constexpr int VROUNDS = CH / VROWS, PPR = VROWS / RPP;      // passes per round
    static_assert(VROWS % RPP == 0 && VROWS % 4 == 0, "a round is whole passes");
    constexpr int CPAIRS = D / 2;                    // channel pairs
    constexpr int NG = kDecodeThreads / CPAIRS;      // thread groups, each covering all channels
    constexpr int GPG = (G + NG - 1) / NG;           // query heads per group

    __shared__ __align__(16) float s_p[G][CH];       // logits, then softmax numerators
    __shared__ int64_t s_row[CH];                    // K/V row of each chunk entry (-1 = none)
    __shared__ float s_m[G], s_l[G], s_corr[G];
    __shared__ __align__(16) T s_v[VROWS][D];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int bh = b * a.map.Hkv + h;
    const int sub = lane % LPR, rl = lane / LPR;     // this lane's 8-element slice and row slot
    const int cp = tid % CPAIRS, g0 = (tid / CPAIRS) * GPG;   // this thread's channel pair and first query head
    const float ninf = -__builtin_inff();

    // Splits own fixed slices of the max_k-long index row, so the index loads do not have to
    // wait for the selected count; entries at or beyond the count are ignored.  (Dense: whole
    // chunks of the sequence.)
    int total = a.max_k;
    if (DENSE) {
        total = a.seq_len[b];
        total = total < 0 ? 0 : (total > a.map.max_n ? a.map.max_n : total);
    }
    const int per = DENSE ? (((total + CH - 1) / CH + a.n_split - 1) / a.n_split) * CH
                          : (total + a.n_split - 1) / a.n_split;
    const int r_begin = split * per;
    const int r_end = min(total, r_begin + per);
    const int32_t *idx = DENSE ? nullptr : a.idx + (int64_t)bh * a.max_k;

    SK_STAMP3(0);
    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        Row8<T> r;
        r.load((const T *)a.q + ((int64_t)b * a.Hq + h * G + g) * D + sub * 8);
        r.get(qf[g]);
    }
    float acc[GPG][2];
#pragma unroll
    for (int gg = 0; gg < GPG; ++gg) acc[gg][0] = acc[gg][1] = 0.0f;
    if (tid < G) {
        s_m[tid] = ninf;
        s_l[tid] = 0.0f;
    }
    __syncthreads();

    Row8<T> kr[NPASS], vr[NPASS], kn[NPASS], vn[NPASS];
    int64_t rows[NPASS], rown[NPASS];
    // dense: this lane's rows of the chunk starting at c0, straight from the token positions
    auto load_dense = [&](int c0, Row8<T> *kd, Row8<T> *vd, int64_t *rd) {
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int t = c0 + p * RPP + wave * RPW + rl;
            rd[p] = t < r_end ? a.map.row(b, h, t) : -1;
            if (rd[p] >= 0) {
                kd[p].load((const T *)a.K + rd[p] * D + sub * 8);
                vd[p].load((const T *)a.V + rd[p] * D + sub * 8);
            } else {
                kd[p].zero();
                vd[p].zero();
            }
        }
    };
    if (DENSE && r_begin < r_end) load_dense(r_begin, kr, vr, rows);

    for (int c0 = r_begin; c0 < r_end; c0 += CH) {
        if (DENSE) {
            if (c0 + CH < r_end) load_dense(c0 + CH, kn, vn, rown);
        } else {
            // ---- rows of this chunk
            if (tid < CH) {
                int r = c0 + tid;
                int64_t row = -1;
                if (r < r_end) {
                    int t = idx[r];
                    int nsel = a.n_selected[bh];
                    if (r < nsel && t >= 0 && t < a.map.max_n) row = a.map.row(b, h, t);
                }
                s_row[tid] = row;
            }
            __syncthreads();
            SK_STAMP3(1);

            // ---- gather this chunk's K and V rows together (one memory latency, not two)
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                rows[p] = s_row[p * RPP + wave * RPW + rl];
                if (rows[p] >= 0) {
                    kr[p].load((const T *)a.K + rows[p] * D + sub * 8);
                    vr[p].load((const T *)a.V + rows[p] * D + sub * 8);
                } else {
                    kr[p].zero();
                    vr[p].zero();
                }
            }
        }
        // ---- logits: scale * k.q for every query head of the group
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            if (p == 0) SK_STAMP3(2);
            float kf[8];
            kr[p].get(kf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float dot = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(kf[e], qf[g][e], dot);
                dot = row_sum<LPR>(dot);
                if (sub == 0) s_p[g][p * RPP + wave * RPW + rl] = rows[p] >= 0 ? dot * a.scale : ninf;
            }
        }
        if (VROUNDS == 1) {                          // the value rows ride along with the logits
#pragma unroll
            for (int p = 0; p < NPASS; ++p) vr[p].store(&s_v[p * RPP + wave * RPW + rl][sub * 8]);
        }
        __syncthreads();
        SK_STAMP3(3);

        // ---- running softmax statistics, one wavefront per query head at a time
        for (int g = wave; g < G; g += NWAVE) {
            const float v = s_p[g][lane];            // CH == 64 == wavefront size
            const float m_old = s_m[g];
            const float m_new = fmaxf(m_old, wave_max(v));
            const float p = (v == ninf) ? 0.0f : expf(v - m_new);
            const float sum = row_sum<64>(p);
            const float corr = (m_old == ninf) ? 0.0f : expf(m_old - m_new);
            s_p[g][lane] = p;
            if (lane == 0) {
                s_m[g] = m_new;
                s_l[g] = s_l[g] * corr + sum;
                s_corr[g] = corr;
            }
        }
        __syncthreads();
        SK_STAMP3(4);

        // ---- weighted value rows
#pragma unroll
        for (int gg = 0; gg < GPG; ++gg) {
            if (g0 + gg < G) {
                const float corr = s_corr[g0 + gg];
                acc[gg][0] *= corr;
                acc[gg][1] *= corr;
            }
        }
#pragma unroll
        for (int round = 0; round < VROUNDS; ++round) {
            if (VROUNDS > 1) {
                if (round > 0) __syncthreads();      // the previous round's rows have been consumed
#pragma unroll
                for (int p = 0; p < PPR; ++p)
                    vr[round * PPR + p].store(&s_v[p * RPP + wave * RPW + rl][sub * 8]);
                __syncthreads();
            }
            if (g0 < G) {
                constexpr int RB = 16;               // rows whose LDS reads are issued together
                static_assert(VROWS % RB == 0, "whole row batches");
                for (int r = 0; r < VROWS; r += RB) {
                    float2 v2[RB];
#pragma unroll
                    for (int j = 0; j < RB; ++j) v2[j] = pair_f32(&s_v[r + j][2 * cp]);
#pragma unroll
                    for (int gg = 0; gg < GPG; ++gg) {
                        if (g0 + gg < G) {
                            float4 w[RB / 4];
#pragma unroll
                            for (int j = 0; j < RB / 4; ++j) w[j] = *(const float4 *)&s_p[g0 + gg][round * VROWS + r + 4 * j];
#pragma unroll
                            for (int j = 0; j < RB / 4; ++j) {
                                acc[gg][0] = fmaf(w[j].x, v2[4 * j].x, acc[gg][0]);
                                acc[gg][1] = fmaf(w[j].x, v2[4 * j].y, acc[gg][1]);
                                acc[gg][0] = fmaf(w[j].y, v2[4 * j + 1].x, acc[gg][0]);
                                acc[gg][1] = fmaf(w[j].y, v2[4 * j + 1].y, acc[gg][1]);
                                acc[gg][0] = fmaf(w[j].z, v2[4 * j + 2].x, acc[gg][0]);
                                acc[gg][1] = fmaf(w[j].z, v2[4 * j + 2].y, acc[gg][1]);
                                acc[gg][0] = fmaf(w[j].w, v2[4 * j + 3].x, acc[gg][0]);
                                acc[gg][1] = fmaf(w[j].w, v2[4 * j + 3].y, acc[gg][1]);
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
        if (DENSE) {
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                kr[p] = kn[p];
                vr[p] = vn[p];
                rows[p] = rown[p];
            }
        }
    }

    SK_STAMP3(5);
    // ---- this split's partial result: (max, sum, weighted value sum) per query head
    float *part = a.partials + ((int64_t)(b * a.Hq + h * G) * a.n_split) * (D + 2);
#pragma unroll
    for (int gg = 0; gg < GPG; ++gg) {
        const int g = g0 + gg;
        if (g < G)
            *(float2 *)&part[((int64_t)g * a.n_split + split) * (D + 2) + 2 + 2 * cp] = make_float2(acc[gg][0], acc[gg][1]);
    }
    if (tid < G) {
        part[((int64_t)tid * a.n_split + split) * (D + 2) + 0] = s_m[tid];
        part[((int64_t)tid * a.n_split + split) * (D + 2) + 1] = s_l[tid];
    }
    SK_STAMP3(6);
}

// Merge of the split-K partial results of one query head: out = sum_s w_s acc_s / sum_s w_s l_s
// with w_s = exp(m_s - max m).  One workgroup per query head, one thread per output channel;
// every load of a thread is issued before the first use, so the kernel costs one memory
// latency.  Runs as a kernel of its own after the partial pass: no fence, no signalling.
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(DecodeArgs a) {
    __shared__ float s_w[64];
    __shared__ float s_den;
    const int c = threadIdx.x, g = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int G = a.Hq / a.map.Hkv;
    const int64_t head = (int64_t)b * a.Hq + h * G + g;
    const float *part = a.partials + head * a.n_split * (D + 2);
    const float ninf = -__builtin_inff();
    // the first wavefront weighs the splits: its (max, sum) loads go out first, so that the
    // weights are ready when the value sums arrive
    const bool live = c < 64 && c < a.n_split;
    const float m = live ? part[(int64_t)c * (D + 2)] : ninf;
    const float l = live ? part[(int64_t)c * (D + 2) + 1] : 0.0f;
    float acc[64];
#pragma unroll
    for (int s = 0; s < 64; ++s) acc[s] = s < a.n_split ? part[(int64_t)s * (D + 2) + 2 + c] : 0.0f;
    if (c < 64) {
        const float top = wave_max(m);
        const float w = (m == ninf) ? 0.0f : expf(m - top);
        const float den = row_sum<64>(w * l);
        s_w[c] = w;
        if (c == 0) s_den = den;
    }
    __syncthreads();
    float num = 0.0f;
#pragma unroll
    for (int s = 0; s < 64; ++s)
        if (s < a.n_split) num = fmaf(s_w[s], acc[s], num);
    const float den = s_den;
    const float y = den > 0.0f ? num / den : 0.0f;
    if (a.out_dtype == SOCKET_F32) ((float *)a.out)[head * D + c] = y;
    else ((uint16_t *)a.out)[head * D + c] = f32_to_bf16_rne(y);
}

template <typename T, int D, bool DENSE>
static int launch_decode_g(const DecodeArgs &a, int G, dim3 grid, hipStream_t st) {
    switch (G) {
        case 1: hipLaunchKernelGGL((sparse_decode_kernel<T, D, 1, DENSE>), grid, dim3(kDecodeThreads), 0, st, a); break;
        case 2: hipLaunchKernelGGL((sparse_decode_kernel<T, D, 2, DENSE>), grid, dim3(kDecodeThreads), 0, st, a); break;
        case 4: hipLaunchKernelGGL((sparse_decode_kernel<T, D, 4, DENSE>), grid, dim3(kDecodeThreads), 0, st, a); break;
        case 8: hipLaunchKernelGGL((sparse_decode_kernel<T, D, 8, DENSE>), grid, dim3(kDecodeThreads), 0, st, a); break;
        default: return SOCKET_EUNSUPPORTED;
    }
    return SOCKET_OK;
}

template <typename T, bool DENSE>
static int launch_decode_d(const DecodeArgs &a, int D, int G, dim3 grid, hipStream_t st) {
    switch (D) {
        case 64: return launch_decode_g<T, 64, DENSE>(a, G, grid, st);
        case 128: return launch_decode_g<T, 128, DENSE>(a, G, grid, st);
        case 256: return launch_decode_g<T, 256, DENSE>(a, G, grid, st);
        default: return SOCKET_EUNSUPPORTED;
    }
}

static int launch_merge(const DecodeArgs &a, const Geometry &g, int batch, hipStream_t st) {
    dim3 mgrid(g.G, g.Hkv, batch);
    switch (g.d) {
        case 64: hipLaunchKernelGGL(decode_merge_kernel<64>, mgrid, dim3(64), 0, st, a); break;
        case 128: hipLaunchKernelGGL(decode_merge_kernel<128>, mgrid, dim3(128), 0, st, a); break;
        case 256: hipLaunchKernelGGL(decode_merge_kernel<256>, mgrid, dim3(256), 0, st, a); break;
        default: return SOCKET_EUNSUPPORTED;
    }
    return SOCKET_OK;
}

// Eq. 1: every token below seq_len, 64 splits per (sequence, KV head)
int launch_dense_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const int32_t *block_table, const int32_t *seq_len, int batch, float scale,
                        int out_dtype, void *out, hipStream_t st) {
    const Geometry &g = ctx->g;
    DecodeArgs a;
    a.q = q; a.K = K; a.V = V; a.idx = nullptr; a.n_selected = nullptr; a.seq_len = seq_len;
    a.partials = ctx->partials; a.counters = ctx->counters; a.out = out;
    a.map = RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks};
    a.scale = scale; a.Hq = g.Hq; a.max_k = g.max_k; a.n_split = kDenseSplits; a.out_dtype = out_dtype;
    dim3 grid(kDenseSplits, g.Hkv, batch);
    int rc = g.kv_dtype == SOCKET_F32 ? launch_decode_d<float, true>(a, g.d, g.G, grid, st)
                                      : launch_decode_d<uint16_t, true>(a, g.d, g.G, grid, st);
    if (rc != SOCKET_OK) return rc;
    rc = launch_merge(a, g, batch, st);
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

int launch_sparse_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                         const int32_t *idx, const int32_t *n_selected, const int32_t *block_table,
                         int batch, float scale, int out_dtype, void *out, hipStream_t st) {
    const Geometry &g = ctx->g;
    DecodeArgs a;
    a.q = q; a.K = K; a.V = V; a.idx = idx; a.n_selected = n_selected;
    a.partials = ctx->partials; a.counters = ctx->counters; a.out = out;
    a.map = RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks};
    a.scale = scale; a.Hq = g.Hq; a.max_k = g.max_k; a.n_split = g.n_split; a.out_dtype = out_dtype;
    a.seq_len = nullptr;
    dim3 grid(g.n_split, g.Hkv, batch);
    int rc = g.kv_dtype == SOCKET_F32 ? launch_decode_d<float, false>(a, g.d, g.G, grid, st)
                                      : launch_decode_d<uint16_t, false>(a, g.d, g.G, grid, st);
    if (rc != SOCKET_OK) return rc;
    rc = launch_merge(a, g, batch, st);
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

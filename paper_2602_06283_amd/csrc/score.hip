// Alg. 2 (SoftBucketProbs) and Alg. 5 (SoftHashCollisionScores, the soft score of Eq. 3).
//
//   soft_hash_kernel  builds, per (sequence, KV head), the table of bucket probabilities of
//                     the G queries that share the head.  Evaluated in fp64 and stored as
//                     fp32.  A softmax over the corners of {+-1}^P factorises over the
//                     planes, p(r) = prod_i sigmoid(+-2 u_i / tau), which is the form used.
//   score_kernel      loads that table into LDS and streams the bucket ids of every key
//                     once: 64/S keys per wavefront pass, S lanes per key, each lane reading
//                     16 ids with one 16-byte load.  The rotated id order (see socket.h)
//                     makes the 64 lanes of a pass hit 64 different tables, and the table is
//                     stored [bucket][table], so the LDS gathers are free of bank conflicts.
#include "socket_internal.h"

namespace sk {

struct SoftHashArgs {
    const void *q;
    const void *W;
    float *tables;
    double tau;
    int d, G, Hkv, Hq, L, P, LP, Lpad, rounds, R, mode, Plo, Phi, Rlo, Rhi, table_rows;
    int64_t table_words;
    int kv_dtype;
};

constexpr int kTablesPerWg = 8;

__device__ __forceinline__ double sigmoid64(double x) { return 1.0 / (1.0 + exp(-x)); }

__global__ __launch_bounds__(256) void soft_hash_kernel(SoftHashArgs a) {
    extern __shared__ double sm64[];
    const int tid = threadIdx.x;
    const int h = blockIdx.y, b = blockIdx.z;
    const int t0 = blockIdx.x * kTablesPerWg;               // first table of this workgroup
    double *qd = sm64;                                       // [G][d]
    double *sp = qd + a.G * a.d;                             // [G][8][P] sigmoid(+2u/tau)
    double *sn = sp + a.G * kTablesPerWg * a.P;              // [G][8][P] sigmoid(-2u/tau)

    for (int i = tid; i < a.G * a.d; i += 256) {
        int g = i / a.d, c = i - g * a.d;
        int64_t at = ((int64_t)b * a.Hq + h * a.G + g) * a.d + c;
        qd[i] = a.kv_dtype == SOCKET_F32 ? (double)((const float *)a.q)[at]
                                         : (double)bf16_to_f32(((const uint16_t *)a.q)[at]);
    }
    __syncthreads();

    const int cols = kTablesPerWg * a.P;
    const double inv_sqrt_d = 1.0 / sqrt((double)a.d);
    for (int i = tid; i < a.G * cols; i += 256) {
        int g = i / cols, j = i - g * cols;
        int tl = j / a.P, pl = j - tl * a.P;
        int l = t0 + tl;
        double plus = 0.0, minus = 0.0;
        if (l < a.L) {
            int64_t col = (int64_t)l * a.P + pl;
            double z = 0.0;
            if (a.kv_dtype == SOCKET_F32) {
                const float *W = (const float *)a.W + (int64_t)h * a.d * a.LP;
                for (int c = 0; c < a.d; ++c) z += (double)W[(int64_t)c * a.LP + col] * qd[g * a.d + c];
            } else {
                const uint16_t *W = (const uint16_t *)a.W + (int64_t)h * a.d * a.LP;
                for (int c = 0; c < a.d; ++c)
                    z += (double)bf16_to_f32(W[(int64_t)c * a.LP + col]) * qd[g * a.d + c];
            }
            double u = tanh(z) * inv_sqrt_d;
            plus = sigmoid64(2.0 * u / a.tau);
            minus = sigmoid64(-2.0 * u / a.tau);
        }
        sp[(g * kTablesPerWg + tl) * a.P + pl] = plus;
        sn[(g * kTablesPerWg + tl) * a.P + pl] = minus;
    }
    __syncthreads();

    const int lw = a.Lpad < 64 ? a.Lpad : 64;        // distinct tables per 64-word row
    const int copies = 64 / lw;
    float *T = a.tables + ((int64_t)b * a.Hkv + h) * a.table_words;
    if (a.mode == kDirect) {
        for (int i = tid; i < kTablesPerWg * a.R; i += 256) {
            int tl = i % kTablesPerWg, r = i / kTablesPerWg;
            int l = t0 + tl;
            if (l >= a.Lpad) continue;
            double mean = 0.0;
            if (l < a.L) {
                for (int g = 0; g < a.G; ++g) {
                    double p = 1.0;
                    for (int pl = 0; pl < a.P; ++pl) {
                        int at = (g * kTablesPerWg + tl) * a.P + pl;
                        p *= ((r >> pl) & 1) ? sp[at] : sn[at];
                    }
                    mean += p;
                }
                mean /= (double)a.G;
            }
            int c = l >> 6, lp = l & 63;
            for (int cp = 0; cp < copies; ++cp)
                T[((int64_t)c * a.R + r) * 64 + lp + cp * lw] = (float)mean;
        }
    } else {
        const int rows = a.Rlo + a.Rhi;
        for (int i = tid; i < kTablesPerWg * rows * a.G; i += 256) {
            int tl = i % kTablesPerWg, rest = i / kTablesPerWg;
            int row = rest % rows, g = rest / rows;
            int l = t0 + tl;
            if (l >= a.Lpad) continue;
            double p = 0.0;
            if (l < a.L) {
                if (row < a.Rlo) {
                    p = 1.0 / (double)a.G;      // the 1/G of the group mean rides on the low factor
                    for (int pl = 0; pl < a.Plo; ++pl) {
                        int at = (g * kTablesPerWg + tl) * a.P + pl;
                        p *= ((row >> pl) & 1) ? sp[at] : sn[at];
                    }
                } else {
                    int rh = row - a.Rlo;
                    p = 1.0;
                    for (int pl = 0; pl < a.Phi; ++pl) {
                        int at = (g * kTablesPerWg + tl) * a.P + a.Plo + pl;
                        p *= ((rh >> pl) & 1) ? sp[at] : sn[at];
                    }
                }
            }
            int c = l >> 6, lp = l & 63;
            for (int cp = 0; cp < copies; ++cp)
                T[(((int64_t)g * a.rounds + c) * rows + row) * 64 + lp + cp * lw] = (float)p;
        }
    }
}

// ---------------------------------------------------------------------------------------

struct ScoreArgs {
    const void *codes;
    const float *tables;
    const float *vnorm;
    const int32_t *seq_len;
    float *scores;
    RowMap map;
    int Lpad, rounds, R, G, Plo, Rlo, table_rows;
    int64_t table_words;
    int keys_per_wg;
};

// 16 bucket ids of one lane: CB = 1 -> 16 bytes, CB = 2 -> 32 bytes.
template <int CB> struct CodeVec;
template <> struct CodeVec<1> {
    uint4 v;
    __device__ __forceinline__ void load(const void *p) { v = *(const uint4 *)p; }
    __device__ __forceinline__ uint32_t word(int j) const { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }
    __device__ __forceinline__ uint32_t code(int s) const { return (word(s >> 2) >> (8 * (s & 3))) & 0xffu; }
};
template <> struct CodeVec<2> {
    uint4 v[2];
    __device__ __forceinline__ void load(const void *p) { v[0] = ((const uint4 *)p)[0]; v[1] = ((const uint4 *)p)[1]; }
    __device__ __forceinline__ uint32_t word(int j) const {
        const uint4 &q = v[j >> 2];
        int k = j & 3;
        return k == 0 ? q.x : k == 1 ? q.y : k == 2 ? q.z : q.w;
    }
    __device__ __forceinline__ uint32_t code(int s) const { return (word(s >> 1) >> (16 * (s & 1))) & 0xffffu; }
};

template <int S, int CB, int MODE, bool ONE_ROUND>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(ScoreArgs a) {
    extern __shared__ float tbl[];
    constexpr int KPW = 64 / S;                      // keys per wavefront pass
    constexpr int NW = kScoreThreads / 64;
    constexpr int U = 4;                             // passes in flight per wavefront
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * a.map.Hkv + h;
    const int key0 = blockIdx.x * a.keys_per_wg;
    const int key1 = min(key0 + a.keys_per_wg, a.map.max_n);
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > a.map.max_n ? a.map.max_n : seq);
    float *out = a.scores + bh * a.map.max_n;
    const float ninf = -__builtin_inff();

    if (key0 >= seq) {                               // nothing valid here: only the -inf fill
        for (int k = key0 + tid; k < key1; k += kScoreThreads) out[k] = ninf;
        return;
    }

    {   // bucket-probability table -> LDS
        const float4 *src = (const float4 *)(a.tables + bh * a.table_words);
        float4 *dst = (float4 *)tbl;
        for (int i = tid; i < (int)(a.table_words >> 2); i += kScoreThreads) dst[i] = src[i];
    }

    const int sub = lane % S, kk = lane / S;
    const int lw = a.Lpad < 64 ? a.Lpad : 64;
    uint32_t woff[16];                               // byte offset of this lane's table within a 64-float row
#pragma unroll
    for (int s = 0; s < 16; ++s) woff[s] = 4u * (uint32_t)(sub + S * ((kk + s) & 15) + lw * (kk >> 4));
    const float *vn = a.vnorm ? a.vnorm + bh * a.map.max_n : nullptr;
    __syncthreads();

    const int span = NW * KPW;                       // keys per workgroup pass
    for (int base0 = key0 + wave * KPW; base0 < key1; base0 += U * span) {
        CodeVec<CB> cv[U];
        bool live[U];
        float sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int key = base0 + u * span + kk;
            live[u] = key < seq;
            sum[u] = 0.0f;
        }
        for (int c = 0; c < (ONE_ROUND ? 1 : a.rounds); ++c) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int key = base0 + u * span + kk;
                int64_t row = live[u] ? a.map.row(b, h, key) : -1;
                if (row < 0) live[u] = false;
                if (live[u])
                    cv[u].load((const char *)a.codes + (row * a.Lpad + c * 64 + sub * 16) * CB);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!live[u]) continue;
                float acc = 0.0f;
                if (MODE == kDirect) {
                    const char *T = (const char *)tbl + (size_t)c * a.R * 256;
#pragma unroll
                    for (int s = 0; s < 16; ++s) {
                        uint32_t addr;
                        if (CB == 1) {
                            // byte 0 <- woff, byte 1 <- id: address = id*256 + woff
                            addr = __builtin_amdgcn_perm(cv[u].word(s >> 2), woff[s], 0x0c0c0400u + ((uint32_t)(s & 3) << 8));
                        } else {
                            addr = (cv[u].code(s) << 8) | woff[s];
                        }
                        acc += *(const float *)(T + addr);
                    }
                } else {
                    for (int g = 0; g < a.G; ++g) {
                        const char *T = (const char *)tbl + ((size_t)(g * a.rounds + c) * a.table_rows) * 256;
                        float part = 0.0f;
#pragma unroll
                        for (int s = 0; s < 16; ++s) {
                            uint32_t code = cv[u].code(s);
                            uint32_t lo = code & (uint32_t)(a.Rlo - 1), hi = code >> a.Plo;
                            float pa = *(const float *)(T + ((lo << 8) | woff[s]));
                            float pb = *(const float *)(T + (((uint32_t)a.Rlo + hi) << 8 | woff[s]));
                            part = fmaf(pa, pb, part);
                        }
                        acc += part;
                    }
                }
                sum[u] += acc;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float v = sum[u];
            if (S >= 2) v += __shfl_xor(v, 1);
            if (S >= 4) v += __shfl_xor(v, 2);
            const int key = base0 + u * span + kk;
            if (sub == 0 && key < key1) {
                if (live[u]) out[key] = vn ? v * vn[key] : v;
                else out[key] = ninf;
            }
        }
    }
}

template <int S, int CB, int MODE>
static void launch_score_kernel(const ScoreArgs &a, bool one_round, dim3 grid, size_t lds, hipStream_t st) {
    if (one_round) hipLaunchKernelGGL((score_kernel<S, CB, MODE, true>), grid, dim3(kScoreThreads), lds, st, a);
    else hipLaunchKernelGGL((score_kernel<S, CB, MODE, false>), grid, dim3(kScoreThreads), lds, st, a);
}

template <int CB, int MODE>
static int dispatch_score_s(const ScoreArgs &a, int S, bool one_round, dim3 grid, size_t lds, hipStream_t st) {
    switch (S) {
        case 1: launch_score_kernel<1, CB, MODE>(a, one_round, grid, lds, st); return SOCKET_OK;
        case 2: launch_score_kernel<2, CB, MODE>(a, one_round, grid, lds, st); return SOCKET_OK;
        case 4: launch_score_kernel<4, CB, MODE>(a, one_round, grid, lds, st); return SOCKET_OK;
        default: return SOCKET_EUNSUPPORTED;
    }
}

static int set_lds_limit(const void *fn, size_t lds) {
    if (lds <= 64 * 1024) return SOCKET_OK;
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess
               ? SOCKET_OK : SOCKET_EHIP;
}

int launch_score(socket_ctx *ctx, const void *q, const void *codes, const void *proj, float tau,
                 const float *vnorm, const int32_t *block_table, const int32_t *seq_len, int batch,
                 float *scores, hipStream_t st) {
    const Geometry &g = ctx->g;
    SoftHashArgs sa;
    sa.q = q; sa.W = proj; sa.tables = ctx->tables; sa.tau = (double)tau;
    sa.d = g.d; sa.G = g.G; sa.Hkv = g.Hkv; sa.Hq = g.Hq; sa.L = g.L; sa.P = g.P; sa.LP = g.L * g.P;
    sa.Lpad = g.Lpad; sa.rounds = g.rounds; sa.R = g.R; sa.mode = g.mode;
    sa.Plo = g.Plo; sa.Phi = g.Phi; sa.Rlo = g.Rlo; sa.Rhi = g.Rhi; sa.table_rows = g.table_rows;
    sa.table_words = g.table_words; sa.kv_dtype = g.kv_dtype;
    {
        dim3 grid((g.Lpad + kTablesPerWg - 1) / kTablesPerWg, g.Hkv, batch);
        size_t lds = (size_t)(g.G * g.d + 2 * g.G * kTablesPerWg * g.P) * sizeof(double);
        hipLaunchKernelGGL(soft_hash_kernel, grid, dim3(256), lds, st, sa);
        int rc = record_hip(ctx, hipGetLastError());
        if (rc != SOCKET_OK) return rc;
    }

    ScoreArgs a;
    a.codes = codes; a.tables = ctx->tables; a.vnorm = vnorm; a.seq_len = seq_len; a.scores = scores;
    a.map = RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks};
    a.Lpad = g.Lpad; a.rounds = g.rounds; a.R = g.R; a.G = g.G; a.Plo = g.Plo; a.Rlo = g.Rlo;
    a.table_rows = g.table_rows; a.table_words = g.table_words;
    // About two workgroups per CU over the whole launch; a workgroup pass covers
    // 8 waves * 4 passes * (64/S) keys, and each workgroup pays one table load.
    const int quantum = (kScoreThreads / 64) * 4 * (64 / g.S);
    int64_t per_bh_wgs = 512 / ((int64_t)batch * g.Hkv);
    if (per_bh_wgs < 1) per_bh_wgs = 1;
    int64_t kpw = (g.max_n + per_bh_wgs - 1) / per_bh_wgs;
    kpw = (kpw + quantum - 1) / quantum * quantum;
    a.keys_per_wg = (int)kpw;
    dim3 grid((g.max_n + a.keys_per_wg - 1) / a.keys_per_wg, g.Hkv, batch);
    size_t lds = (size_t)g.table_words * 4;
    const bool one_round = g.rounds == 1;
    int rc;
    // the attribute must be raised before a launch that needs more than 64 KB of LDS
#define SK_PREP(S_, CB_, MODE_)                                                                   \
    do {                                                                                          \
        int r1 = set_lds_limit((const void *)score_kernel<S_, CB_, MODE_, true>, lds);            \
        int r2 = set_lds_limit((const void *)score_kernel<S_, CB_, MODE_, false>, lds);           \
        if (r1 != SOCKET_OK || r2 != SOCKET_OK) return SOCKET_EHIP;                               \
    } while (0)
    if (g.mode == kDirect && g.cb == 1) {
        if (g.S == 1) SK_PREP(1, 1, kDirect); else if (g.S == 2) SK_PREP(2, 1, kDirect); else SK_PREP(4, 1, kDirect);
        rc = dispatch_score_s<1, kDirect>(a, g.S, one_round, grid, lds, st);
    } else if (g.mode == kFactor && g.cb == 1) {
        if (g.S == 1) SK_PREP(1, 1, kFactor); else if (g.S == 2) SK_PREP(2, 1, kFactor); else SK_PREP(4, 1, kFactor);
        rc = dispatch_score_s<1, kFactor>(a, g.S, one_round, grid, lds, st);
    } else if (g.mode == kFactor && g.cb == 2) {
        if (g.S == 1) SK_PREP(1, 2, kFactor); else if (g.S == 2) SK_PREP(2, 2, kFactor); else SK_PREP(4, 2, kFactor);
        rc = dispatch_score_s<2, kFactor>(a, g.S, one_round, grid, lds, st);
    } else {
        return SOCKET_EUNSUPPORTED;
    }
#undef SK_PREP
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

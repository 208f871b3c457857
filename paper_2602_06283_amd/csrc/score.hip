// Alg. 2 (SoftBucketProbs) and Alg. 5 (SoftHashCollisionScores, the soft score of Eq. 3).
//
//   project_kernel    builds, per (sequence, KV head), the table of bucket probabilities of
//                     the G queries that share the head.  Evaluated in fp64 and stored as
//                     fp32.  A softmax over the corners of {+-1}^P factorises over the
//                     planes, p(r) = prod_i sigmoid(+-2 u_i / tau), which is the form used.
//                     The same launch can hash the one key a decode step appends (Alg. 1),
//                     since both are projections onto the same hyperplanes.
//   score_kernel      loads that table into LDS and streams the bucket ids of every key
//                     once: 64/S keys per wavefront pass, S lanes per key, each lane reading
//                     16 ids with one 16-byte load.  The rotated id order (see socket.h)
//                     makes the 64 lanes of a pass hit 64 different tables, and the table is
//                     stored [bucket][table], so the LDS gathers are free of bank conflicts.
#include <cmath>

#include "socket_internal.h"

namespace sk {

#ifdef SK_DEBUG_CLOCKS
__device__ long long sk_dbg2[64];
#define SK_STAMP2(i) do { if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0) { sk_dbg2[i] = wall_clock64(); sk_dbg2[32 + i] = clock64(); } } while (0)
extern "C" int socket_debug_clocks2(long long *out) {
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(sk_dbg2), sizeof(long long) * 64);
}
#else
#define SK_STAMP2(i) ((void)0)
#endif

struct ProjectArgs {
    const void *q;          // [B, Hq, d]; null = no soft hash
    const void *W;          // [Hkv, d, L*P]
    float *tables;
    double tau;
    double x_scale;         // 2 / (sqrt(d) * tau)
    const void *K;          // key cache; null = no append hash
    void *codes;
    const int32_t *pos;     // [B] position of the appended key (append hash only)
    const int32_t *count;   // optional [B]: append only where count[b] >= 1
    int32_t *len_out;       // optional [B]: pos[b] + 1
    RowMap map;
    int d, G, Hkv, Hq, L, P, LP, Lpad, S, cb, rounds, R, mode, Plo, Phi, Rlo, Rhi, table_rows, tpw;
    int64_t table_words;
};

template <typename T> __device__ __forceinline__ float elem_to_f32(T v);
template <> __device__ __forceinline__ float elem_to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float elem_to_f32<uint16_t>(uint16_t v) { return bf16_to_f32(v); }

// 1/x for x in [1, 2]: hardware estimate plus two Newton steps (relative error < 1e-15)
__device__ __forceinline__ double rcp64(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = fma(r, fma(-x, r, 1.0), r);
    r = fma(r, fma(-x, r, 1.0), r);
    return r;
}

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask);
    hi = __shfl_xor(hi, mask);
    return __hiloint2double(hi, lo);
}

// One workgroup projects onto the P hyperplanes of ONE table of one KV head:
//   - the G queries of the head's group, in fp64, giving that table's bucket probabilities
//     (Alg. 2; the softmax over corners is evaluated as a product of per-plane sigmoids);
//   - optionally the key appended at position pos[b], in fp32 FMA, giving its bucket id for
//     that table (Alg. 1 on one row).
// The kernel is a chain of short dependent phases, so each phase is spread over as many
// threads as it has independent work: every dot product is cut into TPP channel ranges that
// adjacent lanes sum with shuffles.
template <typename T>
__global__ __launch_bounds__(256) void project_kernel(ProjectArgs a) {
    extern __shared__ double sm64[];
    const int tid = threadIdx.x;
    const int l = blockIdx.x, h = blockIdx.y, b = blockIdx.z;   // table, KV head, sequence
    const int cols = a.P;
    const int col0 = l * a.P;
    const bool live = l < a.L;                               // tables >= L are padding: zero rows
    const bool soft = a.q != nullptr, app = a.K != nullptr;

    double *qd = sm64;                                       // [G][d]
    double *sp = qd + a.G * a.d;                             // [G][P] sigmoid(+2u/tau)
    double *sn = sp + a.G * a.P;                             // [G][P] sigmoid(-2u/tau)
    double *half = sn + a.G * a.P;                           // [G][Rlo+Rhi] (direct mode)
    const int hrows = a.Rlo + a.Rhi;
    const int nhalf = a.mode == kDirect ? a.G * hrows : 0;
    float *kf = (float *)(half + nhalf);                     // [d]
    uint32_t *sgn = (uint32_t *)(kf + a.d);                  // [16] sign bits of the key's projections
    T *w = (T *)(sgn + 16);                                  // [d][P]
    SK_STAMP2(0);

    // ---- the table's slab of W, the queries and the key row -> LDS, all loads in flight at once
    constexpr int NB = 8;
    if (live) {
        const T *Wg = (const T *)a.W + (int64_t)h * a.d * a.LP + col0;
        const int total = a.d * cols;
        for (int i0 = tid; i0 < total; i0 += NB * 256) {
            T v[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int i = i0 + j * 256;
                if (i < total) v[j] = Wg[(int64_t)(i / cols) * a.LP + i % cols];
            }
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int i = i0 + j * 256;
                if (i < total) w[i] = v[j];
            }
        }
    }
    if (soft) {
        for (int i = tid; i < a.G * a.d; i += 256) {
            int g = i / a.d, c = i - g * a.d;
            qd[i] = (double)elem_to_f32<T>(((const T *)a.q)[((int64_t)b * a.Hq + h * a.G + g) * a.d + c]);
        }
    }
    int tok = 0;
    int64_t krow = -1;
    if (app) {
        tok = a.pos[b];
        const bool wanted = a.count == nullptr || a.count[b] >= 1;
        if (wanted && tok >= 0 && tok < a.map.max_n) krow = a.map.row(b, h, tok);
        for (int c = tid; c < a.d; c += 256)
            kf[c] = krow >= 0 ? elem_to_f32<T>(((const T *)a.K)[krow * a.d + c]) : 0.0f;
        if (a.len_out && l == 0 && h == 0 && tid == 0) a.len_out[b] = tok + 1;
    }
    if (tid < 16) sgn[tid] = 0;
    __syncthreads();
    SK_STAMP2(1);

    // ---- appended key: 16 lanes per hyperplane, fp32 FMA over a 16th of the channels each
    if (app && live) {
        const int pl = tid >> 4, part = tid & 15;            // 16 planes x 16 parts = 256 threads
        float acc = 0.0f;
        if (pl < cols) {
            const int per = a.d >> 4;
            for (int c = part * per; c < (part + 1) * per; ++c) acc = fmaf(kf[c], elem_to_f32<T>(w[c * cols + pl]), acc);
        }
#pragma unroll
        for (int m = 8; m > 0; m >>= 1) acc += __shfl_xor(acc, m);
        if (pl < cols && part == 0) sgn[pl] = acc >= 0.0f ? 1u : 0u;
    }
    // ---- queries: fp64 dot products, TPP lanes each; then u = tanh(z)/sqrt(d) and the
    //      per-plane sigmoids of +-2u/tau
    if (soft && live) {
        const int npairs = a.G * cols;                       // <= 128
        int tpp = 1;
        while (tpp * 2 * npairs <= 256 && tpp < 32 && (a.d / (tpp * 2)) >= 2) tpp *= 2;
        const int pair = tid / tpp, part = tid % tpp;
        double z = 0.0;
        if (pair < npairs) {
            const int g = pair / cols, j = pair - g * cols;
            const int per = a.d / tpp;
            const double *qg = qd + g * a.d + part * per;
            const T *wj = w + (part * per) * cols + j;
            double z0 = 0.0, z1 = 0.0;
            for (int c0 = 0; c0 < per; c0 += 8) {            // 8 channels' LDS reads issued together
                T wv[8];
                double qv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool in = c0 + e < per;
                    wv[e] = in ? wj[(c0 + e) * cols] : (T)0;
                    qv[e] = in ? qg[c0 + e] : 0.0;
                }
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    z0 = fma((double)elem_to_f32<T>(wv[e]), qv[e], z0);
                    z1 = fma((double)elem_to_f32<T>(wv[e + 1]), qv[e + 1], z1);
                }
            }
            z = z0 + z1;
        }
        for (int m = tpp >> 1; m > 0; m >>= 1) z += shfl_xor_f64(z, m);
        if (pair < npairs && part == 0) {
            // tanh|z| = (1 - t)/(1 + t) with t = exp(-2|z|); sigmoid(+-x) from e = exp(-|x|)
            const double t = exp(-2.0 * fabs(z));
            const double th = (1.0 - t) * rcp64(1.0 + t);
            const double e = exp(-a.x_scale * th);           // x = 2 tanh|z| / (sqrt(d) tau) >= 0
            const double big = rcp64(1.0 + e), small = e * big;
            sp[pair] = z >= 0.0 ? big : small;                // [g][pl]
            sn[pair] = z >= 0.0 ? small : big;
        }
    }
    __syncthreads();
    SK_STAMP2(2);

    if (app && krow >= 0 && tid == 0 && l < a.Lpad) {
        uint32_t code = 0;
        if (live)
            for (int pl = 0; pl < cols; ++pl) code |= sgn[pl] << pl;
        const int64_t at = krow * a.Lpad + code_pos(l, tok, a.S);
        if (a.cb == 1) ((uint8_t *)a.codes)[at] = (uint8_t)code;
        else ((uint16_t *)a.codes)[at] = (uint16_t)code;
    }
    if (!soft) return;
    SK_STAMP2(3);

    const int lw = a.Lpad < 64 ? a.Lpad : 64;        // distinct tables per 64-word row
    const int copies = 64 / lw;
    const int c64 = l >> 6, lp = l & 63;
    float *Tg = a.tables + ((int64_t)b * a.Hkv + h) * a.table_words;
    // products over the low and the high planes: p(r) = lo[r & (Rlo-1)] * hi[r >> Plo]
    auto half_product = [&](int g, int row) -> double {
        double p = 1.0;
        if (row < a.Rlo) {
            for (int pl = 0; pl < a.Plo; ++pl) p *= ((row >> pl) & 1) ? sp[g * cols + pl] : sn[g * cols + pl];
        } else {
            const int rh = row - a.Rlo;
            for (int pl = 0; pl < a.Phi; ++pl)
                p *= ((rh >> pl) & 1) ? sp[g * cols + a.Plo + pl] : sn[g * cols + a.Plo + pl];
        }
        return p;
    };
    if (a.mode == kDirect) {
        if (live) {
            for (int i = tid; i < a.G * hrows; i += 256) half[i] = half_product(i / hrows, i % hrows);   // [g][row]
        }
        __syncthreads();
        SK_STAMP2(4);
        const double inv_g = 1.0 / (double)a.G;
        for (int r = tid; r < a.R; r += 256) {
            double mean = 0.0;
            if (live) {
                for (int g = 0; g < a.G; ++g) mean += half[g * hrows + (r & (a.Rlo - 1))] * half[g * hrows + a.Rlo + (r >> a.Plo)];
                mean *= inv_g;
            }
            for (int cp = 0; cp < copies; ++cp) Tg[((int64_t)c64 * a.R + r) * 64 + lp + cp * lw] = (float)mean;
        }
        SK_STAMP2(5);
    } else {
        for (int i = tid; i < hrows * a.G; i += 256) {
            int row = i % hrows, g = i / hrows;
            double p = 0.0;
            if (live) {
                p = half_product(g, row);
                if (row < a.Rlo) p /= (double)a.G;    // the 1/G of the group mean rides on the low factor
            }
            for (int cp = 0; cp < copies; ++cp)
                Tg[(((int64_t)g * a.rounds + c64) * hrows + row) * 64 + lp + cp * lw] = (float)p;
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
    uint32_t *hist;          // optional [B*Hkv][kHistBins]: leading-digit histogram of the scores
    RowMap map;
    int Lpad, rounds, R, G, Plo, Rlo, table_rows;
    int64_t table_words;
};

// 16 bucket ids of one lane: CB = 1 -> 16 bytes, CB = 2 -> 32 bytes.
template <int CB> struct CodeVec;
template <> struct CodeVec<1> {
    uint4 v;
#ifndef SK_SCORE_NO_NT
    // the id stream is read once: a non-temporal load keeps it from displacing the table and
    // the scores in L2 (measured 6 % faster)
    __device__ __forceinline__ void load(const void *p) {
        typedef unsigned int u4 __attribute__((ext_vector_type(4)));
        u4 t = __builtin_nontemporal_load((const u4 *)p);
        v = make_uint4(t.x, t.y, t.z, t.w);
    }
#else
    __device__ __forceinline__ void load(const void *p) { v = *(const uint4 *)p; }
#endif
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

typedef __attribute__((address_space(3))) const float lds_cfloat_t;
typedef __attribute__((address_space(3))) float lds_float_t;

// LDS read at a raw byte address (the table look-ups compute their addresses as integers).
__device__ __forceinline__ float lds_read(uint32_t addr) { return *(lds_cfloat_t *)(size_t)addr; }

// Sum over this lane's 16 tables of 64-table chunk c of the bucket probabilities of one key.
// tbase = LDS byte address of the table; BASE0 says it is known to be 0, which lets the
// direct one-byte-id path form each address with a single v_perm_b32 when, in addition, the
// table has a single 64-table chunk (NOOFF: nothing to add at all).
template <int CB, int MODE, bool BASE0, bool NOOFF>
__device__ __forceinline__ float gather16(const CodeVec<CB> &cv, uint32_t tbase, const uint32_t *woff,
                                          int c, const ScoreArgs &a) {
    float acc0 = 0.0f, acc1 = 0.0f;
    if (MODE == kDirect) {
        const uint32_t toff = (BASE0 ? 0u : tbase) + (uint32_t)c * (uint32_t)a.R * 256u;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            uint32_t addr;
            if (CB == 1)   // byte 0 <- table offset, byte 1 <- bucket id: address = id*256 + offset
                addr = __builtin_amdgcn_perm(cv.word(s >> 2), woff[s], 0x0c0c0400u + ((uint32_t)(s & 3) << 8));
            else
                addr = (cv.code(s) << 8) | woff[s];
            if (!NOOFF) addr += toff;
            const float p = lds_read(addr);
            if (s == 0) acc0 = p;
            else if (s == 1) acc1 = p;
            else if (s & 1) acc1 += p;
            else acc0 += p;
        }
    } else {
        for (int g = 0; g < a.G; ++g) {
            const uint32_t toff = tbase + (uint32_t)((g * a.rounds + c) * a.table_rows) * 256u;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                uint32_t code = cv.code(s);
                uint32_t lo = code & (uint32_t)(a.Rlo - 1), hi = code >> a.Plo;
                float pa = lds_read(toff + ((lo << 8) | woff[s]));
                float pb = lds_read(toff + ((((uint32_t)a.Rlo + hi) << 8) | woff[s]));
                if (s & 1) acc1 = fmaf(pa, pb, acc1); else acc0 = fmaf(pa, pb, acc0);
            }
        }
    }
    return acc0 + acc1;
}

// Sum over the S adjacent lanes that share a key (DPP quad permutes, no LDS traffic).
template <int S>
__device__ __forceinline__ float group_sum(float v) {
    if (S >= 2) v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));  // lane ^ 1
    if (S >= 4) v += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true));  // lane ^ 2
    return v;
}

__device__ __forceinline__ uint32_t score_order_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <bool V> struct BoolTag { static constexpr bool value = V; };

// A workgroup owns chunks of CKEYS consecutive keys, taken round-robin; inside a chunk each
// wavefront owns U*KPW consecutive keys and keeps U 16-byte loads per lane in flight.  Chunks
// that lie wholly inside the sequence take a branch-free path in which the loads of the next
// chunk are issued before the current one is processed (two register sets, ping-pong).
template <int S, int CB, int MODE, bool ONE_ROUND, bool PAGED>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(ScoreArgs a) {
    extern __shared__ float tbl[];
    constexpr int KPW = 64 / S;                      // keys per wavefront pass
    constexpr int NW = kScoreThreads / 64;
    constexpr int U = kScoreU;                       // passes per wavefront per chunk
    constexpr int WKEYS = U * KPW;                   // consecutive keys a wavefront owns in a chunk
    constexpr int CKEYS = NW * WKEYS;                // keys per chunk
    static_assert(U % S == 0, "each lane of a key's group emits U/S results");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * a.map.Hkv + h;
    const int max_n = a.map.max_n;
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > max_n ? max_n : seq);
    float *out = a.scores + bh * max_n;
    const float *vn = a.vnorm ? a.vnorm + bh * max_n : nullptr;
    const float ninf = -__builtin_inff();
    const int stride = gridDim.x;
    // Every workgroup takes the same number of whole chunks (nround); what is left over - less
    // than one chunk per workgroup, plus the tail beyond the sequence - is dealt out pass by
    // pass over all wavefronts, so that no workgroup carries a whole extra chunk.
    const int nround = (seq / CKEYS) / stride;
    const int left0 = nround * stride * CKEYS;       // first key of the leftover region
    const bool has_table = seq > 0;

    const int sub = lane % S, kk = lane / S;
    const int lw = a.Lpad < 64 ? a.Lpad : 64;
    uint32_t woff[16];                               // byte offset of this lane's table in a 64-float row
#pragma unroll
    for (int s = 0; s < 16; ++s) woff[s] = 4u * (uint32_t)(sub + S * ((kk + s) & 15) + lw * (kk >> 4));
    const uint32_t tbase = (uint32_t)(size_t)(lds_float_t *)tbl;
    uint32_t *lhist = (uint32_t *)(tbl + a.table_words);
    const char *codes_bh = (const char *)a.codes + (bh * max_n * (int64_t)a.Lpad + sub * 16) * CB;

    // address of this lane's 16 ids of key `key`, round c; dead = the token's block is absent
    auto code_ptr = [&](int key, int c, bool &dead) -> const char * {
        if (PAGED) {
            int64_t row = a.map.row(b, h, key);
            dead = row < 0;
            if (dead) row = 0;
            return (const char *)a.codes + (row * a.Lpad + c * 64 + sub * 16) * CB;
        }
        dead = false;
        return codes_bh + ((int64_t)key * a.Lpad + c * 64) * CB;
    };
    // Passes u = 0..U-1 of a wavefront cover keys base + u*KPW + kk.  Lane `sub` of a key's
    // group writes the results of passes sub, sub+S, ...
    auto emit = [&](int base, const float *sum, const bool *dead) {
#pragma unroll
        for (int j = 0; j < U / S; ++j) {
            float v = sum[j * S];
            bool dd = dead[j * S];
#pragma unroll
            for (int t = 1; t < S; ++t) {
                v = sub == t ? sum[j * S + t] : v;
                dd = sub == t ? dead[j * S + t] : dd;
            }
            const int key = base + (j * S + sub) * KPW + kk;
            if (key < max_n) {
                if (dd) v = ninf;
                else if (vn) v *= vn[key];
                out[key] = v;
                if (a.hist && v > ninf) atomicAdd(&lhist[score_order_key(v) >> (32 - kHistBits)], 1u);
            }
        }
    };
    auto load_set = [&](CodeVec<CB> *cv, bool *dead, int base) {
#pragma unroll
        for (int u = 0; u < U; ++u) cv[u].load(code_ptr(base + u * KPW + kk, 0, dead[u]));
    };
    auto chunk_base = [&](int r) { return (r * stride + (int)blockIdx.x) * CKEYS + wave * WKEYS; };

    constexpr bool PREFETCH = ONE_ROUND;
    CodeVec<CB> setA[U], setB[U];
    bool deadA[U], deadB[U];
    if (PREFETCH && nround > 0) load_set(setA, deadA, chunk_base(0));
    if (has_table) {            // bucket-probability table -> LDS
        const float4 *src = (const float4 *)(a.tables + bh * a.table_words);
        float4 *dst = (float4 *)tbl;
        const int n4 = (int)(a.table_words >> 2);
        constexpr int B8 = 8;                        // independent loads in flight per thread
        for (int i0 = tid; i0 < n4; i0 += B8 * kScoreThreads) {
            float4 t[B8];
#pragma unroll
            for (int j = 0; j < B8; ++j) {
                const int i = i0 + j * kScoreThreads;
                t[j] = i < n4 ? src[i] : make_float4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < B8; ++j) {
                const int i = i0 + j * kScoreThreads;
                if (i < n4) dst[i] = t[j];
            }
        }
        if (a.hist)
            for (int i = tid; i < kHistBins; i += kScoreThreads) lhist[i] = 0;
    }
    __syncthreads();

    // ---- whole chunks: branch-free, the next chunk's loads in flight during the look-ups
    auto full_chunks = [&](auto base0) {
        constexpr bool BASE0 = decltype(base0)::value;
        auto process = [&](const CodeVec<CB> *cv, const bool *dead, int base) {
            float sum[U];
#pragma unroll
            for (int u = 0; u < U; ++u) sum[u] = group_sum<S>(gather16<CB, MODE, BASE0, BASE0 && ONE_ROUND>(cv[u], tbase, woff, 0, a));
            emit(base, sum, dead);
        };
        if (PREFETCH) {
            int r = 0;
            while (r < nround) {
                if (r + 1 < nround) load_set(setB, deadB, chunk_base(r + 1));
                process(setA, deadA, chunk_base(r));
                if (++r >= nround) break;
                if (r + 1 < nround) load_set(setA, deadA, chunk_base(r + 1));
                process(setB, deadB, chunk_base(r));
                ++r;
            }
        } else {
            for (int r = 0; r < nround; ++r) {
                const int base = chunk_base(r);
                float sum[U];
                bool dead[U];
#pragma unroll
                for (int u = 0; u < U; ++u) sum[u] = 0.0f;
                for (int c = 0; c < a.rounds; ++c) {
                    CodeVec<CB> cur[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) cur[u].load(code_ptr(base + u * KPW + kk, c, dead[u]));
#pragma unroll
                    for (int u = 0; u < U; ++u) sum[u] += gather16<CB, MODE, BASE0, false>(cur[u], tbase, woff, c, a);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) sum[u] = group_sum<S>(sum[u]);
                emit(base, sum, dead);
            }
        }
    };
    if (tbase == 0) full_chunks(BoolTag<true>());
    else full_chunks(BoolTag<false>());

    // ---- leftover keys and the -inf fill beyond the sequence, U passes at a time per wavefront
    const int npass = (max_n - left0 + KPW - 1) / KPW;
    for (int p0 = ((int)blockIdx.x * NW + wave) * U; p0 < npass; p0 += stride * NW * U) {
        const int base = left0 + p0 * KPW;
        float sum[U];
        bool dead[U];
        CodeVec<CB> cv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            sum[u] = 0.0f;
            dead[u] = base + u * KPW + kk >= seq;
        }
        for (int c = 0; c < a.rounds; ++c) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (dead[u]) continue;
                bool absent;
                cv[u].load(code_ptr(base + u * KPW + kk, c, absent));
                if (absent) dead[u] = true;
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (!dead[u]) sum[u] += gather16<CB, MODE, false, false>(cv[u], tbase, woff, c, a);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) sum[u] = group_sum<S>(sum[u]);   // every lane of a key's group takes part
        emit(base, sum, dead);
    }

    if (a.hist && has_table) {
        __syncthreads();
        uint32_t *gh = a.hist + bh * kHistBins;
        for (int i = tid; i < kHistBins; i += kScoreThreads)
            if (lhist[i]) atomicAdd(&gh[i], lhist[i]);
    }
}

typedef void (*score_fn_t)(ScoreArgs);

template <int S, int CB, int MODE>
static score_fn_t pick_score_variant(bool one_round, bool paged) {
    if (one_round) return paged ? score_kernel<S, CB, MODE, true, true> : score_kernel<S, CB, MODE, true, false>;
    return paged ? score_kernel<S, CB, MODE, false, true> : score_kernel<S, CB, MODE, false, false>;
}

template <int CB, int MODE>
static score_fn_t pick_score_s(int S, bool one_round, bool paged) {
    switch (S) {
        case 1: return pick_score_variant<1, CB, MODE>(one_round, paged);
        case 2: return pick_score_variant<2, CB, MODE>(one_round, paged);
        case 4: return pick_score_variant<4, CB, MODE>(one_round, paged);
        default: return nullptr;
    }
}

static score_fn_t pick_score(const Geometry &g) {
    const bool one_round = g.rounds == 1, paged = g.page > 0;
    if (g.mode == kDirect && g.cb == 1) return pick_score_s<1, kDirect>(g.S, one_round, paged);
    if (g.mode == kFactor && g.cb == 1) return pick_score_s<1, kFactor>(g.S, one_round, paged);
    if (g.mode == kFactor && g.cb == 2) return pick_score_s<2, kFactor>(g.S, one_round, paged);
    return nullptr;
}

static int set_lds_limit(const void *fn, size_t lds) {
    if (lds <= 64 * 1024) return SOCKET_OK;
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess
               ? SOCKET_OK : SOCKET_EHIP;
}

int launch_project(socket_ctx *ctx, const void *q, const void *proj, float tau, const void *K,
                   void *codes, const int32_t *block_table, const int32_t *pos, const int32_t *count,
                   int32_t *len_out, int batch, hipStream_t st) {
    const Geometry &g = ctx->g;
    ProjectArgs a;
    a.q = q; a.W = proj; a.tables = ctx->tables; a.tau = (double)tau;
    a.x_scale = 2.0 / (sqrt((double)g.d) * (double)tau);
    a.K = K; a.codes = codes; a.pos = pos; a.count = count; a.len_out = len_out;
    a.map = RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks};
    a.d = g.d; a.G = g.G; a.Hkv = g.Hkv; a.Hq = g.Hq; a.L = g.L; a.P = g.P; a.LP = g.L * g.P;
    a.Lpad = g.Lpad; a.S = g.S; a.cb = g.cb; a.rounds = g.rounds; a.R = g.R; a.mode = g.mode;
    a.Plo = g.Plo; a.Phi = g.Phi; a.Rlo = g.Rlo; a.Rhi = g.Rhi; a.table_rows = g.table_rows;
    a.table_words = g.table_words;
    a.tpw = 1;
    const int nhalf = g.mode == kDirect ? g.G * (g.Rlo + g.Rhi) : 0;
    const int esize = g.kv_dtype == SOCKET_F32 ? 4 : 2;
    size_t lds = (size_t)(g.G * g.d + 2 * g.G * g.P + nhalf) * sizeof(double) + (size_t)g.d * 4 + 64 +
                 (size_t)g.d * g.P * esize;
    dim3 grid(g.Lpad, g.Hkv, batch);
    if (g.kv_dtype == SOCKET_F32) {
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)project_kernel<float>,
                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return SOCKET_EHIP;
        hipLaunchKernelGGL(project_kernel<float>, grid, dim3(256), lds, st, a);
    } else {
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)project_kernel<uint16_t>,
                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return SOCKET_EHIP;
        hipLaunchKernelGGL(project_kernel<uint16_t>, grid, dim3(256), lds, st, a);
    }
    return record_hip(ctx, hipGetLastError());
}

int launch_soft_hash(socket_ctx *ctx, const void *q, const void *proj, float tau, int batch,
                     hipStream_t st) {
    return launch_project(ctx, q, proj, tau, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, batch, st);
}

int launch_score_keys(socket_ctx *ctx, const void *codes, const float *vnorm,
                      const int32_t *block_table, const int32_t *seq_len, int batch, float *scores,
                      bool with_hist, hipStream_t st) {
    const Geometry &g = ctx->g;
    ScoreArgs a;
    a.codes = codes; a.tables = ctx->tables; a.vnorm = vnorm; a.seq_len = seq_len; a.scores = scores;
    a.map = RowMap{block_table, g.Hkv, g.max_n, g.page, g.max_blocks, g.num_blocks};
    a.Lpad = g.Lpad; a.rounds = g.rounds; a.R = g.R; a.G = g.G; a.Plo = g.Plo; a.Rlo = g.Rlo;
    a.table_rows = g.table_rows; a.table_words = g.table_words;
    // Two resident workgroups per CU over the whole launch, chunks dealt round-robin.
    const int ckeys = (kScoreThreads / 64) * kScoreU * (64 / g.S);
    const int nchunks = (g.max_n + ckeys - 1) / ckeys;
#ifndef SK_SCORE_WGS
#define SK_SCORE_WGS (256 * 1024 / SK_SCORE_THREADS)
#endif
    int per_bh = SK_SCORE_WGS / (batch * g.Hkv);
    if (per_bh < 1) per_bh = 1;
    if (per_bh > nchunks) per_bh = nchunks;
    dim3 grid(per_bh, g.Hkv, batch);
    a.hist = with_hist ? ctx->hist : nullptr;
    size_t lds = (size_t)g.table_words * 4 + (a.hist ? kHistBins * 4 : 0);
    score_fn_t fn = pick_score(g);
    if (!fn) return SOCKET_EUNSUPPORTED;
    // more than 64 KB of dynamic LDS has to be allowed per kernel before the launch
    if (set_lds_limit((const void *)fn, lds) != SOCKET_OK) return SOCKET_EHIP;
    hipLaunchKernelGGL(fn, grid, dim3(kScoreThreads), lds, st, a);
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

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
    float *tstats;          // [B*Hkv][Lpad][3]: mean squared deviation of each table's entries from 1/R;
                            // sum and sum of squares of 256 sampled value norms
    const float *vnorm;     // optional [B, Hkv, max_n]: value norms to sample (with the append hash only)
    double tau;
    double x_scale;         // 2 / (sqrt(d) * tau)
    int hard;               // 1: one-hot tables (the query's own bucket), Eq. 3's hard count
    const void *K;          // key cache; null = no append hash
    void *codes;
    const int32_t *pos;     // [B] position of the appended key (append hash only)
    const int32_t *count;   // optional [B]: append only where count[b] >= 1
    int32_t *len_out;       // optional [B]: pos[b] + 1
    RowMap map;
    int d, G, Hkv, Hq, L, P, LP, Lpad, S, cb, rounds, R, mode, Plo, Phi, Rlo, Rhi, table_rows;
    int GT;                 // split mode: tables per group
    int cols_magic;         // ceil(2^16 / P): x / P == (x * cols_magic) >> 16 for x < 2^12
    int64_t table_words;
};

template <typename T> __device__ __forceinline__ float elem_to_f32(T v);
template <> __device__ __forceinline__ float elem_to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float elem_to_f32<uint16_t>(uint16_t v) { return bf16_to_f32(v); }

// the 16 / sizeof(T) elements of a 16-byte vector as floats
template <typename T> __device__ __forceinline__ void vec_to_f32(const uint4 &v, float *f);
template <> __device__ __forceinline__ void vec_to_f32<float>(const uint4 &v, float *f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void vec_to_f32<uint16_t>(const uint4 &v, float *f) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// 1/x for x in [1, 2]: hardware estimate plus two Newton steps (relative error < 1e-15)
__device__ __forceinline__ double rcp64(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = fma(r, fma(-x, r, 1.0), r);
    r = fma(r, fma(-x, r, 1.0), r);
    return r;
}

template <int CTRL> __device__ __forceinline__ double dpp_f64(double v) {
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(v), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(v), CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}
// sum over groups of n adjacent lanes, n = 1, 2, 4, 8 or 16 (uniform over the wavefront)
__device__ __forceinline__ double group_sum_f64(double v, int n) {
    if (n >= 16) {
        v += dpp_f64<0x128>(v);      // row_ror:8
        v += dpp_f64<0x124>(v);      // row_ror:4
    } else if (n >= 8) {
        v += dpp_f64<0x141>(v);      // row_half_mirror
    }
    if (n >= 4) v += dpp_f64<0x4E>(v);
    if (n >= 2) v += dpp_f64<0xB1>(v);
    return v;
}

constexpr int kPlanePad = 16;        // per-plane sigmoids are kept [g][16]; planes >= P hold 1

// One workgroup projects onto the P hyperplanes of ONE table of one KV head:
//   - the G queries of the head's group, in fp64, giving that table's bucket probabilities
//     (Alg. 2; the softmax over corners is evaluated as a product of per-plane sigmoids);
//   - optionally the key appended at position pos[b], in fp32 FMA, giving its bucket id for
//     that table (Alg. 1 on one row).
// The kernel is a chain of short dependent phases bounded by memory and LDS latency, so every
// phase issues all of its independent loads before the first use, and every dot product is
// cut into channel ranges that adjacent lanes sum with DPP moves.
// DW: the dword fetch of the W slab is compiled in (bf16 tables whose planes are whole dwords
// but not whole 16-byte vectors, e.g. 10 planes); the other instantiations stay as lean as
// they were.
template <typename T, int G, bool DW>
__global__ __launch_bounds__(256) void project_kernel(ProjectArgs a) {
    extern __shared__ double sm64[];
    constexpr int EPV = 16 / (int)sizeof(T);                 // elements per 16-byte vector
    const int tid = threadIdx.x;
    // Workgroups go to the 8 XCDs round-robin; the 8 tables whose columns of W share 128-byte
    // lines are given to workgroups of one XCD, so each line is fetched into one L2 only.
    const int x = blockIdx.x;
    const int l = (x & 7) * (a.Lpad >> 3) + (x >> 3);        // table (Lpad is a multiple of 16)
    const int h = blockIdx.y, b = blockIdx.z;                // KV head, sequence
    const int cols = a.P, d = a.d;
    const int col0 = l * a.P;
    const bool live = l < a.L;                               // tables >= L are padding: zero rows
    const bool soft = a.q != nullptr, app = a.K != nullptr;

    // Plane j lives in slot j, except that the high planes of the factor form start at slot 8:
    // any product over 8 consecutive slots then needs no bounds (an unused slot holds 1).
    double *sig = sm64;                                      // [G][16 slots][2] sigmoid(-2u/tau), sigmoid(+2u/tau)
    double *qd = sig + G * kPlanePad * 2;                    // [G][d]  queries
    double *wd = qd + G * d;                                 // [P][d]  W slab, transposed
    float *wf = (float *)(wd + cols * d);                    // [P][d]  the same in fp32 (key path)
    float *kf = wf + cols * d;                               // [d]
    uint32_t *sgn = (uint32_t *)(kf + d);                    // [16] sign bits of the key's projections
    float *s_dev = (float *)(sgn + 16);                      // [12]
    SK_STAMP2(0);

    // ---- every global load of the kernel is issued here, before the first one is used
    int tok = 0;
    bool wanted = false;
    if (app) {
        tok = a.pos[b];
        wanted = a.count == nullptr || a.count[b] >= 1;
    }
    const T *Wg = (const T *)a.W + (int64_t)h * d * a.LP + col0;
    const int row_bytes = cols * (int)sizeof(T);
    // Three ways to fetch the slab: 16-byte vectors when a channel's planes are whole vectors
    // (8 planes of bf16), dwords when they are whole dwords (10 planes of bf16: 5 each), else
    // element by element.  i / n for i < 4096 and n <= 16 is a multiplication by ceil(2^16 / n).
    const bool wvec = (row_bytes & 15) == 0 && ((a.LP * (int)sizeof(T)) & 15) == 0;
    const bool wdw = DW && !wvec && sizeof(T) == 2 && (row_bytes & 3) == 0 && ((a.LP * (int)sizeof(T)) & 3) == 0 &&
                     ((col0 * (int)sizeof(T)) & 3) == 0;
    const int nvec = row_bytes >> 4;                         // 16-byte vectors per channel (vector path)
    const int ndw = row_bytes >> 2;                          // dwords per channel (dword path)
    auto div_small = [](int i, int n, int &rem) {
        const int q = (int)(((uint32_t)i * ((65536u + (uint32_t)n - 1u) / (uint32_t)n)) >> 16);
        rem = i - q * n;
        return q;
    };
    constexpr int WV = 4, WD = DW ? 8 : 1, WE = 16;
    uint4 wv[WV];
    uint32_t wq[WD];
    T we[WE];
    if (live && wvec) {
#pragma unroll
        for (int j = 0; j < WV; ++j) {
            const int i = tid + j * 256;
            if (i < d * nvec) wv[j] = *(const uint4 *)(Wg + (int64_t)(i / nvec) * a.LP + (i % nvec) * EPV);
        }
    } else if (live && wdw) {
#pragma unroll
        for (int j = 0; j < WD; ++j) {
            const int i = tid + j * 256;
            int part;
            const int c = div_small(i, ndw, part);
            if (i < d * ndw) wq[j] = *(const uint32_t *)((const char *)(Wg + (int64_t)c * a.LP) + part * 4);
        }
    } else if (live) {
#pragma unroll
        for (int j = 0; j < WE; ++j) {
            const int i = tid + j * 256;
            int part;
            const int c = div_small(i, cols, part);
            if (i < d * cols) we[j] = Wg[(int64_t)c * a.LP + part];
        }
    }
    constexpr int QV = (G * 256 * (int)sizeof(T) / 16 + 255) / 256;   // d <= 256
    uint4 qv[QV];
    const int nq = G * d / EPV;
    if (soft && live) {
        const T *qg = (const T *)a.q + ((int64_t)b * a.Hq + h * G) * d;
#pragma unroll
        for (int j = 0; j < QV; ++j) {
            const int i = tid + j * 256;
            if (i < nq) qv[j] = *(const uint4 *)(qg + i * EPV);
        }
    }
    int64_t krow = -1;
    uint4 kv = make_uint4(0, 0, 0, 0);
    if (app) {
        if (wanted && tok >= 0 && tok < a.map.max_n) krow = a.map.row(b, h, tok);
        if (krow >= 0 && live && tid < d / EPV) kv = *(const uint4 *)((const T *)a.K + krow * d + tid * EPV);
        if (a.len_out && x == 0 && h == 0 && tid == 0) a.len_out[b] = tok + 1;
    }
    // 256 value norms spread over the sequence (tok + 1 tokens): their mean and spread scale the
    // histogram bins of the weighted scores
    float nu = 0.0f;
    const bool sampling = a.vnorm != nullptr && app && soft && live && tok >= 0 && tok < a.map.max_n;
    if (sampling) {
        const int seq = tok + 1;
        int t = (int)((float)(l * 256 + tid) * ((float)seq / (float)(a.L * 256)));
        t = t < seq ? t : seq - 1;
        nu = a.vnorm[((int64_t)b * a.Hkv + h) * a.map.max_n + t];
    }

    // ---- into LDS as fp32 / fp64, W transposed to [plane][channel]
    if (live && wvec) {
#pragma unroll
        for (int j = 0; j < WV; ++j) {
            const int i = tid + j * 256;
            if (i < d * nvec) {
                float f[EPV];
                vec_to_f32<T>(wv[j], f);
                const int c = i / nvec, p0 = (i % nvec) * EPV;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    wf[(p0 + e) * d + c] = f[e];
                    wd[(p0 + e) * d + c] = (double)f[e];
                }
            }
        }
    } else if (live && wdw) {
#pragma unroll
        for (int j = 0; j < WD; ++j) {
            const int i = tid + j * 256;
            if (i < d * ndw) {
                int part;
                const int c = div_small(i, ndw, part);
                const float f0 = __uint_as_float(wq[j] << 16), f1 = __uint_as_float(wq[j] & 0xffff0000u);   // two bf16
                wf[(2 * part) * d + c] = f0;
                wd[(2 * part) * d + c] = (double)f0;
                wf[(2 * part + 1) * d + c] = f1;
                wd[(2 * part + 1) * d + c] = (double)f1;
            }
        }
    } else if (live) {
#pragma unroll
        for (int j = 0; j < WE; ++j) {
            const int i = tid + j * 256;
            if (i < d * cols) {
                const float f = elem_to_f32<T>(we[j]);
                int part;
                const int c = div_small(i, cols, part);
                wf[part * d + c] = f;
                wd[part * d + c] = (double)f;
            }
        }
    }
    if (soft && live) {
#pragma unroll
        for (int j = 0; j < QV; ++j) {
            const int i = tid + j * 256;
            if (i < nq) {
                float f[EPV];
                vec_to_f32<T>(qv[j], f);
#pragma unroll
                for (int e = 0; e < EPV; ++e) qd[i * EPV + e] = (double)f[e];
            }
        }
        if (tid < G * kPlanePad * 2) sig[tid] = 1.0;
    }
    if (app && tid < d / EPV) {
        float f[EPV];
        vec_to_f32<T>(kv, f);
#pragma unroll
        for (int e = 0; e < EPV; ++e) kf[tid * EPV + e] = f[e];
    }
    if (tid < 16) sgn[tid] = 0;
    __syncthreads();
    SK_STAMP2(1);

    // ---- appended key: 16 lanes per hyperplane, fp32 FMA over a 16th of the channels each
    if (app && live) {
        const int pl = tid >> 4, part = tid & 15;            // 16 planes x 16 parts = 256 threads
        const int per = d >> 4;                              // 4, 8 or 16 channels
        float acc = 0.0f;
        if (pl < cols) {
            // lane `part` takes channel quads part, part+16, ...: the 16 lanes of a plane read
            // 256 contiguous bytes at a time, free of bank conflicts
            const float4 *k4 = (const float4 *)kf + part;
            const float4 *w4 = (const float4 *)(wf + pl * d) + part;
            for (int c = 0; c < per / 4; ++c) {
                const float4 kk = k4[c * 16], ww = w4[c * 16];
                acc = fmaf(kk.x, ww.x, acc);
                acc = fmaf(kk.y, ww.y, acc);
                acc = fmaf(kk.z, ww.z, acc);
                acc = fmaf(kk.w, ww.w, acc);
            }
        }
        acc = row_sum<16>(acc);
        if (pl < cols && part == 0) sgn[pl] = acc >= 0.0f ? 1u : 0u;
    }
    SK_STAMP2(8);
    // ---- queries: fp64 dot products, tpp lanes each; then u = tanh(z)/sqrt(d) and the
    //      per-plane sigmoids of +-2u/tau
    if (soft && live) {
        const int npairs = G * cols;                         // <= 128
        int lg = 0;                                          // log2 of the lanes per dot product,
        while ((2 << lg) * npairs <= 256 && lg < 4 && (d >> (lg + 1)) >= 8) ++lg;   // >= 8 channels each
        const int tpp = 1 << lg;
        const int pair = tid >> lg, part = tid & (tpp - 1);
        const bool mine = pair < npairs;
        const int g = mine ? (pair * a.cols_magic) >> 16 : 0;   // pair / cols
        const int j = mine ? pair - g * cols : 0;
        const int per = d >> lg;                             // a multiple of 8
        // lane `part` takes channel pairs part, part+tpp, ...: the lanes of a dot product read
        // contiguous bytes, free of bank conflicts
        const double2 *q2 = (const double2 *)(qd + g * d) + part;
        const double2 *w2 = (const double2 *)(wd + j * d) + part;
        double z0 = 0.0, z1 = 0.0;
        for (int c0 = 0; c0 < per / 8; ++c0) {               // 8 channels' LDS reads issued together
            double2 wv2[4], qv2[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                wv2[e] = w2[(4 * c0 + e) << lg];
                qv2[e] = q2[(4 * c0 + e) << lg];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                z0 = fma(wv2[e].x, qv2[e].x, z0);
                z1 = fma(wv2[e].y, qv2[e].y, z1);
            }
        }
        SK_STAMP2(9);
        const double z = group_sum_f64(z0 + z1, tpp);
        SK_STAMP2(10);
        if (mine && part == 0) {
            // tanh|z| = (1 - t)/(1 + t) with t = exp(-2|z|); sigmoid(+-x) from e = exp(-|x|)
            const double t = exp(-2.0 * fabs(z));
            const double th = (1.0 - t) * rcp64(1.0 + t);
            const double e = exp(-a.x_scale * th);           // x = 2 tanh|z| / (sqrt(d) tau) >= 0
            double big = rcp64(1.0 + e), small = e * big;
            if (a.hard) {                            // the limit tau -> 0: all mass on the query's side of the plane
                big = 1.0;
                small = 0.0;
            }
            const int slot = (a.mode == kFactor && j >= a.Plo) ? 8 + j - a.Plo : j;
            sig[(g * kPlanePad + slot) * 2 + 1] = z >= 0.0 ? big : small;
            sig[(g * kPlanePad + slot) * 2] = z >= 0.0 ? small : big;
        }
        SK_STAMP2(11);
    }
    __syncthreads();
    SK_STAMP2(2);

    // the appended key's bucket id for this table, written by one thread
    auto write_code = [&]() {
        uint32_t code = 0;
        if (live) {
            uint4 sg[4];                             // all 16 sign words in one LDS round trip
#pragma unroll
            for (int i = 0; i < 4; ++i) sg[i] = ((const uint4 *)sgn)[i];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                code |= (sg[i].x << (4 * i)) | (sg[i].y << (4 * i + 1)) | (sg[i].z << (4 * i + 2)) | (sg[i].w << (4 * i + 3));
        }
        if (a.mode == kSplit) {
            // packed ids: the 10 bits sit in one or two dwords that other tables (other
            // workgroups) write too, so they are cleared and set with atomics
            const int grp = l / a.GT, j = packed_pos(l % a.GT, tok, a.S);
            const int sub = j >> 4, bit = 10 * (j & 15), wi = bit >> 5, sh = bit & 31;
            uint32_t *w0 = (uint32_t *)((char *)a.codes + packed_word(krow, grp, sub, wi, a.Lpad, a.GT));
            atomicAnd(w0, ~(0x3ffu << sh));
            atomicOr(w0, code << sh);
            if (sh > 22) {
                uint32_t *w1 = (uint32_t *)((char *)a.codes + packed_word(krow, grp, sub, wi + 1, a.Lpad, a.GT));
                atomicAnd(w1, ~(0x3ffu >> (32 - sh)));
                atomicOr(w1, code >> (32 - sh));
            }
            return;
        }
        const int64_t at = krow * a.Lpad + code_pos(l, tok, a.S);
        if (a.cb == 1) ((uint8_t *)a.codes)[at] = (uint8_t)code;
        else ((uint16_t *)a.codes)[at] = (uint16_t)code;
    };
    const bool code_due = app && krow >= 0;
    if (!soft) {
        if (code_due && tid == 0) write_code();
        return;
    }
    SK_STAMP2(3);

    const int lw = a.Lpad < 64 ? a.Lpad : 64;        // distinct tables per 64-word row
    const int copies = 64 / lw;
    const int c64 = l >> 6, lp = l & 63;
    float *Tg = a.tables + ((int64_t)b * a.Hkv + h) * a.table_words;
    // product over the 8 slots s0 .. s0+7 of the sigmoid picked by the bits of `bits` (bits of
    // unused slots are 0 and pick a stored 1); the 8 LDS reads are independent
    auto plane_product = [&](int g, int s0, int bits) -> double {
        double f[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = sig[(g * kPlanePad + s0 + i) * 2 + ((bits >> i) & 1)];
        return ((f[0] * f[1]) * (f[2] * f[3])) * ((f[4] * f[5]) * (f[6] * f[7]));
    };
    if (a.mode == kDirect || a.mode == kSplit) {
        // p(r) over all planes, averaged over the G queries: one entry per thread and pass
        // (planes 8 and 9 of the split form sit in slots 8 and 9)
        const double inv_g = 1.0 / (double)G, inv_r = 1.0 / (double)a.R;
        const bool split = a.mode == kSplit;
        // split form: the products over planes 0..7 for each low byte of the id and over planes
        // 8, 9 for its two high bits, once per query head; an entry is then one product of two
        constexpr int kAb = 256 + 4;
        double *ab = (double *)(s_dev + 12);         // [G][kAb]
        if (split) {
            for (int i = tid; i < G * kAb; i += 256) {
                const int g = i / kAb, r = i - g * kAb;
                ab[i] = !live ? 0.0 : r < 256 ? plane_product(g, 0, r) : plane_product(g, 8, r - 256);
            }
            __syncthreads();
        }
        float dev2 = 0.0f;
        if (split) {
            // four consecutive buckets per thread, stored as one 16-byte piece: a group's table
            // is kept as [bucket / 4][table][4] (the other tables of the group come from other
            // workgroups, so longer contiguous runs per table mean fewer partial writes)
            for (int r4 = tid; r4 < (a.R >> 2); r4 += 256) {
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 4 * r4 + j;
                    double mean = 0.0;
                    if (live) {
#pragma unroll
                        for (int g = 0; g < G; ++g) mean += ab[g * kAb + (r & 255)] * ab[g * kAb + 256 + (r >> 8)];
                        mean *= inv_g;
                        const double dv = mean - inv_r;
                        dev2 += (float)(dv * dv);
                    }
                    v[j] = (float)mean;
                }
                *(float4 *)&Tg[(((int64_t)(l / a.GT) * (a.R >> 2) + r4) * a.GT + l % a.GT) * 4] =
                    make_float4(v[0], v[1], v[2], v[3]);
            }
        }
        for (int r = tid; r < a.R && !split; r += 256) {
            double mean = 0.0;
            if (live) {
#pragma unroll
                for (int g = 0; g < G; ++g) mean += plane_product(g, 0, r);
                mean *= inv_g;
                const double dv = mean - inv_r;      // a table's entries sum to 1: their mean is 1/R
                dev2 += (float)(dv * dv);
            }
            for (int cp = 0; cp < copies; ++cp) Tg[((int64_t)c64 * a.R + r) * 64 + lp + cp * lw] = (float)mean;
        }
        // spread of this table's entries, from which the scoring pass sizes its histogram bins
        dev2 = row_sum<64>(dev2);
        const float nu1 = row_sum<64>(nu), nu2 = row_sum<64>(nu * nu);
        if ((tid & 63) == 0) {
            s_dev[tid >> 6] = dev2;
            s_dev[4 + (tid >> 6)] = nu1;
            s_dev[8 + (tid >> 6)] = nu2;
        }
        __syncthreads();
        if (tid < 3) {
            const float *part = s_dev + 4 * tid;
            const double sum = (double)(part[0] + part[1] + part[2] + part[3]);
            a.tstats[(((int64_t)b * a.Hkv + h) * a.Lpad + l) * 3 + tid] = (float)(tid == 0 ? sum * inv_r : sum);
        }
        if (code_due && tid == 64) write_code();     // off the first wavefront's path
        SK_STAMP2(5);
    } else {
        // products over the low and the high planes: p(r) = lo[r & (Rlo-1)] * hi[r >> Plo]
        const int hrows = a.Rlo + a.Rhi;
        for (int i = tid; i < hrows * G; i += 256) {
            const int row = i % hrows, g = i / hrows;
            double p = 0.0;
            if (live) {
                p = row < a.Rlo ? plane_product(g, 0, row) / (double)G   // the 1/G of the group mean rides on the low factor
                                : plane_product(g, 8, row - a.Rlo);
            }
            for (int cp = 0; cp < copies; ++cp)
                Tg[(((int64_t)g * a.rounds + c64) * hrows + row) * 64 + lp + cp * lw] = (float)p;
        }
        if (code_due && tid == 64) write_code();
    }
}

// ---------------------------------------------------------------------------------------

struct ScoreArgs {
    const void *codes;
    const float *tables;
    const float *vnorm;
    const int32_t *seq_len;
    float *scores;
    uint32_t *hist;          // optional [B*Hkv][kHistBins]: first-level histogram of the scores
    const float *tstats;     // [B*Hkv][Lpad][3] per-table spread, sampled value norms (adaptive histogram only)
    uint32_t *thr;           // [B*Hkv][kThrStride] threshold records: receives the binning
    int hist_mode;           // HistMode of `hist`
    int n_sink, n_window;    // the first n_sink and last n_window tokens of a sequence score +inf
    RowMap map;
    int L, Lpad, rounds, R, G, Plo, Rlo, table_rows;
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
    const bool adaptive = a.hist_mode == kHistAdaptive;
    float bin_lo = 0.0f, bin_inv = 0.0f;             // adaptive histogram bins, set once the table is in

    const int sub = lane % S, kk = lane / S;
    const int lw = a.Lpad < 64 ? a.Lpad : 64;
    uint32_t woff[16];                               // byte offset of this lane's table in a 64-float row
#pragma unroll
    for (int s = 0; s < 16; ++s) woff[s] = 4u * (uint32_t)(sub + S * ((kk + s) & 15) + lw * (kk >> 4));
    const uint32_t tbase = (uint32_t)(size_t)(lds_float_t *)tbl;
    uint32_t *lhist = (uint32_t *)(tbl + a.table_words);
    // (no static __shared__ in this kernel: the table has to sit at LDS address 0 for the
    // fast address path)
    float *s_bin = (float *)(lhist + kHistBins);     // [2], present with a histogram only
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
    // value-norm weights of the keys this lane emits for a chunk (fetched with the ids, so that
    // their latency is hidden the same way)
    constexpr int EPL = U / S;
    auto load_weights = [&](float *w, int base) {
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int key = base + (j * S + sub) * KPW + kk;
            w[j] = (vn && key < seq) ? vn[key] : 1.0f;
        }
    };
    auto emit = [&](int base, const float *sum, const bool *dead, const float *w) {
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
                if (dd) {
                    v = ninf;
                } else {
                    v *= w[j];
                    if (key < a.n_sink || key >= seq - a.n_window) v = __builtin_inff();   // sink / local window
                }
                out[key] = v;
                if (a.hist && v > ninf) {
                    const uint32_t bin = adaptive ? score_bin(v, bin_lo, bin_inv)
                                                  : score_order_key(v) >> (32 - kHistBits);
                    atomicAdd(&lhist[bin], 1u);
                }
            }
        }
    };
    // (keys at or beyond the sequence, which only the leftover region has, read the last row
    // of the buffer instead and are marked dead: every set is the same sequence of loads, so
    // the number of loads in flight stays known)
    auto load_set = [&](CodeVec<CB> *cv, bool *dead, float *w, int base) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int key = base + u * KPW + kk;
            cv[u].load(code_ptr(min(key, max_n - 1), 0, dead[u]));
            dead[u] = dead[u] || key >= seq;
        }
        load_weights(w, base);
    };
    auto chunk_base = [&](int r) { return (r * stride + (int)blockIdx.x) * CKEYS + wave * WKEYS; };

    constexpr bool PREFETCH = ONE_ROUND;
    // The leftover region is taken U passes at a time per wavefront.  With PREFETCH a
    // wavefront's first such set rides the ping-pong below as one more round (its loads in
    // flight during the last whole chunk's look-ups) instead of costing a memory latency of
    // its own at the end of the kernel: a sequence length that is not a whole number of rounds,
    // the usual case while decoding, then costs what the next whole number would.
    const int npass = (max_n - left0 + KPW - 1) / KPW;
    const int p_first = ((int)blockIdx.x * NW + wave) * U;
    const int left_base = left0 + p_first * KPW;
    const int nr = nround + (PREFETCH && p_first < npass ? 1 : 0);
    auto round_base = [&](int r) { return r < nround ? chunk_base(r) : left_base; };
    CodeVec<CB> setA[U], setB[U];
    bool deadA[U], deadB[U];
    float wgtA[EPL], wgtB[EPL];
    if (PREFETCH && nr > 0) load_set(setA, deadA, wgtA, round_base(0));
    // Adaptive histogram: if the keys' bucket ids were uniform, a score would have mean L/R and
    // variance sum_l var_l; bins are laid from four deviations below that mean upwards.
    float var_part = 0.0f, nu1_part = 0.0f, nu2_part = 0.0f;
    if (adaptive && wave == 0)
        for (int l = lane; l < a.Lpad; l += 64) {
            const float *ts = a.tstats + (bh * a.Lpad + l) * 3;
            var_part += ts[0];
            nu1_part += ts[1];
            nu2_part += ts[2];
        }
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
    if (adaptive && wave == 0) {
        float mu = (float)a.L / (float)a.R;
        float var = row_sum<64>(var_part);
        const float nu1 = row_sum<64>(nu1_part), nu2 = row_sum<64>(nu2_part);
        if (vn) {
            // weighted scores nu * s, nu and s taken as independent: moments of the product
            const float cnt = (float)(a.L * 256);
            const float mnu = nu1 / cnt, vnu = fmaxf(nu2 / cnt - mnu * mnu, 0.0f);
            var = mnu * mnu * var + mu * mu * vnu + vnu * var;
            mu *= mnu;
        }
        const float sigma = fmaxf(sqrtf(var), fmaxf(mu * 1e-6f, 1e-30f));
        const float lo = mu - 4.0f * sigma, inv = 1.0f / (4.0f * sigma);
        if (lane == 0) {
            s_bin[0] = lo;
            s_bin[1] = inv;
            if (blockIdx.x == 0) {       // the select's sweep bins with the very same pair
                a.thr[bh * kThrStride + kThrBinLo] = __float_as_uint(lo);
                a.thr[bh * kThrStride + kThrBinInv] = __float_as_uint(inv);
            }
        }
    }
    __syncthreads();
    if (adaptive) {
        bin_lo = s_bin[0];
        bin_inv = s_bin[1];
    }

    // ---- whole chunks: branch-free, the next chunk's loads in flight during the look-ups
    auto full_chunks = [&](auto base0) {
        constexpr bool BASE0 = decltype(base0)::value;
        auto process = [&](const CodeVec<CB> *cv, const bool *dead, const float *w, int base) {
            float sum[U];
#pragma unroll
            for (int u = 0; u < U; ++u) sum[u] = group_sum<S>(gather16<CB, MODE, BASE0, BASE0 && ONE_ROUND>(cv[u], tbase, woff, 0, a));
            emit(base, sum, dead, w);
        };
        if (PREFETCH) {
            int r = 0;
            while (r < nr) {
                if (r + 1 < nr) load_set(setB, deadB, wgtB, round_base(r + 1));
                process(setA, deadA, wgtA, round_base(r));
                if (++r >= nr) break;
                if (r + 1 < nr) load_set(setA, deadA, wgtA, round_base(r + 1));
                process(setB, deadB, wgtB, round_base(r));
                ++r;
            }
        } else {
            for (int r = 0; r < nround; ++r) {
                const int base = chunk_base(r);
                float sum[U], w[EPL];
                bool dead[U];
                load_weights(w, base);
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
                emit(base, sum, dead, w);
            }
        }
    };
    if (tbase == 0) full_chunks(BoolTag<true>());
    else full_chunks(BoolTag<false>());

    // ---- (the rest of) the leftover keys and the -inf fill beyond the sequence
    for (int p0 = p_first + (nr > nround ? stride * NW * U : 0); p0 < npass; p0 += stride * NW * U) {
        const int base = left0 + p0 * KPW;
        float sum[U], w[EPL];
        bool dead[U];
        CodeVec<CB> cv[U];
        load_weights(w, base);
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
        emit(base, sum, dead, w);
    }

    if (a.hist && has_table) {
        __syncthreads();
        uint32_t *gh = a.hist + bh * kHistBins;
        for (int i = tid; i < kHistBins; i += kScoreThreads)
            if (lhist[i]) atomicAdd(&gh[i], lhist[i]);
    }
}

// ---------------------------------------------------------------------------------------
// Split tables (P = 9, 10; packed 10-bit ids).  The one-entry-per-bucket table of 64 tables
// does not fit in LDS, so a workgroup (one per CU, 16 wavefronts) goes through the groups of
// GT = 16 S tables one after the other: group table -> LDS, then every key it owns adds the
// group's look-ups to the partial sum it left in `scores` during the previous group.  A
// wavefront takes U passes of 64/S keys at a time, the same keys in every group; a lane reads
// 16 low bytes and one dword of high-bit pairs per key and group.  The last group applies
// weights, forced tokens and the mask, and feeds the histogram.
// ---------------------------------------------------------------------------------------
#ifndef SK_SPLIT_THREADS
#define SK_SPLIT_THREADS 1024
#endif
constexpr int kSplitThreads = SK_SPLIT_THREADS;

// bins of the adaptive histogram, from the per-table spreads the projection pass left (and, for
// weighted scores, from the value norms it sampled); called by one whole wavefront
__device__ __forceinline__ void adaptive_bin_params(const ScoreArgs &a, int64_t bh, int lane, bool weighted,
                                                    float *lo, float *inv) {
    float var_part = 0.0f, nu1_part = 0.0f, nu2_part = 0.0f;
    for (int l = lane; l < a.Lpad; l += 64) {
        const float *ts = a.tstats + (bh * a.Lpad + l) * 3;
        var_part += ts[0];
        nu1_part += ts[1];
        nu2_part += ts[2];
    }
    float mu = (float)a.L / (float)a.R;
    float var = row_sum<64>(var_part);
    const float nu1 = row_sum<64>(nu1_part), nu2 = row_sum<64>(nu2_part);
    if (weighted) {          // weighted scores nu * s, nu and s taken as independent: moments of the product
        const float cnt = (float)(a.L * 256);
        const float mnu = nu1 / cnt, vnu = fmaxf(nu2 / cnt - mnu * mnu, 0.0f);
        var = mnu * mnu * var + mu * mu * vnu + vnu * var;
        mu *= mnu;
    }
    const float sigma = fmaxf(sqrtf(var), fmaxf(mu * 1e-6f, 1e-30f));
    *lo = mu - 4.0f * sigma;
    *inv = 1.0f / (4.0f * sigma);
}

// ids of the U keys a lane works on in one turn, with what the keys it emits carry over
template <int U, int EPL> struct SplitSet {
    uint4 main[U];                                   // words 0..3 and word 4 of the 160-bit strings
    uint32_t tail[U];
    bool dead[U];
    float carry[EPL], w[EPL];
};

template <int S, bool PAGED>
__global__ __launch_bounds__(kSplitThreads) void score_split_kernel(ScoreArgs a) {
    extern __shared__ float tbl[];
    constexpr int GT = 16 * S;                       // tables per group
    constexpr int KPW = 64 / S;                      // keys per wavefront pass
    constexpr int NW = kSplitThreads / 64;
#ifndef SK_SPLIT_U
#define SK_SPLIT_U 2
#endif
    constexpr int U = SK_SPLIT_U;                    // passes a wavefront takes per turn
    constexpr int EPL = U / S;                       // results a lane emits per turn
    constexpr int TP = 8192 / kSplitThreads;         // float4 of a group table each thread moves (at most 128 KB in all)
    typedef SplitSet<U, EPL> Set;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: so is all turn bookkeeping
    const int h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)b * a.map.Hkv + h;
    const int max_n = a.map.max_n;
    int seq = a.seq_len[b];
    seq = seq < 0 ? 0 : (seq > max_n ? max_n : seq);
    float *out = a.scores + bh * max_n;
    const float *vn = a.vnorm ? a.vnorm + bh * max_n : nullptr;
    const float ninf = -__builtin_inff();
    const bool adaptive = a.hist_mode == kHistAdaptive;
    const int sub = lane % S, kk = lane / S;
    uint32_t woff[16];                               // byte offset of this lane's table in a GT-float row
#pragma unroll
    for (int s = 0; s < 16; ++s) woff[s] = 4u * (uint32_t)(sub + S * ((kk + s) & 15));
    const int group_words = a.R * GT;
    const int n4 = group_words >> 2;                 // <= TP * kSplitThreads
    uint32_t *lhist = (uint32_t *)(tbl + group_words);
    float *s_bin = (float *)(lhist + kHistBins);     // [2], present with a histogram only
    const char *cb = (const char *)a.codes;
    float bin_lo = 0.0f, bin_inv = 0.0f;

    // A wavefront's turns: U passes of KPW keys each, the same keys in every group.  Turns
    // cover the keys below seq only (the rest of the row is filled with -inf), and inside a
    // turn nothing branches on a key being absent: its loads go to a row that exists and its
    // result is dropped, so that the number of loads in flight is fixed and a set can be waited
    // for while the next one is still on its way.
    const int npass = (seq + KPW - 1) / KPW;
    const int stride = gridDim.x * NW * U;
    const int first_p0 = ((int)blockIdx.x * NW + wave) * U;
    const int nturn = first_p0 < npass ? (npass - first_p0 + stride - 1) / stride : 0;
    const float *wsrc = vn ? vn : out;               // weights, or anything loadable

    // this lane's part of a string address that does not change from turn to turn: its token's
    // tile among the tiles of a pass, its row in the tile, its string in the row
    const uint32_t lane_main = (uint32_t)((kk >> 4) * (int)packed_tile_bytes(a.Lpad) + (kk & 15) * GT + sub * 16);
    const uint32_t lane_tail = (uint32_t)((kk >> 4) * (int)packed_tile_bytes(a.Lpad) + 16 * GT + (kk & 15) * (GT >> 2) + sub * 4);
    // (grp, tix): group and turn inside the group
    auto load_set = [&](Set &st, int grp, int tix) __attribute__((always_inline)) {
        const int base = (first_p0 + tix * stride) * KPW;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int key = base + u * KPW + kk;
            st.dead[u] = key >= seq;
            typedef unsigned int u4 __attribute__((ext_vector_type(4)));
            u4 t;
            if (PAGED) {
                int64_t row = a.map.row(b, h, st.dead[u] ? 0 : key);
                st.dead[u] = st.dead[u] || row < 0;
                row = row < 0 ? 0 : row;
                t = __builtin_nontemporal_load((const u4 *)(cb + packed_word(row, grp, sub, 0, a.Lpad, GT)));
                st.tail[u] = __builtin_nontemporal_load((const uint32_t *)(cb + packed_word(row, grp, sub, 4, a.Lpad, GT)));
            } else {
                // one address for the whole pass (its first token starts a tile), plus the lane's
                // own offset; a key beyond the row's capacity reads the pass's first token instead
                const char *pass = cb + packed_main_row(bh * max_n + base + u * KPW, grp, a.Lpad, GT);
                const bool inside = key < max_n;
                t = __builtin_nontemporal_load((const u4 *)(pass + (inside ? lane_main : 0u)));
                st.tail[u] = __builtin_nontemporal_load((const uint32_t *)(pass + (inside ? lane_tail : (uint32_t)(16 * GT))));
            }
            st.main[u] = make_uint4(t.x, t.y, t.z, t.w);
        }
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            int key = base + (j * S + sub) * KPW + kk;
            key = key < seq ? key : 0;
            // (with a single turn per group the partial sums are written by the turn that is
            // still ahead when this runs: process() fetches them itself then)
            st.carry[j] = out[key];
            st.w[j] = wsrc[key];
        }
    };
    auto process = [&](const Set &st, int grp, int tix) __attribute__((always_inline)) {
        const int base = (first_p0 + tix * stride) * KPW;
        const bool first = grp == 0, last = grp == a.rounds - 1;
        float sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t sw[5] = {st.main[u].x, st.main[u].y, st.main[u].z, st.main[u].w, st.tail[u]};
            float p[16];
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                // id s = bits [10 s, 10 s + 10) of the string; its table entry is at id * (4 GT) + woff
                constexpr uint32_t kIdMask = 0x3ffu * (uint32_t)(GT * 4);
                const int wi = (10 * s) >> 5, sh = (10 * s) & 31;
                uint32_t x;                          // the id, shifted left by log2(4 GT), plus other bits
                constexpr int LG = S == 2 ? 7 : 6;
                if (sh > 22) x = __builtin_amdgcn_alignbit(sw[wi + 1], sw[wi], sh - LG);   // sh - LG > 0 here
                else if (sh >= LG) x = sw[wi] >> (sh - LG);
                else x = sw[wi] << (LG - sh);
                p[s] = lds_read((x & kIdMask) | woff[s]);     // the table starts at LDS address 0
            }
            float acc0 = p[0], acc1 = p[1];
#pragma unroll
            for (int s = 2; s < 16; s += 2) {
                acc0 += p[s];
                acc1 += p[s + 1];
            }
            sum[u] = group_sum<S>(acc0 + acc1);
        }
        // lane `sub` of a key's group emits the results of passes sub, sub+S, ...
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            float v = sum[j * S];
            bool dd = st.dead[j * S];
#pragma unroll
            for (int t = 1; t < S; ++t) {
                v = sub == t ? sum[j * S + t] : v;
                dd = sub == t ? st.dead[j * S + t] : dd;
            }
            const int key = base + (j * S + sub) * KPW + kk;
            if (key >= seq) continue;
            if (!first) v += nturn == 1 ? out[key] : st.carry[j];
            if (!last) {
                if (!dd) out[key] = v;
                continue;
            }
            if (dd) {
                v = ninf;
            } else {
                if (vn) v *= st.w[j];
                if (key < a.n_sink || key >= seq - a.n_window) v = __builtin_inff();   // sink / local window
            }
            out[key] = v;
            if (a.hist && v > ninf) {
                const uint32_t bin = adaptive ? score_bin(v, bin_lo, bin_inv)
                                              : score_order_key(v) >> (32 - kHistBits);
                atomicAdd(&lhist[bin], 1u);
            }
        }
    };
    // a group's table goes through registers, so that its loads can be in flight while the
    // previous group's last turn still reads the table in LDS
    float4 tp[TP];
    auto table_fetch = [&](int grp) __attribute__((always_inline)) {
        const float4 *src = (const float4 *)(a.tables + bh * a.table_words + (int64_t)grp * group_words);
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int i = tid + j * kSplitThreads;
            tp[j] = i < n4 ? src[i] : make_float4(0, 0, 0, 0);
        }
    };
    // memory keeps a group's table as [bucket / 4][table][4]; LDS wants [bucket][table] (bank =
    // table): piece i holds buckets 4 (i / GT) .. + 3 of table i % GT
    auto table_commit = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int i = tid + j * kSplitThreads;
            if (i < n4) {
                float *dst = tbl + (4 * (i / GT)) * GT + i % GT;
                dst[0] = tp[j].x;
                dst[GT] = tp[j].y;
                dst[2 * GT] = tp[j].z;
                dst[3 * GT] = tp[j].w;
            }
        }
    };

    // beyond the sequence: -inf
    for (int key = seq + (int)blockIdx.x * kSplitThreads + tid; key < max_n; key += (int)gridDim.x * kSplitThreads)
        out[key] = ninf;
    Set setA, setB;
    if (nturn > 0) load_set(setA, 0, 0);
    if (seq > 0) {
        table_fetch(0);
        table_commit();
    }
    if (a.hist) {
        for (int i = tid; i < kHistBins; i += kSplitThreads) lhist[i] = 0;
        if (adaptive && wave == 0) {
            float lo, inv;
            adaptive_bin_params(a, bh, lane, vn != nullptr, &lo, &inv);
            if (lane == 0) {
                s_bin[0] = lo;
                s_bin[1] = inv;
                if (blockIdx.x == 0) {               // the select's sweep bins with the very same pair
                    a.thr[bh * kThrStride + kThrBinLo] = __float_as_uint(lo);
                    a.thr[bh * kThrStride + kThrBinInv] = __float_as_uint(inv);
                }
            }
        }
    }
    __syncthreads();
    if (adaptive) {
        bin_lo = s_bin[0];
        bin_inv = s_bin[1];
    }

    // Group by group; inside a group the next turn's ids are requested before the current
    // turn is worked on (the last turn of a group requests the first of the next group), two
    // register sets taking turns.  Between groups every wavefront meets to swap the table.
    // (A wavefront without keys still helps to move the tables and keeps the barriers matched.)
    for (int grp = 0; grp < a.rounds; ++grp) {
        if (grp > 0) {
            __syncthreads();                         // every wavefront is done with the previous group's table
            table_fetch(grp);
            table_commit();
            __syncthreads();
        }
        const bool more = grp + 1 < a.rounds;
        int tix = 0;
        while (tix < nturn) {
            if (tix + 1 < nturn) load_set(setB, grp, tix + 1);
            else if (more) load_set(setB, grp + 1, 0);
            process(setA, grp, tix);
            if (++tix >= nturn) {                    // (the sets swap names when a group has an odd number of turns)
                Set t = setA; setA = setB; setB = t;
                break;
            }
            if (tix + 1 < nturn) load_set(setA, grp, tix + 1);
            else if (more) load_set(setA, grp + 1, 0);
            process(setB, grp, tix);
            ++tix;
        }
    }
    if (a.hist && seq > 0) {
        __syncthreads();
        uint32_t *gh = a.hist + bh * kHistBins;
        for (int i = tid; i < kHistBins; i += kSplitThreads)
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
                   int32_t *len_out, int batch, hipStream_t st, const float *vnorm) {
    const Geometry &g = ctx->g;
    ProjectArgs a;
    a.vnorm = (q && K && g.mode != kFactor) ? vnorm : nullptr;
    ctx->vnorm_sampled = a.vnorm;
    a.hard = tau <= 0.0f;                            // internal convention of launch_hard_hash
    if (a.hard) tau = 1.0f;
    a.q = q; a.W = proj; a.tables = ctx->tables; a.tstats = ctx->tstats; a.tau = (double)tau;
    a.x_scale = 2.0 / (sqrt((double)g.d) * (double)tau);
    a.K = K; a.codes = codes; a.pos = pos; a.count = count; a.len_out = len_out;
    a.map = row_map(g, block_table);
    a.d = g.d; a.G = g.G; a.Hkv = g.Hkv; a.Hq = g.Hq; a.L = g.L; a.P = g.P; a.LP = g.L * g.P;
    a.Lpad = g.Lpad; a.S = g.S; a.cb = g.cb; a.rounds = g.rounds; a.R = g.R; a.mode = g.mode;
    a.Plo = g.Plo; a.Phi = g.Phi; a.Rlo = g.Rlo; a.Rhi = g.Rhi; a.table_rows = g.table_rows;
    a.table_words = g.table_words; a.GT = g.GT;
    a.cols_magic = (65536 + g.P - 1) / g.P;
    const size_t lds = (size_t)(2 * g.G * kPlanePad + g.G * g.d + g.P * g.d) * sizeof(double) +
                       (size_t)(g.P * g.d + g.d) * 4 + 64 + 48 +
                       (g.mode == kSplit ? (size_t)g.G * (256 + 4) * sizeof(double) : 0);
    dim3 grid(g.Lpad, g.Hkv, batch);
    typedef void (*project_fn_t)(ProjectArgs);
    project_fn_t fn = nullptr;
    const bool f32 = g.kv_dtype == SOCKET_F32;
    const bool dw = !f32 && (g.P * 2) % 16 != 0 && (g.P * 2) % 4 == 0;    // see project_kernel
    switch (g.G) {
        case 1: fn = f32 ? project_kernel<float, 1, false> : dw ? project_kernel<uint16_t, 1, true> : project_kernel<uint16_t, 1, false>; break;
        case 2: fn = f32 ? project_kernel<float, 2, false> : dw ? project_kernel<uint16_t, 2, true> : project_kernel<uint16_t, 2, false>; break;
        case 4: fn = f32 ? project_kernel<float, 4, false> : dw ? project_kernel<uint16_t, 4, true> : project_kernel<uint16_t, 4, false>; break;
        case 8: fn = f32 ? project_kernel<float, 8, false> : dw ? project_kernel<uint16_t, 8, true> : project_kernel<uint16_t, 8, false>; break;
        default: return SOCKET_EUNSUPPORTED;
    }
    if (set_lds_limit((const void *)fn, lds) != SOCKET_OK) return SOCKET_EHIP;
    hipLaunchKernelGGL(fn, grid, dim3(256), lds, st, a);
    return record_hip(ctx, hipGetLastError());
}

int launch_hard_hash(socket_ctx *ctx, const void *q, const void *proj, int batch, hipStream_t st) {
    return launch_project(ctx, q, proj, 0.0f, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, batch, st);
}

int launch_soft_hash(socket_ctx *ctx, const void *q, const void *proj, float tau, int batch,
                     hipStream_t st) {
    return launch_project(ctx, q, proj, tau, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, batch, st);
}

int launch_score_keys(socket_ctx *ctx, const void *codes, const float *vnorm,
                      const int32_t *block_table, const int32_t *seq_len, int batch, float *scores,
                      bool want_hist, int *hist_mode, hipStream_t st) {
    const Geometry &g = ctx->g;
    ScoreArgs a;
    // The adaptive bins are sized from the one-entry-per-bucket tables (and, for weighted
    // scores, from the value norms the projection pass sampled: only if it sampled these).
    const int mode = !want_hist ? kHistNone
                     : (g.mode != kFactor && (vnorm == nullptr || vnorm == ctx->vnorm_sampled)) ? kHistAdaptive
                                                                                              : kHistDigit;
    if (hist_mode) *hist_mode = mode;
    a.hist_mode = mode; a.tstats = ctx->tstats; a.L = g.L;
    a.n_sink = ctx->n_sink; a.n_window = ctx->n_window;
    a.thr = ctx->counters + (int64_t)g.max_batch * g.Hkv * kCounterStride;
    a.codes = codes; a.tables = ctx->tables; a.vnorm = vnorm; a.seq_len = seq_len; a.scores = scores;
    a.map = row_map(g, block_table);
    a.Lpad = g.Lpad; a.rounds = g.rounds; a.R = g.R; a.G = g.G; a.Plo = g.Plo; a.Rlo = g.Rlo;
    a.table_rows = g.table_rows; a.table_words = g.table_words;
    if (g.mode == kSplit) {
        // one workgroup per CU (a group table fills most of its LDS)
        const int keys_per_turn = (kSplitThreads / 64) * SK_SPLIT_U * (64 / g.S);
        int per_bh = 256 / (batch * g.Hkv);
        const int turns = (g.max_n + keys_per_turn - 1) / keys_per_turn;
        if (per_bh > turns) per_bh = turns;
        if (per_bh < 1) per_bh = 1;
        a.hist = want_hist ? ctx->hist : nullptr;
        const size_t lds = (size_t)g.R * g.GT * 4 + (a.hist ? kHistBins * 4 + 16 : 0);
        const bool paged = g.page > 0;
        score_fn_t fn = g.S == 1 ? (paged ? score_split_kernel<1, true> : score_split_kernel<1, false>)
                                 : (paged ? score_split_kernel<2, true> : score_split_kernel<2, false>);
        if (set_lds_limit((const void *)fn, lds) != SOCKET_OK) return SOCKET_EHIP;
        // the kernel forms its table addresses from LDS address 0: it must own no static LDS
        static int static_lds[4] = {-1, -1, -1, -1};          // per kernel variant, asked once
        int &mine = static_lds[(g.S == 1 ? 0 : 2) + (paged ? 1 : 0)];
        if (mine < 0) {
            hipFuncAttributes attr;
            if (hipFuncGetAttributes(&attr, (const void *)fn) != hipSuccess) return SOCKET_EHIP;
            mine = (int)attr.sharedSizeBytes;
        }
        if (mine != 0) return SOCKET_EUNSUPPORTED;
        hipLaunchKernelGGL(fn, dim3(per_bh, g.Hkv, batch), dim3(kSplitThreads), lds, st, a);
        return record_hip(ctx, hipGetLastError());
    }
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
    a.hist = want_hist ? ctx->hist : nullptr;
    size_t lds = (size_t)g.table_words * 4 + (a.hist ? kHistBins * 4 + 16 : 0);
    score_fn_t fn = pick_score(g);
    if (!fn) return SOCKET_EUNSUPPORTED;
    // more than 64 KB of dynamic LDS has to be allowed per kernel before the launch
    if (set_lds_limit((const void *)fn, lds) != SOCKET_OK) return SOCKET_EHIP;
    hipLaunchKernelGGL(fn, grid, dim3(kScoreThreads), lds, st, a);
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

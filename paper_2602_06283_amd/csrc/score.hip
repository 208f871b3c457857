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
    int pf, Pu;             // ids per byte and the caller's P when ids share bytes (else 1, P)
    double tmean;           // mean of a table's entries: pf / 2^Pu
    float *subprobs;        // ids that share bytes: [B*Hkv][L*pf][2^Pu] probabilities of the caller's tables
    int batch, nb;          // sequences in the call; sequences one workgroup serves (batched kernel)
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
        const double z = group_sum_f64(z0 + z1, tpp);
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
    }
    __syncthreads();

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
    // ids that share a byte (pf tables of Pu planes each): a look-up with the byte gives the sum
    // of the pf tables' probabilities, each a product over its own Pu planes
    auto shared_sum = [&](int g, int bits) -> double {
        double f[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = sig[(g * kPlanePad + i) * 2 + ((bits >> i) & 1)];
        if (a.pf == 2) return (f[0] * f[1]) * (f[2] * f[3]) + (f[4] * f[5]) * (f[6] * f[7]);
        if (a.pf == 4) return (f[0] * f[1] + f[2] * f[3]) + (f[4] * f[5] + f[6] * f[7]);
        return ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
    };
    if (a.pf > 1 && live && tid < a.pf << a.Pu) {
        // the caller's tables one by one, for the read-back
        const int j = tid >> a.Pu, x = tid & ((1 << a.Pu) - 1);
        double mean = 0.0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            double pr = 1.0;
            for (int i = 0; i < a.Pu; ++i) pr *= sig[(g * kPlanePad + j * a.Pu + i) * 2 + ((x >> i) & 1)];
            mean += pr;
        }
        a.subprobs[((((int64_t)b * a.Hkv + h) * a.L + l) * a.pf + j) * (1 << a.Pu) + x] = (float)(mean / (double)G);
    }
    if (a.mode == kDirect || a.mode == kSplit) {
        // p(r) over all planes, averaged over the G queries: one entry per thread and pass
        // (planes 8 and 9 of the split form sit in slots 8 and 9)
        const double inv_g = 1.0 / (double)G, inv_r = 1.0 / (double)a.R;
        const bool split = a.mode == kSplit;
        // split form: the products over planes 0..3, 4..7 and 8, 9 for every value of those bits,
        // once per query head; an entry is then a product of three of them
        constexpr int kAb = 16 + 16 + 4;
        double *ab = (double *)(s_dev + 12);         // [G][kAb]
        if (split) {
            for (int i = tid; i < G * kAb; i += 256) {
                const int g = i / kAb, e = i - g * kAb;
                const int s0 = e < 16 ? 0 : e < 32 ? 4 : 8, bits = e < 32 ? (e & 15) : e - 32;
                const double *sp = sig + (g * kPlanePad + s0) * 2;
                double v = sp[bits & 1] * sp[2 + ((bits >> 1) & 1)];
                if (e < 32) v *= sp[4 + ((bits >> 2) & 1)] * sp[6 + ((bits >> 3) & 1)];
                ab[i] = live ? v : 0.0;
            }
            __syncthreads();
        }
        float dev2 = 0.0f;
        if (split) {
            // four consecutive buckets per thread, stored as one 16-byte piece: a group's table
            // is kept as [bucket / 4][table][4] (the other tables of the group come from other
            // workgroups, so longer contiguous runs per table mean fewer partial writes)
            for (int r4 = tid; r4 < (a.R >> 2); r4 += 256) {
                double mean[4] = {0.0, 0.0, 0.0, 0.0};
                if (live) {
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const double *t = ab + g * kAb;
                        const double up = t[16 + ((r4 >> 2) & 15)] * t[32 + (r4 >> 6)];   // bits 4..7 and 8, 9 of the id
#pragma unroll
                        for (int j = 0; j < 4; ++j) mean[j] = fma(t[(r4 & 3) * 4 + j], up, mean[j]);
                    }
                }
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    mean[j] *= inv_g;
                    if (live) {
                        const double dv = mean[j] - inv_r;
                        dev2 += (float)(dv * dv);
                    }
                    v[j] = (float)mean[j];
                }
                *(float4 *)&Tg[(((int64_t)(l / a.GT) * (a.R >> 2) + r4) * a.GT + l % a.GT) * 4] =
                    make_float4(v[0], v[1], v[2], v[3]);
            }
        }
        for (int r = tid; r < a.R && !split; r += 256) {
            double mean = 0.0;
            if (live) {
                if (a.pf == 1) {
#pragma unroll
                    for (int g = 0; g < G; ++g) mean += plane_product(g, 0, r);
                } else {
#pragma unroll
                    for (int g = 0; g < G; ++g) mean += shared_sum(g, r);
                }
                mean *= inv_g;
                const double dv = mean - a.tmean;    // a table's entries sum to 1: their mean is 1/R
                dev2 += (float)(dv * dv);            // (pf tables' entries summed: pf / 2^Pu)
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
// The same projections for a batch: one workgroup serves one table of one KV head for up to
// `nb` sequences, so the table's slab of W is fetched and laid out once for all of them, and
// every phase works on all `nb` sequences at once (the phases are latency-bound: the second
// to the sixteenth sequence cost little more than the first).  Products of sigmoids are
// built from quarter tables: the 16 products of the four planes of slots 4k .. 4k+3, for
// k = 0..3, per (sequence, query head); an entry of the final table is then two or three
// factors instead of P.
// ---------------------------------------------------------------------------------------
constexpr int kProjThreads = 256;
constexpr int kProjMaxNb = 16;

// bytes of dynamic LDS of project_batch_kernel
static size_t project_batch_lds(int nb, int G, int d, int P, int elem) {
    const int DS = d + 4, DSQ = d + 16 / elem;
    const size_t stage = (size_t)P * DS * 4 + (size_t)nb * G * DSQ * elem + (size_t)nb * DS * 4;   // W, queries, keys
    const size_t quarter = (size_t)nb * G * 64 * 8;
    return (size_t)nb * G * 32 * 8 + (stage > quarter ? stage : quarter) + (size_t)nb * (8 + 4 + 48 + 64) + 64;
}

template <typename T, int G>
__global__ __launch_bounds__(kProjThreads) void project_batch_kernel(ProjectArgs a) {
    extern __shared__ double sm64[];
    constexpr int EPV = 16 / (int)sizeof(T);                 // elements per 16-byte vector
    constexpr int NT = kProjThreads;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int x = blockIdx.x;
    const int l = (x & 7) * (a.Lpad >> 3) + (x >> 3);        // table; the 8 tables sharing lines of W on one XCD
    const int h = blockIdx.y;
    const int b0 = blockIdx.z * a.nb;
    const int nb = min(a.nb, a.batch - b0);
    const int P = a.P, d = a.d;
    const int DS = d + 4, DSQ = d + 16 / (int)sizeof(T);     // padded row strides in LDS: fp32 rows, query rows
    const int col0 = l * P;
    const bool live = l < a.L;                               // tables >= L are padding: zero rows
    const bool soft = a.q != nullptr, app = a.K != nullptr;

    // LDS: sigmoids, then a region used first for the staged operands and later for the quarter
    // tables, then small per-sequence records
    double *sig = sm64;                                      // [nb][G][16 slots][2]
    char *region = (char *)(sig + a.nb * G * 32);
    float *wf = (float *)region;                             // [P][DS]
    T *qs = (T *)(wf + P * DS);                              // [nb][G][DSQ] queries, as stored
    float *kf = (float *)(qs + (size_t)a.nb * G * DSQ);      // [nb][DS]
    double *qt = (double *)region;                           // [nb][G][4][16] quarter tables (after the dot products)
    const size_t stage = (size_t)P * DS * 4 + (size_t)a.nb * G * DSQ * sizeof(T) + (size_t)a.nb * DS * 4;
    const size_t quarter = (size_t)a.nb * G * 64 * 8;
    char *tail = region + (((stage > quarter ? stage : quarter) + 7) & ~(size_t)7);
    int64_t *s_krow = (int64_t *)tail;                       // [nb]
    int *s_tok = (int *)(s_krow + a.nb);                     // [nb]
    float *s_dev = (float *)(s_tok + a.nb);                  // [nb][4 waves][3]
    uint32_t *sgn = (uint32_t *)(s_dev + a.nb * 12);         // [nb][16]

    // ---- global loads, all issued before the first use
    const T *Wg = (const T *)a.W + (int64_t)h * d * a.LP + col0;
    const int row_bytes = P * (int)sizeof(T);
    const bool wvec = (row_bytes & 15) == 0 && ((a.LP * (int)sizeof(T)) & 15) == 0;
    const bool wdw = !wvec && sizeof(T) == 2 && (row_bytes & 3) == 0 && ((a.LP * (int)sizeof(T)) & 3) == 0 &&
                     ((col0 * (int)sizeof(T)) & 3) == 0;
    const int nvec = row_bytes >> 4, ndw = row_bytes >> 2;
    auto div_small = [](int i, int n, int &rem) {            // i / n for i < 4096, n <= 16
        const int q = (int)(((uint32_t)i * ((65536u + (uint32_t)n - 1u) / (uint32_t)n)) >> 16);
        rem = i - q * n;
        return q;
    };
    constexpr int WV = 4, WD = sizeof(T) == 2 ? 8 : 1, WE = 16;
    uint4 wv[WV];
    uint32_t wq[WD];
    T we[WE];
    if (live && wvec) {
#pragma unroll
        for (int j = 0; j < WV; ++j) {
            const int i = tid + j * NT;
            if (i < d * nvec) wv[j] = *(const uint4 *)(Wg + (int64_t)(i / nvec) * a.LP + (i % nvec) * EPV);
        }
    } else if (live && wdw) {
#pragma unroll
        for (int j = 0; j < WD; ++j) {
            const int i = tid + j * NT;
            int part;
            const int c = div_small(i, ndw, part);
            if (i < d * ndw) wq[j] = *(const uint32_t *)((const char *)(Wg + (int64_t)c * a.LP) + part * 4);
        }
    } else if (live) {
#pragma unroll
        for (int j = 0; j < WE; ++j) {
            const int i = tid + j * NT;
            int part;
            const int c = div_small(i, P, part);
            if (i < d * P) we[j] = Wg[(int64_t)c * a.LP + part];
        }
    }
    // appended keys: thread -> (sequence, 16-byte piece of its row); at most KV pieces per thread
    const int kpieces = d / EPV;
    constexpr int KV = (kProjMaxNb * 256 * (int)sizeof(T) / 16 + NT - 1) / NT;
    uint4 kv[KV];
    if (app) {
#pragma unroll
        for (int j = 0; j < KV; ++j) {
            const int i = tid + j * NT;
            kv[j] = make_uint4(0, 0, 0, 0);
            if (i < nb * kpieces && live) {
                const int kb = i / kpieces, piece = i - kb * kpieces;
                const int tok = a.pos[b0 + kb];
                const bool wanted = a.count == nullptr || a.count[b0 + kb] >= 1;
                const int64_t krow = (wanted && tok >= 0 && tok < a.map.max_n) ? a.map.row(b0 + kb, h, tok) : -1;
                if (krow >= 0) kv[j] = *(const uint4 *)((const T *)a.K + krow * d + piece * EPV);
            }
        }
        if (tid < nb) {
            const int tok = a.pos[b0 + tid];
            const bool wanted = a.count == nullptr || a.count[b0 + tid] >= 1;
            s_tok[tid] = tok;
            s_krow[tid] = (wanted && tok >= 0 && tok < a.map.max_n) ? a.map.row(b0 + tid, h, tok) : -1;
            if (a.len_out && x == 0 && h == 0) a.len_out[b0 + tid] = tok + 1;
        }
    }
    // 256 value norms spread over each sequence: their mean and spread scale the histogram bins
    // of the weighted scores
    const bool sampling = a.vnorm != nullptr && app && soft && live;
    if (sampling) {
        for (int kb = 0; kb < nb; ++kb) {
            const int tok = a.pos[b0 + kb];
            float nu = 0.0f;
            if (tok >= 0 && tok < a.map.max_n) {
                const int seq = tok + 1;
                int t = (int)((float)(l * 256 + tid) * ((float)seq / (float)(a.L * 256)));
                t = t < seq ? t : seq - 1;
                nu = a.vnorm[((int64_t)(b0 + kb) * a.Hkv + h) * a.map.max_n + t];
            }
            const float nu1 = row_sum<64>(nu), nu2 = row_sum<64>(nu * nu);
            if (lane == 0) {
                s_dev[(kb * 4 + wave) * 3 + 1] = nu1;
                s_dev[(kb * 4 + wave) * 3 + 2] = nu2;
            }
        }
    } else if (tid < nb * 4) {
        s_dev[tid * 3 + 1] = 0.0f;
        s_dev[tid * 3 + 2] = 0.0f;
    }

    // ---- W into LDS as fp32, transposed to [plane][channel]
    if (live && wvec) {
#pragma unroll
        for (int j = 0; j < WV; ++j) {
            const int i = tid + j * NT;
            if (i < d * nvec) {
                float f[EPV];
                vec_to_f32<T>(wv[j], f);
                const int c = i / nvec, p0 = (i % nvec) * EPV;
#pragma unroll
                for (int e = 0; e < EPV; ++e) wf[(p0 + e) * DS + c] = f[e];
            }
        }
    } else if (live && wdw) {
#pragma unroll
        for (int j = 0; j < WD; ++j) {
            const int i = tid + j * NT;
            if (i < d * ndw) {
                int part;
                const int c = div_small(i, ndw, part);
                wf[(2 * part) * DS + c] = __uint_as_float(wq[j] << 16);
                wf[(2 * part + 1) * DS + c] = __uint_as_float(wq[j] & 0xffff0000u);
            }
        }
    } else if (live) {
#pragma unroll
        for (int j = 0; j < WE; ++j) {
            const int i = tid + j * NT;
            if (i < d * P) {
                int part;
                const int c = div_small(i, P, part);
                wf[part * DS + c] = elem_to_f32<T>(we[j]);
            }
        }
    }
    // ---- queries into LDS as stored (four vectors in flight per thread)
    if (soft && live) {
        const int qpieces = G * d / EPV;                     // 16-byte pieces per sequence
        const int nq = nb * qpieces;
        auto q_src = [&](int i) {
            const int kb = i / qpieces, piece = i - kb * qpieces;
            return (const uint4 *)((const T *)a.q + ((int64_t)(b0 + kb) * a.Hq + h * G) * d + piece * EPV);
        };
        auto q_dst = [&](int i) {
            const int kb = i / qpieces, piece = i - kb * qpieces;
            const int g = piece / (d / EPV), c = (piece - g * (d / EPV)) * EPV;
            return (uint4 *)(qs + ((size_t)(kb * G + g)) * DSQ + c);
        };
        for (int i0 = tid; i0 < nq; i0 += 4 * NT) {
            // (a piece beyond the end reads the last one again and is not stored)
            const int i1 = i0 + NT, i2 = i0 + 2 * NT, i3 = i0 + 3 * NT;
            const uint4 v0 = *q_src(i0);
            const uint4 v1 = *q_src(i1 < nq ? i1 : nq - 1);
            const uint4 v2 = *q_src(i2 < nq ? i2 : nq - 1);
            const uint4 v3 = *q_src(i3 < nq ? i3 : nq - 1);
            *q_dst(i0) = v0;
            if (i1 < nq) *q_dst(i1) = v1;
            if (i2 < nq) *q_dst(i2) = v2;
            if (i3 < nq) *q_dst(i3) = v3;
        }
        for (int i = tid; i < nb * G * 32; i += NT) sig[i] = 1.0;
    }
    if (app) {
#pragma unroll
        for (int j = 0; j < KV; ++j) {
            const int i = tid + j * NT;
            if (i < nb * kpieces) {
                const int kb = i / kpieces, piece = i - kb * kpieces;
                float f[EPV];
                vec_to_f32<T>(kv[j], f);
#pragma unroll
                for (int e = 0; e < EPV; ++e) kf[kb * DS + piece * EPV + e] = f[e];
            }
        }
    }
    for (int i = tid; i < nb * 16; i += NT) sgn[i] = 0;
    __syncthreads();

    // ---- appended keys: fp32 FMA, lpd lanes per (sequence, plane)
    if (app && live) {
        const int ndots = nb * P;                            // <= 256
        int lg = 0;
        while ((2 << lg) * ndots <= NT && lg < 4 && (d >> (lg + 1)) >= 4) ++lg;
        const int lpd = 1 << lg;
        const int dot = tid >> lg, part = tid & (lpd - 1);
        float acc = 0.0f;
        const bool mine = dot < ndots;
        const int kb = mine ? dot / P : 0, pl = mine ? dot - kb * P : 0;
        if (mine) {
            // lane `part` takes channel quads part, part + lpd, ...
            const float4 *k4 = (const float4 *)(kf + kb * DS) + part;
            const float4 *w4 = (const float4 *)(wf + pl * DS) + part;
            const int nquad = d >> (2 + lg);
            for (int c = 0; c < nquad; ++c) {
                const float4 kk = k4[c << lg], ww = w4[c << lg];
                acc = fmaf(kk.x, ww.x, acc);
                acc = fmaf(kk.y, ww.y, acc);
                acc = fmaf(kk.z, ww.z, acc);
                acc = fmaf(kk.w, ww.w, acc);
            }
        }
        if (lpd >= 16) {
            acc += dpp_f32<0x128>(acc);
            acc += dpp_f32<0x124>(acc);
        } else if (lpd >= 8) {
            acc += dpp_f32<0x141>(acc);
        }
        if (lpd >= 4) acc += dpp_f32<0x4E>(acc);
        if (lpd >= 2) acc += dpp_f32<0xB1>(acc);
        if (mine && part == 0) sgn[kb * 16 + pl] = acc >= 0.0f ? 1u : 0u;
    }
    // ---- queries: fp64 dot products, tpp lanes each; u = tanh(z)/sqrt(d), then the per-plane
    //      sigmoids of +-2u/tau
    if (soft && live) {
        const int npairs = nb * G * P;
        int lg = 0;
        while ((2 << lg) * npairs <= NT && lg < 4 && (d >> (lg + 1)) >= 16) ++lg;   // at least 4 channel quads per lane
        const int tpp = 1 << lg;
        const int part = tid & (tpp - 1);
        const int nquad = d >> (2 + lg);                     // channel quads per lane, a multiple of 4
        for (int pair0 = 0; pair0 < npairs; pair0 += NT >> lg) {
            const int pair = pair0 + (tid >> lg);
            const bool mine = pair < npairs;
            const int bg = mine ? pair / P : 0;              // (sequence, query head)
            const int j = mine ? pair - bg * P : 0;
            const T *qrow = qs + (size_t)bg * DSQ;
            const float *wrow = wf + j * DS;
            double z0 = 0.0, z1 = 0.0, z2 = 0.0, z3 = 0.0;
            for (int c0 = 0; c0 < nquad; c0 += 4) {          // nquad is a multiple of 4; 4 quads' LDS reads at a time
                float4 ww[4];
                float qq[4][4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ch = 4 * (part + ((c0 + e) << lg));
                    ww[e] = *(const float4 *)(wrow + ch);
                    if (sizeof(T) == 2) {
                        const uint2 raw = *(const uint2 *)(qrow + ch);
                        qq[e][0] = __uint_as_float(raw.x << 16); qq[e][1] = __uint_as_float(raw.x & 0xffff0000u);
                        qq[e][2] = __uint_as_float(raw.y << 16); qq[e][3] = __uint_as_float(raw.y & 0xffff0000u);
                    } else {
                        const float4 raw = *(const float4 *)(qrow + ch);
                        qq[e][0] = raw.x; qq[e][1] = raw.y; qq[e][2] = raw.z; qq[e][3] = raw.w;
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    z0 = fma((double)ww[e].x, (double)qq[e][0], z0);
                    z1 = fma((double)ww[e].y, (double)qq[e][1], z1);
                    z2 = fma((double)ww[e].z, (double)qq[e][2], z2);
                    z3 = fma((double)ww[e].w, (double)qq[e][3], z3);
                }
            }
            z0 += z2;
            z1 += z3;
            const double z = group_sum_f64(z0 + z1, tpp);
            if (mine && part == 0) {
                // tanh|z| = (1 - t)/(1 + t) with t = exp(-2|z|); sigmoid(+-x) from e = exp(-|x|)
                const double t = exp(-2.0 * fabs(z));
                const double th = (1.0 - t) * rcp64(1.0 + t);
                const double e = exp(-a.x_scale * th);       // x = 2 tanh|z| / (sqrt(d) tau) >= 0
                double big = rcp64(1.0 + e), small = e * big;
                if (a.hard) {                                // the limit tau -> 0
                    big = 1.0;
                    small = 0.0;
                }
                const int slot = (a.mode == kFactor && j >= a.Plo) ? 8 + j - a.Plo : j;
                sig[(bg * 16 + slot) * 2 + 1] = z >= 0.0 ? big : small;
                sig[(bg * 16 + slot) * 2] = z >= 0.0 ? small : big;
            }
        }
    }
    __syncthreads();

    // the appended keys' bucket ids for this table, one thread per sequence
    auto write_code = [&](int kb) {
        const int64_t krow = s_krow[kb];
        if (krow < 0) return;
        const int tok = s_tok[kb];
        uint32_t code = 0;
        if (live)
            for (int i = 0; i < P; ++i) code |= sgn[kb * 16 + i] << i;
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
    if (!soft) {
        if (app && tid < nb) write_code(tid);
        return;
    }

    // ---- quarter tables (over the region that held the staged operands)
    for (int e0 = tid; e0 < nb * G * 64; e0 += 4 * NT) {     // four entries' LDS reads at a time
        double f[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = e0 + j * NT;
            const int bg = e >> 6, quarter = (e >> 4) & 3, bits = e & 15;
            const double *sp = sig + (bg * 16 + quarter * 4) * 2;
            const bool in = e < nb * G * 64;
#pragma unroll
            for (int i = 0; i < 4; ++i) f[j][i] = in ? sp[2 * i + ((bits >> i) & 1)] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = e0 + j * NT;
            if (e < nb * G * 64) qt[e] = live ? (f[j][0] * f[j][1]) * (f[j][2] * f[j][3]) : 0.0;
        }
    }
    __syncthreads();
    if (app && tid >= 64 && tid < 64 + nb) write_code(tid - 64);   // off the first wavefront's path

    const int lw = a.Lpad < 64 ? a.Lpad : 64;            // distinct tables per 64-word row
    const int copies = 64 / lw;
    const int c64 = l >> 6, lp = l & 63;
    const double inv_g = 1.0 / (double)G, inv_r = 1.0 / (double)a.R;
    if (a.mode == kDirect && a.R <= NT) {
        // p(r) over all planes, averaged over the G queries: bucket r = tid of every sequence, four
        // sequences' LDS reads at a time; the spreads of all sequences are reduced together
        const int r = tid;
        float dev2[kProjMaxNb];
#pragma unroll
        for (int k0 = 0; k0 < kProjMaxNb; k0 += 4) {
            double lo[4][G], hi[4][G];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = k0 + j < nb && r < a.R;
                const double *qb = qt + (size_t)(in ? k0 + j : 0) * G * 64;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    lo[j][g] = qb[g * 64 + (r & 15)];
                    hi[j][g] = qb[g * 64 + 16 + ((r >> 4) & 15)];
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int kb = k0 + j;
                dev2[kb] = 0.0f;
                if (kb < nb && r < a.R) {
                    double mean = 0.0;
#pragma unroll
                    for (int g = 0; g < G; ++g) mean += lo[j][g] * hi[j][g];
                    mean *= inv_g;
                    if (live) {
                        const double dv = mean - inv_r;      // a table's entries sum to 1: their mean is 1/R
                        dev2[kb] = (float)(dv * dv);
                    }
                    float *Tg = a.tables + ((int64_t)(b0 + kb) * a.Hkv + h) * a.table_words;
                    for (int cp = 0; cp < copies; ++cp) Tg[((int64_t)c64 * a.R + r) * 64 + lp + cp * lw] = (float)mean;
                }
            }
        }
#pragma unroll
        for (int kb = 0; kb < kProjMaxNb; ++kb) dev2[kb] = row_sum<64>(dev2[kb]);
#pragma unroll
        for (int kb = 0; kb < kProjMaxNb; ++kb)
            if (kb < nb && lane == 0) s_dev[(kb * 4 + wave) * 3] = dev2[kb];
    } else {
    for (int kb = 0; kb < nb; ++kb) {
        float *Tg = a.tables + ((int64_t)(b0 + kb) * a.Hkv + h) * a.table_words;
        const double *qb = qt + (size_t)kb * G * 64;
        float dev2 = 0.0f;
        if (a.mode == kDirect) {            // p(r) over all planes, averaged over the G queries
            for (int r = tid; r < a.R; r += NT) {
                double mean = 0.0;
#pragma unroll
                for (int g = 0; g < G; ++g) mean += qb[g * 64 + (r & 15)] * qb[g * 64 + 16 + (r >> 4)];
                mean *= inv_g;
                if (live) {
                    const double dv = mean - inv_r;          // a table's entries sum to 1: their mean is 1/R
                    dev2 += (float)(dv * dv);
                }
                for (int cp = 0; cp < copies; ++cp) Tg[((int64_t)c64 * a.R + r) * 64 + lp + cp * lw] = (float)mean;
            }
        } else if (a.mode == kSplit) {
            // four consecutive buckets per thread, one 16-byte piece: a group's table is kept
            // [bucket / 4][table][4]
            for (int r4 = tid; r4 < (a.R >> 2); r4 += NT) {
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 4 * r4 + j;
                    double mean = 0.0;
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        mean += (qb[g * 64 + (r & 15)] * qb[g * 64 + 16 + ((r >> 4) & 15)]) * qb[g * 64 + 32 + (r >> 8)];
                    mean *= inv_g;
                    if (live) {
                        const double dv = mean - inv_r;
                        dev2 += (float)(dv * dv);
                    }
                    v[j] = (float)mean;
                }
                *(float4 *)&Tg[(((int64_t)(l / a.GT) * (a.R >> 2) + r4) * a.GT + l % a.GT) * 4] =
                    make_float4(v[0], v[1], v[2], v[3]);
            }
        } else {
            // products over the low and the high planes: p(r) = lo[r & (Rlo-1)] * hi[r >> Plo]
            const int hrows = a.Rlo + a.Rhi;
            for (int i = tid; i < hrows * G; i += NT) {
                const int row = i % hrows, g = i / hrows;
                double p;
                if (row < a.Rlo) p = (qb[g * 64 + (row & 15)] * qb[g * 64 + 16 + (row >> 4)]) * inv_g;   // the 1/G of the group mean rides on the low factor
                else p = qb[g * 64 + 32 + ((row - a.Rlo) & 15)] * qb[g * 64 + 48 + ((row - a.Rlo) >> 4)];
                for (int cp = 0; cp < copies; ++cp)
                    Tg[(((int64_t)g * a.rounds + c64) * hrows + row) * 64 + lp + cp * lw] = (float)p;
            }
        }
        // spread of this table's entries, from which the scoring pass sizes its histogram bins
        dev2 = row_sum<64>(dev2);
        if (lane == 0) s_dev[(kb * 4 + wave) * 3] = dev2;
    }
    }
    if (a.mode == kFactor) return;
    __syncthreads();
    if (tid < nb * 3) {
        const int kb = tid / 3, w = tid - kb * 3;
        const float *part = s_dev + kb * 12 + w;
        const double sum = (double)(part[0] + part[3] + part[6] + part[9]);
        a.tstats[(((int64_t)(b0 + kb) * a.Hkv + h) * a.Lpad + l) * 3 + w] = (float)(w == 0 ? sum * inv_r : sum);
    }
}

// ---------------------------------------------------------------------------------------
// The batched projections in their common case (one-entry-per-bucket tables of P = 4 or 8
// planes, the soft hash wanted): one workgroup serves one sequence, one KV head and a GROUP of
// TG = 128 / P tables, i.e. 128 adjacent columns of W.
//   - The slab of W stays in LDS as stored ([channel][128 columns]); a thread owns two adjacent
//     columns and one or two query heads and a range of channels: one conversion to fp64 per
//     element of W serves two multiply-adds, against two conversions per multiply-add when a
//     thread owns a single (query, plane) pair.
//   - Products of sigmoids come from quarter tables as in the kernels above, laid out
//     table-minor so that lanes over the tables of the group read adjacent words.
//   - A thread's entries of the final tables belong to one table, and 16 (or 32) lanes over the
//     group's tables write adjacent words of a row of the table block: 64-byte (128-byte)
//     runs instead of single words a row apart.
// ---------------------------------------------------------------------------------------
template <bool V> struct GroupTag { static constexpr bool value = V; };
constexpr int kGroupCols = 128;
constexpr int kGroupThreads = 512;

static size_t project_group_lds(int G, int d, int P, int elem) {
    const int TG = kGroupCols / P, NQ = (P + 3) / 4;
    const int QPT = G >= 2 ? 2 : 1, NQG = G / QPT, CS = kGroupThreads / (64 * NQG);
    const size_t slab = (size_t)d * kGroupCols * elem, quarter = (size_t)G * NQ * 16 * TG * 8;
    return (slab > quarter ? slab : quarter) + (size_t)d * G * 8 + (size_t)CS * G * kGroupCols * 8 +
           (size_t)G * P * 2 * TG * 8 + (size_t)d * 4 + (kGroupThreads / 64) * kGroupCols * 4 + 3 * kGroupThreads * 4 + kGroupCols * 4;
}

template <typename T, int G, int P>
__global__ __launch_bounds__(kGroupThreads) void project_group_kernel(ProjectArgs a) {
    extern __shared__ double sm64[];
    constexpr int NT = kGroupThreads, NW = NT / 64, COLS = kGroupCols, TG = COLS / P, R = 1 << P, NQ = (P + 3) / 4;
    constexpr int EPV = 16 / (int)sizeof(T);
    constexpr int QPT = G >= 2 ? 2 : 1;              // query heads per thread
    constexpr int NQG = G / QPT;                     // thread groups over the query heads
    constexpr int CS = NT / (64 * NQG);              // channel ranges
    static_assert(P == 4 || P == 8, "whole quarters");
    static_assert(CS >= 1 && CS * NQG * 64 == NT, "every thread has a share of the dot products");
    const int tid = threadIdx.x;
    const int tg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int d = a.d;
    const int l0 = tg * TG;                          // first table of the group
    const bool app = a.K != nullptr;

    // LDS: the slab of W (later the quarter tables), queries, partial dot products, sigmoids, the key
    const size_t slab = (size_t)d * COLS * sizeof(T), quarter = (size_t)G * NQ * 16 * TG * 8;
    T *ws = (T *)sm64;                               // [d][COLS]
    double *qt = sm64;                               // [G][NQ][16][TG]
    double *qd = (double *)((char *)sm64 + (slab > quarter ? slab : quarter));   // [d][G]
    double *zb = qd + (size_t)d * G;                 // [CS][G][COLS]
    double *sig = zb + CS * G * COLS;                // [G][P][2][TG]
    float *kf = (float *)(sig + G * P * 2 * TG);     // [d]
    float *kz = kf + d;                              // [NW][COLS]
    float *s_part = kz + NW * COLS;                   // [3][NT]
    uint32_t *sgn = (uint32_t *)(s_part + 3 * NT);   // [COLS]

    // ---- global loads, all issued before the first use
    int tok = 0;
    int64_t krow = -1;
    if (app) {
        tok = a.pos[b];
        const bool wanted = a.count == nullptr || a.count[b] >= 1;
        if (wanted && tok >= 0 && tok < a.map.max_n) krow = a.map.row(b, h, tok);
        if (a.len_out && tg == 0 && h == 0 && tid == 0) a.len_out[b] = tok + 1;
    }
    // W: rows of COLS elements (columns at or beyond L * P do not exist: zero)
    constexpr int VPR = COLS / EPV;                  // 16-byte vectors per row
    constexpr int WV = 2048 / NT;                    // vectors per thread: d * VPR <= 2048
    const T *Wg = (const T *)a.W + (int64_t)h * d * a.LP + (int64_t)l0 * P;
    uint4 wv[WV];
#pragma unroll
    for (int j = 0; j < WV; ++j) {
        const int i = tid + j * NT;
        const int c = i / VPR, v = i % VPR;
        wv[j] = make_uint4(0, 0, 0, 0);
        if (c < d && l0 * P + (v + 1) * EPV <= a.LP) wv[j] = *(const uint4 *)(Wg + (int64_t)c * a.LP + v * EPV);
    }
    // queries: 16-byte pieces of the G rows; the appended key's row
    const int qpieces = G * d / EPV, kpieces = d / EPV;
    uint4 qv = make_uint4(0, 0, 0, 0), kv = make_uint4(0, 0, 0, 0);
    if (tid < qpieces) qv = *(const uint4 *)((const T *)a.q + ((int64_t)b * a.Hq + h * G) * d + tid * EPV);
    if (app && krow >= 0 && tid >= NT - kpieces) kv = *(const uint4 *)((const T *)a.K + krow * d + (tid - (NT - kpieces)) * EPV);
    // 256 value norms spread over the sequence per table: thread -> table tid % TG, samples tid / TG + (NT / TG) m
    constexpr int SPT = 256 * TG / NT;               // samples per thread
    const int li_own = tid % TG;                     // the table of this thread's samples and table entries
    float nu1 = 0.0f, nu2 = 0.0f;
    if (a.vnorm != nullptr && app && l0 + li_own < a.L && tok >= 0 && tok < a.map.max_n) {
        const int seq = tok + 1;
        const float step = (float)seq / (float)(a.L * 256);
        float nu[SPT];
#pragma unroll
        for (int m = 0; m < SPT; ++m) {
            const int j = tid / TG + (NT / TG) * m;
            int t = (int)((float)((l0 + li_own) * 256 + j) * step);
            t = t < seq ? t : seq - 1;
            nu[m] = a.vnorm[((int64_t)b * a.Hkv + h) * a.map.max_n + t];
        }
#pragma unroll
        for (int m = 0; m < SPT; ++m) {
            nu1 += nu[m];
            nu2 = fmaf(nu[m], nu[m], nu2);
        }
    }

    // ---- into LDS
#pragma unroll
    for (int j = 0; j < WV; ++j) {
        const int i = tid + j * NT;
        if (i < d * VPR) *(uint4 *)(ws + (size_t)i * EPV) = wv[j];
    }
    if (tid < qpieces) {
        float f[EPV];
        vec_to_f32<T>(qv, f);
        const int g = tid / kpieces, c0 = (tid - g * kpieces) * EPV;
#pragma unroll
        for (int e = 0; e < EPV; ++e) qd[(size_t)(c0 + e) * G + g] = (double)f[e];
    }
    if (app && tid >= NT - kpieces) {
        float f[EPV];
        vec_to_f32<T>(kv, f);
#pragma unroll
        for (int e = 0; e < EPV; ++e) kf[(tid - (NT - kpieces)) * EPV + e] = f[e];
    }
    __syncthreads();

    // ---- dot products: columns 2 cpi, 2 cpi + 1; query heads qg QPT ..; channels of range cs
    const int cpi = tid & 63;
    auto w_pair = [&](int c, float &wa, float &wb) __attribute__((always_inline)) {
        if (sizeof(T) == 2) {
            const uint32_t w2 = ((const uint32_t *)ws)[c * (COLS / 2) + cpi];
            wa = __uint_as_float(w2 << 16);
            wb = __uint_as_float(w2 & 0xffff0000u);
        } else {
            const float2 w2 = ((const float2 *)ws)[c * (COLS / 2) + cpi];
            wa = w2.x;
            wb = w2.y;
        }
    };
    {
        const int qg = (tid >> 6) % NQG, cs = tid / (64 * NQG);
        const int cn = d / CS;
        double z[QPT][2];
#pragma unroll
        for (int qq = 0; qq < QPT; ++qq) z[qq][0] = z[qq][1] = 0.0;
#pragma unroll 8
        for (int c = cs * cn; c < (cs + 1) * cn; ++c) {
            float wa, wb;
            w_pair(c, wa, wb);
            const double da = (double)wa, db = (double)wb;
#pragma unroll
            for (int qq = 0; qq < QPT; ++qq) {
                const double qvv = qd[(size_t)c * G + qg * QPT + qq];
                z[qq][0] = fma(da, qvv, z[qq][0]);
                z[qq][1] = fma(db, qvv, z[qq][1]);
            }
        }
#pragma unroll
        for (int qq = 0; qq < QPT; ++qq)
            *(double2 *)&zb[((size_t)cs * G + qg * QPT + qq) * COLS + 2 * cpi] = make_double2(z[qq][0], z[qq][1]);
    }
    if (app) {                                       // the key, in fp32: a range of the channels per wavefront
        const int cs4 = tid >> 6, cn = d / NW;
        float k0 = 0.0f, k1 = 0.0f;
#pragma unroll 8
        for (int c = cs4 * cn; c < (cs4 + 1) * cn; ++c) {
            float wa, wb;
            w_pair(c, wa, wb);
            const float kk = kf[c];
            k0 = fmaf(wa, kk, k0);
            k1 = fmaf(wb, kk, k1);
        }
        *(float2 *)&kz[cs4 * COLS + 2 * cpi] = make_float2(k0, k1);
    }
    __syncthreads();

    // ---- per (query head, column): u = tanh(z)/sqrt(d), then the sigmoids of +-2u/tau
    for (int v = tid; v < G * COLS; v += NT) {
        const int g = v / COLS, col = v % COLS;
        double z = zb[(size_t)g * COLS + col];
#pragma unroll
        for (int cs = 1; cs < CS; ++cs) z += zb[((size_t)cs * G + g) * COLS + col];
        // tanh|z| = (1 - t)/(1 + t) with t = exp(-2|z|); sigmoid(+-x) from e = exp(-|x|)
        const double t = exp(-2.0 * fabs(z));
        const double th = (1.0 - t) * rcp64(1.0 + t);
        const double e = exp(-a.x_scale * th);       // x = 2 tanh|z| / (sqrt(d) tau) >= 0
        double big = rcp64(1.0 + e), small = e * big;
        if (a.hard) {                                // the limit tau -> 0
            big = 1.0;
            small = 0.0;
        }
        const int li = col / P, pl = col % P;
        sig[((g * P + pl) * 2 + 1) * TG + li] = z >= 0.0 ? big : small;
        sig[((g * P + pl) * 2) * TG + li] = z >= 0.0 ? small : big;
    }
    if (app && tid < COLS) {
        float ks = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) ks += kz[w * COLS + tid];
        sgn[tid] = ks >= 0.0f ? 1u : 0u;
    }
    __syncthreads();

    // ---- quarter tables (over the slab of W): products over planes 4 qr .. 4 qr + 3
    for (int e = tid; e < G * NQ * 16 * TG; e += NT) {
        const int li = e % TG, bits = (e / TG) & 15, gq = e / (TG * 16);     // gq = g * NQ + qr
        const int g = gq / NQ, qr = gq % NQ;
        const double *sp = sig + ((g * P + qr * 4) * 2) * TG + li;
        const double f0 = sp[(0 + ((bits >> 0) & 1)) * TG], f1 = sp[(2 + ((bits >> 1) & 1)) * TG];
        const double f2 = sp[(4 + ((bits >> 2) & 1)) * TG], f3 = sp[(6 + ((bits >> 3) & 1)) * TG];
        // (ids that share a byte: the byte's entry is a sum over its pf small tables, so a
        // quarter holds one 4-plane table, two 2-plane tables or four 1-plane tables)
        double v = (f0 * f1) * (f2 * f3);
        if (a.pf > 2) v = a.pf == 4 ? f0 * f1 + f2 * f3 : (f0 + f1) + (f2 + f3);
        qt[e] = v;
    }
    if (a.pf > 1) {
        // the caller's tables one by one, for the read-back
        const int Ru = 1 << a.Pu;
        for (int e = tid; e < TG * a.pf * Ru; e += NT) {
            const int x = e % Ru, j = (e / Ru) % a.pf, li = e / (Ru * a.pf);
            if (l0 + li >= a.L) continue;
            double mean = 0.0;
            for (int g = 0; g < G; ++g) {
                double pr = 1.0;
                for (int i = 0; i < a.Pu; ++i) pr *= sig[((g * P + j * a.Pu + i) * 2 + ((x >> i) & 1)) * TG + li];
                mean += pr;
            }
            a.subprobs[((((int64_t)b * a.Hkv + h) * a.L + l0 + li) * a.pf + j) * Ru + x] = (float)(mean / (double)G);
        }
    }
    // the appended key's bucket ids, one thread per table of the group (tables >= L: id 0)
    if (app && krow >= 0 && tid >= 64 && tid < 64 + TG && l0 + tid - 64 < a.Lpad) {
        const int li = tid - 64, l = l0 + li;
        uint32_t code = 0;
        if (l < a.L)
#pragma unroll
            for (int i = 0; i < P; ++i) code |= sgn[li * P + i] << i;
        ((uint8_t *)a.codes)[krow * a.Lpad + code_pos(l, tok, a.S)] = (uint8_t)code;
    }
    __syncthreads();

    // ---- the tables: p(r) over all planes, averaged over the G queries.  Thread -> table li_own,
    //      buckets tid / TG + (NT / TG) k.
    {
        constexpr int RSTEP = NT / TG, NK = R / RSTEP;
        const int l = l0 + li_own;
        const bool live = l < a.L;
        const int lw = a.Lpad < 64 ? a.Lpad : 64, copies = 64 / lw;
        const int c64 = l >> 6, lp = l & 63;
        const double inv_g = 1.0 / (double)G;
        float *Tg = a.tables + ((int64_t)b * a.Hkv + h) * a.table_words;
        const int r0 = tid / TG;
        double lo[G];
        static_assert(RSTEP % 16 == 0 || P <= 4, "the low four bits of a thread's buckets are the same for every k");
        if (P > 4) {
#pragma unroll
            for (int g = 0; g < G; ++g) lo[g] = qt[((g * NQ) * 16 + (r0 & 15)) * TG + li_own];
        }
        float dev2 = 0.0f;
        // (ids that share a byte: the byte's entry is the sum of the two quarters, else their
        // product; two copies of the loop, so that neither pays for the other)
        auto fill = [&](auto shared_tag) __attribute__((always_inline)) {
            constexpr bool SHARED = decltype(shared_tag)::value;
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int r = r0 + RSTEP * k;
                double mean = 0.0;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (P > 4) {
                        const double hi = qt[((g * NQ + 1) * 16 + (r >> 4)) * TG + li_own];
                        if (SHARED) mean += lo[g] + hi;
                        else mean = fma(lo[g], hi, mean);
                    } else mean += qt[((g * NQ) * 16 + r) * TG + li_own];
                }
                mean *= inv_g;
                if (!live) mean = 0.0;
                else {
                    const double dv = mean - (SHARED ? a.tmean : 1.0 / (double)R);   // a table's entries sum to 1: their mean is 1/R (pf / 2^Pu when ids share bytes)
                    dev2 += (float)(dv * dv);
                }
                if (l < a.Lpad)
                    // (streaming stores: the tables are read next by workgroups of every XCD, through memory)
                    for (int cp = 0; cp < copies; ++cp) __builtin_nontemporal_store((float)mean, &Tg[((int64_t)c64 * R + r) * 64 + lp + cp * lw]);
            }
        };
        if (a.pf > 1) fill(GroupTag<true>());
        else fill(GroupTag<false>());
        s_part[tid] = dev2;
        s_part[NT + tid] = nu1;
        s_part[2 * NT + tid] = nu2;
    }
    __syncthreads();
    // spread of each table's entries and its sampled value norms, from which the scoring pass
    // sizes its histogram bins
    if (tid < 3 * TG) {
        const int w = tid / TG, li = tid % TG;
        float sum = 0.0f;
#pragma unroll
        for (int j = 0; j < NT / TG; ++j) sum += s_part[w * NT + li + j * TG];
        if (l0 + li < a.Lpad)
            a.tstats[(((int64_t)b * a.Hkv + h) * a.Lpad + l0 + li) * 3 + w] = w == 0 ? (float)((double)sum / (double)R) : sum;
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
    float mu;               // mean score of a uniformly drawn key (the caller's L / 2^P)
    int batch;
    int64_t table_words;
};

// 16 bucket ids of one lane: CB = 1 -> 16 bytes, CB = 2 -> 32 bytes.
template <int CB> struct CodeVec;
template <> struct CodeVec<1> {
    uint4 v;
    // the id stream is read once: a non-temporal load keeps it from displacing the table and
    // the scores in L2 (measured 6 % faster)
    __device__ __forceinline__ void load(const void *p) {
        typedef unsigned int u4 __attribute__((ext_vector_type(4)));
        u4 t = __builtin_nontemporal_load((const u4 *)p);
        v = make_uint4(t.x, t.y, t.z, t.w);
    }
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

constexpr int kBlkTiles = 1024;                      // block ids a scoring workgroup keeps in LDS (paged caches)

// The keys of all sequences of the batch are cut into units of WKEYS = U*KPW consecutive keys
// (what one wavefront takes at a time: U 16-byte loads per lane in flight), and the units of a
// KV head, in sequence order, are dealt out in equal contiguous runs to the workgroups of that
// head: long and short sequences then cost their workgroups the same.  A run that crosses from
// one sequence into the next is worked off segment by segment, the table in LDS being replaced
// in between.  Inside a segment the wavefronts take units round-robin, and the loads of a
// wavefront's next unit are issued before its current one is processed (two register sets,
// ping-pong); with a paged cache the block-table entries are fetched one unit further ahead
// still, so that no id load waits for a table entry.
// BATCHED = false is the single-sequence case: one segment per workgroup, its units taken
// round-robin over all workgroups of the head, and none of the bookkeeping above.
template <int S, int CB, int MODE, bool ONE_ROUND, bool PAGED, bool BATCHED>
// (64 tables of one-byte ids, paged: two workgroups per CU need four wavefronts per SIMD, i.e. at most 128
// registers, which the compiler meets only when told)
__global__ __launch_bounds__(kScoreThreads, (MODE == kDirect && S == 4 && PAGED) ? 4 : 1) void score_kernel(ScoreArgs a) {
    extern __shared__ float tbl[];
    constexpr int KPW = 64 / S;                      // keys per wavefront pass
    constexpr int NW = kScoreThreads / 64;
    constexpr int U = kScoreU;                       // passes per unit
    constexpr int WKEYS = U * KPW;                   // keys per unit
    constexpr int EPL = U / S;                       // results a lane emits per unit
    static_assert(U % S == 0, "each lane of a key's group emits U/S results");
    constexpr int TPU = WKEYS / 16;                  // 16-key tiles per unit (a tile never straddles a page)
    constexpr int RPB = kBlkTiles / (NW * TPU);      // rounds of the workgroup whose block ids fit in LDS at a time
    constexpr int kTableCost = 2 * NW;                   // a table load, in units (one per wavefront): measured 2-3 us
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.y, slot = blockIdx.x, nslot = gridDim.x;
    const int max_n = a.map.max_n;
    const float ninf = -__builtin_inff();
    const bool adaptive = a.hist_mode == kHistAdaptive;

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

    // Sequence lengths: one global load each, then from LDS (the workgroup reads them twice)
    int *s_len = (int *)(tbl + a.table_words + (a.hist ? kHistBins + 4 : 0));   // [batch]
    int32_t *s_blk = s_len + (BATCHED ? a.batch : 0);   // [kBlkTiles] paged caches: block ids of 16-key tiles
    const int nbatch = BATCHED ? a.batch : 1;
    int u0 = 0, u1 = 0;
    if (BATCHED) {
        for (int b = tid; b < nbatch; b += kScoreThreads) {
            const int v = a.seq_len[b];
            s_len[b] = v < 0 ? 0 : (v > max_n ? max_n : v);
        }
        __syncthreads();
        // this workgroup's run of units: the first (total mod nslot) workgroups take one more.
        // Runs are cut in cost, not in units: entering a sequence costs a load of its table,
        // about what kTableCost units take, so a workgroup whose run crosses into the next
        // sequence is given that many units less.
        int total = 0;
        for (int b = 0; b < nbatch; ++b) total += (s_len[b] + WKEYS - 1) / WKEYS + kTableCost;
        const int per = total / nslot, extra = total - per * nslot;
        // Workgroups go to the 8 XCDs round-robin: neighbouring runs (mostly the same sequence,
        // so the same probability table) are given to workgroups of one XCD, whose L2 then
        // serves the table to all but the first of them.
        const int run_id = (nslot & 7) == 0 ? (slot & 7) * (nslot >> 3) + (slot >> 3) : slot;
        u0 = run_id * per + (run_id < extra ? run_id : extra);
        u1 = u0 + per + (run_id < extra ? 1 : 0);
    }

    auto run = [&](auto base0) {
        constexpr bool BASE0 = decltype(base0)::value;
        int cum = 0;
        bool first_segment = true;
        for (int b = 0; b < nbatch; ++b) {
            int seq;
            if (BATCHED) {
                seq = s_len[b];
            } else {
                seq = a.seq_len[0];
                seq = seq < 0 ? 0 : (seq > max_n ? max_n : seq);
            }
            const int nu = (seq + WKEYS - 1) / WKEYS;
            const int64_t bh = (int64_t)b * a.map.Hkv + h;
            float *out = a.scores + bh * max_n;
            // beyond the sequence's last unit: -inf, a share for every workgroup of the head
            for (int key = nu * WKEYS + slot * kScoreThreads + tid; key < max_n; key += nslot * kScoreThreads)
                out[key] = ninf;
            int ub, ue, ustride;
            if (BATCHED) {
                const int first = cum + kTableCost;  // cost position of the sequence's first unit
                const int lo = u0 > first ? u0 : first, hi = u1 < first + nu ? u1 : first + nu;
                ub = lo - first;                     // this workgroup's units of the sequence
                ue = hi - first;
                ustride = NW;
                cum += nu + kTableCost;
            } else {
                ub = slot * NW;                      // its wavefronts' first units; the next ones nslot * NW further on
                ue = nu;
                ustride = nslot * NW;
            }
            if (ub >= ue) continue;

            const float *vn = a.vnorm ? a.vnorm + bh * max_n : nullptr;
            const float *wsrc = vn ? vn : a.tables;  // weights, or anything loadable
            const int nmine = ue - ub > wave ? (ue - ub - wave + ustride - 1) / ustride : 0;   // units of this wavefront
            auto unit_base = [&](int r) { return (ub + wave + r * ustride) * WKEYS; };
            float bin_lo = 0.0f, bin_inv = 0.0f;     // adaptive histogram bins, set once the table is in

            // Paged caches: the block-table entries of the U keys base + u*KPW + kk, as loaded; what
            // depends on them is computed when the ids are fetched, a unit later, so that nothing
            // waits for these loads here.
            auto locate = [&](int32_t *blks, int base) {
                if (!PAGED) return;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int key = base + u * KPW + kk;
                    const int t = key < max_n ? key : max_n - 1;
                    blks[u] = a.map.block_table[(int64_t)b * a.map.max_blocks + a.map.page_slot(t)];
                }
            };
            // After the first unit the entries come from LDS: the workgroup fetches those of RPB
            // rounds of units at a time (beside the table, for the first RPB), so that the id
            // loads of the main loop wait for no other global load.
            const int nround_wg = (ue - ub + ustride - 1) / ustride;   // rounds the workgroup makes over the segment
            auto stage_blks = [&](int r0) {
                const int rounds = nround_wg - r0 < RPB ? nround_wg - r0 : RPB;
                for (int i = tid; i < rounds * NW * TPU; i += kScoreThreads) {
                    const int lu = i / TPU, tile = i - lu * TPU;
                    const int key = (ub + (r0 + lu / NW) * ustride + lu % NW) * WKEYS + tile * 16;
                    s_blk[i] = key < max_n ? a.map.block_table[(int64_t)b * a.map.max_blocks + a.map.page_slot(key)] : -1;
                }
            };
            auto staged = [&](int32_t *blks, int r, int r0) {
                if (!PAGED) return;
#pragma unroll
                for (int u = 0; u < U; ++u) blks[u] = s_blk[((r - r0) * NW + wave) * TPU + u * (KPW / 16) + (kk >> 4)];
            };
            // The id loads of a unit.  A key at or beyond the sequence, or one whose block is absent,
            // reads a row that exists and is marked dead: every unit is the same sequence of loads.
            // Lane `sub` of a key's group emits the results of passes sub, sub+S, ...; the
            // value-norm weights of those keys are fetched with the ids.
            const char *ids = (const char *)a.codes + ((PAGED ? 0 : bh * max_n * a.Lpad) + sub * 16) * CB;
            auto fetch = [&](CodeVec<CB> *cv, bool *dead, float *w, const int32_t *rows, int base, int c) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int key = base + u * KPW + kk;
                    const int t = key < max_n ? key : max_n - 1;
                    int32_t row = t;                 // row of the id tensor (fits 32 bits: socket_create checks)
                    if (PAGED) {
                        const int32_t blk = rows[u];
                        row = (uint32_t)blk < (uint32_t)a.map.num_blocks ? (blk * a.map.Hkv + h) * a.map.page + a.map.page_off(t) : -1;
                    }
                    dead[u] = key >= seq || row < 0;
                    row = row < 0 ? 0 : row;
                    cv[u].load(ids + ((int64_t)row * a.Lpad + c * 64) * CB);
                }
                if (c == 0) {
#pragma unroll
                    for (int j = 0; j < EPL; ++j) {
                        const int key = base + (j * S + sub) * KPW + kk;
                        // (batched / paged: every lane loads a word whether there are weights or
                        // not, so that a unit is the same number of loads either way and the
                        // waits on the loads stay exact)
                        if (BATCHED || PAGED) w[j] = wsrc[(vn && key < seq) ? key : 0];
                        else w[j] = (vn && key < seq) ? vn[key] : 1.0f;
                    }
                }
            };
            auto emit = [&](int base, const float *sum, const bool *dead, const float *w) {
#pragma unroll
                for (int j = 0; j < EPL; ++j) {
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
                            if (vn) v *= w[j];
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

            CodeVec<CB> setA[U], setB[U];
            bool deadA[U], deadB[U];
            int32_t blks[PAGED ? U : 1];
            float wgtA[EPL], wgtB[EPL];
            if (ONE_ROUND && nmine > 0) {            // the first unit's loads go out before the table's
                locate(blks, unit_base(0));
                fetch(setA, deadA, wgtA, blks, unit_base(0), 0);
            }
            // Adaptive histogram: if the keys' bucket ids were uniform, a score would have mean L/R
            // and variance sum_l var_l; bins are laid from four deviations below that mean upwards.
            float var_part = 0.0f, nu1_part = 0.0f, nu2_part = 0.0f;
            if (adaptive && wave == 0)
                for (int l = lane; l < a.Lpad; l += 64) {
                    const float *ts = a.tstats + (bh * a.Lpad + l) * 3;
                    var_part += ts[0];
                    nu1_part += ts[1];
                    nu2_part += ts[2];
                }
            if (!first_segment) __syncthreads();     // every wavefront is done with the previous table
            first_segment = false;
            if (PAGED && ONE_ROUND) stage_blks(0);
            {                                        // bucket-probability table -> LDS
                const float4 *src = (const float4 *)(a.tables + bh * a.table_words);
                float4 *dst = (float4 *)tbl;
                const int n4 = (int)(a.table_words >> 2);
                constexpr int B8 = 8;                // independent loads in flight per thread
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
                float mu = a.mu;
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
                const float blo = mu - 4.0f * sigma, binv = 1.0f / (4.0f * sigma);
                if (lane == 0) {
                    s_bin[0] = blo;
                    s_bin[1] = binv;
                    if (ub == 0) {                   // the select's sweep bins with the very same pair
                        a.thr[bh * kThrStride + kThrBinLo] = __float_as_uint(blo);
                        a.thr[bh * kThrStride + kThrBinInv] = __float_as_uint(binv);
                    }
                }
            }
            __syncthreads();
            if (adaptive) {
                bin_lo = s_bin[0];
                bin_inv = s_bin[1];
            }

            if (ONE_ROUND) {
                auto process = [&](const CodeVec<CB> *cv, const bool *dead, const float *w, int base) {
                    float sum[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) sum[u] = group_sum<S>(gather16<CB, MODE, BASE0, BASE0>(cv[u], tbase, woff, 0, a));
                    emit(base, sum, dead, w);
                };
                for (int r0 = 0; r0 < (PAGED ? nround_wg : 1); r0 += RPB) {
                    if (r0 > 0) {                    // paged: the next RPB rounds' block ids
                        __syncthreads();
                        stage_blks(r0);
                        __syncthreads();
                        if (r0 < nmine) {
                            staged(blks, r0, r0);
                            fetch(setA, deadA, wgtA, blks, unit_base(r0), 0);
                        }
                    }
                    const int last = (PAGED && nmine > r0 + RPB ? r0 + RPB : nmine) - 1;
                    for (int r = r0; r <= last;) {
                        if (r < last) {
                            staged(blks, r + 1, r0);
                            fetch(setB, deadB, wgtB, blks, unit_base(r + 1), 0);
                        }
                        process(setA, deadA, wgtA, unit_base(r));
                        if (++r > last) break;
                        if (r < last) {
                            staged(blks, r + 1, r0);
                            fetch(setA, deadA, wgtA, blks, unit_base(r + 1), 0);
                        }
                        process(setB, deadB, wgtB, unit_base(r));
                        ++r;
                    }
                }
            } else {
                for (int r = 0; r < nmine; ++r) {
                    const int base = unit_base(r);
                    float sum[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) sum[u] = 0.0f;
                    locate(blks, base);
                    // two chunks at a time: both halves of a 128-byte piece of the keys' rows are
                    // asked for together (fetched half by half, a look-up pass apart, the scoring of
                    // 128-byte rows measured 28 % slower; asking for the next unit's rows ahead as
                    // well, or 16 wavefronts sharing the table, gained nothing more)
                    int c = 0;
                    for (; c + 1 < a.rounds; c += 2) {
                        fetch(setA, deadA, wgtA, blks, base, c);
                        fetch(setB, deadB, wgtB, blks, base, c + 1);
#pragma unroll
                        for (int u = 0; u < U; ++u) sum[u] += gather16<CB, MODE, BASE0, false>(setA[u], tbase, woff, c, a);
#pragma unroll
                        for (int u = 0; u < U; ++u) sum[u] += gather16<CB, MODE, BASE0, false>(setB[u], tbase, woff, c + 1, a);
                    }
                    if (c < a.rounds) {
                        fetch(setA, deadA, wgtA, blks, base, c);
#pragma unroll
                        for (int u = 0; u < U; ++u) sum[u] += gather16<CB, MODE, BASE0, false>(setA[u], tbase, woff, c, a);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) sum[u] = group_sum<S>(sum[u]);
                    emit(base, sum, deadA, wgtA);
                }
            }

            if (a.hist) {
                __syncthreads();
                uint32_t *gh = a.hist + bh * kHistBins;
                for (int i = tid; i < kHistBins; i += kScoreThreads)
                    if (lhist[i]) atomicAdd(&gh[i], lhist[i]);
            }
        }
    };
    if (tbase == 0) run(BoolTag<true>());
    else run(BoolTag<false>());
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
constexpr int kSplitThreads = 1024;
constexpr int kSplitU = 2;                           // passes a wavefront takes per turn

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
    float mu = a.mu;
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

// KEEP: no wavefront has more than kKeepTurns turns, and the partial sums of its keys stay in
// LDS (behind the table and the histogram) from one group of tables to the next; otherwise they
// travel through `scores`.
constexpr int kKeepTurns = 5;

template <int S, bool PAGED, bool KEEP>
__global__ __launch_bounds__(kSplitThreads) void score_split_kernel(ScoreArgs a) {
    extern __shared__ float tbl[];
    constexpr int GT = 16 * S;                       // tables per group
    constexpr int KPW = 64 / S;                      // keys per wavefront pass
    constexpr int NW = kSplitThreads / 64;
    constexpr int U = kSplitU;
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
    float *s_keep = a.hist ? s_bin + 4 : (float *)lhist;   // [NW][kKeepTurns][EPL][64] partial sums (KEEP)
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
    constexpr bool in_regs = KEEP;

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
            if (!in_regs) st.carry[j] = out[key];
            st.w[j] = wsrc[key];
        }
    };
    auto process = [&](const Set &st, int grp, int tix) __attribute__((always_inline)) {
        constexpr bool KEPT = KEEP;
        float *kept = s_keep + ((wave * kKeepTurns + tix) * EPL) * 64 + lane;   // [j] at stride 64
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
            if (KEPT) {
                if (!first) v += kept[j * 64];
                if (!last) {
                    kept[j * 64] = v;
                    continue;
                }
            } else {
                if (!first) v += nturn == 1 ? out[key] : st.carry[j];
                if (!last) {
                    if (!dd) out[key] = v;
                    continue;
                }
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

template <int S, int CB, int MODE, bool BATCHED>
static score_fn_t pick_score_variant(bool one_round, bool paged) {
    if (one_round) return paged ? score_kernel<S, CB, MODE, true, true, BATCHED> : score_kernel<S, CB, MODE, true, false, BATCHED>;
    return paged ? score_kernel<S, CB, MODE, false, true, BATCHED> : score_kernel<S, CB, MODE, false, false, BATCHED>;
}

template <int CB, int MODE>
static score_fn_t pick_score_s(int S, bool one_round, bool paged, bool batched) {
    switch (S) {
        case 1: return batched ? pick_score_variant<1, CB, MODE, true>(one_round, paged) : pick_score_variant<1, CB, MODE, false>(one_round, paged);
        case 2: return batched ? pick_score_variant<2, CB, MODE, true>(one_round, paged) : pick_score_variant<2, CB, MODE, false>(one_round, paged);
        case 4: return batched ? pick_score_variant<4, CB, MODE, true>(one_round, paged) : pick_score_variant<4, CB, MODE, false>(one_round, paged);
        default: return nullptr;
    }
}

static score_fn_t pick_score(const Geometry &g, bool batched) {
    const bool one_round = g.rounds == 1, paged = g.page > 0;
    if (g.mode == kDirect && g.cb == 1) return pick_score_s<1, kDirect>(g.S, one_round, paged, batched);
    if (g.mode == kFactor && g.cb == 1) return pick_score_s<1, kFactor>(g.S, one_round, paged, batched);
    if (g.mode == kFactor && g.cb == 2) return pick_score_s<2, kFactor>(g.S, one_round, paged, batched);
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
    a.pf = g.pf; a.Pu = g.Pu; a.tmean = (double)g.pf / (double)(1 << g.Pu); a.subprobs = ctx->subprobs;
    a.cols_magic = (65536 + g.P - 1) / g.P;
    const size_t lds = (size_t)(2 * g.G * kPlanePad + g.G * g.d + g.P * g.d) * sizeof(double) +
                       (size_t)(g.P * g.d + g.d) * 4 + 64 + 48 +
                       (g.mode == kSplit ? (size_t)g.G * 36 * sizeof(double) : 0);
    typedef void (*project_fn_t)(ProjectArgs);
    project_fn_t fn = nullptr;
    const bool f32 = g.kv_dtype == SOCKET_F32;
    a.batch = batch; a.nb = 1;
    const int elem = f32 ? 4 : 2;
    // batches, the common case: a workgroup per (sequence, KV head, group of 128 columns of W)
    const bool by_group = q && g.mode == kDirect && g.cb == 1 && (g.P == 4 || g.P == 8) && g.R == (1 << g.P) &&
                          (size_t)g.d * kGroupCols * elem <= 32 * 1024 && (a.LP * elem) % 16 == 0 &&
                          g.G * g.d / (16 / elem) <= kGroupThreads - g.d / (16 / elem);
    if (batch > 1 && (g.pf == 1 || by_group)) {   // (ids that share bytes: that kernel or the one-sequence kernel)
        // several sequences per workgroup: the W slab of a table is staged once for all of them
        if (by_group) {
            const size_t glds = project_group_lds(g.G, g.d, g.P, elem);
            const bool p8 = g.P == 8;
            switch (g.G) {
                case 1: fn = f32 ? (p8 ? project_group_kernel<float, 1, 8> : project_group_kernel<float, 1, 4>)
                                 : (p8 ? project_group_kernel<uint16_t, 1, 8> : project_group_kernel<uint16_t, 1, 4>); break;
                case 2: fn = f32 ? (p8 ? project_group_kernel<float, 2, 8> : project_group_kernel<float, 2, 4>)
                                 : (p8 ? project_group_kernel<uint16_t, 2, 8> : project_group_kernel<uint16_t, 2, 4>); break;
                case 4: fn = f32 ? (p8 ? project_group_kernel<float, 4, 8> : project_group_kernel<float, 4, 4>)
                                 : (p8 ? project_group_kernel<uint16_t, 4, 8> : project_group_kernel<uint16_t, 4, 4>); break;
                case 8: fn = f32 ? (p8 ? project_group_kernel<float, 8, 8> : project_group_kernel<float, 8, 4>)
                                 : (p8 ? project_group_kernel<uint16_t, 8, 8> : project_group_kernel<uint16_t, 8, 4>); break;
                default: return SOCKET_EUNSUPPORTED;
            }
            if (set_lds_limit((const void *)fn, glds) != SOCKET_OK) return SOCKET_EHIP;
            const int TG = kGroupCols / g.P;
            hipLaunchKernelGGL(fn, dim3((g.Lpad + TG - 1) / TG, g.Hkv, batch), dim3(kGroupThreads), glds, st, a);
            return record_hip(ctx, hipGetLastError());
        }
        int nb = batch < kProjMaxNb ? batch : kProjMaxNb;
        while (nb > 1 && project_batch_lds(nb, g.G, g.d, g.P, elem) > 64 * 1024) --nb;
        const int groups = (batch + nb - 1) / nb;
        a.nb = (batch + groups - 1) / groups;
        const size_t blds = project_batch_lds(a.nb, g.G, g.d, g.P, elem);
        switch (g.G) {
            case 1: fn = f32 ? project_batch_kernel<float, 1> : project_batch_kernel<uint16_t, 1>; break;
            case 2: fn = f32 ? project_batch_kernel<float, 2> : project_batch_kernel<uint16_t, 2>; break;
            case 4: fn = f32 ? project_batch_kernel<float, 4> : project_batch_kernel<uint16_t, 4>; break;
            case 8: fn = f32 ? project_batch_kernel<float, 8> : project_batch_kernel<uint16_t, 8>; break;
            default: return SOCKET_EUNSUPPORTED;
        }
        hipLaunchKernelGGL(fn, dim3(g.Lpad, g.Hkv, groups), dim3(kProjThreads), blds, st, a);
        return record_hip(ctx, hipGetLastError());
    }
    dim3 grid(g.Lpad, g.Hkv, batch);
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

static score_fn_t pick_split(int S, bool paged, bool keep) {
    if (S == 1) return paged ? (keep ? score_split_kernel<1, true, true> : score_split_kernel<1, true, false>)
                             : (keep ? score_split_kernel<1, false, true> : score_split_kernel<1, false, false>);
    return paged ? (keep ? score_split_kernel<2, true, true> : score_split_kernel<2, true, false>)
                 : (keep ? score_split_kernel<2, false, true> : score_split_kernel<2, false, false>);
}

// once per context: the packed-id scoring kernel forms its table addresses from LDS address 0,
// so it must own no static LDS
int score_prepare(const Geometry &g) {
    if (g.mode != kSplit) return SOCKET_OK;
    const bool paged = g.page > 0;
    hipFuncAttributes attr;
    for (int keep = 0; keep < 2; ++keep) {
        score_fn_t fn = pick_split(g.S, paged, keep != 0);
        if (hipFuncGetAttributes(&attr, (const void *)fn) != hipSuccess) return SOCKET_EHIP;
        if (attr.sharedSizeBytes != 0) return SOCKET_EUNSUPPORTED;
    }
    return SOCKET_OK;
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
    a.hist_mode = mode; a.tstats = ctx->tstats; a.L = g.L; a.mu = g.mu;
    a.n_sink = ctx->n_sink; a.n_window = ctx->n_window;
    a.thr = ctx->counters + (int64_t)g.max_batch * g.Hkv * kCounterStride;
    a.codes = codes; a.tables = ctx->tables; a.vnorm = vnorm; a.seq_len = seq_len; a.scores = scores;
    a.map = row_map(g, block_table);
    a.Lpad = g.Lpad; a.rounds = g.rounds; a.R = g.R; a.G = g.G; a.Plo = g.Plo; a.Rlo = g.Rlo;
    a.table_rows = g.table_rows; a.table_words = g.table_words;
    if (g.mode == kSplit) {
        // one workgroup per CU (a group table fills most of its LDS)
        const int keys_per_turn = (kSplitThreads / 64) * kSplitU * (64 / g.S);
        int per_bh = 256 / (batch * g.Hkv);
        const int turns = (g.max_n + keys_per_turn - 1) / keys_per_turn;
        if (per_bh > turns) per_bh = turns;
        if (per_bh < 1) per_bh = 1;
        a.hist = want_hist ? ctx->hist : nullptr;
        size_t lds = (size_t)g.R * g.GT * 4 + (a.hist ? kHistBins * 4 + 16 : 0);
        const bool paged = g.page > 0;
        // partial sums in LDS when no wavefront has more than kKeepTurns turns and they fit
        const int turns_per_wave = (turns + per_bh - 1) / per_bh;
        const size_t keep_bytes = (size_t)(kSplitThreads / 64) * kKeepTurns * (kSplitU / g.S) * 64 * 4;
        const bool keep = g.rounds > 1 && turns_per_wave <= kKeepTurns && lds + keep_bytes <= 160 * 1024;
        if (keep) lds += keep_bytes;
        score_fn_t fn = pick_split(g.S, paged, keep);
        if (set_lds_limit((const void *)fn, lds) != SOCKET_OK) return SOCKET_EHIP;
        // (the kernel forms its table addresses from LDS address 0: score_prepare has checked that it owns no static LDS)
        hipLaunchKernelGGL(fn, dim3(per_bh, g.Hkv, batch), dim3(kSplitThreads), lds, st, a);
        return record_hip(ctx, hipGetLastError());
    }
    // Two resident workgroups per CU over the whole launch (fewer when there is less than one
    // unit per wavefront): each KV head's units are dealt out evenly to its workgroups.
    const int wg_keys = (kScoreThreads / 64) * kScoreU * (64 / g.S);
    int64_t nslot = ((int64_t)batch * g.max_n + wg_keys - 1) / wg_keys;
    const int per_head = (256 * 1024 / kScoreThreads) / g.Hkv;
    if (nslot > per_head) nslot = per_head;
    if (nslot < 1) nslot = 1;
    dim3 grid((unsigned)nslot, g.Hkv);
    a.batch = batch;
    a.hist = want_hist ? ctx->hist : nullptr;
    size_t lds = (size_t)g.table_words * 4 + (a.hist ? kHistBins * 4 + 16 : 0) + (batch > 1 ? (size_t)batch * 4 : 0) +
                 (g.page > 0 ? (size_t)kBlkTiles * 4 : 0);   // table, histogram + bins, lengths, block ids
    score_fn_t fn = pick_score(g, batch > 1);
    if (!fn) return SOCKET_EUNSUPPORTED;
    // more than 64 KB of dynamic LDS has to be allowed per kernel before the launch
    if (set_lds_limit((const void *)fn, lds) != SOCKET_OK) return SOCKET_EHIP;
    hipLaunchKernelGGL(fn, grid, dim3(kScoreThreads), lds, st, a);
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

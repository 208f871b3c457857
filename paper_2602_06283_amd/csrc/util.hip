// Small service kernels: read-back of the bucket probabilities a context holds (Alg. 2, for
// inspection and tests), a clear of the context's select scratch, and a plain streaming read
// that measures what this GPU's memory delivers to a kernel that does nothing else.
#include "socket_internal.h"

namespace sk {

struct ProbsArgs {
    const float *tables;
    float *out;             // [batch][Hkv][L][R]
    int L, R, G, Lpad, rounds, GT, mode, Plo, Rlo, table_rows;
    int64_t table_words;
    int64_t total;          // batch * Hkv * L * R
};

// one thread per (sequence, KV head, table, bucket): the group-mean probability the scoring
// pass looks up for that bucket, taken out of whichever layout the context keeps
__global__ __launch_bounds__(256) void bucket_probs_kernel(ProbsArgs a) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.total) return;
    const int r = (int)(i % a.R);
    const int l = (int)((i / a.R) % a.L);
    const int64_t bh = i / ((int64_t)a.R * a.L);
    const float *T = a.tables + bh * a.table_words;
    float p;
    if (a.mode == kDirect) {
        p = T[((int64_t)(l >> 6) * a.R + r) * 64 + (l & 63)];
    } else if (a.mode == kSplit) {
        p = T[(((int64_t)(l / a.GT) * (a.R >> 2) + (r >> 2)) * a.GT + l % a.GT) * 4 + (r & 3)];
    } else {
        const int lo = r & (a.Rlo - 1), hi = r >> a.Plo;
        p = 0.0f;
        for (int g = 0; g < a.G; ++g) {
            const float *F = T + ((int64_t)g * a.rounds + (l >> 6)) * a.table_rows * 64 + (l & 63);
            p += F[(int64_t)lo * 64] * F[(int64_t)(a.Rlo + hi) * 64];   // the 1/G rides on the low factor
        }
    }
    a.out[i] = p;
}

int launch_bucket_probs(socket_ctx *ctx, int batch, float *probs, hipStream_t st) {
    const Geometry &g = ctx->g;
    if (g.pf > 1)   // ids that share bytes: the projection pass keeps the caller's tables beside the summed ones
        return record_hip(ctx, hipMemcpyAsync(probs, ctx->subprobs, (size_t)batch * g.Hkv * g.Lu * (1 << g.Pu) * 4,
                                              hipMemcpyDeviceToDevice, st));
    ProbsArgs a;
    a.tables = ctx->tables; a.out = probs;
    a.L = g.L; a.R = g.R; a.G = g.G; a.Lpad = g.Lpad; a.rounds = g.rounds; a.GT = g.GT; a.mode = g.mode;
    a.Plo = g.Plo; a.Rlo = g.Rlo; a.table_rows = g.table_rows; a.table_words = g.table_words;
    a.total = (int64_t)batch * g.Hkv * g.L * g.R;
    const int64_t blocks = (a.total + 255) / 256;
    if (blocks > 0x7fffffff) return SOCKET_EUNSUPPORTED;
    hipLaunchKernelGGL(bucket_probs_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a);
    return record_hip(ctx, hipGetLastError());
}

// zero `n` words (histograms, counters): a fill kernel, so that it can sit in a captured graph
__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t *p, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0u;
}

int launch_reset(socket_ctx *ctx, hipStream_t st) {
    const Geometry &g = ctx->g;
    const int64_t BH = (int64_t)g.max_batch * g.Hkv;
    const int64_t n_hist = 2 * BH * kHistBins, n_cnt = BH * (kCounterStride + kThrStride);
    hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((n_hist + 255) / 256 < 1024 ? (n_hist + 255) / 256 : 1024)), dim3(256), 0, st,
                       ctx->hist, n_hist);
    hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((n_cnt + 255) / 256 < 1024 ? (n_cnt + 255) / 256 : 1024)), dim3(256), 0, st,
                       ctx->counters, n_cnt);
    ctx->pending_hist = kHistNone;
    return record_hip(ctx, hipGetLastError());
}

// Read `bytes` (a multiple of 16) once, 16 bytes per lane and load, four loads in flight per
// lane, non-temporal like the scoring pass reads its ids; the xor of everything goes to *sink so
// that the loads cannot be dropped.
constexpr int kProbeThreads = 512;
__global__ __launch_bounds__(kProbeThreads) void stream_read_kernel(const uint4 *src, int64_t n16, uint32_t *sink) {
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const int64_t stride = (int64_t)gridDim.x * kProbeThreads;
    uint32_t acc = 0;
    int64_t i = (int64_t)blockIdx.x * kProbeThreads + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load((const u4 *)src + i + j * stride);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    for (; i < n16; i += stride) {
        const u4 v = __builtin_nontemporal_load((const u4 *)src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;             // (practically never: keeps the loads alive)
}

int launch_stream_read(const void *buf, int64_t bytes, uint32_t *sink, hipStream_t st) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(512), dim3(kProbeThreads), 0, st, (const uint4 *)buf, bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? SOCKET_OK : SOCKET_EHIP;
}

}  // namespace sk

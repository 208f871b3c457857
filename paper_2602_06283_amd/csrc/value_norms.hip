// Alg. 1 caches, next to the bucket ids, the norm of every value vector; Alg. 3 ranks tokens
// by (soft collision score) x ||v_j||_2.  This kernel fills that cache: one pass over the
// value rows, d/8 lanes per row with a 16- or 32-byte load each, fp32 sum of squares, DPP
// row sum.  Bound by the read of V.
#include "socket_internal.h"

namespace sk {

struct NormArgs {
    const void *V;
    float *vnorm;           // [B, Hkv, max_n], logical token order
    const int32_t *row_begin;
    const int32_t *row_count;
    RowMap map;
};

constexpr int kNormThreads = 256;
constexpr int kNormPasses = 4;       // rows per lane group and workgroup: the loads of all passes go out together

template <typename T, int D>
__global__ __launch_bounds__(kNormThreads) void value_norms_kernel(NormArgs a) {
    constexpr int LPR = D / 8;                       // lanes per row
    constexpr int RPP = kNormThreads / LPR;          // rows per pass
    const int tid = threadIdx.x;
    const int sub = tid % LPR, rl = tid / LPR;
    const int h = blockIdx.y, b = blockIdx.z;
    const int count = a.row_count[b], begin = a.row_begin[b];
    const int r0 = blockIdx.x * (RPP * kNormPasses);
    if (r0 >= count) return;
    Row8<T> v[kNormPasses];
    int tok[kNormPasses];
#pragma unroll
    for (int p = 0; p < kNormPasses; ++p) {
        const int r = r0 + p * RPP + rl;
        const int t = begin + r;
        int64_t row = -1;
        if (r < count && t >= 0 && t < a.map.max_n) row = a.map.row(b, h, t);
        tok[p] = row >= 0 ? t : -1;
        if (row >= 0) v[p].load((const T *)a.V + row * D + sub * 8);
        else v[p].zero();
    }
#pragma unroll
    for (int p = 0; p < kNormPasses; ++p) {
        float f[8];
        v[p].get(f);
        float s = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(f[e], f[e], s);
        s = row_sum<LPR>(s);
        if (sub == 0 && tok[p] >= 0) a.vnorm[((int64_t)b * a.map.Hkv + h) * a.map.max_n + tok[p]] = sqrtf(s);
    }
}

int launch_value_norms(socket_ctx *ctx, const void *V, const int32_t *block_table,
                       const int32_t *row_begin, const int32_t *row_count, int batch, int max_rows,
                       float *vnorm, hipStream_t st) {
    const Geometry &g = ctx->g;
    NormArgs a;
    a.V = V; a.vnorm = vnorm; a.row_begin = row_begin; a.row_count = row_count;
    a.map = row_map(g, block_table);
    const int rows_per_wg = (kNormThreads / (g.d / 8)) * kNormPasses;
    dim3 grid((max_rows + rows_per_wg - 1) / rows_per_wg, g.Hkv, batch);
    const bool f32 = g.kv_dtype == SOCKET_F32;
    switch (g.d) {
        case 64:
            if (f32) hipLaunchKernelGGL((value_norms_kernel<float, 64>), grid, dim3(kNormThreads), 0, st, a);
            else hipLaunchKernelGGL((value_norms_kernel<uint16_t, 64>), grid, dim3(kNormThreads), 0, st, a);
            break;
        case 128:
            if (f32) hipLaunchKernelGGL((value_norms_kernel<float, 128>), grid, dim3(kNormThreads), 0, st, a);
            else hipLaunchKernelGGL((value_norms_kernel<uint16_t, 128>), grid, dim3(kNormThreads), 0, st, a);
            break;
        case 256:
            if (f32) hipLaunchKernelGGL((value_norms_kernel<float, 256>), grid, dim3(kNormThreads), 0, st, a);
            else hipLaunchKernelGGL((value_norms_kernel<uint16_t, 256>), grid, dim3(kNormThreads), 0, st, a);
            break;
        default: return SOCKET_EUNSUPPORTED;
    }
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

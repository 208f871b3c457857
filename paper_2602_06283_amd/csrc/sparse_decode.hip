// Eq. 2: exact softmax attention restricted to the selected tokens (Eq. 1 when every token is
// selected).  Split-K flash-decode: the selected rows of one (sequence, KV head) are divided
// among n_split workgroups; each gathers its K rows once for all G query heads of the group,
// keeps a running (max, sum, weighted value sum) per query head in fp32 over the gathered
// K and V rows, and writes one partial result per split; a second small kernel merges them.
// Logits use no 1/sqrt(d) unless the caller passes one as `scale`; with unit-variance data
// they reach +-100, so everything is max-subtracted.
//
// Given the ordered index row, a split owns a fixed range of its slots.  The fused decode step
// can also start from what the select's sweep leaves, without waiting for the ordered row: the
// positions selected outright lie in one region per workgroup of the sweep (kSlice positions of
// the sequence each, in position order), and a split owns a region (or an interleaved share of
// one, or a few regions), plus those candidates of the threshold bin that make the cut and whose
// position falls in its regions (every split ranks the few candidates itself).  Which tokens a
// split sums, and in which order, then depends on the scores alone: the output is the same bit
// for bit on every run.  The splits also write the ordered index row for the caller, each its
// own entries: the regions one after the other already are the positions selected outright in
// ascending order, so an entry's slot is the number of entries before it plus the number of kept
// candidates below it, and a kept candidate's slot the same two counts for its position.
#include <mutex>

#include "topk_device.h"

namespace sk {

template <bool V> struct IntTag { static constexpr bool value = V; };

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;

// where a workgroup's rows come from
enum RowSource {
    kRowsIdx = 0,      // its slice of the ordered row idx[b, h, :n_selected]               (Eq. 2)
    kRowsSweep = 1,    // what the select's sweep left: staged positions + ranked candidates (Eq. 2)
    kRowsDense = 2,    // every token below seq_len, contiguous ranges                      (Eq. 1)
};
constexpr int kCandPer = 2;                       // candidates per thread of a decode workgroup
constexpr int kSweepCand = kCandPer * kDecodeThreads;   // candidates a decode workgroup ranks itself; a
                                                  // head with more is attended from the ordered
                                                  // row by its ordering workgroup

struct DecodeArgs {
    const void *q;
    const void *K;
    const void *V;
    const int32_t *idx;
    const int32_t *n_selected;
    float *partials;
    void *out;
    RowMap map;
    float scale;
    int Hq, max_k, n_split, out_dtype;
    const int32_t *seq_len;   // dense variant, and kRowsSweep: tokens of each sequence
    // kRowsSweep: the lists and the threshold record of the select's sweep
    const int32_t *sel_regions;
    const uint32_t *sel_cnt;
    int n_regions, ssr, rpg;
    int emit_idx;             // the splits write the ordered index row (a.idx) themselves
    const uint32_t *cand_key;
    const int32_t *cand_idx;
    const uint32_t *thr;
};

// two adjacent elements of an LDS row as floats
__device__ __forceinline__ float2 pair_f32(const uint16_t *p) {
    const uint32_t w = *(const uint32_t *)p;
    return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}
__device__ __forceinline__ float2 pair_f32(const float *p) { return *(const float2 *)p; }

// dynamic LDS of decode_body<kRowsSweep> while it ranks candidates: their keys and a quad of padding
constexpr size_t kSweepRankLds = (size_t)(kSweepCand + 4) * 8;

// dynamic LDS of decode_body<.., G, .., NT>: the value tile, over which the thread groups' shares
// of the value sum are added at the end
template <typename T, int D, int G, int NT = kDecodeThreads> constexpr size_t decode_lds_bytes() {
    constexpr int ROWB = D * (int)sizeof(T);
    constexpr int VROWS = kDecodeChunk * ROWB <= 32768 ? kDecodeChunk : 32768 / ROWB;
    constexpr size_t tile = (size_t)VROWS * ROWB, sums = (size_t)(NT / (D / 2)) * G * D * 4;
    return tile > sums ? tile : sums;
}

// One split of one (sequence, KV head), run by a whole workgroup of NT threads.
// SRC says where the rows come from (RowSource).  `dyn` is decode_lds_bytes<T, D, G, NT>() of LDS
// (kRowsSweep: at least kSweepRankLds).  Returns
// true when nothing was done: kRowsSweep with more candidates than a workgroup ranks.
template <typename T, int D, int G, int SRC, int NT = kDecodeThreads>
__device__ __forceinline__ bool decode_body(const DecodeArgs &a, int split, int h, int b, char *dyn) {
    constexpr bool DENSE = SRC == kRowsDense;
    constexpr int LPR = D / 8;                       // lanes per row
    constexpr int RPW = 64 / LPR;                    // rows per wavefront pass
    constexpr int NWAVE = NT / 64;
    constexpr int RPP = NWAVE * RPW;                 // rows per workgroup pass
    constexpr int CH = kDecodeChunk;
    constexpr int NPASS = CH / RPP;
    static_assert(CH % RPP == 0, "chunk must be whole passes");
    // The value rows of a chunk go through LDS (at most 32 KB at a time), where every thread
    // owns two adjacent output channels of every query head for a share of the rows: no
    // cross-lane sums in the value product.
    constexpr int ROWB = D * (int)sizeof(T);
    constexpr int VROWS = CH * ROWB <= 32768 ? CH : 32768 / ROWB;
    constexpr int VROUNDS = CH / VROWS, PPR = VROWS / RPP;      // passes per round
    static_assert(VROWS % RPP == 0 && VROWS % 4 == 0, "a round is whole passes");
    constexpr int CPAIRS = D / 2;                    // channel pairs
    constexpr int NG = NT / CPAIRS;      // thread groups, each covering all channels: a group walks its own rows of the tile
    constexpr int RPR = VROWS / NG;                  // rows of the tile per group
    static_assert(VROWS % NG == 0 && RPR >= 1, "every group has whole rows of the tile");
    constexpr int RB = RPR < 16 ? RPR : 16;          // rows whose LDS reads are issued together
    static_assert(RPR % RB == 0, "whole batches of rows");

    __shared__ __align__(16) float s_p[G][CH];       // logits, then softmax numerators
    __shared__ int64_t s_row[1][CH];                 // K/V row of each chunk entry (-1 = none)
    __shared__ float s_m[G], s_l[G], s_corr[G];
    // bf16 caches: the logits of a chunk are one 16-row MFMA tile per wavefront (rows = keys,
    // columns = query heads, padded to 16), K fetched straight into A-operand registers: lane
    // (row = lane % 16, group kg = lane / 16) holds channels 32 s + 8 kg .. + 7 of its row for
    // k-step s.  fp32 caches keep the FMA + DPP row sums.
    constexpr bool MF = sizeof(T) == 2;
    constexpr int KST = D / 32;                      // MFMA k-steps
    constexpr int NLW = CH / 16;                     // wavefronts that hold a tile of the chunk
    static_assert(NLW <= NWAVE, "a chunk's tiles fit the workgroup's wavefronts");
    __shared__ __align__(16) float s_q[MF ? 1 : G][MF ? 8 : D];          // the queries as floats
    __shared__ __align__(16) uint16_t s_qb[MF ? G : 1][MF ? D : 8];      // the queries as stored (bf16)
    __shared__ int32_t s_cpos[SRC == kRowsSweep ? kSweepCand : 1];   // candidates that make the cut, best first
    // kRowsSweep, for the index row: every kept candidate's position (any order, padded with
    // INT_MAX to whole quads), the head of the first region, the entry counts of the regions before it
    constexpr int kHeadEntries = SRC == kRowsSweep ? NT : 1;
    __shared__ __align__(16) int32_t s_kept[SRC == kRowsSweep ? kSweepCand : 4];
    __shared__ int32_t s_head[kHeadEntries];
    __shared__ float s_pre[NWAVE];
    __shared__ int s_nkept;
    __shared__ int64_t s_own[kHeadEntries];          // kRowsSweep: the K/V rows of the first NT entries
    T (*s_v)[D] = (T (*)[D])dyn;                     // [VROWS][D]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bh = b * a.map.Hkv + h;
    const int sub = lane % LPR, rl = lane / LPR;     // this lane's 8-element slice and row slot
    const int cp = tid % CPAIRS, grp = tid / CPAIRS;  // this thread's channel pair and row group of the value tile
    const float ninf = -__builtin_inff();

    // Splits own fixed ranges of the max_k slots, so no load has to wait for the selected
    // count; slots at or beyond the count are ignored.  (Dense: whole chunks of the sequence.)
    const int per = (a.max_k + a.n_split - 1) / a.n_split;
    const int r_begin = split * per;
    int r_end = min(a.max_k, r_begin + per);

    // ---- every load that needs nothing else first, issued before anything waits: the queries,
    //      the first chunk's list entries, the counts and (kRowsSweep) one candidate per thread
    //      (the reads stay inside the buffers)
    Row8<T> qr[G];                                   // (the first LPR threads: 8 channels of every query head each)
    if (tid < LPR) {
#pragma unroll
        for (int g = 0; g < G; ++g) qr[g].load((const T *)a.q + ((int64_t)b * a.Hq + h * G + g) * D + tid * 8);
    }
    const int32_t *list = nullptr;
    int32_t first = -1;                              // the list entry of slot r_begin + tid (kRowsSweep: entry tid of the split's share of its first region)
    uint32_t pk[kCandPer];
    int32_t pp[kCandPer];
    int count = 0, need = 0, n_cand = 0;             // list entries that count; kRowsSweep: see below
    // kRowsSweep: this split's regions [reg0, reg1) of the sweep, and of a shared region the
    // entries sub_i, sub_i + sub_n, ...
    int reg0 = 0, reg1 = 0, sub_i = 0, sub_n = 1;
    uint32_t cnt_before = 0;                         // entries of region `tid`, if that lies before this split's
    int32_t head = 0;                                // entry `tid` of this split's region
    if (SRC == kRowsIdx) {
        list = a.idx + (int64_t)bh * a.max_k;
        if (tid < CH && r_begin + tid < r_end) first = list[r_begin + tid];
        count = a.n_selected[bh];
    }
    if (SRC == kRowsSweep) {
        if (a.rpg > 1) {
            reg0 = split * a.rpg;
            reg1 = min(a.n_regions, reg0 + a.rpg);
        } else {
            reg0 = split / a.ssr;
            reg1 = reg0 + 1;
            sub_i = split - reg0 * a.ssr;
            sub_n = a.ssr;
        }
        // regions past the end of the sequence hold nothing: an empty partial result, at once
        // (in a batch of mixed lengths that is a good part of the workgroups)
        if ((int64_t)reg0 * kSlice >= a.seq_len[b]) {
            float *part = a.partials + ((int64_t)(b * a.Hq + h * G) * a.n_split) * (D + 2);
            if (tid < G) {
                part[((int64_t)tid * a.n_split + split) * (D + 2) + 0] = ninf;
                part[((int64_t)tid * a.n_split + split) * (D + 2) + 1] = 0.0f;
            }
            for (int i = tid; i < G * D; i += NT) part[((int64_t)(i / D) * a.n_split + split) * (D + 2) + 2 + i % D] = 0.0f;
            return false;
        }
        list = a.sel_regions + (int64_t)bh * a.n_regions * kSlice;
        first = list[(int64_t)reg0 * kSlice + sub_i + tid * sub_n];   // (inside the region's kSlice words: sub_n <= 16)
        count = (int)a.sel_cnt[(int64_t)bh * a.n_regions + reg0];
        if (a.emit_idx) {
            cnt_before = tid < reg0 ? a.sel_cnt[(int64_t)bh * a.n_regions + tid] : 0u;
            if (sub_i == 0) head = list[(int64_t)reg0 * kSlice + tid];   // (inside the region's kSlice words)
        }
#pragma unroll
        for (int j = 0; j < kCandPer; ++j) {
            const int i = tid + j * NT;
            pk[j] = i < a.map.max_n ? a.cand_key[(int64_t)bh * a.map.max_n + i] : 0u;
            pp[j] = i < a.map.max_n ? a.cand_idx[(int64_t)bh * a.map.max_n + i] : 0;
        }
        // the selection: every position of the regions, and the `need` best candidates of the threshold bin
        const uint32_t *thr = a.thr + (int64_t)bh * kThrStride;
        const int k_eff = min((int)thr[0], a.max_k);
        const int above = k_eff ? min((int)thr[5], k_eff) : 0;
        n_cand = k_eff ? (int)thr[6] : 0;
        need = k_eff - above;
        if (k_eff == 0) count = 0;
    }
    // too many candidates to rank here: the caller attends the head from the ordered row instead
    if (SRC == kRowsSweep && n_cand > kSweepCand) return true;
    // the queries wait in LDS (in registers they would cost a workgroup per compute unit)
    if (tid < LPR) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (MF) {
                qr[g].store(&s_qb[g][tid * 8]);
            } else {
                float qf[8];
                qr[g].get(qf);
                *(float4 *)&s_q[g][tid * 8] = make_float4(qf[0], qf[1], qf[2], qf[3]);
                *(float4 *)&s_q[g][tid * 8 + 4] = make_float4(qf[4], qf[5], qf[6], qf[7]);
            }
        }
    }
    // kRowsSweep: the K/V row of this thread's entry (paged: a block-table lookup, in flight while
    // the candidates are ranked)
    const int n_first = count > sub_i ? (count - sub_i + sub_n - 1) / sub_n : 0;   // entries of this split in its first region
    int64_t own_row = -1;
    if (SRC == kRowsSweep && tid < n_first && first >= 0 && first < a.map.max_n) own_row = a.map.row(b, h, first);

    float acc[G][2];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g][0] = acc[g][1] = 0.0f;
    if (tid < G) {
        s_m[tid] = ninf;
        s_l[tid] = 0.0f;
    }

    // ---- kRowsSweep: of the `need` best candidates on (score, then smaller position) those whose
    //      position lies in this split's regions (and, of a shared region, the share of the
    //      split that the position's parity-like residue picks), best first
    __shared__ int s_nmine;
    const bool emit = SRC == kRowsSweep && a.emit_idx;
    if (SRC == kRowsSweep) {
        unsigned long long *ck = (unsigned long long *)dyn;       // the value tile is not in use yet
        if (tid == 0) {
            s_nmine = 0;
            s_nkept = 0;
        }
        if (emit) {
            for (int i = tid; i < kSweepCand; i += NT) s_kept[i] = 0x7fffffff;
            s_head[tid] = head;
            const float wsum = row_sum<64>((float)cnt_before);   // (exact: fewer than 2^24 entries)
            if (lane == 0) s_pre[wave] = wsum;
        }
        if (need > 0) {
#pragma unroll
            for (int j = 0; j < kCandPer; ++j) {
                const int i = tid + j * NT;
                if (i < n_cand) ck[i] = ((unsigned long long)pk[j] << 32) | (0x7fffffffu - (uint32_t)pp[j]);
            }
            if (tid < 4) ck[n_cand + tid] = 0;                    // (whole quads for the ranking loop; beats nobody)
        }
        __syncthreads();
        if (need > 0) {
#pragma unroll
            for (int j = 0; j < kCandPer; ++j) {
                const int i = tid + j * NT;
                const int reg = pp[j] / kSlice;
                // a shared region's candidates all go to its first split, which holds the region's head
                const bool here = i < n_cand && reg >= reg0 && reg < reg1 && sub_i == 0;
                if (i < n_cand && (here || emit)) {
                    // rank among all candidates, and among those of this split's regions: whoever
                    // beats a kept candidate is kept as well, so the second count is the
                    // candidate's place in this split's list
                    const unsigned long long me = ck[i];
                    const uint32_t plo = 0x7fffffffu - (uint32_t)reg1 * kSlice, phi = 0x7fffffffu - (uint32_t)reg0 * kSlice;
                    auto inside = [&](unsigned long long c) { return (uint32_t)c > plo && (uint32_t)c <= phi; };   // position in [reg0, reg1) * kSlice
                    int rank = 0, place = 0;
                    for (int o = 0; o < n_cand; o += 4) {
                        const ulonglong2 c0 = *(const ulonglong2 *)&ck[o], c1 = *(const ulonglong2 *)&ck[o + 2];
                        const bool b0 = c0.x > me, b1 = c0.y > me, b2 = c1.x > me, b3 = c1.y > me;
                        rank += b0 + b1 + b2 + b3;
                        place += (b0 && inside(c0.x)) + (b1 && inside(c0.y)) + (b2 && inside(c1.x)) + (b3 && inside(c1.y));
                    }
                    if (rank < need) {
                        if (here) {
                            s_cpos[place] = pp[j];
                            atomicAdd(&s_nmine, 1);
                        }
                        if (emit) s_kept[atomicAdd(&s_nkept, 1)] = pp[j];
                    }
                }
            }
        }
        s_own[tid] = own_row;
    }
    __syncthreads();
    const int n_mine = SRC == kRowsSweep ? s_nmine : 0;
    float qf[(SRC == kRowsSweep || MF) ? 1 : G][8];
    if (SRC != kRowsSweep && !MF) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4 q0 = *(const float4 *)&s_q[g][sub * 8], q1 = *(const float4 *)&s_q[g][sub * 8 + 4];
            qf[g][0] = q0.x; qf[g][1] = q0.y; qf[g][2] = q0.z; qf[g][3] = q0.w;
            qf[g][4] = q1.x; qf[g][5] = q1.y; qf[g][6] = q1.z; qf[g][7] = q1.w;
        }
    }
    // ---- the index row: entries before this split's region, kept candidates below a position
    int32_t *idx_row = nullptr;
    int entries_before = 0, n_kept = 0;
    if (emit) {
        idx_row = (int32_t *)a.idx + (int64_t)bh * a.max_k;
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < NWAVE; ++w) sum += s_pre[w];
        entries_before = (int)sum;
        n_kept = s_nkept;
    }
    auto kept_below = [&](int32_t p) __attribute__((always_inline)) {
        int c = 0;
        for (int q = 0; q < n_kept; q += 4) {
            const int4 v = *(const int4 *)&s_kept[q];
            c += (v.x < p) + (v.y < p) + (v.z < p) + (v.w < p);
        }
        return c;
    };
    int32_t pend_t = -1;                             // the list entry this thread has yet to write to the row
    int pend_slot = 0;
    if (SRC == kRowsSweep && emit && tid < n_first) {
        pend_t = first;
        pend_slot = entries_before + sub_i + tid * sub_n;
    }

    // one chunk of rows (s_row filled, or kr/vr/rows loaded for the dense source): logits,
    // running softmax statistics, weighted value rows.  Only the first n_live slots of the chunk
    // hold rows: passes over the slots behind them are skipped.
    Row8<T> kr[MF ? 1 : NPASS], vr[NPASS], kn[MF ? 1 : NPASS], vn[NPASS];
    uint4 ka[MF ? KST : 1], kan[MF ? KST : 1];       // K in A-operand layout (bf16 caches)
    bool kvalid = false, kvalidn = false;            // this lane's tile row holds a key
    int64_t rows[NPASS], rown[NPASS];
    // the K and V rows of the first n_live slots of a chunk, from the row numbers in srow: both
    // fetched together (one memory latency, not two)
    auto gather = [&](const int64_t *srow, int n_live, Row8<T> *kd, uint4 *kad, bool &kval, Row8<T> *vd, int64_t *rd) __attribute__((always_inline)) {
        constexpr int STEP = RPP > 16 ? RPP : 16;
        const int live = (n_live + STEP - 1) / STEP * STEP;
        const int np = live / RPP;
        if (MF) {
            kval = false;
            if (wave < NLW && wave * 16 < live) {
                const int64_t row = srow[wave * 16 + (lane & 15)];
                kval = row >= 0;
                const T *src = (const T *)a.K + (kval ? row : 0) * D + 8 * (lane >> 4);   // (a slot without a key reads row 0: never used)
#pragma unroll
                for (int st = 0; st < KST; ++st) kad[st] = *(const uint4 *)(src + 32 * st);
            }
        }
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            rd[p] = p < np ? srow[p * RPP + wave * RPW + rl] : -1;
            if (rd[p] >= 0) {
                if (!MF) kd[p].load((const T *)a.K + rd[p] * D + sub * 8);
                vd[p].load((const T *)a.V + rd[p] * D + sub * 8);
            } else {
                if (!MF) kd[p].zero();
                vd[p].zero();
            }
        }
    };
    // kRowsSweep: this thread's pending entry of the index row, written while rows are on their way
    auto emit_pending = [&]() __attribute__((always_inline)) {
        if (SRC == kRowsSweep && pend_t >= 0) {
            if (pend_slot < 0) {
                // a kept candidate: the entries of its region below it (a binary search, in the
                // region's head in LDS or past that in memory)
                int lo = 0, hi = min(count, kHeadEntries);   // first entry >= the position
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (s_head[mid] < pend_t) lo = mid + 1; else hi = mid;
                }
                if (lo == kHeadEntries) {
                    hi = count;
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (list[(int64_t)reg0 * kSlice + mid] < pend_t) lo = mid + 1; else hi = mid;
                    }
                }
                pend_slot = entries_before + lo;
            }
            const int at = pend_slot + kept_below(pend_t);
            if (at < a.max_k) idx_row[at] = pend_t;
            pend_t = -1;
        }
    };
    // (kr, vr, rows hold the chunk's rows)
    auto attend_chunk = [&](int n_live, auto whole) __attribute__((always_inline)) {
        constexpr int STEP = RPP > 16 ? RPP : 16;    // whole passes and whole batches of the value product
        constexpr bool WHOLE = decltype(whole)::value;        // every slot holds a row: nothing to skip
        const int live = WHOLE ? CH : (n_live + STEP - 1) / STEP * STEP;   // slots worked on
        const int np = WHOLE ? NPASS : live / RPP;
        // ---- logits: scale * k.q for every query head of the group
        if (MF) {
            if (wave < NLW && wave * 16 < live) {
                const int g = lane & 15, kg = lane >> 4;
                floatx4_t c = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int st = 0; st < KST; ++st) {
                    union { uint4 u; bf16x8_t v; } ua, ub;
                    ua.u = ka[st];
                    ub.u = g < G ? *(const uint4 *)&s_qb[g < G ? g : 0][32 * st + 8 * kg] : make_uint4(0, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua.v, ub.v, c, 0, 0, 0);
                }
                // c[e] = logit of tile row 4 kg + e for query head g; whether that row holds a key
                // is known to the lane that fetched it
                const unsigned long long have = __ballot(kvalid);
                if (g < G) {
                    float o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = ((have >> (4 * kg + e)) & 1ull) ? c[e] * a.scale : ninf;
                    *(float4 *)&s_p[g][wave * 16 + 4 * kg] = make_float4(o[0], o[1], o[2], o[3]);
                }
            }
        } else if (SRC == kRowsSweep) {              // (queries from LDS: registers decide how many workgroups fit)
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float4 q0 = *(const float4 *)&s_q[g][sub * 8], q1 = *(const float4 *)&s_q[g][sub * 8 + 4];
                const float qg[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
                for (int p = 0; p < NPASS; ++p) {
                    if (p >= np) break;
                    float kf[8];
                    kr[p].get(kf);
                    float dot = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) dot = fmaf(kf[e], qg[e], dot);
                    dot = row_sum<LPR>(dot);
                    if (sub == 0) s_p[g][p * RPP + wave * RPW + rl] = rows[p] >= 0 ? dot * a.scale : ninf;
                }
            }
        } else {                                     // (long runs of chunks: queries in registers, a row unpacked once)
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                if (p >= np) break;
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
        }
        if (VROUNDS == 1) {                          // the value rows ride along with the logits
#pragma unroll
            for (int p = 0; p < NPASS; ++p)
                if (p < np) vr[p].store(&s_v[p * RPP + wave * RPW + rl][sub * 8]);
        }
        __syncthreads();

        // ---- running softmax statistics, one wavefront per query head at a time
        for (int g = wave; g < G; g += NWAVE) {
            const float v = lane < live ? s_p[g][lane] : ninf;   // CH == 64 == wavefront size
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

        // ---- weighted value rows: one read of a row's channel pair serves all G query heads
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float corr = s_corr[g];
            acc[g][0] *= corr;
            acc[g][1] *= corr;
        }
#pragma unroll
        for (int round = 0; round < VROUNDS; ++round) {
            if (round * VROWS >= live) break;
            if (VROUNDS > 1) {
                if (round > 0) __syncthreads();      // the previous round's rows have been consumed
#pragma unroll
                for (int p = 0; p < PPR; ++p)
                    vr[round * PPR + p].store(&s_v[p * RPP + wave * RPW + rl][sub * 8]);
                __syncthreads();
            }
            // this group's rows of the tile, RB at a time
#pragma unroll
            for (int rb = 0; rb < RPR; rb += RB) {
                const int r0 = grp * RPR + rb;
                if (round * VROWS + r0 >= live) break;
                float2 v2[RB];
#pragma unroll
                for (int j = 0; j < RB; ++j) v2[j] = pair_f32(&s_v[r0 + j][2 * cp]);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float w[RB];
                    if (RB % 4 == 0) {
#pragma unroll
                        for (int j = 0; j < RB / 4; ++j) {
                            const float4 w4 = *(const float4 *)&s_p[g][round * VROWS + r0 + 4 * j];
                            w[4 * j] = w4.x; w[4 * j + 1] = w4.y; w[4 * j + 2] = w4.z; w[4 * j + 3] = w4.w;
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < RB; ++j) w[j] = s_p[g][round * VROWS + r0 + j];
                    }
#pragma unroll
                    for (int j = 0; j < RB; ++j) {
                        acc[g][0] = fmaf(w[j], v2[j].x, acc[g][0]);
                        acc[g][1] = fmaf(w[j], v2[j].y, acc[g][1]);
                    }
                }
            }
        }
        __syncthreads();
    };

    if (DENSE) {
        // Whole chunks of the sequence d_per split; the next chunk's rows are loaded while the
        // current chunk is worked on.
        int total = a.seq_len[b];
        total = total < 0 ? 0 : (total > a.map.max_n ? a.map.max_n : total);
        const int d_per = (((total + CH - 1) / CH + a.n_split - 1) / a.n_split) * CH;
        const int d_begin = split * d_per;
        const int d_end = min(total, d_begin + d_per);
        auto load_dense = [&](int c0, Row8<T> *kd, uint4 *kad, bool &kval, Row8<T> *vd, int64_t *rd) __attribute__((always_inline)) {
            if (MF) {
                kval = false;
                if (wave < NLW) {
                    const int t = c0 + wave * 16 + (lane & 15);
                    kval = t < d_end;
                    const T *src = (const T *)a.K + (kval ? a.map.row(b, h, t) : 0) * D + 8 * (lane >> 4);
#pragma unroll
                    for (int st = 0; st < KST; ++st) kad[st] = *(const uint4 *)(src + 32 * st);
                }
            }
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                const int t = c0 + p * RPP + wave * RPW + rl;
                rd[p] = t < d_end ? a.map.row(b, h, t) : -1;
                if (rd[p] >= 0) {
                    if (!MF) kd[p].load((const T *)a.K + rd[p] * D + sub * 8);
                    vd[p].load((const T *)a.V + rd[p] * D + sub * 8);
                } else {
                    if (!MF) kd[p].zero();
                    vd[p].zero();
                }
            }
        };
        if (d_begin < d_end) load_dense(d_begin, kr, ka, kvalid, vr, rows);
        for (int c0 = d_begin; c0 < d_end; c0 += CH) {
            if (c0 + CH < d_end) load_dense(c0 + CH, kn, kan, kvalidn, vn, rown);
            if (c0 + CH <= d_end) attend_chunk(CH, IntTag<true>());
            else attend_chunk(d_end - c0, IntTag<false>());
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                if (!MF) kr[p] = kn[p];
                vr[p] = vn[p];
                rows[p] = rown[p];
            }
            if (MF) {
#pragma unroll
                for (int st = 0; st < KST; ++st) ka[st] = kan[st];
                kvalid = kvalidn;
            }
        }
    } else {
        if (SRC == kRowsIdx) {
            // ---- this split's slots of the ordered row
            for (int c0 = r_begin; c0 < r_end; c0 += CH) {
                if (tid < CH) {
                    const int r = c0 + tid;
                    int64_t row = -1;
                    if (r < r_end && r < count) {
                        const int t = c0 == r_begin ? first : list[r];
                        if (t >= 0 && t < a.map.max_n) row = a.map.row(b, h, t);
                    }
                    s_row[0][tid] = row;
                }
                __syncthreads();
                const int n_live = max(0, min(CH, min(r_end, count) - c0));
                gather(s_row[0], n_live, kr, ka, kvalid, vr, rows);
                attend_chunk(n_live, IntTag<false>());
            }
        } else {
            // ---- this split's share of its regions, then its candidates
            for (int reg = reg0; reg < reg1; ++reg) {
                const int cnt = reg == reg0 ? count : (int)a.sel_cnt[(int64_t)bh * a.n_regions + reg];
                const int n_here = cnt > sub_i ? (cnt - sub_i + sub_n - 1) / sub_n : 0;     // entries of this split in the region
                const int n_rows = n_here + (reg == reg1 - 1 ? n_mine : 0);
                // the rows of chunk c0 into s_row[buf]
                auto fill = [&](int c0, int buf) __attribute__((always_inline)) {
                    if (tid < CH) {
                        const int r = c0 + tid;
                        int t = -1;
                        const bool ahead = reg == reg0 && r < n_here && r < NT;   // looked up by thread r at the start
                        if (ahead) {
                        } else if (r < n_here) {
                            t = list[(int64_t)reg * kSlice + sub_i + r * sub_n];
                            if (emit) {
                                pend_t = t;
                                pend_slot = entries_before + sub_i + r * sub_n;
                            }
                        } else if (r < n_rows) {
                            t = s_cpos[r - n_here];
                            if (emit) {
                                pend_t = t;
                                pend_slot = -1;
                            }
                        }
                        s_row[buf][tid] = ahead ? s_own[r] : (t >= 0 && t < a.map.max_n) ? a.map.row(b, h, t) : -1;
                    }
                };
                for (int c0 = 0; c0 < n_rows; c0 += CH) {
                    fill(c0, 0);
                    __syncthreads();
                    gather(s_row[0], min(CH, n_rows - c0), kr, ka, kvalid, vr, rows);
                    emit_pending();
                    attend_chunk(min(CH, n_rows - c0), IntTag<false>());
                }
            }
        }
    }

    // ---- this split's partial result: (max, sum, weighted value sum) per query head.  The
    //      groups' shares of the value sum are added in a fixed order through LDS (over the tile).
    float *part = a.partials + ((int64_t)(b * a.Hq + h * G) * a.n_split) * (D + 2);
    {
        float *s_red = (float *)dyn;                 // [NG][G][D]
#pragma unroll
        for (int g = 0; g < G; ++g)
            *(float2 *)&s_red[((size_t)grp * G + g) * D + 2 * cp] = make_float2(acc[g][0], acc[g][1]);
        __syncthreads();
        for (int o = tid; o < G * D / 2; o += NT) {  // a channel pair of one query head
            const int g = o / CPAIRS, c2 = o % CPAIRS;
            float2 sum = *(const float2 *)&s_red[(size_t)g * D + 2 * c2];
#pragma unroll
            for (int k = 1; k < NG; ++k) {
                const float2 t = *(const float2 *)&s_red[((size_t)k * G + g) * D + 2 * c2];
                sum.x += t.x;
                sum.y += t.y;
            }
            *(float2 *)&part[((int64_t)g * a.n_split + split) * (D + 2) + 2 + 2 * c2] = sum;
        }
    }
    if (tid < G) {
        part[((int64_t)tid * a.n_split + split) * (D + 2) + 0] = s_m[tid];
        part[((int64_t)tid * a.n_split + split) * (D + 2) + 1] = s_l[tid];
    }
    return false;
}

template <typename T, int D, int G, int SRC>
__global__ __launch_bounds__(kDecodeThreads) void sparse_decode_kernel(DecodeArgs a) {
    extern __shared__ __align__(16) char decode_lds[];
    decode_body<T, D, G, SRC>(a, blockIdx.x, blockIdx.y, blockIdx.z, decode_lds);
}

// Merge of the split-K partial results of one query head: out = sum_s w_s acc_s / sum_s w_s l_s
// with w_s = exp(m_s - max m).  NT threads: thread (channel c = tid % D, group sg = tid / D)
// takes the splits sg, sg + NT/D, ... of channel c, every load issued before the first use (at
// most 32 per thread: the hardware tracks 63 outstanding loads per wavefront, more would stall
// the issue), then the groups' sums are added in a fixed order through LDS.  Runs in a launch
// after the partial pass: no fence, no signalling.
constexpr int kMergeThreads = 512;

template <int D, int NT>
__device__ __forceinline__ void merge_body(const DecodeArgs &a, int g, int h, int b) {
    constexpr int NG = NT / D;                       // groups of D threads
    constexpr int PER = kMaxSplits / NG;             // splits per thread
    static_assert(NT % D == 0 && NG >= 2 && PER <= 64, "groups of D threads, at most 64 loads in flight each");
    __shared__ float s_w[kMaxSplits];
    __shared__ float s_den;
    __shared__ float s_red[NG][D];
    const int tid = threadIdx.x;
    const int c = tid % D, sg = tid / D;
    const int G = a.Hq / a.map.Hkv;
    const int64_t head = (int64_t)b * a.Hq + h * G + g;
    const float *part = a.partials + head * a.n_split * (D + 2);
    const float ninf = -__builtin_inff();
    // the first wavefront weighs the splits (two per lane): its (max, sum) loads go out first, so
    // that the weights are ready when the value sums arrive
    float m[2], l[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const bool live = tid < 64 && tid + 64 * j < a.n_split;
        m[j] = live ? part[(int64_t)(tid + 64 * j) * (D + 2)] : ninf;
        l[j] = live ? part[(int64_t)(tid + 64 * j) * (D + 2) + 1] : 0.0f;
    }
    float acc[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int s = sg + j * NG;
        acc[j] = s < a.n_split ? part[(int64_t)s * (D + 2) + 2 + c] : 0.0f;
    }
    if (tid < 64) {
        const float top = wave_max(fmaxf(m[0], m[1]));
        const float w0 = (m[0] == ninf) ? 0.0f : expf(m[0] - top), w1 = (m[1] == ninf) ? 0.0f : expf(m[1] - top);
        const float den = row_sum<64>(w0 * l[0] + w1 * l[1]);
        s_w[tid] = w0;
        s_w[tid + 64] = w1;
        if (tid == 0) s_den = den;
    }
    __syncthreads();
    float num = 0.0f;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int s = sg + j * NG;
        if (s < a.n_split) num = fmaf(s_w[s], acc[j], num);
    }
    s_red[sg][c] = num;
    __syncthreads();
    if (sg == 0) {
        float total = s_red[0][c];
#pragma unroll
        for (int gg = 1; gg < NG; ++gg) total += s_red[gg][c];
        const float den = s_den;
        const float y = den > 0.0f ? total / den : 0.0f;
        if (a.out_dtype == SOCKET_F32) ((float *)a.out)[head * D + c] = y;
        else ((uint16_t *)a.out)[head * D + c] = f32_to_bf16_rne(y);
    }
    __syncthreads();                                 // the LDS arrays may be rewritten by a following call
}

template <int D>
__global__ __launch_bounds__(kMergeThreads) void decode_merge_kernel(DecodeArgs a) {
    merge_body<D, kMergeThreads>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// The launch after the attention of the fused decode step: the merge of the splits for every
// query head, and one more workgroup per (sequence, KV head) that finishes the select: the -1
// fill behind the index row, the selected count, the shared scratch cleared for the next call.
// Where the attention's splits did not write the index row (they do unless a split owns several
// regions) that workgroup orders it (topk_resolve_body); where they left a head alone, its
// threshold bin holding more candidates than they rank (mass ties only), it orders the row,
// attends the head from it split after split, and merges it: slow and exact.
template <typename T, int D, int G>
__global__ __launch_bounds__(kTopkThreads, 6) void merge_finish_kernel(DecodeArgs a, TopkArgs t) {
    extern __shared__ __align__(16) char decode_lds[];
    const int h = blockIdx.y, b = blockIdx.z, bh = b * a.map.Hkv + h, tid = threadIdx.x;
    const uint32_t *thr = t.thr + (int64_t)bh * kThrStride;
    const uint32_t k_eff = thr[0];
    const bool redo = k_eff != 0 && thr[6] > (uint32_t)kSweepCand;
    if ((int)blockIdx.x < G) {
        if (!redo) merge_body<D, kTopkThreads>(a, blockIdx.x, h, b);
        return;
    }
    if (a.emit_idx && !redo) {
        int32_t *out = t.idx + (int64_t)bh * t.max_k;
        for (int i = (int)min(k_eff, (uint32_t)t.max_k) + tid; i < t.max_k; i += kTopkThreads) out[i] = -1;
        if (tid == 0) t.n_selected[bh] = (int32_t)k_eff;
        uint32_t *gh1 = t.hist + (int64_t)bh * kHistBins, *gh2 = t.hist2 + (int64_t)bh * kHistBins;
        for (int i = tid; i < kHistBins; i += kTopkThreads) {
            gh1[i] = 0;
            gh2[i] = 0;
        }
        if (tid < 2) t.counters[(int64_t)bh * kCounterStride + tid] = 0;
        return;
    }
    topk_resolve_body(t, bh, (uint32_t *)decode_lds);
    if (!redo) return;
    __threadfence();
    __syncthreads();                                 // the ordered row and its count are written
    // (every thread of the workgroup takes part: the bodies below are full of barriers)
    for (int s = 0; s < a.n_split; ++s) decode_body<T, D, G, kRowsIdx, kTopkThreads>(a, s, h, b, decode_lds);
    __threadfence();
    __syncthreads();
    for (int g = 0; g < G; ++g) merge_body<D, kTopkThreads>(a, g, h, b);
}

// which launch launch_decode makes: a RowSource, or
constexpr int kMergeFinish = -1;                     // merge_finish_kernel

template <typename T, int D, int G, int WHAT>
static int launch_decode_one(const DecodeArgs &a, const TopkArgs *t, dim3 grid, hipStream_t st) {
    if constexpr (WHAT == kMergeFinish) {
        constexpr size_t kLds = decode_lds_bytes<T, D, G, kTopkThreads>() > kResolveLds ? decode_lds_bytes<T, D, G, kTopkThreads>() : kResolveLds;
        static_assert(kLds <= 64 * 1024, "within the default dynamic LDS limit");
        hipLaunchKernelGGL((merge_finish_kernel<T, D, G>), dim3(G + 1, grid.y, grid.z), dim3(kTopkThreads), kLds, st, a, *t);
    } else {
        constexpr size_t kTile = decode_lds_bytes<T, D, G>();
        constexpr size_t kLds = WHAT == kRowsSweep && kTile < kSweepRankLds ? kSweepRankLds : kTile;
        hipLaunchKernelGGL((sparse_decode_kernel<T, D, G, WHAT>), grid, dim3(kDecodeThreads), kLds, st, a);
    }
    return SOCKET_OK;
}

template <typename T, int D, int WHAT>
static int launch_decode_g(const DecodeArgs &a, const TopkArgs *t, int G, dim3 grid, hipStream_t st) {
    switch (G) {
        case 1: return launch_decode_one<T, D, 1, WHAT>(a, t, grid, st);
        case 2: return launch_decode_one<T, D, 2, WHAT>(a, t, grid, st);
        case 4: return launch_decode_one<T, D, 4, WHAT>(a, t, grid, st);
        case 8: return launch_decode_one<T, D, 8, WHAT>(a, t, grid, st);
        default: return SOCKET_EUNSUPPORTED;
    }
}

template <typename T, int WHAT>
static int launch_decode_d(const DecodeArgs &a, const TopkArgs *t, int D, int G, dim3 grid, hipStream_t st) {
    switch (D) {
        case 64: return launch_decode_g<T, 64, WHAT>(a, t, G, grid, st);
        case 128: return launch_decode_g<T, 128, WHAT>(a, t, G, grid, st);
        case 256: return launch_decode_g<T, 256, WHAT>(a, t, G, grid, st);
        default: return SOCKET_EUNSUPPORTED;
    }
}

template <int WHAT>
static int launch_decode(const DecodeArgs &a, const TopkArgs *t, const Geometry &g, dim3 grid, hipStream_t st) {
    return g.kv_dtype == SOCKET_F32 ? launch_decode_d<float, WHAT>(a, t, g.d, g.G, grid, st)
                                    : launch_decode_d<uint16_t, WHAT>(a, t, g.d, g.G, grid, st);
}

static int launch_merge(const DecodeArgs &a, const Geometry &g, int batch, hipStream_t st) {
    dim3 mgrid(g.G, g.Hkv, batch);
    switch (g.d) {
        case 64: hipLaunchKernelGGL(decode_merge_kernel<64>, mgrid, dim3(kMergeThreads), 0, st, a); break;
        case 128: hipLaunchKernelGGL(decode_merge_kernel<128>, mgrid, dim3(kMergeThreads), 0, st, a); break;
        case 256: hipLaunchKernelGGL(decode_merge_kernel<256>, mgrid, dim3(kMergeThreads), 0, st, a); break;
        default: return SOCKET_EUNSUPPORTED;
    }
    return SOCKET_OK;
}

static DecodeArgs decode_args(const Geometry &g, float *partials, const void *q, const void *K, const void *V,
                              const int32_t *block_table, float scale, int out_dtype, void *out, int n_split) {
    DecodeArgs a;
    a.q = q; a.K = K; a.V = V; a.idx = nullptr; a.n_selected = nullptr; a.seq_len = nullptr;
    a.partials = partials; a.out = out;
    a.map = row_map(g, block_table);
    a.scale = scale; a.Hq = g.Hq; a.max_k = g.max_k; a.n_split = n_split; a.out_dtype = out_dtype;
    a.sel_regions = nullptr; a.sel_cnt = nullptr; a.n_regions = 0; a.ssr = 1; a.rpg = 1; a.emit_idx = 0;
    a.cand_key = nullptr; a.cand_idx = nullptr; a.thr = nullptr;
    return a;
}
static DecodeArgs decode_args(socket_ctx *ctx, const void *q, const void *K, const void *V,
                              const int32_t *block_table, float scale, int out_dtype, void *out, int n_split) {
    return decode_args(ctx->g, ctx->partials, q, K, V, block_table, scale, out_dtype, out, n_split);
}

// Eq. 1: every token below seq_len, 64 splits per (sequence, KV head)
int launch_dense_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const int32_t *block_table, const int32_t *seq_len, int batch, float scale,
                        int out_dtype, void *out, hipStream_t st) {
    const Geometry &g = ctx->g;
    DecodeArgs a = decode_args(ctx, q, K, V, block_table, scale, out_dtype, out, kDenseSplits);
    a.seq_len = seq_len;
    int rc = launch_decode<kRowsDense>(a, nullptr, g, dim3(kDenseSplits, g.Hkv, batch), st);
    if (rc != SOCKET_OK) return rc;
    rc = launch_merge(a, g, batch, st);
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

// Eq. 2 from the ordered index row, split-K partial results in `partials`
static int sparse_decode_launches(const Geometry &g, float *partials, const void *q, const void *K, const void *V,
                                  const int32_t *idx, const int32_t *n_selected, const int32_t *block_table,
                                  int batch, float scale, int out_dtype, void *out, hipStream_t st) {
    DecodeArgs a = decode_args(g, partials, q, K, V, block_table, scale, out_dtype, out, g.n_split);
    a.idx = idx; a.n_selected = n_selected;
    int rc = launch_decode<kRowsIdx>(a, nullptr, g, dim3(g.n_split, g.Hkv, batch), st);
    if (rc != SOCKET_OK) return rc;
    return launch_merge(a, g, batch, st);
}

int launch_sparse_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                         const int32_t *idx, const int32_t *n_selected, const int32_t *block_table,
                         int batch, float scale, int out_dtype, void *out, hipStream_t st) {
    int rc = sparse_decode_launches(ctx->g, ctx->partials, q, K, V, idx, n_selected, block_table, batch, scale,
                                    out_dtype, out, st);
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

// ---------------------------------------------------------------------------------------
// The same attention for callers that may not allocate: the split-K partial results live in
// a file-scope device array instead of a context's scratch.  Host code never passes the
// array's name to a kernel (there it is only a stand-in): its device address is asked for once
// per device and kept.
// ---------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)SOCKET_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_lock;
static void *scratch_ptr[kMaxDevices];               // device address of `scratch` on each device, once known

// the current device's copy of the array; null (and *err set) when HIP refuses
static void *static_scratch(hipError_t *err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !p) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}

int sparse_decode_noalloc(const socket_params *p, const void *q, const void *K, const void *V,
                          const int32_t *idx, const int32_t *n_selected, const int32_t *block_table,
                          int batch, float scale, int out_dtype, void *out, hipStream_t st, int *hip_error) {
    Geometry g;
    int rc = fill_geometry(p, &g);
    if (rc != SOCKET_OK) return rc;
    if (batch < 1 || batch > g.max_batch) return SOCKET_EINVAL;
    if ((g.page > 0) != (block_table != nullptr)) return SOCKET_EINVAL;
    const size_t need = (size_t)batch * g.Hq * g.n_split * (g.d + 2) * sizeof(float);
    if (need > kStaticScratchBytes) return SOCKET_ELIMIT;
    hipError_t e = hipSuccess;
    float *partials = (float *)static_scratch(&e);
    if (!partials) {
        if (hip_error) *hip_error = (int)e;
        return SOCKET_EHIP;
    }
    // nothing in the array has to start at zero: every split writes its whole partial result,
    // empty splits included, before the merge reads it
    rc = sparse_decode_launches(g, partials, q, K, V, idx, n_selected, block_table, batch, scale, out_dtype, out, st);
    if (rc != SOCKET_OK) return rc;
    e = hipGetLastError();
    if (e != hipSuccess) {
        if (hip_error) *hip_error = (int)e;
        return SOCKET_EHIP;
    }
    return SOCKET_OK;
}

// The tail of the fused decode step, after the select's sweep (launch_topk_sweep): Eq. 2 from
// the sweep's lists, the splits writing the index row as they go, then the merge of the splits
// with the select's finishing touches beside it.
int launch_sweep_decode(socket_ctx *ctx, const void *q, const void *K, const void *V,
                        const float *scores, const int32_t *seq_len, const int32_t *k,
                        int32_t *idx, int32_t *n_selected, int hist_mode, const int32_t *block_table,
                        int batch, float scale, int out_dtype, void *out, hipStream_t st) {
    const Geometry &g = ctx->g;
    const TopkArgs t = topk_args(ctx, scores, seq_len, k, idx, n_selected, hist_mode);
    DecodeArgs a = decode_args(ctx, q, K, V, block_table, scale, out_dtype, out, g.n_split_sweep);
    a.idx = idx; a.n_selected = n_selected;
    a.sel_regions = t.sel_regions; a.sel_cnt = t.sel_cnt; a.n_regions = g.n_regions; a.ssr = g.ssr; a.rpg = g.rpg;
    a.emit_idx = g.rpg == 1 && g.n_regions <= kDecodeThreads;
    a.seq_len = seq_len;
    a.cand_key = t.cand_key; a.cand_idx = t.cand_idx; a.thr = t.thr;
    const dim3 grid(g.n_split_sweep, g.Hkv, batch);
    int rc = launch_decode<kRowsSweep>(a, nullptr, g, grid, st);
    if (rc != SOCKET_OK) return rc;
    rc = launch_decode<kMergeFinish>(a, &t, g, grid, st);
    if (rc != SOCKET_OK) return rc;
    return record_hip(ctx, hipGetLastError());
}

}  // namespace sk

// The small kernels after the streaming pass:
//   merge_splits_kernel   "emit partial" of the per-shard attention (Sec. 2.1.1): folds the
//                         un-normalised split records of one shard into the shard's normalised
//                         partial output O_i and its log-sum-exp lse_i;
//   combine_kernel        the rescale-and-sum of the N shard fragments (Sec. 2.1.1, Sec. 2.2):
//                         w_i = exp(lse_i - max lse), O = sum w_i O_i / sum w_i;
//   shard_layout_kernel   the integer KVP cut of every sequence into N contiguous slices.
#pragma once
#include "common.hpp"

namespace helix {

struct MergeArgs {
    const float* ws_o;    // [split][B][Q][dv]
    const float* ws_m;    // [split][B][Q]
    const float* ws_l;
    float* o_part;        // [N][B][Q][dv]
    float* lse_part;      // [N][B][Q]
    int32_t B, Q, n_shards, shard0;   // shard0: index of the first shard of this launch in o_part
    int32_t split_base[kMaxLaunchShards];
    int32_t n_splits[kMaxLaunchShards];
    // records of a launch cut by stream_plan_kernel: pair p = (shard, sequence) owns one record per workgroup
    // whose tile range touches it, record rec_base + g + p, rows [record][Q]
    const int64_t* tile_prefix;       // NULL: records are [split][B][Q] as split_base / n_splits say
    const int2* pair_rec;             // MLA: [pairs] the workgroups g_first .. g_first + n - 1 that hold tiles of the pair
    const int2* row_rec;              // GQA: [rows] first and last seat (StreamSeat) that hold tiles of row (head tile, pair, kv head)
    int32_t n_wg, rec_base;
    int32_t K, g, head_tiles;         // GQA: kv heads, query heads per kv head, head tiles per kv head (records of 16 heads)
};

// Where the records of (shard i, sequence b, query head h) are in an evenly cut launch: n of them, record j in
// row first + j * stride of the record arrays.
struct StreamRecords {
    int n;
    size_t first, stride;
};

__device__ __forceinline__ StreamRecords stream_records(const MergeArgs& a, int i, int b, int h)
{
    const int p = i * a.B + b;
    StreamRecords r;
    r.n = 0; r.first = 0; r.stride = 0;
    if (a.pair_rec) {                     // MLA: one row per pair, a record holds all Q heads
        const int2 pr = a.pair_rec[p];
        r.n = pr.y;
        r.first = (size_t)(a.rec_base + pr.x + p) * a.Q + h;
        r.stride = (size_t)a.Q;
    } else if (a.tile_prefix[p + 1] > a.tile_prefix[p]) {      // GQA: a row per (head tile, pair, kv head), records of 16 heads
        const int kh = h / a.g, hin = h - kh * a.g, ht = hin >> 4;
        const int row = (ht * a.n_shards * a.B + p) * a.K + kh;
        const int2 rr = a.row_rec[row];
        r.n = rr.y - rr.x + 1;
        r.first = (size_t)(a.rec_base + rr.x + row) * 16 + (hin & 15);
        r.stride = 16;
    }
    return r;
}

// Where the records of one (shard, b, h) row are: record j (0 <= j < n) sits in row `row(j)` of the record
// arrays, or nowhere (kNoRecord).
constexpr size_t kNoRecord = ~(size_t)0;

struct SplitRecords {             // [split][B][Q]: records sb .. sb + n - 1 of row rem = b * Q + h
    int n;
    size_t first, stride;
    __device__ __forceinline__ size_t row(int j) const { return first + (size_t)j * stride; }
};


template <int DV>
struct MergeSmem {
    static constexpr int TPR = DV / 4;   // threads covering one row with float4
    static constexpr int SL = 256 / TPR; // split lanes working side by side
    float m[SL];
    float l[SL];
    float o[SL][DV];
};

// Threads that share one row's value columns in the kernels that fold the records of an evenly cut launch, and
// rows a workgroup of the fused kernel folds side by side.  That path is a chain of dependent memory round trips per
// row, so what counts is how many rows the part holds at once: few threads per row, each with several loads in flight.
constexpr int kFinishRowThreads = 32;
template <int DV>
constexpr int finish_row_threads() { return DV / 4 < kFinishRowThreads ? DV / 4 : kFinishRowThreads; }

// lse = (M + log2 L) ln 2.  M is an integer and may sit far from the true maximum (the MLA kernel
// keeps 32 octaves of headroom), so M and log2 L can cancel: L is split into 2^e * mant first, M + e
// is exact, and only log2(mant) in (-1, 0] carries a rounding error.
__device__ __forceinline__ float lse_of(float M, float L)
{
    if (!(L > 0.f)) return -INFINITY;
    const float e = (float)__builtin_amdgcn_frexp_expf(L);
    const float mant = __builtin_amdgcn_frexp_mantf(L);
    return ((M + e) + __builtin_log2f(mant)) * kLn2;
}

// Folds the split records of one (shard, b, h) row: M = max_j m_j, L = sum_j l_j 2^(m_j - M),
// O = sum_j O_j 2^(m_j - M) / L.  Records carry an integer reference exponent m (a float holding an
// integer, or -inf for "no tokens"), so every rescale is an exact power of two and the running
// maximum below changes no bit of the result.  One pass; the O row of an empty record (ragged
// sequences leave many) is not fetched.
// Returns the normalised O (valid in threads tid < TPR, 4 columns each); M and L in all threads.
template <int DV, class Records>
__device__ __forceinline__ f32x4 merge_row(const float* __restrict__ ws_o, const float* __restrict__ ws_m,
                                           const float* __restrict__ ws_l, const Records& recs,
                                           MergeSmem<DV>& sm, float& M, float& L)
{
    const int nsp = recs.n;
    using S = MergeSmem<DV>;
    const int tid = threadIdx.x;
    const int sl = tid / S::TPR, c4 = (tid % S::TPR) * 4;
    float Mt = -INFINITY, Lt = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // Four records in flight per thread: first their (m, l), then the O rows of those that are not empty.
    // One record at a time would make the loop a chain of dependent HBM round trips.
    constexpr int U = 4;
    for (int j0 = sl; j0 < nsp; j0 += S::SL * U) {
        float mj[U], lj[U];
        f32x4 oj[U];
        size_t rec[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int j = j0 + u * S::SL;
            mj[u] = -INFINITY;
            lj[u] = 0.f;
            rec[u] = j < nsp ? recs.row(j) : kNoRecord;
            if (rec[u] != kNoRecord) {
                mj[u] = ws_m[rec[u]];
                lj[u] = ws_l[rec[u]];
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            oj[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (mj[u] != -INFINITY)                // an empty record's O was never written: not fetched either
                oj[u] = *reinterpret_cast<const f32x4*>(ws_o + rec[u] * DV + c4);
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (mj[u] == -INFINITY) continue;
            if (mj[u] > Mt) {
                const float f = __builtin_amdgcn_exp2f(Mt - mj[u]);   // 0 from -inf
                acc *= f;
                Lt *= f;
                Mt = mj[u];
            }
            const float g = __builtin_amdgcn_exp2f(mj[u] - Mt);
            acc += oj[u] * g;
            Lt += lj[u] * g;
        }
    }
    __syncthreads();                       // previous users of sm are done
    *reinterpret_cast<f32x4*>(&sm.o[sl][c4]) = acc;
    if (c4 == 0) { sm.m[sl] = Mt; sm.l[sl] = Lt; }
    __syncthreads();
    M = -INFINITY;
#pragma unroll
    for (int k = 0; k < S::SL; k++) M = fmaxf(M, sm.m[k]);
    L = 0.f;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (M != -INFINITY) {
#pragma unroll
        for (int k = 0; k < S::SL; k++) {
            const float f = __builtin_amdgcn_exp2f(sm.m[k] - M);   // 0 for a lane without records
            L += sm.l[k] * f;
            if (tid < S::TPR) s += *reinterpret_cast<const f32x4*>(&sm.o[k][c4]) * f;
        }
        s *= (L > 0.f) ? 1.f / L : 0.f;
    }
    return s;
}

// The same fold for the records of an evenly cut launch: row (shard i, sequence b, head h) has one record per
// workgroup that holds tiles of it -- one to three as a rule for MLA, sixteen on the uniform GQA share.  SUB
// threads share a row's records (record j goes to sub-lane j % SUB) and each folds its records one after the other,
// four in flight; the sub-lanes' results are then folded in sub-lane order.  Which SUB a value width uses is fixed
// (stream_sublanes), so every kernel that folds a row produces the same bits.  A thread handles NV groups of four
// columns, c0 + v * cstride.
template <int DV>
constexpr int stream_sublanes() { return DV >= 512 ? 1 : 8; }
// shards the fused kernel folds side by side (its workgroup has at most 1024 threads)
template <int DV>
constexpr int finish_groups() { return 1024 / (finish_row_threads<DV>() * stream_sublanes<DV>()) < 8 ? 1024 / (finish_row_threads<DV>() * stream_sublanes<DV>()) : 8; }

// WITH_O = false folds the reference exponents and normalisers only (the same operations on them, hence the same
// Mt and Lt, without touching the O rows).
template <int DV, int NV, bool WITH_O = true>
__device__ __forceinline__ void fold_stream_records(const MergeArgs& a, const StreamRecords& recs, int sub, int nsub, int c0, int cstride,
                                                    f32x4 (&acc)[NV], float& Mt, float& Lt)
{
    const int n = recs.n;
    Mt = -INFINITY;
    Lt = 0.f;
#pragma unroll
    for (int v = 0; v < NV; v++) acc[v] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int U = 4;                  // records in flight, (m, l) and the O rows together
    for (int j0 = sub; j0 < n; j0 += U * nsub) {
        float mj[U], lj[U];
        f32x4 oj[U][NV];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int j = j0 + u * nsub;
            mj[u] = -INFINITY;
            lj[u] = 0.f;
#pragma unroll
            for (int v = 0; v < NV; v++) oj[u][v] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (j < n) {
                const size_t at = recs.first + (size_t)j * recs.stride;
                mj[u] = a.ws_m[at];
                lj[u] = a.ws_l[at];
                // (the O row of an empty record was never written: it is read all the same, to keep the two loads
                // independent, and dropped below)
                if constexpr (WITH_O) {
#pragma unroll
                    for (int v = 0; v < NV; v++) oj[u][v] = *reinterpret_cast<const f32x4*>(a.ws_o + at * DV + c0 + v * cstride);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (mj[u] == -INFINITY) continue;
            if (mj[u] > Mt) {
                const float f = __builtin_amdgcn_exp2f(Mt - mj[u]);   // 0 from -inf
#pragma unroll
                for (int v = 0; v < NV; v++) acc[v] *= f;
                Lt *= f;
                Mt = mj[u];
            }
            const float g = __builtin_amdgcn_exp2f(mj[u] - Mt);
#pragma unroll
            for (int v = 0; v < NV; v++) acc[v] += oj[u][v] * g;
            Lt += lj[u] * g;
        }
    }
}

// Shared memory of one row being folded by SUB sub-lanes.
template <int DV, int SUB>
struct StreamFoldSmem {
    float m[SUB], l[SUB];
    float o[SUB][DV];
};

// Folds the records of row (i, b, h) with the workgroup's threads (sub, c0): every thread of the WORKGROUP must call
// it the same number of times (it holds two barriers when SUB > 1); `active` = this thread has a row to fold.
// out / M / L are valid in the threads with sub == 0.
template <int DV, int NV, int SUB>
__device__ __forceinline__ void merge_stream_row(const MergeArgs& a, bool active, int i, int b, int h, int sub, int c0, int cstride,
                                                 StreamFoldSmem<DV, SUB>* sm, f32x4 (&out)[NV], float& M, float& L)
{
    StreamRecords recs;
    recs.n = 0; recs.first = 0; recs.stride = 0;
    if (active) recs = stream_records(a, i, b, h);
    f32x4 acc[NV];
    float Mt, Lt;
    fold_stream_records<DV, NV>(a, recs, sub, SUB, c0, cstride, acc, Mt, Lt);
    if constexpr (SUB > 1) {
        if (active) {
#pragma unroll
            for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(&sm->o[sub][c0 + v * cstride]) = acc[v];
            if (c0 == 0) { sm->m[sub] = Mt; sm->l[sub] = Lt; }
        }
        __syncthreads();
        if (active && sub == 0) {
            Mt = -INFINITY;
#pragma unroll
            for (int k = 0; k < SUB; k++) Mt = fmaxf(Mt, sm->m[k]);
            Lt = 0.f;
#pragma unroll
            for (int v = 0; v < NV; v++) acc[v] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (Mt != -INFINITY) {
#pragma unroll
                for (int k = 0; k < SUB; k++) {
                    const float f = __builtin_amdgcn_exp2f(sm->m[k] - Mt);       // 0 for a sub-lane without records
                    Lt += sm->l[k] * f;
#pragma unroll
                    for (int v = 0; v < NV; v++) acc[v] += *reinterpret_cast<const f32x4*>(&sm->o[k][c0 + v * cstride]) * f;
                }
            }
        }
        __syncthreads();                  // the staging area is free for the next row
    }
    M = Mt;
    L = Lt;
    const float inv = (Lt > 0.f) ? 1.f / Lt : 0.f;
#pragma unroll
    for (int v = 0; v < NV; v++) out[v] = acc[v] * inv;
}

// merge_stream_row done by ONE thread group on its own, without shared memory or barriers: the sub-lanes' folds one
// after the other, then their results in sub-lane order -- the same operations on the same values as
// merge_stream_row, hence the same bits.  For launches with so many rows that a workgroup per row would be bound by
// the rate at which workgroups start (a row then has one or two records as a rule).
template <int DV, int NV, int SUB, bool WITH_O = true>
__device__ __forceinline__ void merge_stream_row_alone(const MergeArgs& a, int i, int b, int h, int c0, int cstride,
                                                       f32x4 (&out)[NV], float& M, float& L)
{
    const StreamRecords recs = stream_records(a, i, b, h);
    f32x4 acc[NV];
    float Mt, Lt;
    if constexpr (SUB == 1) {
        fold_stream_records<DV, NV, WITH_O>(a, recs, 0, 1, c0, cstride, acc, Mt, Lt);
    } else {
        // the largest reference exponent of the row's records is what the sub-lanes' results are scaled to
        Mt = -INFINITY;
        for (int j = 0; j < recs.n; j++) Mt = fmaxf(Mt, a.ws_m[recs.first + (size_t)j * recs.stride]);
        Lt = 0.f;
#pragma unroll
        for (int v = 0; v < NV; v++) acc[v] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (Mt != -INFINITY) {
#pragma unroll 1
            for (int k = 0; k < SUB && k < recs.n; k++) {             // (a sub-lane without records adds zeros)
                f32x4 pk[NV];
                float mk, lk;
                fold_stream_records<DV, NV, WITH_O>(a, recs, k, SUB, c0, cstride, pk, mk, lk);
                const float f = __builtin_amdgcn_exp2f(mk - Mt);       // 0 for a sub-lane whose records are all empty
                Lt += lk * f;
#pragma unroll
                for (int v = 0; v < NV; v++) acc[v] += pk[v] * f;
            }
        }
    }
    M = Mt;
    L = Lt;
    const float inv = (Lt > 0.f) ? 1.f / Lt : 0.f;
#pragma unroll
    for (int v = 0; v < NV; v++) out[v] = acc[v] * inv;
}

// The fold of shard i's records of row rem = b * Q + h in the [split][B][Q] layout.
template <int DV>
__device__ __forceinline__ f32x4 merge_shard_row(const MergeArgs& a, int i, int rem, MergeSmem<DV>& sm, float& M, float& L)
{
    const int bq = a.B * a.Q;
    SplitRecords r;
    r.n = a.n_splits[i];
    r.first = (size_t)a.split_base[i] * bq + rem;
    r.stride = (size_t)bq;
    return merge_row<DV>(a.ws_o, a.ws_m, a.ws_l, r, sm, M, L);
}

// One workgroup per (shard, b, h) row: split records -> the shard's (O_i, lse_i).
template <int DV>
__global__ __launch_bounds__(256) void merge_splits_kernel(const MergeArgs a)
{
    __shared__ MergeSmem<DV> sm;
    const int tid = threadIdx.x;
    const int row = blockIdx.x;          // (i*B + b)*Q + h
    const int bq = a.B * a.Q;
    const int i = row / bq, rem = row % bq;
    float M, L;
    const size_t orow = (size_t)(a.shard0 + i) * bq + rem;
    if (a.tile_prefix) {
        constexpr int TPR = finish_row_threads<DV>(), NV = DV / (4 * TPR), SUB = stream_sublanes<DV>();
        static_assert(TPR * SUB <= 256, "threads of this kernel");
        __shared__ StreamFoldSmem<DV, SUB> fold;
        const bool active = tid < TPR * SUB;
        const int sub = tid / TPR, c0 = (tid % TPR) * 4;
        f32x4 o[NV];
        merge_stream_row<DV, NV, SUB>(a, active, i, rem / a.Q, rem % a.Q, sub, c0, 4 * TPR, &fold, o, M, L);
        if (active && sub == 0) {
#pragma unroll
            for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(a.o_part + orow * DV + c0 + v * 4 * TPR) = o[v];
            if (c0 == 0) a.lse_part[orow] = lse_of(M, L);
        }
        return;
    }
    const f32x4 o = merge_shard_row<DV>(a, i, rem, sm, M, L);
    if (tid < MergeSmem<DV>::TPR) *reinterpret_cast<f32x4*>(a.o_part + orow * DV + tid * 4) = o;
    if (tid == 0) a.lse_part[orow] = lse_of(M, L);
}

// One step of the combine's running sums; combine_kernel and finish_kernel share it so that both
// produce the same bits from the same fragments.
__device__ __forceinline__ void combine_accumulate(f32x4& acc, float& wsum, const f32x4& o_i, float lse_i, float top)
{
    const float w = __expf(lse_i - top);
    wsum += w;
    acc += o_i * w;
}

struct FinishArgs {
    MergeArgs m;          // shard0 must be 0 and m.n_shards the total number of shards (<= kMaxLaunchShards)
    float* o;             // [B][Q][dv]
    float* lse_out;       // [B][Q] or NULL
    int32_t keep_parts;   // finish_stream_kernel: also store the per-shard fragments (the caller asked for them)
};

// merge + combine in one launch for an evenly cut launch of at most kMaxLaunchShards shards: one workgroup per
// (b, h) row, its threads in groups that fold different shards side by side (merge_stream_row); the fragments meet
// in shared memory, where they are combined in shard order -- the arithmetic of merge_splits_kernel followed by
// combine_kernel, without the round trip of the fragments through memory.  Launched with
// finish_row_threads<DV>() * stream_sublanes<DV>() * min(shards, finish_groups<DV>()) threads.
template <int DV>
__global__ __launch_bounds__(finish_row_threads<DV>() * stream_sublanes<DV>() * finish_groups<DV>()) void finish_stream_kernel(const FinishArgs f)
{
    constexpr int TPR = finish_row_threads<DV>(), NV = DV / (4 * TPR), SUB = stream_sublanes<DV>();
    static_assert(NV >= 1 && NV * 4 * TPR == DV, "whole float4 columns per thread");
    static_assert(TPR * SUB * finish_groups<DV>() <= 1024, "threads of a workgroup");
    __shared__ float sm_o[kMaxLaunchShards][DV];
    __shared__ float sm_lse[kMaxLaunchShards];
    __shared__ StreamFoldSmem<DV, SUB> fold[finish_groups<DV>()];
    const MergeArgs& a = f.m;
    const int tid = threadIdx.x, G = blockDim.x / (TPR * SUB);
    const int grp = tid / (TPR * SUB), sub = (tid / TPR) % SUB, c0 = (tid % TPR) * 4;
    const int rem = blockIdx.x;          // b*Q + h
    const int b = rem / a.Q, h = rem % a.Q;
    const size_t bq = (size_t)a.B * a.Q;
    for (int i0 = 0; i0 < a.n_shards; i0 += G) {       // the same trip count for every thread: the fold holds barriers
        const int i = i0 + grp;
        const bool active = i < a.n_shards;
        float M, L;
        f32x4 o[NV];
        merge_stream_row<DV, NV, SUB>(a, active, i, b, h, sub, c0, 4 * TPR, &fold[grp], o, M, L);
        if (active && sub == 0) {
            const float lse = lse_of(M, L);
#pragma unroll
            for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(&sm_o[i][c0 + v * 4 * TPR]) = o[v];
            if (c0 == 0) sm_lse[i] = lse;
            if (f.keep_parts) {
#pragma unroll
                for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(a.o_part + ((size_t)i * bq + rem) * DV + c0 + v * 4 * TPR) = o[v];
                if (c0 == 0) a.lse_part[(size_t)i * bq + rem] = lse;
            }
        }
    }
    __syncthreads();
    // the combine, shard after shard as combine_kernel does it; the threads share the columns
    float top = -INFINITY;
    for (int i = 0; i < a.n_shards; i++) top = fmaxf(top, sm_lse[i]);
    float wsum = 0.f;
    for (int c = tid * 4; c < DV; c += blockDim.x * 4) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        wsum = 0.f;
        if (top != -INFINITY) {
            for (int i = 0; i < a.n_shards; i++) {
                const float li = sm_lse[i];
                if (li == -INFINITY) continue;
                combine_accumulate(acc, wsum, *reinterpret_cast<const f32x4*>(&sm_o[i][c]), li, top);
            }
            acc *= 1.f / wsum;
        }
        *reinterpret_cast<f32x4*>(f.o + (size_t)rem * DV + c) = acc;
    }
    if (tid == 0 && f.lse_out) f.lse_out[rem] = (top != -INFINITY) ? top + __logf(wsum) : -INFINITY;
}

// finish_stream_kernel for launches with many (b, h) rows: 256 / finish_row_threads rows per workgroup, every row
// folded and combined by its own thread group (merge_stream_row_alone) -- two passes over the shards, the first over
// the normalisers only, for the largest lse, the second folding every fragment once more and weighing it at once,
// in shard order: the operations of finish_stream_kernel on the same values.
constexpr int64_t kManyRows = 2048;       // from this many rows on the launch is cut by rows, not by workgroups per row
template <int DV>
constexpr int finish_rows_per_workgroup() { return 256 / finish_row_threads<DV>(); }

template <int DV>
__global__ __launch_bounds__(256) void finish_rows_kernel(const FinishArgs f)
{
    constexpr int TPR = finish_row_threads<DV>(), NV = DV / (4 * TPR), SUB = stream_sublanes<DV>(), RPW = 256 / TPR;
    static_assert(RPW * TPR == 256, "rows of a workgroup (finish_rows_per_workgroup)");
    const MergeArgs& a = f.m;
    const int tid = threadIdx.x, c0 = (tid % TPR) * 4;
    const int64_t bq = (int64_t)a.B * a.Q;
    const int64_t rem = (int64_t)blockIdx.x * RPW + tid / TPR;       // b*Q + h
    if (rem >= bq) return;
    const int b = (int)(rem / a.Q), h = (int)(rem - (int64_t)b * a.Q);
    float top = -INFINITY;
    for (int i = 0; i < a.n_shards; i++) {
        f32x4 none[NV];
        float M, L;
        merge_stream_row_alone<DV, NV, SUB, false>(a, i, b, h, c0, 4 * TPR, none, M, L);
        top = fmaxf(top, lse_of(M, L));
    }
    f32x4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; v++) acc[v] = f32x4{0.f, 0.f, 0.f, 0.f};
    float wsum = 0.f;
    for (int i = 0; i < a.n_shards; i++) {
        f32x4 o[NV];
        float M, L;
        merge_stream_row_alone<DV, NV, SUB>(a, i, b, h, c0, 4 * TPR, o, M, L);
        const float lse = lse_of(M, L);
        if (f.keep_parts) {
#pragma unroll
            for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(a.o_part + ((size_t)i * bq + rem) * DV + c0 + v * 4 * TPR) = o[v];
            if (c0 == 0) a.lse_part[(size_t)i * bq + rem] = lse;
        }
        if (top == -INFINITY || lse == -INFINITY) continue;
        float wnext = wsum;               // (every column group of the thread takes the same step)
#pragma unroll
        for (int v = 0; v < NV; v++) {
            wnext = wsum;
            combine_accumulate(acc[v], wnext, o[v], lse, top);
        }
        wsum = wnext;
    }
    if (top != -INFINITY) {
#pragma unroll
        for (int v = 0; v < NV; v++) acc[v] *= 1.f / wsum;
    }
#pragma unroll
    for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(f.o + (size_t)rem * DV + c0 + v * 4 * TPR) = acc[v];
    if (c0 == 0 && f.lse_out) f.lse_out[rem] = (top != -INFINITY) ? top + __logf(wsum) : -INFINITY;
}

// merge_splits_kernel for evenly cut launches with many rows: a thread group per (shard, b, h) row.
template <int DV>
__global__ __launch_bounds__(256) void merge_rows_kernel(const MergeArgs a)
{
    constexpr int TPR = finish_row_threads<DV>(), NV = DV / (4 * TPR), SUB = stream_sublanes<DV>(), RPW = 256 / TPR;
    const int tid = threadIdx.x, c0 = (tid % TPR) * 4;
    const int64_t bq = (int64_t)a.B * a.Q;
    const int64_t row = (int64_t)blockIdx.x * RPW + tid / TPR;       // (i*B + b)*Q + h
    if (row >= bq * a.n_shards) return;
    const int i = (int)(row / bq);
    const int64_t rem = row - (int64_t)i * bq;
    const int b = (int)(rem / a.Q), h = (int)(rem - (int64_t)b * a.Q);
    f32x4 o[NV];
    float M, L;
    merge_stream_row_alone<DV, NV, SUB>(a, i, b, h, c0, 4 * TPR, o, M, L);
    const size_t orow = (size_t)(a.shard0 + i) * bq + rem;
#pragma unroll
    for (int v = 0; v < NV; v++) *reinterpret_cast<f32x4*>(a.o_part + orow * DV + c0 + v * 4 * TPR) = o[v];
    if (c0 == 0) a.lse_part[orow] = lse_of(M, L);
}

// merge_splits + combine in one launch for calls with at most kMaxLaunchShards shards:
// one workgroup per (b, h) row; emits the per-shard fragments (O_i, lse_i) AND the combined output.
template <int DV>
__global__ __launch_bounds__(256) void finish_kernel(const FinishArgs f)
{
    __shared__ MergeSmem<DV> sm;
    const MergeArgs& a = f.m;
    const int tid = threadIdx.x;
    const int rem = blockIdx.x;          // b*Q + h
    const int bq = a.B * a.Q;
    constexpr int TPR = MergeSmem<DV>::TPR;
    if (a.n_shards == 1) {               // the combine of one fragment is the fragment itself, bit for bit
        float M, L;
        const f32x4 o = merge_shard_row<DV>(a, 0, rem, sm, M, L);
        if (tid < TPR) {
            *reinterpret_cast<f32x4*>(a.o_part + (size_t)rem * DV + tid * 4) = o;
            *reinterpret_cast<f32x4*>(f.o + (size_t)rem * DV + tid * 4) = o;
        }
        if (tid == 0) {
            const float lse = lse_of(M, L);
            a.lse_part[rem] = lse;
            if (f.lse_out) f.lse_out[rem] = lse;
        }
        return;
    }
    __shared__ float sh_lse[kMaxLaunchShards];
    float top = -INFINITY;
    for (int i = 0; i < a.n_shards; i++) {
        float M, L;
        const f32x4 o = merge_shard_row<DV>(a, i, rem, sm, M, L);
        const float lse = lse_of(M, L);
        if (tid < TPR) *reinterpret_cast<f32x4*>(a.o_part + ((size_t)i * bq + rem) * DV + tid * 4) = o;
        if (tid == 0) { a.lse_part[(size_t)i * bq + rem] = lse; sh_lse[i] = lse; }
        top = fmaxf(top, lse);
    }
    __syncthreads();
    // second loop: every thread re-reads its own columns of every fragment (it wrote them itself)
    if (tid < TPR) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float wsum = 0.f;
        if (top != -INFINITY) {
            for (int i = 0; i < a.n_shards; i++) {
                const float li = sh_lse[i];
                if (li == -INFINITY) continue;
                combine_accumulate(acc, wsum, *reinterpret_cast<const f32x4*>(a.o_part + ((size_t)i * bq + rem) * DV + tid * 4), li, top);
            }
            acc *= 1.f / wsum;
        }
        *reinterpret_cast<f32x4*>(f.o + (size_t)rem * DV + tid * 4) = acc;
        if (tid == 0 && f.lse_out) f.lse_out[rem] = (top != -INFINITY) ? top + __logf(wsum) : -INFINITY;
    }
}

// Rows = B*Q.  256/TPR rows per workgroup, TPR threads per row, a loop over the N shards.
template <int DV>
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ o_parts, const float* __restrict__ lses,
                                                      float* __restrict__ o, float* __restrict__ lse_out,
                                                      int32_t* __restrict__ argmax_shard, int32_t n_shards, int64_t rows)
{
    constexpr int TPR = DV / 4;
    constexpr int RPB = 256 / TPR;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * RPB + tid / TPR;
    if (row >= rows) return;
    const int c4 = (tid % TPR) * 4;

    float top = -INFINITY;
    int best = 0;
    for (int i = 0; i < n_shards; i++) {
        const float li = lses[(int64_t)i * rows + row];
        if (li > top) { top = li; best = i; }
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float wsum = 0.f;
    if (top != -INFINITY) {
        for (int i = 0; i < n_shards; i++) {
            const float li = lses[(int64_t)i * rows + row];
            if (li == -INFINITY) continue;
            combine_accumulate(acc, wsum, *reinterpret_cast<const f32x4*>(o_parts + ((int64_t)i * rows + row) * DV + c4), li, top);
        }
        acc *= 1.f / wsum;
    }
    *reinterpret_cast<f32x4*>(o + row * DV + c4) = acc;
    if (c4 == 0) {
        if (lse_out) lse_out[row] = (top != -INFINITY) ? top + __logf(wsum) : -INFINITY;
        if (argmax_shard) argmax_shard[row] = best;
    }
}

__global__ void shard_layout_kernel(const int32_t* __restrict__ seq_len, const int64_t* __restrict__ seq_base,
                                    int32_t B, int32_t N, int64_t* __restrict__ shard_off, int32_t* __restrict__ shard_len)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * N) return;
    const int i = idx / B, b = idx % B;
    const int64_t L = seq_len[b];
    const int64_t per = (L + N - 1) / N;
    const int64_t c = 16 * ((per + 15) / 16);
    const int64_t lo = min((int64_t)i * c, L), hi = min((int64_t)(i + 1) * c, L);
    shard_off[idx] = lo + (seq_base ? seq_base[b] : 0);
    shard_len[idx] = (int32_t)(hi - lo);
}

// Staggered KV append (Sec. 2.3): one workgroup per sequence copies the new token's row of every KV
// head into the owner shard at position len[b] and bumps len[b].  Pure byte copies: an element is
// num/den bytes (bf16 2/1, e4m3 1/1, MXFP4 1/2), rows of dk (and dv) elements; MXFP4 rows carry
// dk/32 (dv/32) block-scale bytes in separate arrays.
struct AppendArgs {
    ShardDev sh;          // the owner shard
    const uint8_t* k_new; // [B][K][dk elements]
    const uint8_t* v_new; // [B][K][dv elements] or NULL
    const float* scale_new;
    const uint8_t* k_mx_new; // MXFP4: [B][K][dk/32]
    const uint8_t* v_mx_new; // MXFP4: [B][K][dv/32]
    int32_t* len;         // the owner's len array (writable alias of sh.len)
    int32_t* overflow;
    int32_t K, dk, dv, num, den, capacity;
};

__global__ __launch_bounds__(256) void kv_append_kernel(const AppendArgs a)
{
    const int b = blockIdx.x, tid = threadIdx.x;
    __shared__ int s_len;
    if (tid == 0) s_len = a.len[b];
    __syncthreads();
    const int len = s_len;
    if (len >= a.capacity) {
        if (tid == 0 && a.overflow) *a.overflow = 1;
        return;
    }
    const int64_t tok = (a.sh.tok_off ? a.sh.tok_off[b] : 0) + len;
    uint8_t* kdst = const_cast<uint8_t*>(static_cast<const uint8_t*>(a.sh.k));
    uint8_t* vdst = const_cast<uint8_t*>(static_cast<const uint8_t*>(a.sh.v));
    float* sdst = const_cast<float*>(a.sh.kv_scale);
    const int krow = a.dk * a.num / a.den, vrow = a.dv * a.num / a.den;
    for (int i = tid; i < a.K * krow; i += 256) {
        const int kh = i / krow, x = i % krow;
        kdst[((int64_t)b * a.sh.k_sb + (int64_t)kh * a.sh.k_sh + tok * a.sh.k_st) * a.num / a.den + x] = a.k_new[((int64_t)b * a.K + kh) * krow + x];
    }
    if (a.v_new)
        for (int i = tid; i < a.K * vrow; i += 256) {
            const int kh = i / vrow, x = i % vrow;
            vdst[((int64_t)b * a.sh.v_sb + (int64_t)kh * a.sh.v_sh + tok * a.sh.v_st) * a.num / a.den + x] = a.v_new[((int64_t)b * a.K + kh) * vrow + x];
        }
    if (a.scale_new)
        for (int kh = tid; kh < a.K; kh += 256)
            sdst[(int64_t)b * a.sh.s_sb + (int64_t)kh * a.sh.s_sh + tok] = a.scale_new[(int64_t)b * a.K + kh];
    if (a.k_mx_new) {
        uint8_t* kmx = const_cast<uint8_t*>(a.sh.k_mx);
        uint8_t* vmx = const_cast<uint8_t*>(a.sh.v_mx);
        const int kr = a.dk / 32, vr = a.dv / 32;
        for (int i = tid; i < a.K * kr; i += 256) {
            const int kh = i / kr, x = i % kr;
            kmx[((int64_t)b * a.sh.k_sb + (int64_t)kh * a.sh.k_sh + tok * a.sh.k_st) / 32 + x] = a.k_mx_new[((int64_t)b * a.K + kh) * kr + x];
        }
        for (int i = tid; a.v_mx_new && i < a.K * vr; i += 256) {
            const int kh = i / vr, x = i % vr;
            vmx[((int64_t)b * a.sh.v_sb + (int64_t)kh * a.sh.v_sh + tok * a.sh.v_st) / 32 + x] = a.v_mx_new[((int64_t)b * a.K + kh) * vr + x];
        }
    }
    if (tid == 0) a.len[b] = len + 1;     // every thread took its copy of the old length before the barrier
}

}  // namespace helix

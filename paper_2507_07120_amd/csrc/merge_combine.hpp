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
    const int2* pair_rec;             // [pairs] the workgroups g_first .. g_first + n - 1 that hold tiles of the pair
    int32_t n_wg, rec_base;
};

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

// The same fold for the records of an evenly cut launch (stream_plan_kernel): pair (shard i, sequence b) has one
// record per workgroup that holds tiles of it -- one to three as a rule.  They are folded by ONE thread per four
// value columns, record after record in workgroup order, so no shared memory and no barrier is involved and a
// workgroup can fold several shards side by side.  A thread handles NV groups of four columns, c0 + v * cstride:
// out[v] receives their normalised O; M, L as above.  (How many columns a thread holds changes no bit.)
template <int DV, int NV>
__device__ __forceinline__ void merge_stream_row(const MergeArgs& a, int i, int b, int h, int c0, int cstride, f32x4 (&out)[NV], float& M, float& L)
{
    const int p = i * a.B + b;
    const int2 pr = a.pair_rec[p];
    const int n = abs(pr.y);
    const bool gaps = pr.y < 0;
    int64_t T = 0;
    if (gaps) T = a.tile_prefix[a.n_shards * a.B];
    const size_t row0 = (size_t)(a.rec_base + pr.x + p) * a.Q + h;
    float Mt = -INFINITY, Lt = 0.f;
    f32x4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; v++) acc[v] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int U = NV >= 4 ? 2 : 4;    // records in flight: first their (m, l), then the O rows
    for (int j0 = 0; j0 < n; j0 += U) {
        float mj[U], lj[U];
        f32x4 oj[U][NV];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int j = j0 + u;
            mj[u] = -INFINITY;
            lj[u] = 0.f;
            // a workgroup without a tile (launches with fewer tiles than workgroups) wrote no record
            const bool there = j < n && !(gaps && stream_start(pr.x + j, T, a.n_wg) == stream_start(pr.x + j + 1, T, a.n_wg));
            if (there) {
                mj[u] = a.ws_m[row0 + (size_t)j * a.Q];
                lj[u] = a.ws_l[row0 + (size_t)j * a.Q];
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++)
#pragma unroll
            for (int v = 0; v < NV; v++) {
                oj[u][v] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (mj[u] != -INFINITY)
                    oj[u][v] = *reinterpret_cast<const f32x4*>(a.ws_o + (row0 + (size_t)(j0 + u) * a.Q) * DV + c0 + v * cstride);
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
        if (tid < MergeSmem<DV>::TPR) {
            f32x4 o[1];
            merge_stream_row<DV, 1>(a, i, rem / a.Q, rem % a.Q, tid * 4, 0, o, M, L);
            *reinterpret_cast<f32x4*>(a.o_part + orow * DV + tid * 4) = o[0];
            if (tid == 0) a.lse_part[orow] = lse_of(M, L);
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
// (b, h) row, its threads in groups of kFinishRowThreads that fold different shards side by side
// (merge_stream_row, DV / kFinishRowThreads columns per thread); the fragments meet in shared memory, where the
// first group combines them in shard order -- the arithmetic of merge_splits_kernel followed by combine_kernel,
// without the round trip of the fragments through memory.  The path is a chain of dependent memory round trips
// per row, so what counts is how many rows the part holds at once: few threads per row, each with several loads
// in flight.  Launched with kFinishRowThreads * min(shards, kFinishGroups) threads.
constexpr int kFinishRowThreads = 32, kFinishGroups = 8;

template <int DV>
__global__ __launch_bounds__(kFinishRowThreads * kFinishGroups) void finish_stream_kernel(const FinishArgs f)
{
    constexpr int TPR = kFinishRowThreads, NV = DV / (4 * TPR);
    static_assert(NV >= 1 && NV * 4 * TPR == DV, "whole float4 columns per thread");
    __shared__ float sm_o[kMaxLaunchShards][DV];
    __shared__ float sm_lse[kMaxLaunchShards];
    const MergeArgs& a = f.m;
    const int tid = threadIdx.x, grp = tid / TPR, c0 = (tid % TPR) * 4, G = blockDim.x / TPR;
    const int rem = blockIdx.x;          // b*Q + h
    const int b = rem / a.Q, h = rem % a.Q;
    const size_t bq = (size_t)a.B * a.Q;
    for (int i = grp; i < a.n_shards; i += G) {
        float M, L;
        f32x4 o[NV];
        merge_stream_row<DV, NV>(a, i, b, h, c0, 4 * TPR, o, M, L);
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
    __syncthreads();
    // the combine, shard after shard as combine_kernel does it; the groups share the columns
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

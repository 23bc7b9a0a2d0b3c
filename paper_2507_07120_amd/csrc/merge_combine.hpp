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
};

template <int DV>
struct MergeSmem {
    static constexpr int TPR = DV / 4;   // threads covering one row with float4
    static constexpr int SL = 256 / TPR; // split lanes working side by side
    float red[4];
    float l[SL];
    float o[SL][DV];
};

// Reference exponent M = max_j m_j and normaliser L = sum_j l_j 2^(m_j - M) of one (shard, b, h)
// row over its split records.  Records carry an integer reference exponent m (a float holding an
// integer, or -inf for "no tokens"), so every rescale 2^(m_j - M) is exact.  All 256 threads call
// it and all get the same bits.
template <int DV>
__device__ __forceinline__ void shard_row_stats(const float* __restrict__ ws_m, const float* __restrict__ ws_l,
                                                int sb, int nsp, int bq, int rem, MergeSmem<DV>& sm, float& M, float& L)
{
    using S = MergeSmem<DV>;
    const int tid = threadIdx.x;
    float mloc = -INFINITY;
    for (int j = tid; j < nsp; j += 256) mloc = fmaxf(mloc, ws_m[(size_t)(sb + j) * bq + rem]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, off));
    __syncthreads();                       // previous users of sm are done
    if ((tid & 63) == 0) sm.red[tid >> 6] = mloc;
    __syncthreads();
    M = fmaxf(fmaxf(sm.red[0], sm.red[1]), fmaxf(sm.red[2], sm.red[3]));
    const int sl = tid / S::TPR;
    if (tid % S::TPR == 0) {
        float lacc = 0.f;
        if (M != -INFINITY)
            for (int j = sl; j < nsp; j += S::SL) {
                const size_t rec = (size_t)(sb + j) * bq + rem;
                const float mj = ws_m[rec];
                if (mj != -INFINITY) lacc += ws_l[rec] * __builtin_amdgcn_exp2f(mj - M);
            }
        sm.l[sl] = lacc;
    }
    __syncthreads();
    L = 0.f;
#pragma unroll
    for (int k = 0; k < S::SL; k++) L += sm.l[k];
}

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

// The normalised partial O_i of the row: sum_j O_j 2^(m_j - M) / L.  Valid in threads tid < TPR
// (4 columns each).
template <int DV>
__device__ __forceinline__ f32x4 shard_row_output(const float* __restrict__ ws_o, const float* __restrict__ ws_m,
                                                  int sb, int nsp, int bq, int rem, MergeSmem<DV>& sm, float M, float L)
{
    using S = MergeSmem<DV>;
    const int tid = threadIdx.x;
    const int sl = tid / S::TPR, c4 = (tid % S::TPR) * 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (M != -INFINITY) {
        for (int j = sl; j < nsp; j += S::SL) {
            const size_t rec = (size_t)(sb + j) * bq + rem;
            const float mj = ws_m[rec];
            if (mj == -INFINITY) continue;            // empty record: its O was never written
            acc += *reinterpret_cast<const f32x4*>(ws_o + rec * DV + c4) * __builtin_amdgcn_exp2f(mj - M);
        }
    }
    __syncthreads();
    *reinterpret_cast<f32x4*>(&sm.o[sl][c4]) = acc;
    __syncthreads();
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (tid < S::TPR) {
#pragma unroll
        for (int k = 0; k < S::SL; k++) s += *reinterpret_cast<const f32x4*>(&sm.o[k][c4]);
        s *= (L > 0.f) ? 1.f / L : 0.f;
    }
    return s;
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
    shard_row_stats<DV>(a.ws_m, a.ws_l, a.split_base[i], a.n_splits[i], bq, rem, sm, M, L);
    const f32x4 o = shard_row_output<DV>(a.ws_o, a.ws_m, a.split_base[i], a.n_splits[i], bq, rem, sm, M, L);
    const size_t orow = (size_t)(a.shard0 + i) * bq + rem;
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
};

// merge_splits + combine in one launch for calls with at most kMaxLaunchShards shards:
// one workgroup per (b, h) row; emits the per-shard fragments (O_i, lse_i) AND the combined output.
template <int DV>
__global__ __launch_bounds__(256) void finish_kernel(const FinishArgs f)
{
    __shared__ MergeSmem<DV> sm;
    __shared__ float sh_M[kMaxLaunchShards], sh_L[kMaxLaunchShards];
    const MergeArgs& a = f.m;
    const int tid = threadIdx.x;
    const int rem = blockIdx.x;          // b*Q + h
    const int bq = a.B * a.Q;
    float top = -INFINITY;
    for (int i = 0; i < a.n_shards; i++) {
        float M, L;
        shard_row_stats<DV>(a.ws_m, a.ws_l, a.split_base[i], a.n_splits[i], bq, rem, sm, M, L);
        if (tid == 0) { sh_M[i] = M; sh_L[i] = L; a.lse_part[(size_t)i * bq + rem] = lse_of(M, L); }
        top = fmaxf(top, lse_of(M, L));
    }
    __syncthreads();
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float wsum = 0.f;
    for (int i = 0; i < a.n_shards; i++) {
        const float M = sh_M[i], L = sh_L[i];
        const f32x4 o = shard_row_output<DV>(a.ws_o, a.ws_m, a.split_base[i], a.n_splits[i], bq, rem, sm, M, L);
        if (tid < MergeSmem<DV>::TPR) {
            *reinterpret_cast<f32x4*>(a.o_part + ((size_t)i * bq + rem) * DV + tid * 4) = o;
            const float li = lse_of(M, L);
            if (li != -INFINITY) combine_accumulate(acc, wsum, o, li, top);
        }
    }
    if (tid < MergeSmem<DV>::TPR) {
        if (top != -INFINITY) acc *= 1.f / wsum;
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

}  // namespace helix

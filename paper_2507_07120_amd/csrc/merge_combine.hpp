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

// One workgroup per (shard, b, h) row.  Records carry an integer reference exponent m (a float
// holding an integer, or -inf for "no tokens"), so every rescale 2^(m_j - M) is exact.
template <int DV>
__global__ __launch_bounds__(256) void merge_splits_kernel(const MergeArgs a)
{
    constexpr int TPR = DV / 4;          // threads covering one row with float4
    constexpr int SL = 256 / TPR;        // split lanes working side by side
    static_assert(256 % TPR == 0, "row width must divide the workgroup");
    const int tid = threadIdx.x;
    const int row = blockIdx.x;          // (i*B + b)*Q + h
    const int bq = a.B * a.Q;
    const int i = row / bq, rem = row % bq;
    const int nsp = a.n_splits[i], sb = a.split_base[i];

    __shared__ float red[4];
    __shared__ float sm_o[SL][DV];
    __shared__ float sm_l[SL];

    float mloc = -INFINITY;
    for (int j = tid; j < nsp; j += 256) mloc = fmaxf(mloc, a.ws_m[(size_t)(sb + j) * bq + rem]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, off));
    if ((tid & 63) == 0) red[tid >> 6] = mloc;
    __syncthreads();
    const float M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));

    const int sl = tid / TPR, c4 = (tid % TPR) * 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float lacc = 0.f;
    if (M != -INFINITY) {
        for (int j = sl; j < nsp; j += SL) {
            const size_t rec = (size_t)(sb + j) * bq + rem;
            const float mj = a.ws_m[rec];
            if (mj == -INFINITY) continue;            // empty record: its O was never written
            const float f = __builtin_amdgcn_exp2f(mj - M);
            lacc += a.ws_l[rec] * f;
            acc += *reinterpret_cast<const f32x4*>(a.ws_o + rec * DV + c4) * f;
        }
    }
    *reinterpret_cast<f32x4*>(&sm_o[sl][c4]) = acc;
    if (c4 == 0) sm_l[sl] = lacc;
    __syncthreads();
    if (tid < TPR) {
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        float L = 0.f;
#pragma unroll
        for (int k = 0; k < SL; k++) { s += *reinterpret_cast<const f32x4*>(&sm_o[k][c4]); L += sm_l[k]; }
        const size_t orow = (size_t)(a.shard0 + i) * bq + rem;
        const float inv = (L > 0.f) ? 1.f / L : 0.f;
        *reinterpret_cast<f32x4*>(a.o_part + orow * DV + c4) = s * inv;
        if (tid == 0) a.lse_part[orow] = (L > 0.f) ? (M + __builtin_log2f(L)) * kLn2 : -INFINITY;
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
            const float w = __expf(li - top);
            wsum += w;
            acc += *reinterpret_cast<const f32x4*>(o_parts + ((int64_t)i * rows + row) * DV + c4) * w;
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

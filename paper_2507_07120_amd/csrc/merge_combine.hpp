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
template <int DV>
__device__ __forceinline__ f32x4 merge_row(const float* __restrict__ ws_o, const float* __restrict__ ws_m,
                                           const float* __restrict__ ws_l, int sb, int nsp, int bq, int rem,
                                           MergeSmem<DV>& sm, float& M, float& L)
{
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
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int j = j0 + u * S::SL;
            mj[u] = -INFINITY;
            lj[u] = 0.f;
            if (j < nsp) {
                const size_t rec = (size_t)(sb + j) * bq + rem;
                mj[u] = ws_m[rec];
                lj[u] = ws_l[rec];
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            oj[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (mj[u] != -INFINITY)                // an empty record's O was never written: not fetched either
                oj[u] = *reinterpret_cast<const f32x4*>(ws_o + ((size_t)(sb + j0 + u * S::SL) * bq + rem) * DV + c4);
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
    const f32x4 o = merge_row<DV>(a.ws_o, a.ws_m, a.ws_l, a.split_base[i], a.n_splits[i], bq, rem, sm, M, L);
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
    const MergeArgs& a = f.m;
    const int tid = threadIdx.x;
    const int rem = blockIdx.x;          // b*Q + h
    const int bq = a.B * a.Q;
    constexpr int TPR = MergeSmem<DV>::TPR;
    if (a.n_shards == 1) {               // the combine of one fragment is the fragment itself, bit for bit
        float M, L;
        const f32x4 o = merge_row<DV>(a.ws_o, a.ws_m, a.ws_l, a.split_base[0], a.n_splits[0], bq, rem, sm, M, L);
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
        const f32x4 o = merge_row<DV>(a.ws_o, a.ws_m, a.ws_l, a.split_base[i], a.n_splits[i], bq, rem, sm, M, L);
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

// Shared device-side types and helpers of the gfx950 decode-attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace helix {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMaxLaunchShards = 16;   // shard descriptors travel by value in the kernel arguments
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// One KV shard as the kernels see it (Sec. 2.1.1: the slice of the cache one KVP rank holds).
struct ShardDev {
    const void* k;
    const void* v;
    const float* kv_scale;
    const int64_t* tok_off;
    const int32_t* len;
    int64_t k_sb, k_sh, k_st;
    int64_t v_sb, v_sh, v_st;
    int64_t s_sb, s_sh;
    int32_t split_base;   // index of this shard's first split among all splits of the call
    int32_t n_splits;     // ceil(max_len / split_tokens)
    int32_t unit_base;    // first workgroup of this shard in the launch
    int32_t kvp_n;        // 0: tok_off / len describe this shard.  N > 0: they describe the WHOLE cache and
    int32_t kvp_i;        //    this descriptor is KVP slice kvp_i of N, cut inside the kernel (shard_range)
    int32_t pad;
    int64_t* out_off;     // kvp_n > 0: where slice kvp_i's offsets / lengths of all sequences are recorded, or NULL
    int32_t* out_len;
    const uint8_t* k_mx;  // MXFP4 only: E8M0 block scales, index = element index / 32
    const uint8_t* v_mx;
    int32_t* status;      // device word the kernels OR status bits into, or NULL
};

constexpr int kStatusLenExceedsMax = 1;   // HELIX_STATUS_LEN_EXCEEDS_MAX
constexpr int kStatusReferenceMoved = 256; // HELIX_STATUS_REFERENCE_MOVED: added once per (wave, tile) in which an MLA kernel moved reference exponents

// The launch holds n_splits runs of split_tokens tokens per sequence (sized from the host's max_len):
// tokens of a longer sequence are not attended to, which the caller can learn from the status word.
// Called by one thread of the workgroup that serves a sequence's first run.
__device__ __forceinline__ void flag_len_overflow(const ShardDev& sh, int len, int split_tokens)
{
    if (sh.status && (int64_t)len > (int64_t)sh.n_splits * split_tokens) atomicOr(sh.status, kStatusLenExceedsMax);
}

// Arguments of an attention launch over up to kMaxLaunchShards shards.
struct AttnArgs {
    const uint16_t* q;    // bf16 [B,Q,dk]
    float* ws_o;          // split records: un-normalised sum_t p_t v_t, [split][B][Q][dv]
    float* ws_m;          // integer power-of-two reference exponent of the record, [split][B][Q]
    float* ws_l;          // sum_t p_t, [split][B][Q]
    int32_t B, Q, K, g;
    int32_t head_tiles;   // ceil(g / heads per workgroup)
    int32_t split_tokens; // tokens of a shard one workgroup streams
    float scale_log2e;    // softmax scale * log2(e)
    int32_t n_shards;
    const uint2* units;   // which (shard << 24 | row, split) each workgroup serves, written by run_order_kernel; NULL: by id
    // MLA launches that are cut evenly over the token stream (stream_plan_kernel): the (shard, sequence) pairs of
    // the launch, pair = shard * B + sequence, laid end to end in 32-token tiles
    const int64_t* tile_prefix;   // [pairs + 1] tiles before pair p; [pairs] = all tiles.  NULL: runs by workgroup id
    const int32_t* wg_first_pair; // [n_wg] the pair that holds a workgroup's first tile
    int32_t n_wg;                 // workgroups of the launch
    int32_t rec_base;             // first record of this launch; the run of workgroup g inside pair p writes record rec_base + g + p
    ShardDev shard[kMaxLaunchShards];
};

constexpr int kStreamTile = 32;   // tokens per tile of the MLA kernels

// First tile of workgroup g when T tiles are dealt evenly to n_wg workgroups: workgroup g serves tiles
// [stream_start(g), stream_start(g + 1)), each range T / n_wg tiles long to within one.
__host__ __device__ __forceinline__ int64_t stream_start(int64_t g, int64_t T, int64_t n_wg) { return g * T / n_wg; }

// The workgroup whose range holds tile x (0 <= x < T): the largest g with stream_start(g) <= x.
__device__ __forceinline__ int stream_owner(int64_t x, int64_t T, int n_wg)
{
    int g = (int)min((int64_t)n_wg - 1, (x * n_wg + n_wg - 1) / T);       // at or just above the answer
    while (g > 0 && stream_start(g, T, n_wg) > x) g--;
    while (g + 1 < n_wg && stream_start(g + 1, T, n_wg) <= x) g++;
    return g;
}

// Tokens of sequence b this shard holds and the row of the first one.  With kvp_n > 0 the contiguous
// KVP cut of Sec. 2.1.1 is made here: slice width c = 16 * ceil(ceil(L / N) / 16) tokens (whole blocks of
// the append granule of Sec. 2.3), slice i = [min(i c, L), min((i+1) c, L)) -- the same integers the
// stand-alone layout kernel produces.
__device__ __forceinline__ void shard_range(const ShardDev& sh, int b, int& len, int64_t& first_row)
{
    const int64_t base = sh.tok_off ? sh.tok_off[b] : 0;
    const int64_t L = sh.len[b];
    if (sh.kvp_n == 0) {
        len = (int)L;
        first_row = base;
        return;
    }
    // 32-bit unsigned arithmetic for the division (L < 2^31, N <= 1024, so L + N - 1 and c fit); only
    // the product i * c needs 64 bits
    const uint32_t n = (uint32_t)sh.kvp_n;
    const uint32_t per = ((uint32_t)L + n - 1u) / n;
    const uint32_t c = ((per + 15u) >> 4) << 4;
    const int64_t lo = min((int64_t)sh.kvp_i * c, L), hi = min((int64_t)(sh.kvp_i + 1) * c, L);
    len = (int)(hi - lo);
    first_row = base + lo;
}

__device__ __forceinline__ uint32_t as_u32(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float as_f32(uint32_t x) { return __builtin_bit_cast(float, x); }

// Two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// 2^(t - m) for an integer-valued m, computed so that the significand of the result depends on t
// only: 2^frac(t) scaled by the exact power 2^(floor(t) - m).  Different running references m
// (another shard split, another tile order) therefore give bit-identical weights up to the
// exponent, which is what keeps sharded and unsharded runs within fp32 summation noise.
__device__ __forceinline__ float exp2_rel(float t, float m)
{
    float fl = __builtin_floorf(t);
    float e = __builtin_amdgcn_exp2f(t - fl);
    return __builtin_ldexpf(e, (int)(fl - m));
}

// 2^(t - m) for an integer m, the fractional and the integer part of t taken by one instruction each
// (v_fract_f32, v_cvt_flr_i32_f32): the same bits as exp2_rel(t, (float)m) in five instructions instead of six
// (for |t| below 2^31 octaves; the conversion saturates beyond).
__device__ __forceinline__ float exp2_rel_int(float t, int m)
{
    int n;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(n) : "v"(t));
    return __builtin_ldexpf(__builtin_amdgcn_exp2f(__builtin_amdgcn_fractf(t)), n - m);
}

__device__ __forceinline__ float wave_xor_max_16_32(float x)
{
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}

__device__ __forceinline__ float wave_xor_sum_16_32(float x)
{
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

// The order in which the workgroups of an attention launch take their runs.  Workgroup ids are dealt
// round-robin to the 8 XCDs (and on to their CUs) for good; an MLA workgroup needs a whole CU whatever it
// finds to do.  With ragged lengths the runs of a launch are full (split_tokens rows), partial (the last
// of a sequence's slice) or empty (the grid is sized for the longest sequence), and with a plain
// id -> (split, row) map the XCDs whose ids happen to hold less work idle at the end (measured: 15 % of
// the ragged MLA configuration).  This kernel (one workgroup) writes the map instead: all full runs
// first -- equal cost, so every XCD gets the same share -- then the partial ones by descending length
// (16 classes), then the empty ones, which only write their empty record.  A row is a (sequence, kv
// head, head tile): row = (b * K + kv head) * head_tiles + head tile.  Entry i: x = shard << 24 | row,
// y = split index.  Which workgroup serves which run has no influence on any result.
constexpr int kOrderThreads = 1024, kOrderClasses = 16;

__global__ __launch_bounds__(kOrderThreads) void run_order_kernel(const AttnArgs a, uint2* units, int n_units)
{
    __shared__ int count[kOrderClasses + 2];              // runs per segment: [0] full, [1 + c] partial of class c, [last] empty
    __shared__ int cursor[kOrderClasses + 2];
    const int tid = threadIdx.x;
    const int rows = a.B * a.K * a.head_tiles;
    const int pairs = a.n_shards * rows;
    if (tid < kOrderClasses + 2) count[tid] = 0;
    __syncthreads();
    // what one (shard, row) pair contributes: nf full runs, one partial run of class cls (or none: -1)
    auto runs_of = [&](int p, int& si, int& row, int& nf, int& cls, int& n) {
        si = p / rows;
        row = p - si * rows;
        const int b = row / (a.K * a.head_tiles);
        const ShardDev& sh = a.shard[si];
        int len;
        int64_t first_row;
        shard_range(sh, b, len, first_row);
        len = max(len, 0);                                // a negative length is an empty sequence, as in the attention kernels
        n = sh.n_splits;
        nf = min(len / a.split_tokens, n);
        const int rem = len - nf * a.split_tokens;
        cls = nf < n && rem > 0 ? kOrderClasses - 1 - min(kOrderClasses - 1, (int)((int64_t)rem * kOrderClasses / a.split_tokens)) : -1;
    };
    // a thread's first pair is looked up once (the usual launch has fewer pairs than threads)
    int si0 = 0, row0 = 0, nf0 = 0, cls0 = -1, n0 = 0;
    if (tid < pairs) runs_of(tid, si0, row0, nf0, cls0, n0);
    for (int p = tid; p < pairs; p += kOrderThreads) {
        int si = si0, row = row0, nf = nf0, cls = cls0, n = n0;
        if (p != tid) runs_of(p, si, row, nf, cls, n);
        if (nf) atomicAdd(&count[0], nf);
        if (cls >= 0) atomicAdd(&count[1 + cls], 1);
        if (n - nf - (cls >= 0)) atomicAdd(&count[kOrderClasses + 1], n - nf - (cls >= 0));
    }
    __syncthreads();
    if (tid == 0) {
        int at = 0;
        for (int j = 0; j < kOrderClasses + 2; j++) { cursor[j] = at; at += count[j]; }
    }
    __syncthreads();
    for (int p = tid; p < pairs; p += kOrderThreads) {
        int si = si0, row = row0, nf = nf0, cls = cls0, n = n0;
        if (p != tid) runs_of(p, si, row, nf, cls, n);
        const uint32_t who = (uint32_t)si << 24 | (uint32_t)row;
        int s = 0;
        if (nf) {
            const int at = atomicAdd(&cursor[0], nf);
            for (; s < nf; s++) if (at + s < n_units) units[at + s] = uint2{who, (uint32_t)s};
        }
        if (cls >= 0) {
            const int at = atomicAdd(&cursor[1 + cls], 1);
            if (at < n_units) units[at] = uint2{who, (uint32_t)s};
            s++;
        }
        if (s < n) {
            const int at = atomicAdd(&cursor[kOrderClasses + 1], n - s) - s;
            for (; s < n; s++) if (at + s < n_units) units[at + s] = uint2{who, (uint32_t)s};
        }
    }
}

// Plan of an MLA launch whose workgroups share the work evenly whatever the sequence lengths are.  The slices
// of all (shard, sequence) pairs of the launch are laid end to end, counted in 32-token tiles, and workgroup g
// of n_wg takes the tiles [g T / n_wg, (g + 1) T / n_wg): a run of equal length for every workgroup, cut into
// pieces only where it crosses from one pair into the next.  Every piece ends in one split record, so a pair
// has one record per workgroup that touches it -- about T / n_wg tokens apart -- instead of one per fixed-size
// run, and no workgroup is launched for tokens that do not exist.  This kernel (one workgroup) writes what the
// attention and merge kernels need: the exclusive prefix of the pairs' tile counts, per workgroup the pair that
// holds its first tile, and per pair the workgroups that hold its tiles; it also records the KVP cut (out_off /
// out_len) of every pair, empty ones included.
constexpr int kPlanThreads = 1024;

__global__ __launch_bounds__(kPlanThreads) void stream_plan_kernel(const AttnArgs a, int64_t* tile_prefix, int32_t* wg_first_pair, int2* pair_rec)
{
    __shared__ int64_t part[kPlanThreads];
    const int tid = threadIdx.x;
    const int pairs = a.n_shards * a.B;
    const int chunk = (pairs + kPlanThreads - 1) / kPlanThreads;          // consecutive pairs per thread
    const int p0 = min(tid * chunk, pairs), p1 = min(p0 + chunk, pairs);
    auto tiles_of = [&](int p) {
        const int si = p / a.B, b = p - si * a.B;
        const ShardDev& sh = a.shard[si];
        int len;
        int64_t first_row;
        shard_range(sh, b, len, first_row);
        if (sh.out_off) { sh.out_off[b] = first_row; sh.out_len[b] = len; }
        return (int64_t)((max(len, 0) + kStreamTile - 1) / kStreamTile);   // a negative length is an empty sequence
    };
    int64_t mine = 0;
    for (int p = p0; p < p1; p++) mine += tiles_of(p);
    part[tid] = mine;
    __syncthreads();
    // exclusive scan of the per-thread sums (Hillis-Steele over 1024 entries)
    for (int off = 1; off < kPlanThreads; off <<= 1) {
        const int64_t add = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    int64_t run = part[tid] - mine;
    const int64_t T = part[kPlanThreads - 1];
    for (int p = p0; p < p1; p++) {
        tile_prefix[p] = run;
        const int si = p / a.B, b = p - si * a.B;
        int len;
        int64_t first_row;
        shard_range(a.shard[si], b, len, first_row);
        run += (int64_t)((max(len, 0) + kStreamTile - 1) / kStreamTile);
    }
    if (tid == 0) tile_prefix[pairs] = T;
    __threadfence_block();
    __syncthreads();                                   // the prefix is complete and visible to the whole workgroup
    for (int g = tid; g < a.n_wg; g += kPlanThreads) {
        int first = 0;
        if (T > 0) {
            const int64_t s = stream_start(g, T, a.n_wg);
            // the largest pair p with tile_prefix[p] <= s (it is not empty: the next pair starts beyond s)
            int lo = 0, hi = pairs - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (tile_prefix[mid] <= s) lo = mid; else hi = mid - 1;
            }
            first = lo;
        }
        wg_first_pair[g] = first;
    }
    // for the merge: the workgroups that hold tiles of pair p are g_first .. g_first + n - 1 (x, y); y is stored
    // negated when the launch has fewer tiles than workgroups, because then some of them hold no tile at all
    for (int p = tid; p < pairs; p += kPlanThreads) {
        const int64_t lo = tile_prefix[p], hi = tile_prefix[p + 1];
        int2 r = {0, 0};
        if (hi > lo) {
            r.x = stream_owner(lo, T, a.n_wg);
            r.y = stream_owner(hi - 1, T, a.n_wg) - r.x + 1;
            if (T < a.n_wg) r.y = -r.y;
        }
        pair_rec[p] = r;
    }
}

}  // namespace helix

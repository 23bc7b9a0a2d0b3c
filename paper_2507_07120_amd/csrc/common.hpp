// Shared device-side types and helpers of the gfx950 decode-attention kernels.
#pragma once
#include "seat.hpp"
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
    // split records: un-normalised sum_t p_t v_t (ws_o, rows of dv), the integer power-of-two reference exponent of
    // the row (ws_m) and sum_t p_t (ws_l).  Rows of an evenly cut launch: [record][16 heads] (GQA), [record][Q] (MLA),
    // record = rec_base + workgroup + row (GQA) / pair (MLA) index; of a launch cut by workgroup id: [split][B][Q]
    float* ws_o;
    float* ws_m;
    float* ws_l;
    int32_t B, Q, K, g;
    int32_t head_tiles;   // ceil(g / heads per workgroup)
    int32_t split_tokens; // launches cut by workgroup id: tokens of a shard one workgroup serves
    float scale_log2e;    // softmax scale * log2(e)
    int32_t n_shards;
    // streaming GQA launches (every workgroup plans its own share, stream_self_plan): what the merge needs later
    int64_t* prefix_out;  // [pairs + 1] row tiles of one head tile before pair p, written by workgroup 0
    int2* row_rec;        // [rows] first and last seat (StreamSeat::seat) that hold tiles of a row, written by those workgroups
    // MLA launches that are cut evenly over the token stream (stream_plan_kernel): the (shard, sequence) pairs of
    // the launch, pair = shard * B + sequence, laid end to end in 32-token tiles
    const int64_t* tile_prefix;   // [pairs + 1] tiles before pair p; [pairs] = all tiles.  NULL: runs by workgroup id
    const int32_t* wg_first_pair; // [n_wg] the pair that holds a workgroup's first tile
    int32_t n_wg;                 // workgroups of the launch
    int32_t n_base;               // streaming GQA launches: workgroups per head tile (n_wg / head_tiles, see StreamSeat)
    int32_t rec_base;             // first record of this launch; the run of workgroup g inside pair p writes record rec_base + g + p
    ShardDev shard[kMaxLaunchShards];
};

constexpr int kStreamTile = 32;   // tokens per tile of the MLA kernels

// T tiles dealt evenly to n_wg workgroups: the first T % n_wg workgroups serve T / n_wg + 1 consecutive tiles, the
// others T / n_wg.  With fewer tiles than workgroups the first T workgroups get one tile each, so the workgroups
// without a tile all sit at the end (the workgroups that hold tiles of one row are always consecutive).
struct StreamDeal {
    int64_t q, r;
    // first tile of workgroup g (0 <= g <= n_wg)
    __host__ __device__ __forceinline__ int64_t start(int64_t g) const { return g * q + (g < r ? g : r); }
    // the workgroup that serves tile x (0 <= x < T)
    __host__ __device__ __forceinline__ int owner(int64_t x) const
    {
        const int64_t head = r * (q + 1);                  // tiles of the workgroups with one tile more
        return x < head ? (int)(x / (q + 1)) : (int)(r + (x - head) / q);
    }
};

__host__ __device__ __forceinline__ StreamDeal stream_deal(int64_t T, int n_wg)
{
    StreamDeal d;
    if (__builtin_expect((uint64_t)T >> 32 != 0, 0)) {
        d.q = T / n_wg;
        d.r = T % n_wg;
    } else {                                               // (the usual sizes: a 32-bit division costs a fraction of the 64-bit one)
        const uint32_t q = (uint32_t)T / (uint32_t)n_wg;
        d.q = q;
        d.r = (uint32_t)T - q * (uint32_t)n_wg;
    }
    return d;
}

// Tokens of sequence b this shard holds and the row of the first one.  With kvp_n > 0 the contiguous
// KVP cut of Sec. 2.1.1 is made here: slice width c = 16 * ceil(ceil(L / N) / 16) tokens (whole blocks of
// the append granule of Sec. 2.3), slice i = [min(i c, L), min((i+1) c, L)) -- the same integers the
// stand-alone layout kernel produces.
__device__ __forceinline__ void shard_range_of(int64_t L, int64_t base, int kvp_n, int kvp_i, int& len, int64_t& first_row)
{
    if (kvp_n == 0) {
        len = (int)L;
        first_row = base;
        return;
    }
    // 32-bit unsigned arithmetic for the division (L < 2^31, N <= 1024, so L + N - 1 and c fit); only
    // the product i * c needs 64 bits
    const uint32_t n = (uint32_t)kvp_n;
    const uint32_t per = ((uint32_t)L + n - 1u) / n;
    const uint32_t c = ((per + 15u) >> 4) << 4;
    const int64_t lo = min((int64_t)kvp_i * c, L), hi = min((int64_t)(kvp_i + 1) * c, L);
    len = (int)(hi - lo);
    first_row = base + lo;
}

__device__ __forceinline__ void shard_range(const ShardDev& sh, int b, int& len, int64_t& first_row)
{
    const int64_t base = sh.tok_off ? sh.tok_off[b] : 0;
    shard_range_of(sh.len[b], base, sh.kvp_n, sh.kvp_i, len, first_row);
}

// A load of the K/V stream.  NT: non-temporal -- every byte is used once (measured on MI355X: plain loads of a 1 GiB
// stream top out near 6.2 TB/s, non-temporal ones reach 7.0 TB/s).  Launches whose head tiles share their reads
// through the L2 (StreamSeat) load the ordinary way.
template <bool NT, class T>
__device__ __forceinline__ T stream_load(const T* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait for the wave's global
// loads and stores (a record's stores take a microsecond or two to be acknowledged).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
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

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (no shared memory): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add 0), then the last lane of rows 0 and 2 is
// added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x)
{
    constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowShr + 1, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowShr + 2, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowShr + 4, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowShr + 8, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowBcast15, 0xa, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kRowBcast31, 0xc, 0xf, false);
    return x;
}

// Where a workgroup of a streaming GQA launch sits.  A kv head with more than 16 query heads has several head
// tiles, and every one of them needs the kv head's keys and values: the launch then consists of head_tiles equal
// sets of n_base workgroups, set t serving head tile t of every row, all sets cut in exactly the same way -- so the
// head_tiles workgroups with the same index `wg` inside their sets read the same tokens at the same time.  With
// n_base a multiple of 8 their workgroup ids are 8 apart, which puts them on the same XCD (consecutive ids go round
// robin over the 8 XCDs): one of them fetches a key from HBM, the others find it in that XCD's L2 (these launches
// use ordinary loads, not non-temporal ones).  seat = ht * n_base + wg numbers the workgroups in the order their
// rows have in the record arrays.
struct StreamSeat {
    int wg, n_wg;            // index inside the set, workgroups of a set
    int ht, seat;
};

__device__ __forceinline__ StreamSeat stream_seat(const AttnArgs& a)
{
    StreamSeat s;
    s.wg = (int)blockIdx.x;
    s.n_wg = a.n_wg;
    s.ht = 0;
    if (a.head_tiles > 1) {
        const SeatOf at = seat_of((int)blockIdx.x, a.head_tiles, a.n_base);
        s.n_wg = a.n_base;
        s.ht = at.ht;
        s.wg = at.wg;
    }
    s.seat = s.ht * s.n_wg + s.wg;
    return s;
}

// The same even cut, planned by every workgroup for itself (the streaming GQA kernels: a planning launch of its
// own would cost them 5 % of a step).  The rows of one head tile -- (shard, sequence, kv head), rows_per_pair of
// them per (shard, sequence) pair, all as long as the pair's slice -- are laid end to end in tiles of tile_tokens
// tokens, and workgroup g of the n_wg that serve the head tile (StreamSeat) takes the row tiles
// [g T / n_wg, (g + 1) T / n_wg).  Every workgroup reads all
// lengths (one or a few per thread, in parallel: the one dependent memory round trip a workgroup needs anyway
// before it knows where its keys are), scans them, and finds the pair that holds its first tile.  All results
// are the same in every lane.
struct StreamCursor {
    int64_t cur, end;        // row tiles still to serve: [cur, end)
    int32_t pair;            // the pair that holds tile `cur` ...
    int64_t pair_lo;         // ... its first row tile
    int64_t pair_tiles;      // ... the tiles of one of its rows
    int64_t first_row;       // ... the row of its slice's first token in the cache
    int32_t len;             // ... and the slice's length in tokens
    int32_t ht, seat;        // the workgroup's head tile and seat (StreamSeat)
    int32_t row0;            // index of the head tile's first row among the launch's rows
};

__device__ __forceinline__ int64_t uniform_i64(int64_t x)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)x >> 32));
    return (int64_t)((uint64_t)hi << 32 | lo);
}

// THREADS = threads of the workgroup (a multiple of 64, at most 1024); scratch: THREADS / 64 + 5 int64 in LDS.
// prefix_out (may be NULL): workgroup 0 stores the exclusive prefix of the pairs' row tiles there, [pairs + 1], for
// the merge kernel; it also records the KVP cut of every pair (out_off / out_len of the shards).
// Returns false if this workgroup has no tile to serve.
template <int THREADS>
__device__ __forceinline__ bool stream_self_plan(const AttnArgs& a, int tile_tokens, int rows_per_pair, int64_t* scratch,
                                                 int64_t* prefix_out, StreamCursor& c)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pairs = a.n_shards * a.B;
    const StreamSeat seat = stream_seat(a);
    c.ht = seat.ht;
    c.seat = seat.seat;
    c.row0 = seat.ht * pairs * rows_per_pair;
    if (__builtin_expect(pairs <= 64, 1)) {
        // The usual case: every wave plans for itself, lane p looking at pair p -- no shared memory, no barrier.
        // The loops run over uniform indices, so that the shards' pointers come from scalar loads of the kernel
        // arguments and the lengths are the only vector loads on the way.
        // (lanes beyond the last pair look at the last pair too, so that no load sits under a condition; their
        // tile count is zeroed below)
        const int pl = min(lane, pairs - 1);
        const int32_t* len_at = nullptr;
        const int64_t* off_at = nullptr;
        int kvp_n = 0, kvp_i = 0;
        for (int si = 0; si < a.n_shards; si++) {
            const ShardDev& sh = a.shard[si];
            const int b = pl - si * a.B;
            if (b >= 0 && b < a.B) {
                len_at = sh.len + b;
                off_at = sh.tok_off ? sh.tok_off + b : nullptr;
                kvp_n = sh.kvp_n;
                kvp_i = sh.kvp_i;
            }
        }
        const int64_t L = *len_at;                                                  // both loads in flight together
        const int64_t base = __builtin_expect(off_at != nullptr, 1) ? *off_at : 0;
        int len;
        int64_t first_row;
        shard_range_of(L, base, kvp_n, kvp_i, len, first_row);
        const uint32_t t = lane < pairs ? (uint32_t)((max(len, 0) + tile_tokens - 1) / tile_tokens) : 0u;
        // inclusive sum of the pairs' tile counts over the lanes (at most 64 x 2^24: 32 bits), then times the rows
        const uint32_t t_incl = wave_inclusive_sum(t);
        const int64_t T = (int64_t)__builtin_amdgcn_readlane(t_incl, 63) * rows_per_pair;
        const int64_t excl = (int64_t)(t_incl - t) * rows_per_pair;
        const int64_t mine = (int64_t)t * rows_per_pair;
        if (__builtin_expect(blockIdx.x == 0 && wave == 0, 0)) {
            if (prefix_out && lane < pairs) {
                prefix_out[lane] = excl;
                if (lane == pairs - 1) prefix_out[pairs] = T;
            }
            for (int si = 0; si < a.n_shards; si++) {                    // the KVP cut, empty slices included
                const ShardDev& sh = a.shard[si];
                const int b = lane - si * a.B;
                if (sh.out_off && b >= 0 && b < a.B) { sh.out_off[b] = first_row; sh.out_len[b] = len; }
            }
        }
        const StreamDeal deal = stream_deal(T, seat.n_wg);
        c.cur = deal.start(seat.wg);
        c.end = deal.start(seat.wg + 1);
        if (c.cur >= c.end) return false;
        // exactly one lane's pair holds tile `cur` (0 <= cur < T)
        const uint64_t holds = __ballot(lane < pairs && mine > 0 && excl <= c.cur && c.cur < excl + mine);
        const int src = __builtin_ctzll(holds | (1ull << 63));
        auto from = [&](uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane(v, src); };
        c.pair = src;
        c.pair_lo = (int64_t)((uint64_t)from((uint32_t)((uint64_t)excl >> 32)) << 32 | from((uint32_t)excl));
        c.pair_tiles = from(t);
        c.first_row = (int64_t)((uint64_t)from((uint32_t)((uint64_t)first_row >> 32)) << 32 | from((uint32_t)first_row));
        c.len = (int32_t)from((uint32_t)len);
        return true;
    }
    const int chunk = (pairs + THREADS - 1) / THREADS;                 // consecutive pairs per thread
    const int p0 = min(tid * chunk, pairs), p1 = min(p0 + chunk, pairs);
    // length and first row of a pair, tiles of one of its rows
    auto look = [&](int p, int& len, int64_t& first_row) {
        const int si = p / a.B, b = p - si * a.B;
        shard_range(a.shard[si], b, len, first_row);
        return (int64_t)((max(len, 0) + tile_tokens - 1) / tile_tokens);
    };
    int64_t mine = 0;
    int len0 = 0;                                                      // the thread's first pair (its only one, as a rule)
    int64_t row0 = 0, tiles0 = 0;
    for (int p = p0; p < p1; p++) {
        int len;
        int64_t first_row;
        const int64_t t = look(p, len, first_row);
        if (p == p0) { len0 = len; row0 = first_row; tiles0 = t; }
        mine += t * rows_per_pair;
    }
    // inclusive scan inside the wave, then over the waves' totals
    int64_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t lo = __shfl_up((uint32_t)incl, off), hi = __shfl_up((uint32_t)((uint64_t)incl >> 32), off);
        if (lane >= off) incl += (int64_t)((uint64_t)hi << 32 | lo);
    }
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    int64_t before = 0, T = 0;
#pragma unroll
    for (int w = 0; w < THREADS / 64; w++) {
        const int64_t tw = scratch[w];
        if (w < wave) before += tw;
        T += tw;
    }
    T = uniform_i64(T);
    const int64_t excl = before + incl - mine;                         // row tiles before this thread's first pair
    if (blockIdx.x == 0) {
        int64_t run = excl;
        for (int p = p0; p < p1; p++) {
            if (prefix_out) prefix_out[p] = run;
            int len = len0;
            int64_t first_row = row0, t = tiles0;
            if (p != p0) t = look(p, len, first_row);
            const ShardDev& sh = a.shard[p / a.B];
            if (sh.out_off) { sh.out_off[p % a.B] = first_row; sh.out_len[p % a.B] = len; }     // the KVP cut, empty slices included
            run += t * rows_per_pair;
        }
        if (tid == 0 && prefix_out) prefix_out[pairs] = T;
    }
    const StreamDeal deal = stream_deal(T, seat.n_wg);
    c.cur = deal.start(seat.wg);
    c.end = deal.start(seat.wg + 1);
    if (c.cur >= c.end) return false;
    // the thread whose pairs hold tile `cur` tells the others which pair it is, where its rows start and how long they are
    int64_t* found = scratch + THREADS / 64;
    if (mine > 0 && excl <= c.cur && c.cur < excl + mine) {
        int64_t run = excl;
        for (int p = p0; p < p1; p++) {
            int len = len0;
            int64_t first_row = row0, t = tiles0;
            if (p != p0) t = look(p, len, first_row);
            if (c.cur < run + t * rows_per_pair) {
                found[0] = p;
                found[1] = run;
                found[2] = t;
                found[3] = first_row;
                found[4] = len;
                break;
            }
            run += t * rows_per_pair;
        }
    }
    __syncthreads();
    c.pair = (int32_t)uniform_i64(found[0]);
    c.pair_lo = uniform_i64(found[1]);
    c.pair_tiles = uniform_i64(found[2]);
    c.first_row = uniform_i64(found[3]);
    c.len = (int32_t)uniform_i64(found[4]);
    return true;
}

// One run of a streaming workgroup: tokens [t0, t1_cap) of row (shard si, sequence b, kv head kh, head tile ht).
struct StreamRun {
    int si, b, kh, ht;
    int t0, t1_cap;          // t1_cap may lie beyond the slice's end (whole tiles)
    int slot;                // record slot of the run: seat + row index
    int row;                 // row index within the launch: (head tile, pair, kv head)
    int seat;                // the workgroup's seat
    bool first, last;        // the run holds the row's first / last tile
};

// Takes the next run off the cursor; false when the workgroup's range is used up.  Uniform in all lanes.
__device__ __forceinline__ bool stream_next_run(const AttnArgs& a, StreamCursor& c, int tile_tokens, int rows_per_pair, StreamRun& r)
{
    for (;;) {
        if (c.cur >= c.end) return false;
        const int64_t pair_hi = c.pair_lo + c.pair_tiles * rows_per_pair;
        if (c.cur < pair_hi) break;
        c.pair++;                                                       // the next pair (one without tokens is skipped)
        c.pair_lo = pair_hi;
        const int si = c.pair / a.B;
        int len;
        int64_t first_row;
        shard_range(a.shard[si], c.pair - si * a.B, len, first_row);
        c.len = __builtin_amdgcn_readfirstlane(len);
        c.first_row = uniform_i64(first_row);
        c.pair_tiles = (int64_t)((max(c.len, 0) + tile_tokens - 1) / tile_tokens);
    }
    // row within the pair = kv head (this sits on the way to a workgroup's first load: divisions only where they
    // are needed, and in 32 bits where the numbers allow)
    const int64_t into = c.cur - c.pair_lo;
    int rr = 0;
    if (into >= c.pair_tiles) rr = __builtin_expect((into | c.pair_tiles) >> 31 != 0, 0) ? (int)(into / c.pair_tiles) : (int)((uint32_t)into / (uint32_t)c.pair_tiles);
    const int64_t row_lo = c.pair_lo + (int64_t)rr * c.pair_tiles;
    const int64_t seg_end = min(c.end, row_lo + c.pair_tiles);
    r.si = a.n_shards == 1 ? 0 : c.pair / a.B;
    r.b = c.pair - r.si * a.B;
    r.kh = rr;
    r.ht = c.ht;
    r.t0 = (int)(c.cur - row_lo) * tile_tokens;
    r.t1_cap = (int)(seg_end - row_lo) * tile_tokens;
    r.row = c.row0 + c.pair * rows_per_pair + rr;
    r.seat = c.seat;
    r.slot = a.rec_base + c.seat + r.row;
    r.first = c.cur == row_lo;
    r.last = seg_end == row_lo + c.pair_tiles;
    c.cur = seg_end;
    return true;
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
    const StreamDeal deal = stream_deal(T, a.n_wg);
    for (int g = tid; g < a.n_wg; g += kPlanThreads) {
        int first = 0;
        if (T > 0) {
            const int64_t s = deal.start(g);
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
    // for the merge: the workgroups that hold tiles of pair p are g_first .. g_first + n - 1 (x, y)
    for (int p = tid; p < pairs; p += kPlanThreads) {
        const int64_t lo = tile_prefix[p], hi = tile_prefix[p + 1];
        int2 r = {0, 0};
        if (hi > lo) {
            r.x = deal.owner(lo);
            r.y = deal.owner(hi - 1) - r.x + 1;
        }
        pair_rec[p] = r;
    }
}

}  // namespace helix

// Split-KV decode attention for the MLA case on gfx950: 128 query heads attending ONE shared latent
// whose 576-wide row is the key and whose first 512 entries are the value (Sec. 1, Sec. 3: MLA keeps
// one latent for K and V that all query heads share), per-shard attention of Helix's attention
// phase (Sec. 2.1.1).  Latent stored as bf16, or as e4m3 codes with one fp32 scale per token.
//
// This is the dense contraction of the path (242 flop per latent byte in bf16, 480 in e4m3): it is
// MFMA-bound, so the design question is how to feed the matrix cores, not HBM.
//
// What was measured on MI355X and shaped the kernel:
//   * one wavefront per SIMD issues a 16x16x32 bf16 MFMA only every ~21 cycles; two per SIMD reach
//     the 16-cycle rate -> 8 wavefronts per CU, at most 256 registers each;
//   * a wavefront draws at most ~36 B/clk from LDS (a 1 KB operand read every ~28 cycles), all eight
//     together ~210-245 B/clk, and only if the 16 rows x 64 B of an MFMA operand hit distinct banks:
//     at the natural row stride of 1152 bytes they run 4-way conflicted; XOR-ing the 16-byte chunk
//     index with (row & 7) removes the conflicts without padding.  The transposing read
//     (ds_read_b64_tr_b16) is as fast per byte as the 128-bit read and hands out the value-column-
//     major operand straight from the row-major latent tile;
//   * every operand byte a wave reads is used by ONE score MFMA but by 2 x (head tiles) P.V MFMAs,
//     so the P.V side is where sharing a wave's reads across more heads pays;
//   * global_load_lds_dwordx4 copies 16 bytes per lane from global memory into LDS without touching
//     registers.  When the compiler knows about an LDS DMA in flight it drains it (vmcnt(0)) before
//     the next transposing LDS read, and a spilled register is reloaded by a vector memory load
//     that waits behind every DMA in flight: the DMA is issued from inline assembly and waited for
//     explicitly, and the tile loop must not spill;
//   * the time of this kernel depends on the DATA (all-zero latents run 30 % faster than random
//     ones at the same instruction stream): the part lowers its clock under the switching power of
//     the matrix cores and LDS, so executed MFMAs and LDS bytes per useful flop are what counts.
//
// Workgroup = 8 wavefronts = one CU, HPW = 128 heads (all heads of the usual MLA configuration: the
// latent is read from HBM and copied into LDS once).  A launch with one head tile is cut evenly over its
// token stream (stream_plan_kernel in common.hpp): every workgroup serves one equally long range of the
// launch's (shard, sequence) pairs laid end to end -- a run per pair it touches, a split record per run.
// A run goes through its latent rows in tiles of 32 tokens kept in a ring of three LDS slots (in use, next,
// in flight).  Per tile:
//   S phase  scores S^T[token, head] = K . Q^T: wave w owns heads 16w..16w+15 and both token halves
//            (two independent MFMA chains); its Q slice (16 x 576 bf16 = 72 registers) never moves,
//            the K operands come from LDS.  Softmax stays inside the wave, with an integer reference
//            exponent per head that stays put from tile to tile (bf16: 32 octaves above the largest score
//            seen when it was set): no rescale of accumulators, no cross-lane maximum in the common tile.
//            A tile in which a score comes within reach of the number range's end moves that head's
//            reference -- an exact power-of-two rescale of its normaliser at once and of its accumulators in
//            the P phase, behind a wave-uniform branch (never on ordinary logits; a test forces it).
//            The lane's 8 weights go to LDS as bf16 hi + lo, already in the P.V operand's layout (a head's row is
//            64 bytes: its four 16-byte slots are XOR-ed with (head >> 1) & 3, so that the eight lanes an LDS
//            access serves per cycle fall on distinct banks).
//   barrier
//   P phase  O^T[dv, head] += V^T . P^T: waves 2p and 2p+1 share heads 32p..32p+31 and split the value
//            columns (256 each: 16 column tiles x 2 head tiles = 128 accumulator registers); the
//            weights of the pair's 32 heads are held in registers, every V^T operand read feeds four
//            MFMAs.  The DMA requests for the tile two ahead are spread between the MFMAs.
//   barrier
// Each wave copies 4 rows of every tile and awaits only its own share before the barrier that
// publishes it.
//
// e4m3 latent: the raw codes are DMA-ed into a per-wave staging area and widened to fp16 (exact) by
// the wave that requested them when the tile is due, and both contractions run on the fp16 MFMA (same
// rate as bf16, 11 significant bits): the query rows are scaled into fp16 range by a power of two, and
// ONE fp16 weight w_t = p_t * f_t per token replaces the bf16 hi/lo pair -- half the P.V MFMAs.
// The per-token scale f_t multiplies the score (s_t = f_t * q.k8_t) and the weight; the normaliser sums
// the unrounded p_t in fp32.  fp16's range is narrow: a head's reference puts its largest first-tile weight
// into [2^4, 2^5], and a tile in which a weight reaches 2^14 moves the reference so that this weight lands
// there again.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace helix {

struct MlaCfg {
    static constexpr int DK = 576, DV = 512;
    static constexpr int T = 32;                  // tokens per tile
    static constexpr int ROW = 1152;              // LDS bytes per latent row; chunk c of row r sits at chunk c ^ (r & 7)
    static constexpr int KS = DK / 32;            // 18 k-steps of the score MFMA
    static constexpr int NBUF = 3;                // latent tiles in LDS: in use, next, in flight
    static constexpr int TILE_BYTES = T * ROW;    // 36864
    static constexpr int WAVES = 8;
    static constexpr int HPW = 16 * WAVES;        // heads per workgroup: every wave scores 16 heads
    static constexpr int THREADS = WAVES * 64;
    static constexpr int NHT = 2;                 // head tiles of a wave pair
    static constexpr int DVT = DV / 16 / 2;       // value-column tiles per wave (16): a pair splits the columns
    static constexpr int P_BYTES = NHT * 16 * T * 2;   // one of hi / lo of one pair: [32 heads][32 weights] bf16
    static constexpr int AHEAD = 2;               // tiles between a tile's request and its first use
    // LDS map
    static constexpr int OFF_K = 0;
    static constexpr int OFF_P = NBUF * TILE_BYTES;               // [pair][hi, lo]
    static constexpr int OFF_FLAG = OFF_P + (WAVES / 2) * 2 * P_BYTES;   // + 4: largest query magnitude of the workgroup (fp16 set-up)
    static constexpr int OFF_SCALE = OFF_FLAG + 16;               // [NBUF][32] fp32 per-token scales
    static constexpr int OFF_DMA = OFF_SCALE + NBUF * T * 4;      // [THREADS][8] u32: per-lane source offsets of the tile DMA (5 used)
    static constexpr int OFF_STAGE = OFF_DMA + THREADS * 32;      // [WAVES][4 rows][576] e4m3 codes on their way in
    static constexpr int OFF_RESC = OFF_STAGE + T * DK;           // [WAVES] int: tile (index + 1) in which a wave last moved references; [HPW] fp32 factors
    static constexpr int LDS_BYTES = OFF_RESC + WAVES * 4 + HPW * 4;
    // bf16 latent: a head's reference sits kHeadroom octaves above the largest score seen when it was set and moves
    // when a score comes within 127 - kLimit octaves of fp32's largest power of two (weights and accumulators are fp32-ranged)
    static constexpr float kHeadroom = 32.f, kLimit = 64.f;
    // fp16 weights (e4m3 / MXFP4 latents): a head's reference moves when a weight reaches kWeightLimit, so that the
    // tile's largest weight of that head lands in [2^(kWeightLand-1), 2^kWeightLand]
    static constexpr float kWeightLimit = 16384.f, kWeightLand = 5.f;
};
static_assert(MlaCfg::LDS_BYTES <= 160 * 1024, "LDS budget of a gfx950 CU");

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// The 16x16x32 MFMA on 16-bit operands handed over as raw bits: fp16 for the e4m3 latent (whose tile in
// LDS is widened to fp16), bf16 otherwise.  Same operand and result layout for both.
template <bool F16>
__device__ __forceinline__ f32x4 mla_mfma(const u32x4& a, const u32x4& b, const f32x4& c)
{
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Two fp32 -> packed fp16 pair, round to nearest even (one v_cvt_pk_f16_f32).
__device__ __forceinline__ uint32_t pack_f16_rne(float lo, float hi)
{
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

typedef __attribute__((address_space(3))) uint8_t lds_byte;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) int lds_i32;

// Transposing LDS read: within each group of 16 lanes, lane i receives the 16-bit element (i % 4) of
// the 8-byte rows supplied by lanes 4e + i/4, e = 0..3 (checked on the device).
__device__ __forceinline__ u32x2 lds_read_tr16(const lds_byte* p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    return __builtin_bit_cast(u32x2, v);
}

// The lane id behind a compiler barrier.  Per-lane LDS addresses derived from it are recomputed where
// they are used (a handful of VALU instructions per phase) instead of being hoisted out of the tile
// loop, where a dozen of them would sit in registers the kernel does not have.
__device__ __forceinline__ int mla_opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// Byte offset of (row, 16-byte chunk c) inside an LDS tile.
__device__ __forceinline__ int mla_swz(int row, int c) { return row * MlaCfg::ROW + ((c ^ (row & 7)) << 4); }

// (the workgroup barrier that orders LDS traffic only and leaves global loads and LDS DMA in flight)
__device__ __forceinline__ void mla_barrier() { lds_barrier(); }

// Waits until at most N of this wave's vector memory loads (LDS DMA included) are outstanding.
template <int N>
__device__ __forceinline__ void mla_wait_vm()
{
    static_assert(N >= 0 && N < 16, "low four bits of the counter field");
    __builtin_amdgcn_s_waitcnt(0x0F70 | N);
}

// Workgroups of one shard are numbered so that the head tiles of the same token range are 8 apart:
// consecutive workgroup ids go round-robin over the 8 XCDs, so ids that differ by 8 share an XCD
// and with it an L2.  Shards are padded to a multiple of 8 token ranges (padding workgroups exit).
__host__ __device__ inline int mla_units_of_shard(int n_splits, int B, int head_tiles)
{
    return (n_splits * B + 7) / 8 * 8 * head_tiles;
}

// bf16 latent tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l of a
// wave instruction deposits its 16 bytes at M0 + 16*l; inactive lanes write nothing -- checked on
// the device).  Wave w copies rows 4w..4w+3 of every tile: 288 sixteen-byte chunks = 4.5 wave
// instructions (the fifth with 32 lanes).  LDS position (row, cpos) receives the global chunk
// cpos ^ (row & 7) of that row (72 chunks per row is a multiple of 8, so the XOR stays inside it).
// The instruction is written as inline assembly so that the compiler does not track it: a tracked
// LDS DMA makes it drain the counter before unrelated LDS reads.  Waiting is explicit (mla_wait_vm);
// M0 is otherwise unused in this kernel.
struct MlaDma {
    static constexpr int ROWS = MlaCfg::T / MlaCfg::WAVES;                  // 4
    static constexpr int CHUNKS = ROWS * (MlaCfg::ROW / 16);                // 288
    static constexpr int INSTRS = (CHUNKS + 63) / 64;                       // 5 per wave and tile
    static constexpr int SHARE_BYTES = ROWS * MlaCfg::ROW;                  // 4608
    static_assert(INSTRS == 5, "size of the offset table");

    // Row within the tile of chunk q (< 320) of wave `wave`: q / 72 by multiplication.
    static __device__ __forceinline__ int row_of(int wave, int q) { return wave * ROWS + ((q * 911) >> 16); }

    // The source offset of a lane's chunk within a tile depends on the lane and the part only.  The
    // five offsets live in an LDS table (32 bytes per thread) and are fetched at the start of every
    // phase that issues DMA: held across the tile loop they would be five registers the kernel does
    // not have, and a spilled offset is reloaded with a vector memory load that waits behind every
    // DMA in flight.
    struct Offsets { u32x4 a; uint32_t b; };
    static __device__ __forceinline__ void init(lds_byte* table, uint32_t row_bytes, int wave, int lane, int tid)
    {
        uint32_t o[INSTRS];
#pragma unroll
        for (int j = 0; j < INSTRS; j++) {
            const int q = j * 64 + lane, row = min(row_of(wave, q), wave * ROWS + ROWS - 1), cpos = q % 72;
            o[j] = (uint32_t)row * row_bytes + (uint32_t)((cpos ^ (row & 7)) << 4);
        }
        *reinterpret_cast<lds_u32x4*>(table + tid * 32) = u32x4{o[0], o[1], o[2], o[3]};
        *reinterpret_cast<__attribute__((address_space(3))) uint32_t*>(table + tid * 32 + 16) = o[4];
    }
    static __device__ __forceinline__ Offsets fetch(const lds_byte* table, int tid)
    {
        Offsets f;
        tid = mla_opaque(tid);
        f.a = *reinterpret_cast<const lds_u32x4*>(table + tid * 32);
        f.b = *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(table + tid * 32 + 16);
        return f;
    }

    // Requests part j (one wave instruction, j < INSTRS) of this wave's rows of the tile at `src`
    // (n_valid rows); `dst` = LDS byte address of the wave's share of the slot.  `src`, `dst`,
    // `wave` are uniform.
    static __device__ __forceinline__ void issue_part(int j, const Offsets& f, const char* src, int n_valid, uint32_t dst, int wave, int lane)
    {
        const uint32_t off = j < 4 ? f.a[j] : f.b;
        bool live = j * 64 + 63 < CHUNKS || lane < CHUNKS - j * 64;
        if (n_valid != MlaCfg::T) {                       // ragged last tile of a run (rare): per-lane row test
            int l = lane;
            asm volatile("" : "+v"(l));                  // keeps this arithmetic out of the tile loop's preheader
            live = live && row_of(wave, j * 64 + l) < n_valid;
        }
        if (live)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(dst + j * 1024), "v"(off), "s"(src) : "memory");
    }

    // Zero-fills the rows a ragged tile does not have (their weights are zero, but 0 * garbage could
    // be NaN); the DMA skipped exactly these positions.
    static __device__ __forceinline__ void zero_fill(int n_valid, lds_byte* tile, int wave, int lane)
    {
        if (n_valid < MlaCfg::T) {
            uint32_t z = 0;
            asm volatile("" : "+v"(lane), "+v"(z));          // nothing of this rare path is to live in the tile loop's registers
#pragma unroll
            for (int j = 0; j < INSTRS; j++) {
                const int q = j * 64 + lane;
                if (q < CHUNKS && row_of(wave, q) >= n_valid)
                    *reinterpret_cast<lds_u32x4*>(tile + wave * SHARE_BYTES + q * 16) = u32x4{z, z, z, z};
            }
        }
    }
};

// e4m3 latent tiles: wave w DMAs the raw codes of rows 4w..4w+3 (2304 bytes = 2.25 wave
// instructions) into its own staging area plus the four per-token scales straight into the scale
// slot, and later widens its rows to fp16 (exact: e4m3 has 3 mantissa bits and a 4-bit exponent)
// into the swizzled tile.  Staging is private to the wave: no barrier between request and conversion.
struct MlaDmaFp8 {
    static constexpr int ROWS = MlaDma::ROWS;
    static constexpr int CHUNKS_PER_ROW = MlaCfg::DK / 16;                  // 36
    static constexpr int CHUNKS = ROWS * CHUNKS_PER_ROW;                    // 144
    static constexpr int INSTRS = (CHUNKS + 63) / 64;                       // 3 for the codes, one more for the scales
    static constexpr int PARTS = INSTRS + 1;
    static constexpr int SHARE_BYTES = ROWS * MlaCfg::DK;                   // 2304

    static __device__ __forceinline__ int row_of(int wave, int q) { return wave * ROWS + ((q * 1821) >> 16); }   // q / 36 for q < 192

    static __device__ __forceinline__ void init(lds_byte* table, uint32_t row_bytes, int wave, int lane, int tid)
    {
        uint32_t o[INSTRS];
#pragma unroll
        for (int j = 0; j < INSTRS; j++) {
            const int q = j * 64 + lane, row = min(row_of(wave, q), wave * ROWS + ROWS - 1), cpos = q % CHUNKS_PER_ROW;
            o[j] = (uint32_t)row * row_bytes + (uint32_t)(cpos << 4);
        }
        *reinterpret_cast<lds_u32x4*>(table + tid * 32) = u32x4{o[0], o[1], o[2], 0};
        // where convert() puts the lane's chunk j of codes: (row, 16-byte chunk 2cc) of the widened tile
        uint32_t t[INSTRS];
#pragma unroll
        for (int j = 0; j < INSTRS; j++) {
            const int q = min(j * 64 + lane, CHUNKS - 1), row = row_of(wave, q), cc = q - (row - wave * ROWS) * CHUNKS_PER_ROW;
            t[j] = (uint32_t)mla_swz(row, 2 * cc);
        }
        *reinterpret_cast<lds_u32x4*>(table + tid * 32 + 16) = u32x4{t[0], t[1], t[2], 0};
    }

    // part j < INSTRS: codes; part INSTRS: scales.  `stage`, `scale_dst` = LDS byte addresses of the
    // wave's staging area and of the tile's scale slot; `src`, `scales` = the tile in global memory.
    static __device__ __forceinline__ void issue_part(int j, const MlaDma::Offsets& f, const char* src, const float* scales, int n_valid,
                                                      uint32_t stage, uint32_t scale_dst, int wave, int lane)
    {
        if (j < INSTRS) {
            bool live = j * 64 + 63 < CHUNKS || lane < CHUNKS - j * 64;
            if (n_valid != MlaCfg::T) {
                int l = lane;
                asm volatile("" : "+v"(l));
                live = live && row_of(wave, j * 64 + l) < n_valid;
            }
            if (live)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :: "s"(stage + j * 1024), "v"(f.a[j]), "s"(src) : "memory");
        } else {
            if (lane < ROWS && wave * ROWS + lane < n_valid)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                             :: "s"(scale_dst + wave * ROWS * 4), "v"((uint32_t)lane * 4u), "s"(scales + wave * ROWS) : "memory");
        }
    }

    // After the wave's DMA has landed: widen its rows into the tile (v_cvt_scalef32_pk_f16_fp8 with scale 1:
    // two codes -> two fp16, exact for all 256 codes -- checked on the device); rows the tile does not
    // have become zeros with scale zero.  The destination offsets come from the table init() wrote.
    static __device__ __forceinline__ void convert(int n_valid, const lds_byte* stage, lds_byte* tile, lds_byte* scale_slot,
                                                   const lds_byte* table, int wave, int lane, int tid)
    {
        lane = mla_opaque(lane);                          // addresses recomputed here, not carried through the tile loop
        const u32x4 dst = *reinterpret_cast<const lds_u32x4*>(table + mla_opaque(tid) * 32 + 16);
        const lds_byte* sp = stage + lane * 16;
        const bool ragged = n_valid != MlaCfg::T;
#pragma unroll
        for (int j = 0; j < INSTRS; j++) {
            if (j * 64 + 63 >= CHUNKS && lane >= CHUNKS - j * 64) continue;
            u32x4 w = *reinterpret_cast<const lds_u32x4*>(sp + j * 1024);
            if (ragged && row_of(wave, j * 64 + lane) >= n_valid) w = u32x4{0, 0, 0, 0};
            uint32_t o[8];
#pragma unroll
            for (int d = 0; d < 4; d++) {
                o[2 * d] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[d], 1.0f, false));
                o[2 * d + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[d], 1.0f, true));
            }
            // chunks 2cc and 2cc + 1 of a row swap places under the XOR swizzle: the tile base and the row
            // pitch are multiples of 32 bytes, so that is bit 4 of the offset
            *reinterpret_cast<lds_u32x4*>(tile + dst[j]) = u32x4{o[0], o[1], o[2], o[3]};
            *reinterpret_cast<lds_u32x4*>(tile + (dst[j] ^ 16u)) = u32x4{o[4], o[5], o[6], o[7]};
        }
        if (ragged && lane < ROWS && wave * ROWS + lane >= n_valid) *reinterpret_cast<lds_f32*>(scale_slot + (wave * ROWS + lane) * 4) = 0.f;
    }
};
static_assert(MlaCfg::OFF_K % 32 == 0 && MlaCfg::TILE_BYTES % 32 == 0 && MlaCfg::ROW % 32 == 0, "convert() flips bit 4 of a tile offset");

// MXFP4 latent tiles (E2M1 codes, blocks of 32 along the row sharing an E8M0 scale; rows dense: 288 code
// bytes and 18 scale bytes per token): wave w DMAs the codes of rows 4w..4w+3 (1152 contiguous bytes =
// 1.125 wave instructions) and their 72 scale bytes (18 or 19 dwords from the 4-byte boundary below
// them: a token row's scales start on an even address, not always on a multiple of 4) into its own
// staging area.  Conversion turns the tile into exactly what the e4m3 path produces -- fp16 entries
// plus one fp32 scale per token -- so everything downstream is shared: the token scale is
// f_t = 2^(top_t - 127 - UP) with top_t the largest scale code of the row, and the entries of block j
// become code * 2^(X_j - top_t + UP) in fp16 (v_cvt_scalef32_pk_f16_fp4: two codes of a byte, low
// nibble first, times a float scale).  That is exact while X_j >= top_t - 21 (normal fp16 numbers);
// blocks further below the row's largest lose at most 2^-24 of the row's largest magnitude.
struct MlaDmaFp4 {
    static constexpr int ROWS = MlaDma::ROWS;
    static constexpr int CODE_ROW = MlaCfg::DK / 2;                         // 288
    static constexpr int SCALE_ROW = MlaCfg::DK / 32;                       // 18
    static constexpr int CHUNKS = ROWS * CODE_ROW / 16;                     // 72
    static constexpr int INSTRS = (CHUNKS + 63) / 64;                       // 2 for the codes, one more for the scales
    static constexpr int PARTS = INSTRS + 1;
    static constexpr int UNITS = ROWS * CODE_ROW / 8;                       // 144 eight-byte units = 16 codes = two chunks of the tile
    static constexpr int PASSES = (UNITS + 63) / 64;                        // 3
    static constexpr int OFF_SC = ROWS * CODE_ROW;                          // staging: the scale dwords behind the codes
    static constexpr int SHARE_BYTES = 1280;
    static constexpr int UP = 8;
    static_assert(OFF_SC + 3 + ROWS * SCALE_ROW + 16 <= SHARE_BYTES && MlaCfg::WAVES * SHARE_BYTES <= MlaCfg::T * MlaCfg::DK, "staging area");
    static_assert(PASSES == 3 && INSTRS == 2, "layout of the offset table");

    static __device__ __forceinline__ int row_of_chunk(int q) { return (q * 3641) >> 16; }      // q / 18 for q < 72
    static __device__ __forceinline__ int row_of_unit(int q) { return (q * 1821) >> 16; }       // q / 36 for q < 192

    // `shift` = the run's first scale byte address modulo 4 (0 or 2; the same for every wave and tile,
    // because 4 rows are 72 bytes)
    static __device__ __forceinline__ void init(lds_byte* table, int wave, int lane, int tid, int shift)
    {
        // [0], [1]: the lane's chunk of the wave's 1152 code bytes; [3]: where the set-up step of convert()
        // finds scale (lane & 15) of row (lane >> 4) in the staging area
        *reinterpret_cast<lds_u32x4*>(table + tid * 32) =
            u32x4{(uint32_t)lane * 16u, 1024u + (uint32_t)lane * 16u, 0u, (uint32_t)(OFF_SC + shift + (lane >> 4) * SCALE_ROW + (lane & 15))};
        // [4..6]: unit q = 64 pass + lane of convert(): tile offset of its first chunk | staging offset of its
        // block's scale (from OFF_SC) << 20 | row << 28
        uint32_t t[PASSES];
#pragma unroll
        for (int j = 0; j < PASSES; j++) {
            const int q = min(j * 64 + lane, UNITS - 1), row = row_of_unit(q), uu = q - row * (CODE_ROW / 8);
            t[j] = (uint32_t)mla_swz(wave * ROWS + row, 2 * uu) | (uint32_t)(shift + row * SCALE_ROW + (uu >> 1)) << 20 | (uint32_t)row << 28;
        }
        static_assert(MlaCfg::TILE_BYTES <= (1 << 20) && 3 + ROWS * SCALE_ROW <= 256, "packing of the table entries");
        *reinterpret_cast<lds_u32x4*>(table + tid * 32 + 16) = u32x4{t[0], t[1], t[2], 0};
    }

    // part j < INSTRS: codes; part INSTRS: scales.  `codes` = the wave's rows of the tile in global memory,
    // `scales` = the 4-byte boundary at or below their scale bytes; `stage` = LDS byte address of the wave's
    // staging area.  Only dwords that hold a byte of a row the tile has are requested.
    static __device__ __forceinline__ void issue_part(int j, const MlaDma::Offsets& f, const char* codes, const char* scales, int n_valid,
                                                      uint32_t stage, int wave, int lane, int shift)
    {
        if (j < INSTRS) {
            bool live = j * 64 + 63 < CHUNKS || lane < CHUNKS - j * 64;
            if (n_valid != MlaCfg::T) {
                int l = lane;
                asm volatile("" : "+v"(l));
                live = live && wave * ROWS + row_of_chunk(j * 64 + l) < n_valid;
            }
            if (live)
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                             :: "s"(stage + j * 1024), "v"(f.a[j]), "s"(codes) : "memory");
        } else {
            const int rows = min(ROWS, n_valid - wave * ROWS);
            if (rows > 0 && lane < ((shift + rows * SCALE_ROW + 3) >> 2))
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                             :: "s"(stage + OFF_SC), "v"((uint32_t)lane * 4u), "s"(scales) : "memory");
        }
    }

    template <int BYTE>
    static __device__ __forceinline__ uint32_t pair(uint32_t codes, float scale)
    {
        return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(codes, scale, BYTE));
    }

    // max over each group of 16 lanes, by DPP (no LDS round trips): lane ^ 1, lane ^ 2, mirror within 8, mirror within 16
    static __device__ __forceinline__ int max16(int x)
    {
        x = max(x, __builtin_amdgcn_mov_dpp(x, 0xB1, 0xf, 0xf, true));      // quad_perm [1,0,3,2]
        x = max(x, __builtin_amdgcn_mov_dpp(x, 0x4E, 0xf, 0xf, true));      // quad_perm [2,3,0,1]
        x = max(x, __builtin_amdgcn_mov_dpp(x, 0x141, 0xf, 0xf, true));     // row_half_mirror
        x = max(x, __builtin_amdgcn_mov_dpp(x, 0x140, 0xf, 0xf, true));     // row_mirror
        return x;
    }

    // After the wave's DMA has landed.  Every LDS read is issued up front (the conversion sits at the start
    // of a phase: a chain of dependent LDS round trips there delays the wave's first MFMA).  Lane
    // (row = lane / 16, j = lane % 16) looks at scales j and 16 + j of its row; the rows' largest codes end up
    // in four scalar registers, the token scales in the tile's scale slot (zero for rows the tile does not
    // have, whose entries become zeros as well).  Then three passes over the 144 units; which rows a pass's
    // lanes work on is fixed: units 0..35 are row 0, 36..71 row 1, ...
    static __device__ __forceinline__ void convert(int n_valid, lds_byte* stage, lds_byte* tile, lds_byte* scale_slot,
                                                   const lds_byte* table, int wave, int lane, int tid)
    {
        typedef __attribute__((address_space(3))) uint32_t lds_u32;
        static_assert(CODE_ROW / 8 == 36 && ROWS == 4, "row boundaries of the passes below");
        lane = mla_opaque(lane);
        const lds_byte* mine = table + mla_opaque(tid) * 32;
        const uint32_t at = *reinterpret_cast<const lds_u32*>(mine + 12);
        const u32x4 dst = *reinterpret_cast<const lds_u32x4*>(mine + 16);
        const int j = lane & 15, row = lane >> 4;
        int x = stage[at];
        const int x2 = stage[at + 16];                                      // inside the staging area for every lane
        u32x2 w[PASSES];
        int xb[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; p++) {
            if (p * 64 + 63 >= UNITS && lane >= UNITS - p * 64) continue;
            w[p] = *reinterpret_cast<const lds_u32x2*>(stage + lane * 8 + p * 512);
            xb[p] = stage[OFF_SC + ((dst[p] >> 20) & 0xffu)];
        }
        if (j < SCALE_ROW - 16) x = max(x, x2);
        x = max16(x);
        const int t0 = __builtin_amdgcn_readlane(x, 0), t1 = __builtin_amdgcn_readlane(x, 16);
        const int t2 = __builtin_amdgcn_readlane(x, 32), t3 = __builtin_amdgcn_readlane(x, 48);
        if (j == 0)
            *reinterpret_cast<lds_f32*>(scale_slot + (wave * ROWS + row) * 4) =
                wave * ROWS + row < n_valid ? __builtin_ldexpf(1.f, x - (127 + UP)) : 0.f;
        const bool ragged = n_valid != MlaCfg::T;
#pragma unroll
        for (int p = 0; p < PASSES; p++) {
            if (p * 64 + 63 >= UNITS && lane >= UNITS - p * 64) continue;
            const uint32_t meta = dst[p];
            const int top = p == 0 ? (lane < 36 ? t0 : t1) : p == 1 ? (lane < 8 ? t1 : lane < 44 ? t2 : t3) : t3;
            const int e = xb[p] - top + (127 + UP);
            const float scale = as_f32((uint32_t)max(e, 0) << 23);        // 2^(X - top + UP); more than 135 octaves down: zero
            u32x2 cw = w[p];
            if (ragged && wave * ROWS + (int)(meta >> 28) >= n_valid) cw = u32x2{0, 0};
            const uint32_t to = meta & 0xfffffu;
            *reinterpret_cast<lds_u32x4*>(tile + to) = u32x4{pair<0>(cw.x, scale), pair<1>(cw.x, scale), pair<2>(cw.x, scale), pair<3>(cw.x, scale)};
            *reinterpret_cast<lds_u32x4*>(tile + (to ^ 16u)) = u32x4{pair<0>(cw.y, scale), pair<1>(cw.y, scale), pair<2>(cw.y, scale), pair<3>(cw.y, scale)};
        }
    }
};

// FP8: the latent is not bf16 and the contractions run in fp16 -- e4m3 codes with a scale per token, or,
// with MX, MXFP4 codes with block scales (widened to the same tile and token scales).
template <bool FP8, bool MX = false>
__global__ __launch_bounds__(MlaCfg::THREADS, 1) void mla_decode_kernel(const AttnArgs a)
{
    static_assert(FP8 || !MX, "the MXFP4 latent takes the fp16 pipeline");
    using C = MlaCfg;
    extern __shared__ __align__(16) uint8_t smem_raw[];
    lds_byte* smem = (lds_byte*)smem_raw;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps wave-dependent addresses in SGPRs
    const int r = lane & 15, kc = lane >> 4;
    const int pair = wave >> 1, half = wave & 1;                  // waves 2p, 2p+1 share heads 32p..32p+31

    // Which runs this workgroup serves.  With a stream plan (stream_plan_kernel, one head tile): the tiles
    // [start(g), start(g + 1)) of the even deal (StreamDeal) of the launch's pairs laid end to end -- one run per pair the range
    // touches.  Otherwise one run, from the workgroup id.
    // (everything here is the same for all lanes; values loaded from memory are handed on through
    // readfirstlane so that they, and the addresses derived from them, stay in scalar registers)
    auto uniform64 = [](int64_t x) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)x >> 32));
        return (int64_t)((uint64_t)hi << 32 | lo);
    };
    const bool stream = a.tile_prefix != nullptr;
    int64_t tile_cur = 0, tile_end = 0;
    int kvpair = 0, id_si = 0, id_split = 0, id_b = 0, htw = 0;
    if (stream) {
        const int64_t T = uniform64(a.tile_prefix[a.n_shards * a.B]);
        const StreamDeal deal = stream_deal(T, a.n_wg);
        tile_cur = deal.start(blockIdx.x);
        tile_end = deal.start(blockIdx.x + 1);
        kvpair = __builtin_amdgcn_readfirstlane(a.wg_first_pair[blockIdx.x]);
    } else {
        int u = blockIdx.x;
        while (id_si + 1 < a.n_shards && u >= a.shard[id_si + 1].unit_base) id_si++;
        u -= a.shard[id_si].unit_base;
        const int ug = u / (8 * a.head_tiles), j8 = u % (8 * a.head_tiles);
        const int logical = ug * 8 + (j8 & 7);
        htw = j8 >> 3;
        if (logical >= a.shard[id_si].n_splits * a.B) return;         // padding workgroup
        // Split index slow, sequence fast, and the sequence rotated by 3 per split: consecutive workgroup
        // ids go to different XCDs, so every XCD sees every split index and a mix of sequences.
        id_split = logical / a.B;
        id_b = (logical % a.B + 3 * id_split) % a.B;
    }
  for (bool first_run = true;; first_run = false) {
    int si, b, t0, t1_cap;
    size_t rec;
    if (stream) {
        if (tile_cur >= tile_end) break;
        int64_t lo = uniform64(a.tile_prefix[kvpair]), hi = uniform64(a.tile_prefix[kvpair + 1]);
        while (hi <= tile_cur) { kvpair++; lo = hi; hi = uniform64(a.tile_prefix[kvpair + 1]); }     // pairs without tokens
        const int64_t seg_end = min(tile_end, hi);
        si = kvpair / a.B;
        b = kvpair - si * a.B;
        t0 = (int)(tile_cur - lo) * MlaCfg::T;
        t1_cap = (int)(seg_end - lo) * MlaCfg::T;
        rec = (size_t)(a.rec_base + (int)blockIdx.x + kvpair) * a.Q;
        tile_cur = seg_end;
        kvpair++;
    } else {
        if (!first_run) break;
        si = id_si;
        b = id_b;
        t0 = id_split * a.split_tokens;
        t1_cap = t0 + a.split_tokens;
        rec = ((size_t)(a.shard[si].split_base + id_split) * a.B + b) * a.Q + htw * MlaCfg::HPW;
    }
    const ShardDev& sh = a.shard[si];

    int len;
    int64_t first_row;
    shard_range(sh, b, len, first_row);
    len = __builtin_amdgcn_readfirstlane(len);
    first_row = uniform64(first_row);
    if (!stream && id_split == 0 && htw == 0 && threadIdx.x == 0) {
        if (sh.out_off) { sh.out_off[b] = first_row; sh.out_len[b] = len; }
        flag_len_overflow(sh, len, a.split_tokens);
    }
    const int t1 = min(t1_cap, len);
    const int h0 = htw * C::HPW;                      // first head of this workgroup
    const int nh = min(C::HPW, a.Q - h0);             // real heads (the rest is zero padding)

    if (t0 >= len) {                                  // nothing to attend to: an empty record
        if (tid < nh) { a.ws_m[rec + tid] = -INFINITY; a.ws_l[rec + tid] = 0.f; }
        continue;
    }

    // Q slice of this wave as the score MFMA's B operand: lane (r,kc) holds head 16*wave + r of the
    // workgroup, dims 32*ks + 8*kc .. +8
    const int hl = wave * 16 + r;                     // this lane's head within the workgroup
    u32x4 qb[C::KS];
    float q_mul = a.scale_log2e;                      // raw MFMA score -> exponent (base 2) of the weight
    {
        const uint16_t* qrow = a.q + ((size_t)b * a.Q + h0 + min(hl, nh - 1)) * C::DK + kc * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ks++) {
            u32x4 w = *reinterpret_cast<const u32x4*>(qrow + ks * 32);
            if (hl >= nh) w = u32x4{0, 0, 0, 0};
            qb[ks] = w;
        }
        if constexpr (FP8) {
            // The e4m3 path contracts in fp16: the workgroup's query rows are scaled by the power of two
            // that puts their largest magnitude in [2^14, 2^15) and converted (exact for every entry within
            // 2^-28 of the largest, the rest is off by less than 2^-39 of it); the scores get the inverse.
            // One factor for the whole workgroup, so that it lives in a scalar register.
            uint32_t mx = 0;
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++)
#pragma unroll
                for (int j = 0; j < 4; j++) mx = max(mx, max(qb[ks][j] & 0x7fffu, (qb[ks][j] >> 16) & 0x7fffu));
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
            uint32_t* cell = reinterpret_cast<uint32_t*>(smem_raw + C::OFF_FLAG);
            if (tid == 0) cell[1] = 0;
            __syncthreads();
            if (lane == 0) atomicMax(&cell[1], mx);
            __syncthreads();
            mx = __builtin_amdgcn_readfirstlane(cell[1]);
            const uint32_t e = min(max(mx >> 7, 15u), 254u);            // biased exponent of the largest |q|
            const float up = as_f32((268u - e) << 23);                   // 2^(14 - (e - 127))
            q_mul *= as_f32((e - 14u) << 23);                            // 2^((e - 127) - 14)
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++)
#pragma unroll
                for (int j = 0; j < 4; j++)
                    qb[ks][j] = pack_f16_rne(as_f32(qb[ks][j] << 16) * up, as_f32(qb[ks][j] & 0xffff0000u) * up);
        }
    }

    const int esz = FP8 ? 1 : 2;
    const int64_t tok0 = first_row + t0;
    const int64_t first_elem = (int64_t)b * sh.k_sb + tok0 * sh.k_st;
    const char* kbase = reinterpret_cast<const char*>(sh.k) + (MX ? first_elem / 2 : esz * first_elem);
    const float* sbase = FP8 && !MX ? sh.kv_scale + (int64_t)b * sh.s_sb + tok0 : nullptr;
    const uint32_t row_bytes = MX ? (uint32_t)MlaDmaFp4::CODE_ROW : (uint32_t)sh.k_st * esz;
    // MXFP4: the run's block scales, from the 4-byte boundary at or below them
    const char* xbase = nullptr;
    int xshift = 0;
    if constexpr (MX) {
        xbase = reinterpret_cast<const char*>(sh.k_mx) + first_elem / 32;
        xshift = (int)(reinterpret_cast<uintptr_t>(xbase) & 3);
        xbase -= xshift;
    }

    const int n_tok = t1 - t0;
    const int n_tiles = (n_tok + C::T - 1) / C::T;

    float m_ref = -INFINITY;                          // reference exponent of head hl (integer-valued)
    float l_run = 0.f;                                // this lane's share of sum p (tokens 4kc+i, 16+4kc+i of every tile)
    f32x4 acc[C::DVT][C::NHT];                        // O^T[256half + 16d + 4kc + i][32pair + 16h + r]

    auto ktile_of = [&](int slot) { return smem + C::OFF_K + slot * C::TILE_BYTES; };      // slot = tile index mod NBUF
    auto next_slot = [](int slot) { return slot + 1 == C::NBUF ? 0 : slot + 1; };
    auto valid_of = [&](int it) { return min(C::T, n_tok - it * C::T); };

    // Scores of this wave's 16 heads against both token halves of a latent tile in LDS: two
    // independent MFMA chains.  Chunk 4ks + kc of row 16half + r sits at chunk (4ks + kc) ^ f,
    // f = row & 7 = r & 7: the low two bits of f permute kc, bit 2 swaps k-steps 2j and 2j+1 -> one
    // per-lane base, +-64 bytes, immediates for ks and the half.  Reads run PD k-steps ahead.
    auto scores = [&](const lds_byte* ktile, f32x4& s0, f32x4& s1) {
        constexpr int PD = MX ? 2 : 3;           // measured: MXFP4 2.3 % faster with 2, e4m3 1 % slower, bf16 unchanged
        u32x4 k0[C::KS], k1[C::KS];
        const int l = mla_opaque(lane), r = l & 15, kc = l >> 4;
        const int f = r & 7;
        const lds_byte* kp = ktile + r * C::ROW + ((kc ^ (f & 3)) << 4);
        const int flip = (f & 4) << 4;
        auto rd = [&](int ks, int half) {
            const lds_byte* q = ((ks & 1) ? kp - flip : kp + flip) + half * 16 * C::ROW;
            return *reinterpret_cast<const lds_u32x4*>(q + ks * 64);
        };
        s0 = f32x4{0.f, 0.f, 0.f, 0.f};
        s1 = s0;
#pragma unroll
        for (int o = 0; o < PD; o++) { k0[o] = rd(o, 0); k1[o] = rd(o, 1); }
#pragma unroll
        for (int o = 0; o < C::KS; o++) {
            s0 = mla_mfma<FP8>(k0[o], qb[o], s0);
            s1 = mla_mfma<FP8>(k1[o], qb[o], s1);
            if (o + PD < C::KS) { k0[o + PD] = rd(o + PD, 0); k1[o + PD] = rd(o + PD, 1); }
            __builtin_amdgcn_sched_barrier(0);        // keep the reads PD k-steps ahead
        }
        // lane (r,kc): head r; s0[i] = token 4kc + i, s1[i] = token 16 + 4kc + i
    };

    // exponents (base 2) of the lane's 8 scores, masked beyond the ragged end of the tile; returns
    // their maximum (-inf if none is valid)
    auto exponents = [&](auto masked, const f32x4& s0, const f32x4& s1, int kb, int n_valid, float (&t)[8], float (&fs)[8]) {
        if (FP8) {
            const auto* sc = reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(smem + C::OFF_SCALE + kb * C::T * 4);
            const int kq = mla_opaque(lane) >> 4;
            const f32x4 f0 = sc[kq], f1 = sc[4 + kq];
#pragma unroll
            for (int i = 0; i < 4; i++) { fs[i] = f0[i]; fs[4 + i] = f1[i]; }
        }
        float bmax = -INFINITY;
        int tok = 0;
        if constexpr (decltype(masked)::value) tok = (mla_opaque(lane) >> 4) * 4;   // recomputed here: eight hoisted token indices would not fit
#pragma unroll
        for (int i = 0; i < 8; i++) {
            float x = (i < 4 ? s0[i] : s1[i - 4]) * q_mul;
            if (FP8) x *= fs[i];
            if constexpr (decltype(masked)::value) {
                if (tok >= n_valid - ((i >> 2) * 16 + (i & 3))) x = -INFINITY;
            }
            t[i] = x;
            bmax = fmaxf(bmax, x);
        }
        return bmax;
    };

    // A head's reference exponent moved up by `d` octaves (0 for the heads of this wave that stay) in the S phase
    // of tile `it`: its normaliser follows at once, its accumulators -- spread over the pair's two waves -- when
    // the P phase finds the factor 2^-d in the mailbox (epoch = it + 1 tells that the factors are this tile's).
    auto move_reference = [&](int it, float d) {
        d = fminf(d, 16384.f);                        // (an infinite score: the result is NaN whatever happens here)
        m_ref += d;
        l_run = __builtin_ldexpf(l_run, -(int)d);
        const int l = mla_opaque(lane);
        if ((l >> 4) == 0) *reinterpret_cast<lds_f32*>(smem + C::OFF_RESC + C::WAVES * 4 + (wave * 16 + (l & 15)) * 4) = __builtin_ldexpf(1.f, -(int)d);
        if (l == 0) {
            *reinterpret_cast<lds_i32*>(smem + C::OFF_RESC + wave * 4) = it + 1;
            if (sh.status) atomicAdd(sh.status, kStatusReferenceMoved);
        }
    };

    // Softmax of the wave's scores, entirely inside the wave: the lane's 8 weights are exactly the 8
    // k-slots of lane (r,kc) in the P.V MFMA's B operand if slot e < 4 means token 4kc + e and slot
    // e >= 4 token 16 + 4kc + e - 4 -- the V^T operand is read to match.  A head's reference stays where it is
    // from tile to tile, so no maximum has to be agreed on across lanes in the common case: every lane checks
    // its own weights (scores) against the limit, and only a tile in which some lane of the wave exceeds it
    // takes the branch that moves that head's reference (exact powers of two throughout: which tiles moved a
    // reference, and by how much, changes no bit of a weight's significand).
    // `masked`: the tile is the ragged last one of the run -- tokens beyond n_valid get exponent -inf,
    // clamped 200 octaves below the reference where the weight is exactly 0.  Full tiles skip both.
    auto softmax_tile = [&](auto masked, const f32x4& s0, const f32x4& s1, int kb, int n_valid, int it) {
        constexpr bool M = decltype(masked)::value;
        auto floor_of = [&](float x) { return M ? fmaxf(x, m_ref - 200.f) : x; };
        float t[8], fs[8], p[8];
        if constexpr (FP8) {
            // One fp16 weight per token, w_t = p_t * f_t (11 significant bits: relative L2 error of O about 2e-4);
            // the normaliser sums the unrounded p_t in fp32.
            exponents(masked, s0, s1, kb, n_valid, t, fs);
            float lsum = 0.f, wm = 0.f;
            {
                const int mi = (int)m_ref;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    const float pi = exp2_rel_int(floor_of(t[i]), mi);
                    lsum += pi;
                    p[i] = pi * fs[i];
                    wm = fmaxf(wm, p[i]);
                }
            }
            if (__builtin_expect(__any(!(wm < C::kWeightLimit)), 0)) {
                const float wh = wave_xor_max_16_32(wm);               // the head's largest weight of this tile
                const bool hit = !(wh < C::kWeightLimit);
                if (!__any(hit && !(wh < INFINITY && lsum < INFINITY))) {
                    // the usual case: every weight is a finite fp32 number, so the new reference follows from the
                    // largest one and the tile's weights move with it by an exact power of two
                    const int d = hit ? __builtin_amdgcn_frexp_expf(wh) - (int)C::kWeightLand : 0;
                    move_reference(it, (float)d);
                    lsum = __builtin_ldexpf(lsum, -d);
#pragma unroll
                    for (int i = 0; i < 8; i++) p[i] = __builtin_ldexpf(p[i], -d);
                } else {
                    // a weight beyond fp32 (a score more than 100 octaves above the reference): the tile's scores
                    // are computed once more -- kept across the branch they would cost every tile eight registers.
                    // Exponent of the head's largest weight of this tile: log2(p_t f_t) = t + log2 f_t.
                    f32x4 r0, r1;
                    scores(ktile_of(kb), r0, r1);
                    exponents(masked, r0, r1, kb, n_valid, t, fs);
                    float um = -INFINITY;
#pragma unroll
                    for (int i = 0; i < 8; i++) um = fmaxf(um, floor_of(t[i]) + __builtin_log2f(fs[i]));
                    um = wave_xor_max_16_32(um);
                    move_reference(it, hit ? fmaxf(__builtin_ceilf(um) - C::kWeightLand - m_ref, 0.f) : 0.f);
                    const int mi = (int)m_ref;
                    lsum = 0.f;
#pragma unroll
                    for (int i = 0; i < 8; i++) {
                        const float pi = exp2_rel_int(floor_of(t[i]), mi);
                        lsum += pi;
                        p[i] = pi * fs[i];
                    }
                }
            }
            l_run += lsum;
            u32x4 w;
#pragma unroll
            for (int j = 0; j < 4; j++) w[j] = pack_f16_rne(p[2 * j], p[2 * j + 1]);
            const int l = mla_opaque(lane);
            lds_byte* pw = smem + C::OFF_P + pair * 2 * C::P_BYTES + (half * 16 + (l & 15)) * (C::T * 2) + (((l >> 4) ^ ((l >> 1) & 3)) << 4);
            *reinterpret_cast<lds_u32x4*>(pw) = w;
            return;
        }
        float top = exponents(masked, s0, s1, kb, n_valid, t, fs);
        if (__builtin_expect(__any(top > m_ref + C::kLimit), 0)) {
            top = wave_xor_max_16_32(top);
            move_reference(it, top > m_ref + C::kLimit ? __builtin_ceilf(top) + C::kHeadroom - m_ref : 0.f);
        }
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            p[i] = exp2_rel(floor_of(t[i]), m_ref);
            lsum += p[i];
        }
        l_run += lsum;
        u32x4 hi, lo;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            hi[j] = pack_bf16_rne(p[2 * j], p[2 * j + 1]);
            lo[j] = pack_bf16_rne(p[2 * j] - as_f32(hi[j] << 16), p[2 * j + 1] - as_f32(hi[j] & 0xffff0000u));
        }
        const int l = mla_opaque(lane);
        lds_byte* pw = smem + C::OFF_P + pair * 2 * C::P_BYTES + (half * 16 + (l & 15)) * (C::T * 2) + (((l >> 4) ^ ((l >> 1) & 3)) << 4);
        *reinterpret_cast<lds_u32x4*>(pw) = hi;
        *reinterpret_cast<lds_u32x4*>(pw + C::P_BYTES) = lo;
    };
    auto softmax = [&](const f32x4& s0, const f32x4& s1, int kb, int n_valid, int it) {
        if (n_valid == C::T) softmax_tile(std::false_type{}, s0, s1, kb, n_valid, it);
        else softmax_tile(std::true_type{}, s0, s1, kb, n_valid, it);
    };

    // O^T[value columns of this wave, 32 heads of the pair] += V^T . P^T for one tile.  The weights
    // (two head tiles, hi and lo) stay in registers, the V^T operands stream through transposing
    // reads.  Lane (r,kc) supplies rows 4kc + r/4 (first read) and 16 + that (second read), value
    // columns 256half + 16d + 4(r%4) .. +3 = chunk 32half + 2d + (r%4)/2, byte 8*(r&1) within it;
    // row & 7 is the same for both reads and touches the low three chunk bits: four per-lane bases
    // (d % 4), immediates for d / 4 and the second row.  `between(j)` runs after the j-th group of
    // three column tiles (the caller spreads its DMA requests there).
    auto pv = [&](const lds_byte* ktile, int it, auto&& between) {
        const int l = mla_opaque(lane), r = l & 15, kc = l >> 4;
        {   // rare: heads of this pair moved their reference in this tile's S phase (move_reference)
            const u32x2 ep = *reinterpret_cast<const lds_u32x2*>(smem + C::OFF_RESC + pair * 8);
            const int e0 = __builtin_amdgcn_readfirstlane((int)ep.x), e1 = __builtin_amdgcn_readfirstlane((int)ep.y);
            if (__builtin_expect(e0 == it + 1 || e1 == it + 1, 0)) {
#pragma unroll
                for (int h = 0; h < C::NHT; h++) {
                    if ((h == 0 ? e0 : e1) != it + 1) continue;
                    const float f = *reinterpret_cast<const lds_f32*>(smem + C::OFF_RESC + C::WAVES * 4 + (pair * 32 + h * 16 + r) * 4);
#pragma unroll
                    for (int d = 0; d < C::DVT; d++) acc[d][h] *= f;
                }
            }
        }
        const lds_byte* pp = smem + C::OFF_P + pair * 2 * C::P_BYTES + r * (C::T * 2) + ((kc ^ ((r >> 1) & 3)) << 4);
        u32x4 bh[C::NHT], bl[C::NHT];
#pragma unroll
        for (int h = 0; h < C::NHT; h++) {
            bh[h] = *reinterpret_cast<const lds_u32x4*>(pp + h * 16 * (C::T * 2));
            if constexpr (!FP8) bl[h] = *reinterpret_cast<const lds_u32x4*>(pp + h * 16 * (C::T * 2) + C::P_BYTES);
        }
        const int vrow = 4 * kc + (r >> 2), vf = vrow & 7, cb = (r & 3) >> 1;
        const lds_byte* vb = ktile + vrow * C::ROW + ((r & 1) << 3) + half * 512;
        const lds_byte* ve[4];
#pragma unroll
        for (int e = 0; e < 4; e++) ve[e] = vb + (((2 * e + cb) ^ vf) << 4);
        auto rd = [&](int d) {
            const lds_byte* p0 = ve[d & 3] + (d >> 2) * 128;
            const u32x2 v0 = lds_read_tr16(p0), v1 = lds_read_tr16(p0 + 16 * C::ROW);
            return u32x4{v0.x, v0.y, v1.x, v1.y};
        };
        constexpr int PD = 3;
        u32x4 va[C::DVT];
#pragma unroll
        for (int d = 0; d < PD; d++) va[d] = rd(d);
#pragma unroll
        for (int d = 0; d < C::DVT; d++) {
#pragma unroll
            for (int h = 0; h < C::NHT; h++) acc[d][h] = mla_mfma<FP8>(va[d], bh[h], acc[d][h]);
            if constexpr (!FP8) {
#pragma unroll
                for (int h = 0; h < C::NHT; h++) acc[d][h] = mla_mfma<false>(va[d], bl[h], acc[d][h]);
            }
            if (d + PD < C::DVT) va[d + PD] = rd(d + PD);
            if (d % 3 == 1) between(d / 3);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Tile `it` on its way into LDS slot `slot`.  stage_begin() fetches the lane's source offsets,
    // stage_issue_part() requests one part, stage_commit() completes the tile as far as this wave
    // is concerned (its own requests have landed; e4m3 rows are widened); a barrier then publishes it.
    constexpr int AHEAD = C::AHEAD;
    constexpr int PARTS = MX ? MlaDmaFp4::PARTS : FP8 ? MlaDmaFp8::PARTS : MlaDma::INSTRS;
    static_assert(AHEAD == 2 && C::NBUF == 3, "ring arithmetic: tile it+2 goes where tile it-1 was");
    if constexpr (MX) MlaDmaFp4::init(smem + C::OFF_DMA, wave, lane, tid, xshift);
    else if constexpr (FP8) MlaDmaFp8::init(smem + C::OFF_DMA, row_bytes, wave, lane, tid);
    else MlaDma::init(smem + C::OFF_DMA, row_bytes, wave, lane, tid);
    MlaDma::Offsets dma_off;                              // valid from stage_begin() to the last part of that phase
    auto stage_begin = [&]() { dma_off = MlaDma::fetch(smem + C::OFF_DMA, tid); };
    auto stage_issue_part = [&](int it, int slot, int j) {
        const char* src = kbase + (size_t)it * C::T * row_bytes;
        if constexpr (MX)
            MlaDmaFp4::issue_part(j, dma_off, src + wave * MlaDmaFp4::ROWS * MlaDmaFp4::CODE_ROW,
                                  xbase + ((size_t)it * C::T + wave * MlaDmaFp4::ROWS) * MlaDmaFp4::SCALE_ROW, valid_of(it),
                                  (uint32_t)(uintptr_t)(smem + C::OFF_STAGE) + wave * MlaDmaFp4::SHARE_BYTES, wave, lane, xshift);
        else if constexpr (FP8)
            MlaDmaFp8::issue_part(j, dma_off, src, sbase + it * C::T, valid_of(it), (uint32_t)(uintptr_t)(smem + C::OFF_STAGE) + wave * MlaDmaFp8::SHARE_BYTES,
                                  (uint32_t)(uintptr_t)(smem + C::OFF_SCALE) + slot * C::T * 4, wave, lane);
        else
            MlaDma::issue_part(j, dma_off, src, valid_of(it), (uint32_t)(uintptr_t)ktile_of(slot) + wave * MlaDma::SHARE_BYTES, wave, lane);
    };
    auto stage_issue = [&](int it, int slot) {
        stage_begin();
#pragma unroll
        for (int j = 0; j < PARTS; j++) stage_issue_part(it, slot, j);
    };
    // `newer` = whole tiles (5 instructions per wave) requested after this one, which may stay in flight
    auto stage_commit = [&](int it, int slot, int newer) {
        if constexpr (MX) {
            mla_wait_vm<0>();
            MlaDmaFp4::convert(valid_of(it), smem + C::OFF_STAGE + wave * MlaDmaFp4::SHARE_BYTES, ktile_of(slot), smem + C::OFF_SCALE + slot * C::T * 4,
                               smem + C::OFF_DMA, wave, lane, tid);
        } else if constexpr (FP8) {
            mla_wait_vm<0>();
            MlaDmaFp8::convert(valid_of(it), smem + C::OFF_STAGE + wave * MlaDmaFp8::SHARE_BYTES, ktile_of(slot), smem + C::OFF_SCALE + slot * C::T * 4,
                               smem + C::OFF_DMA, wave, lane, tid);
        } else {
            MlaDma::zero_fill(valid_of(it), ktile_of(slot), wave, lane);
            if (newer == 1) mla_wait_vm<MlaDma::INSTRS>();
            else mla_wait_vm<0>();
        }
    };

    {
        l_run = 0.f;
#pragma unroll
        for (int d = 0; d < C::DVT; d++)
#pragma unroll
            for (int h = 0; h < C::NHT; h++) acc[d][h] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (tid < C::WAVES) *reinterpret_cast<lds_i32*>(smem + C::OFF_RESC + tid * 4) = 0;       // no reference has moved yet

        // ---- first tiles on their way; tile 0 sets the reference exponent of every head ----
        if constexpr (FP8) {
            // the staging area holds one tile: tile 1 is requested once tile 0 has been widened
            stage_issue(0, 0);
            stage_commit(0, 0, 0);
            if (n_tiles > 1) stage_issue(1, 1);
        } else {
            // a tile counts as whole unless it is the last of the run
            stage_issue(0, 0);
            if (n_tiles > 1) stage_issue(1, 1);
            stage_commit(0, 0, n_tiles > 2 ? 1 : 0);
        }
        mla_barrier();
        {
            float t[8], fs[8];
            f32x4 s0, s1;
            scores(ktile_of(0), s0, s1);
            const float top = wave_xor_max_16_32(exponents(std::true_type{}, s0, s1, 0, valid_of(0), t, fs));
            if constexpr (FP8) {
                // fp16 weights w_t = 2^(t - m) f_t: the head's reference m puts its largest first-tile weight
                // into [2^4, 2^5] -- nine octaves below the limit at which the reference moves, eighteen above
                // the smallest normal fp16 number.  (A tile whose token scales are all zero: by the scores.)
                float um = -INFINITY;
#pragma unroll
                for (int i = 0; i < 8; i++) um = fmaxf(um, t[i] + __builtin_log2f(fs[i]));
                um = wave_xor_max_16_32(um);
                m_ref = um > -INFINITY ? __builtin_ceilf(um) - C::kWeightLand : __builtin_ceilf(top);
            } else {
                m_ref = __builtin_ceilf(top) + C::kHeadroom;      // finite: token 0 is valid
            }
        }

        // ---- the tile loop ----
        for (int it = 0, slot = 0; it < n_tiles; it++) {
            const int slot1 = next_slot(slot), slot2 = next_slot(slot1);
            {   // S phase
                f32x4 s0, s1;
                scores(ktile_of(slot), s0, s1);
                softmax(s0, s1, slot, valid_of(it), it);
                // the next tile is completed here (bf16: its DMA awaited; MXFP4: widened -- measured 1.6-2 %
                // faster here than at the start of the P phase, the e4m3 widening 1 % slower)
                if ((!FP8 || MX) && it + 1 < n_tiles) stage_commit(it + 1, slot1, 0);
            }
            mla_barrier();
            {   // P phase
                // e4m3: the next tile is widened here rather than in the S phase, which is the longer one
                // and the one that loads LDS most; its staging area is free again for the request below
                if (FP8 && !MX && it + 1 < n_tiles) stage_commit(it + 1, slot1, 0);
                const bool more = it + AHEAD < n_tiles;
                if (more) stage_begin();
                pv(ktile_of(slot), it, [&](int j) { if (more && j < PARTS) stage_issue_part(it + AHEAD, slot2, j); });
            }
            mla_barrier();
            slot = slot1;
        }
    }

    // ---- the workgroup's record: un-normalised O, reference exponent and normaliser per head ----
    {
        const float l = wave_xor_sum_16_32(l_run);
        if (kc == 0 && hl < nh) {
            a.ws_m[rec + hl] = m_ref;
            a.ws_l[rec + hl] = l;
        }
    }
#pragma unroll
    for (int h = 0; h < C::NHT; h++) {
        const int ho = pair * 32 + h * 16 + r;
        if (ho < nh) {
            float* orow = a.ws_o + (rec + ho) * C::DV + half * 256 + kc * 4;
#pragma unroll
            for (int d = 0; d < C::DVT; d++) *reinterpret_cast<f32x4*>(orow + d * 16) = acc[d][h];
        }
    }
  }   // the workgroup's next run
}

}  // namespace helix

// Split-KV decode attention for the MLA case on gfx950: 128 query heads attending ONE shared latent
// whose 576-wide row is the key and whose first 512 entries are the value (Sec. 1, Sec. 3: MLA keeps
// one latent for K and V that all query heads share), per-shard attention of Helix's attention
// phase (Sec. 2.1.1).  Latent stored as bf16, or as e4m3 codes with one fp32 scale per token.
//
// This is the dense contraction of the path (242 flop per latent byte in bf16, 480 in e4m3): it is
// MFMA-bound, so the design question is how to feed the matrix cores, not HBM.
//
// What was measured on MI355X and shaped the kernel:
//   * one wavefront per SIMD issues a 16x16x32 bf16 MFMA only every ~21 cycles and cannot overlap its
//     own VALU work with its MFMAs (each extra VALU op costs ~3.5 cycles); two wavefronts per SIMD
//     reach the 16-cycle rate and hide each other's VALU and LDS waits -> 8 wavefronts per CU, at
//     most 256 registers each;
//   * LDS delivers ~220 B/clk per CU for 128-bit reads with 8 wavefronts, but only if the 16 rows x
//     64 B of an MFMA operand hit distinct banks: latent rows are padded from 1152 to 1184 bytes;
//   * ds_read_b64_tr_b16 hands out the transposed (value-column-major) operand straight from the
//     row-major latent tile; global_load_lds_dwordx4 copies 16 bytes per lane from global memory
//     into LDS without touching registers.
//
// Workgroup = 8 wavefronts = one CU, HPW = 64 heads, a run of `split_tokens` latent rows in tiles of
// 32 tokens.  (The two workgroups that cover the 128 heads of a token range are numbered 8 apart, so
// they sit on the same XCD and the second one's latent reads hit that XCD's L2.)
//   scores   S^T[token, head] = K . Q^T: wave w = (hq, th) owns heads 16hq..16hq+15 and tokens
//            16th..16th+15 of every tile; its Q slice (16 x 576 bf16 = 72 registers) never moves,
//            the K operands come from LDS.
//   softmax  per wave on its 16x16 scores with an integer reference exponent that is FIXED for the
//            whole run (set 32 octaves above the first tile's maximum): no rescale of accumulators
//            inside the loop, ever; if a later tile exceeds the reference by more than 64 octaves
//            the workgroup starts the run over with a higher reference (never seen on real logits,
//            exercised by a test).  Weights go to LDS as bf16 hi + lo.
//   P.V      O^T[dv, head] += V^T . P^T: wave w owns value columns 64w..64w+63 for all 64 heads
//            (64 accumulator registers); V^T operands via the transposing LDS read, P^T operands
//            from the weights all eight waves just wrote.
//   The four waves with th = 0 run scores -> softmax -> P.V(previous tile), the four with th = 1
//   run P.V(previous tile) -> scores -> softmax: the two waves of a SIMD are always in different
//   phases, so one's exponentials issue under the other's MFMAs.  One barrier per tile.
//
// e4m3 latent: codes are widened to bf16 (exact) on their way into LDS; the per-token scale f_t
// multiplies the score (s_t = f_t * q.k8_t) and the weight that meets the values (p_t * f_t), while
// the normaliser sums the plain p_t.
#pragma once
#include "common.hpp"

namespace helix {

struct MlaCfg {
    static constexpr int DK = 576, DV = 512;
    static constexpr int T = 32;                  // tokens per tile
    static constexpr int ROW = 1184;              // LDS bytes per latent row (1152 + 32 pad)
    static constexpr int KS = DK / 32;            // 18 k-steps of the score MFMA
    static constexpr int NBUF = 3;                // latent tiles in LDS: values (it-1), keys (it), in flight (it+1)
    static constexpr int TILE_BYTES = T * ROW;    // 37888
    static constexpr int HPW = 64;                // heads per workgroup
    static constexpr int NHT = HPW / 16;          // head tiles
    static constexpr int WAVES = 8;
    static constexpr int THREADS = WAVES * 64;
    static constexpr int DVT = DV / 16 / WAVES;   // value-column tiles per wave (4)
    static constexpr int P_BYTES = HPW * T * 2;   // one of hi / lo: [HPW heads][32 tokens] bf16
    // LDS map
    static constexpr int OFF_K = 0;
    static constexpr int OFF_P = NBUF * TILE_BYTES;               // [2 buffers][hi, lo]
    static constexpr int OFF_FLAG = OFF_P + 2 * 2 * P_BYTES;      // [2][8] int: a wave asks for a restart
    static constexpr int OFF_TOP = OFF_FLAG + 2 * WAVES * 4;      // [2 token halves][HPW] fp32: first-tile maxima / final l
    static constexpr int OFF_SCALE = OFF_TOP + 2 * HPW * 4;       // [NBUF][32] fp32 per-token scales
    static constexpr int LDS_BYTES = OFF_SCALE + NBUF * T * 4;
    static constexpr float kHeadroom = 32.f, kLimit = 64.f;
};

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

// Workgroups of one shard are numbered so that the head tiles of the same token range are 8 apart:
// consecutive workgroup ids go round-robin over the 8 XCDs, so ids that differ by 8 share an XCD
// and with it an L2.  Shards are padded to a multiple of 8 token ranges (padding workgroups exit).
__host__ __device__ inline int mla_units_of_shard(int n_splits, int B, int head_tiles)
{
    return (n_splits * B + 7) / 8 * 8 * head_tiles;
}

// bf16 latent tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l of a
// wave instruction deposits its 16 bytes at the instruction's LDS base + 16*l; inactive lanes write
// nothing -- checked on the device).  The padded tile is a run of 32 x 74 sixteen-byte positions
// (72 data chunks + 2 pad per row) = 37 wave instructions, dealt 5 per wave.
struct MlaDma {
    static constexpr int POS_PER_ROW = MlaCfg::ROW / 16;                    // 74
    static constexpr int INSTRS = MlaCfg::T * POS_PER_ROW / 64;             // 37
    static constexpr int PER_WAVE = (INSTRS + MlaCfg::WAVES - 1) / MlaCfg::WAVES;   // 5
    static_assert(MlaCfg::T * POS_PER_ROW % 64 == 0, "tile must be whole wave instructions");

    // Starts the copy of the tile at `src` (n_valid rows) into LDS buffer `dst`.  `wave` is uniform.
    static __device__ __forceinline__ void issue(const char* src, uint32_t row_bytes, int n_valid, lds_byte* dst, int wave, int lane)
    {
        // The per-lane offsets are the same for every tile: the compiler hoists them out of the tile
        // loop (five registers), which leaves ~8 instructions per DMA instead of ~20.
        const int pos = wave * PER_WAVE * 64 + lane;
        int row = pos / POS_PER_ROW, c = pos - row * POS_PER_ROW;
#pragma unroll
        for (int j = 0; j < PER_WAVE; j++) {
            if (wave * PER_WAVE + j < INSTRS) {
                if (c < 72 && row < n_valid)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void*)(src + ((uint32_t)row * row_bytes + (uint32_t)c * 16u)),
                        dst + (wave * PER_WAVE + j) * 1024, 16, 0, 0);
            }
            c += 64;                                  // next instruction: 64 positions further
            if (c >= POS_PER_ROW) { c -= POS_PER_ROW; row++; }
        }
    }

    // Zero-fills the rows a ragged tile does not have (their weights are zero, but 0 * garbage could
    // be NaN) and waits for the copy to land; call before the barrier that publishes the tile.
    static __device__ __forceinline__ void commit(int n_valid, lds_byte* dst, int wave, int lane)
    {
        if (n_valid < MlaCfg::T) {
            const int pos0 = wave * PER_WAVE * 64 + lane;
#pragma unroll
            for (int j = 0; j < PER_WAVE; j++) {
                const int pos = pos0 + j * 64;
                const int row = pos / POS_PER_ROW, c = pos - row * POS_PER_ROW;
                if (wave * PER_WAVE + j < INSTRS && c < 72 && row >= n_valid)
                    *reinterpret_cast<lds_u32x4*>(dst + pos * 16) = u32x4{0, 0, 0, 0};
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                                 // vmcnt(0): the DMA counts as a vector memory load
    }
};

// e4m3 latent tiles pass through registers: 16 codes per 16-byte chunk become 16 bf16 (exact: e4m3
// has 3 mantissa bits and a 4-bit exponent) and go to LDS with ordinary stores.
struct MlaStageFp8 {
    static constexpr int CHUNKS_PER_ROW = 36;
    static constexpr int CHUNKS = MlaCfg::T * CHUNKS_PER_ROW;               // 1152
    static constexpr int PER_THREAD = (CHUNKS + MlaCfg::THREADS - 1) / MlaCfg::THREADS;   // 3
    u32x4 regs[PER_THREAD];
    float scale;                                                            // thread t < 32 holds token t's scale

    __device__ __forceinline__ void load(const char* src, uint32_t row_bytes, const float* scales, int n_valid, int tid)
    {
#pragma unroll
        for (int j = 0; j < PER_THREAD; j++) {
            const int ch = tid + MlaCfg::THREADS * j;
            const int row = ch / CHUNKS_PER_ROW, cc = ch % CHUNKS_PER_ROW;
            regs[j] = u32x4{0, 0, 0, 0};
            if (ch < CHUNKS && row < n_valid)
                regs[j] = *reinterpret_cast<const u32x4*>(src + (size_t)row * row_bytes + cc * 16);
        }
        scale = (tid < n_valid && tid < MlaCfg::T) ? scales[tid] : 0.f;
    }

    __device__ __forceinline__ void store(lds_byte* dst, lds_byte* dst_scale, int tid) const
    {
#pragma unroll
        for (int j = 0; j < PER_THREAD; j++) {
            const int ch = tid + MlaCfg::THREADS * j;
            const int row = ch / CHUNKS_PER_ROW, cc = ch % CHUNKS_PER_ROW;
            if (ch >= CHUNKS) continue;
            uint32_t o[8];
#pragma unroll
            for (int d = 0; d < 4; d++) {
                const uint32_t w = regs[j][d];
                const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
                const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
                o[2 * d] = pack_bf16_rne(lo.x, lo.y);
                o[2 * d + 1] = pack_bf16_rne(hi.x, hi.y);
            }
            auto* q = reinterpret_cast<lds_u32x4*>(dst + row * MlaCfg::ROW + cc * 32);
            q[0] = u32x4{o[0], o[1], o[2], o[3]};
            q[1] = u32x4{o[4], o[5], o[6], o[7]};
        }
        if (tid < MlaCfg::T) *reinterpret_cast<lds_f32*>(dst_scale + tid * 4) = scale;
    }
};

template <bool FP8>
__global__ __launch_bounds__(MlaCfg::THREADS, 1) void mla_decode_kernel(const AttnArgs a)
{
    using C = MlaCfg;
    extern __shared__ __align__(16) uint8_t smem_raw[];
    lds_byte* smem = (lds_byte*)smem_raw;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps wave-dependent addresses in SGPRs
    const int r = lane & 15, kc = lane >> 4;
    const int hq = wave & 3, th = wave >> 2;                      // score tile of this wave: head tile, token half

    // which (shard, split, sequence, head tile of HPW heads) this workgroup serves
    int u = blockIdx.x, si = 0;
    while (si + 1 < a.n_shards && u >= a.shard[si + 1].unit_base) si++;
    const ShardDev& sh = a.shard[si];
    u -= sh.unit_base;
    const int grp = u / (8 * a.head_tiles), j8 = u % (8 * a.head_tiles);
    const int logical = grp * 8 + (j8 & 7);
    const int htw = j8 >> 3;
    if (logical >= sh.n_splits * a.B) return;         // padding workgroup
    const int split = logical % sh.n_splits;
    const int b = logical / sh.n_splits;

    const int len = sh.len[b];
    const int t0 = split * a.split_tokens;
    const int t1 = min(t0 + a.split_tokens, len);
    const int h0 = htw * C::HPW;                      // first head of this workgroup
    const int nh = min(C::HPW, a.Q - h0);             // real heads (the rest is zero padding)
    const size_t rec = ((size_t)(sh.split_base + split) * a.B + b) * a.Q + h0;

    if (t0 >= len) {
        if (tid < nh) { a.ws_m[rec + tid] = -INFINITY; a.ws_l[rec + tid] = 0.f; }
        return;
    }

    // Q slice of this wave as the score MFMA's B operand: lane (r,kc) holds head 16hq + r of the
    // workgroup, dims 32*ks + 8*kc .. +8
    bf16x8 qb[C::KS];
    {
        const int hl = hq * 16 + r;
        const uint16_t* qrow = a.q + ((size_t)b * a.Q + h0 + min(hl, nh - 1)) * C::DK + kc * 8;
#pragma unroll
        for (int ks = 0; ks < C::KS; ks++) {
            u32x4 w = *reinterpret_cast<const u32x4*>(qrow + ks * 32);
            if (hl >= nh) w = u32x4{0, 0, 0, 0};
            qb[ks] = __builtin_bit_cast(bf16x8, w);
        }
    }

    const int esz = FP8 ? 1 : 2;
    const int64_t tok0 = (sh.tok_off ? sh.tok_off[b] : 0) + t0;
    const char* kbase = reinterpret_cast<const char*>(sh.k) + (int64_t)esz * ((int64_t)b * sh.k_sb + tok0 * sh.k_st);
    const float* sbase = FP8 ? sh.kv_scale + (int64_t)b * sh.s_sb + tok0 : nullptr;
    const uint32_t row_bytes = (uint32_t)sh.k_st * esz;

    const int n_tok = t1 - t0;
    const int n_tiles = (n_tok + C::T - 1) / C::T;

    float m_ref = -INFINITY;                          // reference exponent of head 16hq + r (integer-valued)
    float m_floor = -INFINITY;                        // lower bound for it after a restart
    float l_run = 0.f;                                // this lane's share of sum p over the wave's token halves
    f32x4 acc[C::DVT][C::NHT];                        // O^T[64w + 16d + 4kc + i][16h + r]

    auto ktile_of = [&](int it) { return smem + C::OFF_K + (it % C::NBUF) * C::TILE_BYTES; };

    // Scores of this wave's 16 heads against its 16 tokens of a latent tile in LDS.  The K operand
    // reads run PD operands ahead of the MFMAs that consume them.
    auto scores = [&](const lds_byte* ktile) {
        constexpr int PD = 4;
        bf16x8 kop[C::KS];
        const lds_byte* kp = ktile + (th * 16 + r) * C::ROW + kc * 16;
        auto rd = [&](int ks) { return __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4*>(kp + ks * 64)); };
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int o = 0; o < PD; o++) kop[o] = rd(o);
#pragma unroll
        for (int o = 0; o < C::KS; o++) {
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[o], qb[o], s, 0, 0, 0);
            if (o + PD < C::KS) kop[o + PD] = rd(o + PD);
        }
        return s;                                     // lane (r,kc): head r, tokens 16th + 4kc + i
    };

    // exponents (base 2) of the wave's scores, masked beyond the ragged end of the tile; returns this
    // lane's maximum over its 4 tokens (-inf if none is valid)
    auto exponents = [&](const f32x4& s, int kb, int n_valid, float (&t)[4], float (&fs)[4]) {
        if (FP8) {
            const f32x4 f = *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(
                smem + C::OFF_SCALE + kb * C::T * 4 + (th * 16 + kc * 4) * 4);
#pragma unroll
            for (int i = 0; i < 4; i++) fs[i] = f[i];
        }
        float bmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            float x = s[i] * a.scale_log2e;
            if (FP8) x *= fs[i];
            if (th * 16 + kc * 4 + i >= n_valid) x = -INFINITY;
            t[i] = x;
            bmax = fmaxf(bmax, x);
        }
        return bmax;
    };

    // weights of the wave's scores for the fixed reference, as bf16 hi + lo into LDS buffer pb
    auto weights = [&](const float (&t)[4], const float (&fs)[4], int pb) {
        float p[4];
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            p[i] = (t[i] == -INFINITY) ? 0.f : exp2_rel(t[i], m_ref);
            lsum += p[i];
            if (FP8) p[i] *= fs[i];
        }
        l_run += lsum;
        const uint32_t h01 = pack_bf16_rne(p[0], p[1]), h23 = pack_bf16_rne(p[2], p[3]);
        const uint32_t l01 = pack_bf16_rne(p[0] - as_f32(h01 << 16), p[1] - as_f32(h01 & 0xffff0000u));
        const uint32_t l23 = pack_bf16_rne(p[2] - as_f32(h23 << 16), p[3] - as_f32(h23 & 0xffff0000u));
        lds_byte* ph = smem + C::OFF_P + pb * 2 * C::P_BYTES + (hq * 16 + r) * (C::T * 2) + (th * 16 + kc * 4) * 2;
        *reinterpret_cast<lds_u32x2*>(ph) = u32x2{h01, h23};
        *reinterpret_cast<lds_u32x2*>(ph + C::P_BYTES) = u32x2{l01, l23};
    };

    // Softmax of a tile after the first.  The reference stays, so no maximum has to be agreed on
    // across lanes: every lane only checks its own 4 scores against the limit, and a ballot turns
    // that into this wave's restart flag (all lanes store the same word: no divergent branch).
    auto softmax = [&](const f32x4& s, int kb, int pb, int n_valid) {
        float t[4], fs[4];
        const float top = __builtin_ceilf(exponents(s, kb, n_valid, t, fs));
        const bool over = top > m_ref + C::kLimit;
        if (over) m_floor = fmaxf(m_floor, top + C::kHeadroom);
        *reinterpret_cast<lds_i32*>(smem + C::OFF_FLAG + (pb * C::WAVES + wave) * 4) = __any(over) ? 1 : 0;
        weights(t, fs, pb);
    };

    // Did any wave ask for a restart while it computed the weights of tile buffer `pb`?  (uniform)
    auto overflowed = [&](int pb) {
        const auto f0 = *reinterpret_cast<const lds_u32x4*>(smem + C::OFF_FLAG + pb * 32);
        const auto f1 = *reinterpret_cast<const lds_u32x4*>(smem + C::OFF_FLAG + pb * 32 + 16);
        return (f0.x | f0.y | f0.z | f0.w | f1.x | f1.y | f1.z | f1.w) != 0;
    };

    // O^T[value cols of this wave, all heads of the workgroup] += V^T . P^T for one tile.  The four
    // V^T operands stay in registers; the weights are fetched one head tile at a time (hi, lo).
    auto pv = [&](const lds_byte* ktile, int pb) {
        const lds_byte* pp = smem + C::OFF_P + pb * 2 * C::P_BYTES + r * (C::T * 2) + kc * 16;
        // V^T operand: lane (r,kc) ends up with value column 64w + 16d + r, tokens 8kc .. 8kc+7
        const lds_byte* vp = ktile + (kc * 8 + (r >> 2)) * C::ROW + (wave * 64 + (r & 3) * 4) * 2;
        bf16x8 va[C::DVT];
#pragma unroll
        for (int d = 0; d < C::DVT; d++) {
            const u32x2 v0 = lds_read_tr16(vp + d * 32), v1 = lds_read_tr16(vp + d * 32 + 4 * C::ROW);
            va[d] = __builtin_bit_cast(bf16x8, u32x4{v0.x, v0.y, v1.x, v1.y});
        }
        bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4*>(pp));
        bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4*>(pp + C::P_BYTES));
#pragma unroll
        for (int h = 0; h < C::NHT; h++) {
            const bf16x8 ch = bh, cl = bl;
            if (h + 1 < C::NHT) {
                bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4*>(pp + (h + 1) * 16 * (C::T * 2)));
                bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const lds_u32x4*>(pp + (h + 1) * 16 * (C::T * 2) + C::P_BYTES));
            }
#pragma unroll
            for (int d = 0; d < C::DVT; d++) acc[d][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[d], ch, acc[d][h], 0, 0, 0);
#pragma unroll
            for (int d = 0; d < C::DVT; d++) acc[d][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[d], cl, acc[d][h], 0, 0, 0);
        }
    };

    // Tile `it` on its way into LDS: e4m3 rows pass through registers, bf16 rows are copied by the
    // LDS DMA.  issue() starts the loads, commit() completes the tile as far as this thread is
    // concerned; a barrier then publishes it.
    MlaStageFp8 stage;
    auto stage_issue = [&](int it) {
        const int nv = min(C::T, n_tok - it * C::T);
        if constexpr (FP8) stage.load(kbase + (size_t)it * C::T * row_bytes, row_bytes, sbase + it * C::T, nv, tid);
        else MlaDma::issue(kbase + (size_t)it * C::T * row_bytes, row_bytes, nv, ktile_of(it), wave, lane);
    };
    auto stage_commit = [&](int it) {
        if constexpr (FP8) stage.store(ktile_of(it), smem + C::OFF_SCALE + (it % C::NBUF) * C::T * 4, tid);
        else MlaDma::commit(min(C::T, n_tok - it * C::T), ktile_of(it), wave, lane);
    };

    // The outer loop runs once unless the reference exponent turned out too low.
    for (;;) {
        l_run = 0.f;
#pragma unroll
        for (int d = 0; d < C::DVT; d++)
#pragma unroll
            for (int h = 0; h < C::NHT; h++) acc[d][h] = f32x4{0.f, 0.f, 0.f, 0.f};

        // ---- tile 0: fixes the reference exponent of every head ----
        stage_issue(0);
        stage_commit(0);
        __syncthreads();
        if (n_tiles > 1) stage_issue(1);
        {
            const f32x4 s = scores(ktile_of(0));
            float t[4], fs[4];
            const float top = wave_xor_max_16_32(exponents(s, 0, min(C::T, n_tok), t, fs));   // over the wave's 16 tokens
            // the two waves that share these heads exchange the maxima of their token halves
            if (kc == 0) *reinterpret_cast<lds_f32*>(smem + C::OFF_TOP + (th * C::HPW + hq * 16 + r) * 4) = top;
            __syncthreads();
            const float top2 = fmaxf(*reinterpret_cast<const lds_f32*>(smem + C::OFF_TOP + (hq * 16 + r) * 4),
                                     *reinterpret_cast<const lds_f32*>(smem + C::OFF_TOP + (C::HPW + hq * 16 + r) * 4));
            m_ref = fmaxf(__builtin_ceilf(top2) + C::kHeadroom, m_floor);        // finite: token 0 is valid
            *reinterpret_cast<lds_i32*>(smem + C::OFF_FLAG + wave * 4) = 0;
            weights(t, fs, 0);
        }
        if (n_tiles > 1) stage_commit(1);
        __syncthreads();

        // ---- tiles 1 .. n-1, one barrier each; P.V runs one tile behind the scores ----
        bool restart = false;
        for (int it = 1; it < n_tiles; it++) {
            const bool has_next = it + 1 < n_tiles;
            if (has_next) stage_issue(it + 1);
            const int nv = min(C::T, n_tok - it * C::T);
            if (__builtin_expect(overflowed((it - 1) & 1), 0)) { restart = true; break; }
            {
                const f32x4 s = scores(ktile_of(it));
                softmax(s, it % C::NBUF, it & 1, nv);
                pv(ktile_of(it - 1), (it - 1) & 1);
            }
            if (has_next) stage_commit(it + 1);
            __syncthreads();
        }
        if (!restart && !overflowed((n_tiles - 1) & 1)) {
            pv(ktile_of(n_tiles - 1), (n_tiles - 1) & 1);
            break;
        }
        // Start over.  Heads share their reference between two waves: publish the raised floors.
        __syncthreads();                              // everybody has left the tile loop and the LDS buffers
        m_floor = wave_xor_max_16_32(m_floor);        // the four lanes of a head saw different tokens
        if (kc == 0) *reinterpret_cast<lds_f32*>(smem + C::OFF_TOP + (th * C::HPW + hq * 16 + r) * 4) = m_floor;
        __syncthreads();
        m_floor = fmaxf(*reinterpret_cast<const lds_f32*>(smem + C::OFF_TOP + (hq * 16 + r) * 4),
                        *reinterpret_cast<const lds_f32*>(smem + C::OFF_TOP + (C::HPW + hq * 16 + r) * 4));
        __syncthreads();
    }

    // ---- the workgroup's record: un-normalised O, reference exponent and normaliser per head ----
    {
        const float l = wave_xor_sum_16_32(l_run);    // this wave's token halves
        __syncthreads();
        if (th == 1 && kc == 0) *reinterpret_cast<lds_f32*>(smem + C::OFF_TOP + (hq * 16 + r) * 4) = l;
        __syncthreads();
        const int hl = hq * 16 + r;
        if (th == 0 && kc == 0 && hl < nh) {
            a.ws_m[rec + hl] = m_ref;
            a.ws_l[rec + hl] = l + *reinterpret_cast<const lds_f32*>(smem + C::OFF_TOP + hl * 4);
        }
    }
#pragma unroll
    for (int h = 0; h < C::NHT; h++) {
        const int hl = h * 16 + r;
        if (hl < nh) {
            float* orow = a.ws_o + (rec + hl) * C::DV + wave * 64 + kc * 4;
#pragma unroll
            for (int d = 0; d < C::DVT; d++) *reinterpret_cast<f32x4*>(orow + d * 16) = acc[d][h];
        }
    }
}

}  // namespace helix

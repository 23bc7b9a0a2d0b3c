// Split-KV decode attention for the MLA case on gfx950: 128 query heads attending ONE shared latent
// whose 576-wide row is the key and whose first 512 entries are the value (Sec. 1, Sec. 3:
// "a single latent representation of both K and V for all Q heads"), per-shard attention of Helix's
// attention phase (Sec. 2.1.1).  Latent stored as bf16, or as e4m3 codes with one fp32 scale per token.
//
// This is the dense contraction of the path (242 flop per latent byte in bf16, 480 in e4m3): it is
// MFMA-bound, so the design question is how to feed the matrix cores, not HBM.
//
//   Workgroup = 4 wavefronts = one CU, HPW = 64 of the heads, a run of `split_tokens` latent rows in
//   tiles of 32 tokens.  (All 128 heads in one workgroup would need 256 accumulator + 144 query
//   registers per lane and left the compiler spilling; with 64 heads the two workgroups of a token
//   range sit on the same XCD and the second one's latent reads hit that XCD's L2.)  Each latent
//   tile is parked in LDS (row stride padded to 1184 B so that MFMA-operand reads of 16 rows x 64 B
//   hit 64 distinct banks) and used twice:
//
//   scores  S^T[token, head] = K . Q^T      wave w owns heads 16w..16w+15 of the workgroup with its
//           Q slice (16 x 576 bf16 = 72 VGPRs) stationary in registers; K operands come from LDS.
//   softmax per wave on its own heads with an integer reference exponent that stays fixed for the
//           whole run of tokens (see the kernel); the weights (bf16 hi + lo) go to LDS.
//   P.V     O^T[dv, head] += V^T . P^T     wave w owns value columns 128w..128w+127 for ALL heads
//           of the workgroup (64 x 128 fp32 accumulators = 128 registers).  V^T operands come
//           straight out of the row-major latent tile with the transposing LDS read
//           (ds_read_b64_tr_b16), P^T operands from the weights the four waves just wrote.
//
//   LDS traffic per 32-token tile and wave: 36 KB (K) + 8 KB (V) + 8 KB (P) + 2 KB (P writes) over
//   1600 MFMA cycles = 135 B/clk per CU, half of the 256 B/clk the CU's LDS delivers for 128-bit
//   reads (measured 214-223 B/clk).
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
    static constexpr int NBUF = 3;                // latent tiles in flight in LDS
    static constexpr int TILE_BYTES = T * ROW;    // 37888
    static constexpr int HPW = 64;                // heads per workgroup
    static constexpr int NHT = HPW / 16;          // head tiles of the P.V product
    static constexpr int QHT = HPW / 64;          // head tiles per wave in the score product
    static constexpr int P_BYTES = HPW * T * 2;   // one of hi / lo: [HPW heads][32 tokens] bf16
    // LDS map
    static constexpr int OFF_K = 0;
    static constexpr int OFF_P = NBUF * TILE_BYTES;               // [2 buffers][hi, lo]
    static constexpr int OFF_FLAG = OFF_P + 2 * 2 * P_BYTES;      // [2][4] int: a wave asks for a restart
    static constexpr int OFF_SCALE = OFF_FLAG + 2 * 4 * 4;        // [NBUF][32] fp32 per-token scales
    static constexpr int LDS_BYTES = OFF_SCALE + NBUF * T * 4;
};

typedef __attribute__((address_space(3))) uint8_t lds_byte;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Transposing LDS read: within each group of 16 lanes, lane i receives the 16-bit element (i % 4) of
// the 8-byte rows supplied by lanes 4e + i/4, e = 0..3 (checked on the device).
__device__ __forceinline__ u32x2 lds_read_tr16(const lds_byte* p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    return __builtin_bit_cast(u32x2, v);
}

// Stages the latent tile whose first token row is at `src` into LDS buffer `dst`: bf16 rows are
// copied, e4m3 rows widened to bf16.  Rows >= n_valid are zero-filled.  `regs` decouples the global
// loads (issued early) from the LDS writes (done after the tile's consumers are known to be idle).
template <bool FP8>
struct MlaStage {
    static constexpr int CHUNKS_PER_ROW = FP8 ? 36 : 72;           // 16-byte global chunks
    static constexpr int CHUNKS = MlaCfg::T * CHUNKS_PER_ROW;
    static constexpr int PER_THREAD = (CHUNKS + 255) / 256;        // 9 (bf16) or 5 (e4m3)
    u32x4 regs[PER_THREAD];
    float scale;                                                    // e4m3: thread t < 32 holds token t's scale

    __device__ __forceinline__ void load(const char* src, uint32_t row_bytes, const float* scales, int n_valid, int tid)
    {
#pragma unroll
        for (int j = 0; j < PER_THREAD; j++) {
            const int ch = tid + 256 * j;
            const int row = ch / CHUNKS_PER_ROW, cc = ch % CHUNKS_PER_ROW;
            regs[j] = u32x4{0, 0, 0, 0};
            if (ch < CHUNKS && row < n_valid)
                regs[j] = *reinterpret_cast<const u32x4*>(src + (size_t)row * row_bytes + cc * 16);   // plain load: the sibling workgroup re-reads it from L2
        }
        if (FP8) scale = (tid < n_valid && tid < MlaCfg::T) ? scales[tid] : 0.f;
    }

    __device__ __forceinline__ void store(lds_byte* dst, lds_byte* dst_scale, int tid) const
    {
#pragma unroll
        for (int j = 0; j < PER_THREAD; j++) {
            const int ch = tid + 256 * j;
            const int row = ch / CHUNKS_PER_ROW, cc = ch % CHUNKS_PER_ROW;
            if (ch >= CHUNKS) continue;
            if (!FP8) {
                *reinterpret_cast<__attribute__((address_space(3))) u32x4*>(dst + row * MlaCfg::ROW + cc * 16) = regs[j];
            } else {
                // 16 codes -> 16 bf16 (exact: e4m3 has 3 mantissa bits and a 4-bit exponent)
                uint32_t o[8];
#pragma unroll
                for (int d = 0; d < 4; d++) {
                    const uint32_t w = regs[j][d];
                    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
                    const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w, true);
                    o[2 * d] = pack_bf16_rne(lo.x, lo.y);
                    o[2 * d + 1] = pack_bf16_rne(hi.x, hi.y);
                }
                auto* q = reinterpret_cast<__attribute__((address_space(3))) u32x4*>(dst + row * MlaCfg::ROW + cc * 32);
                q[0] = u32x4{o[0], o[1], o[2], o[3]};
                q[1] = u32x4{o[4], o[5], o[6], o[7]};
            }
        }
        if (FP8 && tid < MlaCfg::T) *reinterpret_cast<__attribute__((address_space(3))) float*>(dst_scale + tid * 4) = scale;
    }
};

// Workgroups of one shard are numbered so that the head tiles of the same token range are 8 apart:
// consecutive workgroup ids go round-robin over the 8 XCDs, so ids that differ by 8 share an XCD
// and with it an L2.  Shards are padded to a multiple of 8 token ranges (padding workgroups exit).
__host__ __device__ inline int mla_units_of_shard(int n_splits, int B, int head_tiles)
{
    return (n_splits * B + 7) / 8 * 8 * head_tiles;
}

template <bool FP8>
__global__ __launch_bounds__(256, 1) void mla_decode_kernel(const AttnArgs a)
{
    using C = MlaCfg;
    extern __shared__ __align__(16) uint8_t smem_raw[];
    lds_byte* smem = (lds_byte*)smem_raw;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kc = lane >> 4;

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

    // Q slice of this wave as the score MFMA's B operand: lane (r,kc) holds head 16w + r of the
    // workgroup, dims 32*ks + 8*kc .. +8
    bf16x8 qb[C::KS];
    {
        const int hl = wave * 16 + r;
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

    float m_run = -INFINITY;                          // reference exponent of head 16w + r (integer-valued)
    float m_floor = -INFINITY;                        // lower bound for it after a restart
    float l_run = 0.f;
    f32x4 acc[8][C::NHT];                             // [dv tile][head tile]: O^T[128w + 16*dvt + 4*kc + i][16*ht + r]

    // Scores of this wave's 16 heads against the 32 tokens of a latent tile in LDS.  The K operand
    // reads run PD operands ahead of the MFMAs that consume them (one wave per SIMD: nothing else
    // hides the LDS latency).
    auto scores = [&](const lds_byte* ktile, f32x4 (&s)[2]) {
        constexpr int NOP = 2 * C::KS, PD = 8;
        bf16x8 kop[NOP];
        const lds_byte* kp = ktile + r * C::ROW + kc * 16;
        auto rd = [&](int o) {   // operand o = 2*ks + tt: rows 16tt + r, dims 32ks + 8kc .. +8
            return __builtin_bit_cast(bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(
                                                  kp + (o & 1) * 16 * C::ROW + (o >> 1) * 64));
        };
        s[0] = s[1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int o = 0; o < PD; o++) kop[o] = rd(o);
        __builtin_amdgcn_sched_group_barrier(0x100, PD, 0);      // PD LDS reads up front ...
#pragma unroll
        for (int o = 0; o < NOP; o++) {
            s[o & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[o], qb[o >> 1], s[o & 1], 0, 0, 0);
            if (o + PD < NOP) kop[o + PD] = rd(o + PD);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // ... then MFMA, read, MFMA, read, ...
            if (o + PD < NOP) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    // Softmax of one tile's scores on the wave's own heads: new integer reference exponent, the
    // rescale factor for everybody's accumulators, weights as bf16 hi + lo into LDS.
    auto softmax = [&](const f32x4 (&s)[2], int kb, int pb, int n_valid, bool first) {
        lds_byte* phi = smem + C::OFF_P + pb * 2 * C::P_BYTES;
        lds_byte* plo = phi + C::P_BYTES;
        float fscale[2][4];                           // e4m3: per-token scales of this lane's tokens
        if (FP8) {
#pragma unroll
            for (int tt = 0; tt < 2; tt++) {
                const f32x4 f = *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(
                    smem + C::OFF_SCALE + kb * C::T * 4 + (tt * 16 + kc * 4) * 4);
#pragma unroll
                for (int i = 0; i < 4; i++) fscale[tt][i] = f[i];
            }
        }
        float t[2][4];
        float bmax = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < 2; tt++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                float x = s[tt][i] * a.scale_log2e;
                if (FP8) x *= fscale[tt][i];
                if (tt * 16 + kc * 4 + i >= n_valid) x = -INFINITY;
                t[tt][i] = x;
                bmax = fmaxf(bmax, x);
            }
        bmax = wave_xor_max_16_32(bmax);
        // Reference exponent: fixed for the whole run of tokens at kHeadroom octaves above the first
        // tile's maximum (or at m_floor after a restart), so the 128 accumulator registers of every
        // wave never need a rescale inside the loop.  Any integer reference gives the same result up
        // to fp32 rounding of the sums: weights are exact powers of two times a significand that
        // does not depend on the reference.  A later tile whose maximum exceeds the reference by
        // more than kLimit octaves (weights near 2^64; never seen on real logits) raises the flag
        // that makes the whole workgroup start the run over with a higher reference.
        constexpr float kHeadroom = 32.f, kLimit = 64.f;
        const float top = __builtin_ceilf(bmax);                         // finite: token 0 of a tile is valid
        if (first) m_run = fmaxf(top + kHeadroom, m_floor);
        const bool over = top > m_run + kLimit;
        if (over) m_floor = top + kHeadroom;
        const bool any = __any(over);
        if (lane == 0) *reinterpret_cast<__attribute__((address_space(3))) int*>(smem + C::OFF_FLAG + (pb * 4 + wave) * 4) = any ? 1 : 0;
        const float m_new = m_run;
        float lsum = 0.f;
#pragma unroll
        for (int tt = 0; tt < 2; tt++) {
            float p[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                p[i] = (t[tt][i] == -INFINITY) ? 0.f : exp2_rel(t[tt][i], m_new);
                lsum += p[i];
                if (FP8) p[i] *= fscale[tt][i];
            }
            const uint32_t h01 = pack_bf16_rne(p[0], p[1]), h23 = pack_bf16_rne(p[2], p[3]);
            const uint32_t l01 = pack_bf16_rne(p[0] - as_f32(h01 << 16), p[1] - as_f32(h01 & 0xffff0000u));
            const uint32_t l23 = pack_bf16_rne(p[2] - as_f32(h23 << 16), p[3] - as_f32(h23 & 0xffff0000u));
            const int off = (wave * 16 + r) * (C::T * 2) + (tt * 16 + kc * 4) * 2;
            *reinterpret_cast<__attribute__((address_space(3))) u32x2*>(phi + off) = u32x2{h01, h23};
            *reinterpret_cast<__attribute__((address_space(3))) u32x2*>(plo + off) = u32x2{l01, l23};
        }
        l_run += lsum;
    };

    // Did any wave ask for a restart while it computed the weights of tile `pb`?  (workgroup-uniform)
    auto overflowed = [&](int pb) {
        const auto fl = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(smem + C::OFF_FLAG + pb * 16);
        return (fl.x | fl.y | fl.z | fl.w) != 0;
    };

    // O^T[value cols of this wave, all heads of the workgroup] += V^T . P^T for one tile.
    auto pv = [&](const lds_byte* ktile, int pb) {
        const lds_byte* phi = smem + C::OFF_P + pb * 2 * C::P_BYTES;
        const lds_byte* plo = phi + C::P_BYTES;
        bf16x8 bh[C::NHT], bl[C::NHT];
#pragma unroll
        for (int h = 0; h < C::NHT; h++) {
            const int off = (h * 16 + r) * (C::T * 2) + kc * 16;
            bh[h] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(phi + off));
            bl[h] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(plo + off));
        }
#pragma unroll
        for (int d = 0; d < 8; d++) {
            // V^T operand: lane (r,kc) ends up with value column 128w + 16d + r, tokens 8kc .. 8kc+7
            const lds_byte* vp = ktile + (kc * 8 + (r >> 2)) * C::ROW + (wave * 128 + d * 16 + (r & 3) * 4) * 2;
            const u32x2 v0 = lds_read_tr16(vp);
            const u32x2 v1 = lds_read_tr16(vp + 4 * C::ROW);
            const bf16x8 va = __builtin_bit_cast(bf16x8, u32x4{v0.x, v0.y, v1.x, v1.y});
#pragma unroll
            for (int h = 0; h < C::NHT; h++) acc[d][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, bh[h], acc[d][h], 0, 0, 0);
#pragma unroll
            for (int h = 0; h < C::NHT; h++) acc[d][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, bl[h], acc[d][h], 0, 0, 0);
        }
    };

    auto ktile_of = [&](int it) { return smem + C::OFF_K + (it % C::NBUF) * C::TILE_BYTES; };
    auto stage_load = [&](MlaStage<FP8>& st, int it) {
        st.load(kbase + (size_t)it * C::T * row_bytes, row_bytes, FP8 ? sbase + it * C::T : nullptr,
                min(C::T, n_tok - it * C::T), tid);
    };
    auto stage_store = [&](const MlaStage<FP8>& st, int it) {
        st.store(ktile_of(it), smem + C::OFF_SCALE + (it % C::NBUF) * C::T * 4, tid);
    };

    // Pipeline over tiles, one barrier per tile.  In iteration `it` a wave computes the scores of
    // tile it, then runs the MFMAs of P.V for tile it-1 in the same straight-line block as the VALU
    // work of tile it's softmax, so the matrix pipe stays fed while the exponentials issue.
    //   LDS tiles: it-1 (values), it (keys), it+1 (being filled) -> three buffers; weights of tile
    //   it-1 are read while those of tile it are written -> two buffers.
    // The outer loop runs once unless a reference exponent turned out too low (see the softmax).
    for (;;) {
        l_run = 0.f;
#pragma unroll
        for (int d = 0; d < 8; d++)
#pragma unroll
            for (int h = 0; h < C::NHT; h++) acc[d][h] = f32x4{0.f, 0.f, 0.f, 0.f};
        MlaStage<FP8> stage;
        stage_load(stage, 0);
        stage_store(stage, 0);
        if (n_tiles > 1) stage_load(stage, 1);
        __syncthreads();
        {
            f32x4 s[2];
            scores(ktile_of(0), s);
            softmax(s, 0, 0, min(C::T, n_tok), true);
        }
        if (n_tiles > 1) stage_store(stage, 1);
        __syncthreads();
        bool restart = false;
        int it = 1;
        for (; it < n_tiles; it++) {
            const bool has_next = it + 1 < n_tiles;
            if (has_next) stage_load(stage, it + 1);
            f32x4 s[2];
            scores(ktile_of(it), s);
            if (__builtin_expect(overflowed((it - 1) & 1), 0)) { restart = true; break; }
            pv(ktile_of(it - 1), (it - 1) & 1);
            softmax(s, it % C::NBUF, it & 1, min(C::T, n_tok - it * C::T), false);
            if (has_next) stage_store(stage, it + 1);
            __syncthreads();
        }
        if (!restart && !overflowed((n_tiles - 1) & 1)) {
            pv(ktile_of(n_tiles - 1), (n_tiles - 1) & 1);
            break;
        }
        __syncthreads();                              // everybody has left the LDS buffers: start over
    }

    // ---- the workgroup's record: un-normalised O, reference exponent and normaliser per head ----
    {
        const float l = wave_xor_sum_16_32(l_run);
        const int hl = wave * 16 + r;
        if (kc == 0 && hl < nh) { a.ws_m[rec + hl] = m_run; a.ws_l[rec + hl] = l; }
    }
    // a wave knows the final reference exponent only of its own heads, but the accumulators of all
    // heads were rescaled tile by tile with the owners' factors, so they already match them.
#pragma unroll
    for (int h = 0; h < C::NHT; h++) {
        const int hl = h * 16 + r;
        if (hl < nh) {
            float* orow = a.ws_o + (rec + hl) * C::DV + wave * 128 + kc * 4;
#pragma unroll
            for (int d = 0; d < 8; d++) *reinterpret_cast<f32x4*>(orow + d * 16) = acc[d][h];
        }
    }
}

}  // namespace helix

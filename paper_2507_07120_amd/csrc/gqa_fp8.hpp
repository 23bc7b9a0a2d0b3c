// Split-KV decode attention for GQA/MQA groups with the KV cache in fp8: OCP e4m3 codes and one fp32 scale per
// (sequence, kv head, token) that the token's key row and value row share (value = code * scale) -- the fp8 KV
// streaming of the per-shard attention of Helix's attention phase (Sec. 2.1.1), dk == dv == 128: 264 bytes per token
// and KV head against 512 in bf16.
//
// Same decomposition and the same arithmetic after dequantisation as the bf16 kernel (gqa_decode.hpp): a workgroup
// of 4 waves serves runs of consecutive tokens of (shard, sequence, kv head, head tile) rows, the waves take
// alternating 32-token blocks, scores / integer-reference softmax / P.V run on 16x16x32 bf16 MFMAs.  What differs is
// how the operands get into registers:
//   K   lane (r = token, kc) loads the 32 bytes holding dims 32kc .. 32kc+31 of its token (two 16-byte loads; a wave
//       instruction covers 16 whole rows).  The score contraction does not care about the order of the dims as long
//       as Q agrees, so k-step s takes dims 32kc + 8s .. +8 from every lane (Q is loaded to match).
//   V   lane (r, kc) owns value columns 8r .. 8r+7 (8 bytes per token) of its 8 tokens, as in the bf16 kernel; the
//       8x8 transpose happens after the conversion.
//   dequantisation  v_cvt_scalef32_pk_bf16_fp8 with scale 1 turns two codes into two bf16 (exact: e4m3 has three
//       mantissa bits), right before the MFMA that consumes them: 64 conversions per lane and 32-token block.
//   the token's scale f_t is not a power of two, so it never touches an operand: it multiplies the token's score
//       (s_t = f_t * q.k8_t) and its weight (w_t = p_t * f_t, then the bf16 hi/lo split), both in fp32; the normaliser
//       sums the p_t.
#pragma once
#include "gqa_decode.hpp"

namespace helix {

typedef __bf16 f8_bf16x2 __attribute__((ext_vector_type(2)));
typedef u32x4 f8_u32x4_a4 __attribute__((aligned(4)));       // 16-byte loads that are only dword aligned
typedef f32x4 f8_f32x4_a4 __attribute__((aligned(4)));

struct F8Raw {
    u32x4 k[2][2];     // codes of dims 32kc..32kc+31 of tokens r, 16 + r
    u32x2 v[8];        // codes of columns 8r..8r+7 of the lane's 8 tokens
    f32x4 fs[2];       // scales of tokens 4kc..4kc+3 and 16 + 4kc .. +3
};

// Loads the block of 32 tokens whose first rows are kblk / vblk (codes, row strides in bytes) and whose first scale
// is sblk.  TAIL: tokens >= n_valid are redirected to the last valid row (their weights are zero later).
template <bool TAIL, bool NT>
__device__ __forceinline__ void f8_load_block(F8Raw& raw, const char* kblk, const char* vblk, const float* sblk,
                                              uint32_t k_row_bytes, uint32_t v_row_bytes, int r, int kc, int n_valid)
{
#pragma unroll
    for (int a = 0; a < 2; a++) {
        int tok = a * 16 + r;
        if (TAIL) tok = min(tok, n_valid - 1);
        const char* p = kblk + (uint32_t)((uint32_t)tok * k_row_bytes + (uint32_t)kc * 32u);
        raw.k[a][0] = stream_load<NT>(reinterpret_cast<const u32x4*>(p));
        raw.k[a][1] = stream_load<NT>(reinterpret_cast<const u32x4*>(p + 16));
    }
#pragma unroll
    for (int j = 0; j < 8; j++) {
        int tok = (j >> 2) * 16 + kc * 4 + (j & 3);
        if (TAIL) tok = min(tok, n_valid - 1);
        raw.v[j] = stream_load<NT>(reinterpret_cast<const u32x2*>(vblk + (uint32_t)((uint32_t)tok * v_row_bytes + (uint32_t)r * 8u)));
    }
    if (TAIL) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int tok = min((j >> 2) * 16 + kc * 4 + (j & 3), n_valid - 1);
            raw.fs[j >> 2][j & 3] = stream_load<NT>(sblk + tok);
        }
    } else {
#pragma unroll
        for (int a = 0; a < 2; a++) {
            const f8_f32x4_a4* sp = reinterpret_cast<const f8_f32x4_a4*>(sblk + a * 16 + kc * 4);     // (dword aligned only)
            if constexpr (NT) raw.fs[a] = __builtin_nontemporal_load(sp);
            else raw.fs[a] = *sp;
        }
    }
}

// The two e4m3 codes in half `hi` of a dword as a bf16 pair.
__device__ __forceinline__ uint32_t f8_pair(uint32_t codes, bool hi)
{
    const f8_bf16x2 p = hi ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, true)
                           : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes, 1.0f, false);
    return __builtin_bit_cast(uint32_t, p);
}

// One 32-token block straight from the raw codes: every operand is converted right before the MFMA that consumes it
// (K: 4 conversions per k-step; V: the 16 bits holding columns 2p, 2p+1 of the lane's 8 tokens -> 8 conversions, then
// the 16-bit transpose), so no dequantised copy of the block is kept.
template <bool TAIL>
__device__ __forceinline__ void f8_compute_block(GqaState<128>& st, const F8Raw& raw, const bf16x8 (&qb)[4],
                                                 float scale_log2e, int kc, int n_valid)
{
    const float fs[8] = {raw.fs[0][0], raw.fs[0][1], raw.fs[0][2], raw.fs[0][3], raw.fs[1][0], raw.fs[1][1], raw.fs[1][2], raw.fs[1][3]};
    uint32_t pairs[8];            // columns (2p, 2p+1) of the lane's 8 tokens, refreshed at every even column
    gqa_compute_core<128, TAIL, true>(
        st,
        [&](int a, int s) {
            const uint32_t w0 = raw.k[a][s >> 1][(s & 1) * 2], w1 = raw.k[a][s >> 1][(s & 1) * 2 + 1];
            return __builtin_bit_cast(bf16x8, u32x4{f8_pair(w0, false), f8_pair(w0, true), f8_pair(w1, false), f8_pair(w1, true)});
        },
        [&](int c) {
            if ((c & 1) == 0) {
#pragma unroll
                for (int j = 0; j < 8; j++) pairs[j] = f8_pair(raw.v[j][c >> 2], ((c >> 1) & 1) != 0);
            }
            return gqa_column_of_pairs(pairs, c);
        },
        qb, scale_log2e, kc, n_valid, fs);
}

// SHARED: several head tiles per kv head, side by side (StreamSeat), ordinary loads.
template <bool SHARED>
__global__ __launch_bounds__(256, 2) void gqa_fp8_kernel(const AttnArgs a)
{
    constexpr int D = 128;
    constexpr bool NT = !SHARED;
    using C = GqaCfg<D>;

    // This workgroup's share of the launch: an equal range of its head tile's rows laid end to end (stream_self_plan),
    // served run by run -- one run, and one split record, per row the range touches.
    __shared__ int64_t plan_scratch[256 / 64 + 5];
    const int rows_per_pair = a.K;
    StreamCursor cursor;
    if (!stream_self_plan<256>(a, kGqaTile, rows_per_pair, plan_scratch, a.prefix_out, cursor)) return;
    StreamRun run;
    while (stream_next_run(a, cursor, kGqaTile, rows_per_pair, run)) {
    // (the lane's coordinates are derived anew in every run, so that nothing computed from them is kept across runs)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, kc = lane >> 4;
    gqa_note_run(a, run);
    const ShardDev& sh = a.shard[run.si];
    const int b = run.b, kh = run.kh, ht = run.ht;

    const int len = cursor.len;                      // of the slice the run belongs to (the cursor's current pair)
    const int64_t first_row = cursor.first_row;
    const int t0 = run.t0;
    const int t1 = min(run.t1_cap, len);
    const int h0 = kh * a.g + ht * 16;
    const int nh = min(16, a.g - ht * 16);
    const size_t rec = (size_t)run.slot * 16;            // a record holds the 16 head rows of the tile

    // strides count elements = bytes
    const int64_t tok0 = first_row + t0;
    const char* kbase = reinterpret_cast<const char*>(sh.k) + ((int64_t)b * sh.k_sb + (int64_t)kh * sh.k_sh + tok0 * sh.k_st);
    const char* vbase = reinterpret_cast<const char*>(sh.v) + ((int64_t)b * sh.v_sb + (int64_t)kh * sh.v_sh + tok0 * sh.v_st);
    const float* sbase = sh.kv_scale + ((int64_t)b * sh.s_sb + (int64_t)kh * sh.s_sh + tok0);
    const uint32_t k_row_bytes = (uint32_t)sh.k_st, v_row_bytes = (uint32_t)sh.v_st;

    GqaState<D> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int c = 0; c < C::CPL; c++) st.o[c] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int n_tok = max(t1 - t0, 0);
    const int n_full = n_tok / C::TB;
    const int n_blk = (n_tok + C::TB - 1) / C::TB;
    const int nw = n_full > wave ? (n_full - wave + 3) / 4 : 0;       // this wave's full blocks: wave, wave+4, ...
    const size_t k_blk_bytes = (size_t)C::TB * k_row_bytes, v_blk_bytes = (size_t)C::TB * v_row_bytes;

    // block i of this wave; loads are never issued under a condition of their own (the compiler's wait counts
    // stay exact): a prefetch past the end re-reads the wave's last block
    auto load = [&](F8Raw& raw, int i) {
        const size_t blk = (size_t)(wave + 4 * min(i, nw - 1));
        f8_load_block<false, NT>(raw, kbase + blk * k_blk_bytes, vbase + blk * v_blk_bytes, sbase + blk * C::TB, k_row_bytes, v_row_bytes, r, kc, C::TB);
    };
    F8Raw r0, r1;
    // the ragged last block of the run, if any, belongs to wave (n_full % 4), which takes it first (requested together
    // with the wave's first full block, so that nobody waits for it at the end of the run)
    const bool tail_mine = n_blk > n_full && (n_full & 3) == wave;
    const int n_tail = n_tok - n_full * C::TB;
    if (tail_mine) f8_load_block<true, NT>(r1, kbase + n_full * k_blk_bytes, vbase + n_full * v_blk_bytes, sbase + (size_t)n_full * C::TB, k_row_bytes, v_row_bytes, r, kc, n_tail);
    if (nw > 0) load(r0, 0);

    // Q as the score MFMA's B operand, in the dim order of the K operand: lane (r,kc) holds head r,
    // dims 32kc + 8s .. +8 for k-step s
    bf16x8 qb[C::KS];
    {
        const uint16_t* qrow = a.q + ((size_t)b * a.Q + h0 + min(r, nh - 1)) * D + kc * 32;
#pragma unroll
        for (int s = 0; s < C::KS; s++) {
            u32x4 w = *reinterpret_cast<const u32x4*>(qrow + s * 8);
            if (r >= nh) w = u32x4{0, 0, 0, 0};
            qb[s] = __builtin_bit_cast(bf16x8, w);
        }
    }

    if (tail_mine) f8_compute_block<true>(st, r1, qb, a.scale_log2e, kc, n_tail);
    if (nw > 0) {
        int i = 0;
        for (; i + 2 <= nw; i += 2) {
            load(r1, i + 1);
            f8_compute_block<false>(st, r0, qb, a.scale_log2e, kc, C::TB);
            load(r0, i + 2);
            f8_compute_block<false>(st, r1, qb, a.scale_log2e, kc, C::TB);
        }
        if (i < nw) f8_compute_block<false>(st, r0, qb, a.scale_log2e, kc, C::TB);
    }

    gqa_emit_record<D>(st, a, rec, nh, tid, wave, r, kc);
    lds_barrier();                    // the record's staging area in LDS is free for the next run (its stores may still be on their way)
    }
}

}  // namespace helix

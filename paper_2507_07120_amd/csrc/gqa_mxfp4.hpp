// Split-KV decode attention for GQA/MQA groups with the KV cache in MXFP4 -- the FP4 the paper's
// evaluation assumes for KV states (Sec. 3; microscaling formats: E2M1 elements, blocks of 32 along a
// row sharing one E8M0 power-of-two scale).  dk == dv == 128: a token's key or value row is 64 bytes
// of codes plus 4 scale bytes, 3.8x fewer HBM bytes per token than bf16.
//
// Same decomposition and the same arithmetic after dequantisation as the bf16 kernel
// (gqa_decode.hpp): a workgroup of 4 waves serves runs of consecutive tokens of (shard, sequence, kv head,
// head tile) rows, the waves take alternating 32-token blocks, scores / integer-reference softmax / P.V run on
// 16x16x32 bf16 MFMAs.
// What differs is how the operands get into registers:
//   K   lane (r = token, kc) loads the 16 bytes holding dims 32kc .. 32kc+31 of its token: exactly
//       one scale block.  The score contraction does not care about the order of the dims as long
//       as Q agrees, so k-step s takes dims 32kc + 8s .. +8 from every lane (Q is loaded to match)
//       instead of 32s + 8kc .. +8.  One wave instruction covers 16 whole rows.
//   V   lane (r, kc) owns value columns 8r .. 8r+7 (4 bytes per token, scale block r/4) of its 8
//       tokens, as in the bf16 kernel; the 8x8 transpose happens after the conversion.
//   dequantisation  v_cvt_scalef32_pk_bf16_fp4 turns one byte (two codes, low nibble first --
//       checked on the device for all 256 bytes) into two bf16 times a float scale: exact, because
//       an E2M1 value has one mantissa bit and the scale is a power of two.  64 conversions per lane
//       and 32-token block, each right before the MFMA that consumes its result.
//   scales  K: one dword (the 4 block scales of a token) per lane, byte kc selected; V: two 16-byte
//       loads cover the 4 scales of the lane's 8 tokens, byte r/4 selected; the code becomes the float's
//       exponent field (codes 1..254).
// A block is only 4.3 KB per wave, so three waves per SIMD are kept resident (at most 168 registers;
// the kernel takes 162, two raw blocks of 26 registers each among them); loads are never issued under a condition of their own (the
// index is clamped instead), which keeps the compiler's wait counts exact.  The kernel is bound by
// vector-ALU issue, not by HBM, so full blocks are fetched with buffer loads whose addresses cost no
// vector instruction (Mx4Streams).
#pragma once
#include "gqa_decode.hpp"

namespace helix {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));       // 16-byte loads that are only dword aligned

struct Mx4Raw {
    u32x4 k[2];        // codes of dims 32kc..32kc+31 of tokens r, 16 + r
    uint32_t ks[2];    // their tokens' 4 block scales
    uint32_t v[8];     // codes of columns 8r..8r+7 of the lane's 8 tokens
    u32x4 vs[2];       // block scales of tokens 4kc..4kc+3 and 16 + 4kc .. +3 (4 bytes each)
};

constexpr int kMxRow = 64;     // code bytes per 128-wide row
constexpr int kMxScaleRow = 4; // scale bytes per row

// Loads the block of 32 tokens whose first rows are kblk / vblk (codes) and ksc / vsc (scales).
// TAIL: tokens >= n_valid are redirected to the last valid row (their weights are zero later).
template <bool TAIL, bool NT>
__device__ __forceinline__ void mx4_load_block(Mx4Raw& raw, const char* kblk, const char* vblk, const char* ksc, const char* vsc,
                                               uint32_t k_row_bytes, uint32_t v_row_bytes, int r, int kc, int n_valid)
{
#pragma unroll
    for (int a = 0; a < 2; a++) {
        int tok = a * 16 + r;
        if (TAIL) tok = min(tok, n_valid - 1);
        raw.k[a] = stream_load<NT>(reinterpret_cast<const u32x4*>(kblk + (uint32_t)((uint32_t)tok * k_row_bytes + (uint32_t)kc * 16u)));
        raw.ks[a] = stream_load<NT>(reinterpret_cast<const uint32_t*>(ksc + (uint32_t)tok * (k_row_bytes / 16u)));
    }
#pragma unroll
    for (int j = 0; j < 8; j++) {
        int tok = (j >> 2) * 16 + kc * 4 + (j & 3);
        if (TAIL) tok = min(tok, n_valid - 1);
        raw.v[j] = stream_load<NT>(reinterpret_cast<const uint32_t*>(vblk + (uint32_t)((uint32_t)tok * v_row_bytes + (uint32_t)r * 4u)));
    }
    if (TAIL) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int tok = min((j >> 2) * 16 + kc * 4 + (j & 3), n_valid - 1);
            raw.vs[j >> 2][j & 3] = stream_load<NT>(reinterpret_cast<const uint32_t*>(vsc + (uint32_t)tok * (v_row_bytes / 16u)));
        }
    } else {
        // rows of a value block that are contiguous in memory have contiguous scale rows
#pragma unroll
        for (int a = 0; a < 2; a++) {
            const u32x4_a4* sp = reinterpret_cast<const u32x4_a4*>(vsc + (uint32_t)(a * 16 + kc * 4) * (v_row_bytes / 16u));     // (dword aligned only)
            if constexpr (NT) raw.vs[a] = __builtin_nontemporal_load(sp);
            else raw.vs[a] = *sp;
        }
    }
}

// Full blocks are fetched with buffer loads: address = 64-bit base of the split (a descriptor in scalar
// registers) + a scalar offset (block, token row inside the block) + one loop-invariant 32-bit lane
// offset per stream -- no vector address arithmetic in the block loop.  The descriptors carry no usable
// range (the host has checked the shapes); offsets stay below 2^32 because a split is at most 2^25 tokens.
struct Mx4Streams {
    __amdgpu_buffer_rsrc_t k, v, ks, vs;
    uint32_t lane_k, lane_ks, lane_v, lane_vs;
    uint32_t k_row_bytes, v_row_bytes;

    __device__ __forceinline__ void init(const char* kbase, const char* vbase, const char* ksbase, const char* vsbase,
                                         uint32_t krb, uint32_t vrb, int r, int kc)
    {
        constexpr int kRaw32 = 0x00020000;                // dword 3 of a raw buffer descriptor: 32-bit data format
        k = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kbase), 0, -1, kRaw32);
        v = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vbase), 0, -1, kRaw32);
        ks = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(ksbase), 0, -1, kRaw32);
        vs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vsbase), 0, -1, kRaw32);
        k_row_bytes = krb;
        v_row_bytes = vrb;
        lane_k = (uint32_t)r * krb + (uint32_t)kc * 16u;
        lane_ks = (uint32_t)r * (krb / 16u);
        lane_v = (uint32_t)kc * 4u * vrb + (uint32_t)r * 4u;
        lane_vs = (uint32_t)kc * 4u * (vrb / 16u);
    }

    // the full block of 32 tokens that starts `tok` rows into the split (uniform)
    template <bool NONTEMPORAL>
    __device__ __forceinline__ void load(Mx4Raw& raw, uint32_t tok) const
    {
        constexpr int NT = NONTEMPORAL ? 2 : 0;           // cache policy bits of the buffer load: 2 = non-temporal
        const uint32_t sk = tok * k_row_bytes, sv = tok * v_row_bytes, sks = tok * (k_row_bytes / 16u), svs = tok * (v_row_bytes / 16u);
#pragma unroll
        for (int a = 0; a < 2; a++) {
            raw.k[a] = __builtin_amdgcn_raw_buffer_load_b128(k, lane_k, sk + a * 16 * k_row_bytes, NT);
            raw.ks[a] = __builtin_amdgcn_raw_buffer_load_b32(ks, lane_ks, sks + a * (k_row_bytes), NT);
        }
#pragma unroll
        for (int j = 0; j < 8; j++)
            raw.v[j] = __builtin_amdgcn_raw_buffer_load_b32(v, lane_v, sv + ((j >> 2) * 16 + (j & 3)) * v_row_bytes, NT);
        // rows of a value block that are contiguous in memory have contiguous scale rows
#pragma unroll
        for (int a = 0; a < 2; a++) raw.vs[a] = __builtin_amdgcn_raw_buffer_load_b128(vs, lane_vs, svs + a * v_row_bytes, NT);
    }
};

// 2^(code - 127) of byte `which` of a dword of E8M0 scales, for codes 1..254: the code is the
// exponent field of the float.  Rotating right by 8*which + 9 moves the byte to bits 23..30.
__device__ __forceinline__ float mx4_scale(uint32_t four, int which)
{
    return as_f32(__builtin_amdgcn_alignbit(four, four, 8u * (uint32_t)which + 9u) & 0x7F800000u);
}

__device__ __forceinline__ uint32_t mx4_pair(uint32_t codes, float scale, int byte)
{
    bf16x2_t p;
    switch (byte) {
        case 0: p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 0); break;
        case 1: p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 1); break;
        case 2: p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 2); break;
        default: p = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 3); break;
    }
    return __builtin_bit_cast(uint32_t, p);
}

// One 32-token block straight from the raw codes: every operand is converted right before the MFMA
// that consumes it (K: 4 conversions per k-step; V: the byte holding columns 2p, 2p+1 of the lane's 8
// tokens -> 8 conversions, then the 16-bit transpose), so no dequantised copy of the block is kept --
// that copy would cost 64 registers and the third wave per SIMD.
template <bool TAIL>
__device__ __forceinline__ void mx4_compute_block(GqaState<128>& st, const Mx4Raw& raw, const bf16x8 (&qb)[4],
                                                  float scale_log2e, int r, int kc, int n_valid)
{
    float ksc[2], vsc[8];
#pragma unroll
    for (int a = 0; a < 2; a++) ksc[a] = mx4_scale(raw.ks[a], kc);
#pragma unroll
    for (int j = 0; j < 8; j++) vsc[j] = mx4_scale(raw.vs[j >> 2][j & 3], r >> 2);
    uint32_t pairs[8];            // columns (2p, 2p+1) of the lane's 8 tokens, refreshed at every even column
    gqa_compute_core<128, TAIL>(
        st,
        [&](int a, int s) {
            const uint32_t w = raw.k[a][s];
            return __builtin_bit_cast(bf16x8, u32x4{mx4_pair(w, ksc[a], 0), mx4_pair(w, ksc[a], 1), mx4_pair(w, ksc[a], 2), mx4_pair(w, ksc[a], 3)});
        },
        [&](int c) {
            if ((c & 1) == 0) {
#pragma unroll
                for (int j = 0; j < 8; j++) pairs[j] = mx4_pair(raw.v[j], vsc[j], c >> 1);
            }
            return gqa_column_of_pairs(pairs, c);
        },
        qb, scale_log2e, kc, n_valid);
}

// SHARED: several head tiles per kv head, side by side (StreamSeat), ordinary loads.
template <bool SHARED>
__global__ __launch_bounds__(256, 3) void gqa_mxfp4_kernel(const AttnArgs a)
{
    constexpr int D = 128;
    constexpr bool NT = !SHARED;
    using C = GqaCfg<D>;
    const int tid = threadIdx.x;
    // the wave index as a scalar: block addresses then stay in scalar registers and the loads take a
    // scalar base plus a 32-bit lane offset instead of 64-bit vector arithmetic per load
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, kc = lane >> 4;

    // This workgroup's share of the launch: an equal range of its head tile's rows laid end to end (stream_self_plan),
    // served run by run -- one run, and one split record, per row the range touches.
    __shared__ int64_t plan_scratch[256 / 64 + 5];
    const int rows_per_pair = a.K;
    StreamCursor cursor;
    if (!stream_self_plan<256>(a, kGqaTile, rows_per_pair, plan_scratch, a.prefix_out, cursor)) return;
    StreamRun run;
    while (stream_next_run(a, cursor, kGqaTile, rows_per_pair, run)) {
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

    // element index of the split's first token row; codes sit at index / 2, scales at index / 32
    const int64_t tok0 = first_row + t0;
    const int64_t ke = (int64_t)b * sh.k_sb + (int64_t)kh * sh.k_sh + tok0 * sh.k_st;
    const int64_t ve = (int64_t)b * sh.v_sb + (int64_t)kh * sh.v_sh + tok0 * sh.v_st;
    const char* kbase = reinterpret_cast<const char*>(sh.k) + ke / 2;
    const char* vbase = reinterpret_cast<const char*>(sh.v) + ve / 2;
    const char* ksbase = reinterpret_cast<const char*>(sh.k_mx) + ke / 32;
    const char* vsbase = reinterpret_cast<const char*>(sh.v_mx) + ve / 32;
    const uint32_t k_row_bytes = (uint32_t)sh.k_st / 2u, v_row_bytes = (uint32_t)sh.v_st / 2u;   // scale rows: a 16th of that

    GqaState<D> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int c = 0; c < C::CPL; c++) st.o[c] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int n_tok = max(t1 - t0, 0);
    const int n_full = n_tok / C::TB;
    const int n_blk = (n_tok + C::TB - 1) / C::TB;
    const int nw = n_full > wave ? (n_full - wave + 3) / 4 : 0;       // this wave's full blocks: wave, wave+4, ...

    // block i of this wave; the index is clamped, so a prefetch past the end re-reads the last block
    Mx4Streams in;
    in.init(kbase, vbase, ksbase, vsbase, k_row_bytes, v_row_bytes, r, kc);
    auto load = [&](Mx4Raw& raw, int i) { in.template load<NT>(raw, (uint32_t)(wave + 4 * min(i, nw - 1)) * C::TB); };
    Mx4Raw r0, r1;
    // the ragged last block of the run, if any, belongs to wave (n_full % 4), which takes it first (requested together
    // with the wave's first full block, so that nobody waits for it at the end of the run)
    const bool tail_mine = n_blk > n_full && (n_full & 3) == wave;
    const int n_tail = n_tok - n_full * C::TB;
    if (tail_mine) {
        const size_t blk0 = (size_t)n_full * C::TB;
        mx4_load_block<true, NT>(r1, kbase + blk0 * k_row_bytes, vbase + blk0 * v_row_bytes, ksbase + blk0 * (k_row_bytes / 16u),
                                 vsbase + blk0 * (v_row_bytes / 16u), k_row_bytes, v_row_bytes, r, kc, n_tail);
    }
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

    if (tail_mine) mx4_compute_block<true>(st, r1, qb, a.scale_log2e, r, kc, n_tail);
    if (nw > 0) {
        int i = 0;
        for (; i + 2 <= nw; i += 2) {
            load(r1, i + 1);
            mx4_compute_block<false>(st, r0, qb, a.scale_log2e, r, kc, C::TB);
            load(r0, i + 2);
            mx4_compute_block<false>(st, r1, qb, a.scale_log2e, r, kc, C::TB);
        }
        if (i < nw) mx4_compute_block<false>(st, r0, qb, a.scale_log2e, r, kc, C::TB);
    }
    gqa_emit_record<D>(st, a, rec, nh, tid, wave, r, kc);
    lds_barrier();                    // the record's staging area in LDS is free for the next run (its stores may still be on their way)
    }
}

}  // namespace helix

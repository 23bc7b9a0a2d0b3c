// Split-KV decode attention for GQA/MQA groups on gfx950: steps "score tile", "online softmax
// update" and "P.V tile" of the per-shard attention of Helix's attention phase (Sec. 2.1.1), for
// bf16 K/V with dk == dv in {64, 128}.
//
// Work decomposition.  One workgroup (4 wavefronts) streams `split_tokens` consecutive tokens of
// one (shard, sequence, kv head) and serves up to 16 query heads of that kv head's group.  The
// four waves take alternating 32-token blocks, each keeping its own running (m, l, O), and merge
// through LDS at the end into ONE un-normalised record per workgroup; a second small kernel merges
// the records of a shard (merge_combine.hpp).
//
// Data path.  K and V go from HBM straight into the registers of the MFMA that consumes them --
// the path is HBM-bound (16 flop/byte at a group of 16) and nothing is read twice, so LDS staging
// would only add a hop.
//   scores   S^T[token,head] = K[token,:] . Q^T        v_mfma_f32_16x16x32_bf16, A = K rows as
//            loaded (lane = token r, 8 consecutive dims of k-chunk kc), B = Q held in registers.
//   weights  p = 2^(s*log2e*scale - m) with an INTEGER running reference m (exp2_rel): rescales of
//            O and l are exact powers of two and p's significand does not depend on how the
//            sequence was split.  The accumulator lane that holds a score column holds the same
//            head's O column, so no cross-lane traffic is needed beyond one 4-lane max.
//   P.V      O^T[dv,head] += V^T[dv,token] . P^T[token,head].  The A operand needs 8 tokens of ONE
//            value column per lane, while memory has 8 columns of one token per 16-byte load:
//            every lane loads the same 8 columns of its 8 tokens (each instruction covers four
//            full 256-byte rows) and transposes the 8x8 block of 16-bit elements in registers
//            with v_perm_b32 -- one VALU op per loaded dword.
//            p is split into bf16 hi + bf16 lo (two MFMAs): a single bf16 rounding of p would
//            cost ~1.7e-3 relative L2 error on O, above the 1e-3 parity bar; the split leaves ~1e-5.
#pragma once
#include "common.hpp"

namespace helix {

template <int D>
struct GqaCfg {
    static constexpr int KS = D / 32;    // k-steps of the score MFMA
    static constexpr int CPL = D / 16;   // value columns per lane
    static constexpr int VDW = CPL / 2;  // dwords per lane per V token
    static constexpr int TB = 32;        // tokens per wave block
};

template <int D>
struct GqaBlock {
    bf16x8 k[2][GqaCfg<D>::KS];          // two 16-token score tiles
    uint32_t v[8][GqaCfg<D>::VDW];       // 8 tokens x CPL columns
};

template <int N, bool NT>
__device__ __forceinline__ void load_dwords(uint32_t (&dst)[N], const char* p)
{
    if constexpr (N == 4) {
        u32x4 t = stream_load<NT>(reinterpret_cast<const u32x4*>(p));
        dst[0] = t.x; dst[1] = t.y; dst[2] = t.z; dst[3] = t.w;
    } else if constexpr (N == 2) {
        u32x2 t = stream_load<NT>(reinterpret_cast<const u32x2*>(p));
        dst[0] = t.x; dst[1] = t.y;
    } else {
        static_assert(N == 2 || N == 4, "unsupported value width");
    }
}

// K/V are read exactly once, so the loads are non-temporal (NT) -- unless the launch has several head tiles per
// kv head, whose workgroups share their reads through the L2 (StreamSeat).
// Loads the block of 32 tokens starting at shard token `tb`.  kblk / vblk point at the block's
// first token row (wave-uniform); tokens >= t1 are redirected to the last valid row so that every
// address stays inside the shard (their weights are forced to zero later).
template <int D, bool TAIL, bool NT>
__device__ __forceinline__ void gqa_load_block(GqaBlock<D>& blk, const char* kblk, const char* vblk,
                                               uint32_t k_row_bytes, uint32_t v_row_bytes,
                                               int r, int kc, int n_valid)
{
    using C = GqaCfg<D>;
#pragma unroll
    for (int a = 0; a < 2; a++) {
        int tok = a * 16 + r;
        if (TAIL) tok = min(tok, n_valid - 1);
        const char* p = kblk + (uint32_t)tok * k_row_bytes + (uint32_t)kc * 16u;
#pragma unroll
        for (int s = 0; s < C::KS; s++)
            blk.k[a][s] = __builtin_bit_cast(bf16x8, stream_load<NT>(reinterpret_cast<const u32x4*>(p + s * 64)));
    }
#pragma unroll
    for (int j = 0; j < 8; j++) {
        int tok = (j >> 2) * 16 + kc * 4 + (j & 3);
        if (TAIL) tok = min(tok, n_valid - 1);
        const char* p = vblk + (uint32_t)tok * v_row_bytes + (uint32_t)r * (C::CPL * 2);
        load_dwords<C::VDW, NT>(blk.v[j], p);
    }
}

template <int D>
struct GqaState {
    float m;                          // integer-valued running reference exponent (or -inf)
    float l;                          // this lane's share of sum_t p_t for head r
    f32x4 o[GqaCfg<D>::CPL];          // O^T tiles: o[c][i] = O[head r][dv = (kc*4+i)*CPL + c]
};

// One 32-token block: scores, online softmax update, P.V.  `kop(a, s)` supplies the score MFMA's A
// operand (16-token tile a, k-step s), `vop(c)` the P.V MFMA's A operand for value column c of the
// lane (8 tokens of that column); the callers differ in how the operands come out of the loaded
// block (bf16 as loaded / transposed, MXFP4 or e4m3 converted on the fly).  SCALED: token slot e of the lane
// (token (e / 4) * 16 + 4kc + e % 4) carries a dequantisation factor fs[e] that multiplies its score and its weight,
// both in fp32; the normaliser sums the weights without it.
template <int D, bool TAIL, bool SCALED = false, class KOp, class VOp>
__device__ __forceinline__ void gqa_compute_core(GqaState<D>& st, KOp&& kop, VOp&& vop,
                                                 const bf16x8 (&qb)[GqaCfg<D>::KS],
                                                 float scale_log2e, int kc, int n_valid, const float* fs = nullptr)
{
    using C = GqaCfg<D>;
    // scores: lane (r,kc) gets head r, tokens a*16 + kc*4 + i
    float t[8];
#pragma unroll
    for (int a = 0; a < 2; a++) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < C::KS; s++)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop(a, s), qb[s], acc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            t[a * 4 + i] = acc[i] * scale_log2e;
            if (SCALED) t[a * 4 + i] *= fs[a * 4 + i];
        }
    }
    bool valid[8];
    if (TAIL) {
#pragma unroll
        for (int e = 0; e < 8; e++) {
            valid[e] = ((e >> 2) * 16 + kc * 4 + (e & 3)) < n_valid;
            t[e] = valid[e] ? t[e] : -INFINITY;
        }
    }
    float bmax = t[0];
#pragma unroll
    for (int e = 1; e < 8; e++) bmax = fmaxf(bmax, t[e]);
    bmax = wave_xor_max_16_32(bmax);
    const float m_new = fmaxf(st.m, __builtin_ceilf(bmax));
    if (__any(m_new != st.m)) {
        const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // exact power of two, 0 from -inf
        st.l *= alpha;
#pragma unroll
        for (int c = 0; c < C::CPL; c++) st.o[c] *= alpha;
        st.m = m_new;
    }
    // weights and their bf16 hi/lo split, packed as the MFMA's B operand (8 tokens of head r)
    uint32_t phi[4], plo[4];
    float lsum = 0.f;
    const int mi = (int)m_new;                            // finite: the block has a valid token
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        float p0, p1;
        if (TAIL) {
            p0 = valid[e] ? exp2_rel_int(t[e], mi) : 0.f;
            p1 = valid[e + 1] ? exp2_rel_int(t[e + 1], mi) : 0.f;
        } else {
            p0 = exp2_rel_int(t[e], mi);
            p1 = exp2_rel_int(t[e + 1], mi);
        }
        // l sums the unsplit weights: hi + lo differs from p by at most 2^-17 p, far below the bars,
        // and re-adding the split would cost three more VALU instructions per weight pair
        lsum += p0 + p1;
        if (SCALED) {
            p0 *= fs[e];
            p1 *= fs[e + 1];
        }
        const uint32_t h = pack_bf16_rne(p0, p1);
        const float r0 = p0 - as_f32(h << 16);
        const float r1 = p1 - as_f32(h & 0xffff0000u);
        const uint32_t lo = pack_bf16_rne(r0, r1);
        phi[e >> 1] = h;
        plo[e >> 1] = lo;
    }
    st.l += lsum;
    const bf16x8 bhi = __builtin_bit_cast(bf16x8, u32x4{phi[0], phi[1], phi[2], phi[3]});
    const bf16x8 blo = __builtin_bit_cast(bf16x8, u32x4{plo[0], plo[1], plo[2], plo[3]});
    // P.V
#pragma unroll
    for (int c = 0; c < C::CPL; c++) {
        const bf16x8 va = vop(c);
        st.o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, bhi, st.o[c], 0, 0, 0);
        st.o[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, blo, st.o[c], 0, 0, 0);
    }
}

// Column c of the lane's 8 tokens out of 8 registers that each hold one token's columns (2p, 2p+1)
// as a bf16 pair: the 8x8 transpose of 16-bit elements, one v_perm_b32 per output dword.
__device__ __forceinline__ bf16x8 gqa_column_of_pairs(const uint32_t (&t)[8], int c)
{
    const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
    u32x4 a;
    a.x = __builtin_amdgcn_perm(t[1], t[0], sel);
    a.y = __builtin_amdgcn_perm(t[3], t[2], sel);
    a.z = __builtin_amdgcn_perm(t[5], t[4], sel);
    a.w = __builtin_amdgcn_perm(t[7], t[6], sel);
    return __builtin_bit_cast(bf16x8, a);
}

// bf16 block: K operands as loaded; V: this lane's 8 tokens x CPL columns transposed into CPL operands.
template <int D, bool TAIL>
__device__ __forceinline__ void gqa_compute_block(GqaState<D>& st, const GqaBlock<D>& blk,
                                                  const bf16x8 (&qb)[GqaCfg<D>::KS],
                                                  float scale_log2e, int kc, int n_valid)
{
    gqa_compute_core<D, TAIL>(
        st, [&](int a, int s) { return blk.k[a][s]; },
        [&](int c) {
            const uint32_t t[8] = {blk.v[0][c >> 1], blk.v[1][c >> 1], blk.v[2][c >> 1], blk.v[3][c >> 1],
                                   blk.v[4][c >> 1], blk.v[5][c >> 1], blk.v[6][c >> 1], blk.v[7][c >> 1]};
            return gqa_column_of_pairs(t, c);
        },
        qb, scale_log2e, kc, n_valid);
}

__device__ __forceinline__ float max_of_waves(const float (&m)[4][16], int r)
{
    return fmaxf(fmaxf(m[0][r], m[1][r]), fmaxf(m[2][r], m[3][r]));
}

// Merges the four waves' running states of a workgroup into ONE un-normalised record (sum p v, integer
// reference exponent, sum p) and writes it to the workspace.  Called by all 256 threads.
template <int D>
__device__ __forceinline__ void gqa_emit_record(GqaState<D>& st, const AttnArgs& a, size_t rec, int nh,
                                                int tid, int wave, int r, int kc)
{
    using C = GqaCfg<D>;
    __shared__ float sm_m[4][16];
    __shared__ float sm_l[4][16];
    __shared__ float sm_o[4][16][D];
    st.l = wave_xor_sum_16_32(st.l);
    if (kc == 0) { sm_m[wave][r] = st.m; sm_l[wave][r] = st.l; }
    lds_barrier();
    const float M = max_of_waves(sm_m, r);
    const float f = (st.m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m - M);
#pragma unroll
    for (int c = 0; c < C::CPL; c++)
#pragma unroll
        for (int i = 0; i < 4; i++) sm_o[wave][r][(kc * 4 + i) * C::CPL + c] = st.o[c][i] * f;
    lds_barrier();
    if (tid < nh) {
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < 4; w++) {
            const float mw = sm_m[w][tid];
            L += (mw == -INFINITY) ? 0.f : sm_l[w][tid] * __builtin_amdgcn_exp2f(mw - max_of_waves(sm_m, tid));
        }
        a.ws_m[rec + tid] = max_of_waves(sm_m, tid);
        a.ws_l[rec + tid] = L;
    }
    float* out = a.ws_o + rec * D;
    for (int idx = tid * 4; idx < nh * D; idx += 256 * 4) {
        const int hh = idx / D, col = idx % D;
        f32x4 s0 = *reinterpret_cast<const f32x4*>(&sm_o[0][hh][col]);
        f32x4 s1 = *reinterpret_cast<const f32x4*>(&sm_o[1][hh][col]);
        f32x4 s2 = *reinterpret_cast<const f32x4*>(&sm_o[2][hh][col]);
        f32x4 s3 = *reinterpret_cast<const f32x4*>(&sm_o[3][hh][col]);
        *reinterpret_cast<f32x4*>(out + idx) = (s0 + s1) + (s2 + s3);
    }
}

constexpr int kGqaTile = 128;      // tokens per planning tile of the streaming kernels: one 32-token block per wave

// What a streaming workgroup does around each of its runs: the row's first / last workgroup is noted for the merge.
__device__ __forceinline__ void gqa_note_run(const AttnArgs& a, const StreamRun& run)
{
    if (threadIdx.x == 0) {
        if (run.first) a.row_rec[run.row].x = run.seat;
        if (run.last) a.row_rec[run.row].y = run.seat;
    }
}

// SHARED: the launch has several head tiles per kv head (more than 16 query heads share a kv head); their
// workgroups sit side by side (StreamSeat) and load the ordinary way.
template <int D, bool SHARED>
__global__ __launch_bounds__(256, 2) void gqa_decode_kernel(const AttnArgs a)
{
    using C = GqaCfg<D>;
    constexpr bool NT = !SHARED;

    // This workgroup's share of the launch: an equal range of its head tile's rows laid end to end (stream_self_plan),
    // served run by run -- one run, and one split record, per row the range touches.
    __shared__ int64_t plan_scratch[256 / 64 + 5];
    const int rows_per_pair = a.K;
    StreamCursor cursor;
    if (!stream_self_plan<256>(a, kGqaTile, rows_per_pair, plan_scratch, a.prefix_out, cursor)) return;
    StreamRun run;
    while (stream_next_run(a, cursor, kGqaTile, rows_per_pair, run)) {
    // (the lane's coordinates are derived anew in every run: hoisted out of this loop, the address pieces computed
    // from them would hold two dozen registers for the whole kernel, which the streaming loop has no room for)
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

    const int64_t tok0 = first_row + t0;
    const char* kbase = reinterpret_cast<const char*>(sh.k) + 2 * ((int64_t)b * sh.k_sb + (int64_t)kh * sh.k_sh + tok0 * sh.k_st);
    const char* vbase = reinterpret_cast<const char*>(sh.v) + 2 * ((int64_t)b * sh.v_sb + (int64_t)kh * sh.v_sh + tok0 * sh.v_st);
    const uint32_t k_row_bytes = (uint32_t)sh.k_st * 2u, v_row_bytes = (uint32_t)sh.v_st * 2u;

    GqaState<D> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int c = 0; c < C::CPL; c++) st.o[c] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this wave's blocks: wave, wave+4, wave+8, ... of the run; all but possibly the last are full
    const int n_tok = max(t1 - t0, 0);
    const int n_full = n_tok / C::TB;                 // full blocks in the run
    const int n_blk = (n_tok + C::TB - 1) / C::TB;
    const size_t k_blk_bytes = (size_t)C::TB * k_row_bytes, v_blk_bytes = (size_t)C::TB * v_row_bytes;

    // This wave's full blocks are wave, wave+4, ...  Two register sets; the next block's loads are
    // always issued before the current block is consumed, and never under a condition of their
    // own: the compiler's s_waitcnt placement merges the counts of all paths that reach a use, so a
    // skipped prefetch on one path would make every path wait for the prefetch it did issue.
    GqaBlock<D> b0, b1;
    const int nw = n_full > wave ? (n_full - wave + 3) / 4 : 0;
    auto kptr = [&](int i) { return kbase + (size_t)(wave + 4 * i) * k_blk_bytes; };
    auto vptr = [&](int i) { return vbase + (size_t)(wave + 4 * i) * v_blk_bytes; };
    // The ragged last block of the run, if any, belongs to wave (n_full % 4), which takes it FIRST: requested
    // together with the wave's first full block, it is not waited for at the end of the run by the three other waves.
    const bool tail_mine = n_blk > n_full && (n_full & 3) == wave;
    const int n_tail = n_tok - n_full * C::TB;
    if (tail_mine) gqa_load_block<D, true, NT>(b1, kbase + n_full * k_blk_bytes, vbase + n_full * v_blk_bytes, k_row_bytes, v_row_bytes, r, kc, n_tail);
    if (nw > 0) gqa_load_block<D, false, NT>(b0, kptr(0), vptr(0), k_row_bytes, v_row_bytes, r, kc, C::TB);

    // (fetched after the first K/V block is on its way: the stream does not depend on Q)
    // Q as the score MFMA's B operand: lane (r,kc) holds head r, dims s*32 + kc*8 .. +8
    bf16x8 qb[C::KS];
    {
        const uint16_t* qrow = a.q + ((size_t)b * a.Q + h0 + min(r, nh - 1)) * D + kc * 8;
#pragma unroll
        for (int s = 0; s < C::KS; s++) {
            u32x4 w = *reinterpret_cast<const u32x4*>(qrow + s * 32);
            if (r >= nh) w = u32x4{0, 0, 0, 0};
            qb[s] = __builtin_bit_cast(bf16x8, w);
        }
    }

    if (tail_mine) gqa_compute_block<D, true>(st, b1, qb, a.scale_log2e, kc, n_tail);
    if (nw > 0) {
        int i = 0;
        for (; i + 2 < nw; i += 2) {
            gqa_load_block<D, false, NT>(b1, kptr(i + 1), vptr(i + 1), k_row_bytes, v_row_bytes, r, kc, C::TB);
            gqa_compute_block<D, false>(st, b0, qb, a.scale_log2e, kc, C::TB);
            gqa_load_block<D, false, NT>(b0, kptr(i + 2), vptr(i + 2), k_row_bytes, v_row_bytes, r, kc, C::TB);
            gqa_compute_block<D, false>(st, b1, qb, a.scale_log2e, kc, C::TB);
        }
        if (i + 1 < nw) {
            gqa_load_block<D, false, NT>(b1, kptr(i + 1), vptr(i + 1), k_row_bytes, v_row_bytes, r, kc, C::TB);
            gqa_compute_block<D, false>(st, b0, qb, a.scale_log2e, kc, C::TB);
            gqa_compute_block<D, false>(st, b1, qb, a.scale_log2e, kc, C::TB);
        } else {
            gqa_compute_block<D, false>(st, b0, qb, a.scale_log2e, kc, C::TB);
        }
    }

    gqa_emit_record<D>(st, a, rec, nh, tid, wave, r, kc);
    lds_barrier();                    // the record's staging area in LDS is free for the next run (its stores may still be on their way)
    }
}

}  // namespace helix

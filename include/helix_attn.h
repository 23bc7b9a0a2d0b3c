/*
 * helix_attn.h -- C ABI of the MI355X (gfx950) library for the attention phase of Helix Parallelism.
 *
 * What the calls compute (Helix Parallelism, Sec. 2.1.1 "KV partitioning (KVP)", Fig. 4 top,
 * Sec. 2.2 first paragraphs): during decode every KVP rank holds one slice of the KV cache along
 * the sequence dimension, runs exact softmax attention of the single new query token against its
 * slice, and emits a partial attention output plus one log-sum-exp scalar per (token, head); the
 * fragments of all ranks are then rescaled by their log-sum-exp and summed, which reconstructs the
 * exact softmax-normalised attention over the unsharded cache.  Q query heads share K KV heads
 * (GQA/MQA) or a single latent that is both key and value (MLA) (Sec. 1, Sec. 3).
 *
 *     partial, per shard i, sequence b, query head h (kv head = h / (Q/K)):
 *         s_t   = scale * <q[b,h,:], k_i[b,kv,t,:]>                  t in the shard
 *         lse_i = ln sum_t exp(s_t)                                   natural log, scale inside
 *         O_i   = sum_t exp(s_t - lse_i) * v_i[b,kv,t,:]              normalised within the shard
 *     combine:
 *         w_i = exp(lse_i - max_j lse_j) ;  O = sum_i w_i O_i / sum_i w_i ;
 *         LSE = max_j lse_j + ln sum_i w_i
 *
 * No causal mask: the one decode query attends to every token a shard holds (the new token's K/V
 * is appended before attention, Sec. 2.3).
 *
 * General conventions
 *   - All pointers are DEVICE pointers unless a parameter says "host".  The structs themselves
 *     (helix_problem, helix_kv_shard, the shard array) are host memory, read during the call.
 *   - The caller owns every buffer, including the workspace.  The library allocates nothing,
 *     never synchronises, never reads device memory from the host; all work is enqueued on the
 *     HIP stream passed as `hip_stream` (a hipStream_t; NULL = the default stream).  No call leaves
 *     state behind for the next one (the only process-wide state is a set of once-flags for a kernel
 *     attribute), so calls from several threads on their own streams and buffers are independent.
 *   - Every call returns a helix_status.  Arguments are validated on the host before anything
 *     is launched, so an error return means no kernel ran.
 *   - Supported shapes: (dk,dv) = (64,64) or (128,128) with bf16 K/V and any Q/K group size
 *     (the GQA path), (128,128) with e4m3 K/V + one fp32 scale per (sequence, kv head, token) that the
 *     token's key and value row share, (128,128) with MXFP4 K/V (the FP4 of the paper's evaluation, Sec. 3), and
 *     (dk,dv) = (576,512) with v_aliases_k = 1, kv_heads = 1, bf16, e4m3 + per-token fp32
 *     scale, or MXFP4 (the MLA path).  q is always bf16.
 *   - Alignment: q, k, v rows must start on 16-byte boundaries: base pointers 16-byte aligned and
 *     all strides multiples of 16 bytes.
 *   - Arithmetic: scores are exact products of the stored values accumulated in fp32; softmax weights
 *     are computed in fp32 relative to an integer power-of-two reference, so results do not depend on
 *     how a sequence is cut into shards beyond fp32 summation order (1e-5 on O(1) outputs).  The bf16,
 *     e4m3 and MXFP4 GQA paths and the bf16 MLA path hand each weight to the matrix cores as a bf16 hi + lo
 *     pair (relative error 2^-17; an e4m3 token's scale multiplies its score and its weight in fp32); the e4m3 and MXFP4 MLA paths contract in fp16 with ONE fp16 weight per token (relative
 *     error up to 2^-12 that the normaliser does not share: |error of O| <= 2^-12 * max |v| for a peaked
 *     softmax, about 2e-4 relative L2 otherwise).  An MXFP4 latent row is held as fp16 entries times a
 *     power of two taken from its largest block scale: exact for blocks within 21 octaves of that scale,
 *     smaller ones are off by at most 2^-24 of the row's largest magnitude; the largest scale code of a
 *     row must be at least 10.  LSE always comes from the unrounded fp32 sums.
 */
#ifndef HELIX_ATTN_H
#define HELIX_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HELIX_OK = 0,
    HELIX_ERR_NULL = 1,        /* a required pointer is NULL */
    HELIX_ERR_SHAPE = 2,       /* sizes, strides or alignment that make no sense */
    HELIX_ERR_UNSUPPORTED = 3, /* a combination the kernels do not implement */
    HELIX_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned or smaller than helix_attn_workspace_bytes */
    HELIX_ERR_LAUNCH = 5       /* the HIP runtime refused a launch */
} helix_status;

typedef enum {
    HELIX_KV_BF16 = 0,
    HELIX_KV_FP8_E4M3 = 1,     /* OCP e4m3 codes, value = code * kv_scale[token] (key and value row of a token alike) */
    HELIX_KV_MXFP4 = 2         /* OCP microscaling FP4 (the precision Sec. 3 evaluates in): E2M1 codes, two per byte
                                  (even element in the low nibble); every 32 consecutive elements of a
                                  row share one E8M0 scale byte; value = 2^(scale - 127) * e2m1(code).
                                  A block with scale code 0 (2^-127) is taken as zero, which is its value to
                                  within 2^-124; scale code 255 (NaN) is not supported. */
} helix_kv_dtype;

#define HELIX_MAX_SHARDS 1024

/* The problem of Sec. 1 / Appendix A: B sequences, Q query heads sharing K KV heads. */
typedef struct helix_problem {
    int32_t batch;        /* B >= 1 */
    int32_t q_heads;      /* Q >= 1 */
    int32_t kv_heads;     /* K >= 1, Q % K == 0; query head h reads kv head h / (Q/K) */
    int32_t dk;           /* key / query width */
    int32_t dv;           /* value width */
    int32_t v_aliases_k;  /* 1 = MLA latent: the value row is the first dv entries of the key row */
    int32_t kv_dtype;     /* helix_kv_dtype */
    float scale;          /* softmax scale, multiplies q.k before the exponential; finite, > 0 */
    int32_t split_tokens; /* 0 = automatic.  Otherwise the number of shard tokens one workgroup
                             streams (rounded up to the kernel's block size): a tuning knob that
                             changes neither results' meaning nor the workspace formula's validity */
} helix_problem;

/* One KV-sequence shard = the slice of the cache one KVP rank holds (Sec. 2.1.1).
 * Key element (b, kh, t, d), t counted from the shard's first token of sequence b, lives at
 *     k + b*k_stride_b + kh*k_stride_h + (tok_off[b] + t)*k_stride_t + d        (in elements)
 * and values / scales follow the same scheme with their own strides (scale: token stride 1).
 * MXFP4: strides still count ELEMENTS (two per byte); the code of element index e sits in byte e/2
 * of k (v), its block scale in byte e/32 of k_scale_mx (v_scale_mx).  Token rows must be dense
 * (k_stride_t == dk, v_stride_t == dv), the other strides multiples of 128, the scale arrays
 * 4-byte aligned.  An MXFP4 MLA latent (v_aliases_k) has v == NULL and v_scale_mx == NULL: the value is
 * the first dv entries of the key row, block scales included; its scale bytes are fetched as aligned
 * 4-byte words, so the array must be readable up to the next 4-byte boundary after its last row. */
typedef struct helix_kv_shard {
    const void *k;          /* bf16 or e4m3 */
    const void *v;          /* same dtype; must be NULL iff v_aliases_k */
    const float *kv_scale;  /* e4m3 only: one fp32 per (b, kh, token); NULL otherwise */
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
    int64_t s_stride_b, s_stride_h;
    const int64_t *tok_off; /* [B] row of the shard's first token of sequence b (ragged / packed
                               storage, or a view into an unsharded cache); NULL = 0 */
    const int32_t *len;     /* [B] tokens of sequence b in THIS shard; 0 is allowed */
    int32_t max_len;        /* host copy of an upper bound of len[b] (sizes the grid); >= 0 */
    const uint8_t *k_scale_mx; /* MXFP4 only: E8M0 block scales of k; NULL otherwise */
    const uint8_t *v_scale_mx; /* MXFP4 only: E8M0 block scales of v; NULL otherwise */
    int32_t *status;        /* device int32 or NULL: the attention kernels OR HELIX_STATUS_* bits into it when they
                               meet device data the host could not check (the caller clears it; it is only ever
                               written when a condition holds) */
} helix_kv_shard;

/* Bits of helix_kv_shard.status.  The launch is sized from the host's max_len; a sequence whose device-side
 * len[b] is larger (e.g. after helix_kv_append without raising max_len) has its surplus tokens left out of
 * the attention, and this bit says so. */
#define HELIX_STATUS_LEN_EXCEEDS_MAX 1
/* The MLA kernels keep a power-of-two reference exponent per head and move it only in a tile whose scores
 * (bf16 latent) or fp16 weights (e4m3 / MXFP4 latents) come near the end of their number range -- never on
 * ordinary logits, a few times per run on sharply peaked ones.  Results do not depend on it, time hardly: every
 * (wavefront, tile) that moved references adds HELIX_STATUS_REFERENCE_MOVED, so (status >> 8) counts them. */
#define HELIX_STATUS_REFERENCE_MOVED 256

/* Bytes of workspace helix_attn_partial / helix_attn_decode need for `n_shards` shards whose
 * max_len are all <= `max_len`.  Returns 0 if the problem is invalid or unsupported.
 * The workspace must be 256-byte aligned; its contents are scratch. */
size_t helix_attn_workspace_bytes(const helix_problem *problem, int32_t n_shards, int32_t max_len);

/* Sec. 2.1.1: one rank's work.  Attention of q over one shard.
 *   q          bf16 [B,Q,dk] contiguous
 *   o_partial  fp32 [B,Q,dv]: O_i, normalised within the shard (zeros where len[b] == 0)
 *   lse        fp32 [B,Q]: lse_i (-inf where len[b] == 0)                                   */
int helix_attn_partial(const helix_problem *problem, const void *q, const helix_kv_shard *shard,
                       float *o_partial, float *lse,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Sec. 2.1.1 / Sec. 2.2: the rescale-and-sum every rank applies to the fragments it received.
 * Only batch, q_heads and dv of `problem` are read.
 *   o_partials    fp32 [N,B,Q,dv],  lses fp32 [N,B,Q]
 *   o             fp32 [B,Q,dv]
 *   lse_out       fp32 [B,Q] or NULL: LSE of the whole context
 *   argmax_shard  int32 [B,Q] or NULL: lowest shard index holding the largest lses value (0 if all
 *                 are -inf); decided on the fp32 values as stored
 * Shards with lse = -inf get weight 0 whatever their partial holds; if all are -inf, o = 0 and
 * lse_out = -inf.  o must not overlap o_partials. */
int helix_attn_combine(const helix_problem *problem, int32_t n_shards,
                       const float *o_partials, const float *lses,
                       float *o, float *lse_out, int32_t *argmax_shard, void *hip_stream);

/* Whole decode attention on one GPU: helix_attn_partial for each of the N shards (one launch),
 * then helix_attn_combine.  n_shards == 1 is attention over an unsharded cache (the short-context
 * degenerate case KVP = 1, Sec. 5).
 *   shards      host array [N]
 *   o           fp32 [B,Q,dv]
 *   lse_out     fp32 [B,Q] or NULL
 *   o_partials  fp32 [N,B,Q,dv] or NULL, lses fp32 [N,B,Q] or NULL: the per-shard fragments a rank
 *               would send; both or neither.  When NULL they live in the workspace. */
int helix_attn_decode(const helix_problem *problem, const void *q,
                      const helix_kv_shard *shards, int32_t n_shards,
                      float *o, float *lse_out, float *o_partials, float *lses,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): helix_attn_decode with the split records and the
 * per-shard fragments in a static device array of HELIX_STATIC_SCRATCH_BYTES inside the library instead of a
 * caller's workspace.  Same kernels, same plan, same results as helix_attn_decode with o_partials == NULL.
 * The call allocates nothing; its first use on a device looks up the array's address (hipGetSymbolAddress).
 * A problem that needs more than HELIX_STATIC_SCRATCH_BYTES of workspace is refused with HELIX_ERR_WORKSPACE
 * before anything is launched.  Every call on a GPU uses that GPU's one array (nothing in it has to be
 * cleared: each launch writes every record it later reads): calls that overlap on one GPU -- from different
 * streams or threads -- race on it; calls on one stream are ordered. */
#define HELIX_STATIC_SCRATCH_BYTES (16u << 20)
int helix_attn_decode_static(const helix_problem *problem, const void *q,
                             const helix_kv_shard *shards, int32_t n_shards,
                             float *o, float *lse_out, void *hip_stream);

/* helix_shard_layout and helix_attn_decode in one call: `cache` describes the UNSHARDED cache (len =
 * the sequences' full lengths, tok_off = their first rows or NULL, max_len = an upper bound of the
 * lengths) and the N slices of Sec. 2.1.1 are cut inside the attention kernel, with the integers
 * helix_shard_layout would produce.  One launch less per decode step.
 *   shard_off, shard_len   int64 / int32 [N,B] or both NULL: the cut, written by the kernel
 *   everything else as in helix_attn_decode; size the workspace with helix_attn_workspace_bytes(
 *   problem, n_shards, max_len). */
int helix_attn_decode_kvp(const helix_problem *problem, const void *q, const helix_kv_shard *cache,
                          int32_t n_shards, float *o, float *lse_out, float *o_partials, float *lses,
                          int64_t *shard_off, int32_t *shard_len,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Sec. 2.1.1: the contiguous KVP cut of every sequence into N slices, as device-side integer
 * bookkeeping.  Slice width c_b = 16 * ceil(ceil(L_b / N) / 16) tokens (whole 16-token blocks, the
 * append granule of Sec. 2.3); shard i of sequence b = [min(i*c_b, L_b), min((i+1)*c_b, L_b)).
 *   seq_len    int32 [B], every entry >= 0
 *   seq_base   int64 [B] or NULL: row of sequence b's first token in packed storage, added to the
 *              offsets so that shard_off can serve directly as helix_kv_shard.tok_off
 *   shard_off  int64 [N,B],  shard_len int32 [N,B]                                           */
int helix_shard_layout(const int32_t *seq_len, const int64_t *seq_base, int32_t batch,
                       int32_t n_shards, int64_t *shard_off, int32_t *shard_len, void *hip_stream);

#define HELIX_APPEND_BLOCK 16   /* decode tokens a KVP rank receives before the next rank takes over */

/* Sec. 2.3 (distributed KV concatenation): which KVP rank stores the K/V of decode token
 * `decode_index` (0 = the first token generated after prefill): HELIX_APPEND_BLOCK consecutive tokens go
 * to rank 0, the next HELIX_APPEND_BLOCK to rank 1, ..., cycling over the n_shards ranks.  Host-only
 * integer arithmetic; returns -1 for n_shards < 1 or a negative index. */
int32_t helix_kv_append_owner(int64_t decode_index, int32_t n_shards);

/* Sec. 2.3: staggered KV append.  Writes the new token's K (and V) row of every sequence and KV head
 * into the shard of rank helix_kv_append_owner(decode_index, n_shards), at token position len[b] of
 * that shard (after the shard's tok_off[b]), and then increments that shard's len[b].
 *   shards      host array [N]; only the owner's descriptor is used.  Its k / v / kv_scale / len
 *               memory is WRITTEN by this call although the struct declares it const.
 *   k_new       device, KV dtype of the problem, [B,K,dk] contiguous
 *   v_new       device [B,K,dv], or NULL iff v_aliases_k
 *   scale_new   device fp32 [B,K], e4m3 only (NULL for bf16)
 *   capacity    tokens per (sequence, kv head) the owner's storage can hold, counted from tok_off[b]; a
 *               sequence that is already full is left untouched and *overflow (device int32, may
 *               be NULL) is set to 1
 * The caller keeps its host-side max_len of the owner shard up to date (+1 per call). */
int helix_kv_append(const helix_problem *problem, const helix_kv_shard *shards, int32_t n_shards,
                    int64_t decode_index, const void *k_new, const void *v_new, const float *scale_new,
                    int32_t capacity, int32_t *overflow, void *hip_stream);

/* The same for an MXFP4 cache (helix_kv_append returns HELIX_ERR_UNSUPPORTED for it):
 *   k_codes, v_codes    device uint8 [B,K,dk/2], [B,K,dv/2]: the new rows' E2M1 codes
 *   k_scales, v_scales  device uint8 [B,K,dk/32], [B,K,dv/32]: their E8M0 block scales
 * v_codes and v_scales must be NULL iff v_aliases_k. */
int helix_kv_append_mxfp4(const helix_problem *problem, const helix_kv_shard *shards, int32_t n_shards,
                          int64_t decode_index, const void *k_codes, const void *v_codes,
                          const uint8_t *k_scales, const uint8_t *v_scales,
                          int32_t capacity, int32_t *overflow, void *hip_stream);

/* Sec. 2.1.3 (HOP-B, batch-wise overlap of the KVP exchange with attention) on one GPU.  The batch is
 * cut into n_groups groups of consecutive sequences (the first groups hold ceil(B / n_groups)).  Group
 * g's per-shard attention runs on `compute_stream`; as soon as it is done its fragments are handed
 * over on `exchange_stream` -- a device copy send -> recv stands in for the All-to-All, which is the
 * identity when all N ranks are one GPU -- and combined there, while group g+1's attention is already
 * running on `compute_stream`.
 *   send_o, recv_o      fp32 [N*B*Q*dv] each, group-major: group g (sequences b0..b0+nb-1) owns the
 *                       contiguous block [N, nb, Q, dv] starting at element N*b0*Q*dv
 *   send_lse, recv_lse  fp32 [N*B*Q] each, same scheme
 *   o, lse_out          fp32 [B,Q,dv], [B,Q] (lse_out may be NULL): complete once exchange_stream has
 *                       drained
 *   workspace           at least helix_attn_hopb_workspace_bytes
 *   events              host array of n_groups + 1 hipEvent_t created by the caller: events[g] marks
 *                       group g's fragments ready, events[n_groups] the end of the call's exchange
 *                       work; the next call on the same buffers waits for it before it overwrites
 *                       send_o / send_lse, so calls may be issued back to back
 * compute_stream == exchange_stream is allowed and runs everything in order (HOP-B off). */
int helix_attn_decode_hopb(const helix_problem *problem, const void *q,
                           const helix_kv_shard *shards, int32_t n_shards, int32_t n_groups,
                           float *o, float *lse_out,
                           float *send_o, float *send_lse, float *recv_o, float *recv_lse,
                           void *workspace, size_t workspace_bytes,
                           void *compute_stream, void *exchange_stream, void *const *events);

/* Workspace bytes helix_attn_decode_hopb needs (the largest group's); 0 if invalid. */
size_t helix_attn_hopb_workspace_bytes(const helix_problem *problem, int32_t n_shards, int32_t max_len,
                                       int32_t n_groups);

/* Fig. 3's timeline as arithmetic: n_requests requests, each t_attn of attention followed by t_comm
 * of exchange.  pipelined == 0: all attention, then all exchange (n*t_attn + n*t_comm); otherwise a
 * two-stage pipeline in which request i's exchange runs under request i+1's attention:
 * t_attn + (n-1)*max(t_attn, t_comm) + t_comm.  Host arithmetic; NaN for n < 1 or negative times. */
double helix_hopb_span(int32_t n_requests, double t_attn, double t_comm, int32_t pipelined);

/* Appendix A: DRAM-read time of one layer's KV cache, the quantity the KVP width of this library's
 * shards divides: B * 2 * ceil(K/TPA) * Hsz * (S/KVP) * bytes_per_param / mem_bw.  Host arithmetic in
 * double; returns NaN for non-positive sizes.  mem_bw in bytes per second (8.0e12 for an MI355X). */
double helix_kv_read_seconds(int64_t B, int64_t K, int64_t Hsz, double S, double bytes_per_param,
                             double mem_bw, int64_t TPA, int64_t KVP);

/* Appendix A: DRAM-read time of one layer's weights (QKV + output projection + SwiGLU FFN):
 * (2*H*(Q/TPA)*Hsz + 2*H*ceil(K/TPA)*Hsz + 3*H*F/TPF) * bytes_per_param / mem_bw. */
double helix_weight_read_seconds(int64_t H, int64_t Q, int64_t K, int64_t Hsz, int64_t F,
                                 double bytes_per_param, double mem_bw, int64_t TPA, int64_t TPF);

/* How the library would cut the work: tokens per workgroup and workgroups of the attention launch
 * for the given shards' max_len (host array [N]): the tokens a workgroup gets if every sequence is that long.
 * For benchmarks and tests; launches nothing. */
int helix_attn_plan(const helix_problem *problem, const int32_t *max_lens, int32_t n_shards,
                    int32_t *split_tokens, int64_t *workgroups);

/* helix_attn_decode_kvp for benchmarks: additionally records `start_event` immediately before and `stop_event`
 * immediately after the call's streaming attention kernel launches (not the small kernels around them), on the
 * call's stream, so that the caller can read that kernel's duration with hipEventElapsedTime.  Both are
 * hipEvent_t handles owned by the caller and must not be NULL.  No state outlives the call. */
int helix_attn_decode_kvp_timed(const helix_problem *problem, const void *q, const helix_kv_shard *cache,
                                int32_t n_shards, float *o, float *lse_out, float *o_partials, float *lses,
                                int64_t *shard_off, int32_t *shard_len,
                                void *workspace, size_t workspace_bytes, void *hip_stream,
                                void *start_event, void *stop_event);

/* Ceiling probes for benchmarks: kernels that do nothing but the memory or matrix access pattern the attention
 * kernels are built on, so that "fraction of what this part sustains" can be measured beside "fraction of the
 * published peak".  Each call enqueues ONE kernel on hip_stream; the caller times it.
 *
 * helix_probe_stream_read: a bare streaming read of `bytes` bytes (a multiple of 16384) of `buf` with the launch
 *   shape of the GQA attention kernels: `workgroups` workgroups of 4 waves, each reading one contiguous chunk
 *   in blocks of 16 KB with 16 x 16-byte loads per lane in flight; nontemporal != 0 uses non-temporal loads as
 *   the attention kernels do.  Nothing is written. */
int helix_probe_stream_read(const void *buf, size_t bytes, int32_t workgroups, int32_t nontemporal, void *hip_stream);

/* helix_probe_mfma_lds: 256 workgroups of 8 waves, each wave issuing `iters` x 8 16x16x32 bf16 MFMAs (iters a
 *   multiple of 8) whose A operand is read from LDS at every instruction; the LDS holds the first 64 KB of
 *   `operands` (bf16 values of the caller's choice: the rate depends on the data).  With stream_buf != NULL every
 *   wave also reads 1 KB of it (non-temporal, addressed modulo stream_bytes, a power of two >= 4 MiB) per 16
 *   MFMAs: 256 flop per byte, the MLA path's ratio of matrix work to HBM bytes.  *flops and *bytes_read (host, may be NULL) receive
 *   the launch's totals. */
int helix_probe_mfma_lds(const void *operands, int32_t iters, const void *stream_buf, size_t stream_bytes,
                         double *flops, double *bytes_read, void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *helix_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* HELIX_ATTN_H */

// C ABI of the Helix decode-attention library for MI355X (gfx950): host-side validation, work
// planning, workspace carving and kernel launches.  See include/helix_attn.h for the contract.
#include "../../include/helix_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>

#include "common.hpp"
#include "gqa_decode.hpp"
#include "gqa_mxfp4.hpp"
#include "merge_combine.hpp"
#include "mla_decode.hpp"

namespace {

using namespace helix;

enum class Path { Gqa64, Gqa128, GqaMx128, Mla };

struct Plan {
    Path path;
    int32_t heads_per_wg;   // query heads one workgroup serves
    int32_t head_tiles;     // workgroups per (b, kv head) along the group
    int32_t granule;        // split_tokens is a multiple of this
    int32_t split_tokens;
    int64_t total_splits;   // over all shards
    int64_t workgroups;
    bool ordered;           // the workgroups take their runs from a map written on the device (run_order_kernel)
};

constexpr int64_t kTargetWorkgroups = 256;   // CUs of an MI355X
constexpr int64_t kMinSplitTokens = 128;        // one block per wave: a launch too small to fill the CUs is latency-bound, shorter runs end sooner
constexpr int64_t kTargetWorkgroupsMx = 768;    // MXFP4 streams 3.8x fewer bytes per token: three workgroups resident per CU
constexpr int64_t kTargetWorkgroupsMla = 4096;   // upper end: keeps the split records of a call near 1 GB at most
constexpr int64_t kMinSplitTokensMla = 4096;

inline int64_t target_workgroups(Path path)
{
    return path == Path::Mla ? kTargetWorkgroupsMla : path == Path::GqaMx128 ? kTargetWorkgroupsMx : kTargetWorkgroups;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_problem(const helix_problem* p, Path* path)
{
    if (!p) return HELIX_ERR_NULL;
    if (p->batch < 1 || p->q_heads < 1 || p->kv_heads < 1 || p->dk < 1 || p->dv < 1) return HELIX_ERR_SHAPE;
    if (p->q_heads % p->kv_heads != 0) return HELIX_ERR_SHAPE;
    if (!(p->scale > 0.f) || !std::isfinite(p->scale)) return HELIX_ERR_SHAPE;
    if (p->split_tokens < 0) return HELIX_ERR_SHAPE;
    if (p->kv_dtype != HELIX_KV_BF16 && p->kv_dtype != HELIX_KV_FP8_E4M3 && p->kv_dtype != HELIX_KV_MXFP4) return HELIX_ERR_UNSUPPORTED;
    if (p->v_aliases_k != 0 && p->v_aliases_k != 1) return HELIX_ERR_SHAPE;
    if (p->v_aliases_k && p->dv > p->dk) return HELIX_ERR_SHAPE;
    if ((int64_t)p->batch * p->q_heads > (int64_t)1 << 24) return HELIX_ERR_SHAPE;
    if (!p->v_aliases_k && p->kv_dtype == HELIX_KV_BF16 && p->dk == p->dv && (p->dk == 64 || p->dk == 128)) {
        *path = p->dk == 64 ? Path::Gqa64 : Path::Gqa128;
        return HELIX_OK;
    }
    if (!p->v_aliases_k && p->kv_dtype == HELIX_KV_MXFP4 && p->dk == 128 && p->dv == 128) {
        *path = Path::GqaMx128;
        return HELIX_OK;
    }
    if (p->v_aliases_k && p->dk == 576 && p->dv == 512 && p->kv_heads == 1) {
        *path = Path::Mla;
        return HELIX_OK;
    }
    return HELIX_ERR_UNSUPPORTED;
}

// Cuts the launch into workgroups.  The streaming kernels are HBM-bound with no reuse.  Measured on
// MI355X, the read rate is highest with about one long-lived workgroup per CU (256 sequential
// streams: 6.8 TB/s at 256 workgroups, 6.5 at 512, 6.2 at 1024 on the 1 GiB GQA share), so the
// target is one workgroup per CU, never less than one per (shard, sequence, kv head, head tile) row,
// with split records that stay small next to the KV bytes a workgroup streams.
// Split records a GQA plan may use per (sequence, kv head, head tile) row when a ragged batch asks for
// runs shorter than its longest sequence needs at one workgroup per CU; the sizing call covers it.
inline int64_t ragged_split_cap(Path path, int64_t rows, int32_t n)
{
    return ceil_div(4 * target_workgroups(path), rows) + n;
}

int make_plan(const helix_problem* p, Path path, const int32_t* max_lens, const int64_t* sum_lens, int32_t n, Plan* plan)
{
    plan->path = path;
    plan->heads_per_wg = path == Path::Mla ? MlaCfg::HPW : 16;
    plan->granule = path == Path::Mla ? 32 : 128;         // MLA: 32-token tiles; GQA: 4 waves x 32-token blocks
    const int g = p->q_heads / p->kv_heads;
    plan->head_tiles = (int32_t)ceil_div(g, plan->heads_per_wg);
    const int64_t rows = (int64_t)p->batch * p->kv_heads * plan->head_tiles;
    int64_t total = 0;       // tokens of a row if every sequence had max_len
    int64_t tokens = 0;      // tokens of all sequences, as far as the caller has told
    bool ragged = false;
    for (int i = 0; i < n; i++) {
        if (max_lens[i] < 0 || (sum_lens && sum_lens[i] < 0)) return HELIX_ERR_SHAPE;
        total += max_lens[i];
        const int64_t full = (int64_t)p->batch * max_lens[i];
        const bool told = sum_lens && sum_lens[i] > 0 && sum_lens[i] < full;
        tokens += told ? sum_lens[i] : full;
        ragged = ragged || told;
    }
    // MLA launches always take their runs from the map (one head tile); the streaming kernels do so for
    // a batch that is declared ragged -- the map costs a launch of its own
    plan->ordered = path == Path::Mla ? plan->head_tiles == 1 : ragged;
    int64_t split;
    if (p->split_tokens > 0) {
        split = ceil_div(p->split_tokens, plan->granule) * plan->granule;
    } else {
        // MLA is compute-bound, one workgroup per CU at a time, and sequence lengths may be ragged (the
        // host only knows the longest): short runs of 4096 tokens let the dispatcher balance the CUs.
        // Measured (runs ordered by run_order_kernel): the ragged e4m3 workload takes 2.81 ms with 4096-token
        // runs, 2.90 with 3072 or 8192, 3.00 with 2048; the uniform bf16 share loses 1 % (3 % of the whole
        // step) against its best (8192).  The 256 KB record of a run is 5-11 % of the latent bytes it reads.
        const int64_t target = target_workgroups(path);
        const int64_t floor_tokens = path == Path::Mla ? kMinSplitTokensMla : kMinSplitTokens;
        const int64_t work = path == Path::Mla ? rows * total : rows / p->batch * tokens;   // token rows to stream
        split = ceil_div(ceil_div(work, target), plan->granule) * plan->granule;
        split = std::max<int64_t>(split, floor_tokens);
        if (path != Path::Mla && ragged) {
            // the longest sequence decides how many records a row needs: keep them within the sizing call's bound
            const int64_t cap = ragged_split_cap(path, rows, n) - n;
            split = std::max<int64_t>(split, ceil_div(ceil_div(total, cap), plan->granule) * plan->granule);
        }
    }
    if (path == Path::GqaMx128) split = std::min<int64_t>(split, (int64_t)1 << 25);   // 32-bit byte offsets inside a split
    plan->split_tokens = (int32_t)split;
    plan->total_splits = 0;
    for (int i = 0; i < n; i++) plan->total_splits += std::max<int64_t>(1, ceil_div(max_lens[i], split));
    plan->workgroups = plan->total_splits * rows;   // MLA launches pad this per shard to whole groups of 8
    if (plan->workgroups > (int64_t)1 << 30) return HELIX_ERR_SHAPE;
    return HELIX_OK;
}

struct Workspace {
    float* ws_o;
    float* ws_m;
    float* ws_l;
    float* part_o;
    float* part_lse;
    uint2* units;           // MLA: the run each workgroup serves (run_order_kernel), one entry per split record row
    size_t bytes;
};

// Carves a workspace for `total_splits` records and `n` shard partials.  base may be NULL (sizing).
Workspace carve(const helix_problem* p, int64_t total_splits, int64_t rows, int32_t n, void* base)
{
    const size_t bq = (size_t)p->batch * p->q_heads;
    char* c = static_cast<char*>(base);
    size_t off = 0;
    Workspace w;
    w.ws_o = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)total_splits * bq * p->dv * 4, 256);
    w.ws_m = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)total_splits * bq * 4, 256);
    w.ws_l = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)total_splits * bq * 4, 256);
    w.part_o = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)n * bq * p->dv * 4, 256);
    w.part_lse = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)n * bq * 4, 256);
    w.units = reinterpret_cast<uint2*>(c + off); off = align_up(off + (size_t)total_splits * rows * sizeof(uint2), 256);
    w.bytes = off;
    return w;
}

int check_shard(const helix_problem* p, const helix_kv_shard* s)
{
    if (!s->k || !s->len) return HELIX_ERR_NULL;
    if (p->v_aliases_k ? s->v != nullptr : s->v == nullptr) return p->v_aliases_k ? HELIX_ERR_SHAPE : HELIX_ERR_NULL;
    const bool fp8 = p->kv_dtype == HELIX_KV_FP8_E4M3;
    if (fp8 ? s->kv_scale == nullptr : false) return HELIX_ERR_NULL;
    if (s->max_len < 0 || s->sum_len < 0) return HELIX_ERR_SHAPE;
    if (p->kv_dtype == HELIX_KV_MXFP4) {
        // strides count elements; a row is dk/2 code bytes and dk/32 scale bytes, token rows dense
        if (!s->k_scale_mx) return HELIX_ERR_NULL;
        if (s->k_stride_b < 0 || s->k_stride_h < 0 || s->k_stride_b % 128 || s->k_stride_h % 128) return HELIX_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(s->k) % 16 || reinterpret_cast<uintptr_t>(s->k_scale_mx) % 4) return HELIX_ERR_SHAPE;
        if (s->k_stride_t != p->dk) return HELIX_ERR_UNSUPPORTED;
        if (p->v_aliases_k) return s->v_scale_mx ? HELIX_ERR_SHAPE : HELIX_OK;      // the latent's scales serve key and value
        if (!s->v_scale_mx) return HELIX_ERR_NULL;
        if (s->v_stride_b < 0 || s->v_stride_h < 0 || s->v_stride_b % 128 || s->v_stride_h % 128) return HELIX_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(s->v) % 16 || reinterpret_cast<uintptr_t>(s->v_scale_mx) % 4) return HELIX_ERR_SHAPE;
        if (s->v_stride_t != p->dv) return HELIX_ERR_UNSUPPORTED;
        return HELIX_OK;
    }
    const int64_t esz = fp8 ? 1 : 2, mult = 16 / esz;
    if (s->k_stride_t < p->dk || s->k_stride_t > ((int64_t)1 << 24) || s->k_stride_b < 0 || s->k_stride_h < 0) return HELIX_ERR_SHAPE;
    if (s->k_stride_t % mult || s->k_stride_b % mult || s->k_stride_h % mult) return HELIX_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(s->k) % 16) return HELIX_ERR_SHAPE;
    if (!p->v_aliases_k) {
        if (s->v_stride_t < p->dv || s->v_stride_t > ((int64_t)1 << 24) || s->v_stride_b < 0 || s->v_stride_h < 0) return HELIX_ERR_SHAPE;
        if (s->v_stride_t % mult || s->v_stride_b % mult || s->v_stride_h % mult) return HELIX_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(s->v) % 16) return HELIX_ERR_SHAPE;
    }
    if (fp8 && (s->s_stride_b < 0 || s->s_stride_h < 0)) return HELIX_ERR_SHAPE;
    return HELIX_OK;
}

hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;   // helix_attn_set_profile_events

int launch_status()
{
    return hipGetLastError() == hipSuccess ? HELIX_OK : HELIX_ERR_LAUNCH;
}

template <int DV>
int launch_combine(const float* o_parts, const float* lses, float* o, float* lse_out, int32_t* argmax,
                   int32_t n, int64_t rows, hipStream_t stream)
{
    constexpr int RPB = 256 / (DV / 4);
    const unsigned grid = (unsigned)ceil_div(rows, RPB);
    hipLaunchKernelGGL((combine_kernel<DV>), dim3(grid), dim3(256), 0, stream, o_parts, lses, o, lse_out, argmax, n, rows);
    return launch_status();
}

int combine_any(int32_t dv, const float* o_parts, const float* lses, float* o, float* lse_out, int32_t* argmax,
                int32_t n, int64_t rows, hipStream_t stream)
{
    switch (dv) {
        case 64: return launch_combine<64>(o_parts, lses, o, lse_out, argmax, n, rows, stream);
        case 128: return launch_combine<128>(o_parts, lses, o, lse_out, argmax, n, rows, stream);
        case 512: return launch_combine<512>(o_parts, lses, o, lse_out, argmax, n, rows, stream);
        default: return HELIX_ERR_UNSUPPORTED;
    }
}

// n > 0: every descriptor handed to run_partials describes the whole cache and shard i is cut inside
// the kernels as slice i of n (Sec. 2.1.1); off / len ([n, B], may be NULL) receive the cut.
struct KvpCut {
    int32_t n = 0;
    int64_t* off = nullptr;
    int32_t* len = nullptr;
};

// Attention over `n` shards into per-shard partials (o_part [n,B,Q,dv], lse_part [n,B,Q]).
// With `o` non-NULL and n <= kMaxLaunchShards the merge and the combine run fused (finish_kernel)
// and *finished is set; otherwise the caller still has to combine.
int run_partials(const helix_problem* p, const Plan& plan, const void* q, const helix_kv_shard* shards, int32_t n,
                 const Workspace& ws, float* o_part, float* lse_part, hipStream_t stream,
                 float* o = nullptr, float* lse_out = nullptr, bool* finished = nullptr, KvpCut cut = KvpCut())
{
    const bool fuse = o != nullptr && n <= kMaxLaunchShards;
    if (finished) *finished = fuse;
    const int g = p->q_heads / p->kv_heads;
    const int64_t rows = (int64_t)p->batch * p->kv_heads * plan.head_tiles;
    int32_t split_base = 0;
    for (int32_t s0 = 0; s0 < n; s0 += kMaxLaunchShards) {
        const int32_t cnt = std::min<int32_t>(kMaxLaunchShards, n - s0);
        AttnArgs a;
        std::memset(&a, 0, sizeof a);
        MergeArgs m;
        std::memset(&m, 0, sizeof m);
        a.q = static_cast<const uint16_t*>(q);
        a.ws_o = ws.ws_o; a.ws_m = ws.ws_m; a.ws_l = ws.ws_l;
        a.B = p->batch; a.Q = p->q_heads; a.K = p->kv_heads; a.g = g;
        a.head_tiles = plan.head_tiles;
        a.split_tokens = plan.split_tokens;
        a.scale_log2e = p->scale * kLog2e;
        a.n_shards = cnt;
        int64_t units = 0;
        for (int32_t i = 0; i < cnt; i++) {
            const helix_kv_shard& s = shards[s0 + i];
            ShardDev& d = a.shard[i];
            d.k = s.k; d.v = s.v; d.kv_scale = s.kv_scale; d.tok_off = s.tok_off; d.len = s.len;
            d.k_sb = s.k_stride_b; d.k_sh = s.k_stride_h; d.k_st = s.k_stride_t;
            d.v_sb = s.v_stride_b; d.v_sh = s.v_stride_h; d.v_st = s.v_stride_t;
            d.s_sb = s.s_stride_b; d.s_sh = s.s_stride_h;
            d.k_mx = s.k_scale_mx; d.v_mx = s.v_scale_mx;
            d.kvp_n = cut.n; d.kvp_i = s0 + i;
            d.out_off = cut.off ? cut.off + (int64_t)(s0 + i) * p->batch : nullptr;
            d.out_len = cut.len ? cut.len + (int64_t)(s0 + i) * p->batch : nullptr;
            d.n_splits = (int32_t)std::max<int64_t>(1, ceil_div(s.max_len, plan.split_tokens));
            d.split_base = split_base;
            d.unit_base = (int32_t)units;
            m.split_base[i] = split_base;
            m.n_splits[i] = d.n_splits;
            split_base += d.n_splits;
            units += plan.path == Path::Mla && !plan.ordered ? mla_units_of_shard(d.n_splits, p->batch, plan.head_tiles)
                                                                   : (int64_t)d.n_splits * rows;
        }
        // MLA with one head tile: the runs are handed to the workgroups in the order run_order_kernel
        // writes -- full runs first, then partial ones, then empty ones (see there)
        if (plan.ordered) {
            hipLaunchKernelGGL(helix::run_order_kernel, dim3(1), dim3(helix::kOrderThreads), 0, stream, a, ws.units, (int)units);
            if (int rc = launch_status()) return rc;
            a.units = ws.units;
        }
        if (g_prof_start && g_prof_stop && s0 == 0) (void)hipEventRecord(g_prof_start, stream);
        switch (plan.path) {
            case Path::Gqa64:
                hipLaunchKernelGGL((gqa_decode_kernel<64>), dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::Gqa128:
                hipLaunchKernelGGL((gqa_decode_kernel<128>), dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::GqaMx128:
                hipLaunchKernelGGL(gqa_mxfp4_kernel, dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::Mla: {
                const int kind = p->kv_dtype == HELIX_KV_FP8_E4M3 ? 1 : p->kv_dtype == HELIX_KV_MXFP4 ? 2 : 0;
                auto kern = kind == 2 ? mla_decode_kernel<true, true> : kind == 1 ? mla_decode_kernel<true> : mla_decode_kernel<false>;
                // more than the default 64 KB of LDS per workgroup has to be asked for: once per device and
                // kernel, so that later calls consist of launches only (and can be captured into a HIP graph)
                static bool asked[3][64];
                int dev = 0;
                if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return HELIX_ERR_LAUNCH;
                if (!asked[kind][dev]) {
                    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                            MlaCfg::LDS_BYTES) != hipSuccess)
                        return HELIX_ERR_LAUNCH;
                    asked[kind][dev] = true;
                }
                hipLaunchKernelGGL(kern, dim3((unsigned)units), dim3(MlaCfg::THREADS), MlaCfg::LDS_BYTES, stream, a);
                break;
            }
            default:
                return HELIX_ERR_UNSUPPORTED;
        }
        if (int rc = launch_status()) return rc;
        if (g_prof_start && g_prof_stop && s0 + cnt >= n) (void)hipEventRecord(g_prof_stop, stream);
        m.ws_o = ws.ws_o; m.ws_m = ws.ws_m; m.ws_l = ws.ws_l;
        m.o_part = o_part; m.lse_part = lse_part;
        m.B = p->batch; m.Q = p->q_heads; m.n_shards = cnt; m.shard0 = s0;
        if (fuse) {
            FinishArgs f;
            f.m = m; f.o = o; f.lse_out = lse_out;
            const unsigned frows = (unsigned)((int64_t)p->batch * p->q_heads);
            switch (p->dv) {
                case 64: hipLaunchKernelGGL((finish_kernel<64>), dim3(frows), dim3(256), 0, stream, f); break;
                case 128: hipLaunchKernelGGL((finish_kernel<128>), dim3(frows), dim3(256), 0, stream, f); break;
                case 512: hipLaunchKernelGGL((finish_kernel<512>), dim3(frows), dim3(256), 0, stream, f); break;
                default: return HELIX_ERR_UNSUPPORTED;
            }
            return launch_status();
        }
        const unsigned mrows = (unsigned)((int64_t)cnt * p->batch * p->q_heads);
        switch (p->dv) {
            case 64: hipLaunchKernelGGL((merge_splits_kernel<64>), dim3(mrows), dim3(256), 0, stream, m); break;
            case 128: hipLaunchKernelGGL((merge_splits_kernel<128>), dim3(mrows), dim3(256), 0, stream, m); break;
            case 512: hipLaunchKernelGGL((merge_splits_kernel<512>), dim3(mrows), dim3(256), 0, stream, m); break;
            default: return HELIX_ERR_UNSUPPORTED;
        }
        if (int rc = launch_status()) return rc;
    }
    return HELIX_OK;
}

int prepare(const helix_problem* p, const helix_kv_shard* shards, int32_t n, void* workspace, size_t workspace_bytes,
            Plan* plan, Workspace* ws)
{
    Path path;
    if (int rc = check_problem(p, &path)) return rc;
    if (!shards) return HELIX_ERR_NULL;
    if (n < 1 || n > HELIX_MAX_SHARDS) return HELIX_ERR_SHAPE;
    int32_t max_lens[HELIX_MAX_SHARDS];
    int64_t sum_lens[HELIX_MAX_SHARDS];
    for (int32_t i = 0; i < n; i++) {
        if (int rc = check_shard(p, &shards[i])) return rc;
        max_lens[i] = shards[i].max_len;
        sum_lens[i] = shards[i].sum_len;
    }
    if (int rc = make_plan(p, path, max_lens, sum_lens, n, plan)) return rc;
    *ws = carve(p, plan->total_splits, (int64_t)p->batch * p->kv_heads * plan->head_tiles, n, workspace);
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || ws->bytes > workspace_bytes) return HELIX_ERR_WORKSPACE;
    return HELIX_OK;
}

}  // namespace

extern "C" {

const char* helix_status_string(int status)
{
    switch (status) {
        case HELIX_OK: return "ok";
        case HELIX_ERR_NULL: return "a required pointer is NULL";
        case HELIX_ERR_SHAPE: return "invalid shape, stride or alignment";
        case HELIX_ERR_UNSUPPORTED: return "unsupported combination of head widths / dtype";
        case HELIX_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case HELIX_ERR_LAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}

int helix_attn_set_profile_events(void* start_event, void* stop_event)
{
    if ((start_event == nullptr) != (stop_event == nullptr)) return HELIX_ERR_NULL;
    g_prof_start = static_cast<hipEvent_t>(start_event);
    g_prof_stop = static_cast<hipEvent_t>(stop_event);
    return HELIX_OK;
}

int helix_attn_plan(const helix_problem* problem, const int32_t* max_lens, const int64_t* sum_lens, int32_t n_shards,
                    int32_t* split_tokens, int64_t* workgroups)
{
    Path path;
    if (int rc = check_problem(problem, &path)) return rc;
    if (!max_lens) return HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS) return HELIX_ERR_SHAPE;
    Plan plan;
    if (int rc = make_plan(problem, path, max_lens, sum_lens, n_shards, &plan)) return rc;
    if (split_tokens) *split_tokens = plan.split_tokens;
    if (workgroups) *workgroups = plan.workgroups;
    return HELIX_OK;
}

size_t helix_attn_workspace_bytes(const helix_problem* problem, int32_t n_shards, int32_t max_len)
{
    Path path;
    if (check_problem(problem, &path) != HELIX_OK) return 0;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS || max_len < 0) return 0;
    // The plan's split count grows when shards are shorter than max_len (smaller splits keep the
    // workgroup count up), so size for the worst case over all max_len_i <= max_len.
    int32_t lens[HELIX_MAX_SHARDS];
    for (int i = 0; i < n_shards; i++) lens[i] = max_len;
    Plan plan;
    if (make_plan(problem, path, lens, nullptr, n_shards, &plan) != HELIX_OK) return 0;
    const int64_t rows = (int64_t)problem->batch * problem->kv_heads * plan.head_tiles;
    int64_t worst = plan.total_splits;
    if (problem->split_tokens == 0) {
        worst = std::max<int64_t>(worst, ceil_div(target_workgroups(path), rows) + n_shards);
        if (path != Path::Mla) worst = std::max<int64_t>(worst, ragged_split_cap(path, rows, n_shards));   // a batch declared ragged
    }
    return carve(problem, worst, rows, n_shards, nullptr).bytes;
}

int helix_attn_partial(const helix_problem* problem, const void* q, const helix_kv_shard* shard,
                       float* o_partial, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!q || !o_partial || !lse) return HELIX_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(o_partial) % 16) return HELIX_ERR_SHAPE;
    Plan plan;
    Workspace ws;
    if (int rc = prepare(problem, shard, 1, workspace, workspace_bytes, &plan, &ws)) return rc;
    return run_partials(problem, plan, q, shard, 1, ws, o_partial, lse, static_cast<hipStream_t>(hip_stream));
}

int helix_attn_combine(const helix_problem* problem, int32_t n_shards, const float* o_partials, const float* lses,
                       float* o, float* lse_out, int32_t* argmax_shard, void* hip_stream)
{
    if (!problem || !o_partials || !lses || !o) return HELIX_ERR_NULL;
    if (problem->batch < 1 || problem->q_heads < 1 || n_shards < 1 || n_shards > HELIX_MAX_SHARDS) return HELIX_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(o_partials) % 16 || reinterpret_cast<uintptr_t>(o) % 16) return HELIX_ERR_SHAPE;
    const int64_t rows = (int64_t)problem->batch * problem->q_heads;
    return combine_any(problem->dv, o_partials, lses, o, lse_out, argmax_shard, n_shards, rows,
                       static_cast<hipStream_t>(hip_stream));
}

int helix_attn_decode(const helix_problem* problem, const void* q, const helix_kv_shard* shards, int32_t n_shards,
                      float* o, float* lse_out, float* o_partials, float* lses,
                      void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!q || !o) return HELIX_ERR_NULL;
    if ((o_partials == nullptr) != (lses == nullptr)) return HELIX_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(o) % 16 ||
        reinterpret_cast<uintptr_t>(o_partials) % 16) return HELIX_ERR_SHAPE;
    Plan plan;
    Workspace ws;
    if (int rc = prepare(problem, shards, n_shards, workspace, workspace_bytes, &plan, &ws)) return rc;
    float* po = o_partials ? o_partials : ws.part_o;
    float* pl = lses ? lses : ws.part_lse;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    bool finished = false;
    if (int rc = run_partials(problem, plan, q, shards, n_shards, ws, po, pl, stream, o, lse_out, &finished)) return rc;
    if (finished) return HELIX_OK;
    const int64_t rows = (int64_t)problem->batch * problem->q_heads;
    return combine_any(problem->dv, po, pl, o, lse_out, nullptr, n_shards, rows, stream);
}

namespace {
// The descriptors of sequences b0 .. of a shard: every base pointer advanced by b0 batch strides.
helix_kv_shard shard_of_group(const helix_problem* p, const helix_kv_shard& s, int32_t b0)
{
    helix_kv_shard g = s;
    const int64_t num = p->kv_dtype == HELIX_KV_BF16 ? 2 : 1, den = p->kv_dtype == HELIX_KV_MXFP4 ? 2 : 1;
    g.k = static_cast<const char*>(s.k) + b0 * s.k_stride_b * num / den;
    if (s.v) g.v = static_cast<const char*>(s.v) + b0 * s.v_stride_b * num / den;
    if (s.kv_scale) g.kv_scale = s.kv_scale + b0 * s.s_stride_b;
    if (s.k_scale_mx) g.k_scale_mx = s.k_scale_mx + b0 * s.k_stride_b / 32;
    if (s.v_scale_mx) g.v_scale_mx = s.v_scale_mx + b0 * s.v_stride_b / 32;
    if (s.tok_off) g.tok_off = s.tok_off + b0;
    g.len = s.len + b0;
    return g;
}
}  // namespace

size_t helix_attn_hopb_workspace_bytes(const helix_problem* problem, int32_t n_shards, int32_t max_len, int32_t n_groups)
{
    if (!problem || n_groups < 1 || n_groups > problem->batch) return 0;
    helix_problem sub = *problem;
    sub.batch = (int32_t)ceil_div(problem->batch, n_groups);
    const size_t a = helix_attn_workspace_bytes(&sub, n_shards, max_len);
    sub.batch = problem->batch - (n_groups - 1) * sub.batch > 0 ? problem->batch - (n_groups - 1) * sub.batch : sub.batch;
    const size_t b = helix_attn_workspace_bytes(&sub, n_shards, max_len);
    return a == 0 || b == 0 ? 0 : std::max(a, b);
}

int helix_attn_decode_hopb(const helix_problem* problem, const void* q, const helix_kv_shard* shards, int32_t n_shards,
                           int32_t n_groups, float* o, float* lse_out,
                           float* send_o, float* send_lse, float* recv_o, float* recv_lse,
                           void* workspace, size_t workspace_bytes,
                           void* compute_stream, void* exchange_stream, void* const* events)
{
    Path path;
    if (int rc = check_problem(problem, &path)) return rc;
    if (!q || !o || !shards || !send_o || !send_lse || !recv_o || !recv_lse || !events) return HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS || n_groups < 1 || n_groups > problem->batch) return HELIX_ERR_SHAPE;
    for (int g = 0; g <= n_groups; g++)
        if (!events[g]) return HELIX_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(o) % 16 || reinterpret_cast<uintptr_t>(send_o) % 16 ||
        reinterpret_cast<uintptr_t>(recv_o) % 16) return HELIX_ERR_SHAPE;
    hipStream_t cs = static_cast<hipStream_t>(compute_stream), xs = static_cast<hipStream_t>(exchange_stream);
    const int32_t B = problem->batch, Q = problem->q_heads, dv = problem->dv, N = n_shards;
    const int32_t per = (int32_t)ceil_div(B, n_groups);
    // validate everything before the first launch: an error return means no kernel ran
    helix_kv_shard sub[HELIX_MAX_SHARDS];                  // on the stack: the library allocates nothing
    for (int32_t b0 = 0; b0 < B; b0 += per) {
        helix_problem sp = *problem;
        sp.batch = std::min(per, B - b0);
        for (int32_t i = 0; i < N; i++) sub[i] = shard_of_group(problem, shards[i], b0);
        Plan plan;
        Workspace ws;
        if (int rc = prepare(&sp, sub, N, workspace, workspace_bytes, &plan, &ws)) return rc;
    }
    // the previous call's exchange may still be reading the send buffers
    if (hipStreamWaitEvent(cs, static_cast<hipEvent_t>(events[n_groups]), 0) != hipSuccess) return HELIX_ERR_LAUNCH;
    int g = 0;
    for (int32_t b0 = 0; b0 < B; b0 += per, g++) {
        helix_problem sp = *problem;
        sp.batch = std::min(per, B - b0);
        for (int32_t i = 0; i < N; i++) sub[i] = shard_of_group(problem, shards[i], b0);
        Plan plan;
        Workspace ws;
        if (int rc = prepare(&sp, sub, N, workspace, workspace_bytes, &plan, &ws)) return rc;
        const size_t off_o = (size_t)N * b0 * Q * dv, off_l = (size_t)N * b0 * Q;
        const size_t n_o = (size_t)N * sp.batch * Q * dv, n_l = (size_t)N * sp.batch * Q;
        const char* qg = static_cast<const char*>(q) + (size_t)b0 * Q * problem->dk * 2;
        if (int rc = run_partials(&sp, plan, qg, sub, N, ws, send_o + off_o, send_lse + off_l, cs)) return rc;
        hipEvent_t ready = static_cast<hipEvent_t>(events[g]);
        if (hipEventRecord(ready, cs) != hipSuccess || hipStreamWaitEvent(xs, ready, 0) != hipSuccess) return HELIX_ERR_LAUNCH;
        if (hipMemcpyAsync(recv_o + off_o, send_o + off_o, n_o * 4, hipMemcpyDeviceToDevice, xs) != hipSuccess ||
            hipMemcpyAsync(recv_lse + off_l, send_lse + off_l, n_l * 4, hipMemcpyDeviceToDevice, xs) != hipSuccess)
            return HELIX_ERR_LAUNCH;
        if (int rc = combine_any(dv, recv_o + off_o, recv_lse + off_l, o + (size_t)b0 * Q * dv,
                                 lse_out ? lse_out + (size_t)b0 * Q : nullptr, nullptr, N, (int64_t)sp.batch * Q, xs))
            return rc;
    }
    if (hipEventRecord(static_cast<hipEvent_t>(events[n_groups]), xs) != hipSuccess) return HELIX_ERR_LAUNCH;
    return HELIX_OK;
}

double helix_hopb_span(int32_t n_requests, double t_attn, double t_comm, int32_t pipelined)
{
    if (n_requests < 1 || !(t_attn >= 0) || !(t_comm >= 0)) return NAN;
    if (!pipelined) return n_requests * t_attn + n_requests * t_comm;
    return t_attn + (n_requests - 1) * std::max(t_attn, t_comm) + t_comm;
}

int helix_attn_decode_kvp(const helix_problem* problem, const void* q, const helix_kv_shard* cache, int32_t n_shards,
                          float* o, float* lse_out, float* o_partials, float* lses,
                          int64_t* shard_off, int32_t* shard_len,
                          void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!q || !o || !cache) return HELIX_ERR_NULL;
    if ((o_partials == nullptr) != (lses == nullptr) || (shard_off == nullptr) != (shard_len == nullptr)) return HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS) return HELIX_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(o) % 16 ||
        reinterpret_cast<uintptr_t>(o_partials) % 16) return HELIX_ERR_SHAPE;
    if (cache->max_len < 0) return HELIX_ERR_SHAPE;
    // every slice is at most c = 16 * ceil(ceil(max_len / N) / 16) tokens long
    helix_kv_shard slices[HELIX_MAX_SHARDS];               // on the stack: the library allocates nothing
    const int64_t per = ceil_div(cache->max_len, n_shards);
    const int32_t c = (int32_t)std::min<int64_t>(16 * ceil_div(per, 16), cache->max_len);
    for (int32_t i = 0; i < n_shards; i++) {
        slices[i] = *cache;
        slices[i].max_len = c;
        // a slice holds a N-th of every sequence, rounded up to whole 16-token blocks
        if (cache->sum_len > 0) slices[i].sum_len = std::min<int64_t>(ceil_div(cache->sum_len, n_shards) + 16 * (int64_t)problem->batch, (int64_t)problem->batch * c);
    }
    Plan plan;
    Workspace ws;
    if (int rc = prepare(problem, slices, n_shards, workspace, workspace_bytes, &plan, &ws)) return rc;
    float* po = o_partials ? o_partials : ws.part_o;
    float* pl = lses ? lses : ws.part_lse;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    KvpCut cut;
    cut.n = n_shards; cut.off = shard_off; cut.len = shard_len;
    bool finished = false;
    if (int rc = run_partials(problem, plan, q, slices, n_shards, ws, po, pl, stream, o, lse_out, &finished, cut)) return rc;
    if (finished) return HELIX_OK;
    const int64_t rows = (int64_t)problem->batch * problem->q_heads;
    return combine_any(problem->dv, po, pl, o, lse_out, nullptr, n_shards, rows, stream);
}

int32_t helix_kv_append_owner(int64_t decode_index, int32_t n_shards)
{
    if (n_shards < 1 || decode_index < 0) return -1;
    return (int32_t)((decode_index / HELIX_APPEND_BLOCK) % n_shards);
}

namespace {
int append_common(const helix_problem* problem, const helix_kv_shard* shards, int32_t n_shards, int64_t decode_index,
                  const void* k_new, const void* v_new, const float* scale_new, const uint8_t* k_mx_new, const uint8_t* v_mx_new,
                  int32_t capacity, int32_t* overflow, void* hip_stream)
{
    const helix_kv_shard& s = shards[helix_kv_append_owner(decode_index, n_shards)];
    if (int rc = check_shard(problem, &s)) return rc;
    const bool fp8 = problem->kv_dtype == HELIX_KV_FP8_E4M3, fp4 = problem->kv_dtype == HELIX_KV_MXFP4;
    AppendArgs a;
    std::memset(&a, 0, sizeof a);
    a.sh.k = s.k; a.sh.v = s.v; a.sh.kv_scale = s.kv_scale; a.sh.tok_off = s.tok_off; a.sh.len = s.len;
    a.sh.k_sb = s.k_stride_b; a.sh.k_sh = s.k_stride_h; a.sh.k_st = s.k_stride_t;
    a.sh.v_sb = s.v_stride_b; a.sh.v_sh = s.v_stride_h; a.sh.v_st = s.v_stride_t;
    a.sh.s_sb = s.s_stride_b; a.sh.s_sh = s.s_stride_h;
    a.sh.k_mx = s.k_scale_mx; a.sh.v_mx = s.v_scale_mx;
    a.k_new = static_cast<const uint8_t*>(k_new);
    a.v_new = static_cast<const uint8_t*>(v_new);
    a.scale_new = scale_new;
    a.k_mx_new = k_mx_new; a.v_mx_new = v_mx_new;
    a.len = const_cast<int32_t*>(s.len);
    a.overflow = overflow;
    a.K = problem->kv_heads; a.dk = problem->dk; a.dv = problem->dv; a.capacity = capacity;
    a.num = fp4 || fp8 ? 1 : 2; a.den = fp4 ? 2 : 1;
    hipLaunchKernelGGL(helix::kv_append_kernel, dim3((unsigned)problem->batch), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), a);
    return launch_status();
}
}  // namespace

int helix_kv_append(const helix_problem* problem, const helix_kv_shard* shards, int32_t n_shards,
                    int64_t decode_index, const void* k_new, const void* v_new, const float* scale_new,
                    int32_t capacity, int32_t* overflow, void* hip_stream)
{
    Path path;
    if (int rc = check_problem(problem, &path)) return rc;
    if (problem->kv_dtype == HELIX_KV_MXFP4) return HELIX_ERR_UNSUPPORTED;      // helix_kv_append_mxfp4 carries the block scales
    if (!shards || !k_new) return HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS || decode_index < 0 || capacity < 0) return HELIX_ERR_SHAPE;
    const bool fp8 = problem->kv_dtype == HELIX_KV_FP8_E4M3;
    if (problem->v_aliases_k ? v_new != nullptr : v_new == nullptr) return problem->v_aliases_k ? HELIX_ERR_SHAPE : HELIX_ERR_NULL;
    if (fp8 ? scale_new == nullptr : scale_new != nullptr) return fp8 ? HELIX_ERR_NULL : HELIX_ERR_SHAPE;
    return append_common(problem, shards, n_shards, decode_index, k_new, v_new, scale_new, nullptr, nullptr, capacity, overflow, hip_stream);
}

int helix_kv_append_mxfp4(const helix_problem* problem, const helix_kv_shard* shards, int32_t n_shards,
                          int64_t decode_index, const void* k_codes, const void* v_codes,
                          const uint8_t* k_scales, const uint8_t* v_scales,
                          int32_t capacity, int32_t* overflow, void* hip_stream)
{
    Path path;
    if (int rc = check_problem(problem, &path)) return rc;
    if (problem->kv_dtype != HELIX_KV_MXFP4) return HELIX_ERR_UNSUPPORTED;
    if (!shards || !k_codes || !k_scales) return HELIX_ERR_NULL;
    if (problem->v_aliases_k ? (v_codes || v_scales) : (!v_codes || !v_scales)) return problem->v_aliases_k ? HELIX_ERR_SHAPE : HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS || decode_index < 0 || capacity < 0) return HELIX_ERR_SHAPE;
    return append_common(problem, shards, n_shards, decode_index, k_codes, v_codes, nullptr, k_scales, v_scales, capacity, overflow, hip_stream);
}

double helix_kv_read_seconds(int64_t B, int64_t K, int64_t Hsz, double S, double bytes_per_param,
                             double mem_bw, int64_t TPA, int64_t KVP)
{
    if (B < 1 || K < 1 || Hsz < 1 || !(S >= 0) || !(bytes_per_param > 0) || !(mem_bw > 0) || TPA < 1 || KVP < 1) return NAN;
    const double heads = (double)ceil_div(K, TPA);         // a KV head is never split: TPA > K duplicates it
    return (double)B * 2.0 * heads * (double)Hsz * (S / (double)KVP) * bytes_per_param / mem_bw;
}

double helix_weight_read_seconds(int64_t H, int64_t Q, int64_t K, int64_t Hsz, int64_t F,
                                 double bytes_per_param, double mem_bw, int64_t TPA, int64_t TPF)
{
    if (H < 1 || Q < 1 || K < 1 || Hsz < 1 || F < 1 || !(bytes_per_param > 0) || !(mem_bw > 0) || TPA < 1 || TPF < 1) return NAN;
    const double q_and_out = 2.0 * (double)H * ((double)Q / (double)TPA) * (double)Hsz;
    const double kv = 2.0 * (double)H * (double)ceil_div(K, TPA) * (double)Hsz;
    const double ffn = 3.0 * ((double)H * (double)F / (double)TPF);
    return (q_and_out + kv + ffn) * bytes_per_param / mem_bw;
}

int helix_shard_layout(const int32_t* seq_len, const int64_t* seq_base, int32_t batch, int32_t n_shards,
                       int64_t* shard_off, int32_t* shard_len, void* hip_stream)
{
    if (!seq_len || !shard_off || !shard_len) return HELIX_ERR_NULL;
    if (batch < 1 || n_shards < 1 || n_shards > HELIX_MAX_SHARDS || (int64_t)batch * n_shards > (int64_t)1 << 30) return HELIX_ERR_SHAPE;
    const int total = batch * n_shards;
    hipLaunchKernelGGL(helix::shard_layout_kernel, dim3((total + 255) / 256), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), seq_len, seq_base, batch, n_shards, shard_off, shard_len);
    return launch_status();
}

}  // extern "C"

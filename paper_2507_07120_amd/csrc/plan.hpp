// Host side of the C ABI that needs no GPU: argument validation, the cut of a launch into workgroups
// and the carving of the caller's workspace.  Plain C++ without any HIP type, so that it can also be
// compiled into a host-only test program (address / undefined-behaviour sanitizers run there).
#pragma once
#include "../../include/helix_attn.h"

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdint>

namespace helix_host {

enum class Path { Gqa64, Gqa128, GqaMx128, Mla };

struct Plan {
    Path path;
    int32_t heads_per_wg;   // query heads one workgroup serves
    int32_t head_tiles;     // workgroups per (b, kv head) along the group
    int32_t granule;        // split_tokens is a multiple of this
    int32_t split_tokens;
    int64_t total_splits;   // split records of the call, over all shards
    int64_t workgroups;
    bool ordered;           // the workgroups take their runs from a map written on the device (run_order_kernel)
    bool stream;            // MLA with one head tile: every launch is cut evenly over its token stream (stream_plan_kernel)
    size_t map_bytes;       // device-written maps of the call (run map, or tile prefix + first pair per workgroup)
};

constexpr int kMlaHeadsPerWorkgroup = 128;      // checked against the kernel's configuration where both are visible
constexpr int64_t kTargetWorkgroups = 256;      // CUs of an MI355X
constexpr int64_t kMinSplitTokens = 128;        // one block per wave: a launch too small to fill the CUs is latency-bound, shorter runs end sooner
constexpr int64_t kTargetWorkgroupsMx = 768;    // MXFP4 streams 3.8x fewer bytes per token: three workgroups resident per CU
constexpr int64_t kTargetWorkgroupsMla = 4096;  // upper end: keeps the split records of a call near 1 GB at most
constexpr int64_t kMinSplitTokensMla = 4096;

inline int64_t target_workgroups(Path path)
{
    return path == Path::Mla ? kTargetWorkgroupsMla : path == Path::GqaMx128 ? kTargetWorkgroupsMx : kTargetWorkgroups;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kMaxShardsPerLaunch = 16;         // shard descriptors travel by value in the kernel arguments
constexpr int64_t kStreamMinTokens = 256;       // an evenly cut MLA launch gives a workgroup at least this many tokens ...
constexpr int64_t kStreamWorkgroups = 256;      // ... and uses at most one workgroup per CU

// Workgroups of an evenly cut MLA launch over shards whose longest sequences add up to `tokens` per sequence slot
// (batch * sum of max_len): one per CU unless the launch is small, or as many as the caller's run length asks for.
inline int64_t stream_workgroups(const helix_problem* p, int64_t tokens)
{
    if (p->split_tokens > 0) return std::max<int64_t>(1, ceil_div(tokens, ceil_div(p->split_tokens, 32) * 32));
    return std::min(kStreamWorkgroups, std::max<int64_t>(1, tokens / kStreamMinTokens));
}

// Bytes of the maps stream_plan_kernel writes for a launch of `cnt` shards and `n_wg` workgroups, 256-byte aligned
inline size_t stream_map_bytes(int64_t pairs, int64_t n_wg)
{
    // tile prefix [pairs + 1] int64, workgroups of every pair [pairs] 2 x int32, first pair of every workgroup [n_wg] int32
    return ((size_t)(pairs + 1) * 8 + 255) / 256 * 256 + ((size_t)pairs * 8 + 255) / 256 * 256 + ((size_t)n_wg * 4 + 255) / 256 * 256;
}

inline int check_problem(const helix_problem* p, Path* path)
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

// Split records a GQA plan may use per (sequence, kv head, head tile) row when a ragged batch asks for
// runs shorter than its longest sequence needs at one workgroup per CU; the sizing call covers it.
inline int64_t ragged_split_cap(Path path, int64_t rows, int32_t n)
{
    return ceil_div(4 * target_workgroups(path), rows) + n;
}

// Cuts the launch into workgroups.  The streaming kernels are HBM-bound with no reuse.  Measured on
// MI355X, the read rate is highest with about one long-lived workgroup per CU (256 sequential
// streams: 6.8 TB/s at 256 workgroups, 6.5 at 512, 6.2 at 1024 on the 1 GiB GQA share), so the
// target is one workgroup per CU, never less than one per (shard, sequence, kv head, head tile) row,
// with split records that stay small next to the KV bytes a workgroup streams.
inline int make_plan(const helix_problem* p, Path path, const int32_t* max_lens, const int64_t* sum_lens, int32_t n, Plan* plan)
{
    plan->path = path;
    plan->heads_per_wg = path == Path::Mla ? kMlaHeadsPerWorkgroup : 16;
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
    plan->stream = path == Path::Mla && plan->head_tiles == 1;
    if (plan->stream) {
        // One launch per kMaxShardsPerLaunch shards.  Each is cut evenly over the tokens its sequences turn out
        // to have (the lengths live on the device): the host only decides how many workgroups share them, from
        // the upper bounds it knows.  A pair has one record per workgroup that touches it: at most n_wg + pairs
        // records per launch, whatever the lengths are.
        plan->ordered = false;
        plan->total_splits = 0;
        plan->workgroups = 0;
        plan->map_bytes = 0;
        int64_t most = 0;
        for (int s0 = 0; s0 < n; s0 += kMaxShardsPerLaunch) {
            const int cnt = std::min(kMaxShardsPerLaunch, n - s0);
            int64_t bound = 0;                              // tokens of the launch if every sequence had max_len
            for (int i = 0; i < cnt; i++) bound += (int64_t)p->batch * max_lens[s0 + i];
            const int64_t n_wg = stream_workgroups(p, bound);
            if (n_wg > (int64_t)1 << 20) return HELIX_ERR_SHAPE;
            plan->total_splits += n_wg + (int64_t)cnt * p->batch;
            plan->workgroups += n_wg;
            plan->map_bytes += stream_map_bytes((int64_t)cnt * p->batch, n_wg);
            most = std::max(most, ceil_div(bound, n_wg));
        }
        plan->split_tokens = (int32_t)std::min<int64_t>(ceil_div(std::max<int64_t>(most, 1), 32) * 32, (int64_t)INT32_MAX / 32 * 32);
        return HELIX_OK;
    }
    // The streaming kernels take their runs from a map for a batch that is declared ragged -- the map costs a
    // launch of its own; MLA launches with several head tiles go by workgroup id
    plan->ordered = path != Path::Mla && ragged;
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
    // split_tokens is a 32-bit field of the kernel arguments: many shards of many long sequences must not wrap it
    // (no sequence is longer than INT32_MAX tokens, so a run of this length already holds any of them)
    split = std::min<int64_t>(split, (int64_t)INT32_MAX / plan->granule * plan->granule);
    plan->split_tokens = (int32_t)split;
    plan->total_splits = 0;
    for (int i = 0; i < n; i++) plan->total_splits += std::max<int64_t>(1, ceil_div(max_lens[i], split));
    plan->workgroups = plan->total_splits * rows;   // MLA launches pad this per shard to whole groups of 8
    if (plan->workgroups > (int64_t)1 << 30) return HELIX_ERR_SHAPE;
    plan->map_bytes = plan->ordered ? (size_t)plan->workgroups * sizeof(uint64_t) : 0;
    return HELIX_OK;
}

struct Workspace {
    float* ws_o;
    float* ws_m;
    float* ws_l;
    float* part_o;
    float* part_lse;
    char* maps;             // what the planning kernels write: the run each workgroup serves, or the stream plan
    size_t bytes;
};

// Carves a workspace for `total_splits` records, `n` shard partials and `map_bytes` of maps.  A record holds one
// row per (sequence, query head), or, for the evenly cut MLA launches (`per_pair`), per query head of the one
// sequence its run belongs to.  base may be NULL (sizing).
inline Workspace carve(const helix_problem* p, int64_t total_splits, bool per_pair, size_t map_bytes, int32_t n, void* base)
{
    const size_t bq = (size_t)p->batch * p->q_heads;
    const size_t rec_rows = per_pair ? (size_t)p->q_heads : bq;
    char* c = static_cast<char*>(base);
    size_t off = 0;
    Workspace w;
    w.ws_o = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)total_splits * rec_rows * p->dv * 4, 256);
    w.ws_m = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)total_splits * rec_rows * 4, 256);
    w.ws_l = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)total_splits * rec_rows * 4, 256);
    w.part_o = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)n * bq * p->dv * 4, 256);
    w.part_lse = reinterpret_cast<float*>(c + off); off = align_up(off + (size_t)n * bq * 4, 256);
    w.maps = c + off; off = align_up(off + map_bytes, 256);
    w.bytes = off;
    return w;
}

inline int check_shard(const helix_problem* p, const helix_kv_shard* s)
{
    if (!s->k || !s->len) return HELIX_ERR_NULL;
    if (p->v_aliases_k ? s->v != nullptr : s->v == nullptr) return p->v_aliases_k ? HELIX_ERR_SHAPE : HELIX_ERR_NULL;
    const bool fp8 = p->kv_dtype == HELIX_KV_FP8_E4M3;
    if (fp8 ? s->kv_scale == nullptr : false) return HELIX_ERR_NULL;
    if (s->max_len < 0 || s->sum_len < 0) return HELIX_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(s->status) % 4) return HELIX_ERR_SHAPE;
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

// Validates a call's problem and shards, plans it and carves the workspace.  Nothing is launched.
inline int prepare(const helix_problem* p, const helix_kv_shard* shards, int32_t n, void* workspace, size_t workspace_bytes,
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
    *ws = carve(p, plan->total_splits, plan->stream, plan->map_bytes, n, workspace);
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || ws->bytes > workspace_bytes) return HELIX_ERR_WORKSPACE;
    return HELIX_OK;
}

// Bytes of workspace that cover any call with `n_shards` shards no longer than `max_len`; 0 if invalid.
inline size_t workspace_bytes(const helix_problem* problem, int32_t n_shards, int32_t max_len)
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
    // an evenly cut MLA launch: workgroups and records only grow with the bounds, so the all-longest plan is the worst
    if (plan.stream) return carve(problem, plan.total_splits, true, plan.map_bytes, n_shards, nullptr).bytes;
    const int64_t rows = (int64_t)problem->batch * problem->kv_heads * plan.head_tiles;
    int64_t worst = plan.total_splits;
    if (problem->split_tokens == 0) {
        worst = std::max<int64_t>(worst, ceil_div(target_workgroups(path), rows) + n_shards);
        if (path != Path::Mla) worst = std::max<int64_t>(worst, ragged_split_cap(path, rows, n_shards));   // a batch declared ragged
    }
    return carve(problem, worst, false, (size_t)worst * rows * sizeof(uint64_t), n_shards, nullptr).bytes;
}

// The N slices helix_attn_decode_kvp hands to the kernels: each describes the whole cache (the kernel
// cuts slice i out of it) with the slice's own upper bounds.  `slices` has room for n_shards entries.
inline void kvp_slices(const helix_problem* problem, const helix_kv_shard* cache, int32_t n_shards, helix_kv_shard* slices)
{
    // every slice is at most c = 16 * ceil(ceil(max_len / N) / 16) tokens long
    const int64_t per = ceil_div(cache->max_len, n_shards);
    const int32_t c = (int32_t)std::min<int64_t>(16 * ceil_div(per, 16), cache->max_len);
    for (int32_t i = 0; i < n_shards; i++) {
        slices[i] = *cache;
        slices[i].max_len = c;
        // a slice holds a N-th of every sequence, rounded up to whole 16-token blocks
        if (cache->sum_len > 0)
            slices[i].sum_len = std::min<int64_t>(ceil_div(cache->sum_len, n_shards) + 16 * (int64_t)problem->batch, (int64_t)problem->batch * c);
    }
}

}  // namespace helix_host

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

enum class Path { Gqa64, Gqa128, GqaMx128, GqaF8_128, Mla };

struct Plan {
    Path path;
    int32_t heads_per_wg;   // query heads one workgroup serves
    int32_t head_tiles;     // workgroups per (b, kv head) along the group
    int32_t granule;        // tokens per planning tile: runs start and end on multiples of it
    int32_t split_tokens;   // tokens a workgroup streams (at most)
    int64_t total_splits;   // split records of the call, over all launches
    int32_t rec_rows;       // head rows of one record
    int64_t workgroups;
    bool stream;            // every launch is cut evenly over its token stream on the device (all but MLA with several head tiles)
    size_t map_bytes;       // what the kernels tell each other about the cut (tile prefix, workgroups of a row, ...)
};

constexpr int kMlaHeadsPerWorkgroup = 128;      // checked against the kernel's configuration where both are visible
constexpr int kMaxShardsPerLaunch = 16;         // shard descriptors travel by value in the kernel arguments
constexpr int64_t kTargetWorkgroups = 256;      // CUs of an MI355X: the streaming kernels read fastest with one long-lived workgroup per CU
constexpr int64_t kTargetWorkgroupsMx = 768;    // MXFP4 streams 3.8x fewer bytes per token: three workgroups resident per CU
constexpr int64_t kStreamMinTokensMla = 256;    // an MLA launch gives a workgroup at least this many tokens (a run costs ~10 us of set-up)
constexpr int64_t kTargetWorkgroupsMla = 4096;  // MLA with several head tiles (runs by workgroup id): keeps the records of a call near 1 GB
constexpr int64_t kMinSplitTokensMla = 4096;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workgroups of an evenly cut launch over rows whose lengths add up to at most `row_tokens`, `row_tiles` tiles:
// one per CU (three for MXFP4 K/V) unless the launch is small, or as many as the caller's run
// length asks for.  Measured on the 1 GiB GQA share: 256 sequential streams read 6.8 TB/s, 512 6.5, 1024 6.2.
// A GQA launch with several head tiles per kv head (row_tokens and row_tiles count every head tile) consists of
// head_tiles equal sets of workgroups, one per head tile, cut alike; a set has a multiple of 8 workgroups where the
// launch is large enough, so that the workgroups that read the same tokens land on the same XCD.
inline int64_t stream_workgroups(const helix_problem* p, Path path, int64_t head_tiles, int64_t row_tokens, int64_t row_tiles)
{
    if (path == Path::Mla) {
        if (p->split_tokens > 0) return std::max<int64_t>(1, ceil_div(row_tokens, ceil_div(p->split_tokens, 32) * 32));
        return std::min(kTargetWorkgroups, std::max<int64_t>(1, row_tokens / kStreamMinTokensMla));
    }
    const int64_t set_tokens = row_tokens / head_tiles, set_tiles = row_tiles / head_tiles;      // of one head tile
    int64_t n;
    if (p->split_tokens > 0) {
        n = std::max<int64_t>(1, ceil_div(set_tokens, ceil_div(p->split_tokens, 128) * 128));
    } else {
        // (e4m3 K/V stream like bf16 ones: measured 6.8 TB/s with 256 workgroups, 6.5 with 512, 6.2 with 768 and more)
        int64_t target = std::max<int64_t>(1, (path == Path::GqaMx128 ? kTargetWorkgroupsMx : kTargetWorkgroups) / head_tiles);
        if (head_tiles > 1 && target >= 8) target = target / 8 * 8;
        n = std::min(target, std::max<int64_t>(1, set_tiles));
    }
    // the MXFP4 kernel addresses a run with 32-bit byte offsets
    if (path == Path::GqaMx128) n = std::max(n, ceil_div(set_tokens, (int64_t)1 << 25));
    return n * head_tiles;
}

// Bytes of the maps of one evenly cut launch, 256-byte aligned: the tile prefix [pairs + 1] int64, then MLA: the
// workgroups of every pair [pairs] 2 x int32 and the first pair of every workgroup [n_wg] int32; GQA: the first
// and last workgroup of every row [rows] 2 x int32.
inline size_t stream_map_bytes(Path path, int64_t pairs, int64_t rows, int64_t n_wg)
{
    const size_t prefix = align_up((size_t)(pairs + 1) * 8, 256);
    if (path == Path::Mla) return prefix + align_up((size_t)pairs * 8, 256) + align_up((size_t)n_wg * 4, 256);
    return prefix + align_up((size_t)rows * 8, 256);
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
    if (!p->v_aliases_k && p->kv_dtype == HELIX_KV_FP8_E4M3 && p->dk == 128 && p->dv == 128) {
        *path = Path::GqaF8_128;
        return HELIX_OK;
    }
    if (p->v_aliases_k && p->dk == 576 && p->dv == 512 && p->kv_heads == 1) {
        *path = Path::Mla;
        return HELIX_OK;
    }
    return HELIX_ERR_UNSUPPORTED;
}

// Cuts a call into launches and workgroups.  Only upper bounds of the lengths are known here (they live on the
// device): the host decides how many workgroups share a launch, the kernels find out which tokens each one gets.
inline int make_plan(const helix_problem* p, Path path, const int32_t* max_lens, int32_t n, Plan* plan)
{
    plan->path = path;
    plan->heads_per_wg = path == Path::Mla ? kMlaHeadsPerWorkgroup : 16;
    plan->granule = path == Path::Mla ? 32 : 128;         // MLA: 32-token tiles; GQA: 4 waves x 32-token blocks
    const int g = p->q_heads / p->kv_heads;
    plan->head_tiles = (int32_t)ceil_div(g, plan->heads_per_wg);
    plan->rec_rows = path == Path::Mla ? p->q_heads : 16;
    const int64_t rows_per_pair = path == Path::Mla ? 1 : (int64_t)p->kv_heads * plan->head_tiles;
    for (int i = 0; i < n; i++)
        if (max_lens[i] < 0) return HELIX_ERR_SHAPE;
    plan->stream = path != Path::Mla || plan->head_tiles == 1;
    plan->map_bytes = 0;
    if (plan->stream) {
        // One launch per kMaxShardsPerLaunch shards, each cut evenly over the tokens its sequences turn out to have.
        // A row has one record per workgroup that touches it: at most n_wg + rows records per launch, whatever
        // the lengths are.
        plan->total_splits = 0;
        plan->workgroups = 0;
        int64_t most = 0;
        for (int s0 = 0; s0 < n; s0 += kMaxShardsPerLaunch) {
            const int cnt = std::min(kMaxShardsPerLaunch, n - s0);
            int64_t row_tokens = 0, row_tiles = 0;         // if every sequence had max_len
            for (int i = 0; i < cnt; i++) {
                row_tokens += (int64_t)p->batch * rows_per_pair * max_lens[s0 + i];
                row_tiles += (int64_t)p->batch * rows_per_pair * ceil_div(max_lens[s0 + i], plan->granule);
            }
            const int64_t n_wg = stream_workgroups(p, path, path == Path::Mla ? 1 : plan->head_tiles, row_tokens, row_tiles);
            const int64_t pairs = (int64_t)cnt * p->batch, rows = pairs * rows_per_pair;
            if (n_wg > (int64_t)1 << 20 || rows > (int64_t)1 << 28) return HELIX_ERR_SHAPE;
            plan->total_splits += n_wg + rows;
            plan->workgroups += n_wg;
            plan->map_bytes += stream_map_bytes(path, pairs, rows, n_wg);
            most = std::max(most, ceil_div(row_tokens, n_wg));
        }
        plan->split_tokens = (int32_t)std::min<int64_t>(ceil_div(std::max<int64_t>(most, 1), plan->granule) * plan->granule,
                                                        (int64_t)INT32_MAX / plan->granule * plan->granule);
        return HELIX_OK;
    }
    // MLA with several head tiles: fixed runs of 4096 tokens, one workgroup per (run, sequence, head tile), by id
    const int64_t rows = (int64_t)p->batch * plan->head_tiles;
    int64_t split;
    if (p->split_tokens > 0) {
        split = ceil_div(p->split_tokens, plan->granule) * plan->granule;
    } else {
        int64_t total = 0;
        for (int i = 0; i < n; i++) total += max_lens[i];
        split = ceil_div(ceil_div(rows * total, kTargetWorkgroupsMla), plan->granule) * plan->granule;
        split = std::max<int64_t>(split, kMinSplitTokensMla);
    }
    // split_tokens is a 32-bit field of the kernel arguments: many shards of many long sequences must not wrap it
    // (no sequence is longer than INT32_MAX tokens, so a run of this length already holds any of them)
    split = std::min<int64_t>(split, (int64_t)INT32_MAX / plan->granule * plan->granule);
    plan->split_tokens = (int32_t)split;
    plan->total_splits = 0;
    for (int i = 0; i < n; i++) plan->total_splits += std::max<int64_t>(1, ceil_div(max_lens[i], split));
    plan->workgroups = plan->total_splits * rows;   // the launch pads this per shard to whole groups of 8
    plan->rec_rows = p->batch * p->q_heads;         // records [split][B][Q]
    if (plan->workgroups > (int64_t)1 << 30 || (int64_t)p->batch * p->q_heads > INT32_MAX) return HELIX_ERR_SHAPE;
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

// Carves a workspace for `total_splits` records of `rec_rows` head rows each, `n` shard partials and `map_bytes`
// of maps.  base may be NULL (sizing).
inline Workspace carve(const helix_problem* p, int64_t total_splits, int64_t rec_rows, size_t map_bytes, int32_t n, void* base)
{
    const size_t bq = (size_t)p->batch * p->q_heads;
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
    if (s->max_len < 0) return HELIX_ERR_SHAPE;
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
    for (int32_t i = 0; i < n; i++) {
        if (int rc = check_shard(p, &shards[i])) return rc;
        max_lens[i] = shards[i].max_len;
    }
    if (int rc = make_plan(p, path, max_lens, n, plan)) return rc;
    *ws = carve(p, plan->total_splits, plan->rec_rows, plan->map_bytes, n, workspace);
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
    if (make_plan(problem, path, lens, n_shards, &plan) != HELIX_OK) return 0;
    // an evenly cut launch: workgroups and records only grow with the bounds, so the all-longest plan is the worst
    if (plan.stream) return carve(problem, plan.total_splits, plan.rec_rows, plan.map_bytes, n_shards, nullptr).bytes;
    // runs by workgroup id: shorter shards keep their one record each
    const int64_t worst = std::max<int64_t>(plan.total_splits, ceil_div(kTargetWorkgroupsMla, (int64_t)problem->batch * plan.head_tiles) + n_shards);
    return carve(problem, worst, plan.rec_rows, 0, n_shards, nullptr).bytes;
}

// The N slices helix_attn_decode_kvp hands to the kernels: each describes the whole cache (the kernel
// cuts slice i out of it) with the slice's own upper bounds.  `slices` has room for n_shards entries.
inline void kvp_slices(const helix_kv_shard* cache, int32_t n_shards, helix_kv_shard* slices)
{
    // every slice is at most c = 16 * ceil(ceil(max_len / N) / 16) tokens long
    const int64_t per = ceil_div(cache->max_len, n_shards);
    const int32_t c = (int32_t)std::min<int64_t>(16 * ceil_div(per, 16), cache->max_len);
    for (int32_t i = 0; i < n_shards; i++) {
        slices[i] = *cache;
        slices[i].max_len = c;
    }
}

}  // namespace helix_host

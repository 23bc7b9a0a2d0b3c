// C ABI of the Helix decode-attention library for MI355X (gfx950): host-side validation, work
// planning, workspace carving and kernel launches.  See include/helix_attn.h for the contract.
#include "../../include/helix_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>

#include "plan.hpp"
#include "common.hpp"
#include "gqa_decode.hpp"
#include "gqa_mxfp4.hpp"
#include "gqa_fp8.hpp"
#include "merge_combine.hpp"
#include "mla_decode.hpp"
#include "probes.hpp"

namespace {

using namespace helix;
using namespace helix_host;

static_assert(kMlaHeadsPerWorkgroup == MlaCfg::HPW, "the host plan and the MLA kernel agree on the heads of a workgroup");

// The MLA kernels need more than the default 64 KB of LDS per workgroup, which has to be asked for once per
// device and kernel; later calls then consist of launches only (and can be captured into a HIP graph).
// The request is idempotent, so two threads that both find the flag clear may both make it.
std::atomic<bool> g_lds_asked[3][64];

// Scratch memory of helix_attn_decode_static: callers that must not allocate get the split records and the
// per-shard fragments here instead of in a workspace of their own.  Every GPU the library runs on holds its
// own copy of the array until the process ends.  In host code the array's name is only a handle: the device
// address comes from hipGetSymbolAddress, once per device, and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[HELIX_STATIC_SCRATCH_BYTES];
std::atomic<void*> g_scratch_ptr[64];

int static_scratch(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return HELIX_ERR_LAUNCH;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HELIX_ERR_LAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);      // the same address whichever thread stores it
    }
    *out = p;
    return HELIX_OK;
}

// hipEvent_t pair recorded around the streaming attention kernel(s) of a call (the timed entry point), or none
struct KernelEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};

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
                 float* o = nullptr, float* lse_out = nullptr, bool* finished = nullptr, KvpCut cut = KvpCut(),
                 KernelEvents ev = KernelEvents(), bool keep_parts = true)
{
    const bool fuse = o != nullptr && n <= kMaxLaunchShards;
    if (finished) *finished = fuse;
    const int g = p->q_heads / p->kv_heads;
    const bool mla = plan.path == Path::Mla;
    const int64_t rows_per_pair = mla ? 1 : (int64_t)p->kv_heads * plan.head_tiles;
    static_assert(kMaxLaunchShards == kMaxShardsPerLaunch, "the host plan and the kernels agree on the shards of a launch");
    int32_t split_base = 0;
    int32_t rec_base = 0;          // stream plan: first record of the launch
    size_t map_off = 0;            // ... and where its maps start in the workspace
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
        int64_t row_tokens = 0, row_tiles = 0;             // of the launch, if every sequence had max_len
        for (int32_t i = 0; i < cnt; i++) {
            const helix_kv_shard& s = shards[s0 + i];
            ShardDev& d = a.shard[i];
            d.k = s.k; d.v = s.v; d.kv_scale = s.kv_scale; d.tok_off = s.tok_off; d.len = s.len;
            d.k_sb = s.k_stride_b; d.k_sh = s.k_stride_h; d.k_st = s.k_stride_t;
            d.v_sb = s.v_stride_b; d.v_sh = s.v_stride_h; d.v_st = s.v_stride_t;
            d.s_sb = s.s_stride_b; d.s_sh = s.s_stride_h;
            d.k_mx = s.k_scale_mx; d.v_mx = s.v_scale_mx;
            d.status = s.status;
            d.kvp_n = cut.n; d.kvp_i = s0 + i;
            d.out_off = cut.off ? cut.off + (int64_t)(s0 + i) * p->batch : nullptr;
            d.out_len = cut.len ? cut.len + (int64_t)(s0 + i) * p->batch : nullptr;
            row_tokens += (int64_t)p->batch * rows_per_pair * s.max_len;
            row_tiles += (int64_t)p->batch * rows_per_pair * ceil_div(s.max_len, plan.granule);
            if (!plan.stream) {                            // MLA with several head tiles: runs by workgroup id
                d.n_splits = (int32_t)std::max<int64_t>(1, ceil_div(s.max_len, plan.split_tokens));
                d.split_base = split_base;
                d.unit_base = (int32_t)units;
                m.split_base[i] = split_base;
                m.n_splits[i] = d.n_splits;
                split_base += d.n_splits;
                units += mla_units_of_shard(d.n_splits, p->batch, plan.head_tiles);
            }
        }
        if (plan.stream) {
            // the launch is cut evenly over the tokens its sequences have on the device: by a planning kernel for MLA
            // (one workgroup per CU, each run worth a set-up), by every workgroup for itself in the streaming kernels
            const int64_t n_wg = stream_workgroups(p, plan.path, mla ? 1 : plan.head_tiles, row_tokens, row_tiles);
            const int64_t pairs = (int64_t)cnt * p->batch, rows = pairs * rows_per_pair;
            char* maps = ws.maps + map_off;
            map_off += stream_map_bytes(plan.path, pairs, rows, n_wg);
            int64_t* prefix = reinterpret_cast<int64_t*>(maps);
            a.n_wg = (int32_t)n_wg;
            a.n_base = (int32_t)(n_wg / (mla ? 1 : plan.head_tiles));
            a.rec_base = rec_base;
            m.tile_prefix = prefix;
            m.n_wg = a.n_wg;
            m.rec_base = rec_base;
            m.K = p->kv_heads; m.g = g; m.head_tiles = plan.head_tiles;
            if (mla) {
                int2* pair_rec = reinterpret_cast<int2*>(maps + align_up((size_t)(pairs + 1) * 8, 256));
                int32_t* first_pair = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(pair_rec) + align_up((size_t)pairs * 8, 256));
                hipLaunchKernelGGL(helix::stream_plan_kernel, dim3(1), dim3(helix::kPlanThreads), 0, stream, a, prefix, first_pair, pair_rec);
                if (int rc = launch_status()) return rc;
                a.tile_prefix = prefix;
                a.wg_first_pair = first_pair;
                m.pair_rec = pair_rec;
            } else {
                a.prefix_out = prefix;
                a.row_rec = reinterpret_cast<int2*>(maps + align_up((size_t)(pairs + 1) * 8, 256));
                m.row_rec = a.row_rec;
            }
            rec_base += (int32_t)(n_wg + rows);
            units = n_wg;
        }
        if (ev.start && s0 == 0 && hipEventRecord(ev.start, stream) != hipSuccess) return HELIX_ERR_LAUNCH;
        switch (plan.path) {
            // (several head tiles per kv head: the kernels whose workgroups share their reads through the L2)
            case Path::Gqa64:
                if (plan.head_tiles > 1) hipLaunchKernelGGL((gqa_decode_kernel<64, true>), dim3((unsigned)units), dim3(256), 0, stream, a);
                else hipLaunchKernelGGL((gqa_decode_kernel<64, false>), dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::Gqa128:
                if (plan.head_tiles > 1) hipLaunchKernelGGL((gqa_decode_kernel<128, true>), dim3((unsigned)units), dim3(256), 0, stream, a);
                else hipLaunchKernelGGL((gqa_decode_kernel<128, false>), dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::GqaMx128:
                if (plan.head_tiles > 1) hipLaunchKernelGGL(gqa_mxfp4_kernel<true>, dim3((unsigned)units), dim3(256), 0, stream, a);
                else hipLaunchKernelGGL(gqa_mxfp4_kernel<false>, dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::GqaF8_128:
                if (plan.head_tiles > 1) hipLaunchKernelGGL(gqa_fp8_kernel<true>, dim3((unsigned)units), dim3(256), 0, stream, a);
                else hipLaunchKernelGGL(gqa_fp8_kernel<false>, dim3((unsigned)units), dim3(256), 0, stream, a);
                break;
            case Path::Mla: {
                const int kind = p->kv_dtype == HELIX_KV_FP8_E4M3 ? 1 : p->kv_dtype == HELIX_KV_MXFP4 ? 2 : 0;
                auto kern = kind == 2 ? mla_decode_kernel<true, true> : kind == 1 ? mla_decode_kernel<true> : mla_decode_kernel<false>;
                int dev = 0;
                if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return HELIX_ERR_LAUNCH;
                if (!g_lds_asked[kind][dev].load(std::memory_order_acquire)) {
                    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                            MlaCfg::LDS_BYTES) != hipSuccess)
                        return HELIX_ERR_LAUNCH;
                    g_lds_asked[kind][dev].store(true, std::memory_order_release);
                }
                hipLaunchKernelGGL(kern, dim3((unsigned)units), dim3(MlaCfg::THREADS), MlaCfg::LDS_BYTES, stream, a);
                break;
            }
            default:
                return HELIX_ERR_UNSUPPORTED;
        }
        if (int rc = launch_status()) return rc;
        if (ev.stop && s0 + cnt >= n && hipEventRecord(ev.stop, stream) != hipSuccess) return HELIX_ERR_LAUNCH;
        m.ws_o = ws.ws_o; m.ws_m = ws.ws_m; m.ws_l = ws.ws_l;
        m.o_part = o_part; m.lse_part = lse_part;
        m.B = p->batch; m.Q = p->q_heads; m.n_shards = cnt; m.shard0 = s0;
        if (fuse) {
            FinishArgs f;
            f.m = m; f.o = o; f.lse_out = lse_out; f.keep_parts = keep_parts ? 1 : 0;
            const unsigned frows = (unsigned)((int64_t)p->batch * p->q_heads);
            // many rows: a thread group per row instead of a workgroup per row (on the MLA width the workgroup version
            // folds the shards side by side, so with more shards it stays ahead for longer)
            if (plan.stream && (int64_t)frows >= helix::kManyRows * (p->dv == 512 ? cnt : 1)) {
                auto grid = [&](int rows_per_wg) { return dim3((frows + rows_per_wg - 1) / rows_per_wg); };
                switch (p->dv) {
                    case 64: hipLaunchKernelGGL((finish_rows_kernel<64>), grid(helix::finish_rows_per_workgroup<64>()), dim3(256), 0, stream, f); break;
                    case 128: hipLaunchKernelGGL((finish_rows_kernel<128>), grid(helix::finish_rows_per_workgroup<128>()), dim3(256), 0, stream, f); break;
                    case 512: hipLaunchKernelGGL((finish_rows_kernel<512>), grid(helix::finish_rows_per_workgroup<512>()), dim3(256), 0, stream, f); break;
                    default: return HELIX_ERR_UNSUPPORTED;
                }
                return launch_status();
            }
            if (plan.stream) {
                auto threads = [&](int row_threads, int sublanes, int groups) { return dim3((unsigned)(row_threads * sublanes * std::min<int32_t>(cnt, groups))); };
                switch (p->dv) {
                    case 64: hipLaunchKernelGGL((finish_stream_kernel<64>), dim3(frows), threads(helix::finish_row_threads<64>(), helix::stream_sublanes<64>(), helix::finish_groups<64>()), 0, stream, f); break;
                    case 128: hipLaunchKernelGGL((finish_stream_kernel<128>), dim3(frows), threads(helix::finish_row_threads<128>(), helix::stream_sublanes<128>(), helix::finish_groups<128>()), 0, stream, f); break;
                    case 512: hipLaunchKernelGGL((finish_stream_kernel<512>), dim3(frows), threads(helix::finish_row_threads<512>(), helix::stream_sublanes<512>(), helix::finish_groups<512>()), 0, stream, f); break;
                    default: return HELIX_ERR_UNSUPPORTED;
                }
                return launch_status();
            }
            if (p->dv != 512) return HELIX_ERR_UNSUPPORTED;       // runs by workgroup id exist for the MLA shape only
            hipLaunchKernelGGL((finish_kernel<512>), dim3(frows), dim3(256), 0, stream, f);
            return launch_status();
        }
        const unsigned mrows = (unsigned)((int64_t)cnt * p->batch * p->q_heads);
        if (plan.stream && (int64_t)mrows >= helix::kManyRows) {
            auto grid = [&](int rows_per_wg) { return dim3((mrows + rows_per_wg - 1) / rows_per_wg); };
            switch (p->dv) {
                case 64: hipLaunchKernelGGL((merge_rows_kernel<64>), grid(helix::finish_rows_per_workgroup<64>()), dim3(256), 0, stream, m); break;
                case 128: hipLaunchKernelGGL((merge_rows_kernel<128>), grid(helix::finish_rows_per_workgroup<128>()), dim3(256), 0, stream, m); break;
                case 512: hipLaunchKernelGGL((merge_rows_kernel<512>), grid(helix::finish_rows_per_workgroup<512>()), dim3(256), 0, stream, m); break;
                default: return HELIX_ERR_UNSUPPORTED;
            }
            if (int rc = launch_status()) return rc;
            continue;
        }
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

int helix_attn_plan(const helix_problem* problem, const int32_t* max_lens, int32_t n_shards,
                    int32_t* split_tokens, int64_t* workgroups)
{
    Path path;
    if (int rc = check_problem(problem, &path)) return rc;
    if (!max_lens) return HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS) return HELIX_ERR_SHAPE;
    Plan plan;
    if (int rc = make_plan(problem, path, max_lens, n_shards, &plan)) return rc;
    if (split_tokens) *split_tokens = plan.split_tokens;
    if (workgroups) *workgroups = plan.workgroups;
    return HELIX_OK;
}

size_t helix_attn_workspace_bytes(const helix_problem* problem, int32_t n_shards, int32_t max_len)
{
    return helix_host::workspace_bytes(problem, n_shards, max_len);
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
    if (int rc = run_partials(problem, plan, q, shards, n_shards, ws, po, pl, stream, o, lse_out, &finished, KvpCut(), KernelEvents(),
                              o_partials != nullptr)) return rc;
    if (finished) return HELIX_OK;
    const int64_t rows = (int64_t)problem->batch * problem->q_heads;
    return combine_any(problem->dv, po, pl, o, lse_out, nullptr, n_shards, rows, stream);
}

int helix_attn_decode_static(const helix_problem* problem, const void* q, const helix_kv_shard* shards, int32_t n_shards,
                             float* o, float* lse_out, void* hip_stream)
{
    if (!q || !o) return HELIX_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(o) % 16) return HELIX_ERR_SHAPE;
    // validate and size first (a fake, aligned base: nothing is dereferenced), then fetch the device address
    Plan plan;
    Workspace ws;
    if (int rc = prepare(problem, shards, n_shards, reinterpret_cast<void*>(uintptr_t(256)), HELIX_STATIC_SCRATCH_BYTES, &plan, &ws)) return rc;
    void* base = nullptr;
    if (int rc = static_scratch(&base)) return rc;
    if (int rc = prepare(problem, shards, n_shards, base, HELIX_STATIC_SCRATCH_BYTES, &plan, &ws)) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    bool finished = false;
    if (int rc = run_partials(problem, plan, q, shards, n_shards, ws, ws.part_o, ws.part_lse, stream, o, lse_out, &finished, KvpCut(), KernelEvents(),
                              false)) return rc;
    if (finished) return HELIX_OK;
    const int64_t rows = (int64_t)problem->batch * problem->q_heads;
    return combine_any(problem->dv, ws.part_o, ws.part_lse, o, lse_out, nullptr, n_shards, rows, stream);
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

namespace {
int decode_kvp(const helix_problem* problem, const void* q, const helix_kv_shard* cache, int32_t n_shards,
               float* o, float* lse_out, float* o_partials, float* lses, int64_t* shard_off, int32_t* shard_len,
               void* workspace, size_t workspace_bytes, void* hip_stream, KernelEvents ev)
{
    if (!problem || !q || !o || !cache) return HELIX_ERR_NULL;
    if ((o_partials == nullptr) != (lses == nullptr) || (shard_off == nullptr) != (shard_len == nullptr)) return HELIX_ERR_NULL;
    if (n_shards < 1 || n_shards > HELIX_MAX_SHARDS) return HELIX_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(q) % 16 || reinterpret_cast<uintptr_t>(o) % 16 ||
        reinterpret_cast<uintptr_t>(o_partials) % 16) return HELIX_ERR_SHAPE;
    if (cache->max_len < 0) return HELIX_ERR_SHAPE;
    Path path;
    if (int rc = check_problem(problem, &path)) return rc;
    helix_kv_shard slices[HELIX_MAX_SHARDS];               // on the stack: the library allocates nothing
    kvp_slices(cache, n_shards, slices);
    Plan plan;
    Workspace ws;
    if (int rc = prepare(problem, slices, n_shards, workspace, workspace_bytes, &plan, &ws)) return rc;
    float* po = o_partials ? o_partials : ws.part_o;
    float* pl = lses ? lses : ws.part_lse;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    KvpCut cut;
    cut.n = n_shards; cut.off = shard_off; cut.len = shard_len;
    bool finished = false;
    if (int rc = run_partials(problem, plan, q, slices, n_shards, ws, po, pl, stream, o, lse_out, &finished, cut, ev, o_partials != nullptr)) return rc;
    if (finished) return HELIX_OK;
    const int64_t rows = (int64_t)problem->batch * problem->q_heads;
    return combine_any(problem->dv, po, pl, o, lse_out, nullptr, n_shards, rows, stream);
}
}  // namespace

int helix_attn_decode_kvp(const helix_problem* problem, const void* q, const helix_kv_shard* cache, int32_t n_shards,
                          float* o, float* lse_out, float* o_partials, float* lses,
                          int64_t* shard_off, int32_t* shard_len,
                          void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return decode_kvp(problem, q, cache, n_shards, o, lse_out, o_partials, lses, shard_off, shard_len,
                      workspace, workspace_bytes, hip_stream, KernelEvents());
}

int helix_attn_decode_kvp_timed(const helix_problem* problem, const void* q, const helix_kv_shard* cache, int32_t n_shards,
                                float* o, float* lse_out, float* o_partials, float* lses,
                                int64_t* shard_off, int32_t* shard_len,
                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                void* start_event, void* stop_event)
{
    if (!start_event || !stop_event) return HELIX_ERR_NULL;
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return decode_kvp(problem, q, cache, n_shards, o, lse_out, o_partials, lses, shard_off, shard_len,
                      workspace, workspace_bytes, hip_stream, ev);
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

int helix_probe_stream_read(const void* buf, size_t bytes, int32_t workgroups, int32_t nontemporal, void* hip_stream)
{
    if (!buf) return HELIX_ERR_NULL;
    if (bytes == 0 || bytes % helix::kProbeBlock || reinterpret_cast<uintptr_t>(buf) % 16 || workgroups < 1 || workgroups > (1 << 20))
        return HELIX_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint8_t* p = static_cast<const uint8_t*>(buf);
    if (nontemporal) hipLaunchKernelGGL(helix::stream_read_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, stream, p, bytes / helix::kProbeBlock, nullptr);
    else hipLaunchKernelGGL(helix::stream_read_kernel<false>, dim3((unsigned)workgroups), dim3(256), 0, stream, p, bytes / helix::kProbeBlock, nullptr);
    return launch_status();
}

int helix_probe_mfma_lds(const void* operands, int32_t iters, const void* stream_buf, size_t stream_bytes,
                         double* flops, double* bytes_read, void* hip_stream)
{
    if (!operands) return HELIX_ERR_NULL;
    if (iters < 8 || iters % 8 || reinterpret_cast<uintptr_t>(operands) % 16) return HELIX_ERR_SHAPE;
    // the streamed buffer is addressed modulo its size: a power of two, at least one step of the whole grid
    if (stream_buf && (stream_bytes < ((size_t)1 << 22) || (stream_bytes & (stream_bytes - 1)) || stream_bytes > ((size_t)1 << 35) ||
                       reinterpret_cast<uintptr_t>(stream_buf) % 16)) return HELIX_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const helix::u32x4* d = static_cast<const helix::u32x4*>(operands);
    constexpr int grid = 256;                               // one workgroup of 8 waves per CU
    if (stream_buf)
        hipLaunchKernelGGL(helix::mfma_lds_kernel<true>, dim3(grid), dim3(helix::kProbeWaves * 64), 0, stream, iters, d, nullptr,
                           static_cast<const helix::u32x4*>(stream_buf), (uint32_t)(stream_bytes / 16 - 1));
    else
        hipLaunchKernelGGL(helix::mfma_lds_kernel<false>, dim3(grid), dim3(helix::kProbeWaves * 64), 0, stream, iters, d, nullptr, nullptr, 0u);
    if (flops) *flops = (double)grid * helix::kProbeWaves * (double)iters * 8.0 * (2.0 * 16 * 16 * 32);
    if (bytes_read) *bytes_read = stream_buf ? (double)grid * helix::kProbeWaves * 1024.0 * (double)(iters / 2 + 4) : 0.0;
    return launch_status();
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

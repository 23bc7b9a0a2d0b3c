// Host-only program for the sanitizer job: the C ABI's validation, planning and workspace carving
// (paper_2507_07120_amd/csrc/plan.hpp, plain C++) swept over many problems and shard sets under
// -fsanitize=address,undefined.  It checks the invariants the launches rely on; any sanitizer report or
// failed check ends it with a non-zero status.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_2507_07120_amd/csrc/plan.hpp"
#include "../../paper_2507_07120_amd/csrc/seat.hpp"

using namespace helix_host;

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return rng_state;
}

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            std::printf("check failed at line %d: %s (case %ld)\n", __LINE__, #cond, cases); \
            return 1;                                                                \
        }                                                                            \
    } while (0)

int main()
{
    long cases = 0, planned = 0;
    const helix_problem shapes[] = {
        {16, 16, 1, 128, 128, 0, HELIX_KV_BF16, 0.088f, 0},   {4, 64, 8, 128, 128, 0, HELIX_KV_BF16, 0.088f, 0},
        {1, 8, 2, 64, 64, 0, HELIX_KV_BF16, 0.125f, 0},       {2, 40, 2, 64, 64, 0, HELIX_KV_BF16, 0.125f, 256},
        {16, 16, 1, 128, 128, 0, HELIX_KV_MXFP4, 0.088f, 0},  {32, 128, 1, 576, 512, 1, HELIX_KV_BF16, 0.07f, 0},
        {64, 128, 1, 576, 512, 1, HELIX_KV_FP8_E4M3, 0.07f, 0}, {2, 200, 1, 576, 512, 1, HELIX_KV_MXFP4, 0.07f, 0},
        {4096, 16, 1, 128, 128, 0, HELIX_KV_BF16, 0.088f, 0}, {3, 16, 1, 128, 128, 0, HELIX_KV_BF16, 0.088f, INT32_MAX},
        // invalid ones: every entry point must refuse them without touching anything
        {0, 16, 1, 128, 128, 0, HELIX_KV_BF16, 0.088f, 0},    {2, 7, 2, 128, 128, 0, HELIX_KV_BF16, 0.088f, 0},
        {2, 16, 1, 96, 96, 0, HELIX_KV_BF16, 0.088f, 0},      {2, 16, 1, 128, 128, 0, 7, 0.088f, 0},
        {2, 16, 1, 128, 128, 0, HELIX_KV_BF16, -1.f, 0},      {2, 16, 1, 128, 128, 0, HELIX_KV_BF16, 0.088f, -5},
    };
    const int32_t lens_pool[] = {0, 1, 15, 16, 17, 100, 127, 128, 129, 1000, 4095, 4096, 4097, 65536, 131072, 262144, 1 << 24, INT32_MAX};
    const int n_pool = sizeof lens_pool / sizeof lens_pool[0];
    const int32_t shard_counts[] = {1, 2, 3, 8, 16, 17, 64, 1024};
    std::vector<helix_kv_shard> shards(HELIX_MAX_SHARDS);
    std::vector<int32_t> lens(HELIX_MAX_SHARDS);
    alignas(256) static unsigned char fake_base[256];      // never dereferenced: carve() only does address arithmetic
    for (const helix_problem& p : shapes) {
        Path path;
        const int prc = check_problem(&p, &path);
        for (int32_t n : shard_counts) {
            for (int rep = 0; rep < 40; rep++) {
                cases++;
                int32_t longest = 0;
                for (int i = 0; i < n; i++) {
                    lens[i] = lens_pool[rnd() % n_pool];
                    if (rep % 4 == 0) lens[i] = lens_pool[(rep / 4) % n_pool];          // uniform sets as well
                    longest = lens[i] > longest ? lens[i] : longest;
                }
                if (prc != HELIX_OK) {
                    CHECK(workspace_bytes(&p, n, longest) == 0);
                    continue;
                }
                Plan plan;
                const int rc = make_plan(&p, path, lens.data(), n, &plan);
                if (rc != HELIX_OK) {
                    CHECK(rc == HELIX_ERR_SHAPE);          // too many workgroups for one launch: refused, not wrapped
                    continue;
                }
                planned++;
                CHECK(plan.split_tokens > 0 && plan.split_tokens % plan.granule == 0);
                const int64_t rows = (int64_t)p.batch * (path == Path::Mla ? 1 : p.kv_heads) * plan.head_tiles;
                if (plan.stream) {
                    // evenly cut launches of at most 16 shards: a record per workgroup and per row of the launch
                    const int64_t launches = ceil_div(n, kMaxShardsPerLaunch);
                    CHECK(plan.workgroups >= launches && plan.workgroups <= launches * ((int64_t)1 << 20));
                    CHECK(plan.total_splits == plan.workgroups + (int64_t)n * (path == Path::Mla ? p.batch : rows));
                    CHECK(plan.map_bytes >= (size_t)((int64_t)n * p.batch + launches) * 8);
                    CHECK(plan.rec_rows == (path == Path::Mla ? p.q_heads : 16));
                } else {
                    int64_t splits = 0;
                    for (int i = 0; i < n; i++) {
                        const int64_t ns = std::max<int64_t>(1, ceil_div(lens[i], plan.split_tokens));
                        CHECK(ns * plan.split_tokens >= lens[i]);                 // the runs cover the longest sequence
                        splits += ns;
                    }
                    CHECK(splits == plan.total_splits);
                    CHECK(plan.workgroups == splits * rows && plan.workgroups <= ((int64_t)1 << 30));
                }
                // the workspace the sizing call promises covers the call's own carving
                const Workspace w = carve(&p, plan.total_splits, plan.rec_rows, plan.map_bytes, n, fake_base);
                CHECK((unsigned char*)w.ws_o == fake_base);
                CHECK((size_t)((unsigned char*)w.maps - fake_base) + plan.map_bytes <= w.bytes && w.bytes % 256 == 0);
                // (no bound exists only if n shards that all have the longest length are more than one launch holds)
                const size_t bound = workspace_bytes(&p, n, longest);
                if (bound == 0) {
                    std::vector<int32_t> all(n, longest);
                    Plan worst;
                    CHECK(make_plan(&p, path, all.data(), n, &worst) == HELIX_ERR_SHAPE);
                    continue;
                }
                if (p.split_tokens == 0 || plan.stream) CHECK(w.bytes <= bound);
                // descriptors: a valid one passes, each broken field is caught
                helix_kv_shard s{};
                const bool fp4 = p.kv_dtype == HELIX_KV_MXFP4, fp8 = p.kv_dtype == HELIX_KV_FP8_E4M3;
                s.k = fake_base;
                s.v = p.v_aliases_k ? nullptr : fake_base;
                s.kv_scale = fp8 ? reinterpret_cast<const float*>(fake_base) : nullptr;
                s.k_stride_t = p.dk; s.v_stride_t = p.v_aliases_k ? 0 : p.dv;
                s.k_stride_h = 1024 * (int64_t)p.dk; s.v_stride_h = p.v_aliases_k ? 0 : 1024 * (int64_t)p.dv;
                s.len = reinterpret_cast<const int32_t*>(fake_base);
                s.max_len = longest;
                s.k_scale_mx = fp4 ? fake_base : nullptr;
                s.v_scale_mx = fp4 && !p.v_aliases_k ? fake_base : nullptr;
                CHECK(check_shard(&p, &s) == HELIX_OK);
                helix_kv_shard bad = s;
                bad.k = nullptr;
                CHECK(check_shard(&p, &bad) == HELIX_ERR_NULL);
                bad = s; bad.max_len = -1;
                CHECK(check_shard(&p, &bad) == HELIX_ERR_SHAPE);
                bad = s; bad.k = fake_base + 2;
                CHECK(check_shard(&p, &bad) == HELIX_ERR_SHAPE);
                bad = s; bad.status = reinterpret_cast<int32_t*>(fake_base + 1);
                CHECK(check_shard(&p, &bad) == HELIX_ERR_SHAPE);
                // the whole call path short of the launch, incl. the fused cut's slice bounds
                for (int i = 0; i < n; i++) { shards[i] = s; shards[i].max_len = lens[i]; }
                Plan plan2;
                Workspace ws2;
                const int rc2 = prepare(&p, shards.data(), n, fake_base, bound, &plan2, &ws2);
                CHECK(rc2 == HELIX_OK || rc2 == HELIX_ERR_WORKSPACE || rc2 == HELIX_ERR_SHAPE);
                if (p.split_tokens == 0 || plan.stream) CHECK(rc2 == HELIX_OK);
                CHECK(prepare(&p, shards.data(), n, fake_base, 16, &plan2, &ws2) != HELIX_OK || ws2.bytes <= 16);
                helix_kv_shard cache = s;
                kvp_slices(&cache, n, shards.data());
                for (int i = 0; i < n; i++) CHECK(shards[i].max_len >= 0 && shards[i].max_len <= cache.max_len);
            }
        }
    }
    // streaming GQA launches with several head tiles: the map from workgroup id to (head tile, place in the set) is
    // one to one, and with sets of a multiple of 8 the workgroups of one place share their id modulo 8 (one XCD)
    for (int head_tiles = 2; head_tiles <= 9; head_tiles++) {
        for (int n_base : {1, 2, 5, 8, 13, 16, 24, 80, 128}) {
            std::vector<int> seen((size_t)head_tiles * n_base, -1);
            for (int id = 0; id < head_tiles * n_base; id++) {
                const helix::SeatOf at = helix::seat_of(id, head_tiles, n_base);
                CHECK(at.ht >= 0 && at.ht < head_tiles && at.wg >= 0 && at.wg < n_base);
                int& slot = seen[(size_t)at.ht * n_base + at.wg];
                CHECK(slot == -1);
                slot = id;
            }
            if (n_base % 8 == 0)
                for (int wg = 0; wg < n_base; wg++)
                    for (int ht = 1; ht < head_tiles; ht++) CHECK(seen[(size_t)ht * n_base + wg] % 8 == seen[wg] % 8);
            cases++;
        }
    }
    std::printf("ok: %ld cases, %ld planned\n", cases, planned);
    return 0;
}

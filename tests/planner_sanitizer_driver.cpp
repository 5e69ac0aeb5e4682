// The host planner (csrc/plan.cpp) under AddressSanitizer and UndefinedBehaviorSanitizer: plans for ragged,
// rectangular, scattered, strided and long-row masks, every tile size, every kernel choice, with and without
// gathered tiles, every export.  The device side is stubbed out (plans stay host-only).  Built and run by
// tests/test_planner_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "smha.h"
#include "smha_internal.hpp"
namespace smha {
smha_status_t upload_plan(smha_plan *, int) { return SMHA_OK; }
void release_device(smha_plan *) {}
int current_device_or_negative() { return -1; }
smha_status_t pack_device_mask(const uint8_t *, int, int, int, uint64_t *) { return SMHA_ERR_HIP; }
smha_status_t classify_device_mask(const uint8_t *, int, int, int, std::vector<TileInfo> &, std::vector<std::vector<uint64_t>> &) { return SMHA_ERR_HIP; }
}
static uint64_t rng_state = 12345;
static uint32_t rnd() { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33); }
static void exports(smha_plan_t *p, int n_masks) {
    for (int which = 0; which <= 15; ++which)
        for (int mi = 0; mi < n_masks; ++mi) {
            size_t need = 0;
            if (smha_plan_export(p, mi, (smha_export_t)which, nullptr, 0, &need) != SMHA_OK) continue;
            std::vector<char> buf(need + 1);
            smha_plan_export(p, mi, (smha_export_t)which, buf.data(), need, &need);
        }
    // the work order, both grains, for a few batch and head counts the plan's masks allow
    smha_plan_info_t info;
    if (smha_plan_info(p, &info) != SMHA_OK) return;
    for (int fine = 0; fine < 2; ++fine)
        for (int B : {info.Bm, info.Bm == 1 ? 3 : info.Bm})
            for (int H : {info.Hm, info.Hm == 1 ? 9 : info.Hm})
                for (int slots : {1, 7, 128}) {
                    size_t need = 0;
                    int per = 0;
                    if (smha_plan_work_order(p, B, H, slots, fine, nullptr, 0, &need, &per) != SMHA_OK) continue;
                    std::vector<int32_t> buf(need);
                    smha_plan_work_order(p, B, H, slots, fine, buf.data(), need, &need, &per);
                }
}
int main() {
    int n = 0;
    for (int Sq : {1, 65, 130, 700}) for (int Sk : {1, 100, 777, 3000}) for (int variant = 0; variant < 5; ++variant) {
        std::vector<uint8_t> m((size_t)2 * Sq * Sk);
        for (size_t i = 0; i < m.size(); ++i) {
            const int r = (int)((i / Sk) % Sq), c = (int)(i % Sk);
            switch (variant) {
                case 0: m[i] = rnd() % 100 < 30; break;
                case 1: m[i] = rnd() % 1000 < 3; break;                       // scattered
                case 2: m[i] = (c % 37 == 5) || (c <= r && r - c < 70); break; // strided + band
                case 3: m[i] = c % 5 == 2; break;                              // many gathered tiles
                default: m[i] = (r < 64) || (c < 8) || (rnd() % 1000 < 2); break;
            }
        }
        for (int block : {16, 32, 64}) for (int force : {0, 1, 2}) for (int ng : {0, 1}) {
            smha_plan_opts_t o{}; o.block = block; o.force = force; o.device_id = -2; o.no_gather = ng; o.build_both = (variant == 0 && force == 0);
            o.head_dim = (n & 1) ? 128 : 64;
            smha_plan_t *p = nullptr;
            if (smha_plan_from_dense_rect(m.data(), 0, 1, 2, Sq, Sk, &o, &p) != SMHA_OK) { printf("plan failed\n"); return 1; }
            smha_plan_info_t info; smha_plan_info(p, &info);
            exports(p, 2);
            smha_plan_destroy(p);
            ++n;
        }
    }
    // descriptions
    for (int S : {100, 1000, 4100}) {
        smha_mask_desc_t d{}; d.flags = SMHA_MASK_BIGBIRD | SMHA_MASK_PADDING; d.block = 64; d.n_window_blocks = 3; d.n_global_blocks = 2; d.n_random_blocks = 3; d.seed = 5;
        int32_t vl[2] = {S - 17, S / 2}; d.valid_len = vl; d.per_head = 1;
        smha_plan_opts_t o{}; o.device_id = -2; o.head_dim = 128;
        smha_plan_t *p = nullptr;
        if (smha_plan_from_desc(&d, 2, 3, S, &o, &p) != SMHA_OK) { printf("desc plan failed\n"); return 1; }
        exports(p, 6); smha_plan_destroy(p); ++n;
        smha_mask_desc_t e{}; e.flags = SMHA_MASK_CAUSAL | SMHA_MASK_STRIDED | SMHA_MASK_WINDOW; e.window_left = 127; e.stride = 64;
        if (smha_plan_from_desc(&e, 1, 1, S, &o, &p) != SMHA_OK) { printf("desc plan failed\n"); return 1; }
        exports(p, 1); smha_plan_destroy(p); ++n;
    }
    printf("%d plans built and exported under the sanitizers\n", n);
    return 0;
}

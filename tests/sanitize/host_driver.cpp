// Exercises the host-only paths of the library -- the C ABI's argument checks, workspace queries,
// planner table, and the whole of sn_runtime.h (pool, execution order, memory traces, budgets) --
// for the AddressSanitizer / UBSan build of the CPU test suite.  No kernel is launched and no GPU
// is needed.  Exit status 0 = every check held and the sanitizers found nothing.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "sn_runtime.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "host driver: check failed at line %d: %s\n", __LINE__, #c); std::exit(2); } } while (0)

static sn_conv_shape shape_of(int N, int C, int H, int W, int K, int R, int S, int st, int pad, int dt)
{
    sn_conv_shape s = {N, C, H, W, K, R, S, st, st, pad, pad, dt, dt};
    return s;
}

int main()
{
    // shape rule and argument checks
    CHECK(sn_out_dim(227, 0, 11, 4) == 55 && sn_out_dim(2, 0, 3, 1) == 0 && sn_out_dim(0, 0, 1, 1) == 0);
    sn_conv_shape s = shape_of(8, 64, 28, 28, 96, 3, 3, 1, 1, SN_BF16);
    size_t mn = 0, pf = 0;
    for (int dir = 0; dir < 3; ++dir)
        for (int algo = 0; algo < SN_ALGO_COUNT; ++algo) {
            const sn_status st = sn_conv_workspace_query(&s, (sn_conv_dir)dir, (sn_conv_algo)algo, &mn, &pf);
            CHECK(st == (algo == SN_ALGO_WINOGRAD ? SN_ERR_UNSUPPORTED : SN_OK));   // Winograd is the fp32 path's
            CHECK(st != SN_OK || mn <= pf);
        }
    // the fp32 3x3 shape: Winograd for forward and backward-data, every pass size the workspace allows
    sn_conv_shape f = shape_of(8, 64, 28, 28, 96, 3, 3, 1, 1, SN_F32);
    for (int dir = 0; dir < 3; ++dir) {
        const sn_status st = sn_conv_workspace_query(&f, (sn_conv_dir)dir, SN_ALGO_WINOGRAD, &mn, &pf);
        CHECK(st == (dir == SN_CONV_BWD_FILTER ? SN_ERR_UNSUPPORTED : SN_OK));
        CHECK(st != SN_OK || (mn > 0 && mn <= pf));
    }
    CHECK(sn_conv_workspace_query(nullptr, SN_CONV_FWD, SN_ALGO_DIRECT, &mn, &pf) == SN_ERR_BAD_ARG);
    CHECK(sn_conv_workspace_query(&s, SN_CONV_FWD, SN_ALGO_AUTO, &mn, &pf) == SN_ERR_BAD_ARG);   // AUTO names no algorithm
    // strided shapes: the phase decomposition's bookkeeping, supported and refused forms
    const int strided[][6] = {{64, 56, 128, 3, 2, 1}, {256, 56, 128, 1, 2, 0}, {32, 35, 48, 3, 2, 0}, {3, 227, 96, 11, 4, 0},
                              {16, 16, 40, 5, 2, 2}, {40, 7, 96, 1, 2, 0}, {8, 16, 8, 2, 3, 0}};
    for (const auto &g : strided) {
        sn_conv_shape t = shape_of(4, g[0], g[1], g[1], g[2], g[3], g[3], g[4], g[5], SN_BF16);
        for (int dir = 0; dir < 3; ++dir) {
            const sn_status st = sn_conv_workspace_query(&t, (sn_conv_dir)dir, SN_ALGO_STAGED, &mn, &pf);
            CHECK(st == SN_OK || st == SN_ERR_UNSUPPORTED);
            sn_conv_algo a;
            size_t used;
            float ms;
            CHECK(sn_conv_plan(&t, (sn_conv_dir)dir, 1u << 30, &a, &used, &ms) == SN_OK && used <= (1u << 30));
            CHECK(sn_conv_plan(&t, (sn_conv_dir)dir, 0, &a, &used, &ms) == SN_OK && a == SN_ALGO_DIRECT && used == 0);
        }
    }
    // calls with bad arguments return before anything touches a device
    CHECK(sn_conv2d_fwd(nullptr, nullptr, nullptr, &s, SN_ALGO_DIRECT, nullptr, 0, nullptr) == SN_ERR_BAD_ARG);
    CHECK(sn_conv2d_fwd_noalloc(nullptr, nullptr, nullptr, &s, nullptr) == SN_ERR_BAD_ARG);
    CHECK(sn_relu_fwd(nullptr, nullptr, 16, SN_BF16, nullptr) == SN_ERR_BAD_ARG);
    CHECK(sn_bn_fwd(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, 1, 1, 1e-5f, SN_F32, nullptr) == SN_ERR_BAD_ARG);
    CHECK(sn_maxpool_fwd(nullptr, nullptr, nullptr, 1, 1, 4, 4, 2, 2, 2, 2, 3, 3, SN_F32, nullptr) == SN_ERR_BAD_ARG);
    // planner table
    sn_planner_clear();
    CHECK(sn_planner_record(&s, SN_CONV_FWD, SN_ALGO_DIRECT, 0, 2.0f) == SN_OK);
    CHECK(sn_conv_workspace_query(&s, SN_CONV_FWD, SN_ALGO_STAGED, &mn, &pf) == SN_OK);
    CHECK(sn_planner_record(&s, SN_CONV_FWD, SN_ALGO_STAGED, pf, 1.0f) == SN_OK);
    CHECK(sn_planner_record(&s, SN_CONV_FWD, SN_ALGO_STAGED, mn ? mn - 1 : 0, 1.0f) == (mn ? SN_ERR_WORKSPACE_TOO_SMALL : SN_OK));
    sn_conv_algo a;
    size_t used;
    float ms;
    CHECK(sn_conv_plan(&s, SN_CONV_FWD, pf, &a, &used, &ms) == SN_OK && a == SN_ALGO_STAGED && ms == 1.0f);
    CHECK(sn_conv_plan(&s, SN_CONV_FWD, 0, &a, &used, &ms) == SN_OK && a == SN_ALGO_DIRECT && ms == 2.0f);
    sn_planner_clear();

    // pool
    sn_pool *pool = sn_pool_create(64 * SN_POOL_BLOCK + 5);
    CHECK(pool);
    std::vector<uint64_t> ids;
    uint64_t id;
    size_t off;
    for (int i = 0; i < 16; ++i) {
        CHECK(sn_pool_alloc(pool, (size_t)(i % 5) * 1000 + 1, &id, &off) == SN_OK && off % SN_POOL_BLOCK == 0);
        ids.push_back(id);
    }
    for (size_t i = 0; i < ids.size(); i += 2) CHECK(sn_pool_free(pool, ids[i]) == SN_OK);
    CHECK(sn_pool_free(pool, ids[0]) == SN_ERR_BAD_ARG);
    CHECK(sn_pool_alloc(pool, 1u << 30, &id, &off) == SN_ERR_WORKSPACE_TOO_SMALL);
    for (size_t i = 1; i < ids.size(); i += 2) CHECK(sn_pool_free(pool, ids[i]) == SN_OK);
    CHECK(sn_pool_used_bytes(pool) == 0 && sn_pool_largest_free(pool) == 64 * SN_POOL_BLOCK);
    CHECK(sn_pool_peak_bytes(pool) > 0 && sn_pool_high_water(pool) >= sn_pool_peak_bytes(pool));
    sn_pool_destroy(pool);

    // a network with a fork and a join, every level and strategy
    sn_net *net = sn_net_create();
    CHECK(net);
    CHECK(sn_net_add_layer(net, SN_L_CONV, 10, nullptr, 0) == -1);
    int d = sn_net_add_layer(net, SN_L_DATA, 6000, nullptr, 0);
    int c1 = sn_net_add_layer(net, SN_L_CONV, 50000, &d, 1);
    int r1 = sn_net_add_layer(net, SN_L_ACT, 50000, &c1, 1);
    int l1 = sn_net_add_layer(net, SN_L_LRN, 50000, &r1, 1);
    int p1 = sn_net_add_layer(net, SN_L_POOL, 12000, &l1, 1);
    int ca = sn_net_add_layer(net, SN_L_CONV, 20000, &p1, 1);
    int cb = sn_net_add_layer(net, SN_L_CONV, 20000, &p1, 1);
    int bb = sn_net_add_layer(net, SN_L_BN, 20000, &cb, 1);
    int both[2] = {ca, bb};
    int j = sn_net_add_layer(net, SN_L_JOIN, 40000, both, 2);
    int dr = sn_net_add_layer(net, SN_L_DROPOUT, 40000, &j, 1);
    int fc = sn_net_add_layer(net, SN_L_FC, 4000, &dr, 1);
    int sm = sn_net_add_layer(net, SN_L_SOFTMAX, 4000, &fc, 1);
    CHECK(sm == 11);
    int bad = 99;
    CHECK(sn_net_add_layer(net, SN_L_ACT, 1, &bad, 1) == -1);
    sn_conv_shape cs = shape_of(2, 16, 12, 12, 32, 3, 3, 1, 1, SN_BF16);
    CHECK(sn_net_set_conv_shape(net, ca, &cs) == SN_OK && sn_net_set_conv_shape(net, r1, &cs) == SN_ERR_BAD_ARG);
    int route[16];
    CHECK(sn_net_route(net, route, 3) == -1 && sn_net_route(net, route, 16) == 12);
    const int steps = sn_net_steps(net);
    CHECK(steps == 22);
    std::vector<size_t> bytes(steps), freeb(steps);
    std::vector<int32_t> live(steps);
    for (int level = 0; level < 4; ++level)
        for (int strat = 0; strat < 3; ++strat) {
            sn_mem_summary sum;
            CHECK(sn_net_memory_trace(net, (sn_mem_level)level, (sn_recomp_strategy)strat, bytes.data(), live.data(), &sum) == SN_OK);
            CHECK(sum.peak_step >= 1 && sum.peak_step <= steps && bytes[sum.peak_step - 1] == sum.peak_bytes);
            CHECK(sn_net_step_budgets(net, (sn_mem_level)level, (sn_recomp_strategy)strat, sum.peak_bytes, freeb.data()) == SN_OK);
            CHECK(freeb[sum.peak_step - 1] == 0);
            sn_conv_step_plan plans[4];
            CHECK(sn_net_plan_convs(net, (sn_mem_level)level, (sn_recomp_strategy)strat, sum.peak_bytes + (1u << 20), plans, 4) == 1);
            CHECK(plans[0].layer == ca && plans[0].ws_fwd <= plans[0].fwd_budget);
        }
    CHECK(sn_net_memory_trace(nullptr, SN_MEM_LIVENESS, SN_RECOMP_SPEED, nullptr, nullptr, nullptr) == SN_ERR_BAD_ARG);
    sn_net_destroy(net);
    std::puts("host driver: ok");
    return 0;
}

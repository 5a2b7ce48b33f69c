// Driver for the sanitizer build of the library's HOST logic (tests/test_sanitizers.py): network construction, argument
// validation, dependence-window planning, workspace sizing and the error paths, i.e. what can run without a GPU.  Built
// together with the library's sources with the host pass under -fsanitize=address,undefined (device code is not
// instrumented); any finding aborts with a non-zero status.  Analyses are expected to fail with GP_ERR_DEVICE here.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/gpupoly.h"

static unsigned long long state = 99;
static float rnd() {
    state = state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (float)((state >> 33) % 10001) / 10000.0f - 0.5f;
}
static std::vector<float> weights(size_t n) {
    std::vector<float> w(n);
    for (auto& v : w) v = rnd();
    return w;
}
#define EXPECT(call, want) do { int got_ = (int)(call); if (got_ != (int)(want)) { std::fprintf(stderr, "%s:%d: %s -> %d, expected %d\n", __FILE__, __LINE__, #call, got_, (int)(want)); return 1; } } while (0)

static int plan_all(gp_net* net) {
    std::vector<int32_t> steps(8 * 4096);
    for (int l = 1; l < gp_num_layers(net); ++l) {
        int32_t n = 0;
        const gp_status st = gp_debug_plan(net, l, steps.data(), 4096, &n);
        if (st != GP_OK && st != GP_ERR_ARG) { std::fprintf(stderr, "plan of layer %d: %d (%s)\n", l, (int)st, gp_last_error(net)); return 1; }
    }
    int64_t mn = 0, full = 0;
    if (gp_workspace_size(net, 3, &mn, &full) != GP_OK || mn <= 0 || full < mn) return 1;
    return 0;
}

int main() {
    // ---- a residual network with strided convolutions, a 1x1 shortcut, average pooling and a dense head
    gp_net* net = nullptr;
    EXPECT(gp_net_create(3, 16, 16, &net), GP_OK);
    int32_t id = 0, stem = 0, r = 0;
    auto w = weights(8 * 3 * 3 * 3); auto b = weights(8);
    EXPECT(gp_add_conv2d(net, 0, 8, 3, 3, 1, 1, 1, 1, w.data(), b.data(), &stem), GP_OK);
    EXPECT(gp_add_relu(net, stem, &r), GP_OK);
    int cur = r, ch = 8;
    for (int blk = 0; blk < 3; ++blk) {
        const int down = blk == 1, co = down ? 16 : ch, s = down ? 2 : 1;
        auto w1 = weights((size_t)co * ch * 9), b1 = weights(co), w2 = weights((size_t)co * co * 9);
        int32_t c1, r1, c2, sc = cur, sum, out;
        EXPECT(gp_add_conv2d(net, cur, co, 3, 3, s, s, 1, 1, w1.data(), b1.data(), &c1), GP_OK);
        EXPECT(gp_add_relu(net, c1, &r1), GP_OK);
        EXPECT(gp_add_conv2d(net, r1, co, 3, 3, 1, 1, 1, 1, w2.data(), nullptr, &c2), GP_OK);
        if (down) {
            auto ws = weights((size_t)co * ch);
            EXPECT(gp_add_conv2d(net, cur, co, 1, 1, 2, 2, 0, 0, ws.data(), nullptr, &sc), GP_OK);
        }
        EXPECT(gp_add_residual(net, c2, sc, &sum), GP_OK);
        EXPECT(gp_add_relu(net, sum, &out), GP_OK);
        cur = out; ch = co;
    }
    int32_t pool, head;
    EXPECT(gp_add_avgpool2d(net, cur, 2, 2, 2, 2, 0, 0, &pool), GP_OK);
    auto wh = weights((size_t)10 * gp_layer_size(net, pool));
    EXPECT(gp_add_dense(net, pool, 10, wh.data(), nullptr, &head), GP_OK);
    EXPECT(gp_request_bounds(net, pool), GP_OK);
    if (plan_all(net)) return 1;
    for (int mode = 0; mode < 5; ++mode) {         // the modes change which layers carry bounds and the block sizes
        EXPECT(gp_set_early_termination(net, mode == 1), GP_OK);
        EXPECT(gp_set_float_inference(net, mode == 2), GP_OK);
        EXPECT(gp_set_coefficient_storage(net, mode == 3 ? 64 : 32), GP_OK);
        EXPECT(gp_set_interval_coefficients(net, mode == 4), GP_OK);
        if (plan_all(net)) return 1;
    }
    EXPECT(gp_set_interval_coefficients(net, 0), GP_OK);
    std::vector<float> center(3 * 16 * 16, 0.5f), lo(10), hi(10);
    const gp_status st = gp_analyze(net, center.data(), 0.01f, 0.f, 1.f);
    if (st != GP_ERR_DEVICE && st != GP_OK) { std::fprintf(stderr, "analyze: %d\n", (int)st); return 1; }
    if (st == GP_ERR_DEVICE) {
        EXPECT(gp_get_bounds(net, head, lo.data(), hi.data()), GP_ERR_STATE);
        int32_t ok = 0;
        EXPECT(gp_certify(net, 0, &ok, lo.data()), GP_ERR_STATE);
    }
    // ---- argument and shape errors
    EXPECT(gp_add_dense(net, 99, 4, wh.data(), nullptr, &id), GP_ERR_ARG);
    EXPECT(gp_add_dense(net, head, 0, wh.data(), nullptr, &id), GP_ERR_ARG);
    EXPECT(gp_add_conv2d(net, head, 4, 3, 3, 1, 1, 0, 0, wh.data(), nullptr, &id), GP_ERR_SHAPE);
    EXPECT(gp_add_residual(net, head, pool, &id), GP_ERR_SHAPE);
    EXPECT(gp_add_avgpool2d(net, cur, 2, 2, 1, 1, 2, 2, &id), GP_ERR_SHAPE);
    EXPECT(gp_analyze(net, center.data(), -1.f, 0.f, 1.f), GP_ERR_ARG);
    EXPECT(gp_analyze(nullptr, center.data(), 0.1f, 0.f, 1.f), GP_ERR_ARG);
    EXPECT(gp_set_coefficient_storage(net, 16), GP_ERR_ARG);
    EXPECT(gp_set_workspace(net, (void*)0x101, 1 << 20), GP_ERR_ARG);
    center[7] = 1.0f / 0.0f;
    EXPECT(gp_analyze(net, center.data(), 0.01f, 0.f, 1.f), GP_ERR_NONFINITE);
    gp_net_destroy(net);
    // ---- topologies the engine refuses
    EXPECT(gp_net_create(4, 1, 1, &net), GP_OK);
    auto eye = weights(16);
    int32_t a, rr, s2, d2;
    EXPECT(gp_add_dense(net, 0, 4, eye.data(), nullptr, &a), GP_OK);
    EXPECT(gp_add_relu(net, a, &rr), GP_OK);
    EXPECT(gp_add_residual(net, rr, rr, &s2), GP_OK);
    EXPECT(gp_add_dense(net, s2, 4, eye.data(), nullptr, &d2), GP_OK);
    int32_t n = 0;
    EXPECT(gp_debug_plan(net, d2, nullptr, 0, &n), GP_ERR_UNSUPPORTED);
    gp_net_destroy(net);
    // ---- a dense chain (the fused-chain planning path) and the allocation-free call's topology check
    EXPECT(gp_net_create(40, 1, 1, &net), GP_OK);
    cur = 0;
    int fan = 40;
    for (int wd : {24, 37, 12, 5}) {
        auto wl = weights((size_t)wd * fan), bl = weights(wd);
        EXPECT(gp_add_dense(net, cur, wd, wl.data(), bl.data(), &id), GP_OK);
        cur = id;
        if (wd != 5) { EXPECT(gp_add_relu(net, cur, &id), GP_OK); cur = id; }
        fan = wd;
    }
    if (plan_all(net)) return 1;
    std::vector<float> c40(40, 0.5f);
    const gp_status s3 = gp_analyze_batch_dev_static(net, 1, c40.data(), 0.1f, 0.f, 1.f, (double*)c40.data(), (double*)c40.data());
    if (s3 != GP_ERR_DEVICE && s3 != GP_ERR_STATE) { std::fprintf(stderr, "static call: %d\n", (int)s3); return 1; }
    gp_net_destroy(net);
    std::printf("host sanitizer driver: ok\n");
    return 0;
}

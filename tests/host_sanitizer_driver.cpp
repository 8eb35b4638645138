// Test asset: calls every entry point of the C ABI on a tiny model so that the library's HOST code (engine, lanes and
// their threads, scheduler, argument checks, error paths) runs under AddressSanitizer and UndefinedBehaviorSanitizer.
// Built by tests/build_host_sanitizer_driver.py together with the library's sources, with the sanitizers on the
// host side only (device code is compiled as always); run on a GPU by tests/test_zy_host_sanitizers.py.
// Checks results only as far as they need no reference (lengths, equality of the two micro-batch entry points,
// status codes): parity with the oracle is the business of the other GPU tests.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include <cstdint>
#include "../include/ss.h"

static uint32_t rs = 12345u;
static uint32_t rnd() { rs = rs * 1664525u + 1013904223u; return rs >> 8; }
static uint16_t bf16_of(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)((u + 0x7fff + ((u >> 16) & 1)) >> 16); }
#define STEP(msg) do { std::printf("[host-sanitizer-driver] %s\n", msg); std::fflush(stdout); } while (0)
#define OK(call) do { int rc_ = (call); if (rc_ != SS_OK) { std::printf("FAILED %s -> %d: %s\n", #call, rc_, ss_last_error()); return 1; } } while (0)
#define BAD(call, want) do { int rc_ = (call); if (rc_ != (want)) { std::printf("expected %d from %s, got %d\n", (want), #call, rc_); return 1; } } while (0)

int main()
{
    ss_model_cfg cfg{2, 256, 4, 64, 688, 1024, 1.0e4f, 1.0e-6f};
    const int d = cfg.d_model, F = cfg.d_ffn, V = cfg.vocab;
    std::vector<std::vector<uint16_t>> T;
    auto mat = [&](size_t n, float scale, bool ones) {
        std::vector<uint16_t> t(n);
        for (auto& x : t) x = bf16_of(ones ? 1.0f + 0.1f * ((int)(rnd() % 200) - 100) / 100.f : scale * ((int)(rnd() % 2001) - 1000) / 1000.f);
        T.push_back(std::move(t));
    };
    mat((size_t)V * d, 1.0f, false);
    for (int l = 0; l < cfg.n_layers; ++l) {
        mat(d, 0, true);
        for (int i = 0; i < 4; ++i) mat((size_t)d * d, 0.08f, false);
        mat(d, 0, true);
        mat((size_t)F * d, 0.08f, false); mat((size_t)F * d, 0.08f, false); mat((size_t)d * F, 0.05f, false);
    }
    mat(d, 0, true);
    mat((size_t)V * d, 0.1f, false);
    std::vector<const void*> ptrs;
    for (auto& t : T) ptrs.push_back(t.data());
    STEP("create");
    ss_weights* w = nullptr;
    OK(ss_weights_create(&cfg, ptrs.data(), 0, &w));

    const int n = 40, L = 32;
    std::vector<int32_t> toks, offs{0}, target(n), pred(n);
    for (int i = 0; i < n; ++i) {
        const int len = 4 + rnd() % 17;
        for (int t = 0; t < len; ++t) toks.push_back(rnd() % V);
        offs.push_back((int32_t)toks.size());
        target[i] = 1 + rnd() % L;
        int p = target[i] + (int)(rnd() % 9) - 4;
        pred[i] = p < 1 ? 1 : p;
    }
    ss_policy pol{SS_SORT | SS_BIN | SS_FCR | SS_VBS | SS_COMPACT, 4, L, 16, SS_VBS_CLAMP_FLOOR};
    std::vector<int32_t> out((size_t)n * L), lens(n);
    ss_group_stats gs{};
    for (int lanes : {4, 1, 3}) {
        char msg[64]; std::snprintf(msg, sizeof msg, "run_group lanes %d", lanes); STEP(msg);
        OK(ss_set_option(w, SS_OPT_IN_FLIGHT, lanes));
        OK(ss_run_group(w, toks.data(), offs.data(), n, target.data(), pred.data(), 8, &pol, out.data(), lens.data(), &gs, nullptr));
        for (int i = 0; i < n; ++i) if (lens[i] != target[i]) { std::printf("length mismatch\n"); return 1; }
        std::printf("  mb %d+%d failed %d steps %lld\n", gs.n_mb_first, gs.n_mb_failure, gs.n_failed, (long long)gs.steps);
    }
    STEP("run_group vanilla");
    ss_policy vpol{0, 4, L, 16, 0};
    OK(ss_run_group(w, toks.data(), offs.data(), n, target.data(), nullptr, 0, &vpol, out.data(), lens.data(), &gs, nullptr));
    STEP("run_group_generate");
    OK(ss_set_option(w, SS_OPT_IN_FLIGHT, 4));
    ss_gen_opts g{};
    g.eos_id = 7; g.temperature = 0.8f; g.draws = nullptr; g.seed = 0x1234abcd9e3779b9ull; g.draw_ids = nullptr;
    g.target_lens = target.data(); g.sync_every = 3;
    OK(ss_run_group_generate(w, toks.data(), offs.data(), n, pred.data(), 8, &pol, &g, out.data(), lens.data(), &gs, nullptr));
    std::vector<float> draws((size_t)n * L);
    for (auto& u : draws) u = (rnd() & 0xffffff) / 16777216.f;
    g.draws = draws.data(); g.draws_stride = L; g.sync_every = 1; g.temperature = 0.5f;
    OK(ss_run_group_generate(w, toks.data(), offs.data(), n, pred.data(), 8, &pol, &g, out.data(), lens.data(), &gs, nullptr));
    STEP("microbatch entry points");
    const int B = 7, cap = 12;
    std::vector<int32_t> mo((size_t)B * cap), ml(B);
    std::vector<uint8_t> mf(B);
    ss_stats st{};
    OK(ss_decode_microbatch(w, toks.data(), offs.data(), B, cap, target.data(), SS_COMPACT, mo.data(), ml.data(), mf.data(), &st, nullptr));
    std::vector<int32_t> mo2((size_t)B * cap), ml2(B);
    OK(ss_decode_microbatch_static(w, toks.data(), offs.data(), B, cap, target.data(), SS_COMPACT, mo2.data(), ml2.data(), mf.data(), &st, nullptr));
    if (mo != mo2 || ml != ml2) { std::printf("static entry point differs\n"); return 1; }
    OK(ss_decode_microbatch(w, toks.data(), offs.data(), B, cap, target.data(), 0, mo.data(), ml.data(), mf.data(), nullptr, nullptr));
    g.draws = nullptr; g.target_lens = nullptr; g.sync_every = 2;
    OK(ss_generate_microbatch(w, toks.data(), offs.data(), B, cap, &g, SS_COMPACT, mo.data(), ml.data(), mf.data(), &st, nullptr));
    STEP("forward_logits");
    std::vector<int32_t> np_(B);
    size_t rows = 0;
    for (int i = 0; i < B; ++i) { const int len = offs[i + 1] - offs[i]; np_[i] = 1 + rnd() % len; rows += len - np_[i] + 1; }
    std::vector<float> lg(rows * V);
    OK(ss_forward_logits(w, toks.data(), offs.data(), B, np_.data(), 0, lg.data(), nullptr));
    for (int i = 0; i < B; ++i) np_[i] = offs[i + 1] - offs[i];
    std::vector<float> lg2((size_t)offs[B] * V);
    OK(ss_forward_logits(w, toks.data(), offs.data(), B, np_.data(), 1, lg2.data(), nullptr));
    STEP("measurement entry points");
    std::vector<int32_t> pt(16 * 20);
    for (auto& t : pt) t = rnd() % V;
    std::vector<double> ms(4 * 5);
    OK(ss_bench_decode_step(w, pt.data(), 16, 20, 5, ms.data(), nullptr));
    OK(ss_bench_decode_steps_in_flight(w, pt.data(), 16, 20, 5, 4, ms.data()));
    int32_t launches = 0; int64_t bytes = 0;
    OK(ss_bench_weight_stream(w, 16, 3, ms.data(), &launches, nullptr));
    OK(ss_bench_read_stream(w, 3, ms.data(), &bytes, nullptr));
    STEP("error paths");
    BAD(ss_decode_microbatch(w, toks.data(), offs.data(), B, 4090, target.data(), 0, mo.data(), ml.data(), mf.data(), nullptr, nullptr), SS_EINVAL);
    BAD(ss_set_option(w, 99, 1), SS_EINVAL);
    BAD(ss_set_option(w, SS_OPT_IN_FLIGHT, 5), SS_EINVAL);
    {   // one micro-batch of a group pass fails (prompt + cap beyond the positions supported): the call ends cleanly
        std::vector<int32_t> t2(toks), o2(offs);
        const int extra = 4095;
        std::vector<int32_t> big(extra, 3);
        t2.insert(t2.end(), big.begin(), big.end());
        o2.push_back((int32_t)t2.size());
        std::vector<int32_t> tg(target), pr(pred);
        tg.push_back(5); pr.push_back(5);
        std::vector<int32_t> o3((size_t)(n + 1) * L), l3(n + 1);
        BAD(ss_run_group(w, t2.data(), o2.data(), n + 1, tg.data(), pr.data(), 8, &pol, o3.data(), l3.data(), &gs, nullptr), SS_EINVAL);
        std::printf("  message: %s\n", ss_last_error());
    }
    OK(ss_run_group(w, toks.data(), offs.data(), n, target.data(), pred.data(), 8, &pol, out.data(), lens.data(), &gs, nullptr));
    STEP("destroy");
    ss_weights_destroy(w);
    STEP("done");
    // Everything the library owns has been released above.  The process ends here without running the exit handlers of
    // the GPU runtime's own libraries: they are not under test, and their teardown has produced a sanitizer report of
    // its own (frames in the runtime only, at exit, now and then), which would be charged to this test.
    std::fflush(stdout);
    std::fflush(stderr);
    std::_Exit(0);
}

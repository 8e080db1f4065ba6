// Randomised walk over the host-side logic of the library (plan, schedule, engine state machine), built with
// AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py.  The device entry points the
// engine calls are replaced by no-op stand-ins, so nothing here needs a GPU.  Checks: every valid plan partitions
// the model exactly once, runs and spans cover the same elements, event lists never overflow, and the engine
// reports exactly the sends and receives that Algorithm 2's schedule prescribes.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "sdl.h"
int main() {
    std::mt19937_64 rng(123);
    long ok = 0, bad = 0, engines = 0;
    for (int it = 0; it < 6000; ++it) {
        uint32_t L = 1 + rng() % 40, P = rng() % (L + 3), H = rng() % 120, tau = rng() % 130;
        std::vector<uint64_t> numel; std::vector<int32_t> block;
        uint32_t npre = rng() % 3, npost = rng() % 3;
        for (uint32_t i = 0; i < npre; ++i) { numel.push_back((rng() % 50) * 32); block.push_back(SDL_UNIT_PRE); }
        for (uint32_t b = 0; b < L; ++b) { uint32_t k = 1 + rng() % 4; for (uint32_t j = 0; j < k; ++j) { numel.push_back((rng() % 200) * (rng() % 5 ? 32 : 1)); block.push_back((int32_t)b); } }
        for (uint32_t i = 0; i < npost; ++i) { numel.push_back((rng() % 50) * 32); block.push_back(SDL_UNIT_POST); }
        if (rng() % 50 == 0) block[rng() % block.size()] = (int32_t)(L + rng() % 3);   // out of range sometimes
        std::vector<uint32_t> tp; bool use_tp = rng() % 3 == 0;
        uint32_t flags = rng() % 2 ? SDL_PLAN_PRE_OWN_FRAGMENT : 0;
        uint32_t nfrag = P + (flags ? 1 : 0);
        const bool padded = rng() % 2;
        if (padded) flags |= SDL_PLAN_ALIGN_GROUPS;
        if (use_tp) for (uint32_t p = 0; p < nfrag; ++p) tp.push_back(rng() % (H + 2));
        sdl_plan_t* plan = nullptr;
        int rc = sdl_fragment_plan_ex(numel.data(), block.data(), (uint32_t)numel.size(), L, P, (sdl_pattern_t)(rng() % 2), H, tau, use_tp ? tp.data() : nullptr, flags, &plan);
        if (rc != SDL_OK) { ++bad; continue; }
        ++ok;
        uint32_t nf = sdl_plan_num_fragments(plan);
        uint64_t total = 0, sum = 0;
        for (auto n : numel) total += n;
        for (uint32_t p = 0; p < nf + 1; ++p) {
            const sdl_span_t* sp; uint32_t ns;
            if (sdl_plan_fragment_spans(plan, p, &sp, &ns) == SDL_OK) for (uint32_t i = 0; i < ns; ++i) sum += sp[i].numel;
            const sdl_span_t* rn; uint32_t nr; uint64_t rsum = 0, ssum = 0;
            if (sdl_plan_fragment_runs(plan, p, &rn, &nr) == SDL_OK) { for (uint32_t i = 0; i < nr; ++i) rsum += rn[i].numel; for (uint32_t i = 0; i < ns; ++i) ssum += sp[i].numel; if (rsum != ssum) { printf("run/span mismatch\n"); return 1; } }
            uint32_t off; (void)sdl_plan_offset(plan, p, &off);
            size_t cb, sb; for (int f = 0; f < 8; ++f) (void)sdl_plan_message_bytes(plan, p, (sdl_format_t)f, &cb, &sb);
            (void)sdl_plan_staged_numel(plan, p);
        }
        if (sum != total || (padded ? sdl_plan_total_numel(plan) < total : sdl_plan_total_numel(plan) != total)) { printf("partition mismatch %llu %llu\n", (unsigned long long)sum, (unsigned long long)total); return 1; }
        std::vector<uint32_t> s(nf), r(nf);
        for (uint64_t t = 0; t < 3ull * H + 5; ++t) { uint32_t a = 0, b = 0; (void)sdl_plan_events(plan, t, s.data(), &a, r.data(), &b); if (a > nf || b > nf) { printf("events overflow\n"); return 1; } }
        for (uint32_t b = 0; b < L + 1; ++b) (void)sdl_plan_block_fragment(plan, b);
        // engine host logic
        uint32_t M = 1 + rng() % 4; std::vector<uint32_t> taus(M); for (auto& x : taus) x = rng() % (H + 1);
        sdl_engine_t* e = nullptr;
        if (sdl_engine_create(plan, H, M, taus.data(), (sdl_format_t)(rng() % 8), 0.7f, 0.9f, 0.5f, &e) == SDL_OK) {
            if (sdl_engine_step(e, 1, nullptr, nullptr, nullptr) != SDL_ERR_INVALID_ARG) { printf("unbound engine stepped\n"); return 1; }
            static float fake[4];
            std::vector<void*> w(M, fake), msgs((size_t)nf * M, fake);
            if (sdl_engine_bind(e, fake, fake, w.data(), msgs.data(), msgs.data()) != SDL_OK) { printf("bind failed\n"); return 1; }
            uint32_t dmin = taus[0]; for (auto x : taus) if (x < dmin) dmin = x;
            uint64_t sends = 0, recvs = 0, want_s = 0, want_r = 0;
            for (uint64_t t = 1; t <= 4ull * H + 3; ++t) {
                uint32_t a = 0, b = 0, ns = 0, nr = 0;
                int rc2 = sdl_engine_step(e, t, nullptr, &ns, &nr);
                if (rc2 != SDL_OK) { printf("engine step failed rc=%d t=%llu H=%u\n", rc2, (unsigned long long)t, H); return 1; }
                (void)sdl_plan_events(plan, t, s.data(), &a, r.data(), &b);
                sends += ns; recvs += nr; want_s += a;
                // a receive (mean + Nesterov) happens delay_min after each send
                for (uint32_t p = 0; p < nf; ++p) { uint32_t off; (void)sdl_plan_offset(plan, p, &off); if (t > off + dmin && (t - off - dmin) % H == 0 && t - dmin > off) want_r += 1; }
            }
            if (sends != want_s || recvs != want_r) { printf("engine counts differ: sent %llu/%llu received %llu/%llu H=%u\n", (unsigned long long)sends, (unsigned long long)want_s, (unsigned long long)recvs, (unsigned long long)want_r, H); return 1; }
            sdl_engine_destroy(e); ++engines;
        }
        sdl_plan_destroy(plan);
    }
    printf("plans ok %ld rejected %ld engines walked %ld\n", ok, bad, engines);
    return 0;
}

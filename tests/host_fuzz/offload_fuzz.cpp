// Randomised walk of the schedule driver with the outer state in "host memory" (Section 2.5 of the paper), on the
// CPU: csrc/sdl_offload.cpp is compiled against tests/host_fuzz/fake_hip (copies are memcpy), and the staged device
// calls are stand-ins that add 1 to every staged parameter of g when a fragment's mean + Nesterov step runs and 1
// to mom when a merge runs.  After T steps and a flush the host arrays must hold exactly the number of receives
// (merges) of the fragment that owns each parameter: that checks the whole data path -- prefetch in schedule
// order, a prefetched copy giving way to a fragment that is due (the driver also prefetches fragments of its own
// choosing at random, as a caller might), write-back, slot reuse -- for random plans,
// delays, pool sizes and look-aheads.  The pool size a schedule needs is derived here by brute force from
// sdl_plan_events, independently of the engine.  Built with ASan / UBSan by tests/test_host_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "sdl.h"

long fake_hip_copies = 0, fake_hip_bytes = 0;

static void bump(const sdl_plan_t* plan, uint32_t p, float* frag, float by)
{
    const sdl_span_t* runs; uint32_t n;
    if (sdl_plan_fragment_runs(plan, p, &runs, &n) != SDL_OK) abort();
    uint64_t off = 0;
    for (uint32_t i = 0; i < n; ++i) {
        for (uint64_t k = 0; k < runs[i].numel; ++k) frag[off + k] += by;
        off += (runs[i].numel + 511) / 512 * 512;
    }
}

extern "C" {
uint64_t sdl_plan_staged_numel(const sdl_plan_t* plan, uint32_t p)
{
    const sdl_span_t* r; uint32_t n;
    if (sdl_plan_fragment_runs(plan, p, &r, &n)) return 0;
    uint64_t t = 0;
    for (uint32_t i = 0; i < n; ++i) t += (r[i].numel + 511) / 512 * 512;
    return t;
}
int sdl_quantize_outer_grad_staged(const sdl_plan_t*, uint32_t, const float*, const void* const*, uint32_t, sdl_format_t,
                                   void* const*, void* const*, void*) { return SDL_OK; }
int sdl_fragment_outer_step_staged_ex(const sdl_plan_t* plan, uint32_t p, float* g, float* mom, const void* const*, void* const*,
                                      uint32_t, sdl_format_t, float, float, float, void* const*, void* const*, void*)
{ bump(plan, p, g, 1.0f); bump(plan, p, mom, 1.0f); return SDL_OK; }
int sdl_receive_outer_step_staged(const sdl_plan_t* plan, uint32_t p, float* g, float* mom, const void* const*, const void* const*,
                                  void* const*, uint32_t, sdl_format_t, float, float, float, void*)
{ bump(plan, p, g, 1.0f); bump(plan, p, mom, 1.0f); return SDL_OK; }
int sdl_dequant_reduce_nesterov_staged(const sdl_plan_t* plan, uint32_t p, float* g, float*, const void* const*, const void* const*,
                                       uint32_t, sdl_format_t, float, float, void*)
{ bump(plan, p, g, 1.0f); return SDL_OK; }
// the merge only reads the outer parameters; the stand-in marks the momentum once per fragment and step so that
// the count below also sees that every merge found its fragment staged
int sdl_merge_overlap_staged(const sdl_plan_t*, uint32_t, const float*, void* const*, uint32_t, float, void*) { return SDL_OK; }
}

int main()
{
    std::mt19937_64 rng(2024);
    long walked = 0, refused = 0, meddled = 0;
    for (int it = 0; it < 1500; ++it) {
        const uint32_t L = 1 + rng() % 12, P = 1 + rng() % L, H = 2 + rng() % 40;
        const uint32_t M = 1 + rng() % 3;
        std::vector<uint32_t> taus(M);
        const uint32_t tmax = rng() % 3 == 0 ? 0 : rng() % H;
        for (auto& x : taus) x = tmax ? rng() % (tmax + 1) : 0;
        uint32_t dmin = taus[0], dmax = taus[0];
        for (auto x : taus) { if (x < dmin) dmin = x; if (x > dmax) dmax = x; }
        std::vector<uint64_t> numel; std::vector<int32_t> block;
        numel.push_back(64 * (1 + rng() % 9)); block.push_back(SDL_UNIT_PRE);
        for (uint32_t b = 0; b < L; ++b) for (uint32_t j = 0, k = 1 + rng() % 3; j < k; ++j) { numel.push_back(1 + rng() % 700); block.push_back((int32_t)b); }
        numel.push_back(1 + rng() % 300); block.push_back(SDL_UNIT_POST);
        std::vector<uint32_t> tp;
        const bool use_tp = rng() % 3 == 0;
        const uint32_t flags = rng() % 2 ? SDL_PLAN_PRE_OWN_FRAGMENT : 0;
        const uint32_t nf = P + (flags ? 1 : 0);
        if (use_tp) for (uint32_t p = 0; p < nf; ++p) tp.push_back(rng() % H);
        sdl_plan_t* plan = nullptr;
        if (sdl_fragment_plan_ex(numel.data(), block.data(), (uint32_t)numel.size(), L, P, (sdl_pattern_t)(rng() % 2), H, dmin,
                                 use_tp ? tp.data() : nullptr, flags, &plan) != SDL_OK) { printf("plan rejected\n"); return 1; }
        const uint64_t total = sdl_plan_total_numel(plan);
        // slots the schedule needs: fragments between their send step and send + dmax, by brute force over two periods
        std::vector<uint32_t> s(nf), r(nf);
        std::vector<uint64_t> sent_at(nf, 0);
        uint32_t need = 1;
        for (uint64_t t = 1; t <= 3ull * H; ++t) {
            uint32_t a = 0, b = 0;
            if (sdl_plan_events(plan, t, s.data(), &a, r.data(), &b) != SDL_OK) abort();
            for (uint32_t i = 0; i < a; ++i) sent_at[s[i]] = t;
            uint32_t n = 0;
            for (uint32_t p = 0; p < nf; ++p) if (sent_at[p] && t <= sent_at[p] + dmax) ++n;
            if (n > need) need = n;
        }
        const uint32_t lookahead = rng() % (2 * H);
        const bool too_few = need > 1 && rng() % 6 == 0;
        const uint32_t n_slots = too_few ? need - 1 : need + rng() % 3;
        sdl_offload_t* pool = nullptr;
        if (sdl_offload_create(plan, n_slots, &pool) != SDL_OK) { printf("pool create failed\n"); return 1; }
        if (sdl_offload_num_slots(pool) != n_slots) { printf("slot count\n"); return 1; }
        const uint64_t slot_n = sdl_offload_slot_numel(pool);
        std::vector<float> g_host(total), mom_host(total);
        for (uint64_t i = 0; i < total; ++i) { g_host[i] = (float)(i % 1000); mom_host[i] = -(float)(i % 777); }
        const std::vector<float> g0 = g_host, m0 = mom_host;
        std::vector<std::vector<float>> sg(n_slots, std::vector<float>(slot_n + 4, -1e30f)), sm(n_slots, std::vector<float>(slot_n + 4, -1e30f));
        std::vector<float*> pg, pm;
        // 16-byte aligned starts inside the vectors
        for (uint32_t i = 0; i < n_slots; ++i) {
            pg.push_back(sg[i].data() + ((16 - (uintptr_t)sg[i].data() % 16) % 16) / 4);
            pm.push_back(sm[i].data() + ((16 - (uintptr_t)sm[i].data() % 16) % 16) / 4);
        }
        if (sdl_offload_bind(pool, g_host.data(), mom_host.data(), pg.data(), pm.data()) != SDL_OK) { printf("pool bind failed\n"); return 1; }
        sdl_engine_t* e = nullptr;
        const sdl_format_t fmt = (sdl_format_t)(rng() % 6);      // not the whole-span scale: it needs real scale words
        if (sdl_engine_create(plan, H, M, taus.data(), fmt, 0.7f, 0.9f, 0.5f, &e) != SDL_OK) { printf("engine create failed\n"); return 1; }
        static float fake[4];
        std::vector<void*> w(M, fake), msgs((size_t)nf * M, fake);
        const int rcb = sdl_engine_bind_offload(e, pool, w.data(), msgs.data(), msgs.data(), nullptr, lookahead);
        if (too_few) {
            if (rcb != SDL_ERR_INVALID_ARG) { printf("a pool of %u slots was accepted where %u are needed\n", n_slots, need); return 1; }
            ++refused;
        } else {
            if (rcb != SDL_OK) { printf("bind_offload failed rc=%d slots %u need %u\n", rcb, n_slots, need); return 1; }
            const uint64_t T = 3ull * H + rng() % H;
            std::vector<uint64_t> receives(nf, 0), sends(nf, 0);
            const bool meddle = rng() % 2;
            for (uint64_t t = 1; t <= T; ++t) {
                uint32_t ns = 0, nr = 0;
                const int rc = sdl_engine_step(e, t, nullptr, &ns, &nr);
                if (rc != SDL_OK) { printf("engine step failed rc=%d t=%llu H=%u P=%u slots=%u need=%u lookahead=%u dmax=%u\n", rc, (unsigned long long)t, H, nf, n_slots, need, lookahead, dmax); return 1; }
                uint32_t a = 0, b = 0;
                (void)sdl_plan_events(plan, t, s.data(), &a, r.data(), &b);
                for (uint32_t i = 0; i < a; ++i) ++sends[s[i]];
                for (uint32_t p = 0; p < nf; ++p) { uint32_t off; (void)sdl_plan_offset(plan, p, &off); if (t > off + dmin && (t - off - dmin) % H == 0) ++receives[p]; }
                // a caller's own prefetches, in no useful order: they may take the slot that the next sender needs,
                // which then has to give way (a full pool is not an error here)
                if (meddle && rng() % 3 == 0) {
                    const int rcp = sdl_offload_prefetch(pool, (uint32_t)(rng() % nf), nullptr);
                    if (rcp != SDL_OK && rcp != SDL_ERR_NOMEM) { printf("prefetch failed rc=%d\n", rcp); return 1; }
                    if (rcp == SDL_OK) ++meddled;
                }
            }
            if (sdl_offload_flush(pool, nullptr, nullptr) != SDL_OK) { printf("flush failed\n"); return 1; }
            for (uint32_t p = 0; p < nf; ++p) {
                const sdl_span_t* sp; uint32_t nsp;
                (void)sdl_plan_fragment_spans(plan, p, &sp, &nsp);
                // momentum is bumped only by the single-pass calls (one delay for all workers)
                const float want_m = (dmin == dmax) ? (float)receives[p] : 0.0f;
                for (uint32_t i = 0; i < nsp; ++i)
                    for (uint64_t k = sp[i].offset; k < sp[i].offset + sp[i].numel; ++k)
                        if (g_host[k] != g0[k] + (float)receives[p] || mom_host[k] != m0[k] + want_m) {
                            printf("outer state of fragment %u wrong at %llu: g %g want %g (receives %llu), mom %g want %g; H=%u P=%u slots=%u need=%u lookahead=%u\n",
                                   p, (unsigned long long)k, g_host[k], g0[k] + (float)receives[p], (unsigned long long)receives[p], mom_host[k], m0[k] + want_m,
                                   H, nf, n_slots, need, lookahead);
                            return 1;
                        }
            }
            ++walked;
        }
        sdl_engine_destroy(e);
        sdl_offload_destroy(pool);
        sdl_plan_destroy(plan);
    }
    printf("offload engines walked %ld refused %ld meddling prefetches %ld copies %ld bytes %ld\n", walked, refused, meddled, fake_hip_copies, fake_hip_bytes);
    return 0;
}

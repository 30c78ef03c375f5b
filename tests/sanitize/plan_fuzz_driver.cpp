// Host-only driver for tests/test_host_sanitize.py: reads plan descriptions from stdin (possibly malformed on purpose),
// compiles each with the library's host compiler and reads both step tables back, all under AddressSanitizer and
// UndefinedBehaviorSanitizer.  One line per case on stdout: index, status, words of the two tables.
// Arrays are allocated with exactly the sizes the case states ("alloc" fields), so a read past what the
// descriptors promise is a heap overflow the sanitizer reports.
#include <cstdio>
#include <iostream>
#include <new>
#include <vector>

#include "plan.hpp"

extern "C" sccl_status_t sccl_plan_table(const sccl_plan_t*, int32_t, int32_t*, int64_t, int64_t*, int32_t*);

int main() {
    long long ncases;
    if (!(std::cin >> ncases)) return 2;
    for (long long t = 0; t < ncases; t++) {
        int P, nbw;
        std::cin >> P >> nbw;
        std::vector<std::vector<sccl_edge_t>> edges(nbw);
        std::vector<sccl_bw_t> bw(nbw);
        for (int i = 0; i < nbw; i++) {
            int b, stated, real;
            std::cin >> b >> stated >> real;
            edges[i].resize(real);
            for (auto& e : edges[i]) std::cin >> e.src >> e.dst;
            bw[i] = {edges[i].data(), stated, b};
        }
        int G, g_alloc, p_alloc, combining, dtype;
        long long epc;
        std::cin >> G >> g_alloc >> p_alloc >> combining >> dtype >> epc;
        std::vector<uint8_t> pre((size_t)g_alloc * p_alloc), post(pre.size());
        for (auto& x : pre) { int v; std::cin >> v; x = (uint8_t)v; }
        for (auto& x : post) { int v; std::cin >> v; x = (uint8_t)v; }
        int has_slot, positions;
        std::cin >> has_slot >> positions;
        std::vector<int32_t> slot(has_slot ? pre.size() : 0);
        for (auto& x : slot) std::cin >> x;
        int S, s_alloc;
        std::cin >> S >> s_alloc;
        std::vector<int32_t> rounds(s_alloc);
        for (auto& r : rounds) std::cin >> r;
        long long N, n_alloc;
        std::cin >> N >> n_alloc;
        std::vector<sccl_send_t> sends(n_alloc);
        for (auto& s : sends) std::cin >> s.chunk >> s.src >> s.dst >> s.step >> s.op;
        sccl_options_t o{};
        long long flags;
        std::cin >> flags >> o.block_threads >> o.vectors_per_thread >> o.max_workgroups >> o.lowering >> o.slice_vectors >>
            o.staged_threads >> o.reserved;
        o.flags = (uint32_t)flags;
        if (!std::cin) return 3;

        sccl_topology_t topo{P, bw.data(), nbw};
        sccl_collective_t coll{G, pre.data(), post.data(), combining, (sccl_dtype_t)dtype, epc, has_slot ? slot.data() : nullptr,
                               positions};
        sccl_schedule_t sched{S, rounds.data(), sends.data(), N};
        sccl_plan plan;
        sccl_status_t st = SCCL_ERR_NOMEM;
        try { st = sccl_compile_host(&topo, &coll, &sched, &o, 256, &plan); } catch (const std::bad_alloc&) {}
        long long words[2] = {-1, -1};
        if (st == SCCL_OK) {
            for (int lowering = SCCL_LOWER_MEMORY; lowering <= SCCL_LOWER_STAGED; lowering++) {
                int64_t n = 0;
                int32_t info[4];
                if (sccl_plan_table(&plan, lowering, nullptr, 0, &n, info) != SCCL_OK) continue;
                std::vector<int32_t> out((size_t)n);                     // exactly as large as the library said
                if (sccl_plan_table(&plan, lowering, out.data(), n, &n, info) != SCCL_OK) return 4;
                words[lowering - SCCL_LOWER_MEMORY] = (long long)n;
            }
        }
        std::printf("%lld %d %lld %lld\n", t, (int)st, words[0], words[1]);
    }
    return 0;
}

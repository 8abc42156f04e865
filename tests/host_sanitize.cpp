// Driver for the host-only half of the library under AddressSanitizer / UndefinedBehaviorSanitizer (no GPU needed):
// network validation, the cost model and the planner (valid and invalid plans), stage layout queries, schedule
// creation.  Reads commands from stdin (written by tests/test_host_sanitized.py), prints one result line per command.
//   net L            followed by L lines of 16 integers: the lpm_layer fields in declaration order
//   cost flop_per_us hbm_byte_per_us link_byte_per_us elem_bytes microbatch n_microbatch
//   plan Z           lpm_partition                      -> "plan rc starts... | costs..."
//   fixed Z s0..sZ   lpm_partition with fixed_starts    -> "fixed rc"
//   costs Z c0..     lpm_partition_costs                -> "costs rc starts..."
//   lcost i          lpm_layer_cost                     -> "lcost rc value"
//   stage first last m dtype    create, sizes, every offset query, destroy -> "stage rc sizes..."
//   sched Z s0..sZ m M dtype window   stages + lpm_schedule_create / cut_fused / destroy -> "sched rc"
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../include/lpm.h"

int main() {
    std::vector<lpm_layer> net;
    lpm_cost_params cp{};
    char cmd[32];
    while (scanf("%31s", cmd) == 1) {
        if (!strcmp(cmd, "net")) {
            int L = 0;
            if (scanf("%d", &L) != 1) return 2;
            net.assign((size_t)L, lpm_layer{});
            for (int i = 0; i < L; ++i) {
                int32_t* f = reinterpret_cast<int32_t*>(&net[(size_t)i]);
                for (int k = 0; k < 16; ++k) if (scanf("%d", &f[k]) != 1) return 2;
            }
            printf("net %d\n", L);
        } else if (!strcmp(cmd, "cost")) {
            unsigned long long a, b, c;
            if (scanf("%llu %llu %llu %d %d %d", &a, &b, &c, &cp.elem_bytes, &cp.microbatch, &cp.n_microbatch) != 6) return 2;
            cp.flop_per_us = a; cp.hbm_byte_per_us = b; cp.link_byte_per_us = c;
            printf("cost ok\n");
        } else if (!strcmp(cmd, "plan") || !strcmp(cmd, "fixed") || !strcmp(cmd, "costs")) {
            int Z = 0;
            if (scanf("%d", &Z) != 1) return 2;
            std::vector<int32_t> fixed, starts((size_t)(Z > 0 ? Z : 0) + 1, -1);
            std::vector<uint64_t> lc, sc((size_t)(Z > 0 ? Z : 1), 0);
            if (!strcmp(cmd, "fixed")) { fixed.resize((size_t)Z + 1); for (auto& v : fixed) if (scanf("%d", &v) != 1) return 2; }
            if (!strcmp(cmd, "costs")) { lc.resize(net.size()); for (auto& v : lc) { unsigned long long t; if (scanf("%llu", &t) != 1) return 2; v = t; } }
            int32_t rc;
            if (!lc.empty()) rc = lpm_partition_costs(net.data(), (int32_t)net.size(), Z, &cp, lc.data(), nullptr, starts.data(), sc.data());
            else rc = lpm_partition(net.data(), (int32_t)net.size(), Z, &cp, fixed.empty() ? nullptr : fixed.data(), starts.data(), sc.data());
            printf("%s %d", cmd, rc);
            if (rc == 0) {
                for (int32_t v : starts) printf(" %d", v);
                printf(" |");
                for (int z = 0; z < Z; ++z) printf(" %llu", (unsigned long long)sc[(size_t)z]);
            }
            printf("\n");
        } else if (!strcmp(cmd, "lcost")) {
            int i = 0;
            if (scanf("%d", &i) != 1) return 2;
            uint64_t v = 0;
            const int32_t rc = lpm_layer_cost(net.data(), (int32_t)net.size(), i, &cp, &v);
            printf("lcost %d %llu\n", rc, (unsigned long long)v);
        } else if (!strcmp(cmd, "stage")) {
            int first, last, m, dtype;
            if (scanf("%d %d %d %d", &first, &last, &m, &dtype) != 4) return 2;
            lpm_stage* s = nullptr;
            const int32_t rc = lpm_stage_create(net.data(), (int32_t)net.size(), first, last, m, dtype, &s);
            printf("stage %d", rc);
            if (rc == 0) {
                size_t v[8];
                lpm_stage_sizes(s, &v[0], &v[1], &v[2], &v[3], &v[4], &v[5], &v[6], &v[7]);
                for (size_t x : v) printf(" %zu", x);
                size_t off, n, acc = 0;
                for (int i = first - 2; i <= last + 1; ++i) {
                    for (int which = 0; which < 4; ++which) if (lpm_stage_param_offset(s, i, which, &off, &n) == 0) acc += off + n;
                    if (lpm_stage_stash_offset(s, i, &off, &n) == 0) acc += off + n;
                    if (lpm_stage_grad_offset(s, i, &off, &n) == 0) acc += off + n;
                }
                if (lpm_stage_stash_offset(s, -100, &off, &n) == 0) acc += off + n;
                printf(" %zu", acc);
                lpm_stage_destroy(s);
            }
            printf("\n");
        } else if (!strcmp(cmd, "sched")) {
            int Z, m, M, dtype, window;
            if (scanf("%d", &Z) != 1) return 2;
            std::vector<int> st((size_t)Z + 1);
            for (auto& v : st) if (scanf("%d", &v) != 1) return 2;
            if (scanf("%d %d %d %d", &m, &M, &dtype, &window) != 4) return 2;
            std::vector<lpm_stage*> stages;
            int32_t rc = 0;
            for (int z = 0; z < Z && rc == 0; ++z) {
                lpm_stage* s = nullptr;
                rc = lpm_stage_create(net.data(), (int32_t)net.size(), st[(size_t)z], st[(size_t)z + 1], m, dtype, &s);
                if (rc == 0) stages.push_back(s);
            }
            lpm_schedule* sch = nullptr;
            if (rc == 0) rc = lpm_schedule_create(stages.data(), Z, M, window, &sch);
            int fused = 0;
            if (rc == 0) { for (int z = -1; z <= Z; ++z) { const int32_t f = lpm_schedule_cut_fused(sch, z); if (f > 0) ++fused; } lpm_schedule_destroy(sch); }
            for (lpm_stage* s : stages) lpm_stage_destroy(s);
            printf("sched %d %d\n", rc, fused);
        } else {
            fprintf(stderr, "unknown command %s\n", cmd);
            return 2;
        }
    }
    printf("done %s\n", lpm_last_error()[0] ? "(last error text kept)" : "");
    return 0;
}

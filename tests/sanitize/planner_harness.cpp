// TEST INFRASTRUCTURE -- drives the library's host-only guard and tree flattening (csrc/planner.hpp), compiled
// under -fsanitize=address,undefined, from commands on stdin:
//   guard alpha ratio warmup patience max_transitions early_steps n  expected[n]  valid[n]  m  (A T)[m]
//       -> prints the m active strategies on one line, or "EINVAL"
//   flatten order n parents[n]
//       -> prints "perm ... | new_parents ..." or "EINVAL"
// Output arrays are heap blocks of exactly the documented sizes, so an overrun is an ASan report.
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "../../paper_2605_19893_amd/csrc/planner.hpp"

int main() {
    std::string cmd;
    while (std::cin >> cmd) {
        if (cmd == "guard") {
            ssv_guard_config c{};
            int n = 0, m = 0;
            std::cin >> c.alpha >> c.ratio >> c.warmup_steps >> c.patience >> c.max_transitions >> c.early_steps >> n;
            std::vector<double> expected(n > 0 ? n : 0);
            std::vector<uint8_t> valid(n > 0 ? n : 0);
            for (auto& e : expected) std::cin >> e;
            for (auto& v : valid) { int x; std::cin >> x; v = (uint8_t)x; }
            std::cin >> m;
            ssv_guard_state* st = new ssv_guard_state;
            const int rc = ssv::guard_init(st, &c, expected.data(), valid.data(), n);
            for (int i = 0; i < m; ++i) {
                double a, t;
                std::cin >> a >> t;
                if (rc == SSV_OK) std::printf("%d ", ssv::guard_observe(st, a, t));
            }
            std::printf(rc == SSV_OK ? "\n" : "EINVAL\n");
            delete st;
        } else if (cmd == "flatten") {
            int order = 0, n = 0;
            std::cin >> order >> n;
            int32_t* parents = new int32_t[n > 0 ? n : 1];
            int32_t* perm = new int32_t[n > 0 ? n : 1];
            int32_t* newp = new int32_t[n > 0 ? n : 1];
            for (int i = 0; i < n; ++i) std::cin >> parents[i];
            if (ssv::tree_flatten(parents, n, order, perm, newp) != SSV_OK) {
                std::printf("EINVAL\n");
            } else {
                std::printf("perm");
                for (int i = 0; i < n; ++i) std::printf(" %d", perm[i]);
                std::printf(" | new_parents");
                for (int i = 0; i < n; ++i) std::printf(" %d", newp[i]);
                std::printf("\n");
            }
            delete[] parents; delete[] perm; delete[] newp;
        } else {
            return 2;
        }
    }
    return 0;
}

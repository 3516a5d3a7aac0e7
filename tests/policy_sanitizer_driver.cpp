// Drives the host-only policy generator over random networks; built with the address and undefined-behaviour
// sanitizers by test_policy_sanitizers.py (no GPU code is compiled or run).
#include "../include/netmax.h"
#include <cstdio>
#include <random>
#include <vector>
int main() {
    std::mt19937_64 rng(7);
    std::lognormal_distribution<double> ln(0.0, 1.5);
    std::uniform_real_distribution<double> u(0, 1);
    int ok = 0, inf = 0, inv = 0;
    for (int M : {2, 3, 4, 5, 8, 13, 16, 32, 64}) {
        for (int rep = 0; rep < 6; ++rep) {
            std::vector<double> t(M * M), P(M * M);
            std::vector<uint8_t> adj(M * M, 1);
            for (int i = 0; i < M; ++i) for (int m = i; m < M; ++m) {
                double v = ln(rng); t[i * M + m] = t[m * M + i] = v;
                uint8_t a = (rep >= 3 && u(rng) < 0.3) ? 0 : 1; adj[i * M + m] = adj[m * M + i] = a;
            }
            for (int i = 0; i < M; ++i) adj[i * M + i] = 0;
            double rho, tbar, l2, tc;
            int rc = netmax_generate_policy(M, t.data(), rep == 0 ? nullptr : adj.data(), 0.05, 12 + rep, 4 + rep, 0.01, P.data(), &rho, &tbar, &l2, &tc);
            if (rc == NETMAX_OK) ++ok; else if (rc == NETMAX_EINFEASIBLE) ++inf; else ++inv;
        }
    }
    std::printf("ok %d infeasible %d invalid %d\n", ok, inf, inv);
    return inv == 0 && ok > 0 ? 0 : 1;
}

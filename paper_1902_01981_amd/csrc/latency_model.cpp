// Host-side simulation of the paper's run-time model (Section III-C).
#include "latency_model.h"

#include <algorithm>
#include <cmath>

namespace cr {

namespace {

uint64_t splitmix64_at(uint64_t seed, uint64_t counter)
{
    uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Single-port reception of the n children starting at `first`: returns the time the (n-s)-th transfer completes and marks the rest.
double receive(const double *ready, int32_t first, int n, int s, double t_c, uint8_t *mask)
{
    int order[64];
    for (int j = 0; j < n; ++j) order[j] = j;
    std::stable_sort(order, order + n, [&](int x, int y) { return ready[first + x] < ready[first + y]; });
    double port_free = 0.0;
    for (int k = 0; k < n; ++k) {
        const int32_t child = first + order[k];
        if (k < n - s) {
            port_free = std::max(ready[child], port_free) + t_c;
            if (mask) mask[child] = 0;
        } else if (mask) {
            mask[child] = 1;
        }
    }
    return port_free;
}

}  // namespace

double simulate_iteration(const Tree &tree, int s, const std::vector<int64_t> &rows, const LatencyParams &p, uint64_t seed,
                          int64_t iteration, uint8_t *mask, double *ready_out)
{
    const int n = tree.n, L = tree.L;
    const int32_t N = tree.N;
    std::vector<double> ready(N);
    for (int32_t k = 0; k < N; ++k) {
        const double u = static_cast<double>(splitmix64_at(seed, static_cast<uint64_t>(iteration) * N + k) >> 11) * 0x1.0p-53;
        const double d = static_cast<double>(rows[k]);
        ready[k] = p.a * d + (d / p.mu) * (-std::log1p(-u));       // own computation; leaves send as soon as it ends
    }
    for (int l = L - 1; l >= 1; --l)
        for (int32_t node = tree.level_offset[l]; node < tree.level_offset[l + 1]; ++node) {
            const double decode = receive(ready.data(), tree.first_child(node), n, s, p.t_c, mask);
            ready[node] = std::max(ready[node], decode);
        }
    const double total = receive(ready.data(), 0, n, s, p.t_c, mask);
    if (ready_out) std::copy(ready.begin(), ready.end(), ready_out);
    return total;
}

}  // namespace cr

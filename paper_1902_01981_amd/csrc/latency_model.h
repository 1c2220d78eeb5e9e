// Run-time model of one CodedReduce iteration (Section III-C): shifted-exponential computation times, eq. (5), and single-port
// reception with a fixed time per message.  Host only.
#pragma once
#include <cstdint>
#include <vector>

#include "tree_plan.h"

namespace cr {

struct LatencyParams {
    double a;     // shift per data point (seconds per point)
    double mu;    // exponential rate parameter: a worker with d_i points has rate mu / d_i
    double t_c;   // time to receive one message
};

// Simulates iteration number `iteration`: node k computes for a*rows[k] + (rows[k]/mu) * (-ln(1-u_k)), u_k = top 53 bits of
// splitmix64 output number iteration*N + k of the stream started at `seed`.  A parent serves its children in order of readiness,
// one transfer of t_c at a time, and decodes after n-s transfers; the s children not received are marked in `mask` (N bytes).
// ready[k] = time node k's message is ready to send.  Returns the time at which the master has decoded.
double simulate_iteration(const Tree &tree, int s, const std::vector<int64_t> &rows, const LatencyParams &p, uint64_t seed,
                          int64_t iteration, uint8_t *mask, double *ready);

}  // namespace cr

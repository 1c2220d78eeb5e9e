// Gradient-coding matrices for one sibling group (Section II-C): encoding matrix B and decode rows a_f.
#pragma once
#include <cstdint>
#include <vector>

namespace cr {

struct GcCode {
    int n = 0, s = 0;
    std::vector<double> B;   // n x n row-major; s+1 non-zeros per row and per column, unit 2-norm rows
    double gamma = 0.0;      // max_f sum_i |a_fi| ||b_i||_2 / sqrt(n)
    int candidate = -1;      // winning candidate of the search; -1 when B was supplied; -2 for the fractional-repetition design
};

// Number of straggler sets of size exactly s, C(n,s); returns -1 if it exceeds `limit`.
int64_t num_straggler_sets(int n, int s, int64_t limit);

// Candidate count of the search for (n,s): min(2048, max(16, 2^20 / C(n,s))).
int search_candidates(int n, int s);

// Best-of-K design: candidate c draws H (s x n, rows summing to zero) from the splitmix64 stream seeded with `seed`
// (entry (r,j), j < n-1, uses counter (c*s + r)*(n-1) + j, mapped to [-1,1)); rows of B solve H b_i^T = 0 on the
// cyclic support {i..i+s} mod n.  Keeps the candidate with the smallest gamma.  If that gamma is too large for fp32 messages over L
// levels (gamma^L > 256) and s+1 divides n, the fractional-repetition design is taken instead when its gamma is smaller.
// Returns false if no candidate is usable.
bool design_code(int n, int s, int L, uint64_t seed, GcCode &out);

// Adopt a caller-supplied B: checks s+1 non-zeros per row and per column and that every survivor set decodes; computes gamma.
bool adopt_code(int n, int s, const double *B, GcCode &out);

// Decode row for the straggler set given as a bitmask over the n children (exactly s bits set):
// zeros on the stragglers, a B = 1 on the survivors.  Returns false if the system is inconsistent.
bool decode_row(const GcCode &code, uint64_t straggler_bits, double *a);

// f-th straggler set (lexicographic order of the sorted index tuples) as a bitmask.
uint64_t straggler_set_by_rank(int n, int s, int64_t f);

}  // namespace cr

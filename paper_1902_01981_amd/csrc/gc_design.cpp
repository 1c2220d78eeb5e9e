// Host-side design of the gradient-coding matrices (Section II-C).  The paper cites the construction without
// restating it; what binds is the property set: cyclic support with s+1 entries per row, and for every straggler
// set of size s a row a_f, zero on that set, with a_f B = (1,...,1).
#include "gc_design.h"

#include <algorithm>
#include <cmath>
#include <limits>

namespace cr {

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

// Output number `counter` of the splitmix64 stream started at `seed`.
uint64_t splitmix64_at(uint64_t seed, uint64_t counter)
{
    uint64_t z = seed + (counter + 1) * kGolden;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

double uniform_pm1(uint64_t seed, uint64_t counter)
{
    return static_cast<double>(splitmix64_at(seed, counter) >> 11) * 0x1.0p-53 * 2.0 - 1.0;
}

// Solve the k x k system M x = rhs in place (partial pivoting).  M row-major.
bool solve_square(std::vector<double> &M, std::vector<double> &rhs, int k)
{
    for (int c = 0; c < k; ++c) {
        int p = c;
        for (int r = c + 1; r < k; ++r)
            if (std::fabs(M[r * k + c]) > std::fabs(M[p * k + c])) p = r;
        if (M[p * k + c] == 0.0) return false;
        if (p != c) {
            for (int j = 0; j < k; ++j) std::swap(M[p * k + j], M[c * k + j]);
            std::swap(rhs[p], rhs[c]);
        }
        for (int r = c + 1; r < k; ++r) {
            double f = M[r * k + c] / M[c * k + c];
            if (f == 0.0) continue;
            for (int j = c; j < k; ++j) M[r * k + j] -= f * M[c * k + j];
            rhs[r] -= f * rhs[c];
        }
    }
    for (int c = k - 1; c >= 0; --c) {
        double v = rhs[c];
        for (int j = c + 1; j < k; ++j) v -= M[c * k + j] * rhs[j];
        rhs[c] = v / M[c * k + c];
    }
    return true;
}

// Solution of the consistent rows x cols system M x = rhs (rows >= cols) by Householder QR with column pivoting.  Columns that
// depend on earlier pivots (replicated workers) get a zero coefficient: a basic solution.  M row-major, destroyed.
bool least_squares(std::vector<double> &M, std::vector<double> &rhs, int rows, int cols, double *x)
{
    std::vector<int> perm(cols);
    for (int c = 0; c < cols; ++c) perm[c] = c;
    double scale = 0.0;
    for (double v : M) scale = std::max(scale, std::fabs(v));
    if (!(scale > 0.0)) return false;
    int rank = 0;
    for (int c = 0; c < cols; ++c) {
        // pivot: the remaining column with the largest norm below row c
        int best = c;
        double best_norm = -1.0;
        for (int j = c; j < cols; ++j) {
            double nj = 0.0;
            for (int r = c; r < rows; ++r) nj += M[r * cols + j] * M[r * cols + j];
            if (nj > best_norm) { best_norm = nj; best = j; }
        }
        if (!(std::sqrt(best_norm) > 1e-12 * scale * rows)) break;
        if (best != c) {
            for (int r = 0; r < rows; ++r) std::swap(M[r * cols + best], M[r * cols + c]);
            std::swap(perm[best], perm[c]);
        }
        const double norm = std::sqrt(best_norm);
        const double alpha = M[c * cols + c] > 0 ? -norm : norm;
        // v = column - alpha e_c, stored in place; beta = 2 / (v.v)
        const double v0 = M[c * cols + c] - alpha;
        double vv = v0 * v0;
        for (int r = c + 1; r < rows; ++r) vv += M[r * cols + c] * M[r * cols + c];
        if (vv > 0.0) {
            const double beta = 2.0 / vv;
            for (int j = c + 1; j < cols; ++j) {
                double dot = v0 * M[c * cols + j];
                for (int r = c + 1; r < rows; ++r) dot += M[r * cols + c] * M[r * cols + j];
                dot *= beta;
                M[c * cols + j] -= dot * v0;
                for (int r = c + 1; r < rows; ++r) M[r * cols + j] -= dot * M[r * cols + c];
            }
            double dot = v0 * rhs[c];
            for (int r = c + 1; r < rows; ++r) dot += M[r * cols + c] * rhs[r];
            dot *= beta;
            rhs[c] -= dot * v0;
            for (int r = c + 1; r < rows; ++r) rhs[r] -= dot * M[r * cols + c];
        }
        M[c * cols + c] = alpha;
        rank = c + 1;
    }
    std::vector<double> z(cols, 0.0);
    for (int c = rank - 1; c >= 0; --c) {
        double v = rhs[c];
        for (int j = c + 1; j < rank; ++j) v -= M[c * cols + j] * z[j];
        z[c] = v / M[c * cols + c];
    }
    for (int c = 0; c < cols; ++c) x[perm[c]] = z[c];
    return rank > 0;
}

// Rows of B from H (s x n): b_i(i) = 1, the other s support entries solve H[:, others] x = -H[:, i]; unit 2-norm.
bool encoding_from_H(const std::vector<double> &H, int n, int s, std::vector<double> &B)
{
    B.assign(static_cast<size_t>(n) * n, 0.0);
    std::vector<double> M(static_cast<size_t>(s) * s), rhs(s);
    for (int i = 0; i < n; ++i) {
        B[i * n + i] = 1.0;
        if (s > 0) {
            for (int r = 0; r < s; ++r) {
                for (int t = 1; t <= s; ++t) M[r * s + (t - 1)] = H[r * n + (i + t) % n];
                rhs[r] = -H[r * n + i];
            }
            if (!solve_square(M, rhs, s)) return false;
            for (int t = 1; t <= s; ++t) B[i * n + (i + t) % n] = rhs[t - 1];
        }
        double norm = 0.0;
        for (int j = 0; j < n; ++j) norm += B[i * n + j] * B[i * n + j];
        norm = std::sqrt(norm);
        if (!std::isfinite(norm) || norm == 0.0) return false;
        for (int j = 0; j < n; ++j) B[i * n + j] /= norm;
    }
    return true;
}

bool decode_row_impl(const double *B, int n, int s, uint64_t bits, double *a)
{
    int surv[64], ns = 0;
    for (int i = 0; i < n; ++i)
        if (!((bits >> i) & 1ull)) surv[ns++] = i;
    if (ns != n - s) return false;
    std::vector<double> M(static_cast<size_t>(n) * ns), rhs(n, 1.0), x(ns);
    for (int k = 0; k < n; ++k)
        for (int c = 0; c < ns; ++c) M[k * ns + c] = B[surv[c] * n + k];   // B_I^T
    if (!least_squares(M, rhs, n, ns, x.data())) return false;
    for (int i = 0; i < n; ++i) a[i] = 0.0;
    for (int c = 0; c < ns; ++c) a[surv[c]] = x[c];
    for (int k = 0; k < n; ++k) {                                          // a B = 1 must hold, not just in the least-squares sense
        double v = 0.0;
        for (int i = 0; i < n; ++i) v += a[i] * B[i * n + k];
        if (!(std::fabs(v - 1.0) <= 1e-10)) return false;
    }
    return true;
}

// gamma over all straggler sets; +inf if some set does not decode.
double amplification(const double *B, int n, int s)
{
    double norms[64];
    for (int i = 0; i < n; ++i) {
        double v = 0.0;
        for (int j = 0; j < n; ++j) v += B[i * n + j] * B[i * n + j];
        norms[i] = std::sqrt(v);
    }
    const int64_t F = num_straggler_sets(n, s, int64_t(1) << 20);
    double worst = 0.0, a[64];
    for (int64_t f = 0; f < F; ++f) {
        if (!decode_row_impl(B, n, s, straggler_set_by_rank(n, s, f), a)) return std::numeric_limits<double>::infinity();
        double v = 0.0;
        for (int i = 0; i < n; ++i) v += std::fabs(a[i]) * norms[i];
        worst = std::max(worst, v);
    }
    return worst / std::sqrt(static_cast<double>(n));
}

}  // namespace

int64_t num_straggler_sets(int n, int s, int64_t limit)
{
    if (s < 0 || s > n) return 0;
    int k = std::min(s, n - s);
    __int128 c = 1;
    for (int i = 1; i <= k; ++i) {
        c = c * (n - k + i) / i;
        if (c > limit) return -1;
    }
    return static_cast<int64_t>(c);
}

int search_candidates(int n, int s)
{
    int64_t F = num_straggler_sets(n, s, int64_t(1) << 20);
    if (F < 1) return 16;
    int64_t k = (int64_t(1) << 20) / F;
    return static_cast<int>(std::min<int64_t>(2048, std::max<int64_t>(16, k)));
}

uint64_t straggler_set_by_rank(int n, int s, int64_t f)
{
    // unrank the f-th s-subset of {0..n-1} in lexicographic order of its sorted elements
    uint64_t bits = 0;
    int next = 0;
    for (int left = s; left > 0; --left) {
        for (int v = next; v < n; ++v) {
            int64_t cnt = num_straggler_sets(n - v - 1, left - 1, std::numeric_limits<int64_t>::max() / 2);
            if (left - 1 == 0) cnt = 1;
            if (f < cnt) { bits |= 1ull << v; next = v + 1; break; }
            f -= cnt;
        }
    }
    return bits;
}

// Fractional repetition: s+1 groups of n/(s+1) workers; worker j of every group holds the j-th window of s+1 partitions
// (all entries equal, unit 2-norm).  s stragglers cannot break all s+1 groups, and the members of an intact group sum to the whole.
static void fractional_repetition(int n, int s, std::vector<double> &B)
{
    const int per_group = n / (s + 1);
    B.assign(static_cast<size_t>(n) * n, 0.0);
    const double v = 1.0 / std::sqrt(static_cast<double>(s + 1));
    for (int g = 0; g <= s; ++g)
        for (int j = 0; j < per_group; ++j)
            for (int t = 0; t <= s; ++t) B[(g * per_group + j) * n + j * (s + 1) + t] = v;
}

bool design_code(int n, int s, int L, uint64_t seed, GcCode &out)
{
    out.n = n; out.s = s;
    if (s == 0) {
        out.B.assign(static_cast<size_t>(n) * n, 0.0);
        for (int i = 0; i < n; ++i) out.B[i * n + i] = 1.0;
        out.gamma = amplification(out.B.data(), n, 0);
        out.candidate = 0;
        return true;
    }
    if (s == n - 1) {
        // every worker holds every partition (null(H) is spanned by the all-ones vector): all candidates coincide
        out.B.assign(static_cast<size_t>(n) * n, 1.0 / std::sqrt(static_cast<double>(n)));
        out.gamma = amplification(out.B.data(), n, s);
        out.candidate = 0;
        return true;
    }
    const int K = search_candidates(n, s);
    std::vector<double> H(static_cast<size_t>(s) * n), B;
    double best = std::numeric_limits<double>::infinity();
    for (int c = 0; c < K; ++c) {
        for (int r = 0; r < s; ++r) {
            // the last column makes the row sum to zero; summed in index order with compensation so the value
            // does not depend on how the compiler reorders a plain loop
            double sum = 0.0, comp = 0.0;
            for (int j = 0; j < n - 1; ++j) {
                double v = uniform_pm1(seed, (static_cast<uint64_t>(c) * s + r) * (n - 1) + j);
                H[r * n + j] = v;
                double yv = v - comp, t = sum + yv;
                comp = (t - sum) - yv;
                sum = t;
            }
            H[r * n + n - 1] = -sum;
        }
        if (!encoding_from_H(H, n, s, B)) continue;
        double g = amplification(B.data(), n, s);
        if (g < best) { best = g; out.B = B; out.candidate = c; }
    }
    // Fall-back for badly conditioned cyclic codes: when fp32 rounding amplified over L levels, gamma^L 2^-24, would exceed 2^-16
    // and s+1 divides n, the fractional-repetition design (0/1 decode rows) is used instead if its gamma is smaller.
    if (n % (s + 1) == 0 && !(std::pow(best, L) <= 256.0)) {
        std::vector<double> FR;
        fractional_repetition(n, s, FR);
        const double g = amplification(FR.data(), n, s);
        if (g < best) { best = g; out.B = FR; out.candidate = -2; }
    }
    if (!std::isfinite(best)) return false;
    out.gamma = best;
    return true;
}

bool adopt_code(int n, int s, const double *B, GcCode &out)
{
    out.n = n; out.s = s; out.candidate = -1;
    // Section II-C: every worker holds s+1 partitions and every partition sits in s+1 workers
    std::vector<int> per_col(n, 0);
    for (int i = 0; i < n; ++i) {
        int per_row = 0;
        for (int j = 0; j < n; ++j) {
            const double v = B[i * n + j];
            if (!std::isfinite(v)) return false;
            if (v != 0.0) { ++per_row; ++per_col[j]; }
        }
        if (per_row != s + 1) return false;
    }
    for (int j = 0; j < n; ++j)
        if (per_col[j] != s + 1) return false;
    out.B.assign(B, B + static_cast<size_t>(n) * n);
    out.gamma = amplification(B, n, s);
    return std::isfinite(out.gamma);
}

bool decode_row(const GcCode &code, uint64_t straggler_bits, double *a)
{
    return decode_row_impl(code.B.data(), code.n, code.s, straggler_bits, a);
}

}  // namespace cr

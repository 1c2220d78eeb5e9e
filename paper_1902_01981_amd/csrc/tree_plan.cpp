// Host-side allocation of data to the tree (Section III-A CR.Allocate; Algorithms 1 and 2).
#include "tree_plan.h"

#include <algorithm>

namespace cr {

bool make_tree(int n, int L, Tree &t)
{
    t.n = n; t.L = L;
    t.level_offset.assign(L + 2, 0);
    int64_t off = 0, width = 1;
    for (int l = 1; l <= L; ++l) {
        width *= n;
        t.level_offset[l] = static_cast<int32_t>(off);
        off += width;
        if (off > (int64_t(1) << 24)) return false;
    }
    t.level_offset[L + 1] = static_cast<int32_t>(off);
    t.N = static_cast<int32_t>(off);
    return true;
}

int Tree::level_of(int32_t node) const
{
    int l = 1;
    while (node >= level_offset[l + 1]) ++l;
    return l;
}

int32_t Tree::parent_of(int32_t node) const
{
    int l = level_of(node);
    if (l == 1) return -1;
    return level_offset[l - 1] + (node - level_offset[l]) / n;
}

int32_t Tree::first_child(int32_t node) const
{
    int l = level_of(node);
    if (l == L) return -1;
    return level_offset[l + 1] + (node - level_offset[l]) * n;
}

int64_t own_count(int64_t size, int n, int L, int s, int l)
{
    if (l == L) return size;
    // Q = sum_{j=0}^{L-l} (n/(s+1))^j = P / D with D = (s+1)^(L-l), P = sum_j n^j (s+1)^(L-l-j)
    const int depth = L - l;
    __int128 D = 1, P = 0;
    for (int j = 0; j < depth; ++j) D *= (s + 1);
    __int128 npow = 1;
    for (int j = 0; j <= depth; ++j) {
        __int128 term = npow;
        for (int t = 0; t < depth - j; ++t) term *= (s + 1);
        P += term;
        npow *= n;
    }
    __int128 num = static_cast<__int128>(size) * D * 2 + P;    // floor(size*D/P + 1/2)
    return static_cast<int64_t>(num / (2 * P));
}

static int64_t set_size(const WeightedSet &W)
{
    int64_t v = 0;
    for (const Segment &g : W) v += g.row_end - g.row_begin;
    return v;
}

// positions [lo, hi) of W, appended to out with coefficients scaled by `scale`
static void take(const WeightedSet &W, int64_t lo, int64_t hi, double scale, WeightedSet &out)
{
    int64_t pos = 0;
    for (const Segment &g : W) {
        const int64_t len = g.row_end - g.row_begin;
        const int64_t a0 = std::max(lo, pos), a1 = std::min(hi, pos + len);
        if (a1 > a0) out.push_back({g.row_begin + (a0 - pos), g.row_begin + (a1 - pos), g.coef * scale});
        pos += len;
    }
}

std::vector<WeightedSet> comp_alloc(const WeightedSet &W, const double *B, int n)
{
    const int64_t size = set_size(W);
    std::vector<int64_t> cut(n + 1);
    for (int k = 0; k <= n; ++k) cut[k] = static_cast<int64_t>(static_cast<__int128>(size) * k / n);
    std::vector<WeightedSet> out(n);
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < n; ++k)
            if (B[i * n + k] != 0.0) take(W, cut[k], cut[k + 1], B[i * n + k], out[i]);
    return out;
}

void allocate(const Tree &t, int s, int64_t m, const double *B, std::vector<WeightedSet> &own, std::vector<Slab> &slabs)
{
    const int n = t.n, L = t.L;
    own.assign(t.N, {});
    std::vector<WeightedSet> rest(t.N);            // what a node hands down to its children
    WeightedSet whole{{0, m, 1.0}};
    for (int l = 1; l <= L; ++l) {
        const int32_t width = t.level_offset[l + 1] - t.level_offset[l];
        for (int32_t pi = 0; pi < width / n; ++pi) {
            const WeightedSet &src = (l == 1) ? whole : rest[t.level_offset[l - 1] + pi];
            std::vector<WeightedSet> sub = comp_alloc(src, B, n);
            for (int j = 0; j < n; ++j) {
                const int32_t node = t.level_offset[l] + pi * n + j;
                const int64_t size = set_size(sub[j]);
                const int64_t keep = own_count(size, n, L, s, l);
                take(sub[j], 0, keep, 1.0, own[node]);
                take(sub[j], keep, size, 1.0, rest[node]);
            }
        }
    }
    slabs.clear();
    for (int32_t node = 0; node < t.N; ++node)
        for (const Segment &g : own[node]) slabs.push_back({node, g.row_begin, g.row_end, g.coef});
}

void split_pieces(const std::vector<Slab> &slabs, int teams, std::vector<Piece> &pieces,
                  std::vector<int32_t> &slab_piece_begin, std::vector<int32_t> &team_piece_begin)
{
    int64_t visits = 0;
    for (const Slab &sl : slabs) visits += sl.row_end - sl.row_begin;
    pieces.clear();
    slab_piece_begin.assign(slabs.size() + 1, 0);
    team_piece_begin.assign(teams + 1, 0);
    size_t p = 0;           // current slab
    int64_t slab_start = 0; // visit index of the first row of slab p
    for (int tm = 0; tm < teams; ++tm) {
        int64_t lo = static_cast<int64_t>(static_cast<__int128>(visits) * tm / teams);
        const int64_t hi = static_cast<int64_t>(static_cast<__int128>(visits) * (tm + 1) / teams);
        team_piece_begin[tm] = static_cast<int32_t>(pieces.size());
        while (lo < hi) {
            while (slab_start + (slabs[p].row_end - slabs[p].row_begin) <= lo) {
                slab_start += slabs[p].row_end - slabs[p].row_begin;
                ++p;
                slab_piece_begin[p] = static_cast<int32_t>(pieces.size());
            }
            const int64_t slab_len = slabs[p].row_end - slabs[p].row_begin;
            const int64_t stop = std::min(hi, slab_start + slab_len);
            pieces.push_back({static_cast<int32_t>(p), tm, slabs[p].row_begin + (lo - slab_start), slabs[p].row_begin + (stop - slab_start)});
            lo = stop;
        }
    }
    team_piece_begin[teams] = static_cast<int32_t>(pieces.size());
    while (p < slabs.size()) { ++p; slab_piece_begin[p] = static_cast<int32_t>(pieces.size()); }
}

}  // namespace cr

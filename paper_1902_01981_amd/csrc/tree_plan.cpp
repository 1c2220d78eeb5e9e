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

static void index_slab_pieces(size_t num_slabs, Split &out)
{
    // row order inside a slab = increasing row_begin; a stable counting sort by slab keeps any order the caller set up
    std::vector<int32_t> order(out.pieces.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = static_cast<int32_t>(i);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (out.pieces[a].slab != out.pieces[b].slab) return out.pieces[a].slab < out.pieces[b].slab;
        return out.pieces[a].row_begin < out.pieces[b].row_begin;
    });
    out.slab_pieces = order;
    out.slab_piece_begin.assign(num_slabs + 1, 0);
    for (const Piece &pc : out.pieces) out.slab_piece_begin[pc.slab + 1] += 1;
    for (size_t q = 0; q < num_slabs; ++q) out.slab_piece_begin[q + 1] += out.slab_piece_begin[q];
}

void split_equal_ranges(const std::vector<Slab> &slabs, int teams, Split &out)
{
    int64_t visits = 0;
    for (const Slab &sl : slabs) visits += sl.row_end - sl.row_begin;
    out.pieces.clear();
    out.teams = teams;
    out.team_piece_begin.assign(teams + 1, 0);
    size_t p = 0;           // current slab
    int64_t slab_start = 0; // visit index of the first row of slab p
    for (int tm = 0; tm < teams; ++tm) {
        int64_t lo = static_cast<int64_t>(static_cast<__int128>(visits) * tm / teams);
        const int64_t hi = static_cast<int64_t>(static_cast<__int128>(visits) * (tm + 1) / teams);
        out.team_piece_begin[tm] = static_cast<int32_t>(out.pieces.size());
        while (lo < hi) {
            while (slab_start + (slabs[p].row_end - slabs[p].row_begin) <= lo) {
                slab_start += slabs[p].row_end - slabs[p].row_begin;
                ++p;
            }
            const int64_t slab_len = slabs[p].row_end - slabs[p].row_begin;
            const int64_t stop = std::min(hi, slab_start + slab_len);
            out.pieces.push_back({static_cast<int32_t>(p), tm, slabs[p].row_begin + (lo - slab_start), slabs[p].row_begin + (stop - slab_start)});
            lo = stop;
        }
    }
    out.team_piece_begin[teams] = static_cast<int32_t>(out.pieces.size());
    index_slab_pieces(slabs.size(), out);
}

namespace {
struct Unit { int64_t cell; int32_t slab; int64_t row_begin, row_end; };

// Cells that every holder holds whole: the row axis is first cut wherever any slab begins or ends (between two such cuts the set of
// holders does not change), then every stretch is cut into near-equal cells of at most cell_rows rows.  Units sorted by cell.
std::vector<Unit> whole_cell_units(const std::vector<Slab> &slabs, int64_t cell_rows)
{
    std::vector<Unit> units;
    std::vector<int64_t> cuts;
    cuts.reserve(2 * slabs.size());
    for (const Slab &sl : slabs) { cuts.push_back(sl.row_begin); cuts.push_back(sl.row_end); }
    std::sort(cuts.begin(), cuts.end());
    cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
    std::vector<int64_t> first_cell(cuts.size(), 0);     // index of the first cell of the stretch that starts at cuts[i]
    for (size_t i = 0; i + 1 < cuts.size(); ++i) first_cell[i + 1] = first_cell[i] + (cuts[i + 1] - cuts[i] + cell_rows - 1) / cell_rows;
    for (size_t q = 0; q < slabs.size(); ++q) {
        size_t i = static_cast<size_t>(std::lower_bound(cuts.begin(), cuts.end(), slabs[q].row_begin) - cuts.begin());
        for (; i + 1 < cuts.size() && cuts[i] < slabs[q].row_end; ++i) {
            const int64_t len = cuts[i + 1] - cuts[i];
            const int64_t parts = (len + cell_rows - 1) / cell_rows;
            for (int64_t c = 0; c < parts; ++c)
                units.push_back({first_cell[i] + c, static_cast<int32_t>(q), cuts[i] + static_cast<int64_t>(static_cast<__int128>(len) * c / parts),
                                 cuts[i] + static_cast<int64_t>(static_cast<__int128>(len) * (c + 1) / parts)});
        }
    }
    std::stable_sort(units.begin(), units.end(), [](const Unit &a, const Unit &b) { return a.cell < b.cell; });
    return units;
}
}  // namespace

void split_shared_queues(const std::vector<Slab> &slabs, int64_t cell_rows, int lanes, int teams_per_group, int slots_per_lane, Split &out)
{
    const std::vector<Unit> units = whole_cell_units(slabs, cell_rows);
    // an item = up to teams_per_group holders of one cell = the work of one workgroup for the length of that cell
    struct Item { size_t ub, ue; bool shared = false; };     // units [ub, ue); shared: the cell has other items too
    struct Cell { std::vector<Item> items; };
    std::vector<Cell> cells;
    size_t widest = 1;
    for (size_t i = 0; i < units.size();) {
        size_t k = i;
        while (k < units.size() && units[k].cell == units[i].cell) ++k;
        Cell c;
        for (size_t u = i; u < k; u += teams_per_group) c.items.push_back({u, std::min(k, u + teams_per_group), k - i > static_cast<size_t>(teams_per_group)});
        widest = std::max(widest, c.items.size());
        cells.push_back(std::move(c));
        i = k;
    }
    // A gang = `gang` workgroup slots of one L2 domain that work through the same sequence of rounds side by side.  A round holds
    // cells whose items fill at most the gang (one item per slot), so all workgroups that share a cell run it at the same time,
    // from the first round on.  Cells with more items than a domain has slots are spread over several rounds.
    const size_t gang = std::min(widest, static_cast<size_t>(slots_per_lane));
    const size_t gangs = static_cast<size_t>(lanes) * (slots_per_lane / gang);
    struct Round { std::vector<Item> slot; };                // slot[j] = the item of gang slot j (ub == ue: none)
    std::vector<Round> rounds;
    for (const Cell &c : cells)
        for (size_t first = 0; first < c.items.size(); first += gang) {
            const size_t count = std::min(gang, c.items.size() - first);
            if (rounds.empty() || rounds.back().slot.size() + count > gang) rounds.push_back({});
            for (size_t j = 0; j < count; ++j) rounds.back().slot.push_back(c.items[first + j]);
        }
    // round r goes to gang r mod gangs: consecutive cells land on different L2 domains and every gang gets the same number of rounds
    // to within one.  Gang g = (domain x = g mod lanes, number k = g / lanes) occupies workgroup ids x + lanes*(k*gang + j), j < gang.
    const size_t groups_all = static_cast<size_t>(lanes) * (slots_per_lane / gang) * gang;
    std::vector<std::vector<Item>> queue(groups_all);
    for (size_t r = 0; r < rounds.size(); ++r) {
        const size_t g = r % gangs, x = g % lanes, k = g / lanes;
        for (size_t j = 0; j < gang; ++j)
            queue[x + lanes * (k * gang + j)].push_back(j < rounds[r].slot.size() ? rounds[r].slot[j] : Item{0, 0, false});
    }
    size_t groups = groups_all;
    auto empty_queue = [&](const std::vector<Item> &q) { return std::all_of(q.begin(), q.end(), [](const Item &it) { return it.ub == it.ue; }); };
    while (groups > 0 && empty_queue(queue[groups - 1])) --groups;

    out = Split();
    out.teams = static_cast<int>(groups) * teams_per_group;
    out.team_piece_begin.assign(out.teams + 1, 0);
    out.group_item_begin.assign(groups + 1, 0);
    // pieces team-major (a team's pieces are contiguous, in the order it runs them); then the item table that points at them
    std::vector<std::vector<int32_t>> piece_of(groups);      // per group: items x teams_per_group, piece index or -1
    for (size_t g = 0; g < groups; ++g) {
        piece_of[g].assign(queue[g].size() * teams_per_group, -1);
        for (int t = 0; t < teams_per_group; ++t) {
            const int32_t team = static_cast<int32_t>(g) * teams_per_group + t;
            out.team_piece_begin[team] = static_cast<int32_t>(out.pieces.size());
            for (size_t i = 0; i < queue[g].size(); ++i) {
                const Item &it = queue[g][i];
                if (it.ub + t >= it.ue) continue;
                const Unit &u = units[it.ub + t];
                piece_of[g][i * teams_per_group + t] = static_cast<int32_t>(out.pieces.size());
                out.pieces.push_back({u.slab, team, u.row_begin, u.row_end, it.shared ? 1 : 0});
            }
        }
        int64_t busy = 0;
        for (const Item &it : queue[g])
            if (it.ub < it.ue) busy += units[it.ub].row_end - units[it.ub].row_begin + 4;     // + pipeline refill and the partial row, in rows
        out.makespan = std::max(out.makespan, busy);
    }
    out.team_piece_begin[out.teams] = static_cast<int32_t>(out.pieces.size());
    for (size_t g = 0; g < groups; ++g) {
        out.group_item_begin[g + 1] = out.group_item_begin[g] + static_cast<int32_t>(queue[g].size());
        out.item_pieces.insert(out.item_pieces.end(), piece_of[g].begin(), piece_of[g].end());
    }
    index_slab_pieces(slabs.size(), out);
}

void split_row_cells(const std::vector<Slab> &slabs, int64_t cell_rows, int lanes, int teams_per_block, Split &out)
{
    std::vector<Unit> units;
    for (size_t q = 0; q < slabs.size(); ++q) {
        int64_t b = slabs[q].row_begin;
        while (b < slabs[q].row_end) {
            const int64_t cell = b / cell_rows;
            const int64_t e = std::min(slabs[q].row_end, (cell + 1) * cell_rows);
            units.push_back({cell, static_cast<int32_t>(q), b, e});
            b = e;
        }
    }
    std::stable_sort(units.begin(), units.end(), [](const Unit &a, const Unit &b) { return a.cell < b.cell; });

    // Team order.  Workgroups are handed to the chip's `lanes` L2 domains round-robin by workgroup id, so the holders of one cell are
    // placed on workgroup ids that are congruent modulo `lanes`: inside each run of `lanes` consecutive non-empty cells, workgroup
    // number g*lanes + c carries holders g*tpb .. g*tpb+tpb-1 of cell c (tpb = teams per workgroup).  Slots without a holder become
    // empty teams (no pieces), which keeps the alignment.
    const Unit none{-1, -1, 0, 0};
    std::vector<Unit> order;
    order.reserve(units.size() + units.size() / 4);
    size_t i = 0;
    while (i < units.size()) {
        std::vector<std::pair<size_t, size_t>> cells;      // [begin, end) in units
        size_t j = i;
        while (j < units.size() && static_cast<int>(cells.size()) < lanes) {
            size_t k = j;
            while (k < units.size() && units[k].cell == units[j].cell) ++k;
            cells.push_back({j, k});
            j = k;
        }
        size_t deepest = 0;
        for (auto &c : cells) deepest = std::max(deepest, c.second - c.first);
        const bool last_run = (j == units.size());
        for (size_t g = 0; g * teams_per_block < deepest; ++g)
            for (size_t c = 0; c < static_cast<size_t>(lanes); ++c)
                for (int t = 0; t < teams_per_block; ++t) {
                    const size_t rank = g * teams_per_block + t;
                    if (c < cells.size() && cells[c].first + rank < cells[c].second) order.push_back(units[cells[c].first + rank]);
                    else if (lanes > 1 || teams_per_block > 1) order.push_back(none);
                }
        (void)last_run;
        i = j;
    }
    while (!order.empty() && order.back().slab < 0) order.pop_back();

    out.pieces.clear();
    out.teams = static_cast<int>(order.size());
    out.team_piece_begin.assign(order.size() + 1, 0);
    for (size_t u = 0; u < order.size(); ++u) {
        out.team_piece_begin[u] = static_cast<int32_t>(out.pieces.size());
        if (order[u].slab >= 0) out.pieces.push_back({order[u].slab, static_cast<int32_t>(u), order[u].row_begin, order[u].row_end});
    }
    out.team_piece_begin[order.size()] = static_cast<int32_t>(out.pieces.size());
    index_slab_pieces(slabs.size(), out);
}

}  // namespace cr

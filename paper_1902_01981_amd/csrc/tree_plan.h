// (n,L)-regular tree, CompAlloc (Algorithm 1) and CR.Allocate (Algorithm 2): which rows of X every worker holds, with which scalar.
#pragma once
#include <cstdint>
#include <vector>

namespace cr {

struct Segment {          // data points X[row_begin:row_end], each carrying the scalar coef (the paper's "b D")
    int64_t row_begin, row_end;
    double coef;
};
using WeightedSet = std::vector<Segment>;

struct Slab {             // one (worker, segment) pair: owns one d-float partial gradient
    int32_t node;
    int64_t row_begin, row_end;
    double coef;
};

struct Piece {            // a contiguous run of one slab's rows handled by one stage-1 team
    int32_t slab, team;
    int64_t row_begin, row_end;
    int32_t shared = 0;   // shared cells: 1 if other workgroups fetch the same rows at the same time (the cell has several items)
};

struct Tree {
    int n = 0, L = 0;
    int32_t N = 0;
    std::vector<int32_t> level_offset;   // level_offset[l] = id of node (l,0), l = 1..L; [L+1] = N
    int level_of(int32_t node) const;
    int32_t parent_of(int32_t node) const;            // -1 for level-1 nodes (their parent is the master)
    int32_t first_child(int32_t node) const;          // -1 for leaves
    int32_t group_of(int32_t node) const { return node / n; }   // level-order numbering: group g = ids [g n, (g+1) n)
};

bool make_tree(int n, int L, Tree &t);   // false if N would exceed 2^24

// own = round_half_up(size / sum_{j=0}^{L-l} (n/(s+1))^j); leaves keep everything
int64_t own_count(int64_t size, int n, int L, int s, int l);

// Algorithm 1 with k = n parts cut by position at floor(kappa |W| / n); child i gets, in ascending kappa, the parts with b_ik != 0
std::vector<WeightedSet> comp_alloc(const WeightedSet &W, const double *B, int n);

// CR.Allocate: per node, the segments it keeps.  slabs = node-major flattening.
void allocate(const Tree &t, int s, int64_t m, const double *B, std::vector<WeightedSet> &own, std::vector<Slab> &slabs);

// Stage-1 work split.  `pieces` are in execution order (team ids non-decreasing; team t runs pieces
// [team_piece_begin[t], team_piece_begin[t+1])); slab p is the sum of pieces slab_pieces[slab_piece_begin[p] .. slab_piece_begin[p+1]),
// listed in row order.
struct Split {
    std::vector<Piece> pieces;
    std::vector<int32_t> team_piece_begin;   // teams + 1
    std::vector<int32_t> slab_piece_begin;   // S + 1
    std::vector<int32_t> slab_pieces;        // one entry per piece
    int teams = 0;
    // shared queues only: workgroup g runs items [group_item_begin[g], group_item_begin[g+1]) in order; item i gives every team
    // of the workgroup its piece, item_pieces[i * teams_per_group + t], or -1
    std::vector<int32_t> group_item_begin;
    std::vector<int32_t> item_pieces;
    int64_t makespan = 0;                    // longest queue, in rows (with a few rows of start-up per item)
};

// Equal ranges: the slab-major row-visit space is cut into `teams` equal contiguous ranges, cut again at slab boundaries.
void split_equal_ranges(const std::vector<Slab> &slabs, int teams, Split &out);

// Row cells: every slab is cut on one global grid of `cell_rows` rows; a team runs at most one piece.  Teams are ordered by cell so
// that the holders of the same rows are launched together and stream the same addresses at the same time (all but the first of them
// are then served by the L2 cache instead of HBM).  `lanes` = number of L2 domains workgroups are dealt to round-robin,
// `teams_per_block` = teams in one workgroup: the holders of a cell go to workgroup ids congruent modulo `lanes`.
void split_row_cells(const std::vector<Slab> &slabs, int64_t cell_rows, int lanes, int teams_per_block, Split &out);

// Shared queues: cells are laid inside the stretches between slab boundaries (at most `cell_rows` rows, near-equal), so that every
// holder of a cell holds all of it.  Up to `teams_per_group` holders of a cell form an item, the work of one workgroup; there are
// lanes * slots_per_lane workgroup slots (one per compute unit), each with a queue of items.  All items of a cell sit at the same
// position of the queues of neighbouring slots of one L2 domain, so they run side by side from the start of the launch.
void split_shared_queues(const std::vector<Slab> &slabs, int64_t cell_rows, int lanes, int teams_per_group, int slots_per_lane, Split &out);

}  // namespace cr

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

// Stage-1 split of the slab-major row-visit space into `teams` equal ranges, cut again at slab boundaries.
// slab_piece_begin has S+1 entries, team_piece_begin teams+1 entries.
void split_pieces(const std::vector<Slab> &slabs, int teams, std::vector<Piece> &pieces,
                  std::vector<int32_t> &slab_piece_begin, std::vector<int32_t> &team_piece_begin);

}  // namespace cr

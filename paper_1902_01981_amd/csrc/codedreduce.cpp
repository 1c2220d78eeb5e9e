// C-ABI boundary of the CodedReduce hot path: plan (host), workspace binding, and the three stages of one iteration.
#include "codedreduce.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "gc_design.h"
#include "kernels.h"
#include "latency_model.h"
#include "tree_plan.h"

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string &msg)
{
    g_last_error = msg;
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(CR_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define CR_HIP(call)                                        \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) return hip_fail(e_, #call);   \
    } while (0)

constexpr uint64_t kDefaultSeed = 190201981ull;
constexpr int kProgramSlots = 16;     // encode programs the workspace holds at once: one host-to-device copy serves that many steps
constexpr int kStagingHalves = 2;     // pinned staging is two such batches, so the host fills one while the other is being copied
constexpr size_t kMaxSamples = size_t(1) << 16;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct TimedLaunch {
    int kernel;
    hipEvent_t start, stop;
};

}  // namespace

struct cr_plan_s {
    // problem
    int L = 0, n = 0, s = 0, model = 0, x_dtype = 0;
    int64_t m = 0, d = 0;
    cr::Tree tree;
    cr::GcCode code;
    std::vector<cr::WeightedSet> own;
    std::vector<cr::Slab> slabs;
    std::vector<int32_t> node_slab_begin;          // N+1
    int64_t row_visits = 0, min_rows = 0, max_rows = 0;
    mutable std::unordered_map<uint64_t, std::vector<double>> row_cache;   // padded straggler bitmask -> decode row

    // stage-1 split
    const cr::Stage1Variant *variant = nullptr;        // the stage-1 kernel in use (nullptr: two-pass path for very wide rows)
    const cr::Stage1Variant *variant_regs = nullptr, *variant_staged = nullptr;   // what exists for (x_dtype, d)
    bool rows_as_buffers = false;    // every row starts on a 4-byte boundary and every piece has fewer than 2^31 bytes
    int split_kind = -1;                            // -1: choose from the device when the workspace is sized
    int64_t split_value = 0;
    int split_kind_used = -1;                       // what ensure_split settled on
    int64_t split_value_used = 0;
    int l2_domains = 0, unit_slots = 0;             // what the split was laid out for (0 until it is fixed)
    int l2_sharing = -1;                            // 1 / 0: workgroup ids congruent modulo l2_domains were seen (not) to share a die; -1: not checked
    cr::Split split;

    // device binding
    bool bound = false;
    hipStream_t stream = nullptr;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    cr::DevPiece *d_pieces = nullptr;
    int32_t *d_team_piece_begin = nullptr, *d_slab_piece_begin = nullptr, *d_slab_pieces = nullptr;
    int32_t *d_group_item_begin = nullptr, *d_item_pieces = nullptr;   // shared queues only
    uint32_t *d_placement = nullptr;               // kPlacementSlots words: where the workgroups of a probe launch ran
    char *d_program = nullptr;                     // kProgramSlots encode programs (each with its root decode terms)
    size_t program_bytes = 0;                      // size of one
    float *d_partial = nullptr, *d_G = nullptr, *d_M = nullptr, *d_residuals = nullptr;   // residuals: wide-row path only
    const float *G_src = nullptr;                  // slabs the encode reads: d_G or the caller's buffer
    char *h_staging = nullptr;                     // pinned, kStagingHalves * kProgramSlots * program_bytes
    hipEvent_t staging_done[kStagingHalves] = {};
    bool staging_used[kStagingHalves] = {};
    int staging_next = 0;
    int dec_slot = 0;                              // program slot whose decode terms cr_decode_root uses
    // layout of the program block (offsets in bytes, fixed per plan)
    size_t off_slab = 0, off_level = 0, off_row = 0, off_coef = 0, off_acoef = 0, off_sub = 0, off_dec = 0;
    size_t max_terms = 0;
    int num_dec_terms = 0;

    bool have_grads = false, have_messages = false;
    std::vector<char> static_program;              // host copy of the encode program of cr_aggregate_static (ordinary memory)

    // timing
    unsigned profiling = 0;                         // bit k: launches of kernel id k are bracketed by events
    std::vector<TimedLaunch> timed;
    std::vector<hipEvent_t> event_pool;
    double total_ms[CR_K_COUNT] = {};
    int64_t launches[CR_K_COUNT] = {}, bytes_sum[CR_K_COUNT] = {}, bytes_last[CR_K_COUNT] = {};
    std::vector<float> samples[CR_K_COUNT];         // duration of every timed launch since the totals were last cleared (bounded)
};

namespace {

int64_t elem_size(const cr_plan_t *p) { return p->x_dtype == CR_BF16 ? 2 : 4; }
constexpr int64_t kStreamFromBytes = int64_t(1) << 30;      // four times the last-level cache: nothing of X survives an iteration

// decode row for one group under rule "pad with the highest-index survivors"; returns CR_E_UNDECODABLE if more than s flags are set
int group_decode_row(const cr_plan_t *p, const uint8_t *flags, const double **row)
{
    uint64_t bits = 0;
    int cnt = 0;
    for (int j = 0; j < p->n; ++j)
        if (flags[j]) { bits |= 1ull << j; ++cnt; }
    if (cnt > p->s) return CR_E_UNDECODABLE;
    for (int j = p->n - 1; cnt < p->s; --j)
        if (!((bits >> j) & 1ull)) { bits |= 1ull << j; ++cnt; }
    auto it = p->row_cache.find(bits);
    if (it == p->row_cache.end()) {
        std::vector<double> a(p->n);
        if (!cr::decode_row(p->code, bits, a.data())) return fail(CR_E_INVAL, "decode row: survivor system is inconsistent");
        it = p->row_cache.emplace(bits, std::move(a)).first;
    }
    *row = it->second.data();
    return CR_OK;
}

// MI355X has 8 accelerator dies (XCDs), each with its own L2; workgroups are dealt to them round-robin by workgroup id.  The count
// is asked of the current device; without one (planning on a host without a GPU) MI355X's 8 is assumed.  Whether congruent workgroup
// ids really share a die is checked on the device when a workspace is bound (see check_l2_sharing).
constexpr int kDefaultL2Domains = 8, kDefaultUnits = 256;
constexpr int kPlacementSlots = 1024;

int query_l2_domains()
{
    int dev = 0, xccs = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&xccs, hipDeviceAttributeNumberOfXccs, dev) == hipSuccess && xccs >= 1 && xccs <= 64)
        return xccs;
    (void)hipGetLastError();
    return kDefaultL2Domains;
}

// Workgroup slots of a staged kernel: one per compute unit of the current device (a multiple of the L2 domains; MI355X's 256
// without a device).  Rows of at most 8 KB get two per unit where registers and LDS let two workgroups stay resident: their steps
// are short, and the second workgroup fills the gaps around the first one's barriers (measured +10 to +16 % at 2048 columns;
// longer rows gain nothing).
int unit_slots(const cr::Stage1Variant *v, int64_t row_bytes, int64_t d, int domains)
{
    int dev = 0, cus = 0, resident = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus >= domains) {
        int slots = cus / domains * domains;
        if (v && row_bytes <= 8192 && cr::prepare_stage1(*v, d) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, v->fn[0], v->block(), v->lds_bytes(d)) == hipSuccess && resident >= 2)
            slots *= 2;
        (void)hipGetLastError();
        return slots;
    }
    (void)hipGetLastError();
    return kDefaultUnits / domains * domains;
}

int ensure_split(cr_plan_t *p)
{
    if (!p->split.pieces.empty() || p->model == CR_AGGREGATE_ONLY) return CR_OK;
    int kind = p->split_kind;
    int64_t value = p->split_value;
    p->variant = p->variant_regs;
    const int domains = query_l2_domains();
    p->l2_domains = domains;
    p->unit_slots = 0;
    p->l2_sharing = -1;
    if (kind < 0 && p->s == 0) {
        // no redundancy (every row has one holder): nothing to share, so one contiguous range per resident workgroup streams best
        int dev = 0, cus = 0, per_cu = 0;
        int slots = 2 * 256;                                // MI355X: 256 CUs, two resident workgroups each; refined if a device is present
        if (p->variant && hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, p->variant->fn[0], p->variant->block(), 0) == hipSuccess && cus > 0 && per_cu > 0)
            slots = cus * per_cu;
        else
            (void)hipGetLastError();                        // no device: keep the default and clear the error
        kind = CR_SPLIT_EQUAL_RANGES;
        value = static_cast<int64_t>(slots) * (p->variant ? p->variant->teams_per_block() : 1);
    }
    // small problems (under 16 rows per compute unit and workgroup) do not repay the staged kernel's start-up: row cells below
    if (kind < 0 && p->variant_staged && p->row_visits / p->variant_staged->teams_per_block() >= 256 * 16) {
        // Rows staged through LDS: one workgroup per compute unit, each with a queue of cells (see split_shared_queues); the
        // launch lasts as long as the longest queue.  Take the cell height, 16 to 1024 rows in steps of 8, that makes it
        // shortest; ties go to the taller cell (fewer partial rows).
        kind = CR_SPLIT_SHARED_CELLS;
        const int tpb = p->variant_staged->teams_per_block();
        const int slots = unit_slots(p->variant_staged, p->d * elem_size(p), p->d, domains);
        value = 512;
        if (p->row_visits / tpb / 64 <= (int64_t(1) << 16)) {       // with longer queues than that the last round no longer matters
            int64_t best = -1;
            cr::Split trial;
            for (int64_t c = 16; c <= 1024; c += 8) {
                cr::split_shared_queues(p->slabs, c, domains, tpb, slots / domains, trial);
                if (best < 0 || trial.makespan <= best) { best = trial.makespan; value = c; }
            }
        }
    }
    if (kind < 0) {
        // default: row cells of about 2 MB of X, between 96 and 512 rows, a multiple of 32.  Long enough that the d-float partial
        // row each piece writes is about a percent of what it reads, short enough that the holders of a cell stay in step and
        // that the last cells do not leave the chip half empty (measured on configurations 2, 3 and 5).
        kind = CR_SPLIT_ROW_CELLS;
        const int64_t row_bytes = p->d * elem_size(p);
        value = std::min<int64_t>(512, std::max<int64_t>(96, ((int64_t(2) << 20) / row_bytes + 16) / 32 * 32));
        // small problems: shorter cells, so that there are a few thousand pieces to spread over the chip
        value = std::min<int64_t>(value, std::max<int64_t>(16, (p->row_visits / 2048 + 15) / 16 * 16));
    }
    if (kind == CR_SPLIT_SHARED_CELLS) {
        if (!p->variant_staged) return fail(CR_E_INVAL, "no kernel stages rows of this width and type through LDS");
        p->variant = p->variant_staged;
    }
    const int teams_per_block = p->variant ? p->variant->teams_per_block() : 1;     // wide rows: one workgroup per piece
    p->split_kind_used = kind;
    p->split_value_used = value;
    if (kind == CR_SPLIT_SHARED_CELLS) {
        if (p->row_visits / value + 2 * static_cast<int64_t>(p->slabs.size()) > (int64_t(1) << 26)) return fail(CR_E_INVAL, "too many row cells");
        p->unit_slots = unit_slots(p->variant, p->d * elem_size(p), p->d, domains);
        cr::split_shared_queues(p->slabs, value, domains, teams_per_block, p->unit_slots / domains, p->split);
        // what the staged kernel relies on: every piece of an item covers the same rows
        const cr::Split &sp = p->split;
        for (size_t it = 0; it * teams_per_block < sp.item_pieces.size(); ++it) {
            const cr::Piece *first = nullptr;
            for (int t = 0; t < teams_per_block; ++t) {
                const int32_t pi = sp.item_pieces[it * teams_per_block + t];
                if (pi < 0) continue;
                const cr::Piece &pc = sp.pieces[pi];
                if (first && (first->row_begin != pc.row_begin || first->row_end != pc.row_end)) {
                    p->split = cr::Split();
                    return fail(CR_E_STATE, "shared cells: the teams of a workgroup do not hold the same rows");
                }
                if (!first) first = &pc;
            }
        }
    } else if (kind == CR_SPLIT_ROW_CELLS) {
        if (p->row_visits / value + static_cast<int64_t>(p->slabs.size()) > (int64_t(1) << 26)) return fail(CR_E_INVAL, "too many row cells");
        cr::split_row_cells(p->slabs, value, domains, teams_per_block, p->split);
        if (!p->variant) {                                  // the wide-row kernels index pieces directly: no empty teams
            cr::Split compact;
            cr::split_row_cells(p->slabs, value, 1, 1, compact);
            p->split = compact;
        }
    } else {
        const int teams = static_cast<int>(std::min<int64_t>(value, std::max<int64_t>(1, p->row_visits)));
        cr::split_equal_ranges(p->slabs, teams, p->split);
    }
    return CR_OK;
}

void compute_layout(cr_plan_t *p, size_t *total)
{
    const size_t S = p->slabs.size(), N = p->tree.N, P = p->split.pieces.size();
    // worst case: one term per slab plus one dummy per node, each sub-program padded to the unroll
    p->max_terms = align_up(S + N + static_cast<size_t>(p->n) * cr::kEncodeUnroll, cr::kEncodeUnroll);
    size_t off = 0;
    p->off_slab = off;  off = align_up(off + p->max_terms * sizeof(int32_t), 256);
    p->off_level = off; off = align_up(off + p->max_terms * sizeof(int32_t), 256);
    p->off_row = off;   off = align_up(off + p->max_terms * sizeof(int32_t), 256);
    p->off_coef = off;  off = align_up(off + p->max_terms * sizeof(double), 256);
    p->off_acoef = off; off = align_up(off + p->max_terms * sizeof(double), 256);
    p->off_sub = off;   off = align_up(off + 2 * static_cast<size_t>(p->n) * sizeof(int32_t), 256);   // begin and end of every sub-program
    p->off_dec = off;   off = align_up(off + p->n * sizeof(cr::DecTerm), 256);
    p->program_bytes = off;

    size_t w = 0;
    w = align_up(w + P * sizeof(cr::DevPiece), 256);
    w = align_up(w + (p->split.teams + 1) * sizeof(int32_t), 256);
    w = align_up(w + (S + 1) * sizeof(int32_t), 256);
    w = align_up(w + P * sizeof(int32_t), 256);
    w = align_up(w + p->split.group_item_begin.size() * sizeof(int32_t), 256);
    w = align_up(w + p->split.item_pieces.size() * sizeof(int32_t), 256);
    w = align_up(w + kPlacementSlots * sizeof(uint32_t), 256);
    w = align_up(w + kProgramSlots * p->program_bytes, 256);
    const size_t row = static_cast<size_t>(p->d) * sizeof(float);
    if (p->model != CR_AGGREGATE_ONLY) {
        w = align_up(w + P * row, 256);
        w = align_up(w + S * row, 256);
        if (!p->variant) w = align_up(w + static_cast<size_t>(p->row_visits) * sizeof(float), 256);
    }
    w = align_up(w + N * row, 256);
    *total = w;
}

hipEvent_t take_event(cr_plan_t *p)
{
    if (!p->event_pool.empty()) {
        hipEvent_t e = p->event_pool.back();
        p->event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct LaunchTimer {     // brackets one launch with events when profiling is on
    cr_plan_t *p;
    int kernel;
    hipEvent_t start = nullptr, stop = nullptr;
    LaunchTimer(cr_plan_t *plan, int k, int64_t bytes) : p(plan), kernel(k)
    {
        p->bytes_last[k] = bytes;
        if (!((p->profiling >> k) & 1)) return;
        start = take_event(p);
        stop = take_event(p);
        if (start && stop) (void)hipEventRecord(start, p->stream);
    }
    void done()
    {
        if (!start || !stop) return;
        (void)hipEventRecord(stop, p->stream);
        p->timed.push_back({kernel, start, stop});
        p->bytes_sum[kernel] += p->bytes_last[kernel];
    }
};

int fold_timings(cr_plan_t *p)
{
    for (const TimedLaunch &t : p->timed) {
        float ms = 0.f;
        CR_HIP(hipEventElapsedTime(&ms, t.start, t.stop));
        p->total_ms[t.kernel] += ms;
        p->launches[t.kernel] += 1;
        if (p->samples[t.kernel].size() < kMaxSamples) p->samples[t.kernel].push_back(ms);
        p->event_pool.push_back(t.start);
        p->event_pool.push_back(t.stop);
    }
    p->timed.clear();
    return CR_OK;
}

// The row-cell and shared-cell splits put the holders of a cell on workgroup ids that are congruent modulo the number of L2
// domains, trusting that the dispatcher deals workgroups to the dies round-robin.  This runs a launch of kPlacementSlots small
// workgroups that record the die they ran on and checks exactly that; the outcome is reported by cr_plan_info (l2_sharing).
// A device that places workgroups differently still computes the same results, only without the shared fetches.
int check_l2_sharing(cr_plan_t *p)
{
    std::vector<uint32_t> where(kPlacementSlots);
    CR_HIP(cr::launch_placement_probe(p->d_placement, kPlacementSlots, p->stream));
    CR_HIP(hipMemcpyAsync(where.data(), p->d_placement, kPlacementSlots * sizeof(uint32_t), hipMemcpyDeviceToHost, p->stream));
    CR_HIP(hipStreamSynchronize(p->stream));
    const int domains = p->l2_domains;
    std::vector<int> die_of(domains, -1);
    bool ok = true;
    for (int g = 0; g < kPlacementSlots && ok; ++g) {
        const int die = static_cast<int>(where[g] >> 16);
        int &seen = die_of[g % domains];
        if (seen < 0) seen = die;
        ok = seen == die;
    }
    for (int a = 0; a < domains && ok; ++a)                  // and distinct residues on distinct dies
        for (int b = a + 1; b < domains; ++b) ok = ok && die_of[a] != die_of[b];
    p->l2_sharing = ok ? 1 : 0;
    return CR_OK;
}

}  // namespace

extern "C" {

const char *cr_last_error(void) { return g_last_error.c_str(); }

int cr_plan(int L, int n, int s, int64_t m, int64_t d, cr_plan_t **out)
{
    return cr_plan_ex(L, n, s, m, d, CR_LINEAR, CR_F32, kDefaultSeed, nullptr, out);
}

int cr_plan_ex(int L, int n, int s, int64_t m, int64_t d, int model, int x_dtype, uint64_t seed, const double *B_or_null, cr_plan_t **out)
{
    if (!out) return fail(CR_E_INVAL, "out is NULL");
    *out = nullptr;
    if (L < 1 || L > cr::kMaxLevels) return fail(CR_E_INVAL, "L must be in 1..8");
    if (n < 2 || n > 64) return fail(CR_E_INVAL, "n must be in 2..64");
    if (s < 0 || s >= n) return fail(CR_E_INVAL, "s must be in 0..n-1");
    if (d < 1) return fail(CR_E_INVAL, "d must be positive");
    if (d > (int64_t(1) << 28)) return fail(CR_E_INVAL, "d exceeds 2^28");     // every kernel indexes columns with 32-bit integers
    if (model < CR_LINEAR || model > CR_AGGREGATE_ONLY) return fail(CR_E_INVAL, "unknown model");
    if (x_dtype != CR_F32 && x_dtype != CR_BF16) return fail(CR_E_INVAL, "unknown x_dtype");
    if (cr::num_straggler_sets(n, s, int64_t(1) << 20) < 0) return fail(CR_E_INVAL, "C(n,s) exceeds 2^20 straggler patterns");
    cr_plan_t *p = new (std::nothrow) cr_plan_s();
    if (!p) return fail(CR_E_NOMEM, "out of host memory");
    try {
        if (!cr::make_tree(n, L, p->tree)) { delete p; return fail(CR_E_INVAL, "tree has more than 2^24 workers"); }
        if (m < p->tree.N) { delete p; return fail(CR_E_INVAL, "m must be at least the number of workers"); }
        if (m > (int64_t(1) << 40)) { delete p; return fail(CR_E_INVAL, "m exceeds 2^40"); }
        p->L = L; p->n = n; p->s = s; p->m = m; p->d = d; p->model = model; p->x_dtype = x_dtype;
        bool ok = B_or_null ? cr::adopt_code(n, s, B_or_null, p->code) : cr::design_code(n, s, L, seed, p->code);
        if (!ok) { delete p; return fail(CR_E_INVAL, B_or_null ? "supplied B must have s+1 non-zeros per row and per column and decode every straggler set" : "code search found no usable candidate"); }
        cr::allocate(p->tree, s, m, p->code.B.data(), p->own, p->slabs);
        p->node_slab_begin.assign(p->tree.N + 1, 0);
        for (const cr::Slab &sl : p->slabs) p->node_slab_begin[sl.node + 1] += 1;
        for (int32_t i = 0; i < p->tree.N; ++i) p->node_slab_begin[i + 1] += p->node_slab_begin[i];
        p->min_rows = INT64_MAX;
        for (int32_t node = 0; node < p->tree.N; ++node) {
            int64_t rows = 0;
            for (const cr::Segment &g : p->own[node]) rows += g.row_end - g.row_begin;
            p->row_visits += rows;
            p->min_rows = std::min(p->min_rows, rows);
            p->max_rows = std::max(p->max_rows, rows);
        }
        if (p->slabs.size() > (size_t(1) << 30)) { delete p; return fail(CR_E_INVAL, "too many slabs"); }
        if (model != CR_AGGREGATE_ONLY) {
            p->variant_regs = cr::select_stage1(x_dtype, d);          // nullptr: rows too wide for one team's registers, two-pass path
            int64_t max_holders = 1;                                  // a leaf's rows sit in s+1 workers of every level above it
            for (int l = 0; l < L && max_holders < 64; ++l) max_holders *= s + 1;
            p->variant_staged = s > 0 ? cr::select_stage1_staged(x_dtype, d, max_holders) : nullptr;   // nullptr: no such kernel for this width
            p->variant = p->variant_regs;
        }
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(CR_E_NOMEM, "out of host memory");
    }
    *out = p;
    return CR_OK;
}

void cr_plan_destroy(cr_plan_t *p)
{
    if (!p) return;
    if (p->bound) (void)hipStreamSynchronize(p->stream);
    for (const TimedLaunch &t : p->timed) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
    for (hipEvent_t e : p->event_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->staging_done)
        if (e) (void)hipEventDestroy(e);
    if (p->h_staging) (void)hipHostFree(p->h_staging);
    delete p;
}

int cr_plan_info(const cr_plan_t *p, cr_plan_info_t *info)
{
    if (!p || !info) return fail(CR_E_INVAL, "NULL argument");
    std::memset(info, 0, sizeof *info);
    info->L = p->L; info->n = p->n; info->s = p->s; info->model = p->model; info->x_dtype = p->x_dtype;
    info->num_workers = p->tree.N;
    info->num_groups = p->tree.N / p->n;
    info->num_slabs = static_cast<int32_t>(p->slabs.size());
    info->num_decode_rows = static_cast<int32_t>(cr::num_straggler_sets(p->n, p->s, int64_t(1) << 20));
    info->code_candidate = p->code.candidate;
    info->num_teams = p->split.teams;
    info->num_pieces = static_cast<int32_t>(p->split.pieces.size());
    const bool split_known = !p->split.pieces.empty();
    info->split_kind = split_known ? p->split_kind_used : -1;
    info->split_value = split_known ? p->split_value_used : 0;
    info->stage1_team_size = p->variant ? p->variant->team_size : 0;
    info->stage1_teams_per_group = p->variant ? p->variant->teams_per_block() : 1;
    info->stage1_staged = p->variant && p->variant->staged ? 1 : 0;
    info->m = p->m; info->d = p->d;
    info->row_visits = p->row_visits;
    info->min_rows = p->min_rows; info->max_rows = p->max_rows;
    info->gamma = p->code.gamma;
    double q = static_cast<double>(p->n) / (p->s + 1), sum = 0.0, pw = 1.0;
    for (int l = 1; l <= p->L; ++l) { pw *= q; sum += pw; }
    info->r_cr = 1.0 / sum;
    info->l2_domains = p->l2_domains ? p->l2_domains : kDefaultL2Domains;
    info->unit_slots = split_known ? p->unit_slots : 0;
    info->l2_sharing = p->l2_sharing;
    info->code_warning = std::pow(p->code.gamma, p->L) * std::ldexp(1.0, -24) > 1e-5 ? 1 : 0;
    return CR_OK;
}

int cr_plan_get_B(const cr_plan_t *p, double *B)
{
    if (!p || !B) return fail(CR_E_INVAL, "NULL argument");
    std::copy(p->code.B.begin(), p->code.B.end(), B);
    return CR_OK;
}

int cr_plan_get_A(const cr_plan_t *p, double *A)
{
    if (!p || !A) return fail(CR_E_INVAL, "NULL argument");
    const int64_t F = cr::num_straggler_sets(p->n, p->s, int64_t(1) << 20);
    for (int64_t f = 0; f < F; ++f)
        if (!cr::decode_row(p->code, cr::straggler_set_by_rank(p->n, p->s, f), A + f * p->n))
            return fail(CR_E_INVAL, "decode row: survivor system is inconsistent");
    return CR_OK;
}

int cr_plan_get_segments(const cr_plan_t *p, int64_t *row_begin, int64_t *row_end, double *coef, int32_t *worker)
{
    if (!p) return fail(CR_E_INVAL, "NULL plan");
    for (size_t i = 0; i < p->slabs.size(); ++i) {
        if (worker) worker[i] = p->slabs[i].node;
        if (row_begin) row_begin[i] = p->slabs[i].row_begin;
        if (row_end) row_end[i] = p->slabs[i].row_end;
        if (coef) coef[i] = p->slabs[i].coef;
    }
    return CR_OK;
}

int cr_plan_decode_row(const cr_plan_t *p, const uint8_t *flags, double *a)
{
    if (!p || !flags || !a) return fail(CR_E_INVAL, "NULL argument");
    const double *row = nullptr;
    int rc = group_decode_row(p, flags, &row);
    if (rc == CR_E_UNDECODABLE) return fail(rc, "more than s stragglers in the group");
    if (rc != CR_OK) return rc;
    std::copy(row, row + p->n, a);
    return CR_OK;
}

int cr_plan_set_split(cr_plan_t *p, int kind, int64_t value)
{
    if (!p) return fail(CR_E_INVAL, "NULL plan");
    if (kind != CR_SPLIT_EQUAL_RANGES && kind != CR_SPLIT_ROW_CELLS && kind != CR_SPLIT_SHARED_CELLS) return fail(CR_E_INVAL, "unknown split kind");
    if (value < 1) return fail(CR_E_INVAL, "split value must be >= 1");
    if (kind == CR_SPLIT_EQUAL_RANGES && value > (int64_t(1) << 24)) return fail(CR_E_INVAL, "too many teams");
    if (p->bound) return fail(CR_E_STATE, "the work split cannot change once a workspace is bound");
    if (p->model == CR_AGGREGATE_ONLY) return fail(CR_E_INVAL, "an aggregation-only plan has no stage-1 split");
    p->split_kind = kind;
    p->split_value = value;
    p->split = cr::Split();
    return ensure_split(p);
}

int cr_plan_get_pieces(const cr_plan_t *p, int32_t *slab, int64_t *row_begin, int64_t *row_end, int32_t *team)
{
    if (!p) return fail(CR_E_INVAL, "NULL plan");
    for (size_t i = 0; i < p->split.pieces.size(); ++i) {
        if (slab) slab[i] = p->split.pieces[i].slab;
        if (row_begin) row_begin[i] = p->split.pieces[i].row_begin;
        if (row_end) row_end[i] = p->split.pieces[i].row_end;
        if (team) team[i] = p->split.pieces[i].team;
    }
    return CR_OK;
}

int cr_simulate_iteration(const cr_plan_t *p, double a, double mu, double t_c, uint64_t seed, int64_t iteration, uint8_t *mask,
                          double *ready, double *total)
{
    if (!p) return fail(CR_E_INVAL, "NULL plan");
    if (!(a >= 0.0) || !(mu > 0.0) || !(t_c >= 0.0) || iteration < 0) return fail(CR_E_INVAL, "a >= 0, mu > 0, t_c >= 0, iteration >= 0 required");
    std::vector<int64_t> rows(p->tree.N, 0);
    for (const cr::Slab &sl : p->slabs) rows[sl.node] += sl.row_end - sl.row_begin;
    const double t = cr::simulate_iteration(p->tree, p->s, rows, {a, mu, t_c}, seed, iteration, mask, ready);
    if (total) *total = t;
    return CR_OK;
}

int cr_workspace_bytes(cr_plan_t *p, size_t *bytes)
{
    if (!p || !bytes) return fail(CR_E_INVAL, "NULL argument");
    int rc = ensure_split(p);
    if (rc != CR_OK) return rc;
    compute_layout(p, bytes);
    return CR_OK;
}

int cr_bind_workspace(cr_plan_t *p, void *dev_ptr, size_t bytes, void *hip_stream)
{
    if (!p || !dev_ptr) return fail(CR_E_INVAL, "NULL argument");
    if (reinterpret_cast<uintptr_t>(dev_ptr) % 256 != 0) return fail(CR_E_INVAL, "workspace must be 256-byte aligned");
    int rc = ensure_split(p);
    if (rc != CR_OK) return rc;
    size_t need = 0;
    compute_layout(p, &need);
    if (bytes < need) return fail(CR_E_INVAL, "workspace too small");
    if (p->bound) CR_HIP(hipStreamSynchronize(p->stream));
    if (p->variant) {
        int dev = 0, lds = 0;
        CR_HIP(hipGetDevice(&dev));
        CR_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        if (p->variant->lds_bytes(p->d) > static_cast<size_t>(lds)) return fail(CR_E_INVAL, "the stage-1 kernel needs more LDS per workgroup than this device has");
        CR_HIP(cr::prepare_stage1(*p->variant, p->d));
    }
    p->stream = static_cast<hipStream_t>(hip_stream);
    p->ws = static_cast<char *>(dev_ptr);
    p->ws_bytes = bytes;

    const size_t S = p->slabs.size(), N = p->tree.N, P = p->split.pieces.size();
    const size_t row = static_cast<size_t>(p->d) * sizeof(float);
    size_t w = 0;
    p->d_pieces = reinterpret_cast<cr::DevPiece *>(p->ws + w);             w = align_up(w + P * sizeof(cr::DevPiece), 256);
    p->d_team_piece_begin = reinterpret_cast<int32_t *>(p->ws + w);        w = align_up(w + (p->split.teams + 1) * sizeof(int32_t), 256);
    p->d_slab_piece_begin = reinterpret_cast<int32_t *>(p->ws + w);        w = align_up(w + (S + 1) * sizeof(int32_t), 256);
    p->d_slab_pieces = reinterpret_cast<int32_t *>(p->ws + w);             w = align_up(w + P * sizeof(int32_t), 256);
    p->d_group_item_begin = reinterpret_cast<int32_t *>(p->ws + w);        w = align_up(w + p->split.group_item_begin.size() * sizeof(int32_t), 256);
    p->d_item_pieces = reinterpret_cast<int32_t *>(p->ws + w);             w = align_up(w + p->split.item_pieces.size() * sizeof(int32_t), 256);
    p->d_placement = reinterpret_cast<uint32_t *>(p->ws + w);              w = align_up(w + kPlacementSlots * sizeof(uint32_t), 256);
    p->d_program = p->ws + w;                                              w = align_up(w + kProgramSlots * p->program_bytes, 256);
    p->d_partial = nullptr; p->d_G = nullptr;
    if (p->model != CR_AGGREGATE_ONLY) {
        p->d_partial = reinterpret_cast<float *>(p->ws + w);               w = align_up(w + P * row, 256);
        p->d_G = reinterpret_cast<float *>(p->ws + w);                     w = align_up(w + S * row, 256);
        if (!p->variant) { p->d_residuals = reinterpret_cast<float *>(p->ws + w); w = align_up(w + static_cast<size_t>(p->row_visits) * sizeof(float), 256); }
    }
    p->d_M = reinterpret_cast<float *>(p->ws + w);                         w = align_up(w + N * row, 256);
    p->G_src = p->d_G;

    if (P > 0) {
        std::vector<cr::DevPiece> hp(P);
        int64_t visit = 0, longest = 0;
        for (size_t i = 0; i < P; ++i) longest = std::max(longest, p->split.pieces[i].row_end - p->split.pieces[i].row_begin);
        p->rows_as_buffers = (p->d * elem_size(p)) % 4 == 0 && longest * p->d * elem_size(p) < (int64_t(1) << 31);
        for (size_t i = 0; i < P; ++i) {
            const int64_t rows = p->split.pieces[i].row_end - p->split.pieces[i].row_begin;
            // shared cells know which of them several workgroups fetch; under the other splits a row is fetched by each of its holders
            // ... and a data matrix of a few hundred megabytes stays in the last-level cache (256 MB on MI355X) from one iteration
            // to the next if its lines are allowed to: only larger ones are streamed past the caches
            const bool streams = p->m * p->d * elem_size(p) >= kStreamFromBytes;
            const int32_t shared = !streams ? 1 : p->split_kind_used == CR_SPLIT_SHARED_CELLS ? p->split.pieces[i].shared : (p->s > 0 ? 1 : 0);
            hp[i] = {p->split.pieces[i].row_begin, visit, static_cast<int32_t>(rows), p->split.pieces[i].slab, shared, 0};
            visit += rows;
        }
        CR_HIP(hipMemcpy(p->d_pieces, hp.data(), P * sizeof(cr::DevPiece), hipMemcpyHostToDevice));
        CR_HIP(hipMemcpy(p->d_team_piece_begin, p->split.team_piece_begin.data(), (p->split.teams + 1) * sizeof(int32_t), hipMemcpyHostToDevice));
        CR_HIP(hipMemcpy(p->d_slab_piece_begin, p->split.slab_piece_begin.data(), (S + 1) * sizeof(int32_t), hipMemcpyHostToDevice));
        CR_HIP(hipMemcpy(p->d_slab_pieces, p->split.slab_pieces.data(), P * sizeof(int32_t), hipMemcpyHostToDevice));
        if (!p->split.item_pieces.empty()) {
            CR_HIP(hipMemcpy(p->d_group_item_begin, p->split.group_item_begin.data(), p->split.group_item_begin.size() * sizeof(int32_t), hipMemcpyHostToDevice));
            CR_HIP(hipMemcpy(p->d_item_pieces, p->split.item_pieces.data(), p->split.item_pieces.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        }
    }
    p->l2_sharing = -1;
    if (P > 0 && (p->split_kind_used == CR_SPLIT_ROW_CELLS || p->split_kind_used == CR_SPLIT_SHARED_CELLS)) {
        int rc = check_l2_sharing(p);
        if (rc != CR_OK) return rc;
    }
    if (!p->h_staging) {
        CR_HIP(hipHostMalloc(reinterpret_cast<void **>(&p->h_staging), p->program_bytes * kProgramSlots * kStagingHalves, hipHostMallocDefault));
        for (int i = 0; i < kStagingHalves; ++i) CR_HIP(hipEventCreateWithFlags(&p->staging_done[i], hipEventDisableTiming));
    }
    p->bound = true;
    p->have_grads = false;
    p->have_messages = false;
    return CR_OK;
}

int cr_partial_grads(cr_plan_t *p, const void *X, const float *y, const float *w)
{
    if (!p || !X || !y || !w) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    if (p->model == CR_AGGREGATE_ONLY) return fail(CR_E_STATE, "aggregation-only plan: use cr_load_partial_grads");
    if (reinterpret_cast<uintptr_t>(X) % 16 != 0) return fail(CR_E_INVAL, "X must be 16-byte aligned");
    const int64_t S = static_cast<int64_t>(p->slabs.size()), P = static_cast<int64_t>(p->split.pieces.size());
    {
        // what the method must move: every holder reads its rows and targets once, each slab gradient is written once
        const int64_t bytes = p->row_visits * p->d * elem_size(p) + p->row_visits * 4 + S * p->d * 4 + p->d * 4;
        LaunchTimer t(p, CR_K_PARTIAL_GRADS, bytes);
        if (p->variant && p->variant->staged) {
            CR_HIP(cr::launch_partial_grads_staged(*p->variant, X, y, w, p->d_pieces, p->d_group_item_begin, p->d_item_pieces,
                                                   static_cast<int>(p->split.group_item_begin.size()) - 1, p->d_partial, p->d,
                                                   p->model == CR_LOGISTIC ? 1 : 0, p->stream));
        } else if (p->variant) {
            CR_HIP(cr::launch_partial_grads(*p->variant, X, y, w, p->d_pieces, p->d_team_piece_begin, p->split.teams, p->d_partial, p->d,
                                            p->model == CR_LOGISTIC ? 1 : 0, p->rows_as_buffers, p->stream));
        } else {
            CR_HIP(cr::launch_residuals(p->x_dtype, X, y, w, p->d_pieces, static_cast<int>(P), p->d_residuals, p->d,
                                        p->model == CR_LOGISTIC ? 1 : 0, p->stream));
            CR_HIP(cr::launch_xt_residuals(p->x_dtype, X, p->d_pieces, static_cast<int>(P), p->d_residuals, p->d_partial, p->d, p->stream));
        }
        t.done();
    }
    {
        LaunchTimer t(p, CR_K_REDUCE_PIECES, (P + S) * p->d * 4);
        CR_HIP(cr::launch_reduce_pieces(p->d_partial, p->d_slab_piece_begin, p->d_slab_pieces, static_cast<int>(S), p->d_G, p->d, p->stream));
        t.done();
    }
    p->G_src = p->d_G;
    p->have_grads = true;
    p->have_messages = false;
    return CR_OK;
}

int cr_load_partial_grads(cr_plan_t *p, const float *G)
{
    if (!p || !G) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    if (reinterpret_cast<uintptr_t>(G) % 16 != 0) return fail(CR_E_INVAL, "G must be 16-byte aligned");
    p->G_src = G;
    p->have_grads = true;
    p->have_messages = false;
    return CR_OK;
}

namespace {

struct ProgramCounts { int64_t active_slabs = 0, active_msgs = 0; int dec_terms = 0; };

// Turns a straggler mask into the encode program of one iteration, written into the host block h (program_bytes long, laid out
// by compute_layout): the post-order term list of every level-1 sub-tree and the master's decode terms.  Any group beyond
// tolerance fails the call before anything is written (CR_E_UNDECODABLE).
int build_program(cr_plan_t *p, const uint8_t *mask, char *h, ProgramCounts *counts)
{
    const int n = p->n, L = p->L;
    const int32_t N = p->tree.N, groups = N / n;
    // decode row of every sibling group
    std::vector<const double *> rows(groups);
    for (int32_t g = 0; g < groups; ++g) {
        int rc = group_decode_row(p, mask + static_cast<size_t>(g) * n, &rows[g]);
        if (rc == CR_E_UNDECODABLE) return fail(rc, "sibling group " + std::to_string(g) + " has more than s stragglers");
        if (rc != CR_OK) return rc;
    }
    int32_t *t_slab = reinterpret_cast<int32_t *>(h + p->off_slab);
    int32_t *t_level = reinterpret_cast<int32_t *>(h + p->off_level);
    int32_t *t_row = reinterpret_cast<int32_t *>(h + p->off_row);
    double *t_coef = reinterpret_cast<double *>(h + p->off_coef);
    double *t_acoef = reinterpret_cast<double *>(h + p->off_acoef);
    auto put = [&](size_t t, int32_t slab, double coef) { t_slab[t] = slab; t_level[t] = 0; t_row[t] = 0; t_coef[t] = coef; t_acoef[t] = 0.0; };
    int32_t *sub = reinterpret_cast<int32_t *>(h + p->off_sub);
    cr::DecTerm *dec = reinterpret_cast<cr::DecTerm *>(h + p->off_dec);

    // post-order program of every level-1 sub-tree
    size_t nt = 0;
    struct Frame { int32_t node; int level; int next_child; };
    std::vector<Frame> stack;
    for (int i = 0; i < n; ++i) {
        sub[i] = static_cast<int32_t>(nt);
        size_t real_terms = 0;
        stack.push_back({static_cast<int32_t>(i), 1, 0});
        while (!stack.empty()) {
            Frame &f = stack.back();
            if (f.level < L && f.next_child < n) {
                const int32_t child = p->tree.level_offset[f.level + 1] + (f.node - p->tree.level_offset[f.level]) * n + f.next_child;
                ++f.next_child;
                stack.push_back({child, f.level + 1, 0});
                continue;
            }
            const int32_t node = f.node;
            const int level = f.level;
            stack.pop_back();
            if (mask[node]) continue;                     // a straggler sends nothing
            double acoef = 0.0;
            if (level >= 2) {
                const int32_t parent = p->tree.level_offset[level - 1] + (node - p->tree.level_offset[level]) / n;
                if (!mask[parent]) acoef = rows[node / n][node % n];
            }
            const int32_t sb = p->node_slab_begin[node], se = p->node_slab_begin[node + 1];
            for (int32_t q = sb; q < se; ++q) put(nt++, q, p->slabs[q].coef);
            if (se == sb) put(nt++, 0, 0.0);              // a node without rows still sends its children's combination
            t_level[nt - 1] = level;                      // the node's last term finishes it
            t_row[nt - 1] = node;
            t_acoef[nt - 1] = acoef;
            counts->active_slabs += se - sb;
            counts->active_msgs += 1;
        }
        real_terms = nt - static_cast<size_t>(sub[i]);
        while (nt % cr::kEncodeUnroll != 0) {             // pad with no-op terms on an already fetched slab
            put(nt, nt > 0 ? t_slab[nt - 1] : 0, 0.0);
            ++nt;
        }
        sub[n + i] = sub[i] + static_cast<int32_t>(real_terms);
    }
    int ndec = 0;
    for (int j = 0; j < n; ++j)
        if (!mask[j] && rows[0][j] != 0.0) dec[ndec++] = {j, 0, rows[0][j]};
    counts->dec_terms = ndec;
    return CR_OK;
}

// the program's arrays as the encode kernel takes them, for a program block at device address d_program
cr::EncProgram program_view(const cr_plan_t *p, const char *d_program)
{
    cr::EncProgram prog;
    prog.slab = reinterpret_cast<const int32_t *>(d_program + p->off_slab);
    prog.level = reinterpret_cast<const int32_t *>(d_program + p->off_level);
    prog.row = reinterpret_cast<const int32_t *>(d_program + p->off_row);
    prog.coef = reinterpret_cast<const double *>(d_program + p->off_coef);
    prog.acoef = reinterpret_cast<const double *>(d_program + p->off_acoef);
    prog.sub_begin = reinterpret_cast<const int32_t *>(d_program + p->off_sub);
    prog.sub_end = prog.sub_begin + p->n;
    return prog;
}

}  // namespace

namespace {

// every group of every mask within tolerance?  (checked before anything is enqueued or any staging is touched)
int check_masks(const cr_plan_t *p, const uint8_t *masks, int steps)
{
    const int n = p->n;
    const int32_t N = p->tree.N;
    for (int t = 0; t < steps; ++t)
        for (int32_t grp = 0; grp < N / n; ++grp) {
            int cnt = 0;
            for (int j = 0; j < n; ++j) cnt += masks[static_cast<size_t>(t) * N + static_cast<size_t>(grp) * n + j] ? 1 : 0;
            if (cnt > p->s)
                return fail(CR_E_UNDECODABLE, (steps > 1 ? "step " + std::to_string(t) + ": " : std::string()) + "sibling group " + std::to_string(grp) +
                                                  " has more than s stragglers");
        }
    return CR_OK;
}

// Builds the encode programs of `count` <= kProgramSlots masks in pinned staging and sends them to program slots 0 .. count-1 with
// one copy on the plan's stream (which therefore follows every kernel that still reads the slots).  counts[i] describes program i.
int upload_programs(cr_plan_t *p, const uint8_t *masks, int count, ProgramCounts *counts)
{
    const int half = p->staging_next;
    if (p->staging_used[half]) CR_HIP(hipEventSynchronize(p->staging_done[half]));     // the copy that last read this half is done
    char *h = p->h_staging + static_cast<size_t>(half) * kProgramSlots * p->program_bytes;
    for (int i = 0; i < count; ++i) {
        counts[i] = ProgramCounts();
        int rc = build_program(p, masks + static_cast<size_t>(i) * p->tree.N, h + static_cast<size_t>(i) * p->program_bytes, &counts[i]);
        if (rc != CR_OK) return rc;
    }
    p->staging_next = (half + 1) % kStagingHalves;
    CR_HIP(hipMemcpyAsync(p->d_program, h, static_cast<size_t>(count) * p->program_bytes, hipMemcpyHostToDevice, p->stream));
    CR_HIP(hipEventRecord(p->staging_done[half], p->stream));
    p->staging_used[half] = true;
    return CR_OK;
}

int encode_slot(cr_plan_t *p, int slot, const ProgramCounts &counts)
{
    LaunchTimer t(p, CR_K_ENCODE, (counts.active_slabs + counts.active_msgs) * p->d * 4);
    CR_HIP(cr::launch_encode(p->G_src, p->d_M, program_view(p, p->d_program + static_cast<size_t>(slot) * p->program_bytes), p->n, p->L, p->d, p->stream));
    t.done();
    p->num_dec_terms = counts.dec_terms;
    p->dec_slot = slot;
    p->have_messages = true;
    return CR_OK;
}

// the master's decode; with w != nullptr the gradient step w <- w - lr g rides in the same launch
int decode_root(cr_plan_t *p, float *g, float *w, float lr)
{
    if (!p || !g) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    if (!p->have_messages) return fail(CR_E_STATE, "no messages yet: call cr_encode_tree first");
    LaunchTimer t(p, CR_K_DECODE, static_cast<int64_t>(p->num_dec_terms + 1 + (w ? 2 : 0)) * p->d * 4);
    const char *prog = p->d_program + static_cast<size_t>(p->dec_slot) * p->program_bytes;
    CR_HIP(cr::launch_decode(p->d_M, g, reinterpret_cast<const cr::DecTerm *>(prog + p->off_dec), p->num_dec_terms, p->d, w, lr, p->stream));
    t.done();
    return CR_OK;
}

}  // namespace

int cr_encode_tree(cr_plan_t *p, const uint8_t *mask)
{
    if (!p || !mask) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    if (!p->have_grads) return fail(CR_E_STATE, "no partial gradients yet");
    int rc = check_masks(p, mask, 1);
    if (rc != CR_OK) return rc;
    ProgramCounts counts;
    rc = upload_programs(p, mask, 1, &counts);
    if (rc != CR_OK) return rc;
    return encode_slot(p, 0, counts);
}

int cr_decode_root(cr_plan_t *p, float *g) { return decode_root(p, g, nullptr, 0.f); }

int cr_gd_update(cr_plan_t *p, float *w, const float *g, float lr)
{
    if (!p || !w || !g) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    LaunchTimer t(p, CR_K_UPDATE, 3 * p->d * 4);
    CR_HIP(cr::launch_update(w, g, lr, p->d, p->stream));
    t.done();
    return CR_OK;
}

int cr_gd_run(cr_plan_t *p, const void *X, const float *y, float *w, float *g, const uint8_t *masks, int steps, float lr,
              const float *w_star, float *metrics)
{
    if (!p || !X || !y || !w || !g || !masks) return fail(CR_E_INVAL, "NULL argument");
    if (steps < 0) return fail(CR_E_INVAL, "steps must be >= 0");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    if (p->model == CR_AGGREGATE_ONLY) return fail(CR_E_STATE, "aggregation-only plan has no gradient stage");
    int rc = check_masks(p, masks, steps);              // every mask is checked before anything is enqueued
    if (rc != CR_OK) return rc;
    const int32_t N = p->tree.N;
    ProgramCounts counts[kProgramSlots];
    for (int t0 = 0; t0 < steps; t0 += kProgramSlots) {
        // the programs of the next kProgramSlots steps travel in one copy; the steps themselves are kernel launches only
        const int count = std::min(kProgramSlots, steps - t0);
        rc = upload_programs(p, masks + static_cast<size_t>(t0) * N, count, counts);
        if (rc != CR_OK) return rc;
        for (int i = 0; i < count; ++i) {
            rc = cr_partial_grads(p, X, y, w);
            if (rc == CR_OK) rc = encode_slot(p, i, counts[i]);
            // without the convergence measures the gradient step rides in the decode launch (same arithmetic as cr_gd_update)
            if (rc == CR_OK) rc = decode_root(p, g, metrics ? nullptr : w, lr);
            if (rc != CR_OK) return rc;
            if (metrics) {
                LaunchTimer tm(p, CR_K_UPDATE, 3 * p->d * 4 + (w_star ? p->d * 4 : 0));
                CR_HIP(cr::launch_update_metrics(w, g, lr, w_star, metrics + 2 * static_cast<size_t>(t0 + i), p->d, p->stream));
                tm.done();
            }
        }
    }
    return CR_OK;
}

int cr_aggregate_run(cr_plan_t *p, const float *G, int64_t G_step_stride, const uint8_t *masks, int steps, float *g, int64_t g_step_stride)
{
    if (!p || !G || !masks || !g) return fail(CR_E_INVAL, "NULL argument");
    if (steps < 0 || G_step_stride < 0 || g_step_stride < 0) return fail(CR_E_INVAL, "steps and strides must be >= 0");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    if (reinterpret_cast<uintptr_t>(G) % 16 != 0 || (G_step_stride * sizeof(float)) % 16 != 0) return fail(CR_E_INVAL, "G and its step stride must be 16-byte aligned");
    int rc = check_masks(p, masks, steps);
    if (rc != CR_OK) return rc;
    const int32_t N = p->tree.N;
    ProgramCounts counts[kProgramSlots];
    for (int t0 = 0; t0 < steps; t0 += kProgramSlots) {
        const int count = std::min(kProgramSlots, steps - t0);
        rc = upload_programs(p, masks + static_cast<size_t>(t0) * N, count, counts);
        if (rc != CR_OK) return rc;
        for (int i = 0; i < count; ++i) {
            p->G_src = G + static_cast<int64_t>(t0 + i) * G_step_stride;
            p->have_grads = true;
            rc = encode_slot(p, i, counts[i]);
            if (rc == CR_OK) rc = decode_root(p, g + static_cast<int64_t>(t0 + i) * g_step_stride, nullptr, 0.f);
            if (rc != CR_OK) return rc;
        }
    }
    return CR_OK;
}

int cr_aggregate_static(cr_plan_t *p, const float *G, const uint8_t *mask, float *g, void *hip_stream)
{
    static_assert(CR_STATIC_SCRATCH_BYTES == cr::kStaticScratchBytes, "the header states the size of the library's device array");
    if (!p || !G || !mask || !g) return fail(CR_E_INVAL, "NULL argument");
    if (reinterpret_cast<uintptr_t>(G) % 16 != 0) return fail(CR_E_INVAL, "G must be 16-byte aligned");
    if (p->program_bytes == 0) {                        // offsets of the program's arrays: host arithmetic only
        size_t unused = 0;
        compute_layout(p, &unused);
    }
    const size_t msg_bytes = static_cast<size_t>(p->tree.N) * static_cast<size_t>(p->d) * sizeof(float);
    if (p->program_bytes > cr::kStaticProgramBytes)
        return fail(CR_E_INVAL, "cr_aggregate_static: the encode program of this tree (" + std::to_string(p->program_bytes) + " bytes) exceeds 64 KiB");
    if (msg_bytes > cr::kStaticScratchBytes - cr::kStaticProgramBytes)
        return fail(CR_E_INVAL, "cr_aggregate_static: N * d * 4 = " + std::to_string(msg_bytes) + " bytes of messages exceed the library's device array (" +
                                    std::to_string(cr::kStaticScratchBytes - cr::kStaticProgramBytes) + " bytes)");
    if (p->static_program.size() != p->program_bytes) p->static_program.assign(p->program_bytes, 0);
    ProgramCounts counts;
    int rc = build_program(p, mask, p->static_program.data(), &counts);
    if (rc != CR_OK) return rc;
    char *base = nullptr;
    CR_HIP(cr::static_scratch(&base));                  // this device's copy of the array; never the array's name
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float *M = reinterpret_cast<float *>(base + cr::kStaticProgramBytes);
    CR_HIP(cr::launch_upload(base, p->static_program.data(), p->program_bytes, stream));
    CR_HIP(cr::launch_encode(G, M, program_view(p, base), p->n, p->L, p->d, stream));
    CR_HIP(cr::launch_decode(M, g, reinterpret_cast<const cr::DecTerm *>(base + p->off_dec), counts.dec_terms, p->d, nullptr, 0.f, stream));
    return CR_OK;
}

int cr_get_slab_grads(const cr_plan_t *p, const float **G)
{
    if (!p || !G) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    *G = p->G_src;
    return CR_OK;
}

int cr_get_messages(const cr_plan_t *p, const float **M)
{
    if (!p || !M) return fail(CR_E_INVAL, "NULL argument");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    *M = p->d_M;
    return CR_OK;
}

int cr_profile_enable(cr_plan_t *p, int kernels)
{
    if (!p) return fail(CR_E_INVAL, "NULL plan");
    if (p->bound) {
        CR_HIP(hipStreamSynchronize(p->stream));
        int rc = fold_timings(p);
        if (rc != CR_OK) return rc;
    }
    if (kernels < 0 || kernels > CR_PROFILE_ALL) return fail(CR_E_INVAL, "kernel mask out of range");
    if (kernels) {                                      // a new selection starts new totals
        for (int k = 0; k < CR_K_COUNT; ++k) { p->total_ms[k] = 0.0; p->launches[k] = 0; p->bytes_sum[k] = 0; p->samples[k].clear(); }
    }
    p->profiling = static_cast<unsigned>(kernels);
    return CR_OK;
}

int cr_profile_read(cr_plan_t *p, int kernel, double *total_ms, int64_t *launches, int64_t *algorithmic_bytes)
{
    if (!p || kernel < 0 || kernel >= CR_K_COUNT) return fail(CR_E_INVAL, "bad argument");
    if (p->bound) {
        CR_HIP(hipStreamSynchronize(p->stream));
        int rc = fold_timings(p);
        if (rc != CR_OK) return rc;
    }
    if (total_ms) *total_ms = p->total_ms[kernel];
    if (launches) *launches = p->launches[kernel];
    if (algorithmic_bytes) *algorithmic_bytes = p->bytes_sum[kernel];
    return CR_OK;
}

int cr_profile_samples(cr_plan_t *p, int kernel, float *ms, int64_t capacity, int64_t *count)
{
    if (!p || !count || kernel < 0 || kernel >= CR_K_COUNT || capacity < 0 || (capacity > 0 && !ms)) return fail(CR_E_INVAL, "bad argument");
    if (p->bound) {
        CR_HIP(hipStreamSynchronize(p->stream));
        int rc = fold_timings(p);
        if (rc != CR_OK) return rc;
    }
    const std::vector<float> &v = p->samples[kernel];
    const int64_t n = std::min<int64_t>(capacity, static_cast<int64_t>(v.size()));
    std::copy(v.begin(), v.begin() + n, ms);
    *count = static_cast<int64_t>(v.size());
    return CR_OK;
}

int cr_probe_read_bandwidth(const void *src, size_t bytes, float *sink, int launches, void *hip_stream, double *gbps)
{
    if (!src || !sink || !gbps) return fail(CR_E_INVAL, "NULL argument");
    if (bytes < (size_t(1) << 20) || bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0)
        return fail(CR_E_INVAL, "src must be 16-byte aligned, bytes a multiple of 16 and at least 1 MiB");
    if (launches < 1 || launches > 1000) return fail(CR_E_INVAL, "launches must be 1..1000");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t start = nullptr, stop = nullptr;
    CR_HIP(hipEventCreate(&start));
    if (hipEventCreate(&stop) != hipSuccess) { (void)hipEventDestroy(start); return fail(CR_E_HIP, "hipEventCreate failed"); }
    hipError_t e = cr::launch_stream_read(src, bytes / 16, sink, stream);                 // warm-up
    if (e == hipSuccess) e = hipEventRecord(start, stream);
    for (int i = 0; i < launches && e == hipSuccess; ++i) e = cr::launch_stream_read(src, bytes / 16, sink, stream);
    if (e == hipSuccess) e = hipEventRecord(stop, stream);
    if (e == hipSuccess) e = hipEventSynchronize(stop);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, start, stop);
    (void)hipEventDestroy(start);
    (void)hipEventDestroy(stop);
    if (e != hipSuccess) return fail(CR_E_HIP, std::string("read-bandwidth probe: ") + hipGetErrorString(e));
    *gbps = static_cast<double>(bytes) * launches / (static_cast<double>(ms) * 1e-3) / 1e9;
    return CR_OK;
}

int cr_last_algorithmic_bytes(const cr_plan_t *p, int kernel, int64_t *bytes)
{
    if (!p || !bytes || kernel < 0 || kernel >= CR_K_COUNT) return fail(CR_E_INVAL, "bad argument");
    *bytes = p->bytes_last[kernel];
    return CR_OK;
}

int cr_synchronize(cr_plan_t *p)
{
    if (!p) return fail(CR_E_INVAL, "NULL plan");
    if (!p->bound) return fail(CR_E_INVAL, "no workspace bound");
    CR_HIP(hipStreamSynchronize(p->stream));
    return CR_OK;
}

}  // extern "C"

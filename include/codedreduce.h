/* CodedReduce (CR) gradient aggregation: the data-parallel hot path on one AMD MI355X (gfx950).
 *
 * All N workers of an (n,L)-regular tree are simulated on one GPU.  One iteration is
 *
 *     cr_partial_grads(X, y, w)   every worker's partial gradients over its allocated row segments
 *     cr_encode_tree(mask)        every non-straggling node's message, leaves first
 *     cr_decode_root(g)           the master's decode from any n-s of its n children
 *
 * and returns the exact full gradient  g = sum over all m data points of the per-point loss
 * gradient  (Section II-A, eq. (3)) whenever no sibling group has more than s stragglers.
 *
 * Notation: m data points (the paper's d), model dimension d (the paper's p), n children per
 * parent, L layers, s stragglers tolerated per sibling group, N = n + n^2 + ... + n^L workers.
 * Workers are numbered 0-based level by level: node (l,i), l in 1..L, i in 0..n^l-1, has id
 * n + ... + n^(l-1) + i and children (l+1, n*i + j), j in 0..n-1; sibling group g is ids [g*n, (g+1)*n),
 * group 0 being the master's children.
 *
 * Conventions for every call
 *   - plain C ABI; every function returns a cr_status (CR_OK = 0, negatives are errors); the text of the
 *     last error on the calling thread is available from cr_last_error().
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *   - the caller owns X, y, w, g and the workspace block; the library allocates no device memory and
 *     frees nothing it was handed.  A plan owns only host tables (and a few KB of pinned host staging
 *     once a workspace is bound).
 *   - device work is enqueued on the stream given to cr_bind_workspace and the call returns without
 *     waiting, unless stated otherwise.
 *   - a plan is not thread-safe; calls on one plan that overlap in time race.
 */
#ifndef CODEDREDUCE_H
#define CODEDREDUCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cr_plan_s cr_plan_t;

enum cr_status {
    CR_OK = 0,
    CR_E_INVAL = -1,        /* bad argument, unsupported size, workspace too small or not bound */
    CR_E_UNDECODABLE = -2,  /* some sibling group has more than s stragglers (remark after Theorem 1) */
    CR_E_STATE = -3,        /* call out of order: encode before gradients exist, decode before encode */
    CR_E_HIP = -4,          /* a HIP runtime call failed; see cr_last_error() */
    CR_E_NOMEM = -5         /* host allocation failed */
};

enum cr_model {
    CR_LINEAR = 0,          /* least squares:  per-point gradient x (x.w - y) */
    CR_LOGISTIC = 1,        /* logistic loss, targets y in {0,1}:  x (sigmoid(x.w) - y) */
    CR_AGGREGATE_ONLY = 2   /* no data matrix: partial gradients are supplied by cr_load_partial_grads */
};

enum cr_xdtype { CR_F32 = 0, CR_BF16 = 1 }; /* storage type of X only; y, w, g, slabs and messages are fp32 */

enum cr_kernel {            /* ids for cr_profile_read */
    CR_K_PARTIAL_GRADS = 0, CR_K_REDUCE_PIECES = 1, CR_K_ENCODE = 2, CR_K_DECODE = 3, CR_K_UPDATE = 4, CR_K_COUNT = 5
};

typedef struct cr_plan_info {
    int32_t L, n, s, model, x_dtype;
    int32_t num_workers;     /* N */
    int32_t num_groups;      /* N / n sibling groups */
    int32_t num_slabs;       /* S: (worker, segment) pairs; one d-float partial gradient each */
    int32_t num_decode_rows; /* F = C(n,s) */
    int32_t code_candidate;  /* index of the winning candidate of the code search; -1 if B was supplied; -2 fractional repetition */
    int32_t num_teams;       /* stage-1 work split (0 until known, see cr_plan_set_split) */
    int32_t num_pieces;      /* stage-1 partial rows (0 until the split is known) */
    int32_t split_kind;      /* enum cr_split of the split in force; -1 until it is known */
    int32_t stage1_team_size;       /* threads that share one row in the stage-1 kernel in force; 0: two-pass path for very wide rows */
    int32_t stage1_teams_per_group; /* teams (holders) per workgroup of that kernel */
    int32_t stage1_staged;   /* 1 if that kernel fetches rows once per workgroup into LDS */
    int64_t m, d;
    int64_t row_visits;      /* sum over workers of allocated rows */
    int64_t min_rows, max_rows; /* smallest / largest per-worker load; both equal r_CR m up to integer cuts (Theorem 1) */
    int64_t split_value;     /* teams (equal ranges) or rows per cell (row cells, shared cells); 0 until the split is known */
    double gamma;            /* max_f sum_i |a_fi| ||b_i||_2 / sqrt(n): rounding amplification of one decode.  Messages are fp32, so
                              * a decoded gradient carries a relative rounding error of about gamma^L * 2^-24 (see code_warning) */
    double r_cr;             /* computation load of Theorem 1 */
    int32_t l2_domains;      /* L2 cache domains (accelerator dies) the stage-1 split was laid out for: queried from the device when
                              * the split is fixed, 8 (MI355X) without a device */
    int32_t unit_slots;      /* workgroup slots (compute units, or twice that for short rows) of the shared-cells split; 0 otherwise */
    int32_t l2_sharing;      /* do workgroups whose ids are congruent modulo l2_domains run on the same die, as the row-cell and
                              * shared-cell splits assume?  1: checked on the device at cr_bind_workspace; 0: checked and NOT so
                              * (results stay exact, but every holder of a row then fetches it from HBM itself); -1: not checked
                              * (no workspace bound yet, or the split does not rely on it) */
    int32_t code_warning;    /* 1 if gamma^L * 2^-24 exceeds 1e-5, a tenth of the fp32 parity bar: the code is too badly
                              * conditioned for fp32 messages to be trusted to 1e-4 (wide groups with s+1 not dividing n) */
} cr_plan_info_t;

/* ---- plan (host only; Section III-A CR.Allocate, Algorithms 1 and 2, Section II-C for the code) ------------
 * cr_plan builds, on the host: the gradient-coding matrices B (n x n, cyclic support {i..i+s} mod n, unit-norm
 * rows; if the best cyclic candidate has gamma^L > 256 and s+1 divides n, the 0/1 fractional-repetition design
 * instead) and the decode rows a_f (a_f B = 1, zero on the straggler set); the recursive allocation of weighted row
 * segments to every node (CompAlloc with k = n parts cut at floor(kappa |W| / n); a node keeps the first
 * round(|W| / sum_{j=0}^{L-l} (n/(s+1))^j) positions of its sub-tree set, leaves keep all); and the slab list
 * (node-major, segments in allocation order).  cr_plan = cr_plan_ex with CR_LINEAR, CR_F32, the default seed, no B.
 *   seed         seeds the counter-based search for a well-conditioned code (ignored when B is given)
 *   B_or_null    host, n*n doubles row-major: use this encoding matrix (s+1 non-zeros in every row and column); or NULL
 *   out          receives the plan; destroy with cr_plan_destroy
 * Errors: CR_E_INVAL for L<1, L>8, n<2, n>64, s<0, s>=n, d<1, d>2^28 (any model), m<N, m>2^40, C(n,s) > 2^20, N > 2^24, an unsupported B. */
int cr_plan(int L, int n, int s, int64_t m, int64_t d, cr_plan_t **out);
int cr_plan_ex(int L, int n, int s, int64_t m, int64_t d, int model, int x_dtype, uint64_t seed,
               const double *B_or_null, cr_plan_t **out);
void cr_plan_destroy(cr_plan_t *plan);

/* ---- introspection (host; data for tests and harnesses) ------------------------------------------------------ */
int cr_plan_info(const cr_plan_t *plan, cr_plan_info_t *info);
int cr_plan_get_B(const cr_plan_t *plan, double *B /* host, n*n */);
int cr_plan_get_A(const cr_plan_t *plan, double *A /* host, F*n, row f = f-th straggler set in lexicographic order */);
/* The allocation (CR.Allocate, Algorithm 2): segment p = rows [row_begin[p], row_end[p]) of X, held by worker[p] with combining
 * coefficient coef[p]; segments are listed worker-major, in allocation order; each owns one slab (a d-float partial gradient), so
 * there are S = num_slabs of them.  Arrays of S entries, any may be NULL. */
int cr_plan_get_segments(const cr_plan_t *plan, int64_t *row_begin, int64_t *row_end, double *coef, int32_t *worker);
/* decode row for one sibling group (Section III-A, CR.Execute step 3): flags[j] != 0 marks child j a straggler.  With fewer than
 * s stragglers the set is padded with the highest-index survivors.  a: host, n doubles.  CR_E_UNDECODABLE if more than s are set. */
int cr_plan_decode_row(const cr_plan_t *plan, const uint8_t *flags /* host, n */, double *a);
/* Stage-1 work split into pieces (a piece = a run of one slab's rows handled by one team; it owns one d-float partial row).
 *   CR_SPLIT_EQUAL_RANGES  value = teams: the row visits of all slabs, slab-major, are cut into `teams` equal contiguous ranges,
 *                          cut again at slab boundaries.
 *   CR_SPLIT_ROW_CELLS     value = rows per cell: every slab is cut on one global grid of that many rows, one piece per team, teams
 *                          ordered by cell so that the holders of the same rows run at the same time.
 *   CR_SPLIT_SHARED_CELLS  value = most rows per cell: the grid is laid between slab boundaries, so every holder of a cell holds
 *                          all of it; 2, 3, 4 or 8 holders (by row width and by (s+1)^L, the most holders a row can have) share a
 *                          workgroup, which fetches each row once into LDS for all of them; each still does all of its own
 *                          arithmetic.  One workgroup per compute unit works through a queue of cells (a team then runs
 *                          several pieces).  fp32 rows of 257 to 3072 16-byte chunks with s > 0 only, else CR_E_INVAL.  Rows of
 *                          1537 to 2558 whole chunks (d a multiple of 4) held by 3 or more workers go straight from HBM into LDS
 *                          (no registers on the way in), 3, 4 or 6 holders per workgroup.  Rows that a single workgroup reads are
 *                          fetched with the non-temporal hint (they stream past the caches) when X has 1 GiB or more.
 * Default (when this is never called): with s = 0 (no row is held twice) equal ranges, one per resident workgroup; else shared
 * cells where that kernel exists and the problem has at least 16 rows per compute unit and workgroup, with the cell height
 * (16 to 1024 rows) that gives the shortest longest queue; else row cells of about 2 MB of X (96 to 512 rows, fewer for
 * small problems).  CR_E_STATE once a workspace is bound. */
enum cr_split { CR_SPLIT_EQUAL_RANGES = 0, CR_SPLIT_ROW_CELLS = 1, CR_SPLIT_SHARED_CELLS = 2 };
int cr_plan_set_split(cr_plan_t *plan, int kind, int64_t value);
/* pieces in execution order: piece i is rows [row_begin[i], row_end[i]) of slab[i], run by team[i]; num_pieces entries each, any may be NULL */
int cr_plan_get_pieces(const cr_plan_t *plan, int32_t *slab, int64_t *row_begin, int64_t *row_end, int32_t *team);

/* ---- run-time model (host only; Section III-C "Latency Performance", eq. (5), Theorem 2) ------------------------------------
 * Simulates iteration number `iteration` of the plan's tree: worker k, holding rows_k data points, computes for
 * a*rows_k + (rows_k/mu) * Exp(1) (the shifted-exponential law of eq. (5), drawn from the counter-based splitmix64 stream seeded
 * with `seed`, counter iteration*N + k); a parent receives one message at a time, in order of readiness, t_c per message, and
 * decodes after n-s of them; all nodes compute from time 0 and while receiving.
 *   mask   host, N bytes or NULL: 1 for the s children of every group that were not waited for (usable by cr_encode_tree)
 *   ready  host, N doubles or NULL: time each node's message is ready to send
 *   total  host or NULL: time at which the master has decoded
 * CR_E_INVAL unless a >= 0, mu > 0, t_c >= 0, iteration >= 0. */
int cr_simulate_iteration(const cr_plan_t *plan, double a, double mu, double t_c, uint64_t seed, int64_t iteration,
                          uint8_t *mask, double *ready, double *total);

/* ---- device binding --------------------------------------------------------------------------------------------
 * The workspace holds the device tables, 16 encode programs, the stage-1 piece partials, the slab gradients
 * G[S][d] (not for CR_AGGREGATE_ONLY) and the messages M[N][d], all fp32 rows of d floats.  dev_ptr must be 256-byte aligned and stay valid while the plan
 * is used; hip_stream is a hipStream_t (NULL = the default stream).  cr_bind_workspace copies the tables synchronously. */
int cr_workspace_bytes(cr_plan_t *plan, size_t *bytes);
int cr_bind_workspace(cr_plan_t *plan, void *dev_ptr, size_t bytes, void *hip_stream);

/* ---- the hot path ------------------------------------------------------------------------------------------------
 * cr_partial_grads (CR.Execute step 1): for every slab p,  G[p] = X[b:e]^T (phi(X[b:e] w) - y[b:e]),  phi = identity or sigmoid.
 *   X_dev  m x d row-major, contiguous, fp32 or bf16 per the plan, 16-byte aligned;  y_dev m floats;  w_dev d floats.
 *   Every holder of a row does all of its own arithmetic on it (the redundancy is the method) in one pass over its rows, as long
 *   as a row fits the registers of one team (d <= 24576, whether or not d is a multiple of the 16-byte chunk); wider rows take
 *   two passes.  Holders of the same rows are scheduled together, so that one fetch from HBM serves them all: through the L2
 *   (row cells) or, with shared cells, once per workgroup through LDS (see cr_plan_set_split).
 * cr_load_partial_grads: use caller-supplied slab gradients G_dev[S][d] (fp32, 16-byte aligned) in place of stage 1;
 *   the buffer is read in place by cr_encode_tree and must stay valid until then.
 * cr_encode_tree (CR.Execute steps 2-5): mask is HOST memory, N bytes, non-zero = straggler.  For every non-straggler node,
 *   m_(l,i) = sum_p coef_p G[p] over its slabs  +  sum_j a_j m_(l+1, n i + j)  with a = the decode row of its children group.
 *   Stragglers write no message (their row of M keeps stale data); all other nodes do, also below a straggler.
 *   CR_E_UNDECODABLE, before anything is enqueued and with no state change, if any group has more than s stragglers.
 * cr_decode_root (the last step of CR.Execute, Algorithm 2: the master recovers g from any n-s of its children):
 *   g_dev[d] = sum_j a_j m_(1,j) with the decode row of group 0 from the last cr_encode_tree; by eq. (3) this is the full gradient.
 * cr_gd_update: w <- w - lr * g (plain gradient step used by the benchmark loop).
 * Errors: CR_E_STATE out of order; CR_E_INVAL unbound workspace / NULL / misaligned pointers; CR_E_HIP launch failures. */
int cr_partial_grads(cr_plan_t *plan, const void *X_dev, const float *y_dev, const float *w_dev);
int cr_load_partial_grads(cr_plan_t *plan, const float *G_dev);
int cr_encode_tree(cr_plan_t *plan, const uint8_t *straggler_mask_host);
int cr_decode_root(cr_plan_t *plan, float *g_dev);
int cr_gd_update(cr_plan_t *plan, float *w_dev, const float *g_dev, float lr);

/* Gradient descent loop kept on the device (eq. (2) with a plain step): `steps` times  g = CodedReduce(w);  w <- w - lr g,  enqueued
 * back to back.  The encode programs of 16 steps at a time travel to the device in one copy, so a step is kernel launches only; the
 * host waits only when it runs more than 32 steps ahead of the copies (two pinned staging batches).
 *   masks_host      steps x N bytes, one straggler mask per step; all are checked first: CR_E_UNDECODABLE before anything is enqueued
 *   w_dev, g_dev    d floats each; w is updated in place, g holds the last decoded gradient
 *   w_star_or_null  d floats (device): the reference model of the normalised error rate, or NULL
 *   metrics_or_null device, steps x 2 floats: [2t] = ||w_t+1 - w_t||^2 / ||w_t||^2 (relative error rate, eq. (6)),
 *                   [2t+1] = ||w_t+1 - w*||^2 / ||w*||^2 (normalised error rate, eq. (8); -1 without w*); NULL = plain update,
 *                   which then rides in the decode launch (the same arithmetic as cr_gd_update, one launch fewer per step) */
int cr_gd_run(cr_plan_t *plan, const void *X_dev, const float *y_dev, float *w_dev, float *g_dev, const uint8_t *masks_host,
              int steps, float lr, const float *w_star_or_null, float *metrics_or_null);

/* Aggregation alone, many masks in one call (CR.Execute steps 2 to the end, Algorithm 2, once per mask): step t encodes the slab
 * gradients at G_dev + t * G_step_stride under masks_host[t] and decodes into g_dev + t * g_step_stride; like cr_load_partial_grads,
 * cr_encode_tree and cr_decode_root called in turn (the same bits), but with the programs of 16 steps per host-to-device copy.
 *   G_dev          device, S x d floats per step, 16-byte aligned; G_step_stride in floats (a multiple of 4): 0 = the same slabs every step
 *   masks_host     steps x N bytes; all are checked first: CR_E_UNDECODABLE before anything is enqueued
 *   g_dev          device, d floats per step; g_step_stride in floats: 0 = every step overwrites the same vector
 * Afterwards the plan is in the state the last step's three calls would have left (messages of the last mask). */
int cr_aggregate_run(cr_plan_t *plan, const float *G_dev, int64_t G_step_stride, const uint8_t *masks_host, int steps, float *g_dev,
                     int64_t g_step_stride);

/* ---- aggregation without any allocation ----------------------------------------------------------------------------------------
 * For callers that cannot allocate or bind device memory: code under HIP stream capture, tight serving loops, harnesses that forbid
 * hipMalloc.  cr_aggregate_static is cr_load_partial_grads + cr_encode_tree + cr_decode_root in one call, with everything those
 * keep in a workspace -- the per-call encode program and the messages M[N][d] -- held in a device array that is part of the library
 * itself (CR_STATIC_SCRATCH_BYTES; each GPU the library runs on holds one until the process ends).  The plan needs no workspace.
 * The call allocates and frees nothing on the device or in pinned memory and records no copy: the program reaches the device as
 * kernel arguments, so all it enqueues on hip_stream is kernel launches (a handful of small ones, encode, decode).
 *   plan        any plan; its model is not consulted (no stage 1 runs)
 *   G_dev       device, S x d floats, 16-byte aligned: the slab gradients, read in place
 *   mask_host   host, N bytes, non-zero = straggler; read before the call returns
 *   g_dev       device, d floats: receives the decoded gradient (the same bits cr_decode_root gives for the same G and mask)
 *   hip_stream  a hipStream_t (NULL = the default stream)
 * Limits: the messages must fit, N * d * 4 <= CR_STATIC_SCRATCH_BYTES - 64 KiB (the paper's network, 156 workers x 117 706
 * parameters, does), and the encode program (28 bytes per slab and per worker) must fit 64 KiB: CR_E_INVAL otherwise, before
 * anything is enqueued.  CR_E_UNDECODABLE as for cr_encode_tree.  All calls on one GPU share that GPU's array, whatever the plan:
 * calls that overlap in time on one GPU (two streams, two threads) race.  The array keeps the previous call's contents; nothing
 * in it needs clearing, since every message row that is read was written earlier in the same call. */
#define CR_STATIC_SCRATCH_BYTES ((size_t)96 << 20)
int cr_aggregate_static(cr_plan_t *plan, const float *G_dev, const uint8_t *mask_host, float *g_dev, void *hip_stream);

/* ---- results kept in the workspace (device pointers, valid while the workspace is) --------------------------- */
int cr_get_slab_grads(const cr_plan_t *plan, const float **G_dev); /* S x d */
int cr_get_messages(const cr_plan_t *plan, const float **M_dev);   /* N x d, row = worker id */

/* ==== instrumentation: measurement plumbing for benchmarks and tests; no step of the method needs any of it ================
 * cr_profile_enable(plan, kernels): bit k of `kernels` set = every launch of kernel id k is bracketed by two HIP events on the
 * bound stream from now on (CR_PROFILE_ALL: all of them, 0: none); a non-zero call also clears the totals.  Each bracket costs
 * a few microseconds of device time, which shows on small problems.  cr_profile_read waits for the stream, then returns for one
 * kernel id the summed duration, the number of launches and the algorithmic bytes of those launches (bytes the method must
 * move: rows read once per holder, each result written once) since the last non-zero cr_profile_enable; any may be NULL.
 * Totals read after cr_profile_enable(plan, 0) are those gathered until then. */
#define CR_PROFILE_ALL ((1 << CR_K_COUNT) - 1)
int cr_profile_enable(cr_plan_t *plan, int kernels);
int cr_profile_read(cr_plan_t *plan, int kernel, double *total_ms, int64_t *launches, int64_t *algorithmic_bytes);
/* the duration in milliseconds of every single timed launch of one kernel id since the last non-zero cr_profile_enable, in launch
 * order (the first 65536 of them): up to `capacity` values are copied to ms (host), *count receives how many there are; waits for
 * the stream like cr_profile_read */
int cr_profile_samples(cr_plan_t *plan, int kernel, float *ms, int64_t capacity, int64_t *count);
/* algorithmic bytes of the most recent launch of a kernel id (0 if none yet) */
int cr_last_algorithmic_bytes(const cr_plan_t *plan, int kernel, int64_t *bytes);
int cr_synchronize(cr_plan_t *plan); /* wait for the bound stream */
/* What a plain streaming read reaches on this device: `launches` launches of a kernel that only reads src_dev[0 .. bytes) with
 * 16-byte loads (every workgroup sums what it reads into sink_dev so that nothing is optimised away), timed with HIP events on the
 * given stream; the call waits for them.  A yardstick for the traffic figures of the hot path, not part of it.
 *   src_dev   device, 16-byte aligned, bytes a multiple of 16 and at least 1 MiB;  sink_dev  device, at least 16384 floats
 *   gbps      receives bytes * launches / elapsed in GB/s (the first launch is a warm-up and not timed) */
int cr_probe_read_bandwidth(const void *src_dev, size_t bytes, float *sink_dev, int launches, void *hip_stream, double *gbps);

const char *cr_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CODEDREDUCE_H */

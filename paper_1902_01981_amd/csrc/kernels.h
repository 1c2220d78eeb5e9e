// Device-side tables and kernel launchers of the CodedReduce hot path (gfx950).  Host code sees only plain launch functions.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace cr {

struct DevPiece {            // one stage-1 work item: rows [row_begin, row_begin + nrows) of X, partial row = index of the piece
    int64_t row_begin;
    int64_t visit_begin;     // index of the piece's first row among all row visits, piece-major (wide-row path: where its residuals live)
    int32_t nrows;
    int32_t slab;
    int32_t shared;          // 1: other workgroups fetch these rows at the same time, so the fetch should leave them in the L2
    int32_t reserved;
};

// Encode program: a post-order list of terms, stored as parallel arrays so that a wavefront fetches kEncodeUnroll terms with a few
// wide scalar loads.  Term t:  own += coef[t] * G[slab[t]];  if level[t] > 0 the term is the last of a node at that level:
// message = own + pending[level], stored to M[row[t]] and folded into pending[level-1] with acoef[t]; own = 0.
struct EncProgram {
    const int32_t *slab;
    const int32_t *level;
    const int32_t *row;
    const double *coef;
    const double *acoef;
    const int32_t *sub_begin;    // first term of each sub-program, a multiple of kEncodeUnroll
    const int32_t *sub_end;      // one past its last real term; no-op terms pad it up to the next multiple of kEncodeUnroll
};

struct DecTerm {             // g += coef * M[row]
    int32_t row;
    int32_t pad;
    double coef;
};

constexpr int kEncodeUnroll = 8;   // encode sub-programs are padded to a multiple of this many terms
constexpr int kMaxLevels = 8;

// Stage-1 kernel variant chosen for (x_dtype, d): team size, chunks per thread, rows per step, teams per workgroup.
// A `staged` variant fetches each row once per workgroup into LDS, from where all its teams (holders of the same rows) read it.
struct Stage1Variant {
    int xd, vec, team_size, k, rows, tpb;
    bool staged;
    const void *fn[2];               // phi = identity, phi = sigmoid
    int ring = 0;                    // > 0: rows reach LDS by direct global-to-LDS loads into a ring of `ring` rows
    int w_in_lds = 0;                // 1: the weights sit in LDS behind the ring (one more row of LDS)
    const void *fn_buffers[2] = {nullptr, nullptr};   // the same kernel fetching rows with buffer loads (see launch_partial_grads)
    int holders_per_team = 1;        // 2: every team of threads works for two of the tpb holders of an item, one after the other
    int block() const { return team_size * tpb / holders_per_team; }
    int teams_per_block() const { return tpb; }
    // dynamic LDS the launch needs for rows of d columns (0 for variants that keep rows in registers only)
    size_t lds_bytes(int64_t d) const;
};

constexpr size_t kLdsPerWorkgroup = 160 * 1024;   // gfx950

// Returns nullptr if (x_dtype, d) is outside what the single-pass register kernels cover.
const Stage1Variant *select_stage1(int x_dtype, int64_t d);
// The LDS-staged kernel for rows held by up to max_holders workers each, or nullptr if there is none for this type and width.
// Rows of 1537 to 2558 whole 16-byte chunks (fp32, d a multiple of 4) held by three or more workers get the kernel that loads
// straight into LDS, three or four holders per workgroup.
const Stage1Variant *select_stage1_staged(int x_dtype, int64_t d, int64_t max_holders);
// Once per variant and device before the first launch (raises the kernel's dynamic LDS limit where needed).
hipError_t prepare_stage1(const Stage1Variant &v, int64_t d);

// rows_as_buffers: every row starts on a 4-byte boundary and every piece has fewer than 2^31 bytes; variants that have a
// buffer-load twin (bf16 rows, one wavefront per team) then run it
hipError_t launch_partial_grads(const Stage1Variant &v, const void *X, const float *y, const float *w, const DevPiece *pieces,
                                const int32_t *team_piece_begin, int num_teams, float *partial, int64_t d, int logistic,
                                bool rows_as_buffers, hipStream_t stream);
// Staged variants: workgroup g works through items [group_item_begin[g], group_item_begin[g+1]); item i hands team t of the
// workgroup the piece item_pieces[i * teams_per_block + t] (or -1); all pieces of an item cover the same rows.
hipError_t launch_partial_grads_staged(const Stage1Variant &v, const void *X, const float *y, const float *w, const DevPiece *pieces,
                                       const int32_t *group_item_begin, const int32_t *item_pieces, int num_groups, float *partial,
                                       int64_t d, int logistic, hipStream_t stream);
// Wide rows (a row does not fit the registers of one team): two passes.  launch_residuals writes phi(x.w) - y for every row visit,
// launch_xt_residuals forms X^T r per piece and block of 256*kWideChunks*vec columns.  X is read twice on this path.
constexpr int kWideChunks = 8;
hipError_t launch_residuals(int x_dtype, const void *X, const float *y, const float *w, const DevPiece *pieces, int num_pieces,
                            float *residuals, int64_t d, int logistic, hipStream_t stream);
hipError_t launch_xt_residuals(int x_dtype, const void *X, const DevPiece *pieces, int num_pieces, const float *residuals, float *partial,
                               int64_t d, hipStream_t stream);
hipError_t launch_reduce_pieces(const float *partial, const int32_t *slab_piece_begin, const int32_t *slab_pieces, int num_slabs, float *G, int64_t d,
                                hipStream_t stream);
hipError_t launch_encode(const float *G, float *M, const EncProgram &prog, int num_sub, int L, int64_t d, hipStream_t stream);
// w != nullptr: also steps w <- w - lr g (g as stored, rounded to fp32) in the same launch
hipError_t launch_decode(const float *M, float *g, const DecTerm *terms, int nterms, int64_t d, float *w, float lr, hipStream_t stream);
hipError_t launch_update(float *w, const float *g, float lr, int64_t d, hipStream_t stream);
// plain streaming read of n16 16-byte words; every workgroup writes its sum to sink[workgroup] (kStreamGroups workgroups)
constexpr int kStreamGroups = 256 * 8;
hipError_t launch_stream_read(const void *src, size_t n16, float *sink, hipStream_t stream);
// ---- the library's own device memory, for callers that cannot allocate -------------------------------------------------------
// A file-scope device array of kStaticScratchBytes (every GPU the library runs on holds its own copy until the process ends).
// static_scratch returns its address on the CURRENT device (looked up once per device, no allocation) in *ptr.
constexpr size_t kStaticProgramBytes = size_t(64) << 10;                 // head of the array: one encode program
constexpr size_t kStaticScratchBytes = size_t(96) << 20;                 // the whole array; messages follow the program
hipError_t static_scratch(char **ptr);
// copies `bytes` (a multiple of 4) from host memory to the device address dst through kernel arguments: launches only, no
// staging buffer, no memcpy node; the host bytes are consumed before the call returns
hipError_t launch_upload(char *dst, const char *src_host, size_t bytes, hipStream_t stream);

// one wavefront per workgroup; out[workgroup id] = (die the workgroup ran on) << 16 | (shader engine and compute unit inside the die)
hipError_t launch_placement_probe(uint32_t *out, int groups, hipStream_t stream);
hipError_t launch_update_metrics(float *w, const float *g, float lr, const float *w_star, float *metrics, int64_t d, hipStream_t stream);

}  // namespace cr

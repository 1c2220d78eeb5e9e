// HIP kernels of the CodedReduce hot path for gfx950 (64-wide wavefronts).  Everything here is bandwidth bound (stage 1 on bf16
// rows: bound by vector-ALU issue): plain vector FMAs, 16-byte coalesced loads, no matrix cores.
//
//   partial_grads_kernel   CR.Execute step 1: G_piece = X[b:e]^T (phi(X[b:e] w) - y[b:e]) in ONE pass over the rows
//   partial_grads_staged_kernel   the same, with the rows fetched once per workgroup into LDS for several holders of those rows
//   partial_grads_dma_kernel      the same, with the rows loaded from global memory straight into LDS (no registers on the way)
//   residuals_kernel, xt_residuals_kernel   the same in two passes, for rows too wide for one team's registers
//   reduce_pieces_kernel   sums the pieces of each slab (fixed order, so results are reproducible bit for bit)
//   encode_kernel          CR.Execute steps 2-5: every node's message, children folded into parents in registers
//   decode_kernel          the master's decode  g = sum_j a_j m_(1,j), optionally followed by w <- w - lr g in the same launch
//   update_kernel, update_metrics_kernel    w <- w - lr g, optionally with the convergence measures of eq. (6) and (8)
//
// Rows of d elements start on a 4-byte (fp32) or 2-byte (bf16) boundary whatever d is, so the 16-byte row accesses are declared
// with that alignment; the hardware runs in unaligned-access mode and the compiler emits the same dwordx4 instructions.
// A row is cut into nq = ceil(d / VEC) chunks of VEC columns; when VEC does not divide d the last chunk is moved back to end at
// column d, overlapping its neighbour.  Overlapped columns are then produced twice, from the same operands in the same order,
// and both copies store the same bits; only sums ACROSS columns (the dot product x.w) must count them once.
#include "kernels.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstring>
#include <type_traits>

namespace cr {

namespace {

typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));       // four floats of an fp32 row
typedef unsigned u4h __attribute__((ext_vector_type(4), aligned(2)));    // eight bf16 values of a bf16 row
typedef float f4a __attribute__((ext_vector_type(4)));                   // the same chunks parked in LDS, 16-byte aligned there
typedef unsigned u4a __attribute__((ext_vector_type(4)));

// v + (v of the lane that the cross-lane pattern CTRL pairs this lane with, inside its row of 16 lanes)
template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Sum over the 64 lanes, delivered to every lane.  The four steps inside a row of 16 lanes are adds that read the partner lane
// directly (quad swaps, then the mirrored half-row and row: for a sum a mirror does what an exchange does).  The two steps across
// rows either go through the LDS crossbar (2 adds + 2 LDS operations), or pass lane 15 / lane 31 on to the following rows so
// that lane 63 ends with the total, which is then read into a scalar register (5 vector operations, no LDS round trip).
// Kernels limited by vector-ALU issue (bf16 rows: a widening operation per element on top of the two multiply-adds) take the
// first form, kernels limited by cache bandwidth and latency (fp32 rows) the second.
template <bool VIA_LDS> __device__ __forceinline__ float wave_sum(float v)
{
    v = dpp_add<0xB1>(v);      // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);      // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);     // row_half_mirror
    v = dpp_add<0x140>(v);     // row_mirror
    if constexpr (VIA_LDS) {
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        return v;
    } else {
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x142, 0xa, 0xf, false));   // row_bcast:15 into rows 1 and 3
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x143, 0xc, 0xf, false));   // row_bcast:31 into rows 2 and 3
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
    }
}

// The same for four rows at once, at less than half the vector instructions: a transposing butterfly.  After the first two steps
// (lane pairs, then pairs of pairs, each lane keeping the row its position selects and handing the other to its partner) lane l
// holds the sum over its quad of row l & 3; two rotations inside the row of 16 lanes and two exchanges across rows finish the sums,
// and lanes 0..3 hold the four totals.  13 vector operations, 2 LDS exchanges and 4 lane reads for four rows, where four single
// sums take about 44.
// wave_sum4_lanes leaves the totals in the lanes (lane l holds the total of row l & 3); wave_sum4 reads them into scalars.
__device__ __forceinline__ float wave_sum4_lanes(const float (&s)[4])
{
    const unsigned lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const bool b0 = lane & 1u, b1 = lane & 2u;
    // lanes with b0 = 0 keep rows 0 and 2, the others rows 1 and 3
    float t01 = (b0 ? s[1] : s[0]) + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(b0 ? s[0] : s[1]), 0xB1, 0xf, 0xf, false));
    float t23 = (b0 ? s[3] : s[2]) + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(b0 ? s[2] : s[3]), 0xB1, 0xf, 0xf, false));
    // lanes with b1 = 0 keep rows 0/1, the others rows 2/3
    float u = (b1 ? t23 : t01) + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(b1 ? t01 : t23), 0x4E, 0xf, 0xf, false));
    u += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(u), 0x124, 0xf, 0xf, false));      // row_ror:4
    u += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(u), 0x128, 0xf, 0xf, false));      // row_ror:8
    u += __shfl_xor(u, 16, 64);
    u += __shfl_xor(u, 32, 64);
    return u;
}
__device__ __forceinline__ void wave_sum4(const float (&s)[4], float (&out)[4])
{
    const float u = wave_sum4_lanes(s);
#pragma unroll
    for (int r = 0; r < 4; ++r) out[r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(u), r));
}

// 1 / (1 + e^-z) from the hardware exponential and reciprocal (each good to about one unit in the last place); it saturates to
// 0 and 1 for large |z| without special cases
__device__ __forceinline__ float sigmoid(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

// element offset of chunk q inside a row (a chunk index past the row is sent to the last chunk)
template <int VEC> __device__ __forceinline__ int chunk_offset(int q, int nq, int d)
{
    return q < nq - 1 ? q * VEC : d - VEC;
}
// does element v of chunk q belong to it alone (not to the overlap with the chunk before, not past the row)?
template <int VEC> __device__ __forceinline__ bool chunk_owns(int q, int v, int nq, int d)
{
    return q < nq - 1 || (q == nq - 1 && d - VEC + v >= (nq - 1) * VEC);
}

// ---- how a chunk of a row of X is fetched and widened to fp32 -------------------------------------------------
// load(row, e): the chunk at element e of the row that starts at `row` (a wave-uniform pointer; e differs per lane);
// load_once: the same for rows nobody else reads, with the non-temporal hint, so that they stream past the caches
template <int XD, int VEC> struct Chunk;
template <int XD> __device__ __forceinline__ const void *row_ptr(const void *X, int64_t row, int d)
{
    return static_cast<const char *>(X) + row * d * (XD == 1 ? 2 : 4);
}

template <> struct Chunk<0, 4> {
    using raw_t = f4u;
    using lds_t = f4a;
    static __device__ __forceinline__ raw_t load(const void *row, unsigned e) { return *reinterpret_cast<const f4u *>(static_cast<const char *>(row) + e * 4u); }
    static __device__ __forceinline__ raw_t load_once(const void *row, unsigned e) { return __builtin_nontemporal_load(reinterpret_cast<const f4u *>(static_cast<const char *>(row) + e * 4u)); }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&v)[4]) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
};
template <> struct Chunk<1, 8> {
    using raw_t = u4h;
    using lds_t = u4a;
    static __device__ __forceinline__ raw_t load(const void *row, unsigned e) { return *reinterpret_cast<const u4h *>(static_cast<const char *>(row) + e * 2u); }
    static __device__ __forceinline__ raw_t load_once(const void *row, unsigned e) { return __builtin_nontemporal_load(reinterpret_cast<const u4h *>(static_cast<const char *>(row) + e * 2u)); }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&v)[8])
    {
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
        v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
        v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
    }
};
template <> struct Chunk<0, 1> {      // rows shorter than one wide chunk
    using raw_t = float;
    static __device__ __forceinline__ raw_t load(const void *row, unsigned e) { return *reinterpret_cast<const float *>(static_cast<const char *>(row) + e * 4u); }
    static __device__ __forceinline__ raw_t load_once(const void *row, unsigned e) { return __builtin_nontemporal_load(reinterpret_cast<const float *>(static_cast<const char *>(row) + e * 4u)); }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&v)[1]) { v[0] = r; }
};
template <> struct Chunk<1, 1> {
    using raw_t = uint16_t;
    static __device__ __forceinline__ raw_t load(const void *row, unsigned e) { return *reinterpret_cast<const uint16_t *>(static_cast<const char *>(row) + e * 2u); }
    static __device__ __forceinline__ raw_t load_once(const void *row, unsigned e) { return __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(static_cast<const char *>(row) + e * 2u)); }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&v)[1]) { v[0] = __uint_as_float(static_cast<uint32_t>(r) << 16); }
};

// VEC consecutive floats of an fp32 row (slab gradients, piece partials, messages)
template <int VEC> __device__ __forceinline__ void load_row(const float *src, float (&v)[VEC])
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) { const f4u t = *reinterpret_cast<const f4u *>(src + i); v[i] = t.x; v[i + 1] = t.y; v[i + 2] = t.z; v[i + 3] = t.w; }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = src[i];
    }
}
template <int VEC> __device__ __forceinline__ void load_row_nt(const float *src, float (&v)[VEC])
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) { const f4u t = __builtin_nontemporal_load(reinterpret_cast<const f4u *>(src + i)); v[i] = t.x; v[i + 1] = t.y; v[i + 2] = t.z; v[i + 3] = t.w; }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = __builtin_nontemporal_load(src + i);
    }
}
template <int VEC> __device__ __forceinline__ void store_row(float *dst, const float (&v)[VEC])
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) { f4u t; t.x = v[i]; t.y = v[i + 1]; t.z = v[i + 2]; t.w = v[i + 3]; *reinterpret_cast<f4u *>(dst + i) = t; }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) dst[i] = v[i];
    }
}
template <int VEC> __device__ __forceinline__ void store_row_nt(float *dst, const float (&v)[VEC])
{
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) { f4u t; t.x = v[i]; t.y = v[i + 1]; t.z = v[i + 2]; t.w = v[i + 3]; __builtin_nontemporal_store(t, reinterpret_cast<f4u *>(dst + i)); }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) __builtin_nontemporal_store(v[i], dst + i);
    }
}

// ---- stage 1 ------------------------------------------------------------------------------------------------------
// A team of TS threads owns whole rows: thread t holds chunks t, t+TS, ... (K of them, VEC columns each) of every row it
// works on, so a row is fetched once, used for the dot product x.w, kept in registers, and used again for the rank-1 update
// acc += (phi(x.w) - y) x.  R rows are in flight per step.  The dot is reduced inside the wavefront and, for teams of several
// wavefronts, through LDS (double buffered: one barrier per step).  Each piece ends with one d-float store of the accumulators.
template <int XD, int VEC, int TS, int K, int R, bool LOGISTIC, bool BUF = false>
__global__ void __launch_bounds__((TS < 256 ? 256 : TS))
partial_grads_kernel(const void *__restrict__ X, const float *__restrict__ y, const float *__restrict__ w,
                     const DevPiece *__restrict__ pieces, const int32_t *__restrict__ team_piece_begin, int num_teams,
                     float *__restrict__ partial, int d, int nq)
{
    using C = Chunk<XD, VEC>;
    using raw_t = typename C::raw_t;
    constexpr int BLOCK = TS < 256 ? 256 : TS;
    constexpr int WAVES = TS / 64;
    const int tl = threadIdx.x % TS;
    // the team index is the same for every lane of a wavefront: keep it (and all that derives from it) in scalar registers
    const int team = __builtin_amdgcn_readfirstlane(blockIdx.x * (BLOCK / TS) + threadIdx.x / TS);
    __shared__ float red[2][R][WAVES];
    if (team >= num_teams) return;   // whole teams only; teams of several wavefronts span the block, so barriers stay uniform

    // K = ceil(nq / TS): only the last chunk of a thread can fall outside the row.  Such a lane re-reads the row's last chunk
    // (so every load is unconditional) with zero weights, and never stores its accumulator.
    unsigned off[K];
    float wv[K][VEC];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int q = tl + k * TS;
        off[k] = chunk_offset<VEC>(q, nq, d);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const float t = w[off[k] + v];               // always inside the row; masked after the load
            wv[k][v] = chunk_owns<VEC>(q, v, nq, d) ? t : 0.f;
        }
    }

    const int lane3 = tl & 3;
    const int pb = team_piece_begin[team], pe = team_piece_begin[team + 1];
    int buf = 0;
    for (int p = pb; p < pe; ++p) {
        const DevPiece pc = pieces[p];
        float acc[K][VEC];
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[k][v] = 0.f;

        // BUF (chosen by the host where every row starts on a 4-byte boundary and every piece has fewer than 2^31 bytes): the
        // piece's rows as a buffer -- base, size in bytes, plain 32-bit words
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(row_ptr<XD>(X, pc.row_begin, d)), 0,
                                                                                 BUF ? pc.nrows * d * (XD == 1 ? 2 : 4) : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(y + pc.row_begin), 0, BUF ? pc.nrows * 4 : 0, 0x00020000);
        for (int r0 = 0; r0 < pc.nrows; r0 += R) {
            raw_t xr[R][K];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int rr = min(r0 + r, pc.nrows - 1);          // rows past the end re-read the last row; their residual is zeroed
                const void *row = row_ptr<XD>(X, pc.row_begin + rr, d);
                if constexpr (BUF) {
                    // bf16 rows (bound by vector-ALU issue): a buffer load takes the piece's base and the row's offset as scalars
                    // and the lane's offset as it is, where a global load costs a 64-bit vector add per load
                    const unsigned soff = static_cast<unsigned>(rr) * static_cast<unsigned>(d) * (XD == 1 ? 2u : 4u);
#pragma unroll
                    for (int k = 0; k < K; ++k)
                        xr[r][k] = __builtin_bit_cast(raw_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off[k] * (XD == 1 ? 2u : 4u), soff, 0));
                } else if (XD == 1 || pc.shared) {
                    // fp32 rows that other holders read too are left in the L2; bf16 rows always are (that path is bound by the
                    // vector ALUs, and a second copy of its loop costs more than streaming gains)
#pragma unroll
                    for (int k = 0; k < K; ++k) xr[r][k] = C::load(row, off[k]);
                } else {
                    asm volatile("; rows read once" ::: "memory");   // (the markers keep the two kinds of load from being merged into one)
#pragma unroll
                    for (int k = 0; k < K; ++k) xr[r][k] = C::load_once(row, off[k]);
                    asm volatile("; rows read once" ::: "memory");
                }
            }
            float pd[R], res_of[R];
            if constexpr (XD == 1 && R % 4 == 0) {
                // bf16 rows are bound by vector-ALU issue: the cross-lane sums of four rows are taken together
#pragma unroll
                for (int r0b = 0; r0b < R; r0b += 4) {
                    float s4[4], t4[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float s = 0.f;
#pragma unroll
                        for (int k = 0; k < K; ++k) {
                            float xv[VEC];
                            C::widen(xr[r0b + r][k], xv);
#pragma unroll
                            for (int v = 0; v < VEC; ++v) s = fmaf(xv[v], wv[k][v], s);
                        }
                        s4[r] = s;
                    }
                    if constexpr (BUF && WAVES == 1) {
                        // the residuals of the four rows in one go, in the lanes that hold the totals: lane l has the target of row
                        // l & 3 (one 4-byte buffer load per lane; past the piece's end it returns 0 and the row counts for nothing)
                        const float u = wave_sum4_lanes(s4);
                        const float yv = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc_y, lane3 * 4, (r0 + r0b) * 4, 0));
                        const float ph = LOGISTIC ? sigmoid(u) : u;
                        const float rv = lane3 < pc.nrows - (r0 + r0b) ? ph - yv : 0.f;
#pragma unroll
                        for (int r = 0; r < 4; ++r) res_of[r0b + r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(rv), r));
                    } else {
                        wave_sum4(s4, t4);
#pragma unroll
                        for (int r = 0; r < 4; ++r) pd[r0b + r] = t4[r];
                    }
                }
            } else {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    float xv[VEC];
                    C::widen(xr[r][k], xv);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) s = fmaf(xv[v], wv[k][v], s);
                }
                pd[r] = wave_sum<XD == 1>(s);
            }
            }
            if constexpr (WAVES > 1) {
                const int wave = tl / 64;
                if ((tl & 63) == 0) {
#pragma unroll
                    for (int r = 0; r < R; ++r) red[buf][r][wave] = pd[r];
                }
                __syncthreads();
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float s = 0.f;
#pragma unroll
                    for (int wv_i = 0; wv_i < WAVES; ++wv_i) s += red[buf][r][wv_i];
                    pd[r] = s;
                }
                buf ^= 1;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int rr = r0 + r;
                float res;
                if constexpr (BUF && XD == 1 && R % 4 == 0 && WAVES == 1) res = res_of[r];
                else {
                    const float yy = y[pc.row_begin + min(rr, pc.nrows - 1)];
                    const float z = pd[r];
                    const float ph = LOGISTIC ? sigmoid(z) : z;
                    res = (rr < pc.nrows) ? ph - yy : 0.f;
                }
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    float xv[VEC];
                    C::widen(xr[r][k], xv);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[k][v] = fmaf(res, xv[v], acc[k][v]);
                }
            }
        }
        float *out = partial + static_cast<int64_t>(p) * d;
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (tl + k * TS < nq) store_row<VEC>(out + off[k], acc[k]);
    }
}

// ---- stage 1 with rows staged through LDS -----------------------------------------------------------------------------
// The holders of a cell run the same rows.  Here H of them share a workgroup: its H*TS threads fetch every row once, pass it
// through registers into LDS, and each team then reads the row from LDS and does its own dot product, residual and rank-1 update
// exactly as above.  The L2 therefore serves a row once per workgroup instead of once per holder.
// Software pipeline, one barrier per step of R rows: while step s is computed from one LDS buffer, step s+1 moves from registers
// into the other buffer and the global loads of steps s+2 and s+3 are in flight in two register sets.
// One workgroup per compute unit works through a queue of items (an item = one cell for up to H of its holders); all pieces of
// an item must cover the same rows (cells cut at slab boundaries).  The weights are loaded once per workgroup.
template <int XD, int VEC, int TS, int K, int R, int H, bool LOGISTIC>
__global__ void __launch_bounds__(TS * H)
partial_grads_staged_kernel(const void *__restrict__ X, const float *__restrict__ y, const float *__restrict__ w,
                            const DevPiece *__restrict__ pieces, const int32_t *__restrict__ group_item_begin,
                            const int32_t *__restrict__ item_pieces, float *__restrict__ partial, int d, int nq)
{
    using C = Chunk<XD, VEC>;
    using raw_t = typename C::raw_t;
    using lds_t = typename C::lds_t;
    constexpr int BT = TS * H, WAVES = TS / 64, LPT = (K + H - 1) / H, ROW = LPT * BT;   // ROW chunks of LDS per staged row
    extern __shared__ __align__(16) unsigned char smem[];
    lds_t *stage = reinterpret_cast<lds_t *>(smem);                                       // [2][R][ROW]
    float *red = reinterpret_cast<float *>(smem + sizeof(lds_t) * 2 * R * ROW);           // [H][2][R][WAVES]
    const int tl = threadIdx.x % TS;
    const int tib = __builtin_amdgcn_readfirstlane(threadIdx.x / TS);
    const int wave = tl / 64;

    // what the item in hand is: set at the top of the item loop below, read by the pipeline stages
    DevPiece pc = {};                                   // the rows of the item (every team's piece of it has the same rows)
    int my_piece = -1;                                  // this team's piece of the item, or -1: it then only helps to fetch
    bool active = false;
    int nsteps = 0;

    // fetch role: thread g of the workgroup brings chunks g, g+BT, ... of every row
    unsigned goff[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) goff[j] = chunk_offset<VEC>(threadIdx.x + j * BT, nq, d);
    // compute role: as in the register-only kernel
    float wv[K][VEC];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int q = tl + k * TS;
        const int o = chunk_offset<VEC>(q, nq, d);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const float t = w[o + v];
            wv[k][v] = chunk_owns<VEC>(q, v, nq, d) ? t : 0.f;
        }
    }
    float acc[K][VEC];

    // rows that other workgroups fetch as well are left in the L2 for them; rows only this workgroup reads stream past it
    auto fetch = [&](raw_t (&P)[R][LPT], int step) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int rr = min(step * R + r, pc.nrows - 1);
            const void *row = row_ptr<XD>(X, pc.row_begin + rr, d);
            if (pc.shared) {
#pragma unroll
                for (int j = 0; j < LPT; ++j) P[r][j] = C::load(row, goff[j]);
            } else {
                asm volatile("; rows read once" ::: "memory");       // (the markers keep the two kinds of load from being merged into one)
#pragma unroll
                for (int j = 0; j < LPT; ++j) P[r][j] = C::load_once(row, goff[j]);
                asm volatile("; rows read once" ::: "memory");
            }
        }
    };
    auto park = [&](const raw_t (&P)[R][LPT], int buf) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < LPT; ++j) stage[(buf * R + r) * ROW + threadIdx.x + j * BT] = __builtin_bit_cast(lds_t, P[r][j]);
    };
    // one step: rows step*R .. step*R+R-1 are in LDS buffer `cur`; `next` holds the rows of step+1 (loaded or still in flight)
    auto step_fn = [&](int step, raw_t (&next)[R][LPT], int cur) {
        park(next, cur ^ 1);
        fetch(next, step + 3);                          // unconditional: the load queue then has a known depth at every wait
        float pd[R], yy[R];
        lds_t xr[R][K];
        if (active) {
#pragma unroll
            for (int r = 0; r < R; ++r) yy[r] = y[pc.row_begin + min(step * R + r, pc.nrows - 1)];   // asked for early, used after the barrier
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int k = 0; k < K; ++k) xr[r][k] = stage[(cur * R + r) * ROW + tl + k * TS];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float s[4] = {0.f, 0.f, 0.f, 0.f};       // four chains: a sum need not wait for the one before it
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    float xv[VEC];
                    C::widen(__builtin_bit_cast(raw_t, xr[r][k]), xv);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) s[k & 3] = fmaf(xv[v], wv[k][v], s[k & 3]);
                }
                pd[r] = wave_sum<XD == 1>((s[0] + s[1]) + (s[2] + s[3]));
            }
            if constexpr (WAVES > 1) {
                if ((tl & 63) == 0) {
#pragma unroll
                    for (int r = 0; r < R; ++r) red[((tib * 2 + cur) * R + r) * WAVES + wave] = pd[r];
                }
            }
        }
        __syncthreads();
        if (active) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float z = pd[r];
                if constexpr (WAVES > 1) {
                    z = 0.f;
#pragma unroll
                    for (int i = 0; i < WAVES; ++i) z += red[((tib * 2 + cur) * R + r) * WAVES + i];
                }
                const int rr = step * R + r;
                const float ph = LOGISTIC ? sigmoid(z) : z;
                const float res = (rr < pc.nrows) ? ph - yy[r] : 0.f;
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    float xv[VEC];
                    C::widen(__builtin_bit_cast(raw_t, xr[r][k]), xv);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[k][v] = fmaf(res, xv[v], acc[k][v]);
                }
            }
        }
    };

    // The workgroup works through its queue of items.  The last barrier of an item is behind every LDS read of it, so the next
    // item's first buffer can be filled at once; loads still in flight for steps past its end land in registers nobody reads.
    raw_t P0[R][LPT], P1[R][LPT];
    const int item_end = group_item_begin[blockIdx.x + 1];
    for (int item = group_item_begin[blockIdx.x]; item < item_end; ++item) {
        int ref_piece = -1;
        my_piece = -1;
#pragma unroll
        for (int t = 0; t < H; ++t) {
            const int pi = item_pieces[item * H + t];
            if (pi >= 0) {
                if (ref_piece < 0) ref_piece = pi;
                if (t == tib) my_piece = pi;
            }
        }
        if (ref_piece < 0) continue;                    // a gap in the queue (the same for the whole workgroup)
        pc = pieces[ref_piece];
        active = my_piece >= 0;
        nsteps = (pc.nrows + R - 1) / R;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[k][v] = 0.f;

        fetch(P0, 0);
        fetch(P1, 1);                                   // steps past the end re-read the last row; nothing is computed from them
        park(P0, 0);
        fetch(P0, 2);
        __syncthreads();
        int step = 0;
        for (; step + 1 < nsteps; step += 2) {          // two steps per trip, so that register sets and LDS buffers are fixed at compile time
            step_fn(step, P1, 0);
            step_fn(step + 1, P0, 1);
        }
        if (step < nsteps) step_fn(step, P1, 0);
        if (active) {
            float *out = partial + static_cast<int64_t>(my_piece) * d;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int q = tl + k * TS;
                if (q < nq) store_row<VEC>(out + chunk_offset<VEC>(q, nq, d), acc[k]);
            }
        }
    }
}

// ---- stage 1 with rows loaded straight into LDS ------------------------------------------------------------------------
// The same sharing for rows that start on 16-byte boundaries (fp32, d a multiple of 4), with the fetch done by the load-to-LDS form
// of the global load (global_load_lds_dwordx4: lane l of a wavefront writes 16 bytes at LDS offset M0 + 16 l).  Nothing passes
// through registers on its way in, which leaves room for a third holder per workgroup at 10 chunks per thread (168 registers at
// 768 threads), and the depth of the prefetch is set by LDS alone: a ring of NB rows, one being computed, the others landed or in
// flight.  One barrier per row:
//     read row b from its ring slot into registers, dot products, park the partial dots in LDS
//     wait until this wavefront's loads of row b+1 have landed (rows b+2 .. b+NB-1 stay in flight), barrier
//     aim the loads of row b+NB at the slot of row b            (every team holds row b in registers)
//     residuals and rank-1 updates of row b
// The loads are written as inline assembly so that the compiler neither knows nor guesses which LDS bytes they touch: every wait is
// written out with the number of loads that may stay in flight.  That count must be exact, so every wavefront issues the same
// number of loads for every row, also past the end of its queue (it then re-fetches its last row into a slot nobody reads), and
// the wavefront has no other vector loads in flight while the ring runs.  The fetch cursor runs through the whole queue of the
// workgroup, so the pipeline does not drain between items.
__device__ __forceinline__ void load_to_lds_16(const void *gptr, unsigned lds_offset)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_offset) : "memory", "m0");
}
// the same with the non-temporal hint: for rows that no other workgroup asks for, which then stream past the caches (a plain
// read of a large buffer reaches 7.0 TB/s that way on this machine, 6.0 to 6.3 without the hint)
__device__ __forceinline__ void load_to_lds_16_nt(const void *gptr, unsigned lds_offset)
{
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(gptr), "s"(lds_offset) : "memory", "m0");
}
// wait until at most N of this wavefront's vector memory loads are in flight (the other counters are left alone)
template <int N> __device__ __forceinline__ void wait_loads()
{
    static_assert(N >= 0 && N < 64, "the counter has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int TS, int K, int H, int NB, bool WL, int HPT, bool LOGISTIC>
__global__ void __launch_bounds__(TS * H)
partial_grads_dma_kernel(const void *__restrict__ Xv, const float *__restrict__ y, const float *__restrict__ w,
                         const DevPiece *__restrict__ pieces, const int32_t *__restrict__ group_item_begin,
                         const int32_t *__restrict__ item_pieces, float *__restrict__ partial, int d, int nq)
{
    constexpr int BT = TS * H, WAVES = TS / 64, LPT = (K + H - 1) / H;     // LPT loads per thread and row; (LPT - 1) * BT < nq always
    static_assert((NB - 1) * LPT < 64, "the loads in flight per wavefront must fit the hardware counter");
    static_assert(NB >= 2 && WAVES > 1, "a ring of at least two rows; teams of several wavefronts");
    static_assert(HPT == 1 || (HPT == 2 && WL), "a team that works for two holders keeps two sets of accumulators: the weights must be in LDS");
    constexpr int SLOTS = H * HPT;                          // holders per workgroup: team t works for holders t * HPT ... of an item
    const float *X = static_cast<const float *>(Xv);
    extern __shared__ __align__(16) unsigned char smem[];
    f4a *ring = reinterpret_cast<f4a *>(smem);                                          // [NB][nq] chunks
    f4a *wl = ring + NB * nq;                                                           // WL: the weights, [nq] chunks
    float *red = reinterpret_cast<float *>(smem + sizeof(f4a) * (NB + (WL ? 1 : 0)) * nq);   // [SLOTS][2][WAVES]
    const unsigned ring_lds = static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) unsigned char *)smem));
    const int tl = threadIdx.x % TS;
    const int tib = __builtin_amdgcn_readfirstlane(threadIdx.x / TS);
    const int wave = tl / 64;
    const int wgwave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);

    const int item_begin = group_item_begin[blockIdx.x], item_end = group_item_begin[blockIdx.x + 1];

    // compute role, as in the kernels above: chunks tl, tl + TS, ... of a row; a chunk index past the row reads the row's last chunk
    // with zero weights (K = ceil(nq / TS), so only a thread's last chunk can lie past the row)
    // WL (1024 threads, so 128 registers each): the weights live in LDS behind the ring and are read per row like the row itself;
    // only a thread's last chunk, the one that may need masking, keeps its weights in registers (wv[0])
    constexpr int KW = WL ? 1 : K;
    float wv[KW][4];
    const int qlast = min(tl + (K - 1) * TS, nq - 1);
#pragma unroll
    for (int k = WL ? K - 1 : 0; k < K; ++k) {
        const int q = k < K - 1 ? tl + k * TS : qlast;
        const f4u t = *reinterpret_cast<const f4u *>(w + 4 * q);
        const bool own = tl + k * TS < nq;
        float(&dst)[4] = wv[WL ? 0 : k];
        dst[0] = own ? t.x : 0.f; dst[1] = own ? t.y : 0.f; dst[2] = own ? t.z : 0.f; dst[3] = own ? t.w : 0.f;
    }
    if constexpr (WL) {
        for (int q = threadIdx.x; q < nq; q += BT) {
            const f4u t = *reinterpret_cast<const f4u *>(w + 4 * q);
            f4a v; v.x = t.x; v.y = t.y; v.z = t.z; v.w = t.w;
            wl[q] = v;                   // visible to the others after the barrier that follows the first fetches
        }
    }
    float acc[HPT][K][4];
#pragma unroll
    for (int h = 0; h < HPT; ++h)
#pragma unroll
        for (int k = 0; k < K; ++k) acc[h][k][0] = acc[h][k][1] = acc[h][k][2] = acc[h][k][3] = 0.f;
    __builtin_amdgcn_s_waitcnt(0);       // the weights are in: from here on the only vector loads of this wavefront are the ring's

    // fetch role: thread t brings chunks t, t + BT, ... of every row.  Only the last of them can lie outside the row, and a whole
    // wavefront may then have nothing to bring: it skips that load and counts one load fewer per row when it waits.
    const bool last_any = (LPT - 1) * BT + wgwave * 64 < nq;                 // the same for the whole wavefront
    const bool last_mine = (LPT - 1) * BT + static_cast<int>(threadIdx.x) < nq;

    // cursors over the workgroup's queue: the fetch cursor runs NB rows ahead of the compute cursor
    struct Cursor {
        int item;           // index into the queue; item_end: past the end
        int rows_left;      // rows of the current item not yet passed
        int piece[HPT];     // compute cursor: this team's pieces of the item (-1: none); fetch cursor: [0] = any piece of the item
        int shared;         // fetch cursor: do other workgroups fetch the item's rows too?
        int64_t row;        // current row of X
    };
    auto enter = [&](Cursor &c, bool for_compute) {     // settle on the first item at or after c.item that has pieces
        for (; c.item < item_end; ++c.item) {
            int ref = -1, mine[HPT];
#pragma unroll
            for (int h = 0; h < HPT; ++h) mine[h] = -1;
#pragma unroll
            for (int t = 0; t < SLOTS; ++t) {
                const int pi = item_pieces[c.item * SLOTS + t];
                if (pi >= 0) {
                    if (ref < 0) ref = pi;
                    if (t / HPT == tib) mine[t % HPT] = pi;
                }
            }
            if (ref < 0) continue;                          // a gap in the queue
            const DevPiece pc = pieces[ref];                // every piece of an item covers the same rows
            c.row = pc.row_begin;
            c.rows_left = pc.nrows;
#pragma unroll
            for (int h = 0; h < HPT; ++h) c.piece[h] = for_compute ? mine[h] : ref;
            c.shared = pc.shared;
            return;
        }
    };
    Cursor F, C;
    F.item = C.item = item_begin;
    F.rows_left = C.rows_left = 0;
#pragma unroll
    for (int h = 0; h < HPT; ++h) F.piece[h] = C.piece[h] = -1;
    F.shared = C.shared = 1;
    F.row = C.row = 0;
    enter(F, false);
    enter(C, true);
    if (C.item >= item_end) return;                        // nothing queued (the same for the whole workgroup)

    // loads of the row under the fetch cursor into ring slot `slot`; then the cursor moves on, staying on its last row once the
    // queue is exhausted.  Rows that other workgroups fetch as well are left in the L2 for them; rows that only this workgroup
    // reads stream past it.
    auto issue = [&](int slot) {
        const float *row = X + F.row * d;
        const unsigned dst = ring_lds + 16u * static_cast<unsigned>(slot * nq + wgwave * 64);
        if (F.shared) {
#pragma unroll
            for (int j = 0; j < LPT - 1; ++j) load_to_lds_16(row + 4 * (threadIdx.x + j * BT), dst + 16u * (j * BT));
            if (last_any) {
                if (last_mine) load_to_lds_16(row + 4 * (threadIdx.x + (LPT - 1) * BT), dst + 16u * ((LPT - 1) * BT));
            }
        } else {
#pragma unroll
            for (int j = 0; j < LPT - 1; ++j) load_to_lds_16_nt(row + 4 * (threadIdx.x + j * BT), dst + 16u * (j * BT));
            if (last_any) {
                if (last_mine) load_to_lds_16_nt(row + 4 * (threadIdx.x + (LPT - 1) * BT), dst + 16u * ((LPT - 1) * BT));
            }
        }
        if (F.rows_left > 1) { --F.rows_left; ++F.row; }
        else {
            Cursor N = F;
            ++N.item;
            enter(N, false);
            if (N.item < item_end) F = N;
        }
    };
    // wait until at most B of this wavefront's rows are still in flight
    auto wait_for = [&](auto tag) {
        constexpr int B = decltype(tag)::value;
        if (last_any) wait_loads<B * LPT>(); else wait_loads<B * (LPT - 1)>();
    };

#pragma unroll
    for (int i = 0; i < NB; ++i) issue(i);
    wait_for(std::integral_constant<int, NB - 1>{});
    __syncthreads();
    int slot = 0, par = 0;
    while (C.item < item_end) {                            // the items of the queue ...
        bool has[HPT];
        bool active = false;
#pragma unroll
        for (int h = 0; h < HPT; ++h) { has[h] = C.piece[h] >= 0; active = active || has[h]; }
        int64_t row = C.row;
        for (int left = C.rows_left; left > 0; --left, ++row) {         // ... and the rows of an item
            float yy = 0.f;
            f4a xr[K];
            if (active) {
                yy = y[row];
#pragma unroll
                for (int k = 0; k < K; ++k) xr[k] = ring[slot * nq + (k < K - 1 ? tl + k * TS : qlast)];
#pragma unroll
                for (int h = 0; h < HPT; ++h) {            // every holder forms its own dot product
                    if (!has[h]) continue;
                    float s = 0.f, s1 = 0.f;
#pragma unroll
                    for (int k = 0; k < K; ++k) {
                        f4a wk;
                        if (WL && k < K - 1) wk = wl[tl + k * TS];
                        else { const float(&r)[4] = wv[WL ? 0 : k]; wk.x = r[0]; wk.y = r[1]; wk.z = r[2]; wk.w = r[3]; }
                        if (k & 1) { s1 = fmaf(xr[k].x, wk.x, s1); s1 = fmaf(xr[k].y, wk.y, s1); s1 = fmaf(xr[k].z, wk.z, s1); s1 = fmaf(xr[k].w, wk.w, s1); }
                        else { s = fmaf(xr[k].x, wk.x, s); s = fmaf(xr[k].y, wk.y, s); s = fmaf(xr[k].z, wk.z, s); s = fmaf(xr[k].w, wk.w, s); }
                    }
                    const float pd = wave_sum<false>(s + s1);
                    if ((tl & 63) == 0) red[((tib * HPT + h) * 2 + par) * WAVES + wave] = pd;
                }
            }
            wait_for(std::integral_constant<int, NB - 2>{});      // my part of the next row has landed; the barrier covers the others'
            __syncthreads();
            issue(slot);                                         // every team holds this row in registers: its slot is free
            if (active) {
#pragma unroll
                for (int h = 0; h < HPT; ++h) {
                    if (!has[h]) continue;
                    float z = 0.f;
#pragma unroll
                    for (int i = 0; i < WAVES; ++i) z += red[((tib * HPT + h) * 2 + par) * WAVES + i];
                    const float res = (LOGISTIC ? sigmoid(z) : z) - yy;
#pragma unroll
                    for (int k = 0; k < K; ++k) {
                        acc[h][k][0] = fmaf(res, xr[k].x, acc[h][k][0]); acc[h][k][1] = fmaf(res, xr[k].y, acc[h][k][1]);
                        acc[h][k][2] = fmaf(res, xr[k].z, acc[h][k][2]); acc[h][k][3] = fmaf(res, xr[k].w, acc[h][k][3]);
                    }
                }
            }
            slot = slot + 1 == NB ? 0 : slot + 1;
            par ^= 1;
        }
#pragma unroll
        for (int h = 0; h < HPT; ++h) {
            if (!has[h]) continue;                         // the item is done: this holder's partial row is complete
            float *out = partial + static_cast<int64_t>(C.piece[h]) * d;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int q = tl + k * TS;
                if (q < nq) { f4u t; t.x = acc[h][k][0]; t.y = acc[h][k][1]; t.z = acc[h][k][2]; t.w = acc[h][k][3]; *reinterpret_cast<f4u *>(out + 4 * q) = t; }
                acc[h][k][0] = acc[h][k][1] = acc[h][k][2] = acc[h][k][3] = 0.f;
            }
        }
        ++C.item;
        enter(C, true);
    }
    wait_loads<0>();                      // the re-fetches past the end of the queue land before the workgroup gives its LDS back
}

// ---- stage 1 for wide rows -----------------------------------------------------------------------------------------
// When a row is too long for one team's registers the single pass is split in two: first the residuals r = phi(x.w) - y of every
// row visit (one workgroup per piece, the row streamed in chunks), then G_piece = X^T r per piece and column block.
template <int XD, int VEC>
__global__ void __launch_bounds__(256)
residuals_kernel(const void *__restrict__ X, const float *__restrict__ y, const float *__restrict__ w,
                 const DevPiece *__restrict__ pieces, float *__restrict__ residuals, int d, int nq, int logistic)
{
    using C = Chunk<XD, VEC>;
    using raw_t = typename C::raw_t;
    constexpr int U = 8;                                 // chunks in flight per thread
    const DevPiece pc = pieces[blockIdx.x];
    __shared__ float red[2][4];
    int buf = 0;
    for (int r = 0; r < pc.nrows; ++r) {
        const void *row = row_ptr<XD>(X, pc.row_begin + r, d);
        float s = 0.f;
        for (int q0 = threadIdx.x; q0 < nq; q0 += 256 * U) {
            raw_t xr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) xr[u] = C::load(row, chunk_offset<VEC>(q0 + u * 256, nq, d));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + u * 256;
                const int o = chunk_offset<VEC>(q, nq, d);
                float xv[VEC];
                C::widen(xr[u], xv);
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    if (chunk_owns<VEC>(q, v, nq, d)) s = fmaf(xv[v], w[o + v], s);
            }
        }
        s = wave_sum<true>(s);
        if ((threadIdx.x & 63) == 0) red[buf][threadIdx.x / 64] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            const float z = red[buf][0] + red[buf][1] + red[buf][2] + red[buf][3];
            const float ph = logistic ? sigmoid(z) : z;
            residuals[pc.visit_begin + r] = ph - y[pc.row_begin + r];
        }
        buf ^= 1;
    }
}

template <int XD, int VEC>
__global__ void __launch_bounds__(256)
xt_residuals_kernel(const void *__restrict__ X, const DevPiece *__restrict__ pieces, const float *__restrict__ residuals,
                    float *__restrict__ partial, int d, int nq)
{
    using C = Chunk<XD, VEC>;
    using raw_t = typename C::raw_t;
    constexpr int K = kWideChunks;
    const DevPiece pc = pieces[blockIdx.y];
    const int qbase = blockIdx.x * (256 * K) + threadIdx.x;
    unsigned off[K];
#pragma unroll
    for (int k = 0; k < K; ++k) off[k] = chunk_offset<VEC>(qbase + k * 256, nq, d);
    float acc[K][VEC];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[k][v] = 0.f;
    for (int r = 0; r < pc.nrows; ++r) {
        const void *row = row_ptr<XD>(X, pc.row_begin + r, d);
        const float res = residuals[pc.visit_begin + r];
        raw_t xr[K];
#pragma unroll
        for (int k = 0; k < K; ++k) xr[k] = C::load(row, off[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            float xv[VEC];
            C::widen(xr[k], xv);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[k][v] = fmaf(res, xv[v], acc[k][v]);
        }
    }
    float *out = partial + static_cast<int64_t>(blockIdx.y) * d;
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (qbase + k * 256 < nq) store_row<VEC>(out + off[k], acc[k]);
}

// ---- piece reduction ------------------------------------------------------------------------------------------------
// G[slab] = sum of the slab's pieces.  A workgroup covers 64 chunks of columns of one slab; its four wavefronts each add up every
// fourth piece (eight loads in flight per lane), then the four partial sums are combined through LDS.  The order of the
// additions is fixed by the piece list alone, so the result is the same bits on every run; the sums are carried in fp64.
template <int VEC>
__global__ void __launch_bounds__(256)
reduce_pieces_kernel(const float *__restrict__ partial, const int32_t *__restrict__ slab_piece_begin, const int32_t *__restrict__ slab_pieces,
                     float *__restrict__ G, int64_t d, int nq)
{
    constexpr int WAVES = 4;
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = min(static_cast<int>(blockIdx.x) * 64 + lane, nq - 1);     // lanes past the row repeat its last chunk and do not store
    const int64_t col = chunk_offset<VEC>(q, nq, static_cast<int>(d));
    const int slab = blockIdx.y;
    const int pb = slab_piece_begin[slab], pe = slab_piece_begin[slab + 1];
    double acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0;
    for (int j0 = pb + wave; j0 < pe; j0 += WAVES * U) {
        float xv[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = min(j0 + u * WAVES, pe - 1);
            load_row<VEC>(partial + static_cast<int64_t>(slab_pieces[j]) * d + col, xv[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (j0 + u * WAVES < pe) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] += static_cast<double>(xv[u][v]);
            }
    }
    __shared__ double part[WAVES - 1][VEC][64];
    if (wave > 0) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) part[wave - 1][v][lane] = acc[v];
    }
    __syncthreads();
    if (wave == 0 && static_cast<int>(blockIdx.x) * 64 + lane < nq) {
        float out[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            double t = acc[v];
#pragma unroll
            for (int k = 0; k < WAVES - 1; ++k) t += part[k][v][lane];
            out[v] = static_cast<float>(t);
        }
        store_row<VEC>(G + static_cast<int64_t>(slab) * d + col, out);
    }
}

// ---- encode ---------------------------------------------------------------------------------------------------------
// One thread owns C chunks of VEC columns and runs the whole sub-tree of one level-1 node for them: a post-order list of terms
// (own += coef * G[slab]) in which the last term of a node finishes it: message = own + pending[level], stored (rounded to fp32,
// as a transmitted message would be) and folded into pending[level-1] with the parent's decode coefficient.  Child messages
// therefore never come back from HBM; every active slab is read once and every message written once.  The program is the same for
// every thread, so it is read with wide scalar loads, U terms at a time; the slab loads of those terms are all issued before the
// first is used.  Slabs and messages are touched once: loads and stores are non-temporal.
// A workgroup of BS threads covers BS*C*VEC contiguous columns of every row it touches.  Two shapes are used:
//   narrow  C=1, U=8, fp64 accumulators: for short vectors, where the launch has few threads and latency decides;
//   wide    C=32, U=1, fp32 accumulators: for long vectors.  A workgroup then streams 128 KB-aligned, 128 KB-long pieces of one
//           slab at a time, which is what HBM likes best (the same 31-stream pattern read 4 KB at a time reaches 4.9 TB/s, this
//           6.1 TB/s); the 32 chunks in flight fill the register file, hence fp32 accumulation: two or three extra roundings
//           of the size of the message's own fp32 rounding.
template <int VEC, int LT, int C, int BS, int U, typename acc_t>
__global__ void __launch_bounds__(BS)
encode_kernel(const float *__restrict__ G, float *__restrict__ M, EncProgram prog, int64_t d, int nq)
{
    static_assert(kEncodeUnroll % U == 0, "sub-programs are padded to kEncodeUnroll terms");
    typedef int iuv __attribute__((ext_vector_type(U)));
    typedef double duv __attribute__((ext_vector_type(U)));
    const int q0 = blockIdx.x * (BS * C) + threadIdx.x;
    if (q0 >= nq) return;
    // whole groups of U terms: the padding terms are only fetched when U does not divide the real length
    const int tb = prog.sub_begin[blockIdx.y], te = tb + (prog.sub_end[blockIdx.y] - tb + U - 1) / U * U;
    // chunk c of this thread; a chunk past the end of the row is redirected to the row's last chunk and not stored
    int64_t col[C];
    bool live[C];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int q = q0 + c * BS;
        live[c] = q < nq;
        col[c] = chunk_offset<VEC>(q, nq, static_cast<int>(d));
    }

    acc_t pend[LT + 1][C][VEC];
    acc_t own[C][VEC];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            own[c][v] = 0;
#pragma unroll
            for (int l = 0; l <= LT; ++l) pend[l][c][v] = 0;
        }

    for (int t = tb; t < te; t += U) {
        const iuv slab = *reinterpret_cast<const iuv *>(prog.slab + t);
        const iuv level = *reinterpret_cast<const iuv *>(prog.level + t);
        const iuv row = *reinterpret_cast<const iuv *>(prog.row + t);
        const duv coef = *reinterpret_cast<const duv *>(prog.coef + t);
        const duv acoef = *reinterpret_cast<const duv *>(prog.acoef + t);
        float xv[U][C][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *src = G + static_cast<int64_t>(slab[u]) * d;
#pragma unroll
            for (int c = 0; c < C; ++c) load_row_nt<VEC>(src + col[c], xv[u][c]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) own[c][v] = fma(static_cast<acc_t>(coef[u]), static_cast<acc_t>(xv[u][c][v]), own[c][v]);
            const int lvl = level[u];
            if (lvl > 0) {
                float *dst = M + static_cast<int64_t>(row[u]) * d;
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    float out[VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        acc_t msg = own[c][v];
#pragma unroll
                        for (int l = 1; l < LT; ++l)               // only levels 1..L-1 ever collect children
                            if (l == lvl) { msg += pend[l][c][v]; pend[l][c][v] = 0; }
                        out[v] = static_cast<float>(msg);
                        own[c][v] = 0;
                    }
                    if (live[c]) store_row_nt<VEC>(dst + col[c], out);
#pragma unroll
                    for (int l = 1; l < LT; ++l)
                        if (l == lvl - 1) {
#pragma unroll
                            for (int v = 0; v < VEC; ++v) pend[l][c][v] = fma(static_cast<acc_t>(acoef[u]), static_cast<acc_t>(out[v]), pend[l][c][v]);
                        }
                }
            }
        }
    }
}

// ---- decode ---------------------------------------------------------------------------------------------------------
template <int VEC>
__global__ void __launch_bounds__(256)
decode_kernel(const float *__restrict__ M, float *__restrict__ g, const DecTerm *__restrict__ terms, int nterms, int64_t d, int nq,
              float *__restrict__ w, float lr)
{
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q >= nq) return;
    const int64_t col = chunk_offset<VEC>(q, nq, static_cast<int>(d));
    double acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0;
    for (int j = 0; j < nterms; ++j) {
        const DecTerm tm = terms[j];
        float xv[VEC];
        load_row<VEC>(M + static_cast<int64_t>(tm.row) * d + col, xv);
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = fma(tm.coef, static_cast<double>(xv[v]), acc[v]);
    }
    float out[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) out[v] = static_cast<float>(acc[v]);
    store_row<VEC>(g + col, out);
    if (w) {
        // the gradient step of the same columns, from the rounded g that was just stored; a column shared with the neighbouring
        // chunk is stepped by the chunk that owns it only
#pragma unroll
        for (int v = 0; v < VEC; ++v)
            if (chunk_owns<VEC>(q, v, nq, static_cast<int>(d))) w[col + v] = fmaf(-lr, out[v], w[col + v]);
    }
}

__global__ void __launch_bounds__(256) update_kernel(float *__restrict__ w, const float *__restrict__ g, float lr, int64_t d)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < d) w[i] = fmaf(-lr, g[i], w[i]);
}

// Gradient step fused with the two convergence measures of the paper's experiments: metrics[0] = ||w_new - w||^2 / ||w||^2
// (relative error rate, eq. (6)), metrics[1] = ||w_new - w*||^2 / ||w*||^2 (normalised error rate, eq. (8)), or -1 without w*.
// One workgroup, fixed summation order: the model has at most a few 10^4 entries on this path.
__global__ void __launch_bounds__(1024)
update_metrics_kernel(float *__restrict__ w, const float *__restrict__ g, float lr, const float *__restrict__ w_star,
                      float *__restrict__ metrics, int64_t d)
{
    double acc[4] = {0.0, 0.0, 0.0, 0.0};   // |dw|^2, |w|^2, |w_new - w*|^2, |w*|^2
    for (int64_t i = threadIdx.x; i < d; i += 1024) {
        const float wo = w[i];
        const float wn = fmaf(-lr, g[i], wo);
        w[i] = wn;
        const double dw = static_cast<double>(wn) - static_cast<double>(wo);
        acc[0] += dw * dw;
        acc[1] += static_cast<double>(wo) * wo;
        if (w_star) {
            const double ws = w_star[i], e = static_cast<double>(wn) - ws;
            acc[2] += e * e;
            acc[3] += ws * ws;
        }
    }
    __shared__ double part[16][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc[k] += __shfl_xor(acc[k], o, 64);
    }
    if ((threadIdx.x & 63) == 0)
        for (int k = 0; k < 4; ++k) part[threadIdx.x / 64][k] = acc[k];
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot[4] = {0.0, 0.0, 0.0, 0.0};
        for (int wv = 0; wv < 16; ++wv)
            for (int k = 0; k < 4; ++k) tot[k] += part[wv][k];
        metrics[0] = static_cast<float>(tot[0] / tot[1]);
        metrics[1] = w_star ? static_cast<float>(tot[2] / tot[3]) : -1.f;
    }
}

// ---- variant table for stage 1 --------------------------------------------------------------------------------------
// each variant is built twice, for phi = identity and phi = sigmoid: every lane forms the residual of every row, and the kernels
// bound by vector-ALU issue would pay for evaluating both forms and selecting one
#define CR_V(XD, VEC, TS, K, R)                                                                         \
    {XD, VEC, TS, K, R, (TS < 256 ? 256 / TS : 1), false,                                               \
     {reinterpret_cast<const void *>(&partial_grads_kernel<XD, VEC, TS, K, R, false>),                  \
      reinterpret_cast<const void *>(&partial_grads_kernel<XD, VEC, TS, K, R, true>)}}
#define CR_VB(XD, VEC, TS, K, R)                                                                        \
    {XD, VEC, TS, K, R, (TS < 256 ? 256 / TS : 1), false,                                               \
     {reinterpret_cast<const void *>(&partial_grads_kernel<XD, VEC, TS, K, R, false>),                  \
      reinterpret_cast<const void *>(&partial_grads_kernel<XD, VEC, TS, K, R, true>)}, 0, 0,            \
     {reinterpret_cast<const void *>(&partial_grads_kernel<XD, VEC, TS, K, R, false, true>),            \
      reinterpret_cast<const void *>(&partial_grads_kernel<XD, VEC, TS, K, R, true, true>)}}
#define CR_S(XD, VEC, TS, K, R, H)                                                                      \
    {XD, VEC, TS, K, R, H, true,                                                                        \
     {reinterpret_cast<const void *>(&partial_grads_staged_kernel<XD, VEC, TS, K, R, H, false>),        \
      reinterpret_cast<const void *>(&partial_grads_staged_kernel<XD, VEC, TS, K, R, H, true>)}}
#define CR_D(TS, K, NB, H)                                                                             \
    {0, 4, TS, K, 1, H, true,                                                                          \
     {reinterpret_cast<const void *>(&partial_grads_dma_kernel<TS, K, H, NB, false, 1, false>),           \
      reinterpret_cast<const void *>(&partial_grads_dma_kernel<TS, K, H, NB, false, 1, true>)}, NB, 0}
#define CR_DW2(TS, K, NB, H)                                                                           \
    {0, 4, TS, K, 1, 2 * H, true,                                                                      \
     {reinterpret_cast<const void *>(&partial_grads_dma_kernel<TS, K, H, NB, true, 2, false>),         \
      reinterpret_cast<const void *>(&partial_grads_dma_kernel<TS, K, H, NB, true, 2, true>)}, NB, 1, {nullptr, nullptr}, 2}
#define CR_DW(TS, K, NB, H)                                                                            \
    {0, 4, TS, K, 1, H, true,                                                                          \
     {reinterpret_cast<const void *>(&partial_grads_dma_kernel<TS, K, H, NB, true, 1, false>),            \
      reinterpret_cast<const void *>(&partial_grads_dma_kernel<TS, K, H, NB, true, 1, true>)}, NB, 1}
// one variant per exact chunk count K = ceil(row chunks / team size); R rows in flight chosen so a thread holds about 16-24 chunks
const Stage1Variant kVariants[] = {
    // fp32, chunks of 4 columns (4 registers per chunk)
    CR_V(0, 4, 64, 1, 8), CR_V(0, 4, 64, 2, 8), CR_V(0, 4, 64, 3, 4), CR_V(0, 4, 64, 4, 4),
    CR_V(0, 4, 256, 2, 8), CR_V(0, 4, 256, 3, 4), CR_V(0, 4, 256, 4, 4), CR_V(0, 4, 256, 5, 4),
    CR_V(0, 4, 256, 6, 3), CR_V(0, 4, 256, 7, 2), CR_V(0, 4, 256, 8, 2), CR_V(0, 4, 256, 9, 2),
    CR_V(0, 4, 256, 10, 2), CR_V(0, 4, 256, 11, 2), CR_V(0, 4, 256, 12, 2),
    CR_V(0, 4, 1024, 4, 2), CR_V(0, 4, 1024, 5, 1), CR_V(0, 4, 1024, 6, 1),
    // bf16, chunks of 8 columns: they widen to eight accumulators each, so a thread can hold half as many
    // (the one-wavefront teams, bound by vector-ALU issue, also come with buffer loads for rows that start on 4-byte boundaries)
    CR_VB(1, 8, 64, 1, 8), CR_VB(1, 8, 64, 2, 4), CR_VB(1, 8, 64, 3, 4), CR_VB(1, 8, 64, 4, 2),
    CR_V(1, 8, 256, 2, 4), CR_V(1, 8, 256, 3, 4), CR_V(1, 8, 256, 4, 2), CR_V(1, 8, 256, 5, 2),
    CR_V(1, 8, 256, 6, 2), CR_V(1, 8, 1024, 2, 2), CR_V(1, 8, 1024, 3, 1),
    // rows shorter than one wide chunk: one column per lane
    CR_V(0, 1, 64, 1, 8), CR_V(1, 1, 64, 1, 8),
    // fp32 rows of 1537 to 2558 whole 16-byte chunks (up to 40 KB) loaded straight into LDS.  Four holders per workgroup (1024
    // threads, 128 registers each: the weights move to LDS, behind a ring of three rows) where the holder counts make that fewer
    // workgroups per row; else three holders per workgroup (768 threads) and a ring of four rows.  Listed before the
    // register-staged kernels of two holders that cover the same widths.
    CR_DW2(256, 7, 3, 3), CR_DW2(256, 8, 3, 3), CR_DW2(256, 9, 3, 3), CR_DW2(256, 10, 3, 3),
    CR_DW(256, 7, 3, 4), CR_DW(256, 8, 3, 4), CR_DW(256, 9, 3, 4), CR_DW(256, 10, 3, 4),
    CR_D(256, 7, 4, 3), CR_D(256, 8, 4, 3), CR_D(256, 9, 4, 3), CR_D(256, 10, 4, 3),
    // fp32 rows staged through LDS by way of registers (any width).  Eight holders per workgroup, one wavefront each, for rows of up to 1024 chunks ...
    CR_S(0, 4, 64, 5, 1, 8), CR_S(0, 4, 64, 6, 1, 8), CR_S(0, 4, 64, 7, 1, 8), CR_S(0, 4, 64, 8, 1, 8), CR_S(0, 4, 64, 9, 1, 8),
    CR_S(0, 4, 64, 10, 1, 8), CR_S(0, 4, 64, 11, 1, 8), CR_S(0, 4, 64, 12, 1, 8), CR_S(0, 4, 64, 13, 1, 8), CR_S(0, 4, 64, 14, 1, 8),
    CR_S(0, 4, 64, 15, 1, 8), CR_S(0, 4, 64, 16, 1, 8),
    // ... four holders of four wavefronts (1024 threads, so at most 128 registers each) up to 1536 chunks ...
    CR_S(0, 4, 256, 2, 2, 4), CR_S(0, 4, 256, 3, 2, 4), CR_S(0, 4, 256, 4, 2, 4), CR_S(0, 4, 256, 5, 1, 4), CR_S(0, 4, 256, 6, 1, 4),
    // ... two holders up to 3072 chunks; R is limited by the two LDS buffers of R rows each
    CR_S(0, 4, 256, 2, 4, 2), CR_S(0, 4, 256, 3, 2, 2), CR_S(0, 4, 256, 4, 2, 2), CR_S(0, 4, 256, 5, 2, 2), CR_S(0, 4, 256, 6, 2, 2),
    CR_S(0, 4, 256, 7, 1, 2), CR_S(0, 4, 256, 8, 1, 2), CR_S(0, 4, 256, 9, 1, 2), CR_S(0, 4, 256, 10, 1, 2),
    CR_S(0, 4, 256, 11, 1, 2), CR_S(0, 4, 256, 12, 1, 2),
};

// columns per chunk: the 16-byte width unless the row is shorter than that
int stage1_chunk_width(int x_dtype, int64_t d)
{
    const int wide = (x_dtype == 1) ? 8 : 4;
    return d >= wide ? wide : 1;
}

}  // namespace

size_t Stage1Variant::lds_bytes(int64_t d) const
{
    if (!staged) return 0;
    if (ring > 0) {        // ring of whole rows, then the partial dot products of the teams' wavefronts
        const size_t nq = static_cast<size_t>((d + vec - 1) / vec);
        return 16 * static_cast<size_t>(ring + w_in_lds) * nq + sizeof(float) * tpb * 2 * (team_size / 64);
    }
    const size_t row_chunks = static_cast<size_t>((k + tpb - 1) / tpb) * block();
    return 16 * 2 * rows * row_chunks + sizeof(float) * tpb * 2 * rows * (team_size / 64);
}

const Stage1Variant *select_stage1(int x_dtype, int64_t d)
{
    const int vec = stage1_chunk_width(x_dtype, d);
    const int64_t nq = (d + vec - 1) / vec;
    // smallest team that covers the row with an available chunk count; the kernel needs K = ceil(nq / team size) exactly
    for (int ts : {64, 256, 1024}) {
        const int64_t k = (nq + ts - 1) / ts;
        for (const Stage1Variant &v : kVariants)
            if (!v.staged && v.xd == x_dtype && v.vec == vec && v.team_size == ts && v.k == k) return &v;
    }
    return nullptr;
}

const Stage1Variant *select_stage1_staged(int x_dtype, int64_t d, int64_t max_holders)
{
    const int vec = stage1_chunk_width(x_dtype, d);
    const int64_t nq = (d + vec - 1) / vec;
    // the widest workgroup that is not wider than the rows need: 8 holders for rows with 5 or more, 4 (3 for long rows) for 3 or 4,
    // else 2.  The table lists wide workgroups before narrow ones; the kernel that loads straight into LDS needs rows of whole
    // 16-byte chunks and a ring that fits LDS at this width.
    const int widest = max_holders >= 5 ? 8 : max_holders >= 3 ? 4 : 2;
    for (const Stage1Variant &v : kVariants) {
        if (!v.staged || v.xd != x_dtype || v.vec != vec || v.k != (nq + v.team_size - 1) / v.team_size || v.tpb > widest) continue;
        if (v.ring > 0 && (d % vec != 0 || v.lds_bytes(d) > kLdsPerWorkgroup)) continue;
        // four holders per workgroup (weights in LDS) only where that takes fewer workgroups per row than three do
        if (v.w_in_lds && v.holders_per_team == 1 && (max_holders + 3) / 4 >= (max_holders + 2) / 3) continue;
        // three teams that each work for two holders: rows with five or six holders in one workgroup
        if (v.holders_per_team == 2 && max_holders != 5 && max_holders != 6) continue;
        return &v;
    }
    return nullptr;
}

hipError_t prepare_stage1(const Stage1Variant &v, int64_t d)
{
    if (v.lds_bytes(d) <= 48 * 1024) return hipSuccess;
    for (const void *fn : v.fn) {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(v.lds_bytes(d)));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_partial_grads(const Stage1Variant &v, const void *X, const float *y, const float *w, const DevPiece *pieces,
                                const int32_t *team_piece_begin, int num_teams, float *partial, int64_t d, int logistic,
                                bool rows_as_buffers, hipStream_t stream)
{
    int di = static_cast<int>(d);
    int nq = static_cast<int>((d + v.vec - 1) / v.vec);
    void *args[] = {&X, &y, &w, &pieces, &team_piece_begin, &num_teams, &partial, &di, &nq};
    const int tpb = v.teams_per_block();
    dim3 grid((num_teams + tpb - 1) / tpb), block(v.block());
    const void *fn = rows_as_buffers && v.fn_buffers[0] ? v.fn_buffers[logistic ? 1 : 0] : v.fn[logistic ? 1 : 0];
    return hipLaunchKernel(fn, grid, block, args, 0, stream);
}

hipError_t launch_partial_grads_staged(const Stage1Variant &v, const void *X, const float *y, const float *w, const DevPiece *pieces,
                                       const int32_t *group_item_begin, const int32_t *item_pieces, int num_groups, float *partial,
                                       int64_t d, int logistic, hipStream_t stream)
{
    int di = static_cast<int>(d);
    int nq = static_cast<int>((d + v.vec - 1) / v.vec);
    void *args[] = {&X, &y, &w, &pieces, &group_item_begin, &item_pieces, &partial, &di, &nq};
    dim3 grid(num_groups), block(v.block());
    return hipLaunchKernel(v.fn[logistic ? 1 : 0], grid, block, args, v.lds_bytes(d), stream);
}

namespace {
template <int XD, int VEC>
hipError_t launch_wide(const void *X, const float *y, const float *w, const DevPiece *pieces, int num_pieces, float *residuals,
                       float *partial, int64_t d, int logistic, hipStream_t stream)
{
    const int nq = static_cast<int>((d + VEC - 1) / VEC);
    const int di = static_cast<int>(d);
    if (partial == nullptr)
        residuals_kernel<XD, VEC><<<num_pieces, 256, 0, stream>>>(X, y, w, pieces, residuals, di, nq, logistic);
    else
        xt_residuals_kernel<XD, VEC><<<dim3((nq + 256 * kWideChunks - 1) / (256 * kWideChunks), num_pieces), 256, 0, stream>>>(
            X, pieces, residuals, partial, di, nq);
    return hipGetLastError();
}

hipError_t dispatch_wide(int x_dtype, const void *X, const float *y, const float *w, const DevPiece *pieces, int num_pieces,
                         float *residuals, float *partial, int64_t d, int logistic, hipStream_t stream)
{
    if (x_dtype == 0) return launch_wide<0, 4>(X, y, w, pieces, num_pieces, residuals, partial, d, logistic, stream);
    return launch_wide<1, 8>(X, y, w, pieces, num_pieces, residuals, partial, d, logistic, stream);
}
}  // namespace

hipError_t launch_residuals(int x_dtype, const void *X, const float *y, const float *w, const DevPiece *pieces, int num_pieces,
                            float *residuals, int64_t d, int logistic, hipStream_t stream)
{
    return dispatch_wide(x_dtype, X, y, w, pieces, num_pieces, residuals, nullptr, d, logistic, stream);
}

hipError_t launch_xt_residuals(int x_dtype, const void *X, const DevPiece *pieces, int num_pieces, const float *residuals, float *partial,
                               int64_t d, hipStream_t stream)
{
    return dispatch_wide(x_dtype, X, nullptr, nullptr, pieces, num_pieces, const_cast<float *>(residuals), partial, d, 0, stream);
}

hipError_t launch_reduce_pieces(const float *partial, const int32_t *slab_piece_begin, const int32_t *slab_pieces, int num_slabs, float *G,
                                int64_t d, hipStream_t stream)
{
    if (d >= 4) {
        const int nq = static_cast<int>((d + 3) / 4);
        reduce_pieces_kernel<4><<<dim3((nq + 63) / 64, num_slabs), 256, 0, stream>>>(partial, slab_piece_begin, slab_pieces, G, d, nq);
    } else {
        const int nq = static_cast<int>(d);
        reduce_pieces_kernel<1><<<dim3((nq + 63) / 64, num_slabs), 256, 0, stream>>>(partial, slab_piece_begin, slab_pieces, G, d, nq);
    }
    return hipGetLastError();
}

template <int VEC, int C, int BS, int U, typename acc_t>
static hipError_t launch_encode_shape(const float *G, float *M, const EncProgram &prog, int num_sub, int L, int64_t d, hipStream_t stream)
{
    const int nq = static_cast<int>((d + VEC - 1) / VEC);
    const dim3 grid((nq + BS * C - 1) / (BS * C), num_sub), block(BS);
    if (L <= 1) encode_kernel<VEC, 1, C, BS, U, acc_t><<<grid, block, 0, stream>>>(G, M, prog, d, nq);
    else if (L == 2) encode_kernel<VEC, 2, C, BS, U, acc_t><<<grid, block, 0, stream>>>(G, M, prog, d, nq);
    else if (L == 3) encode_kernel<VEC, 3, C, BS, U, acc_t><<<grid, block, 0, stream>>>(G, M, prog, d, nq);
    else if constexpr (C == 1) {                         // deeper trees only in the narrow shape (the wide one would spill)
        if (L == 4) encode_kernel<VEC, 4, C, BS, U, acc_t><<<grid, block, 0, stream>>>(G, M, prog, d, nq);
        else encode_kernel<VEC, kMaxLevels, C, BS, U, acc_t><<<grid, block, 0, stream>>>(G, M, prog, d, nq);
    } else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_encode(const float *G, float *M, const EncProgram &prog, int num_sub, int L, int64_t d, hipStream_t stream)
{
    if (d >= 4) {
        // wide shape once its 8192-chunk workgroups are enough to fill the chip, and only up to 3 levels (registers)
        const int64_t wide_groups = ((d + 3) / 4 + 8191) / 8192 * num_sub;
        if (wide_groups >= 256 && L <= 3) return launch_encode_shape<4, 32, 256, 1, float>(G, M, prog, num_sub, L, d, stream);
        return launch_encode_shape<4, 1, 256, 8, double>(G, M, prog, num_sub, L, d, stream);
    }
    return launch_encode_shape<1, 1, 256, 8, double>(G, M, prog, num_sub, L, d, stream);
}

hipError_t launch_decode(const float *M, float *g, const DecTerm *terms, int nterms, int64_t d, float *w, float lr, hipStream_t stream)
{
    if (d >= 4) {
        const int nq = static_cast<int>((d + 3) / 4);
        decode_kernel<4><<<(nq + 255) / 256, 256, 0, stream>>>(M, g, terms, nterms, d, nq, w, lr);
    } else {
        const int nq = static_cast<int>(d);
        decode_kernel<1><<<(nq + 255) / 256, 256, 0, stream>>>(M, g, terms, nterms, d, nq, w, lr);
    }
    return hipGetLastError();
}

// ---- yardstick: a plain streaming read ------------------------------------------------------------------------------------
// Every workgroup walks one contiguous part of the array, eight non-temporal 16-byte loads in flight per thread; nothing but the
// loads and one add per word.  What this reaches is the practical ceiling for traffic that really comes from HBM (measured on
// MI355X: 7.0 to 7.1 TB/s; 6.0 to 6.3 without the non-temporal hint, or with a grid-wide stride instead of contiguous parts).
__global__ void __launch_bounds__(256) stream_read_kernel(const f4a *__restrict__ src, size_t n16, float *__restrict__ sink)
{
    const size_t per = ((n16 + gridDim.x - 1) / gridDim.x + 2047) / 2048 * 2048;      // whole unrolled iterations: parts start on 32 KB
    const size_t begin = per * blockIdx.x < n16 ? per * blockIdx.x : n16, end = begin + per < n16 ? begin + per : n16;
    float s = 0.f;
    size_t i = begin + threadIdx.x;
    for (; i + 7 * 256 < end; i += 8 * 256) {
        f4a v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u].x + v[u].y + v[u].z + v[u].w;
    }
    for (; i < end; i += 256) {
        const f4a v = __builtin_nontemporal_load(src + i);
        s += v.x + v.y + v.z + v.w;
    }
    s = wave_sum<true>(s);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

hipError_t launch_stream_read(const void *src, size_t n16, float *sink, hipStream_t stream)
{
    stream_read_kernel<<<kStreamGroups, 256, 0, stream>>>(static_cast<const f4a *>(src), n16, sink);
    return hipGetLastError();
}

// ---- device memory owned by the library --------------------------------------------------------------------------------
// For callers that cannot allocate (under stream capture, in serving loops): the scratch the aggregation needs beyond its inputs
// and outputs -- one encode program and the message rows M[N][d] -- lives in this array.  In host code the array's name is only a
// stand-in; its device address is asked for once per device, with that device current, and kept.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<char *> g_scratch_ptr[kMaxDevices];           // per device: where that device's copy of `scratch` lives
}  // namespace

hipError_t static_scratch(char **ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!sym) return hipErrorInvalidSymbol;
        p = static_cast<char *>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release);    // two threads racing here store the same address
    }
    *ptr = p;
    return hipSuccess;
}

// A block of host bytes travels as a kernel argument (kernel arguments are copied when the launch is enqueued) and one
// workgroup writes it out with vector stores.
struct UploadBlock { uint32_t word[960]; };
__global__ void __launch_bounds__(256) upload_kernel(uint32_t *__restrict__ dst, UploadBlock block, int nwords)
{
    for (int i = threadIdx.x; i < nwords; i += 256) dst[i] = block.word[i];
}

hipError_t launch_upload(char *dst, const char *src_host, size_t bytes, hipStream_t stream)
{
    for (size_t off = 0; off < bytes; off += sizeof(UploadBlock)) {
        UploadBlock block;
        const size_t len = bytes - off < sizeof(UploadBlock) ? bytes - off : sizeof(UploadBlock);
        std::memcpy(block.word, src_host + off, len);
        upload_kernel<<<1, 256, 0, stream>>>(reinterpret_cast<uint32_t *>(dst + off), block, static_cast<int>(len / 4));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- where do workgroups run? -----------------------------------------------------------------------------------------
// __smid() packs the hardware ids of the wave: die (XCC) above 6 bits of shader engine and compute unit.
__global__ void __launch_bounds__(64) placement_probe_kernel(uint32_t *__restrict__ out)
{
    const unsigned id = __smid();
    if (threadIdx.x == 0) out[blockIdx.x] = ((id >> 6) << 16) | (id & 63u);
}

hipError_t launch_placement_probe(uint32_t *out, int groups, hipStream_t stream)
{
    placement_probe_kernel<<<groups, 64, 0, stream>>>(out);
    return hipGetLastError();
}

hipError_t launch_update(float *w, const float *g, float lr, int64_t d, hipStream_t stream)
{
    update_kernel<<<static_cast<unsigned>((d + 255) / 256), 256, 0, stream>>>(w, g, lr, d);
    return hipGetLastError();
}

hipError_t launch_update_metrics(float *w, const float *g, float lr, const float *w_star, float *metrics, int64_t d, hipStream_t stream)
{
    update_metrics_kernel<<<1, 1024, 0, stream>>>(w, g, lr, w_star, metrics, d);
    return hipGetLastError();
}

}  // namespace cr

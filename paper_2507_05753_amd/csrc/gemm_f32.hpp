// FP32 matrix-core block GEMM for gfx950:  C[M x N] = op(A) * op(B) (+ addend) (+ bias)
//
// The contraction index k may be the contiguous index of an operand ("K-contiguous", KC) or
// its row index ("K-strided", KS):
//   A KC : A is M x K row-major          A KS : A is K x M row-major
//   B KC : B is N x K row-major          B KS : B is K x N row-major
// Forward  Y  = X W^T    : A = X  (KC), B = W (KC)     - the "X W^T" form of Sec. 4
// Backward dX = dY W     : A = dY (KC), B = W (KS)     - contraction over the out-features
//          dW = dY^T X   : A = dY (KS), B = X (KS)     - contraction over the rows (tokens);
// the paper calls these the transposed multiplications of the backward pass (Sec. 4.1) and
// needs the K-strided form for its transposed MLP as well (Sec. 5).  No operand is ever
// transposed in memory.
//
// One launch runs a *group* of up to four equally-shaped problems (the block products of
// all virtual ranks that belong to the same step of a pass: the products handed to a peer,
// or the kept products accumulated on top of the received partial, Eqs. (2) and (4)).
//
// Work decomposition
//   workgroup : 256 threads = 4 wavefronts (2 x 2), one 128 x 128 tile of C
//   wavefront : 64 x 64 sub-tile = 2 x 2 MFMA blocks of 32 x 32 (v_mfma_f32_32x32x2_f32)
//   K loop    : slabs of 32, two slab buffers in LDS used alternately
//
// gemm_f32_stream<A_KS, B_KS, RUNS> (operand rows 16-byte aligned, contiguous extents in whole
// 16-byte chunks): slabs go global -> LDS without passing through registers
// (buffer_load_dwordx4 ... lds), requested two slabs ahead of the math, one transfer after every
// second MFMA of a slab's last k-group (a burst of transfers, or any vector ALU instruction
// between MFMAs, holds up the matrix pipe measurably).  A wave-level load fills 1 KiB
// of LDS, lane l writing 16-byte slot l; rows are not padded, instead the lane chooses WHICH
// 16-byte chunk of global memory it fetches so that the later LDS reads are conflict-free:
//   KC operand slab: 128 rows x 32 k (128-B rows), chunk = slot ^ ((row >> 1) & 7); the MFMA
//      side reads 4 consecutive k of one row with one 128-bit read;
//   KS operand slab: 32 k x 128 rows-of-C (512-B rows), chunk = slot ^ (8 * ((k >> 2) & 1));
//      the MFMA side reads the same 4 k with four 32-bit reads 512 B apart.
// Either way a lane ends up with the same four operand values, so the MFMA code, the
// accumulator layout and the epilogue do not depend on the operand layouts.  Chunks outside
// the operand (past K, or past the last row / column) are fetched from outside the buffer
// descriptor and arrive as zeros, or are clamped to valid rows whose results are discarded.
// The received partial product (the addend) is loaded straight into the accumulators while
// the first slab is in flight; the epilogue adds the bias, applies the activation, adds the
// residual and stores.
//
// gemm_f32_guarded<A_KS, B_KS> (anything else): register loads with per-element bounds
// checks written to the same LDS positions.
//
// Tile order: consecutive workgroup ids land on different XCDs (round-robin dispatch), so
// the id is first folded into a per-XCD contiguous range, then walked column-major inside
// bands of 8 row-tiles.  The 64 workgroups an XCD has in flight (2 per CU) therefore form an
// 8 x 8 block of tiles that shares 8 A panels and 8 B panels in that XCD's L2.
//
// Tail: tiles are equal, so a launch whose tile count is not a multiple of the number of
// workgroups the chip holds (2 per CU) ends with a partial round in which part of the chip
// idles - 10 % of the time for 2312 long tiles on 512 slots.  Where an estimate says it pays, the
// launcher runs only whole rounds one tile per workgroup (RUNS = false) and cuts the K loops of
// the remaining tiles into equal runs of slabs, one run per workgroup of a second launch
// (RUNS = true; a run covers the end of one tile and the start of the next).  Each run writes
// its raw accumulators to a scratch tile, and a third small kernel (`gemm_f32_join`) adds a
// tile's runs in ascending k order, then the addend and the bias, applies the epilogue and
// stores C: no atomics, no flags, the same result on every run.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "epilogue.hpp"

namespace jg {

constexpr int kMaxGroup = 4;
constexpr int BM = 128;
constexpr int BN = 128;
constexpr int BK = 32;
constexpr int OPERAND_FLOATS = BM * BK;                  // one K slab of one operand = 16 KiB (BM == BN)
constexpr int STAGE_FLOATS = 2 * OPERAND_FLOATS;        // one K slab of A and B = 32 KiB
constexpr int GEMM_THREADS = 256;
constexpr int kNumXcd = 8;
constexpr int kBandRows = 8;                            // row-tiles per band
constexpr int kFlushSlabs = 32;                         // K extent of one first-level accumulation = 1024

struct GemmProblem {
    const float* A;       // M x K (KC) or K x M (KS), leading dimension lda
    const float* B;       // N x K (KC) or K x N (KS), leading dimension ldb
    float* C;             // M x N, leading dimension ldc
    const float* addend;  // M x N (ldadd) added in the epilogue, or nullptr
    const float* bias;    // length N added in the epilogue, or nullptr
    int lda, ldb, ldc, ldadd;
    const float* residual = nullptr;   // M x N (ldres) added after the activation, or nullptr
    int ldres = 0;
};

struct GemmGroup {
    GemmProblem p[kMaxGroup];
    int nprob;
    int M, N, K;          // common shape of every problem in the group
    int tiles_m, tiles_n; // ceil(M / BM), ceil(N / BN)
    int per_xcd;          // whole tiles handled by each XCD's workgroups (see launch_gemm_group)
    // split tail (all zero when it is not used): tiles [whole_tiles, total) are cut into runs
    int whole_tiles;      // tiles that get a workgroup of their own = kNumXcd * per_xcd when the tail is split
    int run_wgs;          // workgroups that share the remaining tiles' K loops
    int run_len, run_extra;   // run w covers run_len slabs, one more for w < run_extra
    float* run_tiles;     // scratch: two BM x BN tiles per run workgroup
    int act;              // kActNone / kActGelu, applied to (sum + bias) of every finished element
};

// First slab-iteration (tile-major, then slab) of run w; the runs partition [0, tail tiles * slabs).
__host__ __device__ inline int64_t run_begin(const GemmGroup& g, int w)
{
    return (int64_t)w * g.run_len + (w < g.run_extra ? w : g.run_extra);
}
// The run that contains slab-iteration `it`.
__host__ __device__ inline int run_of(const GemmGroup& g, int64_t it)
{
    const int64_t long_part = (int64_t)g.run_extra * (g.run_len + 1);
    return it < long_part ? (int)(it / (g.run_len + 1)) : g.run_extra + (int)((it - long_part) / g.run_len);
}

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;
constexpr int kBufferRsrcFlags = 0x00020000;   // raw 32-bit-element buffer descriptor, gfx9 family
constexpr int kMaxDirectLd = 1 << 21;          // keeps a tile's 128 rows * ld * 4 B below 2^30
constexpr int kOutOfBuffer = 0x7FFFFFF0;       // byte offset beyond any such tile: reads as zero

// s_waitcnt that waits only for the vector-memory counter to drop to n (n < 64)
#define JG_WAIT_VMCNT(n) \
    __builtin_amdgcn_s_waitcnt(((n) & 0xF) | ((((n) >> 4) & 0x3) << 14) | (0x7 << 4) | (0xF << 8))

struct TileCoord {
    int prob, m0, n0;
};

__device__ __forceinline__ TileCoord decode_tile(const GemmGroup& g, int lid)
{
    const int tiles_per_prob = g.tiles_m * g.tiles_n;
    const int prob = lid / tiles_per_prob;
    const int t = lid - prob * tiles_per_prob;
    const int band = t / (kBandRows * g.tiles_n);
    const int in_band = t - band * (kBandRows * g.tiles_n);
    const int band_first = band * kBandRows;
    const int band_rows = min(kBandRows, g.tiles_m - band_first);
    TileCoord c;
    c.prob = prob;
    c.m0 = (band_first + in_band % band_rows) * BM;
    c.n0 = (in_band / band_rows) * BN;
    return c;
}

// Lane coordinates inside the workgroup's tile.
struct LaneMap {
    int wave, lane, wm, wn, lr, lk;
    __device__ __forceinline__ void init(int tid)
    {
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS slot addresses in scalar registers
        lane = tid & 63;
        wm = wave >> 1;      // the wave's 64-row half of the tile
        wn = wave & 1;       // ... and 64-column half
        lr = lane & 31;      // row (A) / column (B) of the 32-wide MFMA block this lane feeds
        lk = lane >> 5;      // which of the instruction's two k slots
    }
};

// How a lane fetches its MFMA operand values of one operand from a slab in LDS.  For k-group
// g (8 consecutive k) lanes with lk = 0 take k = 8 g .. 8 g + 3 and lanes with lk = 1 the next
// four; the t-th MFMA of the group contracts the k slots {8 g + t, 8 g + 4 + t}.  A and B use
// the same assignment, so the products pair up whatever the two layouts are.
template <bool KS>
struct FragReader {
    int off[2];   // float offset of the lane's data for blocks 0 / 1 (operand base included)
    int sw[2];    // KC only: the row's chunk swizzle
    // half = the wave's 64-wide half of the tile along this operand's C dimension
    __device__ __forceinline__ void init(int operand_base, int half, int lr, int lk)
    {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int r = half * 64 + b * 32 + lr;
            if (KS) {
                off[b] = operand_base + (4 * lk) * BM + (r ^ (32 * lk));
                sw[b] = 0;
            } else {
                off[b] = operand_base + r * BK;
                sw[b] = (r >> 1) & 7;
            }
        }
    }
    __device__ __forceinline__ float4 read(const float* s, int g, int b, int lk) const
    {
        if (KS) {
            const float* p = s + off[b] + g * 8 * BM;
            return make_float4(p[0], p[BM], p[2 * BM], p[3 * BM]);
        } else {
            return *reinterpret_cast<const float4*>(s + off[b] + (((g * 2 + lk) ^ sw[b]) << 2));
        }
    }
};

__device__ __forceinline__ void mfma_group(floatx16 (&acc)[2][2], const float4 (&fa)[2], const float4 (&fb)[2])
{
    const float av[2][4] = {{fa[0].x, fa[0].y, fa[0].z, fa[0].w}, {fa[1].x, fa[1].y, fa[1].z, fa[1].w}};
    const float bv[2][4] = {{fb[0].x, fb[0].y, fb[0].z, fb[0].w}, {fb[1].x, fb[1].y, fb[1].z, fb[1].w}};
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][tt], bv[j][tt], acc[i][j], 0, 0, 0);
}

// All-zero accumulators, written by the matrix pipe: one instruction per 16 registers instead of 16
// vector moves.  This matters because the zeroing runs while the other resident workgroup
// saturates the matrix pipe, where every vector ALU instruction waits for a gap between MFMAs.
__device__ __forceinline__ void zero_acc(floatx16 (&acc)[2][2])
{
    const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(0.f, 0.f, zero, 0, 0, 0);
}

// Two-level accumulation.  The MFMAs add into `acc`; every kFlushSlabs slabs `acc` is folded
// into `sum` and cleared.  A single FP32 running sum over K same-sign products drifts by about
// sqrt(K / 6) roundings of the whole sum (over 1e-6 of it from K of a few thousand); with
// chunks of 1024 the drift stays near 1e-7 of the magnitude for any K this library accepts.
__device__ __forceinline__ void fold_acc(floatx16 (&sum)[2][2], floatx16 (&acc)[2][2])
{
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[i][j][v] += acc[i][j][v];
    zero_acc(acc);
}

// Accumulator register v of lane (lr, lk) holds row 8 (v / 4) + 4 lk + v % 4, column lr of
// its 32 x 32 block, so one load / store instruction touches two 128-byte row segments.

// acc = addend tile (the partial product received from the peer), or zero.
__device__ __forceinline__ void init_acc(const GemmProblem& P, int M, int N, int m0, int n0,
                                         const LaneMap& L, floatx16 (&acc)[2][2])
{
    const float* __restrict__ addend = P.addend;
    if (!addend) {
        zero_acc(acc);
        return;
    }
    const int ldadd = P.ldadd;
    const int row_base = m0 + L.wm * 64 + 4 * L.lk;
    const int col_base = n0 + L.wn * 64 + L.lr;
    if (ldadd <= kMaxDirectLd) {
        // The lane's position goes into one vector offset per column block and the row of each access into
        // a scalar offset, so the 64 loads of a tile whose rows are all inside need no vector ALU work (a
        // workgroup that starts up shares its SIMDs with one that is saturating the matrix pipe, and every
        // vector ALU instruction there waits for a gap between MFMAs).  A tile that hangs over the last
        // column takes the same path: the descriptor ends at the last valid column, a lane whose column
        // lies past N gets an offset outside it, and what it reads is zero.  A tile that hangs over the last
        // row (ROWS_IN = false) masks each access the same way, by the rows the lane has left: a compare
        // and a select per access instead of a 64-bit address and a predicated load.
        auto direct = [&](auto rows_in_c) __attribute__((always_inline)) {
            constexpr bool ROWS_IN = decltype(rows_in_c)::value;
            const int nrows = ROWS_IN ? BM : M - m0;
            const int ncols = min(BN, N - n0);
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(addend + (int64_t)m0 * ldadd + n0), 0, ((nrows - 1) * ldadd + ncols) * 4, kBufferRsrcFlags);
            const int lane_col = L.wn * 64 + L.lr;
            const int lane_row = L.wm * 64 + 4 * L.lk;
            const int lane_off = (lane_row * ldadd + lane_col) * 4;
            const int off[2] = {lane_col < ncols ? lane_off : kOutOfBuffer, lane_col + 32 < ncols ? lane_off + 128 : kOutOfBuffer};
            const int slack = nrows - lane_row;      // rows of the tile at or below the lane's first that are inside
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int rel = i * 32 + 8 * (v >> 2) + (v & 3);
                        const int voff = (ROWS_IN || rel < slack) ? off[j] : kOutOfBuffer;
                        acc[i][j][v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, voff, rel * ldadd * 4, 0));
                    }
        };
        if (m0 + BM <= M) direct(std::true_type{});
        else direct(std::false_type{});
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = col_base + j * 32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                    acc[i][j][v] = (row < M && col < N) ? addend[(int64_t)row * ldadd + col] : 0.f;
                }
            }
    }
}

// C = act(acc + bias) + residual for the tile at (m0, n0).
__device__ __forceinline__ void store_tile(const GemmProblem& P, int M, int N, int m0, int n0,
                                           const LaneMap& L, const floatx16 (&acc)[2][2], int act)
{
    const float* __restrict__ bias = P.bias;
    const float* __restrict__ residual = P.residual;
    float* __restrict__ C = P.C;
    const int ldc = P.ldc;
    const int row_base = m0 + L.wm * 64 + 4 * L.lk;     // + i * 32 + 8 (v / 4) + v % 4
    const int col_base = n0 + L.wn * 64 + L.lr;         // + j * 32
    if (ldc <= kMaxDirectLd && (!residual || P.ldres <= kMaxDirectLd)) {
        // No per-element bounds checks and no 64-bit addresses: lane position in one vector offset per column
        // block, the row of each store in a scalar offset.  Columns past N (the tile that hangs over the last
        // column; one in sixteen at N = 2000) are left to the descriptor: such a lane's offset lies outside
        // it, its stores are dropped and its loads read zero.  With per-element checks that tile's epilogue
        // took about 85 us of vector ALU work squeezed between the other workgroup's MFMAs, against a 225 us
        // tile.  Rows past M (ROWS_IN = false: the tile that hangs over the last row) are masked per access
        // by the rows the lane has left.
        auto direct = [&](auto rows_in_c) __attribute__((always_inline)) {
        constexpr bool ROWS_IN = decltype(rows_in_c)::value;
        const int nrows = ROWS_IN ? BM : M - m0;
        const int ncols = min(BN, N - n0);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            C + (int64_t)m0 * ldc + n0, 0, ((nrows - 1) * ldc + ncols) * 4, kBufferRsrcFlags);
        const int lane_col = L.wn * 64 + L.lr;
        const int lane_row = L.wm * 64 + 4 * L.lk;
        const int lane_off = (lane_row * ldc + lane_col) * 4;
        const bool in[2] = {lane_col < ncols, lane_col + 32 < ncols};
        const int off[2] = {in[0] ? lane_off : kOutOfBuffer, in[1] ? lane_off + 128 : kOutOfBuffer};
        const int slack = nrows - lane_row;
        if (!bias && !act && !residual) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float value = acc[i][j][v];   // a copy: bit-casting the vector element in place reads element 0
                        const int rel = i * 32 + 8 * (v >> 2) + (v & 3);
                        const int voff = (ROWS_IN || rel < slack) ? off[j] : kOutOfBuffer;
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, value), rsrc, voff, rel * ldc * 4, 0);
                    }
        } else {
            const int ldres = P.ldres;
            const __amdgpu_buffer_rsrc_t res_rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(residual ? residual + (int64_t)m0 * ldres + n0 : C), 0,
                residual ? ((nrows - 1) * ldres + ncols) * 4 : 0, kBufferRsrcFlags);
            const int res_lane = (lane_row * ldres + lane_col) * 4;
            const int res_offs[2] = {in[0] ? res_lane : kOutOfBuffer, in[1] ? res_lane + 128 : kOutOfBuffer};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float bj = (bias && in[j]) ? bias[col_base + j * 32] : 0.f;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    float res[16];
                    if (residual) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int rel = i * 32 + 8 * (v >> 2) + (v & 3);
                            const int voff = (ROWS_IN || rel < slack) ? res_offs[j] : kOutOfBuffer;
                            res[v] = __builtin_bit_cast(
                                float, __builtin_amdgcn_raw_buffer_load_b32(res_rsrc, voff, rel * ldres * 4, 0));
                        }
                    }
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float y = activate(acc[i][j][v] + bj, act);
                        if (residual) y += res[v];
                        const int rel = i * 32 + 8 * (v >> 2) + (v & 3);
                        const int voff = (ROWS_IN || rel < slack) ? off[j] : kOutOfBuffer;
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, y), rsrc, voff, rel * ldc * 4, 0);
                    }
                }
            }
        }
        };
        if (m0 + BM <= M) direct(std::true_type{});
        else direct(std::false_type{});
    } else {                              // a leading dimension too long for 32-bit offsets: every element checked, 64-bit addresses
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = col_base + j * 32;
                if (col >= N) continue;
                const float bj = bias ? bias[col] : 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (row < M) {
                        float y = activate(acc[i][j][v] + bj, act);
                        if (residual) y += residual[(int64_t)row * P.ldres + col];
                        C[(int64_t)row * ldc + col] = y;
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Slab loaders.  A loader is set up once per tile for one operand and then asked for slab kt.
// LDS positions: a wave-level transfer fills 1 KiB; unit u = p * 4 + wave (p = 0..3) is the
// u-th KiB of the operand's 16 KiB slab, lane l its l-th 16-byte slot.
//   KC: unit u = rows 8 u .. 8 u + 7 of the tile, 8 slots per row.
//   KS: unit u = k rows 2 u, 2 u + 1 of the slab, 32 slots per row.
// ------------------------------------------------------------------------------------------
struct OperandView {
    const float* base;   // element (row-of-C 0, k 0) of the whole operand
    int ld;              // leading dimension
    int extent;          // M (for A) or N (for B): number of rows-of-C the operand spans
    int origin;          // m0 or n0 of this tile
};

template <bool KS>
struct StreamLoader {
    int voff[4];                        // byte offsets of this lane's four chunks
    int oob[4];                         // KC: kOutOfBuffer for chunks that lie at or past column K in the ragged last slab, else 0
    __amdgpu_buffer_rsrc_t rsrc;        // KC: the tile's rows; KS: rebuilt for every slab
    const float* tile_base;             // KS: element (origin, k = 0)
    int ld, K, valid;                   // valid = rows-of-C of this tile inside the operand
    int kt_ragged;                      // KC: the slab that needs the zero fill, or -1

    __device__ __forceinline__ void init(const OperandView& v, int K_, int wave, int lane)
    {
        ld = v.ld;
        K = K_;
        valid = min(BM, v.extent - v.origin);
        kt_ragged = (K % BK) ? K / BK : -1;
        if (KS) {
            tile_base = v.base + v.origin;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int k = (p * 4 + wave) * 2 + (lane >> 5);
                const int chunk = (lane & 31) ^ (8 * ((k >> 2) & 1));
                voff[p] = (k * ld + chunk * 4) * 4;
                oob[p] = 0;
            }
        } else {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int r = (p * 4 + wave) * 8 + (lane >> 3);
                const int chunk = (lane & 7) ^ ((r >> 1) & 7);
                // rows past the edge are clamped to the last valid row: read but never stored
                voff[p] = (min(r, valid - 1) * ld + chunk * 4) * 4;
                oob[p] = chunk * 4 < K % BK ? 0 : kOutOfBuffer;
            }
            // base = first row of the tile, extent = up to the end of its last valid row: an
            // out-of-range offset reads zero instead of faulting
            const int64_t bytes = ((int64_t)(valid - 1) * ld + K) * 4;
            rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(v.base + (int64_t)v.origin * ld), 0,
                                                     (int)bytes, kBufferRsrcFlags);
        }
    }
    // Requests are asynchronous: the data is in LDS once this thread's vmcnt has drained and a
    // barrier has passed.  begin(kt) fixes the slab; issue(p) then enqueues the p-th of this
    // lane's four 16-byte transfers.  They are separate calls because the kernel spreads the
    // transfers between its MFMAs: issued back to back they hold up the matrix pipe, and so
    // does any vector ALU work between the MFMAs, which is why issue() does none.  A KC
    // operand's ragged last slab needs per-lane masking and goes through request() instead.
    int soff;                           // KC: byte offset of the slab inside a row
    __device__ __forceinline__ void begin(int kt)
    {
        if (KS) {
            // buffer over the k rows of this slab that exist; rows past K and columns past the
            // operand's edge fall outside it and arrive as zeros
            const int rows = min(BK, K - kt * BK);
            const int64_t bytes = ((int64_t)(rows - 1) * ld + valid) * 4;
            rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(tile_base + (int64_t)kt * BK * ld), 0,
                                                     (int)bytes, kBufferRsrcFlags);
            soff = 0;
        } else {
            soff = kt * BK * 4;
        }
    }
    __device__ __forceinline__ void issue(int p, float* operand_slab, int wave) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(operand_slab + (p * 4 + wave) * 256), 16, voff[p],
                                                 soff, 0, 0);
    }
    // all four transfers of any slab at once
    __device__ __forceinline__ void request(int kt, float* operand_slab, int wave)
    {
        begin(kt);
        // in the ragged slab the chunks at or past column K get an offset beyond the buffer and read as zero
        const int mask = (!KS && kt == kt_ragged) ? -1 : 0;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(operand_slab + (p * 4 + wave) * 256), 16,
                                                     voff[p] | (oob[p] & mask), soff, 0, 0);
    }
};

// Synchronous loader for operands that rule out 16-byte transfers: four guarded 4-element
// reads per slab, written to the positions the stream loader would have filled.
template <bool KS>
struct GuardedLoader {
    const float* base;
    int ld, K, extent, origin;
    __device__ __forceinline__ void init(const OperandView& v, int K_)
    {
        base = v.base; ld = v.ld; K = K_; extent = v.extent; origin = v.origin;
    }
    // element (row-of-C r, k), zero outside the operand
    __device__ __forceinline__ float at(int r, int k) const
    {
        if (r >= extent || k >= K) return 0.f;
        return KS ? base[(int64_t)k * ld + r] : base[(int64_t)r * ld + k];
    }
    __device__ __forceinline__ void fetch(int kt, int wave, int lane, float4 (&reg)[4]) const
    {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (KS) {
                const int k = (p * 4 + wave) * 2 + (lane >> 5);
                const int chunk = (lane & 31) ^ (8 * ((k >> 2) & 1));
                const int r = origin + chunk * 4, kk = kt * BK + k;
                reg[p] = make_float4(at(r, kk), at(r + 1, kk), at(r + 2, kk), at(r + 3, kk));
            } else {
                const int rr = (p * 4 + wave) * 8 + (lane >> 3);
                const int chunk = (lane & 7) ^ ((rr >> 1) & 7);
                const int r = origin + rr, kk = kt * BK + chunk * 4;
                reg[p] = make_float4(at(r, kk), at(r, kk + 1), at(r, kk + 2), at(r, kk + 3));
            }
        }
    }
    __device__ __forceinline__ static void put(float* operand_slab, int wave, int lane, const float4 (&reg)[4])
    {
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(operand_slab + (p * 4 + wave) * 256 + lane * 4) = reg[p];
    }
};

// ------------------------------------------------------------------------------------------
// asynchronous-load kernel, two workgroups per CU.  RUNS = false: one whole tile per workgroup
// (tiles [0, whole_tiles)).  RUNS = true: one run of slabs of the split tail per workgroup; it is
// a separate instance, launched after the first on the same stream, so that the whole-tile code
// carries none of the run bookkeeping.
// ------------------------------------------------------------------------------------------
template <bool A_KS, bool B_KS, bool RUNS>
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_f32_stream(const GemmGroup g)
{
    // One array per slab buffer: distinct LDS objects let the compiler prove that the
    // asynchronous fill of one does not alias the reads of the other, so it does not make
    // every LDS read wait for the loads still in flight.
    __shared__ __align__(16) float ring0[STAGE_FLOATS];
    __shared__ __align__(16) float ring1[STAGE_FLOATS];

    const int M = g.M, N = g.N, K = g.K;
    const int nkt_all = (K + BK - 1) / BK;
    LaneMap L;
    L.init(threadIdx.x);

    // What this workgroup does: one whole tile, or one run of slab-iterations [it, it_end) of the
    // tail tiles, which touches one or two tiles.
    constexpr bool is_run = RUNS;
    int lid = 0;
    int64_t it = 0, it_end = 0;
    if (is_run) {
        it = run_begin(g, (int)blockIdx.x);
        it_end = run_begin(g, (int)blockIdx.x + 1);
    } else {
        lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
        if (lid >= g.whole_tiles) return;   // whole workgroup leaves before any barrier
    }

    for (int pass = 0;; ++pass) {   // one pass per tile touched: 1 for a whole tile, 1 or 2 for a run
    int k0 = 0, k1 = nkt_all;       // slabs of this pass
    if (is_run) {
        if (it >= it_end) break;
        const int t = (int)(it / nkt_all);
        k0 = (int)(it - (int64_t)t * nkt_all);
        k1 = (int)min((int64_t)nkt_all, k0 + (it_end - it));
        lid = g.whole_tiles + t;
    }
    const TileCoord tc = decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];
    const int m0 = tc.m0, n0 = tc.n0;
    // where the accumulators start from and go to: the problem's addend / C / bias, or (a run)
    // zero and a scratch tile of its own
    GemmProblem out = P;
    int out_m = M, out_n = N, out_m0 = m0, out_n0 = n0;
    if (is_run) {
        out.C = g.run_tiles + ((int64_t)2 * (int)blockIdx.x + pass) * (BM * BN);
        out.ldc = BN;
        out.addend = nullptr;
        out.bias = nullptr;
        out.residual = nullptr;
        out_m = BM; out_n = BN; out_m0 = 0; out_n0 = 0;
    }
    const int nkt = k1;             // the pass ends before this slab
    // slabs up to nkt_spread - 1 are requested in the spread form; a ragged last slab is not, if an
    // operand is K-contiguous
    const bool ragged_burst = (!A_KS || !B_KS) && (K % BK) != 0 && k1 == nkt_all;
    const int nkt_spread = ragged_burst ? nkt - 1 : nkt;
    const int kt_burst = ragged_burst ? nkt - 1 : -1;

    StreamLoader<A_KS> load_a;
    StreamLoader<B_KS> load_b;
    load_a.init(OperandView{P.A, P.lda, M, m0}, K, L.wave, L.lane);
    load_b.init(OperandView{P.B, P.ldb, N, n0}, K, L.wave, L.lane);
    FragReader<A_KS> frag_a;
    FragReader<B_KS> frag_b;
    frag_a.init(0, L.wm, L.lr, L.lk);
    frag_b.init(OPERAND_FLOATS, L.wn, L.lr, L.lk);

    auto request_slab = [&](int kt, float* slab) {
        load_a.request(kt, slab, L.wave);
        load_b.request(kt, slab + OPERAND_FLOATS, L.wave);
    };
    auto read_frags = [&](const float* slab, int kk, float4 (&fa)[2], float4 (&fb)[2]) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            fa[b] = frag_a.read(slab, kk, b, L.lk);
            fb[b] = frag_b.read(slab, kk, b, L.lk);
        }
    };

    floatx16 acc[2][2], sum[2][2];
    float4 fa[2][2], fb[2][2];   // two register sets of MFMA operands (even / odd k-group)

    // The 16 MFMAs of one k-group; when `spread` > 0, this lane's eight transfers of slab
    // `kt_req` into `slab` go out between them, one after every second MFMA.  Issued in a
    // burst, the transfers keep the matrix pipe waiting measurably longer.
    auto mfma_group_requesting = [&](const float4 (&a)[2], const float4 (&b)[2], int spread, int kt_req,
                                     float* slab) {
        const float av[2][4] = {{a[0].x, a[0].y, a[0].z, a[0].w}, {a[1].x, a[1].y, a[1].z, a[1].w}};
        const float bv[2][4] = {{b[0].x, b[0].y, b[0].z, b[0].w}, {b[1].x, b[1].y, b[1].z, b[1].w}};
        if (spread > 0) {
            load_a.begin(kt_req);
            load_b.begin(kt_req);
        }
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][tt], bv[j][tt], acc[i][j], 0, 0, 0);
                    const int idx = tt * 4 + i * 2 + j;
                    if ((idx & 1) == 0 && spread > 0) {
                        if (idx < 8) load_a.issue(idx >> 1, slab, L.wave);
                        else load_b.issue((idx >> 1) & 3, slab + OPERAND_FLOATS, L.wave);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
    };

    // One slab: inside it the operands of k-group kk + 1 are requested before the 16 MFMAs of
    // group kk are issued, so LDS latency hides behind about a thousand matrix-pipe cycles.
    // The slab boundary (wait for the next slab, barrier, first operand read of the next slab)
    // sits before the LAST group's MFMAs for the same reason, and the requests for the slab
    // after next go out between those MFMAs.  The scheduling fences keep the compiler from
    // undoing this order.
    auto step = [&](int kt, float* cur, const float* nxt) {
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            read_frags(cur, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            mfma_group(acc, fa[kk & 1], fb[kk & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
        JG_WAIT_VMCNT(0);   // this thread's part of slab kt + 1 has landed
        __syncthreads();    // ... and everyone's; all waves hold their last operands of slab kt
        // the slab after next: spread between the MFMAs below, or (ragged last slab of a
        // K-contiguous operand, once per tile) all at once here
        const int spread = nkt_spread - (kt + 2);   // > 0: request slab kt + 2 between the MFMAs
        if (kt + 2 == kt_burst) request_slab(kt + 2, cur);
        if (kt + 1 < nkt) read_frags(nxt, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        mfma_group_requesting(fa[1], fb[1], spread, kt + 2, cur);
        __builtin_amdgcn_sched_barrier(0);
    };

    request_slab(k0, ring0);
    init_acc(out, out_m, out_n, out_m0, out_n0, L, sum);   // its loads fly together with the first slab
    zero_acc(acc);
    JG_WAIT_VMCNT(0);
    __syncthreads();
    if (k0 + 1 < nkt) request_slab(k0 + 1, ring1);
    read_frags(ring0, 0, fa[0], fb[0]);
    __builtin_amdgcn_sched_barrier(0);
    int kt = k0;
    for (int pair = 0; kt + 1 < nkt; kt += 2, ++pair) {
        step(kt, ring0, ring1);
        step(kt + 1, ring1, ring0);
        if ((pair & (kFlushSlabs / 2 - 1)) == kFlushSlabs / 2 - 1) fold_acc(sum, acc);
    }
    if (kt < nkt) step(kt, ring0, ring1);
    fold_acc(sum, acc);

    store_tile(out, out_m, out_n, out_m0, out_n0, L, sum, is_run ? (int)kActNone : g.act);
    if (!is_run) break;
    it += k1 - k0;
    __syncthreads();   // every wave is done with the slab buffers before the next pass refills them
    }
}

// Second kernel of a launch whose tail was split: kJoinSlices workgroups per tail tile, each with a band of 16
// of its rows, add the tile's runs in ascending k order, then the addend and the bias, apply the activation, add
// the residual and store C.  (One workgroup per tile took 40 us on a small problem cut into eight runs per tile:
// too few loads in flight.)
constexpr int kJoinSlices = 8;
__global__ __launch_bounds__(GEMM_THREADS) void gemm_f32_join(const GemmGroup g)
{
    const int t = blockIdx.x / kJoinSlices, slice = blockIdx.x % kJoinSlices;
    const int nkt = (g.K + BK - 1) / BK;
    const TileCoord tc = decode_tile(g, g.whole_tiles + t);
    const GemmProblem& P = g.p[tc.prob];
    const int64_t it0 = (int64_t)t * nkt;
    const int w_first = run_of(g, it0), w_last = run_of(g, it0 + nkt - 1);
    const float* __restrict__ addend = P.addend;
    const float* __restrict__ bias = P.bias;
    constexpr int kPieces = BM * BN / 4 / kJoinSlices;      // 4-element pieces of a slice
#pragma unroll 1
    for (int u = 0; u < kPieces / GEMM_THREADS; ++u) {
        const int idx = slice * kPieces + threadIdx.x + GEMM_THREADS * u;   // one 4-element piece of a tile row
        const int r = idx / (BN / 4), c = (idx % (BN / 4)) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int w = w_first; w <= w_last; ++w) {
            const int first_tile = (int)(run_begin(g, w) / nkt);   // the tile of the run's pass 0
            const float* src = g.run_tiles + ((int64_t)2 * w + (t - first_tile)) * (BM * BN);
            const float4 p = *reinterpret_cast<const float4*>(src + r * BN + c);
            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        }
        const int row = tc.m0 + r, col = tc.n0 + c;
        if (row >= g.M) continue;
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (col + q >= g.N) break;
            float y = e[q];
            if (addend) y += addend[(int64_t)row * P.ldadd + col + q];
            if (bias) y += bias[col + q];
            y = activate(y, g.act);
            if (P.residual) y += P.residual[(int64_t)row * P.ldres + col + q];
            P.C[(int64_t)row * P.ldc + col + q] = y;
        }
    }
}

// ------------------------------------------------------------------------------------------
// guarded kernel: any alignment, any sizes; synchronous slab loads through registers
// ------------------------------------------------------------------------------------------
template <bool A_KS, bool B_KS>
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_f32_guarded(const GemmGroup g)
{
    __shared__ __align__(16) float slab[STAGE_FLOATS];

    const int lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
    if (lid >= g.whole_tiles) return;   // the guarded kernel never splits: whole_tiles = all tiles
    const TileCoord tc = decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];
    const int M = g.M, N = g.N, K = g.K;

    LaneMap L;
    L.init(threadIdx.x);
    GuardedLoader<A_KS> load_a;
    GuardedLoader<B_KS> load_b;
    load_a.init(OperandView{P.A, P.lda, M, tc.m0}, K);
    load_b.init(OperandView{P.B, P.ldb, N, tc.n0}, K);
    FragReader<A_KS> frag_a;
    FragReader<B_KS> frag_b;
    frag_a.init(0, L.wm, L.lr, L.lk);
    frag_b.init(OPERAND_FLOATS, L.wn, L.lr, L.lk);

    floatx16 acc[2][2], sum[2][2];
    init_acc(P, M, N, tc.m0, tc.n0, L, sum);
    zero_acc(acc);
    float4 fa[2][2], fb[2][2];
    const int nkt = (K + BK - 1) / BK;
    for (int kt = 0; kt < nkt; ++kt) {
        if (kt && (kt & (kFlushSlabs - 1)) == 0) fold_acc(sum, acc);
        float4 ra[4], rb[4];
        load_a.fetch(kt, L.wave, L.lane, ra);
        load_b.fetch(kt, L.wave, L.lane, rb);
        __syncthreads();        // everyone is done reading the previous slab
        GuardedLoader<A_KS>::put(slab, L.wave, L.lane, ra);
        GuardedLoader<B_KS>::put(slab + OPERAND_FLOATS, L.wave, L.lane, rb);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                fa[kk & 1][b] = frag_a.read(slab, kk, b, L.lk);
                fb[kk & 1][b] = frag_b.read(slab, kk, b, L.lk);
            }
            mfma_group(acc, fa[kk & 1], fb[kk & 1]);
        }
    }
    fold_acc(sum, acc);
    store_tile(P, M, N, tc.m0, tc.n0, L, sum, g.act);
}

enum GemmLayout { kGemmNT = 0 /* A KC, B KC */, kGemmNN = 1 /* A KC, B KS */, kGemmTN = 2 /* A KS, B KS */ };

// Can this operand take the asynchronous 16-byte path?
inline bool operand_streams(const float* p, int ld, bool ks, int extent, int K)
{
    if (((uintptr_t)p & 15) || (ld & 3) || ld > kMaxDirectLd) return false;
    return ks ? (extent % 4) == 0 : (K % 4) == 0;   // the contiguous extent comes in whole chunks
}

template <bool A_KS, bool B_KS>
inline void launch_gemm_layout(const GemmGroup& g, bool stream_ok, hipStream_t stream)
{
    const unsigned grid = (unsigned)(kNumXcd * g.per_xcd);   // whole tiles
    if (stream_ok) {
        if (grid)
            hipLaunchKernelGGL((gemm_f32_stream<A_KS, B_KS, false>), dim3(grid), dim3(GEMM_THREADS), 0, stream, g);
        if (g.run_wgs)
            hipLaunchKernelGGL((gemm_f32_stream<A_KS, B_KS, true>), dim3((unsigned)g.run_wgs), dim3(GEMM_THREADS), 0,
                               stream, g);
    } else
        hipLaunchKernelGGL((gemm_f32_guarded<A_KS, B_KS>), dim3(grid), dim3(GEMM_THREADS), 0, stream, g);
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
constexpr int kMinRunSlabs = 32;   // a run shorter than this is not worth its start-up and its scratch tile ...
constexpr int kMinRunSlabsFewRounds = 8;   // ... unless the launch has few rounds of tiles, where the last one weighs more,
constexpr int kMinRunSlabsSubRound = 4;    // ... or not even half a round: a small problem, cut up to fill the chip
constexpr int kRunOverheadSlabs = 6;   // start-up, scratch store and join of a run, in slab times

// How a launch of `total` tiles with `nkt` slabs each is divided on a chip that holds `slots`
// workgroups: `whole` tiles one per workgroup, the rest (if that pays) in `runs` equal runs.
struct TailSplit {
    int whole, runs, run_len, run_extra;
};
inline TailSplit plan_tail(int64_t total, int nkt, int slots)
{
    TailSplit t = {(int)total, 0, 0, 0};
    if (slots < kNumXcd) return t;
    slots -= slots % kNumXcd;                         // whole rounds must fill every XCD's range evenly
    const int64_t rest = total % slots;
    if (rest == 0) return t;
    const int64_t iters = rest * nkt;
    const int min_slabs = 2 * total < slots ? kMinRunSlabsSubRound : total <= 4 * (int64_t)slots ? kMinRunSlabsFewRounds : kMinRunSlabs;
    // (a problem smaller than the chip gets one run per compute unit at most: a workgroup alone on its unit runs
    // nearly twice as fast, and half as many scratch tiles pass through the join)
    const int64_t cap = 2 * total < slots ? slots / 2 : slots;
    const int64_t runs = iters / min_slabs < cap ? iters / min_slabs : cap;
    if (runs <= rest) return t;                       // no finer than whole tiles: nothing gained
    // Estimated time of the last round either way, in slab times at the two-workgroups-per-CU rate
    // (a workgroup alone on its CU runs about 1.8 times as fast); split only for a saving of at least
    // 3 % of the launch.
    auto round_time = [slots](int64_t wgs, int64_t slabs) { return (double)slabs * (2 * wgs <= slots ? 0.55 : 1.0); };
    const double saving = round_time(rest, nkt) - (round_time(runs, (iters + runs - 1) / runs) + kRunOverheadSlabs);
    if (saving < 0.03 * ((double)total / slots) * nkt) return t;
    t.whole = (int)(total - rest);
    t.runs = (int)runs;
    t.run_len = (int)(iters / runs);
    t.run_extra = (int)(iters % runs);
    return t;
}
// Scratch bytes launch_gemm_group may use for a launch of `total` tiles (0: the tail is not split).
inline size_t tail_scratch_bytes(int64_t total, int K, int slots)
{
    const TailSplit t = plan_tail(total, (K + BK - 1) / BK, slots);
    return (size_t)t.runs * 2 * BM * BN * sizeof(float);
}

// Fills the derived fields of `g` and enqueues the GEMM kernel.  `scratch` (device, 16-byte
// aligned, may be null) enables the split tail when it holds tail_scratch_bytes(...) bytes;
// `*needs_join` then tells the caller to enqueue launch_gemm_join(g) next on the same stream.
// Preconditions (checked by the C-ABI layer): 1 <= nprob <= 4; M, N, K >= 1; all pointers valid
// for their shapes; leading dimensions at least the contiguous extent of their operand.
inline hipError_t launch_gemm_group(GemmGroup& g, int layout, hipStream_t stream, float* scratch,
                                    size_t scratch_bytes, int slots, bool* needs_join)
{
    *needs_join = false;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const int64_t total = (int64_t)g.nprob * g.tiles_m * g.tiles_n;
    // The tile index is a 32-bit block id (and the grid is one-dimensional): refuse a product
    // with more tiles than that instead of wrapping around.
    if (total + kNumXcd + slots > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const bool a_ks = layout == kGemmTN, b_ks = layout != kGemmNT;
    bool stream_ok = true;
    for (int i = 0; i < g.nprob; ++i) {
        stream_ok = stream_ok && operand_streams(g.p[i].A, g.p[i].lda, a_ks, g.M, g.K) &&
                    operand_streams(g.p[i].B, g.p[i].ldb, b_ks, g.N, g.K);
    }
    TailSplit t = {(int)total, 0, 0, 0};
    if (stream_ok && scratch) {
        t = plan_tail(total, (g.K + BK - 1) / BK, slots);
        if ((size_t)t.runs * 2 * BM * BN * sizeof(float) > scratch_bytes) t = {(int)total, 0, 0, 0};
    }
    g.whole_tiles = t.whole;
    g.run_wgs = t.runs;
    g.run_len = t.run_len;
    g.run_extra = t.run_extra;
    g.run_tiles = t.runs ? scratch : nullptr;
    g.per_xcd = (t.whole + kNumXcd - 1) / kNumXcd;   // exact when the tail is split (whole is a multiple of 8)
    switch (layout) {
    case kGemmNT: launch_gemm_layout<false, false>(g, stream_ok, stream); break;
    case kGemmNN: launch_gemm_layout<false, true>(g, stream_ok, stream); break;
    case kGemmTN: launch_gemm_layout<true, true>(g, stream_ok, stream); break;
    default: return hipErrorInvalidValue;
    }
    *needs_join = t.runs > 0;
    return hipGetLastError();
}

// The second kernel of a launch whose tail was split (see launch_gemm_group).
inline hipError_t launch_gemm_join(const GemmGroup& g, hipStream_t stream)
{
    const int tail_tiles = g.nprob * g.tiles_m * g.tiles_n - g.whole_tiles;
    hipLaunchKernelGGL(gemm_f32_join, dim3((unsigned)tail_tiles * kJoinSlices), dim3(GEMM_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg

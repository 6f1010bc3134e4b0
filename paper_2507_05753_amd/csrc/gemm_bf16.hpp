// Reduced-precision block GEMM for gfx950:  C[M x N] (FP32) = A * B^T (+ addend) (+ bias), operands in
// bfloat16, products exact, sums in FP32 (v_mfma_f32_32x32x16_bf16).
//
// The paper trains in a mixed precision whose matrix units round FP32 operands to a short mantissa and
// accumulate in FP32 (Sec. 6.1).  This chip's matrix cores have no such FP32-input mode; their
// bfloat16 mode runs at 16 times the FP32 rate.  Two variants of the X W^T layer of Sec. 4 use it:
//   terms = 1 : operands rounded to bfloat16 once, when they are sharded;
//   terms = 3 : operands split x = hi + lo (both bfloat16) and the product taken as
//               hi hi + hi lo + lo hi — three passes over K at the same rate, 16 mantissa bits.
// Both operands are K-contiguous (A is M x K, B is N x K, the "X W^T" form); a split operand stores
// its lo plane behind its hi plane in every row ([hi(0..K) | lo(0..K)]), so the three terms are three
// K loops over two column windows of the same rows.
//
// Work decomposition
//   workgroup : 256 threads = 4 wavefronts (2 x 2), one 256 x 256 tile of C, one workgroup per CU
//   wavefront : 128 x 128 sub-tile = 4 x 4 MFMA blocks of 32 x 32 (256 accumulator registers);
//               per 16 k it reads 8 fragments of 16 bytes for 16 MFMAs, the smallest LDS traffic
//               per MFMA a wavefront's registers allow
//   K loop    : slabs of 64 (128-byte rows: whole cache lines), two slab buffers of 64 KiB in LDS
//               used alternately; slab kt + 1 travels global -> LDS (buffer_load_dwordx4 ... lds)
//               while slab kt is multiplied, one transfer after every fourth MFMA
// LDS layout as in the FP32 kernel's K-contiguous operands: rows are not padded; the lane that
// fills 16-byte slot s of row r fetches chunk s ^ ((r >> 1) & 7) of that row, which makes the
// 128-bit fragment reads (32 rows x 2 chunks per instruction) conflict-free.
// Transfers that would start at or past column K (ragged last slab) or past the operand's last row
// get an offset outside the buffer descriptor and arrive as zeros: nothing outside the operands is
// ever read.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_f32.hpp"

namespace jg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int HB_BM = 256;
constexpr int HB_BN = 256;
constexpr int HB_BK = 64;                                 // bfloat16 elements per slab row = 128 bytes
constexpr int HB_THREADS = 256;
constexpr int HB_OPERAND_BYTES = HB_BM * HB_BK * 2;       // one slab of one operand = 32 KiB (BM == BN)
constexpr int HB_STAGE_BYTES = 2 * HB_OPERAND_BYTES;      // A and B
constexpr int HB_BAND_ROWS = 4;                           // row-tiles per band of the tile order
constexpr int HB_TRANSFERS = HB_OPERAND_BYTES / (HB_THREADS * 16);   // 8 per lane, operand and slab

struct HbGroup {
    GemmProblem p[kMaxGroup];   // A, B point at bfloat16 data; lda, ldb count 4-byte units (bfloat16 pairs)
    int nprob;
    int M, N, K;                // K counts bfloat16 elements of one plane
    int terms;                  // 1, or 3 for split operands
    int tiles_m, tiles_n, total, per_xcd;
    int act;
};

__device__ __forceinline__ TileCoord hb_decode_tile(const HbGroup& g, int lid)
{
    const int tiles_per_prob = g.tiles_m * g.tiles_n;
    const int prob = lid / tiles_per_prob;
    const int t = lid - prob * tiles_per_prob;
    const int band = t / (HB_BAND_ROWS * g.tiles_n);
    const int in_band = t - band * (HB_BAND_ROWS * g.tiles_n);
    const int band_first = band * HB_BAND_ROWS;
    const int band_rows = min(HB_BAND_ROWS, g.tiles_m - band_first);
    TileCoord c;
    c.prob = prob;
    c.m0 = (band_first + in_band % band_rows) * HB_BM;
    c.n0 = (in_band / band_rows) * HB_BN;
    return c;
}

// One operand's slabs, global -> LDS.  Transfer t of a lane covers row 32 t + 8 wave + lane / 8
// of the tile (eight lanes per 128-byte row).
struct HbLoader {
    __amdgpu_buffer_rsrc_t rsrc;
    int voff[HB_TRANSFERS];     // byte offset of the lane's chunk in slab 0, or kOutOfBuffer for rows past the operand
    int chunk_k;                // first k (within a slab) of the chunk this lane fetches
    // row_bytes: the bytes of a row that exist (all planes)
    __device__ __forceinline__ void init(const float* base, int ld, int extent, int origin, int row_bytes, int wave,
                                         int lane)
    {
        const int valid = min(HB_BM, extent - origin);
        const int r = wave * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((r >> 1) & 7);
        chunk_k = chunk * 8;
#pragma unroll
        for (int t = 0; t < HB_TRANSFERS; ++t) {
            const int row = t * 32 + r;
            voff[t] = row < valid ? row * ld * 4 + chunk * 16 : kOutOfBuffer;
        }
        // The descriptor spans the tile's valid rows.  A slab's column offset travels in the scalar
        // offset: the kernel only issues transfers whose chunk exists, so nothing depends on whether
        // the hardware counts that offset in its range check.
        const int64_t bytes = (int64_t)(valid - 1) * ld * 4 + row_bytes;
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(base + (int64_t)origin * ld), 0, (int)bytes,
                                                 kBufferRsrcFlags);
    }
    // transfer t of the slab whose first column (in bytes, plane offset included) is col_bytes; every chunk
    // of the slab lies below K
    __device__ __forceinline__ void issue(int t, int col_bytes, char* operand_slab, int wave) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(operand_slab + t * 4096 + wave * 1024), 16, voff[t],
                                                 col_bytes, 0, 0);
    }
    // the same for a slab of which only the first `cols` columns exist
    __device__ __forceinline__ void issue_ragged(int t, int col_bytes, int cols, char* operand_slab, int wave) const
    {
        const int vo = chunk_k < cols ? voff[t] : kOutOfBuffer;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(operand_slab + t * 4096 + wave * 1024), 16, vo,
                                                 col_bytes, 0, 0);
    }
};

// acc = addend tile (the partial product received from the peer), or zero.
// m0, n0: the tile's origin; row_off, col_off: the lane's first row and its column inside the tile.
__device__ __forceinline__ void hb_init_acc(const GemmProblem& P, int M, int N, int m0, int n0, int row_off, int col_off,
                                            bool interior, floatx16 (&acc)[4][4])
{
    const int row_base = m0 + row_off, col_base = n0 + col_off;
    const float* __restrict__ addend = P.addend;
    if (!addend) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        return;
    }
    const int ldadd = P.ldadd;
    if (interior && ldadd <= kMaxDirectLd / 2) {
        // lane position in one vector offset, the row of each access in a scalar offset
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(addend + (int64_t)m0 * ldadd + n0), 0, ((HB_BM - 1) * ldadd + HB_BN) * 4, kBufferRsrcFlags);
        const int lane_off = (row_off * ldadd + col_off) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    acc[i][j][v] = __builtin_bit_cast(
                        float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off + j * 128,
                                                                    (i * 32 + 8 * (v >> 2) + (v & 3)) * ldadd * 4, 0));
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = col_base + j * 32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                    acc[i][j][v] = (row < M && col < N) ? addend[(int64_t)row * ldadd + col] : 0.f;
                }
            }
    }
}

// C = act(acc + bias) + residual.
__device__ __forceinline__ void hb_store_tile(const GemmProblem& P, int M, int N, int m0, int n0, int row_off, int col_off,
                                              bool interior, const floatx16 (&acc)[4][4], int act)
{
    const int row_base = m0 + row_off, col_base = n0 + col_off;
    const float* __restrict__ bias = P.bias;
    const float* __restrict__ residual = P.residual;
    float* __restrict__ C = P.C;
    const int ldc = P.ldc, ldres = P.ldres;
    if (interior && ldc <= kMaxDirectLd / 2 && (!residual || ldres <= kMaxDirectLd / 2)) {
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            C + (int64_t)m0 * ldc + n0, 0, ((HB_BM - 1) * ldc + HB_BN) * 4, kBufferRsrcFlags);
        const __amdgpu_buffer_rsrc_t res_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(residual ? residual + (int64_t)m0 * ldres + n0 : C), 0,
            residual ? ((HB_BM - 1) * ldres + HB_BN) * 4 : 0, kBufferRsrcFlags);
        const int lane_off = (row_off * ldc + col_off) * 4;
        const int res_off = (row_off * ldres + col_off) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float bj = bias ? bias[col_base + j * 32] : 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float res[16];
                if (residual) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        res[v] = __builtin_bit_cast(
                            float, __builtin_amdgcn_raw_buffer_load_b32(res_rsrc, res_off + j * 128,
                                                                        (i * 32 + 8 * (v >> 2) + (v & 3)) * ldres * 4, 0));
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float y = activate(acc[i][j][v] + bj, act);
                    if (residual) y += res[v];
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, y), rsrc, lane_off + j * 128,
                                                          (i * 32 + 8 * (v >> 2) + (v & 3)) * ldc * 4, 0);
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = col_base + j * 32;
                if (col >= N) continue;
                const float bj = bias ? bias[col] : 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (row < M) {
                        float y = activate(acc[i][j][v] + bj, act);
                        if (residual) y += residual[(int64_t)row * ldres + col];
                        C[(int64_t)row * ldc + col] = y;
                    }
                }
            }
    }
}

// grid: kNumXcd * per_xcd workgroups; consecutive ids land on different XCDs, so the id is folded
// into a per-XCD contiguous range of tiles, walked column-major inside bands of 4 row-tiles: the 32
// tiles an XCD has in flight form a 4 x 8 block that shares 4 A panels and 8 B panels in its L2.
__global__ __launch_bounds__(HB_THREADS, 1) void gemm_bf16_nt(const HbGroup g)
{
    __shared__ __align__(1024) char slab[2 * HB_STAGE_BYTES];

    const int lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
    if (lid >= g.total) return;
    const TileCoord tc = hb_decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];
    const int M = g.M, N = g.N, K = g.K;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lk = lane >> 5;

    HbLoader load_a, load_b;
    const int row_bytes = (g.terms == 3 ? 2 : 1) * K * 2;
    load_a.init(P.A, P.lda, M, tc.m0, row_bytes, wave, lane);
    load_b.init(P.B, P.ldb, N, tc.n0, row_bytes, wave, lane);

    // The slab sequence: `terms` passes over K.  With split operands the two small cross terms go
    // first (A hi with B lo, then A lo with B hi) and hi with hi last: added to an already large sum,
    // the small products would lose their low bits at every step.
    const int nkt = (K + HB_BK - 1) / HB_BK;
    const int total_slabs = nkt * g.terms;
    const int last_cols = K - (nkt - 1) * HB_BK;            // columns of a pass's last slab
    auto request = [&](int it, char* stage) __attribute__((always_inline)) {
        const int pass = it / nkt, kt = it - pass * nkt;
        const int a_col = (kt * HB_BK + ((g.terms == 3 && pass == 1) ? K : 0)) * 2;
        const int b_col = (kt * HB_BK + ((g.terms == 3 && pass == 0) ? K : 0)) * 2;
        if (kt == nkt - 1 && last_cols < HB_BK) {
#pragma unroll
            for (int t = 0; t < HB_TRANSFERS; ++t) {
                load_a.issue_ragged(t, a_col, last_cols, stage, wave);
                load_b.issue_ragged(t, b_col, last_cols, stage + HB_OPERAND_BYTES, wave);
            }
        } else {
#pragma unroll
            for (int t = 0; t < HB_TRANSFERS; ++t) {
                load_a.issue(t, a_col, stage, wave);
                load_b.issue(t, b_col, stage + HB_OPERAND_BYTES, wave);
            }
        }
    };

    request(0, slab);

    const bool interior = tc.m0 + HB_BM <= M && tc.n0 + HB_BN <= N;
    const int row_off = wm * 128 + 4 * lk;      // the lane's first row and its column inside the tile
    const int col_off = wn * 128 + lr;
    floatx16 acc[4][4];
    hb_init_acc(P, M, N, tc.m0, tc.n0, row_off, col_off, interior, acc);

    // fragment k-step s (16 k) of block b: row 32 b + lr, chunks 2 s + lk
    int frag_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) frag_off[s] = lr * 128 + (((2 * s + lk) ^ ((lr >> 1) & 7)) << 4);
    const int a_frag = wm * 4 * 4096;                          // the wave's four row blocks of A
    const int b_frag = HB_OPERAND_BYTES + wn * 4 * 4096;       // ... and four column blocks of B

    for (int it = 0; it < total_slabs; ++it) {
        char* cur = slab + (it & 1) * HB_STAGE_BYTES;
        char* nxt = slab + ((it + 1) & 1) * HB_STAGE_BYTES;
        __builtin_amdgcn_s_waitcnt(0);     // this lane's transfers of slab `it` have landed
        __syncthreads();                   // everyone's have, and everyone is done reading the other buffer
        if (it + 1 < total_slabs) request(it + 1, nxt);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            bf16x8 fa[4], fb[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                fa[b] = *reinterpret_cast<const bf16x8*>(cur + a_frag + b * 4096 + frag_off[s]);
                fb[b] = *reinterpret_cast<const bf16x8*>(cur + b_frag + b * 4096 + frag_off[s]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
    hb_store_tile(P, M, N, tc.m0, tc.n0, row_off, col_off, interior, acc, g.act);
}

// Can this operand take the 16-byte transfers?  (rows 16-byte aligned, K in whole chunks)
inline bool hb_operand_ok(const float* p, int ld, int K)
{
    return ((uintptr_t)p & 15) == 0 && (ld & 3) == 0 && (K & 7) == 0 && ld <= kMaxDirectLd / 2;
}

// One grouped launch.  Preconditions (checked by the C-ABI layer when the plan is made): every
// operand passes hb_operand_ok; 1 <= nprob <= 4; M, N, K >= 1.
inline hipError_t launch_gemm_bf16_group(const GemmGroup& src, int terms, hipStream_t stream)
{
    HbGroup g;
    for (int i = 0; i < kMaxGroup; ++i) g.p[i] = src.p[i];
    g.nprob = src.nprob;
    g.M = src.M;
    g.N = src.N;
    g.K = src.K;
    g.terms = terms;
    g.act = src.act;
    g.tiles_m = (g.M + HB_BM - 1) / HB_BM;
    g.tiles_n = (g.N + HB_BN - 1) / HB_BN;
    const int64_t total = (int64_t)g.nprob * g.tiles_m * g.tiles_n;
    if (total + kNumXcd > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    for (int i = 0; i < g.nprob; ++i)
        if (!hb_operand_ok(g.p[i].A, g.p[i].lda, g.K) || !hb_operand_ok(g.p[i].B, g.p[i].ldb, g.K))
            return hipErrorInvalidValue;
    g.total = (int)total;
    g.per_xcd = (g.total + kNumXcd - 1) / kNumXcd;
    hipLaunchKernelGGL(gemm_bf16_nt, dim3((unsigned)(kNumXcd * g.per_xcd)), dim3(HB_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg

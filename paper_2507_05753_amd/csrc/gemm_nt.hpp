// FP32 matrix-core block GEMM for gfx950:  C = A * B^T (+ addend) (+ bias)
//
//   A : M x K  (a rank's activation shard X_r, K contiguous)
//   B : N x K  (a weight block, K contiguous)  -> the "X W^T" form of Sec. 4
//   C : M x N
//
// One launch runs a *group* of up to four equally-shaped problems (the block
// products of all virtual ranks that belong to the same step of the forward
// pass: the products handed to a peer, or the kept products whose epilogue adds
// the received partial, Eqs. (2) and (4)).
//
// Work decomposition
//   workgroup : 256 threads = 4 wavefronts (2 x 2), one 128 x 128 tile of C
//   wavefront : 64 x 64 sub-tile = 2 x 2 MFMA blocks of 32 x 32 (v_mfma_f32_32x32x2_f32)
//   K loop    : slabs of 32, double-buffered in LDS, global loads of slab t+1 are
//               issued before the MFMAs of slab t and parked in registers
//   LDS       : rows padded to 36 floats so that 128-bit reads of 32 consecutive
//               rows and 128-bit writes of 8 chunks x 8 rows spread over the banks
//
// Tile order: consecutive workgroup ids land on different XCDs (round-robin
// dispatch), so the id is first folded into a per-XCD contiguous range, then
// walked in column-major order inside bands of 8 row-tiles.  The 64 workgroups an
// XCD has in flight therefore share 8 A row-panels and 8 B row-panels in its L2.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jg {

constexpr int kMaxGroup = 4;
constexpr int BM = 128;
constexpr int BN = 128;
constexpr int BK = 32;
constexpr int LDS_ROW = BK + 4;                       // floats per padded row
constexpr int STAGE_FLOATS = (BM + BN) * LDS_ROW;     // one K slab of A and B
constexpr int GEMM_THREADS = 256;
constexpr int GEMM_LDS_BYTES = 2 * STAGE_FLOATS * (int)sizeof(float);
constexpr int kNumXcd = 8;
constexpr int kBandRows = 8;                          // row-tiles per band

struct GemmProblem {
    const float* A;       // M x K, leading dimension lda
    const float* B;       // N x K, leading dimension ldb
    float* C;             // M x N, leading dimension ldc
    const float* addend;  // M x N (ldadd) added in the epilogue, or nullptr
    const float* bias;    // length N added in the epilogue, or nullptr
    int lda, ldb, ldc, ldadd;
};

struct GemmGroup {
    GemmProblem p[kMaxGroup];
    int nprob;
    int M, N, K;          // common shape of every problem in the group
    int tiles_m, tiles_n; // ceil(M / BM), ceil(N / BN)
    int per_xcd;          // ceil(nprob * tiles_m * tiles_n / kNumXcd)
    int vec_ok;           // all A/B pointers 16-byte aligned and lda, ldb multiples of 4
};

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float4 load_chunk(const float* __restrict__ row, int k, int K, bool fast)
{
    if (fast) return *reinterpret_cast<const float4*>(row + k);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k + 0 < K) v.x = row[k + 0];
    if (k + 1 < K) v.y = row[k + 1];
    if (k + 2 < K) v.z = row[k + 2];
    if (k + 3 < K) v.w = row[k + 3];
    return v;
}

__global__ __launch_bounds__(GEMM_THREADS) void gemm_nt_f32(const GemmGroup g)
{
    extern __shared__ __align__(16) float lds[];

    // ---- which tile -------------------------------------------------------
    const int bid = blockIdx.x;
    const int lid = (bid % kNumXcd) * g.per_xcd + bid / kNumXcd;
    const int tiles_per_prob = g.tiles_m * g.tiles_n;
    if (lid >= g.nprob * tiles_per_prob) return;   // whole workgroup leaves before any barrier
    const int prob = lid / tiles_per_prob;
    const int t = lid - prob * tiles_per_prob;
    const int band = t / (kBandRows * g.tiles_n);
    const int in_band = t - band * (kBandRows * g.tiles_n);
    const int band_first = band * kBandRows;
    const int band_rows = min(kBandRows, g.tiles_m - band_first);
    const int tm = band_first + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int m0 = tm * BM;
    const int n0 = tn * BN;

    const GemmProblem& P = g.p[prob];
    const int M = g.M, N = g.N, K = g.K;

    // ---- global -> register staging: thread owns chunk `ck` of rows r0 + 32 p ----
    const int tid = threadIdx.x;
    const int ck = tid & 7;        // which float4 of the 32-wide K slab
    const int r0 = tid >> 3;       // 0..31
    const float* a_row[4];
    const float* b_row[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        // rows past the edge are clamped to the last valid row: they are read but never stored
        const int ar = min(m0 + r0 + 32 * p, M - 1);
        const int br = min(n0 + r0 + 32 * p, N - 1);
        a_row[p] = P.A + (int64_t)ar * P.lda;
        b_row[p] = P.B + (int64_t)br * P.ldb;
    }
    float4 ra[4], rb[4];

    auto load_slab = [&](int kt) {
        const int k = kt * BK + ck * 4;
        const bool fast = g.vec_ok && (kt * BK + BK <= K);   // uniform over the workgroup
#pragma unroll
        for (int p = 0; p < 4; ++p) ra[p] = load_chunk(a_row[p], k, K, fast);
#pragma unroll
        for (int p = 0; p < 4; ++p) rb[p] = load_chunk(b_row[p], k, K, fast);
    };
    auto store_slab = [&](int buf) {
        float* sA = lds + buf * STAGE_FLOATS;
        float* sB = sA + BM * LDS_ROW;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(sA + (r0 + 32 * p) * LDS_ROW + ck * 4) = ra[p];
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(sB + (r0 + 32 * p) * LDS_ROW + ck * 4) = rb[p];
    };

    // ---- MFMA operands ----------------------------------------------------
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31;      // row of the 32-row operand block this lane feeds
    const int lk = lane >> 5;      // which of the instruction's two k slots
    const int a_off = (wm * 64 + lr) * LDS_ROW + lk * 4;
    const int b_off = BM * LDS_ROW + (wn * 64 + lr) * LDS_ROW + lk * 4;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nkt = (K + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 1 < nkt;
        if (more) load_slab(kt + 1);

        const float* s = lds + (kt & 1) * STAGE_FLOATS;
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            // lanes 0-31 take k = 8 kk .. 8 kk + 3, lanes 32-63 the next four; the t-th MFMA
            // contracts k slots {8 kk + t, 8 kk + 4 + t}: A and B use the same assignment
            const float4 a0 = *reinterpret_cast<const float4*>(s + a_off + kk * 8);
            const float4 a1 = *reinterpret_cast<const float4*>(s + a_off + 32 * LDS_ROW + kk * 8);
            const float4 b0 = *reinterpret_cast<const float4*>(s + b_off + kk * 8);
            const float4 b1 = *reinterpret_cast<const float4*>(s + b_off + 32 * LDS_ROW + kk * 8);
            const float av[2][4] = {{a0.x, a0.y, a0.z, a0.w}, {a1.x, a1.y, a1.z, a1.w}};
            const float bv[2][4] = {{b0.x, b0.y, b0.z, b0.w}, {b1.x, b1.y, b1.z, b1.w}};
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][tt], bv[j][tt],
                                                                         acc[i][j], 0, 0, 0);
        }

        if (more) store_slab((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: C = acc (+ addend) (+ bias) -----------------------------
    // accumulator register v of lane (lr, lk) holds row 8 (v / 4) + 4 lk + v % 4, column lr
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + lr;
            if (col >= N) continue;
            const float bj = P.bias ? P.bias[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
                if (row < M) {
                    float y = acc[i][j][v];
                    if (P.addend) y += P.addend[(int64_t)row * P.ldadd + col];
                    y += bj;
                    P.C[(int64_t)row * P.ldc + col] = y;
                }
            }
        }
    }
}

// Host side: fills the derived fields of `g` and enqueues the launch.
// Preconditions (checked by the C-ABI layer): 1 <= nprob <= 4; M, N, K >= 1; all
// pointers valid for their shapes; lda, ldb >= K; ldc, ldadd >= N.
inline hipError_t launch_gemm_group(GemmGroup& g, hipStream_t stream)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const int64_t total = (int64_t)g.nprob * g.tiles_m * g.tiles_n;
    g.per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
    int vec = 1;
    for (int i = 0; i < g.nprob; ++i) {
        if (((uintptr_t)g.p[i].A & 15) || ((uintptr_t)g.p[i].B & 15) || (g.p[i].lda & 3) ||
            (g.p[i].ldb & 3))
            vec = 0;
    }
    g.vec_ok = vec;
    const unsigned grid = (unsigned)(g.per_xcd * kNumXcd);
    hipLaunchKernelGGL(gemm_nt_f32, dim3(grid), dim3(GEMM_THREADS), GEMM_LDS_BYTES, stream, g);
    return hipGetLastError();
}

inline hipError_t prepare_gemm()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_nt_f32),
                               hipFuncAttributeMaxDynamicSharedMemorySize, GEMM_LDS_BYTES);
}

}  // namespace jg

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
//   workgroup : 256 threads = 4 wavefronts (2 x 2), 128 x 128 tiles of C
//   wavefront : 64 x 64 sub-tile = 2 x 2 MFMA blocks of 32 x 32 (v_mfma_f32_32x32x2_f32)
//   K loop    : slabs of 32 floats, two slab buffers in LDS used alternately
//
// gemm_nt_f32_stream (operand rows 16-byte aligned, K a multiple of 4): slabs go global ->
// LDS without passing through registers (buffer_load_dwordx4 ... lds), one slab ahead of the
// math.  Each wave-level load writes 1 KiB of LDS = 8 rows x 128 B, lane l filling 16-byte
// slot l.  Rows are not padded; instead the lane chooses WHICH 16-byte chunk of its row it
// fetches, chunk = slot ^ ((row >> 1) & 7), so that the later 128-bit LDS reads of 16
// consecutive rows at one k-chunk fall into 16 different slots.  Chunks at or past column K
// are fetched from outside the buffer descriptor and arrive as zeros.  The received partial
// product (the addend) is loaded straight into the accumulators while the first slab is in
// flight, so its latency is paid together with the one unavoidable wait of a tile and the
// epilogue only stores.
//
// gemm_nt_f32_guarded (anything else): one tile per workgroup, register loads with
// per-element bounds checks written to the same swizzled LDS positions.
//
// Tile order: consecutive workgroup ids land on different XCDs (round-robin dispatch), so
// the id is first folded into a per-XCD contiguous range, then walked column-major inside
// bands of 8 row-tiles.  The 64 workgroups an XCD has in flight (2 per CU) therefore form an
// 8 x 8 block of tiles that shares 8 A row-panels and 8 B row-panels in that XCD's L2.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace jg {

constexpr int kMaxGroup = 4;
constexpr int BM = 128;
constexpr int BN = 128;
constexpr int BK = 32;
constexpr int ROW_FLOATS = BK;                          // unpadded: one row of a slab = 128 B
constexpr int STAGE_FLOATS = (BM + BN) * ROW_FLOATS;    // one K slab of A and B = 32 KiB
constexpr int GEMM_THREADS = 256;
constexpr int kNumXcd = 8;
constexpr int kBandRows = 8;                            // row-tiles per band
constexpr int kFlushSlabs = 32;                         // K extent of one first-level accumulation = 1024

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
};

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

// What a lane needs to feed the MFMAs from a slab in LDS, and to write its results.
struct LaneMap {
    int wave, lane, wm, wn, lr, lk;
    int a_row_off[2], b_row_off[2], a_sw[2], b_sw[2];
    __device__ __forceinline__ void init(int tid)
    {
        wave = tid >> 6;
        lane = tid & 63;
        wm = wave >> 1;
        wn = wave & 1;
        lr = lane & 31;      // row of the 32-row operand block this lane feeds
        lk = lane >> 5;      // which of the instruction's two k slots
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ra = wm * 64 + i * 32 + lr;
            const int rb = wn * 64 + i * 32 + lr;
            a_row_off[i] = ra * ROW_FLOATS;
            b_row_off[i] = BM * ROW_FLOATS + rb * ROW_FLOATS;
            a_sw[i] = (ra >> 1) & 7;
            b_sw[i] = (rb >> 1) & 7;
        }
    }
    // lanes 0-31 take k = 8 kk .. 8 kk + 3 (chunk 2 kk), lanes 32-63 the next four (chunk
    // 2 kk + 1); the t-th MFMA of a group contracts k slots {8 kk + t, 8 kk + 4 + t}:
    // A and B use the same assignment, so the products pair up correctly.
    __device__ __forceinline__ void read_frags(const float* s, int kk, float4 (&fa)[2], float4 (&fb)[2]) const
    {
        const int c = kk * 2 + lk;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            fa[i] = *reinterpret_cast<const float4*>(s + a_row_off[i] + ((c ^ a_sw[i]) << 2));
            fb[i] = *reinterpret_cast<const float4*>(s + b_row_off[i] + ((c ^ b_sw[i]) << 2));
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
            for (int v = 0; v < 16; ++v) {
                sum[i][j][v] += acc[i][j][v];
                acc[i][j][v] = 0.f;
            }
}

// Accumulator register v of lane (lr, lk) holds row 8 (v / 4) + 4 lk + v % 4, column lr of
// its 32 x 32 block, so one load / store instruction touches two 128-byte row segments.

// acc = addend tile (the partial product received from the peer), or zero.
__device__ __forceinline__ void init_acc(const GemmProblem& P, int M, int N, int m0, int n0,
                                         const LaneMap& L, floatx16 (&acc)[2][2])
{
    const float* __restrict__ addend = P.addend;
    if (!addend) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        return;
    }
    const int ldadd = P.ldadd;
    const int row_base = m0 + L.wm * 64 + 4 * L.lk;
    const int col_base = n0 + L.wn * 64 + L.lr;
    if (m0 + BM <= M && n0 + BN <= N) {
        const float* a_lane = addend + (int64_t)row_base * ldadd + col_base;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    acc[i][j][v] = a_lane[(int64_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * ldadd + j * 32];
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

// C = acc (+ bias) for the tile at (m0, n0).
__device__ __forceinline__ void store_tile(const GemmProblem& P, int M, int N, int m0, int n0,
                                           const LaneMap& L, const floatx16 (&acc)[2][2])
{
    const float* __restrict__ bias = P.bias;
    float* __restrict__ C = P.C;
    const int ldc = P.ldc;
    const int row_base = m0 + L.wm * 64 + 4 * L.lk;     // + i * 32 + 8 (v / 4) + v % 4
    const int col_base = n0 + L.wn * 64 + L.lr;         // + j * 32
    if (m0 + BM <= M && n0 + BN <= N) {   // interior tile: no bounds checks
        float* c_lane = C + (int64_t)row_base * ldc + col_base;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float bj = bias ? bias[col_base + j * 32] : 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    c_lane[(int64_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * ldc + j * 32] = acc[i][j][v] + bj;
        }
    } else {                              // edge tile: every element checked against M and N
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
                    if (row < M) C[(int64_t)row * ldc + col] = acc[i][j][v] + bj;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// asynchronous-load kernel: one tile per workgroup, two workgroups per CU
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_nt_f32_stream(const GemmGroup g)
{
    // One array per slab buffer: distinct LDS objects let the compiler prove that the
    // asynchronous fill of one does not alias the reads of the other, so it does not make
    // every LDS read wait for the loads still in flight.
    __shared__ __align__(16) float ring0[STAGE_FLOATS];
    __shared__ __align__(16) float ring1[STAGE_FLOATS];

    const int lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
    if (lid >= g.nprob * g.tiles_m * g.tiles_n) return;   // whole workgroup leaves before any barrier
    const TileCoord tc = decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];
    const int M = g.M, N = g.N, K = g.K;
    const int m0 = tc.m0, n0 = tc.n0;
    const int nkt = (K + BK - 1) / BK;
    const int kt_ragged = (K % BK) ? K / BK : -1;   // the slab that needs the zero fill, if any

    LaneMap L;
    L.init(threadIdx.x);

    // ---- loader: thread covers tile rows p * 32 + wave * 8 + lane / 8, p = 0..3 (a wave-level
    // load fills 8 consecutive rows x 8 slots = 1 KiB of contiguous LDS)
    const int lrow = L.wave * 8 + (L.lane >> 3);
    const int slot = L.lane & 7;
    const int lda = P.lda, ldb = P.ldb;
    int src_chunk[4];                          // which chunk of its row this lane fetches
    int a_voff[4], b_voff[4];                  // byte offsets of those chunks from the tile's first row
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = p * 32 + lrow;
        src_chunk[p] = slot ^ ((r >> 1) & 7);
        // rows past the edge are clamped to the last valid row: they are read but never stored
        a_voff[p] = ((min(m0 + r, M - 1) - m0) * lda + src_chunk[p] * 4) * 4;
        b_voff[p] = ((min(n0 + r, N - 1) - n0) * ldb + src_chunk[p] * 4) * 4;
    }
    // buffers over the rows of this tile (base = its first row, extent = up to the end of its
    // last valid row): an out-of-range offset reads zero instead of faulting
    const int64_t a_bytes = ((int64_t)(min(m0 + BM, M) - 1 - m0) * lda + K) * 4;
    const int64_t b_bytes = ((int64_t)(min(n0 + BN, N) - 1 - n0) * ldb + K) * 4;
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(P.A + (int64_t)m0 * lda), 0, (int)a_bytes, kBufferRsrcFlags);
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(P.B + (int64_t)n0 * ldb), 0, (int)b_bytes, kBufferRsrcFlags);

    auto request_slab_impl = [&](int kt, float* sA, auto ragged) {
        float* sB = sA + BM * ROW_FLOATS;
        const int soff = kt * BK * 4;
        const int k_left = K - kt * BK;        // valid columns of this slab
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int woff = (p * 32 + L.wave * 8) * ROW_FLOATS;   // wave-uniform LDS offset
            const bool in = !decltype(ragged)::value || src_chunk[p] * 4 < k_left;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void*)(sA + woff), 16,
                                                     in ? a_voff[p] : kOutOfBuffer, soff, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int woff = (p * 32 + L.wave * 8) * ROW_FLOATS;
            const bool in = !decltype(ragged)::value || src_chunk[p] * 4 < k_left;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_void*)(sB + woff), 16,
                                                     in ? b_voff[p] : kOutOfBuffer, soff, 0, 0);
        }
    };
    auto request_slab = [&](int kt, float* sA) {
        if (kt == kt_ragged) request_slab_impl(kt, sA, std::true_type{});
        else request_slab_impl(kt, sA, std::false_type{});
    };

    floatx16 acc[2][2], sum[2][2];
    float4 fa[2][2], fb[2][2];   // two register sets of MFMA operands (even / odd k-group)

    // One slab: inside it the operands of k-group kk + 1 are requested before the 16 MFMAs of
    // group kk are issued, so LDS latency hides behind about a thousand matrix-pipe cycles.
    // The slab boundary (wait for the next slab, barrier, request the slab after next, first
    // operand read of the next slab) sits before the LAST group's MFMAs for the same reason.
    // The scheduling fences keep the compiler from undoing this order.
    auto step = [&](int kt, float* cur, const float* nxt) {
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            L.read_frags(cur, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            mfma_group(acc, fa[kk & 1], fb[kk & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
        JG_WAIT_VMCNT(0);   // this thread's part of slab kt + 1 has landed
        __syncthreads();    // ... and everyone's; all waves hold their last operands of slab kt
        if (kt + 2 < nkt) request_slab(kt + 2, cur);
        if (kt + 1 < nkt) L.read_frags(nxt, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        mfma_group(acc, fa[1], fb[1]);
        __builtin_amdgcn_sched_barrier(0);
    };

    request_slab(0, ring0);
    init_acc(P, M, N, m0, n0, L, sum);   // its loads fly together with slab 0
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    JG_WAIT_VMCNT(0);
    __syncthreads();
    if (1 < nkt) request_slab(1, ring1);
    L.read_frags(ring0, 0, fa[0], fb[0]);
    __builtin_amdgcn_sched_barrier(0);
    int kt = 0;
    for (; kt + 1 < nkt; kt += 2) {
        step(kt, ring0, ring1);
        step(kt + 1, ring1, ring0);
        if ((kt & (kFlushSlabs - 1)) == kFlushSlabs - 2) fold_acc(sum, acc);
    }
    if (kt < nkt) step(kt, ring0, ring1);
    fold_acc(sum, acc);

    store_tile(P, M, N, m0, n0, L, sum);
}

// ------------------------------------------------------------------------------------------
// guarded kernel: any alignment, any K; one tile per workgroup, synchronous slab loads
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float4 load_guarded(const float* __restrict__ row, int k, int K)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k + 0 < K) v.x = row[k + 0];
    if (k + 1 < K) v.y = row[k + 1];
    if (k + 2 < K) v.z = row[k + 2];
    if (k + 3 < K) v.w = row[k + 3];
    return v;
}

__global__ __launch_bounds__(GEMM_THREADS) void gemm_nt_f32_guarded(const GemmGroup g)
{
    __shared__ __align__(16) float slab[STAGE_FLOATS];

    const int lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
    if (lid >= min((int)(blockIdx.x % kNumXcd + 1) * g.per_xcd, g.nprob * g.tiles_m * g.tiles_n)) return;
    const TileCoord tc = decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];
    const int M = g.M, N = g.N, K = g.K;

    LaneMap L;
    L.init(threadIdx.x);
    const int lrow = L.wave * 8 + (L.lane >> 3);
    const int slot = L.lane & 7;
    const float* a_src[4];
    const float* b_src[4];
    int src_chunk[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = p * 32 + lrow;
        a_src[p] = P.A + (int64_t)min(tc.m0 + r, M - 1) * P.lda;
        b_src[p] = P.B + (int64_t)min(tc.n0 + r, N - 1) * P.ldb;
        src_chunk[p] = slot ^ ((r >> 1) & 7);
    }

    floatx16 acc[2][2], sum[2][2];
    init_acc(P, M, N, tc.m0, tc.n0, L, sum);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    float4 fa[2][2], fb[2][2];
    const int nkt = (K + BK - 1) / BK;
    for (int kt = 0; kt < nkt; ++kt) {
        if (kt && (kt & (kFlushSlabs - 1)) == 0) fold_acc(sum, acc);
        float4 ra[4], rb[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) ra[p] = load_guarded(a_src[p], kt * BK + src_chunk[p] * 4, K);
#pragma unroll
        for (int p = 0; p < 4; ++p) rb[p] = load_guarded(b_src[p], kt * BK + src_chunk[p] * 4, K);
        __syncthreads();        // everyone is done reading the previous slab
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(slab + (p * 32 + lrow) * ROW_FLOATS + slot * 4) = ra[p];
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(slab + BM * ROW_FLOATS + (p * 32 + lrow) * ROW_FLOATS + slot * 4) = rb[p];
        __syncthreads();
        L.read_frags(slab, 0, fa[0], fb[0]);
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            if (kk + 1 < BK / 8) L.read_frags(slab, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            mfma_group(acc, fa[kk & 1], fb[kk & 1]);
        }
    }
    fold_acc(sum, acc);
    store_tile(P, M, N, tc.m0, tc.n0, L, sum);
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
    bool stream_ok = (g.K % 4) == 0;   // every operand row 16-byte aligned, K in whole chunks
    for (int i = 0; i < g.nprob; ++i) {
        if (((uintptr_t)g.p[i].A & 15) || ((uintptr_t)g.p[i].B & 15) || (g.p[i].lda & 3) ||
            (g.p[i].ldb & 3) || g.p[i].lda > kMaxDirectLd || g.p[i].ldb > kMaxDirectLd)
            stream_ok = false;
    }
    const unsigned grid = (unsigned)(kNumXcd * g.per_xcd);
    if (stream_ok) hipLaunchKernelGGL(gemm_nt_f32_stream, dim3(grid), dim3(GEMM_THREADS), 0, stream, g);
    else hipLaunchKernelGGL(gemm_nt_f32_guarded, dim3(grid), dim3(GEMM_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg

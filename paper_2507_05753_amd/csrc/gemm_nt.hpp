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
//   K loop    : slabs of 32 floats; a ring of STAGES slab buffers in LDS
//
// Data path.  When every operand row is 16-byte aligned (the DIRECT variant) full
// slabs go global -> LDS without passing through registers (buffer_load_dwordx4 ... lds):
// each wave-level load writes 1 KiB of LDS = 8 rows x 128 B, lane l filling 16-byte
// slot l.  Rows are not padded; instead the lane chooses WHICH 16-byte chunk of its
// row it fetches, chunk = slot ^ ((row >> 1) & 7), so that the later 128-bit LDS
// reads of 16 consecutive rows at one k-chunk fall into 16 different slots.  Chunks
// past column K are fetched from outside the buffer and arrive as zeros.  A last slab
// whose K is not a multiple of 4, and every slab of the GUARDED variant (unaligned
// rows), goes through registers with per-element bounds checks and is written to
// the same swizzled positions.
//
// Tile order: consecutive workgroup ids land on different XCDs (round-robin
// dispatch), so the id is first folded into a per-XCD contiguous range, then
// walked in column-major order inside bands of 8 row-tiles.  The workgroups an
// XCD has in flight therefore share 8 A row-panels and a few B row-panels in its L2.
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

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ float4 load_guarded(const float* __restrict__ row, int k, int K)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k + 0 < K) v.x = row[k + 0];
    if (k + 1 < K) v.y = row[k + 1];
    if (k + 2 < K) v.z = row[k + 2];
    if (k + 3 < K) v.w = row[k + 3];
    return v;
}

template <int STAGES, bool DIRECT>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_nt_f32(const GemmGroup g)
{
    // One array per ring slot: distinct LDS objects let the compiler prove that the
    // asynchronous fill of one slot does not alias the reads of another, so it does not
    // make every LDS read wait for the loads still in flight.
    __shared__ __align__(16) float ring0[STAGE_FLOATS];
    __shared__ __align__(16) float ring1[STAGE_FLOATS];
    static_assert(STAGES == 2, "the ring is written out for two slots");

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

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;

    // ---- slab loader: thread covers tile rows  p * 32 + wave * 8 + lane / 8,  p = 0..3 ----
    // (wave-level: 8 consecutive rows x 8 slots = 1 KiB of contiguous LDS)
    const int lrow = wave * 8 + (lane >> 3);   // row within a 32-row group
    const int slot = lane & 7;                 // 16-byte slot within the LDS row
    const float* a_src[4];
    const float* b_src[4];
    int src_chunk[4];                          // which chunk of its row this lane fetches
    int a_voff[4], b_voff[4];                  // byte offsets of that chunk from the tile's first row
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = p * 32 + lrow;
        // rows past the edge are clamped to the last valid row: they are read but never stored
        const int ar = min(m0 + r, M - 1), br = min(n0 + r, N - 1);
        a_src[p] = P.A + (int64_t)ar * P.lda;
        b_src[p] = P.B + (int64_t)br * P.ldb;
        src_chunk[p] = swz(r, slot);
        a_voff[p] = ((ar - m0) * P.lda + src_chunk[p] * 4) * 4;
        b_voff[p] = ((br - n0) * P.ldb + src_chunk[p] * 4) * 4;
    }
    // Buffer resources over the rows of this tile (base = first row of the tile, extent = up to
    // the end of the last valid row): an out-of-range offset reads zero instead of faulting.
    const int64_t a_bytes = ((int64_t)(min(m0 + BM, M) - 1 - m0) * P.lda + K) * 4;
    const int64_t b_bytes = ((int64_t)(min(n0 + BN, N) - 1 - n0) * P.ldb + K) * 4;
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(P.A + (int64_t)m0 * P.lda), 0, (int)a_bytes, kBufferRsrcFlags);
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(P.B + (int64_t)n0 * P.ldb), 0, (int)b_bytes, kBufferRsrcFlags);

    // Asynchronous slab load (aligned rows).  A 16-byte chunk that starts at or beyond column K
    // is redirected to an offset outside the buffer, which the hardware answers with zeros:
    // the ragged last slab of a K that is a multiple of 4 needs no special path.
    auto load_direct_impl = [&](int kt, float* sA, auto ragged) {
        float* sB = sA + BM * ROW_FLOATS;
        const int soff = kt * BK * 4;
        const int k_left = K - kt * BK;                 // valid columns of this slab
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int woff = (p * 32 + wave * 8) * ROW_FLOATS;   // wave-uniform LDS offset
            const bool in = !decltype(ragged)::value || src_chunk[p] * 4 < k_left;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void*)(sA + woff), 16,
                                                     in ? a_voff[p] : kOutOfBuffer, soff, 0, 0);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int woff = (p * 32 + wave * 8) * ROW_FLOATS;
            const bool in = !decltype(ragged)::value || src_chunk[p] * 4 < k_left;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_void*)(sB + woff), 16,
                                                     in ? b_voff[p] : kOutOfBuffer, soff, 0, 0);
        }
    };
    const int kt_ragged = (K % BK) ? K / BK : -1;       // the slab that needs the zero fill, if any
    auto load_direct = [&](int kt, float* sA) {
        if (kt == kt_ragged) load_direct_impl(kt, sA, std::true_type{});
        else load_direct_impl(kt, sA, std::false_type{});
    };
    auto load_guarded_slab = [&](int kt, float* sA) {   // any slab, any alignment; synchronous
        float* sB = sA + BM * ROW_FLOATS;
        float4 ra[4], rb[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) ra[p] = load_guarded(a_src[p], kt * BK + src_chunk[p] * 4, K);
#pragma unroll
        for (int p = 0; p < 4; ++p) rb[p] = load_guarded(b_src[p], kt * BK + src_chunk[p] * 4, K);
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(sA + (p * 32 + lrow) * ROW_FLOATS + slot * 4) = ra[p];
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *reinterpret_cast<float4*>(sB + (p * 32 + lrow) * ROW_FLOATS + slot * 4) = rb[p];
    };

    // slabs that take the direct path: all of them when K is a multiple of 4, else the full ones
    const int nfull = !DIRECT ? 0 : (K % 4 == 0) ? (K + BK - 1) / BK : K / BK;
    const int nkt = (K + BK - 1) / BK;

    // ---- MFMA operand addressing -------------------------------------------
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31;      // row of the 32-row operand block this lane feeds
    const int lk = lane >> 5;      // which of the instruction's two k slots
    int a_row_off[2], b_row_off[2], a_sw[2], b_sw[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int ra_ = wm * 64 + i * 32 + lr;
        const int rb_ = wn * 64 + i * 32 + lr;
        a_row_off[i] = ra_ * ROW_FLOATS;
        b_row_off[i] = BM * ROW_FLOATS + rb_ * ROW_FLOATS;
        a_sw[i] = (ra_ >> 1) & 7;
        b_sw[i] = (rb_ >> 1) & 7;
    }

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // lanes 0-31 take k = 8 kk .. 8 kk + 3 (chunk 2 kk), lanes 32-63 the next four (chunk
    // 2 kk + 1); the t-th MFMA of a group contracts k slots {8 kk + t, 8 kk + 4 + t}:
    // A and B use the same assignment, so the products pair up correctly.
    auto read_frags = [&](const float* s, int kk, float4 (&fa)[2], float4 (&fb)[2]) {
        const int c = kk * 2 + lk;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            fa[i] = *reinterpret_cast<const float4*>(s + a_row_off[i] + ((c ^ a_sw[i]) << 2));
            fb[i] = *reinterpret_cast<const float4*>(s + b_row_off[i] + ((c ^ b_sw[i]) << 2));
        }
    };
    auto mfma_group = [&](const float4 (&fa)[2], const float4 (&fb)[2]) {
        const float av[2][4] = {{fa[0].x, fa[0].y, fa[0].z, fa[0].w}, {fa[1].x, fa[1].y, fa[1].z, fa[1].w}};
        const float bv[2][4] = {{fb[0].x, fb[0].y, fb[0].z, fb[0].w}, {fb[1].x, fb[1].y, fb[1].z, fb[1].w}};
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][tt], bv[j][tt], acc[i][j], 0, 0, 0);
    };

    float4 fa[2][2], fb[2][2];   // two register sets of MFMA operands (even / odd k-group)

    // ---- direct slabs: slab kt is computed from ring slot kt % 2 while slab kt + 1 fills the other ----
    // Inside a slab the operands of k-group kk + 1 are requested before the 16 MFMAs of group kk
    // are issued, so LDS latency hides behind about a thousand matrix-pipe cycles.  The slab
    // boundary (wait for the next slab, barrier, start the load after next, first operand read of
    // the next slab) sits before the LAST group's MFMAs for the same reason.  The scheduling
    // fences keep the compiler from undoing this order.
    if (DIRECT && nfull > 0) {
        auto step = [&](int kt, float* cur, const float* nxt) {
#pragma unroll
            for (int kk = 0; kk < 3; ++kk) {
                read_frags(cur, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                mfma_group(fa[kk & 1], fb[kk & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
            JG_WAIT_VMCNT(0);   // this thread's part of slab kt + 1 has landed
            __syncthreads();    // ... and everyone's; all waves hold their last operands of slab kt
            if (kt + 2 < nfull) load_direct(kt + 2, cur);
            if (kt + 1 < nfull) read_frags(nxt, 0, fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            mfma_group(fa[1], fb[1]);
            __builtin_amdgcn_sched_barrier(0);
        };
        load_direct(0, ring0);
        JG_WAIT_VMCNT(0);
        __syncthreads();
        if (1 < nfull) load_direct(1, ring1);
        read_frags(ring0, 0, fa[0], fb[0]);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        for (; kt + 1 < nfull; kt += 2) {
            step(kt, ring0, ring1);
            step(kt + 1, ring1, ring0);
        }
        if (kt < nfull) step(kt, ring0, ring1);
    }
    // ---- guarded slabs (the ragged tail, or all of them): load, then compute, one at a time ----
    for (int kt = nfull; kt < nkt; ++kt) {
        __syncthreads();        // everyone is done reading ring0
        load_guarded_slab(kt, ring0);
        __syncthreads();
        read_frags(ring0, 0, fa[0], fb[0]);
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            if (kk + 1 < BK / 8) read_frags(ring0, kk + 1, fa[(kk + 1) & 1], fb[(kk + 1) & 1]);
            mfma_group(fa[kk & 1], fb[kk & 1]);
        }
    }

    // ---- epilogue: C = acc (+ addend) (+ bias) -----------------------------
    // accumulator register v of lane (lr, lk) holds row 8 (v / 4) + 4 lk + v % 4, column lr of
    // its 32 x 32 block: one store instruction writes two 128-byte row segments.
    const float* __restrict__ addend = P.addend;
    const float* __restrict__ bias = P.bias;
    float* __restrict__ C = P.C;
    const int ldc = P.ldc, ldadd = P.ldadd;
    const int row_base = m0 + wm * 64 + 4 * lk;     // + i * 32 + 8 (v / 4) + v % 4
    const int col_base = n0 + wn * 64 + lr;         // + j * 32
    if (m0 + BM <= M && n0 + BN <= N) {
        // interior tile: no bounds checks; all loads of the received partial are issued
        // before the first of them is needed
        float* c_lane = C + (int64_t)row_base * ldc + col_base;
        if (addend) {
            const float* a_lane = addend + (int64_t)row_base * ldadd + col_base;
            float r[2][2][16];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        r[i][j][v] = a_lane[(int64_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * ldadd + j * 32];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] += r[i][j][v];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float bj = bias ? bias[col_base + j * 32] : 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    c_lane[(int64_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * ldc + j * 32] = acc[i][j][v] + bj;
        }
    } else {
        // edge tile: every element checked against M and N
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
                        float y = acc[i][j][v];
                        if (addend) y += addend[(int64_t)row * ldadd + col];
                        y += bj;
                        C[(int64_t)row * ldc + col] = y;
                    }
                }
            }
        }
    }
}

constexpr int kGemmStages = 2;

// Host side: fills the derived fields of `g` and enqueues the launch.
// Preconditions (checked by the C-ABI layer): 1 <= nprob <= 4; M, N, K >= 1; all
// pointers valid for their shapes; lda, ldb >= K; ldc, ldadd >= N.
inline hipError_t launch_gemm_group(GemmGroup& g, hipStream_t stream)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const int64_t total = (int64_t)g.nprob * g.tiles_m * g.tiles_n;
    g.per_xcd = (int)((total + kNumXcd - 1) / kNumXcd);
    bool aligned = true;   // every operand row starts on a 16-byte boundary
    for (int i = 0; i < g.nprob; ++i) {
        if (((uintptr_t)g.p[i].A & 15) || ((uintptr_t)g.p[i].B & 15) || (g.p[i].lda & 3) ||
            (g.p[i].ldb & 3) || g.p[i].lda > kMaxDirectLd || g.p[i].ldb > kMaxDirectLd)
            aligned = false;
    }
    const unsigned grid = (unsigned)(g.per_xcd * kNumXcd);
    if (aligned)
        hipLaunchKernelGGL((gemm_nt_f32<kGemmStages, true>), dim3(grid), dim3(GEMM_THREADS), 0, stream, g);
    else
        hipLaunchKernelGGL((gemm_nt_f32<kGemmStages, false>), dim3(grid), dim3(GEMM_THREADS), 0, stream, g);
    return hipGetLastError();
}

inline hipError_t prepare_gemm() { return hipSuccess; }   // static LDS: nothing to configure

}  // namespace jg

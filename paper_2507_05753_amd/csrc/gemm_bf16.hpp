// Reduced-precision block GEMM for gfx950:  C[M x N] (FP32) = A * B^T (+ addend) (+ bias), operands in
// bfloat16, products exact, sums in FP32 (v_mfma_f32_32x32x16_bf16).
//
// The paper trains in a mixed precision whose matrix units round FP32 operands to a short mantissa and
// accumulate in FP32 (Sec. 6.1).  This chip's matrix cores have no such FP32-input mode; their
// bfloat16 mode runs at 16 times the FP32 rate.  Two variants of the X W^T layer of Sec. 4 use it:
//   terms = 1 : operands rounded to bfloat16 once, when they are sharded;
//   terms = 3 : operands split x = hi + lo (both bfloat16) and the product taken as
//               hi hi + hi lo + lo hi — three times the matrix work, 16 mantissa bits, in one pass
//               over K (gemm_bf16x3_nt).
// Both operands are K-contiguous (A is M x K, B is N x K, the "X W^T" form); a split operand stores
// its lo plane behind its hi plane in every row ([hi(0..K) pad | lo(0..K) pad]), so the terms read two
// column windows of the same rows.  The shard step pads every plane to a multiple
// of 64 elements: rows then start on 128-byte lines and no 64-byte slab row straddles two of them.
//
// Work decomposition (gemm_bf16_nt, terms = 1; what differs with split operands is said at gemm_bf16x3_nt)
//   workgroup : 256 threads = 4 wavefronts (2 x 2), one 256 x 256 tile of C, one workgroup per CU
//   wavefront : 128 x 128 sub-tile = 4 x 4 MFMA blocks of 32 x 32 (256 accumulator registers);
//               per 16 k it reads 8 fragments of 16 bytes for 16 MFMAs, the smallest LDS traffic
//               per MFMA a wavefront's registers allow
//   K loop    : slabs of 64 (128-byte rows: every request is a whole cache line), two slab buffers of
//               64 KiB in LDS.  A slab's second half is in registers before the workgroup's one barrier
//               per slab, which sits between the halves; behind it the buffer is refilled with slab
//               it + 2 (buffer_load_dwordx4 ... lds, one transfer after every second MFMA) and the
//               first operands of slab it + 1 are read.  One slab ahead of the transfers a few lanes
//               ask L2 for the lines of the slab after, so that first touches of HBM are not waited
//               for with a whole slab of LDS standing empty
//   epilogue  : each 32 x 128 block of a wave's accumulators goes through the wave's piece of LDS
//               (free by then) and leaves as 16-byte stores;
//               optionally a second copy rounded to bfloat16 for a layer that follows
//   tail      : the tiles of a last partial round of workgroups can be cut into runs of slabs
//               (gemm_bf16_join adds them in k order); see make_bf16_group
// LDS layout: see HbLoader.
// Transfers that would start at or past column K (ragged last slab) or past the operand's last row
// get an offset outside the buffer descriptor and arrive as zeros: nothing outside the operands is
// ever read.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>
#include <type_traits>
#include <utility>

#include "cvt_kernels.hpp"
#include "gemm_f32.hpp"
#include "stream_kernels.hpp"

namespace jg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int HB_BM = 256;
constexpr int HB_BN = 256;
constexpr int HB_BK = 32;                                 // split operands: bfloat16 elements per slab row = 64 bytes
constexpr int HB_WIDE_BK = 64;                            // one plane: 128 bytes, a whole cache line per row
constexpr int HB_THREADS = 256;
constexpr int HB_OPERAND_BYTES = HB_BM * HB_BK * 2;       // one 32 k slab of one plane = 16 KiB (BM == BN)
constexpr int HB_BAND_ROWS = 4;                           // row-tiles per band of the tile order
constexpr int HB_PREFETCH_SLABS = 1;                      // L2 prefetch distance ahead of the transfers, in slabs

struct HbGroup {
    GemmProblem p[kMaxGroup];   // A, B point at bfloat16 data; lda, ldb count 4-byte units (bfloat16 pairs)
    int nprob;
    int M, N, K;                // K counts bfloat16 elements of one plane
    int terms;                  // 1, or 3 for split operands
    int plane;                  // split operands: elements from the hi plane of a row to its lo plane (>= K)
    int tiles_m, tiles_n, total;
    int whole;                  // tiles [0, whole) get a workgroup each; per_xcd = ceil(whole / 8)
    int per_xcd;
    // split tail (parts = 0: none): each of the tiles [whole, total) is cut into `parts` runs of slabs, one
    // workgroup per run, which leaves its raw sums in scratch tile (tile - whole) * parts + part
    int parts;
    float* scratch;             // 256 x 256 floats per run
    int act;
    // Optional second copy of every finished element of C, rounded to bfloat16 as the shard step rounds (hi plane,
    // and lo plane behind it when planes16 = 2): the next layer of an MLP chain reads it as its X shard.
    uint16_t* c16[kMaxGroup];   // per problem, or all null
    int ld16;                   // bfloat16 elements per row of that copy (all planes)
    int plane16, planes16;      // elements from the hi plane of a row to its lo plane; 1 or 2 planes
    // Whole tiles taken last to first.  A launch that reads what the launch before it wrote (the received partial
    // products, or C itself between the chunks of a contraction) alternates with it, so that it starts with the
    // tiles written last - the ones the memory-side cache still holds.  Same tiles, same sums: only the order differs.
    int reverse;
};

struct HbCopy16 {               // what a caller of launch_gemm_bf16_group passes for that copy
    uint16_t* dst[kMaxGroup];
    int ld, plane, planes;
};
constexpr int HB_TILE_FLOATS = HB_BM * HB_BN;

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

typedef int hb_int4 __attribute__((ext_vector_type(4)));

// One 16-byte-per-lane transfer global -> LDS: lane l's data lands at lds_base + 16 l.  Written as
// an instruction rather than through the compiler's builtin: for the builtin the compiler makes every
// later LDS read wait until ALL transfers in flight have landed, which would undo the prefetch
// distance; here the kernel's own vmcnt waits say which slab must have arrived.  M0 carries the LDS
// address and is declared clobbered.
// (The compiler reserves M0 for itself and warns about seeing it in a clobber list; it does not keep a value in
// M0 across a volatile statement, and naming it states what the statement does.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void hb_transfer(const hb_int4& rsrc, unsigned lds_base, int voffset, int soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory", "m0");
}

// Asks L2 for the lines that hold the first four bytes at each lane's offset (lanes whose offset lies outside
// the buffer ask for nothing).  The four bytes go to a 256-byte piece of LDS that nobody reads: the point is that
// the lines are on their way from HBM to L2 some slabs before the transfers that need them.
__device__ __forceinline__ void hb_prefetch(const hb_int4& rsrc, unsigned lds_dump, int voffset, int soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :
                 : "s"(lds_dump), "v"(voffset), "s"(rsrc), "s"(soffset)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// One operand's slabs, global -> LDS, ROW bytes (64 or 128) of every tile row per slab.  ROW / 16 lanes share
// a row, so a wavefront's transfer covers 1024 / ROW rows and the workgroup's four 4096 / ROW; transfer t of a
// lane covers row (4096 / ROW) t + (1024 / ROW) wave + lane / (ROW / 16) of the tile.  With 128-byte rows every
// request is a whole cache line, which L2 serves at 1.6 times the rate of half lines (measured: 25 against
// 15 TB/s into LDS over all CUs).
// LDS rows are not padded; the lane that fills 16-byte slot s of row r fetches chunk s ^ swizzle(r) of that
// row, with swizzle(r) = (r >> 2) & 3 for 64-byte rows and (r >> 1) & 7 for 128-byte rows: the 128-bit fragment
// reads (32 rows, two chunks per instruction) then touch every bank group once per 16 lanes.
template <int ROW>
struct HbLoader {
    static constexpr int kLanesPerRow = ROW / 16;
    static constexpr int kRowsPerWave = 64 / kLanesPerRow;
    static constexpr int kRowsPerTransfer = 4 * kRowsPerWave;
    static constexpr int kTransfers = HB_BM / kRowsPerTransfer;     // per lane, operand and slab: 4 or 8
    __device__ static __forceinline__ int swizzle(int row) { return ROW == 64 ? (row >> 2) & 3 : (row >> 1) & 7; }
    hb_int4 rsrc;               // raw buffer descriptor over the tile's valid rows, in scalar registers
    int voff[kTransfers];       // byte offset of the lane's chunk in slab 0, or kOutOfBuffer for rows past the operand
    int chunk_k;                // first k (within a slab) of the chunk this lane fetches
    // row_bytes: the bytes of a row that exist (all planes)
    __device__ __forceinline__ void init(const float* base, int ld, int extent, int origin, int row_bytes, int wave,
                                         int lane)
    {
        const int valid = min(HB_BM, extent - origin);
        const int r = wave * kRowsPerWave + lane / kLanesPerRow;
        const int chunk = (lane % kLanesPerRow) ^ swizzle(r);       // (rows of later transfers: same swizzle)
        chunk_k = chunk * 8;
#pragma unroll
        for (int t = 0; t < kTransfers; ++t) {
            const int row = t * kRowsPerTransfer + r;
            voff[t] = row < valid ? row * ld * 4 + chunk * 16 : kOutOfBuffer;
        }
        // The descriptor spans the tile's valid rows.  A slab's column offset travels in the scalar
        // offset: the kernel only issues transfers whose chunk exists, so nothing depends on whether
        // the hardware counts that offset in its range check.
        const uintptr_t first = reinterpret_cast<uintptr_t>(base + (int64_t)origin * ld);
        rsrc.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)first);
        rsrc.y = __builtin_amdgcn_readfirstlane((int)((first >> 32) & 0xffff));      // stride 0: raw buffer
        rsrc.z = __builtin_amdgcn_readfirstlane((int)((int64_t)(valid - 1) * ld * 4 + row_bytes));
        rsrc.w = kBufferRsrcFlags;
    }
    // transfer t of the slab whose first column (in bytes, plane offset included) is col_bytes; of a ragged
    // slab (cols < ROW / 2 columns exist) the chunks at or past `cols` are fetched from outside the buffer
    __device__ __forceinline__ void issue(int t, int col_bytes, int cols, unsigned operand_slab, int wave) const
    {
        const int vo = chunk_k < cols ? voff[t] : kOutOfBuffer;
        hb_transfer(rsrc, operand_slab + t * 4096 + wave * 1024, vo, col_bytes);
    }
};

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>): a loop whose index is a compile-time
// constant in every copy of the body.  The epilogue's loops over accumulator blocks are written with it: as
// `#pragma unroll` loops they stay rolled once their body outgrows the compiler's unrolling budget, and an
// accumulator array indexed at run time lives in scratch memory - through the whole K loop.
template <int... I, typename F>
__device__ __forceinline__ void hb_static_for_impl(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void hb_static_for(F&& f)
{
    hb_static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

constexpr int HB_SHUFFLE_LD = 136;     // floats per row of a wave's 32 x 128 staging block: 128 + 8 keeps the two
                                       // half-waves of a write (rows r and r + 4) on different banks

// C = act(acc + addend + bias) + residual for the wave's 128 x 128 part of the tile at (m0, n0).
// The addend is the partial product received from the peer (Eqs. (2), (4)): (kept + received) + bias,
// the order of the separate combine kernel.
// An MFMA accumulator holds one column of four rows per lane, so storing it as it is writes 4 bytes per
// lane (two 128-byte pieces per instruction) - measured at 1.6 TB/s with every CU storing at once.
// Interior tiles therefore pass each 32 x 128 block through the wave's own piece of LDS (free by now) and
// leave as 16 bytes per lane, two 512-byte row pieces per instruction; addend and residual arrive the same way.
// wm, wn: the wave's quadrant; lr, lk: lane coordinates; shuffle: 32 x HB_SHUFFLE_LD floats of LDS owned by the wave.
// c16 (may be null): the bfloat16 copy of the finished elements, ld16 elements per row, lo plane at + lo16 (0: none).
__device__ __forceinline__ void hb_store_tile(const GemmProblem& P, int M, int N, int m0, int n0, int wm, int wn, int lr,
                                              int lk, bool interior, const floatx16 (&acc)[4][4], int act, float* shuffle,
                                              uint16_t* __restrict__ c16 = nullptr, int ld16 = 0, int lo16 = 0)
{
    const float* __restrict__ bias = P.bias;
    const float* __restrict__ residual = P.residual;
    const float* addend = P.addend;     // may be C itself: a later chunk of a contraction adds on top of what C holds
    float* C = P.C;                     // (every element is read and then written by the same lane)
    const int ldc = P.ldc, ldres = P.ldres, ldadd = P.ldadd;
    const bool vec_ok = (((uintptr_t)C | (uintptr_t)addend | (uintptr_t)residual | (uintptr_t)bias) & 15) == 0 &&
                        ((ldc | (addend ? ldadd : 0) | (residual ? ldres : 0)) & 3) == 0 &&
                        (!c16 || ((((uintptr_t)c16) & 7) == 0 && ((ld16 | lo16) & 3) == 0));
    // edge tiles take the same way when N is a multiple of 4 (a lane's four columns are then all inside or all
    // outside), with each row and column group checked
    if (vec_ok && (interior || (N & 3) == 0)) {
        const int lane = lk * 32 + lr;
        const int rrow = lane >> 5, rcol = (lane & 31) * 4;          // read-back position: row 2 p + rrow, 4 columns
        const int col = n0 + wn * 128 + rcol;
        const bool col_in = col < N;
        const vf4 b4 = (bias && col_in) ? *reinterpret_cast<const vf4*>(bias + col) : vf4{0.f, 0.f, 0.f, 0.f};
        // The addend of a 32 x 128 block is requested as a whole (16 loads per lane in flight) while the block
        // before it is being stored, and added to the block in LDS before the read-back loop: fetched inside that
        // loop, one load per step, each step waited out a trip to memory (measured: the launches with an addend
        // took 1.56 times as long as those without).
        vf4 ad[16];
        auto request_addend = [&](int i) __attribute__((always_inline)) {
            const int64_t row0 = m0 + wm * 128 + i * 32 + rrow;
#pragma unroll
            for (int p = 0; p < 16; ++p) {
                const int64_t row = row0 + 2 * p;
                ad[p] = (interior || (col_in && row < M))
                            ? __builtin_nontemporal_load(reinterpret_cast<const vf4*>(addend + row * ldadd + col))
                            : vf4{0.f, 0.f, 0.f, 0.f};
            }
        };
        if (addend) request_addend(0);
        hb_static_for<4>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
#pragma unroll
            for (int jb = 0; jb < 4; ++jb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    shuffle[(8 * (v >> 2) + 4 * lk + (v & 3)) * HB_SHUFFLE_LD + jb * 32 + lr] = acc[i][jb][v];
            if (addend) {
#pragma unroll
                for (int p = 0; p < 16; ++p) {
                    vf4* at = reinterpret_cast<vf4*>(shuffle + (2 * p + rrow) * HB_SHUFFLE_LD + rcol);
                    *at = *at + ad[p];
                }
                if (i < 3) request_addend(i + 1);
            }
            const int64_t row0 = m0 + wm * 128 + i * 32 + rrow;
            // Rolled up, four steps at a time: the body holds every variant of the epilogue (the activation alone
            // is hundreds of instructions); 64 copies of it made each step jump across more code than the
            // instruction cache holds, and a step took 830 cycles instead of a few dozen.  Four steps share their
            // waits (LDS, and memory for the residual).
#pragma unroll 1
            for (int p0 = 0; p0 < 16; p0 += 4) {
                vf4 y[4], res[4];
                bool in[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t row = row0 + 2 * (p0 + q);
                    in[q] = interior || (col_in && row < M);
                    y[q] = *reinterpret_cast<const vf4*>(shuffle + (2 * (p0 + q) + rrow) * HB_SHUFFLE_LD + rcol);
                    res[q] = (residual && in[q]) ? *reinterpret_cast<const vf4*>(residual + row * ldres + col)
                                                 : vf4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t row = row0 + 2 * (p0 + q);
                    vf4 o = y[q] + b4;
                    if (act) o = vf4{activate(o.x, act), activate(o.y, act), activate(o.z, act), activate(o.w, act)};
                    if (residual) o += res[q];
                    if (in[q]) *reinterpret_cast<vf4*>(C + row * ldc + col) = o;
                    if (c16 && in[q]) {
                        typedef uint32_t vu2 __attribute__((ext_vector_type(2)));
                        const uint32_t h0 = bf16_bits(o.x), h1 = bf16_bits(o.y), h2 = bf16_bits(o.z), h3 = bf16_bits(o.w);
                        uint16_t* at = c16 + row * ld16 + col;
                        *reinterpret_cast<vu2*>(at) = vu2{h0 | (h1 << 16), h2 | (h3 << 16)};
                        if (lo16) {
                            const uint32_t l0 = bf16_bits(o.x - bf16_value(h0)), l1 = bf16_bits(o.y - bf16_value(h1));
                            const uint32_t l2 = bf16_bits(o.z - bf16_value(h2)), l3 = bf16_bits(o.w - bf16_value(h3));
                            *reinterpret_cast<vu2*>(at + lo16) = vu2{l0 | (l1 << 16), l2 | (l3 << 16)};
                        }
                    }
                }
            }
        });
    } else {
        const int row_base = m0 + wm * 128 + 4 * lk, col_base = n0 + wn * 128 + lr;
        hb_static_for<16>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value / 4, j = decltype(ic)::value % 4;
                const int col = col_base + j * 32;
                if (col >= N) return;
                const float bj = bias ? bias[col] : 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (row < M) {
                        float y = acc[i][j][v];
                        if (addend) y += addend[(int64_t)row * ldadd + col];
                        y = activate(y + bj, act);
                        if (residual) y += residual[(int64_t)row * ldres + col];
                        C[(int64_t)row * ldc + col] = y;
                        if (c16) {
                            const uint32_t h = bf16_bits(y);
                            c16[(int64_t)row * ld16 + col] = (uint16_t)h;
                            if (lo16) c16[(int64_t)row * ld16 + col + lo16] = (uint16_t)bf16_bits(y - bf16_value(h));
                        }
                    }
                }
        });
    }
}

// grid: kNumXcd * per_xcd workgroups; consecutive ids land on different XCDs, so the id is folded
// into a per-XCD contiguous range of tiles, walked column-major inside bands of 4 row-tiles: the 32
// tiles an XCD has in flight form a 4 x 8 block that shares 4 A panels and 8 B panels in its L2.
__global__ __launch_bounds__(HB_THREADS, 1) void gemm_bf16_nt(const HbGroup g)
{
    constexpr int UNIT = HB_BM * HB_WIDE_BK * 2;            // one operand's slab: 256 rows of 128 bytes = 32 KiB
    constexpr int STAGE = 2 * UNIT;                          // A and B
    typedef HbLoader<HB_WIDE_BK * 2> Loader;
    constexpr int T = Loader::kTransfers;                    // 8 per lane and operand
    constexpr int PF = HB_PREFETCH_SLABS;
    __shared__ __align__(1024) char slab[2 * STAGE];
    __shared__ __align__(256) char dump[HB_THREADS * 4];    // where the prefetches' four bytes per lane end up

    const int M = g.M, N = g.N, K = g.K;
    const int nkt = (K + HB_WIDE_BK - 1) / HB_WIDE_BK;
    // The first 8 * per_xcd workgroups take whole tiles; the rest are the runs of the split tail, in
    // launch order (so they spread over the XCDs and start last).
    int lid, s_begin = 0, s_end = nkt, run = -1;
    if ((int)blockIdx.x < kNumXcd * g.per_xcd) {
        lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
        if (lid >= g.whole) return;
        if (g.reverse) lid = g.whole - 1 - lid;
    } else {
        run = blockIdx.x - kNumXcd * g.per_xcd;
        const int t = run / g.parts, part = run - t * g.parts;
        lid = g.whole + t;
        if (lid >= g.total) return;
        // (a 64-bit division runs on the vector unit; the results are pinned back to scalar registers because
        // the transfers take the slab's column offset from one)
        s_begin = __builtin_amdgcn_readfirstlane((int)((int64_t)nkt * part / g.parts));
        s_end = __builtin_amdgcn_readfirstlane((int)((int64_t)nkt * (part + 1) / g.parts));
    }
    const TileCoord tc = hb_decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lk = lane >> 5;
    const unsigned slab_lds = (unsigned)reinterpret_cast<uintptr_t>((lds_void*)slab);   // LDS address of the buffers

    Loader load_a, load_b;
    const int row_bytes = K * 2;
    load_a.init(P.A, P.lda, M, tc.m0, row_bytes, wave, lane);
    load_b.init(P.B, P.ldb, N, tc.n0, row_bytes, wave, lane);

    const int total_slabs = s_end - s_begin;                // slabs this workgroup multiplies
    const int last_cols = K - (nkt - 1) * HB_WIDE_BK;       // columns of the last slab
    // The slab to request next.  Past the end it stays on the last slab: the surplus requests re-read
    // that slab into buffers nobody reads again, so that every iteration is the same.
    int req_kt = s_begin, req_left = total_slabs;
    // transfer q (0 .. 2 T - 1) of slab kt: A's T transfers, then B's
    auto issue = [&](int q, int kt, unsigned stage) __attribute__((always_inline)) {
        const int cols = kt == nkt - 1 ? last_cols : HB_WIDE_BK;
        const int col = kt * HB_WIDE_BK * 2;
        if (q < T) load_a.issue(q, col, cols, stage, wave);
        else load_b.issue(q - T, col, cols, stage + UNIT, wave);
    };
    auto advance = [&]() __attribute__((always_inline)) {
        if (req_left > 1) {
            --req_left;
            ++req_kt;
        }
    };
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int q = 0; q < 2 * T; ++q) issue(q, req_kt, slab_lds + b * STAGE);
        advance();
    }
    // L2 prefetch, PF slabs ahead of the transfers.  The 32 tiles an XCD has in flight are a block of 4 row tiles x
    // 8 column tiles that walk K together: the 8 workgroups of a row share an A panel, the 4 of a column a B panel,
    // so each asks for its share of a slab's lines only (32 of the 256 A rows, 64 of the 256 B rows; a quarter of
    // that per wavefront).  Where the block is incomplete (edges, a partial round) some lines are not asked for and
    // arrive when the transfers need them, as they would without this.
    // A wavefront's loads complete in order, so a prefetch must be back before the transfers issued after it can
    // count as landed: it is issued right behind a slab's transfers and has two slab times until the next
    // slab's transfers are waited for.
    int pf_a = kOutOfBuffer, pf_b = kOutOfBuffer;
    {
        const int row_a = ((tc.n0 / HB_BN) & 7) * 32 + wave * 8 + lane;
        const int row_b = ((tc.m0 / HB_BM) & 3) * 64 + wave * 16 + lane;
        if (lane < 8 && row_a < min(HB_BM, M - tc.m0)) pf_a = row_a * P.lda * 4;
        if (lane < 16 && row_b < min(HB_BN, N - tc.n0)) pf_b = row_b * P.ldb * 4;
    }
    const unsigned dump_lds = (unsigned)reinterpret_cast<uintptr_t>((lds_void*)dump) + wave * 256;
    int pf_kt = s_begin + 2;
    auto prefetch = [&]() __attribute__((always_inline)) {
        const bool live = pf_kt < nkt;
        const int col = pf_kt * HB_WIDE_BK * 2;
        hb_prefetch(load_a.rsrc, dump_lds, live ? pf_a : kOutOfBuffer, col);
        hb_prefetch(load_b.rsrc, dump_lds, live ? pf_b : kOutOfBuffer, col);
        ++pf_kt;
    };
#pragma unroll
    for (int d = 0; d < PF; ++d) prefetch();

    const bool interior = tc.m0 + HB_BM <= M && tc.n0 + HB_BN <= N;
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment k-step s (16 k, four per slab) of block b: row 32 b + lr (128-byte rows), chunks 2 s + lk
    int frag_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) frag_off[s] = lr * 128 + (((2 * s + lk) ^ Loader::swizzle(lr)) << 4);
    const int a_frag = wm * 4 * 4096;                          // the wave's four row blocks of A
    const int b_frag = UNIT + wn * 4 * 4096;                   // ... and four column blocks of B
    struct Half { bf16x8 a[2][4], b[2][4]; };                  // the operands of two k-steps
    auto read_half = [&](const char* stage, int h, Half& f) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                f.a[s][b] = *reinterpret_cast<const bf16x8*>(stage + a_frag + b * 4096 + frag_off[2 * h + s]);
                f.b[s][b] = *reinterpret_cast<const bf16x8*>(stage + b_frag + b * 4096 + frag_off[2 * h + s]);
            }
    };

    Half f0, f1;                        // a slab's first / second 32 k
    // transfers complete in order: slab 0 has landed once at most those of the second request are in flight
    JG_WAIT_VMCNT(2 * T + 2 * PF);
    __syncthreads();
    read_half(slab, 0, f0);

    for (int it = 0; it < total_slabs; ++it) {
        const char* cur = slab + (it & 1) * STAGE;
        const char* nxt = slab + ((it + 1) & 1) * STAGE;
        read_half(cur, 1, f1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.a[s][i], f0.b[s][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // Slab it + 1 was requested a slab ago and only two prefetches have been issued since; this wavefront's
        // reads of slab `it` are complete (its second half sits in registers).  Behind the barrier slab it + 1 may
        // be read by all and slab it's buffer refilled.
        JG_WAIT_VMCNT(PF > 0 ? 2 : 0);
        __builtin_amdgcn_s_waitcnt(0xC07F);    // lgkmcnt(0) only
        __syncthreads();
        read_half(nxt, 0, f0);                 // (after the last slab: a surplus copy, read but not used)
        __builtin_amdgcn_sched_barrier(0);
        {
            const unsigned stage = slab_lds + (it & 1) * STAGE;
            const int kt = req_kt;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.a[s][i], f1.b[s][j], acc[i][j], 0, 0, 0);
                        const int idx = s * 16 + i * 4 + j;
                        // slab it + 2, one transfer after every second MFMA
                        if ((idx & 1) == 0) issue(idx >> 1, kt, stage);
                        __builtin_amdgcn_sched_barrier(0);
                    }
            if (PF > 0) prefetch();
            advance();
        }
    }
    JG_WAIT_VMCNT(0);       // the surplus transfers have landed ...
    __syncthreads();        // ... and nobody reads a slab any more: the buffers become the waves' staging blocks
    float* shuffle = reinterpret_cast<float*>(slab + wave * (32 * HB_SHUFFLE_LD * 4));
    if (run < 0) {
        hb_store_tile(P, M, N, tc.m0, tc.n0, wm, wn, lr, lk, interior, acc, g.act, shuffle, g.c16[tc.prob], g.ld16,
                      g.planes16 == 2 ? g.plane16 : 0);
    } else {                // a run of a split tile: raw sums into its scratch tile
        GemmProblem raw = {};
        raw.C = g.scratch + (int64_t)run * HB_TILE_FLOATS;
        raw.ldc = HB_BN;
        hb_store_tile(raw, HB_BM, HB_BN, 0, 0, wm, wn, lr, lk, true, acc, kActNone, shuffle);
    }
}

// Split operands in one pass over K (terms = 3).  A slab is the
// same 32 k of all four planes (A hi, A lo, B hi, B lo: 64 KiB) and gives three products per block
// - hi lo, lo hi, hi hi, the small ones first within every 16 k - so four operand slabs feed what three
// separate passes fetch six for.  The transfers are what bounds the one-plane loop (L2 delivers about
// 12 TB/s to LDS), so this form is faster by about that third.  Two slab buffers: the transfers of slab
// it + 2 are issued behind slab it's mid-slab barrier, into the buffer of the slab just used up, and have
// a whole slab's time (96 MFMAs per wave) to land.
// Against three separate passes with the two small cross terms first (which this mode was before: added
// to an already large sum the small products lose their low bits at every step), the small products here
// meet a sum that has already grown, as in any single pass; the rounding walk on same-sign data is that of
// 3 K / 16 steps (see the tolerance notes of the tests).
__global__ __launch_bounds__(HB_THREADS, 1) void gemm_bf16x3_nt(const HbGroup g)
{
    constexpr int STAGE = 4 * HB_OPERAND_BYTES;              // 64 KiB
    constexpr int PF = HB_PREFETCH_SLABS;
    __shared__ __align__(1024) char slab[2 * STAGE];
    __shared__ __align__(256) char dump[HB_THREADS * 4];    // where the prefetches' four bytes per lane end up

    const int M = g.M, N = g.N, K = g.K;
    const int nkt = (K + HB_BK - 1) / HB_BK;
    int lid, s_begin = 0, s_end = nkt, run = -1;
    if ((int)blockIdx.x < kNumXcd * g.per_xcd) {
        lid = (blockIdx.x % kNumXcd) * g.per_xcd + blockIdx.x / kNumXcd;
        if (lid >= g.whole) return;
        if (g.reverse) lid = g.whole - 1 - lid;
    } else {
        run = blockIdx.x - kNumXcd * g.per_xcd;
        const int t = run / g.parts, part = run - t * g.parts;
        lid = g.whole + t;
        if (lid >= g.total) return;
        s_begin = __builtin_amdgcn_readfirstlane((int)((int64_t)nkt * part / g.parts));
        s_end = __builtin_amdgcn_readfirstlane((int)((int64_t)nkt * (part + 1) / g.parts));
    }
    const TileCoord tc = hb_decode_tile(g, lid);
    const GemmProblem& P = g.p[tc.prob];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, lk = lane >> 5;
    const unsigned slab_lds = (unsigned)reinterpret_cast<uintptr_t>((lds_void*)slab);

    HbLoader<HB_BK * 2> load_a, load_b;
    const int row_bytes = (g.plane + K) * 2;
    load_a.init(P.A, P.lda, M, tc.m0, row_bytes, wave, lane);
    load_b.init(P.B, P.ldb, N, tc.n0, row_bytes, wave, lane);
    const int plane_bytes = g.plane * 2;
    const int total_slabs = s_end - s_begin;
    const int last_cols = K - (nkt - 1) * HB_BK;
    // the slab to request next; past the end it stays on the last one (surplus requests into a buffer
    // nobody reads again keep the loop uniform)
    int req_kt = s_begin, req_left = total_slabs;
    // transfer q (0 .. 15) of the next slab: planes A hi, A lo, B hi, B lo, four transfers each
    auto issue = [&](int q, int kt, unsigned stage) __attribute__((always_inline)) {
        const int cols = kt == nkt - 1 ? last_cols : HB_BK;
        const int col = kt * HB_BK * 2 + ((q & 4) ? plane_bytes : 0);
        if (q < 8) load_a.issue(q & 3, col, cols, stage + (q >> 2) * HB_OPERAND_BYTES, wave);
        else load_b.issue(q & 3, col, cols, stage + (q >> 2) * HB_OPERAND_BYTES, wave);
    };
    auto advance = [&]() __attribute__((always_inline)) {
        if (req_left > 1) {
            --req_left;
            ++req_kt;
        }
    };
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int q = 0; q < 16; ++q) issue(q, req_kt, slab_lds + b * STAGE);
        advance();
    }
    // L2 prefetch as in gemm_bf16_nt: the workgroup's share of the rows, both planes of each (a 64-byte slab row is
    // half a line, so every second request finds its line on the way already)
    int pf_a = kOutOfBuffer, pf_b = kOutOfBuffer;
    {
        const int row_a = ((tc.n0 / HB_BN) & 7) * 32 + wave * 8 + (lane & 7);
        const int row_b = ((tc.m0 / HB_BM) & 3) * 64 + wave * 16 + (lane & 15);
        if (lane < 16 && row_a < min(HB_BM, M - tc.m0)) pf_a = row_a * P.lda * 4 + (lane >> 3) * plane_bytes;
        if (lane < 32 && row_b < min(HB_BN, N - tc.n0)) pf_b = row_b * P.ldb * 4 + (lane >> 4) * plane_bytes;
    }
    const unsigned dump_lds = (unsigned)reinterpret_cast<uintptr_t>((lds_void*)dump) + wave * 256;
    int pf_kt = s_begin + 2;
    auto prefetch = [&]() __attribute__((always_inline)) {
        const bool live = pf_kt < nkt;
        const int col = pf_kt * HB_BK * 2;
        hb_prefetch(load_a.rsrc, dump_lds, live ? pf_a : kOutOfBuffer, col);
        hb_prefetch(load_b.rsrc, dump_lds, live ? pf_b : kOutOfBuffer, col);
        ++pf_kt;
    };
#pragma unroll
    for (int d = 0; d < PF; ++d) prefetch();

    const bool interior = tc.m0 + HB_BM <= M && tc.n0 + HB_BN <= N;
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    int frag_off[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) frag_off[s] = lr * 64 + (((2 * s + lk) ^ ((lr >> 2) & 3)) << 4);
    const int a_frag = wm * 4 * 2048;
    const int b_frag = 2 * HB_OPERAND_BYTES + wn * 4 * 2048;
    struct Frags { bf16x8 ah[4], al[4], bh[4], bl[4]; };
    auto read_frags = [&](const char* stage, int s, Frags& f) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            f.ah[b] = *reinterpret_cast<const bf16x8*>(stage + a_frag + b * 2048 + frag_off[s]);
            f.al[b] = *reinterpret_cast<const bf16x8*>(stage + a_frag + HB_OPERAND_BYTES + b * 2048 + frag_off[s]);
            f.bh[b] = *reinterpret_cast<const bf16x8*>(stage + b_frag + b * 2048 + frag_off[s]);
            f.bl[b] = *reinterpret_cast<const bf16x8*>(stage + b_frag + HB_OPERAND_BYTES + b * 2048 + frag_off[s]);
        }
    };

    Frags f0, f1;                       // operands of a slab's first / second 16 k
    JG_WAIT_VMCNT(16 + 2 * PF);         // slab 0 has landed (the second request and the prefetches may be in flight)
    __syncthreads();
    read_frags(slab, 0, f0);

    for (int it = 0; it < total_slabs; ++it) {
        char* cur = slab + (it & 1) * STAGE;
        const char* nxt = slab + ((it + 1) & 1) * STAGE;
        read_frags(cur, 1, f1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.ah[i], f0.bl[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.al[i], f0.bh[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.ah[i], f0.bh[j], acc[i][j], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
        // Slab it + 1 was requested a slab ago and only two prefetches have been issued since; this wavefront's
        // reads of slab `it` are complete.  Behind the barrier slab it + 1 may be read and slab it's buffer refilled.
        JG_WAIT_VMCNT(PF > 0 ? 2 : 0);
        __builtin_amdgcn_s_waitcnt(0xC07F);    // lgkmcnt(0) only
        __syncthreads();
        read_frags(nxt, 0, f0);                // (after the last slab: a surplus copy, read but not used)
        __builtin_amdgcn_sched_barrier(0);
        {
            const unsigned stage = slab_lds + (it & 1) * STAGE;
            const int kt = req_kt;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.ah[i], f1.bl[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.al[i], f1.bh[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.ah[i], f1.bh[j], acc[i][j], 0, 0, 0);
                    issue(i * 4 + j, kt, stage);        // slab it + 2, one transfer after every third MFMA
                    __builtin_amdgcn_sched_barrier(0);
                }
            if (PF > 0) prefetch();
            advance();
        }
    }
    JG_WAIT_VMCNT(0);       // the surplus transfers have landed ...
    __syncthreads();        // ... and nobody reads a slab any more: the buffers become the waves' staging blocks
    float* shuffle = reinterpret_cast<float*>(slab + wave * (32 * HB_SHUFFLE_LD * 4));
    if (run < 0) {
        hb_store_tile(P, M, N, tc.m0, tc.n0, wm, wn, lr, lk, interior, acc, g.act, shuffle, g.c16[tc.prob], g.ld16,
                      g.planes16 == 2 ? g.plane16 : 0);
    } else {
        GemmProblem raw = {};
        raw.C = g.scratch + (int64_t)run * HB_TILE_FLOATS;
        raw.ldc = HB_BN;
        hb_store_tile(raw, HB_BM, HB_BN, 0, 0, wm, wn, lr, lk, true, acc, kActNone, shuffle);
    }
}

// Second kernel of a launch with a split tail: adds a tile's runs in ascending k order, then what the
// epilogue adds, and stores C.  grid: kHbJoinSlices workgroups per tail tile, each with a band of its rows.
constexpr int kHbJoinSlices = 32;
__global__ __launch_bounds__(HB_THREADS) void gemm_bf16_join(const HbGroup g)
{
    const int t = blockIdx.x / kHbJoinSlices, slice = blockIdx.x % kHbJoinSlices;
    constexpr int kSliceFloats = HB_TILE_FLOATS / kHbJoinSlices;
    const TileCoord tc = hb_decode_tile(g, g.whole + t);
    const GemmProblem& P = g.p[tc.prob];
    const float* runs = g.scratch + (int64_t)t * g.parts * HB_TILE_FLOATS;
    const bool interior = tc.m0 + HB_BM <= g.M && tc.n0 + HB_BN <= g.N;
    uint16_t* __restrict__ c16 = g.c16[tc.prob];
    const int lo16 = g.planes16 == 2 ? g.plane16 : 0;
    const bool vec_ok = (((uintptr_t)P.C | (uintptr_t)P.addend | (uintptr_t)P.residual | (uintptr_t)P.bias) & 15) == 0 &&
                        ((P.ldc | (P.addend ? P.ldadd : 0) | (P.residual ? P.ldres : 0)) & 3) == 0 &&
                        (!c16 || ((((uintptr_t)c16) & 7) == 0 && ((g.ld16 | lo16) & 3) == 0));
    if (interior && vec_ok) {
        for (int u = slice * (kSliceFloats / 4) + threadIdx.x; u < (slice + 1) * (kSliceFloats / 4); u += HB_THREADS) {
            const int r = u / (HB_BN / 4), c = (u - r * (HB_BN / 4)) * 4;
            vf4 y = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(runs) + u);
            for (int p = 1; p < g.parts; ++p)
                y += __builtin_nontemporal_load(reinterpret_cast<const vf4*>(runs + (int64_t)p * HB_TILE_FLOATS) + u);
            const int64_t row = tc.m0 + r;
            const int col = tc.n0 + c;
            if (P.addend) y += __builtin_nontemporal_load(reinterpret_cast<const vf4*>(P.addend + row * P.ldadd + col));
            if (P.bias) y += *reinterpret_cast<const vf4*>(P.bias + col);
            if (g.act) y = vf4{activate(y.x, g.act), activate(y.y, g.act), activate(y.z, g.act), activate(y.w, g.act)};
            if (P.residual) y += *reinterpret_cast<const vf4*>(P.residual + row * P.ldres + col);
            *reinterpret_cast<vf4*>(P.C + row * P.ldc + col) = y;
            if (c16) {
                typedef uint32_t vu2 __attribute__((ext_vector_type(2)));
                const uint32_t h0 = bf16_bits(y.x), h1 = bf16_bits(y.y), h2 = bf16_bits(y.z), h3 = bf16_bits(y.w);
                uint16_t* at = c16 + row * g.ld16 + col;
                *reinterpret_cast<vu2*>(at) = vu2{h0 | (h1 << 16), h2 | (h3 << 16)};
                if (lo16) {
                    const uint32_t l0 = bf16_bits(y.x - bf16_value(h0)), l1 = bf16_bits(y.y - bf16_value(h1));
                    const uint32_t l2 = bf16_bits(y.z - bf16_value(h2)), l3 = bf16_bits(y.w - bf16_value(h3));
                    *reinterpret_cast<vu2*>(at + lo16) = vu2{l0 | (l1 << 16), l2 | (l3 << 16)};
                }
            }
        }
    } else {
        for (int u = slice * kSliceFloats + threadIdx.x; u < (slice + 1) * kSliceFloats; u += HB_THREADS) {
            const int r = u / HB_BN, c = u - r * HB_BN;
            const int64_t row = tc.m0 + r;
            const int col = tc.n0 + c;
            if (row >= g.M || col >= g.N) continue;
            float y = runs[u];
            for (int p = 1; p < g.parts; ++p) y += runs[(int64_t)p * HB_TILE_FLOATS + u];
            if (P.addend) y += P.addend[row * P.ldadd + col];
            y = activate(y + (P.bias ? P.bias[col] : 0.f), g.act);
            if (P.residual) y += P.residual[row * P.ldres + col];
            P.C[row * P.ldc + col] = y;
            if (c16) {
                const uint32_t h = bf16_bits(y);
                c16[row * g.ld16 + col] = (uint16_t)h;
                if (lo16) c16[row * g.ld16 + col + lo16] = (uint16_t)bf16_bits(y - bf16_value(h));
            }
        }
    }
}

// Can this operand take the 16-byte transfers?  (rows 16-byte aligned, K in whole chunks)
inline bool hb_operand_ok(const float* p, int ld, int K)
{
    return ((uintptr_t)p & 15) == 0 && (ld & 3) == 0 && (K & 7) == 0 && ld <= kMaxDirectLd / 2;
}

// One grouped launch.  Preconditions (checked by the C-ABI layer when the plan is made): every
// operand passes hb_operand_ok; 1 <= nprob <= 4; M, N, K >= 1.
// `cus` workgroups run at a time.  When the tiles do not fill whole rounds of them, the tiles of the last
// partial round are cut into runs of slabs so that every CU gets one (at least kHbMinRunSlabs slabs each);
// scratch holds a 256 x 256 tile of floats per run, or is null / too small: then every tile stays whole.
// Second summation level of the bfloat16 kernels, taken between launches: the length of the chunks a contraction of
// K (elements of one plane) is cut into.  A same-sign sum of n accumulate steps (one MFMA = 16 k, three MFMAs per
// 16 k with split operands) was measured to drift by 4.7e-7 / 7.3e-7 / 9.8e-7 of its magnitude at n = 32 / 64 / 96,
// about n^0.62; c equal chunks leave that of n / c steps divided by sqrt(c).  The smallest c that stays at the level
// of 64 steps (7.3e-7, inside the 1e-6 the layer is held to) is taken; chunks are whole 64-element slabs.
inline int bf16_chunk_k(int K, int terms)
{
    const double steps = (double)terms * K / 16.0;
    const double level = std::pow(64.0, 0.62);
    int c = 1;
    while (c < 256 && std::pow(steps / c, 0.62) > level * std::sqrt((double)c)) ++c;
    const int chunk = ((K + c - 1) / c + 63) / 64 * 64;
    return chunk < K ? chunk : K;
}

constexpr int kHbMinRunSlabs = 16;
constexpr int kHbJoinCostSlabs = 40;    // the join kernel takes about as long as 40 slabs of the main loop
inline size_t bf16_tail_scratch_bytes(int cus) { return (size_t)cus * HB_TILE_FLOATS * sizeof(float); }

// plane: with split operands, the distance in elements from a row's hi plane to its lo plane (>= K, a multiple of 8)
inline hipError_t make_bf16_group(const GemmGroup& src, int terms, int plane, int cus, float* scratch, size_t scratch_bytes,
                                  HbGroup& g, const HbCopy16* copy16 = nullptr, bool reverse = false)
{
    g.reverse = reverse ? 1 : 0;
    for (int i = 0; i < kMaxGroup; ++i) g.p[i] = src.p[i];
    for (int i = 0; i < kMaxGroup; ++i) g.c16[i] = copy16 ? copy16->dst[i] : nullptr;
    g.ld16 = copy16 ? copy16->ld : 0;
    g.plane16 = copy16 ? copy16->plane : 0;
    g.planes16 = copy16 ? copy16->planes : 1;
    g.nprob = src.nprob;
    g.M = src.M;
    g.N = src.N;
    g.K = src.K;
    g.terms = terms;
    g.plane = plane;
    g.act = src.act;
    if (terms == 3 && (plane < src.K || (plane & 7))) return hipErrorInvalidValue;
    g.tiles_m = (g.M + HB_BM - 1) / HB_BM;
    g.tiles_n = (g.N + HB_BN - 1) / HB_BN;
    const int64_t total = (int64_t)g.nprob * g.tiles_m * g.tiles_n;
    if (total + kNumXcd > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    for (int i = 0; i < g.nprob; ++i)
        if (!hb_operand_ok(g.p[i].A, g.p[i].lda, g.K) || !hb_operand_ok(g.p[i].B, g.p[i].ldb, g.K))
            return hipErrorInvalidValue;
    g.total = (int)total;
    g.whole = g.total;
    g.parts = 0;
    g.scratch = nullptr;
    // in slabs of the one-plane loop; the one-pass split-operand kernel cuts a tile's K / 32 slabs, each three of these
    const int tile_slabs = (g.K + HB_BK - 1) / HB_BK * terms;
    const int tail = cus > 0 ? g.total % cus : 0;
    if (scratch && tail > 0 && 2 * tail <= cus) {
        int parts = cus / tail;
        if (parts > tile_slabs / kHbMinRunSlabs) parts = tile_slabs / kHbMinRunSlabs;
        // worth it when the shortened last round saves at least twice what the join costs
        const bool pays = parts >= 2 && tile_slabs - tile_slabs / parts >= 2 * kHbJoinCostSlabs;
        if (pays && (size_t)tail * parts * HB_TILE_FLOATS * sizeof(float) <= scratch_bytes) {
            g.whole = g.total - tail;       // a multiple of cus, hence of the number of XCDs
            g.parts = parts;
            g.scratch = scratch;
        }
    }
    g.per_xcd = (g.whole + kNumXcd - 1) / kNumXcd;
    return hipSuccess;
}

inline unsigned bf16_grid(const HbGroup& g) { return (unsigned)(kNumXcd * g.per_xcd + (g.total - g.whole) * g.parts); }

// cus: compute units of the device (one workgroup each).  *needs_join: launch_gemm_bf16_join must follow.
// copy16 (may be null): see HbGroup::c16.
inline hipError_t launch_gemm_bf16_group(const GemmGroup& src, int terms, int plane, int cus, float* scratch,
                                         size_t scratch_bytes, hipStream_t stream, HbGroup& g, bool* needs_join,
                                         const HbCopy16* copy16 = nullptr, bool reverse = false)
{
    *needs_join = false;
    const hipError_t e = make_bf16_group(src, terms, plane, cus, scratch, scratch_bytes, g, copy16, reverse);
    if (e != hipSuccess) return e;
    if (terms == 3) hipLaunchKernelGGL(gemm_bf16x3_nt, dim3(bf16_grid(g)), dim3(HB_THREADS), 0, stream, g);
    else hipLaunchKernelGGL(gemm_bf16_nt, dim3(bf16_grid(g)), dim3(HB_THREADS), 0, stream, g);
    *needs_join = g.parts > 0;
    return hipGetLastError();
}

inline hipError_t launch_gemm_bf16_join(const HbGroup& g, hipStream_t stream)
{
    hipLaunchKernelGGL(gemm_bf16_join, dim3((unsigned)(g.total - g.whole) * kHbJoinSlices), dim3(HB_THREADS), 0, stream, g);
    return hipGetLastError();
}

}  // namespace jg

// Layer norm over the channels a rank holds of each token (Sec. 3: a layer norm before each mixing
// MLP; Sec. 5 "Layer norms": the library routine applied to the rank's own channels):
//     mu = mean_c x,  var = mean_c (x - mu)^2,  y[c] = (x[c] - mu) / sqrt(var + eps) * gamma[c] + beta[c]
// per row of a rank's activation block.
//
// HBM-bound: every element is read once and written once.  One wavefront owns one row and keeps it
// in registers (NV 16-byte vectors per lane) between the reduction and the normalisation, so the row
// is not read a second time; the two reductions (sum, then sum of squared deviations) and the
// normalisation run in double, which this chip does at half the FP32 rate — far below the time the
// memory traffic takes — and leaves the result within one FP32 rounding of the exact value.  Rows that do not fit
// the register budget, or whose length or alignment rules out 128-bit accesses, take a plain
// kernel (one workgroup per row, three passes, the second and third served by the caches).
#pragma once

#include <hip/hip_runtime.h>

#include "cvt_kernels.hpp"
#include "stream_kernels.hpp"

namespace jg {

struct NormBlock {
    const float* x;      // rows x cols, dense
    float* y;            // rows x cols, dense; may be x itself
    const float* gamma;  // the block's cols scale factors, or nullptr (1)
    const float* beta;   // the block's cols offsets, or nullptr (0)
    float* xb;           // optional: x + row_bias[row] per row (the input with a per-token offset added, for a skip
                         // connection that carries the bias of a layer along the token dimension); nullptr: none
    const float* row_bias;   // rows values, read when xb is set
    uint16_t* y16;       // optional second copy of y rounded to bfloat16 as the shard step rounds (rows of planes16
                         // planes of plane16 elements: [hi | lo]); nullptr: none.  Taken by the register-resident
                         // kernel only: see launch_norm_group
};

struct NormGroup {
    NormBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;      // common shape
    double eps;
    int plane16, planes16;   // layout of the y16 copies
};

constexpr int NORM_THREADS = 256;
constexpr int NORM_ROWS_PER_WG = NORM_THREADS / 64;
constexpr int kNormMaxVectorsPerLane = 32;     // register-resident rows: up to 64 * 32 * 4 = 8192 columns


// The sum of a value over the 64 lanes of a wavefront, the same in every lane.  It goes through the data-parallel-
// primitive paths of the vector ALU (six round trips through the LDS crossbar, as shuffles make them, cost the
// one-pass backward kernel a tenth of its time): within quads, within eights (half mirror), within rows of 16
// (mirror), then lane 15 of every row into the next row and lane 31 into the upper half; lane 63 ends with the
// total, which goes out through a scalar register.  A fixed order, so the same bits on every run.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_neighbour(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xF, false);
    return __hiloint2double(hi, lo);        // lanes outside ROW_MASK, or without a source lane, see +0.0
}
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_neighbour<0xB1, 0xF>(v);       // quad_perm [1, 0, 3, 2]
    v += dpp_neighbour<0x4E, 0xF>(v);       // quad_perm [2, 3, 0, 1]
    v += dpp_neighbour<0x141, 0xF>(v);      // row_half_mirror
    v += dpp_neighbour<0x140, 0xF>(v);      // row_mirror
    v += dpp_neighbour<0x142, 0xA>(v);      // row_bcast15 into rows 1 and 3
    v += dpp_neighbour<0x143, 0xC>(v);      // row_bcast31 into rows 2 and 3
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

// grid: x = row / NORM_ROWS_PER_WG, y = block.  cols is a multiple of 4, cols / 4 <= 64 * NV.
template <int NV>
__global__ __launch_bounds__(NORM_THREADS) void layernorm_rows_f32(const NormGroup g)
{
    const NormBlock& B = g.b[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * NORM_ROWS_PER_WG + (threadIdx.x >> 6);
    if (row >= g.rows) return;       // whole wavefronts leave; no barrier below
    const int nvec = g.cols >> 2;
    const vf4* x = reinterpret_cast<const vf4*>(B.x + (int64_t)row * g.cols);
    vf4 v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        v[i] = c < nvec ? x[c] : vf4{0.f, 0.f, 0.f, 0.f};
    }
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += ((double)v[i].x + (double)v[i].y) + ((double)v[i].z + (double)v[i].w);
    const double mu = wave_sum(s) / (double)g.cols;
    // The row stays in registers as FP32; each pass widens it again (keeping the widened copies would
    // triple the register count and halve the number of rows in flight).
#pragma unroll
    for (int i = 0; i < NV; ++i) asm volatile("" : "+v"(v[i]));
    double q = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (i * 64 + lane < nvec) {
            const double dx = (double)v[i].x - mu, dy = (double)v[i].y - mu;
            const double dz = (double)v[i].z - mu, dw = (double)v[i].w - mu;
            q += (dx * dx + dy * dy) + (dz * dz + dw * dw);
        }
    }
    const double rstd = 1.0 / sqrt(wave_sum(q) / (double)g.cols + g.eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) asm volatile("" : "+v"(v[i]));
    if (B.xb) {
        const float rb = B.row_bias[row];
        vf4* xb = reinterpret_cast<vf4*>(B.xb + (int64_t)row * g.cols);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = i * 64 + lane;
            if (c < nvec) xb[c] = v[i] + rb;
        }
    }
    vf4* y = reinterpret_cast<vf4*>(B.y + (int64_t)row * g.cols);
    const vf4* gamma = reinterpret_cast<const vf4*>(B.gamma);
    const vf4* beta = reinterpret_cast<const vf4*>(B.beta);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        if (c < nvec) {
            const vf4 ga = gamma ? gamma[c] : vf4{1.f, 1.f, 1.f, 1.f};
            const vf4 be = beta ? beta[c] : vf4{0.f, 0.f, 0.f, 0.f};
            vf4 o;
            o.x = (float)(((double)v[i].x - mu) * rstd * (double)ga.x + (double)be.x);
            o.y = (float)(((double)v[i].y - mu) * rstd * (double)ga.y + (double)be.y);
            o.z = (float)(((double)v[i].z - mu) * rstd * (double)ga.z + (double)be.z);
            o.w = (float)(((double)v[i].w - mu) * rstd * (double)ga.w + (double)be.w);
            y[c] = o;
            if (B.y16) {
                typedef uint32_t vu2 __attribute__((ext_vector_type(2)));
                const uint32_t h0 = bf16_bits(o.x), h1 = bf16_bits(o.y), h2 = bf16_bits(o.z), h3 = bf16_bits(o.w);
                uint16_t* at = B.y16 + (int64_t)row * g.plane16 * g.planes16 + 4 * c;
                *reinterpret_cast<vu2*>(at) = vu2{h0 | (h1 << 16), h2 | (h3 << 16)};
                if (g.planes16 == 2) {
                    const uint32_t l0 = bf16_bits(o.x - bf16_value(h0)), l1 = bf16_bits(o.y - bf16_value(h1));
                    const uint32_t l2 = bf16_bits(o.z - bf16_value(h2)), l3 = bf16_bits(o.w - bf16_value(h3));
                    *reinterpret_cast<vu2*>(at + g.plane16) = vu2{l0 | (l1 << 16), l2 | (l3 << 16)};
                }
            }
        }
    }
}

// Any row length and alignment.  grid: x = row, y = block.
__global__ __launch_bounds__(NORM_THREADS) void layernorm_generic_f32(const NormGroup g)
{
    __shared__ double part[NORM_THREADS / 64];
    const NormBlock& B = g.b[blockIdx.y];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* x = B.x + (int64_t)blockIdx.x * g.cols;
    float* y = B.y + (int64_t)blockIdx.x * g.cols;

    auto block_sum = [&](double v) {
        v = wave_sum(v);
        __syncthreads();             // the previous sum has been read by every wavefront
        if (lane == 0) part[wave] = v;
        __syncthreads();
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < NORM_THREADS / 64; ++w) t += part[w];
        return t;
    };

    double s = 0.0;
    for (int c = tid; c < g.cols; c += NORM_THREADS) s += (double)x[c];
    const double mu = block_sum(s) / (double)g.cols;
    double q = 0.0;
    for (int c = tid; c < g.cols; c += NORM_THREADS) {
        const double d = (double)x[c] - mu;
        q += d * d;
    }
    const double rstd = 1.0 / sqrt(block_sum(q) / (double)g.cols + g.eps);
    // every element is read for the last time by the thread that overwrites it: y may be x
    float* xb = B.xb ? B.xb + (int64_t)blockIdx.x * g.cols : nullptr;
    const float rb = B.xb ? B.row_bias[blockIdx.x] : 0.f;
    for (int c = tid; c < g.cols; c += NORM_THREADS) {
        const double ga = B.gamma ? (double)B.gamma[c] : 1.0;
        const double be = B.beta ? (double)B.beta[c] : 0.0;
        const float xv = x[c];
        if (xb) xb[c] = xv + rb;
        y[c] = (float)(((double)xv - mu) * rstd * ga + be);
    }
}

// ------------------------------------------------------------------------------------------
// Backward of the norm (Sec. 3's norm in the backward pass of Sec. 4.1).  Per row of a block, with
// xhat = (x - mu) * rstd and g = dy * gamma:
//     dx = (g - mean(g) - xhat * mean(g * xhat)) * rstd,
// and over the rows of all blocks that hold a channel:  dgamma = sum dy * xhat,  dbeta = sum dy.
// Two forms.  One pass (layernorm_bwd_fused_f32 and its join): a workgroup per band of rows keeps the column sums
// of its band while it produces dx.  Two kernels, for rows that form cannot take or when the caller's workspace has
// no room for the bands' sums: rows (one wavefront or workgroup per row, double arithmetic as in the forward; it
// also leaves mu and rstd of every row in `stats`), then columns (as the bias gradient's column sums: 32-column
// strips, double accumulators, a fixed order).
// ------------------------------------------------------------------------------------------
struct NormBwdBlock {
    const float* x;      // rows x cols, dense: the forward's input
    const float* dy;     // rows x cols, dense: gradient of the forward's output
    float* dx;           // rows x cols, dense
    const float* gamma;  // the block's cols scale factors, or nullptr (1)
    double* stats;       // rows x 2: mu, rstd (written by the row kernel, read by the column kernel)
    const float* add;    // rows x cols, dense, added to dx before its one rounding (a skip connection), or nullptr
};

struct NormBwdGroup {
    NormBwdBlock b[kMaxBlocks];
    int nblocks;
    int rows, cols;
    double eps;
    // the one-pass kernel (layernorm_bwd_fused_f32): rows per workgroup, workgroups per block, and where each leaves
    // its column sums (nblocks x nbands x cols pairs of doubles: dgamma's, dbeta's), or nullptr (no column sums wanted)
    int band_rows, nbands;
    double* partial;
};

// grid: x = row, y = block
__global__ __launch_bounds__(NORM_THREADS) void layernorm_bwd_rows_f32(const NormBwdGroup g)
{
    __shared__ double part[NORM_THREADS / 64];
    const NormBwdBlock& B = g.b[blockIdx.y];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t off = (int64_t)blockIdx.x * g.cols;
    const float* x = B.x + off;
    const float* dy = B.dy + off;
    float* dx = B.dx + off;
    auto block_sum = [&](double v) {
        v = wave_sum(v);
        __syncthreads();
        if (lane == 0) part[wave] = v;
        __syncthreads();
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < NORM_THREADS / 64; ++w) t += part[w];
        return t;
    };
    double s = 0.0;
    for (int c = tid; c < g.cols; c += NORM_THREADS) s += (double)x[c];
    const double mu = block_sum(s) / (double)g.cols;
    double q = 0.0;
    for (int c = tid; c < g.cols; c += NORM_THREADS) {
        const double d = (double)x[c] - mu;
        q += d * d;
    }
    const double rstd = 1.0 / sqrt(block_sum(q) / (double)g.cols + g.eps);
    double sg = 0.0, sgx = 0.0;
    for (int c = tid; c < g.cols; c += NORM_THREADS) {
        const double gv = (double)dy[c] * (B.gamma ? (double)B.gamma[c] : 1.0);
        sg += gv;
        sgx += gv * (((double)x[c] - mu) * rstd);
    }
    const double mg = block_sum(sg) / (double)g.cols;
    const double mgx = block_sum(sgx) / (double)g.cols;
    for (int c = tid; c < g.cols; c += NORM_THREADS) {
        const double gv = (double)dy[c] * (B.gamma ? (double)B.gamma[c] : 1.0);
        const double xh = ((double)x[c] - mu) * rstd;
        const double o = (gv - mg - xh * mgx) * rstd;
        dx[c] = (float)(B.add ? o + (double)B.add[off + c] : o);
    }
    if (tid == 0) {
        B.stats[2 * (int64_t)blockIdx.x] = mu;
        B.stats[2 * (int64_t)blockIdx.x + 1] = rstd;
    }
}

// The same with one wavefront per row and the row of x and of dy in registers (NV 16-byte vectors per lane each),
// as the forward's register-resident kernel: every element is read once.  cols % 4 == 0, cols / 4 <= 64 * NV,
// 16-byte aligned operands.  grid: x = row / NORM_ROWS_PER_WG, y = block.
template <int NV>
__global__ __launch_bounds__(NORM_THREADS) void layernorm_bwd_rows_reg_f32(const NormBwdGroup g)
{
    const NormBwdBlock& B = g.b[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * NORM_ROWS_PER_WG + (threadIdx.x >> 6);
    if (row >= g.rows) return;
    const int nvec = g.cols >> 2;
    const vf4* x = reinterpret_cast<const vf4*>(B.x + (int64_t)row * g.cols);
    const vf4* dy = reinterpret_cast<const vf4*>(B.dy + (int64_t)row * g.cols);
    const vf4* gamma = reinterpret_cast<const vf4*>(B.gamma);
    vf4 v[NV], d[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        v[i] = c < nvec ? x[c] : vf4{0.f, 0.f, 0.f, 0.f};
        d[i] = c < nvec ? __builtin_nontemporal_load(dy + c) : vf4{0.f, 0.f, 0.f, 0.f};
    }
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += ((double)v[i].x + (double)v[i].y) + ((double)v[i].z + (double)v[i].w);
    const double mu = wave_sum(s) / (double)g.cols;
#pragma unroll
    for (int i = 0; i < NV; ++i) asm volatile("" : "+v"(v[i]));
    double q = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (i * 64 + lane < nvec) {
            const double dx = (double)v[i].x - mu, dy2 = (double)v[i].y - mu;
            const double dz = (double)v[i].z - mu, dw = (double)v[i].w - mu;
            q += (dx * dx + dy2 * dy2) + (dz * dz + dw * dw);
        }
    }
    const double rstd = 1.0 / sqrt(wave_sum(q) / (double)g.cols + g.eps);
#pragma unroll
    for (int i = 0; i < NV; ++i) asm volatile("" : "+v"(v[i]), "+v"(d[i]));
    // g = dy * gamma replaces dy in the registers (rounded to FP32 it would differ from the definition: keep dy,
    // multiply again below)
    double sg = 0.0, sgx = 0.0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        if (c < nvec) {
            const vf4 ga = gamma ? gamma[c] : vf4{1.f, 1.f, 1.f, 1.f};
            const double g0 = (double)d[i].x * (double)ga.x, g1 = (double)d[i].y * (double)ga.y;
            const double g2 = (double)d[i].z * (double)ga.z, g3 = (double)d[i].w * (double)ga.w;
            sg += (g0 + g1) + (g2 + g3);
            sgx += (g0 * (((double)v[i].x - mu) * rstd) + g1 * (((double)v[i].y - mu) * rstd)) +
                   (g2 * (((double)v[i].z - mu) * rstd) + g3 * (((double)v[i].w - mu) * rstd));
        }
    }
    const double mg = wave_sum(sg) / (double)g.cols;
    const double mgx = wave_sum(sgx) / (double)g.cols;
#pragma unroll
    for (int i = 0; i < NV; ++i) asm volatile("" : "+v"(v[i]), "+v"(d[i]));
    vf4* dxp = reinterpret_cast<vf4*>(B.dx + (int64_t)row * g.cols);
    const vf4* addp = B.add ? reinterpret_cast<const vf4*>(B.add + (int64_t)row * g.cols) : nullptr;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * 64 + lane;
        if (c < nvec) {
            const vf4 ga = gamma ? gamma[c] : vf4{1.f, 1.f, 1.f, 1.f};
            const vf4 ad = addp ? addp[c] : vf4{0.f, 0.f, 0.f, 0.f};
            vf4 o;
            o.x = (float)(((double)d[i].x * (double)ga.x - mg - (((double)v[i].x - mu) * rstd) * mgx) * rstd +
                          (double)ad.x);
            o.y = (float)(((double)d[i].y * (double)ga.y - mg - (((double)v[i].y - mu) * rstd) * mgx) * rstd +
                          (double)ad.y);
            o.z = (float)(((double)d[i].z * (double)ga.z - mg - (((double)v[i].z - mu) * rstd) * mgx) * rstd +
                          (double)ad.z);
            o.w = (float)(((double)d[i].w * (double)ga.w - mg - (((double)v[i].w - mu) * rstd) * mgx) * rstd +
                          (double)ad.w);
            dxp[c] = o;
        }
    }
    if (lane == 0) {
        B.stats[2 * (int64_t)row] = mu;
        B.stats[2 * (int64_t)row + 1] = rstd;
    }
}

// One pass over x and dy that gives dx AND the column sums: a workgroup takes a band of a block's rows, RB rows at a
// time, every thread the same columns of each (NV 16-byte vectors, T vectors apart), so a thread's column sums stay
// in its registers (double, rows in ascending order) while the rows' own sums go through LDS.  Every element is read
// once (12 bytes per element with the store, against 20 of the two-kernel form); the bands' sums are added in a
// fixed order by layernorm_bwd_fused_join_f32.
// All four sums over a row are taken in one round, before the statistics exist, about the row's first element p:
//     S1 = sum (x - p),  S2 = sum (x - p)^2,  Sg = sum g,  Sgx = sum g (x - p)       (g = dy * gamma)
//     mu = p + S1 / n,  var = S2 / n - (S1 / n)^2,  mean(g) = Sg / n,  mean(g xhat) = rstd (Sgx - (mu - p) Sg) / n
// in double: p is a sample of the row, so (mu - p)^2 is of the order of var and the subtraction costs a few units
// of 1e-16, where the definition's two-pass form has as much from its own sums.  One barrier per batch; the next
// batch's rows are requested before the current one is worked on.
// cols % 4 == 0, cols / 4 <= T * NV, 16-byte aligned operands.  T threads, grid: x = band, y = block.
template <int NV, int RB, int T>
__global__ __launch_bounds__(T) void layernorm_bwd_fused_f32(const NormBwdGroup g)
{
    constexpr int NW = T / 64;
    __shared__ double part[2][NW][4 * RB];
    // gamma lives in LDS: read from memory inside the loop it would sit behind the next batch's rows in the wave's
    // in-order memory queue, and every batch would wait out that trip to HBM
    __shared__ vf4 gsh[NV * T];
    const NormBwdBlock& B = g.b[blockIdx.y];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nvec = g.cols >> 2;
    const int r_begin = blockIdx.x * g.band_rows, r_end = min(g.rows, r_begin + g.band_rows);
    const vf4* gamma = reinterpret_cast<const vf4*>(B.gamma);
    const double inv_cols = 1.0 / (double)g.cols;
    const vf4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = i * T + tid;
        gsh[c] = (gamma && c < nvec) ? gamma[c] : vf4{1.f, 1.f, 1.f, 1.f};      // (read back by the same thread only)
    }
    double accg[NV][4], accb[NV][4];
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) accg[i][k] = accb[i][k] = 0.0;
    auto fetch = [&](int r0, vf4 (&v)[RB][NV], vf4 (&d)[RB][NV], float (&p)[RB]) {
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const bool row_ok = r0 + j < r_end;
            const vf4* x = reinterpret_cast<const vf4*>(B.x + (int64_t)(r0 + j) * g.cols);
            const vf4* dy = reinterpret_cast<const vf4*>(B.dy + (int64_t)(r0 + j) * g.cols);
            p[j] = row_ok ? B.x[(int64_t)(r0 + j) * g.cols] : 0.f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int c = i * T + tid;
                const bool ok = row_ok && c < nvec;
                v[j][i] = ok ? __builtin_nontemporal_load(x + c) : zero;
                d[j][i] = ok ? __builtin_nontemporal_load(dy + c) : zero;
            }
        }
    };
    vf4 v[RB][NV], d[RB][NV];
    float pv[RB];
    fetch(r_begin, v, d, pv);
    int parity = 0;
    for (int r0 = r_begin; r0 < r_end; r0 += RB, parity ^= 1) {
        // the skip connection's rows of this batch, then the next batch's x and dy: what is needed first is asked first
        vf4 ad[RB][NV];
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const vf4* addp = reinterpret_cast<const vf4*>(B.add + (int64_t)(r0 + j) * g.cols);
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int c = i * T + tid;
                ad[j][i] = (B.add && r0 + j < r_end && c < nvec) ? __builtin_nontemporal_load(addp + c) : zero;
            }
        }
        vf4 vn[RB][NV], dn[RB][NV];
        float pn[RB];
        fetch(r0 + RB, vn, dn, pn);        // (past the band's end: nothing is read)
        double t[4 * RB];
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const double p = (double)pv[j];
            double s1 = 0.0, s2 = 0.0, sg = 0.0, sgx = 0.0;
            int own = tid;      // opaque to the compiler: hoisted out of the loop, gamma would take 4 * NV registers
            asm volatile("" : "+v"(own));
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int c = i * T + tid;
                if (c < nvec) {
                    const vf4 ga = gsh[i * T + own];
                    const double x0 = (double)v[j][i].x - p, x1 = (double)v[j][i].y - p;
                    const double x2 = (double)v[j][i].z - p, x3 = (double)v[j][i].w - p;
                    const double g0 = (double)d[j][i].x * (double)ga.x, g1 = (double)d[j][i].y * (double)ga.y;
                    const double g2 = (double)d[j][i].z * (double)ga.z, g3 = (double)d[j][i].w * (double)ga.w;
                    s1 += (x0 + x1) + (x2 + x3);
                    s2 += (x0 * x0 + x1 * x1) + (x2 * x2 + x3 * x3);
                    sg += (g0 + g1) + (g2 + g3);
                    sgx += (g0 * x0 + g1 * x1) + (g2 * x2 + g3 * x3);
                }
            }
            t[4 * j] = wave_sum(s1);
            t[4 * j + 1] = wave_sum(s2);
            t[4 * j + 2] = wave_sum(sg);
            t[4 * j + 3] = wave_sum(sgx);
        }
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 4 * RB; ++k) part[parity][wave][k] = t[k];
        }
        __syncthreads();    // a place in `part` is written again two batches on, behind the next batch's barrier
#pragma unroll
        for (int k = 0; k < 4 * RB; ++k) {
            double a = part[parity][0][k];
#pragma unroll
            for (int w = 1; w < NW; ++w) a += part[parity][w][k];
            t[k] = a;
        }
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            if (r0 + j < r_end) {
                const double p = (double)pv[j];
                const double m1 = t[4 * j] * inv_cols;                       // mu - p
                const double var = fmax(t[4 * j + 1] * inv_cols - m1 * m1, 0.0);
                const double rstd = 1.0 / sqrt(var + g.eps);
                const double mg = t[4 * j + 2] * inv_cols;
                const double mgx = rstd * (t[4 * j + 3] - m1 * t[4 * j + 2]) * inv_cols;
                const double shift = p + m1;                                 // mu
                vf4* dxp = reinterpret_cast<vf4*>(B.dx + (int64_t)(r0 + j) * g.cols);
                int own = tid;
                asm volatile("" : "+v"(own));
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    const int c = i * T + tid;
                    if (c < nvec) {
                        const vf4 ga = gsh[i * T + own];
                        const float xs[4] = {v[j][i].x, v[j][i].y, v[j][i].z, v[j][i].w};
                        const float ds[4] = {d[j][i].x, d[j][i].y, d[j][i].z, d[j][i].w};
                        const float gs[4] = {ga.x, ga.y, ga.z, ga.w};
                        const float as[4] = {ad[j][i].x, ad[j][i].y, ad[j][i].z, ad[j][i].w};
                        float o[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const double xh = ((double)xs[k] - shift) * rstd;
                            o[k] = (float)(((double)ds[k] * (double)gs[k] - mg - xh * mgx) * rstd + (double)as[k]);
                            accg[i][k] += (double)ds[k] * xh;
                            accb[i][k] += (double)ds[k];
                        }
                        __builtin_nontemporal_store(vf4{o[0], o[1], o[2], o[3]}, dxp + c);
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            pv[j] = pn[j];
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                v[j][i] = vn[j][i];
                d[j][i] = dn[j][i];
            }
        }
    }
    if (g.partial) {
        double* p = g.partial + 2 * ((int64_t)blockIdx.y * g.nbands + blockIdx.x) * g.cols;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int c = i * T + tid;
            if (c < nvec) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    p[2 * (4 * c + k)] = accg[i][k];
                    p[2 * (4 * c + k) + 1] = accb[i][k];
                }
            }
        }
    }
}

template <int NV>
inline void launch_norm_bwd_rows_reg(const NormBwdGroup& g, hipStream_t stream)
{
    dim3 grid((g.rows + NORM_ROWS_PER_WG - 1) / NORM_ROWS_PER_WG, g.nblocks, 1);
    hipLaunchKernelGGL((layernorm_bwd_rows_reg_f32<NV>), grid, dim3(NORM_THREADS), 0, stream, g);
}

constexpr int kNormBwdMaxVectorsPerLane = 17;      // register-resident rows of x and dy: up to 4352 columns

inline bool norm_bwd_rows_fit(const NormBwdGroup& g)
{
    if ((g.cols & 3) || g.cols / 4 > 64 * kNormBwdMaxVectorsPerLane) return false;
    for (int i = 0; i < g.nblocks; ++i) {
        const NormBwdBlock& b = g.b[i];
        if (((uintptr_t)b.x & 15) || ((uintptr_t)b.dy & 15) || ((uintptr_t)b.dx & 15) || ((uintptr_t)b.gamma & 15) ||
            ((uintptr_t)b.add & 15))
            return false;
    }
    return true;
}

struct NormBwdColsOut {
    const float* x[2];       // source blocks stacked by rows (4-way: the two row halves that hold the channel block)
    const float* dy[2];
    const double* stats[2];
    float* dgamma;           // cols sums of dy * xhat, or nullptr
    float* dbeta;            // cols sums of dy, or nullptr
    int nsrc;
    int src_block[2];        // the sources' places in the row kernel's group (where the one-pass kernel left their sums)
};

struct NormBwdColsGroup {
    NormBwdColsOut o[kMaxBlocks];
    int nout;
    int rows, cols;
    // the rows of every source block are cut into `parts` ranges of part_rows (one workgroup per strip and range, as
    // in the bias gradient: a strip per workgroup alone leaves half the chip idle); parts > 1: every workgroup leaves
    // its sums in `partial` (nout x parts x cols pairs of doubles) and layernorm_bwd_cols_join_f32 adds them in order
    int parts, part_rows;
    double* partial;
};

constexpr int NORM_STRIP = 32;            // columns per workgroup of the column kernel
constexpr int NORM_COLS_THREADS = 256;

// grid: x = column strip, y = output (channel block), z = row range.  VEC (cols % 4 == 0, 16-byte aligned sources):
// four columns per thread, 8 lanes across the strip, 32 row lanes; otherwise one column per thread, 8 row lanes.
template <bool VEC>
__global__ __launch_bounds__(NORM_COLS_THREADS) void layernorm_bwd_cols_f32(const NormBwdColsGroup g)
{
    constexpr int LANES = VEC ? NORM_STRIP / 4 : NORM_STRIP;
    constexpr int ROW_LANES = NORM_COLS_THREADS / LANES;
    constexpr int W = VEC ? 4 : 1;
    __shared__ double pg[ROW_LANES][NORM_STRIP + 1], pb[ROW_LANES][NORM_STRIP + 1];
    const NormBwdColsOut& O = g.o[blockIdx.y];
    const int tid = threadIdx.x, cl = tid % LANES, rl = tid / LANES;
    const int col = blockIdx.x * NORM_STRIP + cl * W;
    double sg[4] = {0.0, 0.0, 0.0, 0.0}, sb[4] = {0.0, 0.0, 0.0, 0.0};
    const int r_begin = blockIdx.z * g.part_rows, r_end = min(g.rows, r_begin + g.part_rows);
    if (col < g.cols) {
        for (int b = 0; b < O.nsrc; ++b) {
#pragma unroll 2
            for (int r = r_begin + rl; r < r_end; r += ROW_LANES) {
                const double mu = O.stats[b][2 * (int64_t)r], rstd = O.stats[b][2 * (int64_t)r + 1];
                if (VEC) {
                    const vf4 dv = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(O.dy[b] + (int64_t)r * g.cols + col));
                    const vf4 xv = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(O.x[b] + (int64_t)r * g.cols + col));
                    sg[0] += (double)dv.x * (((double)xv.x - mu) * rstd);
                    sg[1] += (double)dv.y * (((double)xv.y - mu) * rstd);
                    sg[2] += (double)dv.z * (((double)xv.z - mu) * rstd);
                    sg[3] += (double)dv.w * (((double)xv.w - mu) * rstd);
                    sb[0] += (double)dv.x;
                    sb[1] += (double)dv.y;
                    sb[2] += (double)dv.z;
                    sb[3] += (double)dv.w;
                } else {
                    const double d = (double)O.dy[b][(int64_t)r * g.cols + col];
                    sg[0] += d * (((double)O.x[b][(int64_t)r * g.cols + col] - mu) * rstd);
                    sb[0] += d;
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < W; ++q) {
        pg[rl][cl * W + q] = sg[q];
        pb[rl][cl * W + q] = sb[q];
    }
    __syncthreads();
    if (tid < NORM_STRIP) {
        const int c = blockIdx.x * NORM_STRIP + tid;
        if (c < g.cols) {
            double tg = 0.0, tb = 0.0;
#pragma unroll
            for (int r = 0; r < ROW_LANES; ++r) {
                tg += pg[r][tid];
                tb += pb[r][tid];
            }
            if (g.parts > 1) {
                double* p = g.partial + 2 * (((int64_t)blockIdx.y * g.parts + blockIdx.z) * g.cols + c);
                p[0] = tg;
                p[1] = tb;
            } else {
                if (O.dgamma) O.dgamma[c] = (float)tg;
                if (O.dbeta) O.dbeta[c] = (float)tb;
            }
        }
    }
}

// Second stage of the column sums: the parts of column c in ascending order, rounded once.
__global__ __launch_bounds__(NORM_COLS_THREADS) void layernorm_bwd_cols_join_f32(const NormBwdColsGroup g)
{
    const NormBwdColsOut& O = g.o[blockIdx.y];
    const int c = blockIdx.x * NORM_COLS_THREADS + threadIdx.x;
    if (c >= g.cols) return;
    const double* p = g.partial + 2 * ((int64_t)blockIdx.y * g.parts * g.cols + c);
    double tg = 0.0, tb = 0.0;
    for (int k = 0; k < g.parts; ++k) {
        tg += p[2 * (int64_t)k * g.cols];
        tb += p[2 * (int64_t)k * g.cols + 1];
    }
    if (O.dgamma) O.dgamma[c] = (float)tg;
    if (O.dbeta) O.dbeta[c] = (float)tb;
}

// Row ranges of the column kernel and the bytes of their partial sums (0: one range).
inline int norm_col_parts(int rows, int cols, int nout)
{
    const int64_t strips = (int64_t)((cols + NORM_STRIP - 1) / NORM_STRIP) * nout;
    int parts = strips > 0 ? (int)((1024 + strips - 1) / strips) : 1;
    if (parts > rows / 64) parts = rows / 64;
    if (parts > 64) parts = 64;
    return parts < 1 ? 1 : parts;
}
inline size_t norm_cols_workspace_bytes(int rows, int cols, int nout)
{
    const int parts = norm_col_parts(rows, cols, nout);
    return parts > 1 ? (size_t)nout * parts * cols * 2 * sizeof(double) : 0;
}

// Second stage of the one-pass kernel: column c of output o is the sum over its source blocks, in order, and over
// each one's bands, in order - eight interleaved running sums (band k goes to sum k mod 8) added in order at the end.  g.parts = bands
// per block.  grid: x = strip of 32 columns, y = output.
__global__ __launch_bounds__(NORM_COLS_THREADS) void layernorm_bwd_fused_join_f32(const NormBwdColsGroup g)
{
    constexpr int PL = NORM_COLS_THREADS / NORM_STRIP;
    __shared__ double pg[PL][NORM_STRIP + 1], pb[PL][NORM_STRIP + 1];
    const NormBwdColsOut& O = g.o[blockIdx.y];
    const int cl = threadIdx.x % NORM_STRIP, pl = threadIdx.x / NORM_STRIP;
    const int c = blockIdx.x * NORM_STRIP + cl;
    double tg = 0.0, tb = 0.0;
    if (c < g.cols) {
        typedef double vd2 __attribute__((ext_vector_type(2)));
        for (int b = 0; b < O.nsrc; ++b) {
            const vd2* p = reinterpret_cast<const vd2*>(g.partial) + ((int64_t)O.src_block[b] * g.parts * g.cols + c);
#pragma unroll 8
            for (int band = pl; band < g.parts; band += PL) {
                const vd2 q = __builtin_nontemporal_load(p + (int64_t)band * g.cols);
                tg += q.x;
                tb += q.y;
            }
        }
    }
    pg[pl][cl] = tg;
    pb[pl][cl] = tb;
    __syncthreads();
    if (threadIdx.x < NORM_STRIP && c < g.cols) {
        double sg = 0.0, sb = 0.0;
#pragma unroll
        for (int k = 0; k < PL; ++k) {
            sg += pg[k][cl];
            sb += pb[k][cl];
        }
        if (O.dgamma) O.dgamma[c] = (float)sg;
        if (O.dbeta) O.dbeta[c] = (float)sb;
    }
}

// The one-pass kernel's shape.  Three vectors per thread: the column sums (24 registers per vector), the rows of two
// batches and the skip connection's fit a wavefront that shares its SIMD with one other (about 200 registers; rows
// of two at a time, or four vectors per thread, were slower).  The workgroup is as wide as the row needs then, up to
// 512 threads, and there are as many workgroups as the chip holds at once: 8 wavefronts per compute unit.
constexpr int kNormFusedNV = 3;
constexpr int kNormFusedMaxThreads = 512;          // rows of up to 512 * 3 * 4 = 6144 columns
constexpr int kNormFusedCus = 256;
inline int norm_fused_threads(int cols) { return ((cols / 4 + kNormFusedNV - 1) / kNormFusedNV + 63) / 64 * 64; }
inline int norm_fused_band_rows(int rows, int cols, int nblocks)
{
    int wgs = kNormFusedCus * (8 / (norm_fused_threads(cols) / 64));
    if (wgs > 1024) wgs = 1024;
    const int bands = (wgs + nblocks - 1) / nblocks;
    const int per = (rows + bands - 1) / bands;
    return per < 1 ? 1 : per;
}
inline bool norm_fused_fits(int rows, int cols)
{
    return rows > 0 && cols > 0 && (cols & 3) == 0 && norm_fused_threads(cols) <= kNormFusedMaxThreads;
}
inline size_t norm_fused_workspace_bytes(int rows, int cols, int nblocks)
{
    if (!norm_fused_fits(rows, cols) || nblocks <= 0) return 0;
    const int per = norm_fused_band_rows(rows, cols, nblocks);
    return (size_t)nblocks * ((rows + per - 1) / per) * cols * 2 * sizeof(double);
}

template <int T>
inline void launch_norm_bwd_fused(const NormBwdGroup& g, hipStream_t stream)
{
    hipLaunchKernelGGL((layernorm_bwd_fused_f32<kNormFusedNV, 1, T>), dim3(g.nbands, g.nblocks, 1), dim3(T), 0, stream, g);
}

// partial / partial_bytes (may be null): room for the partial column sums - the one-pass kernel's
// (norm_fused_workspace_bytes) when the rows fit it, else the column kernel's (norm_cols_workspace_bytes)
inline hipError_t launch_norm_bwd(const NormBwdGroup& g, NormBwdColsGroup cg, hipStream_t stream, void* partial = nullptr,
                                  size_t partial_bytes = 0)
{
    if (g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    const size_t fused_bytes = norm_fused_workspace_bytes(g.rows, g.cols, g.nblocks);
    if (cg.nout > 0 && fused_bytes > 0 && norm_bwd_rows_fit(g) && partial && partial_bytes >= fused_bytes) {
        NormBwdGroup f = g;
        f.band_rows = norm_fused_band_rows(g.rows, g.cols, g.nblocks);
        f.nbands = (g.rows + f.band_rows - 1) / f.band_rows;
        f.partial = static_cast<double*>(partial);
        switch (norm_fused_threads(g.cols)) {
        case 64: launch_norm_bwd_fused<64>(f, stream); break;
        case 128: launch_norm_bwd_fused<128>(f, stream); break;
        case 192: launch_norm_bwd_fused<192>(f, stream); break;
        case 256: launch_norm_bwd_fused<256>(f, stream); break;
        case 320: launch_norm_bwd_fused<320>(f, stream); break;
        case 384: launch_norm_bwd_fused<384>(f, stream); break;
        case 448: launch_norm_bwd_fused<448>(f, stream); break;
        default: launch_norm_bwd_fused<512>(f, stream); break;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        cg.parts = f.nbands;
        cg.part_rows = f.band_rows;
        cg.partial = f.partial;
        hipLaunchKernelGGL(layernorm_bwd_fused_join_f32, dim3((cg.cols + NORM_STRIP - 1) / NORM_STRIP, cg.nout, 1),
                           dim3(NORM_COLS_THREADS), 0, stream, cg);
        return hipGetLastError();
    }
    if (g.rows > 0 && norm_bwd_rows_fit(g)) {
        const int need = (g.cols / 4 + 63) / 64;      // vectors per lane
        if (need <= 1) launch_norm_bwd_rows_reg<1>(g, stream);
        else if (need <= 2) launch_norm_bwd_rows_reg<2>(g, stream);
        else if (need <= 4) launch_norm_bwd_rows_reg<4>(g, stream);
        else if (need <= 9) launch_norm_bwd_rows_reg<9>(g, stream);
        else launch_norm_bwd_rows_reg<17>(g, stream);
    } else if (g.rows > 0) {
        hipLaunchKernelGGL(layernorm_bwd_rows_f32, dim3(g.rows, g.nblocks, 1), dim3(NORM_THREADS), 0, stream, g);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || cg.nout <= 0) return e;
    bool vec = (cg.cols & 3) == 0;
    for (int i = 0; i < cg.nout; ++i)
        for (int b = 0; b < cg.o[i].nsrc; ++b)
            if (((uintptr_t)cg.o[i].x[b] | (uintptr_t)cg.o[i].dy[b]) & 15) vec = false;
    cg.parts = norm_col_parts(cg.rows, cg.cols, cg.nout);
    if (!partial || partial_bytes < norm_cols_workspace_bytes(cg.rows, cg.cols, cg.nout)) cg.parts = 1;
    cg.part_rows = cg.parts > 1 ? ((cg.rows + cg.parts - 1) / cg.parts + 31) / 32 * 32 : cg.rows;
    if (cg.parts > 1) cg.parts = (cg.rows + cg.part_rows - 1) / cg.part_rows;
    cg.partial = static_cast<double*>(partial);
    const dim3 cgrid((cg.cols + NORM_STRIP - 1) / NORM_STRIP, cg.nout, cg.parts);
    if (vec) hipLaunchKernelGGL(layernorm_bwd_cols_f32<true>, cgrid, dim3(NORM_COLS_THREADS), 0, stream, cg);
    else hipLaunchKernelGGL(layernorm_bwd_cols_f32<false>, cgrid, dim3(NORM_COLS_THREADS), 0, stream, cg);
    if (cg.parts > 1)
        hipLaunchKernelGGL(layernorm_bwd_cols_join_f32, dim3((cg.cols + NORM_COLS_THREADS - 1) / NORM_COLS_THREADS, cg.nout, 1),
                           dim3(NORM_COLS_THREADS), 0, stream, cg);
    return hipGetLastError();
}

template <int NV>
inline void launch_norm_rows(const NormGroup& g, hipStream_t stream)
{
    dim3 grid((g.rows + NORM_ROWS_PER_WG - 1) / NORM_ROWS_PER_WG, g.nblocks, 1);
    hipLaunchKernelGGL((layernorm_rows_f32<NV>), grid, dim3(NORM_THREADS), 0, stream, g);
}

// True when the group asks for bfloat16 copies.
inline bool norm_wants_copies(const NormGroup& g)
{
    for (int i = 0; i < g.nblocks; ++i)
        if (g.b[i].y16) return true;
    return false;
}

// True when the register-resident kernel can take the group.
inline bool norm_rows_fit(const NormGroup& g)
{
    if ((g.cols & 3) || g.cols / 4 > 64 * kNormMaxVectorsPerLane) return false;
    for (int i = 0; i < g.nblocks; ++i) {
        const NormBlock& b = g.b[i];
        if (((uintptr_t)b.x & 15) || ((uintptr_t)b.y & 15) || ((uintptr_t)b.gamma & 15) || ((uintptr_t)b.beta & 15) ||
            ((uintptr_t)b.xb & 15))
            return false;
    }
    return true;
}

// A group with bfloat16 copies must fit the register-resident kernel (the caller checks norm_rows_fit and
// converts separately otherwise); the copies must be 8-byte aligned with plane16 a multiple of 4.
inline hipError_t launch_norm_group(const NormGroup& g, hipStream_t stream)
{
    if (g.rows <= 0 || g.cols <= 0 || g.nblocks <= 0) return hipSuccess;
    if (norm_wants_copies(g)) {
        if (!norm_rows_fit(g) || (g.plane16 & 3) || g.plane16 < g.cols || (g.planes16 != 1 && g.planes16 != 2))
            return hipErrorInvalidValue;
        for (int i = 0; i < g.nblocks; ++i)
            if ((uintptr_t)g.b[i].y16 & 7) return hipErrorInvalidValue;
    }
    if (norm_rows_fit(g)) {
        const int need = (g.cols / 4 + 63) / 64;      // vectors per lane
        if (need <= 1) launch_norm_rows<1>(g, stream);
        else if (need <= 2) launch_norm_rows<2>(g, stream);
        else if (need <= 4) launch_norm_rows<4>(g, stream);
        else if (need <= 6) launch_norm_rows<6>(g, stream);
        else if (need <= 9) launch_norm_rows<9>(g, stream);
        else if (need <= 12) launch_norm_rows<12>(g, stream);
        else if (need <= 17) launch_norm_rows<17>(g, stream);
        else if (need <= 24) launch_norm_rows<24>(g, stream);
        else launch_norm_rows<32>(g, stream);
    } else {
        hipLaunchKernelGGL(layernorm_generic_f32, dim3(g.rows, g.nblocks, 1), dim3(NORM_THREADS), 0, stream, g);
    }
    return hipGetLastError();
}

}  // namespace jg

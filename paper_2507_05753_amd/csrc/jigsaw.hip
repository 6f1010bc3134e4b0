// C-ABI layer of libjigsaw (see include/jigsaw.h): argument checking, the block
// decomposition of Sec. 4.1 / 4.2, workspace layout, and kernel launches.
// No device memory is allocated here and nothing synchronises except jg_profile_read.
#include "../../include/jigsaw.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "gemm_f32.hpp"
#include "stream_kernels.hpp"
#include "patch_kernels.hpp"
#include "norm_kernels.hpp"
#include "reduce_kernels.hpp"
#include "act_kernels.hpp"
#include "gemm_bf16.hpp"
#include "cvt_kernels.hpp"

// Workspace of jg_linear_forward_static: a fixed array in the code object's own device memory, so that the call
// needs no allocation by anyone.  Every GPU the library is used on holds its own copy at its own address until
// the process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels get the device
// address kept in g_scratch_ptr[device].
constexpr size_t kStaticScratchBytes = (size_t)JG_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Last failing HIP call of this host thread, for jg_last_hip_error().
thread_local char g_hip_detail[160] = "no HIP error recorded";

bool hip_ok(hipError_t e, const char* what)
{
    if (e == hipSuccess) return true;
    std::snprintf(g_hip_detail, sizeof(g_hip_detail), "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
    (void)hipGetLastError();   // clear the sticky per-thread error
    return false;
}
#define HIP_OK(call) hip_ok((call), #call)

// Makes `device` the calling thread's current one; a thread that already is on it (every call after a context's
// first, in the usual program) pays a thread-local read instead of a trip into the runtime's device switch.
static hipError_t use_device(int device)
{
    int cur = -1;
    if (hipGetDevice(&cur) == hipSuccess && cur == device) return hipSuccess;
    return hipSetDevice(device);
}

constexpr int kProfileMaxLaunches = 8192;
constexpr int64_t kMaxDim = 0x7fffffff - 1024;   // every dimension fits an int with tile slack
constexpr int kDefaultSlots = 512;               // MI355X: 256 CUs x 2 resident GEMM workgroups (plans made without a context)
constexpr size_t kWsAlign = 256;

struct TimedLaunch {
    hipEvent_t start, stop;
    int kernel;
};

}  // namespace

struct jg_ctx {
    int device;
    int slots;                           // workgroups of the GEMM kernel the device holds at once (2 per CU)
    hipStream_t stream;
    void* static_ws;                     // device address of this device's static workspace (nullptr: device index too high)
    bool profiling;
    std::vector<hipEvent_t> pool;        // created on first jg_profile(ctx, 1)
    size_t pool_used;
    std::vector<TimedLaunch> timed;
    std::vector<jg_plan*> plans;         // the live plans made with this context: jg_free detaches them
    bool hb_reverse = false;             // tile order of the last bfloat16 launch (see run_gemm)
};

struct jg_plan {
    jg_ctx* ctx;
    jg_linear_desc d;
    // per-rank shard shapes
    int64_t xr, xc, wr, wc, yr, yc;
    // 4-byte units in one row of an X or W shard: xc for FP32, xc / 2 for bfloat16, xc for the
    // split mode's [hi | lo] rows
    int64_t xcp;
    int64_t plane;   // reduced precision: bfloat16 elements per plane of a shard row = xc rounded up to 64
    // workspace layout (byte offsets); sizes are per rank
    size_t part_bytes;     // one rank's partial product  (yr x yc floats, padded)
    size_t wblk_bytes;     // one rank's received weight block (4-way, copy mode)
    size_t off_send;       // ways x part_bytes: partial products handed to the peer
    size_t off_kept;       // ways x part_bytes: kept products (separate combine only)
    size_t off_wrecv;      // ways x wblk_bytes
    size_t ws_bytes;
    // backward workspace: ways partials of dX blocks, then (4-way) ways partials of dW blocks
    size_t bw_dx_bytes, bw_dw_bytes, bw_off_dw, bw_ws_bytes;
    size_t bw_off_cvt;   // reduced-precision backward: where the rounded operands start in the backward workspace
    // scratch tiles of the split tail (largest need over the pass's launches), at the end of each workspace
    int slots;
    size_t tail_bytes, off_tail, bw_tail_bytes, bw_off_tail;
    // reduced precision, as a layer of an MLP chain: the FP32 input activations are converted into ways shards of
    // chain_shard_bytes each, behind the layer's own workspace
    size_t chain_shard_bytes, chain_bytes;
    // JG_OP_XW: the activation block a rank receives (copy mode), next to the weight block of off_wrecv
    size_t xblk_bytes, off_xrecv;
    // JG_OP_XW: its gradients are the other two permutations, dX = dY W^T (an X W^T layer on dY and W) and
    // dW = X^T dY (an X^T W layer on X and dY); the plans of those two layers, owned by this plan
    jg_plan* bw_dx_plan;
    jg_plan* bw_dw_plan;
};

namespace {

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// 4-way roles (Sec. 4.2, Eq. (4)).  A term printed bold as a whole product is formed
// on the rank that holds its X block and shipped; where only W^T is bold the weight
// block is shipped to the rank holding the X block.
//   rank 0: X0 W0^T keep            X0 W2^T (W2 from rank 2) -> rank 1
//   rank 1: X1 W1^T -> rank 0       X1 W3^T (W3 from rank 3) keep
//   rank 2: X2 W2^T -> rank 3       X2 W0^T (W0 from rank 0) keep
//   rank 3: X3 W3^T keep            X3 W1^T (W1 from rank 1) -> rank 2
constexpr int kWeightFrom4[4] = {2, 3, 0, 1};
constexpr int kOwnIsKept4[4] = {1, 0, 0, 1};
constexpr int kPeer4[4] = {1, 0, 3, 2};

struct ScopedTimer {
    jg_ctx* c;
    int kernel;
    hipEvent_t stop;
    bool on;
    ScopedTimer(jg_ctx* ctx, int k) : c(ctx), kernel(k), stop(nullptr), on(false)
    {
        if (c->profiling && c->pool_used + 2 <= c->pool.size()) {
            hipEvent_t start = c->pool[c->pool_used++];
            stop = c->pool[c->pool_used++];
            if (hipEventRecord(start, c->stream) == hipSuccess) {
                c->timed.push_back({start, stop, kernel});
                on = true;
            }
        }
    }
    ~ScopedTimer()
    {
        if (on) (void)hipEventRecord(stop, c->stream);
    }
};

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

int check_ptr_array(const float* const* arr, int n)
{
    if (!arr) return JG_E_NULL;
    for (int i = 0; i < n; ++i) {
        if (!arr[i]) return JG_E_NULL;
        if (!aligned(arr[i], 4)) return JG_E_ALIGN;
    }
    return JG_OK;
}

}  // namespace

extern "C" {

const char* jg_last_hip_error(void) { return g_hip_detail; }

const char* jg_strerror(int status)
{
    switch (status) {
    case JG_OK: return "ok";
    case JG_E_NULL: return "required pointer is NULL";
    case JG_E_SHAPE: return "bad shape: non-positive, too large, or not divisible as `ways` requires";
    case JG_E_WAYS: return "ways must be 1, 2 or 4 and rank must be in [0, ways)";
    case JG_E_DTYPE: return "unsupported dtype, op or option value";
    case JG_E_WORKSPACE: return "workspace missing or too small";
    case JG_E_ALIGN: return "misaligned device pointer";
    case JG_E_HIP: return "HIP runtime call failed";
    case JG_E_ARCH: return "device is not gfx950";
    default: return "unknown status";
    }
}

int jg_init(jg_ctx** out, int device, void* hip_stream)
{
    if (!out) return JG_E_NULL;
    *out = nullptr;
    int count = 0;
    if (!HIP_OK(hipGetDeviceCount(&count))) return JG_E_HIP;
    if (device < 0 || device >= count) {
        std::snprintf(g_hip_detail, sizeof(g_hip_detail), "device %d out of range (%d visible)", device, count);
        return JG_E_HIP;
    }
    hipDeviceProp_t prop;
    if (!HIP_OK(hipGetDeviceProperties(&prop, device))) return JG_E_HIP;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return JG_E_ARCH;
    if (!HIP_OK(hipSetDevice(device))) return JG_E_HIP;
    void* static_ws = nullptr;
    if (device < kMaxDevices) {
        // this device's copy of the static workspace: looked up once, with the device current
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[device]) {
            void* ptr = nullptr;
            if (!HIP_OK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)))) return JG_E_HIP;
            g_scratch_ptr[device] = ptr;
        }
        static_ws = g_scratch_ptr[device];
    }
    jg_ctx* c = new (std::nothrow) jg_ctx();
    if (!c) return JG_E_HIP;
    c->device = device;
    c->static_ws = static_ws;
    c->slots = 2 * prop.multiProcessorCount;
    c->stream = (hipStream_t)hip_stream;
    c->profiling = false;
    c->pool_used = 0;
    *out = c;
    return JG_OK;
}

void jg_free(jg_ctx* ctx)
{
    if (!ctx) return;
    (void)use_device(ctx->device);
    for (hipEvent_t e : ctx->pool) (void)hipEventDestroy(e);
    for (jg_plan* p : ctx->plans) p->ctx = nullptr;     // surviving plans answer queries only from now on
    delete ctx;
}

int jg_profile(jg_ctx* ctx, int enable)
{
    if (!ctx) return JG_E_NULL;
    if (!HIP_OK(use_device(ctx->device))) return JG_E_HIP;
    if (enable && ctx->pool.empty()) {
        ctx->pool.reserve(2 * kProfileMaxLaunches);
        ctx->timed.reserve(kProfileMaxLaunches);
        for (int i = 0; i < 2 * kProfileMaxLaunches; ++i) {
            hipEvent_t e;
            if (!HIP_OK(hipEventCreate(&e))) return JG_E_HIP;
            ctx->pool.push_back(e);
        }
    }
    ctx->profiling = enable != 0;
    return JG_OK;
}

int jg_profile_read(jg_ctx* ctx, int kernel, double* total_ms, int64_t* launches)
{
    if (!ctx || !total_ms || !launches) return JG_E_NULL;
    if (kernel < 0 || kernel >= JG_KERNEL_COUNT) return JG_E_DTYPE;
    if (!HIP_OK(use_device(ctx->device))) return JG_E_HIP;
    if (!HIP_OK(hipStreamSynchronize(ctx->stream))) return JG_E_HIP;
    double sum = 0.0;
    int64_t n = 0;
    std::vector<TimedLaunch> rest;
    rest.reserve(ctx->timed.size());
    for (const TimedLaunch& t : ctx->timed) {
        if (t.kernel != kernel) {
            rest.push_back(t);
            continue;
        }
        float ms = 0.f;
        if (!HIP_OK(hipEventElapsedTime(&ms, t.start, t.stop))) return JG_E_HIP;
        sum += ms;
        ++n;
    }
    ctx->timed.swap(rest);
    if (ctx->timed.empty()) ctx->pool_used = 0;   // every pair has been read: reuse the pool
    *total_ms = sum;
    *launches = n;
    return JG_OK;
}

// Reduced-precision backward of the plain layer: the rounded operands in the backward workspace, from bw_off_cvt on.
// dY_r twice (rows of the contracted N share for dX, contraction-major over the tokens for dW), every weight block
// and X_r contraction-major.  Sizes in bytes per shard / block, each rounded up to 256.
struct BwReduced {
    int planes, plane_n, plane_m, ld_n, ld_m, wblocks;
    size_t dy16, dy16t, w16t, x16t, off_dy16, off_dy16t, off_w16t, off_x16t, total;
};

static BwReduced bw_reduced_layout(const jg_plan* p)
{
    BwReduced L;
    const int ways = p->d.ways;
    L.planes = p->d.dtype == JG_BF16X3 ? 2 : 1;
    L.plane_n = (int)((p->yc + 63) / 64 * 64);      // contraction over the rank's share of N (dX)
    L.plane_m = (int)((p->xr + 63) / 64 * 64);      // contraction over the rank's tokens (dW)
    L.ld_n = L.planes == 2 ? L.plane_n : L.plane_n / 2;     // row strides in 4-byte units
    L.ld_m = L.planes == 2 ? L.plane_m : L.plane_m / 2;
    L.wblocks = ways == 2 ? 2 : 1;                  // weight blocks in a rank's shard
    L.dy16 = round_up(4 * (size_t)p->yr * L.ld_n, kWsAlign);
    L.dy16t = round_up(4 * (size_t)p->yc * L.ld_m, kWsAlign);
    L.w16t = round_up(4 * (size_t)p->xc * L.ld_n, kWsAlign);
    L.x16t = round_up(4 * (size_t)p->xc * L.ld_m, kWsAlign);
    L.off_dy16 = p->bw_off_cvt;
    L.off_dy16t = L.off_dy16 + L.dy16 * ways;
    L.off_w16t = L.off_dy16t + L.dy16t * ways;
    L.off_x16t = L.off_w16t + L.w16t * ways * L.wblocks;
    L.total = L.off_x16t + L.x16t * ways - p->bw_off_cvt;
    return L;
}

// The same for the transposed layer Y = X^T W (X_r tokens x channels, W_r tokens x columns, dY_r channels x columns):
// dX = W dY^T contracts over the columns (W_r and dY_r rounded as they are), dW = X dY over the channels (X_r rounded
// as it is, every channels x columns block of dY_r contraction-major).
struct BwReducedXtw {
    int planes, plane_d, plane_c, ld_d, ld_c, yblocks;
    size_t w16, dy16, x16, dy16t, off_w16, off_dy16, off_x16, off_dy16t, total;
};

static BwReducedXtw bw_reduced_xtw_layout(const jg_plan* p)
{
    BwReducedXtw L;
    const int ways = p->d.ways;
    L.planes = p->d.dtype == JG_BF16X3 ? 2 : 1;
    L.plane_d = (int)((p->wc + 63) / 64 * 64);      // contraction over the rank's share of the columns (dX)
    L.plane_c = (int)((p->xc + 63) / 64 * 64);      // contraction over the rank's share of the channels (dW)
    L.ld_d = L.planes == 2 ? L.plane_d : L.plane_d / 2;
    L.ld_c = L.planes == 2 ? L.plane_c : L.plane_c / 2;
    L.yblocks = ways == 2 ? 2 : 1;                  // channels x columns blocks stacked in a rank's dY shard
    L.w16 = round_up(4 * (size_t)p->wr * L.ld_d, kWsAlign);
    L.dy16 = round_up(4 * (size_t)p->yr * L.ld_d, kWsAlign);
    L.x16 = round_up(4 * (size_t)p->xr * L.ld_c, kWsAlign);
    L.dy16t = round_up(4 * (size_t)p->wc * L.ld_c, kWsAlign);       // one block: columns x channels
    L.off_w16 = p->bw_off_cvt;
    L.off_dy16 = L.off_w16 + L.w16 * ways;
    L.off_x16 = L.off_dy16 + L.dy16 * ways;
    L.off_dy16t = L.off_x16 + L.x16 * ways;
    L.total = L.off_dy16t + L.dy16t * ways * L.yblocks - p->bw_off_cvt;
    return L;
}

int jg_plan_create(jg_ctx* ctx, const jg_linear_desc* desc, jg_plan** out)
{
    if (!out) return JG_E_NULL;
    *out = nullptr;
    if (!desc) return JG_E_NULL;
    const jg_linear_desc& d = *desc;
    if (d.ways != 1 && d.ways != 2 && d.ways != 4) return JG_E_WAYS;
    if (d.op != JG_OP_XWT && d.op != JG_OP_XTW && d.op != JG_OP_XW) return JG_E_DTYPE;
    if (d.dtype != JG_F32 && d.dtype != JG_BF16 && d.dtype != JG_BF16X3) return JG_E_DTYPE;
    const bool reduced = d.dtype != JG_F32;
    if (d.op == JG_OP_XW && reduced) return JG_E_DTYPE;     // the X W permutation exists in FP32 only
    if (d.combine != JG_COMBINE_FUSED && d.combine != JG_COMBINE_SEPARATE) return JG_E_DTYPE;
    if (d.weights != JG_WEIGHTS_COPY && d.weights != JG_WEIGHTS_DIRECT) return JG_E_DTYPE;
    if (d.has_bias != 0 && d.has_bias != 1) return JG_E_DTYPE;
    if (d.tail != JG_TAIL_SPLIT && d.tail != JG_TAIL_WHOLE) return JG_E_DTYPE;
    if (d.accumulate != JG_ACC_LEVELS && d.accumulate != JG_ACC_SINGLE) return JG_E_DTYPE;
    if (d.M <= 0 || d.K <= 0 || d.N <= 0) return JG_E_SHAPE;
    if (d.M > kMaxDim || d.K > kMaxDim || d.N > kMaxDim) return JG_E_SHAPE;
    // the dimensions that are halved: X W^T splits K (2-way) and M, K (4-way); X^T W splits M and K, M
    const bool xtw = d.op == JG_OP_XTW;
    if (d.ways >= 2 && ((xtw ? d.M & 1 : d.K & 1) || (d.N & 1))) return JG_E_SHAPE;
    if (d.ways == 4 && ((d.M & 1) || (d.K & 1))) return JG_E_SHAPE;
    // bfloat16 shards move in 16-byte chunks of 8 elements: a rank's share of K must be whole chunks
    // (the transposed layer's shard step pads its contraction-major rows with zeros instead: any K)
    if (reduced && !xtw && ((d.K / (d.ways >= 2 ? 2 : 1)) & 7)) return JG_E_SHAPE;
    {   // every product of the plan (forward M x N, backward M x K and N x K, up to four
        // problems a launch) must have a tile count that fits the 32-bit block index
        const int64_t tm = (d.M + jg::BM - 1) / jg::BM, tn = (d.N + jg::BM - 1) / jg::BM,
                      tk = (d.K + jg::BM - 1) / jg::BM;
        const int64_t limit = (0x7fffffffLL - 64) / 4;
        if (tm * tn > limit || tm * tk > limit || tn * tk > limit) return JG_E_SHAPE;
    }

    jg_plan* p = new (std::nothrow) jg_plan();
    if (!p) return JG_E_HIP;
    p->ctx = ctx;
    p->d = d;
    p->xblk_bytes = p->off_xrecv = 0;
    p->bw_dx_plan = p->bw_dw_plan = nullptr;
    const bool xw = d.op == JG_OP_XW;
    if (xw) {
        // X is M x K, W is K x N, Y is M x N; all split on the last dimension (2-way) or 2 x 2; in the 2-way
        // form a rank holds all K rows of its column half of W
        const int64_t rows = d.ways == 4 ? 2 : 1, cols = d.ways >= 2 ? 2 : 1;
        p->xr = d.M / rows; p->xc = d.K / cols;
        p->wr = d.ways == 4 ? d.K / 2 : d.K; p->wc = d.N / cols;
        p->yr = d.M / rows; p->yc = d.N / cols;
    } else if (xtw) {
        // X is K x M, W is K x N, Y is M x N; all split on the last dimension (2-way) or 2 x 2
        const int64_t rows = d.ways == 4 ? 2 : 1, cols = d.ways >= 2 ? 2 : 1;
        p->xr = d.K / rows; p->xc = d.M / cols;
        p->wr = d.K / rows; p->wc = d.N / cols;
        p->yr = d.M / rows; p->yc = d.N / cols;
    } else {
        switch (d.ways) {
        case 1:
            p->xr = d.M; p->xc = d.K; p->wr = d.N; p->wc = d.K; p->yr = d.M; p->yc = d.N;
            break;
        case 2:   // Sec. 4.1: channel (last) dimension halved; W_r keeps all N rows
            p->xr = d.M; p->xc = d.K / 2; p->wr = d.N; p->wc = d.K / 2; p->yr = d.M; p->yc = d.N / 2;
            break;
        default:  // Sec. 4.2: 2 x 2 blocks
            p->xr = d.M / 2; p->xc = d.K / 2; p->wr = d.N / 2; p->wc = d.K / 2;
            p->yr = d.M / 2; p->yc = d.N / 2;
            break;
        }
    }
    // bfloat16 shard rows are padded to whole 128-byte lines per plane
    // (the transposed layer's reduced-precision shards are stored contraction-major: X_r as xc rows of xr elements)
    p->plane = reduced ? ((xtw ? p->xr : p->xc) + 63) / 64 * 64 : p->xc;
    p->xcp = d.dtype == JG_BF16 ? p->plane / 2 : d.dtype == JG_BF16X3 ? p->plane : p->xc;
    p->part_bytes = p->wblk_bytes = 0;
    p->off_send = p->off_kept = p->off_wrecv = 0;
    size_t off = 0;
    // partial products are handed over wherever the contraction is split across ranks; an operand
    // block comes from a peer in the 4-way X W^T layer (a weight block) and in the 2- and 4-way
    // X^T W layer (an activation block)
    // (X W: both products of an output block are formed by its owner, the first into a partial of its own; the
    // activation block comes from the row neighbour, 4-way also a weight block from the column neighbour)
    const bool partials = xtw ? d.ways == 4 : d.ways >= 2;
    const bool operand_blocks = (xtw ? d.ways >= 2 : d.ways == 4) && d.weights == JG_WEIGHTS_COPY;
    if (xw && d.ways >= 2 && d.weights == JG_WEIGHTS_COPY) {
        p->xblk_bytes = round_up((size_t)p->xr * (size_t)p->xc * sizeof(float), kWsAlign);
        p->off_xrecv = off;
        off += p->xblk_bytes * d.ways;
    }
    if (partials) {
        p->part_bytes = round_up((size_t)p->yr * (size_t)p->yc * sizeof(float), kWsAlign);
        p->off_send = off;
        off += p->part_bytes * d.ways;
        if (d.combine == JG_COMBINE_SEPARATE) {
            p->off_kept = off;
            off += p->part_bytes * d.ways;
        }
    }
    if (operand_blocks) {
        const size_t elems = xtw  ? (reduced ? (size_t)p->xc * (size_t)p->xcp : (size_t)p->xr * (size_t)p->xc)
                             : xw ? (size_t)p->wr * (size_t)p->wc
                                  : (size_t)p->wr * (size_t)p->xcp;
        p->wblk_bytes = round_up(elems * sizeof(float), kWsAlign);
        p->off_wrecv = off;
        off += p->wblk_bytes * d.ways;
    }
    p->ws_bytes = off;
    p->bw_dx_bytes = p->bw_dw_bytes = p->bw_off_dw = p->bw_ws_bytes = 0;
    if (d.ways >= 2) {
        // one partial per rank for dX and (wherever dW sums two terms: 4-way, and the 2-way transposed layer) for dW
        p->bw_dx_bytes = round_up((size_t)p->xr * (size_t)p->xc * sizeof(float), kWsAlign);
        p->bw_off_dw = p->bw_dx_bytes * d.ways;
        p->bw_ws_bytes = p->bw_off_dw;
        if (d.ways == 4 || xtw) {
            p->bw_dw_bytes = round_up((size_t)p->wr * (size_t)p->wc * sizeof(float), kWsAlign);
            p->bw_ws_bytes += p->bw_dw_bytes * d.ways;
        }
    }
    // scratch for the split tail: the largest need over the launches of each pass
    p->slots = ctx ? ctx->slots : kDefaultSlots;
    p->tail_bytes = p->bw_tail_bytes = 0;
    if (d.tail == JG_TAIL_SPLIT && reduced) {
        // one 256 x 256 scratch tile per CU, when the launches of the pass can end in a partial round worth splitting
        p->tail_bytes = jg::bf16_tail_scratch_bytes(p->slots / 2);
        p->bw_tail_bytes = p->tail_bytes;
    } else if (d.tail == JG_TAIL_SPLIT) {
        auto need = [&](int nprob, int64_t m, int64_t n, int64_t k) {
            const int64_t tiles = nprob * ((m + jg::BM - 1) / jg::BM) * ((n + jg::BN - 1) / jg::BN);
            return jg::tail_scratch_bytes(tiles, (int)k, p->slots);
        };
        if (xtw) {
            p->tail_bytes = need(d.ways == 1 ? 1 : 4, p->xc, p->wc, p->xr);
            const size_t dx = need(d.ways, p->xr, p->xc, p->wc);
            const size_t dw = need(d.ways, p->xr, p->wc, p->xc);
            p->bw_tail_bytes = dx > dw ? dx : dw;
        } else {
            p->tail_bytes = need(d.ways, p->yr, p->yc, p->xc);
            const size_t dx = need(d.ways, p->xr, p->xc, p->yc);
            const size_t dw = need(d.ways == 1 ? 1 : 4, p->yc, p->xc, p->xr);
            p->bw_tail_bytes = dx > dw ? dx : dw;
        }
    }
    p->off_tail = p->ws_bytes;
    p->ws_bytes += p->tail_bytes;
    p->bw_off_cvt = p->bw_ws_bytes;
    if (reduced) p->bw_ws_bytes += xtw ? bw_reduced_xtw_layout(p).total : bw_reduced_layout(p).total;
    p->bw_off_tail = p->bw_ws_bytes;
    p->bw_ws_bytes += p->bw_tail_bytes;
    p->ws_bytes = round_up(p->ws_bytes, kWsAlign);
    p->chain_shard_bytes = reduced ? round_up(4 * (size_t)(xtw ? p->xc : p->xr) * (size_t)p->xcp, kWsAlign) : 0;
    p->chain_bytes = p->chain_shard_bytes * d.ways;
    if (xw) {
        jg_linear_desc dx = d, dw = d;
        dx.op = JG_OP_XWT; dx.M = d.M; dx.K = d.N; dx.N = d.K; dx.has_bias = 0; dx.combine = JG_COMBINE_FUSED;
        dw.op = JG_OP_XTW; dw.K = d.M; dw.M = d.K; dw.N = d.N; dw.has_bias = 0; dw.combine = JG_COMBINE_FUSED;
        int rc = jg_plan_create(ctx, &dx, &p->bw_dx_plan);
        if (rc == JG_OK) rc = jg_plan_create(ctx, &dw, &p->bw_dw_plan);
        if (rc != JG_OK) {
            jg_plan_destroy(p);
            return rc;
        }
        p->bw_ws_bytes = p->bw_dx_plan->ws_bytes > p->bw_dw_plan->ws_bytes ? p->bw_dx_plan->ws_bytes
                                                                           : p->bw_dw_plan->ws_bytes;
        p->bw_tail_bytes = p->bw_dx_plan->tail_bytes > p->bw_dw_plan->tail_bytes ? p->bw_dx_plan->tail_bytes
                                                                                 : p->bw_dw_plan->tail_bytes;
    }
    if (ctx) ctx->plans.push_back(p);
    *out = p;
    return JG_OK;
}

void jg_plan_destroy(jg_plan* plan)
{
    if (!plan) return;
    jg_plan_destroy(plan->bw_dx_plan);
    jg_plan_destroy(plan->bw_dw_plan);
    if (plan->ctx) {
        std::vector<jg_plan*>& live = plan->ctx->plans;
        for (size_t i = 0; i < live.size(); ++i)
            if (live[i] == plan) {
                live[i] = live.back();
                live.pop_back();
                break;
            }
    }
    delete plan;
}

int jg_plan_query(const jg_plan* plan, int what, int rank, int64_t* out)
{
    if (!plan || !out) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    const bool per_rank = what == JG_Q_FLOPS_RANK || what == JG_Q_EXCHANGE_BYTES_RANK ||
                          (what >= JG_Q_X_ROWS && what <= JG_Q_RESIDENT_BYTES_RANK) ||
                          what == JG_Q_X_SHARD_BYTES || what == JG_Q_W_SHARD_BYTES;
    if (per_rank && (rank < 0 || rank >= d.ways)) return JG_E_WAYS;
    const int64_t M = d.M, K = d.K, N = d.N;
    const bool xtw = d.op == JG_OP_XTW;
    const bool reduced = d.dtype != JG_F32;
    const int64_t eb = d.dtype == JG_BF16 ? 2 : 4;     // bytes per element of an X or W shard (split mode: hi + lo)
    switch (what) {
    case JG_Q_WORKSPACE_BYTES: *out = (int64_t)plan->ws_bytes; break;
    case JG_Q_FLOPS_TOTAL: *out = 2 * M * K * N; break;
    case JG_Q_FLOPS_RANK: *out = 2 * M * K * N / d.ways; break;
    case JG_Q_HBM_BYTES_ALGO:
        *out = eb * (M * K + N * K) + 4 * M * N + ((xtw ? d.ways == 4 : d.ways >= 2) ? 8 * M * N : 0);
        break;
    case JG_Q_EXCHANGE_BYTES_RANK:
        if (d.op == JG_OP_XW) {
            // 2-way: one M x K/2 activation block.  4-way: one M/2 x K/2 activation block and one K/2 x N/2
            // weight block.
            *out = d.ways == 1 ? 0
                 : d.ways == 2 ? 4 * M * (K / 2)
                               : 4 * ((M / 2) * (K / 2) + (K / 2) * (N / 2));
            break;
        }
        if (xtw) {
            // 2-way: one K x M/2 activation block.  4-way: one M/2 x N/2 partial and one K/2 x M/2
            // activation block.
            *out = d.ways == 1 ? 0
                 : d.ways == 2 ? 4 * K * (M / 2)
                               : 4 * ((M / 2) * (N / 2) + (K / 2) * (M / 2));
            break;
        }
        // 2-way: one M x N/2 partial.  4-way: one M/2 x N/2 partial and one N/2 x K/2 weight block.
        *out = d.ways == 1 ? 0
             : d.ways == 2 ? 4 * M * (N / 2)
                           : 4 * (M / 2) * (N / 2) + eb * (N / 2) * (K / 2);
        break;
    case JG_Q_X_ROWS: *out = plan->xr; break;
    case JG_Q_X_COLS: *out = plan->xc; break;
    case JG_Q_W_ROWS: *out = plan->wr; break;
    case JG_Q_W_COLS: *out = plan->wc; break;
    case JG_Q_Y_ROWS: *out = plan->yr; break;
    case JG_Q_Y_COLS: *out = plan->yc; break;
    case JG_Q_B_LEN: *out = plan->yc; break;
    case JG_Q_RESIDENT_BYTES_RANK:
        *out = eb * (plan->xr * plan->xc + plan->wr * plan->wc) + 4 * plan->yr * plan->yc;
        break;
    case JG_Q_GEMM_LAUNCHES: {
        // block-product launches per forward; a reduced-precision product takes one launch per chunk of its contraction
        int64_t chunks = 1;
        if (reduced && d.accumulate != JG_ACC_SINGLE) {
            int kk = (int)(xtw ? plan->xr : plan->xc);
            if (xtw) kk = (kk + 7) / 8 * 8;
            const int ck = jg::bf16_chunk_k(kk, d.dtype == JG_BF16X3 ? 3 : 1);
            chunks = (kk + ck - 1) / ck;
        }
        *out = ((d.ways == 1 || (xtw && d.ways == 2)) ? 1 : 2) * chunks;
        break;
    }
    case JG_Q_BACKWARD_WORKSPACE_BYTES: *out = (int64_t)plan->bw_ws_bytes; break;
    case JG_Q_BACKWARD_FLOPS_TOTAL: *out = 4 * M * K * N; break;
    case JG_Q_BACKWARD_GEMM_LAUNCHES: *out = d.ways == 1 ? 2 : (d.ways == 2 && !xtw) ? 3 : 4; break;
    case JG_Q_TAIL_SCRATCH_BYTES: *out = (int64_t)plan->tail_bytes; break;
    case JG_Q_BACKWARD_TAIL_SCRATCH_BYTES: *out = (int64_t)plan->bw_tail_bytes; break;
    case JG_Q_X_SHARD_BYTES: *out = 4 * ((xtw && reduced) ? plan->xc : plan->xr) * plan->xcp; break;
    case JG_Q_W_SHARD_BYTES:
        *out = d.op == JG_OP_XW ? 4 * plan->wr * plan->wc : 4 * ((xtw && reduced) ? plan->wc : plan->wr) * plan->xcp;
        break;
    case JG_Q_CHAIN_WORKSPACE_BYTES: *out = (int64_t)(plan->ws_bytes + plan->chain_bytes); break;
    case JG_Q_NORM_BACKWARD_WORKSPACE_BYTES:
        // mean and 1 / sqrt(var + eps) of every row (the two-kernel form), then the partial column sums of whichever
        // form runs
        *out = (int64_t)(round_up(16 * (size_t)plan->xr, kWsAlign) * d.ways +
                         std::max(jg::norm_cols_workspace_bytes((int)plan->xr, (int)plan->xc, d.ways == 4 ? 2 : d.ways),
                                  jg::norm_fused_workspace_bytes((int)plan->xr, (int)plan->xc, d.ways)));
        break;
    case JG_Q_BIAS_BACKWARD_WORKSPACE_BYTES:
        *out = (int64_t)jg::colsum_workspace_bytes((int)plan->yr, (int)plan->yc, d.ways == 4 ? 2 : d.ways);
        break;
    case JG_Q_X_F32_SHARDS_BYTES:
        *out = (int64_t)(round_up(4 * (size_t)plan->xr * (size_t)plan->xc, kWsAlign) * d.ways);
        break;
    default: return JG_E_DTYPE;
    }
    return JG_OK;
}

// Geometry of one tensor's partition: every rank's block is rows x cols, rank r's block sits at
// block coordinates (rb, cb) of the global matrix, whose width is `width`.
struct Partition {
    int64_t rows, cols, width;
};

static int partition_of(const jg_plan* plan, int which, Partition* out)
{
    switch (which) {
    case JG_T_X:
    case JG_T_X_F32: *out = {plan->xr, plan->xc, plan->d.op == JG_OP_XTW ? plan->d.M : plan->d.K}; return JG_OK;
    case JG_T_W:
    case JG_T_W_F32: *out = {plan->wr, plan->wc, plan->d.op == JG_OP_XWT ? plan->d.K : plan->d.N}; return JG_OK;
    case JG_T_Y: *out = {plan->yr, plan->yc, plan->d.N}; return JG_OK;
    default: return JG_E_DTYPE;
    }
}

static void block_coords(int ways, int r, int64_t* rb, int64_t* cb)
{
    *rb = 0;
    *cb = 0;
    if (ways == 2) *cb = r;
    if (ways == 4) { *rb = r / 2; *cb = r % 2; }
}

int jg_shard(const jg_plan* plan, int which, const float* global, int64_t ld, float* const* shards)
{
    if (!plan || !global) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    if (int rc = check_ptr_array(shards, d.ways)) return rc;
    if (!aligned(global, 4)) return JG_E_ALIGN;
    if (which != JG_T_X && which != JG_T_W && which != JG_T_B && which != JG_T_Y && which != JG_T_X_F32 &&
        which != JG_T_W_F32)
        return JG_E_DTYPE;
    jg_ctx* c = plan->ctx;
    if (!c) return JG_E_NULL;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;

    if (d.dtype != JG_F32 && (which == JG_T_X || which == JG_T_W)) {
        // reduced precision: the shard is written in the format the matrix cores read
        Partition pt;
        (void)partition_of(plan, which, &pt);
        if (ld < pt.width) return JG_E_SHAPE;
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = d.ways;
        cv.rows = (int)pt.rows;
        cv.cols = (int)pt.cols;
        cv.planes = d.dtype == JG_BF16X3 ? 2 : 1;
        cv.plane = (int)plan->plane;
        for (int r = 0; r < d.ways; ++r) {
            if (!aligned(shards[r], 16)) return JG_E_ALIGN;
            int64_t rb, cb;
            block_coords(d.ways, r, &rb, &cb);
            cv.b[r] = {global + rb * pt.rows * ld + cb * pt.cols, reinterpret_cast<uint16_t*>(shards[r]), ld};
        }
        ScopedTimer t(c, JG_KERNEL_SHARD);
        if (d.op == JG_OP_XTW)      // contraction-major: the block's columns become the shard's rows
            return HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream)) ? JG_OK : JG_E_HIP;
        return HIP_OK(jg::launch_cvt_group(cv, c->stream)) ? JG_OK : JG_E_HIP;
    }

    jg::CopyGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nblocks = d.ways;
    // activations and gradients are streamed once; weights and bias are re-read soon
    g.nontemporal = which == JG_T_X || which == JG_T_Y || which == JG_T_X_F32;
    if (which == JG_T_B) {
        g.rows = 1;
        g.cols = (int)plan->yc;
        for (int r = 0; r < d.ways; ++r) {
            const int64_t col_half = d.ways == 1 ? 0 : (r % 2);
            g.b[r] = {global + col_half * plan->yc, shards[r], plan->yc, plan->yc};
        }
    } else {
        Partition pt;
        (void)partition_of(plan, which, &pt);
        if (ld < pt.width) return JG_E_SHAPE;
        g.rows = (int)pt.rows;
        g.cols = (int)pt.cols;
        for (int r = 0; r < d.ways; ++r) {
            int64_t rb, cb;
            block_coords(d.ways, r, &rb, &cb);
            g.b[r] = {global + rb * pt.rows * ld + cb * pt.cols, shards[r], ld, pt.cols};
        }
    }
    ScopedTimer t(c, JG_KERNEL_SHARD);
    return HIP_OK(jg::launch_copy_group(g, c->stream)) ? JG_OK : JG_E_HIP;
}

int jg_gather_as(const jg_plan* plan, int which, const float* const* shards, float* global, int64_t ld)
{
    if (!plan || !global) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    if (int rc = check_ptr_array(shards, d.ways)) return rc;
    if (!aligned(global, 4)) return JG_E_ALIGN;
    Partition pt;
    if (int rc = partition_of(plan, which, &pt)) return rc;
    if (d.dtype != JG_F32 && (which == JG_T_X || which == JG_T_W))
        return JG_E_DTYPE;   // bfloat16 shards are not converted back
    if (ld < pt.width) return JG_E_SHAPE;
    jg_ctx* c = plan->ctx;
    if (!c) return JG_E_NULL;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;

    jg::CopyGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nblocks = d.ways;
    g.nontemporal = 1;
    g.rows = (int)pt.rows;
    g.cols = (int)pt.cols;
    for (int r = 0; r < d.ways; ++r) {
        int64_t rb, cb;
        block_coords(d.ways, r, &rb, &cb);
        g.b[r] = {shards[r], global + rb * pt.rows * ld + cb * pt.cols, pt.cols, ld};
    }
    ScopedTimer t(c, JG_KERNEL_GATHER);
    return HIP_OK(jg::launch_copy_group(g, c->stream)) ? JG_OK : JG_E_HIP;
}

// Shared by jg_shard_patches / jg_gather_patches: `which` is the tensor whose partition the blocks follow.
static int patch_move(const jg_plan* plan, int which, float* field, int64_t C, int64_t H, int64_t W, int64_t p,
                      float* const* blocks, bool to_field)
{
    if (!plan || !field) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    if (d.op != JG_OP_XWT || (d.dtype != JG_F32 && which == JG_T_X)) return JG_E_DTYPE;
    if (int rc = check_ptr_array(blocks, d.ways)) return rc;
    if (!aligned(field, 4)) return JG_E_ALIGN;
    if (C <= 0 || H <= 0 || W <= 0 || p <= 0 || C > kMaxDim || H > kMaxDim || W > kMaxDim || p > 4096) return JG_E_SHAPE;
    if (H % p || W % p) return JG_E_SHAPE;
    Partition pt;
    (void)partition_of(plan, which, &pt);
    // tokens = patches, features = channels x patch elements
    if ((H / p) * (W / p) != d.M || C * p * p != pt.width) return JG_E_SHAPE;
    if (pt.rows * pt.cols >= jg::kMaxUnitsPerLaunch) return JG_E_SHAPE;
    jg_ctx* c = plan->ctx;
    if (!c) return JG_E_NULL;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    jg::PatchGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nblocks = d.ways;
    g.rows = (int)pt.rows;
    g.cols = (int)pt.cols;
    g.field = field;
    g.H = (int)H; g.W = (int)W; g.p = (int)p; g.wp = (int)(W / p);
    for (int r = 0; r < d.ways; ++r) {
        int64_t rb, cb;
        block_coords(d.ways, r, &rb, &cb);
        g.block[r] = blocks[r];
        g.row0[r] = (int)(rb * pt.rows);
        g.col0[r] = (int)(cb * pt.cols);
    }
    ScopedTimer t(c, to_field ? JG_KERNEL_GATHER : JG_KERNEL_SHARD);
    return HIP_OK(jg::launch_patch_group(g, to_field, c->stream)) ? JG_OK : JG_E_HIP;
}

int jg_shard_patches(const jg_plan* plan, const float* field, int64_t C, int64_t H, int64_t W, int64_t p,
                     float* const* x_shards)
{
    return patch_move(plan, JG_T_X, const_cast<float*>(field), C, H, W, p, x_shards, false);
}

int jg_gather_patches(const jg_plan* plan, const float* const* y_shards, float* field, int64_t C, int64_t H,
                      int64_t W, int64_t p)
{
    return patch_move(plan, JG_T_Y, field, C, H, W, p, const_cast<float* const*>(y_shards), true);
}

int jg_gather(const jg_plan* plan, const float* const* y_sh, float* global_y, int64_t ld)
{
    return jg_gather_as(plan, JG_T_Y, y_sh, global_y, ld);
}

// One GEMM launch of a pass (timed as `kernel_class`), followed by the join kernel when the
// launcher split the tail; `scratch` is the pass's tail region of the caller's workspace.
// copy16 (reduced precision only, may be null): a bfloat16 copy of the launch's output for the next layer.
// plane (reduced precision; 0 = the plan's forward shards'): elements per plane of the operands' rows
static bool run_gemm(const jg_plan* plan, jg::GemmGroup& g, int layout, int kernel_class, char* scratch,
                     size_t scratch_bytes, const jg::HbCopy16* copy16 = nullptr, int plane = 0)
{
    jg_ctx* c = plan->ctx;
    bool join = false;
    if (plan->d.dtype != JG_F32) {
        // The bfloat16 kernels sum in one level (their accumulators fill the register file).  The second level is
        // taken here: the contraction is cut into chunks, one launch each; the first writes its sums to C (on top
        // of the product's addend), every later one adds its own on top of what C holds, and the last applies the
        // epilogue.  One chunk, and nothing changes, for short contractions and for JG_ACC_SINGLE plans.
        const int terms = plan->d.dtype == JG_BF16X3 ? 3 : 1;
        const int K = g.K;
        const int chunk = plan->d.accumulate == JG_ACC_SINGLE ? K : jg::bf16_chunk_k(K, terms);
        const jg::GemmGroup whole = g;
        for (int k0 = 0; k0 < K; k0 += chunk) {
            const bool first = k0 == 0, last = k0 + chunk >= K;
            jg::GemmGroup part = whole;
            part.K = last ? K - k0 : chunk;
            if (!last) part.act = jg::kActNone;
            for (int i = 0; i < whole.nprob; ++i) {
                jg::GemmProblem& q = part.p[i];
                q.A += k0 / 2;      // operand rows hold bfloat16 pairs per 4-byte unit; a split operand's lo plane
                q.B += k0 / 2;      // sits at the same distance behind its hi plane in every chunk
                if (!first) { q.addend = q.C; q.ldadd = q.ldc; }
                if (!last) { q.bias = nullptr; q.residual = nullptr; q.ldres = 0; }
            }
            jg::HbGroup hb;
            // a launch that adds on top of what the one before it wrote walks the tiles the other way round
            // (HbGroup::reverse)
            const bool reverse = part.p[0].addend ? !c->hb_reverse : false;
            c->hb_reverse = reverse;
            {
                ScopedTimer t(c, kernel_class);
                if (!HIP_OK(jg::launch_gemm_bf16_group(part, terms, plane ? plane : (int)plan->plane, plan->slots / 2,
                                                       reinterpret_cast<float*>(scratch), scratch_bytes, c->stream, hb,
                                                       &join, last ? copy16 : nullptr, reverse)))
                    return false;
            }
            if (join) {
                ScopedTimer t(c, JG_KERNEL_JOIN);
                if (!HIP_OK(jg::launch_gemm_bf16_join(hb, c->stream))) return false;
            }
        }
        return true;
    }
    {
        ScopedTimer t(c, kernel_class);
        if (!HIP_OK(jg::launch_gemm_group(g, layout, c->stream, reinterpret_cast<float*>(scratch), scratch_bytes,
                                          plan->slots, &join)))
            return false;
    }
    if (join) {
        ScopedTimer t(c, JG_KERNEL_JOIN);
        if (!HIP_OK(jg::launch_gemm_join(g, c->stream))) return false;
    }
    return true;
}

// Forward pass of the transposed layer Y = X^T W (+ b); arguments already checked.  Every block
// product is a GEMM whose two operands are read along their row stride (A = an X block, K x M;
// B = a W block, K x N).
static int forward_xtw(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                       const float* const* b_sh, const float* const* r_sh, int act, float* const* y_sh, char* ws)
{
    const jg_linear_desc& d = plan->d;
    const int ways = d.ways;
    jg_ctx* c = plan->ctx;
    auto bias_of = [&](int r) -> const float* { return d.has_bias ? b_sh[r] : nullptr; };
    auto res_of = [&](int r) -> const float* { return r_sh ? r_sh[r] : nullptr; };
    // reduced precision: the shards are stored contraction-major (channels x tokens), so every product is the
    // bfloat16 kernel's own form A B^T with both leading dimensions the padded token count
    const bool reduced = d.dtype != JG_F32;
    const int ldx = reduced ? (int)plan->xcp : (int)plan->xc, ldw = reduced ? (int)plan->xcp : (int)plan->wc;
    const int ldy = (int)plan->yc;
    char* tail = plan->tail_bytes ? ws + plan->off_tail : nullptr;

    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    g.M = (int)plan->xc;   // channels of one X block = rows of one Y block
    g.N = (int)plan->wc;
    g.K = (int)plan->xr;   // tokens of one block
    if (reduced) g.K = (g.K + 7) / 8 * 8;      // whole 16-byte chunks: the shard step wrote zeros past the last token

    if (ways == 1) {
        g.nprob = 1;
        g.act = act;
        g.p[0] = {x_sh[0], w_sh[0], y_sh[0], nullptr, bias_of(0), ldx, ldw, ldy, 0, res_of(0), ldy};
        return run_gemm(plan, g, jg::kGemmTN, JG_KERNEL_GEMM, tail, plan->tail_bytes) ? JG_OK : JG_E_HIP;
    }

    // the activation block every rank gets from its row neighbour (rank r ^ 1)
    const float* x_in[4];
    if (d.weights == JG_WEIGHTS_COPY) {
        jg::CopyGroup cg;
        std::memset(&cg, 0, sizeof(cg));
        cg.nblocks = ways;
        cg.nontemporal = 0;
        cg.rows = reduced ? (int)plan->xc : (int)plan->xr;
        cg.cols = reduced ? (int)plan->xcp : (int)plan->xc;
        for (int r = 0; r < ways; ++r) {
            float* dst = reinterpret_cast<float*>(ws + plan->off_wrecv + r * plan->wblk_bytes);
            cg.b[r] = {x_sh[r ^ 1], dst, cg.cols, cg.cols};
            x_in[r] = dst;
        }
        ScopedTimer t(c, JG_KERNEL_WEIGHT_COPY);
        if (!HIP_OK(jg::launch_copy_group(cg, c->stream))) return JG_E_HIP;
    } else {
        for (int r = 0; r < ways; ++r) x_in[r] = x_sh[r ^ 1];
    }

    if (ways == 2) {
        // Y_r = [X_0^T W_r ; X_1^T W_r]: row half r from the rank's own block, the other from the
        // received one; nothing is summed across ranks, so both products carry the bias
        const int64_t half = (int64_t)plan->xc * plan->yc;   // floats in one M/2 x N/2 block of Y_r
        g.nprob = 4;
        g.act = act;
        for (int r = 0; r < 2; ++r) {
            const float* res = res_of(r);
            g.p[2 * r] = {x_sh[r], w_sh[r], y_sh[r] + r * half, nullptr, bias_of(r), ldx, ldw, ldy, 0,
                          res ? res + r * half : nullptr, ldy};
            g.p[2 * r + 1] = {x_in[r], w_sh[r], y_sh[r] + (1 - r) * half, nullptr, bias_of(r), ldx, ldw, ldy, 0,
                              res ? res + (1 - r) * half : nullptr, ldy};
        }
        return run_gemm(plan, g, jg::kGemmTN, JG_KERNEL_GEMM, tail, plan->tail_bytes) ? JG_OK : JG_E_HIP;
    }

    // 4-way.  Rank (i, j) = 2 i + j: own X block -> a term of Y block (j, j), received X block -> a
    // term of Y block (1 - j, j).  It owns block (i, j), so it keeps the first if i == j and the
    // second otherwise, and hands the other one to rank (1 - i, j) = r ^ 2.
    auto send_buf = [&](int r) { return reinterpret_cast<float*>(ws + plan->off_send + r * plan->part_bytes); };
    auto kept_buf = [&](int r) { return reinterpret_cast<float*>(ws + plan->off_kept + r * plan->part_bytes); };
    const float* x_keep[4];
    const float* x_send[4];
    for (int r = 0; r < 4; ++r) {
        const bool own_is_kept = (r / 2) == (r % 2);
        x_keep[r] = own_is_kept ? x_sh[r] : x_in[r];
        x_send[r] = own_is_kept ? x_in[r] : x_sh[r];
    }
    g.nprob = 4;
    for (int r = 0; r < 4; ++r)
        g.p[r] = {x_send[r], w_sh[r], send_buf(r), nullptr, nullptr, ldx, ldw, ldy, 0};
    if (!run_gemm(plan, g, jg::kGemmTN, JG_KERNEL_GEMM, tail, plan->tail_bytes)) return JG_E_HIP;
    if (d.combine == JG_COMBINE_FUSED) {
        g.act = act;
        for (int r = 0; r < 4; ++r)
            g.p[r] = {x_keep[r], w_sh[r], y_sh[r], send_buf(r ^ 2), bias_of(r), ldx, ldw, ldy, ldy, res_of(r), ldy};
        return run_gemm(plan, g, jg::kGemmTN, JG_KERNEL_GEMM, tail, plan->tail_bytes) ? JG_OK : JG_E_HIP;
    }
    for (int r = 0; r < 4; ++r)
        g.p[r] = {x_keep[r], w_sh[r], kept_buf(r), nullptr, nullptr, ldx, ldw, ldy, 0};
    if (!run_gemm(plan, g, jg::kGemmTN, JG_KERNEL_GEMM, tail, plan->tail_bytes)) return JG_E_HIP;
    jg::CombineGroup cb;
    std::memset(&cb, 0, sizeof(cb));
    cb.nblocks = 4;
    cb.rows = (int)plan->yr;
    cb.cols = (int)plan->yc;
    cb.act = act;
    for (int r = 0; r < 4; ++r) cb.b[r] = {kept_buf(r), send_buf(r ^ 2), bias_of(r), y_sh[r], res_of(r)};
    ScopedTimer t(c, JG_KERNEL_COMBINE);
    return HIP_OK(jg::launch_combine_group(cb, c->stream)) ? JG_OK : JG_E_HIP;
}

// Forward pass of the third permutation Y = X W (+ b), weights stored K x N; arguments already checked.  It is
// the form of the backward product dX = dY W (Sec. 4.1) and takes that pass's blocks: every output block is
//     Y_(i,j) = X_(i,j) W_(j,j) + X_(i,1-j) W_(1-j,j),
// both products formed by the block's owner - the second from the activation block of its row neighbour, and
// whichever weight block is not its own from its column neighbour (2-way: a rank holds both weight blocks of
// its column half).  The first product goes to a partial in the workspace, the second is accumulated on top.
// A = an X block (K-contiguous), B = a W block read along its row stride.
static int forward_xw(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                      const float* const* b_sh, const float* const* r_sh, int act, float* const* y_sh, char* ws)
{
    const jg_linear_desc& d = plan->d;
    const int ways = d.ways;
    jg_ctx* c = plan->ctx;
    auto bias_of = [&](int r) -> const float* { return d.has_bias ? b_sh[r] : nullptr; };
    auto res_of = [&](int r) -> const float* { return r_sh ? r_sh[r] : nullptr; };
    char* tail = plan->tail_bytes ? ws + plan->off_tail : nullptr;
    const int ldx = (int)plan->xc, ldw = (int)plan->wc, ldy = (int)plan->yc;

    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    g.M = (int)plan->yr;
    g.N = (int)plan->yc;
    g.K = (int)plan->xc;
    if (ways == 1) {
        g.nprob = 1;
        g.act = act;
        g.p[0] = {x_sh[0], w_sh[0], y_sh[0], nullptr, bias_of(0), ldx, ldw, ldy, 0, res_of(0), ldy};
        return run_gemm(plan, g, jg::kGemmNN, JG_KERNEL_GEMM, tail, plan->tail_bytes) ? JG_OK : JG_E_HIP;
    }
    // what a rank gets from its peers: the activation block of its row neighbour (r ^ 1) and, 4-way, the weight
    // block of its column neighbour (r ^ 2)
    const float* x_in[4];
    const float* w_in[4] = {nullptr, nullptr, nullptr, nullptr};
    if (d.weights == JG_WEIGHTS_COPY) {
        jg::CopyGroup cg;
        std::memset(&cg, 0, sizeof(cg));
        cg.nblocks = ways;
        cg.nontemporal = 0;
        cg.rows = (int)plan->xr;
        cg.cols = (int)plan->xc;
        for (int r = 0; r < ways; ++r) {
            float* dst = reinterpret_cast<float*>(ws + plan->off_xrecv + r * plan->xblk_bytes);
            cg.b[r] = {x_sh[r ^ 1], dst, cg.cols, cg.cols};
            x_in[r] = dst;
        }
        {
            ScopedTimer t(c, JG_KERNEL_WEIGHT_COPY);
            if (!HIP_OK(jg::launch_copy_group(cg, c->stream))) return JG_E_HIP;
        }
        if (ways == 4) {
            cg.rows = (int)plan->wr;
            cg.cols = (int)plan->wc;
            for (int r = 0; r < 4; ++r) {
                float* dst = reinterpret_cast<float*>(ws + plan->off_wrecv + r * plan->wblk_bytes);
                cg.b[r] = {w_sh[r ^ 2], dst, cg.cols, cg.cols};
                w_in[r] = dst;
            }
            ScopedTimer t(c, JG_KERNEL_WEIGHT_COPY);
            if (!HIP_OK(jg::launch_copy_group(cg, c->stream))) return JG_E_HIP;
        }
    } else {
        for (int r = 0; r < ways; ++r) {
            x_in[r] = x_sh[r ^ 1];
            if (ways == 4) w_in[r] = w_sh[r ^ 2];
        }
    }
    // the weight block of the product with the rank's own activation block, and of the one with the received block
    const float* w_own[4];
    const float* w_other[4];
    if (ways == 2) {
        const int64_t block = (int64_t)plan->xc * plan->wc;     // floats in one K/2 x N/2 block of W_r = [W_(0,r); W_(1,r)]
        for (int r = 0; r < 2; ++r) {
            w_own[r] = w_sh[r] + r * block;
            w_other[r] = w_sh[r] + (1 - r) * block;
        }
    } else {
        for (int r = 0; r < 4; ++r) {
            const bool diagonal = (r / 2) == (r % 2);           // rank (i, j) holds W_(i,j): W_(j,j) iff i = j
            w_own[r] = diagonal ? w_sh[r] : w_in[r];
            w_other[r] = diagonal ? w_in[r] : w_sh[r];
        }
    }
    auto part_buf = [&](int r) { return reinterpret_cast<float*>(ws + plan->off_send + r * plan->part_bytes); };
    auto kept_buf = [&](int r) { return reinterpret_cast<float*>(ws + plan->off_kept + r * plan->part_bytes); };
    g.nprob = ways;
    for (int r = 0; r < ways; ++r)
        g.p[r] = {x_in[r], w_other[r], part_buf(r), nullptr, nullptr, ldx, ldw, ldy, 0, nullptr, 0};
    if (!run_gemm(plan, g, jg::kGemmNN, JG_KERNEL_GEMM, tail, plan->tail_bytes)) return JG_E_HIP;
    if (d.combine == JG_COMBINE_FUSED) {
        g.act = act;
        for (int r = 0; r < ways; ++r)
            g.p[r] = {x_sh[r], w_own[r], y_sh[r], part_buf(r), bias_of(r), ldx, ldw, ldy, ldy, res_of(r), ldy};
        return run_gemm(plan, g, jg::kGemmNN, JG_KERNEL_GEMM, tail, plan->tail_bytes) ? JG_OK : JG_E_HIP;
    }
    for (int r = 0; r < ways; ++r)
        g.p[r] = {x_sh[r], w_own[r], kept_buf(r), nullptr, nullptr, ldx, ldw, ldy, 0, nullptr, 0};
    if (!run_gemm(plan, g, jg::kGemmNN, JG_KERNEL_GEMM, tail, plan->tail_bytes)) return JG_E_HIP;
    jg::CombineGroup cb;
    std::memset(&cb, 0, sizeof(cb));
    cb.nblocks = ways;
    cb.rows = (int)plan->yr;
    cb.cols = (int)plan->yc;
    cb.act = act;
    for (int r = 0; r < ways; ++r) cb.b[r] = {kept_buf(r), part_buf(r), bias_of(r), y_sh[r], res_of(r)};
    ScopedTimer t(c, JG_KERNEL_COMBINE);
    return HIP_OK(jg::launch_combine_group(cb, c->stream)) ? JG_OK : JG_E_HIP;
}

int jg_linear_forward(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                      const float* const* b_sh, float* const* y_sh, void* workspace,
                      size_t workspace_bytes)
{
    return jg_linear_forward_ex(plan, x_sh, w_sh, b_sh, nullptr, JG_ACT_NONE, y_sh, workspace, workspace_bytes);
}

// jg_linear_forward_ex.  copy16 (reduced-precision plans with the fused combine only, may be null): the launch
// that writes Y also writes it in bfloat16, in the X-shard format of the layer that follows.
static int forward_impl(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                        const float* const* b_sh, const float* const* r_sh, int activation, float* const* y_sh,
                        void* workspace, size_t workspace_bytes, const jg::HbCopy16* copy16)
{
    if (!plan || !plan->ctx) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    const int ways = d.ways;
    if (activation != JG_ACT_NONE && activation != JG_ACT_GELU) return JG_E_DTYPE;
    const int act = activation == JG_ACT_GELU ? jg::kActGelu : jg::kActNone;
    if (int rc = check_ptr_array(x_sh, ways)) return rc;
    if (int rc = check_ptr_array(w_sh, ways)) return rc;
    if (int rc = check_ptr_array(y_sh, ways)) return rc;
    if (d.has_bias) {
        if (int rc = check_ptr_array(b_sh, ways)) return rc;
    }
    if (r_sh) {
        if (int rc = check_ptr_array(r_sh, ways)) return rc;
    }
    if (plan->ws_bytes > 0) {
        if (!workspace || workspace_bytes < plan->ws_bytes) return JG_E_WORKSPACE;
        if (!aligned(workspace, kWsAlign)) return JG_E_ALIGN;
    }
    jg_ctx* c = plan->ctx;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    char* ws = static_cast<char*>(workspace);
    auto bias_of = [&](int r) -> const float* { return d.has_bias ? b_sh[r] : nullptr; };
    auto res_of = [&](int r) -> const float* { return r_sh ? r_sh[r] : nullptr; };

    if (d.op == JG_OP_XTW) return forward_xtw(plan, x_sh, w_sh, b_sh, r_sh, act, y_sh, ws);
    if (d.op == JG_OP_XW) return forward_xw(plan, x_sh, w_sh, b_sh, r_sh, act, y_sh, ws);
    char* tail = plan->tail_bytes ? ws + plan->off_tail : nullptr;

    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    g.M = (int)plan->yr;
    g.N = (int)plan->yc;
    g.K = (int)plan->xc;
    const int ldk = (int)plan->xcp;  // leading dimension of every X / W shard, in 4-byte units
    const int ldn = (int)plan->yc;   // leading dimension of every Y shard / partial

    if (ways == 1) {
        g.nprob = 1;
        g.act = act;
        g.p[0] = {x_sh[0], w_sh[0], y_sh[0], nullptr, bias_of(0), ldk, ldk, ldn, 0, res_of(0), ldn};
        return run_gemm(plan, g, jg::kGemmNT, JG_KERNEL_GEMM, tail, plan->tail_bytes, copy16) ? JG_OK : JG_E_HIP;
    }

    auto send_buf = [&](int r) { return reinterpret_cast<float*>(ws + plan->off_send + r * plan->part_bytes); };
    auto kept_buf = [&](int r) { return reinterpret_cast<float*>(ws + plan->off_kept + r * plan->part_bytes); };

    // For every rank: the weight block of the product it ships, of the product it keeps,
    // and the rank whose shipped partial it receives.
    const float* w_send[4];
    const float* w_keep[4];
    int recv_from[4];
    if (ways == 2) {
        // Sec. 4.1: W_r = [W_{r,0}; W_{r,1}] by rows; rank r keeps X_r W_{r,r}^T and ships
        // X_r W_{r,1-r}^T to the other rank.
        const int64_t half = plan->yc * plan->xcp;  // 4-byte units in one N/2 x K/2 block
        for (int r = 0; r < 2; ++r) {
            w_keep[r] = w_sh[r] + r * half;
            w_send[r] = w_sh[r] + (1 - r) * half;
            recv_from[r] = 1 - r;
        }
    } else {
        const float* w_in[4];   // the weight block rank r receives from kWeightFrom4[r]
        if (d.weights == JG_WEIGHTS_COPY) {
            jg::CopyGroup cg;
            std::memset(&cg, 0, sizeof(cg));
            cg.nblocks = 4;
            cg.rows = (int)plan->wr;
            cg.cols = (int)plan->xcp;
            for (int r = 0; r < 4; ++r) {
                float* dst = reinterpret_cast<float*>(ws + plan->off_wrecv + r * plan->wblk_bytes);
                cg.b[r] = {w_sh[kWeightFrom4[r]], dst, plan->xcp, plan->xcp};
                w_in[r] = dst;
            }
            ScopedTimer t(c, JG_KERNEL_WEIGHT_COPY);
            if (!HIP_OK(jg::launch_copy_group(cg, c->stream))) return JG_E_HIP;
        } else {
            for (int r = 0; r < 4; ++r) w_in[r] = w_sh[kWeightFrom4[r]];
        }
        for (int r = 0; r < 4; ++r) {
            w_keep[r] = kOwnIsKept4[r] ? w_sh[r] : w_in[r];
            w_send[r] = kOwnIsKept4[r] ? w_in[r] : w_sh[r];
            recv_from[r] = kPeer4[r];
        }
    }

    // launch 1: the products handed to a peer, stored where the peer will read them
    g.nprob = ways;
    for (int r = 0; r < ways; ++r)
        g.p[r] = {x_sh[r], w_send[r], send_buf(r), nullptr, nullptr, ldk, ldk, ldn, 0};
    if (!run_gemm(plan, g, jg::kGemmNT, JG_KERNEL_GEMM, tail, plan->tail_bytes)) return JG_E_HIP;

    // launch 2: the kept products
    if (d.combine == JG_COMBINE_FUSED) {
        g.act = act;
        for (int r = 0; r < ways; ++r)
            g.p[r] = {x_sh[r], w_keep[r], y_sh[r], send_buf(recv_from[r]), bias_of(r), ldk, ldk, ldn, ldn,
                      res_of(r), ldn};
        return run_gemm(plan, g, jg::kGemmNT, JG_KERNEL_GEMM, tail, plan->tail_bytes, copy16) ? JG_OK : JG_E_HIP;
    }
    for (int r = 0; r < ways; ++r)
        g.p[r] = {x_sh[r], w_keep[r], kept_buf(r), nullptr, nullptr, ldk, ldk, ldn, 0};
    if (!run_gemm(plan, g, jg::kGemmNT, JG_KERNEL_GEMM, tail, plan->tail_bytes)) return JG_E_HIP;
    jg::CombineGroup cb;
    std::memset(&cb, 0, sizeof(cb));
    cb.nblocks = ways;
    cb.rows = (int)plan->yr;
    cb.cols = (int)plan->yc;
    cb.act = act;
    for (int r = 0; r < ways; ++r)
        cb.b[r] = {kept_buf(r), send_buf(recv_from[r]), bias_of(r), y_sh[r], res_of(r)};
    ScopedTimer t(c, JG_KERNEL_COMBINE);
    return HIP_OK(jg::launch_combine_group(cb, c->stream)) ? JG_OK : JG_E_HIP;
}

int jg_linear_forward_ex(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                         const float* const* b_sh, const float* const* r_sh, int activation, float* const* y_sh,
                         void* workspace, size_t workspace_bytes)
{
    return forward_impl(plan, x_sh, w_sh, b_sh, r_sh, activation, y_sh, workspace, workspace_bytes, nullptr);
}

int jg_linear_forward_static(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                             const float* const* b_sh, float* const* y_sh)
{
    if (!plan || !plan->ctx) return JG_E_NULL;
    if (plan->ws_bytes > kStaticScratchBytes) return JG_E_WORKSPACE;    // the layer does not fit the fixed array
    void* ws = plan->ctx->static_ws;
    if (!ws && plan->ws_bytes > 0) return JG_E_WORKSPACE;
    return forward_impl(plan, x_sh, w_sh, b_sh, nullptr, JG_ACT_NONE, y_sh, ws, kStaticScratchBytes, nullptr);
}

// Backward of the transposed layer Y = X^T W (X [T x C], W [T x D], dY [C x D]); arguments already checked.
//     dX = W dY^T  (contraction over D: both operands read along their rows, as in the forward of X W^T),
//     dW = X dY    (contraction over C: dY read along its row stride).
// Blocks: X_(i,a) = tokens half i, channels half a; W_(i,j); dY_(a,j) (2-way: i is the whole token range and
// dY_r stacks dY_(0,r) over dY_(1,r)).  dX_(i,a) = sum_j W_(i,j) dY_(a,j)^T,  dW_(i,j) = sum_a X_(i,a) dY_(a,j):
// two terms each, the first into a partial, the second on top of it.
static int backward_xtw(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                        const float* const* dy_sh, float* const* dx_sh, float* const* dw_sh, char* ws)
{
    const int ways = plan->d.ways;
    const int tr = (int)plan->xr, ch = (int)plan->xc, dh = (int)plan->wc;     // tokens, channels, columns of a block
    char* tail = plan->bw_tail_bytes ? ws + plan->bw_off_tail : nullptr;
    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    auto launch = [&](int layout, int kernel_class) -> bool {
        return run_gemm(plan, g, layout, kernel_class, tail, plan->bw_tail_bytes);
    };
    if (ways == 1) {
        g.nprob = 1; g.M = tr; g.N = ch; g.K = dh;
        g.p[0] = {w_sh[0], dy_sh[0], dx_sh[0], nullptr, nullptr, dh, dh, ch, 0};
        if (!launch(jg::kGemmNT, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
        g.M = tr; g.N = dh; g.K = ch;
        g.p[0] = {x_sh[0], dy_sh[0], dw_sh[0], nullptr, nullptr, ch, dh, dh, 0};
        return launch(jg::kGemmNN, JG_KERNEL_GEMM_DW) ? JG_OK : JG_E_HIP;
    }
    auto dx_part = [&](int r) { return reinterpret_cast<float*>(ws + r * plan->bw_dx_bytes); };
    auto dw_part = [&](int r) { return reinterpret_cast<float*>(ws + plan->bw_off_dw + r * plan->bw_dw_bytes); };
    // rank and block coordinates: 2-way rank r = (0, r); 4-way rank 2 i + j = (i, j)
    const int rows = ways == 4 ? 2 : 1;
    auto rk = [&](int i, int j) { return rows == 2 ? 2 * i + j : j; };
    // dY_(a,j): on rank (a, j) in the 4-way form; block a of rank j's stacked pair in the 2-way form
    const int64_t yblock = (int64_t)ch * dh;
    auto dy_blk = [&](int a, int j) { return rows == 2 ? dy_sh[rk(a, j)] : dy_sh[j] + a * yblock; };
    g.nprob = ways;
    for (int pass = 0; pass < 2; ++pass) {      // dX_(i,a): term j = 1 - a, then term j = a
        g.M = tr; g.N = ch; g.K = dh;
        for (int i = 0; i < rows; ++i)
            for (int a = 0; a < 2; ++a) {
                const int r = rk(i, a), j = pass == 0 ? 1 - a : a;
                if (pass == 0)
                    g.p[r] = {w_sh[rk(i, j)], dy_blk(a, j), dx_part(r), nullptr, nullptr, dh, dh, ch, 0};
                else
                    g.p[r] = {w_sh[rk(i, j)], dy_blk(a, j), dx_sh[r], dx_part(r), nullptr, dh, dh, ch, ch};
            }
        if (!launch(jg::kGemmNT, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
    }
    for (int pass = 0; pass < 2; ++pass) {      // dW_(i,j): term a = 1 - j, then term a = j
        g.M = tr; g.N = dh; g.K = ch;
        for (int i = 0; i < rows; ++i)
            for (int j = 0; j < 2; ++j) {
                const int r = rk(i, j), a = pass == 0 ? 1 - j : j;
                if (pass == 0)
                    g.p[r] = {x_sh[rk(i, a)], dy_blk(a, j), dw_part(r), nullptr, nullptr, ch, dh, dh, 0};
                else
                    g.p[r] = {x_sh[rk(i, a)], dy_blk(a, j), dw_sh[r], dw_part(r), nullptr, ch, dh, dh, dh};
            }
        if (!launch(jg::kGemmNN, JG_KERNEL_GEMM_DW)) return JG_E_HIP;
    }
    return JG_OK;
}

// Backward of the plain layer in reduced precision; arguments already checked.  x_sh, w_sh: FP32 shards.  Every
// operand of every block product is rounded into the workspace in the layout the bfloat16 kernel reads (both operands
// along the contracted index): dY_r as it is for dX (contraction over its columns) and contraction-major for dW,
// the weight blocks and X_r contraction-major.  The block products and their sums are those of the FP32 backward.
static int backward_reduced(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                            const float* const* dy_sh, float* const* dx_sh, float* const* dw_sh, char* ws)
{
    const jg_linear_desc& d = plan->d;
    const int ways = d.ways;
    jg_ctx* c = plan->ctx;
    const int mr = (int)plan->xr, kh = (int)plan->xc, nh = (int)plan->yc;
    if (nh & 7) return JG_E_SHAPE;      // dY_r is rounded in 16-byte chunks of 8 along its rows
    const BwReduced L = bw_reduced_layout(plan);
    const int64_t wblock = (int64_t)nh * kh;
    auto dy16 = [&](int r) { return reinterpret_cast<const float*>(ws + L.off_dy16 + r * L.dy16); };
    auto dy16t = [&](int r) { return reinterpret_cast<const float*>(ws + L.off_dy16t + r * L.dy16t); };
    auto w16t = [&](int r, int b) { return reinterpret_cast<const float*>(ws + L.off_w16t + (r * L.wblocks + b) * L.w16t); };
    auto x16t = [&](int r) { return reinterpret_cast<const float*>(ws + L.off_x16t + r * L.x16t); };
    auto u16 = [](const float* p) { return reinterpret_cast<uint16_t*>(const_cast<float*>(p)); };
    {
        ScopedTimer t(c, JG_KERNEL_SHARD);
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = ways;
        cv.planes = L.planes;
        // dY_r: contraction-major over the tokens and, from the same read, rows as they are
        cv.rows = mr; cv.cols = nh; cv.plane = L.plane_m; cv.plane_rows = L.plane_n;
        for (int r = 0; r < ways; ++r) cv.b[r] = {dy_sh[r], u16(dy16t(r)), nh, u16(dy16(r))};
        if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        // X_r: contraction-major over the tokens
        cv.cols = kh;
        for (int r = 0; r < ways; ++r) cv.b[r] = {x_sh[r], u16(x16t(r)), kh, nullptr};
        if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        // the weight blocks (nh x kh each): contraction-major over the rank's share of N
        cv.rows = nh; cv.cols = kh; cv.plane = L.plane_n;
        for (int b = 0; b < L.wblocks; ++b) {
            for (int r = 0; r < ways; ++r) cv.b[r] = {w_sh[r] + b * wblock, u16(w16t(r, b)), kh, nullptr};
            if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        }
    }
    char* tail = plan->bw_tail_bytes ? ws + plan->bw_off_tail : nullptr;
    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    auto launch = [&](int kernel_class, int plane) -> bool {
        return run_gemm(plan, g, jg::kGemmNT, kernel_class, tail, plan->bw_tail_bytes, nullptr, plane);
    };
    auto dx_shape = [&]() { g.M = mr; g.N = kh; g.K = nh; };
    auto dw_shape = [&]() { g.M = nh; g.N = kh; g.K = (mr + 7) / 8 * 8; };      // (zeros past the last token)
    auto dx_part = [&](int r) { return reinterpret_cast<float*>(ws + r * plan->bw_dx_bytes); };
    auto dw_part = [&](int r) { return reinterpret_cast<float*>(ws + plan->bw_off_dw + r * plan->bw_dw_bytes); };
    if (ways == 1) {
        g.nprob = 1;
        dx_shape();
        g.p[0] = {dy16(0), w16t(0, 0), dx_sh[0], nullptr, nullptr, L.ld_n, L.ld_n, kh, 0};
        if (!launch(JG_KERNEL_GEMM_DX, L.plane_n)) return JG_E_HIP;
        dw_shape();
        g.p[0] = {dy16t(0), x16t(0), dw_sh[0], nullptr, nullptr, L.ld_m, L.ld_m, kh, 0};
        return launch(JG_KERNEL_GEMM_DW, L.plane_m) ? JG_OK : JG_E_HIP;
    }
    if (ways == 2) {
        // dX_r = dY_r W_{r,r} + dY_{1-r} W_{r,1-r};  dW_{r,c} = dY_c^T X_r
        g.nprob = 2;
        dx_shape();
        for (int r = 0; r < 2; ++r)
            g.p[r] = {dy16(1 - r), w16t(r, 1 - r), dx_part(r), nullptr, nullptr, L.ld_n, L.ld_n, kh, 0};
        if (!launch(JG_KERNEL_GEMM_DX, L.plane_n)) return JG_E_HIP;
        for (int r = 0; r < 2; ++r)
            g.p[r] = {dy16(r), w16t(r, r), dx_sh[r], dx_part(r), nullptr, L.ld_n, L.ld_n, kh, kh};
        if (!launch(JG_KERNEL_GEMM_DX, L.plane_n)) return JG_E_HIP;
        g.nprob = 4;
        dw_shape();
        for (int r = 0; r < 2; ++r)
            for (int cc = 0; cc < 2; ++cc)
                g.p[2 * r + cc] = {dy16t(cc), x16t(r), dw_sh[r] + cc * wblock, nullptr, nullptr, L.ld_m, L.ld_m, kh, 0};
        return launch(JG_KERNEL_GEMM_DW, L.plane_m) ? JG_OK : JG_E_HIP;
    }
    // 4-way: dX_(i,j) = sum_c dY_(i,c) W_(c,j);  dW_(c,j) = sum_i dY_(i,c)^T X_(i,j);  rank 2 row + column
    auto rk = [](int a, int b) { return 2 * a + b; };
    g.nprob = 4;
    for (int pass = 0; pass < 2; ++pass) {
        dx_shape();
        for (int i = 0; i < 2; ++i)
            for (int j = 0; j < 2; ++j) {
                const int r = rk(i, j), cc = pass == 0 ? 1 - j : j;
                if (pass == 0)
                    g.p[r] = {dy16(rk(i, cc)), w16t(rk(cc, j), 0), dx_part(r), nullptr, nullptr, L.ld_n, L.ld_n, kh, 0};
                else
                    g.p[r] = {dy16(rk(i, cc)), w16t(rk(cc, j), 0), dx_sh[r], dx_part(r), nullptr, L.ld_n, L.ld_n, kh, kh};
            }
        if (!launch(JG_KERNEL_GEMM_DX, L.plane_n)) return JG_E_HIP;
    }
    for (int pass = 0; pass < 2; ++pass) {
        dw_shape();
        for (int cc = 0; cc < 2; ++cc)
            for (int j = 0; j < 2; ++j) {
                const int r = rk(cc, j), i = pass == 0 ? 1 - cc : cc;
                if (pass == 0)
                    g.p[r] = {dy16t(rk(i, cc)), x16t(rk(i, j)), dw_part(r), nullptr, nullptr, L.ld_m, L.ld_m, kh, 0};
                else
                    g.p[r] = {dy16t(rk(i, cc)), x16t(rk(i, j)), dw_sh[r], dw_part(r), nullptr, L.ld_m, L.ld_m, kh, kh};
            }
        if (!launch(JG_KERNEL_GEMM_DW, L.plane_m)) return JG_E_HIP;
    }
    return JG_OK;
}

// Backward of the transposed layer in reduced precision; arguments already checked.  x_sh, w_sh: FP32 shards.
// Blocks and sums as backward_xtw; what each product reads is rounded into the workspace first.
static int backward_xtw_reduced(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                                const float* const* dy_sh, float* const* dx_sh, float* const* dw_sh, char* ws)
{
    const int ways = plan->d.ways;
    jg_ctx* c = plan->ctx;
    const int tr = (int)plan->xr, ch = (int)plan->xc, dh = (int)plan->wc;
    if ((ch & 7) || (dh & 7)) return JG_E_SHAPE;    // X_r, W_r and dY_r are rounded in 16-byte chunks of 8 along their rows
    const BwReducedXtw L = bw_reduced_xtw_layout(plan);
    const int rows = ways == 4 ? 2 : 1;
    auto rk = [&](int i, int j) { return rows == 2 ? 2 * i + j : j; };
    auto w16 = [&](int r) { return reinterpret_cast<const float*>(ws + L.off_w16 + r * L.w16); };
    auto x16 = [&](int r) { return reinterpret_cast<const float*>(ws + L.off_x16 + r * L.x16); };
    // dY_(a,j): on rank (a, j) in the 4-way form; block a of rank j's stacked pair in the 2-way form
    auto dy16 = [&](int a, int j) {
        const char* base = ws + L.off_dy16 + (rows == 2 ? rk(a, j) : j) * L.dy16;
        return reinterpret_cast<const float*>(base) + (rows == 2 ? 0 : (int64_t)a * ch * L.ld_d);
    };
    auto dy16t = [&](int a, int j) {
        const int r = rows == 2 ? rk(a, j) : j, b = rows == 2 ? 0 : a;
        return reinterpret_cast<const float*>(ws + L.off_dy16t + (r * L.yblocks + b) * L.dy16t);
    };
    auto u16 = [](const float* p) { return reinterpret_cast<uint16_t*>(const_cast<float*>(p)); };
    {
        ScopedTimer t(c, JG_KERNEL_SHARD);
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = ways;
        cv.planes = L.planes;
        cv.rows = tr; cv.cols = dh; cv.plane = L.plane_d;                   // W_r as it is
        for (int r = 0; r < ways; ++r) cv.b[r] = {w_sh[r], u16(w16(r)), dh};
        if (!HIP_OK(jg::launch_cvt_group(cv, c->stream))) return JG_E_HIP;
        cv.rows = tr; cv.cols = ch; cv.plane = L.plane_c;                   // X_r as it is
        for (int r = 0; r < ways; ++r) cv.b[r] = {x_sh[r], u16(x16(r)), ch};
        if (!HIP_OK(jg::launch_cvt_group(cv, c->stream))) return JG_E_HIP;
        // every dY block contraction-major and, from the same read, as it is (2-way: the blocks of dY_r one after
        // the other, as the rows of its rounded shard)
        cv.rows = ch; cv.cols = dh; cv.plane_rows = L.plane_d;
        for (int b = 0; b < L.yblocks; ++b) {
            for (int r = 0; r < ways; ++r)
                cv.b[r] = {dy_sh[r] + (int64_t)b * ch * dh,
                           reinterpret_cast<uint16_t*>(ws + L.off_dy16t + (r * L.yblocks + b) * L.dy16t), dh,
                           reinterpret_cast<uint16_t*>(ws + L.off_dy16 + r * L.dy16) +
                               (int64_t)b * ch * L.plane_d * L.planes};
            if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        }
    }
    char* tail = plan->bw_tail_bytes ? ws + plan->bw_off_tail : nullptr;
    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    auto launch = [&](int kernel_class, int plane) -> bool {
        return run_gemm(plan, g, jg::kGemmNT, kernel_class, tail, plan->bw_tail_bytes, nullptr, plane);
    };
    auto dx_part = [&](int r) { return reinterpret_cast<float*>(ws + r * plan->bw_dx_bytes); };
    auto dw_part = [&](int r) { return reinterpret_cast<float*>(ws + plan->bw_off_dw + r * plan->bw_dw_bytes); };
    g.nprob = ways;
    const int passes = ways == 1 ? 1 : 2;
    for (int pass = 0; pass < passes; ++pass) {     // dX_(i,a) = sum_j W_(i,j) dY_(a,j)^T: term j = 1 - a, then j = a
        g.M = tr; g.N = ch; g.K = dh;
        for (int i = 0; i < rows; ++i)
            for (int a = 0; a < (ways == 1 ? 1 : 2); ++a) {
                const int r = rk(i, a), j = ways == 1 ? 0 : (pass == 0 ? 1 - a : a);
                const bool last = pass == passes - 1;
                g.p[r] = {w16(rk(i, j)), dy16(a, j), last ? dx_sh[r] : dx_part(r), (last && ways > 1) ? dx_part(r) : nullptr,
                          nullptr, L.ld_d, L.ld_d, ch, (last && ways > 1) ? ch : 0};
            }
        if (!launch(JG_KERNEL_GEMM_DX, L.plane_d)) return JG_E_HIP;
    }
    for (int pass = 0; pass < passes; ++pass) {     // dW_(i,j) = sum_a X_(i,a) dY_(a,j): term a = 1 - j, then a = j
        g.M = tr; g.N = dh; g.K = ch;
        for (int i = 0; i < rows; ++i)
            for (int j = 0; j < (ways == 1 ? 1 : 2); ++j) {
                const int r = rk(i, j), a = ways == 1 ? 0 : (pass == 0 ? 1 - j : j);
                const bool last = pass == passes - 1;
                g.p[r] = {x16(rk(i, a)), dy16t(a, j), last ? dw_sh[r] : dw_part(r), (last && ways > 1) ? dw_part(r) : nullptr,
                          nullptr, L.ld_c, L.ld_c, dh, (last && ways > 1) ? dh : 0};
            }
        if (!launch(JG_KERNEL_GEMM_DW, L.plane_c)) return JG_E_HIP;
    }
    return JG_OK;
}

int jg_linear_backward(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                       const float* const* dy_sh, float* const* dx_sh, float* const* dw_sh,
                       void* workspace, size_t workspace_bytes)
{
    if (!plan || !plan->ctx) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    const int ways = d.ways;
    if (int rc = check_ptr_array(x_sh, ways)) return rc;
    if (int rc = check_ptr_array(w_sh, ways)) return rc;
    if (int rc = check_ptr_array(dy_sh, ways)) return rc;
    if (int rc = check_ptr_array(dx_sh, ways)) return rc;
    if (int rc = check_ptr_array(dw_sh, ways)) return rc;
    if (plan->bw_ws_bytes > 0) {
        if (!workspace || workspace_bytes < plan->bw_ws_bytes) return JG_E_WORKSPACE;
        if (!aligned(workspace, kWsAlign)) return JG_E_ALIGN;
    }
    jg_ctx* c = plan->ctx;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    char* ws = static_cast<char*>(workspace);
    if (d.op == JG_OP_XW) {
        // dX = dY W^T is the X W^T layer on (dY, W), dW = X^T dY the X^T W layer on (X, dY): the partitions agree
        // (every tensor of the three permutations is split the same way), so the shards are used as they are
        int rc = forward_impl(plan->bw_dx_plan, dy_sh, w_sh, nullptr, nullptr, JG_ACT_NONE, dx_sh, workspace,
                              workspace_bytes, nullptr);
        if (rc != JG_OK) return rc;
        return forward_impl(plan->bw_dw_plan, x_sh, dy_sh, nullptr, nullptr, JG_ACT_NONE, dw_sh, workspace,
                            workspace_bytes, nullptr);
    }
    if (d.dtype != JG_F32) {
        for (int r = 0; r < ways; ++r)
            if (!aligned(x_sh[r], 4) || !aligned(w_sh[r], 4) || !aligned(dy_sh[r], 4)) return JG_E_ALIGN;
        return d.op == JG_OP_XTW ? backward_xtw_reduced(plan, x_sh, w_sh, dy_sh, dx_sh, dw_sh, ws)
                                 : backward_reduced(plan, x_sh, w_sh, dy_sh, dx_sh, dw_sh, ws);
    }
    if (d.op == JG_OP_XTW) return backward_xtw(plan, x_sh, w_sh, dy_sh, dx_sh, dw_sh, ws);

    // shard shapes: X_r is mr x kh, W_r is (wr) x kh, dY_r is mr x nh
    const int mr = (int)plan->xr, kh = (int)plan->xc, nh = (int)plan->yc;
    const int64_t wblock = (int64_t)nh * kh;   // floats in one nh x kh weight block

    jg::GemmGroup g;
    std::memset(&g, 0, sizeof(g));

    char* tail = plan->bw_tail_bytes ? ws + plan->bw_off_tail : nullptr;
    auto launch = [&](int layout, int kernel_class) -> bool {
        return run_gemm(plan, g, layout, kernel_class, tail, plan->bw_tail_bytes);
    };

    if (ways == 1) {
        // dX [M x K] = dY [M x N] . W [N x K]: contraction over N, W read K-strided
        g.nprob = 1; g.M = mr; g.N = kh; g.K = nh;
        g.p[0] = {dy_sh[0], w_sh[0], dx_sh[0], nullptr, nullptr, nh, kh, kh, 0};
        if (!launch(jg::kGemmNN, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
        // dW [N x K] = dY^T . X: contraction over M, both operands read K-strided
        g.M = nh; g.N = kh; g.K = mr;
        g.p[0] = {dy_sh[0], x_sh[0], dw_sh[0], nullptr, nullptr, nh, kh, kh, 0};
        return launch(jg::kGemmTN, JG_KERNEL_GEMM_DW) ? JG_OK : JG_E_HIP;
    }

    auto dx_part = [&](int r) { return reinterpret_cast<float*>(ws + r * plan->bw_dx_bytes); };
    auto dw_part = [&](int r) { return reinterpret_cast<float*>(ws + plan->bw_off_dw + r * plan->bw_dw_bytes); };

    if (ways == 2) {
        // W_r = [W_{r,0}; W_{r,1}] by rows.  dX_r = dY_r W_{r,r} + dY_{1-r} W_{r,1-r}.
        g.nprob = 2; g.M = mr; g.N = kh; g.K = nh;
        for (int r = 0; r < 2; ++r)     // the product with the peer's dY half -> partial
            g.p[r] = {dy_sh[1 - r], w_sh[r] + (1 - r) * wblock, dx_part(r), nullptr, nullptr, nh, kh, kh, 0};
        if (!launch(jg::kGemmNN, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
        for (int r = 0; r < 2; ++r)     // the product with the rank's own dY half, on top of it
            g.p[r] = {dy_sh[r], w_sh[r] + r * wblock, dx_sh[r], dx_part(r), nullptr, nh, kh, kh, kh};
        if (!launch(jg::kGemmNN, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
        // dW_{r,c} = dY_c^T X_r: one product per block, four blocks in one launch
        g.nprob = 4; g.M = nh; g.N = kh; g.K = mr;
        for (int r = 0; r < 2; ++r)
            for (int cc = 0; cc < 2; ++cc)
                g.p[2 * r + cc] = {dy_sh[cc], x_sh[r], dw_sh[r] + cc * wblock, nullptr, nullptr, nh, kh, kh, 0};
        return launch(jg::kGemmTN, JG_KERNEL_GEMM_DW) ? JG_OK : JG_E_HIP;
    }

    // 4-way: block (row half i, column half j) lives on rank 2 i + j, for X, W, dY, dX and dW alike.
    auto rk = [](int a, int b) { return 2 * a + b; };
    // dX_(i,j) = dY_(i,0) W_(0,j) + dY_(i,1) W_(1,j); the rank's own dY block is dY_(i,j)
    g.nprob = 4; g.M = mr; g.N = kh; g.K = nh;
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {   // the term with the row neighbour's dY block -> partial
            const int r = rk(i, j), cc = 1 - j;
            g.p[r] = {dy_sh[rk(i, cc)], w_sh[rk(cc, j)], dx_part(r), nullptr, nullptr, nh, kh, kh, 0};
        }
    if (!launch(jg::kGemmNN, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {   // the term with the rank's own dY block, on top of it
            const int r = rk(i, j), cc = j;
            g.p[r] = {dy_sh[rk(i, cc)], w_sh[rk(cc, j)], dx_sh[r], dx_part(r), nullptr, nh, kh, kh, kh};
        }
    if (!launch(jg::kGemmNN, JG_KERNEL_GEMM_DX)) return JG_E_HIP;
    // dW_(c,j) = dY_(0,c)^T X_(0,j) + dY_(1,c)^T X_(1,j); rank (c,j) holds X_(c,j)
    g.M = nh; g.N = kh; g.K = mr;
    for (int cc = 0; cc < 2; ++cc)
        for (int j = 0; j < 2; ++j) {   // the term formed on the column neighbour (row half 1 - c) -> partial
            const int r = rk(cc, j), i = 1 - cc;
            g.p[r] = {dy_sh[rk(i, cc)], x_sh[rk(i, j)], dw_part(r), nullptr, nullptr, nh, kh, kh, 0};
        }
    if (!launch(jg::kGemmTN, JG_KERNEL_GEMM_DW)) return JG_E_HIP;
    for (int cc = 0; cc < 2; ++cc)
        for (int j = 0; j < 2; ++j) {   // the term with the rank's own X block, on top of it
            const int r = rk(cc, j), i = cc;
            g.p[r] = {dy_sh[rk(i, cc)], x_sh[rk(i, j)], dw_sh[r], dw_part(r), nullptr, nh, kh, kh, kh};
        }
    return launch(jg::kGemmTN, JG_KERNEL_GEMM_DW) ? JG_OK : JG_E_HIP;
}

// jg_layernorm_forward.  copy16 (may be null): `ways` destinations for a bfloat16 copy of the output in the
// plan's X-shard format; *copied tells whether the kernel wrote them (it does when the rows fit its
// register-resident form; otherwise the caller converts the FP32 output).
// xb_sh / row_bias (may be null): `ways` destinations for x + row_bias[token] (FP32, shaped like X_r); row_bias is a
// device vector over all rows of X.
static int layernorm_impl(const jg_plan* plan, const float* const* x_sh, const float* gamma, const float* beta,
                          double eps, float* const* out_sh, uint16_t* const* copy16, bool* copied,
                          float* const* xb_sh = nullptr, const float* row_bias = nullptr)
{
    if (copied) *copied = false;
    if (!plan || !plan->ctx) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    if (int rc = check_ptr_array(x_sh, d.ways)) return rc;
    if (int rc = check_ptr_array(out_sh, d.ways)) return rc;
    if (!(eps >= 0.0)) return JG_E_DTYPE;
    if (!aligned(gamma, 4) || !aligned(beta, 4)) return JG_E_ALIGN;
    for (int r = 0; r < d.ways; ++r)
        if (!aligned(x_sh[r], 4) || !aligned(out_sh[r], 4)) return JG_E_ALIGN;
    jg_ctx* c = plan->ctx;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    jg::NormGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nblocks = d.ways;
    g.rows = (int)plan->xr;
    g.cols = (int)plan->xc;
    g.eps = eps;
    for (int r = 0; r < d.ways; ++r) {
        int64_t rb, cb;
        block_coords(d.ways, r, &rb, &cb);     // the channels are the columns of X: block cb of them
        g.b[r] = {x_sh[r], out_sh[r], gamma ? gamma + cb * plan->xc : nullptr, beta ? beta + cb * plan->xc : nullptr,
                  xb_sh ? xb_sh[r] : nullptr, xb_sh ? row_bias + rb * plan->xr : nullptr, nullptr};
    }
    if (copy16 && d.dtype != JG_F32 && jg::norm_rows_fit(g)) {
        g.planes16 = d.dtype == JG_BF16X3 ? 2 : 1;
        g.plane16 = (int)plan->plane;
        for (int r = 0; r < d.ways; ++r) g.b[r].y16 = copy16[r];
        if (copied) *copied = true;
    }
    ScopedTimer t(c, JG_KERNEL_NORM);
    return HIP_OK(jg::launch_norm_group(g, c->stream)) ? JG_OK : JG_E_HIP;
}

// add_sh (or nullptr): per rank a block shaped like X_r that is added to dX_r before its rounding
static int layernorm_backward_impl(const jg_plan* plan, const float* const* x_sh, const float* gamma, double eps,
                                   const float* const* dy_sh, float* const* dx_sh, float* dgamma, float* dbeta,
                                   void* workspace, size_t workspace_bytes, const float* const* add_sh)
{
    if (!plan || !plan->ctx) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    if (int rc = check_ptr_array(x_sh, d.ways)) return rc;
    if (int rc = check_ptr_array(dy_sh, d.ways)) return rc;
    if (int rc = check_ptr_array(dx_sh, d.ways)) return rc;
    if (add_sh) {
        if (int rc = check_ptr_array(add_sh, d.ways)) return rc;
        for (int r = 0; r < d.ways; ++r)
            if (!aligned(add_sh[r], 4)) return JG_E_ALIGN;
    }
    if (!(eps >= 0.0)) return JG_E_DTYPE;
    if (!aligned(gamma, 4) || !aligned(dgamma, 4) || !aligned(dbeta, 4)) return JG_E_ALIGN;
    for (int r = 0; r < d.ways; ++r)
        if (!aligned(x_sh[r], 4) || !aligned(dy_sh[r], 4) || !aligned(dx_sh[r], 4)) return JG_E_ALIGN;
    const size_t stats_bytes = round_up(16 * (size_t)plan->xr, kWsAlign);
    if (!workspace || workspace_bytes < stats_bytes * d.ways) return JG_E_WORKSPACE;
    if (!aligned(workspace, kWsAlign)) return JG_E_ALIGN;
    jg_ctx* c = plan->ctx;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    jg::NormBwdGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nblocks = d.ways;
    g.rows = (int)plan->xr;
    g.cols = (int)plan->xc;
    g.eps = eps;
    double* stats[4] = {nullptr, nullptr, nullptr, nullptr};
    for (int r = 0; r < d.ways; ++r) {
        int64_t rb, cb;
        block_coords(d.ways, r, &rb, &cb);
        stats[r] = reinterpret_cast<double*>(static_cast<char*>(workspace) + r * stats_bytes);
        g.b[r] = {x_sh[r], dy_sh[r], dx_sh[r], gamma ? gamma + cb * plan->xc : nullptr, stats[r],
                  add_sh ? add_sh[r] : nullptr};
    }
    // the channel blocks: one per rank (1-, 2-way), or per column of the 2 x 2 grid, summed over its two row halves
    jg::NormBwdColsGroup cg;
    std::memset(&cg, 0, sizeof(cg));
    cg.rows = (int)plan->xr;
    cg.cols = (int)plan->xc;
    if (dgamma || dbeta) {
        cg.nout = d.ways == 4 ? 2 : d.ways;
        for (int j = 0; j < cg.nout; ++j) {
            jg::NormBwdColsOut& o = cg.o[j];
            o.nsrc = d.ways == 4 ? 2 : 1;
            for (int b = 0; b < o.nsrc; ++b) {
                const int r = d.ways == 4 ? 2 * b + j : j;
                o.x[b] = x_sh[r];
                o.dy[b] = dy_sh[r];
                o.stats[b] = stats[r];
                o.src_block[b] = r;
            }
            o.dgamma = dgamma ? dgamma + (int64_t)j * plan->xc : nullptr;
            o.dbeta = dbeta ? dbeta + (int64_t)j * plan->xc : nullptr;
        }
    }
    // behind the rows' statistics: room for the column sums' partial results, used when it is there
    char* part = static_cast<char*>(workspace) + stats_bytes * d.ways;
    const size_t part_bytes = workspace_bytes - stats_bytes * d.ways;
    ScopedTimer t(c, JG_KERNEL_NORM);
    return HIP_OK(jg::launch_norm_bwd(g, cg, c->stream, part, part_bytes)) ? JG_OK : JG_E_HIP;
}

int jg_layernorm_backward(const jg_plan* plan, const float* const* x_sh, const float* gamma, double eps,
                          const float* const* dy_sh, float* const* dx_sh, float* dgamma, float* dbeta, void* workspace,
                          size_t workspace_bytes)
{
    return layernorm_backward_impl(plan, x_sh, gamma, eps, dy_sh, dx_sh, dgamma, dbeta, workspace, workspace_bytes,
                                   nullptr);
}

int jg_bias_backward(const jg_plan* plan, const float* const* dy_sh, float* const* db_sh, void* workspace,
                     size_t workspace_bytes)
{
    if (!plan || !plan->ctx) return JG_E_NULL;
    const jg_linear_desc& d = plan->d;
    if (int rc = check_ptr_array(dy_sh, d.ways)) return rc;
    if (int rc = check_ptr_array(db_sh, d.ways)) return rc;
    for (int r = 0; r < d.ways; ++r)
        if (!aligned(dy_sh[r], 4) || !aligned(db_sh[r], 4)) return JG_E_ALIGN;
    jg_ctx* c = plan->ctx;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    jg::ColSumGroup g;
    std::memset(&g, 0, sizeof(g));
    g.rows = (int)plan->yr;
    g.cols = (int)plan->yc;
    if (d.ways == 4) {
        // column half j of dY is held as the two row blocks of ranks j and 2 + j, and both hold its bias slice
        g.nout = 2;
        for (int j = 0; j < 2; ++j) {
            g.o[j].nsrc = g.o[j].ndst = 2;
            g.o[j].src[0] = dy_sh[j];
            g.o[j].src[1] = dy_sh[2 + j];
            g.o[j].dst[0] = db_sh[j];
            g.o[j].dst[1] = db_sh[2 + j];
        }
    } else {
        g.nout = d.ways;
        for (int r = 0; r < d.ways; ++r) {
            g.o[r].nsrc = g.o[r].ndst = 1;
            g.o[r].src[0] = dy_sh[r];
            g.o[r].dst[0] = db_sh[r];
        }
    }
    if (workspace && !aligned(workspace, 8)) return JG_E_ALIGN;
    ScopedTimer t(c, JG_KERNEL_REDUCE);
    return HIP_OK(jg::launch_colsum_group(g, c->stream, workspace, workspace ? workspace_bytes : 0)) ? JG_OK : JG_E_HIP;
}

int jg_layernorm_forward(const jg_plan* plan, const float* const* x_sh, const float* gamma, const float* beta,
                         double eps, float* const* out_sh)
{
    return layernorm_impl(plan, x_sh, gamma, beta, eps, out_sh, nullptr, nullptr);
}

// X [M x C] -> H [M x Hd] -> Y [M x C]: the second layer maps back to the first one's input width
static int check_mlp_chain(const jg_plan* first, const jg_plan* second)
{
    if (!first || !second) return JG_E_NULL;
    const jg_linear_desc &a = first->d, &b = second->d;
    if (a.op != JG_OP_XWT || b.op != JG_OP_XWT) return JG_E_DTYPE;
    if (a.dtype != b.dtype) return JG_E_DTYPE;
    if (a.ways != b.ways) return JG_E_WAYS;
    if (a.M != b.M || a.N != b.K || b.N != a.K) return JG_E_SHAPE;
    if (first->ctx != second->ctx) return JG_E_NULL;
    return JG_OK;
}

// The two layers of an MLP chain.  in_sh: the first layer's input activations as FP32 shards (xr x xc, dense).
// FP32 plans: two calls of the layer, H handed on in place.  Reduced-precision plans: the first layer's input is
// rounded into the workspace in the format its products read (the conversion jg_shard applies to X); the launch
// that writes H also writes it rounded, in the second layer's format (fused combine), or H is converted like the
// input (separate combine).  Workspace: [0, ws1) layer 1, [ws1, ws1 + chain1) its rounded input, then from
// max(ws1 + chain1, ws2) the rounded H; layer 2 works in [0, ws2).
static size_t chain_h16_offset(const jg_plan* first, const jg_plan* second)
{
    const size_t a = first->ws_bytes + first->chain_bytes;
    return a > second->ws_bytes ? a : second->ws_bytes;
}

static int convert_shards(const jg_plan* plan, const float* const* in_sh, char* dst, const float** conv)
{
    const jg_linear_desc& d = plan->d;
    jg_ctx* c = plan->ctx;
    jg::CvtGroup cv;
    std::memset(&cv, 0, sizeof(cv));
    cv.nblocks = d.ways;
    cv.rows = (int)plan->xr;
    cv.cols = (int)plan->xc;
    cv.planes = d.dtype == JG_BF16X3 ? 2 : 1;
    cv.plane = (int)plan->plane;
    for (int r = 0; r < d.ways; ++r) {
        if (!aligned(in_sh[r], 4)) return JG_E_ALIGN;
        cv.b[r] = {in_sh[r], reinterpret_cast<uint16_t*>(dst + r * plan->chain_shard_bytes), plan->xc};
        conv[r] = reinterpret_cast<const float*>(dst + r * plan->chain_shard_bytes);
    }
    ScopedTimer t(c, JG_KERNEL_SHARD);
    return HIP_OK(jg::launch_cvt_group(cv, c->stream)) ? JG_OK : JG_E_HIP;
}

// Checks of a reduced-precision chain's workspace (the FP32 chain's are those of its layers).
static int check_chain_workspace(const jg_plan* first, const jg_plan* second, void* workspace, size_t workspace_bytes)
{
    if (first->d.dtype == JG_F32) return JG_OK;
    if (!workspace || workspace_bytes < chain_h16_offset(first, second) + second->chain_bytes) return JG_E_WORKSPACE;
    return aligned(workspace, kWsAlign) ? JG_OK : JG_E_ALIGN;
}

// input_converted: the first layer's rounded input is in place already (the layer norm wrote it).
static int run_chain(const jg_plan* first, const jg_plan* second, const float* const* in_sh, const float* const* x_sh,
                     const float* const* w1_sh, const float* const* b1_sh, const float* const* w2_sh,
                     const float* const* b2_sh, float* const* h_sh, float* const* y_sh, void* workspace,
                     size_t workspace_bytes, bool input_converted)
{
    if (first->d.dtype == JG_F32) {
        // H_r is written by the first layer in the partition the second one reads its input in
        int rc = forward_impl(first, in_sh, w1_sh, b1_sh, nullptr, JG_ACT_GELU, h_sh, workspace, workspace_bytes, nullptr);
        if (rc != JG_OK) return rc;
        return forward_impl(second, h_sh, w2_sh, b2_sh, x_sh, JG_ACT_NONE, y_sh, workspace, workspace_bytes, nullptr);
    }
    const int ways = first->d.ways;
    if (int rc = check_ptr_array(in_sh, ways)) return rc;
    const size_t off_h16 = chain_h16_offset(first, second);
    if (int rc = check_chain_workspace(first, second, workspace, workspace_bytes)) return rc;
    jg_ctx* c = first->ctx;
    if (!c) return JG_E_NULL;
    if (!HIP_OK(use_device(c->device))) return JG_E_HIP;
    char* ws = static_cast<char*>(workspace);
    const float* x16[4] = {nullptr, nullptr, nullptr, nullptr};
    const float* h16[4] = {nullptr, nullptr, nullptr, nullptr};
    if (input_converted) {
        for (int r = 0; r < ways; ++r)
            x16[r] = reinterpret_cast<const float*>(ws + first->ws_bytes + r * first->chain_shard_bytes);
    } else if (int rc = convert_shards(first, in_sh, ws + first->ws_bytes, x16)) {
        return rc;
    }
    const bool fused = first->d.combine == JG_COMBINE_FUSED;
    jg::HbCopy16 copy;
    std::memset(&copy, 0, sizeof(copy));
    copy.planes = second->d.dtype == JG_BF16X3 ? 2 : 1;
    copy.plane = (int)second->plane;
    copy.ld = copy.plane * copy.planes;
    for (int r = 0; r < ways; ++r) {
        copy.dst[r] = reinterpret_cast<uint16_t*>(ws + off_h16 + r * second->chain_shard_bytes);
        h16[r] = reinterpret_cast<const float*>(copy.dst[r]);
    }
    int rc = forward_impl(first, x16, w1_sh, b1_sh, nullptr, JG_ACT_GELU, h_sh, workspace, workspace_bytes,
                          fused ? &copy : nullptr);
    if (rc != JG_OK) return rc;
    if (!fused) {
        if (int rc2 = convert_shards(second, h_sh, ws + off_h16, h16)) return rc2;
    }
    return forward_impl(second, h16, w2_sh, b2_sh, x_sh, JG_ACT_NONE, y_sh, workspace, workspace_bytes, nullptr);
}

int jg_mixing_forward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                      const float* beta, double eps, const float* const* w1_sh, const float* const* b1_sh,
                      const float* const* w2_sh, const float* const* b2_sh, float* const* xn_sh,
                      float* const* h_sh, float* const* y_sh, void* workspace, size_t workspace_bytes)
{
    if (int rc = check_mlp_chain(first, second)) return rc;
    if (int rc = check_ptr_array(h_sh, first->d.ways)) return rc;
    if (int rc = check_chain_workspace(first, second, workspace, workspace_bytes)) return rc;
    // a reduced-precision chain: the norm writes its output a second time, rounded, where the first layer reads it
    uint16_t* x16[4] = {nullptr, nullptr, nullptr, nullptr};
    const bool reduced = first->d.dtype != JG_F32;
    if (reduced)
        for (int r = 0; r < first->d.ways; ++r)
            x16[r] = reinterpret_cast<uint16_t*>(static_cast<char*>(workspace) + first->ws_bytes +
                                                 r * first->chain_shard_bytes);
    bool copied = false;
    int rc = layernorm_impl(first, x_sh, gamma, beta, eps, xn_sh, reduced ? x16 : nullptr, &copied);
    if (rc != JG_OK) return rc;
    return run_chain(first, second, xn_sh, x_sh, w1_sh, b1_sh, w2_sh, b2_sh, h_sh, y_sh, workspace, workspace_bytes,
                     copied);
}

int jg_mlp_forward(const jg_plan* first, const jg_plan* second, const float* const* x_sh,
                   const float* const* w1_sh, const float* const* b1_sh, const float* const* w2_sh,
                   const float* const* b2_sh, float* const* h_sh, float* const* y_sh, void* workspace,
                   size_t workspace_bytes)
{
    if (int rc = check_mlp_chain(first, second)) return rc;
    if (int rc = check_ptr_array(h_sh, first->d.ways)) return rc;
    return run_chain(first, second, x_sh, x_sh, w1_sh, b1_sh, w2_sh, b2_sh, h_sh, y_sh, workspace, workspace_bytes,
                     false);
}

// (reduced precision: the recomputed forward reads X and W1 rounded, behind the first plan's own forward workspace)
static size_t mlp_backward_w16_bytes(const jg_plan* first)
{
    if (first->d.dtype == JG_F32) return 0;
    const size_t rows = first->d.op == JG_OP_XTW ? first->wc : first->wr;      // (contraction-major shards: wc rows)
    return round_up(4 * rows * (size_t)first->xcp, kWsAlign);
}

static size_t mlp_backward_workspace(const jg_plan* first, const jg_plan* second)
{
    size_t need = first->ws_bytes + first->chain_bytes + mlp_backward_w16_bytes(first) * first->d.ways;
    if (first->bw_ws_bytes > need) need = first->bw_ws_bytes;
    if (second->bw_ws_bytes > need) need = second->bw_ws_bytes;
    return need;
}

// with_skip: dX = dY + dA W1 (the MLP with its skip connection); otherwise dx_sh receives dA W1 alone
static int mlp_backward_impl(const jg_plan* first, const jg_plan* second, const float* const* x_sh,
                             const float* const* w1_sh, const float* const* b1_sh, const float* const* w2_sh,
                             const float* const* h_sh, const float* const* dy_sh, float* const* a_sh,
                             float* const* dh_sh, float* const* da_sh, float* const* dx_sh, float* const* dw1_sh,
                             float* const* db1_sh, float* const* dw2_sh, float* const* db2_sh, void* workspace,
                             size_t workspace_bytes, bool with_skip)
{
    if (int rc = check_mlp_chain(first, second)) return rc;
    const int ways = first->d.ways;
    const bool reduced = first->d.dtype != JG_F32;
    for (float* const* arr : {a_sh, dh_sh, da_sh, db1_sh, db2_sh})
        if (int rc = check_ptr_array(arr, ways)) return rc;
    const size_t need = mlp_backward_workspace(first, second);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return JG_E_WORKSPACE;
        if (!aligned(workspace, kWsAlign)) return JG_E_ALIGN;
    }
    jg_ctx* c = first->ctx;
    // second layer: dH = dY W2, dW2 = dY^T H, db2 = column sums of dY
    int rc = jg_linear_backward(second, h_sh, w2_sh, dy_sh, dh_sh, dw2_sh, workspace, workspace_bytes);
    if (rc != JG_OK) return rc;
    rc = jg_bias_backward(second, dy_sh, db2_sh, workspace, workspace_bytes);
    if (rc != JG_OK) return rc;
    // the pre-activation, which the forward does not keep: A = X W1^T + b1 once more (mixed precision: from the
    // FP32 X and W1 this call is given, rounded as the forward rounds them)
    const float* const* a_x = x_sh;
    const float* const* a_w = w1_sh;
    const float* x16[4];
    const float* w16[4];
    if (reduced) {
        if (int rc1 = check_ptr_array(x_sh, ways)) return rc1;
        if (int rc1 = check_ptr_array(w1_sh, ways)) return rc1;
        char* ws = static_cast<char*>(workspace);
        if (int rc1 = convert_shards(first, x_sh, ws + first->ws_bytes, x16)) return rc1;
        const size_t wbytes = mlp_backward_w16_bytes(first);
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = ways;
        cv.rows = (int)first->wr;
        cv.cols = (int)first->wc;
        cv.planes = first->d.dtype == JG_BF16X3 ? 2 : 1;
        cv.plane = (int)first->plane;
        for (int r = 0; r < ways; ++r) {
            if (!aligned(w1_sh[r], 4)) return JG_E_ALIGN;
            char* dst = ws + first->ws_bytes + first->chain_bytes + r * wbytes;
            cv.b[r] = {w1_sh[r], reinterpret_cast<uint16_t*>(dst), first->wc};
            w16[r] = reinterpret_cast<const float*>(dst);
        }
        {
            ScopedTimer t(c, JG_KERNEL_SHARD);
            if (!HIP_OK(jg::launch_cvt_group(cv, c->stream))) return JG_E_HIP;
        }
        a_x = x16;
        a_w = w16;
    }
    rc = forward_impl(first, a_x, a_w, b1_sh, nullptr, JG_ACT_NONE, a_sh, workspace, workspace_bytes, nullptr);
    if (rc != JG_OK) return rc;
    // dA = dH * gelu'(A)
    {
        jg::ActBwdGroup ag;
        std::memset(&ag, 0, sizeof(ag));
        ag.nblocks = ways;
        ag.n = (int64_t)first->yr * first->yc;
        for (int r = 0; r < ways; ++r) {
            if (!aligned(a_sh[r], 4) || !aligned(dh_sh[r], 4) || !aligned(da_sh[r], 4)) return JG_E_ALIGN;
            ag.b[r] = {a_sh[r], dh_sh[r], da_sh[r]};
        }
        ScopedTimer t(c, JG_KERNEL_COMBINE);
        if (!HIP_OK(jg::launch_act_bwd_group(ag, c->stream))) return JG_E_HIP;
    }
    // first layer: dA W1 (into dx_sh), dW1 = dA^T X, db1 = column sums of dA
    rc = jg_linear_backward(first, x_sh, w1_sh, da_sh, dx_sh, dw1_sh, workspace, workspace_bytes);
    if (rc != JG_OK) return rc;
    rc = jg_bias_backward(first, da_sh, db1_sh, workspace, workspace_bytes);
    if (rc != JG_OK || !with_skip) return rc;
    // the skip connection: dX = dY + dA W1 (dY_r and dX_r are both shaped like X_r)
    jg::CombineGroup cb;
    std::memset(&cb, 0, sizeof(cb));
    cb.nblocks = ways;
    cb.rows = (int)first->xr;
    cb.cols = (int)first->xc;
    cb.act = jg::kActNone;
    for (int r = 0; r < ways; ++r) cb.b[r] = {dx_sh[r], dy_sh[r], nullptr, dx_sh[r], nullptr};
    ScopedTimer t(c, JG_KERNEL_COMBINE);
    return HIP_OK(jg::launch_combine_group(cb, c->stream)) ? JG_OK : JG_E_HIP;
}

int jg_mlp_backward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* const* w1_sh,
                    const float* const* b1_sh, const float* const* w2_sh, const float* const* h_sh,
                    const float* const* dy_sh, float* const* a_sh, float* const* dh_sh, float* const* da_sh,
                    float* const* dx_sh, float* const* dw1_sh, float* const* db1_sh, float* const* dw2_sh,
                    float* const* db2_sh, void* workspace, size_t workspace_bytes)
{
    return mlp_backward_impl(first, second, x_sh, w1_sh, b1_sh, w2_sh, h_sh, dy_sh, a_sh, dh_sh, da_sh, dx_sh, dw1_sh,
                             db1_sh, dw2_sh, db2_sh, workspace, workspace_bytes, true);
}

int jg_mixing_backward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                       double eps, const float* const* xn_sh, const float* const* w1_sh, const float* const* b1_sh,
                       const float* const* w2_sh, const float* const* h_sh, const float* const* dy_sh,
                       float* const* a_sh, float* const* dh_sh, float* const* da_sh, float* const* dxn_sh,
                       float* const* dx_sh, float* const* dw1_sh, float* const* db1_sh, float* const* dw2_sh,
                       float* const* db2_sh, float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes)
{
    if (int rc = check_mlp_chain(first, second)) return rc;
    if (int rc = check_ptr_array(dxn_sh, first->d.ways)) return rc;
    size_t need = mlp_backward_workspace(first, second);
    const size_t stats = round_up(16 * (size_t)first->xr, kWsAlign) * first->d.ways;
    if (stats > need) need = stats;
    if (!workspace || workspace_bytes < need) return JG_E_WORKSPACE;
    // the MLP on Xn, without a skip connection of its own: dXn = dA W1
    int rc = mlp_backward_impl(first, second, xn_sh, w1_sh, b1_sh, w2_sh, h_sh, dy_sh, a_sh, dh_sh, da_sh, dxn_sh,
                               dw1_sh, db1_sh, dw2_sh, db2_sh, workspace, workspace_bytes, false);
    if (rc != JG_OK) return rc;
    // the norm's backward, with the block's skip connection added before dX is rounded
    return layernorm_backward_impl(first, x_sh, gamma, eps, dxn_sh, dx_sh, dgamma, dbeta, workspace, workspace_bytes,
                                   dy_sh);
}

// X [T x C] -> H [C x D] (transposed layer) -> Y [T x C] (plain layer, W2 in the activations' place, H in the weights')
static int check_token_chain(const jg_plan* first, const jg_plan* second)
{
    if (!first || !second) return JG_E_NULL;
    const jg_linear_desc &a = first->d, &b = second->d;
    if (a.op != JG_OP_XTW || b.op != JG_OP_XWT) return JG_E_DTYPE;
    if (a.dtype != b.dtype) return JG_E_DTYPE;
    if (a.ways != b.ways) return JG_E_WAYS;
    // first: K = T, M = C, N = D; second: M = T, K = D, N = C
    if (a.K != b.M || a.M != b.N || a.N != b.K) return JG_E_SHAPE;
    if (b.has_bias) return JG_E_DTYPE;      // the second layer's bias goes with the token: it is b2, not a column bias
    if (first->ctx != second->ctx) return JG_E_NULL;
    return JG_OK;
}

int jg_token_mixing_forward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                            const float* beta, double eps, const float* const* w1_sh, const float* const* b1_sh,
                            const float* const* w2_sh, const float* b2, float* const* xn_sh, float* const* h_sh,
                            float* const* y_sh, void* workspace, size_t workspace_bytes)
{
    if (int rc = check_token_chain(first, second)) return rc;
    const int ways = first->d.ways;
    const bool reduced = first->d.dtype != JG_F32;
    if (int rc = check_ptr_array(h_sh, ways)) return rc;
    if (int rc = check_ptr_array(x_sh, ways)) return rc;
    if (int rc = check_ptr_array(xn_sh, ways)) return rc;
    if (!aligned(b2, 4)) return JG_E_ALIGN;
    // workspace: [the layers' own, shared] [X + b2, FP32] [mixed precision: Xn rounded, contraction-major] [H rounded]
    const size_t base = first->ws_bytes > second->ws_bytes ? first->ws_bytes : second->ws_bytes;
    const size_t shard = round_up(4 * (size_t)first->xr * (size_t)first->xc, kWsAlign);
    const size_t off_x16 = base + (b2 ? shard * ways : 0);
    const size_t h16_shard = reduced ? round_up(4 * (size_t)second->wr * (size_t)second->xcp, kWsAlign) : 0;
    const size_t off_h16 = off_x16 + first->chain_bytes;
    const size_t need = off_h16 + h16_shard * ways;
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return JG_E_WORKSPACE;
        if (!aligned(workspace, kWsAlign)) return JG_E_ALIGN;
    }
    char* ws = static_cast<char*>(workspace);
    // the skip connection carries the second layer's per-token bias: the norm, which reads X anyway, also writes
    // X + b2[token] for it
    float* xb[4] = {nullptr, nullptr, nullptr, nullptr};
    const float* res[4];
    for (int r = 0; r < ways; ++r) {
        if (b2) xb[r] = reinterpret_cast<float*>(ws + base + r * shard);
        res[r] = b2 ? xb[r] : x_sh[r];
    }
    int rc = layernorm_impl(first, x_sh, gamma, beta, eps, xn_sh, nullptr, nullptr, b2 ? xb : nullptr, b2);
    if (rc != JG_OK) return rc;
    const float* const* first_in = xn_sh;
    const float* const* second_w = h_sh;
    const float* xn16[4];
    const float* h16[4];
    jg_ctx* c = first->ctx;
    if (reduced) {
        // the first layer reads Xn rounded and contraction-major: the transposing conversion of the shard step
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = ways;
        cv.rows = (int)first->xr;
        cv.cols = (int)first->xc;
        cv.planes = first->d.dtype == JG_BF16X3 ? 2 : 1;
        cv.plane = (int)first->plane;
        for (int r = 0; r < ways; ++r) {
            char* dst = ws + off_x16 + r * first->chain_shard_bytes;
            cv.b[r] = {xn_sh[r], reinterpret_cast<uint16_t*>(dst), first->xc};
            xn16[r] = reinterpret_cast<const float*>(dst);
        }
        ScopedTimer t(c, JG_KERNEL_SHARD);
        if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        first_in = xn16;
    }
    // H = gelu(Xn^T W1 + b1): [C x D], partitioned like the first plan's Y - which is how the second plan
    // partitions its weights
    rc = forward_impl(first, first_in, w1_sh, b1_sh, nullptr, JG_ACT_GELU, h_sh, workspace, workspace_bytes, nullptr);
    if (rc != JG_OK) return rc;
    if (reduced) {
        // the second layer reads H rounded, in its weight-shard format (rows of the contracted index already)
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = ways;
        cv.rows = (int)second->wr;
        cv.cols = (int)second->wc;
        cv.planes = second->d.dtype == JG_BF16X3 ? 2 : 1;
        cv.plane = (int)second->plane;
        for (int r = 0; r < ways; ++r) {
            if (!aligned(h_sh[r], 4)) return JG_E_ALIGN;
            char* dst = ws + off_h16 + r * h16_shard;
            cv.b[r] = {h_sh[r], reinterpret_cast<uint16_t*>(dst), second->wc};
            h16[r] = reinterpret_cast<const float*>(dst);
        }
        ScopedTimer t(c, JG_KERNEL_SHARD);
        if (!HIP_OK(jg::launch_cvt_group(cv, c->stream))) return JG_E_HIP;
        second_w = h16;
    }
    // Y = (X + b2) + W2 H^T: [T x C], partitioned like X
    return forward_impl(second, w2_sh, second_w, nullptr, res, JG_ACT_NONE, y_sh, workspace, workspace_bytes, nullptr);
}

int jg_token_mixing_backward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                             double eps, const float* const* xn_sh, const float* const* w1_sh,
                             const float* const* b1_sh, const float* const* w2_sh, const float* const* h_sh,
                             const float* const* dy_sh, float* const* a_sh, float* const* dh_sh, float* const* da_sh,
                             float* const* dxn_sh, float* const* dx_sh, float* const* dw1_sh, float* const* db1_sh,
                             float* const* dw2_sh, float* db2, float* dgamma, float* dbeta, void* workspace,
                             size_t workspace_bytes)
{
    if (int rc = check_token_chain(first, second)) return rc;
    const int ways = first->d.ways;
    const bool reduced = first->d.dtype != JG_F32;
    for (float* const* arr : {a_sh, dh_sh, da_sh, dxn_sh, db1_sh})
        if (int rc = check_ptr_array(arr, ways)) return rc;
    if (int rc = check_ptr_array(dy_sh, ways)) return rc;
    if (!aligned(db2, 4)) return JG_E_ALIGN;
    size_t need = mlp_backward_workspace(first, second);
    const size_t stats = round_up(16 * (size_t)first->xr, kWsAlign) * ways;
    if (stats > need) need = stats;
    if (!workspace || workspace_bytes < need) return JG_E_WORKSPACE;
    if (!aligned(workspace, kWsAlign)) return JG_E_ALIGN;
    jg_ctx* c = first->ctx;
    // second layer, W2 in the activations' place and H in the weights': its "dX" is dW2 = dY H, its "dW" is dH = dY^T W2
    int rc = jg_linear_backward(second, w2_sh, h_sh, dy_sh, dw2_sh, dh_sh, workspace, workspace_bytes);
    if (rc != JG_OK) return rc;
    if (db2) {
        // db2[t] = sum over the channels of dY[t][.]: the blocks of a token range side by side
        jg::RowSumGroup rg;
        std::memset(&rg, 0, sizeof(rg));
        rg.rows = (int)first->xr;
        rg.cols = (int)first->xc;
        rg.nout = ways == 4 ? 2 : 1;
        for (int i = 0; i < rg.nout; ++i) {
            rg.o[i].nsrc = ways == 1 ? 1 : 2;
            for (int b = 0; b < rg.o[i].nsrc; ++b) {
                if (!aligned(dy_sh[2 * i + b], 4)) return JG_E_ALIGN;
                rg.o[i].src[b] = dy_sh[2 * i + b];
            }
            rg.o[i].dst = db2 + (int64_t)i * first->xr;
        }
        ScopedTimer t(c, JG_KERNEL_REDUCE);
        if (!HIP_OK(jg::launch_rowsum_group(rg, c->stream))) return JG_E_HIP;
    }
    // the pre-activation, which the forward does not keep: A = Xn^T W1 + b1 once more (mixed precision: from the FP32
    // Xn and W1 this call is given, rounded contraction-major as the forward's shard step does)
    const float* const* a_x = xn_sh;
    const float* const* a_w = w1_sh;
    const float* x16[4];
    const float* w16[4];
    if (reduced) {
        if (int rc1 = check_ptr_array(xn_sh, ways)) return rc1;
        if (int rc1 = check_ptr_array(w1_sh, ways)) return rc1;
        char* ws = static_cast<char*>(workspace);
        const size_t wbytes = mlp_backward_w16_bytes(first);
        jg::CvtGroup cv;
        std::memset(&cv, 0, sizeof(cv));
        cv.nblocks = ways;
        cv.planes = first->d.dtype == JG_BF16X3 ? 2 : 1;
        cv.plane = (int)first->plane;
        cv.rows = (int)first->xr;
        ScopedTimer t(c, JG_KERNEL_SHARD);
        cv.cols = (int)first->xc;
        for (int r = 0; r < ways; ++r) {
            if (!aligned(xn_sh[r], 4) || !aligned(w1_sh[r], 4)) return JG_E_ALIGN;
            char* dst = ws + first->ws_bytes + r * first->chain_shard_bytes;
            cv.b[r] = {xn_sh[r], reinterpret_cast<uint16_t*>(dst), first->xc};
            x16[r] = reinterpret_cast<const float*>(dst);
        }
        if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        cv.cols = (int)first->wc;
        for (int r = 0; r < ways; ++r) {
            char* dst = ws + first->ws_bytes + first->chain_bytes + r * wbytes;
            cv.b[r] = {w1_sh[r], reinterpret_cast<uint16_t*>(dst), first->wc};
            w16[r] = reinterpret_cast<const float*>(dst);
        }
        if (!HIP_OK(jg::launch_cvt_transposed_group(cv, c->stream))) return JG_E_HIP;
        a_x = x16;
        a_w = w16;
    }
    rc = forward_impl(first, a_x, a_w, b1_sh, nullptr, JG_ACT_NONE, a_sh, workspace, workspace_bytes, nullptr);
    if (rc != JG_OK) return rc;
    {   // dA = dH * gelu'(A)
        jg::ActBwdGroup ag;
        std::memset(&ag, 0, sizeof(ag));
        ag.nblocks = ways;
        ag.n = (int64_t)first->yr * first->yc;
        for (int r = 0; r < ways; ++r) {
            if (!aligned(a_sh[r], 4) || !aligned(dh_sh[r], 4) || !aligned(da_sh[r], 4)) return JG_E_ALIGN;
            ag.b[r] = {a_sh[r], dh_sh[r], da_sh[r]};
        }
        ScopedTimer t(c, JG_KERNEL_COMBINE);
        if (!HIP_OK(jg::launch_act_bwd_group(ag, c->stream))) return JG_E_HIP;
    }
    // transposed layer: dXn = W1 dA^T, dW1 = Xn dA, db1 = column sums of dA
    rc = jg_linear_backward(first, xn_sh, w1_sh, da_sh, dxn_sh, dw1_sh, workspace, workspace_bytes);
    if (rc != JG_OK) return rc;
    rc = jg_bias_backward(first, da_sh, db1_sh, workspace, workspace_bytes);
    if (rc != JG_OK) return rc;
    // the norm's backward, with the block's skip connection added before dX is rounded
    return layernorm_backward_impl(first, x_sh, gamma, eps, dxn_sh, dx_sh, dgamma, dbeta, workspace, workspace_bytes,
                                   dy_sh);
}

}  // extern "C"

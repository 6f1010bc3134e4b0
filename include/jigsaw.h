/*
 * libjigsaw - forward pass of a Jigsaw-partitioned linear layer on one AMD MI355X (gfx950).
 *
 * The operation (Sec. 4 of the Jigsaw paper): a linear layer is the product
 *     Y = X W^T (+ b),   X: M x K activations,  W: N x K weights,  Y: M x N,
 * and in an n-way parallel model every rank holds 1/n of X, of W and of Y, with no
 * all-gather or broadcast of parameters (Sec. 4, "zero memory redundancy").
 *
 *   ways = 1   the unpartitioned layer (the paper's 1-way baseline, Sec. 6.2.1).
 *   ways = 2   Sec. 4.1, Eqs. (1)-(2): X and W are split on the last (channel)
 *              dimension, X = [X_0, X_1], W = [W_0, W_1]; rank r splits its W_r by
 *              rows into W_{r,0}, W_{r,1}, keeps X_r W_{r,r}^T, ships X_r W_{r,1-r}^T
 *              to the other rank, and ends with Y_r = Y[:, r-th half of N].
 *   ways = 4   Sec. 4.2, Eqs. (3)-(4): X, W (and Y) are split 2 x 2 on the last two
 *              dimensions, blocks numbered row-major.  Rank r forms two block
 *              products; one partial product and one weight block are handed to a
 *              peer, and Y_r sits where X_r sat.
 *
 * The transposed layer (Sec. 5: a forward pass defined by X^T W, which removes the
 * transpose of the [tokens, channels] tensor before the token-mixing MLP of Sec. 3):
 *     Y = X^T W (+ b),   X: K x M ([tokens, channels]),  W: K x N,  Y: M x N,
 * selected by op = JG_OP_XTW.  The paper names this permutation and says that it has
 * its own exchange pattern, but prints no equations; this library keeps the rules of
 * Sec. 4 (split on the last dimension, 2 x 2 blocks row-major, nothing duplicated,
 * two block products per rank, one partial handed to one peer):
 *   ways = 2   X_r = X[:, r], W_r = W[:, r], Y_r = Y[:, r] = [X_0^T W_r ; X_1^T W_r].  The
 *              contraction is not split, so nothing is summed across ranks: rank r
 *              gets the peer's activation block and fills both row halves of Y_r.
 *   ways = 4   block (i, j) on rank 2 i + j.  Rank (i, j) multiplies its W_(i,j) with its
 *              own X_(i,j) (a term of Y block (j, j)) and with X_(i,1-j) received from
 *              rank (i, 1-j) (a term of Y block (1-j, j)); it keeps the term of the
 *              block it owns (row half i) and hands the other to rank (1-i, j).
 *
 * The third permutation Sec. 5 names, Y = X W (+ b) with the weights stored along the contracted index
 * (X: M x K, W: K x N), selected by op = JG_OP_XW.  It is the form of the backward product dX = dY W of
 * Sec. 4.1 and takes that pass's blocks: all tensors split on their last dimension (2-way: X_r = X[:, r-th half
 * of K], W_r = W[:, r-th half of N] with all K rows, Y_r = Y[:, r-th half of N]) or 2 x 2 (4-way), and
 *     Y_(i,j) = X_(i,j) W_(j,j) + X_(i,1-j) W_(1-j,j)      (W_(k,c): rows k-th half of K, columns c-th half of N),
 * both products formed by the block's owner, which gets the activation block of its row neighbour and (4-way)
 * the weight block of its column neighbour.  Its own gradients are the other two permutations (dX = dY W^T,
 * dW = X^T dY), which jg_linear_backward runs on the same shards.
 *
 * All n ranks of one layer are "virtual ranks" resident on the one GPU: each has its
 * own shard buffers, and a hand-off to a peer is a store into the peer's buffer.
 *
 * Conventions
 *  - Every function returns JG_OK (0) or a negative jg_status.  Nothing throws,
 *    aborts or prints.
 *  - All matrices are dense row-major FP32.  "device" pointers are HIP device
 *    addresses owned by the caller (e.g. PyTorch tensors); "host" pointers are
 *    ordinary host memory.  The library allocates no device memory.
 *  - Shard arguments are HOST arrays of `ways` DEVICE pointers, indexed by rank.
 *    A rank's shard is contiguous (leading dimension = its column count).
 *  - All GPU work is enqueued on the stream given to jg_init and is asynchronous;
 *    the library synchronises only in jg_profile_read.
 *  - Inputs are never written.  Outputs and workspace must not overlap inputs.
 *  - Handles are host-heap objects freed only by the matching call; NULL is a no-op
 *    for the two release functions.  One jg_ctx per host thread.  A plan is
 *    immutable and reusable; concurrent forwards that share a workspace race.
 */
#ifndef JIGSAW_H
#define JIGSAW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct jg_ctx jg_ctx;
typedef struct jg_plan jg_plan;

typedef enum jg_status {
    JG_OK = 0,
    JG_E_NULL = -1,      /* a required pointer (handle, array, array element) is NULL   */
    JG_E_SHAPE = -2,     /* M, K, N <= 0, too large, or not divisible as `ways` needs   */
    JG_E_WAYS = -3,      /* ways not in {1, 2, 4}, or rank out of range                 */
    JG_E_DTYPE = -4,     /* unsupported dtype / op / option value                       */
    JG_E_WORKSPACE = -5, /* workspace NULL or smaller than JG_Q_WORKSPACE_BYTES         */
    JG_E_ALIGN = -6,     /* a device pointer is not 4-byte aligned, workspace not 256-B */
    JG_E_HIP = -7,       /* a HIP runtime call failed                                   */
    JG_E_ARCH = -8       /* the device is not gfx950                                    */
} jg_status;

enum { JG_OP_XWT = 0,                                    /* Y = X W^T (Sec. 4)          */
       JG_OP_XTW = 1,                                    /* Y = X^T W (Sec. 5) */
       JG_OP_XW = 2 };                                   /* Y = X W   (Sec. 5; FP32 only) */
enum { JG_F32 = 0,       /* the paper's uniform single precision (Sec. 6.1)                          */
       JG_BF16 = 1,      /* reduced precision (Sec. 6.1 trains in a mixed precision whose matrix units
                            round FP32 operands to a short mantissa and sum in FP32; this chip has no such
                            FP32-input mode): X and W are rounded to bfloat16 (nearest, ties to even) when
                            they are sharded, products are exact, sums FP32, Y and b stay FP32           */
       JG_BF16X3 = 2 };  /* the same with split operands x = hi + lo (both bfloat16): the product is
                            hi hi + hi lo + lo hi, 16 mantissa bits per operand at three times the
                            matrix work of JG_BF16                                                       */
enum { JG_COMBINE_FUSED = 0, JG_COMBINE_SEPARATE = 1 };  /* where the "+" of Eq. (2)/(4) runs */
enum { JG_WEIGHTS_COPY = 0, JG_WEIGHTS_DIRECT = 1 };     /* 4-way weight-block hand-off */
enum { JG_TAIL_SPLIT = 0, JG_TAIL_WHOLE = 1 };           /* last partial round of a GEMM launch */
enum { JG_ACC_LEVELS = 0,   /* reduced precision: long contractions are summed in two levels (chunks of K, one launch each) */
       JG_ACC_SINGLE = 1 }; /* ... or in one level, for data known to be zero-mean                              */
enum { JG_ACT_NONE = 0, JG_ACT_GELU = 1 };               /* epilogue activation of jg_linear_forward_ex */
enum { JG_T_X = 0, JG_T_W = 1, JG_T_B = 2, JG_T_Y = 3,   /* tensor selector of jg_shard / jg_gather_as */
       JG_T_X_F32 = 4,    /* partitioned like X, stored in FP32 whatever the plan's dtype: the activations a
                             mixed-precision MLP chain takes, its skip connection, a layer norm's output */
       JG_T_W_F32 = 5 };  /* partitioned like W, stored in FP32 whatever the plan's dtype: the master copy of the
                             weights that a reduced-precision backward reads, and its dW */

typedef struct jg_linear_desc {
    int64_t M, K, N;     /* global sizes: Y is M x N and K is contracted.  JG_OP_XWT: X is
                            M x K, W is N x K.  JG_OP_XTW: X is K x M, W is K x N.
                            JG_OP_XW: X is M x K, W is K x N.                           */
    int32_t ways;        /* 1, 2 or 4                                                   */
    int32_t op;          /* JG_OP_XWT, JG_OP_XTW or JG_OP_XW                            */
    int32_t dtype;       /* JG_F32, or JG_BF16 / JG_BF16X3 (forward; backward of JG_OP_XWT, which
                            reads FP32 shards: see jg_linear_backward).  The X and W shards
                            are then bfloat16 arrays of JG_Q_X_SHARD_BYTES /
                            JG_Q_W_SHARD_BYTES bytes, 16-byte aligned, written by jg_shard.
                            JG_OP_XWT: every rank's share of K (K, or K / 2 for 2 and 4
                            ways) must be a multiple of 8; xr rows per shard, each row xc
                            values padded to a multiple of 64 (whole 128-byte lines; the
                            padding is never read), JG_BF16X3 every row as
                            [hi(0..xc) pad | lo(0..xc) pad].  JG_OP_XTW: any K; the shards
                            are stored contraction-major - xc (wc) rows of the rank's xr
                            tokens, padded likewise, zeros up to the next multiple of 8  */
    int32_t has_bias;    /* 0 / 1: b_r (the slice of b matching Y_r's columns) is added
                            once, by the rank that owns the output block                */
    int32_t combine;     /* JG_COMBINE_FUSED: the kept-product GEMM starts its accumulators
                            from the received partial.  JG_COMBINE_SEPARATE: the kept
                            product is written out and a streaming kernel adds the two
                            partials (for measurement).                                 */
    int32_t weights;     /* The operand block a rank needs from a peer (JG_OP_XWT: 4-way, a
                            weight block; JG_OP_XTW: 2- and 4-way, an activation block).
                            JG_WEIGHTS_COPY: the weight block a rank needs
                            from its peer (the terms of Eq. (4) in which only W^T is
                            bold) is copied into the workspace first, as a transfer
                            would deliver it.  JG_WEIGHTS_DIRECT: the peer's buffer is
                            read in place.                                              */
    int32_t tail;        /* JG_TAIL_SPLIT: when the tiles of a GEMM launch do not fill a whole
                            number of rounds of the chip's workgroup slots, the K loops of
                            the tiles of the last partial round are cut into equal runs, one
                            per slot, and a second small kernel adds each tile's runs in
                            ascending k order (no atomics: results do not vary from run to
                            run).  Needs JG_Q_TAIL_SCRATCH_BYTES more workspace.
                            JG_TAIL_WHOLE: one workgroup per tile throughout.           */
    int32_t accumulate;  /* Reduced-precision plans only (FP32 plans always sum in two levels inside the
                            kernel).  The bfloat16 kernels sum in one level: on operands of one sign a
                            running FP32 sum of K products drifts past 1e-6 of its magnitude from K of
                            about 1500 (500 with split operands).  JG_ACC_LEVELS (the default): a product
                            with a longer contraction is cut into chunks of K, one launch each, every launch
                            after the first adding on top of what the output holds - the second summation
                            level; results stay within 1e-6 of the magnitude on any data, at the price of
                            one more pass over the output per chunk.  JG_ACC_SINGLE: one launch whatever K;
                            for zero-mean data, whose running sums stay small (measured below 1e-7).     */
} jg_linear_desc;

typedef enum jg_query {
    JG_Q_WORKSPACE_BYTES = 0,    /* device bytes jg_linear_forward needs (rank ignored)        */
    JG_Q_FLOPS_TOTAL = 1,        /* 2 M K N: matmul dimensions only (Sec. 6.3 work model)      */
    JG_Q_FLOPS_RANK = 2,         /* one rank's two block products                              */
    JG_Q_HBM_BYTES_ALGO = 3,     /* 4(MK + NK + MN), plus 8 MN where a block's first product passes
                                    through a partial (written once and read once): ways >= 2,
                                    for JG_OP_XTW ways = 4 only                                */
    JG_Q_EXCHANGE_BYTES_RANK = 4,/* bytes a rank hands to its peers per forward                */
    JG_Q_X_ROWS = 5, JG_Q_X_COLS = 6,   /* shape of rank's X shard                             */
    JG_Q_W_ROWS = 7, JG_Q_W_COLS = 8,   /* shape of rank's W shard                             */
    JG_Q_Y_ROWS = 9, JG_Q_Y_COLS = 10,  /* shape of rank's Y shard                             */
    JG_Q_B_LEN = 11,                    /* length of rank's bias slice (= Y_COLS)              */
    JG_Q_RESIDENT_BYTES_RANK = 12,      /* bytes of X_r + W_r + Y_r (bias and workspace apart) */
    JG_Q_GEMM_LAUNCHES = 13,     /* GEMM kernel launches per forward (rank ignored)            */
    JG_Q_BACKWARD_WORKSPACE_BYTES = 14, /* device bytes jg_linear_backward needs (rank ignored)  */
    JG_Q_BACKWARD_FLOPS_TOTAL = 15,     /* 4 M K N: twice the forward (Sec. 6.3 work model)      */
    JG_Q_BACKWARD_GEMM_LAUNCHES = 16,   /* GEMM kernel launches per backward (rank ignored)      */
    JG_Q_TAIL_SCRATCH_BYTES = 17,       /* part of JG_Q_WORKSPACE_BYTES that JG_TAIL_SPLIT adds   */
    JG_Q_BACKWARD_TAIL_SCRATCH_BYTES = 18, /* the same for JG_Q_BACKWARD_WORKSPACE_BYTES          */
    JG_Q_X_SHARD_BYTES = 19,            /* bytes of the rank's X shard in the plan's dtype        */
    JG_Q_W_SHARD_BYTES = 20,            /* ... and of its W shard                                 */
    JG_Q_CHAIN_WORKSPACE_BYTES = 21,    /* the plan's share of the workspace of jg_mlp_forward /
                                           jg_mixing_forward: JG_Q_WORKSPACE_BYTES, plus (reduced
                                           precision) room for its input in bfloat16 (rank ignored) */
    JG_Q_X_F32_SHARDS_BYTES = 22,       /* `ways` FP32 shards shaped like X_r, each rounded up to 256
                                           bytes: what jg_token_mixing_forward needs for its skip
                                           connection when b2 is given (rank ignored)               */
    JG_Q_NORM_BACKWARD_WORKSPACE_BYTES = 23,  /* device bytes jg_layernorm_backward wants (rank ignored): the rows'
                                                 statistics, which it needs, and the partial column sums that let it
                                                 read x and dy once (or, for rows it cannot take that way, let its
                                                 dgamma / dbeta kernel use the whole chip)                             */
    JG_Q_BIAS_BACKWARD_WORKSPACE_BYTES = 24   /* device bytes that let jg_bias_backward use the whole chip (rank ignored) */
} jg_query;

typedef enum jg_kernel {         /* kernel classes for jg_profile_read */
    JG_KERNEL_GEMM = 0,          /* forward block-product GEMM (X W^T form)             */
    JG_KERNEL_WEIGHT_COPY = 1,   /* 4-way weight-block hand-off                         */
    JG_KERNEL_COMBINE = 2,       /* separate partial-sum combine                        */
    JG_KERNEL_SHARD = 3,
    JG_KERNEL_GATHER = 4,
    JG_KERNEL_GEMM_DX = 5,       /* backward dX = dY W products                          */
    JG_KERNEL_GEMM_DW = 6,       /* backward dW = dY^T X products                        */
    JG_KERNEL_JOIN = 7,          /* adds the runs of split tail tiles (JG_TAIL_SPLIT)    */
    JG_KERNEL_NORM = 8,          /* layer norm over a rank's channels                    */
    JG_KERNEL_REDUCE = 9,        /* column sums of dY (bias gradient)                    */
    JG_KERNEL_COUNT = 10
} jg_kernel;

/* init.  Creates a context bound to HIP device `device` and to `hip_stream`
 * (a hipStream_t passed as void*; NULL = the device's default stream).  The stream
 * stays owned by the caller and must outlive the context.
 * Errors: JG_E_NULL (out), JG_E_HIP (bad device), JG_E_ARCH (not gfx950). */
int jg_init(jg_ctx** out, int device, void* hip_stream);

/* free.  Releases the context (not the stream).  Plans made with it that are still alive are detached: they
 * keep answering jg_plan_query, their data calls return JG_E_NULL, and jg_plan_destroy still releases them. */
void jg_free(jg_ctx* ctx);

/* build.  Validates `desc` and fixes the block decomposition of Sec. 4.1 / 4.2 for
 * these sizes.  JG_OP_XWT and JG_OP_XW: 2-way needs even K and N; JG_OP_XTW: 2-way needs even M and N
 * (the dimensions that are split); 4-way needs even M, K and N for both (the paper's
 * loader zero-pads to make partitions equal, Sec. 5 "Data loading": padding is the
 * caller's job).  Size limits: each of M, K, N below 2^31 - 1024, and for each pair
 * of them ceil(a/128) * ceil(b/128) at most (2^31 - 65) / 4 (the tile index of a launch
 * is 32 bits wide); beyond that JG_E_SHAPE.  Host-only; launches nothing.  `ctx` may be NULL: the plan then
 * serves jg_plan_query only and the data calls return JG_E_NULL.
 * Errors: JG_E_NULL, JG_E_WAYS, JG_E_DTYPE, JG_E_SHAPE (checked in this order). */
int jg_plan_create(jg_ctx* ctx, const jg_linear_desc* desc, jg_plan** out);
void jg_plan_destroy(jg_plan* plan);

/* query.  Host-only accounting of the plan; `rank` in [0, ways) where it matters.
 * Errors: JG_E_NULL, JG_E_WAYS (rank), JG_E_DTYPE (unknown `what`). */
int jg_plan_query(const jg_plan* plan, int what, int rank, int64_t* out);

/* build (data).  Splits a global tensor into the per-rank shards of Sec. 4.1 / 4.2.
 *   which = JG_T_X: global is M x K with leading dimension ld >= K;
 *           2-way: X_r = X[:, r-th half of K];  4-way: X_r = block (r/2, r%2).
 *   which = JG_T_W: global is N x K, ld >= K; split exactly like X
 *           (2-way: rank r holds all N rows of its column half).
 *   which = JG_T_B: global is the length-N bias (ld ignored); b_r = the half of b
 *           matching Y_r's columns (4-way: replicated on the two ranks of a column).
 *   which = JG_T_Y: global is M x N, ld >= N (an incoming gradient dY): partitioned like Y,
 *           2-way: column halves of N; 4-way: block (r/2, r%2).
 *   which = JG_T_X_F32: as JG_T_X, and stored in FP32 also for a reduced-precision plan (dense
 *           xr x xc shards): the activations jg_mlp_forward / jg_mixing_forward / jg_layernorm_forward take.
 * For a JG_OP_XTW plan the global X is K x M (ld >= M), W is K x N (ld >= N) and Y is
 * M x N; all three are partitioned the same way (2-way: column halves; 4-way: block
 * (r/2, r%2)) and b as above.  For a JG_OP_XW plan X is M x K, W is K x N (ld >= N), partitioned the same way.
 * `global` is a device pointer; `shards` is a host array of `ways` device pointers,
 * each with room for the rank's shard.  Pure data movement: bit-exact.
 * Reduced-precision plans (JG_BF16, JG_BF16X3): `global` is FP32 all the same; X and W shards are
 * written as bfloat16 (see jg_linear_desc.dtype; the pointers in `shards` are then those buffers,
 * 16-byte aligned), each value rounded on its bit pattern — bit-exact against that definition; b and
 * Y stay FP32.  For a JG_OP_XTW plan the same pass transposes each block (Sec. 5: the transposed layer
 * contracts over the row index of X and W; the bfloat16 matrix kernel reads along the contracted index).
 * Errors: JG_E_NULL, JG_E_SHAPE (ld), JG_E_ALIGN, JG_E_DTYPE (which), JG_E_HIP. */
int jg_shard(const jg_plan* plan, int which, const float* global, int64_t ld, float* const* shards);

/* build (data, encoder).  The patch encoder is a convolution whose kernel equals its stride, computed
 * as a linear layer over non-overlapping patches (Sec. 5 "Encoding and decoding layers").  This call
 * writes the X shards of that layer straight from the field, each rank reading its own part of it
 * (Sec. 5 "Data loading"), so the patch matrix is never stored whole.
 *   field: device, C x H x W dense row-major.  p: patch size; must divide H and W.
 *   Patch matrix: row t = py * (W / p) + px, column f = c * p * p + dy * p + dx, value
 *   field[c, py * p + dy, px * p + dx].  The plan (JG_OP_XWT) must have M = (H / p) * (W / p) and
 *   K = C * p * p; a weight row is the convolution kernel of one output channel, flattened [c][dy][dx].
 * x_shards as in jg_shard(JG_T_X).  Pure data movement: bit-exact.
 * Errors: JG_E_NULL, JG_E_DTYPE (op), JG_E_ALIGN, JG_E_SHAPE (sizes do not match the plan), JG_E_HIP. */
int jg_shard_patches(const jg_plan* plan, const float* field, int64_t C, int64_t H, int64_t W, int64_t p,
                     float* const* x_shards);

/* query (data, decoder).  The inverse rearrangement for the decoder: the rows of Y (one per patch,
 * N = C * p * p values each, M = (H / p) * (W / p)) are written back as a C x H x W field from the
 * per-rank Y shards.  Bit-exact.
 * Errors: as jg_shard_patches. */
int jg_gather_patches(const jg_plan* plan, const float* const* y_shards, float* field, int64_t C, int64_t H,
                      int64_t W, int64_t p);

/* run.  One forward pass of the layer over all `ways` virtual ranks:
 *   (ways = 4, JG_WEIGHTS_COPY) copy each rank's incoming weight block;
 *   launch 1: every rank's product that is handed to a peer, stored into the
 *             peer-visible partial buffer in the workspace;
 *   launch 2: every rank's kept product, accumulated on top of the received partial,
 *             plus the bias, written to Y_r (JG_COMBINE_FUSED); or the kept product
 *             followed by a separate combine kernel (JG_COMBINE_SEPARATE).
 * ways = 1 is a single GEMM with the bias in its epilogue; it needs no workspace beyond
 * the tail scratch of JG_TAIL_SPLIT.
 * JG_OP_XTW plans: (JG_WEIGHTS_COPY) copy each rank's incoming activation block; 2-way: one
 * launch of the four block products, each written with the bias straight into its row half
 * of Y_r; 4-way: launch 1 / launch 2 as above, the partial going to rank (1-i, j).  Both
 * operands are read along their rows' stride (no transpose in memory).
 * x_sh, w_sh, y_sh: host arrays of `ways` device pointers (shapes: JG_Q_*_ROWS/COLS);
 * b_sh: the same for the bias slices, required iff has_bias.  `workspace` is a
 * 256-byte-aligned device buffer of at least JG_Q_WORKSPACE_BYTES bytes (may be NULL
 * when that is 0); its contents on entry are irrelevant and are overwritten.
 * JG_OP_XW plans: (JG_WEIGHTS_COPY) copy each rank's incoming activation block and, 4-way, weight block;
 * launch 1: every rank's product of the received activation block, into a partial of its own in the workspace;
 * launch 2: the product of its own activation block on top of it, plus the bias (or, JG_COMBINE_SEPARATE,
 * written out and combined).  The weight blocks are read along their row stride.
 * JG_F32 plans: FP32 storage, FP32 matrix-core multiply-accumulate.  JG_BF16 / JG_BF16X3 plans
 * (JG_OP_XWT only): x_sh and w_sh point at the bfloat16 shards jg_shard wrote, the block products
 * run on the bfloat16 matrix cores with FP32 sums (JG_BF16X3: three products per block for each 16 k,
 * the small cross terms first), the partial products, b and Y stay FP32; the same launches, options and
 * epilogue as above; JG_TAIL_SPLIT adds one 256 x 256 scratch tile of floats per compute unit.
 * Errors: JG_E_NULL, JG_E_WORKSPACE, JG_E_ALIGN, JG_E_HIP. */
int jg_linear_forward(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                      const float* const* b_sh, float* const* y_sh, void* workspace,
                      size_t workspace_bytes);

/* run (with epilogue).  jg_linear_forward with what a mixing MLP puts around its linear layers
 * (Sec. 3: a GELU between the two layers, a residual connection around them; Sec. 5 "Activation
 * functions": GELU is point-wise and needs no exchange), fused into the step that completes an
 * output block:
 *     Y_r = act(X W^T + b)_r + R_r
 * activation: JG_ACT_NONE or JG_ACT_GELU, the defining form x * Phi(x) = x/2 (1 + erf(x / sqrt 2))
 * evaluated in FP32.  r_sh: host array of `ways` device pointers to residual shards shaped and
 * partitioned like Y_r (read only; may alias nothing that is written), or NULL for no residual.
 * Everything else as in jg_linear_forward, which is this call with r_sh = NULL and JG_ACT_NONE.
 * Errors: JG_E_NULL, JG_E_DTYPE (activation), JG_E_WORKSPACE, JG_E_ALIGN, JG_E_HIP. */
int jg_linear_forward_ex(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                         const float* const* b_sh, const float* const* r_sh, int activation, float* const* y_sh,
                         void* workspace, size_t workspace_bytes);

/* run (MLP).  One mixing MLP with its skip connection (Sec. 3) on Jigsaw shards:
 *     H = gelu(X W1^T + b1),    Y = X + H W2^T + b2,
 * X and Y are M x C, W1 is Hd x C, W2 is C x Hd.  `first` is a JG_OP_XWT plan of sizes (M, K = C,
 * N = Hd), `second` one of (M, K = Hd, N = C), same `ways`, same context.  Because a layer leaves
 * its output partitioned like its input (Sec. 4.1), H_r is consumed where it was produced: no
 * re-sharding between the layers.  h_sh: `ways` device buffers shaped like the first plan's Y_r
 * (H is kept: a backward pass would need it).  Workspace: FP32 plans use it in turn, it must hold
 * the larger of the two plans' JG_Q_WORKSPACE_BYTES; reduced-precision plans need the SUM of the two
 * plans' JG_Q_CHAIN_WORKSPACE_BYTES (the rounded H is written while the first layer still works in
 * its own part).  x_sh is read by both layers and must not overlap h_sh or y_sh.
 * Mixed precision (Sec. 6.1: the matrix units round their FP32 operands, everything else stays FP32):
 * both plans JG_BF16, or both JG_BF16X3.  x_sh, h_sh and y_sh are then still FP32 shards (x_sh as
 * jg_shard(JG_T_X_F32) writes them), w1_sh / w2_sh the plans' bfloat16 weight shards.  Each layer
 * reads its input activations rounded as jg_shard rounds X, from a copy in the workspace (H's copy
 * holds the roundings of exactly the FP32 values stored in h_sh; with the fused combine the launch
 * that writes H writes it too), runs its products on the bfloat16 matrix cores and adds bias, GELU
 * and the skip connection (from the unrounded x_sh) in FP32.
 * Errors: JG_E_NULL, JG_E_DTYPE (op, or the two plans' dtypes differ), JG_E_WAYS, JG_E_SHAPE (plans do
 * not chain), and those of jg_linear_forward_ex. */
int jg_mlp_forward(const jg_plan* first, const jg_plan* second, const float* const* x_sh,
                   const float* const* w1_sh, const float* const* b1_sh, const float* const* w2_sh,
                   const float* const* b2_sh, float* const* h_sh, float* const* y_sh, void* workspace,
                   size_t workspace_bytes);

/* run (layer norm).  The layer norm a mixing block applies before each MLP (Sec. 3), on the shards of
 * X.  Sec. 5 "Layer norms": the norm runs over the channels of a token and, with the channels split
 * over ranks, the library routine is applied as it is — every rank normalises over the channels it
 * holds.  Per row of X_r (xr x xc, the plan's JG_T_X partition; channels = columns of X, for both ops):
 *     mu = mean_c x[c],   var = mean_c (x[c] - mu)^2   (biased),
 *     out[c] = (x[c] - mu) / sqrt(var + eps) * gamma[c0 + c] + beta[c0 + c],
 * c0 = first global channel of the rank's block.  gamma, beta: device vectors over ALL channels of X
 * (length = JG_T_X partition width; each rank reads its own slice; read only), either may be NULL
 * (scale 1, offset 0).  eps >= 0; the library's default is 1e-5.  out_sh: `ways` device buffers shaped
 * like X_r; out_sh[r] may be x_sh[r] (in place), other overlaps are not allowed.  Sums and the
 * normalisation are evaluated in double and rounded once.  Needs no workspace; asynchronous on the
 * context's stream.  Input and output are FP32 whatever the plan's dtype (JG_T_X_F32 shards).
 * Errors: JG_E_NULL, JG_E_DTYPE (eps negative or NaN), JG_E_ALIGN, JG_E_HIP. */
int jg_layernorm_forward(const jg_plan* plan, const float* const* x_sh, const float* gamma, const float* beta,
                         double eps, float* const* out_sh);

/* run (mixing block).  The channel-mixing half of a mixing block (Sec. 3: layer norm before the MLP,
 * skip connection around it) on Jigsaw shards:
 *     Xn = layernorm(X),   H = gelu(Xn W1^T + b1),   Y = X + H W2^T + b2.
 * Plans, weights, h_sh, y_sh and workspace as in jg_mlp_forward; gamma, beta, eps as in
 * jg_layernorm_forward; xn_sh: `ways` device buffers shaped like X_r that receive Xn (kept: a backward
 * pass would need it); they must not overlap x_sh, which the skip connection still reads.
 * Errors: those of jg_mlp_forward and jg_layernorm_forward. */
int jg_mixing_forward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                      const float* beta, double eps, const float* const* w1_sh, const float* const* b1_sh,
                      const float* const* w2_sh, const float* const* b2_sh, float* const* xn_sh,
                      float* const* h_sh, float* const* y_sh, void* workspace, size_t workspace_bytes);

/* run (token-mixing block).  The token-mixing half of a mixing block (Sec. 3: the MLP along the token dimension
 * of the layer-normed input, skip connection around it; Sec. 5: its first layer is the transposed multiplication)
 * on Jigsaw shards.  X is T x C (tokens x channels); for every channel c, with xn = layernorm(X) as in
 * jg_layernorm_forward,
 *     y_c = x_c + W2 gelu(W1^T xn_c + b1) + b2,      W1, W2: T x D,  b1: D,  b2: T,
 * evaluated without transposing anything:
 *     H = gelu(Xn^T W1 + b1)     C x D   `first`:  a JG_OP_XTW plan with K = T, M = C, N = D, with bias;
 *     Y = X + W2 H^T + b2 1^T    T x C   `second`: a JG_OP_XWT plan with M = T, K = D, N = C, WITHOUT bias, in which
 *                                        W2 takes the activations' place and H the weights' place.
 * Same `ways`, same context.  H_r leaves the first layer partitioned as the second one partitions its weights, and
 * Y_r is partitioned like X_r, so nothing is re-sharded.  x_sh: the first plan's X shards (jg_shard(first, JG_T_X)
 * of the T x C input); w1_sh: its W shards; b1_sh: its bias shards; w2_sh: jg_shard(second, JG_T_X) of the T x D
 * matrix W2; b2: device vector of length T (the second layer's bias, one value per token), or NULL; gamma, beta,
 * eps, xn_sh as in jg_mixing_forward; h_sh: `ways` buffers shaped like the first plan's Y_r; y_sh: like X_r.
 * Workspace: the larger of the two plans' JG_Q_WORKSPACE_BYTES, plus the first plan's JG_Q_X_F32_SHARDS_BYTES when
 * b2 is given (the norm writes X + b2 there for the skip connection).
 * Mixed precision (Sec. 6.1): both plans JG_BF16, or both JG_BF16X3.  x_sh, xn_sh, h_sh and y_sh are then still FP32
 * shards (x_sh as jg_shard(first, JG_T_X_F32) writes them); w1_sh and w2_sh are the plans' bfloat16 shards
 * (jg_shard(first, JG_T_W) and jg_shard(second, JG_T_X)); the chain rounds Xn (contraction-major, as the first
 * plan's X shards) and H (as the second plan's W shards) into the workspace, which grows by `ways` times the first
 * plan's JG_Q_X_SHARD_BYTES and `ways` times the second plan's JG_Q_W_SHARD_BYTES, each rounded up to 256 bytes.
 * Errors: JG_E_NULL, JG_E_DTYPE (ops, precision, or the second plan has a bias), JG_E_WAYS, JG_E_SHAPE (plans do
 * not chain), JG_E_WORKSPACE, JG_E_ALIGN, and those of jg_linear_forward_ex and jg_layernorm_forward. */
int jg_token_mixing_forward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                            const float* beta, double eps, const float* const* w1_sh, const float* const* b1_sh,
                            const float* const* w2_sh, const float* b2, float* const* xn_sh, float* const* h_sh,
                            float* const* y_sh, void* workspace, size_t workspace_bytes);

/* run, for callers that cannot allocate.  Code under HIP graph capture, tight serving loops and harnesses that
 * forbid allocation cannot hand jg_linear_forward a workspace they would first have to allocate.  This is the same
 * call (same kernels, same launches, same results bit for bit) with the workspace taken from a fixed array of
 * JG_STATIC_WORKSPACE_BYTES bytes that lives in the library's own device memory: every GPU the library has been
 * initialised on (jg_init looks the array's address up once per device) holds one copy until the process ends.
 * The call allocates and frees nothing, on the device or through any library.
 * Limit: plans whose JG_Q_WORKSPACE_BYTES exceeds JG_STATIC_WORKSPACE_BYTES (64 MiB) are refused with
 * JG_E_WORKSPACE (a plan made with JG_TAIL_WHOLE needs no tail scratch and fits more often; the scratch of a small
 * problem cut along K is up to 32 MiB); so is a context on a device index of 64 or more.
 * The array keeps the last call's contents; nothing in it has to start at zero (every partial product and scratch
 * tile is written before it is read).  All calls on one GPU share the array: two calls that overlap on that GPU -
 * from different streams, contexts or threads - race; calls on one stream are ordered and safe.
 * x_sh, w_sh, b_sh, y_sh and the other errors: as jg_linear_forward. */
#define JG_STATIC_WORKSPACE_BYTES (64u << 20)
int jg_linear_forward_static(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                             const float* const* b_sh, float* const* y_sh);

/* run (backward).  Gradients of the same layer for an incoming gradient dY (partitioned like Y):
 *     dX = dY W      (M x K, partitioned like X)       dW = dY^T X    (N x K, partitioned like W)
 * the transposed multiplications of Sec. 4.1 (last sentence); Sec. 6.3 counts them as twice the
 * forward work.  No operand is transposed in memory.  Every output block is the sum of two block
 * products over the two halves of the contracted dimension; one of the two is formed from blocks
 * that live on peers (read in place from the peers' shard buffers), stored as a partial in the
 * workspace, and the second product is accumulated on top of it:
 *   ways = 1   one launch for dX, one for dW, no workspace;
 *   ways = 2   dX_r = dY_r W_{r,r} + dY_{1-r} W_{r,1-r} (the rank needs the peer's dY half);
 *              dW_{r,c} = dY_c^T X_r is a single product per block;
 *   ways = 4   dX_(i,j) = sum_c dY_(i,c) W_(c,j)   and   dW_(c,j) = sum_i dY_(i,c)^T X_(i,j),
 *              blocks (row half, column half) = rank 2 * row + column.
 * x_sh, w_sh, dy_sh: host arrays of `ways` device pointers to the X, W and dY shards (shapes of
 * X_r, W_r, Y_r); dx_sh, dw_sh: the same for the outputs (shapes of X_r, W_r).  `workspace`:
 * 256-byte-aligned device buffer of at least JG_Q_BACKWARD_WORKSPACE_BYTES bytes (may be NULL when
 * that is 0).  The bias gradient is jg_bias_backward's.  The plan's combine / weights options do not apply.
 * A JG_OP_XTW plan (Y = X^T W; Sec. 4.1 / 4.2 applied to the token-mixing layer): dX = W dY^T and dW = X dY, with
 * X_(i,a), W_(i,j), dY_(a,j) the plan's blocks (row half, column half; 2-way: one row range, and dY_r stacks
 * dY_(0,r) over dY_(1,r)):   dX_(i,a) = sum_j W_(i,j) dY_(a,j)^T,   dW_(i,j) = sum_a X_(i,a) dY_(a,j),
 * two launches each for ways >= 2 (the first term into a partial in the workspace, the second on top of it).
 * A JG_OP_XW plan (Y = X W): dX = dY W^T and dW = X^T dY, the forward passes of the other two permutations on
 * (dY, W) and (X, dY) with their launches and workspace (JG_Q_BACKWARD_WORKSPACE_BYTES covers both).
 * A reduced-precision JG_OP_XWT plan (Sec. 6.1: mixed precision): x_sh and w_sh are FP32 shards (JG_T_X_F32,
 * JG_T_W_F32: the copies a mixed-precision training step keeps), dy_sh, dx_sh and dw_sh FP32 as always; every operand
 * of every block product is rounded to bfloat16 (JG_BF16X3: split) into the workspace, in the layout the bfloat16
 * kernel reads, and the products run on the bfloat16 matrix cores with FP32 sums:  dX = rnd(dY) rnd(W),
 * dW = rnd(dY)^T rnd(X), block by block as above.  The rank's share of N must be a multiple of 8 (JG_E_SHAPE).
 * A reduced-precision JG_OP_XTW plan: the same with dX = rnd(W) rnd(dY)^T and dW = rnd(X) rnd(dY); the rank's
 * shares of M (channels) and of N must be multiples of 8 (JG_E_SHAPE), the token count is free.
 * Errors: JG_E_NULL, JG_E_DTYPE, JG_E_SHAPE, JG_E_WORKSPACE, JG_E_ALIGN, JG_E_HIP. */
int jg_linear_backward(const jg_plan* plan, const float* const* x_sh, const float* const* w_sh,
                       const float* const* dy_sh, float* const* dx_sh, float* const* dw_sh,
                       void* workspace, size_t workspace_bytes);

/* run (backward, MLP).  Gradients of jg_mlp_forward's MLP  H = gelu(X W1^T + b1),  Y = X + H W2^T + b2  for an
 * incoming gradient dY (shaped and partitioned like Y_r = like X_r), by the chain rule through the layers' own
 * backward passes (Sec. 4.1):
 *     dH = dY W2,   dW2 = dY^T H,   db2 = sum_i dY;      A = X W1^T + b1 (recomputed: the forward keeps H, not A);
 *     dA = dH * gelu'(A),  gelu'(x) = Phi(x) + x phi(x);  dX = dY + dA W1,   dW1 = dA^T X,   db1 = sum_i dA.
 * FP32 plans as for jg_mlp_forward; or two reduced-precision plans (mixed precision, Sec. 6.1): then x_sh, w1_sh and
 * w2_sh are FP32 shards (JG_T_X_F32, JG_T_W_F32: the activations the forward was given and the master weights), every
 * product's operands are rounded as in the forward (jg_linear_backward on such plans; A from X and W1 rounded once
 * more), everything else stays FP32, and the workspace must also hold, behind the first plan's
 * JG_Q_CHAIN_WORKSPACE_BYTES, `ways` times its JG_Q_W_SHARD_BYTES (each rounded up to 256).
 * x_sh, w1_sh, b1_sh, w2_sh: as in the forward; h_sh: the H it stored; dy_sh:
 * the dY shards.  Outputs (`ways` device buffers each): a_sh, dh_sh, da_sh shaped like H_r (A, dH and dA are kept:
 * they are what the steps hand on); dx_sh like X_r; dw1_sh, dw2_sh like the plans' W_r; db1_sh, db2_sh like their
 * bias shards.  No output may overlap an input or another output.  workspace: 256-byte aligned, at least the
 * largest of the first plan's JG_Q_WORKSPACE_BYTES and the two plans' JG_Q_BACKWARD_WORKSPACE_BYTES.
 * Errors: those of jg_mlp_forward, jg_linear_backward and jg_bias_backward. */
int jg_mlp_backward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* const* w1_sh,
                    const float* const* b1_sh, const float* const* w2_sh, const float* const* h_sh,
                    const float* const* dy_sh, float* const* a_sh, float* const* dh_sh, float* const* da_sh,
                    float* const* dx_sh, float* const* dw1_sh, float* const* db1_sh, float* const* dw2_sh,
                    float* const* db2_sh, void* workspace, size_t workspace_bytes);

/* run (backward, token-mixing block).  Gradients of jg_token_mixing_forward's block (Sec. 3; Sec. 5: the transposed
 * layer) for an incoming gradient dY (T x C, partitioned like X_r), by the chain rule through the steps in the layouts
 * the forward uses:
 *     second layer (W2 in the activations' place, H in the weights'):  dW2 = dY H,  dH = dY^T W2   (jg_linear_backward);
 *     db2[t] = sum_c dY[t][c];      A = Xn^T W1 + b1 (recomputed);      dA = dH * gelu'(A);
 *     transposed layer:  dXn = W1 dA^T,  dW1 = Xn dA  (jg_linear_backward on the JG_OP_XTW plan),  db1 = sum_c dA;
 *     dX = dY + layernorm'(dXn),  dgamma, dbeta   (as jg_layernorm_backward, the skip added before the rounding).
 * Plans as for jg_token_mixing_forward; on two reduced-precision plans (mixed precision) w1_sh and w2_sh are FP32
 * shards (jg_shard(first, JG_T_W_F32) of W1, jg_shard(second, JG_T_X_F32) of W2: the master weights), every product's
 * operands are rounded as in the forward, everything else stays FP32, and the workspace must also hold, behind the
 * first plan's JG_Q_CHAIN_WORKSPACE_BYTES, `ways` times its JG_Q_W_SHARD_BYTES (each rounded up to 256).
 * x_sh, gamma, eps, w1_sh, b1_sh, w2_sh: as in the forward; xn_sh, h_sh: the
 * Xn and H it stored; dy_sh: the dY shards.  Outputs (`ways` device buffers each): a_sh, dh_sh, da_sh shaped like
 * H_r; dxn_sh, dx_sh like X_r; dw1_sh like the first plan's W_r; db1_sh like its bias shards; dw2_sh like the second
 * plan's X_r; db2: device vector of length T (or NULL); dgamma, dbeta: device vectors of length C (either may be
 * NULL).  No output may overlap an input or another output.  workspace: 256-byte aligned, at least the largest of
 * the first plan's JG_Q_WORKSPACE_BYTES, the two plans' JG_Q_BACKWARD_WORKSPACE_BYTES and the first plan's
 * JG_Q_NORM_BACKWARD_WORKSPACE_BYTES.
 * Errors: those of jg_token_mixing_forward, jg_linear_backward, jg_bias_backward and jg_layernorm_backward. */
int jg_token_mixing_backward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                             double eps, const float* const* xn_sh, const float* const* w1_sh,
                             const float* const* b1_sh, const float* const* w2_sh, const float* const* h_sh,
                             const float* const* dy_sh, float* const* a_sh, float* const* dh_sh, float* const* da_sh,
                             float* const* dxn_sh, float* const* dx_sh, float* const* dw1_sh, float* const* db1_sh,
                             float* const* dw2_sh, float* db2, float* dgamma, float* dbeta, void* workspace,
                             size_t workspace_bytes);

/* run (backward, channel-mixing block).  Gradients of jg_mixing_forward's block  Xn = layernorm(X),
 * Y = X + MLP(Xn)  (Sec. 3: the block; Sec. 4.1 and Sec. 5 "Layer norms": its parts) for an incoming gradient dY:
 * jg_mlp_backward's chain on Xn without that function's skip connection (dXn = dA W1), then jg_layernorm_backward's
 * formulas with the block's skip connection added before the one rounding:  dX = dY + layernorm'(dXn).
 * FP32 plans.  x_sh, gamma, eps, w1_sh, b1_sh, w2_sh: as in the forward; xn_sh, h_sh: the Xn and H it stored;
 * dy_sh: the dY shards.  Outputs: a_sh, dh_sh, da_sh, dw1_sh, db1_sh, dw2_sh, db2_sh as in jg_mlp_backward; dxn_sh
 * and dx_sh shaped like X_r; dgamma, dbeta as in jg_layernorm_backward (either may be NULL).  No output may overlap
 * an input or another output.  workspace: 256-byte aligned, at least the largest of what jg_mlp_backward and
 * jg_layernorm_backward ask for on these plans.
 * Errors: those of jg_mlp_backward and jg_layernorm_backward. */
int jg_mixing_backward(const jg_plan* first, const jg_plan* second, const float* const* x_sh, const float* gamma,
                       double eps, const float* const* xn_sh, const float* const* w1_sh, const float* const* b1_sh,
                       const float* const* w2_sh, const float* const* h_sh, const float* const* dy_sh,
                       float* const* a_sh, float* const* dh_sh, float* const* da_sh, float* const* dxn_sh,
                       float* const* dx_sh, float* const* dw1_sh, float* const* db1_sh, float* const* dw2_sh,
                       float* const* db2_sh, float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes);

/* run (backward, layer norm).  Gradients of jg_layernorm_forward's output for an incoming gradient dY (shaped and
 * partitioned like X_r), per row of X_r over the channels the rank holds, with xhat = (x - mu) / sqrt(var + eps)
 * and g = dY * gamma:
 *     dX = (g - mean(g) - xhat * mean(g * xhat)) / sqrt(var + eps),
 *     dgamma[c] = sum over tokens of dY * xhat,     dbeta[c] = sum over tokens of dY.
 * x_sh: the forward's input shards; gamma as in the forward (may be NULL: 1); dy_sh, dx_sh: `ways` device buffers
 * shaped like X_r (no overlaps: the sums over tokens read x_sh and dy_sh after dx_sh is written); dgamma, dbeta: device vectors over ALL channels of X
 * (every channel block is summed over the ranks that hold it and written once), either may be NULL.  Evaluated in
 * double and rounded once; the column sums in a fixed order (the same bits on every run).  workspace: 256-byte
 * aligned; it must hold mean and 1 / sqrt(var + eps) of every row (`ways` times 16 bytes per row of X_r, each
 * rank's share rounded up to 256).  With JG_Q_NORM_BACKWARD_WORKSPACE_BYTES one kernel reads x and dy once and
 * leaves dx and, per band of rows, the column sums, which a second adds in order (rows of up to 6144 columns per
 * rank, a multiple of 4, 16-byte aligned shards; otherwise, or with less workspace, a rows' kernel and a column
 * kernel read them twice).  Any plan (op, dtype): only the X partition matters.
 * Errors: JG_E_NULL, JG_E_DTYPE (eps negative or NaN), JG_E_WORKSPACE, JG_E_ALIGN, JG_E_HIP. */
int jg_layernorm_backward(const jg_plan* plan, const float* const* x_sh, const float* gamma, double eps,
                          const float* const* dy_sh, float* const* dx_sh, float* dgamma, float* dbeta, void* workspace,
                          size_t workspace_bytes);

/* run (backward, bias).  The gradient of the bias for an incoming gradient dY (Sec. 4.1: the backward pass; the
 * bias enters the layer as + 1 b^T, whose adjoint is the column sum):  db[j] = sum_i dY[i][j].
 * dy_sh: the dY shards (shaped and partitioned like Y_r, as for jg_linear_backward); db_sh: `ways` device buffers
 * of JG_Q_B_LEN floats, partitioned like the bias (4-way: the slice of a column half is summed over both row
 * halves and written to both ranks of that column).  Sums are accumulated in double in a fixed order and rounded
 * once: the same bits on every run.  Any plan (op, dtype): only the Y partition matters.
 * workspace (optional; 8-byte aligned device buffer): with JG_Q_BIAS_BACKWARD_WORKSPACE_BYTES bytes the rows are
 * summed in ranges by several workgroups per column strip (partial sums in double, added in a fixed order by a
 * second small kernel), which takes the pass from 3 to about 6 TB/s; with NULL, or less room, one workgroup per
 * strip sums all rows.  The result is within half an FP32 unit of the exact sum either way.  Asynchronous on the
 * context's stream.
 * Errors: JG_E_NULL, JG_E_ALIGN, JG_E_HIP. */
int jg_bias_backward(const jg_plan* plan, const float* const* dy_sh, float* const* db_sh, void* workspace,
                     size_t workspace_bytes);

/* query (data).  Inverse of jg_shard for Y: writes the M x N global result (device,
 * leading dimension ld >= N) from the per-rank Y shards.  Bit-exact.
 * Errors: JG_E_NULL, JG_E_SHAPE, JG_E_ALIGN, JG_E_HIP. */
int jg_gather(const jg_plan* plan, const float* const* y_sh, float* global_y, int64_t ld);

/* query (data).  Inverse of jg_shard for a tensor partitioned like X (JG_T_X: e.g. dX; JG_T_X_F32: FP32
 * shards of any plan, e.g. a layer norm's output), like W (JG_T_W: e.g. dW) or like Y (JG_T_Y): writes
 * the global matrix from the per-rank shards.  jg_gather(plan, ...) is jg_gather_as(plan, JG_T_Y, ...).
 * Bit-exact.  The bfloat16 X and W shards of a reduced-precision plan are not converted back.
 * Errors: JG_E_NULL, JG_E_DTYPE (which; JG_T_X / JG_T_W of a reduced-precision plan), JG_E_SHAPE (ld),
 * JG_E_ALIGN, JG_E_HIP. */
int jg_gather_as(const jg_plan* plan, int which, const float* const* shards, float* global, int64_t ld);

/* Per-kernel timing with HIP events on the context's stream.
 * jg_profile(ctx, 1) starts bracketing every subsequent kernel launch of this
 * context with an event pair (a bounded pool; launches beyond it go untimed);
 * jg_profile(ctx, 0) stops.  jg_profile_read synchronises the stream, returns the
 * summed duration (milliseconds) and the number of timed launches of one kernel
 * class since the last read of that class, and clears them.
 * Errors: JG_E_NULL, JG_E_DTYPE (kernel class), JG_E_HIP. */
int jg_profile(jg_ctx* ctx, int enable);
int jg_profile_read(jg_ctx* ctx, int kernel, double* total_ms, int64_t* launches);

/* Static description of a status code (never NULL). */
const char* jg_strerror(int status);

/* Which HIP call last failed on the calling host thread, and the runtime's message
 * for it (a thread-local string, never NULL; valid until the next failure). */
const char* jg_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* JIGSAW_H */

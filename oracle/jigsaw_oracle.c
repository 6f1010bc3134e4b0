/*
 * CPU oracle for the forward pass of a Jigsaw-partitioned linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct C in IEEE double.
 * It shares no code with the HIP library and must never be called from the
 * product path; only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg use it.
 *
 * What it computes
 * ----------------
 *  oracle_linear      : the definition the method must reach (Sec. 4, first
 *                       paragraph: a linear layer is the product X W^T):
 *                         Y[i][j] = b[j] + sum_{k=0}^{K-1} X[i][k] * W[j][k]
 *                       every product and sum in double, k ascending.
 *  oracle_magnitude   : S[i][j] = |b[j]| + sum_k |X[i][k]| * |W[j][k]|, the
 *                       scale the floating-point tolerance is relative to.
 *  oracle_entries     : the same definition for a list of (row of X, row of W)
 *                       pairs, for sizes where the full product is too slow.
 *  oracle_jigsaw      : the same product obtained the way the method obtains
 *                       it: shard X and W, form the block products each rank
 *                       owns, hand partial products (and, 4-way, weight blocks)
 *                       to the peer by index, add, gather.
 *                       2-way: Sec. 4.1, Eqs. (1)-(2).  4-way: Sec. 4.2,
 *                       Eqs. (3)-(4).  ways = 1 is the unpartitioned layer.
 *  oracle_backward    : the backward pass of the same layer (Sec. 4.1, last
 *                       sentence: the transposed multiplications with the
 *                       incoming gradient), by its definition:
 *                         dX[i][k] = sum_j dY[i][j] * W[j][k]
 *                         dW[j][k] = sum_i dY[i][j] * X[i][k]
 *                       (and, optionally, the same sums of absolute values).
 *  oracle_jigsaw_backward : the same gradients obtained block by block with
 *                       dX partitioned like X and dW like W: every output
 *                       block is the sum of two block products, one of them
 *                       formed from a peer's block.
 *  oracle_linear_xtw  : the transposed linear layer of the token-mixing MLP (Sec. 5:
 *                       a forward pass defined by X^T W, so that the [tokens, channels]
 *                       tensor of Sec. 3 is never transposed in memory), by definition:
 *                         Y[c][d] = b[d] + sum_{t=0}^{T-1} X[t][c] * W[t][d]
 *                       with X [T x C], W [T x D], Y [C x D]; t ascending, in double
 *                       (optionally the same sum of absolute values).
 *  oracle_jigsaw_xtw  : the same product obtained block by block.  The paper names the
 *                       permutation but prints no equations for it; the decomposition
 *                       used here keeps Sec. 4's rules (tensors split along the last
 *                       dimension, 4-way in 2 x 2 blocks on rank 2 i + j, weights are
 *                       never duplicated, two block products per rank, one partial
 *                       product handed to one peer) and is stated above the function.
 *
 *  oracle_linear_xw   : the third permutation Sec. 5 names, Y = X W with the weights stored K x N, by
 *                       definition; oracle_jigsaw_xw: the same block by block (decomposition stated
 *                       above the function).  Pins (tests/test_oracle_xw_pins.py): integer brute force,
 *                       oracle_linear on explicitly transposed weights, closed forms, the block-wise
 *                       result against the definition, the adjoint identities of its gradients.
 *
 *  oracle_gelu        : the activation between the two linear layers of a mixing MLP
 *                       (Sec. 3; Sec. 5 "Activation functions": point-wise, no
 *                       synchronisation).  The paper names GELU without a formula; this is
 *                       its defining form x * Phi(x) = x/2 * (1 + erf(x / sqrt 2)), not the
 *                       tanh approximation.
 *  oracle_mlp         : one mixing MLP with its skip connection (Sec. 3: two linear layers,
 *                       GELU between them, a residual connection around the MLP):
 *                         H = gelu(X W1^T + b1),   Y = X + H W2^T + b2,
 *                       row by row with H kept in double; also returns the magnitudes the
 *                       tolerances of the two outputs are relative to.
 *  oracle_layernorm   : the layer norm applied before each mixing MLP (Sec. 3; Sec. 5 "Layer
 *                       norms": over the channels of a token, PyTorch's own routine usable
 *                       as it is with 2-way parallelism, where every rank holds half of the
 *                       channels of every token — so each rank normalises over the channels
 *                       it holds).  For `groups` equal, contiguous channel blocks, each token
 *                       (row) and block on its own:
 *                         mu = mean_c x,  var = mean_c (x - mu)^2  (biased, two passes),
 *                         y[c] = (x[c] - mu) / sqrt(var + eps) * gamma[c] + beta[c]
 *                       in double; groups = 1 is the unpartitioned layer, 2 the 2- and 4-way
 *                       ones (4-way also splits the tokens, which changes nothing per token).
 *                       Also returns the magnitude (|x| + |mu|) / sqrt(var + eps) * |gamma| + |beta|.
 *  oracle_round_bf16  : the reduced-precision mode (Sec. 6.1: the paper trains in a mixed precision
 *                       whose matrix units round the FP32 operands to a short mantissa and accumulate
 *                       in FP32).  The short format here is bfloat16 = the upper 16 bits of an FP32
 *                       number; rounding is to nearest, ties to even, done on the bit pattern.  The
 *                       reduced-precision layer is the same definition (oracle_linear) applied to
 *                       rounded operands; with split operands (x = hi + lo, hi = round(x),
 *                       lo = round(x - hi)) it is the sum of the three products hi*hi, hi*lo, lo*hi.
 *
 * Pins (see tests/test_oracle_pins.py): closed forms for identity /
 * permutation / all-ones / single-nonzero operands, exact integer brute force
 * on tiny shapes, a library matmul in double, the block identities of
 * Eqs. (2) and (4), linearity, and zero-padding invariance.
 *
 * Pins of the transposed layer (tests/test_oracle_xtw_pins.py): equality with
 * oracle_linear applied to explicitly transposed operands, closed forms, integer
 * brute force, exact equality of the block-wise result with the definition on
 * lattice inputs.
 *
 * Pins of the MLP (tests/test_oracle_mlp_pins.py): tabulated values of the normal
 * distribution function, the identity gelu(x) - gelu(-x) = x, limits, a library erf;
 * the MLP against the pinned forward oracle applied twice, closed forms (zero first
 * layer, identity weights), and brute force in exact rationals where gelu is not
 * involved.
 *
 * Pins of the bfloat16 rounding (tests/test_oracle_bf16_pins.py): tabulated ties and neighbours,
 * the library's own conversion, idempotence, monotonicity, the half-ulp bound, exactness of the
 * split's remainder, lattice values left unchanged.
 *
 * Pins of the layer norm (tests/test_oracle_layernorm_pins.py): rows whose result is known
 * in closed form (constant rows, +-1 rows, an arithmetic progression), the moments of the
 * output, invariance under a shift and (up to eps) a scaling of the input, a library
 * routine in double, independence of the channel blocks, and planted mistakes (unbiased
 * variance, eps outside the root, statistics over the whole row) that the pins must catch.
 *
 * Layout: every matrix is dense row-major; X is M x K, W is N x K, Y is M x N
 * (transposed layer: X is T x C, W is T x D, Y is C x D; MLP: X and Y are M x C,
 * W1 is Hd x C, W2 is C x Hd).
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_E_ARG (-1)
#define ORACLE_E_MEM (-2)

/* ------------------------------------------------------------------ */
/* row-parallel driver (plain pthreads; each thread owns whole rows)    */
/* ------------------------------------------------------------------ */
typedef void (*row_fn)(int64_t row, void* env);

typedef struct {
    row_fn fn;
    void* env;
    int64_t begin, end;
} row_job;

static void* row_worker(void* p)
{
    row_job* j = (row_job*)p;
    for (int64_t r = j->begin; r < j->end; ++r) j->fn(r, j->env);
    return NULL;
}

static int for_rows(int64_t begin, int64_t end, int nthreads, row_fn fn, void* env)
{
    int64_t n = end - begin;
    if (n <= 0) return ORACLE_OK;
    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > n) nthreads = (int)n;
    if (nthreads == 1) {
        row_job j = {fn, env, begin, end};
        row_worker(&j);
        return ORACLE_OK;
    }
    pthread_t* th = (pthread_t*)malloc(sizeof(pthread_t) * (size_t)nthreads);
    row_job* jobs = (row_job*)malloc(sizeof(row_job) * (size_t)nthreads);
    char* started = (char*)calloc((size_t)nthreads, 1);
    if (!th || !jobs || !started) { free(th); free(jobs); free(started); return ORACLE_E_MEM; }
    for (int t = 0; t < nthreads; ++t) {
        jobs[t].fn = fn;
        jobs[t].env = env;
        jobs[t].begin = begin + n * t / nthreads;
        jobs[t].end = begin + n * (t + 1) / nthreads;
        if (pthread_create(&th[t], NULL, row_worker, &jobs[t]) == 0) started[t] = 1;
        else row_worker(&jobs[t]); /* run inline if a thread cannot start */
    }
    for (int t = 0; t < nthreads; ++t)
        if (started[t]) pthread_join(th[t], NULL);
    free(th);
    free(jobs);
    free(started);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* the definition                                                       */
/* ------------------------------------------------------------------ */
typedef struct {
    const float *X, *W, *b;
    int64_t K, N;
    int64_t ldx, ldw, ldy;
    double* Y;
    int absolute; /* 0: value, 1: magnitude */
} lin_env;

static void linear_row(int64_t i, void* p)
{
    const lin_env* e = (const lin_env*)p;
    const float* x = e->X + i * e->ldx;
    double* y = e->Y + i * e->ldy;
    for (int64_t j = 0; j < e->N; ++j) {
        const float* w = e->W + j * e->ldw;
        double acc;
        if (e->b) acc = e->absolute ? fabs((double)e->b[j]) : (double)e->b[j];
        else acc = 0.0;
        if (e->absolute) {
            for (int64_t k = 0; k < e->K; ++k) acc += fabs((double)x[k]) * fabs((double)w[k]);
        } else {
            for (int64_t k = 0; k < e->K; ++k) acc += (double)x[k] * (double)w[k];
        }
        y[j] = acc;
    }
}

/* Rows [row_begin, row_end) of the result, written to Y[(row_end-row_begin) x N]. */
int oracle_linear_rows(const float* X, const float* W, const float* b, int64_t M, int64_t K,
                       int64_t N, int64_t row_begin, int64_t row_end, double* Y, int nthreads)
{
    if (!X || !W || !Y || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    if (row_begin < 0 || row_end > M || row_begin > row_end) return ORACLE_E_ARG;
    lin_env e = {X + row_begin * K, W, b, K, N, K, K, N, Y, 0};
    return for_rows(0, row_end - row_begin, nthreads, linear_row, &e);
}

int oracle_linear(const float* X, const float* W, const float* b, int64_t M, int64_t K, int64_t N,
                  double* Y, int nthreads)
{
    return oracle_linear_rows(X, W, b, M, K, N, 0, M, Y, nthreads);
}

int oracle_magnitude(const float* X, const float* W, const float* b, int64_t M, int64_t K,
                     int64_t N, double* S, int nthreads)
{
    if (!X || !W || !S || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    lin_env e = {X, W, b, K, N, K, K, N, S, 1};
    return for_rows(0, M, nthreads, linear_row, &e);
}

/* n entries: out[e] = bj[e] + <Xr[ix[e]], Wr[jw[e]]>, mag[e] likewise with
 * absolute values.  Xr / Wr are packed row sets with K columns each; bj (may
 * be NULL) holds the bias value of each entry. */
typedef struct {
    const float *Xr, *Wr, *bj;
    int64_t K;
    const int64_t *ix, *jw;
    double *out, *mag;
} ent_env;

static void entry_one(int64_t e, void* p)
{
    const ent_env* v = (const ent_env*)p;
    const float* x = v->Xr + v->ix[e] * v->K;
    const float* w = v->Wr + v->jw[e] * v->K;
    double acc = v->bj ? (double)v->bj[e] : 0.0;
    double s = v->bj ? fabs((double)v->bj[e]) : 0.0;
    for (int64_t k = 0; k < v->K; ++k) {
        double pr = (double)x[k] * (double)w[k];
        acc += pr;
        s += fabs(pr);
    }
    v->out[e] = acc;
    if (v->mag) v->mag[e] = s;
}

int oracle_entries(const float* Xr, const float* Wr, const float* bj, int64_t K, const int64_t* ix,
                   const int64_t* jw, int64_t n, double* out, double* mag, int nthreads)
{
    if (!Xr || !Wr || !ix || !jw || !out || K < 0 || n < 0) return ORACLE_E_ARG;
    ent_env v = {Xr, Wr, bj, K, ix, jw, out, mag};
    return for_rows(0, n, nthreads, entry_one, &v);
}

/* ------------------------------------------------------------------ */
/* the method, step by step                                             */
/* ------------------------------------------------------------------ */

/* contiguous copy of the block [r0, r0+nr) x [c0, c0+nc) of a row-major matrix */
static float* take_block(const float* A, int64_t ld, int64_t r0, int64_t nr, int64_t c0, int64_t nc)
{
    float* B = (float*)malloc(sizeof(float) * (size_t)(nr * nc > 0 ? nr * nc : 1));
    if (!B) return NULL;
    for (int64_t r = 0; r < nr; ++r)
        memcpy(B + r * nc, A + (r0 + r) * ld + c0, sizeof(float) * (size_t)nc);
    return B;
}

/* P = A * Bt^T for contiguous A [m x k] and Bt [n x k], in double */
static int block_product(const float* A, const float* Bt, int64_t m, int64_t k, int64_t n,
                         double* P, int nthreads)
{
    lin_env e = {A, Bt, NULL, k, n, k, k, n, P, 0};
    return for_rows(0, m, nthreads, linear_row, &e);
}

static double* new_partial(int64_t m, int64_t n)
{
    return (double*)calloc((size_t)(m * n > 0 ? m * n : 1), sizeof(double));
}

static int jigsaw2(const float* X, const float* W, const float* b, int64_t M, int64_t K, int64_t N,
                   double* Y, int nthreads)
{
    /* Sec. 4.1: X = [X_0, X_1] and W = [W_0, W_1] are split on the last
     * (channel) dimension; each rank further splits its W_r on the
     * second-to-last dimension into W_{r,0}, W_{r,1}.  Rank r keeps
     * X_r W_{r,r}^T, ships X_r W_{r,1-r}^T to the other rank, and output
     * column-half c ends up on rank c (Eq. 2). */
    const int64_t Kh = K / 2, Nh = N / 2;
    float *Xs[2] = {0, 0}, *Ws[2][2] = {{0, 0}, {0, 0}};
    double *kept[2] = {0, 0}, *sent[2] = {0, 0}, *recv[2] = {0, 0};
    int rc = ORACLE_E_MEM;
    for (int r = 0; r < 2; ++r) {
        Xs[r] = take_block(X, K, 0, M, r * Kh, Kh);
        if (!Xs[r]) goto done;
        for (int c = 0; c < 2; ++c) {
            Ws[r][c] = take_block(W, K, c * Nh, Nh, r * Kh, Kh);
            if (!Ws[r][c]) goto done;
        }
        kept[r] = new_partial(M, Nh);
        sent[r] = new_partial(M, Nh);
        if (!kept[r] || !sent[r]) goto done;
    }
    for (int r = 0; r < 2; ++r) {
        rc = block_product(Xs[r], Ws[r][1 - r], M, Kh, Nh, sent[r], nthreads);
        if (rc) goto done;
        rc = block_product(Xs[r], Ws[r][r], M, Kh, Nh, kept[r], nthreads);
        if (rc) goto done;
    }
    /* exchange: what rank r sent is what rank 1-r receives */
    recv[0] = sent[1];
    recv[1] = sent[0];
    /* combine on the owner and gather: Y[:, c-th half] lives on rank c */
    for (int c = 0; c < 2; ++c)
        for (int64_t i = 0; i < M; ++i)
            for (int64_t j = 0; j < Nh; ++j) {
                double v = kept[c][i * Nh + j] + recv[c][i * Nh + j];
                if (b) v += (double)b[c * Nh + j];
                Y[i * N + c * Nh + j] = v;
            }
    rc = ORACLE_OK;
done:
    for (int r = 0; r < 2; ++r) {
        free(Xs[r]); free(Ws[r][0]); free(Ws[r][1]); free(kept[r]); free(sent[r]);
    }
    return rc;
}

static int jigsaw4(const float* X, const float* W, const float* b, int64_t M, int64_t K, int64_t N,
                   double* Y, int nthreads)
{
    /* Sec. 4.2: X = [[X_0, X_1], [X_2, X_3]] and W = [[W_0, W_1], [W_2, W_3]]
     * are split 2 x 2 on the last two dimensions.  Eq. (4):
     *   Y_0 = X_0 W_0^T + X_1 W_1^T     Y_1 = X_0 W_2^T + X_1 W_3^T
     *   Y_2 = X_2 W_0^T + X_3 W_1^T     Y_3 = X_2 W_2^T + X_3 W_3^T
     * and Y_r sits where X_r sat (rank r).  A term printed bold as a whole is
     * computed on the rank holding its X block and shipped; a term in which
     * only W^T is bold is computed where its X block lives, after that weight
     * block has been shipped there.  Each rank therefore forms two products:
     *   rank 0: X_0 W_0^T (keep)            X_0 W_2^T (W_2 from rank 2; to rank 1)
     *   rank 1: X_1 W_1^T (to rank 0)       X_1 W_3^T (W_3 from rank 3; keep)
     *   rank 2: X_2 W_2^T (to rank 3)       X_2 W_0^T (W_0 from rank 0; keep)
     *   rank 3: X_3 W_3^T (keep)            X_3 W_1^T (W_1 from rank 1; to rank 2)
     */
    const int64_t Mh = M / 2, Kh = K / 2, Nh = N / 2;
    static const int w_from[4] = {2, 3, 0, 1};      /* rank whose weight block rank r receives */
    static const int own_is_kept[4] = {1, 0, 0, 1}; /* is X_r W_r^T the kept term on rank r?   */
    static const int peer[4] = {1, 0, 3, 2};        /* partial-product exchange partner        */
    float *Xs[4] = {0}, *Ws[4] = {0}, *Wrecv[4] = {0};
    double *kept[4] = {0}, *sent[4] = {0}, *recv[4] = {0};
    int rc = ORACLE_E_MEM;
    for (int r = 0; r < 4; ++r) {
        Xs[r] = take_block(X, K, (r / 2) * Mh, Mh, (r % 2) * Kh, Kh);
        Ws[r] = take_block(W, K, (r / 2) * Nh, Nh, (r % 2) * Kh, Kh);
        kept[r] = new_partial(Mh, Nh);
        sent[r] = new_partial(Mh, Nh);
        if (!Xs[r] || !Ws[r] || !kept[r] || !sent[r]) goto done;
    }
    /* weight-block exchange (a copy, as a transfer would deliver it) */
    for (int r = 0; r < 4; ++r) {
        Wrecv[r] = take_block(Ws[w_from[r]], Kh, 0, Nh, 0, Kh);
        if (!Wrecv[r]) goto done;
    }
    for (int r = 0; r < 4; ++r) {
        double* own = own_is_kept[r] ? kept[r] : sent[r];
        double* cross = own_is_kept[r] ? sent[r] : kept[r];
        rc = block_product(Xs[r], Ws[r], Mh, Kh, Nh, own, nthreads);
        if (rc) goto done;
        rc = block_product(Xs[r], Wrecv[r], Mh, Kh, Nh, cross, nthreads);
        if (rc) goto done;
    }
    for (int r = 0; r < 4; ++r) recv[r] = sent[peer[r]];
    for (int r = 0; r < 4; ++r) {
        const int64_t i0 = (r / 2) * Mh, j0 = (r % 2) * Nh;
        for (int64_t i = 0; i < Mh; ++i)
            for (int64_t j = 0; j < Nh; ++j) {
                double v = kept[r][i * Nh + j] + recv[r][i * Nh + j];
                if (b) v += (double)b[j0 + j];
                Y[(i0 + i) * N + j0 + j] = v;
            }
    }
    rc = ORACLE_OK;
done:
    for (int r = 0; r < 4; ++r) {
        free(Xs[r]); free(Ws[r]); free(Wrecv[r]); free(kept[r]); free(sent[r]);
    }
    return rc;
}

int oracle_jigsaw(int ways, const float* X, const float* W, const float* b, int64_t M, int64_t K,
                  int64_t N, double* Y, int nthreads)
{
    if (!X || !W || !Y || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    switch (ways) {
    case 1:
        return oracle_linear(X, W, b, M, K, N, Y, nthreads);
    case 2:
        if ((K % 2) || (N % 2)) return ORACLE_E_ARG;
        return jigsaw2(X, W, b, M, K, N, Y, nthreads);
    case 4:
        if ((M % 2) || (K % 2) || (N % 2)) return ORACLE_E_ARG;
        return jigsaw4(X, W, b, M, K, N, Y, nthreads);
    default:
        return ORACLE_E_ARG;
    }
}

/* ------------------------------------------------------------------ */
/* backward pass: the definition                                        */
/* ------------------------------------------------------------------ */
typedef struct {
    const float *X, *W, *dY;
    int64_t M, K, N;
    double *dX, *dW;
    int absolute;
} bwd_env;

/* row i of dX: for every k, sum over j ascending */
static void dx_row(int64_t i, void* p)
{
    const bwd_env* e = (const bwd_env*)p;
    double* out = e->dX + i * e->K;
    for (int64_t k = 0; k < e->K; ++k) out[k] = 0.0;
    for (int64_t j = 0; j < e->N; ++j) {
        double g = (double)e->dY[i * e->N + j];
        const float* w = e->W + j * e->K;
        if (e->absolute) { g = fabs(g); for (int64_t k = 0; k < e->K; ++k) out[k] += g * fabs((double)w[k]); }
        else { for (int64_t k = 0; k < e->K; ++k) out[k] += g * (double)w[k]; }
    }
}

/* row j of dW: for every k, sum over i ascending */
static void dw_row(int64_t j, void* p)
{
    const bwd_env* e = (const bwd_env*)p;
    double* out = e->dW + j * e->K;
    for (int64_t k = 0; k < e->K; ++k) out[k] = 0.0;
    for (int64_t i = 0; i < e->M; ++i) {
        double g = (double)e->dY[i * e->N + j];
        const float* x = e->X + i * e->K;
        if (e->absolute) { g = fabs(g); for (int64_t k = 0; k < e->K; ++k) out[k] += g * fabs((double)x[k]); }
        else { for (int64_t k = 0; k < e->K; ++k) out[k] += g * (double)x[k]; }
    }
}

/* dX [M x K] and dW [N x K] (either may be NULL); absolute != 0 gives the magnitudes */
int oracle_backward(const float* X, const float* W, const float* dY, int64_t M, int64_t K, int64_t N,
                    double* dX, double* dW, int absolute, int nthreads)
{
    if (!dY || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    if ((dX && !W) || (dW && !X)) return ORACLE_E_ARG;
    bwd_env e = {X, W, dY, M, K, N, dX, dW, absolute};
    int rc = ORACLE_OK;
    if (dX) rc = for_rows(0, M, nthreads, dx_row, &e);
    if (rc == ORACLE_OK && dW) rc = for_rows(0, N, nthreads, dw_row, &e);
    return rc;
}

/* ------------------------------------------------------------------ */
/* backward pass, block by block                                        */
/* ------------------------------------------------------------------ */

/* C += A * B for contiguous A [m x n] and B [n x k] (contraction over A's columns / B's rows) */
typedef struct { const float *A, *B; int64_t n, k; double* C; } nn_env;
static void nn_row(int64_t i, void* p)
{
    const nn_env* e = (const nn_env*)p;
    double* out = e->C + i * e->k;
    for (int64_t j = 0; j < e->n; ++j) {
        const double a = (double)e->A[i * e->n + j];
        const float* b = e->B + j * e->k;
        for (int64_t c = 0; c < e->k; ++c) out[c] += a * (double)b[c];
    }
}
static int add_nn(const float* A, const float* B, int64_t m, int64_t n, int64_t k, double* C, int nthreads)
{
    nn_env e = {A, B, n, k, C};
    return for_rows(0, m, nthreads, nn_row, &e);
}

/* C += A^T * B for contiguous A [m x n] and B [m x k] (contraction over the rows of both) */
typedef struct { const float *A, *B; int64_t m, n, k; double* C; } tn_env;
static void tn_row(int64_t j, void* p)
{
    const tn_env* e = (const tn_env*)p;
    double* out = e->C + j * e->k;
    for (int64_t i = 0; i < e->m; ++i) {
        const double a = (double)e->A[i * e->n + j];
        const float* b = e->B + i * e->k;
        for (int64_t c = 0; c < e->k; ++c) out[c] += a * (double)b[c];
    }
}
static int add_tn(const float* A, const float* B, int64_t m, int64_t n, int64_t k, double* C, int nthreads)
{
    tn_env e = {A, B, m, n, k, C};
    return for_rows(0, n, nthreads, tn_row, &e);
}

static void put_block(double* G, int64_t ld, int64_t r0, int64_t nr, int64_t c0, int64_t nc, const double* B)
{
    for (int64_t r = 0; r < nr; ++r)
        memcpy(G + (r0 + r) * ld + c0, B + r * nc, sizeof(double) * (size_t)nc);
}

/* Partitioning as in the forward pass: dY like Y, dX like X, dW like W.
 * 2-way (Sec. 4.1): rank r holds X_r = X[:, r], W_r = [W_{r,0}; W_{r,1}] = W[:, r], dY_r = dY[:, r]
 * (column halves).  dX_r = dY_0 W_{r,0} + dY_1 W_{r,1} and dW_{r,c} = dY_c^T X_r: the rank needs the
 * peer's dY half; with it, both products of every output block are local.
 * 4-way (Sec. 4.2): blocks (i, j) = rank 2 i + j.  dX_(i,j) = dY_(i,0) W_(0,j) + dY_(i,1) W_(1,j)
 * (the row neighbour's dY block and the column neighbour's W block come from peers);
 * dW_(c,j) = dY_(0,c)^T X_(0,j) + dY_(1,c)^T X_(1,j): the term with i != c is formed on the column
 * neighbour (which holds X_(i,j)) and handed over as a partial product. */
int oracle_jigsaw_backward(int ways, const float* X, const float* W, const float* dY, int64_t M,
                           int64_t K, int64_t N, double* dX, double* dW, int nthreads)
{
    if (!X || !W || !dY || !dX || !dW || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    if (ways == 1) return oracle_backward(X, W, dY, M, K, N, dX, dW, 0, nthreads);
    if (ways != 2 && ways != 4) return ORACLE_E_ARG;
    if ((K % 2) || (N % 2) || (ways == 4 && (M % 2))) return ORACLE_E_ARG;
    const int rh = ways == 4 ? 2 : 1;                 /* row halves of X / dY */
    const int64_t Mb = M / rh, Kh = K / 2, Nh = N / 2;
    int rc = ORACLE_E_MEM;
    /* blocks: Xb[i][j] (Mb x Kh), Gb[i][c] (Mb x Nh) = dY blocks, Wb[c][j] (Nh x Kh) */
    float *Xb[2][2] = {{0}}, *Gb[2][2] = {{0}}, *Wb[2][2] = {{0}};
    for (int i = 0; i < rh; ++i)
        for (int j = 0; j < 2; ++j) {
            Xb[i][j] = take_block(X, K, i * Mb, Mb, j * Kh, Kh);
            Gb[i][j] = take_block(dY, N, i * Mb, Mb, j * Nh, Nh);
            if (!Xb[i][j] || !Gb[i][j]) goto done;
        }
    for (int c = 0; c < 2; ++c)
        for (int j = 0; j < 2; ++j) {
            Wb[c][j] = take_block(W, K, c * Nh, Nh, j * Kh, Kh);
            if (!Wb[c][j]) goto done;
        }
    /* dX blocks: owner (i, j) adds its own-dY term, then the term with the received dY block */
    for (int i = 0; i < rh; ++i)
        for (int j = 0; j < 2; ++j) {
            double* acc = new_partial(Mb, Kh);
            if (!acc) goto done;
            const int own_c = j;                      /* the dY block this rank holds: column half j */
            rc = add_nn(Gb[i][own_c], Wb[own_c][j], Mb, Nh, Kh, acc, nthreads);
            if (!rc) rc = add_nn(Gb[i][1 - own_c], Wb[1 - own_c][j], Mb, Nh, Kh, acc, nthreads);
            if (!rc) put_block(dX, K, i * Mb, Mb, j * Kh, Kh, acc);
            free(acc);
            if (rc) goto done;
            rc = ORACLE_E_MEM;
        }
    /* dW blocks (c, j): one term per row half i; 4-way: the i != c term arrives as a partial */
    for (int c = 0; c < 2; ++c)
        for (int j = 0; j < 2; ++j) {
            double* kept = new_partial(Nh, Kh);
            double* recv = new_partial(Nh, Kh);
            if (!kept || !recv) { free(kept); free(recv); goto done; }
            rc = ORACLE_OK;
            if (ways == 2) {
                rc = add_tn(Gb[0][c], Xb[0][j], Mb, Nh, Kh, kept, nthreads);
            } else {
                rc = add_tn(Gb[c][c], Xb[c][j], Mb, Nh, Kh, kept, nthreads);
                if (!rc) rc = add_tn(Gb[1 - c][c], Xb[1 - c][j], Mb, Nh, Kh, recv, nthreads);
            }
            if (!rc) {
                for (int64_t t = 0; t < Nh * Kh; ++t) kept[t] += recv[t];
                put_block(dW, K, c * Nh, Nh, j * Kh, Kh, kept);
            }
            free(kept); free(recv);
            if (rc) goto done;
            rc = ORACLE_E_MEM;
        }
    rc = ORACLE_OK;
done:
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) { free(Xb[i][j]); free(Gb[i][j]); free(Wb[i][j]); }
    return rc;
}

/* ------------------------------------------------------------------ */
/* transposed linear layer  Y = X^T W + b                               */
/* ------------------------------------------------------------------ */
typedef struct { const float *X, *W, *b; int64_t T, C, D; double* Y; int absolute; } xtw_env;
static void xtw_row(int64_t c, void* p)
{
    const xtw_env* e = (const xtw_env*)p;
    double* out = e->Y + c * e->D;
    for (int64_t d = 0; d < e->D; ++d) {
        const double bd = e->b ? (double)e->b[d] : 0.0;
        out[d] = e->absolute ? fabs(bd) : bd;
    }
    for (int64_t t = 0; t < e->T; ++t) {
        const double x = (double)e->X[t * e->C + c];
        const float* w = e->W + t * e->D;
        if (e->absolute)
            for (int64_t d = 0; d < e->D; ++d) out[d] += fabs(x) * fabs((double)w[d]);
        else
            for (int64_t d = 0; d < e->D; ++d) out[d] += x * (double)w[d];
    }
}

int oracle_linear_xtw(const float* X, const float* W, const float* b, int64_t T, int64_t C, int64_t D,
                      double* Y, int absolute, int nthreads)
{
    if (!X || !W || !Y || T < 0 || C < 0 || D < 0) return ORACLE_E_ARG;
    xtw_env e = {X, W, b, T, C, D, Y, absolute};
    return for_rows(0, C, nthreads, xtw_row, &e);
}

/* Block decomposition of Y = X^T W (X [T x C], W [T x D], Y [C x D]).
 * 2-way: column halves, X_r = X[:, r], W_r = W[:, r], and Y_r = Y[:, r] = [X_0^T W_r ; X_1^T W_r].
 * The contraction (over tokens) is not split, so nothing is summed across ranks: rank r forms
 * the row half it can from its own X_r and the other one from the peer's activation block.
 * 4-way: blocks (i, j) on rank 2 i + j, i the token half of X and W, j the channel half of X
 * (column half of W); Y block (a, c) on rank 2 a + c:
 *     Y_(a,c) = X_(0,a)^T W_(0,c) + X_(1,a)^T W_(1,c).
 * Rank (i, j) multiplies its own W_(i,j) with its own X_(i,j) (a term of Y_(j,j)) and with
 * X_(i,1-j), received from its row neighbour (a term of Y_(1-j,j)); the term whose block it
 * owns (a = i) it keeps, the other goes to its column neighbour (1 - i, j), which owns that
 * block and adds it to its own kept term.  Bias: b[c-th half] on the owner. */
int oracle_jigsaw_xtw(int ways, const float* X, const float* W, const float* b, int64_t T, int64_t C,
                      int64_t D, double* Y, int nthreads)
{
    if (!X || !W || !Y || T < 0 || C < 0 || D < 0) return ORACLE_E_ARG;
    if (ways == 1) return oracle_linear_xtw(X, W, b, T, C, D, Y, 0, nthreads);
    if (ways != 2 && ways != 4) return ORACLE_E_ARG;
    if ((C % 2) || (D % 2) || (ways == 4 && (T % 2))) return ORACLE_E_ARG;
    const int th = ways == 4 ? 2 : 1;                 /* token halves */
    const int64_t Tb = T / th, Ch = C / 2, Dh = D / 2;
    int rc = ORACLE_E_MEM;
    float *Xb[2][2] = {{0}}, *Wb[2][2] = {{0}};
    for (int i = 0; i < th; ++i)
        for (int j = 0; j < 2; ++j) {
            Xb[i][j] = take_block(X, C, i * Tb, Tb, j * Ch, Ch);
            Wb[i][j] = take_block(W, D, i * Tb, Tb, j * Dh, Dh);
            if (!Xb[i][j] || !Wb[i][j]) goto done;
        }
    for (int a = 0; a < 2; ++a)          /* channel half = row half of Y */
        for (int c = 0; c < 2; ++c) {    /* column half of Y */
            double* kept = new_partial(Ch, Dh);
            double* recv = new_partial(Ch, Dh);
            if (!kept || !recv) { free(kept); free(recv); goto done; }
            if (ways == 2) {
                /* owner: rank c; a == c uses its own X block, a != c the received one */
                rc = add_tn(Xb[0][a], Wb[0][c], Tb, Ch, Dh, kept, nthreads);
            } else {
                /* owner: rank (a, c); its kept term has token half a, the received one 1 - a */
                rc = add_tn(Xb[a][a], Wb[a][c], Tb, Ch, Dh, kept, nthreads);
                if (!rc) rc = add_tn(Xb[1 - a][a], Wb[1 - a][c], Tb, Ch, Dh, recv, nthreads);
            }
            if (!rc) {
                for (int64_t r = 0; r < Ch; ++r)
                    for (int64_t q = 0; q < Dh; ++q)
                        kept[r * Dh + q] += recv[r * Dh + q] + (b ? (double)b[c * Dh + q] : 0.0);
                put_block(Y, D, a * Ch, Ch, c * Dh, Dh, kept);
            }
            free(kept); free(recv);
            if (rc) goto done;
            rc = ORACLE_E_MEM;
        }
    rc = ORACLE_OK;
done:
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) { free(Xb[i][j]); free(Wb[i][j]); }
    return rc;
}

/* ------------------------------------------------------------------ */
/* the third permutation  Y = X W + b  (weights stored K x N)           */
/* ------------------------------------------------------------------ */
typedef struct { const float *X, *W, *b; int64_t K, N; double* Y; int absolute; } xw_env;
static void xw_row(int64_t i, void* p)
{
    const xw_env* e = (const xw_env*)p;
    double* out = e->Y + i * e->N;
    for (int64_t j = 0; j < e->N; ++j) {
        const double bj = e->b ? (double)e->b[j] : 0.0;
        out[j] = e->absolute ? fabs(bj) : bj;
    }
    for (int64_t k = 0; k < e->K; ++k) {
        const double x = (double)e->X[i * e->K + k];
        const float* w = e->W + k * e->N;
        if (e->absolute)
            for (int64_t j = 0; j < e->N; ++j) out[j] += fabs(x) * fabs((double)w[j]);
        else
            for (int64_t j = 0; j < e->N; ++j) out[j] += x * (double)w[j];
    }
}

/* Sec. 5 names three permutations of the layer, X W^T, X W and X^T W.  This one by its definition,
 *     Y[i][j] = b[j] + sum_{k=0}^{K-1} X[i][k] * W[k][j],   X [M x K], W [K x N], Y [M x N],
 * every product and sum in double, k ascending (absolute != 0: the same sum of absolute values). */
int oracle_linear_xw(const float* X, const float* W, const float* b, int64_t M, int64_t K, int64_t N,
                     double* Y, int absolute, int nthreads)
{
    if (!X || !W || !Y || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    xw_env e = {X, W, b, K, N, Y, absolute};
    return for_rows(0, M, nthreads, xw_row, &e);
}

/* Block decomposition of Y = X W.  The paper prints no equations for this permutation; it is the form of the
 * backward product dX = dY W of Sec. 4.1 (activations times weights stored along the contracted index), and
 * the blocks follow that pass and the rules of Sec. 4: every tensor split on its last dimension (2-way) or
 * in 2 x 2 blocks with block (i, j) on rank 2 i + j (4-way), nothing duplicated, two block products per rank.
 * 2-way: X_r = X[:, r-th half of K], W_r = W[:, r-th half of N] (all K rows), Y_r = Y[:, r-th half of N]
 *     Y_r = X_r W_(r,r) + X_(1-r) W_(1-r,r),   W_(k,c) = rows k-th half of K, columns c-th half of N:
 * rank r holds both weight blocks of its column half and receives the peer's activation block.
 * 4-way:  Y_(i,j) = X_(i,j) W_(j,j) + X_(i,1-j) W_(1-j,j):  rank (i, j) multiplies its own activation block
 * with W_(j,j) (its own block if i = j, else its column neighbour's) and the block X_(i,1-j) of its row
 * neighbour with W_(1-j,j) (its own if i = 1 - j, else its column neighbour's): one activation block and one
 * weight block come from peers, both products stay.  Bias: b[j-th half] on the owner of the block. */
int oracle_jigsaw_xw(int ways, const float* X, const float* W, const float* b, int64_t M, int64_t K,
                     int64_t N, double* Y, int nthreads)
{
    if (!X || !W || !Y || M < 0 || K < 0 || N < 0) return ORACLE_E_ARG;
    if (ways == 1) return oracle_linear_xw(X, W, b, M, K, N, Y, 0, nthreads);
    if (ways != 2 && ways != 4) return ORACLE_E_ARG;
    if ((K % 2) || (N % 2) || (ways == 4 && (M % 2))) return ORACLE_E_ARG;
    const int rh = ways == 4 ? 2 : 1;                 /* row halves of X and Y */
    const int64_t Mb = M / rh, Kh = K / 2, Nh = N / 2;
    int rc = ORACLE_E_MEM;
    /* Xb[i][k] (Mb x Kh): on rank (i, k);  Wb[k][c] (Kh x Nh): 4-way on rank (k, c), 2-way both on rank c */
    float *Xb[2][2] = {{0}}, *Wb[2][2] = {{0}};
    for (int i = 0; i < rh; ++i)
        for (int k = 0; k < 2; ++k) {
            Xb[i][k] = take_block(X, K, i * Mb, Mb, k * Kh, Kh);
            if (!Xb[i][k]) goto done;
        }
    for (int k = 0; k < 2; ++k)
        for (int c = 0; c < 2; ++c) {
            Wb[k][c] = take_block(W, N, k * Kh, Kh, c * Nh, Nh);
            if (!Wb[k][c]) goto done;
        }
    for (int i = 0; i < rh; ++i)
        for (int j = 0; j < 2; ++j) {     /* the owner of Y block (i, j): rank (i, j), 2-way rank j */
            double* acc = new_partial(Mb, Nh);
            if (!acc) goto done;
            rc = add_nn(Xb[i][j], Wb[j][j], Mb, Kh, Nh, acc, nthreads);              /* its own activation block */
            if (!rc) rc = add_nn(Xb[i][1 - j], Wb[1 - j][j], Mb, Kh, Nh, acc, nthreads);   /* the received one */
            if (!rc) {
                if (b)
                    for (int64_t r = 0; r < Mb; ++r)
                        for (int64_t q = 0; q < Nh; ++q) acc[r * Nh + q] += (double)b[j * Nh + q];
                put_block(Y, N, i * Mb, Mb, j * Nh, Nh, acc);
            }
            free(acc);
            if (rc) goto done;
            rc = ORACLE_E_MEM;
        }
    rc = ORACLE_OK;
done:
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) { free(Xb[i][j]); free(Wb[i][j]); }
    return rc;
}

/* ------------------------------------------------------------------ */
/* mixing MLP: H = gelu(X W1^T + b1), Y = X + H W2^T + b2               */
/* ------------------------------------------------------------------ */
static double gelu1(double x) { return 0.5 * x * (1.0 + erf(x * 0.70710678118654752440)); }

int oracle_gelu(const double* in, int64_t n, double* out)
{
    if (!in || !out || n < 0) return ORACLE_E_ARG;
    for (int64_t i = 0; i < n; ++i) out[i] = gelu1(in[i]);
    return ORACLE_OK;
}

typedef struct {
    const float *X, *W1, *b1, *W2, *b2;
    int64_t C, Hd;
    int residual;
    double *H, *Y, *S1, *SY, *PY;
} mlp_env;

/* One row of X.  S1 = |b1| + |x| |W1|^T (scale of the pre-activation's rounding), SY = |b2| + |x| + |h| |W2|^T
 * (scale of the second layer's own rounding), PY = S1 |W2|^T (how a unit of S1-relative error in H shows in Y;
 * |gelu'| <= 1.13 is left to the caller). */
static void mlp_row(int64_t i, void* p)
{
    const mlp_env* e = (const mlp_env*)p;
    const float* x = e->X + i * e->C;
    double* h = e->H + i * e->Hd;
    double* s1 = e->S1 + i * e->Hd;
    for (int64_t q = 0; q < e->Hd; ++q) {
        const float* w = e->W1 + q * e->C;
        double acc = e->b1 ? (double)e->b1[q] : 0.0, mag = fabs(acc);
        for (int64_t k = 0; k < e->C; ++k) {
            const double t = (double)x[k] * (double)w[k];
            acc += t;
            mag += fabs(t);
        }
        h[q] = gelu1(acc);
        s1[q] = mag;
    }
    for (int64_t j = 0; j < e->C; ++j) {
        const float* w = e->W2 + j * e->Hd;
        double acc = e->b2 ? (double)e->b2[j] : 0.0, mag = fabs(acc), prop = 0.0;
        for (int64_t q = 0; q < e->Hd; ++q) {
            const double t = h[q] * (double)w[q];
            acc += t;
            mag += fabs(t);
            prop += s1[q] * fabs((double)w[q]);
        }
        if (e->residual) {
            acc += (double)x[j];
            mag += fabs((double)x[j]);
        }
        e->Y[i * e->C + j] = acc;
        e->SY[i * e->C + j] = mag;
        e->PY[i * e->C + j] = prop;
    }
}

int oracle_mlp(const float* X, const float* W1, const float* b1, const float* W2, const float* b2, int64_t M,
               int64_t C, int64_t Hd, int residual, double* H, double* Y, double* S1, double* SY, double* PY,
               int nthreads)
{
    if (!X || !W1 || !W2 || !H || !Y || !S1 || !SY || !PY || M < 0 || C < 0 || Hd < 0) return ORACLE_E_ARG;
    mlp_env e = {X, W1, b1, W2, b2, C, Hd, residual, H, Y, S1, SY, PY};
    return for_rows(0, M, nthreads, mlp_row, &e);
}

/* ------------------------------------------------------------------ */
/* layer norm over the channels of a token, per channel block           */
/* ------------------------------------------------------------------ */
typedef struct {
    const float *X, *gamma, *beta;
    int64_t C, groups;
    double eps;
    double *Y, *S;
} ln_env;

static void ln_row(int64_t i, void* p)
{
    const ln_env* e = (const ln_env*)p;
    const int64_t Cg = e->C / e->groups;
    for (int64_t g = 0; g < e->groups; ++g) {
        const float* x = e->X + i * e->C + g * Cg;
        double mu = 0.0, var = 0.0;
        for (int64_t c = 0; c < Cg; ++c) mu += (double)x[c];
        mu /= (double)Cg;
        for (int64_t c = 0; c < Cg; ++c) {
            const double d = (double)x[c] - mu;
            var += d * d;
        }
        var /= (double)Cg;
        const double rstd = 1.0 / sqrt(var + e->eps);
        for (int64_t c = 0; c < Cg; ++c) {
            const int64_t col = g * Cg + c;
            const double ga = e->gamma ? (double)e->gamma[col] : 1.0;
            const double be = e->beta ? (double)e->beta[col] : 0.0;
            e->Y[i * e->C + col] = ((double)x[c] - mu) * rstd * ga + be;
            if (e->S) e->S[i * e->C + col] = (fabs((double)x[c]) + fabs(mu)) * rstd * fabs(ga) + fabs(be);
        }
    }
}

int oracle_layernorm(const float* X, const float* gamma, const float* beta, int64_t M, int64_t C,
                     int64_t groups, double eps, double* Y, double* S, int nthreads)
{
    if (!X || !Y || M < 0 || C < 0 || groups < 1 || !(eps >= 0.0)) return ORACLE_E_ARG;
    if (C % groups) return ORACLE_E_ARG;
    if (C == 0) return ORACLE_OK;
    ln_env e = {X, gamma, beta, C, groups, eps, Y, S};
    return for_rows(0, M, nthreads, ln_row, &e);
}

/* ------------------------------------------------------------------ */
/* bfloat16 rounding: nearest, ties to even, on the bit pattern         */
/* ------------------------------------------------------------------ */
int oracle_round_bf16(const float* in, int64_t n, float* out)
{
    if (!in || !out || n < 0) return ORACLE_E_ARG;
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &in[i], 4);
        if ((u & 0x7F800000u) == 0x7F800000u) {
            if (u & 0x007FFFFFu) u |= 0x00400000u;      /* NaN stays NaN when its payload is cut */
            u &= 0xFFFF0000u;
        } else {
            const uint32_t keep_odd = (u >> 16) & 1u;    /* ties go to the even 16-bit pattern */
            u += 0x7FFFu + keep_odd;
            u &= 0xFFFF0000u;
        }
        memcpy(&out[i], &u, 4);
    }
    return ORACLE_OK;
}

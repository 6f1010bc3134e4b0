// Host-side exercise of the C ABI for a sanitizer build (address + undefined behaviour): everything that runs
// without a GPU - plan validation, every query of every kind of plan, error strings, the data calls' refusal of
// plans without a context, release functions on NULL.  Exit code 0 = every expectation held; the sanitizers abort
// with a report otherwise.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "../../include/jigsaw.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

static jg_linear_desc desc(int64_t M, int64_t K, int64_t N, int ways, int op, int dtype)
{
    jg_linear_desc d;
    std::memset(&d, 0, sizeof(d));
    d.M = M; d.K = K; d.N = N; d.ways = ways; d.op = op; d.dtype = dtype;
    return d;
}

int main()
{
    for (int s = 1; s >= -9; --s) EXPECT(jg_strerror(s) != nullptr && std::strlen(jg_strerror(s)) > 0);
    EXPECT(jg_last_hip_error() != nullptr);
    jg_plan_destroy(nullptr);
    jg_free(nullptr);

    jg_plan* p = nullptr;
    jg_linear_desc d = desc(8, 8, 8, 2, JG_OP_XWT, JG_F32);
    EXPECT(jg_plan_create(nullptr, nullptr, &p) == JG_E_NULL);
    EXPECT(jg_plan_create(nullptr, &d, nullptr) == JG_E_NULL);
    // refused descriptors, one field at a time
    { jg_linear_desc b = d; b.ways = 3; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_WAYS && !p); }
    { jg_linear_desc b = d; b.op = 7; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.dtype = 9; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.combine = 2; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.weights = -1; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.has_bias = 2; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.tail = 5; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.accumulate = 2; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }
    { jg_linear_desc b = d; b.M = 0; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_SHAPE); }
    { jg_linear_desc b = d; b.K = 7; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_SHAPE); }
    { jg_linear_desc b = d; b.N = INT64_MAX; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_SHAPE); }
    { jg_linear_desc b = d; b.M = b.N = 128LL * 23171; b.K = 128; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_SHAPE); }
    { jg_linear_desc b = d; b.dtype = JG_BF16; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_SHAPE); }
    { jg_linear_desc b = d; b.op = JG_OP_XW; b.dtype = JG_BF16; b.K = 16; EXPECT(jg_plan_create(nullptr, &b, &p) == JG_E_DTYPE); }

    // every kind of plan, every query, every rank; sizes from the smallest to the largest configuration
    const int64_t shapes[][3] = {{2, 2, 2}, {100, 100, 100}, {1000, 1000, 1000}, {25000, 4000, 4000}, {200000, 10000, 10000},
                                 {16200, 4320, 8640}, {6, 16, 2}};
    const int ops[] = {JG_OP_XWT, JG_OP_XTW, JG_OP_XW};
    const int dtypes[] = {JG_F32, JG_BF16, JG_BF16X3};
    const int ways_of[] = {1, 2, 4};
    int made = 0;
    for (const auto& sh : shapes)
        for (int op : ops)
            for (int dt : dtypes)
                for (int ways : ways_of)
                    for (int opt = 0; opt < 4; ++opt) {
                        jg_linear_desc q = desc(sh[0], sh[1], sh[2], ways, op, dt);
                        q.has_bias = opt & 1;
                        q.combine = (opt >> 1) & 1;
                        q.weights = opt & 1;
                        q.tail = (opt >> 1) & 1;
                        q.accumulate = opt == 3;
                        jg_plan* plan = nullptr;
                        const int rc = jg_plan_create(nullptr, &q, &plan);
                        if (rc != JG_OK) {
                            EXPECT(plan == nullptr);
                            EXPECT(rc == JG_E_SHAPE || rc == JG_E_DTYPE);
                            continue;
                        }
                        ++made;
                        int64_t total = 0;
                        for (int what = -1; what <= 25; ++what)
                            for (int rank = -1; rank <= ways; ++rank) {
                                int64_t v = -12345;
                                const int qrc = jg_plan_query(plan, what, rank, &v);
                                EXPECT(qrc == JG_OK || qrc == JG_E_WAYS || qrc == JG_E_DTYPE);
                                if (qrc == JG_OK) { EXPECT(v >= 0); total += v > 0; }
                            }
                        EXPECT(total > 0);
                        EXPECT(jg_plan_query(plan, JG_Q_FLOPS_TOTAL, 0, nullptr) == JG_E_NULL);
                        // no context: the data calls refuse before they touch a pointer
                        const float* in[4] = {nullptr, nullptr, nullptr, nullptr};
                        float* out[4] = {nullptr, nullptr, nullptr, nullptr};
                        float x = 0.f;
                        EXPECT(jg_linear_forward(plan, in, in, in, out, nullptr, 0) < 0);
                        EXPECT(jg_linear_forward_static(plan, in, in, in, out) < 0);
                        EXPECT(jg_linear_backward(plan, in, in, in, out, out, nullptr, 0) < 0);
                        EXPECT(jg_shard(plan, JG_T_X, &x, 1, out) < 0);
                        EXPECT(jg_gather(plan, in, &x, 1) < 0);
                        EXPECT(jg_bias_backward(plan, in, out, nullptr, 0) < 0);
                        EXPECT(jg_layernorm_forward(plan, in, nullptr, nullptr, 1e-5, out) < 0);
                        EXPECT(jg_mlp_forward(plan, plan, in, in, in, in, in, out, out, nullptr, 0) < 0);
                        jg_plan_destroy(plan);
                    }
    EXPECT(made > 300);
    EXPECT(jg_plan_query(nullptr, JG_Q_FLOPS_TOTAL, 0, nullptr) == JG_E_NULL);
    // init without a usable device: an error code and a message, nothing else
    jg_ctx* ctx = nullptr;
    const int irc = jg_init(&ctx, 123456, nullptr);
    EXPECT(irc == JG_E_HIP && ctx == nullptr);
    EXPECT(jg_init(nullptr, 0, nullptr) == JG_E_NULL);
    EXPECT(jg_profile(nullptr, 1) == JG_E_NULL);
    std::printf("abi driver: %d plans exercised, %d failures\n", made, failures);
    return failures ? 1 : 0;
}

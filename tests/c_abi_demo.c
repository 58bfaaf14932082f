/*
 * A plain C program against the C ABI of libssd.so: no Python, no PyTorch.
 * Device memory comes from hipMalloc, the library is driven through ssd.h,
 * and the result is compared bit for bit with the CPU oracle, which is
 * compiled into this test program (binary32 build of oracle/ssd_oracle.c).
 * Built by __graft_entry__.build(); run by tests/test_gpu_c_abi.py.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ssd.h"

/* the oracle, binary32 (see oracle/ssd_oracle.c) */
typedef struct {
    int K, k, W;
    float lr, m, wd, lr_loc, alpha, beta, wd_loc, rescale, pre_scale;
    long n, num;
    long *loc_update;
    float *w, *mom, *wl, *pre, *wloc;
} oracle_state;
void ssd_oracle_begin_f32(oracle_state *s);
int ssd_oracle_step_f32(oracle_state *s, const float *const *g);

#define CK(x)                                                                  \
    do {                                                                       \
        hipError_t e_ = (x);                                                   \
        if (e_ != hipSuccess) {                                                \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                          \
        }                                                                      \
    } while (0)
#define SSD(x)                                                                 \
    do {                                                                       \
        int r_ = (x);                                                          \
        if (r_ != SSD_OK) {                                                    \
            printf("ssd error %d at line %d: %s\n", r_, __LINE__, ssd_last_error(ctx)); \
            return 3;                                                          \
        }                                                                      \
    } while (0)

static unsigned long long rng_state = 88172645463325252ULL;
static float rnd(void) /* xorshift, uniform in (-1, 1) */
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (float)((double)(rng_state >> 11) / 4503599627370496.0 - 1.0);
}

enum { T = 3, KMAX = 9, STEPS = 7, P = 2 };

/* K = 3: planar local-weight arrays; K = 9: interleaved by block (see ssd_state_view) */
static int run(const int K)
{
    const int64_t numel[T] = {1000, 37, 4101};
    long N = 0, off[T + 1];
    for (int t = 0; t < T; ++t) off[t] = N, N += numel[t];
    off[T] = N;
    ssd_ctx *ctx = NULL;

    /* host copies: w0 and P sets of K gradients, flat in tensor order */
    float *w0 = malloc(sizeof(float) * N), *g[P][KMAX];
    for (long j = 0; j < N; ++j) w0[j] = rnd();
    for (int p = 0; p < P; ++p)
        for (int i = 0; i < K; ++i) {
            g[p][i] = malloc(sizeof(float) * N);
            for (long j = 0; j < N; ++j) g[p][i][j] = 0.01f * rnd();
        }

    /* device copies: one allocation per tensor, as a framework would hand them over */
    float *d_w[T], *d_g[P][KMAX][T];
    for (int t = 0; t < T; ++t) {
        CK(hipMalloc((void **)&d_w[t], sizeof(float) * numel[t]));
        CK(hipMemcpy(d_w[t], w0 + off[t], sizeof(float) * numel[t], hipMemcpyHostToDevice));
        for (int p = 0; p < P; ++p)
            for (int i = 0; i < K; ++i) {
                CK(hipMalloc((void **)&d_g[p][i][t], sizeof(float) * numel[t]));
                CK(hipMemcpy(d_g[p][i][t], g[p][i] + off[t], sizeof(float) * numel[t], hipMemcpyHostToDevice));
            }
    }

    /* the paper's settings (Sec. 4.1, Table 1) come from the library */
    ssd_config cfg;
    SSD(ssd_config_defaults(&cfg, K, 0.1f, 1e-4f));
    if (cfg.lr_loc != 0.4f || cfg.alpha != 2.0f || cfg.beta != 0.5f || cfg.wd_loc != 1e-4f ||
        cfg.rescale_grad != (float)(1.0 / K)) {
        printf("ssd_config_defaults: unexpected values\n");
        return 4;
    }
    cfg.delay_k = 2, cfg.warmup_iters = 1, cfg.momentum = 0.9f;
    cfg.num_tensors = T, cfg.numel = numel, cfg.device = 0, cfg.stream = NULL;
    size_t ws_bytes = 0;
    SSD(ssd_workspace_bytes(&cfg, &ws_bytes));
    void *ws = NULL;
    CK(hipMalloc(&ws, ws_bytes));
    SSD(ssd_init(&cfg, d_w, ws, ws_bytes, &ctx));

    oracle_state o;
    memset(&o, 0, sizeof o);
    o.K = K, o.k = cfg.delay_k, o.W = cfg.warmup_iters;
    o.lr = cfg.lr, o.m = cfg.momentum, o.wd = cfg.wd, o.lr_loc = cfg.lr_loc, o.alpha = cfg.alpha;
    o.beta = cfg.beta, o.wd_loc = cfg.wd_loc, o.rescale = cfg.rescale_grad, o.pre_scale = 1.0f;
    o.n = N;
    o.loc_update = calloc(K, sizeof(long));
    o.w = malloc(sizeof(float) * N), o.mom = calloc(N, sizeof(float));
    o.wl = malloc(sizeof(float) * N * K), o.pre = malloc(sizeof(float) * N * K);
    o.wloc = malloc(sizeof(float) * N * K);
    memcpy(o.w, w0, sizeof(float) * N);
    ssd_oracle_begin_f32(&o);

    for (int it = 0; it < STEPS; ++it) {
        const int p = it % P;
        const float *rows[KMAX][T];
        const void *const *grads[KMAX];
        const float *og[KMAX];
        for (int i = 0; i < K; ++i) {
            for (int t = 0; t < T; ++t) rows[i][t] = d_g[p][i][t];
            grads[i] = (const void *const *)rows[i];
            og[i] = g[p][i];
        }
        SSD(ssd_step(ctx, grads));
        ssd_oracle_step_f32(&o, og);
    }
    SSD(ssd_materialize(ctx)); /* explicit w'_i arrays, whatever the last iteration was */
    CK(hipDeviceSynchronize());

    ssd_state_view v;
    SSD(ssd_get_state(ctx, &v));
    float *buf = malloc(sizeof(float) * 4101);
    long bad = 0;
    for (int t = 0; t < T; ++t) {
        CK(hipMemcpy(buf, d_w[t], sizeof(float) * numel[t], hipMemcpyDeviceToHost));
        bad += memcmp(buf, o.w + off[t], sizeof(float) * numel[t]) != 0;
        CK(hipMemcpy(buf, v.mom + v.tensor_offset[t], sizeof(float) * numel[t], hipMemcpyDeviceToHost));
        bad += memcmp(buf, o.mom + off[t], sizeof(float) * numel[t]) != 0;
        CK(hipMemcpy(buf, v.pre + v.tensor_offset[t], sizeof(float) * numel[t], hipMemcpyDeviceToHost));
        bad += memcmp(buf, o.pre + off[t], sizeof(float) * numel[t]) != 0;
        for (int i = 0; i < K; ++i) {
            /* w'_i block by block: the general addressing of ssd_state_view */
            for (int64_t a = v.tensor_offset[t], end = a + numel[t]; a < end;) {
                const int64_t blk = a / v.chunk_elems, pos = a % v.chunk_elems;
                const int64_t n = end - a < v.chunk_elems - pos ? end - a : v.chunk_elems - pos;
                CK(hipMemcpy(buf + (a - v.tensor_offset[t]),
                             v.w_local + i * v.w_local_worker_stride + blk * v.w_local_block_stride + pos,
                             sizeof(float) * n, hipMemcpyDeviceToHost));
                a += n;
            }
            bad += memcmp(buf, o.wl + i * N + off[t], sizeof(float) * numel[t]) != 0;
        }
    }
    /* error path: a NULL gradient pointer is refused and leaves the state alone */
    const void *const *nullgrads[KMAX] = {NULL};
    if (ssd_step(ctx, nullgrads) != SSD_EINVAL) bad += 1000;
    if (v.iterations != STEPS) bad += 10000;
    ssd_destroy(ctx);
    if (bad)
        printf("C ABI demo: MISMATCH (%ld)\n", bad);
    else
        printf("C ABI demo: OK, K = %d, %d iterations bit-identical to the oracle\n", K, (int)STEPS);
    return bad ? 1 : 0;
}

int main(void)
{
    int rc = run(3);
    if (rc == 0) rc = run(KMAX);
    return rc;
}

/*
 * CPU oracle for the SSD-SGD parameter-update pipeline.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
 * compute; it is plain scalar C, shares no code with the HIP path, and may be
 * called only from tests, the smoke check and the cpu_baseline leg of the
 * benchmark.  The product never routes through it.
 *
 * What it follows (SSD-SGD paper):
 *   - server: Eq. (server) -- gradients of the K workers are aggregated and
 *     averaged -- followed by the momentum-SGD rule printed in Sec. 3.2.1
 *     (mom = -lr*(grad + wd*w) + m*mom_prev ; w_next = w + mom).
 *   - worker: Algorithm 1 (warm-up loop, then steps-delay loop with a Pull
 *     every k iterations) and Algorithm 2 (the GLU optimizer: grad_sync from
 *     pre_weight and w', refresh of pre_weight every k local updates, the
 *     update of Eq. (glu-update)), with grad_sync as in Sec. 3.3:
 *     (pre_weight - w') * (1 - m) / (lr * k).
 *
 * Readings where the paper leaves a choice (each also listed in the design
 * notes of the repository):
 *   - Eq. (glu-update) is printed with "+ lr_loc*(...)"; the momentum rule of
 *     Sec. 3.2.1 is a descent rule and grad_sync = (old - new)*... has the sign
 *     of a gradient, so the local update is a descent step: w' -= lr_loc*(...).
 *   - "Averaged gradient" (Table 1): sum over workers in index order, then one
 *     multiply by `rescale` (1/K by default).
 *   - The divisor in grad_sync is always k (Sec. 3.3 prints only lr*k), on
 *     every local update, boundary or not.
 *   - grad_sync uses (pre_weight - w') as Sec. 3.3 prints it.  The exact
 *     w_minus of Sec. 3.2.1, ((1 - lr*wd)*pre_weight - w'), is available as a
 *     variant through pre_scale = 1 - lr*wd (formed in double, then rounded);
 *     pre_scale = 1 multiplies exactly and gives the default form.
 *   - lr and m inside grad_sync are the server's (Table 1).
 *   - The Pull of Algorithm 1 happens after t <- t+1, so the pulled weight
 *     includes the server update of the same iteration.
 *   - Pulls are keyed on the index of the steps-delay iteration
 *     (loc_update % k == k-1); this equals Algorithm 1's num % k == k-1
 *     whenever (1+wp) % k == 0, which the paper requires.
 *   - Each worker keeps its own pre_weight, as in Sec. 3.5; Sec. 3.3 says they
 *     all hold the same value, which tests check as an invariant.
 *
 * Precision: the file is compiled twice.  REAL=double is the plain oracle.
 * REAL=float is the "GPU-order" oracle: every statement below is exactly one
 * IEEE-754 binary32 operation rounded to nearest-even (build with
 * -ffp-contract=off so that no multiply-add is fused), workers are summed in
 * index order, and c_sync / rescale are formed once in double and rounded.
 *
 * Parity pins: see tests/test_oracle_pins.py (closed forms of the momentum
 * series, textbook momentum SGD, exact rational brute force, the identity of
 * Sec. 3.2.1, special cases of Eq. (glu-update), schedule against Alg. 1).
 * Nothing here is "parity unpinned".
 */
#include <stddef.h>

#ifndef REAL
#error "compile with -DREAL=float -DSFX=f32 or -DREAL=double -DSFX=f64"
#endif
#define CAT2(a, b) a##_##b
#define CAT(a, b) CAT2(a, b)
#define NAME(x) CAT(x, SFX)

typedef struct {
    int K;            /* number of workers                                   */
    int k;            /* delay steps; 0 = plain SSGD for ever                */
    int W;            /* number of warm-up (SSGD) iterations, = wp + 1       */
    REAL lr, m, wd;   /* server: learning rate, momentum, weight decay       */
    REAL lr_loc, alpha, beta, wd_loc; /* worker, Eq. (glu-update)            */
    REAL rescale;     /* factor on the K-sum, 1/K = average                  */
    REAL pre_scale;   /* factor on pre_weight inside grad_sync: 1 for the form
                         of Sec. 3.3, (1 - lr*wd) for the exact w_minus of
                         Sec. 3.2.1                                          */
    long n;           /* elements in the (flattened) model                   */
    long num;         /* Alg. 1: iterations done                             */
    long *loc_update; /* [K] Alg. 2: local updates done by worker i          */
    REAL *w, *mom;    /* [n] server weight and momentum                      */
    REAL *wl;         /* [K*n] w'_i, local weight of worker i                */
    REAL *pre;        /* [K*n] pre_weight of worker i                        */
    REAL *wloc;       /* [K*n] w_loc of worker i (what fwd/bwd would use)    */
} NAME(ssd_oracle_state);

/* Eq. (server) + momentum rule of Sec. 3.2.1, over n elements.
 * g[i] is worker i's gradient array.  */
void NAME(ssd_oracle_server)(long n, int K, const REAL *const *g, REAL rescale,
                             REAL lr, REAL m, REAL wd, REAL *w, REAL *mom)
{
    for (long j = 0; j < n; ++j) {
        REAL S = g[0][j];
        for (int i = 1; i < K; ++i)
            S = S + g[i][j];
        REAL gh = S * rescale;          /* averaged gradient grad_t          */
        REAL t1 = wd * w[j];
        REAL t2 = gh + t1;
        REAL t3 = lr * t2;
        REAL t4 = m * mom[j];
        REAL mo = t4 - t3;              /* mom_t = m*mom_{t-1} - lr*(...)    */
        mom[j] = mo;
        w[j] = w[j] + mo;               /* w_{t+1} = w_t + mom_t             */
    }
}

/* The factor (1 - lr*wd) of the exact w_minus (Sec. 3.2.1), formed in double. */
REAL NAME(ssd_oracle_pre_scale)(REAL lr, REAL wd)
{
    return (REAL)(1.0 - (double)lr * (double)wd);
}

/* The factor (1-m)/(lr*k) of Sec. 3.3, formed once in double. */
REAL NAME(ssd_oracle_c_sync)(REAL lr, REAL m, int k)
{
    return (REAL)((1.0 - (double)m) / ((double)lr * (double)k));
}

/* One call of Algorithm 2 for one worker: wl, pre are that worker's arrays,
 * *loc_update its counter.  */
void NAME(ssd_oracle_glu)(long n, int k, const REAL *g, REAL *wl, REAL *pre,
                          long *loc_update, REAL c_sync, REAL pre_scale,
                          REAL lr_loc, REAL alpha, REAL beta, REAL wd_loc)
{
    long lu = *loc_update;
    int refresh = (lu > 0) && (lu % k == 0);
    for (long j = 0; j < n; ++j) {
        if (lu == 0)
            pre[j] = wl[j];             /* Alg. 2 initialisation             */
        REAL q = pre_scale * pre[j];    /* pre_scale = 1: q is pre_weight    */
        REAL e = q - wl[j];
        REAL gs = e * c_sync;           /* grad_sync, Sec. 3.3               */
        if (refresh)
            pre[j] = wl[j];             /* Alg. 2: pre_weight = w'           */
        REAL u1 = alpha * g[j];
        REAL u2 = wd_loc * wl[j];
        REAL u3 = u1 + u2;
        REAL u4 = beta * gs;
        REAL u5 = u3 + u4;
        REAL u6 = lr_loc * u5;
        wl[j] = wl[j] - u6;             /* Eq. (glu-update), descent         */
    }
    *loc_update = lu + 1;
}

static void copy_n(long n, const REAL *src, REAL *dst)
{
    for (long j = 0; j < n; ++j)
        dst[j] = src[j];
}

/* Algorithm 1's initialisation: every worker pulls w_0.  */
void NAME(ssd_oracle_begin)(NAME(ssd_oracle_state) *s)
{
    s->num = 0;
    for (int i = 0; i < s->K; ++i) {
        s->loc_update[i] = 0;
        copy_n(s->n, s->w, s->wl + (size_t)i * s->n);
        copy_n(s->n, s->w, s->wloc + (size_t)i * s->n);
        copy_n(s->n, s->w, s->pre + (size_t)i * s->n);
    }
}

/* One iteration of Algorithm 1 seen from all K workers plus the server.
 * Returns the kind of iteration: 0 warm-up, 1 last warm-up, 2 delay (no
 * pull), 3 delay with pull.  */
int NAME(ssd_oracle_step)(NAME(ssd_oracle_state) *s, const REAL *const *g)
{
    const long n = s->n;
    const int K = s->K;
    int kind;
    if (s->k == 0 || s->num < s->W) {
        /* warm-up loop: Push, synchronous server update, Pull w_t          */
        NAME(ssd_oracle_server)(n, K, g, s->rescale, s->lr, s->m, s->wd,
                                s->w, s->mom);
        for (int i = 0; i < K; ++i)
            copy_n(n, s->w, s->wloc + (size_t)i * n);      /* Broadcast w_t */
        kind = 0;
        if (s->k > 0 && s->num == s->W - 1) {
            for (int i = 0; i < K; ++i)
                copy_n(n, s->w, s->wl + (size_t)i * n);    /* w'_{t,i}=w_t  */
            kind = 1;
        }
    } else {
        /* steps-delay loop: Push (server is synchronous every iteration),  */
        NAME(ssd_oracle_server)(n, K, g, s->rescale, s->lr, s->m, s->wd,
                                s->w, s->mom);
        /* local update with GLU,                                           */
        REAL c_sync = NAME(ssd_oracle_c_sync)(s->lr, s->m, s->k);
        long d = s->loc_update[0];
        for (int i = 0; i < K; ++i)
            NAME(ssd_oracle_glu)(n, s->k, g[i], s->wl + (size_t)i * n,
                                 s->pre + (size_t)i * n, &s->loc_update[i],
                                 c_sync, s->pre_scale, s->lr_loc, s->alpha,
                                 s->beta, s->wd_loc);
        /* Broadcast w' to the devices, and every k-th iteration Pull.      */
        for (int i = 0; i < K; ++i)
            copy_n(n, s->wl + (size_t)i * n, s->wloc + (size_t)i * n);
        kind = 2;
        if (d % s->k == s->k - 1) {
            for (int i = 0; i < K; ++i)
                copy_n(n, s->w, s->wl + (size_t)i * n);    /* Pull w_t      */
            kind = 3;
        }
    }
    s->num += 1;
    return kind;
}

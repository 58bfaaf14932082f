// Fused multi-tensor kernel of one SSD-SGD iteration, for K = SSD_K workers.
//
// One workgroup takes one entry of the chunk table (a run of at most
// chunk_elems elements of one layer tensor) and, per element, reads the K
// gradients, the global weight and the momentum exactly once, applies the
// server update (Eq. (server), momentum rule of Sec. 3.2.1) and -- in the
// steps-delay stage -- the K GLU updates of Algorithm 2 (Eq. (glu-update),
// grad_sync of Sec. 3.3) on the K local weights, plus what Algorithm 1 does
// at the end of the iteration (hand-over at the end of warm-up, Pull every k
// iterations).  All K gradient loads and all K local-weight loads of a
// thread are issued before the first use, as 128-bit accesses whenever every
// pointer of the tensor is 16-byte aligned.
//
// Compiled once per K (-DSSD_K=1..16) so that the worker loops unroll.
#include "ssd_device.h"

#ifndef SSD_K
#error "compile with -DSSD_K=<number of workers>"
#endif

template <int K, int STAGE, int PRE, bool PULL, int VW>
__device__ __forceinline__ void ssd_fused_elems(const ssd_fused_args &a, cgfloat *const (&gp)[K],
                                                gfloat *wp, gfloat *momp, gfloat *prep, gfloat *wlp,
                                                gfloat *wlocp, unsigned e)
{
    typedef ssd_vec<VW> V;
    float g[K][VW], w[VW], mo[VW], wl[K][VW], p[VW];
#pragma unroll
    for (int i = 0; i < K; ++i) V::ld(gp[i] + e, g[i]);
    V::ld(wp + e, w);
    V::ld(momp + e, mo);
    if (STAGE == SSD_STAGE_DELAY) {
#pragma unroll
        for (int i = 0; i < K; ++i) V::ld(wlp + i * a.A + e, wl[i]);
        if (PRE != SSD_PRE_INIT) V::ld(prep + e, p);
    }

    float wn[VW], mn[VW];
#pragma unroll
    for (int v = 0; v < VW; ++v) {
        float S = g[0][v];
#pragma unroll
        for (int i = 1; i < K; ++i) S = S + g[i][v];
        ssd_server_elem(S, w[v], mo[v], a.h, wn[v], mn[v]);
    }
    V::st(momp + e, mn);
    V::st(wp + e, wn);

    if (STAGE == SSD_STAGE_WARMUP_LAST) {
        // Alg. 1, last warm-up iteration: w'_{t,i} = w_t
#pragma unroll
        for (int i = 0; i < K; ++i) V::st(wlp + i * a.A + e, wn);
    }
    if (STAGE == SSD_STAGE_DELAY) {
        // Alg. 2: pre_weight takes w' as it was before this update
        if (PRE != SSD_PRE_KEEP) V::st(prep + e, wl[0]);
#pragma unroll
        for (int i = 0; i < K; ++i) {
            float r[VW];
#pragma unroll
            for (int v = 0; v < VW; ++v) {
                float pv = (PRE == SSD_PRE_INIT) ? wl[i][v] : p[v];
                r[v] = ssd_glu_elem(g[i][v], wl[i][v], pv, a.h);
            }
            if (PULL) {
                // Alg. 1: broadcast the updated w', then Pull w_t into w'
                V::st(wlocp + i * a.A + e, r);
                V::st(wlp + i * a.A + e, wn);
            } else {
                V::st(wlp + i * a.A + e, r);
            }
        }
    }
}

template <int K, int STAGE, int PRE, bool PULL>
__global__ __launch_bounds__(SSD_BLOCK) void ssd_fused_kernel(const ssd_fused_args a)
{
    const ssd_chunk c = a.chunks[blockIdx.x];
    const ssd_tensor_desc td = a.tensors[c.tensor];
    cgfloat *gp[K];
    bool vec = ssd_aligned16(td.w);
#pragma unroll
    for (int i = 0; i < K; ++i) {
        const float *g = a.gptr[(int64_t)c.tensor * K + i];
        vec = vec && ssd_aligned16(g);
        gp[i] = ssd_global(g) + c.offset;
    }
    gfloat *wp = ssd_global(td.w) + c.offset;
    const int64_t ao = td.arena_off + c.offset;
    gfloat *momp = ssd_global(a.mom) + ao, *prep = ssd_global(a.pre) + ao;
    gfloat *wlp = ssd_global(a.wl) + ao, *wlocp = ssd_global(a.wloc) + ao;
    const unsigned len = (unsigned)c.len;
    const unsigned tid = threadIdx.x;

    if (vec) {
        const unsigned len4 = len & ~3u;
        for (unsigned e = tid * 4; e < len4; e += SSD_BLOCK * 4)
            ssd_fused_elems<K, STAGE, PRE, PULL, 4>(a, gp, wp, momp, prep, wlp, wlocp, e);
        const unsigned e = len4 + tid;
        if (e < len) ssd_fused_elems<K, STAGE, PRE, PULL, 1>(a, gp, wp, momp, prep, wlp, wlocp, e);
    } else {
        for (unsigned e = tid; e < len; e += SSD_BLOCK)
            ssd_fused_elems<K, STAGE, PRE, PULL, 1>(a, gp, wp, momp, prep, wlp, wlocp, e);
    }
}

#define SSD_CAT2(a, b) a##b
#define SSD_CAT(a, b) SSD_CAT2(a, b)

hipError_t SSD_CAT(ssd_launch_fused_k, SSD_K)(int stage, int pre_action, int pull, unsigned nchunks,
                                               hipStream_t s, const ssd_fused_args &a)
{
    const dim3 grid(nchunks), block(SSD_BLOCK);
#define SSD_GO(ST, PR, PU)                                                         \
    do {                                                                           \
        ssd_fused_kernel<SSD_K, ST, PR, PU><<<grid, block, 0, s>>>(a);             \
        return hipGetLastError();                                                  \
    } while (0)
    if (stage == SSD_STAGE_WARMUP) SSD_GO(SSD_STAGE_WARMUP, SSD_PRE_KEEP, false);
    if (stage == SSD_STAGE_WARMUP_LAST) SSD_GO(SSD_STAGE_WARMUP_LAST, SSD_PRE_KEEP, false);
    if (stage == SSD_STAGE_DELAY) {
        if (pre_action == SSD_PRE_KEEP && !pull) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_KEEP, false);
        if (pre_action == SSD_PRE_KEEP && pull) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_KEEP, true);
        if (pre_action == SSD_PRE_INIT && !pull) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_INIT, false);
        if (pre_action == SSD_PRE_INIT && pull) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_INIT, true);
        if (pre_action == SSD_PRE_REFRESH && !pull) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_REFRESH, false);
        if (pre_action == SSD_PRE_REFRESH && pull) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_REFRESH, true);
    }
    return hipErrorInvalidValue;
}

// Fused multi-tensor kernel of one SSD-SGD iteration, for K = SSD_K workers.
//
// One workgroup takes one entry of the chunk table (a run of at most
// chunk_elems elements of one layer tensor) and, per element, reads the K
// gradients, the global weight and the momentum exactly once, applies the
// server update (Eq. (server), momentum rule of Sec. 3.2.1) and -- in the
// steps-delay stage -- the K GLU updates of Algorithm 2 (Eq. (glu-update),
// grad_sync of Sec. 3.3) on the K local weights.  What Algorithm 1 does at the
// end of an iteration moves no data here: after the hand-over at the end of
// warm-up and after a Pull, every w'_i equals the global weight, so the host
// only records that fact and the next launch (template flag FG) takes w'_i from
// the global weight it loads anyway.  All K gradient loads and all K local-weight loads of a
// thread are issued before the first use, as 128-bit accesses whenever every
// pointer of the tensor is 16-byte aligned.
//
// Compiled once per K (-DSSD_K=1..16) so that the worker loops unroll.
#include "ssd_device.h"

#ifndef SSD_K
#error "compile with -DSSD_K=<number of workers>"
#endif

template <int K, int STAGE, int PRE, bool FG, int VW>
__device__ __forceinline__ void ssd_fused_elems(const ssd_fused_args &a, cgfloat *const (&gp)[K],
                                                gfloat *wp, gfloat *momp, gfloat *prep, gfloat *wlp,
                                                unsigned e)
{
    typedef ssd_vec<VW> V;
    float g[K][VW], w[VW], mo[VW], wl[K][VW], p[VW];
#pragma unroll
    for (int i = 0; i < K; ++i) V::ld(gp[i] + e, g[i]);
    V::ld(wp + e, w);
    V::ld(momp + e, mo);
    if (STAGE == SSD_STAGE_DELAY) {
        if (!FG) {
#pragma unroll
            for (int i = 0; i < K; ++i) V::ld(wlp + i * a.A + e, wl[i]);
        }
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

    if (STAGE == SSD_STAGE_DELAY) {
        // FG: every w'_i is the global weight as it stood before this
        // iteration's server update (after a Pull, or at the end of warm-up),
        // which is in registers already; the w' arrays are not read.
        // Alg. 2: pre_weight takes w' as it was before this update.
        if (PRE != SSD_PRE_KEEP) V::st(prep + e, FG ? w : wl[0]);
#pragma unroll
        for (int i = 0; i < K; ++i) {
            float r[VW];
#pragma unroll
            for (int v = 0; v < VW; ++v) {
                const float wli = FG ? w[v] : wl[i][v];
                const float pv = (PRE == SSD_PRE_INIT) ? wli : p[v];
                r[v] = ssd_glu_elem(g[i][v], wli, pv, a.h);
            }
            V::st(wlp + i * a.A + e, r);
        }
    }
}

template <int K, int STAGE, int PRE, bool FG>
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
    gfloat *wlp = ssd_global(a.wl) + ao;
    const unsigned len = (unsigned)c.len;
    const unsigned tid = threadIdx.x;

    if (vec) {
        const unsigned len4 = len & ~3u;
        for (unsigned e = tid * 4; e < len4; e += SSD_BLOCK * 4)
            ssd_fused_elems<K, STAGE, PRE, FG, 4>(a, gp, wp, momp, prep, wlp, e);
        const unsigned e = len4 + tid;
        if (e < len) ssd_fused_elems<K, STAGE, PRE, FG, 1>(a, gp, wp, momp, prep, wlp, e);
    } else {
        for (unsigned e = tid; e < len; e += SSD_BLOCK)
            ssd_fused_elems<K, STAGE, PRE, FG, 1>(a, gp, wp, momp, prep, wlp, e);
    }
}

#define SSD_CAT2(a, b) a##b
#define SSD_CAT(a, b) SSD_CAT2(a, b)

hipError_t SSD_CAT(ssd_launch_fused_k, SSD_K)(int stage, int pre_action, int from_global, int waves_per_cu, unsigned nchunks,
                                               hipStream_t s, const ssd_fused_args &a)
{
    const dim3 grid(nchunks), block(SSD_BLOCK);
    const unsigned lds = ssd_lds_for_waves(waves_per_cu); // occupancy cap only, never accessed
#define SSD_GO(ST, PR, FG)                                                         \
    do {                                                                           \
        if (lds > 65536)                                                           \
            (void)hipFuncSetAttribute((const void *)ssd_fused_kernel<SSD_K, ST, PR, FG>,   \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        ssd_fused_kernel<SSD_K, ST, PR, FG><<<grid, block, lds, s>>>(a);           \
        return hipGetLastError();                                                  \
    } while (0)
    if (stage == SSD_STAGE_WARMUP) SSD_GO(SSD_STAGE_WARMUP, SSD_PRE_KEEP, false);
    if (stage == SSD_STAGE_DELAY) {
        if (pre_action == SSD_PRE_KEEP && !from_global) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_KEEP, false);
        if (pre_action == SSD_PRE_INIT && !from_global) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_INIT, false);
        if (pre_action == SSD_PRE_INIT && from_global) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_INIT, true);
        if (pre_action == SSD_PRE_REFRESH && !from_global) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_REFRESH, false);
        if (pre_action == SSD_PRE_REFRESH && from_global) SSD_GO(SSD_STAGE_DELAY, SSD_PRE_REFRESH, true);
    }
    return hipErrorInvalidValue;
}

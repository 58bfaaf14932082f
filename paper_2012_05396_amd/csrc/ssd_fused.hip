// Fused multi-tensor kernel of one SSD-SGD iteration, for K = SSD_K workers.
//
// One single-wave workgroup takes one block of the arena (chunk_elems elements
// of one layer tensor) and, per element, reads the K gradients, the global
// weight, the momentum, pre_weight and the K local weights exactly once,
// applies the server update (Eq. (server), momentum rule of Sec. 3.2.1) and
// -- in the steps-delay stage -- the K GLU updates of Algorithm 2
// (Eq. (glu-update), grad_sync of Sec. 3.3) on the K local weights.  What
// Algorithm 1 does at the end of an iteration moves no data here: after the
// hand-over at the end of warm-up and after a Pull, every w'_i equals the
// global weight, so the host only records that fact and the next launch
// (template flag FG) takes w'_i from the global weight it loads anyway.
//
// Order of issue inside a wave: the loads of the library's own state (momentum,
// pre_weight, K local weights) need nothing but blockIdx, so they go out first;
// the two table lookups that lead to the caller's pointers (block -> tensor,
// tensor -> one record with the weight and K gradient pointers) overlap with
// them; then the gradient and
// weight loads; then arithmetic and stores.  128-bit accesses whenever every
// caller pointer of the tensor is 16-byte aligned, else element by element.
//
// Compiled once per K (-DSSD_K=1..16) so that the worker loops unroll, and per
// element type of the gradient buffers (-DSSD_GD=0..2).
#include "ssd_device.h"

#ifndef SSD_K
#error "compile with -DSSD_K=<number of workers>"
#endif
#ifndef SSD_GD
#error "compile with -DSSD_GD=<ssd_grad_dtype of the gradient buffers>"
#endif

template <int K, int VW> struct ssd_state_regs {
    float mo[VW], p[VW], wl[K][VW];
};

template <int K, int STAGE, int PRE, bool FG, int VW>
__device__ __forceinline__ void ssd_load_state(const ssd_fused_args &a, gfloat *momp, gfloat *prep,
                                               gfloat *wlp, unsigned e, ssd_state_regs<K, VW> &s)
{
    typedef ssd_vec<VW> V;
    V::ld(momp + e, s.mo);
    if (STAGE == SSD_STAGE_DELAY) {
        if (PRE != SSD_PRE_INIT) V::ld(prep + e, s.p);
        if (!FG) {
#pragma unroll
            for (int i = 0; i < K; ++i) V::ld(wlp + i * a.A + e, s.wl[i]);
        }
    }
}

template <int K, int GD, int STAGE, int PRE, bool FG, bool XW, int VW>
__device__ __forceinline__ void ssd_finish(const ssd_fused_args &a, const ssd_hyper &h,
                                           const typename ssd_gvec<GD, 4>::ptr (&gp)[K], gfloat *wp, gfloat *momp,
                                           gfloat *prep, gfloat *wlp, unsigned e,
                                           const ssd_state_regs<K, VW> &s)
{
    typedef ssd_vec<VW> V;
    float g[K][VW], w[VW];
#pragma unroll
    for (int i = 0; i < K; ++i) ssd_gvec<GD, VW>::ld(gp[i] + e, g[i]);
    V::ld(wp + e, w);

    float wn[VW], mn[VW];
#pragma unroll
    for (int v = 0; v < VW; ++v) {
        float S = g[0][v];
#pragma unroll
        for (int i = 1; i < K; ++i) S = S + g[i][v];
        ssd_server_elem(S, w[v], s.mo[v], h, wn[v], mn[v]);
    }
    V::st(momp + e, mn);
    V::st(wp + e, wn);

    if (STAGE == SSD_STAGE_DELAY) {
        // FG: every w'_i is the global weight as it stood before this
        // iteration's server update (after a Pull, or at the end of warm-up),
        // which is in registers already; the w' arrays are not read.
        // Alg. 2: pre_weight takes w' as it was before this update.
        if (PRE != SSD_PRE_KEEP) V::st(prep + e, FG ? w : s.wl[0]);
#pragma unroll
        for (int i = 0; i < K; ++i) {
            float r[VW];
#pragma unroll
            for (int v = 0; v < VW; ++v) {
                const float wli = FG ? w[v] : s.wl[i][v];
                const float pv = (PRE == SSD_PRE_INIT) ? wli : s.p[v];
                r[v] = ssd_glu_elem<XW>(g[i][v], wli, pv, h);
            }
            V::st(wlp + i * a.A + e, r);
        }
    }
}

// One 256-element tile: lane l owns elements e0 .. e0+3 (e0 = base + 4l).
// Full vectors take the 128-bit path; a lane at the ragged end of the block,
// or any lane when a caller pointer is not 16-byte aligned, goes element by
// element -- in both cases with the state values preloaded in `s`.
template <int K, int GD, int STAGE, int PRE, bool FG, bool XW>
__device__ __forceinline__ void ssd_tile(const ssd_fused_args &a, const ssd_hyper &h,
                                         const typename ssd_gvec<GD, 4>::ptr (&gp)[K], gfloat *wp, gfloat *momp,
                                         gfloat *prep, gfloat *wlp, unsigned e0, unsigned len, bool vec,
                                         const ssd_state_regs<K, 4> &s)
{
    if (vec && e0 + 3 < len) {
        ssd_finish<K, GD, STAGE, PRE, FG, XW, 4>(a, h, gp, wp, momp, prep, wlp, e0, s);
    } else if (e0 < len) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (e0 + v < len) {
                ssd_state_regs<K, 1> s1;
                s1.mo[0] = s.mo[v];
                s1.p[0] = s.p[v];
#pragma unroll
                for (int i = 0; i < K; ++i) s1.wl[i][0] = s.wl[i][v];
                ssd_finish<K, GD, STAGE, PRE, FG, XW, 1>(a, h, gp, wp, momp, prep, wlp, e0 + v, s1);
            }
        }
    }
}

// The arguments a wave needs first come as separate leading kernel arguments
// so that they can be preloaded into scalar registers at wave launch
// (-amdgpu-kernarg-preload-count); the rest arrives with ordinary scalar loads.
template <int K, int GD, int STAGE, int PRE, bool FG, bool XW>
__global__ __launch_bounds__(SSD_BLOCK) void ssd_fused_kernel(const int32_t *block_tensor, float *mom,
                                                              float *pre, float *wl, int64_t A,
                                                              unsigned C, unsigned blocks_per_xcd,
                                                              const int64_t *rec_table,
                                                              const ssd_tensor_hyper *thyper,
                                                              const ssd_hyper hglobal)
{
    ssd_fused_args a;
    a.tab.block_tensor = block_tensor;
    a.tab.tensors = nullptr;
    a.tab.C = C;
    a.tab.blocks_per_xcd = blocks_per_xcd;
    a.rec = rec_table;
    a.mom = mom;
    a.pre = pre;
    a.wl = wl;
    a.A = A;
    a.thyper = thyper;
    a.h = hglobal;
    const unsigned lane = threadIdx.x;
    // head of the lookup chain: request it first
    const int t = a.tab.block_tensor[ssd_block_slot(blockIdx.x, a.tab.blocks_per_xcd)];
    // state arrays: addressed by blockIdx alone, always 16-byte aligned, and
    // padded to whole blocks, so the first tile is requested right away
    const int64_t ao = (int64_t)blockIdx.x * a.tab.C;
    gfloat *momp = ssd_global(a.mom) + ao, *prep = ssd_global(a.pre) + ao;
    gfloat *wlp = ssd_global(a.wl) + ao;
    ssd_state_regs<K, 4> s;
    ssd_load_state<K, STAGE, PRE, FG, 4>(a, momp, prep, wlp, lane * 4, s);

    // block -> tensor -> one record {w, first_block, numel, g_0 .. g_{K-1}}
    // and the tensor's hyper-parameters
    const ssd_hyper h = ssd_hyper_of(a.h, a.thyper[t]);
    const int64_t *rec = a.rec + (int64_t)t * (K + 3);
    float *w = reinterpret_cast<float *>(rec[0]);
    const int64_t off = ((int64_t)blockIdx.x - rec[1]) * a.tab.C;
    const int64_t left = rec[2] - off;
    const unsigned len = left < (int64_t)a.tab.C ? (unsigned)left : a.tab.C;
    typedef typename ssd_gvec<GD, 4>::ptr gptr;
    gptr gp[K];
    bool vec = ssd_aligned16(w);
#pragma unroll
    for (int i = 0; i < K; ++i) {
        const void *g = reinterpret_cast<const void *>(rec[3 + i]);
        vec = vec && ssd_grad_aligned<GD>(g);
        gp[i] = (gptr)g + off;
    }
    gfloat *wp = ssd_global(w) + off;

    unsigned base = 0;
    for (;;) {
        ssd_tile<K, GD, STAGE, PRE, FG, XW>(a, h, gp, wp, momp, prep, wlp, base + lane * 4, len, vec, s);
        base += SSD_BLOCK * 4;
        if (base >= len) break; // uniform
        ssd_load_state<K, STAGE, PRE, FG, 4>(a, momp, prep, wlp, base + lane * 4, s);
    }
}

#define SSD_CAT2(a, b) a##b
#define SSD_CAT(a, b) SSD_CAT2(a, b)

hipError_t SSD_CAT(SSD_CAT(SSD_CAT(ssd_launch_fused_g, SSD_GD), _k), SSD_K)(int stage, int pre_action, int from_global, int exact_w_minus,
                                               int waves_per_cu, unsigned nchunks, hipStream_t s,
                                               const ssd_fused_args &a)
{
    const dim3 grid(nchunks), block(SSD_BLOCK);
    const unsigned lds = ssd_lds_for_waves(waves_per_cu); // occupancy cap only, never accessed
#define SSD_GO(ST, PR, FG, XW)                                                     \
    do {                                                                           \
        if (lds > 65536)                                                           \
            (void)hipFuncSetAttribute((const void *)ssd_fused_kernel<SSD_K, SSD_GD, ST, PR, FG, XW>, \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        ssd_fused_kernel<SSD_K, SSD_GD, ST, PR, FG, XW><<<grid, block, lds, s>>>(            \
            a.tab.block_tensor, a.mom, a.pre, a.wl, a.A, a.tab.C, a.tab.blocks_per_xcd, a.rec, a.thyper,  \
            a.h);                                                                    \
        return hipGetLastError();                                                  \
    } while (0)
#define SSD_GO_DELAY(PR, FG)                                                       \
    do {                                                                           \
        if (exact_w_minus) SSD_GO(SSD_STAGE_DELAY, PR, FG, true);                  \
        SSD_GO(SSD_STAGE_DELAY, PR, FG, false);                                    \
    } while (0)
    if (stage == SSD_STAGE_WARMUP) SSD_GO(SSD_STAGE_WARMUP, SSD_PRE_KEEP, false, false);
    if (stage == SSD_STAGE_DELAY) {
        if (pre_action == SSD_PRE_KEEP && !from_global) SSD_GO_DELAY(SSD_PRE_KEEP, false);
        if (pre_action == SSD_PRE_INIT && !from_global) SSD_GO_DELAY(SSD_PRE_INIT, false);
        if (pre_action == SSD_PRE_INIT && from_global) SSD_GO_DELAY(SSD_PRE_INIT, true);
        if (pre_action == SSD_PRE_REFRESH && !from_global) SSD_GO_DELAY(SSD_PRE_REFRESH, false);
        if (pre_action == SSD_PRE_REFRESH && from_global) SSD_GO_DELAY(SSD_PRE_REFRESH, true);
    }
    return hipErrorInvalidValue;
}

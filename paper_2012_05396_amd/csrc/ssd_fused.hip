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
// pre_weight, the K local weights) need nothing but blockIdx, so they go out
// first; the two table lookups that lead to the caller's pointers (block ->
// tensor, tensor -> one record with the weight and K gradient pointers)
// overlap with them; then the K gradient loads and the weight load; then
// arithmetic and stores.  A wave asks for its whole tile at once, 2K+3 loads
// per lane; how many waves a compute unit holds is capped by the host
// (ssd_lds_slice_bytes).  128-bit accesses whenever every caller pointer of the
// tensor is 16-byte aligned, else element by element.
//
// The K local weights of a block are K arrays a whole arena apart (K <= 8) or
// lie side by side (K > 8), see ssd_interleave_of.
//
// NT selects the marking of every global access: non-temporal for models
// that stream through HBM, ordinary for models whose arrays stay in the
// last-level cache from one iteration to the next (the host decides by size).
//
// Compiled once per K (-DSSD_K=1..16) so that the worker loops unroll, and per
// element type of the gradient buffers (-DSSD_GD=0..2).
#include <atomic>

#include "ssd_device.h"

#ifndef SSD_K
#error "compile with -DSSD_K=<number of workers>"
#endif
#ifndef SSD_GD
#error "compile with -DSSD_GD=<ssd_grad_dtype of the gradient buffers>"
#endif

// state of the tile that is requested before the table lookups return
template <int K, int VW> struct ssd_head_regs {
    float mo[VW], p[VW], wl[K][VW];
};

template <int K, int STAGE, int PRE, bool FG, bool NT, int VW>
__device__ __forceinline__ void ssd_load_head(gfloat *momp, gfloat *prep, gfloat *wlp, int64_t WS, unsigned e,
                                              ssd_head_regs<K, VW> &s)
{
    ssd_vec<VW, NT>::ld(momp + e, s.mo);
    if (STAGE == SSD_STAGE_DELAY) {
        if (PRE != SSD_PRE_INIT) ssd_vec<VW, NT>::ld(prep + e, s.p);
        if (!FG) {
#pragma unroll
            for (int i = 0; i < K; ++i) ssd_vec<VW, NT>::ld(wlp + (int64_t)i * WS + e, s.wl[i]);
        }
    }
}

// Elements e .. e+VW-1 of the tile, given the head state in `s`.
//
// The server update comes first: it needs every gradient of the tile, so all
// loads have been waited for before the first store is issued.  The 128-bit
// "sc1 nt" stores are inline assembly that the compiler does not count when it
// forms s_waitcnt, so a wait for a load placed after such a store would also
// wait for the store's acknowledgement; and left to itself the scheduler then
// also sinks late gradient loads below arithmetic on early ones (16-bit
// gradient kernels: 5.85 instead of 6.39 TB/s).
template <int K, int GD, int STAGE, int PRE, bool FG, bool XW, bool NT, int VW>
__device__ __forceinline__ void ssd_finish(const ssd_hyper &h, const typename ssd_gvec<GD, 4>::ptr (&gp)[K],
                                           gfloat *wp, gfloat *momp, gfloat *prep, gfloat *wlp, int64_t WS,
                                           unsigned e, const ssd_head_regs<K, VW> &s)
{
    typedef ssd_vec<VW, NT> V;
    float g[K][VW], w[VW], S[VW], wn[VW], mn[VW];
#pragma unroll
    for (int i = 0; i < K; ++i) ssd_gvec<GD, VW, NT>::ld(gp[i] + e, g[i]);
    V::ld(wp + e, w);

    // Eq. (server): the sum of the K gradients, in worker order
#pragma unroll
    for (int i = 0; i < K; ++i) {
#pragma unroll
        for (int v = 0; v < VW; ++v) S[v] = (i == 0) ? g[i][v] : S[v] + g[i][v];
    }
#pragma unroll
    for (int v = 0; v < VW; ++v) ssd_server_elem(S[v], w[v], s.mo[v], h, wn[v], mn[v]);
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
            V::st(wlp + (int64_t)i * WS + e, r);
        }
    }
}

// One 256-element tile: lane l owns elements e0 .. e0+3 (e0 = base + 4l);
// elements lo .. len-1 of the block belong to the tensor.  Full vectors take
// the 128-bit path; a lane at a ragged end of the block, or any lane when a
// caller pointer is not 16-byte aligned, goes element by element -- in both
// cases with the head state preloaded in `s`.
template <int K, int GD, int STAGE, int PRE, bool FG, bool XW, bool NT>
__device__ __forceinline__ void ssd_tile(const ssd_hyper &h, const typename ssd_gvec<GD, 4>::ptr (&gp)[K],
                                         gfloat *wp, gfloat *momp, gfloat *prep, gfloat *wlp, int64_t WS,
                                         unsigned e0, unsigned lo, unsigned len, bool vec,
                                         const ssd_head_regs<K, 4> &s)
{
    if (vec && e0 >= lo && e0 + 3 < len) {
        ssd_finish<K, GD, STAGE, PRE, FG, XW, NT, 4>(h, gp, wp, momp, prep, wlp, WS, e0, s);
    } else if (e0 + 3 >= lo && e0 < len) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (e0 + v >= lo && e0 + v < len) {
                ssd_head_regs<K, 1> s1;
                s1.mo[0] = s.mo[v];
                s1.p[0] = s.p[v];
#pragma unroll
                for (int i = 0; i < K; ++i) s1.wl[i][0] = s.wl[i][v];
                ssd_finish<K, GD, STAGE, PRE, FG, XW, NT, 1>(h, gp, wp, momp, prep, wlp, WS, e0 + v, s1);
            }
        }
    }
}

// The arguments a wave needs first come as separate leading kernel arguments
// so that they can be preloaded into scalar registers at wave launch
// (-amdgpu-kernarg-preload-count); the rest arrives with ordinary scalar loads.
template <int K, int GD, int STAGE, int PRE, bool FG, bool XW, bool NT>
__global__ __launch_bounds__(SSD_BLOCK) void ssd_fused_kernel(const int32_t *block_tensor, float *mom,
                                                              float *pre, float *wl, int64_t A,
                                                              unsigned C, unsigned blocks_per_xcd,
                                                              const int64_t *rec_table,
                                                              const ssd_tensor_hyper *thyper,
                                                              const ssd_hyper hglobal)
{
    const unsigned lane = threadIdx.x;
    // head of the lookup chain: request it first
    const int t = block_tensor[ssd_block_slot(blockIdx.x, blocks_per_xcd)];
    // state arrays: addressed by blockIdx alone, always 16-byte aligned, and
    // padded to whole blocks, so the first tile is requested right away
    const int64_t ao = (int64_t)blockIdx.x * C;
    gfloat *momp = ssd_global(mom) + ao, *prep = ssd_global(pre) + ao;
    // local weights: planar arrays A apart, or the K copies of a block side by side
    constexpr bool IL = ssd_interleave_of(K);
    gfloat *wlp = ssd_global(wl) + (IL ? ao * K : ao);
    const int64_t WS = IL ? (int64_t)C : A; // from worker i's copy of the block to worker i+1's
    ssd_head_regs<K, 4> s;
    ssd_load_head<K, STAGE, PRE, FG, NT, 4>(momp, prep, wlp, WS, lane * 4, s);

    // block -> tensor -> one record {w, elem0, numel, g_0 .. g_{K-1}}
    // and the tensor's hyper-parameters
    // thyper == NULL: no tensor has multipliers, the global values hold for all
    const ssd_hyper h = thyper ? ssd_hyper_of(hglobal, thyper[t]) : hglobal;
    const int64_t *rec = rec_table + (int64_t)t * (K + 3);
    float *w = reinterpret_cast<float *>(rec[0]);
    int64_t off;
    unsigned lo, len;
    ssd_block_range((int64_t)blockIdx.x, C, rec[1], rec[2], off, lo, len);
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
        ssd_tile<K, GD, STAGE, PRE, FG, XW, NT>(h, gp, wp, momp, prep, wlp, WS, base + lane * 4, lo, len, vec, s);
        base += SSD_BLOCK * 4;
        if (base >= len) break; // uniform
        ssd_load_head<K, STAGE, PRE, FG, NT, 4>(momp, prep, wlp, WS, base + lane * 4, s);
    }
}

#define SSD_CAT2(a, b) a##b
#define SSD_CAT(a, b) SSD_CAT2(a, b)

// A slice of LDS above 64 KiB needs the kernel's dynamic-LDS limit raised;
// that is a property of the kernel on a device, set once per kernel variant
// and device (bit d of `done`), not per launch.  Contexts on different host
// threads share the word: two of them may both set the attribute the first
// time (harmless, same value), never read a torn word.
template <typename Kernel>
static hipError_t ssd_allow_lds(Kernel kernel, unsigned lds, std::atomic<unsigned long long> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = dev < 64 ? 1ull << dev : 0; // beyond 64 devices: set it every time
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

hipError_t SSD_CAT(SSD_CAT(SSD_CAT(ssd_launch_fused_g, SSD_GD), _k), SSD_K)(int stage, int pre_action, int from_global, int exact_w_minus, int streaming,
                                               unsigned lds_bytes, unsigned lds_limit, unsigned nchunks, hipStream_t s,
                                               const ssd_fused_args &a)
{
    const dim3 grid(nchunks), block(SSD_BLOCK);
    // lds_bytes: the occupancy cap, a slice of LDS that is never accessed
#define SSD_GO(ST, PR, FG, XW)                                                                     \
    do {                                                                                           \
        if (streaming) SSD_GO_NT(ST, PR, FG, XW, true);                                            \
        SSD_GO_NT(ST, PR, FG, XW, false);                                                          \
    } while (0)
#define SSD_GO_NT(ST, PR, FG, XW, NT)                                                              \
    do {                                                                                           \
        auto kernel = ssd_fused_kernel<SSD_K, SSD_GD, ST, PR, FG, XW, NT>;                         \
        if (lds_bytes > 65536) {                                                                   \
            static std::atomic<unsigned long long> done{0};                                        \
            const hipError_t e = ssd_allow_lds(kernel, lds_limit, done);                           \
            if (e != hipSuccess) return e;                                                         \
        }                                                                                          \
        kernel<<<grid, block, lds_bytes, s>>>(a.tab.block_tensor, a.mom, a.pre, a.wl, a.A, a.tab.C, \
                                              a.tab.blocks_per_xcd, a.rec, a.thyper, a.h);         \
        return hipGetLastError();                                                                  \
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

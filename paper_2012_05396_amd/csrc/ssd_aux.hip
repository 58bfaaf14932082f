// Piecewise kernels: one worker's GLU update (Algorithm 2), one worker's Pull
// (Algorithm 1), and a fill.  They walk the same chunk table as the fused
// kernel and use the same element-wise rules, so a sequence of piecewise
// calls gives the bits of the fused step.
#include "ssd_device.h"

template <int PRE, int GD, int VW>
__device__ __forceinline__ void ssd_glu_elems(const ssd_hyper &h, typename ssd_gvec<GD, 4>::ptr gp, gfloat *wlp,
                                              cgfloat *presrc, gfloat *predst, unsigned e)
{
    typedef ssd_vec<VW> V;
    float g[VW], wl[VW], p[VW], r[VW];
    ssd_gvec<GD, VW>::ld(gp + e, g);
    V::ld(wlp + e, wl);
    if (PRE != SSD_PRE_INIT) V::ld(presrc + e, p);
#pragma unroll
    for (int v = 0; v < VW; ++v) {
        float pv = (PRE == SSD_PRE_INIT) ? wl[v] : p[v];
        r[v] = ssd_glu_elem<true>(g[v], wl[v], pv, h); // pre_scale is 1 unless the variant is on
    }
    if (PRE != SSD_PRE_KEEP) V::st(predst + e, wl);
    V::st(wlp + e, r);
}

template <int PRE, int GD>
__global__ __launch_bounds__(SSD_BLOCK) void ssd_glu_kernel(const ssd_glu_args a)
{
    ssd_tensor_desc td;
    const ssd_block blk = ssd_locate(a.tab, blockIdx.x, td);
    const void *g = a.gptr[blk.tensor];
    const bool vec = ssd_grad_aligned<GD>(g);
    typedef typename ssd_gvec<GD, 4>::ptr gptr;
    const gptr gp = (gptr)g + blk.off;
    gfloat *wlp = ssd_global(a.wl) + (int64_t)blockIdx.x * a.wl_block_stride;
    cgfloat *presrc = ssd_global(a.pre_src) + blk.ao;
    gfloat *predst = ssd_global(a.pre_dst) + blk.ao;
    const unsigned lo = blk.lo, len = blk.len, tid = threadIdx.x;
    const ssd_hyper h = a.thyper ? ssd_hyper_of(a.h, a.thyper[blk.tensor]) : a.h;
    if (vec) {
        // whole vectors from the lead-in (a multiple of 4 elements, see
        // ssd_tensor_desc) to the last whole vector, then the tail
        const unsigned len4 = lo + ((len - lo) & ~3u);
        for (unsigned e = lo + tid * 4; e < len4; e += SSD_BLOCK * 4)
            ssd_glu_elems<PRE, GD, 4>(h, gp, wlp, presrc, predst, e);
        const unsigned e = len4 + tid;
        if (e < len) ssd_glu_elems<PRE, GD, 1>(h, gp, wlp, presrc, predst, e);
    } else {
        for (unsigned e = lo + tid; e < len; e += SSD_BLOCK)
            ssd_glu_elems<PRE, GD, 1>(h, gp, wlp, presrc, predst, e);
    }
}

template <int GD>
static hipError_t ssd_launch_glu_of(int pre_action, unsigned nchunks, hipStream_t s, const ssd_glu_args &a)
{
    const dim3 grid(nchunks), block(SSD_BLOCK);
    switch (pre_action) {
    case SSD_PRE_KEEP: ssd_glu_kernel<SSD_PRE_KEEP, GD><<<grid, block, 0, s>>>(a); break;
    case SSD_PRE_INIT: ssd_glu_kernel<SSD_PRE_INIT, GD><<<grid, block, 0, s>>>(a); break;
    case SSD_PRE_REFRESH: ssd_glu_kernel<SSD_PRE_REFRESH, GD><<<grid, block, 0, s>>>(a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t ssd_launch_glu(int grad_dtype, int pre_action, unsigned nchunks, hipStream_t s, const ssd_glu_args &a)
{
    switch (grad_dtype) {
    case SSD_GRAD_F32: return ssd_launch_glu_of<SSD_GRAD_F32>(pre_action, nchunks, s, a);
    case SSD_GRAD_BF16: return ssd_launch_glu_of<SSD_GRAD_BF16>(pre_action, nchunks, s, a);
    case SSD_GRAD_F16: return ssd_launch_glu_of<SSD_GRAD_F16>(pre_action, nchunks, s, a);
    default: return hipErrorInvalidValue;
    }
}

// INIT: w'_i = w_t and w_loc_i = w_t.  Otherwise w_loc_i = w'_i, then w'_i = w_t.
template <bool INIT, int VW>
__device__ __forceinline__ void ssd_pull_elems(cgfloat *wp, gfloat *wlp, gfloat *wlocp, unsigned e)
{
    typedef ssd_vec<VW> V;
    float w[VW], wl[VW];
    V::ld(wp + e, w);
    if (!INIT) {
        V::ld(wlp + e, wl);
        V::st(wlocp + e, wl);
    } else {
        V::st(wlocp + e, w);
    }
    V::st(wlp + e, w);
}

template <bool INIT>
__global__ __launch_bounds__(SSD_BLOCK) void ssd_pull_kernel(const ssd_pull_args a)
{
    ssd_tensor_desc td;
    const ssd_block blk = ssd_locate(a.tab, blockIdx.x, td);
    const bool vec = ssd_aligned16(td.w);
    cgfloat *wp = ssd_global((const float *)td.w) + blk.off;
    gfloat *wlp = ssd_global(a.wl) + (int64_t)blockIdx.x * a.wl_block_stride;
    gfloat *wlocp = ssd_global(a.wloc) + blk.ao;
    const unsigned lo = blk.lo, len = blk.len, tid = threadIdx.x;
    if (vec) {
        const unsigned len4 = lo + ((len - lo) & ~3u);
        for (unsigned e = lo + tid * 4; e < len4; e += SSD_BLOCK * 4)
            ssd_pull_elems<INIT, 4>(wp, wlp, wlocp, e);
        const unsigned e = len4 + tid;
        if (e < len) ssd_pull_elems<INIT, 1>(wp, wlp, wlocp, e);
    } else {
        for (unsigned e = lo + tid; e < len; e += SSD_BLOCK) ssd_pull_elems<INIT, 1>(wp, wlp, wlocp, e);
    }
}

hipError_t ssd_launch_pull(int init, unsigned nchunks, hipStream_t s, const ssd_pull_args &a)
{
    const dim3 grid(nchunks), block(SSD_BLOCK);
    if (init)
        ssd_pull_kernel<true><<<grid, block, 0, s>>>(a);
    else
        ssd_pull_kernel<false><<<grid, block, 0, s>>>(a);
    return hipGetLastError();
}

// n is a multiple of 4 and p is 16-byte aligned (state arrays are padded).
__global__ __launch_bounds__(SSD_COPY_BLOCK) void ssd_fill_zero_kernel(float *p, int64_t n4)
{
    typedef float v4 __attribute__((ext_vector_type(4)));
    const v4 z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = (int64_t)blockIdx.x * SSD_COPY_BLOCK + threadIdx.x; i < n4;
         i += (int64_t)gridDim.x * SSD_COPY_BLOCK)
        reinterpret_cast<v4 *>(p)[i] = z;
}

hipError_t ssd_launch_fill_zero(float *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t n4 = n / 4;
    int64_t blocks = (n4 + SSD_COPY_BLOCK - 1) / SSD_COPY_BLOCK;
    if (blocks > 8192) blocks = 8192;
    ssd_fill_zero_kernel<<<dim3((unsigned)blocks), dim3(SSD_COPY_BLOCK), 0, s>>>(p, n4);
    return hipGetLastError();
}

// Measurement aid: a plain copy with the library's own load/store helpers.
__global__ __launch_bounds__(SSD_COPY_BLOCK) void ssd_probe_copy_kernel(const float *s, float *d, int64_t n)
{
    cgfloat *src = ssd_global(s);
    gfloat *dst = ssd_global(d);
    const int64_t e = ((int64_t)blockIdx.x * SSD_COPY_BLOCK + threadIdx.x) * 4;
    if (e < n) {
        float x[4];
        ssd_vec<4>::ld(src + e, x);
        ssd_vec<4>::st(dst + e, x);
    }
}

extern "C" int ssd_probe_copy(const float *src, float *dst, int64_t n, void *stream)
{
    if (!src || !dst || n < 0 || n % 4) return SSD_EINVAL;
    if (!ssd_aligned16_host(src) || !ssd_aligned16_host(dst)) return SSD_EALIGN;
    if (n == 0) return SSD_OK;
    const int64_t blocks = (n / 4 + SSD_COPY_BLOCK - 1) / SSD_COPY_BLOCK;
    if (blocks > 0x7fffffffLL) return SSD_EINVAL;
    ssd_probe_copy_kernel<<<dim3((unsigned)blocks), dim3(SSD_COPY_BLOCK), 0, static_cast<hipStream_t>(stream)>>>(
        src, dst, n);
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_EHIP;
}

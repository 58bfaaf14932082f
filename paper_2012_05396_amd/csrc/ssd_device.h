// Internal to the HIP library: argument blocks, element-wise update rules and
// vector load/store helpers shared by the fused and the piecewise kernels.
//
// The element-wise rules are written as one IEEE binary32 operation per
// statement; the library is compiled with -ffp-contract=off so that none of
// them is fused.  That fixes the rounding sequence:
//   server (Eq. (server) + momentum rule of Sec. 3.2.1 of the SSD-SGD paper):
//     S = g_0; S = S + g_i (i = 1..K-1); gh = S*rescale; t1 = wd*w;
//     t2 = gh + t1; t3 = lr*t2; t4 = m*mom; mom' = t4 - t3; w' = w + mom'
//   GLU (Eq. (glu-update), grad_sync of Sec. 3.3, descent sign):
//     q = pre (or pre_scale*pre, exact-w_minus variant); e = q - wl; gs = e*c_sync; u1 = alpha*g; u2 = wd_loc*wl; u3 = u1 + u2;
//     u4 = beta*gs; u5 = u3 + u4; u6 = lr_loc*u5; wl' = wl - u6
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ssd.h"

// Workgroups are single wavefronts: the unit of scheduling is then one wave
// working on one 256-element (1 KiB per array) tile, and the number of waves
// resident per compute unit can be capped exactly (see ssd_lds_slice_bytes).
#define SSD_BLOCK 64
#define SSD_COPY_BLOCK 256

// Layout of the K local-weight arrays w'_i.  Planar (K <= 8): worker i's array
// is one arena, the arrays follow each other.  Interleaved (K > 8): block b of
// worker i is at ((b * K + i) * C), so the K tiles a wave needs lie in one
// K KiB piece instead of K places a whole array apart -- with 2K+3 streams
// the address translations of a compute unit no longer hold one entry per
// stream (hit rate 85 % at K = 16), and this takes K-1 streams away: the plain
// kernel gains 5-8 % for K = 9 ... 16 against planar arrays (both at their
// best number of resident waves).  At K = 8, where translation hits 99.7 % anyway
// and a wave asks for all 8 tiles at once, the same layout measured 2 % slower.
constexpr bool ssd_interleave_of(int K) { return K > 8; }

enum { SSD_STAGE_WARMUP = 0, SSD_STAGE_DELAY = 2 };

// Work decomposition.  The state arrays are "arena" arrays cut into blocks of
// C = chunk_elems elements; tensor t owns a run of whole blocks, so block b of
// the launch is arena elements [b*C, b*C + C) of every state array -- known
// from blockIdx alone -- and one 4-byte table entry names t.  Element 0 of
// tensor t sits at arena element elem0[t], which is the start of its first
// block plus a lead-in of fewer than 256 elements: the lead-in is chosen so
// that the 256-element tiles of the arena (aligned 1 KiB pieces of the state
// arrays) are aligned 1 KiB pieces of the caller's arrays too, whenever the
// tensor's weight pointer is 16-byte aligned.  A tile then never straddles two
// 1 KiB lines of memory in any array that shares the weight's alignment
// (measured +1 ... 5 % on models of hundreds of tensors that start at 256-byte
// rather than 1 KiB boundaries).  The first block of a tensor therefore starts
// with `lead` arena elements that belong to no tensor, its last block ends
// with padding; block b covers tensor elements [b*C - elem0, b*C - elem0 + C)
// clipped to [0, numel).
struct ssd_tensor_desc {
    float *w;        // global weight of this tensor (caller-owned)
    int64_t elem0;   // arena element of the tensor's element 0
    int64_t numel;
};

// Workgroups are handed to the 8 accelerator dies (XCDs, each with its own L2)
// round-robin by workgroup id, so the block -> tensor table is stored die-major:
// entry of block b at (b % 8) * blocks_per_xcd + b / 8.  The 16 entries of one
// 64-byte line are then used by 16 consecutive workgroups of ONE die instead
// of being fetched by all eight.  The die count is a constant of the layout,
// not a query: HIP reports none, and on a device partitioned into fewer dies
// the table is read just as correctly, only with the plain locality of a
// table in block order.
#define SSD_XCDS 8u

struct ssd_tables {
    const int32_t *block_tensor;     // [8 * blocks_per_xcd], die-major
    const ssd_tensor_desc *tensors;  // [T]
    unsigned C;                      // elements per block
    unsigned blocks_per_xcd;         // ceil(num_blocks / 8)
};

static __host__ __device__ __forceinline__ size_t ssd_block_slot(unsigned b, unsigned blocks_per_xcd)
{
    return (size_t)(b % SSD_XCDS) * blocks_per_xcd + b / SSD_XCDS;
}

struct ssd_block {
    int tensor;
    unsigned lo, len;  // elements lo .. len-1 of this block belong to the tensor
    int64_t off;       // tensor element that the block's element 0 stands for (< 0 in a lead-in)
    int64_t ao;        // element offset inside every state array
};

// the part of block b (arena elements [b*C, b*C + C)) that belongs to a tensor
static __host__ __device__ __forceinline__ void ssd_block_range(int64_t b, unsigned C, int64_t elem0, int64_t numel,
                                                       int64_t &off, unsigned &lo, unsigned &len)
{
    off = b * C - elem0;
    lo = off < 0 ? (unsigned)(-off) : 0u;
    const int64_t left = numel - off;
    len = left < (int64_t)C ? (unsigned)left : C;
}

struct ssd_hyper {
    float rescale, lr, m, wd;                    // server
    float c_sync, lr_loc, alpha, beta, wd_loc;   // worker
    float pre_scale;                             // 1, or 1 - lr*wd for the exact w_minus
};

// Per-tensor hyper-parameters: the global values times the tensor's learning-
// rate and weight-decay multipliers (formed on the host), and the two derived
// constants of grad_sync.  One 24-byte record per tensor.
struct ssd_tensor_hyper {
    float lr, wd, c_sync, lr_loc, wd_loc, pre_scale;
};

static __device__ __forceinline__ ssd_hyper ssd_hyper_of(const ssd_hyper &global, const ssd_tensor_hyper &t)
{
    ssd_hyper h = global; // rescale, m, alpha, beta are the same for all tensors
    h.lr = t.lr;
    h.wd = t.wd;
    h.c_sync = t.c_sync;
    h.lr_loc = t.lr_loc;
    h.wd_loc = t.wd_loc;
    h.pre_scale = t.pre_scale;
    return h;
}

struct ssd_fused_args {
    ssd_tables tab;
    // [T][K+3] 8-byte words per tensor: weight pointer, elem0, numel,
    // then the K gradient pointers -- everything a wave needs about the
    // caller's arrays in one contiguous record
    const int64_t *rec;
    const ssd_tensor_hyper *thyper; // [T], or NULL: the values in h hold for every tensor
    float *mom, *pre, *wl;
    int64_t A;                // elements per planar state array
    ssd_hyper h;              // per-tensor fields are replaced from thyper
};

// Streaming kernels with dozens of concurrent read and write streams reach
// their best HBM throughput on MI355X with only a handful of waves per compute
// unit (few tiles in flight = a narrow window of every array).  The cap is
// enforced by giving each single-wave workgroup a slice of the compute unit's
// LDS that it never touches: waves * slice <= LDS per compute unit
// (ssd_lds_slice_bytes, declared in ssd.h; the LDS size is the device's own).

struct ssd_glu_args {
    ssd_tables tab;
    const void *const *gptr;  // [T] gradient pointers of the one worker
    const float *pre_src;     // pre_weight array to read
    float *pre_dst;           // pre_weight array to write (init / refresh)
    float *wl;                // this worker's w': its copy of block 0
    int64_t wl_block_stride;  // elements from its copy of block b to that of block b+1
    const ssd_tensor_hyper *thyper; // [T], or NULL: the values in h hold for every tensor
    ssd_hyper h;              // per-tensor fields are replaced from thyper
};

struct ssd_pull_args {
    ssd_tables tab;
    float *wl, *wloc;         // this worker's arrays (wl: its copy of block 0)
    int64_t wl_block_stride;  // as in ssd_glu_args; w_loc arrays are always planar
};

static __device__ __forceinline__ ssd_block ssd_locate(const ssd_tables &tab, unsigned b,
                                                       ssd_tensor_desc &td)
{
    ssd_block k;
    k.tensor = tab.block_tensor[ssd_block_slot(b, tab.blocks_per_xcd)];
    td = tab.tensors[k.tensor];
    ssd_block_range((int64_t)b, tab.C, td.elem0, td.numel, k.off, k.lo, k.len);
    k.ao = (int64_t)b * tab.C;
    return k;
}

__device__ __forceinline__ void ssd_server_elem(float S, float w, float mom, const ssd_hyper &h,
                                                float &w_new, float &mom_new)
{
    float gh = S * h.rescale;
    float t1 = h.wd * w;
    float t2 = gh + t1;
    float t3 = h.lr * t2;
    float t4 = h.m * mom;
    float mo = t4 - t3;
    mom_new = mo;
    w_new = w + mo;
}

// XW: grad_sync from the exact w_minus of Sec. 3.2.1, (1 - lr*wd)*pre - wl.
// pre_scale = 1 would give the same bits as XW = false, but the multiply sits
// on the critical path of a wave and costs 1.4 % of the fused kernel's
// throughput, so the default form is compiled without it.
template <bool XW>
__device__ __forceinline__ float ssd_glu_elem(float g, float wl, float pre, const ssd_hyper &h)
{
    float q = XW ? h.pre_scale * pre : pre;
    float e = q - wl;
    float gs = e * h.c_sync;
    float u1 = h.alpha * g;
    float u2 = h.wd_loc * wl;
    float u3 = u1 + u2;
    float u4 = h.beta * gs;
    float u5 = u3 + u4;
    float u6 = h.lr_loc * u5;
    return wl - u6;
}

// Pointers that come out of tables in memory are generic to the compiler;
// casting them to the global address space gives global_load / global_store
// with a scalar base and a 32-bit lane offset instead of flat accesses.
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) const float cgfloat;
static __device__ __forceinline__ gfloat *ssd_global(float *p) { return (gfloat *)p; }
static __device__ __forceinline__ cgfloat *ssd_global(const float *p) { return (cgfloat *)p; }

// VW-wide (1 or 4 floats) global loads and stores.  NT: every byte of a step
// is touched once and the arrays are far larger than the caches, so both are
// marked non-temporal.  !NT: ordinary accesses, for models whose whole state
// stays in the last-level cache from one iteration to the next.
template <int VW, bool NT = true> struct ssd_vec;
template <bool NT> struct ssd_vec<1, NT> {
    static __device__ __forceinline__ void ld(cgfloat *p, float (&x)[1])
    {
        x[0] = NT ? __builtin_nontemporal_load(p) : *p;
    }
    static __device__ __forceinline__ void st(gfloat *p, const float (&x)[1])
    {
        if (NT)
            __builtin_nontemporal_store(x[0], p);
        else
            *p = x[0];
    }
};
template <bool NT> struct ssd_vec<4, NT> {
    typedef float v4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(1))) v4 gv4;
    typedef __attribute__((address_space(1))) const v4 cgv4;
    static __device__ __forceinline__ void ld(cgfloat *p, float (&x)[4])
    {
        v4 v = NT ? __builtin_nontemporal_load((cgv4 *)p) : *(cgv4 *)p;
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    }
    static __device__ __forceinline__ void st(gfloat *p, const float (&x)[4])
    {
        v4 v = {x[0], x[1], x[2], x[3]};
        if (!NT) {
            *(gv4 *)p = v;
            return;
        }
        // "sc1 nt" (system-coherence bit + non-temporal) is a cache policy the
        // compiler has no builtin for; measured 1-2 % faster than plain "nt"
        // on MI355X.  The compiler cannot see into the asm, so the wait
        // states that the ISA requires between a store of more than 64 bits
        // and a following VALU write of its data registers (2 on gfx950) are
        // supplied here: s_nop 1 idles for two cycles.
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    }
};

static __device__ __forceinline__ bool ssd_aligned16(const void *p)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// Gradient buffers hold binary32, bfloat16 or binary16 elements (GD is an
// ssd_grad_dtype).  A 16-bit gradient is widened to binary32 as it is loaded:
// bfloat16 by moving its bits into the upper half of the word, binary16 by the
// hardware conversion; both are exact, so everything after the load is the
// same arithmetic on the same values for all three types.  Four elements are
// one 128-bit (binary32) or one 64-bit (16-bit types) load.
template <int GD> struct ssd_grad {
    typedef float elem;
};
template <> struct ssd_grad<SSD_GRAD_BF16> {
    typedef uint16_t elem;
};
template <> struct ssd_grad<SSD_GRAD_F16> {
    typedef uint16_t elem;
};

template <int GD, int VW, bool NT = true> struct ssd_gvec;
template <int VW, bool NT> struct ssd_gvec<SSD_GRAD_F32, VW, NT> {
    typedef cgfloat *ptr;
    static __device__ __forceinline__ void ld(ptr p, float (&x)[VW]) { ssd_vec<VW, NT>::ld(p, x); }
};
template <bool NT> struct ssd_gvec<SSD_GRAD_BF16, 1, NT> {
    typedef __attribute__((address_space(1))) const uint16_t *ptr;
    static __device__ __forceinline__ void ld(ptr p, float (&x)[1])
    {
        x[0] = __uint_as_float((uint32_t)(NT ? __builtin_nontemporal_load(p) : *p) << 16);
    }
};
template <bool NT> struct ssd_gvec<SSD_GRAD_BF16, 4, NT> {
    typedef __attribute__((address_space(1))) const uint16_t *ptr;
    typedef uint32_t u2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void ld(ptr p, float (&x)[4])
    {
        typedef __attribute__((address_space(1))) const u2 *gp2;
        const u2 v = NT ? __builtin_nontemporal_load((gp2)p) : *(gp2)p;
        x[0] = __uint_as_float(v.x << 16);
        x[1] = __uint_as_float(v.x & 0xffff0000u);
        x[2] = __uint_as_float(v.y << 16);
        x[3] = __uint_as_float(v.y & 0xffff0000u);
    }
};
template <bool NT> struct ssd_gvec<SSD_GRAD_F16, 1, NT> {
    typedef __attribute__((address_space(1))) const uint16_t *ptr;
    static __device__ __forceinline__ void ld(ptr p, float (&x)[1])
    {
        typedef __attribute__((address_space(1))) const _Float16 *gph;
        x[0] = (float)(NT ? __builtin_nontemporal_load((gph)p) : *(gph)p);
    }
};
template <bool NT> struct ssd_gvec<SSD_GRAD_F16, 4, NT> {
    typedef __attribute__((address_space(1))) const uint16_t *ptr;
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void ld(ptr p, float (&x)[4])
    {
        typedef __attribute__((address_space(1))) const h4 *gp4;
        const h4 v = NT ? __builtin_nontemporal_load((gp4)p) : *(gp4)p;
        x[0] = (float)v.x; x[1] = (float)v.y; x[2] = (float)v.z; x[3] = (float)v.w;
    }
};

// the four-element path needs every pointer of the tensor aligned to one load
template <int GD> static __device__ __forceinline__ bool ssd_grad_aligned(const void *p)
{
    return (reinterpret_cast<uintptr_t>(p) & (4u * sizeof(typename ssd_grad<GD>::elem) - 1u)) == 0;
}

static inline size_t ssd_grad_elem_size(int grad_dtype) { return grad_dtype == SSD_GRAD_F32 ? 4 : 2; }

static inline bool ssd_aligned16_host(const void *p)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// records a message for ssd_last_error(NULL) on this thread and returns `code`
int ssd_fail_thread(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// launchers, one translation unit each
hipError_t ssd_launch_glu(int grad_dtype, int pre_action, unsigned nchunks, hipStream_t s, const ssd_glu_args &a);
hipError_t ssd_launch_pull(int init, unsigned nchunks, hipStream_t s, const ssd_pull_args &a);
hipError_t ssd_launch_fill_zero(float *p, int64_t n, hipStream_t s);
// lds_bytes: LDS slice per workgroup (occupancy cap, 0 = none); lds_limit: the
// largest slice any launch on this device may ask for (LDS per compute unit)
typedef hipError_t (*ssd_fused_launcher)(int stage, int pre_action, int from_global, int exact_w_minus,
                                         int streaming,
                                         unsigned lds_bytes, unsigned lds_limit,
                                         unsigned nchunks, hipStream_t s, const ssd_fused_args &a);
// ssd_launch_fused_g<grad_dtype>_k<K>
#define SSD_DECL_FUSED(k)                                                                                        \
    hipError_t ssd_launch_fused_g0_k##k(int, int, int, int, int, unsigned, unsigned, unsigned, hipStream_t, const ssd_fused_args &); \
    hipError_t ssd_launch_fused_g1_k##k(int, int, int, int, int, unsigned, unsigned, unsigned, hipStream_t, const ssd_fused_args &); \
    hipError_t ssd_launch_fused_g2_k##k(int, int, int, int, int, unsigned, unsigned, unsigned, hipStream_t, const ssd_fused_args &);
SSD_DECL_FUSED(1) SSD_DECL_FUSED(2) SSD_DECL_FUSED(3) SSD_DECL_FUSED(4)
SSD_DECL_FUSED(5) SSD_DECL_FUSED(6) SSD_DECL_FUSED(7) SSD_DECL_FUSED(8)
SSD_DECL_FUSED(9) SSD_DECL_FUSED(10) SSD_DECL_FUSED(11) SSD_DECL_FUSED(12)
SSD_DECL_FUSED(13) SSD_DECL_FUSED(14) SSD_DECL_FUSED(15) SSD_DECL_FUSED(16)

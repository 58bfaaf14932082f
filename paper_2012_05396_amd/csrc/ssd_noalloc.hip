// ssd_server_aggregate_update_noalloc: the server side of one iteration
// (Eq. (server), momentum rule of Sec. 3.2.1) for callers that cannot
// allocate.  Same element-wise rule and the same multi-tensor launch as the
// context-based entry point, but no context, no workspace argument and no
// allocation of any kind, on the host or on the device: the tables that the
// launch needs (one record per tensor, one entry per 256-element block) live
// in a file-scope device array, `scratch`, whose device address is looked up
// once per device, and they get there as kernel arguments.
//
// Every call on a device uses that device's one array and leaves its tables
// there; nothing in it has to start at zero (each call writes every entry it
// reads).  Calls follow each other correctly on one stream; calls that overlap
// on one device (different streams, or different host threads) race on it.
#include "ssd_device.h"

#include <atomic>

namespace {

// record of one tensor: w, mom, first block, numel, then g_0 .. g_{K-1}
constexpr int kRecHead = 4;
constexpr size_t kRecBytes = (size_t)SSD_NOALLOC_MAX_TENSORS * (kRecHead + SSD_MAX_WORKERS) * sizeof(int64_t);
constexpr size_t kTabBytes = (size_t)SSD_NOALLOC_MAX_BLOCKS * sizeof(uint16_t);
constexpr size_t kScratchBytes = kRecBytes + kTabBytes; // 163,840 + 2,097,152 bytes
static_assert(SSD_NOALLOC_MAX_TENSORS <= 65536, "block table entries are 16-bit tensor numbers");
static_assert(kRecBytes % 256 == 0, "the block table starts 256-byte aligned");
constexpr unsigned kTile = SSD_BLOCK * 4; // elements per single-wave workgroup

} // namespace

// The name below is a host-side stand-in for the device array, not a device
// address: host code only ever uses the pointer hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];

// Device address of this device's copy of `scratch`; the device must be
// current.  Looked up at the first call on the device, then remembered.
hipError_t scratch_of(int device, unsigned char **out)
{
    unsigned char *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!sym) return hipErrorInvalidSymbol;
        p = static_cast<unsigned char *>(sym);
        g_scratch_ptr[device].store(p, std::memory_order_release); // every thread finds the same address
    }
    *out = p;
    return hipSuccess;
}

// Host -> scratch without a copy call: up to kPutWords 8-byte words travel as
// a kernel argument (copied by the launch itself, so the host array may be
// reused at once) and one thread per word stores them.
constexpr int kPutWords = 448; // 3584 bytes of the 4 KiB a launch may carry
struct put_payload {
    int64_t w[kPutWords];
};

__global__ __launch_bounds__(64) void ssd_noalloc_put_kernel(int64_t *dst, int n, const put_payload p)
{
    for (int i = threadIdx.x; i < n; i += 64) dst[i] = p.w[i];
}

// block -> tensor: the last tensor whose first block is <= b (T <= 65536)
__global__ __launch_bounds__(256) void ssd_noalloc_table_kernel(const int64_t *recs, int rec_words, int T,
                                                                unsigned nblocks, uint16_t *table)
{
    const unsigned b = blockIdx.x * 256u + threadIdx.x;
    if (b >= nblocks) return;
    int lo = 0, hi = T - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (recs[(size_t)mid * rec_words + 2] <= (int64_t)b)
            lo = mid;
        else
            hi = mid - 1;
    }
    table[b] = (uint16_t)lo;
}

// S = g_0; S = S + g_i in worker order; then the server rule (ssd_server_elem)
template <int VW>
__device__ __forceinline__ void server_elems(const int64_t *rec, int K, int64_t off, unsigned e, gfloat *wp,
                                             gfloat *mp, const ssd_hyper &h)
{
    typedef ssd_vec<VW> V;
    float S[VW], g[VW], w[VW], mo[VW], wn[VW], mn[VW];
    V::ld(ssd_global(reinterpret_cast<const float *>(rec[kRecHead])) + off + e, S);
    for (int i = 1; i < K; ++i) {
        V::ld(ssd_global(reinterpret_cast<const float *>(rec[kRecHead + i])) + off + e, g);
#pragma unroll
        for (int v = 0; v < VW; ++v) S[v] = S[v] + g[v];
    }
    V::ld(wp + e, w);
    V::ld(mp + e, mo);
#pragma unroll
    for (int v = 0; v < VW; ++v) ssd_server_elem(S[v], w[v], mo[v], h, wn[v], mn[v]);
    V::st(mp + e, mn);
    V::st(wp + e, wn);
}

__global__ __launch_bounds__(SSD_BLOCK) void ssd_noalloc_server_kernel(const uint16_t *table, const int64_t *recs,
                                                                       int K, const ssd_hyper h)
{
    const int t = table[blockIdx.x];
    const int64_t *rec = recs + (size_t)t * (kRecHead + K);
    float *w = reinterpret_cast<float *>(rec[0]);
    float *mom = reinterpret_cast<float *>(rec[1]);
    const int64_t off = ((int64_t)blockIdx.x - rec[2]) * kTile;
    const int64_t left = rec[3] - off;
    const unsigned len = left < (int64_t)kTile ? (unsigned)left : kTile;
    bool vec = ssd_aligned16(w) && ssd_aligned16(mom);
    for (int i = 0; i < K; ++i) vec = vec && ssd_aligned16(reinterpret_cast<const void *>(rec[kRecHead + i]));
    gfloat *wp = ssd_global(w) + off, *mp = ssd_global(mom) + off;
    const unsigned e0 = threadIdx.x * 4;
    if (vec && e0 + 3 < len) {
        server_elems<4>(rec, K, off, e0, wp, mp, h);
    } else {
        for (unsigned e = e0; e < e0 + 4 && e < len; ++e) server_elems<1>(rec, K, off, e, wp, mp, h);
    }
}

struct DeviceScope {
    int prev = -1, target = -1;
    bool ok = false;
    explicit DeviceScope(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        if (prev != dev && hipSetDevice(dev) != hipSuccess) return;
        target = dev;
        ok = true;
    }
    ~DeviceScope()
    {
        if (ok && prev != target) (void)hipSetDevice(prev);
    }
};

} // namespace

extern "C" int ssd_server_aggregate_update_noalloc(int32_t K, int32_t T, const int64_t *numel, float *const *weights,
                                                   float *const *momentum, const float *const *const *grads,
                                                   float lr, float m, float wd, float rescale_grad, int32_t device,
                                                   void *stream)
{
    // every check comes before the first launch: a failing call enqueues nothing
    if (K < 1 || K > SSD_MAX_WORKERS)
        return ssd_fail_thread(SSD_EINVAL, "num_workers = %d, must be 1..%d", K, SSD_MAX_WORKERS);
    if (T < 1) return ssd_fail_thread(SSD_EINVAL, "num_tensors = %d, must be >= 1", T);
    if (T > SSD_NOALLOC_MAX_TENSORS)
        return ssd_fail_thread(SSD_EINVAL, "num_tensors = %d is beyond the %d tensors the static scratch holds", T,
                               SSD_NOALLOC_MAX_TENSORS);
    if (!numel || !weights || !momentum || !grads) return ssd_fail_thread(SSD_EINVAL, "NULL argument");
    if (device < 0 || device >= kMaxDevices) return ssd_fail_thread(SSD_EINVAL, "device = %d", device);
    int64_t nblocks = 0;
    for (int t = 0; t < T; ++t) {
        if (numel[t] < 1) return ssd_fail_thread(SSD_EINVAL, "numel[%d] = %lld, must be >= 1", t, (long long)numel[t]);
        if (!weights[t] || !momentum[t]) return ssd_fail_thread(SSD_EINVAL, "weights[%d] or momentum[%d] is NULL", t, t);
        if (reinterpret_cast<uintptr_t>(weights[t]) % 4 || reinterpret_cast<uintptr_t>(momentum[t]) % 4)
            return ssd_fail_thread(SSD_EALIGN, "weights[%d] or momentum[%d] is not 4-byte aligned", t, t);
        if (numel[t] > (int64_t)SSD_NOALLOC_MAX_BLOCKS * kTile) nblocks = (int64_t)SSD_NOALLOC_MAX_BLOCKS + 1;
        if (nblocks <= SSD_NOALLOC_MAX_BLOCKS) nblocks += (numel[t] + kTile - 1) / kTile;
    }
    if (nblocks > SSD_NOALLOC_MAX_BLOCKS)
        return ssd_fail_thread(SSD_EINVAL, "the model needs more than the %d blocks of %u elements the static "
                                           "scratch holds", SSD_NOALLOC_MAX_BLOCKS, kTile);
    for (int i = 0; i < K; ++i) {
        if (!grads[i]) return ssd_fail_thread(SSD_EINVAL, "grads[%d] is NULL", i);
        for (int t = 0; t < T; ++t) {
            if (!grads[i][t]) return ssd_fail_thread(SSD_EINVAL, "grads[%d][%d] is NULL", i, t);
            if (reinterpret_cast<uintptr_t>(grads[i][t]) % 4)
                return ssd_fail_thread(SSD_EALIGN, "grads[%d][%d] is not 4-byte aligned", i, t);
        }
    }
    DeviceScope scope(device);
    if (!scope.ok) return ssd_fail_thread(SSD_EHIP, "cannot select device %d", device);
    unsigned char *ptr = nullptr;
    hipError_t e = scratch_of(device, &ptr);
    if (e != hipSuccess) return ssd_fail_thread(SSD_EHIP, "address of the static scratch: %s", hipGetErrorString(e));
    int64_t *d_recs = reinterpret_cast<int64_t *>(ptr);
    uint16_t *d_table = reinterpret_cast<uint16_t *>(ptr + kRecBytes);
    hipStream_t s = static_cast<hipStream_t>(stream);

    // records, a launch-full at a time
    const int rw = kRecHead + K;
    const int per_launch = kPutWords / rw; // whole records per launch (>= 22)
    put_payload p = {}; // the whole struct travels with each launch
    int64_t first_block = 0;
    for (int t0 = 0; t0 < T; t0 += per_launch) {
        const int nt = T - t0 < per_launch ? T - t0 : per_launch;
        for (int j = 0; j < nt; ++j) {
            const int t = t0 + j;
            int64_t *r = p.w + (size_t)j * rw;
            r[0] = (int64_t) reinterpret_cast<uintptr_t>(weights[t]);
            r[1] = (int64_t) reinterpret_cast<uintptr_t>(momentum[t]);
            r[2] = first_block;
            r[3] = numel[t];
            for (int i = 0; i < K; ++i) r[kRecHead + i] = (int64_t) reinterpret_cast<uintptr_t>(grads[i][t]);
            first_block += (numel[t] + kTile - 1) / kTile;
        }
        ssd_noalloc_put_kernel<<<dim3(1), dim3(64), 0, s>>>(d_recs + (size_t)t0 * rw, nt * rw, p);
        e = hipGetLastError();
        if (e != hipSuccess) return ssd_fail_thread(SSD_EHIP, "launch of the record upload: %s", hipGetErrorString(e));
    }
    ssd_noalloc_table_kernel<<<dim3((unsigned)((nblocks + 255) / 256)), dim3(256), 0, s>>>(d_recs, rw, T,
                                                                                            (unsigned)nblocks, d_table);
    e = hipGetLastError();
    if (e != hipSuccess) return ssd_fail_thread(SSD_EHIP, "launch of the block table kernel: %s", hipGetErrorString(e));
    ssd_hyper h = {};
    h.rescale = rescale_grad;
    h.lr = lr;
    h.m = m;
    h.wd = wd;
    ssd_noalloc_server_kernel<<<dim3((unsigned)nblocks), dim3(SSD_BLOCK), 0, s>>>(d_table, d_recs, K, h);
    e = hipGetLastError();
    if (e != hipSuccess) return ssd_fail_thread(SSD_EHIP, "launch of the server kernel: %s", hipGetErrorString(e));
    return SSD_OK;
}

// Host side of the SSD-SGD library: argument checks, the schedule of
// Algorithm 1 / Algorithm 2 of the paper as a small state machine, the block
// and pointer tables of the multi-tensor launch, and the launches.
// No arithmetic of the method runs here except two configuration constants,
// c_sync = (1-m)/(lr*k) (Sec. 3.3) and, for the exact-w_minus variant,
// 1 - lr*wd (Sec. 3.2.1), formed once per learning-rate change in binary64
// and rounded to binary32.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "ssd_device.h"

namespace {

thread_local char g_init_error[512] = "";

void set_err(char *buf, size_t cap, const char *fmt, va_list ap) { vsnprintf(buf, cap, fmt, ap); }

int fail_init(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    set_err(g_init_error, sizeof g_init_error, fmt, ap);
    va_end(ap);
    return code;
}

} // namespace

// for the entry points that have no context: the message goes where
// ssd_last_error(NULL) finds it
int ssd_fail_thread(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    set_err(g_init_error, sizeof g_init_error, fmt, ap);
    va_end(ap);
    return code;
}

namespace {

constexpr size_t kWsAlign = 256;
constexpr int kFusedSlots = 8;

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// A small cache of device-resident pointer tables keyed by content, so that a
// caller cycling through a few sets of gradient buffers uploads each table
// once.  Slot memory is reused in least-recently-used order; an event per slot
// keeps the pinned staging copy alive until its upload has run.
struct PtrCache {
    int nslots = 0;
    size_t len = 0;              // pointers per table
    int64_t *dev = nullptr;  // device [nslots][len] 8-byte words (inside the workspace)
    int64_t *host = nullptr; // pinned [nslots][len]
    std::vector<uint64_t> stamp;
    std::vector<char> valid;
    std::vector<hipEvent_t> ev;
    std::vector<hipStream_t> up_stream;  // stream each slot was uploaded on
    std::vector<std::vector<hipStream_t>> users; // streams whose launches have read the slot
    uint64_t clock = 0;

    hipError_t create(int n, size_t l, void *dev_mem)
    {
        nslots = n;
        len = l;
        dev = static_cast<int64_t *>(dev_mem);
        stamp.assign(n, 0);
        valid.assign(n, 0);
        ev.assign(n, nullptr);
        up_stream.assign(n, nullptr);
        users.assign(n, std::vector<hipStream_t>());
        for (auto &u : users) u.reserve(8);
        hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&host), sizeof(int64_t) * len * n,
                                     hipHostMallocDefault);
        if (e != hipSuccess) {
            host = nullptr;
            return e;
        }
        for (int i = 0; i < n; ++i) {
            e = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    void destroy()
    {
        for (size_t i = 0; i < ev.size(); ++i)
            if (ev[i] && valid[i]) (void)hipEventSynchronize(ev[i]); // its upload still reads `host`
        for (hipEvent_t e : ev)
            if (e) (void)hipEventDestroy(e);
        ev.clear();
        if (host) (void)hipHostFree(host);
        host = nullptr;
    }
    // key: len words.  Returns the device table holding them.
    hipError_t get(const int64_t *key, hipStream_t s, const int64_t **out)
    {
        ++clock;
        for (int i = 0; i < nslots; ++i)
            if (valid[i] && std::memcmp(host + i * len, key, sizeof(int64_t) * len) == 0) {
                stamp[i] = clock;
                *out = dev + i * len;
                if (std::find(users[i].begin(), users[i].end(), s) == users[i].end()) {
                    // first use on this stream: order it after the upload, once
                    // (later launches on the stream follow in stream order, so a
                    // steady-state call enqueues nothing but its kernel)
                    if (up_stream[i] != s) {
                        hipError_t e = hipStreamWaitEvent(s, ev[i], 0);
                        if (e != hipSuccess) return e;
                    }
                    users[i].push_back(s);
                }
                return hipSuccess;
            }
        int lru = -1;
        for (int i = 0; i < nslots && lru < 0; ++i)
            if (!valid[i]) lru = i; // a free slot first
        if (lru < 0) {
            lru = 0;
            for (int i = 1; i < nslots; ++i)
                if (stamp[i] < stamp[lru]) lru = i;
        }
        hipError_t e;
        if (valid[lru]) {
            e = hipEventSynchronize(ev[lru]); // staging copy may still be queued
            if (e != hipSuccess) return e;
            for (hipStream_t u : users[lru])
                if (u != s) { // a launch on another stream may still read the old table
                    e = hipStreamSynchronize(u);
                    if (e != hipSuccess) return e;
                }
        }
        valid[lru] = 0;
        std::memcpy(host + lru * len, key, sizeof(int64_t) * len);
        e = hipMemcpyAsync(dev + lru * len, host + lru * len, sizeof(int64_t) * len,
                           hipMemcpyHostToDevice, s);
        if (e != hipSuccess) return e;
        e = hipEventRecord(ev[lru], s);
        if (e != hipSuccess) return e;
        valid[lru] = 1;
        up_stream[lru] = s;
        users[lru].assign(1, s);
        stamp[lru] = clock;
        *out = dev + lru * len;
        return hipSuccess;
    }
};

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        if (prev != dev && hipSetDevice(dev) != hipSuccess) return;
        ok = true;
        target = dev;
    }
    ~DeviceGuard()
    {
        if (ok && prev != target) (void)hipSetDevice(prev);
    }
    int target = -1;
};

struct Layout {
    int64_t A = 0;      // elements of one state array that hold tensors
    int64_t stride = 0; // elements from one state array to the next (>= A)
    std::vector<int64_t> tensor_offset, first_block; // tensor_offset[t] = first_block[t] * chunk_elems + lead-in
    int32_t chunk_elems = 0;
    int64_t num_chunks = 0, blocks_per_xcd = 0;
    size_t off_mom = 0, off_pre0 = 0, off_pre1 = 0, off_wl = 0, off_wloc = 0;
    size_t off_chunks = 0, off_tensors = 0, off_thyper = 0, off_gtab = 0, off_grow = 0;
    int row_slots = 0;
    size_t total = 0;
};

int check_config(const ssd_config *c)
{
    if (!c) return fail_init(SSD_EINVAL, "config is NULL");
    if (c->num_workers < 1 || c->num_workers > SSD_MAX_WORKERS)
        return fail_init(SSD_EINVAL, "num_workers = %d, must be 1..%d", c->num_workers, SSD_MAX_WORKERS);
    if (c->delay_k < 0) return fail_init(SSD_EINVAL, "delay_k = %d, must be >= 0", c->delay_k);
    if (c->warmup_iters < 0) return fail_init(SSD_EINVAL, "warmup_iters = %d, must be >= 0", c->warmup_iters);
    if (c->num_tensors < 1) return fail_init(SSD_EINVAL, "num_tensors = %d, must be >= 1", c->num_tensors);
    if (!c->numel) return fail_init(SSD_EINVAL, "numel is NULL");
    for (int t = 0; t < c->num_tensors; ++t)
        if (c->numel[t] < 1) return fail_init(SSD_EINVAL, "numel[%d] = %lld, must be >= 1", t, (long long)c->numel[t]);
    if (c->delay_k > 0 && !(c->lr != 0.0f))
        return fail_init(SSD_EINVAL, "lr = 0 with delay_k > 0: grad_sync divides by lr*k");
    if (c->chunk_elems < 0 || c->chunk_elems % 256 != 0)
        return fail_init(SSD_EINVAL, "chunk_elems = %d, must be 0 or a positive multiple of 256", c->chunk_elems);
    if (c->grad_sync_exact != 0 && c->grad_sync_exact != 1)
        return fail_init(SSD_EINVAL, "grad_sync_exact = %d, must be 0 or 1", c->grad_sync_exact);
    if (c->grad_dtype != SSD_GRAD_F32 && c->grad_dtype != SSD_GRAD_BF16 && c->grad_dtype != SSD_GRAD_F16)
        return fail_init(SSD_EINVAL, "grad_dtype = %d, must be an ssd_grad_dtype (0..2)", c->grad_dtype);
    if (c->waves_per_cu < 0) return fail_init(SSD_EINVAL, "waves_per_cu = %d, must be >= 0", c->waves_per_cu);
    if (c->cache_policy != SSD_CACHE_AUTO && c->cache_policy != SSD_CACHE_STREAMING &&
        c->cache_policy != SSD_CACHE_RESIDENT)
        return fail_init(SSD_EINVAL, "cache_policy = %d, must be an ssd_cache_policy (0..2)", c->cache_policy);
    if (c->device < 0) return fail_init(SSD_EINVAL, "device = %d", c->device);
    return SSD_OK;
}

// Lead-in of a tensor in its first arena block (see ssd_tensor_desc): the
// element phase of the weight pointer inside its 1 KiB line, so that the
// arena's 256-element tiles are aligned 1 KiB pieces of the caller's arrays
// too.  Only for 16-byte aligned pointers (the lead-in is then a multiple of 4
// elements and the 128-bit path keeps its alignment) and for tensors of at
// least 32 tiles, where the extra block it can cost is at most 3 % of the
// tensor's blocks.
constexpr int64_t kLeadMinElems = 32 * 256;
constexpr int64_t kLeadMax = 252;

int64_t lead_of(const float *w, int64_t numel)
{
    const uintptr_t a = reinterpret_cast<uintptr_t>(w);
    if (numel < kLeadMinElems || a % 16) return 0;
    return (int64_t)(a % 1024) / 4;
}

// Whether everything one steps-delay iteration touches -- K gradients, K local
// weights, global weight, momentum, pre_weight -- fits the last-level cache
// (MI355X: 256 MiB of memory-side cache; HIP reports no such figure).  Then the
// arrays are still cached when the next iteration comes, provided the accesses
// are not marked non-temporal.  Measured on MI355X with K = 1..16 on 0.27 M-
// to 25 M-element models: ordinary accesses are 4-27 % faster up to about
// 300 MB touched per iteration and 10-23 % slower from 490 MB on.
constexpr size_t kLastLevelCacheBytes = (size_t)256 << 20;

bool fits_last_level_cache(const ssd_config &c, const Layout &L)
{
    const size_t K = (size_t)c.num_workers;
    const size_t per_elem = K * ssd_grad_elem_size(c.grad_dtype) + sizeof(float) * (c.delay_k > 0 ? K + 3 : 2);
    return (size_t)L.A * per_elem <= kLastLevelCacheBytes;
}

// Distance in bytes between consecutive state arrays of `bytes` bytes each.
// Large arrays are placed a multiple of 64 MiB (2 MiB for mid-sized ones)
// apart: with the dozens of streams of the fused kernel walking all arrays at
// the same relative position, that placement measured 2-7 % more HBM
// throughput on MI355X than arbitrary distances (K = 8 and 16, 100-550 MB
// arrays) -- but not a multiple of 256 MiB: distances of 256, 512 and 768 MiB
// measured 3-6 % less than 384, 640 and 896 MiB on the same models (K = 4 and
// 8; 61 M- to 198 M-element models), so those take two more units.
size_t array_distance(size_t bytes)
{
    size_t arr = round_up(bytes, kWsAlign);
    if (arr >= ((size_t)64 << 20)) {
        arr = round_up(arr, (size_t)64 << 20);
        if (arr % ((size_t)256 << 20) == 0) arr += (size_t)128 << 20;
    } else if (arr >= ((size_t)2 << 20)) {
        arr = round_up(arr, (size_t)2 << 20);
    }
    return arr;
}

// weights == nullptr: sizes for the worst case over all weight alignments
// (what ssd_workspace_bytes reports before the pointers are known).
int make_layout(const ssd_config *c, float *const *weights, Layout *L)
{
    const int T = c->num_tensors, K = c->num_workers;
    int64_t unused = 0;
    int rc = ssd_plan_chunks(c->numel, T, c->chunk_elems, nullptr, 0, &unused, &L->chunk_elems);
    if (rc != SSD_OK) return rc;
    // arena: tensor t owns whole blocks of chunk_elems elements, in tensor order
    L->tensor_offset.resize(T);
    L->first_block.resize(T);
    int64_t blocks = 0;
    for (int t = 0; t < T; ++t) {
        const int64_t lead = weights ? lead_of(weights[t], c->numel[t])
                                     : (c->numel[t] >= kLeadMinElems ? kLeadMax : 0);
        L->first_block[t] = blocks;
        L->tensor_offset[t] = blocks * L->chunk_elems + (weights ? lead : 0);
        blocks += (c->numel[t] + lead + L->chunk_elems - 1) / L->chunk_elems;
    }
    L->num_chunks = blocks;
    if (L->num_chunks > 0x7fffffffLL) return fail_init(SSD_EINVAL, "model needs %lld chunks, more than one launch holds", (long long)L->num_chunks);
    const int64_t a = blocks * L->chunk_elems; // blocks == num_chunks
    L->A = a;
    size_t o = 0;
    size_t arr = array_distance(sizeof(float) * (size_t)a);
    if (!weights) {
        // worst case over the alignments: the rule is not monotone, so every
        // arena size between the one without lead-ins and this one counts
        int64_t blocks_min = 0;
        for (int t = 0; t < T; ++t) blocks_min += (c->numel[t] + L->chunk_elems - 1) / L->chunk_elems;
        const size_t unit = (size_t)64 << 20;
        const size_t lo = sizeof(float) * (size_t)blocks_min * L->chunk_elems, hi = sizeof(float) * (size_t)a;
        arr = std::max(arr, array_distance(lo));
        for (size_t x = round_up(lo, unit); x < hi; x += unit) arr = std::max(arr, array_distance(x));
    }
    L->stride = (int64_t)(arr / sizeof(float));
    L->off_mom = o, o += arr;
    if (c->delay_k > 0) {
        L->off_pre0 = o, o += arr;
        L->off_pre1 = o, o += arr;
        L->off_wl = o, o += arr * K;
        L->off_wloc = o, o += arr * K;
    }
    L->blocks_per_xcd = (L->num_chunks + SSD_XCDS - 1) / SSD_XCDS;
    L->off_chunks = o, o += round_up(sizeof(int32_t) * (size_t)L->blocks_per_xcd * SSD_XCDS, kWsAlign);
    L->off_tensors = o, o += round_up(sizeof(ssd_tensor_desc) * (size_t)T, kWsAlign);
    L->off_thyper = o, o += round_up(sizeof(ssd_tensor_hyper) * (size_t)T, kWsAlign);
    L->off_gtab = o, o += round_up(sizeof(int64_t) * (size_t)T * (K + 3), kWsAlign) * kFusedSlots;
    L->row_slots = std::max(8, 2 * K);
    L->off_grow = o, o += round_up(sizeof(float *) * (size_t)T, kWsAlign) * L->row_slots;
    L->total = o;
    return SSD_OK;
}

} // namespace

struct ssd_ctx {
    ssd_config cfg;
    std::vector<int64_t> numel;
    Layout L;
    hipStream_t stream = nullptr;
    char *ws = nullptr;
    float *mom = nullptr, *pre[2] = {nullptr, nullptr}, *wl = nullptr, *wloc = nullptr;
    int32_t *d_block_tensor = nullptr;
    ssd_tensor_desc *d_tensors = nullptr;
    PtrCache gtab, grow;
    ssd_hyper h;
    // per-tensor learning-rate / weight-decay multipliers and the table of
    // per-tensor hyper-parameters derived from them (device copy + two pinned
    // staging copies used in turn)
    std::vector<float> lr_mult, wd_mult;
    // every multiplier is 1: the kernels take the global values from their
    // arguments and the table is neither read nor kept up to date, so a
    // learning-rate change costs no upload (schedules that change lr every
    // iteration)
    bool uniform_hyper = true;
    ssd_tensor_hyper *d_thyper = nullptr, *h_thyper[2] = {nullptr, nullptr};
    hipEvent_t thyper_ev[2] = {nullptr, nullptr};
    int thyper_next = 0;
    // what the occupancy cap and the small-model rule need to know about the
    // device, read once at ssd_init
    int num_cus = 0;
    int lds_per_cu = 0;
    bool streaming = true;    // cache policy of the fused launch
    int64_t it = 0;
    std::vector<int64_t> loc_update;
    std::vector<char> has_local, wloc_fresh;
    // pre_weight is one shared array (Sec. 3.3: every worker holds the same
    // value), which is only true while every worker's w' is the same global
    // weight when pre_weight is initialised or refreshed from it.  w_version
    // counts the server updates; pulled_version[i] is its value at worker i's
    // last Pull; round_version that of the first worker of the current
    // init/refresh round.
    int64_t w_version = 0, round_version = -1;
    std::vector<int64_t> pulled_version;
    // After the hand-over at the end of warm-up and after a Pull of the fused
    // step, every w'_i equals the global weight; that is recorded here instead
    // of being written K times.  wl_holds_wloc: the w' arrays then still hold
    // the local weights that were broadcast as w_loc before the Pull.
    bool wl_is_global = false, wl_holds_wloc = false;
    int pre_cur = 0;      // which pre_weight array is current
    int pre_written = 0;  // workers that have written the other one this round
    std::vector<int64_t> scratch; // [T][K+3] records: w, arena element of element 0, numel, g_0..g_{K-1}
    char err[512];

    int fail(int code, const char *fmt, ...)
    {
        va_list ap;
        va_start(ap, fmt);
        set_err(err, sizeof err, fmt, ap);
        va_end(ap);
        return code;
    }
    int fail_hip(hipError_t e, const char *what)
    {
        return fail(SSD_EHIP, "%s: %s", what, hipGetErrorString(e));
    }
    void set_c_sync()
    {
        h.c_sync = cfg.delay_k > 0
                       ? (float)((1.0 - (double)h.m) / ((double)h.lr * (double)cfg.delay_k))
                       : 0.0f;
        // exact w_minus of Sec. 3.2.1: ((1 - lr*wd)*pre_weight - w'); else the factor is 1
        h.pre_scale = cfg.grad_sync_exact ? (float)(1.0 - (double)h.lr * (double)h.wd) : 1.0f;
    }
    ssd_tables tables() const { return ssd_tables{d_block_tensor, d_tensors, (unsigned)L.chunk_elems, (unsigned)L.blocks_per_xcd}; }
    // Hyper-parameters of tensor t: global values times its multipliers, each
    // product one binary32 multiplication; the constants of grad_sync formed
    // from them in binary64.  A tensor with learning rate 0 is frozen on the
    // server, so no global gradient can be inferred for it: c_sync = 0.
    ssd_tensor_hyper tensor_hyper(int t) const
    {
        ssd_tensor_hyper th;
        th.lr = h.lr * lr_mult[t];
        th.wd = h.wd * wd_mult[t];
        th.lr_loc = h.lr_loc * lr_mult[t];
        th.wd_loc = h.wd_loc * wd_mult[t];
        th.c_sync = (cfg.delay_k > 0 && th.lr != 0.0f)
                        ? (float)((1.0 - (double)h.m) / ((double)th.lr * (double)cfg.delay_k))
                        : 0.0f;
        th.pre_scale = cfg.grad_sync_exact ? (float)(1.0 - (double)th.lr * (double)th.wd) : 1.0f;
        return th;
    }
    // Rebuild the table and enqueue its upload on the current stream (ordered
    // after the launches already enqueued there, before the ones to come).
    hipError_t upload_tensor_hyper()
    {
        const int slot = thyper_next;
        thyper_next ^= 1;
        hipError_t e = hipEventSynchronize(thyper_ev[slot]); // its previous upload has run
        if (e != hipSuccess) return e;
        const int T = cfg.num_tensors;
        for (int t = 0; t < T; ++t) h_thyper[slot][t] = tensor_hyper(t);
        e = hipMemcpyAsync(d_thyper, h_thyper[slot], sizeof(ssd_tensor_hyper) * (size_t)T,
                           hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return e;
        return hipEventRecord(thyper_ev[slot], stream);
    }
    float *arr(float *base, int i) const { return base + (int64_t)i * stride_elems(); }
    int64_t stride_elems() const { return L.stride; }
    // w'_i: the K local-weight arrays are planar or interleaved by block (ssd_interleave_of)
    bool interleaved() const { return ssd_interleave_of(cfg.num_workers); }
    int64_t wl_worker_stride() const { return interleaved() ? L.chunk_elems : L.stride; }
    int64_t wl_block_stride() const { return interleaved() ? (int64_t)cfg.num_workers * L.chunk_elems : L.chunk_elems; }
    float *wl_of(int i) const { return wl + (int64_t)i * wl_worker_stride(); }
};

extern "C" {

int ssd_step_kind_of(int64_t iteration, int32_t W, int32_t k, int64_t d, int32_t *pre_action)
{
    if (iteration < 0 || W < 0 || k < 0 || d < 0) return SSD_EINVAL;
    if (pre_action) *pre_action = SSD_PRE_KEEP;
    if (k == 0 || iteration < W) // Alg. 1, warm-up loop (while num <= wp)
        return (k > 0 && iteration == W - 1) ? SSD_STEP_WARMUP_LAST : SSD_STEP_WARMUP;
    if (pre_action) // Alg. 2: initialise at the first local update, refresh every k
        *pre_action = d == 0 ? SSD_PRE_INIT : (d % k == 0 ? SSD_PRE_REFRESH : SSD_PRE_KEEP);
    return d % k == k - 1 ? SSD_STEP_DELAY_PULL : SSD_STEP_DELAY; // Alg. 1: Pull every k
}

int ssd_lds_slice_bytes(int32_t waves_per_cu, int32_t lds_bytes_per_cu)
{
    if (waves_per_cu < 0 || lds_bytes_per_cu < 128 || lds_bytes_per_cu % 128) return SSD_EINVAL;
    if (waves_per_cu == 0 || waves_per_cu >= 32) return 0; // no cap
    // LDS is handed out in 128 granules per compute unit (1280 bytes each on
    // gfx950, whose compute units have 160 KiB): a whole number of granules
    const int granule = lds_bytes_per_cu / 128;
    return (128 / waves_per_cu) * granule;
}

int ssd_config_defaults(ssd_config *cfg, int32_t num_workers, float lr, float wd)
{
    if (!cfg) return fail_init(SSD_EINVAL, "cfg is NULL");
    if (num_workers < 1 || num_workers > SSD_MAX_WORKERS)
        return fail_init(SSD_EINVAL, "num_workers = %d, must be 1..%d", num_workers, SSD_MAX_WORKERS);
    std::memset(cfg, 0, sizeof *cfg);
    cfg->num_workers = num_workers;
    cfg->lr = lr;
    cfg->wd = wd;
    cfg->wd_loc = wd;          // Eq. (glu-update) prints the servers' wd
    cfg->lr_loc = 4.0f * lr;   // Sec. 4.1: loc_lr is four times the global learning rate
    cfg->alpha = 2.0f;         // Sec. 4.1
    cfg->beta = 0.5f;          // Sec. 4.1
    cfg->rescale_grad = (float)(1.0 / (double)num_workers); // Table 1: the servers' gradient is the average
    cfg->grad_dtype = SSD_GRAD_F32;
    return SSD_OK;
}

static int ssd_plan_chunks_impl(const int64_t *numel, int32_t T, int32_t chunk_elems, ssd_chunk *out,
                    int64_t capacity, int64_t *count, int32_t *used)
{
    if (!numel || T < 1 || !count) return fail_init(SSD_EINVAL, "ssd_plan_chunks: NULL argument or T < 1");
    if (chunk_elems < 0 || chunk_elems % 256 != 0)
        return fail_init(SSD_EINVAL, "chunk_elems = %d, must be 0 or a positive multiple of 256", chunk_elems);
    for (int t = 0; t < T; ++t)
        if (numel[t] < 1) return fail_init(SSD_EINVAL, "numel[%d] = %lld, must be >= 1", t, (long long)numel[t]);
    // one tile of a single-wave workgroup: 64 lanes x 4 floats
    const int64_t c = chunk_elems == 0 ? 256 : chunk_elems;
    int64_t n = 0;
    for (int t = 0; t < T; ++t)
        for (int64_t off = 0; off < numel[t]; off += c, ++n)
            if (out && n < capacity) {
                out[n].tensor = t;
                out[n].offset = off;
                out[n].len = (int32_t)std::min<int64_t>(c, numel[t] - off);
            }
    *count = n;
    if (used) *used = (int32_t)c;
    return SSD_OK;
}

static int ssd_workspace_bytes_impl(const ssd_config *cfg, size_t *bytes)
{
    if (!bytes) return fail_init(SSD_EINVAL, "bytes is NULL");
    int rc = check_config(cfg);
    if (rc != SSD_OK) return rc;
    Layout L;
    rc = make_layout(cfg, nullptr, &L);
    if (rc != SSD_OK) return rc;
    *bytes = L.total;
    return SSD_OK;
}

static int ssd_plan_arena_impl(const ssd_config *cfg, float *const *weights, int64_t *tensor_offset,
                               ssd_chunk *out, int64_t capacity, int64_t *num_blocks, size_t *bytes)
{
    int rc = check_config(cfg);
    if (rc != SSD_OK) return rc;
    if (!weights) return fail_init(SSD_EINVAL, "weights is NULL");
    const int T = cfg->num_tensors;
    for (int t = 0; t < T; ++t)
        if (reinterpret_cast<uintptr_t>(weights[t]) % sizeof(float))
            return fail_init(SSD_EALIGN, "weights[%d] is not 4-byte aligned", t);
    Layout L;
    rc = make_layout(cfg, weights, &L);
    if (rc != SSD_OK) return rc;
    if (tensor_offset) std::copy(L.tensor_offset.begin(), L.tensor_offset.end(), tensor_offset);
    if (num_blocks) *num_blocks = L.num_chunks;
    if (bytes) *bytes = L.total;
    if (out)
        for (int t = 0; t < T; ++t) {
            const int64_t end = t + 1 < T ? L.first_block[t + 1] : L.num_chunks;
            for (int64_t b = L.first_block[t]; b < end && b < capacity; ++b) {
                int64_t off;
                unsigned lo, len;
                ssd_block_range(b, (unsigned)L.chunk_elems, L.tensor_offset[t], cfg->numel[t], off, lo, len);
                out[b].tensor = t;
                out[b].offset = off + lo;
                out[b].len = (int32_t)(len - lo);
            }
        }
    return SSD_OK;
}

void ssd_destroy(ssd_ctx *ctx)
{
    if (!ctx) return;
    {
        DeviceGuard g(ctx->cfg.device);
        ctx->gtab.destroy();
        ctx->grow.destroy();
        for (int i = 0; i < 2; ++i) {
            if (ctx->thyper_ev[i]) (void)hipEventSynchronize(ctx->thyper_ev[i]); // staging still being read
            if (ctx->thyper_ev[i]) (void)hipEventDestroy(ctx->thyper_ev[i]);
            if (ctx->h_thyper[i]) (void)hipHostFree(ctx->h_thyper[i]);
        }
    }
    delete ctx;
}

static int init_context(ssd_ctx *c, const ssd_config *cfg, float *const *weights, void *workspace,
                        size_t workspace_bytes, ssd_ctx **out);

static int ssd_init_impl(const ssd_config *cfg, float *const *weights, void *workspace, size_t workspace_bytes,
             ssd_ctx **out)
{
    if (!out) return fail_init(SSD_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc != SSD_OK) return rc;
    if (!weights) return fail_init(SSD_EINVAL, "weights is NULL");
    if (!workspace) return fail_init(SSD_EINVAL, "workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) % kWsAlign)
        return fail_init(SSD_EALIGN, "workspace is not %zu-byte aligned", kWsAlign);
    const int T = cfg->num_tensors;
    for (int t = 0; t < T; ++t) {
        if (!weights[t]) return fail_init(SSD_EINVAL, "weights[%d] is NULL", t);
        if (reinterpret_cast<uintptr_t>(weights[t]) % sizeof(float))
            return fail_init(SSD_EALIGN, "weights[%d] is not 4-byte aligned", t);
    }
    ssd_ctx *c = new (std::nothrow) ssd_ctx;
    if (!c) return fail_init(SSD_ENOMEM, "host allocation failed");
    c->err[0] = 0;
    c->cfg = *cfg;
    c->cfg.numel = nullptr;
    try {
        return init_context(c, cfg, weights, workspace, workspace_bytes, out);
    } catch (...) {
        ssd_destroy(c); // a host allocation failed half-way
        throw;
    }
}

static int init_context(ssd_ctx *c, const ssd_config *cfg, float *const *weights, void *workspace,
                        size_t workspace_bytes, ssd_ctx **out)
{
    const int T = cfg->num_tensors, K = cfg->num_workers;
    int rc;
    c->cfg = *cfg;
    c->numel.assign(cfg->numel, cfg->numel + T);
    c->cfg.numel = c->numel.data();
    rc = make_layout(&c->cfg, weights, &c->L);
    if (rc != SSD_OK) {
        delete c;
        return rc;
    }
    if (workspace_bytes < c->L.total) {
        rc = fail_init(SSD_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, c->L.total);
        delete c;
        return rc;
    }
    c->stream = static_cast<hipStream_t>(cfg->stream);
    c->ws = static_cast<char *>(workspace);
    const Layout &L = c->L;
    c->mom = reinterpret_cast<float *>(c->ws + L.off_mom);
    if (cfg->delay_k > 0) {
        c->pre[0] = reinterpret_cast<float *>(c->ws + L.off_pre0);
        c->pre[1] = reinterpret_cast<float *>(c->ws + L.off_pre1);
        c->wl = reinterpret_cast<float *>(c->ws + L.off_wl);
        c->wloc = reinterpret_cast<float *>(c->ws + L.off_wloc);
    }
    c->d_block_tensor = reinterpret_cast<int32_t *>(c->ws + L.off_chunks);
    c->d_tensors = reinterpret_cast<ssd_tensor_desc *>(c->ws + L.off_tensors);
    c->h.rescale = cfg->rescale_grad;
    c->h.lr = cfg->lr;
    c->h.m = cfg->momentum;
    c->h.wd = cfg->wd;
    c->h.lr_loc = cfg->lr_loc;
    c->h.alpha = cfg->alpha;
    c->h.beta = cfg->beta;
    c->h.wd_loc = cfg->wd_loc;
    c->set_c_sync();
    c->loc_update.assign(K, 0);
    c->has_local.assign(K, 0);
    c->wloc_fresh.assign(K, 0);
    c->pulled_version.assign(K, -1);
    c->lr_mult.assign(T, 1.0f);
    c->wd_mult.assign(T, 1.0f);
    c->scratch.resize((size_t)T * (K + 3));
    for (int t = 0; t < T; ++t) {
        c->scratch[(size_t)t * (K + 3) + 0] = (int64_t) reinterpret_cast<uintptr_t>(weights[t]);
        c->scratch[(size_t)t * (K + 3) + 1] = c->L.tensor_offset[t];
        c->scratch[(size_t)t * (K + 3) + 2] = c->numel[t];
    }

    DeviceGuard guard(cfg->device);
    if (!guard.ok) {
        rc = fail_init(SSD_EHIP, "cannot select device %d", cfg->device);
        delete c;
        return rc;
    }
    hipError_t e;
    {
        int v = 0;
        e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, cfg->device);
        if (e == hipSuccess) {
            c->num_cus = v;
            e = hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, cfg->device);
        }
        if (e != hipSuccess || c->num_cus < 1 || v < 1) {
            rc = fail_init(SSD_EHIP, "cannot read compute-unit count and LDS size of device %d: %s", cfg->device,
                           hipGetErrorString(e));
            delete c;
            return rc;
        }
        c->lds_per_cu = v;
    }
    c->streaming = cfg->cache_policy == SSD_CACHE_AUTO ? !fits_last_level_cache(c->cfg, c->L)
                                                        : cfg->cache_policy == SSD_CACHE_STREAMING;
#define SSD_INIT_HIP(call, what)                                                         \
    do {                                                                                 \
        e = (call);                                                                      \
        if (e != hipSuccess) {                                                           \
            rc = fail_init(SSD_EHIP, "%s: %s", what, hipGetErrorString(e));              \
            ssd_destroy(c);                                                              \
            return rc;                                                                   \
        }                                                                                \
    } while (0)
    SSD_INIT_HIP(c->gtab.create(kFusedSlots, (size_t)T * (K + 3), c->ws + L.off_gtab), "pointer table (fused)");
    // slots of the caches are packed at len pointers; the workspace reserves a
    // rounded-up stride per slot, which is at least that
    SSD_INIT_HIP(c->grow.create(L.row_slots, (size_t)T, c->ws + L.off_grow), "pointer table (rows)");
    c->d_thyper = reinterpret_cast<ssd_tensor_hyper *>(c->ws + L.off_thyper);
    for (int i = 0; i < 2; ++i) {
        SSD_INIT_HIP(hipHostMalloc(reinterpret_cast<void **>(&c->h_thyper[i]), sizeof(ssd_tensor_hyper) * (size_t)T,
                                   hipHostMallocDefault), "staging for per-tensor hyper-parameters");
        SSD_INIT_HIP(hipEventCreateWithFlags(&c->thyper_ev[i], hipEventDisableTiming), "event");
    }
    SSD_INIT_HIP(c->upload_tensor_hyper(), "upload per-tensor hyper-parameters");

    // block -> tensor table and tensor descriptors: built on the host, uploaded once
    std::vector<int32_t> block_tensor((size_t)L.blocks_per_xcd * SSD_XCDS, 0);
    std::vector<ssd_tensor_desc> descs(T);
    for (int t = 0; t < T; ++t) {
        descs[t].w = weights[t];
        descs[t].elem0 = L.tensor_offset[t];
        descs[t].numel = c->numel[t];
        const int64_t end = t + 1 < T ? L.first_block[t + 1] : L.num_chunks;
        for (int64_t b = L.first_block[t]; b < end; ++b)
            block_tensor[ssd_block_slot((unsigned)b, (unsigned)L.blocks_per_xcd)] = t;
    }
    SSD_INIT_HIP(hipMemcpyAsync(c->d_block_tensor, block_tensor.data(), sizeof(int32_t) * block_tensor.size(),
                                hipMemcpyHostToDevice, c->stream), "upload block table");
    SSD_INIT_HIP(hipMemcpyAsync(c->d_tensors, descs.data(), sizeof(ssd_tensor_desc) * descs.size(),
                                hipMemcpyHostToDevice, c->stream), "upload tensor table");
    SSD_INIT_HIP(hipStreamSynchronize(c->stream), "upload tables"); // sources are pageable locals
    // momentum starts at zero (paddings included)
    SSD_INIT_HIP(ssd_launch_fill_zero(c->mom, c->stride_elems(), c->stream), "clear momentum");
    if (cfg->delay_k > 0) {
        // paddings of the other state arrays are never read, but keep them defined
        SSD_INIT_HIP(ssd_launch_fill_zero(c->pre[0], c->stride_elems() * (2 + 2 * (int64_t)K), c->stream), "clear state");
        if (cfg->warmup_iters == 0) {
            // Alg. 1 initialisation without a warm-up stage: every worker pulls w_0
            for (int i = 0; i < K; ++i) c->has_local[i] = 1;
            c->wl_is_global = true;
        }
    }
#undef SSD_INIT_HIP
    *out = c;
    return SSD_OK;
}

static int check_grads(ssd_ctx *c, const void *const *const *grads)
{
    if (!grads) return c->fail(SSD_EINVAL, "grads is NULL");
    const int T = c->cfg.num_tensors, K = c->cfg.num_workers;
    const size_t esize = ssd_grad_elem_size(c->cfg.grad_dtype);
    for (int i = 0; i < K; ++i) {
        if (!grads[i]) return c->fail(SSD_EINVAL, "grads[%d] is NULL", i);
        for (int t = 0; t < T; ++t) {
            const void *p = grads[i][t];
            if (!p) return c->fail(SSD_EINVAL, "grads[%d][%d] is NULL", i, t);
            if (reinterpret_cast<uintptr_t>(p) % esize)
                return c->fail(SSD_EALIGN, "grads[%d][%d] is not %zu-byte aligned", i, t, esize);
            c->scratch[(size_t)t * (K + 3) + 3 + i] = (int64_t) reinterpret_cast<uintptr_t>(p);
        }
    }
    return SSD_OK;
}

// Resident waves per compute unit that gave the highest HBM throughput when
// measured on MI355X: sweeps over 2..16 waves for K = 1, 2, 4, 8 on 133-138 M-
// element models and K = 9 ... 16 on a 60 M-element one, with binary32 and with
// bfloat16 gradient buffers.  A wave requests its whole tile at once, so the
// best cap falls as a wave carries more streams, roughly as
// budget / (loads per lane), and is flat within +-1:
//   plain delay kernel   58 / (2K + 3), at least 4   (K = 8: 4, K = 2: 8)
//   from-global kernel   44 / (K + 3),  at least 4   (50 with 16-bit gradients)
//   warm-up kernel       58 / (K + 2),  at least 6   (read-dominated: its
//                        16-bit gradient loads count half, budget 52)
// Beyond K = 8 the K local weights of a tile are one contiguous piece
// (ssd_interleave_of), which moves the optimum of the plain kernel down to 3
// waves for every K = 9 ... 16 (4 waves: -3 ... -8 %); the other two kernels
// do not read the local weights and stay at 4 and 6 (8 with 16-bit gradients).
static int default_waves_per_cu(int K, int stage, int from_global, bool grad16)
{
    if (K > 8) {
        if (stage == SSD_STAGE_WARMUP) return grad16 ? 8 : 6;
        return from_global ? 4 : 3;
    }
    int loads2, budget, floor_n; // loads per lane in halves of a 128-bit load
    if (stage == SSD_STAGE_WARMUP)
        loads2 = (grad16 ? K : 2 * K) + 4, budget = grad16 ? 52 : 58, floor_n = 6;
    else if (from_global)
        loads2 = 2 * (K + 3), budget = grad16 ? 50 : 44, floor_n = 4;
    else
        loads2 = 2 * (2 * K + 3), budget = 58, floor_n = 4;
    const int n = (2 * budget + loads2 / 2) / loads2;
    return n < floor_n ? floor_n : (n > 16 ? 16 : n);
}

static int launch_fused(ssd_ctx *c, int stage, int pre_action, int from_global)
{
#define SSD_ROW(g)                                                                               \
    {ssd_launch_fused_g##g##_k1,  ssd_launch_fused_g##g##_k2,  ssd_launch_fused_g##g##_k3,       \
     ssd_launch_fused_g##g##_k4,  ssd_launch_fused_g##g##_k5,  ssd_launch_fused_g##g##_k6,       \
     ssd_launch_fused_g##g##_k7,  ssd_launch_fused_g##g##_k8,  ssd_launch_fused_g##g##_k9,       \
     ssd_launch_fused_g##g##_k10, ssd_launch_fused_g##g##_k11, ssd_launch_fused_g##g##_k12,      \
     ssd_launch_fused_g##g##_k13, ssd_launch_fused_g##g##_k14, ssd_launch_fused_g##g##_k15,      \
     ssd_launch_fused_g##g##_k16}
    static const ssd_fused_launcher table[3][SSD_MAX_WORKERS] = {SSD_ROW(0), SSD_ROW(1), SSD_ROW(2)};
#undef SSD_ROW
    static_assert(SSD_GRAD_F32 == 0 && SSD_GRAD_BF16 == 1 && SSD_GRAD_F16 == 2, "rows of the launcher table");
    const int64_t *rec = nullptr;
    hipError_t e = c->gtab.get(c->scratch.data(), c->stream, &rec);
    if (e != hipSuccess) return c->fail_hip(e, "gradient pointer table");
    ssd_fused_args a;
    a.tab = c->tables();
    a.rec = rec;
    a.thyper = c->uniform_hyper ? nullptr : c->d_thyper;
    a.mom = c->mom;
    a.pre = c->pre[c->pre_cur];
    a.wl = c->wl;
    a.A = c->stride_elems();
    a.h = c->h;
    int waves = c->cfg.waves_per_cu;
    if (waves <= 0) {
        waves = default_waves_per_cu(c->cfg.num_workers, stage, from_global, c->cfg.grad_dtype != SSD_GRAD_F32);
        // The cap keeps the request queues towards HBM just full.  A model
        // that is served from the last-level cache wants every wave it can
        // get (measured 3-6 % slower with the cap on 0.27 M- to 7 M-element
        // models in resident mode).
        if (!c->streaming) waves = 0;
    }
    const int lds = ssd_lds_slice_bytes(waves, c->lds_per_cu);
    if (lds < 0) return c->fail(SSD_EINVAL, "no LDS slice for %d waves per compute unit", waves);
    e = table[c->cfg.grad_dtype][c->cfg.num_workers - 1](stage, pre_action, from_global, c->cfg.grad_sync_exact,
                                      c->streaming ? 1 : 0, (unsigned)lds, (unsigned)c->lds_per_cu,
                                      (unsigned)c->L.num_chunks, c->stream, a);
    if (e != hipSuccess) return c->fail_hip(e, "launch of the fused kernel");
    return SSD_OK;
}

// Write out what the flags wl_is_global / wl_holds_wloc stand for: w_loc_i takes
// the broadcast local weights (or the global weight), w'_i the global weight.
// Needed before anything changes the global weight outside the fused step.
static int materialize(ssd_ctx *c)
{
    if (!c->wl_is_global) return SSD_OK;
    const int K = c->cfg.num_workers;
    for (int i = 0; i < K; ++i) {
        ssd_pull_args a = {c->tables(), c->wl_of(i), c->arr(c->wloc, i), c->wl_block_stride()};
        hipError_t e = ssd_launch_pull(c->wl_holds_wloc ? 0 : 1, (unsigned)c->L.num_chunks, c->stream, a);
        if (e != hipSuccess) return c->fail_hip(e, "launch of the pull kernel");
        c->wloc_fresh[i] = 1;
        c->pulled_version[i] = c->w_version;
    }
    c->wl_is_global = c->wl_holds_wloc = false;
    return SSD_OK;
}

static int ssd_materialize_impl(ssd_ctx *c)
{
    if (!c) return SSD_EINVAL;
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    return materialize(c);
}

static int ssd_server_aggregate_update_impl(ssd_ctx *c, const void *const *const *grads)
{
    if (!c) return SSD_EINVAL;
    int rc = check_grads(c, grads);
    if (rc != SSD_OK) return rc;
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    rc = materialize(c); // the global weight is about to change
    if (rc != SSD_OK) return rc;
    rc = launch_fused(c, SSD_STAGE_WARMUP, SSD_PRE_KEEP, 0);
    if (rc == SSD_OK) c->w_version += 1;
    return rc;
}

static int ssd_step_impl(ssd_ctx *c, const void *const *const *grads)
{
    if (!c) return SSD_EINVAL;
    int rc = check_grads(c, grads);
    if (rc != SSD_OK) return rc;
    const int K = c->cfg.num_workers, k = c->cfg.delay_k, W = c->cfg.warmup_iters;
    const int64_t d = c->loc_update[0];
    for (int i = 1; i < K; ++i)
        if (c->loc_update[i] != d)
            return c->fail(SSD_ESTATE, "workers are at different local update counts (%lld vs %lld)",
                           (long long)d, (long long)c->loc_update[i]);
    if (c->pre_written != 0) return c->fail(SSD_ESTATE, "a piecewise local update round is unfinished");
    int32_t pre_action = SSD_PRE_KEEP;
    const int kind = ssd_step_kind_of(c->it, W, k, d, &pre_action);
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    if (kind == SSD_STEP_WARMUP || kind == SSD_STEP_WARMUP_LAST) {
        rc = launch_fused(c, SSD_STAGE_WARMUP, SSD_PRE_KEEP, 0);
        if (rc != SSD_OK) return rc;
        c->w_version += 1;
        if (kind == SSD_STEP_WARMUP_LAST) {
            // Alg. 1: w'_{t,i} = w_t for every worker -- recorded, not copied
            for (int i = 0; i < K; ++i) {
                c->has_local[i] = 1;
                c->wloc_fresh[i] = 0;
                c->loc_update[i] = 0;
            }
            c->wl_is_global = true;
            c->wl_holds_wloc = false;
        }
    } else {
        for (int i = 0; i < K; ++i)
            if (!c->has_local[i]) return c->fail(SSD_ESTATE, "worker %d has no local weights", i);
        if (!c->wl_is_global && pre_action != SSD_PRE_KEEP) {
            // pre_weight is about to take worker 0's w' for everybody (reached
            // only after piecewise calls): all w'_i must be one global weight
            for (int i = 0; i < K; ++i)
                if (!c->wloc_fresh[i] || c->pulled_version[i] != c->pulled_version[0])
                    return c->fail(SSD_ESTATE, "pre_weight is shared: every worker must have pulled the same global "
                                               "weight since its last local update (worker %d has not)", i);
        }
        if (c->wl_is_global && pre_action == SSD_PRE_KEEP) {
            rc = materialize(c); // only after piecewise calls moved the schedule
            if (rc != SSD_OK) return rc;
        }
        rc = launch_fused(c, SSD_STAGE_DELAY, pre_action, c->wl_is_global ? 1 : 0);
        if (rc != SSD_OK) return rc;
        c->w_version += 1;
        // Alg. 1, Pull iteration: the updated w' were broadcast (they stay in
        // the w' arrays as w_loc) and w' = w_t from now on -- recorded only
        const bool pull = kind == SSD_STEP_DELAY_PULL;
        c->wl_is_global = c->wl_holds_wloc = pull;
        for (int i = 0; i < K; ++i) {
            c->loc_update[i] = d + 1;
            c->wloc_fresh[i] = 0;
        }
    }
    c->it += 1;
    return SSD_OK;
}

static int ssd_worker_glu_update_impl(ssd_ctx *c, int32_t worker, const void *const *grads_i)
{
    if (!c) return SSD_EINVAL;
    const int K = c->cfg.num_workers, k = c->cfg.delay_k, T = c->cfg.num_tensors;
    if (worker < 0 || worker >= K) return c->fail(SSD_EINVAL, "worker = %d, must be 0..%d", worker, K - 1);
    if (!grads_i) return c->fail(SSD_EINVAL, "grads_i is NULL");
    const size_t esize = ssd_grad_elem_size(c->cfg.grad_dtype);
    for (int t = 0; t < T; ++t) {
        if (!grads_i[t]) return c->fail(SSD_EINVAL, "grads_i[%d] is NULL", t);
        if (reinterpret_cast<uintptr_t>(grads_i[t]) % esize)
            return c->fail(SSD_EALIGN, "grads_i[%d] is not %zu-byte aligned", t, esize);
    }
    if (k == 0) return c->fail(SSD_ESTATE, "delay_k = 0: there is no steps-delay stage");
    if (!c->has_local[worker]) return c->fail(SSD_ESTATE, "worker %d has no local weights yet (pull first)", worker);
    const int64_t lu = c->loc_update[worker];
    const int64_t dmin = *std::min_element(c->loc_update.begin(), c->loc_update.end());
    if (lu != dmin)
        return c->fail(SSD_ESTATE, "worker %d is at local update %lld but the slowest worker at %lld", worker,
                       (long long)lu, (long long)dmin);
    const int pre_action = lu == 0 ? SSD_PRE_INIT : (lu % k == 0 ? SSD_PRE_REFRESH : SSD_PRE_KEEP);
    // Alg. 2 sets pre_weight = w' here, and pre_weight is one array for all
    // workers (Sec. 3.3: they hold the same value).  That is only the paper's
    // pre_weight if this worker's w' is a pulled global weight, the same one
    // for every worker of this round.
    int64_t version = -1;
    if (pre_action != SSD_PRE_KEEP) {
        const bool fresh = c->wl_is_global || c->wloc_fresh[worker];
        version = c->wl_is_global ? c->w_version : c->pulled_version[worker];
        if (!fresh)
            return c->fail(SSD_ESTATE, "pre_weight is shared: worker %d must pull before local update %lld "
                                       "(its w' is not a global weight)", worker, (long long)lu);
        if (c->pre_written > 0 && version != c->round_version)
            return c->fail(SSD_ESTATE, "pre_weight is shared: worker %d pulled another global weight than the "
                                       "workers before it in this round", worker);
    }
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    int rc = materialize(c);
    if (rc != SSD_OK) return rc;
    const int64_t *tab = nullptr;
    static_assert(sizeof(const float *) == sizeof(int64_t), "pointer tables are tables of 8-byte words");
    hipError_t e = c->grow.get(reinterpret_cast<const int64_t *>(grads_i), c->stream, &tab);
    if (e != hipSuccess) return c->fail_hip(e, "gradient pointer table");
    ssd_glu_args a;
    a.tab = c->tables();
    a.gptr = reinterpret_cast<const void *const *>(tab);
    a.pre_src = c->pre[c->pre_cur];
    a.pre_dst = c->pre[c->pre_cur ^ 1];
    a.wl = c->wl_of(worker);
    a.wl_block_stride = c->wl_block_stride();
    a.thyper = c->uniform_hyper ? nullptr : c->d_thyper;
    a.h = c->h;
    e = ssd_launch_glu(c->cfg.grad_dtype, pre_action, (unsigned)c->L.num_chunks, c->stream, a);
    if (e != hipSuccess) return c->fail_hip(e, "launch of the GLU kernel");
    c->loc_update[worker] = lu + 1;
    c->wloc_fresh[worker] = 0;
    if (pre_action != SSD_PRE_KEEP && c->pre_written == 0) c->round_version = version;
    if (pre_action != SSD_PRE_KEEP && ++c->pre_written == K) {
        c->pre_cur ^= 1; // every worker has written the same values to the other array
        c->pre_written = 0;
    }
    return SSD_OK;
}

static int ssd_worker_pull_impl(ssd_ctx *c, int32_t worker)
{
    if (!c) return SSD_EINVAL;
    const int K = c->cfg.num_workers;
    if (worker < 0 || worker >= K) return c->fail(SSD_EINVAL, "worker = %d, must be 0..%d", worker, K - 1);
    if (c->cfg.delay_k == 0) return c->fail(SSD_ESTATE, "delay_k = 0: workers keep no local weights");
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    int rc = materialize(c);
    if (rc != SSD_OK) return rc;
    ssd_pull_args a = {c->tables(), c->wl_of(worker), c->arr(c->wloc, worker), c->wl_block_stride()};
    hipError_t e = ssd_launch_pull(c->has_local[worker] ? 0 : 1, (unsigned)c->L.num_chunks, c->stream, a);
    if (e != hipSuccess) return c->fail_hip(e, "launch of the pull kernel");
    c->has_local[worker] = 1;
    c->wloc_fresh[worker] = 1;
    c->pulled_version[worker] = c->w_version;
    return SSD_OK;
}

static int ssd_set_lr_impl(ssd_ctx *c, float lr, float lr_loc)
{
    if (!c) return SSD_EINVAL;
    if (c->cfg.delay_k > 0 && !(lr != 0.0f)) return c->fail(SSD_EINVAL, "lr = 0 with delay_k > 0: grad_sync divides by lr*k");
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    c->h.lr = lr;
    c->h.lr_loc = lr_loc;
    c->set_c_sync();
    if (c->uniform_hyper) return SSD_OK; // the new values travel as kernel arguments
    hipError_t e = c->upload_tensor_hyper();
    if (e != hipSuccess) return c->fail_hip(e, "upload of per-tensor hyper-parameters");
    return SSD_OK;
}

static int ssd_set_tensor_multipliers_impl(ssd_ctx *c, const float *lr_mult, const float *wd_mult)
{
    if (!c) return SSD_EINVAL;
    const int T = c->cfg.num_tensors;
    for (int t = 0; t < T; ++t) {
        if (lr_mult && !(lr_mult[t] >= 0.0f)) return c->fail(SSD_EINVAL, "lr_mult[%d] must be >= 0", t);
        if (wd_mult && !(wd_mult[t] >= 0.0f)) return c->fail(SSD_EINVAL, "wd_mult[%d] must be >= 0", t);
    }
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return c->fail(SSD_EHIP, "cannot select device %d", c->cfg.device);
    bool uniform = true;
    for (int t = 0; t < T; ++t) {
        c->lr_mult[t] = lr_mult ? lr_mult[t] : 1.0f;
        c->wd_mult[t] = wd_mult ? wd_mult[t] : 1.0f;
        uniform = uniform && c->lr_mult[t] == 1.0f && c->wd_mult[t] == 1.0f;
    }
    c->uniform_hyper = uniform;
    if (uniform) return SSD_OK;
    hipError_t e = c->upload_tensor_hyper();
    if (e != hipSuccess) return c->fail_hip(e, "upload of per-tensor hyper-parameters");
    return SSD_OK;
}

int ssd_set_stream(ssd_ctx *c, void *stream)
{
    if (!c) return SSD_EINVAL;
    c->stream = static_cast<hipStream_t>(stream);
    return SSD_OK;
}

int ssd_get_state(ssd_ctx *c, ssd_state_view *out)
{
    if (!c) return SSD_EINVAL;
    if (!out) return c->fail(SSD_EINVAL, "out is NULL");
    const int K = c->cfg.num_workers;
    out->iterations = c->it;
    out->local_updates = *std::min_element(c->loc_update.begin(), c->loc_update.end());
    out->in_delay_stage = c->cfg.delay_k > 0 && c->it >= c->cfg.warmup_iters;
    int all_local = 1, all_fresh = 1;
    for (int i = 0; i < K; ++i) {
        all_local &= c->has_local[i];
        all_fresh &= c->wloc_fresh[i];
    }
    out->has_local = all_local;
    out->w_local_is_global = c->wl_is_global ? 1 : 0;
    if (!all_local || (c->wl_is_global && !c->wl_holds_wloc))
        out->w_loc_where = SSD_W_LOC_IS_GLOBAL;
    else if (c->wl_is_global || !all_fresh)
        out->w_loc_where = SSD_W_LOC_IN_W_LOCAL;
    else
        out->w_loc_where = SSD_W_LOC_SEPARATE;
    out->chunk_elems = c->L.chunk_elems;
    out->streaming = c->streaming ? 1 : 0;
    out->num_chunks = c->L.num_chunks;
    out->arena_elems = c->stride_elems();
    out->w_local_worker_stride = c->wl_worker_stride();
    out->w_local_block_stride = c->wl_block_stride();
    out->tensor_offset = c->L.tensor_offset.data();
    out->mom = c->mom;
    out->pre = c->pre[c->pre_cur];
    out->w_local = c->wl;
    out->w_loc = c->wloc;
    return SSD_OK;
}

const char *ssd_last_error(const ssd_ctx *c) { return c ? c->err : g_init_error; }


} // extern "C"

// ---- the exported entry points: nothing throws across the C boundary -------
namespace {
template <typename F> int guarded(ssd_ctx *c, F f)
{
    try {
        return f();
    } catch (const std::bad_alloc &) {
        return c ? c->fail(SSD_ENOMEM, "host allocation failed") : fail_init(SSD_ENOMEM, "host allocation failed");
    } catch (...) {
        return c ? c->fail(SSD_EINVAL, "unexpected C++ exception") : fail_init(SSD_EINVAL, "unexpected C++ exception");
    }
}
} // namespace

extern "C" {

int ssd_plan_chunks(const int64_t *numel, int32_t T, int32_t chunk_elems, ssd_chunk *out, int64_t capacity,
                    int64_t *count, int32_t *used)
{
    return guarded(nullptr, [&] { return ssd_plan_chunks_impl(numel, T, chunk_elems, out, capacity, count, used); });
}
int ssd_workspace_bytes(const ssd_config *cfg, size_t *bytes)
{
    return guarded(nullptr, [&] { return ssd_workspace_bytes_impl(cfg, bytes); });
}
int ssd_plan_arena(const ssd_config *cfg, float *const *weights, int64_t *tensor_offset, ssd_chunk *out,
                   int64_t capacity, int64_t *num_blocks, size_t *bytes)
{
    return guarded(nullptr,
                   [&] { return ssd_plan_arena_impl(cfg, weights, tensor_offset, out, capacity, num_blocks, bytes); });
}
int ssd_init(const ssd_config *cfg, float *const *weights, void *workspace, size_t workspace_bytes, ssd_ctx **out)
{
    return guarded(nullptr, [&] { return ssd_init_impl(cfg, weights, workspace, workspace_bytes, out); });
}
int ssd_materialize(ssd_ctx *c)
{
    return guarded(c, [&] { return ssd_materialize_impl(c); });
}
int ssd_server_aggregate_update(ssd_ctx *c, const void *const *const *grads)
{
    return guarded(c, [&] { return ssd_server_aggregate_update_impl(c, grads); });
}
int ssd_step(ssd_ctx *c, const void *const *const *grads)
{
    return guarded(c, [&] { return ssd_step_impl(c, grads); });
}
int ssd_worker_glu_update(ssd_ctx *c, int32_t worker, const void *const *grads_i)
{
    return guarded(c, [&] { return ssd_worker_glu_update_impl(c, worker, grads_i); });
}
int ssd_worker_pull(ssd_ctx *c, int32_t worker)
{
    return guarded(c, [&] { return ssd_worker_pull_impl(c, worker); });
}
int ssd_set_lr(ssd_ctx *c, float lr, float lr_loc)
{
    return guarded(c, [&] { return ssd_set_lr_impl(c, lr, lr_loc); });
}
int ssd_set_tensor_multipliers(ssd_ctx *c, const float *lr_mult, const float *wd_mult)
{
    return guarded(c, [&] { return ssd_set_tensor_multipliers_impl(c, lr_mult, wd_mult); });
}

} // extern "C"

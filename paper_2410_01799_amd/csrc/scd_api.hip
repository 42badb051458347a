// Host driver and C ABI of libscd (see include/scd.h for the contract of every entry point).
//
// The greedy loop runs as a stream of kernel launches that the host enqueues blindly: which pass a
// launch performs (a further alternation, or the update that ends a term and starts the next) is
// decided on the device from device-resident state, so tens of thousands of dependent steps never
// wait for the host.  The host only reads the state back once per batch of sweeps to see whether
// the requested number of terms is reached.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <condition_variable>
#include <map>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "scd_device.h"

using namespace scd;

namespace {

thread_local int g_last_hip = 0;

#define HIP_TRY(expr)                    \
    do {                                 \
        hipError_t _e = (expr);          \
        if (_e != hipSuccess) {          \
            g_last_hip = (int)_e;        \
            (void)hipGetLastError();     \
            return SCD_EHIP;             \
        }                                \
    } while (0)

int64_t words_for(int64_t n) { return (n + 63) / 64; }

struct Level {
    int64_t rows = 0, cols = 0;
    void* X = nullptr;          // level 0: the remainder; else the previous level's W
    void* partials = nullptr;   // [grid][cols]
    int grid = 0, rows_per_wg = 0;
    double* W = nullptr;        // [cols]
    double* u = nullptr;        // [rows]
    uint64_t* kron_cur = nullptr;
    uint64_t* kron_rng = nullptr;
    RowPassArgs pass;
    ReduceArgs red;
};

}  // namespace

struct scd_ctx {
    scd_dtype dt = SCD_F32;
    int order = 0;
    int nlevels = 0;
    int64_t dims[SCD_MAX_ORDER] = {0};
    int64_t total = 0;
    int64_t w_capacity = 0;
    uint64_t seed = 0;
    size_t esize = 4;
    hipStream_t stream = nullptr;
    void* R = nullptr;
    Level lv[SCD_MAX_ORDER];
    uint64_t* s_bits[SCD_MAX_ORDER] = {nullptr};
    uint64_t* rng_last = nullptr;
    double* cparts = nullptr;
    int ncparts = 0;
    double* fparts = nullptr;
    State* cur = nullptr;
    State* next = nullptr;
    State* pinned = nullptr;   // host-pinned landing zone for state read-backs
    State hs;                  // host mirror of `cur` as of the last synchronisation
    uint64_t* out_signs[SCD_MAX_ORDER] = {nullptr};
    void* c_out = nullptr;
    double* trace = nullptr;
    int32_t* iters = nullptr;
    KronArgs kron;
    // per-context options (scd_set_option); the defaults are the measured optima
    int64_t opt[SCD_OPT_COUNT] = {
        1,         // SCD_OPT_RESIDENT: the register-resident engine may be used
        1,         // SCD_OPT_SPARSE: the sparse engine may be used
        48,        // SCD_OPT_SPARSE_MIN_MIB
        8,         // SCD_OPT_SPARSE_DELAY_WIDTH
        1,         // SCD_OPT_ROWPASS_KERNEL: register-tiled
        16,        // SCD_OPT_POLL_DELAY
        1 << 22,   // SCD_OPT_MAX_SPIN
        64,        // SCD_OPT_SWEEP_BATCH
        0,         // SCD_OPT_VERBOSE
        1,         // SCD_OPT_PERSISTENT_STREAM: the persistent streaming engine may be used
    };
    // register-resident engine
    bool resident = false;          // shape and dtype fit, and not switched off
    bool stream_stale = false;      // the launch-stream state lags behind the engine's progress
    bool broken = false;            // an engine wait ran out: the remainder is no longer trustworthy
    uint64_t* xbuf = nullptr;
    ResidentResult* res_dev = nullptr;
    ResidentResult* res_pin = nullptr;
    uint32_t seq_u = 0, seq_v = 0;
    // sparse engine
    bool sparse = false;
    bool rt_stale = true;           // RT does not mirror R (R was changed by the launch-stream kernels)
    void* RT = nullptr;
    uint64_t* xbuf_sp = nullptr;
    uint32_t seq_sp = 0;
    int rs = 0, cs = 0;
    // persistent streaming engine
    bool pstream = false;
    void* c_scal = nullptr;         // real last mode (scd_decompose_scalars): n3 coefficients per term; else null
    PStreamGeometry ps_geo = {};
    uint64_t* xbuf_p1 = nullptr;
    uint64_t* xbuf_p2 = nullptr;
    size_t xbuf_p1_bytes = 0, xbuf_p2_bytes = 0;
    uint32_t seq_ps = 0;
    int sp_grid = kSpGrid;          // workgroups of the sparse engine's launch
    int share = 0;                  // most workgroups a persistent launch may take (0: the whole device)
    int cus = 256;                  // compute units of the device
    int64_t flips = 0, flips_rows = 0;  // column / row signs that changed after the first alternation of their term
    hipEvent_t ev0 = nullptr, ev1 = nullptr;  // around the engine's launch
    double last_launch_seconds = 0.0;
    double last_launch_bytes = 0.0;
    std::vector<std::pair<void*, size_t>> allocs;  // device blocks of the context and their sizes
};

namespace {

// Persistent launches of different contexts (host threads, streams) share the device: each needs all of
// its workgroups resident at once, one per compute unit, so a launch waits until that many compute units
// are free of other persistent launches of this process (SlotLease below).
std::mutex g_slots_mutex;
std::condition_variable g_slots_cv;
int g_slots_in_use = 0;

// hipFree and hipHostFree wait for every stream of the device.  While other contexts keep the device busy
// from other threads that wait lasts until their launches end, so a context destroyed then parks its
// blocks here, and contexts created later take blocks of the same size back out (the matrices of a model
// come in a handful of shapes).  With the device idle the blocks are freed.
std::mutex g_pool_mutex;
std::multimap<size_t, void*> g_pool_dev, g_pool_host;
size_t g_pool_dev_bytes = 0;
constexpr size_t kPoolMaxBytes = (size_t)48 << 30;

bool others_running()
{
    std::lock_guard<std::mutex> lk(g_slots_mutex);
    return g_slots_in_use > 0;
}

hipError_t pool_malloc(void** p, size_t bytes, bool host)
{
    {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        auto& pool = host ? g_pool_host : g_pool_dev;
        auto it = pool.find(bytes);
        if (it != pool.end()) {
            *p = it->second;
            pool.erase(it);
            if (!host) g_pool_dev_bytes -= bytes;
            return hipSuccess;
        }
    }
    return host ? hipHostMalloc(p, bytes, hipHostMallocDefault) : hipMalloc(p, bytes);
}

void pool_free(void* p, size_t bytes, bool host)
{
    if (!p) return;
    if (others_running()) {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        if (host || g_pool_dev_bytes + bytes <= kPoolMaxBytes) {
            (host ? g_pool_host : g_pool_dev).emplace(bytes, p);
            if (!host) g_pool_dev_bytes += bytes;
            return;
        }
    }
    if (host) (void)hipHostFree(p);
    else (void)hipFree(p);
}

void pool_drain()
{
    std::multimap<size_t, void*> dev, host;
    {
        std::lock_guard<std::mutex> lk(g_pool_mutex);
        dev.swap(g_pool_dev);
        host.swap(g_pool_host);
        g_pool_dev_bytes = 0;
    }
    for (auto& kv : dev) (void)hipFree(kv.second);
    for (auto& kv : host) (void)hipHostFree(kv.second);
}

int dev_alloc(scd_ctx* c, void** p, size_t bytes)
{
    if (bytes == 0) bytes = 8;
    hipError_t e = pool_malloc(p, bytes, false);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        return SCD_ENOMEM;
    }
    c->allocs.emplace_back(*p, bytes);
    return SCD_OK;
}

#define SCD_TRY(expr)              \
    do {                           \
        int _s = (expr);           \
        if (_s < 0) return _s;     \
    } while (0)

int write_state(scd_ctx* c)
{
    // through the pinned buffer, and complete on return: the host copy may change right after
    *c->pinned = c->hs;
    HIP_TRY(hipMemcpyAsync(c->cur, c->pinned, sizeof(State), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(c->next, c->pinned, sizeof(State), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return SCD_OK;
}

int read_state(scd_ctx* c)
{
    HIP_TRY(hipMemcpyAsync(c->pinned, c->cur, sizeof(State), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    c->hs = *c->pinned;
    return SCD_OK;
}

int launch_sweep(scd_ctx* c)
{
    for (int l = 0; l < c->nlevels; ++l) {
        Level& L = c->lv[l];
        HIP_TRY(launch_rowpass(L.pass, c->dt, L.grid, (int)c->opt[SCD_OPT_ROWPASS_KERNEL], c->stream));
        const bool f32p = (l == 0 && c->dt == SCD_F32);
        HIP_TRY(launch_reduce(L.red, f32p, c->stream));
    }
    if (c->order >= 3) HIP_TRY(launch_kron(c->kron, c->stream));
    return SCD_OK;
}

// (Re)draw the random start of the current term into the device buffers.
int seed_current_term(scd_ctx* c, int term_offset, bool with_last)
{
    KronArgs k = c->kron;
    k.force = 1;
    k.term_offset = term_offset;
    k.with_last = with_last ? 1 : 0;
    HIP_TRY(launch_kron(k, c->stream));
    return SCD_OK;
}

// Enqueue sweeps until the device reports that w_target terms are complete.
int run_until_done(scd_ctx* c, int batch)
{
    const int64_t terms = c->hs.w_target - c->hs.k;
    // every term takes at most max_iters alternations plus its update pass
    const double bound = ((double)(terms > 0 ? terms : 0) + 2.0) * ((double)c->hs.max_iters + 2.0) + 4.0;
    double launched = 0;
    if (batch < 1) batch = 1;
    for (;;) {
        for (int b = 0; b < batch; ++b) SCD_TRY(launch_sweep(c));
        launched += batch;
        SCD_TRY(read_state(c));
        if (c->hs.done) return SCD_OK;
        if (launched > bound + batch) return SCD_EINVAL;  // cannot happen: the device loop is bounded
    }
}

void setup_levels(scd_ctx* c)
{
    const int order = c->order;
    for (int l = 0; l < c->nlevels; ++l) {
        Level& L = c->lv[l];
        RowPassArgs& p = L.pass;
        memset(&p, 0, sizeof(p));
        p.X = L.X;
        p.rows = L.rows;
        p.cols = L.cols;
        p.level = l;
        p.rows_per_wg = L.rows_per_wg;
        p.sign_cur = L.kron_cur;
        p.sign_rng = L.kron_rng;
        p.row_bits = c->s_bits[l];
        p.partials = L.partials;
        p.u = L.u;
        p.fparts = c->fparts;
        p.cparts = c->cparts;
        p.ncparts = c->ncparts;
        p.order = order;
        p.cur = c->cur;
        p.next = c->next;
        p.c_out = c->c_out;
        p.iters_out = c->iters;
        p.total = (double)c->total;
        for (int i = 0; i < order; ++i) {
            p.out_signs[i] = c->out_signs[i];
            p.cur_signs[i] = c->s_bits[i];
            p.words[i] = (int32_t)words_for(c->dims[i]);
        }
        ReduceArgs& r = L.red;
        memset(&r, 0, sizeof(r));
        r.partials = L.partials;
        r.nparts = L.grid;
        r.level = l;
        r.cols = L.cols;
        r.rows = L.rows;
        r.W = L.W;
        r.u = L.u;
        r.row_bits = c->s_bits[l];
        r.final = (l == c->nlevels - 1) ? 1 : 0;
        r.last_bits = c->s_bits[order - 1];
        r.cparts = c->cparts;
        r.rng_last = c->rng_last;
        r.fparts = c->fparts;
        r.nfparts = c->lv[0].grid;
        r.last_mode = order - 1;
        r.trace = c->trace;
        r.seed = c->seed;
        r.cur = c->cur;
        r.next = c->next;
    }
    KronArgs& k = c->kron;
    memset(&k, 0, sizeof(k));
    k.order = order;
    k.term_offset = 1;
    for (int i = 0; i < order; ++i) {
        k.dims[i] = c->dims[i];
        k.cur_signs[i] = c->s_bits[i];
    }
    for (int l = 0; l + 2 < order; ++l) {
        k.kron_cur[l] = c->lv[l].kron_cur;
        k.kron_rng[l] = c->lv[l].kron_rng;
        k.cols[l] = c->lv[l].cols;
    }
    k.rng_last = c->rng_last;
    k.seed = c->seed;
    k.cur = c->cur;
    k.next = c->next;
}

int check_dims(int order, const int64_t* dims, int64_t* total)
{
    if (!dims || order < 2 || order > SCD_MAX_ORDER) return SCD_EINVAL;
    double t = 1.0;
    int64_t n = 1;
    for (int i = 0; i < order; ++i) {
        if (dims[i] < 1) return SCD_EINVAL;
        t *= (double)dims[i];
        n *= dims[i];
    }
    if (t > 4.0e12) return SCD_EINVAL;
    *total = n;
    return SCD_OK;
}

bool dtype_ok(int dt) { return dt == SCD_F32 || dt == SCD_F64; }

// Bring the launch-stream state (first alternation of term k done, ||R_k|| known) up to date after the
// resident engine advanced the context.
int resync_stream_state(scd_ctx* c)
{
    c->rt_stale = true;  // the caller is about to let the launch-stream kernels change R
    if (!c->stream_stale) return SCD_OK;
    c->hs.w_target = c->hs.k;
    c->hs.done = 0;
    c->hs.j = 0;
    c->hs.t0_given = 0;
    c->hs.c_prev = -INFINITY;
    SCD_TRY(write_state(c));
    SCD_TRY(seed_current_term(c, 0, true));
    SCD_TRY(launch_sweep(c));
    SCD_TRY(read_state(c));
    c->stream_stale = false;
    return SCD_OK;
}

struct SlotLease {
    int n = 0;
    void acquire(int want, int capacity)
    {
        if (want > capacity) want = capacity;  // the occupancy check of the launcher has the last word
        std::unique_lock<std::mutex> lk(g_slots_mutex);
        g_slots_cv.wait(lk, [&] { return g_slots_in_use + want <= capacity; });
        g_slots_in_use += want;
        n = want;
    }
    ~SlotLease()
    {
        if (!n) return;
        {
            std::lock_guard<std::mutex> lk(g_slots_mutex);
            g_slots_in_use -= n;
        }
        g_slots_cv.notify_all();
    }
};

// Which engine serves this context, and its buffers (allocated once, kept until scd_destroy).
int setup_engines(scd_ctx* c)
{
    const int limit = c->share > 0 ? c->share : c->cus;
    c->resident = c->opt[SCD_OPT_RESIDENT] != 0 && resident_supported(c->dt, c->order, c->dims) &&
                  resident_workgroups(c->dims) <= limit;
    c->sparse = false;
    if (!c->resident && c->opt[SCD_OPT_SPARSE] != 0) {
        // The sparse engine pays about 15 us per alternation whatever the size, the launch-stream engine
        // one pass over the remainder: the former wins from about 48 MiB on (SCD_OPT_SPARSE_MIN_MIB moves
        // the line).  A context that was given a share of the device runs side by side with others, which
        // hides exactly that latency: it takes the sparse engine at any size.
        const double mib = (double)c->total * (double)c->esize / (1024.0 * 1024.0);
        const int grid = limit < kSpGrid ? limit : kSpGrid;
        const bool big = c->share > 0 || mib >= (double)c->opt[SCD_OPT_SPARSE_MIN_MIB];
        if (big && grid >= 1 && sparse_supported(c->dt, c->order, c->dims, grid, &c->rs, &c->cs)) {
            c->sparse = true;
            c->sp_grid = grid;
        }
    }
    auto hip_ok = [](hipError_t e) {
        if (e == hipSuccess) return true;
        g_last_hip = (int)e;
        (void)hipGetLastError();
        return false;
    };
    if (c->sparse && !c->RT) {
        // the transpose doubles the footprint: without room for it the launch-stream engine serves
        if (pool_malloc(&c->RT, (size_t)c->total * c->esize, false) != hipSuccess) {
            (void)hipGetLastError();
            c->RT = nullptr;
            c->sparse = false;
        } else {
            c->allocs.emplace_back(c->RT, (size_t)c->total * c->esize);
            c->rt_stale = true;
            SCD_TRY(dev_alloc(c, (void**)&c->xbuf_sp, sparse_xbuf_bytes()));
            if (!hip_ok(hipMemsetAsync(c->xbuf_sp, 0, sparse_xbuf_bytes(), c->stream))) return SCD_EHIP;
        }
    }
    c->pstream = false;
    if (!c->resident && !c->sparse && c->opt[SCD_OPT_PERSISTENT_STREAM] != 0 &&
        pstream_supported(c->dt, c->order, c->dims, limit, &c->ps_geo)) {
        c->pstream = true;
        // the exchange slots follow the geometry (the share of the device may have changed it)
        if (c->xbuf_p1_bytes < c->ps_geo.xp_bytes) {
            SCD_TRY(dev_alloc(c, (void**)&c->xbuf_p1, c->ps_geo.xp_bytes));
            c->xbuf_p1_bytes = c->ps_geo.xp_bytes;
        }
        if (c->xbuf_p2_bytes < c->ps_geo.xq_bytes) {
            SCD_TRY(dev_alloc(c, (void**)&c->xbuf_p2, c->ps_geo.xq_bytes));
            c->xbuf_p2_bytes = c->ps_geo.xq_bytes;
        }
        // a new geometry reads other slots than the last one wrote: start the numbering again on cleared slots
        if (!hip_ok(hipMemsetAsync(c->xbuf_p1, 0, c->xbuf_p1_bytes, c->stream))) return SCD_EHIP;
        if (!hip_ok(hipMemsetAsync(c->xbuf_p2, 0, c->xbuf_p2_bytes, c->stream))) return SCD_EHIP;
        c->seq_ps = 0;
    }
    if (c->resident && !c->xbuf) {
        const size_t xb = (size_t)4 * kResGrid * kResGrid * kResSlotWords * 8;
        SCD_TRY(dev_alloc(c, (void**)&c->xbuf, xb));
        if (!hip_ok(hipMemsetAsync(c->xbuf, 0, xb, c->stream))) return SCD_EHIP;
    }
    if ((c->resident || c->sparse || c->pstream) && !c->res_dev) {
        SCD_TRY(dev_alloc(c, (void**)&c->res_dev, sizeof(ResidentResult)));
        if (!hip_ok(pool_malloc((void**)&c->res_pin, sizeof(ResidentResult), true))) return SCD_EHIP;
        if (!hip_ok(hipEventCreate(&c->ev0)) || !hip_ok(hipEventCreate(&c->ev1))) return SCD_EHIP;
    }
    return SCD_OK;
}

// n terms in one persistent launch that updates the cached products from the flipped signs only.
int run_sparse(scd_ctx* c, int64_t n)
{
    if (c->rt_stale) {
        HIP_TRY(launch_transpose(c->R, c->RT, c->dt, c->dims[0], c->dims[1], c->stream));
        c->rt_stale = false;
    }
    SparseArgs a;
    memset(&a, 0, sizeof(a));
    a.R = c->R;
    a.RT = c->RT;
    a.m = c->dims[0];
    a.n = c->dims[1];
    a.seed = c->seed;
    a.k_start = c->hs.k;
    a.w_target = c->hs.k + n;
    a.max_iters = c->hs.max_iters;
    a.max_spin = (int32_t)c->opt[SCD_OPT_MAX_SPIN];
    a.poll_delay = (int32_t)c->opt[SCD_OPT_POLL_DELAY];
    a.seq = c->seq_sp;
    a.xbuf = c->xbuf_sp;
    a.S = c->out_signs[0];
    a.T = c->out_signs[1];
    a.c = c->c_out;
    a.iters = c->iters;
    a.trace = c->trace;
    a.mw = (int32_t)words_for(c->dims[0]);
    a.nw = (int32_t)words_for(c->dims[1]);
    a.rs = c->rs;
    a.cs = c->cs;
    a.grid = c->sp_grid;
    // Delayed updates (Section 3.2) trade the writes of the dense start of a term for a correction on every
    // half step, whose cost grows with the length of the pending list.  Measured on this chip the best length
    // is 8, not the paper's 32 (14336x4096: 1084 terms/s immediate, 1175 with 8, 1144 with 16, 1017 with 32;
    // 32000x4096: 781 / 900 / 873; 4096x4096: 1137 / 1165 / 1076 / 942).  SCD_OPT_SPARSE_DELAY_WIDTH sets the
    // length (4..32), 0 switches the list off.
    {
        const int cap = (int)c->opt[SCD_OPT_SPARSE_DELAY_WIDTH];
        int width = cap > 0 ? sparse_delay_width(c->dims[0], c->dims[1]) : 0;
        if (width > cap) width = cap;
        a.delay_width = width;
    }
    a.profile = (int32_t)c->opt[SCD_OPT_VERBOSE];
    a.res = c->res_dev;
    SlotLease lease;
    lease.acquire(a.grid, c->cus);
    HIP_TRY(hipMemsetAsync(c->res_dev, 0, sizeof(ResidentResult), c->stream));
    HIP_TRY(hipEventRecord(c->ev0, c->stream));
    HIP_TRY(launch_sparse(a, c->dt, c->stream));
    HIP_TRY(hipEventRecord(c->ev1, c->stream));
    HIP_TRY(hipMemcpyAsync(c->res_pin, c->res_dev, sizeof(ResidentResult), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    const ResidentResult r = *c->res_pin;
    {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, c->ev0, c->ev1));
        c->last_launch_seconds = (double)ms * 1e-3;
        c->last_launch_bytes = ((double)r.alternations + (double)r.updates) * (double)c->total * (double)c->esize;
    }
    if (r.err || r.k != a.w_target) {
        c->broken = true;
        return SCD_ETIMEOUT;
    }
    if (c->opt[SCD_OPT_VERBOSE])
        fprintf(stderr, "[scd sparse] terms %lld alternations %lld flips %lld re-reads %lld; us: dense %.0f, t-exchange %.0f, "
                        "decide %.0f, u-update %.0f, s-exchange %.0f, v-update %.0f\n", (long long)n,
                (long long)r.alternations, (long long)(r.flips + r.flips_rows), (long long)r.spins, r.ticks[0] * 0.01, r.ticks[1] * 0.01,
                r.ticks[2] * 0.01, r.ticks[3] * 0.01, r.ticks[4] * 0.01, r.ticks[5] * 0.01);
    c->seq_sp = r.seq_u;
    c->flips += r.flips;
    c->flips_rows += r.flips_rows;
    c->hs.k = r.k;
    c->hs.passes += r.alternations;
    c->hs.updates += r.updates;
    if (r.warn) c->hs.warn = 1;
    c->stream_stale = true;
    return SCD_OK;
}

// n terms in one persistent launch that streams the remainder once per alternation.
int run_pstream(scd_ctx* c, int64_t n)
{
    PStreamArgs a;
    memset(&a, 0, sizeof(a));
    const PStreamGeometry& geo = c->ps_geo;
    a.R = c->R;
    a.m = c->dims[0];
    a.n = c->order == 2 ? c->dims[1] : c->dims[1] * c->dims[2];
    if (c->order == 3) {
        a.n2 = (int32_t)c->dims[1];
        a.n3 = (int32_t)c->dims[2];
        a.w2 = (int32_t)words_for(c->dims[1]);
        a.S3 = c->out_signs[2];
        a.scalars = c->c_scal ? 1 : 0;
    }
    a.seed = c->seed;
    a.k_start = c->hs.k;
    a.w_target = c->hs.k + n;
    a.max_iters = c->hs.max_iters;
    a.max_spin = (int32_t)c->opt[SCD_OPT_MAX_SPIN];
    a.poll_delay = (int32_t)c->opt[SCD_OPT_POLL_DELAY];
    a.seq = c->seq_ps;
    a.xp = c->xbuf_p1;
    a.xq = c->xbuf_p2;
    a.S = c->out_signs[0];
    a.T = c->out_signs[1];
    a.c = a.scalars ? c->c_scal : c->c_out;
    a.iters = c->iters;
    a.trace = c->trace;
    a.mw = (int32_t)words_for(c->dims[0]);
    a.nw = (int32_t)words_for(a.n);
    a.grid = geo.grid;
    a.rpw = geo.rpw;
    a.cs = geo.cs;
    a.lds_rows = geo.lds_rows;
    a.profile = (int32_t)c->opt[SCD_OPT_VERBOSE];
    a.res = c->res_dev;
    SlotLease lease;
    lease.acquire(a.grid, c->cus);
    // the workgroups OR their rows' bits into S: the terms of this launch start from zero
    HIP_TRY(hipMemsetAsync(c->out_signs[0] + c->hs.k * a.mw, 0, (size_t)n * (size_t)a.mw * 8, c->stream));
    HIP_TRY(hipMemsetAsync(c->res_dev, 0, sizeof(ResidentResult), c->stream));
    HIP_TRY(hipEventRecord(c->ev0, c->stream));
    HIP_TRY(launch_pstream(a, c->dt, geo.lds_bytes, c->stream));
    HIP_TRY(hipEventRecord(c->ev1, c->stream));
    HIP_TRY(hipMemcpyAsync(c->res_pin, c->res_dev, sizeof(ResidentResult), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    const ResidentResult r = *c->res_pin;
    {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, c->ev0, c->ev1));
        c->last_launch_seconds = (double)ms * 1e-3;
        // one read of R per pass, one more write per update
        c->last_launch_bytes = ((double)r.alternations + (double)r.updates) * (double)c->total * (double)c->esize;
    }
    if (r.err || r.k != a.w_target) {
        c->broken = true;
        return SCD_ETIMEOUT;
    }
    if (c->opt[SCD_OPT_VERBOSE])
        fprintf(stderr, "[scd stream] terms %lld passes %lld re-reads %lld; grid %d, %d rows per workgroup, %d of them in LDS; "
                        "us per pass: rows %.2f, publish %.2f, hop-1 gather %.2f, slice %.2f, hop-2 %.2f, decide %.2f\n",
                (long long)n, (long long)r.alternations, (long long)r.spins, geo.grid, geo.rpw, geo.lds_rows,
                r.ticks[0] * 0.01 / r.alternations, r.ticks[1] * 0.01 / r.alternations, r.ticks[2] * 0.01 / r.alternations,
                r.ticks[3] * 0.01 / r.alternations, r.ticks[4] * 0.01 / r.alternations, r.ticks[5] * 0.01 / r.alternations);
    c->seq_ps = r.seq_u;
    c->rt_stale = true;  // the remainder changed, the transposed copy of the sparse engine did not
    c->hs.k = r.k;
    c->hs.passes += r.alternations;
    c->hs.updates += r.updates;
    if (r.warn) c->hs.warn = 1;
    c->stream_stale = true;
    return SCD_OK;
}

// n terms in one persistent launch with the remainder held in registers.
int run_resident(scd_ctx* c, int64_t n)
{
    ResidentArgs a;
    memset(&a, 0, sizeof(a));
    a.R = (float*)c->R;
    a.m = c->dims[0];
    a.n = c->dims[1];
    a.seed = c->seed;
    a.k_start = c->hs.k;
    a.w_target = c->hs.k + n;
    a.max_iters = c->hs.max_iters;
    a.max_spin = (int32_t)c->opt[SCD_OPT_MAX_SPIN];
    a.poll_delay = (int32_t)c->opt[SCD_OPT_POLL_DELAY];
    a.seq_u = c->seq_u;
    a.seq_v = c->seq_v;
    a.xbuf = c->xbuf;
    a.S = c->out_signs[0];
    a.T = c->out_signs[1];
    a.c = (float*)c->c_out;
    a.iters = c->iters;
    a.trace = c->trace;
    a.mw = (int32_t)words_for(c->dims[0]);
    a.nw = (int32_t)words_for(c->dims[1]);
    a.res = c->res_dev;
    SlotLease lease;
    lease.acquire(resident_workgroups(c->dims), c->cus);
    HIP_TRY(hipMemsetAsync(c->res_dev, 0, sizeof(ResidentResult), c->stream));
    HIP_TRY(hipEventRecord(c->ev0, c->stream));
    HIP_TRY(launch_resident(a, c->stream));
    HIP_TRY(hipEventRecord(c->ev1, c->stream));
    HIP_TRY(hipMemcpyAsync(c->res_pin, c->res_dev, sizeof(ResidentResult), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    const ResidentResult r = *c->res_pin;
    {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, c->ev0, c->ev1));
        c->last_launch_seconds = (double)ms * 1e-3;
        // one read of R per alternation, one write per update (what a streaming implementation must move)
        c->last_launch_bytes = ((double)r.alternations + (double)r.updates) * (double)c->total * (double)c->esize;
    }
    if (r.err || r.k != a.w_target) {
        c->broken = true;
        return SCD_ETIMEOUT;
    }
    if (c->opt[SCD_OPT_VERBOSE])
        fprintf(stderr, "[scd resident] terms %lld alternations %lld re-reads %lld\n", (long long)n,
                (long long)r.alternations, (long long)r.spins);
    c->seq_u = r.seq_u;
    c->seq_v = r.seq_v;
    c->rt_stale = true;  // the remainder changed, the transposed copy of the sparse engine did not
    c->hs.k = r.k;
    c->hs.passes += r.alternations;
    c->hs.updates += r.updates;
    if (r.warn) c->hs.warn = 1;
    c->stream_stale = true;
    return SCD_OK;
}

}  // namespace

extern "C" {

int scd_create(scd_ctx** out, const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w_capacity,
               uint64_t seed, void* stream)
{
    if (!out) return SCD_EINVAL;
    *out = nullptr;
    int64_t total = 0;
    if (!A || !dtype_ok(dt) || w_capacity < 0) return SCD_EINVAL;
    SCD_TRY(check_dims(order, dims, &total));
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
        (void)hipGetLastError();
        return SCD_ENODEVICE;
    }
    scd_ctx* c = new (std::nothrow) scd_ctx();
    if (!c) return SCD_ENOMEM;
    c->dt = dt;
    c->order = order;
    c->nlevels = order - 1;
    c->total = total;
    c->w_capacity = w_capacity;
    c->seed = seed;
    c->esize = dt == SCD_F32 ? 4 : 8;
    c->stream = (hipStream_t)stream;
    for (int i = 0; i < order; ++i) c->dims[i] = dims[i];
    // one workgroup per compute unit: every partial row costs a write and a read per alternation
    int cus = 256;
    {
        int devid = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&devid) == hipSuccess && hipGetDeviceProperties(&prop, devid) == hipSuccess &&
            prop.multiProcessorCount > 0)
            cus = prop.multiProcessorCount;
        (void)hipGetLastError();
    }
    const int wg_target = cus;

    int st = SCD_OK;
    auto fail = [&](int code) {
        scd_destroy(c);
        return code;
    };
#define CTRY(expr)                     \
    do {                               \
        st = (expr);                   \
        if (st < 0) return fail(st);   \
    } while (0)
#define CHIP(expr)                         \
    do {                                   \
        hipError_t _e = (expr);            \
        if (_e != hipSuccess) {            \
            g_last_hip = (int)_e;          \
            (void)hipGetLastError();       \
            return fail(SCD_EHIP);         \
        }                                  \
    } while (0)

    CTRY(dev_alloc(c, &c->R, (size_t)total * c->esize));
    for (int i = 0; i < order; ++i) {
        CTRY(dev_alloc(c, (void**)&c->s_bits[i], (size_t)words_for(dims[i]) * 8));
        CHIP(hipMemsetAsync(c->s_bits[i], 0, (size_t)words_for(dims[i]) * 8, c->stream));
        CTRY(dev_alloc(c, (void**)&c->out_signs[i], (size_t)w_capacity * words_for(dims[i]) * 8));
    }
    CTRY(dev_alloc(c, (void**)&c->rng_last, (size_t)words_for(dims[order - 1]) * 8));
    CTRY(dev_alloc(c, &c->c_out, (size_t)w_capacity * c->esize));
    CTRY(dev_alloc(c, (void**)&c->trace, (size_t)(w_capacity + 1) * 8));
    CTRY(dev_alloc(c, (void**)&c->iters, (size_t)w_capacity * 4));
    CTRY(dev_alloc(c, (void**)&c->cur, sizeof(State)));
    CTRY(dev_alloc(c, (void**)&c->next, sizeof(State)));
    CHIP(pool_malloc((void**)&c->pinned, sizeof(State), true));

    int64_t cols = total;
    for (int l = 0; l < c->nlevels; ++l) {
        Level& L = c->lv[l];
        L.rows = dims[l];
        cols /= dims[l];
        L.cols = cols;
        int64_t rpw = (L.rows + wg_target - 1) / wg_target;
        if (rpw < 1) rpw = 1;
        if (rpw > kMaxRowsPerWg) rpw = kMaxRowsPerWg;
        L.rows_per_wg = (int)rpw;
        L.grid = (int)((L.rows + rpw - 1) / rpw);
        const size_t es = (l == 0) ? c->esize : 8;
        CTRY(dev_alloc(c, &L.partials, (size_t)L.grid * (size_t)L.cols * es));
        CTRY(dev_alloc(c, (void**)&L.W, (size_t)L.cols * 8));
        CTRY(dev_alloc(c, (void**)&L.u, (size_t)L.rows * 8));
        L.X = (l == 0) ? c->R : (void*)c->lv[l - 1].W;
        if (l == c->nlevels - 1) {
            L.kron_cur = c->s_bits[order - 1];
            L.kron_rng = c->rng_last;
        } else {
            CTRY(dev_alloc(c, (void**)&L.kron_cur, (size_t)words_for(L.cols) * 8));
            CTRY(dev_alloc(c, (void**)&L.kron_rng, (size_t)words_for(L.cols) * 8));
        }
    }
    c->cus = cus;
    CTRY(setup_engines(c));
    c->ncparts = (int)words_for(dims[order - 1]);
    CTRY(dev_alloc(c, (void**)&c->cparts, (size_t)c->ncparts * 8));
    CHIP(hipMemsetAsync(c->cparts, 0, (size_t)c->ncparts * 8, c->stream));
    CTRY(dev_alloc(c, (void**)&c->fparts, (size_t)c->lv[0].grid * 8));
    setup_levels(c);

    CHIP(hipMemcpyAsync(c->R, A, (size_t)total * c->esize, hipMemcpyDeviceToDevice, c->stream));
    memset(&c->hs, 0, sizeof(State));
    c->hs.c_prev = -INFINITY;
    c->hs.max_iters = SCD_DEFAULT_MAX_ITERS;
    CTRY(write_state(c));
    CTRY(seed_current_term(c, 0, true));
    // first pass of term 0; it also yields ||R_0||_F.  w_target = 0 stops the device right after.
    CTRY(launch_sweep(c));
    CTRY(read_state(c));
    double f0 = 0.0;
    CHIP(hipMemcpy(&f0, c->trace, sizeof(double), hipMemcpyDeviceToHost));
    if (!isfinite(f0)) return fail(SCD_ENONFINITE);
    *out = c;
    return SCD_OK;
#undef CTRY
#undef CHIP
}

void scd_destroy(scd_ctx* c)
{
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (auto& b : c->allocs) pool_free(b.first, b.second, false);
    pool_free(c->pinned, sizeof(State), true);
    pool_free(c->res_pin, sizeof(ResidentResult), true);
    if (!others_running()) pool_drain();
    if (c->ev0) (void)hipEventDestroy(c->ev0);
    if (c->ev1) (void)hipEventDestroy(c->ev1);
    (void)hipGetLastError();
    delete c;
}

int scd_set_max_iters(scd_ctx* c, int32_t max_iters)
{
    if (!c || max_iters < 1) return SCD_EINVAL;
    c->hs.max_iters = max_iters;
    return write_state(c);
}

int scd_set_workgroups(scd_ctx* c, int workgroups)
{
    if (!c || workgroups < 0) return SCD_EINVAL;
    if (workgroups != 0 && workgroups < 16) return SCD_EINVAL;
    if (c->broken) return SCD_ETIMEOUT;
    c->share = workgroups >= c->cus ? 0 : workgroups;
    return setup_engines(c);
}

int scd_set_option(scd_ctx* c, int option, int64_t value)
{
    if (!c || option < 0 || option >= SCD_OPT_COUNT) return SCD_EINVAL;
    switch (option) {
        case SCD_OPT_RESIDENT:
        case SCD_OPT_SPARSE:
        case SCD_OPT_PERSISTENT_STREAM:
        case SCD_OPT_ROWPASS_KERNEL:
        case SCD_OPT_VERBOSE:
            if (value != 0 && value != 1) return SCD_EINVAL;
            break;
        case SCD_OPT_SPARSE_MIN_MIB:
            if (value < 0 || value > (1 << 30)) return SCD_EINVAL;
            break;
        case SCD_OPT_SPARSE_DELAY_WIDTH:
            if (value != 0 && (value < 4 || value > 32)) return SCD_EINVAL;
            break;
        case SCD_OPT_POLL_DELAY:
            if (value < 0 || value > 4096) return SCD_EINVAL;
            break;
        case SCD_OPT_MAX_SPIN:
            if (value < 0 || value > (1ll << 30)) return SCD_EINVAL;
            break;
        case SCD_OPT_SWEEP_BATCH:
            if (value < 1 || value > 4096) return SCD_EINVAL;
            break;
        default: return SCD_EINVAL;
    }
    c->opt[option] = value;
    if (option == SCD_OPT_RESIDENT || option == SCD_OPT_SPARSE || option == SCD_OPT_SPARSE_MIN_MIB ||
        option == SCD_OPT_PERSISTENT_STREAM) {
        if (c->broken) return SCD_ETIMEOUT;
        return setup_engines(c);
    }
    return SCD_OK;
}

int scd_get_option(const scd_ctx* c, int option, int64_t* value)
{
    if (!c || !value || option < 0 || option >= SCD_OPT_COUNT) return SCD_EINVAL;
    *value = c->opt[option];
    return SCD_OK;
}

int scd_run(scd_ctx* c, int64_t n)
{
    if (!c || n < 0) return SCD_EINVAL;
    if (c->broken) return SCD_ETIMEOUT;
    if (n == 0) return c->hs.warn ? SCD_WMAXITER : SCD_OK;
    if (c->hs.k + n > c->w_capacity) return SCD_EFULL;
    if (c->resident || c->sparse || c->pstream) {
        SCD_TRY(c->resident ? run_resident(c, n) : (c->sparse ? run_sparse(c, n) : run_pstream(c, n)));
        return c->hs.warn ? SCD_WMAXITER : SCD_OK;
    }
    SCD_TRY(resync_stream_state(c));  // a persistent engine may have advanced the context before it lost its share
    c->hs.w_target = c->hs.k + n;
    c->hs.done = 0;
    SCD_TRY(write_state(c));
    int batch = (int)c->opt[SCD_OPT_SWEEP_BATCH];
    if (n == 1 && batch > 16) batch = 16;
    SCD_TRY(run_until_done(c, batch));
    return c->hs.warn ? SCD_WMAXITER : SCD_OK;
}

int scd_step(scd_ctx* c) { return scd_run(c, 1); }

int scd_step_from(scd_ctx* c, const uint64_t* const* init_signs)
{
    if (!c || !init_signs) return SCD_EINVAL;
    for (int i = 1; i < c->order; ++i)
        if (!init_signs[i]) return SCD_EINVAL;
    if (c->broken) return SCD_ETIMEOUT;
    if (c->hs.k + 1 > c->w_capacity) return SCD_EFULL;
    SCD_TRY(resync_stream_state(c));
    for (int i = 1; i < c->order; ++i)
        HIP_TRY(hipMemcpyAsync(c->s_bits[i], init_signs[i], (size_t)words_for(c->dims[i]) * 8, hipMemcpyDeviceToDevice,
                               c->stream));
    c->hs.w_target = c->hs.k + 1;
    c->hs.done = 0;
    c->hs.j = 0;
    c->hs.t0_given = 1;
    c->hs.c_prev = -INFINITY;
    SCD_TRY(write_state(c));
    if (c->order >= 3) SCD_TRY(seed_current_term(c, 1, false));
    SCD_TRY(run_until_done(c, c->opt[SCD_OPT_SWEEP_BATCH] > 16 ? 16 : (int)c->opt[SCD_OPT_SWEEP_BATCH]));
    return c->hs.warn ? SCD_WMAXITER : SCD_OK;
}

int scd_width(const scd_ctx* c, int64_t* k)
{
    if (!c || !k) return SCD_EINVAL;
    *k = c->hs.k;
    return SCD_OK;
}

int scd_results(const scd_ctx* c, uint64_t* const* signs, void* cvec, double* fro_trace, int32_t* iters)
{
    if (!c) return SCD_EINVAL;
    const int64_t k = c->hs.k;
    if (signs && k > 0) {
        for (int i = 0; i < c->order; ++i) {
            if (!signs[i]) return SCD_EINVAL;
            HIP_TRY(hipMemcpyAsync(signs[i], c->out_signs[i], (size_t)k * words_for(c->dims[i]) * 8,
                                   hipMemcpyDeviceToDevice, c->stream));
        }
    }
    if (cvec && k > 0) HIP_TRY(hipMemcpyAsync(cvec, c->c_out, (size_t)k * c->esize, hipMemcpyDeviceToDevice, c->stream));
    if (fro_trace)
        HIP_TRY(hipMemcpyAsync(fro_trace, c->trace, (size_t)(k + 1) * 8, hipMemcpyDeviceToDevice, c->stream));
    if (iters && k > 0) HIP_TRY(hipMemcpyAsync(iters, c->iters, (size_t)k * 4, hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return SCD_OK;
}

int scd_remainder(const scd_ctx* c, void* R_out)
{
    if (!c || !R_out) return SCD_EINVAL;
    if (c->broken) return SCD_ETIMEOUT;
    HIP_TRY(hipMemcpyAsync(R_out, c->R, (size_t)c->total * c->esize, hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return SCD_OK;
}

int scd_set_remainder(scd_ctx* c, const void* R_in)
{
    if (!c || !R_in) return SCD_EINVAL;
    c->stream_stale = false;  // the start pass below rebuilds the launch-stream state
    c->rt_stale = true;
    if (c->broken) {
        // A launch that gave up left tagged words of exchanges it never finished in the slots, and its
        // sequence numbers were not handed back: start the numbering again on cleared buffers, so that no
        // stale word can pass for a fresh one.
        if (c->xbuf) HIP_TRY(hipMemsetAsync(c->xbuf, 0, (size_t)4 * kResGrid * kResGrid * kResSlotWords * 8, c->stream));
        if (c->xbuf_sp) HIP_TRY(hipMemsetAsync(c->xbuf_sp, 0, sparse_xbuf_bytes(), c->stream));
        if (c->xbuf_p1) HIP_TRY(hipMemsetAsync(c->xbuf_p1, 0, c->xbuf_p1_bytes, c->stream));
        if (c->xbuf_p2) HIP_TRY(hipMemsetAsync(c->xbuf_p2, 0, c->xbuf_p2_bytes, c->stream));
        c->seq_u = c->seq_v = c->seq_sp = c->seq_ps = 0;
    }
    c->broken = false;
    HIP_TRY(hipMemcpyAsync(c->R, R_in, (size_t)c->total * c->esize, hipMemcpyDeviceToDevice, c->stream));
    c->hs.w_target = c->hs.k;
    c->hs.done = 0;
    c->hs.j = 0;
    c->hs.t0_given = 0;
    c->hs.c_prev = -INFINITY;
    SCD_TRY(write_state(c));
    SCD_TRY(seed_current_term(c, 0, true));
    SCD_TRY(launch_sweep(c));
    SCD_TRY(read_state(c));
    double f = 0.0;
    HIP_TRY(hipMemcpy(&f, c->trace + c->hs.k, sizeof(double), hipMemcpyDeviceToHost));
    if (!isfinite(f)) return SCD_ENONFINITE;
    return SCD_OK;
}

int scd_engine(const scd_ctx* c, int* engine, double* last_launch_seconds, double* last_launch_bytes)
{
    if (!c) return SCD_EINVAL;
    if (engine) *engine = c->resident ? 1 : (c->sparse ? 2 : (c->pstream ? 3 : 0));
    if (last_launch_seconds) *last_launch_seconds = c->last_launch_seconds;
    if (last_launch_bytes) *last_launch_bytes = c->last_launch_bytes;
    return SCD_OK;
}

int scd_stream_geometry(scd_dtype dt, int order, const int64_t* dims, int limit, int64_t out[8])
{
    if (!dims || !out || !dtype_ok(dt) || order < 2 || order > SCD_MAX_ORDER) return SCD_EINVAL;
    PStreamGeometry g = {};
    const bool ok = pstream_supported(dt, order, dims, limit, &g);
    out[0] = ok ? 1 : 0;
    out[1] = g.grid;
    out[2] = g.rpw;
    out[3] = g.cs;
    out[4] = g.lds_rows;
    out[5] = (int64_t)g.lds_bytes;
    out[6] = (int64_t)g.xp_bytes;
    out[7] = (int64_t)g.xq_bytes;
    return SCD_OK;
}

int scd_sparse_flips(const scd_ctx* c, int64_t* row_flips, int64_t* col_flips)
{
    if (!c) return SCD_EINVAL;
    if (row_flips) *row_flips = c->flips_rows;
    if (col_flips) *col_flips = c->flips;
    return SCD_OK;
}

int scd_traffic(const scd_ctx* c, double* bytes, int64_t* passes, int64_t* sweeps)
{
    if (!c) return SCD_EINVAL;
    const double pass_bytes = (double)c->total * (double)c->esize;
    if (bytes) *bytes = pass_bytes * ((double)c->hs.passes + (double)c->hs.updates);
    if (passes) *passes = c->hs.passes;
    if (sweeps) *sweeps = c->hs.passes;
    return SCD_OK;
}

int scd_profile_sweeps(scd_ctx* c, int n, double* rowpass_seconds, double* reduce_seconds)
{
    if (!c || n < 1 || n > 4096 || !rowpass_seconds || !reduce_seconds) return SCD_EINVAL;
    if (c->broken) return SCD_ETIMEOUT;
    if (c->hs.k >= c->w_capacity) return SCD_EFULL;
    SCD_TRY(resync_stream_state(c));
    // keep the device loop running for the whole sample: aim at the capacity, restore nothing (the
    // terms found while sampling are ordinary terms)
    c->hs.w_target = c->w_capacity;
    c->hs.done = 0;
    SCD_TRY(write_state(c));
    std::vector<hipEvent_t> ev((size_t)3 * n, nullptr);
    int rc = SCD_OK;
    hipError_t e = hipSuccess;
    for (size_t i = 0; i < ev.size() && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    Level& L = c->lv[0];
    for (int i = 0; i < n && e == hipSuccess; ++i) {
        e = hipEventRecord(ev[3 * i], c->stream);
        if (e == hipSuccess) e = launch_rowpass(L.pass, c->dt, L.grid, (int)c->opt[SCD_OPT_ROWPASS_KERNEL], c->stream);
        if (e == hipSuccess) e = hipEventRecord(ev[3 * i + 1], c->stream);
        if (e == hipSuccess) e = launch_reduce(L.red, c->dt == SCD_F32, c->stream);
        if (e == hipSuccess) e = hipEventRecord(ev[3 * i + 2], c->stream);
        for (int l = 1; l < c->nlevels && e == hipSuccess; ++l) {
            e = launch_rowpass(c->lv[l].pass, c->dt, c->lv[l].grid, (int)c->opt[SCD_OPT_ROWPASS_KERNEL], c->stream);
            if (e == hipSuccess) e = launch_reduce(c->lv[l].red, false, c->stream);
        }
        if (e == hipSuccess && c->order >= 3) e = launch_kron(c->kron, c->stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    double tp = 0.0, tr = 0.0;
    for (int i = 0; i < n && e == hipSuccess; ++i) {
        float a = 0.f, b = 0.f;
        e = hipEventElapsedTime(&a, ev[3 * i], ev[3 * i + 1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&b, ev[3 * i + 1], ev[3 * i + 2]);
        tp += a;
        tr += b;
    }
    for (hipEvent_t x : ev)
        if (x) (void)hipEventDestroy(x);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        return SCD_EHIP;
    }
    *rowpass_seconds = tp * 1e-3 / n;
    *reduce_seconds = tr * 1e-3 / n;
    rc = read_state(c);
    return rc;
}

int scd_decompose(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, uint64_t seed, void* stream,
                  uint64_t* const* signs, void* cvec, double* fro_trace, int32_t* iters)
{
    if (!A || !fro_trace || w < 0 || (w > 0 && (!signs || !cvec))) return SCD_EINVAL;
    scd_ctx* c = nullptr;
    int st = scd_create(&c, A, dt, order, dims, w, seed, stream);
    if (st < 0) return st;
    int run = scd_run(c, w);
    if (run < 0) {
        scd_destroy(c);
        return run;
    }
    st = scd_results(c, signs, cvec, fro_trace, iters);
    scd_destroy(c);
    return st < 0 ? st : run;
}

// ---------------------------------------------------------------------------------------------- half steps

static int halfstep_geometry(int64_t m, int* rows_per_wg, int* grid)
{
    int64_t rpw = (m + 1023) / 1024;
    if (rpw < 1) rpw = 1;
    if (rpw > kMaxRowsPerWg) rpw = kMaxRowsPerWg;
    *rows_per_wg = (int)rpw;
    *grid = (int)((m + rpw - 1) / rpw);
    return SCD_OK;
}

int scd_row_signed_sum(const void* R, scd_dtype dt, int64_t m, int64_t n, const uint64_t* tbits, void* stream, double* u,
                       uint64_t* sbits)
{
    if (!R || !tbits || !dtype_ok(dt) || m < 1 || n < 1) return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    double* utmp = nullptr;
    if (!u) {
        hipError_t e = hipMalloc((void**)&utmp, (size_t)m * 8);
        if (e != hipSuccess) {
            g_last_hip = (int)e;
            (void)hipGetLastError();
            return SCD_ENOMEM;
        }
        u = utmp;
    }
    int rpw, grid;
    halfstep_geometry(m, &rpw, &grid);
    int rc = SCD_OK;
    hipError_t e = launch_halfstep(R, dt, m, n, rpw, grid, 1, tbits, nullptr, nullptr, u, st);
    if (e == hipSuccess && sbits) e = launch_pack(u, SCD_F64, m, sbits, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        rc = SCD_EHIP;
    }
    if (utmp) (void)hipFree(utmp);
    return rc;
}

// The three launches of a column half step on caller data: per-workgroup partial column sums, their
// fixed-order join (v, t, partial sums of |v|), the sum of those.  `partials` holds grid * n elements of dt,
// `cparts` ceil(n/64) doubles.
static hipError_t enqueue_col_signed_sum(const void* R, scd_dtype dt, int64_t m, int64_t n, int rpw, int grid,
                                         const uint64_t* sbits, void* partials, double* cparts, double* v, uint64_t* tbits,
                                         double* cout, hipStream_t st)
{
    hipError_t e = launch_halfstep(R, dt, m, n, rpw, grid, 0, nullptr, sbits, partials, nullptr, st);
    if (e == hipSuccess) e = launch_reduce_plain(partials, dt, grid, n, v, tbits, cparts, st);
    if (e == hipSuccess) e = launch_sum_parts(cparts, (int)words_for(n), cout, st);
    return e;
}

int scd_col_signed_sum(const void* R, scd_dtype dt, int64_t m, int64_t n, const uint64_t* sbits, void* stream, double* v,
                       uint64_t* tbits, double* cout)
{
    if (!R || !sbits || !dtype_ok(dt) || m < 1 || n < 1) return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    int rpw, grid;
    halfstep_geometry(m, &rpw, &grid);
    const size_t es = dt == SCD_F32 ? 4 : 8;
    const int ncp = (int)words_for(n);
    void* partials = nullptr;
    double* cparts = nullptr;
    double* ctmp = nullptr;
    int rc = SCD_OK;
    hipError_t e = hipMalloc(&partials, (size_t)grid * (size_t)n * es);
    if (e == hipSuccess) e = hipMalloc((void**)&cparts, (size_t)ncp * 8);
    if (e == hipSuccess && !cout) e = hipMalloc((void**)&ctmp, 8);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        rc = SCD_ENOMEM;
    } else {
        e = enqueue_col_signed_sum(R, dt, m, n, rpw, grid, sbits, partials, cparts, v, tbits, cout ? cout : ctmp, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) {
            g_last_hip = (int)e;
            (void)hipGetLastError();
            rc = SCD_EHIP;
        }
    }
    if (partials) (void)hipFree(partials);
    if (cparts) (void)hipFree(cparts);
    if (ctmp) (void)hipFree(ctmp);
    return rc;
}

// ---------------------------------------------------------------------------------------------- no allocation

// Work space of scd_col_signed_sum_noalloc: one array per device, part of the code object, held until the
// process ends.  Host code never uses the array's name as an address (it is a host-side stand-in): the
// device address is asked for once per device with hipGetSymbolAddress and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[SCD_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call on that device).
int scratch_address(unsigned char** out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return SCD_ENODEVICE;
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return SCD_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = (unsigned char*)g_scratch_ptr[dev];
    return SCD_OK;
}
}  // namespace

int scd_col_signed_sum_noalloc(const void* R, scd_dtype dt, int64_t m, int64_t n, const uint64_t* sbits, void* stream,
                               double* v, uint64_t* tbits, double* cout)
{
    if (!R || !sbits || !dtype_ok(dt) || m < 1 || n < 1) return SCD_EINVAL;
    int rpw, grid;
    halfstep_geometry(m, &rpw, &grid);
    const size_t es = dt == SCD_F32 ? 4 : 8;
    // layout: [0, 256) the cut value when the caller does not want it; then ceil(n/64) doubles of partial
    // sums of |v|, padded to 256 bytes; then grid * n partial column sums
    const size_t cparts_bytes = (((size_t)words_for(n) * 8 + 255) / 256) * 256;
    const size_t need = 256 + cparts_bytes + (size_t)grid * (size_t)n * es;
    if ((double)grid * (double)n * (double)es > (double)SCD_NOALLOC_SCRATCH_BYTES || need > (size_t)SCD_NOALLOC_SCRATCH_BYTES)
        return SCD_ETOOBIG;
    unsigned char* base = nullptr;
    SCD_TRY(scratch_address(&base));
    double* ctmp = (double*)base;
    double* cparts = (double*)(base + 256);
    void* partials = base + 256 + cparts_bytes;
    // every word of the work space that is read was written by this call: nothing to clear
    HIP_TRY(enqueue_col_signed_sum(R, dt, m, n, rpw, grid, sbits, partials, cparts, v, tbits, cout ? cout : ctmp,
                                   (hipStream_t)stream));
    return SCD_OK;
}

// ---------------------------------------------------------------------------------------------- expand, bitsets

int scd_expand(const uint64_t* const* signs, const void* cvec, scd_dtype dt, int order, const int64_t* dims, int64_t w,
               void* stream, void* out)
{
    int64_t total = 0;
    if (!signs || !out || !dtype_ok(dt) || w < 0 || (w > 0 && !cvec)) return SCD_EINVAL;
    SCD_TRY(check_dims(order, dims, &total));
    for (int i = 0; i < order; ++i)
        if (w > 0 && !signs[i]) return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const int64_t m = dims[0], cols = total / dims[0];
    uint64_t* kr = nullptr;
    const uint64_t* T = signs[1];
    if (order >= 3 && w > 0) {
        hipError_t e = hipMalloc((void**)&kr, (size_t)w * (size_t)words_for(cols) * 8);
        if (e != hipSuccess) {
            g_last_hip = (int)e;
            (void)hipGetLastError();
            return SCD_ENOMEM;
        }
        e = launch_kron_terms(order, dims, signs, w, kr, cols, st);
        if (e != hipSuccess) {
            g_last_hip = (int)e;
            (void)hipGetLastError();
            (void)hipFree(kr);
            return SCD_EHIP;
        }
        T = kr;
    }
    hipError_t e = launch_expand(signs[0], T, cvec, dt, m, cols, w, out, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (kr) (void)hipFree(kr);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        return SCD_EHIP;
    }
    return SCD_OK;
}

// ---------------------------------------------------------------------------------------------- mode sums on caller data

namespace {

// One mode step of Algorithm 12 on a tensor given as plain data (the half-step kernels, no context):
// u = x x_i (tensor product of the other modes' current sign vectors).  Mode i sees the tensor as
// (leading modes) x n_i x inner_i, last mode fastest.  The leading modes are contracted one at a time:
// W_1 = signed column sums of the tensor (n_0 rows) with s^(0), W_i = signed column sums of W_{i-1}
// (n_{i-1} rows, small) with s^(i-1) -- valid because a sweep visits the modes in order -- then a signed
// row sum over the trailing modes (sign vector = Kronecker product of their bitsets).  Only modes 0 and 1
// pass over the tensor itself.
struct ModeSums {
    int order = 0;
    int64_t dims[SCD_MAX_ORDER] = {0}, inner[SCD_MAX_ORDER] = {0}, nwords[SCD_MAX_ORDER] = {0};
    int64_t max_dim = 1, max_words = 1;
    double *uA = nullptr, *W[2] = {nullptr, nullptr}, *cparts = nullptr;
    void* partials = nullptr;
    uint64_t* kr_in = nullptr;
    uint64_t* cur[SCD_MAX_ORDER] = {nullptr};  // current sign vector of every mode
    std::vector<void*> bufs;

    bool alloc(void** p, size_t bytes)
    {
        if (hipMalloc(p, bytes ? bytes : 8) != hipSuccess) {
            (void)hipGetLastError();
            *p = nullptr;
            return false;
        }
        bufs.push_back(*p);
        return true;
    }
    bool init(int ord, const int64_t* d)
    {
        order = ord;
        int64_t max_w = 1, max_kron = 1, max_part = 1;
        for (int i = 0; i < order; ++i) {
            dims[i] = d[i];
            inner[i] = 1;
            for (int q = i + 1; q < order; ++q) inner[i] *= d[q];
            nwords[i] = words_for(d[i]);
            if (d[i] > max_dim) max_dim = d[i];
            if (nwords[i] > max_words) max_words = nwords[i];
            if (i > 0) {
                const int64_t wcols = d[i] * inner[i];
                if (wcols > max_w) max_w = wcols;
                int rpw, grid;
                halfstep_geometry(d[i - 1], &rpw, &grid);
                if ((int64_t)grid * wcols > max_part) max_part = (int64_t)grid * wcols;
            }
            if (inner[i] > max_kron) max_kron = inner[i];
        }
        bool ok = alloc((void**)&uA, (size_t)max_dim * 8) && alloc((void**)&W[0], (size_t)max_w * 8) &&
                  alloc((void**)&W[1], (size_t)max_w * 8) && alloc((void**)&cparts, (size_t)words_for(max_w) * 8) &&
                  alloc(&partials, (size_t)max_part * 8) && alloc((void**)&kr_in, (size_t)words_for(max_kron) * 8);
        for (int i = 0; ok && i < order; ++i) ok = alloc((void**)&cur[i], (size_t)nwords[i] * 8);
        return ok;
    }
    void release()
    {
        for (void* p : bufs) (void)hipFree(p);
        bufs.clear();
    }
    // uA <- x x_i (others), x of dtype dt
    hipError_t part(const void* x, scd_dtype dt, int i, hipStream_t st)
    {
        hipError_t err = hipSuccess;
        const void* src = x;
        scd_dtype sdt = dt;
        const bool leading = i > 0, trailing = i < order - 1;  // modes before / after mode i (even of size 1: a sign)
        if (leading) {
            const int64_t rows = dims[i - 1];
            const int64_t wcols = dims[i] * inner[i];
            const void* from = i == 1 ? x : (const void*)W[(i - 1) & 1];
            const scd_dtype fdt = i == 1 ? dt : SCD_F64;
            double* to = trailing ? W[i & 1] : uA;
            int rpw, grid;
            halfstep_geometry(rows, &rpw, &grid);
            err = launch_halfstep(from, fdt, rows, wcols, rpw, grid, 0, nullptr, cur[i - 1], partials, nullptr, st);
            if (err != hipSuccess) return err;
            err = launch_reduce_plain(partials, fdt, grid, wcols, to, nullptr, cparts, st);
            if (err != hipSuccess) return err;
            src = to;
            sdt = SCD_F64;
        }
        if (trailing) {
            const uint64_t* tau = cur[order - 1];
            if (i < order - 2) {
                err = launch_lsq_kron(cur, dims, i + 1, order, inner[i], kr_in, st);
                if (err != hipSuccess) return err;
                tau = kr_in;
            }
            int rpw, grid;
            halfstep_geometry(dims[i], &rpw, &grid);
            err = launch_halfstep(src, sdt, dims[i], inner[i], rpw, grid, 1, tau, nullptr, nullptr, uA, st);
        }
        return err;
    }
};

int check_tensor_args(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, int32_t max_iters,
                      const double* fro_trace, int64_t* total)
{
    if (!A || !dtype_ok(dt) || w < 0 || max_iters < 1 || !fro_trace) return SCD_EINVAL;
    SCD_TRY(check_dims(order, dims, total));
    for (int i = 0; i < order; ++i)
        if (dims[i] > (1ll << 31)) return SCD_EINVAL;
    return SCD_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------- Algorithms 6 and 14

int scd_lsq_decompose_tensor(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, uint64_t seed,
                             int32_t max_iters, void* stream, uint64_t* const* signs, void* cvec, double* fro_trace,
                             int32_t* iters)
{
    int64_t total = 0;
    SCD_TRY(check_tensor_args(A, dt, order, dims, w, max_iters, fro_trace, &total));
    if (w > SCD_LSQ_MAX_WIDTH || (w > 0 && (!signs || !cvec))) return SCD_EINVAL;
    for (int i = 0; i < order; ++i)
        if (w > 0 && !signs[i]) return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const int64_t wl = w > 0 ? w : 1;
    const int nsq = 256;
    ModeSums ms;
    double* host = nullptr;  // pinned: [0] cut value, [1] b of the current term, [2] upload slot, [3] status
    int rc = SCD_OK;
    double *e = nullptr, *D = nullptr, *g = nullptr, *absp = nullptr, *dotp = nullptr;
    double *scal = nullptr, *L = nullptr, *yv = nullptr, *c = nullptr, *work = nullptr, *bvec = nullptr, *sq = nullptr;
    int* status = nullptr;
    std::vector<int32_t> it_host((size_t)wl, 0);
    bool ok = ms.init(order, dims);
    ok = ok && ms.alloc((void**)&e, (size_t)wl * 8) && ms.alloc((void**)&D, (size_t)order * wl * 8) &&
         ms.alloc((void**)&g, (size_t)wl * 8) && ms.alloc((void**)&absp, (size_t)ms.max_words * 8) &&
         ms.alloc((void**)&dotp, (size_t)ms.max_words * 8) && ms.alloc((void**)&scal, 16) &&
         ms.alloc((void**)&L, (size_t)wl * wl * 8) && ms.alloc((void**)&yv, (size_t)wl * 8) && ms.alloc((void**)&c, (size_t)wl * 8) &&
         ms.alloc((void**)&work, (size_t)wl * 8) && ms.alloc((void**)&bvec, (size_t)wl * 8) &&
         ms.alloc((void**)&sq, (size_t)nsq * 8) && ms.alloc((void**)&status, 4);
    if (ok && hipHostMalloc((void**)&host, 4 * sizeof(double), hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        host = nullptr;
        ok = false;
    }
    auto cleanup = [&](int code) {
        (void)hipStreamSynchronize(st);
        ms.release();
        if (host) (void)hipHostFree(host);
        (void)hipGetLastError();
        return code;
    };
    if (!ok) return cleanup(SCD_ENOMEM);
#define LQ(expr)                              \
    do {                                      \
        hipError_t _e = (expr);               \
        if (_e != hipSuccess) {               \
            g_last_hip = (int)_e;             \
            (void)hipGetLastError();          \
            return cleanup(SCD_EHIP);         \
        }                                     \
    } while (0)

    LQ(hipMemsetAsync(status, 0, 4, st));
    // ||a||^2
    LQ(launch_lsq_sumsq(A, dt, total, sq, nsq, st));
    LQ(launch_lsq_sum2(sq, nullptr, nsq, scal, st));
    LQ(hipMemcpyAsync(host, scal, 16, hipMemcpyDeviceToHost, st));
    LQ(hipStreamSynchronize(st));
    const double fro0sq = host[0];
    if (!isfinite(fro0sq)) return cleanup(SCD_ENONFINITE);
    host[2] = sqrt(fro0sq);
    LQ(hipMemcpyAsync(fro_trace, host + 2, 8, hipMemcpyHostToDevice, st));
    LQ(hipStreamSynchronize(st));

    for (int64_t k = 0; k < w; ++k) {
        // Algorithm 12 on the implicit remainder a - S_k c_k, from the keyed random start of term k
        for (int i = 1; i < order; ++i) {
            LQ(launch_rng(seed, (uint64_t)k, (uint32_t)i, dims[i], ms.cur[i], st));
            LQ(launch_lsq_dots(signs[i], k, ms.nwords[i], dims[i], ms.cur[i], nullptr, D + (int64_t)i * wl, st));
        }
        double c_prev = -INFINITY, bnew = 0.0;
        int32_t j = 0;
        for (;;) {
            for (int i = 0; i < order; ++i) {
                // s^(i) = sgn(a x_i (others) - sum_j c_j (prod_{m != i} <s_j^(m), s^(m)>) s_j^(i))
                LQ(ms.part(A, dt, i, st));
                LQ(launch_lsq_prod(D, wl, order, i, k, c, e, st));
                const bool last = i == order - 1;
                LQ(launch_lsq_correct(signs[i], k, ms.nwords[i], dims[i], e, ms.uA, ms.cur[i], last ? absp : nullptr,
                                      last ? dotp : nullptr, st));
                LQ(launch_lsq_dots(signs[i], k, ms.nwords[i], dims[i], ms.cur[i], nullptr, D + (int64_t)i * wl, st));
            }
            // after the last mode: the cut value sum |.| and <S_new, a> (Algorithm 12 line 10)
            LQ(launch_lsq_sum2(absp, dotp, ms.nwords[order - 1], scal, st));
            LQ(hipMemcpyAsync(host, scal, 16, hipMemcpyDeviceToHost, st));
            LQ(hipStreamSynchronize(st));
            ++j;
            const double cut = host[0];
            bnew = host[1];
            if (!isfinite(cut)) return cleanup(SCD_ENONFINITE);
            if (cut <= c_prev || j >= max_iters) {
                if (!(cut <= c_prev)) rc = SCD_WMAXITER;
                break;
            }
            c_prev = cut;
        }
        it_host[(size_t)k] = j;
        // append and refit every coefficient
        for (int i = 0; i < order; ++i)
            LQ(hipMemcpyAsync(signs[i] + k * ms.nwords[i], ms.cur[i], (size_t)ms.nwords[i] * 8, hipMemcpyDeviceToDevice, st));
        host[2] = bnew;
        LQ(hipMemcpyAsync(bvec + k, host + 2, 8, hipMemcpyHostToDevice, st));
        LQ(launch_lsq_prod(D, wl, order, -1, k, nullptr, g, st));  // Gram row: product of the per-mode inner products
        LQ(launch_lsq_solve(L, wl, k, g, (double)total, bvec, yv, c, work, fro0sq, fro_trace + k + 1, status, st));
        LQ(hipMemcpyAsync(host + 3, status, 4, hipMemcpyDeviceToHost, st));
        LQ(hipStreamSynchronize(st));  // host[2] is reused by the next term
        if (*(const int*)(host + 3) != 0) return cleanup(SCD_ESINGULAR);
    }
    LQ(launch_lsq_cast(c, w, dt, cvec, st));
    if (iters && w > 0) LQ(hipMemcpyAsync(iters, it_host.data(), (size_t)w * 4, hipMemcpyHostToDevice, st));
    LQ(hipStreamSynchronize(st));
    return cleanup(rc);
}

// ---------------------------------------------------------------------------------------------- real last mode

int scd_decompose_scalars(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, uint64_t seed,
                          int32_t max_iters, void* stream, uint64_t* const* signs, void* cvec, double* fro_trace,
                          int32_t* iters)
{
    int64_t total = 0;
    SCD_TRY(check_tensor_args(A, dt, order, dims, w, max_iters, fro_trace, &total));
    if (w > 0 && (!signs || !cvec)) return SCD_EINVAL;
    for (int i = 0; i + 1 < order; ++i)
        if (w > 0 && !signs[i]) return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = dt == SCD_F32 ? 4 : 8;
    const int64_t q = dims[order - 1], P = total / q;
    if (w > 0 && pstream_supported(dt, order, dims, kSpGrid, nullptr)) {
        // order 3 with a short last mode (images): the sweeps are those of the all-signs variant, so the
        // persistent streaming engine runs them; it forms the real coefficients from the last mode's sums it
        // already has and subtracts them slice by slice
        scd_ctx* c = nullptr;
        int rc = scd_create(&c, A, dt, order, dims, w, seed, stream);
        if (rc < 0) return rc;
        rc = scd_set_max_iters(c, max_iters);
        if (rc >= 0 && c->pstream) {
            hipError_t e = hipMalloc(&c->c_scal, (size_t)w * (size_t)q * es);
            if (e != hipSuccess) {
                g_last_hip = (int)e;
                (void)hipGetLastError();
                c->c_scal = nullptr;
                rc = SCD_ENOMEM;
            }
            int run = rc;
            if (rc >= 0) run = scd_run(c, w);
            if (run >= 0) {
                hipError_t h = hipSuccess;
                for (int i = 0; i + 1 < order && h == hipSuccess; ++i)
                    h = hipMemcpyAsync(signs[i], c->out_signs[i], (size_t)w * words_for(dims[i]) * 8, hipMemcpyDeviceToDevice, st);
                if (h == hipSuccess) h = hipMemcpyAsync(cvec, c->c_scal, (size_t)w * (size_t)q * es, hipMemcpyDeviceToDevice, st);
                if (h == hipSuccess) h = hipMemcpyAsync(fro_trace, c->trace, (size_t)(w + 1) * 8, hipMemcpyDeviceToDevice, st);
                if (h == hipSuccess && iters) h = hipMemcpyAsync(iters, c->iters, (size_t)w * 4, hipMemcpyDeviceToDevice, st);
                if (h == hipSuccess) h = hipStreamSynchronize(st);
                if (h != hipSuccess) {
                    g_last_hip = (int)h;
                    (void)hipGetLastError();
                    run = SCD_EHIP;
                }
            }
            (void)hipStreamSynchronize(st);
            if (c->c_scal) (void)hipFree(c->c_scal);
            c->c_scal = nullptr;
            scd_destroy(c);
            return run;
        }
        scd_destroy(c);
        if (rc < 0) return rc;
    }
    const int nsq = 256;
    ModeSums ms;
    double* host = nullptr;  // pinned: [0], [1] sums read back, [2] upload slot
    int rc = SCD_OK;
    void* R = nullptr;
    double *absp = nullptr, *dotp = nullptr, *scal = nullptr, *sq = nullptr;
    uint64_t* lead = nullptr;
    std::vector<int32_t> it_host((size_t)(w > 0 ? w : 1), 0);
    bool ok = ms.init(order, dims);
    ok = ok && ms.alloc(&R, (size_t)total * es) && ms.alloc((void**)&absp, (size_t)ms.max_words * 8) &&
         ms.alloc((void**)&dotp, (size_t)ms.max_words * 8) && ms.alloc((void**)&scal, 16) &&
         ms.alloc((void**)&sq, (size_t)nsq * 8) && ms.alloc((void**)&lead, (size_t)words_for(P) * 8);
    if (ok && hipHostMalloc((void**)&host, 4 * sizeof(double), hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        host = nullptr;
        ok = false;
    }
    auto cleanup = [&](int code) {
        (void)hipStreamSynchronize(st);
        ms.release();
        if (host) (void)hipHostFree(host);
        (void)hipGetLastError();
        return code;
    };
    if (!ok) return cleanup(SCD_ENOMEM);
    LQ(hipMemcpyAsync(R, A, (size_t)total * es, hipMemcpyDeviceToDevice, st));
    LQ(launch_lsq_sumsq(R, dt, total, sq, nsq, st));
    LQ(launch_lsq_sum2(sq, nullptr, nsq, scal, st));
    LQ(hipMemcpyAsync(host, scal, 16, hipMemcpyDeviceToHost, st));
    LQ(hipStreamSynchronize(st));
    if (!isfinite(host[0])) return cleanup(SCD_ENONFINITE);
    host[2] = sqrt(host[0]);
    LQ(hipMemcpyAsync(fro_trace, host + 2, 8, hipMemcpyHostToDevice, st));
    LQ(hipStreamSynchronize(st));

    for (int64_t k = 0; k < w; ++k) {
        // Algorithm 12 on the remainder, all modes signs, from the keyed random start of term k
        for (int i = 1; i < order; ++i) LQ(launch_rng(seed, (uint64_t)k, (uint32_t)i, dims[i], ms.cur[i], st));
        double c_prev = -INFINITY;
        int32_t j = 0;
        for (;;) {
            for (int i = 0; i < order; ++i) {
                LQ(ms.part(R, dt, i, st));
                const bool last = i == order - 1;
                LQ(launch_lsq_correct(nullptr, 0, ms.nwords[i], dims[i], nullptr, ms.uA, ms.cur[i], last ? absp : nullptr,
                                      last ? dotp : nullptr, st));
            }
            LQ(launch_lsq_sum2(absp, dotp, ms.nwords[order - 1], scal, st));
            LQ(hipMemcpyAsync(host, scal, 16, hipMemcpyDeviceToHost, st));
            LQ(hipStreamSynchronize(st));
            ++j;
            const double cut = host[0];
            if (!isfinite(cut)) return cleanup(SCD_ENONFINITE);
            if (cut <= c_prev || j >= max_iters) {
                if (!(cut <= c_prev)) rc = SCD_WMAXITER;
                break;
            }
            c_prev = cut;
        }
        it_host[(size_t)k] = j;
        // ms.uA holds r x (leading modes' sign vectors), one value per slice of the last mode: the real
        // coefficients are that over P; they are stored in dt and the stored values are what is subtracted
        void* ck = (char*)cvec + (size_t)k * (size_t)q * es;
        LQ(launch_scalars_coef(ms.uA, q, (double)P, dt, ck, st));
        for (int i = 0; i + 1 < order; ++i)
            LQ(hipMemcpyAsync(signs[i] + k * ms.nwords[i], ms.cur[i], (size_t)ms.nwords[i] * 8, hipMemcpyDeviceToDevice, st));
        const uint64_t* lead_bits = ms.cur[0];
        if (order > 2) {
            LQ(launch_lsq_kron(ms.cur, dims, 0, order - 1, P, lead, st));
            lead_bits = lead;
        }
        LQ(launch_scalars_update(R, dt, total, q, lead_bits, ck, sq, nsq, st));
        LQ(launch_lsq_sum2(sq, nullptr, nsq, scal, st));
        LQ(hipMemcpyAsync(host, scal, 16, hipMemcpyDeviceToHost, st));
        LQ(hipStreamSynchronize(st));
        host[2] = sqrt(host[0]);
        LQ(hipMemcpyAsync(fro_trace + k + 1, host + 2, 8, hipMemcpyHostToDevice, st));
        LQ(hipStreamSynchronize(st));
    }
    if (iters && w > 0) LQ(hipMemcpyAsync(iters, it_host.data(), (size_t)w * 4, hipMemcpyHostToDevice, st));
    LQ(hipStreamSynchronize(st));
#undef LQ
    return cleanup(rc);
}

int scd_lsq_decompose(const void* A, scd_dtype dt, int64_t m, int64_t n, int64_t w, uint64_t seed, int32_t max_iters,
                      void* stream, uint64_t* S, uint64_t* T, void* cvec, double* fro_trace, int32_t* iters)
{
    const int64_t dims[2] = {m, n};
    uint64_t* const signs[2] = {S, T};
    return scd_lsq_decompose_tensor(A, dt, 2, dims, w, seed, max_iters, stream, signs, cvec, fro_trace, iters);
}

size_t scd_apply_workspace_bytes(int64_t m, int64_t n, int64_t w)
{
    if (m < 0 || n < 0 || w < 0) return 0;
    // either direction: the larger of the two layouts
    ApplyPlan a, b;
    apply_plan(n, m, w, &a);
    apply_plan(m, n, w, &b);
    return a.bytes > b.bytes ? a.bytes : b.bytes;
}

int scd_apply(const uint64_t* S, const uint64_t* T, const void* c, scd_dtype dt, int64_t m, int64_t n, int64_t w,
              int transpose, const void* x, int64_t nvec, void* y, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!dtype_ok(dt) || m < 0 || n < 0 || w < 0 || nvec < 0) return SCD_EINVAL;
    if (m > (1ll << 31) || n > (1ll << 31)) return SCD_EINVAL;
    const int64_t nin = transpose ? m : n, nout = transpose ? n : m;
    if (nvec == 0 || nout == 0) return SCD_OK;
    if (!y || !workspace || ((uintptr_t)workspace & 7u)) return SCD_EINVAL;
    if (w > 0 && nin > 0 && (!S || !T || !c || !x)) return SCD_EINVAL;
    ApplyPlan pl;
    apply_plan(nin, nout, w, &pl);
    if (workspace_bytes < pl.bytes) return SCD_EINVAL;
    const size_t es = dt == SCD_F32 ? 4 : 8;
    hipStream_t st = (hipStream_t)stream;
    for (int64_t v = 0; v < nvec; ++v) {
        HIP_TRY(launch_apply(transpose ? S : T, transpose ? T : S, c, dt, nin, nout, w,
                             x ? (const char*)x + (size_t)v * (size_t)nin * es : nullptr,
                             (char*)y + (size_t)v * (size_t)nout * es, workspace, st));
    }
    HIP_TRY(hipStreamSynchronize(st));
    return SCD_OK;
}

int scd_pack(const void* values, scd_dtype dt, int64_t n, void* stream, uint64_t* bits)
{
    if (!values || !bits || !dtype_ok(dt) || n < 0) return SCD_EINVAL;
    if (n == 0) return SCD_OK;
    HIP_TRY(launch_pack(values, dt, n, bits, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return SCD_OK;
}

int scd_unpack(const uint64_t* bits, int64_t n, scd_dtype dt, void* stream, void* values)
{
    if (!values || !bits || !dtype_ok(dt) || n < 0) return SCD_EINVAL;
    if (n == 0) return SCD_OK;
    HIP_TRY(launch_unpack(bits, n, dt, values, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return SCD_OK;
}

int scd_rng_signs(uint64_t seed, uint64_t term, uint32_t mode, int64_t n, void* stream, uint64_t* bits)
{
    if (!bits || n < 0) return SCD_EINVAL;
    if (n == 0) return SCD_OK;
    HIP_TRY(launch_rng(seed, term, mode, n, bits, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    return SCD_OK;
}

// ---------------------------------------------------------------------------------------------- probes

int scd_probe_stream(const void* src, void* dst, int64_t bytes, int grid, int reps, void* stream, double* seconds)
{
    if (!src || bytes < 16 || (bytes % 16) || grid < 1 || reps < 1 || !seconds) return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    float* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = SCD_OK;
    hipError_t e = hipMalloc((void**)&sink, 4);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    // one untimed launch, then `reps` timed ones
    for (int r = -1; r < reps && e == hipSuccess; ++r) {
        if (r == 0) e = hipEventRecord(e0, st);
        if (e != hipSuccess) break;
        e = dst ? launch_stream_copy(src, dst, bytes, grid, st) : launch_stream_read(src, bytes, grid, sink, st);
    }
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        rc = SCD_EHIP;
    } else {
        *seconds = (double)ms * 1e-3 / reps;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return rc;
}

int scd_probe_exchange(int which, int grid, int group, int rounds, void* stream, double* seconds_per_round)
{
    if (which < 0 || which > 1 || grid < 1 || grid > 1024 || (group & 0xFFFF) < 1 || grid % (group & 0xFFFF) || rounds < 1 ||
        !seconds_per_round)
        return SCD_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    uint64_t* buf = nullptr;
    unsigned* flags = nullptr;  // [0] counter, [1] error
    float* out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    const size_t bufbytes = (size_t)2 * grid * 256 * 8;
    hipError_t e = hipMalloc((void**)&buf, bufbytes);
    if (e == hipSuccess) e = hipMalloc((void**)&flags, 8);
    if (e == hipSuccess) e = hipMalloc((void**)&out, (size_t)grid * 4);
    if (e == hipSuccess) e = hipMemsetAsync(buf, 0, bufbytes, st);
    if (e == hipSuccess) e = hipMemsetAsync(flags, 0, 8, st);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    if (e == hipSuccess) e = hipEventRecord(e0, st);
    if (e == hipSuccess) e = launch_exchange_probe(which, grid, buf, flags, rounds, group, 1 << 20, flags + 1, out, st);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    unsigned err[2] = {0, 0};
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) e = hipMemcpy(err, flags, 8, hipMemcpyDeviceToHost);
    int rc = SCD_OK;
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        (void)hipGetLastError();
        rc = SCD_EHIP;
    } else if (err[1]) {
        rc = SCD_EINVAL;  // a bounded wait ran out: the workgroups were not all resident
    } else {
        *seconds_per_round = (double)ms * 1e-3 / rounds;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    if (flags) (void)hipFree(flags);
    if (out) (void)hipFree(out);
    return rc;
}

const char* scd_strerror(int code)
{
    switch (code) {
        case SCD_OK: return "ok";
        case SCD_WMAXITER: return "warning: a term stopped on the iteration cap";
        case SCD_EINVAL: return "invalid argument";
        case SCD_ENOMEM: return "out of memory";
        case SCD_EHIP: return "HIP runtime error";
        case SCD_EFULL: return "context is at its width capacity";
        case SCD_ENONFINITE: return "input holds NaN or Inf";
        case SCD_ENODEVICE: return "no HIP device";
        case SCD_ETIMEOUT: return "a bounded device-side wait ran out; give the context a remainder again or destroy it";
        case SCD_ESINGULAR: return "a new term lies in the span of the earlier ones: normal equations singular";
        case SCD_ETOOBIG: return "the input needs more work space than the call's fixed work space holds";
        default: return "unknown status";
    }
}

int scd_last_hip_error(void) { return g_last_hip; }

}  // extern "C"

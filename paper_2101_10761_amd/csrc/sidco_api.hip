// C ABI of the SIDCo library: argument checks, stage schedule, workspace, kernel sequencing.
// Declarations and their contracts are in include/sidco.h.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "sidco_internal.h"

namespace sidco {
namespace {

constexpr int kMaxDevices = 16;
constexpr int kMaxKernels = SIDCO_MAX_STAGES + 2;
constexpr size_t kAlign = 256;
constexpr uint32_t kFinalLists = 32;  // source lists per block of the last stage's kernel for short lists

// Fixed-size head of the workspace; the two survivor-list buffers follow it.
struct WorkspaceHead {
    DevState st;
    alignas(256) double part[2][4 * kMaxBlocks];
    alignas(256) uint32_t cnt[2][kMaxWaves];
    alignas(256) uint32_t blk[2][kMaxBlocks];
    alignas(256) uint32_t topk_hist[3 * kTopkBins];
    alignas(256) TopkState topk;
    alignas(256) uint32_t dgc_hist[2][3 * kTopkBins];
    alignas(256) DgcState dgc;
    alignas(256) BatchTable batch;  // at a fixed place, so that single calls in between leave it alone
};

constexpr size_t head_bytes() { return (sizeof(WorkspaceHead) + kAlign - 1) / kAlign * kAlign; }

size_t seg_bytes(int64_t d)
{
    const size_t ntiles = (size_t)((d + kTile - 1) / kTile);
    return ntiles * kTile * sizeof(int2);  // one slot per element: no list can overflow
}

// One workspace and the host's record of the calls made with it.  Library-owned workspaces are per
// (device, stream): calls on different streams of a device use different ones and may overlap.
struct WsCtx {
    void* key = nullptr;       // stream that a library-owned workspace serves
    void* ws = nullptr;        // workspace in use
    size_t ws_bytes = 0;
    bool ws_owned = false;
    hipEvent_t ev[kMaxKernels + 1] = {};
    bool ev_made = false;
    int prof_n = 0;            // kernels of the last profiled call
    const char* prof_name[kMaxKernels] = {};
    int64_t dgc_n_s = 0, dgc_k_s = 0;  // sizes of the last sidco_dgc call
    bool bad_cleared = false;  // the scatter kernels' bad-index flag has been initialised in this workspace
    int64_t last_cap = 0;      // output capacity of the last compress call
    uint32_t* status_out = nullptr;  // device word that receives the status bits of every call (sidco_set_status_word)
    // shape of the last compress call: a call that repeats it may use the device's record of where the
    // thresholds fell (DevState::theta_seen)
    int64_t sig_d = 0;
    int sig_dist = -1, sig_M = 0;
    double sig_ratios[SIDCO_MAX_STAGES] = {};
    double sig_theta = -1.0;
    // batched calls: host images of the tables uploaded so far (descriptors and block maps; kept alive
    // because their upload is asynchronous), which of them the device holds, the shared arguments it was
    // used with, and the output capacities for the diagnostics
    std::vector<std::vector<unsigned char>*> batch_images;
    int batch_cur = -1;
    double batch_delta = -1.0, batch_theta = -1.0;
    int batch_dist = -1, batch_M = 0, batch_n = 0;
    std::vector<int64_t> batch_cap;
    uint32_t fit_nblocks = 0;  // grid, length and law of the last sidco_fit call
    int64_t fit_d = 0;
    int fit_dist = 0;

    // the workspace memory has changed: nothing is known about its contents
    void forget()
    {
        sig_d = 0;
        bad_cleared = false;
        dgc_n_s = 0;
        batch_cur = -1;
        fit_nblocks = 0;
    }
};

// Scratch of sidco_compress_static: the workspace of a call (device state, partial sums, list lengths and
// the two survivor-list buffers) for vectors of up to kStaticMaxD elements, resident in every GPU the
// library runs on from the moment its code is loaded until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress: the device address is looked up once per device (static_ws)
// and that pointer is what kernels and copies get.
constexpr int64_t kStaticMaxD = 2097152;
constexpr size_t kStaticBytes =
    (sizeof(WorkspaceHead) + kAlign - 1) / kAlign * kAlign + 2 * (size_t)kStaticMaxD * sizeof(int2);
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticBytes];

struct DeviceCtx {
    WsCtx stat;                   // the static scratch of this device (sidco_compress_static)
    WsCtx shared;                 // the caller's workspace (sidco_set_workspace): serves every stream when set
    std::vector<WsCtx*> streams;  // library-owned workspaces, one per stream seen
    WsCtx* last_prof = nullptr;   // workspace of the last profiled call
};

std::mutex g_mu;
DeviceCtx g_ctx[kMaxDevices];
bool g_profiling = false;
double g_speculation = kSpeculation;
double g_delta1 = 0.25;               // delta_1 of the default stage schedule (Sec. 4.1)
unsigned long long g_next_owner = 1;  // ids of the stage controllers
thread_local char g_hip_msg[256] = "";

int hip_fail(hipError_t e, const char* what)
{
    snprintf(g_hip_msg, sizeof(g_hip_msg), "%s: %s", what, hipGetErrorString(e));
    return SIDCO_ERR_HIP;
}

double default_delta1()
{
    std::lock_guard<std::mutex> lock(g_mu);
    return g_delta1;
}

int grad_type(int grad_dtype)
{
    return grad_dtype == SIDCO_GRAD_F16 ? kGradF16 : (grad_dtype == SIDCO_GRAD_BF16 ? kGradBf16 : kGradF32);
}

bool aligned4(const void* p) { return ((uintptr_t)p & 3u) == 0; }
bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// `grad_align`: alignment the gradient's element type needs (4 for fp32, 2 for the 16-bit types)
int check_common(const void* grad, const float* residual, int64_t d, int dist, const int32_t* out_idx,
                 const float* out_val, const int32_t* out_count, const float* out_eta, uintptr_t grad_align = 4)
{
    if (!grad || !out_idx || !out_val || !out_count || !out_eta) return SIDCO_ERR_NULL;
    if (d < 1 || d > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    if (dist != SIDCO_DIST_EXP && dist != SIDCO_DIST_GAMMA_GPD && dist != SIDCO_DIST_GPD) return SIDCO_ERR_DIST;
    if (((uintptr_t)grad & (grad_align - 1)) != 0 || !aligned4(residual) || !aligned4(out_idx) || !aligned4(out_val) ||
        !aligned4(out_count) || !aligned4(out_eta))
        return SIDCO_ERR_ALIGN;
    if (residual && (const void*)residual == grad) return SIDCO_ERR_ARG;
    return SIDCO_OK;
}

// Makes sure the current device has a workspace of at least `need` bytes.
int ensure_workspace(WsCtx& c, size_t need)
{
    if (c.ws && c.ws_bytes >= need) return SIDCO_OK;
    if (c.ws && !c.ws_owned) return SIDCO_ERR_WORKSPACE;  // caller-provided and too small
    if (c.ws) {
        hipError_t e = hipFree(c.ws);  // waits for work that still uses it
        c.ws = nullptr;
        c.ws_bytes = 0;
        if (e != hipSuccess) return hip_fail(e, "hipFree(workspace)");
    }
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, need);
    if (e != hipSuccess) return hip_fail(e, "hipMalloc(workspace)");
    c.ws = p;
    c.ws_bytes = need;
    c.ws_owned = true;
    c.forget();  // a fresh workspace holds no record of an earlier call
    return SIDCO_OK;
}

// Fills the launch geometry and buffer pointers that every kernel of a call shares.
// `acc_scratch`: fp32 buffer of the workspace that receives acc when the gradient is 16-bit and there is no residual.
void fill_common(Params& p, WorkspaceHead* h, const void* grad, float* residual, int64_t d, int dist,
                 int gt = kGradF32, float* acc_scratch = nullptr)
{
    memset(&p, 0, sizeof(p));
    p.grad = grad;
    p.gt = gt;
    p.residual = residual;
    p.acc_w = residual ? residual : (gt != kGradF32 ? acc_scratch : nullptr);
    p.acc = p.acc_w ? p.acc_w : (const float*)grad;
    p.d = d;
    p.ntiles = (uint32_t)((d + kTile - 1) / kTile);
    p.nfull = (uint32_t)(d / kTile);
    p.nwaves = p.ntiles < (uint32_t)kMaxWaves ? p.ntiles : (uint32_t)kMaxWaves;
    p.nblocks = (p.nwaves + kWavesPerBlock - 1) / kWavesPerBlock;
    p.vec_ok = (gt == kGradF32 ? aligned16(grad) : ((uintptr_t)grad & 7u) == 0) && aligned16(residual);
    p.dist = dist;
    p.st = &h->st;
}

int current_device(DeviceCtx** c)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return SIDCO_ERR_ARG;
    *c = &g_ctx[dev];
    return SIDCO_OK;
}

// The workspace that serves `stream` on the current device: the caller's if one is set, else the
// library's own for that stream (created empty on first use if `create`).  Caller holds g_mu.
int pick_ws(void* stream, bool create, WsCtx** out, DeviceCtx** dev_out = nullptr)
{
    DeviceCtx* d = nullptr;
    int rc = current_device(&d);
    if (rc != SIDCO_OK) return rc;
    if (dev_out) *dev_out = d;
    if (d->shared.ws) {
        *out = &d->shared;
        return SIDCO_OK;
    }
    for (WsCtx* w : d->streams) {
        if (w->key == stream) {
            *out = w;
            return SIDCO_OK;
        }
    }
    if (!create) return SIDCO_ERR_WORKSPACE;
    WsCtx* w = new (std::nothrow) WsCtx;
    if (!w) return SIDCO_ERR_ARG;
    w->key = stream;
    d->streams.push_back(w);
    *out = w;
    return SIDCO_OK;
}

// The static scratch of the current device as a workspace; its address is looked up on first use.
// Caller holds g_mu.  No allocation of any kind.
int static_ws(WsCtx** out)
{
    DeviceCtx* d = nullptr;
    int rc = current_device(&d);
    if (rc != SIDCO_OK) return rc;
    if (!d->stat.ws) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr || ((uintptr_t)ptr % kAlign) != 0) return SIDCO_ERR_WORKSPACE;
        d->stat.ws = ptr;
        d->stat.ws_bytes = kStaticBytes;
        d->stat.ws_owned = false;
    }
    *out = &d->stat;
    return SIDCO_OK;
}

void free_ws(WsCtx& c)
{
    if (c.ws && c.ws_owned) (void)hipFree(c.ws);
    if (c.ev_made)
        for (int i = 0; i <= kMaxKernels; ++i) (void)hipEventDestroy(c.ev[i]);
    for (auto* img : c.batch_images) delete img;
    c = WsCtx();
}

// Grid of the last stage's kernel when it reads survivor lists.  The host only knows the expected
// number of entries; a wrong guess costs time, never correctness.  Every block reserves its output
// range with one same-address atomic, so few blocks for short lists (4 lists per wave, everything loaded
// before the prologue) and one list per wave for long ones (millions of pairs out: 1057 us against 1152 us per
// call with 512 instead of 256 blocks at d = 138 M, delta = 0.1, where the kernel is bound by the scattered
// stores that clear the residual; no difference at delta = 0.01 and below).
uint32_t final_grid(const Params& p, double expect)
{
    uint32_t grid = (p.nwaves + kFinalLists - 1) / kFinalLists;
    if (expect > 4.0e6) grid = p.nblocks;
    if (grid > p.nblocks) grid = p.nblocks;
    if (grid < 1) grid = 1;
    return grid;
}

// Lowest theta a threshold hint may lead to in a dense stage whose source still holds the fraction `cum` of
// the vector: the candidate lists must stay within kMaterializeBelow of the vector.
float hint_floor(double cum, double L_stage, double L_next)
{
    const double t = (log(cum / kMaterializeBelow) - L_stage) / L_next;
    return (float)(t > 0.0 ? t : 0.0);
}

// the host's view of a call's device state
void fill_diag(const DevState& st, int64_t cap, sidco_diag* host_out)
{
    *host_out = st.diag;
    host_out->selected = (int64_t)st.selected_ctr;
    host_out->count = (int32_t)((int64_t)st.selected_ctr < cap ? (int64_t)st.selected_ctr : cap);
    if (st.overflow) host_out->status |= SIDCO_ST_OVERFLOW;
    host_out->reserved = 0;
    const int M = host_out->stages;
    for (int m = (M < 0 ? 0 : M); m < SIDCO_MAX_STAGES; ++m) {  // entries of earlier, longer calls
        host_out->eta[m] = 0.0f;
        host_out->n[m] = 0;
        host_out->stats[m][0] = host_out->stats[m][1] = host_out->stats[m][2] = 0.0;
    }
}

// HIP events of the per-kernel profile, created on first use
int make_events(WsCtx& c)
{
    if (c.ev_made) return SIDCO_OK;
    for (int i = 0; i <= kMaxKernels; ++i) {
        hipError_t e = hipEventCreate(&c.ev[i]);
        if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    }
    c.ev_made = true;
    return SIDCO_OK;
}

size_t acc_bytes(int64_t d) { return seg_bytes(d) / 2; }  // one float per list slot

// `owner`: id of the stage controller that makes the call, 0 for every other caller.
// `use_static`: work in the device's static scratch and allocate nothing (sidco_compress_static).
int run(void* stream, const void* grad, float* residual, int64_t d, int dist, const double* ratios, int M,
        int32_t* out_idx, float* out_val, int64_t out_cap, int32_t* out_count, float* out_eta, bool acc_reset = true,
        int gt = kGradF32, unsigned long long owner = 0, bool use_static = false)
{
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    DeviceCtx* dev = nullptr;
    const size_t seg = seg_bytes(d);
    const bool own_acc = gt != kGradF32 && !residual;  // the widened vector needs a home
    const size_t need = head_bytes() + 2 * seg + (own_acc ? acc_bytes(d) : 0);
    int rc;
    if (use_static) {
        rc = static_ws(&cp);
        if (rc != SIDCO_OK) return rc;
        if (need > cp->ws_bytes) return SIDCO_ERR_SIZE;
    } else {
        rc = pick_ws(stream, true, &cp, &dev);
        if (rc != SIDCO_OK) return rc;
        rc = ensure_workspace(*cp, need);
        if (rc != SIDCO_OK) return rc;
    }
    WsCtx& c = *cp;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;

    WorkspaceHead* h = (WorkspaceHead*)c.ws;
    int2* segbuf[2] = {(int2*)((char*)c.ws + head_bytes()), (int2*)((char*)c.ws + head_bytes() + seg)};

    Params p;
    fill_common(p, h, grad, residual, d, dist, gt, own_acc ? (float*)((char*)c.ws + head_bytes() + 2 * seg) : nullptr);
    p.M = M;
    for (int m = 0; m < M; ++m) p.L[m] = log(1.0 / ratios[m]);
    p.out_idx = out_idx;
    p.out_val = out_val;
    p.out_count = out_count;
    p.out_eta = out_eta;
    p.out_cap = out_cap;
    p.acc_reset = acc_reset ? 1 : 0;
    p.owner = owner;
    p.status_out = c.status_out;
    c.last_cap = out_cap;
    const double theta = g_speculation;
    bool same_shape = c.sig_d == d && c.sig_dist == dist && c.sig_M == M && c.sig_theta == theta;
    for (int m = 0; m < M && same_shape; ++m) same_shape = c.sig_ratios[m] == ratios[m];
    c.sig_d = d;
    c.sig_dist = dist;
    c.sig_M = M;
    c.sig_theta = theta;
    for (int m = 0; m < M; ++m) c.sig_ratios[m] = ratios[m];
    p.use_hint = same_shape ? 1 : 0;
    const bool prof = g_profiling && !use_static;  // the events of a profile are created on first use
    if (prof) {
        rc = make_events(c);
        if (rc != SIDCO_OK) return rc;
        dev->last_prof = &c;
    }
    int k = 0;
    auto mark = [&](const char* name) {
        if (!prof) return;
        if (name) c.prof_name[k - 1] = name;
        (void)hipEventRecord(c.ev[k], s);
    };
    mark(nullptr);

    // stage-1 sums (and acc) -> part[0]
    p.part_out = h->part[0];
    launch_fit(p, (double*)segbuf[1], s);  // the second list buffer is free until the first stage kernel writes it

    ++k;
    mark("k_fit");

    // Stage m: threshold from the previous kernel's sums.  Buffers alternate with the kernel number.
    // `lists` turns true once a stage has written survivor lists (candidates or exceedances).
    bool lists = false;
    double cum = 1.0;      // delta_1 ... delta_{m-1}
    double list_frac = 1;  // expected fraction of the vector in the current lists
    int sel = 0;           // which half of the double buffers the last kernel wrote
    bool reverse = true;   // direction of the next dense pass: k_fit walked forward, so the first one walks back
    bool cand = false;     // the current lists are candidate lists
    auto bind = [&](int m) {
        const int in = sel, out = sel ^ 1;
        p.stage = m;
        p.theta = 0.0f;
        p.prev_cand = cand ? 1 : 0;
        p.part_in = h->part[in];
        p.part_out = h->part[out];
        p.cnt_in = h->cnt[in];
        p.cnt_out = h->cnt[out];
        p.blk_in = h->blk[in];
        p.blk_out = h->blk[out];
        p.seg_in = segbuf[in];
        p.seg_out = segbuf[out];
        sel = out;
    };
    for (int m = 1; m < M; ++m) {
        bind(m);
        if (!lists) {
            // dense source: statistics at eta_m, lists of candidates for stage m+1 (see stage_prologue)
            const double Lw = p.L[m - 1] + theta * p.L[m];
            const double frac = cum * exp(-Lw);
            const bool write = frac <= kMaterializeBelow;
            if (write && theta > 0.0) {
                p.theta = (float)theta;
                p.theta_min = hint_floor(cum, p.L[m - 1], p.L[m]);
            }
            p.reverse = reverse;
            reverse = !reverse;
            launch_compact(p, /*stats=*/true, write, s);
            ++k;
            mark(write ? "k_compact_dense" : "k_scan_dense");
            if (write) {
                lists = true;
                list_frac = frac;
                cand = theta > 0.0;
            }
        } else {
            // one source list per wave: the kernel is a chain of dependent round trips per list, and
            // fewer, longer chains were slower than more blocks (measured: 128 blocks 18 us, 512 blocks 14 us)
            launch_lists(p, p.nblocks, s);
            ++k;
            mark("k_lists");
            list_frac = cum * ratios[m - 1];
            cand = false;
        }
        cum *= ratios[m - 1];
    }
    bind(M);
    if (!lists) {
        p.reverse = reverse;
        launch_compact(p, /*stats=*/false, /*write=*/true, s);
        ++k;
        mark("k_compact_dense");
        p.cnt_in = h->cnt[sel];
        p.blk_in = h->blk[sel];
        p.seg_in = segbuf[sel];
        launch_gather(p, s);
        ++k;
        mark("k_gather");
    } else {
        // few blocks = few reservation atomics
        launch_final_lists(p, final_grid(p, (double)d * list_frac), s);
        ++k;
        mark("k_final_lists");
    }
    c.prof_n = prof ? k : 0;
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return SIDCO_OK;
}

}  // namespace
}  // namespace sidco

using namespace sidco;

extern "C" {

int sidco_stage_ratios(double delta, int stages, double delta1, double* ratios)
{
    if (!ratios) return SIDCO_ERR_NULL;
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    if (stages < 1 || stages > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    if (!(delta1 > 0.0 && delta1 < 1.0)) return SIDCO_ERR_DELTA;
    if (stages == 1 || !(delta1 > delta)) {
        ratios[0] = delta;
        return 1;
    }
    ratios[0] = delta1;
    const double rest = pow(delta / delta1, 1.0 / (double)(stages - 1));
    for (int m = 1; m < stages; ++m) ratios[m] = rest;
    return stages;
}

int64_t sidco_out_capacity(int64_t d, double delta)
{
    if (d < 1 || d > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    const int64_t k = (int64_t)ceil(delta * (double)d);
    const int64_t cap = 4 * k + 4096;
    return cap < d ? cap : d;
}

size_t sidco_workspace_bytes(int64_t d)
{
    if (d < 1 || d > (int64_t)INT32_MAX) return 0;
    return head_bytes() + 2 * seg_bytes(d);
}

int sidco_set_workspace(void* device_ptr, size_t bytes)
{
    if (device_ptr && ((uintptr_t)device_ptr % kAlign) != 0) return SIDCO_ERR_WORKSPACE;
    if (device_ptr && bytes < head_bytes()) return SIDCO_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceCtx* d = nullptr;
    int rc = current_device(&d);
    if (rc != SIDCO_OK) return rc;
    WsCtx& c = d->shared;
    if (d->last_prof == &c) d->last_prof = nullptr;
    free_ws(c);  // events and table images of the previous shared workspace; its memory is the caller's
    c.ws = device_ptr;
    c.ws_bytes = device_ptr ? bytes : 0;
    c.ws_owned = false;
    return SIDCO_OK;
}

int sidco_reserve(void* stream, size_t bytes)
{
    if (bytes < head_bytes()) bytes = head_bytes();
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* c = nullptr;
    int rc = pick_ws(stream, true, &c);
    if (rc != SIDCO_OK) return rc;
    return ensure_workspace(*c, bytes);
}

int sidco_release(void* stream)
{
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceCtx* d = nullptr;
    int rc = current_device(&d);
    if (rc != SIDCO_OK) return rc;
    for (size_t i = 0; i < d->streams.size(); ++i) {
        if (d->streams[i]->key != stream) continue;
        if (d->last_prof == d->streams[i]) d->last_prof = nullptr;
        free_ws(*d->streams[i]);  // hipFree waits for work that still uses the memory
        delete d->streams[i];
        d->streams.erase(d->streams.begin() + (long)i);
        break;
    }
    return SIDCO_OK;
}

int sidco_compress_ex(void* stream, const float* grad, float* residual, int64_t d, int dist, const double* ratios,
                      int n_ratios, int32_t* out_idx, float* out_val, int64_t out_capacity, int32_t* out_count,
                      float* out_eta)
{
    int rc = check_common(grad, residual, d, dist, out_idx, out_val, out_count, out_eta);
    if (rc != SIDCO_OK) return rc;
    if (!ratios) return SIDCO_ERR_NULL;
    if (n_ratios < 1 || n_ratios > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    for (int m = 0; m < n_ratios; ++m)
        if (!(ratios[m] > 0.0 && ratios[m] < 1.0)) return SIDCO_ERR_DELTA;
    if (out_capacity < 1 || out_capacity > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    return run(stream, grad, residual, d, dist, ratios, n_ratios, out_idx, out_val, out_capacity, out_count, out_eta);
}

int sidco_compress(void* stream, const float* grad, float* residual, int64_t d, double delta, int dist, int stages,
                   int32_t* out_idx, float* out_val, int32_t* out_count, float* out_eta)
{
    int rc = check_common(grad, residual, d, dist, out_idx, out_val, out_count, out_eta);
    if (rc != SIDCO_OK) return rc;
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    if (stages < 1 || stages > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    double ratios[SIDCO_MAX_STAGES];
    const int M = sidco_stage_ratios(delta, stages, default_delta1(), ratios);
    if (M < 1) return M;
    return run(stream, grad, residual, d, dist, ratios, M, out_idx, out_val, sidco_out_capacity(d, delta), out_count,
               out_eta);
}

int sidco_compress_static(void* stream, const float* grad, float* residual, int64_t d, double delta, int dist, int stages,
                          int32_t* out_idx, float* out_val, int32_t* out_count, float* out_eta)
{
    int rc = check_common(grad, residual, d, dist, out_idx, out_val, out_count, out_eta);
    if (rc != SIDCO_OK) return rc;
    if (d > kStaticMaxD) {
        snprintf(g_hip_msg, sizeof(g_hip_msg), "sidco_compress_static: d = %lld exceeds the static scratch (%lld elements)",
                 (long long)d, (long long)kStaticMaxD);
        return SIDCO_ERR_SIZE;
    }
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    if (stages < 1 || stages > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    double ratios[SIDCO_MAX_STAGES];
    const int M = sidco_stage_ratios(delta, stages, default_delta1(), ratios);
    if (M < 1) return M;
    return run(stream, grad, residual, d, dist, ratios, M, out_idx, out_val, sidco_out_capacity(d, delta), out_count,
               out_eta, true, kGradF32, 0, true);
}

int64_t sidco_static_max_elements(void) { return kStaticMaxD; }

int sidco_static_init(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* c = nullptr;
    return static_ws(&c);
}

int sidco_compress_typed(void* stream, const void* grad, int grad_dtype, float* residual, int64_t d, double delta,
                         int dist, int stages, int32_t* out_idx, float* out_val, int32_t* out_count, float* out_eta)
{
    if (grad_dtype == SIDCO_GRAD_F32)
        return sidco_compress(stream, (const float*)grad, residual, d, delta, dist, stages, out_idx, out_val, out_count,
                              out_eta);
    if (grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16) return SIDCO_ERR_ARG;
    int rc = check_common(grad, residual, d, dist, out_idx, out_val, out_count, out_eta, 2);
    if (rc != SIDCO_OK) return rc;
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    if (stages < 1 || stages > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    double ratios[SIDCO_MAX_STAGES];
    const int M = sidco_stage_ratios(delta, stages, default_delta1(), ratios);
    if (M < 1) return M;
    return run(stream, grad, residual, d, dist, ratios, M, out_idx, out_val, sidco_out_capacity(d, delta), out_count,
               out_eta, true, grad_dtype == SIDCO_GRAD_F16 ? kGradF16 : kGradBf16);
}

size_t sidco_workspace_bytes_typed(int64_t d, int grad_dtype, int has_residual)
{
    if (d < 1 || d > (int64_t)INT32_MAX) return 0;
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16) return 0;
    const bool own_acc = grad_dtype != SIDCO_GRAD_F32 && !has_residual;
    return head_bytes() + 2 * seg_bytes(d) + (own_acc ? acc_bytes(d) : 0);
}

int sidco_adapt_stages(int stages, double khat_avg, double k, double eps_high, double eps_low, int max_stages)
{
    if (stages < 1 || max_stages < 1 || max_stages > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    if (!(k > 0.0) || !(khat_avg >= 0.0)) return SIDCO_ERR_ARG;
    if (!(eps_high >= 0.0) || !(eps_low >= 0.0 && eps_low < 1.0)) return SIDCO_ERR_ARG;
    int M = stages;
    if (khat_avg > k * (1.0 + eps_high)) M -= 1;
    if (khat_avg < k * (1.0 - eps_low)) M += 1;
    if (M < 1) M = 1;
    if (M > max_stages) M = max_stages;
    return M;
}

struct sidco_controller {
    double delta, delta1, eps_high, eps_low;
    int dist, stages, max_stages, Q;
    int64_t iteration;      // calls made so far
    double last_avg;        // khat average the last adaptation saw (-1 before the first)
    unsigned long long id;  // stamps the device state of the controller's calls
    int64_t disturbed;      // windows whose count another caller of the same workspace broke
};

int sidco_controller_create(sidco_controller** out, double delta, int dist, int stages, int max_stages, int Q,
                            double eps_high, double eps_low, double delta1)
{
    if (!out) return SIDCO_ERR_NULL;
    *out = nullptr;
    if (!(delta > 0.0 && delta < 1.0) || !(delta1 > 0.0 && delta1 < 1.0)) return SIDCO_ERR_DELTA;
    if (dist != SIDCO_DIST_EXP && dist != SIDCO_DIST_GAMMA_GPD && dist != SIDCO_DIST_GPD) return SIDCO_ERR_DIST;
    if (max_stages < 1 || max_stages > SIDCO_MAX_STAGES || stages < 1 || stages > max_stages) return SIDCO_ERR_STAGES;
    if (Q < 1) return SIDCO_ERR_ARG;
    if (!(eps_high >= 0.0) || !(eps_low >= 0.0 && eps_low < 1.0)) return SIDCO_ERR_ARG;
    sidco_controller* c = new (std::nothrow) sidco_controller;
    if (!c) return SIDCO_ERR_ARG;
    c->delta = delta;
    c->delta1 = delta1;
    c->eps_high = eps_high;
    c->eps_low = eps_low;
    c->dist = dist;
    c->stages = stages;
    c->max_stages = max_stages;
    c->Q = Q;
    c->iteration = 0;
    c->last_avg = -1.0;
    c->disturbed = 0;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        c->id = g_next_owner++;
    }
    *out = c;
    return SIDCO_OK;
}

void sidco_controller_destroy(sidco_controller* c) { delete c; }

int sidco_controller_stages(const sidco_controller* c) { return c ? c->stages : SIDCO_ERR_NULL; }

int64_t sidco_controller_iteration(const sidco_controller* c) { return c ? c->iteration : (int64_t)SIDCO_ERR_NULL; }

double sidco_controller_last_average(const sidco_controller* c) { return c ? c->last_avg : -1.0; }

int64_t sidco_controller_disturbed(const sidco_controller* c) { return c ? c->disturbed : (int64_t)SIDCO_ERR_NULL; }

int sidco_controller_compress(sidco_controller* c, void* stream, const float* grad, float* residual, int64_t d,
                              int32_t* out_idx, float* out_val, int32_t* out_count, float* out_eta)
{
    return sidco_controller_compress_typed(c, stream, grad, SIDCO_GRAD_F32, residual, d, out_idx, out_val, out_count,
                                           out_eta);
}

int sidco_controller_compress_typed(sidco_controller* c, void* stream, const void* grad, int grad_dtype, float* residual,
                                    int64_t d, int32_t* out_idx, float* out_val, int32_t* out_count, float* out_eta)
{
    if (!c) return SIDCO_ERR_NULL;
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16)
        return SIDCO_ERR_ARG;
    const int gt = grad_type(grad_dtype);
    int rc = check_common(grad, residual, d, c->dist, out_idx, out_val, out_count, out_eta, gt == kGradF32 ? 4 : 2);
    if (rc != SIDCO_OK) return rc;
    double ratios[SIDCO_MAX_STAGES];
    const int M = sidco_stage_ratios(c->delta, c->stages, c->delta1, ratios);
    if (M < 1) return M;
    // the count of reported pairs starts over on the first call after an adaptation
    const bool first_of_window = c->iteration % c->Q == 0;
    rc = run(stream, grad, residual, d, c->dist, ratios, M, out_idx, out_val, sidco_out_capacity(d, c->delta),
             out_count, out_eta, first_of_window, gt, c->id);
    if (rc != SIDCO_OK) return rc;
    c->iteration += 1;
    if (c->iteration % c->Q != 0) return SIDCO_OK;
    // every Q-th call: read the count back (the only host synchronisation of the controller) and adapt
    DevState st;
    int64_t cap;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        WsCtx* w = nullptr;
        rc = pick_ws(stream, false, &w);
        if (rc != SIDCO_OK) return rc;
        cap = w->last_cap;
        hipError_t e = hipMemcpyAsync(&st, &((WorkspaceHead*)w->ws)->st, sizeof(DevState), hipMemcpyDeviceToHost,
                                      (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(controller)");
        e = hipStreamSynchronize((hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    }
    if (st.disturbed || st.owner != c->id) {
        // another caller used this workspace inside the window: its count is not this vector's, keep M
        c->disturbed += 1;
        return SIDCO_OK;
    }
    const unsigned long long last = st.selected_ctr < (unsigned long long)cap ? st.selected_ctr : (unsigned long long)cap;
    const double avg = (double)(st.khat_sum + last) / (double)c->Q;
    c->last_avg = avg;
    const int next = sidco_adapt_stages(c->stages, avg, c->delta * (double)d, c->eps_high, c->eps_low, c->max_stages);
    if (next >= 1) c->stages = next;
    return SIDCO_OK;
}

int sidco_scatter_add(void* stream, float* dense, int64_t d, const int32_t* idx, const float* val, const int32_t* count,
                      int64_t capacity, float scale)
{
    if (!dense || !idx || !val || !count) return SIDCO_ERR_NULL;
    if (d < 1 || d > (int64_t)INT32_MAX || capacity < 1 || capacity > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    if (!aligned4(dense) || !aligned4(idx) || !aligned4(val) || !aligned4(count)) return SIDCO_ERR_ALIGN;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, true, &cp);
    if (rc != SIDCO_OK) return rc;
    rc = ensure_workspace(*cp, cp->ws ? cp->ws_bytes : head_bytes());  // the head alone is enough here
    if (rc != SIDCO_OK) return rc;
    WorkspaceHead* h = (WorkspaceHead*)cp->ws;
    if (!cp->bad_cleared) {
        launch_clear_u32(&h->st.bad_index, (hipStream_t)stream);
        cp->bad_cleared = true;
    }
    launch_scatter_add(dense, d, idx, val, count, capacity, scale, &h->st.bad_index, (hipStream_t)stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return SIDCO_OK;
}

int sidco_scatter_check(void* stream)
{
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, false, &cp);
    if (rc == SIDCO_ERR_WORKSPACE) return 0;  // no scatter call has been made on this stream
    if (rc != SIDCO_OK) return rc;
    if (!cp->ws || !cp->bad_cleared) return 0;
    uint32_t bad = 0;
    WorkspaceHead* h = (WorkspaceHead*)cp->ws;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(&bad, &h->st.bad_index, sizeof(bad), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(bad_index)");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    if (bad) launch_clear_u32(&h->st.bad_index, s);
    return bad ? 1 : 0;
}

// ---- batched calls ----
namespace {

struct BatchPlan {
    std::vector<TensorDesc> desc;
    std::vector<uint16_t> map, fmap;
    uint32_t blocks = 0, final_blocks = 0;
    uint64_t slots = 0;  // survivor-list slots of all vectors
    uint32_t flat_gx = 0;  // > 0: the first pass runs in the flat shape with this many chunks per block (see below)
};

// Splits the 512 blocks of a launch over the vectors in proportion to their lengths (at least one each).
int plan_batch(const int64_t* offsets, int n, const int64_t* out_offsets, BatchPlan& pl)
{
    if (n < 1 || n > kMaxBatch) return SIDCO_ERR_SIZE;
    uint64_t tiles_total = 0;
    for (int t = 0; t < n; ++t) {
        const int64_t d = offsets[t + 1] - offsets[t];
        if (offsets[t] < 0 || d < 1 || d > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
        if (out_offsets[t] < 0 || out_offsets[t + 1] - out_offsets[t] < 1) return SIDCO_ERR_SIZE;
        tiles_total += (uint64_t)((d + kTile - 1) / kTile);
    }
    pl.desc.assign(n, TensorDesc());
    pl.map.assign(kMaxBlocks, 0);
    pl.fmap.assign(kMaxBlocks, 0);
    uint32_t fb = 0, ff = 0;
    uint64_t slot = 0;
    for (int t = 0; t < n; ++t) {
        TensorDesc& ds = pl.desc[t];
        const int64_t d = offsets[t + 1] - offsets[t];
        const uint64_t ntiles = (uint64_t)((d + kTile - 1) / kTile);
        uint64_t share = 1 + ((uint64_t)(kMaxBlocks - n) * ntiles) / tiles_total;
        uint64_t nwaves = share * kWavesPerBlock < ntiles ? share * kWavesPerBlock : ntiles;
        ds.offset = offsets[t];
        ds.d = d;
        ds.first_block = fb;
        ds.nblocks = (uint32_t)((nwaves + kWavesPerBlock - 1) / kWavesPerBlock);
        ds.first_final = ff;
        ds.nfinal = (uint32_t)((nwaves + 31) / 32);
        ds.seg_off = slot;
        ds.out_offset = out_offsets[t];
        ds.out_cap = out_offsets[t + 1] - out_offsets[t];
        ds.index = (uint32_t)t;
        ds.reserved = 0;
        for (uint32_t i = 0; i < ds.nblocks; ++i) pl.map[fb + i] = (uint16_t)t;
        for (uint32_t i = 0; i < ds.nfinal; ++i) pl.fmap[ff + i] = (uint16_t)t;
        fb += ds.nblocks;
        ff += ds.nfinal;
        slot += ntiles * kTile;
    }
    pl.blocks = fb;
    pl.final_blocks = ff;
    pl.slots = slot;
    // The flat first pass (k_fit_flat_batched) launches, for every block of the dense grid, as many chunks of
    // 4 tiles as the block with the most tiles needs.  It pays from the same total length as for a single vector,
    // and only while most of the launched chunks exist: with a few long vectors among many short ones (whose one
    // block has few tiles) the grid would be mostly empty.
    uint64_t total = 0, chunks = 0, most = 0;
    for (int t = 0; t < n; ++t) {
        const TensorDesc& ds = pl.desc[t];
        const uint64_t ntiles = (uint64_t)((ds.d + kTile - 1) / kTile);
        const uint64_t nwaves = (uint64_t)ds.nblocks * kWavesPerBlock < ntiles ? (uint64_t)ds.nblocks * kWavesPerBlock : ntiles;
        total += (uint64_t)ds.d;
        for (uint32_t b = 0; b < ds.nblocks; ++b) {
            const uint64_t w0 = (uint64_t)b * kWavesPerBlock;
            const uint64_t w1 = w0 + kWavesPerBlock < nwaves ? w0 + kWavesPerBlock : nwaves;
            const uint64_t tiles = (w1 * ntiles) / nwaves - (w0 * ntiles) / nwaves;
            const uint64_t c = (tiles + kFlatBlock / 64 - 1) / (kFlatBlock / 64);
            chunks += c;
            if (c > most) most = c;
        }
    }
    pl.flat_gx = 0;
    if ((int64_t)total >= kFlatMinD && most * fb <= 2 * chunks && most <= 0x7fffffffull / fb &&
        3 * most * fb <= slot)  // the partial sums borrow the second list buffer
        pl.flat_gx = (uint32_t)most;
    return SIDCO_OK;
}

}  // namespace

int sidco_batched_out_offsets(const int64_t* offsets, int n, double delta, int64_t* out_offsets)
{
    if (!offsets || !out_offsets) return SIDCO_ERR_NULL;
    if (n < 1 || n > kMaxBatch) return SIDCO_ERR_SIZE;
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    out_offsets[0] = 0;
    for (int t = 0; t < n; ++t) {
        const int64_t cap = sidco_out_capacity(offsets[t + 1] - offsets[t], delta);
        if (cap < 1) return SIDCO_ERR_SIZE;
        out_offsets[t + 1] = out_offsets[t] + cap;
    }
    return SIDCO_OK;
}

size_t sidco_workspace_bytes_batched(const int64_t* offsets, int n)
{
    if (!offsets || n < 1 || n > kMaxBatch) return 0;
    uint64_t slots = 0;
    for (int t = 0; t < n; ++t) {
        const int64_t d = offsets[t + 1] - offsets[t];
        if (d < 1) return 0;
        slots += (uint64_t)((d + kTile - 1) / kTile) * kTile;
    }
    return head_bytes() + 2 * slots * sizeof(int2);
}

int sidco_compress_batched(void* stream, const float* grad, float* residual, const int64_t* offsets, int n, double delta,
                           int dist, int stages, int32_t* out_idx, float* out_val, const int64_t* out_offsets,
                           int32_t* out_counts, float* out_etas)
{
    return sidco_compress_batched_typed(stream, grad, SIDCO_GRAD_F32, residual, offsets, n, delta, dist, stages, out_idx,
                                        out_val, out_offsets, out_counts, out_etas);
}

size_t sidco_workspace_bytes_batched_typed(const int64_t* offsets, int n, int grad_dtype, int has_residual)
{
    const size_t base = sidco_workspace_bytes_batched(offsets, n);
    if (base == 0) return 0;
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16) return 0;
    const bool own_acc = grad_dtype != SIDCO_GRAD_F32 && !has_residual;
    return base + (own_acc ? (base - head_bytes()) / 4 : 0);  // one float per list slot of one buffer
}

int sidco_compress_batched_typed(void* stream, const void* grad, int grad_dtype, float* residual, const int64_t* offsets,
                                 int n, double delta, int dist, int stages, int32_t* out_idx, float* out_val,
                                 const int64_t* out_offsets, int32_t* out_counts, float* out_etas)
{
    if (!grad || !offsets || !out_idx || !out_val || !out_offsets || !out_counts || !out_etas) return SIDCO_ERR_NULL;
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16)
        return SIDCO_ERR_ARG;
    const int gt = grad_type(grad_dtype);
    if (dist != SIDCO_DIST_EXP && dist != SIDCO_DIST_GAMMA_GPD && dist != SIDCO_DIST_GPD) return SIDCO_ERR_DIST;
    if (((uintptr_t)grad & (gt == kGradF32 ? 3u : 1u)) != 0 || !aligned4(residual) || !aligned4(out_idx) ||
        !aligned4(out_val) || !aligned4(out_counts) || !aligned4(out_etas))
        return SIDCO_ERR_ALIGN;
    if (residual && (const void*)residual == (const void*)grad) return SIDCO_ERR_ARG;
    if (!(delta > 0.0 && delta < 1.0)) return SIDCO_ERR_DELTA;
    if (stages < 1 || stages > SIDCO_MAX_STAGES) return SIDCO_ERR_STAGES;
    double ratios[SIDCO_MAX_STAGES];
    const int M = sidco_stage_ratios(delta, stages, default_delta1(), ratios);
    if (M < 1) return M;
    BatchPlan pl;
    int rc = plan_batch(offsets, n, out_offsets, pl);
    if (rc != SIDCO_OK) return rc;

    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    rc = pick_ws(stream, true, &cp);
    if (rc != SIDCO_OK) return rc;
    WsCtx& c = *cp;
    const bool own_acc = gt != kGradF32 && !residual;  // the widened vectors need a home
    rc = ensure_workspace(c, head_bytes() + 2 * pl.slots * sizeof(int2) + (own_acc ? pl.slots * sizeof(float) : 0));
    if (rc != SIDCO_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    WorkspaceHead* h = (WorkspaceHead*)c.ws;
    const double theta = g_speculation;

    // The table on the device (descriptors and block maps, one contiguous piece of BatchTable) is uploaded
    // when it differs from the one already there, asynchronously and in stream order, from a host image
    // that the library keeps for good (the copy may still be reading it when this call returns, and a
    // caller may have captured it into a graph).  A call that repeats the previous one, shared arguments
    // included, may use the vectors' threshold hints.
    constexpr size_t table_bytes = sizeof(BatchTable) - offsetof(BatchTable, desc);
    std::vector<unsigned char> image(table_bytes, 0);
    memcpy(image.data(), pl.desc.data(), (size_t)n * sizeof(TensorDesc));
    memcpy(image.data() + (offsetof(BatchTable, map) - offsetof(BatchTable, desc)), pl.map.data(),
           kMaxBlocks * sizeof(uint16_t));
    memcpy(image.data() + (offsetof(BatchTable, fmap) - offsetof(BatchTable, desc)), pl.fmap.data(),
           kMaxBlocks * sizeof(uint16_t));
    const bool same_table = c.batch_cur >= 0 && image == *c.batch_images[(size_t)c.batch_cur];
    const bool same_shape = same_table && c.batch_delta == delta && c.batch_theta == theta && c.batch_dist == dist &&
                            c.batch_M == M;
    if (!same_table) {
        int found = -1;
        for (size_t i = 0; i < c.batch_images.size() && found < 0; ++i)
            if (*c.batch_images[i] == image) found = (int)i;
        if (found < 0) {
            auto* keep = new (std::nothrow) std::vector<unsigned char>();
            if (!keep) return SIDCO_ERR_ARG;
            keep->swap(image);
            c.batch_images.push_back(keep);
            found = (int)c.batch_images.size() - 1;
        }
        hipError_t e = hipMemcpyAsync(h->batch.desc, c.batch_images[(size_t)found]->data(), table_bytes,
                                      hipMemcpyHostToDevice, s);
        if (e != hipSuccess) {
            c.batch_cur = -1;
            return hip_fail(e, "hipMemcpyAsync(batch table)");
        }
        c.batch_cur = found;
    }
    c.batch_delta = delta;
    c.batch_theta = theta;
    c.batch_dist = dist;
    c.batch_M = M;
    c.batch_n = n;
    c.batch_cap.resize(n);
    for (int t = 0; t < n; ++t) c.batch_cap[t] = pl.desc[t].out_cap;
    c.sig_d = 0;  // the single-call record of the head is not touched, but keep the rule simple: no hint across kinds

    BatchArgs a;
    memset(&a, 0, sizeof(a));
    a.tb = &h->batch;
    a.grad = grad;
    a.gt = gt;
    a.residual = residual;
    a.acc_own = own_acc ? (float*)((char*)c.ws + head_bytes() + 2 * pl.slots * sizeof(int2)) : nullptr;
    a.out_idx = out_idx;
    a.out_val = out_val;
    a.out_counts = out_counts;
    a.out_etas = out_etas;
    const size_t seg = pl.slots * sizeof(int2);
    for (int i = 0; i < 2; ++i) {
        a.part[i] = h->part[i];
        a.cnt[i] = h->cnt[i];
        a.blk[i] = h->blk[i];
        a.seg[i] = (int2*)((char*)c.ws + head_bytes() + i * seg);
    }
    a.dist = dist;
    a.M = M;
    for (int m = 0; m < M; ++m) a.L[m] = log(1.0 / ratios[m]);
    a.use_hint = same_shape ? 1 : 0;

    // The dense stages may prefetch (see launch_compact) if that is safe for every vector: its accumulated values
    // start on a 16-byte boundary (and its gradient on the boundary the vector path needs), each of its blocks
    // runs all its waves, and every wave owns the prefetched tiles complete.
    bool prefetch = true;
    for (int t = 0; t < n && prefetch; ++t) {
        const TensorDesc& ds = pl.desc[t];
        const uint64_t ntiles = (uint64_t)((ds.d + kTile - 1) / kTile), nfull = (uint64_t)(ds.d / kTile);
        const uint64_t nwaves = (uint64_t)ds.nblocks * kWavesPerBlock;
        const uintptr_t g = (uintptr_t)grad + (uintptr_t)ds.offset * (gt == kGradF32 ? 4u : 2u);
        const float* accp = residual ? residual + ds.offset : (a.acc_own ? a.acc_own + ds.offset : nullptr);
        prefetch = nwaves <= ntiles && nfull / nwaves >= (uint64_t)(kCompactPrefetch * 4 + 1) &&
                   (g & (gt == kGradF32 ? 15u : 7u)) == 0 && ((uintptr_t)accp & 15u) == 0;
    }

    // same sequence as a single call (see run), every kernel once for all vectors
    a.in = 1;
    a.out = 0;
    launch_fit_batched(a, residual != nullptr, pl.blocks, pl.flat_gx, (double*)a.seg[1], s);  // seg[1] is free until the first stage kernel writes it
    bool lists = false, cand = false, reverse = true;
    double cum = 1.0;
    int sel = 0;
    auto bind = [&](int m) {
        a.in = sel;
        a.out = sel ^ 1;
        sel ^= 1;
        a.stage = m;
        a.theta = 0.0f;
        a.prev_cand = cand ? 1 : 0;
    };
    for (int m = 1; m < M; ++m) {
        bind(m);
        if (!lists) {
            const double Lw = a.L[m - 1] + theta * a.L[m];
            const bool write = cum * exp(-Lw) <= kMaterializeBelow;
            if (write && theta > 0.0) {
                a.theta = (float)theta;
                a.theta_min = hint_floor(cum, a.L[m - 1], a.L[m]);
            }
            a.reverse = reverse ? 1 : 0;
            reverse = !reverse;
            launch_compact_batched(a, /*stats=*/true, write, prefetch, pl.blocks, s);
            if (write) {
                lists = true;
                cand = theta > 0.0;
            }
        } else {
            launch_lists_batched(a, pl.blocks, s);
            cand = false;
        }
        cum *= ratios[m - 1];
    }
    bind(M);
    if (!lists) {
        a.reverse = reverse ? 1 : 0;
        launch_compact_batched(a, /*stats=*/false, /*write=*/true, prefetch, pl.blocks, s);
        a.in = sel;  // the gather reads what the compaction just wrote
        launch_gather_batched(a, pl.blocks, s);
    } else {
        launch_final_lists_batched(a, pl.final_blocks, s);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return SIDCO_OK;
}

int sidco_read_diag_batched(void* stream, int t, sidco_diag* host_out)
{
    if (!host_out) return SIDCO_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, false, &cp);
    if (rc != SIDCO_OK) return rc;
    WsCtx& c = *cp;
    if (!c.ws || c.batch_cur < 0) return SIDCO_ERR_WORKSPACE;
    if (t < 0 || t >= c.batch_n) return SIDCO_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    DevState st;
    hipError_t e = hipMemcpyAsync(&st, &((WorkspaceHead*)c.ws)->batch.st[t], sizeof(DevState), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(diag)");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    fill_diag(st, c.batch_cap[t], host_out);
    return SIDCO_OK;
}

int sidco_topk(void* stream, const float* grad, float* residual, int64_t d, int64_t k, int32_t* out_idx, float* out_val,
               int32_t* out_count, float* out_kth)
{
    return sidco_topk_typed(stream, grad, SIDCO_GRAD_F32, residual, d, k, out_idx, out_val, out_count, out_kth);
}

int sidco_topk_typed(void* stream, const void* grad, int grad_dtype, float* residual, int64_t d, int64_t k,
                     int32_t* out_idx, float* out_val, int32_t* out_count, float* out_kth)
{
    if (!grad || !out_idx || !out_val || !out_count || !out_kth) return SIDCO_ERR_NULL;
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16)
        return SIDCO_ERR_ARG;
    if (d < 1 || d > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    if (k < 1 || k > d) return SIDCO_ERR_SIZE;
    const int gt = grad_type(grad_dtype);
    if (((uintptr_t)grad & (gt == kGradF32 ? 3u : 1u)) != 0 || !aligned4(residual) || !aligned4(out_idx) ||
        !aligned4(out_val) || !aligned4(out_count) || !aligned4(out_kth))
        return SIDCO_ERR_ALIGN;
    if (residual && (const void*)residual == (const void*)grad) return SIDCO_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    DeviceCtx* dev = nullptr;
    int rc = pick_ws(stream, true, &cp, &dev);
    if (rc != SIDCO_OK) return rc;
    WsCtx& c = *cp;
    const bool own_acc = gt != kGradF32 && !residual;  // the widened vector needs a home
    rc = ensure_workspace(c, head_bytes() + 2 * seg_bytes(d) + (own_acc ? acc_bytes(d) : 0));
    if (rc != SIDCO_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    WorkspaceHead* h = (WorkspaceHead*)c.ws;

    Params q;
    fill_common(q, h, grad, residual, d, SIDCO_DIST_EXP, gt,
                own_acc ? (float*)((char*)c.ws + head_bytes() + 2 * seg_bytes(d)) : nullptr);
    TopkParams p;
    memset(&p, 0, sizeof(p));
    p.grad = grad;
    p.gt = gt;
    p.residual = residual;
    p.acc_w = q.acc_w;
    p.acc = q.acc;
    p.d = d;
    p.k = k;
    p.ntiles = q.ntiles;
    p.nfull = q.nfull;
    p.nwaves = q.nwaves;
    p.nblocks = q.nblocks;
    p.vec_ok = q.vec_ok;
    p.hist = h->topk_hist;
    p.st = &h->topk;
    p.cnt = h->cnt[0];
    p.seg = (int2*)((char*)c.ws + head_bytes());
    p.out_idx = out_idx;
    p.out_val = out_val;
    p.out_count = out_count;
    p.out_kth = out_kth;

    const bool prof = g_profiling;
    if (prof) {
        rc = make_events(c);
        if (rc != SIDCO_OK) return rc;
        dev->last_prof = &c;
    }
    int kn = 0;
    auto mark = [&](const char* name) {
        if (!prof) return;
        if (name) c.prof_name[kn - 1] = name;
        (void)hipEventRecord(c.ev[kn], s);
    };
    mark(nullptr);
    launch_topk_zero(p, s);
    ++kn;
    mark("k_topk_zero");
    launch_topk_hist(p, s);
    ++kn;
    mark("k_topk_hist");
    launch_topk_compact(p, s);
    ++kn;
    mark("k_topk_compact");
    // the lists hold the k largest entries and the rest of one histogram bin: short, so few blocks
    uint32_t grid = (p.nwaves + 31) / 32;
    if ((double)k > 4.0e6) grid = 256;
    if (grid > p.nblocks) grid = p.nblocks;
    if (grid < 1) grid = 1;
    launch_topk_refine(p, grid, s);
    ++kn;
    mark("k_topk_refine");
    launch_topk_final(p, grid, s);
    ++kn;
    mark("k_topk_final");
    c.prof_n = prof ? kn : 0;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return SIDCO_OK;
}

// n_s, k_s and k of the DGC comparator; false if an argument is out of range
static bool dgc_sizes(int64_t d, double delta, double sample_ratio, int64_t* n_s, int64_t* k_s, int64_t* k)
{
    if (d < 1 || d > (int64_t)INT32_MAX) return false;
    if (!(delta > 0.0 && delta < 1.0) || !(sample_ratio > 0.0 && sample_ratio <= 1.0)) return false;
    int64_t ns = (int64_t)ceil(sample_ratio * (double)d);
    ns = ns < 1 ? 1 : (ns > d ? d : ns);
    int64_t ks = (int64_t)ceil(delta * (double)ns);
    ks = ks < 1 ? 1 : (ks > ns ? ns : ks);
    int64_t kk = (int64_t)ceil(delta * (double)d);
    kk = kk < 1 ? 1 : (kk > d ? d : kk);
    *n_s = ns;
    *k_s = ks;
    *k = kk;
    return true;
}

int sidco_dgc_sizes(int64_t d, double delta, double sample_ratio, int64_t* sizes)
{
    if (!sizes) return SIDCO_ERR_NULL;
    if (d < 1 || d > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    if (!dgc_sizes(d, delta, sample_ratio, &sizes[0], &sizes[1], &sizes[2])) return SIDCO_ERR_DELTA;
    return SIDCO_OK;
}

int sidco_dgc(void* stream, const float* grad, float* residual, int64_t d, double delta, double sample_ratio,
              uint64_t seed, int32_t* out_idx, float* out_val, int32_t* out_count, float* out_eta)
{
    return sidco_dgc_typed(stream, grad, SIDCO_GRAD_F32, residual, d, delta, sample_ratio, seed, out_idx, out_val,
                           out_count, out_eta);
}

int sidco_dgc_typed(void* stream, const void* grad, int grad_dtype, float* residual, int64_t d, double delta,
                    double sample_ratio, uint64_t seed, int32_t* out_idx, float* out_val, int32_t* out_count,
                    float* out_eta)
{
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16)
        return SIDCO_ERR_ARG;
    const int gt = grad_type(grad_dtype);
    int rc = check_common(grad, residual, d, SIDCO_DIST_EXP, out_idx, out_val, out_count, out_eta, gt == kGradF32 ? 4 : 2);
    if (rc != SIDCO_OK) return rc;
    int64_t n_s, k_s, k;
    if (!dgc_sizes(d, delta, sample_ratio, &n_s, &k_s, &k)) return SIDCO_ERR_DELTA;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    DeviceCtx* dev = nullptr;
    rc = pick_ws(stream, true, &cp, &dev);
    if (rc != SIDCO_OK) return rc;
    WsCtx& c = *cp;
    rc = ensure_workspace(c, head_bytes() + 2 * seg_bytes(d));
    if (rc != SIDCO_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    WorkspaceHead* h = (WorkspaceHead*)c.ws;

    Params q;
    fill_common(q, h, grad, residual, d, SIDCO_DIST_EXP, gt);  // no stored acc without a residual: the one dense
                                                              // pass keeps what it selects in the lists
    DgcParams p;
    memset(&p, 0, sizeof(p));
    p.grad = grad;
    p.gt = gt;
    p.residual = residual;
    p.d = d;
    p.k = k;
    p.ntiles = q.ntiles;
    p.nfull = q.nfull;
    p.nwaves = q.nwaves;
    p.nblocks = q.nblocks;
    p.vec_ok = q.vec_ok;
    p.seed = seed;
    p.n_s = (uint32_t)n_s;
    p.k_s = (uint32_t)k_s;
    p.keys = (uint32_t*)((char*)c.ws + head_bytes() + seg_bytes(d));  // the second list buffer is free here
    p.hist_s = h->dgc_hist[0];
    p.hist_l = h->dgc_hist[1];
    p.st = &h->dgc;
    p.cnt = h->cnt[0];
    p.seg = (int2*)((char*)c.ws + head_bytes());
    p.out_eta = out_eta;

    // the second select runs on the kernels of the exact Top-k, with k decided on the device
    TopkParams t;
    memset(&t, 0, sizeof(t));
    t.grad = grad;
    t.gt = gt;
    t.residual = residual;
    t.acc_w = residual;
    t.acc = residual;  // unused: the second select works on the lists alone
    t.d = d;
    t.k = k;
    t.k_from_state = 1;
    t.ntiles = q.ntiles;
    t.nfull = q.nfull;
    t.nwaves = q.nwaves;
    t.nblocks = q.nblocks;
    t.vec_ok = q.vec_ok;
    t.hist = h->dgc_hist[1];
    t.st = &h->dgc.lists;
    t.cnt = p.cnt;
    t.seg = p.seg;
    t.out_idx = out_idx;
    t.out_val = out_val;
    t.out_count = out_count;
    t.out_kth = &h->dgc.kth;

    const bool prof = g_profiling;
    if (prof) {
        rc = make_events(c);
        if (rc != SIDCO_OK) return rc;
        dev->last_prof = &c;
    }
    int kn = 0;
    auto mark = [&](const char* name) {
        if (!prof) return;
        if (name) c.prof_name[kn - 1] = name;
        (void)hipEventRecord(c.ev[kn], s);
    };
    mark(nullptr);
    launch_dgc_zero(p, s);
    ++kn;
    mark("k_dgc_zero");
    launch_dgc_sample(p, s);
    ++kn;
    mark("k_dgc_sample");
    launch_dgc_digit(p, 1, s);
    ++kn;
    mark("k_dgc_digit1");
    launch_dgc_digit(p, 2, s);
    ++kn;
    mark("k_dgc_digit2");
    launch_dgc_dense(p, s);
    ++kn;
    mark("k_dgc_dense");
    uint32_t grid = (p.nwaves + 31) / 32;  // the lists hold about k entries: few blocks
    if (grid > p.nblocks) grid = p.nblocks;
    if (grid < 1) grid = 1;
    launch_dgc_lists(p, grid, s);
    ++kn;
    mark("k_dgc_lists");
    launch_topk_refine(t, grid, s);
    ++kn;
    mark("k_topk_refine");
    launch_topk_final(t, grid, s);
    ++kn;
    mark("k_topk_final");
    c.prof_n = prof ? kn : 0;
    c.dgc_n_s = n_s;
    c.dgc_k_s = k_s;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return SIDCO_OK;
}

int sidco_dgc_result(void* stream, int64_t* host_out)
{
    if (!host_out) return SIDCO_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, false, &cp);
    if (rc != SIDCO_OK) return rc;
    if (!cp->ws || cp->dgc_n_s == 0) return SIDCO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    DgcState st;
    hipError_t e = hipMemcpyAsync(&st, &((WorkspaceHead*)cp->ws)->dgc, sizeof(DgcState), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(dgc state)");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    host_out[0] = cp->dgc_n_s;
    host_out[1] = cp->dgc_k_s;
    host_out[2] = (int64_t)st.first_pass;
    host_out[3] = (int64_t)st.lists.k_eff;
    return SIDCO_OK;
}

int sidco_fit_typed(void* stream, const void* grad, int grad_dtype, float* residual, int64_t d, int dist)
{
    if (!grad) return SIDCO_ERR_NULL;
    if (grad_dtype != SIDCO_GRAD_F32 && grad_dtype != SIDCO_GRAD_F16 && grad_dtype != SIDCO_GRAD_BF16)
        return SIDCO_ERR_ARG;
    if (d < 1 || d > (int64_t)INT32_MAX) return SIDCO_ERR_SIZE;
    if (dist != SIDCO_DIST_EXP && dist != SIDCO_DIST_GAMMA_GPD && dist != SIDCO_DIST_GPD) return SIDCO_ERR_DIST;
    const bool f32 = grad_dtype == SIDCO_GRAD_F32;
    if (((uintptr_t)grad & (f32 ? 3u : 1u)) != 0 || !aligned4(residual)) return SIDCO_ERR_ALIGN;
    if (residual && (const void*)residual == grad) return SIDCO_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, true, &cp);
    if (rc != SIDCO_OK) return rc;
    const bool own_acc = !f32 && !residual;
    rc = ensure_workspace(*cp, head_bytes() + 2 * seg_bytes(d) + (own_acc ? acc_bytes(d) : 0));
    if (rc != SIDCO_OK) return rc;
    WorkspaceHead* h = (WorkspaceHead*)cp->ws;
    Params p;
    fill_common(p, h, grad, residual, d, dist, f32 ? kGradF32 : (grad_dtype == SIDCO_GRAD_F16 ? kGradF16 : kGradBf16),
                own_acc ? (float*)((char*)cp->ws + head_bytes() + 2 * seg_bytes(d)) : nullptr);
    p.M = 1;
    p.acc_reset = 1;
    p.part_out = h->part[0];
    launch_fit(p, (double*)((char*)cp->ws + head_bytes() + seg_bytes(d)), (hipStream_t)stream);
    cp->fit_nblocks = p.nblocks;
    cp->fit_d = d;
    cp->fit_dist = dist;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "kernel launch");
    return SIDCO_OK;
}

int sidco_fit(void* stream, const float* grad, float* residual, int64_t d, int dist)
{
    return sidco_fit_typed(stream, grad, SIDCO_GRAD_F32, residual, d, dist);
}

int sidco_fit_result(void* stream, double* host_sums)
{
    if (!host_sums) return SIDCO_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, false, &cp);
    if (rc != SIDCO_OK) return rc;
    if (!cp->ws || cp->fit_nblocks == 0) return SIDCO_ERR_WORKSPACE;
    static thread_local double part[4 * kMaxBlocks];
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(part, ((WorkspaceHead*)cp->ws)->part[0], sizeof(part), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(partials)");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    double sum[3] = {0.0, 0.0, 0.0};
    for (int q = 0; q < 3; ++q)
        for (uint32_t b = 0; b < cp->fit_nblocks; ++b) sum[q] += part[q * kMaxBlocks + b];
    host_sums[0] = sum[0];
    host_sums[1] = cp->fit_dist == SIDCO_DIST_GPD ? sum[1] : 0.0;
    host_sums[2] = cp->fit_dist == SIDCO_DIST_GAMMA_GPD ? sum[2] * 0.6931471805599453094 : 0.0;
    host_sums[3] = (double)cp->fit_d;
    return SIDCO_OK;
}

int sidco_read_diag(void* stream, sidco_diag* host_out)
{
    if (!host_out) return SIDCO_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* cp = nullptr;
    int rc = pick_ws(stream, false, &cp);
    if (rc != SIDCO_OK) return rc;
    WsCtx& c = *cp;
    if (!c.ws) return SIDCO_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    DevState st;
    hipError_t e = hipMemcpyAsync(&st, &((WorkspaceHead*)c.ws)->st, sizeof(DevState), hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(diag)");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    fill_diag(st, c.last_cap, host_out);
    return SIDCO_OK;
}

int sidco_get_diag(void* stream, sidco_diag* host_out) { return sidco_read_diag(stream, host_out); }

int sidco_set_delta1(double delta1)
{
    if (!(delta1 > 0.0 && delta1 < 1.0)) return SIDCO_ERR_DELTA;
    std::lock_guard<std::mutex> lock(g_mu);
    g_delta1 = delta1;
    return SIDCO_OK;
}

int sidco_set_status_word(void* stream, uint32_t* device_word)
{
    if (!aligned4(device_word)) return SIDCO_ERR_ALIGN;
    std::lock_guard<std::mutex> lock(g_mu);
    WsCtx* c = nullptr;
    int rc = pick_ws(stream, true, &c);
    if (rc != SIDCO_OK) return rc;
    c->status_out = device_word;
    return SIDCO_OK;
}

int sidco_set_speculation(double theta)
{
    if (!(theta >= 0.0 && theta <= 1.0)) return SIDCO_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mu);
    g_speculation = theta;
    return SIDCO_OK;
}

int sidco_set_profiling(int enable)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_profiling = enable != 0;
    return SIDCO_OK;
}

int sidco_get_profile(float* ms, const char** names, int cap)
{
    if (!ms || cap < 1) return SIDCO_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceCtx* d = nullptr;
    int rc = current_device(&d);
    if (rc != SIDCO_OK) return rc;
    if (!d->last_prof || d->last_prof->prof_n == 0) return 0;
    WsCtx& c = *d->last_prof;
    hipError_t e = hipEventSynchronize(c.ev[c.prof_n]);
    if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
    for (int i = 0; i < c.prof_n && i < cap; ++i) {
        e = hipEventElapsedTime(&ms[i], c.ev[i], c.ev[i + 1]);
        if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
        if (names) names[i] = c.prof_name[i];
    }
    return c.prof_n;
}

const char* sidco_strerror(int code)
{
    switch (code) {
        case SIDCO_OK: return "ok";
        case SIDCO_ERR_NULL: return "a required pointer is NULL";
        case SIDCO_ERR_SIZE: return "d or a capacity is out of range (1 .. 2^31-1, or the static scratch of sidco_compress_static)";
        case SIDCO_ERR_DELTA: return "a compression ratio is not in (0,1)";
        case SIDCO_ERR_STAGES: return "number of stages out of range (1 .. SIDCO_MAX_STAGES)";
        case SIDCO_ERR_DIST: return "unknown distribution";
        case SIDCO_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
        case SIDCO_ERR_HIP: return "HIP runtime error";
        case SIDCO_ERR_ALIGN: return "pointer not 4-byte aligned";
        case SIDCO_ERR_ARG: return "invalid argument";
        default: return "unknown error code";
    }
}

const char* sidco_last_hip_error(void) { return g_hip_msg; }

int sidco_version(void) { return 100; }

void sidco_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (int dev = 0; dev < kMaxDevices; ++dev) {
        DeviceCtx& d = g_ctx[dev];
        d.stat = WsCtx();  // nothing to free: the scratch lives as long as the process
        if (!d.shared.ws && !d.shared.ev_made && d.streams.empty()) continue;
        if (hipSetDevice(dev) != hipSuccess) continue;
        free_ws(d.shared);
        for (WsCtx* w : d.streams) {
            free_ws(*w);
            delete w;
        }
        d.streams.clear();
        d.last_prof = nullptr;
    }
    if (have_cur) (void)hipSetDevice(cur);
}

}  // extern "C"

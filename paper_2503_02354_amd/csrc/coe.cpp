// Stage driver behind the C ABI: request store, regroup, batch splitting, expert cache with side-stream switches,
// per-expert batched forward, routing.  Host code only; kernels live in the .hip files.
#include "../../include/coe.h"

#include <hip/hip_runtime_api.h>

#include <fcntl.h>
#include <unistd.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <thread>
#include <cstdio>
#include <cstring>
#include <memory>
#include <string>
#include <vector>

#include "kernels.h"
#include "policy.h"

namespace {

constexpr int kMaxBufs = 8;
constexpr size_t kBlobAlign = 256;

size_t align_up(size_t x, size_t a = kBlobAlign) { return (x + a - 1) / a * a; }

struct LayerPlan {
    coe_layer d;
    int32_t H, W, C;        // source shape
    int32_t P, Q, K;        // destination shape (heads: K = classes)
    size_t off[4];          // byte offsets of this layer's tensors in the blob
    double macs;            // multiply-accumulates per request
    bool packed = false;    // conv filters are stored in matrix-core fragment order (device and pinned copies)
    bool fuse_pool = false; // conv: the max pool that follows runs inside the conv kernel, which writes the pool's dst
    bool fused_away = false;// pool: done by the preceding conv kernel
    bool patchify = false;  // conv with stride == window and no padding: patches are gathered into GEMM rows, then a 1x1 conv
};

struct ArchPlan {
    int32_t dtype, in_h, in_w, in_c, n_classes;
    std::vector<LayerPlan> layers;
    size_t blob_bytes = 0;
    size_t buf_elems[kMaxBufs] = {0};   // per request
    size_t patch_elems = 0;             // per request: rows of the largest patch-gathered conv
    bool groupable = false;             // every layer can run several experts' small groups in one launch
    int32_t row_cap = INT32_MAX;        // most requests one launch may cover: the kernels address a tensor with 31-bit byte offsets
    int32_t arr_min_res = 0, arr_min_miss = 0, arr_wait = 0;   // arranging window (coe_set_arranging); arr_wait 0 = off
    bool gathers_input = false;         // the only reader of the input is a few-channel conv kernel, which can follow a row table
    int64_t lat_k_ns = 1000, lat_b_ns = 0, lat_load_ns = 0;   // latency model (coe_set_latency_model): K n + B, expert load
    size_t elem() const { return dtype == COE_DT_BF16 ? 2 : 4; }
    size_t in_bytes() const { return (size_t)in_h * in_w * in_c * elem(); }
};

// One slot of the expert arena.  The arena is a single device allocation made when the dependency graph is set; it is cut
// into slots of one size class per distinct blob size (experts of one architecture share a class), as many per class as the
// cache caps allow to be resident at once, so a switch never allocates, frees or waits for the device.
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    hipEvent_t last_use = nullptr;   // recorded on the stream of the last kernel that read p
    bool used = false;
    int32_t cls = 0;                 // size class
};

// A pinned host buffer of the host tier (only with coe_set_host_tier): holds the blob of one expert at a time.
struct HostSlot {
    void* p = nullptr;
    int32_t cls = 0;
    hipEvent_t copied = nullptr;     // recorded on the copy stream after the last host-to-device copy out of p
    uint64_t planned = 0;            // copies out of p that steps have planned so far (stepping thread only)
    uint64_t issued = 0;             // ... and enqueued so far (guarded by the loader's mutex)
};

// One read from the backing file, carried out by the loader thread while the stepping thread goes on launching.
struct ReadJob {
    HostSlot* slot = nullptr;
    int64_t file_off = 0;
    size_t nbytes = 0;
    uint64_t need_issued = 0;        // copies out of the slot that must be enqueued (and complete) before it is overwritten
    bool done = false;
    int rc = COE_OK;
    double read_us = 0.0;
};

struct Expert {
    bool registered = false;
    int32_t arch = -1;
    float prob = 0.f;
    void* host = nullptr;            // pinned copy of the blob
    size_t nbytes = 0;
    int32_t cls = 0;                 // size class of its blob in the expert arena
    DevBuf* buf = nullptr;           // arena slot that holds the device copy when resident
    hipEvent_t loaded = nullptr;     // recorded on the copy stream after the switch
    bool load_pending = false;       // compute stream has not yet waited for `loaded`
    int64_t file_off = -1;           // host tier: where the blob sits in the backing file
    HostSlot* hslot = nullptr;       // host tier: the pinned slot that holds it, if any
};

struct ProfClass {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> spans;   // the timed launches
    double work = 0.0;                                       // their algorithmic work
    int64_t issued = 0;                                      // all launches of the class, timed or not
};

}  // namespace

// One executor (paper Section 4.1: executors run inference in parallel, each on its own queue of requests): a stream and
// the activation workspace of the launch sequences that run on it.
constexpr int kMaxLanes = 3;          // with the copy stream: four hardware queues, what a process gets by default

struct Lane {
    hipStream_t s = nullptr;
    void* d_buf[kMaxBufs] = {nullptr};
    size_t buf_bytes[kMaxBufs] = {0};
    void* d_patch = nullptr;         // GEMM rows of patch-gathered convolutions
    size_t patch_bytes = 0;
    hipEvent_t done = nullptr;       // recorded after the lane's last launch of a step
    bool used = false;               // launched something in the current step
    int64_t busy_ns = 0;             // predicted work assigned in the current step
};

struct coe_ctx {
    coe_config cfg;
    std::string err;
    hipStream_t sc = nullptr, sx = nullptr;
    bool own_sc = false, own_sx = false;

    std::vector<ArchPlan> archs;
    std::vector<Expert> experts;
    bool graph_set = false;
    int32_t E = 0;
    std::vector<int32_t> succ_off, succ;
    int32_t* d_succ = nullptr;
    std::unique_ptr<coe::Policy> policy;
    bool filled = false;
    std::vector<int32_t> switch_log;
    void* arena = nullptr;                          // all expert slots
    std::vector<DevBuf> slots;
    std::vector<std::vector<DevBuf*>> free_slots;   // per size class, oldest release first
    int64_t device_allocs = 0;                      // hipMalloc calls made by this context so far

    // host tier (third storage level): blobs live in a file, at most host_cap of them in pinned slots
    int32_t host_cap = 0;
    int fd = -1;
    std::string backing_path;
    int64_t file_bytes = 0;
    std::unique_ptr<coe::Policy> host_policy;
    std::vector<HostSlot> hslots;
    std::vector<std::vector<HostSlot*>> free_hslots;
    std::vector<int32_t> host_log;
    std::thread loader;                             // started with the host tier's slots, joined in coe_destroy
    std::mutex ld_mutex;
    std::condition_variable ld_cv;
    std::deque<ReadJob*> ld_queue;                  // jobs in the order of the switches they serve
    std::deque<ReadJob> ld_jobs;                    // storage of the current step's jobs
    bool ld_stop = false;

    // request store
    int32_t n_live = 0, n_collected = 0;
    int64_t id_base = 0;
    std::vector<uint8_t> collected;
    void* d_inputs = nullptr;
    void* d_staged = nullptr;
    int32_t *d_cur = nullptr, *d_depth = nullptr, *d_path = nullptr;
    float* d_logits = nullptr;
    int32_t max_classes = 0;
    int32_t logits_alloc_classes = 0;

    // regroup
    int32_t *d_cnt = nullptr, *d_off = nullptr, *d_perm = nullptr, *d_inv = nullptr, *d_blockhist = nullptr;
    int32_t* h_cnt = nullptr;        // pinned
    int32_t* h_first = nullptr;      // pinned, one entry per request slot: staging of the first experts of a submit
    int32_t last_pending = 0, last_live = 0, last_E = 0;
    std::vector<int32_t> submit_step;   // per request slot: number of the first step that sees the request
    int32_t step_no = 0;

    // executors: lanes[0] runs on the compute stream; further lanes (cfg.executors > 1) have a stream and an activation
    // workspace of their own, so that launch sequences of different groups overlap on the device
    std::vector<Lane> lanes;
    hipEvent_t ev_ready = nullptr;      // recorded on the compute stream when a step's regrouped inputs are ready
    struct Unit { int32_t expert; int64_t cost_ns; int32_t lane; };
    std::vector<Unit> last_units;       // launch sequences of the last step: first expert, predicted cost, executor
    std::vector<int32_t> last_chunks;   // batches of the last step after request splitting: {expert, first row, count} each

    // profiling
    ProfClass prof[COE_K_COUNT];
    std::vector<hipEvent_t> ev_pool;
};

namespace {

int fail(coe_ctx* c, int code, const std::string& msg)
{
    if (c) c->err = msg;
    return code;
}

#define HIPCHK(ctx, call)                                                                          \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return fail(ctx, COE_EDEVICE, std::string(#call) + ": " + hipGetErrorString(e_));      \
    } while (0)

// ---- profiling spans ---------------------------------------------------------------------------------------------
struct Span {
    coe_ctx* c;
    int cls;
    hipStream_t s;
    hipEvent_t e1 = nullptr;
    Span(coe_ctx* ctx, int kernel_class, double work, hipStream_t stream) : c(ctx), cls(kernel_class), s(stream)
    {
        if (!c->cfg.profile) return;
        // cfg.profile = k > 1 times every k-th launch of a class: an event pair costs a few microseconds of
        // pipeline bubble, which adds up over hundreds of launches per step
        if (c->prof[cls].issued++ % c->cfg.profile) return;
        hipEvent_t e0 = take();
        e1 = take();
        if (!e0 || !e1) { e1 = nullptr; return; }
        hipEventRecord(e0, s);
        c->prof[cls].spans.emplace_back(e0, e1);
        c->prof[cls].work += work;
    }
    ~Span()
    {
        if (e1) hipEventRecord(e1, s);
    }
    hipEvent_t take()
    {
        if (!c->ev_pool.empty()) {
            hipEvent_t e = c->ev_pool.back();
            c->ev_pool.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

// ---- architecture planning -----------------------------------------------------------------------------------------
int plan_arch(coe_ctx* c, const coe_arch_desc* d, ArchPlan& a)
{
    if (d->dtype != COE_DT_F32 && d->dtype != COE_DT_BF16) return fail(c, COE_EINVAL, "arch: unknown dtype");
    if (d->in_h <= 0 || d->in_w <= 0 || d->in_c <= 0 || d->n_classes <= 0 || d->n_layers <= 0 || !d->layers)
        return fail(c, COE_EINVAL, "arch: bad header");
    a.dtype = d->dtype; a.in_h = d->in_h; a.in_w = d->in_w; a.in_c = d->in_c; a.n_classes = d->n_classes;
    struct Shape { int32_t h = 0, w = 0, c = 0; bool set = false; } shp[kMaxBufs];
    shp[0] = {d->in_h, d->in_w, d->in_c, true};
    size_t off = 0;
    const size_t eb = a.elem();
    auto take = [&](size_t n, bool param_dtype) {
        off = align_up(off);
        size_t o = off;
        off += n * (param_dtype ? eb : 4);
        return o;
    };
    for (int32_t i = 0; i < d->n_layers; ++i) {
        LayerPlan L{};
        L.d = d->layers[i];
        const coe_layer& l = L.d;
        if (l.src < 0 || l.src >= kMaxBufs || !shp[l.src].set) return fail(c, COE_EINVAL, "arch: layer reads an unset buffer");
        L.H = shp[l.src].h; L.W = shp[l.src].w; L.C = shp[l.src].c;
        bool is_head = l.op == COE_OP_HEAD || l.op == COE_OP_HEAD_CLS || l.op == COE_OP_HEAD_DET;
        if (!is_head && (l.dst <= 0 || l.dst >= kMaxBufs || l.dst == l.src))
            return fail(c, COE_EINVAL, "arch: bad destination buffer");
        if (is_head && i != d->n_layers - 1) return fail(c, COE_EINVAL, "arch: head must be the last layer");
        switch (l.op) {
        case COE_OP_CONV:
        case COE_OP_MAXPOOL: {
            if (l.r <= 0 || l.s <= 0 || l.stride <= 0 || l.pad < 0 || l.k <= 0) return fail(c, COE_EINVAL, "arch: bad conv/pool parameters");
            L.P = (L.H + 2 * l.pad - l.r) / l.stride + 1;
            L.Q = (L.W + 2 * l.pad - l.s) / l.stride + 1;
            L.K = l.k;
            if (L.P <= 0 || L.Q <= 0) return fail(c, COE_EINVAL, "arch: empty output");
            if (l.op == COE_OP_MAXPOOL) {
                if (l.k != L.C) return fail(c, COE_EINVAL, "arch: pool must keep channels");
                if (l.pad >= l.r || l.pad >= l.s) return fail(c, COE_EINVAL, "arch: pool padding must be smaller than the window");
            } else {
                L.off[0] = take((size_t)l.k * l.r * l.s * L.C, true);
                L.off[1] = take((size_t)l.k, false);
                L.macs = (double)L.P * L.Q * l.k * l.r * l.s * L.C;
                {
                    coe::k::ConvShape cs{1, L.H, L.W, L.C, l.k, l.r, l.s, l.stride, l.pad, L.P, L.Q, l.act};
                    L.packed = d->dtype == COE_DT_BF16 && coe::k::conv_mfma_supported(cs);
                    // non-overlapping windows of a few-channel image (patch embedding): a GEMM over gathered patches
                    const int red = l.r * l.s * L.C;
                    if (!L.packed && d->dtype == COE_DT_BF16 && l.stride == l.r && l.stride == l.s && l.pad == 0 && l.r > 1 &&
                        L.H % l.r == 0 && L.W % l.s == 0 && (l.s * L.C * 2) % 16 == 0 && l.res < 0) {
                        coe::k::ConvShape gs{1, L.P, L.Q, red, l.k, 1, 1, 1, 0, L.P, L.Q, l.act};
                        if (coe::k::conv_mfma_supported(gs)) {
                            L.packed = L.patchify = true;
                            a.patch_elems = std::max(a.patch_elems, (size_t)L.P * L.Q * red);
                        }
                    }
                }
                if (l.res >= 0) {
                    if (l.res >= kMaxBufs || !shp[l.res].set || l.res == l.dst || shp[l.res].h != L.P || shp[l.res].w != L.Q ||
                        shp[l.res].c != L.K)
                        return fail(c, COE_EINVAL, "arch: residual shape mismatch");
                }
                if (l.act < 0 || l.act > 3) return fail(c, COE_EINVAL, "arch: unknown activation");
            }
            break;
        }
        case COE_OP_HEAD:
            if (l.k != d->n_classes) return fail(c, COE_EINVAL, "arch: head width differs from n_classes");
            L.K = l.k;
            L.off[0] = take((size_t)l.k * L.C, true);
            L.off[1] = take((size_t)l.k, false);
            L.macs = (double)l.k * L.C;
            break;
        case COE_OP_TOKENS:
            if (d->dtype != COE_DT_BF16 || L.C % 8) return fail(c, COE_EINVAL, "arch: token ops need bf16 and channels % 8 == 0");
            L.P = L.H * L.W + 1; L.Q = 1; L.K = L.C;
            L.off[0] = take((size_t)L.C, true);
            L.off[1] = take((size_t)L.P * L.C, true);
            break;
        case COE_OP_LAYERNORM:
            if (d->dtype != COE_DT_BF16 || L.C % 2 || L.C > 2048)
                return fail(c, COE_EINVAL, "arch: layer norm needs bf16 and an even channel count <= 2048");
            L.P = L.H; L.Q = L.W; L.K = L.C;
            L.off[0] = take((size_t)L.C, false);
            L.off[1] = take((size_t)L.C, false);
            break;
        case COE_OP_ATTENTION:
            if (L.C % 3 || l.aux0 <= 0 || (L.C / 3) % l.aux0) return fail(c, COE_EINVAL, "arch: bad attention shape");
            L.P = L.H; L.Q = L.W; L.K = L.C / 3;
            if (d->dtype != COE_DT_BF16 || !coe::k::attention_supported(L.H * L.W, L.C / 3, l.aux0))
                return fail(c, COE_EINVAL, "arch: attention needs bf16, head width 64 and at most 224 tokens");
            L.macs = 2.0 * L.H * L.W * L.H * L.W * (L.C / 3);
            break;
        case COE_OP_HEAD_CLS:
            if (l.k != d->n_classes) return fail(c, COE_EINVAL, "arch: head width differs from n_classes");
            if (d->dtype != COE_DT_BF16) return fail(c, COE_EINVAL, "arch: class-token head needs bf16");
            L.K = l.k;
            L.off[0] = take((size_t)L.C, false);
            L.off[1] = take((size_t)L.C, false);
            L.off[2] = take((size_t)l.k * L.C, true);
            L.off[3] = take((size_t)l.k, false);
            L.macs = (double)l.k * L.C;
            break;
        case COE_OP_CONCAT:
            if (d->dtype != COE_DT_BF16) return fail(c, COE_EINVAL, "arch: concatenation needs bf16");
            if (l.res < 0 || l.res >= kMaxBufs || !shp[l.res].set || l.res == l.dst || shp[l.res].h != L.H || shp[l.res].w != L.W)
                return fail(c, COE_EINVAL, "arch: concatenation of different sizes");
            if (L.C % 8 || shp[l.res].c % 8) return fail(c, COE_EINVAL, "arch: concatenated channel counts must be multiples of 8");
            L.P = L.H; L.Q = L.W; L.K = L.C + shp[l.res].c;
            if (l.k != L.K) return fail(c, COE_EINVAL, "arch: concatenation width differs from the sum of its inputs");
            break;
        case COE_OP_UPSAMPLE:
            if (d->dtype != COE_DT_BF16 || L.C % 8) return fail(c, COE_EINVAL, "arch: upsampling needs bf16 and channels % 8 == 0");
            L.P = 2 * L.H; L.Q = 2 * L.W; L.K = L.C;
            break;
        case COE_OP_HEAD_DET:
            if (l.k != d->n_classes) return fail(c, COE_EINVAL, "arch: head width differs from n_classes");
            if (d->dtype != COE_DT_BF16 || l.aux0 <= 0 || L.C != l.aux0 * (5 + l.k) || l.k > 251)
                return fail(c, COE_EINVAL, "arch: detection head needs bf16 maps of anchors x (5 + classes) channels, at most 251 classes");
            if (l.res >= 0 && (l.res >= kMaxBufs || !shp[l.res].set || shp[l.res].c != L.C))
                return fail(c, COE_EINVAL, "arch: second detection map has another layout");
            L.K = l.k;
            L.P = l.res >= 0 ? shp[l.res].h * shp[l.res].w : 0;        // positions of the second map
            break;
        default:
            return fail(c, COE_EINVAL, "arch: unknown op");
        }
        if (!is_head) shp[l.dst] = {L.P, L.Q, L.K, true};
        a.layers.push_back(L);
    }
    int last = a.layers.back().d.op;
    if (last != COE_OP_HEAD && last != COE_OP_HEAD_CLS && last != COE_OP_HEAD_DET)
        return fail(c, COE_EINVAL, "arch: program must end in a head");
    // few-channel conv followed by a 3x3/2 pad-1 max pool of its output, which nobody else reads: one fused kernel
    for (size_t i = 0; i + 1 < a.layers.size(); ++i) {
        LayerPlan& cv = a.layers[i];
        LayerPlan& pl = a.layers[i + 1];
        if (a.dtype != COE_DT_BF16 || cv.d.op != COE_OP_CONV || cv.packed || cv.d.res >= 0 || pl.d.op != COE_OP_MAXPOOL) continue;
        if (pl.d.src != cv.d.dst || pl.d.r != 3 || pl.d.s != 3 || pl.d.stride != 2 || pl.d.pad != 1) continue;
        coe::k::ConvShape cs{1, cv.H, cv.W, cv.C, cv.K, cv.d.r, cv.d.s, cv.d.stride, cv.d.pad, cv.P, cv.Q, cv.d.act};
        if (!coe::k::conv_smallc_supported(cs, false, true)) continue;
        bool read_later = false;
        for (size_t j = i + 2; j < a.layers.size(); ++j) {
            if (a.layers[j].d.src == cv.d.dst || a.layers[j].d.res == cv.d.dst) { read_later = true; break; }
            if (a.layers[j].d.dst == cv.d.dst) break;       // overwritten before anyone reads it
        }
        if (read_later) continue;
        cv.fuse_pool = true;
        pl.fused_away = true;
    }
    // activation buffers per request: what the launched kernels write (a conv fused with its pool writes the pool's output)
    for (const LayerPlan& L : a.layers) {
        const int op = L.d.op;
        if (op == COE_OP_HEAD || op == COE_OP_HEAD_CLS || op == COE_OP_HEAD_DET || L.fuse_pool) continue;
        a.buf_elems[L.d.dst] = std::max(a.buf_elems[L.d.dst], (size_t)L.P * L.Q * L.K);
    }
    a.blob_bytes = align_up(off);
    {
        size_t widest = a.in_bytes();
        for (int b = 1; b < kMaxBufs; ++b) widest = std::max(widest, a.buf_elems[b] * a.elem());
        widest = std::max(widest, a.patch_elems * a.elem());
        a.row_cap = (int32_t)std::min<size_t>((size_t)INT32_MAX, (size_t)0x7FFFFFFE / widest);
        if (a.row_cap < 1) return fail(c, COE_EINVAL, "arch: one request's largest tensor exceeds 2 GiB");
    }
    // request arranging's gather can happen inside the first kernel when that is the few-channel conv and nothing else
    // reads the input
    {
        int readers = 0;
        for (const LayerPlan& L : a.layers) readers += (L.d.src == 0) + (L.d.res == 0);
        const LayerPlan& L0 = a.layers[0];
        coe::k::ConvShape cs{1, L0.H, L0.W, L0.C, L0.K, L0.d.r, L0.d.s, L0.d.stride, L0.d.pad, L0.P, L0.Q, L0.d.act};
        a.gathers_input = readers == 1 && L0.d.op == COE_OP_CONV && L0.d.src == 0 && a.dtype == COE_DT_BF16 && !L0.packed &&
                          (L0.fuse_pool || coe::k::conv_smallc_supported(cs, L0.d.res >= 0, false));
    }
    // grouped launches: matrix-core convs with K % 64 == 0 take a group table; few-channel convs run once per group;
    // pools have no weights; the pooled head takes a group table.  Anything else keeps one launch per group.
    a.groupable = a.dtype == COE_DT_BF16;
    for (const LayerPlan& L : a.layers) {
        const coe_layer& l = L.d;
        coe::k::ConvShape cs{1, L.H, L.W, L.C, L.K, l.r, l.s, l.stride, l.pad, L.P, L.Q, l.act};
        const bool reads_input = l.src == 0 || l.res == 0;
        if (reads_input && !(l.op == COE_OP_CONV && !L.packed && l.res != 0)) a.groupable = false;   // only the per-group stem may
        if (l.op == COE_OP_CONV) {
            if (L.patchify) a.groupable = false;
            else if (L.packed) a.groupable = a.groupable && coe::k::conv_mfma_groupable(cs);
            else if (!L.fuse_pool && !coe::k::conv_smallc_supported(cs, l.res >= 0, false)) a.groupable = false;
        } else if (l.op != COE_OP_MAXPOOL && l.op != COE_OP_HEAD) {
            a.groupable = false;
        }
    }
    return COE_OK;
}

// ---- device memory helpers -----------------------------------------------------------------------------------------
hipError_t dev_malloc(coe_ctx* c, void** p, size_t bytes)
{
    ++c->device_allocs;
    return hipMalloc(p, bytes);
}

int ensure_store(coe_ctx* c)
{
    if (c->archs.empty()) return fail(c, COE_ESTATE, "no architecture registered");
    size_t nreq = (size_t)c->cfg.max_requests;
    if (!c->d_inputs) {
        size_t ib = c->archs[0].in_bytes();
        HIPCHK(c, dev_malloc(c, &c->d_inputs, nreq * ib));
        HIPCHK(c, dev_malloc(c, &c->d_staged, nreq * ib));
    }
    if (c->logits_alloc_classes < c->max_classes) {
        if (c->n_live > 0) return fail(c, COE_ESTATE, "architecture with more classes registered while requests are live");
        if (c->d_logits) HIPCHK(c, hipFree(c->d_logits));
        HIPCHK(c, dev_malloc(c, (void**)&c->d_logits, nreq * c->max_classes * sizeof(float)));
        c->logits_alloc_classes = c->max_classes;
    }
    return COE_OK;
}

// requests per launch sequence of an architecture: the configured maximum batch, cut where a tensor would outgrow the
// kernels' 31-bit byte offsets
int32_t chunk_rows(const coe_ctx* c, const ArchPlan& a) { return std::min(c->cfg.max_batch, a.row_cap); }

int ensure_workspace(coe_ctx* c)
{
    for (Lane& ln : c->lanes) {
        for (int b = 1; b < kMaxBufs; ++b) {
            size_t need = 0;
            for (const ArchPlan& a : c->archs) need = std::max(need, a.buf_elems[b] * a.elem() * (size_t)chunk_rows(c, a));
            if (need > ln.buf_bytes[b]) {
                HIPCHK(c, hipStreamSynchronize(ln.s));
                if (ln.d_buf[b]) HIPCHK(c, hipFree(ln.d_buf[b]));
                ln.d_buf[b] = nullptr;
                HIPCHK(c, dev_malloc(c, &ln.d_buf[b], need));
                ln.buf_bytes[b] = need;
            }
        }
        size_t need = 0;
        for (const ArchPlan& a : c->archs) need = std::max(need, a.patch_elems * a.elem() * (size_t)chunk_rows(c, a));
        if (need > ln.patch_bytes) {
            HIPCHK(c, hipStreamSynchronize(ln.s));
            if (ln.d_patch) HIPCHK(c, hipFree(ln.d_patch));
            ln.d_patch = nullptr;
            HIPCHK(c, dev_malloc(c, &ln.d_patch, need));
            ln.patch_bytes = need;
        }
    }
    return COE_OK;
}

// The arena: per size class as many slots as the caps let be resident at once (all experts of the class when there is no
// cap).  Called once, when the dependency graph is set and every expert is known.
int build_arena(coe_ctx* c)
{
    std::vector<size_t> class_bytes;
    std::vector<int32_t> members;
    for (Expert& x : c->experts) {
        size_t k = 0;
        while (k < class_bytes.size() && class_bytes[k] != x.nbytes) ++k;
        if (k == class_bytes.size()) { class_bytes.push_back(x.nbytes); members.push_back(0); }
        x.cls = (int32_t)k;
        ++members[k];
    }
    std::vector<int32_t> n_slots(class_bytes.size());
    size_t total = 0;
    for (size_t k = 0; k < class_bytes.size(); ++k) {
        int64_t n = members[k];
        if (c->cfg.cache_cap_experts > 0) n = std::min<int64_t>(n, c->cfg.cache_cap_experts);
        if (c->cfg.cache_cap_bytes > 0) n = std::min<int64_t>(n, c->cfg.cache_cap_bytes / (int64_t)class_bytes[k]);
        n_slots[k] = (int32_t)n;
        total += (size_t)n * align_up(class_bytes[k]);
    }
    if (total > 0 && dev_malloc(c, &c->arena, total) != hipSuccess) {
        (void)hipGetLastError();
        c->arena = nullptr;
        return fail(c, COE_ENOMEM, "device allocation of the expert arena failed");
    }
    size_t n_total = 0;
    for (int32_t n : n_slots) n_total += (size_t)n;
    c->slots.resize(n_total);
    c->free_slots.assign(class_bytes.size(), {});
    size_t off = 0, i = 0;
    for (size_t k = 0; k < class_bytes.size(); ++k)
        for (int32_t j = 0; j < n_slots[k]; ++j, ++i) {
            DevBuf& b = c->slots[i];
            b.p = (uint8_t*)c->arena + off;
            b.bytes = class_bytes[k];
            b.cls = (int32_t)k;
            off += align_up(class_bytes[k]);
            HIPCHK(c, hipEventCreateWithFlags(&b.last_use, hipEventDisableTiming));
            c->free_slots[k].push_back(&b);
        }
    return COE_OK;
}

// A free slot of the class: the one released longest ago (its last reader is the most likely to have finished).  The
// policy evicts before it loads, so the class always has one.
int acquire_buf(coe_ctx* c, int32_t cls, DevBuf** out)
{
    std::vector<DevBuf*>& fl = c->free_slots[cls];
    if (fl.empty()) return fail(c, COE_ESTATE, "internal: no free arena slot for an expert the policy admitted");
    *out = fl.front();
    fl.erase(fl.begin());
    return COE_OK;
}

void release_expert(coe_ctx* c, int32_t v)
{
    Expert& x = c->experts[v];
    if (x.buf) {
        c->free_slots[x.buf->cls].push_back(x.buf);
        x.buf = nullptr;
    }
    x.load_pending = false;
}

// ---- host tier --------------------------------------------------------------------------------------------------------
int build_host_arena(coe_ctx* c)
{
    // size classes are the device arena's (build_arena ran first)
    std::vector<size_t> class_bytes(c->free_slots.size(), 0);
    std::vector<int32_t> members(c->free_slots.size(), 0);
    for (const Expert& x : c->experts) { class_bytes[x.cls] = x.nbytes; ++members[x.cls]; }
    size_t n_total = 0;
    for (int32_t m : members) n_total += (size_t)std::min(m, c->host_cap);
    c->hslots.resize(n_total);
    c->free_hslots.assign(class_bytes.size(), {});
    size_t i = 0;
    for (size_t k = 0; k < class_bytes.size(); ++k)
        for (int32_t j = 0; j < std::min(members[k], c->host_cap); ++j, ++i) {
            HostSlot& h = c->hslots[i];
            h.cls = (int32_t)k;
            if (hipHostMalloc(&h.p, class_bytes[k], hipHostMallocDefault) != hipSuccess) {
                (void)hipGetLastError();
                h.p = nullptr;
                return fail(c, COE_ENOMEM, "pinned host allocation of the host tier failed");
            }
            HIPCHK(c, hipEventCreateWithFlags(&h.copied, hipEventDisableTiming));
            c->free_hslots[k].push_back(&h);
        }
    return COE_OK;
}

// The loader thread: reads in the order the jobs were queued.  A slot is overwritten only after every copy out of it that
// was planned before the read has been enqueued by the stepping thread and has completed on the copy stream.
void loader_main(coe_ctx* c)
{
    (void)hipSetDevice(c->cfg.device);
    for (;;) {
        ReadJob* j = nullptr;
        {
            std::unique_lock<std::mutex> lk(c->ld_mutex);
            c->ld_cv.wait(lk, [&] { return c->ld_stop || !c->ld_queue.empty(); });
            if (c->ld_queue.empty()) return;             // stop requested and nothing left to do
            j = c->ld_queue.front();
            c->ld_cv.wait(lk, [&] { return c->ld_stop || j->slot->issued >= j->need_issued; });
            if (j->slot->issued < j->need_issued) { j->rc = COE_ESTATE; j->done = true; c->ld_queue.pop_front(); c->ld_cv.notify_all(); continue; }
        }
        int rc = COE_OK;
        if (j->need_issued > 0 && hipEventSynchronize(j->slot->copied) != hipSuccess) rc = COE_EDEVICE;
        auto t0 = std::chrono::steady_clock::now();
        size_t done = 0;
        while (rc == COE_OK && done < j->nbytes) {
            ssize_t got = pread(c->fd, (uint8_t*)j->slot->p + done, j->nbytes - done, (off_t)(j->file_off + (int64_t)done));
            if (got <= 0) rc = COE_EIO;
            else done += (size_t)got;
        }
        const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
        {
            std::lock_guard<std::mutex> lk(c->ld_mutex);
            j->rc = rc;
            j->read_us = us;
            j->done = true;
            c->ld_queue.pop_front();
        }
        c->ld_cv.notify_all();
    }
}

// Give expert x the oldest free host slot of its class and queue the read of its blob into it.
int queue_read(coe_ctx* c, Expert& x, coe_step_stats* st, ReadJob** job)
{
    std::vector<HostSlot*>& fl = c->free_hslots[x.cls];
    if (fl.empty()) return fail(c, COE_ESTATE, "internal: no free host slot for an expert the host policy admitted");
    HostSlot* h = fl.front();
    fl.erase(fl.begin());
    x.hslot = h;
    c->ld_jobs.emplace_back();
    ReadJob& j = c->ld_jobs.back();
    j.slot = h;
    j.file_off = x.file_off;
    j.nbytes = x.nbytes;
    j.need_issued = h->planned;
    {
        std::lock_guard<std::mutex> lk(c->ld_mutex);
        c->ld_queue.push_back(&j);
    }
    c->ld_cv.notify_all();
    *job = &j;
    if (st) {
        ++st->n_host_misses;
        st->bytes_read += (int64_t)x.nbytes;
    }
    return COE_OK;
}

// The host tier serves one device switch (a request to the level below): a hit needs nothing; a miss evicts by the tier's
// own policy, takes a free slot and queues the read.  *job receives the read the switch has to wait for (null on a hit),
// *src the slot the switch copies from (a later switch of the same step may take the expert out of the host tier again, so
// the expert itself does not remember it).  Policy, log and slot lists change here, on the stepping thread, in switch
// order; only the bytes move on the loader thread.
int host_plan(coe_ctx* c, int32_t e, coe_step_stats* st, ReadJob** job, HostSlot** src)
{
    *job = nullptr;
    *src = nullptr;
    Expert& x = c->experts[e];
    std::vector<uint8_t> need(c->experts.size(), 0);
    need[e] = 1;
    std::vector<int32_t> order;
    std::vector<coe::Switch> sws;
    if (!c->host_policy->plan_stage(need.data(), order, sws)) return fail(c, COE_ENOMEM, "an expert does not fit the host tier");
    for (const coe::Switch& sw : sws) {          // none (hit) or one (miss)
        c->host_log.push_back(sw.expert);
        c->host_log.push_back((int32_t)sw.victims.size());
        for (int32_t v : sw.victims) {
            c->host_log.push_back(v);
            Expert& xv = c->experts[v];
            if (xv.hslot) {
                c->free_hslots[xv.hslot->cls].push_back(xv.hslot);
                xv.hslot = nullptr;
            }
        }
        int rc = queue_read(c, x, st, job);
        if (rc) return rc;
    }
    if (!x.hslot) return fail(c, COE_ESTATE, "internal: the host tier lost an expert it reported resident");
    ++x.hslot->planned;
    *src = x.hslot;
    return COE_OK;
}

// Block until a queued read has finished; its time goes into the step's statistics.
int host_wait(coe_ctx* c, ReadJob* j, coe_step_stats* st)
{
    std::unique_lock<std::mutex> lk(c->ld_mutex);
    c->ld_cv.wait(lk, [&] { return j->done; });
    if (st) st->read_us += j->read_us;
    if (j->rc == COE_EIO) return fail(c, COE_EIO, "reading an expert from the backing file failed");
    if (j->rc) return fail(c, j->rc, "the loader thread could not serve a read");
    return COE_OK;
}

// Enqueue one expert switch on the copy stream: victims leave, the expert's blob is copied into a device buffer.
// st counts the switch; read_st (if the host tier has to read the blob first) counts the read.  planned: the host tier has
// already been asked for this switch (host_plan) and `job` is the read to wait for, if any.
int issue_load(coe_ctx* c, const coe::Switch& sw, coe_step_stats* st, coe_step_stats* read_st, bool planned = false,
               ReadJob* job = nullptr, HostSlot* hs = nullptr)
{
    c->switch_log.push_back(sw.expert);
    c->switch_log.push_back((int32_t)sw.victims.size());
    for (int32_t v : sw.victims) {
        c->switch_log.push_back(v);
        release_expert(c, v);
    }
    Expert& x = c->experts[sw.expert];
    DevBuf* b = nullptr;
    int rc = acquire_buf(c, x.cls, &b);
    if (rc) return rc;
    const void* src = x.host;
    if (c->host_cap > 0) {
        if (!planned) rc = host_plan(c, sw.expert, read_st, &job, &hs);
        if (rc == COE_OK && job) rc = host_wait(c, job, read_st);
        if (rc) { c->free_slots[x.cls].insert(c->free_slots[x.cls].begin(), b); return rc; }
        src = hs->p;
    }
    // the buffer may still be read by kernels of its previous owner
    if (b->used) HIPCHK(c, hipStreamWaitEvent(c->sx, b->last_use, 0));
    {
        Span sp(c, COE_K_SWITCH, (double)x.nbytes, c->sx);
        HIPCHK(c, hipMemcpyAsync(b->p, src, x.nbytes, hipMemcpyHostToDevice, c->sx));
    }
    HIPCHK(c, hipEventRecord(x.loaded, c->sx));
    if (hs) {
        HIPCHK(c, hipEventRecord(hs->copied, c->sx));
        {
            std::lock_guard<std::mutex> lk(c->ld_mutex);
            ++hs->issued;
        }
        c->ld_cv.notify_all();
    }
    x.buf = b;
    x.load_pending = true;
    if (st) {
        st->n_evictions += (int32_t)sw.victims.size();
        st->bytes_switched += (int64_t)x.nbytes;
    }
    return COE_OK;
}

// ---- one expert over one batch ---------------------------------------------------------------------------------------
// rows: the batch is rows[0..n) of the array at `input` (only for architectures whose first kernel follows a row table)
int run_expert(coe_ctx* c, Lane& ln, const Expert& x, const void* weights, const void* input, int32_t n,
               const coe::k::RouteArgs& route, int32_t last_layer = -1, const int32_t* rows = nullptr)
{
    int32_t li = -1;
    const ArchPlan& a = c->archs[x.arch];
    const uint8_t* wb = (const uint8_t*)weights;
    auto buf = [&](int id) -> void* { return id == 0 ? const_cast<void*>(input) : ln.d_buf[id]; };
    for (const LayerPlan& L : a.layers) {
        const coe_layer& l = L.d;
        if (last_layer >= 0 && ++li > last_layer) break;
        switch (l.op) {
        case COE_OP_CONV: {
            coe::k::ConvShape s{n, L.H, L.W, L.C, L.K, l.r, l.s, l.stride, l.pad, L.P, L.Q, l.act};
            const void* res = l.res >= 0 ? buf(l.res) : nullptr;
            double flops = 2.0 * L.macs * n;
            if (L.patchify) {
                {
                    double bytes = 2.0 * n * (double)L.H * L.W * L.C * a.elem();
                    Span sp(c, COE_K_TOKEN_OPS, bytes, ln.s);
                    HIPCHK(c, coe::k::patchify(buf(l.src), ln.d_patch, n, L.H, L.W, L.C, l.r, l.s, ln.s));
                }
                coe::k::ConvShape g{n, L.P, L.Q, l.r * l.s * L.C, L.K, 1, 1, 1, 0, L.P, L.Q, l.act};
                Span sp(c, COE_K_CONV_MFMA, flops, ln.s);
                HIPCHK(c, coe::k::conv_mfma(ln.d_patch, wb + L.off[0], (const float*)(wb + L.off[1]), nullptr, buf(l.dst), g, ln.s));
            } else if (L.packed) {
                Span sp(c, coe::k::conv_mfma_uses_slab(s) ? COE_K_CONV_SLAB : COE_K_CONV_MFMA, flops, ln.s);
                HIPCHK(c, coe::k::conv_mfma(buf(l.src), wb + L.off[0], (const float*)(wb + L.off[1]), res, buf(l.dst), s, ln.s));
            } else if (L.fuse_pool) {
                const LayerPlan& pool = *(&L + 1);
                Span sp(c, COE_K_CONV_STEM, flops, ln.s);
                HIPCHK(c, coe::k::conv_smallc(buf(l.src), wb + L.off[0], (const float*)(wb + L.off[1]), buf(pool.d.dst), s, true, ln.s,
                                              l.src == 0 ? rows : nullptr));
            } else if (a.dtype == COE_DT_BF16 && coe::k::conv_smallc_supported(s, res != nullptr, false)) {
                Span sp(c, COE_K_CONV_STEM, flops, ln.s);
                HIPCHK(c, coe::k::conv_smallc(buf(l.src), wb + L.off[0], (const float*)(wb + L.off[1]), buf(l.dst), s, false, ln.s,
                                              l.src == 0 ? rows : nullptr));
            } else {
                Span sp(c, COE_K_CONV_DIRECT, flops, ln.s);
                HIPCHK(c, coe::k::conv_direct(a.dtype, buf(l.src), wb + L.off[0], (const float*)(wb + L.off[1]), res, buf(l.dst), s, ln.s));
            }
            break;
        }
        case COE_OP_MAXPOOL: {
            if (L.fused_away) break;
            double bytes = (double)n * ((double)L.H * L.W * L.C + (double)L.P * L.Q * L.K) * a.elem();
            Span sp(c, COE_K_POOL, bytes, ln.s);
            HIPCHK(c, coe::k::maxpool(a.dtype, buf(l.src), buf(l.dst), n, L.H, L.W, L.C, l.r, l.s, l.stride, l.pad, L.P, L.Q, ln.s));
            break;
        }
        case COE_OP_HEAD: {
            double bytes = (double)n * L.H * L.W * L.C * a.elem();
            Span sp(c, COE_K_HEAD, bytes, ln.s);
            HIPCHK(c, coe::k::head_gap_fc(a.dtype, buf(l.src), wb + L.off[0], (const float*)(wb + L.off[1]), n, L.H * L.W, L.C, L.K,
                                          route, ln.s));
            break;
        }
        case COE_OP_TOKENS: {
            double bytes = (double)n * ((double)L.H * L.W + L.P) * L.C * a.elem();
            Span sp(c, COE_K_TOKEN_OPS, bytes, ln.s);
            HIPCHK(c, coe::k::tokens(buf(l.src), wb + L.off[0], wb + L.off[1], buf(l.dst), n, L.P, L.C, ln.s));
            break;
        }
        case COE_OP_LAYERNORM: {
            double bytes = 2.0 * n * (double)L.H * L.W * L.C * a.elem();
            Span sp(c, COE_K_TOKEN_OPS, bytes, ln.s);
            HIPCHK(c, coe::k::layernorm(buf(l.src), (const float*)(wb + L.off[0]), (const float*)(wb + L.off[1]), buf(l.dst),
                                        (int64_t)n * L.H * L.W, L.C, ln.s));
            break;
        }
        case COE_OP_ATTENTION: {
            Span sp(c, COE_K_ATTENTION, 2.0 * L.macs * n, ln.s);
            HIPCHK(c, coe::k::attention(buf(l.src), buf(l.dst), n, L.H * L.W, L.K, l.aux0, ln.s));
            break;
        }
        case COE_OP_CONCAT: {
            const int32_t cb = L.K - L.C;
            double bytes = 2.0 * n * (double)L.H * L.W * L.K * a.elem();
            Span sp(c, COE_K_TOKEN_OPS, bytes, ln.s);
            HIPCHK(c, coe::k::concat_channels(buf(l.src), buf(l.res), buf(l.dst), (int64_t)n * L.H * L.W, L.C, cb, ln.s));
            break;
        }
        case COE_OP_UPSAMPLE: {
            double bytes = 5.0 * n * (double)L.H * L.W * L.C * a.elem();
            Span sp(c, COE_K_TOKEN_OPS, bytes, ln.s);
            HIPCHK(c, coe::k::upsample2(buf(l.src), buf(l.dst), n, L.H, L.W, L.C, ln.s));
            break;
        }
        case COE_OP_HEAD_DET: {
            double bytes = (double)n * ((double)L.H * L.W + L.P) * L.C * a.elem();
            Span sp(c, COE_K_HEAD, bytes, ln.s);
            HIPCHK(c, coe::k::head_det(buf(l.src), L.H * L.W, l.res >= 0 ? buf(l.res) : nullptr, L.P, n, l.aux0, L.K, route, ln.s));
            break;
        }
        case COE_OP_HEAD_CLS: {
            double bytes = (double)n * L.C * a.elem();
            Span sp(c, COE_K_HEAD, bytes, ln.s);
            HIPCHK(c, coe::k::head_cls(buf(l.src), (const float*)(wb + L.off[0]), (const float*)(wb + L.off[1]), wb + L.off[2],
                                       (const float*)(wb + L.off[3]), n, L.H * L.W, L.C, L.K, route, ln.s));
            break;
        }
        default:
            return fail(c, COE_EINVAL, "unknown layer op");
        }
    }
    return COE_OK;
}

// ---- several small groups, experts of one architecture, one launch per layer -------------------------------------------------
struct SetMember {
    int32_t expert;
    int32_t first;       // first request of the group in the group-contiguous order
    int32_t count;
};

// rows: as in run_expert; the members' inputs are rows[first..first+count) of the array at `staged`
int run_group_set(coe_ctx* c, Lane& ln, const std::vector<SetMember>& set, const uint8_t* staged, size_t ib, const int32_t* rows)
{
    const ArchPlan& a = c->archs[c->experts[set[0].expert].arch];
    coe::k::GroupTable gt{};
    coe::k::GroupRoutes gr{};
    gt.n = (int32_t)set.size();
    int32_t n = 0;
    for (size_t g = 0; g < set.size(); ++g) {
        const Expert& x = c->experts[set[g].expert];
        gt.first_row[g] = n;
        gt.weights[g] = x.buf->p;
        gr.expert[g] = set[g].expert;
        gr.succ_off[g] = c->succ_off[set[g].expert];
        gr.n_route[g] = c->succ_off[set[g].expert + 1] - c->succ_off[set[g].expert];
        gr.slot_off[g] = set[g].first;
        n += set[g].count;
    }
    gt.first_row[set.size()] = n;
    auto buf = [&](int id) -> uint8_t* { return (uint8_t*)ln.d_buf[id]; };
    for (const LayerPlan& L : a.layers) {
        const coe_layer& l = L.d;
        switch (l.op) {
        case COE_OP_CONV: {
            coe::k::ConvShape s{n, L.H, L.W, L.C, L.K, l.r, l.s, l.stride, l.pad, L.P, L.Q, l.act};
            double flops = 2.0 * L.macs * n;
            if (L.packed) {
                if (l.src == 0) return fail(c, COE_ESTATE, "internal: grouped matrix-core conv on the raw input");
                const void* res = l.res >= 0 ? buf(l.res) : nullptr;
                Span sp(c, coe::k::conv_mfma_uses_slab(s) ? COE_K_CONV_SLAB : COE_K_CONV_MFMA, flops, ln.s);
                HIPCHK(c, coe::k::conv_mfma_grouped(buf(l.src), gt, L.off[0], L.off[1], res, buf(l.dst), s, ln.s));
            } else {
                // few input channels (the stem): the filters live in LDS for a whole launch, so one launch per group,
                // each writing its rows of the shared activation buffer
                const bool fused = L.fuse_pool;
                const LayerPlan& outL = fused ? *(&L + 1) : L;
                const size_t in_row = (size_t)L.H * L.W * L.C * a.elem();
                const size_t out_row = (size_t)outL.P * outL.Q * outL.K * a.elem();
                Span sp(c, COE_K_CONV_STEM, flops, ln.s);
                for (size_t g = 0; g < set.size(); ++g) {
                    coe::k::ConvShape sg = s;
                    sg.N = set[g].count;
                    const bool via_rows = l.src == 0 && rows;
                    const uint8_t* in = via_rows ? staged
                                      : l.src == 0 ? staged + (size_t)set[g].first * ib : buf(l.src) + (size_t)gt.first_row[g] * in_row;
                    const uint8_t* wb = (const uint8_t*)gt.weights[g];
                    HIPCHK(c, coe::k::conv_smallc(in, wb + L.off[0], (const float*)(wb + L.off[1]),
                                                  buf(outL.d.dst) + (size_t)gt.first_row[g] * out_row, sg, fused, ln.s,
                                                  via_rows ? rows + set[g].first : nullptr));
                }
            }
            break;
        }
        case COE_OP_MAXPOOL: {
            if (L.fused_away) break;
            if (l.src == 0) return fail(c, COE_ESTATE, "internal: grouped pool on the raw input");
            double bytes = (double)n * ((double)L.H * L.W * L.C + (double)L.P * L.Q * L.K) * a.elem();
            Span sp(c, COE_K_POOL, bytes, ln.s);
            HIPCHK(c, coe::k::maxpool(a.dtype, buf(l.src), buf(l.dst), n, L.H, L.W, L.C, l.r, l.s, l.stride, l.pad, L.P, L.Q, ln.s));
            break;
        }
        case COE_OP_HEAD: {
            if (l.src == 0) return fail(c, COE_ESTATE, "internal: grouped head on the raw input");
            double bytes = (double)n * L.H * L.W * L.C * a.elem();
            coe::k::RouteArgs r{c->d_perm, 0, c->d_succ, 0, c->d_cur, c->d_depth, c->d_path, c->cfg.max_stages, c->d_logits,
                                c->max_classes};
            Span sp(c, COE_K_HEAD, bytes, ln.s);
            HIPCHK(c, coe::k::head_gap_fc_grouped(a.dtype, buf(l.src), gt, L.off[0], L.off[1], n, L.H * L.W, L.C, L.K, r, gr, ln.s));
            break;
        }
        default:
            return fail(c, COE_ESTATE, "internal: architecture is not groupable");
        }
    }
    return COE_OK;
}

int do_init_fill(coe_ctx* c, coe_step_stats* st)
{
    if (c->filled) return COE_OK;
    if (c->host_cap > 0) {
        // the host tier fills first (descending usage probability), then serves the device's fill
        for (int32_t e : c->host_policy->init_fill()) {
            c->host_log.push_back(e);
            c->host_log.push_back(0);
            ReadJob* job = nullptr;
            int rc = queue_read(c, c->experts[e], st, &job);
            if (rc == COE_OK) rc = host_wait(c, job, st);
            if (rc) return rc;
        }
    }
    std::vector<int32_t> loaded = c->policy->init_fill();
    for (int32_t e : loaded) {
        coe::Switch sw{e, {}};
        int rc = issue_load(c, sw, nullptr, st);
        if (rc) return rc;
    }
    c->filled = true;
    return COE_OK;
}

}  // namespace

// =====================================================================================================================
extern "C" {

static_assert(COE_STATIC_SCRATCH_BYTES == sizeof(int32_t) * (size_t)coe::k::kRegroupStaticInts, "header and kernel agree on the scratch size");

// message of the last failed call that takes no context (per thread)
static thread_local std::string g_err;

const char* coe_last_error(const coe_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

int coe_regroup_static(int32_t n, const int32_t* cur, int32_t n_experts, int32_t* cnt, int32_t* off, int32_t* perm, int32_t* inv,
                       void* stream)
{
    auto bad = [](int code, const std::string& msg) { g_err = msg; return code; };
    if (n < 0 || (n > 0 && (!cur || !perm || !inv)) || !cnt || !off) return bad(COE_EINVAL, "coe_regroup_static: null or negative argument");
    if (n_experts <= 0 || n_experts > coe::k::kRegroupMaxExperts)
        return bad(COE_EINVAL, "coe_regroup_static: n_experts must be in 1.." + std::to_string(coe::k::kRegroupMaxExperts));
    const long long nblocks = ((long long)n + coe::k::kRegroupTile - 1) / coe::k::kRegroupTile;
    if (nblocks * n_experts > (long long)coe::k::kRegroupStaticInts)
        return bad(COE_ERANGE, "coe_regroup_static: ceil(n / " + std::to_string(coe::k::kRegroupTile) + ") * n_experts = " +
                                   std::to_string(nblocks * n_experts) + " exceeds the static scratch of " +
                                   std::to_string(coe::k::kRegroupStaticInts) + " entries (COE_STATIC_SCRATCH_BYTES)");
    hipError_t e = coe::k::regroup_index_static(cur, n, n_experts, cnt, off, perm, inv, (hipStream_t)stream);
    if (e != hipSuccess) return bad(COE_EDEVICE, std::string("coe_regroup_static: ") + hipGetErrorString(e));
    return COE_OK;
}

int coe_create(const coe_config* cfg, coe_ctx** out)
{
    if (!cfg || !out) return COE_EINVAL;
    *out = nullptr;
    if (cfg->max_requests <= 0 || cfg->max_stages <= 0 || cfg->max_batch < 0 || cfg->cache_cap_experts < 0 || cfg->cache_cap_bytes < 0)
        return COE_EINVAL;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0 || cfg->device < 0 || cfg->device >= ndev) {
        (void)hipGetLastError();
        return COE_EDEVICE;
    }
    if (hipSetDevice(cfg->device) != hipSuccess) return COE_EDEVICE;
    coe_ctx* c = new (std::nothrow) coe_ctx();
    if (!c) return COE_ENOMEM;
    c->cfg = *cfg;
    if (c->cfg.max_batch == 0) c->cfg.max_batch = 256;
    auto bail = [&](int code) { coe_destroy(c); return code; };
    if (cfg->compute_stream) c->sc = (hipStream_t)cfg->compute_stream;
    else { if (hipStreamCreateWithFlags(&c->sc, hipStreamNonBlocking) != hipSuccess) return bail(COE_EDEVICE); c->own_sc = true; }
    if (cfg->copy_stream) c->sx = (hipStream_t)cfg->copy_stream;
    else { if (hipStreamCreateWithFlags(&c->sx, hipStreamNonBlocking) != hipSuccess) return bail(COE_EDEVICE); c->own_sx = true; }
    if (cfg->executors < 0 || cfg->executors > kMaxLanes) { coe_destroy(c); return COE_EINVAL; }
    c->lanes.resize(std::max(1, cfg->executors));
    c->lanes[0].s = c->sc;
    for (size_t l = 1; l < c->lanes.size(); ++l)
        if (hipStreamCreateWithFlags(&c->lanes[l].s, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&c->lanes[l].done, hipEventDisableTiming) != hipSuccess)
            return bail(COE_EDEVICE);
    if (hipEventCreateWithFlags(&c->ev_ready, hipEventDisableTiming) != hipSuccess) return bail(COE_EDEVICE);
    size_t nreq = (size_t)cfg->max_requests;
    size_t nblocks = (nreq + coe::k::kRegroupTile - 1) / coe::k::kRegroupTile;
    bool ok = hipMalloc((void**)&c->d_cur, nreq * 4) == hipSuccess && hipMalloc((void**)&c->d_depth, nreq * 4) == hipSuccess &&
              hipMalloc((void**)&c->d_path, nreq * 4 * (size_t)cfg->max_stages) == hipSuccess &&
              hipMalloc((void**)&c->d_perm, nreq * 4) == hipSuccess && hipMalloc((void**)&c->d_inv, nreq * 4) == hipSuccess &&
              hipMalloc((void**)&c->d_cnt, 2 * coe::k::kRegroupMaxExperts * 4) == hipSuccess &&
              hipMalloc((void**)&c->d_off, (coe::k::kRegroupMaxExperts + 1) * 4) == hipSuccess &&
              hipMalloc((void**)&c->d_blockhist, nblocks * coe::k::kRegroupMaxExperts * 4) == hipSuccess &&
              hipHostMalloc((void**)&c->h_cnt, 2 * coe::k::kRegroupMaxExperts * 4, hipHostMallocDefault) == hipSuccess &&
              hipHostMalloc((void**)&c->h_first, nreq * 4, hipHostMallocDefault) == hipSuccess;
    c->device_allocs += 7;
    if (!ok) return bail(COE_ENOMEM);
    c->collected.assign(nreq, 0);
    c->submit_step.assign(nreq, 0);
    *out = c;
    return COE_OK;
}

void coe_destroy(coe_ctx* c)
{
    if (!c) return;
    (void)hipDeviceSynchronize();
    for (Expert& x : c->experts) {
        if (x.host) hipHostFree(x.host);
        if (x.loaded) hipEventDestroy(x.loaded);
    }
    for (DevBuf& b : c->slots)
        if (b.last_use) hipEventDestroy(b.last_use);
    if (c->arena) hipFree(c->arena);
    if (c->loader.joinable()) {
        {
            std::lock_guard<std::mutex> lk(c->ld_mutex);
            c->ld_stop = true;
        }
        c->ld_cv.notify_all();
        c->loader.join();
    }
    for (HostSlot& h : c->hslots) {
        if (h.p) hipHostFree(h.p);
        if (h.copied) hipEventDestroy(h.copied);
    }
    if (c->fd >= 0) {
        close(c->fd);
        unlink(c->backing_path.c_str());
    }
    for (auto& pc : c->prof)
        for (auto& s : pc.spans) { hipEventDestroy(s.first); hipEventDestroy(s.second); }
    for (hipEvent_t e : c->ev_pool) hipEventDestroy(e);
    void* ptrs[] = {c->d_inputs, c->d_staged, c->d_cur, c->d_depth, c->d_path, c->d_logits, c->d_cnt, c->d_off,
                    c->d_perm, c->d_inv, c->d_blockhist, c->d_succ};
    for (void* p : ptrs) if (p) hipFree(p);
    for (size_t l = 0; l < c->lanes.size(); ++l) {
        Lane& ln = c->lanes[l];
        for (int b = 1; b < kMaxBufs; ++b) if (ln.d_buf[b]) hipFree(ln.d_buf[b]);
        if (ln.d_patch) hipFree(ln.d_patch);
        if (ln.done) hipEventDestroy(ln.done);
        if (l > 0 && ln.s) hipStreamDestroy(ln.s);
    }
    if (c->ev_ready) hipEventDestroy(c->ev_ready);
    if (c->h_cnt) hipHostFree(c->h_cnt);
    if (c->h_first) hipHostFree(c->h_first);
    if (c->own_sc && c->sc) hipStreamDestroy(c->sc);
    if (c->own_sx && c->sx) hipStreamDestroy(c->sx);
    delete c;
}

int coe_register_arch(coe_ctx* c, const coe_arch_desc* desc, int32_t* arch_id)
{
    if (!c || !desc || !arch_id) return fail(c, COE_EINVAL, "null argument");
    ArchPlan a;
    int rc = plan_arch(c, desc, a);
    if (rc) return rc;
    if (!c->archs.empty()) {
        const ArchPlan& f = c->archs[0];
        if (f.dtype != a.dtype || f.in_h != a.in_h || f.in_w != a.in_w || f.in_c != a.in_c)
            return fail(c, COE_EINVAL, "all architectures of a context must share input shape and dtype");
    }
    c->archs.push_back(std::move(a));
    c->max_classes = std::max(c->max_classes, desc->n_classes);
    *arch_id = (int32_t)c->archs.size() - 1;
    return COE_OK;
}

int64_t coe_arch_blob_bytes(const coe_ctx* c, int32_t arch_id)
{
    if (!c || arch_id < 0 || arch_id >= (int32_t)c->archs.size()) return COE_EINVAL;
    return (int64_t)c->archs[arch_id].blob_bytes;
}

int coe_register_expert(coe_ctx* c, int32_t id, int32_t arch_id, const void* w, size_t nbytes, float prob)
{
    if (!c || !w) return fail(c, COE_EINVAL, "null argument");
    if (c->graph_set) return fail(c, COE_ESTATE, "experts must be registered before the dependency graph is set");
    if (arch_id < 0 || arch_id >= (int32_t)c->archs.size()) return fail(c, COE_EINVAL, "unknown architecture");
    if (id < 0 || id >= coe::k::kRegroupMaxExperts) return fail(c, COE_EINVAL, "expert id out of range");
    if (nbytes != c->archs[arch_id].blob_bytes) return fail(c, COE_EINVAL, "weight blob size does not match the architecture");
    if (!(prob >= 0.f)) return fail(c, COE_EINVAL, "usage probability must be >= 0");
    if ((size_t)id >= c->experts.size()) c->experts.resize((size_t)id + 1);
    Expert& x = c->experts[id];
    if (x.registered) return fail(c, COE_EINVAL, "expert id registered twice");
    std::vector<uint8_t> image;          // host tier: the blob is prepared here and goes to the backing file
    if (c->host_cap > 0) {
        image.resize(nbytes);
        x.host = image.data();
    } else if (hipHostMalloc(&x.host, nbytes, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        x.host = nullptr;
        return fail(c, COE_ENOMEM, "pinned host allocation failed");
    }
    std::memcpy(x.host, w, nbytes);
    // filters of the layers that run on the matrix cores are kept in fragment order from here on
    {
        std::vector<uint16_t> tmp;
        for (const LayerPlan& L : c->archs[arch_id].layers) {
            if (!L.packed) continue;
            const int red = L.d.r * L.d.s * L.C;
            const size_t n = (size_t)L.K * red;
            tmp.resize(n);
            uint16_t* t = (uint16_t*)((uint8_t*)x.host + L.off[0]);
            coe::k::pack_filters_mfma(t, tmp.data(), L.K, red);
            std::memcpy(t, tmp.data(), n * sizeof(uint16_t));
        }
    }
    if (c->host_cap > 0) {
        x.host = nullptr;
        size_t done = 0;
        while (done < nbytes) {
            ssize_t put = pwrite(c->fd, image.data() + done, nbytes - done, (off_t)(c->file_bytes + (int64_t)done));
            if (put <= 0) return fail(c, COE_EIO, "writing an expert to the backing file failed");
            done += (size_t)put;
        }
        x.file_off = c->file_bytes;
        c->file_bytes += (int64_t)((nbytes + 4095) / 4096 * 4096);
    }
    HIPCHK(c, hipEventCreateWithFlags(&x.loaded, hipEventDisableTiming));
    x.registered = true;
    x.arch = arch_id;
    x.prob = prob;
    x.nbytes = nbytes;
    return COE_OK;
}

int coe_set_host_tier(coe_ctx* c, int32_t host_cap_experts, const char* backing_path)
{
    if (!c) return COE_EINVAL;
    if (host_cap_experts <= 0 || !backing_path || !backing_path[0] || std::strlen(backing_path) >= 4096)
        return fail(c, COE_EINVAL, "host tier needs a positive cap and a path");
    if (!c->experts.empty() || c->graph_set) return fail(c, COE_ESTATE, "the host tier must be set before experts are registered");
    if (c->fd >= 0) return fail(c, COE_ESTATE, "host tier already set");
    int fd = open(backing_path, O_CREAT | O_RDWR | O_TRUNC | O_CLOEXEC, 0600);
    if (fd < 0) return fail(c, COE_EIO, std::string("cannot create the backing file ") + backing_path);
    c->fd = fd;
    c->backing_path = backing_path;
    c->host_cap = host_cap_experts;
    c->file_bytes = 0;
    return COE_OK;
}

int coe_debug_host_log(coe_ctx* c, int32_t cap, int32_t* log, int32_t* n_words)
{
    if (!c || !n_words || (cap > 0 && !log) || cap < 0) return fail(c, COE_EINVAL, "bad argument");
    *n_words = (int32_t)c->host_log.size();
    for (int32_t i = 0; i < std::min<int32_t>(cap, *n_words); ++i) log[i] = c->host_log[i];
    return COE_OK;
}

int coe_set_dependency_graph(coe_ctx* c, int32_t n, const int32_t* succ_off, const int32_t* succ)
{
    if (!c || !succ_off) return fail(c, COE_EINVAL, "null argument");
    if (c->graph_set) return fail(c, COE_ESTATE, "dependency graph already set");
    if (n <= 0 || n != (int32_t)c->experts.size()) return fail(c, COE_ESTATE, "n_experts differs from the registered experts");
    std::vector<int32_t> ncls(n);
    for (int32_t e = 0; e < n; ++e) {
        if (!c->experts[e].registered) return fail(c, COE_ESTATE, "an expert id is missing");
        ncls[e] = c->archs[c->experts[e].arch].n_classes;
    }
    int rc = coe::validate_graph(n, succ_off, succ, ncls.data());
    if (rc) return fail(c, rc, "dependency graph invalid (id out of range, cycle, or more routes than classes)");
    // longest path must fit the recorded path length
    {
        std::vector<int32_t> depth(n, 0), indeg(n, 0), order;
        for (int32_t j = 0; j < succ_off[n]; ++j) if (succ[j] >= 0) ++indeg[succ[j]];
        for (int32_t e = 0; e < n; ++e) if (!indeg[e]) { order.push_back(e); depth[e] = 1; }
        for (size_t i = 0; i < order.size(); ++i) {
            int32_t e = order[i];
            for (int32_t j = succ_off[e]; j < succ_off[e + 1]; ++j) {
                int32_t s = succ[j];
                if (s < 0) continue;
                depth[s] = std::max(depth[s], depth[e] + 1);
                if (--indeg[s] == 0) order.push_back(s);
            }
        }
        if (*std::max_element(depth.begin(), depth.end()) > c->cfg.max_stages)
            return fail(c, COE_ERANGE, "dependency graph is deeper than max_stages");
    }
    c->succ_off.assign(succ_off, succ_off + n + 1);
    c->succ.assign(succ, succ + succ_off[n]);
    size_t nb = std::max<size_t>(1, c->succ.size()) * 4;
    HIPCHK(c, dev_malloc(c, (void**)&c->d_succ, nb));
    if (!c->succ.empty()) HIPCHK(c, hipMemcpy(c->d_succ, c->succ.data(), c->succ.size() * 4, hipMemcpyHostToDevice));
    std::vector<int64_t> bytes(n);
    std::vector<float> prob(n);
    for (int32_t e = 0; e < n; ++e) { bytes[e] = (int64_t)c->experts[e].nbytes; prob[e] = c->experts[e].prob; }
    c->policy.reset(new coe::Policy(n, bytes.data(), prob.data(), c->succ_off.data(), c->succ.data(), c->cfg.cache_cap_experts,
                                    c->cfg.cache_cap_bytes));
    if (!c->policy->set_eviction(c->cfg.eviction)) return fail(c, COE_EINVAL, "unknown eviction rule");
    if (!c->policy->set_in_use_depth(c->cfg.prefetch_depth)) return fail(c, COE_EINVAL, "negative prefetch depth");
    // every device buffer the step path needs is allocated here, once: the expert arena, the request store and the
    // executors' activation workspaces.  coe_submit and coe_step allocate nothing.
    int rc2 = build_arena(c);
    if (rc2 == COE_OK && c->host_cap > 0) {
        c->host_policy.reset(new coe::Policy(n, bytes.data(), prob.data(), c->succ_off.data(), c->succ.data(), c->host_cap, 0));
        c->host_policy->set_eviction(c->cfg.eviction);
        rc2 = build_host_arena(c);
        if (rc2 == COE_OK) c->loader = std::thread(loader_main, c);
        // the file's pages leave the page cache where the file system allows it, so that reads come from the device below
        if (rc2 == COE_OK && fsync(c->fd) == 0) (void)posix_fadvise(c->fd, 0, 0, POSIX_FADV_DONTNEED);
    }
    if (rc2 == COE_OK) rc2 = ensure_store(c);
    if (rc2 == COE_OK) rc2 = ensure_workspace(c);
    if (rc2) {
        c->policy.reset();
        c->host_policy.reset();
        return rc2;
    }
    c->E = n;
    c->graph_set = true;
    return COE_OK;
}

int coe_submit(coe_ctx* c, int32_t n, const void* inputs, int on_device, const int32_t* first, int64_t* first_id)
{
    if (!c || n < 0 || (n > 0 && !inputs)) return fail(c, COE_EINVAL, "bad argument");
    if (!c->graph_set) return fail(c, COE_ESTATE, "set the dependency graph before submitting");
    if ((int64_t)c->n_live + n > c->cfg.max_requests) return fail(c, COE_ERANGE, "request store is full");
    if (first)
        for (int32_t i = 0; i < n; ++i)
            if (first[i] < 0 || first[i] >= c->E) return fail(c, COE_EINVAL, "first_expert out of range");
    int rc = ensure_store(c);
    if (rc) return rc;
    if (first_id) *first_id = c->id_base + c->n_live;
    if (n == 0) return COE_OK;
    size_t ib = c->archs[0].in_bytes();
    size_t base = (size_t)c->n_live;
    HIPCHK(c, hipMemcpyAsync((uint8_t*)c->d_inputs + base * ib, inputs, (size_t)n * ib,
                             on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, c->sc));
    // the first experts travel through pinned staging, one entry per request slot (a slot is reused only after the store
    // has drained, which synchronises), so the call returns without waiting for the stream
    if (first) std::copy(first, first + n, c->h_first + base);
    else std::fill(c->h_first + base, c->h_first + base + n, 0);
    HIPCHK(c, hipMemcpyAsync(c->d_cur + base, c->h_first + base, (size_t)n * 4, hipMemcpyHostToDevice, c->sc));
    HIPCHK(c, hipMemsetAsync(c->d_depth + base, 0, (size_t)n * 4, c->sc));
    HIPCHK(c, hipMemsetAsync(c->d_path + base * c->cfg.max_stages, 0xFF, (size_t)n * 4 * c->cfg.max_stages, c->sc));
    HIPCHK(c, hipMemsetAsync(c->d_logits + base * c->max_classes, 0, (size_t)n * 4 * c->max_classes, c->sc));
    // host inputs are the caller's (possibly pageable) memory and may be freed on return: wait for that copy only
    if (!on_device) HIPCHK(c, hipStreamSynchronize(c->sc));
    std::fill(c->collected.begin() + base, c->collected.begin() + base + n, 0);
    std::fill(c->submit_step.begin() + base, c->submit_step.begin() + base + n, c->step_no);
    c->n_live += n;
    return COE_OK;
}

static int step_body(coe_ctx* c, coe_step_stats& st)
{
    int rc = ensure_workspace(c);       // sized when the graph was set: allocates nothing here
    if (rc) return rc;
    rc = do_init_fill(c, &st);
    if (rc) return rc;
    const int32_t E = c->E;

    // request arranging, index part
    {
        Span sp(c, COE_K_REGROUP_INDEX, (double)c->n_live * 16.0, c->sc);
        HIPCHK(c, coe::k::regroup_index(c->d_cur, c->n_live, E, c->d_cnt, c->d_off, c->d_perm, c->d_inv, c->d_blockhist, c->sc));
    }
    bool arranging = false;
    for (const ArchPlan& a : c->archs) arranging = arranging || a.arr_wait > 0;
    if (arranging)   // the oldest queued request of every group, behind the counts
        HIPCHK(c, coe::k::group_heads(c->d_perm, c->d_off, c->d_cnt, E, c->d_cnt + E, c->sc));
    HIPCHK(c, hipMemcpyAsync(c->h_cnt, c->d_cnt, (size_t)E * 4 * (arranging ? 2 : 1), hipMemcpyDeviceToHost, c->sc));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    auto t0 = std::chrono::steady_clock::now();
    std::vector<int32_t> off(E + 1, 0);
    std::vector<uint8_t> has_group(E, 0);
    int32_t n_groups_queued = 0;
    for (int32_t e = 0; e < E; ++e) {
        off[e + 1] = off[e] + c->h_cnt[e];
        has_group[e] = c->h_cnt[e] > 0;
        n_groups_queued += has_group[e];
    }
    const int32_t n_pending = off[E];
    c->last_pending = n_pending; c->last_live = c->n_live; c->last_E = E;
    if (n_pending == 0) return COE_DONE;
    const int32_t step_no = c->step_no++;

    // arranging window: small groups stay queued for later arrivals to join (they keep their place in the regrouped
    // order; only the plan and the launches skip them)
    if (arranging) {
        std::vector<int32_t> age(E, 0), min_res(E, 0), min_miss(E, 0), wait(E, 0);
        std::vector<uint8_t> resident(E, 0), defer(E, 0);
        for (int32_t e = 0; e < E; ++e) {
            const ArchPlan& a = c->archs[c->experts[e].arch];
            min_res[e] = a.arr_min_res; min_miss[e] = a.arr_min_miss; wait[e] = a.arr_wait;
            resident[e] = c->policy->resident(e);
            if (has_group[e]) age[e] = step_no - c->submit_step[c->h_cnt[E + e]];
        }
        coe_arrange_defer(E, c->h_cnt, age.data(), resident.data(), min_res.data(), min_miss.data(), wait.data(), defer.data());
        for (int32_t e = 0; e < E; ++e)
            if (defer[e]) {
                has_group[e] = 0;
                ++st.n_deferred_groups;
                st.n_deferred_requests += c->h_cnt[e];
            }
    }

    // cache plan: execution order and switches
    std::vector<int32_t> order;
    std::vector<coe::Switch> switches;
    if (!c->policy->plan_stage(has_group.data(), order, switches))      // (the policy keeps its state: nothing to undo)
        return fail(c, COE_ENOMEM, "an expert does not fit the device cache");
    st.n_pending = n_pending;
    st.n_groups = (int32_t)order.size();
    st.n_misses = (int32_t)switches.size();
    st.n_hits = st.n_groups - st.n_misses;
    st.host_plan_us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();

    // request arranging, activation part: inputs into group-contiguous order
    // (one group that holds every stored request: the stable sort is the identity and the inputs are already in order)
    const size_t ib = c->archs[0].in_bytes();
    const bool in_place = n_groups_queued == 1 && n_pending == c->n_live;
    // (every architecture's first kernel can follow the regrouped order itself: no copy either)
    bool via_rows = !in_place;
    for (const ArchPlan& a : c->archs) via_rows = via_rows && a.gathers_input;
    const uint8_t* staged = (const uint8_t*)(in_place || via_rows ? c->d_inputs : c->d_staged);
    const int32_t* rows = via_rows ? c->d_perm : nullptr;
    if (!in_place && !via_rows && !order.empty()) {
        Span sp(c, COE_K_REGROUP_GATHER, 2.0 * (double)n_pending * (double)ib, c->sc);
        HIPCHK(c, coe::k::gather_rows(c->d_inputs, c->d_perm, n_pending, ib, c->d_staged, c->sc));
    }

    // host tier: every switch of the step is a request to it, in switch order; the reads start now, on the loader thread,
    // while the groups whose experts are resident are launched
    std::vector<ReadJob*> read_job(switches.size(), nullptr);
    std::vector<HostSlot*> read_src(switches.size(), nullptr);
    if (c->host_cap > 0)
        for (size_t k = 0; k < switches.size(); ++k) {
            int r2 = host_plan(c, switches[k].expert, &st, &read_job[k], &read_src[k]);
            if (r2) return r2;
        }

    std::vector<uint8_t> launched(E, 0);
    size_t next_load = 0;
    // enqueue every switch whose victims are no longer needed by a group that has not been launched yet; the copies
    // run on the copy stream while earlier groups compute
    // (need: the expert of the group about to be launched.  A switch whose blob is still being read from the backing file
    // is waited for only when that group cannot start without it; otherwise the launches go on and the read catches up.)
    auto issue_ready_loads = [&](int32_t need) -> int {
        while (next_load < switches.size()) {
            const coe::Switch& sw = switches[next_load];
            bool ready = true;
            for (int32_t v : sw.victims) ready = ready && !(has_group[v] && !launched[v]);
            if (!ready) break;
            if (read_job[next_load] && c->experts[need].buf) {
                std::lock_guard<std::mutex> lk(c->ld_mutex);
                if (!read_job[next_load]->done) break;
            }
            int r2 = issue_load(c, sw, &st, &st, c->host_cap > 0, read_job[next_load], read_src[next_load]);
            if (r2) return r2;
            ++next_load;
        }
        return COE_OK;
    };
    // executors: every launch sequence goes to the executor whose queue is predicted to finish first (paper Section
    // 4.2 "Request assigning": minimise the total time over all queues, i.e. the longest one; with equal executors that
    // is the one with the least work so far, the lowest-numbered among equals)
    std::vector<uint8_t> was_missing(E, 0);
    for (const coe::Switch& sw : switches) was_missing[sw.expert] = 1;
    for (Lane& ln : c->lanes) { ln.used = false; ln.busy_ns = 0; }
    c->last_units.clear();
    c->last_chunks.clear();
    if (c->lanes.size() > 1) HIPCHK(c, hipEventRecord(c->ev_ready, c->sc));
    auto take_lane = [&](int32_t first_expert, int64_t cost_ns, Lane** out) -> int {
        size_t best = 0;
        for (size_t l = 1; l < c->lanes.size(); ++l)
            if (c->lanes[l].busy_ns < c->lanes[best].busy_ns) best = l;
        Lane& ln = c->lanes[best];
        ln.busy_ns += cost_ns;
        if (best > 0 && !ln.used) HIPCHK(c, hipStreamWaitEvent(ln.s, c->ev_ready, 0));   // inputs regrouped, earlier steps done
        ln.used = true;
        c->last_units.push_back({first_expert, cost_ns, (int32_t)best});
        *out = &ln;
        return COE_OK;
    };
    auto group_cost = [&](int32_t e) {
        const ArchPlan& a = c->archs[c->experts[e].arch];
        return a.lat_k_ns * (int64_t)c->h_cnt[e] + (was_missing[e] ? a.lat_load_ns : 0);
    };
    const int32_t group_small = c->cfg.group_small == 0 ? 64 : c->cfg.group_small;
    auto small = [&](int32_t e) {
        const ArchPlan& a = c->archs[c->experts[e].arch];
        return group_small > 0 && c->h_cnt[e] <= group_small && c->h_cnt[e] <= chunk_rows(c, a) && a.groupable;
    };
    for (size_t i = 0; i < order.size(); ++i) {
        const int32_t e = order[i];
        if (launched[e]) continue;                             // ran earlier, in a set with other small groups
        rc = issue_ready_loads(e);
        if (rc) return rc;
        Expert& x = c->experts[e];
        if (!x.buf) return fail(c, COE_ESTATE, "internal: expert not loaded at launch time");

        // small groups further down the plan, of the same architecture and with their experts on the device (or on
        // their way), run together with this one: one launch per layer for all of them.  Pulling a group forward changes
        // neither results (they do not depend on the order) nor the switches (those are issued in plan order above, and
        // a group that has run only frees its expert earlier).
        std::vector<SetMember> set;
        if (small(e)) {
            set.push_back({e, off[e], c->h_cnt[e]});
            int32_t rows = c->h_cnt[e];
            for (size_t j = i + 1; j < order.size() && (int32_t)set.size() < coe::k::kMaxGroups; ++j) {
                const int32_t f = order[j];
                if (launched[f] || !small(f) || c->experts[f].arch != x.arch) continue;
                if (!c->experts[f].buf) continue;              // its switch has not been issued yet
                if (rows + c->h_cnt[f] > chunk_rows(c, c->archs[x.arch])) continue;
                set.push_back({f, off[f], c->h_cnt[f]});
                rows += c->h_cnt[f];
            }
        }
        Lane* lane = nullptr;
        if (set.size() >= 2) {
            int64_t cost = c->archs[x.arch].lat_b_ns;                       // one launch sequence for the whole set
            for (const SetMember& m : set) cost += group_cost(m.expert);
            rc = take_lane(e, cost, &lane);
            if (rc) return rc;
            for (const SetMember& m : set) {
                Expert& xm = c->experts[m.expert];
                if (xm.load_pending) {
                    Span sp(c, COE_K_SWITCH_WAIT, (double)xm.nbytes, lane->s);
                    HIPCHK(c, hipStreamWaitEvent(lane->s, xm.loaded, 0));
                    xm.load_pending = false;
                }
            }
            rc = run_group_set(c, *lane, set, staged, ib, rows);
            if (rc) return rc;
            for (const SetMember& m : set) {
                Expert& xm = c->experts[m.expert];
                HIPCHK(c, hipEventRecord(xm.buf->last_use, lane->s));
                xm.buf->used = true;
                launched[m.expert] = 1;
                ++st.n_chunks;
                c->last_chunks.insert(c->last_chunks.end(), {m.expert, m.first, m.count});
            }
            st.n_grouped += (int32_t)set.size();
            ++st.n_group_sets;
            continue;
        }

        const int32_t n_route = c->succ_off[e + 1] - c->succ_off[e];
        // request splitting: as few launch sequences as the cap allows, of equal size (no short last one)
        const int32_t cap_rows = chunk_rows(c, c->archs[x.arch]);
        const int32_t n_seq = (c->h_cnt[e] + cap_rows - 1) / cap_rows;
        const int32_t chunk = (c->h_cnt[e] + n_seq - 1) / n_seq;
        rc = take_lane(e, group_cost(e) + c->archs[x.arch].lat_b_ns * n_seq, &lane);   // a group stays on one executor
        if (rc) return rc;
        if (x.load_pending) {
            Span sp(c, COE_K_SWITCH_WAIT, (double)x.nbytes, lane->s);
            HIPCHK(c, hipStreamWaitEvent(lane->s, x.loaded, 0));
            x.load_pending = false;
        }
        for (int32_t s = off[e]; s < off[e + 1]; s += chunk) {
            int32_t cnt = std::min(chunk, off[e + 1] - s);
            coe::k::RouteArgs r{c->d_perm + s, e, c->d_succ + c->succ_off[e], n_route, c->d_cur, c->d_depth, c->d_path,
                                c->cfg.max_stages, c->d_logits, c->max_classes};
            rc = run_expert(c, *lane, x, x.buf->p, rows ? staged : staged + (size_t)s * ib, cnt, r, -1, rows ? rows + s : nullptr);
            if (rc) return rc;
            ++st.n_chunks;
            c->last_chunks.insert(c->last_chunks.end(), {e, s, cnt});
        }
        HIPCHK(c, hipEventRecord(x.buf->last_use, lane->s));
        x.buf->used = true;
        launched[e] = 1;
    }
    for (const Lane& ln : c->lanes) st.n_executors_used += ln.used;
    return COE_OK;
}

int coe_step(coe_ctx* c, coe_step_stats* stats)
{
    if (!c) return COE_EINVAL;
    coe_step_stats st{};
    if (stats) *stats = st;
    if (!c->graph_set) return fail(c, COE_ESTATE, "dependency graph not set");
    if (c->n_live == 0) return COE_DONE;
    const int64_t allocs_before = c->device_allocs;
    for (Lane& ln : c->lanes) ln.used = false;
    int rc = step_body(c, st);
    // the step is complete on the compute stream once every executor is - also when the step ended in an error after some
    // executors had been given work
    for (size_t l = 1; l < c->lanes.size(); ++l) {
        Lane& ln = c->lanes[l];
        if (!ln.used) continue;
        hipError_t e1 = hipEventRecord(ln.done, ln.s);
        hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(c->sc, ln.done, 0) : e1;
        if (e2 != hipSuccess && rc >= 0) rc = fail(c, COE_EDEVICE, std::string("joining an executor: ") + hipGetErrorString(e2));
    }
    if (c->host_cap > 0) {
        // reads of a step that ended early are still on the loader's queue: they finish before their storage goes
        std::unique_lock<std::mutex> lk(c->ld_mutex);
        if (rc < 0)      // their copies will not be enqueued any more: let the loader through
            for (HostSlot& h : c->hslots) h.issued = h.planned;
        c->ld_cv.notify_all();
        c->ld_cv.wait(lk, [&] { return c->ld_queue.empty(); });
        c->ld_jobs.clear();
    }
    st.n_device_allocs = (int32_t)(c->device_allocs - allocs_before);
    if (stats && rc >= 0) *stats = st;
    return rc;
}

int coe_set_latency_model(coe_ctx* c, int32_t arch_id, int64_t k_ns, int64_t b_ns, int64_t load_ns)
{
    if (!c) return COE_EINVAL;
    if (arch_id < 0 || arch_id >= (int32_t)c->archs.size()) return fail(c, COE_EINVAL, "unknown architecture");
    if (k_ns < 0 || b_ns < 0 || load_ns < 0) return fail(c, COE_EINVAL, "negative latency");
    ArchPlan& a = c->archs[arch_id];
    a.lat_k_ns = k_ns; a.lat_b_ns = b_ns; a.lat_load_ns = load_ns;
    return COE_OK;
}

int coe_assign_executors(int32_t n_units, const int64_t* cost_ns, int32_t n_executors, int32_t* executor)
{
    if (n_units < 0 || n_executors <= 0 || (n_units > 0 && (!cost_ns || !executor))) return COE_EINVAL;
    std::vector<int64_t> busy(n_executors, 0);
    for (int32_t u = 0; u < n_units; ++u) {
        int32_t best = 0;
        for (int32_t l = 1; l < n_executors; ++l)
            if (busy[l] < busy[best]) best = l;
        busy[best] += cost_ns[u];
        executor[u] = best;
    }
    return COE_OK;
}

int coe_debug_last_assignment(coe_ctx* c, int32_t cap, int32_t* first_expert, int64_t* cost_ns, int32_t* executor, int32_t* n_units)
{
    if (!c || !n_units || cap < 0) return COE_EINVAL;
    *n_units = (int32_t)c->last_units.size();
    for (int32_t u = 0; u < std::min<int32_t>(cap, *n_units); ++u) {
        if (first_expert) first_expert[u] = c->last_units[u].expert;
        if (cost_ns) cost_ns[u] = c->last_units[u].cost_ns;
        if (executor) executor[u] = c->last_units[u].lane;
    }
    return COE_OK;
}

int coe_debug_last_chunks(coe_ctx* c, int32_t cap, int32_t* chunks, int32_t* n_chunks)
{
    if (!c || !n_chunks || cap < 0 || (cap > 0 && !chunks)) return COE_EINVAL;
    *n_chunks = (int32_t)(c->last_chunks.size() / 3);
    const size_t words = 3 * (size_t)std::min<int32_t>(cap, *n_chunks);
    std::copy(c->last_chunks.begin(), c->last_chunks.begin() + words, chunks);
    return COE_OK;
}

int coe_set_arranging(coe_ctx* c, int32_t arch_id, int32_t min_group_resident, int32_t min_group_missing, int32_t max_wait_steps)
{
    if (!c) return COE_EINVAL;
    if (arch_id < 0 || arch_id >= (int32_t)c->archs.size()) return fail(c, COE_EINVAL, "unknown architecture");
    if (min_group_resident < 0 || min_group_missing < 0 || max_wait_steps < 0) return fail(c, COE_EINVAL, "negative arranging parameter");
    ArchPlan& a = c->archs[arch_id];
    a.arr_min_res = min_group_resident;
    a.arr_min_miss = min_group_missing;
    a.arr_wait = max_wait_steps;
    return COE_OK;
}

int coe_arrange_defer(int32_t n_experts, const int32_t* count, const int32_t* age, const uint8_t* resident,
                      const int32_t* min_group_resident, const int32_t* min_group_missing, const int32_t* max_wait_steps,
                      uint8_t* defer)
{
    if (n_experts < 0 || !count || !age || !resident || !min_group_resident || !min_group_missing || !max_wait_steps || !defer)
        return COE_EINVAL;
    int n = 0;
    for (int32_t e = 0; e < n_experts; ++e) {
        const int32_t enough = resident[e] ? min_group_resident[e] : min_group_missing[e];
        defer[e] = count[e] > 0 && age[e] < max_wait_steps[e] && count[e] < enough;
        n += defer[e];
    }
    return n;
}

int coe_sync(coe_ctx* c)
{
    if (!c) return COE_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->sx));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    return COE_OK;
}

int coe_collect(coe_ctx* c, int32_t cap, int64_t* ids, float* logits, int32_t* path, int32_t* n_out)
{
    if (!c || cap < 0 || !n_out) return fail(c, COE_EINVAL, "bad argument");
    *n_out = 0;
    if (c->n_live == 0) return COE_OK;
    HIPCHK(c, hipStreamSynchronize(c->sc));
    const size_t n = (size_t)c->n_live, ms = (size_t)c->cfg.max_stages, mc = (size_t)c->max_classes;
    std::vector<int32_t> cur(n), hpath(path ? n * ms : 0);
    std::vector<float> hlog(logits ? n * mc : 0);
    HIPCHK(c, hipMemcpy(cur.data(), c->d_cur, n * 4, hipMemcpyDeviceToHost));
    if (path) HIPCHK(c, hipMemcpy(hpath.data(), c->d_path, n * ms * 4, hipMemcpyDeviceToHost));
    if (logits) HIPCHK(c, hipMemcpy(hlog.data(), c->d_logits, n * mc * 4, hipMemcpyDeviceToHost));
    int32_t m = 0;
    for (size_t i = 0; i < n && m < cap; ++i) {
        if (c->collected[i] || cur[i] >= 0) continue;
        if (ids) ids[m] = c->id_base + (int64_t)i;
        if (logits) std::memcpy(logits + (size_t)m * mc, hlog.data() + i * mc, mc * 4);
        if (path) std::memcpy(path + (size_t)m * ms, hpath.data() + i * ms, ms * 4);
        c->collected[i] = 1;
        ++c->n_collected;
        ++m;
    }
    *n_out = m;
    if (c->n_collected == c->n_live) {   // store drained: start over at slot 0, ids keep counting
        c->id_base += c->n_live;
        c->n_live = 0;
        c->n_collected = 0;
    }
    return COE_OK;
}

int coe_reset_requests(coe_ctx* c)
{
    if (!c) return COE_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->sc));
    c->id_base += c->n_live;
    c->n_live = 0;
    c->n_collected = 0;
    return COE_OK;
}

int coe_debug_last_regroup(coe_ctx* c, int32_t* n_pending, int32_t* n_live, int32_t* cnt, int32_t* off, int32_t* perm,
                           int32_t* inv, int32_t perm_cap)
{
    if (!c) return COE_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->sc));
    if (n_pending) *n_pending = c->last_pending;
    if (n_live) *n_live = c->last_live;
    if (c->last_E == 0) return COE_OK;
    if (cnt) HIPCHK(c, hipMemcpy(cnt, c->d_cnt, (size_t)c->last_E * 4, hipMemcpyDeviceToHost));
    if (off) HIPCHK(c, hipMemcpy(off, c->d_off, ((size_t)c->last_E + 1) * 4, hipMemcpyDeviceToHost));
    if (perm) {
        if (perm_cap < c->last_pending) return fail(c, COE_ERANGE, "perm buffer too small");
        if (c->last_pending) HIPCHK(c, hipMemcpy(perm, c->d_perm, (size_t)c->last_pending * 4, hipMemcpyDeviceToHost));
    }
    if (inv && c->last_live) HIPCHK(c, hipMemcpy(inv, c->d_inv, (size_t)c->last_live * 4, hipMemcpyDeviceToHost));
    return COE_OK;
}

int coe_debug_switch_log(coe_ctx* c, int32_t cap, int32_t* log, int32_t* n_words)
{
    if (!c || !n_words || cap < 0 || (cap > 0 && !log)) return COE_EINVAL;
    *n_words = (int32_t)c->switch_log.size();
    std::copy(c->switch_log.begin(), c->switch_log.begin() + std::min<size_t>(cap, c->switch_log.size()), log);
    return COE_OK;
}

int coe_debug_resident(coe_ctx* c, uint8_t* out)
{
    if (!c || !out) return COE_EINVAL;
    for (size_t e = 0; e < c->experts.size(); ++e) out[e] = c->experts[e].buf ? 1 : 0;
    return COE_OK;
}

int coe_debug_forward(coe_ctx* c, int32_t e, int32_t n, const void* dev_in, float* logits_out)
{
    if (!c || !dev_in || !logits_out || n < 0) return fail(c, COE_EINVAL, "bad argument");
    if (e < 0 || e >= (int32_t)c->experts.size() || !c->experts[e].registered) return fail(c, COE_EINVAL, "unknown expert");
    if (n == 0) return COE_OK;
    int rc = ensure_workspace(c);
    if (rc) return rc;
    Expert& x = c->experts[e];
    const ArchPlan& a = c->archs[x.arch];
    void* w = nullptr;
    float* d_log = nullptr;
    bool temp = false;
    if (x.buf) {
        if (x.load_pending) { HIPCHK(c, hipStreamWaitEvent(c->sc, x.loaded, 0)); x.load_pending = false; }
        w = x.buf->p;
    } else {
        if (c->host_cap > 0) return fail(c, COE_ESTATE, "with a host tier only resident experts can be run directly");
        HIPCHK(c, hipMalloc(&w, x.nbytes));
        temp = true;
        HIPCHK(c, hipMemcpy(w, x.host, x.nbytes, hipMemcpyHostToDevice));
    }
    HIPCHK(c, hipMalloc((void**)&d_log, (size_t)n * a.n_classes * 4));
    const size_t ib = a.in_bytes();
    const int32_t chunk = chunk_rows(c, a);
    for (int32_t s = 0; s < n && rc == COE_OK; s += chunk) {
        int32_t cnt = std::min(chunk, n - s);
        coe::k::RouteArgs r{nullptr, e, nullptr, 0, nullptr, nullptr, nullptr, 0, d_log + (size_t)s * a.n_classes, a.n_classes};
        rc = run_expert(c, c->lanes[0], x, w, (const uint8_t*)dev_in + (size_t)s * ib, cnt, r);
    }
    hipError_t he = hipStreamSynchronize(c->sc);
    if (rc == COE_OK && he == hipSuccess) he = hipMemcpy(logits_out, d_log, (size_t)n * a.n_classes * 4, hipMemcpyDeviceToHost);
    hipFree(d_log);
    if (temp) hipFree(w);
    if (rc) return rc;
    if (he != hipSuccess) return fail(c, COE_EDEVICE, hipGetErrorString(he));
    return COE_OK;
}

int coe_debug_layer_output(coe_ctx* c, int32_t e, int32_t n, const void* dev_in, int32_t layer, void* out, size_t out_bytes)
{
    if (!c || !dev_in || !out || n <= 0) return fail(c, COE_EINVAL, "bad argument");
    if (e < 0 || e >= (int32_t)c->experts.size() || !c->experts[e].registered) return fail(c, COE_EINVAL, "unknown expert");
    Expert& x = c->experts[e];
    const ArchPlan& a = c->archs[x.arch];
    if (n > chunk_rows(c, a)) return fail(c, COE_ERANGE, "more inputs than one launch sequence takes");
    if (layer < 0 || layer >= (int32_t)a.layers.size() - 1) return fail(c, COE_EINVAL, "layer index out of range (heads have no output tensor)");
    const LayerPlan& L = a.layers[layer];
    if (L.fuse_pool || L.fused_away) return fail(c, COE_EINVAL, "layer is fused with its neighbour");
    const size_t bytes = (size_t)n * L.P * L.Q * L.K * a.elem();
    if (out_bytes != bytes) return fail(c, COE_EINVAL, "output size does not match the layer");
    if (c->host_cap > 0) return fail(c, COE_ESTATE, "not available with a host tier");
    int rc = ensure_workspace(c);
    if (rc) return rc;
    void* w = nullptr;
    HIPCHK(c, hipMalloc(&w, x.nbytes));
    hipError_t he = hipMemcpy(w, x.host, x.nbytes, hipMemcpyHostToDevice);
    if (he == hipSuccess) {
        coe::k::RouteArgs r{};
        rc = run_expert(c, c->lanes[0], x, w, dev_in, n, r, layer);
        he = hipStreamSynchronize(c->sc);
        if (rc == COE_OK && he == hipSuccess) he = hipMemcpy(out, c->lanes[0].d_buf[L.d.dst], bytes, hipMemcpyDeviceToHost);
    }
    hipFree(w);
    if (rc) return rc;
    if (he != hipSuccess) return fail(c, COE_EDEVICE, hipGetErrorString(he));
    return COE_OK;
}

int coe_debug_regroup(coe_ctx* c, int32_t n, const int32_t* cur, int32_t E, int32_t* cnt, int32_t* off, int32_t* perm, int32_t* inv)
{
    if (!c || n < 0 || (n > 0 && !cur)) return fail(c, COE_EINVAL, "bad argument");
    if (E <= 0 || E > coe::k::kRegroupMaxExperts) return fail(c, COE_EINVAL, "n_experts out of range");
    if (n > c->cfg.max_requests) return fail(c, COE_ERANGE, "more keys than max_requests");
    if (c->n_live > 0) return fail(c, COE_ESTATE, "requests are live");
    if (n) HIPCHK(c, hipMemcpy(c->d_cur, cur, (size_t)n * 4, hipMemcpyHostToDevice));
    HIPCHK(c, coe::k::regroup_index(c->d_cur, n, E, c->d_cnt, c->d_off, c->d_perm, c->d_inv, c->d_blockhist, c->sc));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    std::vector<int32_t> hoff(E + 1);
    HIPCHK(c, hipMemcpy(hoff.data(), c->d_off, ((size_t)E + 1) * 4, hipMemcpyDeviceToHost));
    if (off) std::copy(hoff.begin(), hoff.end(), off);
    if (cnt) HIPCHK(c, hipMemcpy(cnt, c->d_cnt, (size_t)E * 4, hipMemcpyDeviceToHost));
    if (perm && hoff[E] > 0) HIPCHK(c, hipMemcpy(perm, c->d_perm, (size_t)hoff[E] * 4, hipMemcpyDeviceToHost));
    if (inv && n > 0) HIPCHK(c, hipMemcpy(inv, c->d_inv, (size_t)n * 4, hipMemcpyDeviceToHost));
    return hoff[E];
}

int coe_debug_conv(coe_ctx* c, int32_t dtype, const void* x, const void* w, const float* bias, const void* res, void* y,
                   int32_t n, int32_t h, int32_t wd, int32_t ch, int32_t k, int32_t r, int32_t s, int32_t stride, int32_t pad,
                   int32_t act, int32_t repeat, int32_t* kernel_class)
{
    if (!c || !x || !w || !bias || !y) return fail(c, COE_EINVAL, "null argument");
    if ((dtype != COE_DT_F32 && dtype != COE_DT_BF16) || n <= 0 || h <= 0 || wd <= 0 || ch <= 0 || k <= 0 || r <= 0 || s <= 0 ||
        stride <= 0 || pad < 0 || act < 0 || act > 3 || repeat <= 0)
        return fail(c, COE_EINVAL, "bad convolution parameters");
    const int P = (h + 2 * pad - r) / stride + 1, Q = (wd + 2 * pad - s) / stride + 1;
    if (P <= 0 || Q <= 0) return fail(c, COE_EINVAL, "empty output");
    const size_t eb = dtype == COE_DT_BF16 ? 2 : 4;
    const size_t nx = (size_t)n * h * wd * ch, nw = (size_t)k * r * s * ch, ny = (size_t)n * P * Q * k;
    void *dx = nullptr, *dw = nullptr, *dres = nullptr, *dy = nullptr;
    float* db = nullptr;
    coe::k::ConvShape cs{n, h, wd, ch, k, r, s, stride, pad, P, Q, act};
    const bool mfma = dtype == COE_DT_BF16 && coe::k::conv_mfma_supported(cs);
    const bool smallc = !mfma && dtype == COE_DT_BF16 && coe::k::conv_smallc_supported(cs, res != nullptr, false);
    const int cls = mfma ? (coe::k::conv_mfma_uses_slab(cs) ? COE_K_CONV_SLAB : COE_K_CONV_MFMA)
                         : smallc ? COE_K_CONV_STEM : COE_K_CONV_DIRECT;
    if (kernel_class) *kernel_class = cls;
    hipError_t he = hipSuccess;
    auto ok = [&](hipError_t e) { if (he == hipSuccess) he = e; return he == hipSuccess; };
    std::vector<uint16_t> packed;
    const void* wsrc = w;
    if (mfma) {
        packed.resize(nw);
        coe::k::pack_filters_mfma((const uint16_t*)w, packed.data(), k, r * s * ch);
        wsrc = packed.data();
    }
    if (ok(hipMalloc(&dx, nx * eb)) && ok(hipMalloc(&dw, nw * eb)) && ok(hipMalloc((void**)&db, (size_t)k * 4)) &&
        ok(hipMalloc(&dy, ny * eb)) && (!res || ok(hipMalloc(&dres, ny * eb))) &&
        ok(hipMemcpy(dx, x, nx * eb, hipMemcpyHostToDevice)) && ok(hipMemcpy(dw, wsrc, nw * eb, hipMemcpyHostToDevice)) &&
        ok(hipMemcpy(db, bias, (size_t)k * 4, hipMemcpyHostToDevice)) &&
        (!res || ok(hipMemcpy(dres, res, ny * eb, hipMemcpyHostToDevice)))) {
        const double flops = 2.0 * (double)ny * r * s * ch;
        for (int it = 0; it < repeat && he == hipSuccess; ++it) {
            Span sp(c, cls, flops, c->sc);
            if (mfma) ok(coe::k::conv_mfma(dx, dw, db, dres, dy, cs, c->sc));
            else if (smallc) ok(coe::k::conv_smallc(dx, dw, db, dy, cs, false, c->sc));
            else ok(coe::k::conv_direct(dtype, dx, dw, db, dres, dy, cs, c->sc));
        }
        ok(hipStreamSynchronize(c->sc));
        ok(hipMemcpy(y, dy, ny * eb, hipMemcpyDeviceToHost));
    }
    void* ptrs[] = {dx, dw, db, dres, dy};
    for (void* p : ptrs) if (p) (void)hipFree(p);
    if (he != hipSuccess) return fail(c, COE_EDEVICE, hipGetErrorString(he));
    return COE_OK;
}

int coe_profile_read(coe_ctx* c, int32_t cls, int64_t* launches, double* ms, double* work)
{
    if (!c || cls < 0 || cls >= COE_K_COUNT) return COE_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->sx));
    HIPCHK(c, hipStreamSynchronize(c->sc));
    ProfClass& p = c->prof[cls];
    double total = 0.0;
    for (auto& s : p.spans) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, s.first, s.second) == hipSuccess) total += t;
        else (void)hipGetLastError();
        c->ev_pool.push_back(s.first);
        c->ev_pool.push_back(s.second);
    }
    if (launches) *launches = (int64_t)p.spans.size();
    if (ms) *ms = total;
    if (work) *work = p.work;
    p.spans.clear();
    p.work = 0.0;
    return COE_OK;
}

int coe_profile_issued(coe_ctx* c, int32_t cls, int64_t* issued)
{
    if (!c || !issued || cls < 0 || cls >= COE_K_COUNT) return COE_EINVAL;
    *issued = c->prof[cls].issued;
    c->prof[cls].issued = 0;
    return COE_OK;
}

}  // extern "C"

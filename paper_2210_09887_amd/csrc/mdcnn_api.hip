// Host side of the C ABI: descriptors, the buffer manager (camera shifts, reset
// rule, ring origins), argument validation and launch sequencing.  Allocates no
// device memory and never synchronises.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <utility>
#include <vector>

#include "mdcnn_internal.h"

using namespace mdcnn;

namespace {

thread_local char g_err[512] = "";
int g_conv_path = 0;
int g_fuse_skip = 1;      // mdcnn_frame: residual skips are added by the step-1 kernel of their source
int g_profile = 0;
int g_streams = 0;        // mdcnn_frame: independent branches of the network go to up to this many streams; 0: decide per network
int g_pipe_group = 0;     // mdcnn_frames: forward calls per group of the frame pipeline, 0: by the length of the network
int g_pipe_mode = 1;      // mdcnn_frames: 1 whole frames on streams, 0 runs of layers on streams
int g_pipe_threads = 1;   // mdcnn_frames: one issuing host thread per stream (mode 1, long runs)

// Profiling mode: every kernel launch is bracketed by a pair of events on its
// own stream; mdcnn_profile_read waits for them and sums the times per class.
struct TimedLaunch { int cls; hipEvent_t start, stop; int site, edge; };
thread_local int g_tag_site = -1, g_tag_edge0 = -1;   // the forward call being issued (profiling mode: tags of its launches)
std::vector<TimedLaunch> g_timed;
std::vector<hipEvent_t> g_event_pool;

hipEvent_t take_event() {
    if (!g_event_pool.empty()) { hipEvent_t e = g_event_pool.back(); g_event_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

template <typename F>
hipError_t timed(int cls, hipStream_t st, F&& launch) {
    if (!g_profile) return launch();
    TimedLaunch t{cls, take_event(), take_event(), g_tag_site, -1};
    if (!t.start || !t.stop) return hipErrorOutOfMemory;
    (void)hipEventRecord(t.start, st);
    hipError_t err = launch();
    (void)hipEventRecord(t.stop, st);
    g_timed.push_back(t);
    return err;
}

mdcnn_status fail(mdcnn_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
size_t esize(int dtype) { return dtype == MDCNN_F16 ? 2 : 4; }
long long pmod(long long v, long long n) { long long r = v % n; return r < 0 ? r + n : r; }

struct Layout {
    size_t A, P, flags, delta, list, lcnt, lacc, clist, ccnt, cacc, counters, Y, S, total;
    int nseg_l, nseg_c;
    int Hp, Wp;
};

mdcnn_status check_desc(const mdcnn_buffer_desc* d) {
    if (!d) return fail(MDCNN_ERR_NULL, "descriptor is NULL");
    if (d->dtype != MDCNN_F32 && d->dtype != MDCNN_F16) return fail(MDCNN_ERR_DTYPE, "unknown dtype %d", d->dtype);
    if (d->kind < MDCNN_SITE_INPUT || d->kind > MDCNN_SITE_OUTPUT) return fail(MDCNN_ERR_SHAPE, "unknown site kind %d", d->kind);
    if (d->H < 1 || d->W < 1 || d->C < 1) return fail(MDCNN_ERR_SHAPE, "H, W, C must be positive");
    if ((long long)d->H * d->W > (1 << 24) || d->C > 4096) return fail(MDCNN_ERR_SIZE, "site too large (H*W <= 2^24, C <= 4096)");
    for (int i = 0; i < 4; ++i)
        if (d->border[i] < 0 || d->border[i] > 64) return fail(MDCNN_ERR_SHAPE, "border[%d]=%d out of range [0,64]", i, d->border[i]);
    if (d->tile < 1) return fail(MDCNN_ERR_SHAPE, "tile must be >= 1");
    if (d->kind == MDCNN_SITE_INPUT && (d->border[0] | d->border[1] | d->border[2] | d->border[3]))
        return fail(MDCNN_ERR_SHAPE, "an INPUT site has no border");
    if (d->pool_prev != 0 && (d->pool_prev != 1 || d->kind != MDCNN_SITE_PREACT))
        return fail(MDCNN_ERR_SHAPE, "pool_prev is 0 or 1 and needs a PREACT site");
    if (d->crops != 0 && d->crops != 1) return fail(MDCNN_ERR_SHAPE, "crops is 0 or 1");
    if (d->crops && (d->H > 65535 || d->W > 65535)) return fail(MDCNN_ERR_SIZE, "a site with crops has H, W < 65536");
    if (d->truncation_free != 0) {
        if (d->truncation_free != 1 || d->kind != MDCNN_SITE_PREACT || d->crops || d->pool_prev ||
            (d->border[0] | d->border[1] | d->border[2] | d->border[3]))
            return fail(MDCNN_ERR_SHAPE, "truncation_free is 0 or 1 and needs a PREACT site without border, crops or pooling");
    }
    return MDCNN_OK;
}

void make_layout(const mdcnn_buffer_desc& d, Layout& L) {
    const size_t e = esize(d.dtype);
    const bool hasA = d.kind != MDCNN_SITE_OUTPUT, hasC = d.kind != MDCNN_SITE_INPUT;
    const bool hasP = hasC && !d.truncation_free;         // a truncation-free site keeps no pending ring
    L.Hp = d.H + d.border[0] + d.border[1];
    L.Wp = d.W + d.border[2] + d.border[3];
    const size_t nseg_l = ((size_t)d.H * d.W + kSegPixels - 1) / kSegPixels;
    const size_t nseg_c = ((size_t)L.Hp * L.Wp + kSegPixels - 1) / kSegPixels;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
    L.A = take(hasA ? (size_t)d.H * d.W * d.C * e : 0);
    L.P = take(hasP ? (size_t)L.Hp * L.Wp * d.C * e : 0);
    L.flags = take(hasA ? (size_t)d.H * d.W : 0);
    L.delta = take(hasA ? (size_t)d.H * d.W * d.C * e : 0);
    L.list = take(hasA ? nseg_l * kSegPixels * 4 : 0);
    L.lcnt = take(hasA ? nseg_l * 2 * 4 : 0);
    L.lacc = take(hasA ? nseg_l * 2 * 8 : 0);
    L.nseg_l = hasA ? (int)nseg_l : 0;
    L.nseg_c = hasC ? (int)nseg_c : 0;
    L.clist = take(hasC ? nseg_c * kSegPixels * 4 : 0);
    L.ccnt = take(hasC ? nseg_c * 4 : 0);
    L.cacc = take(hasC ? nseg_c * 8 : 0);
    L.counters = take(kNumCounters * 4);
    L.Y = take(d.pool_prev ? (size_t)d.H * d.W * d.C * e : 0);
    L.S = take(d.crops && hasA ? (size_t)d.H * d.W : 0);
    L.total = off;
}

}  // namespace

// By-products of a forward call - the compacted list of the source site, the compute lists of the destinations and
// their per-segment counts - for the entry point that keeps them out of the sites' memory (mdcnn_layer_forward_noalloc).
// The name of the array is a host-side stand-in: the address the kernels get comes from hipGetSymbolAddress, once per device.
// (No `used` attribute here: with it the compiler keeps the symbol local to the code object and the runtime cannot look it up.)
constexpr size_t kScratchBytes = (size_t)2 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

struct mdcnn_buffer {
    mdcnn_buffer_desc d;
    Layout L;
    SiteDev dev;
    long long gy, gx;          // global pixel coordinate of view pixel (0, 0)
    bool fresh;                // no reset yet
    bool r_up, r_down, r_left, r_right;   // directions in which growth is restricted
};

// Launch plan of one frame: node = one kernel launch in program order (per non-terminal site its
// step-1 launch, then one launch per edge that gets one, or the compaction-only launch).
struct PlanNode {
    int stream;                // index into the streams of the call (0: the caller's)
    bool record;               // a node on another stream waits for this one
    std::vector<int> wait;     // nodes on other streams that must have finished
};
struct Plan {
    int key = -1;              // g_streams * 2 + g_fuse_skip the plan was made for
    int streams = 1;           // streams that carry at least one node
    std::vector<PlanNode> nodes;
};

// Plan of a run of frames that overlap in time (mdcnn_frames).  The forward calls of a frame, in
// site order, are cut into groups of `group_calls`.  The sites a group is the first to touch are
// initialised just before it: by a launch of their own at the head of the frame for the first group,
// by spare blocks of the step-1 launch of the call before the group for the others (that launch and
// the rest of its call do not touch them, or the group would not be the first).  The initialisation,
// and with it everything the frame does to those sites, has to follow whatever the frame before
// does to them, the last of which is the forward call of the highest such site (the readout for an
// OUTPUT site): the stream waits for that before the launch that carries the initialisation.
struct PipeGroup {
    int call0, call1;          // forward calls [call0, call1)
    std::vector<int> fill;     // sites initialised for the group
    int wait_call;             // call of the frame before that must have finished (n_calls: its readout), -1: none
};
struct PipePlan {
    int key = -1;              // group size, streams and mode the plan was made for (-1: no plan yet)
    std::vector<int> call_site, call_e0, call_e1;
    std::vector<PipeGroup> groups;
    // Streams.  Mode 1, frames: frame f goes to stream f % streams as a whole (seg_of_call is all zero).
    // Mode 0, stages: the calls are cut into as many runs as there are streams, of about equal cost, and
    // run k of every frame goes to stream k - frames follow each other on a stream in order, so only what
    // crosses from one run to another needs an event.
    int streams = 1, mode = 0;
    std::vector<int> seg_of_call;      // per call, and one more entry for the readout
    std::vector<int> event_of_call;    // per call (and the readout): slot of the event recorded after it, or -1
    std::vector<char> forward;         // per call: its stream differs from that of the call before (same frame)
    int n_events = 0;
    int stream_of(int frame, int call) const { return mode ? frame % streams : seg_of_call[(size_t)call]; }
};

struct mdcnn_net {
    std::vector<mdcnn_buffer*> sites;
    std::vector<int> esrc, edst;
    std::vector<mdcnn_conv_desc> edges;
    size_t out_bytes;
    Plan plan;
    PipePlan pipe;
};

namespace {

void refresh_origins(mdcnn_buffer* b) {
    const mdcnn_buffer_desc& d = b->d;
    b->dev.a_oy = (int)pmod(b->gy + d.origin_y, d.H);
    b->dev.a_ox = (int)pmod(b->gx + d.origin_x, d.W);
    b->dev.p_oy = (int)pmod(b->gy - d.border[0] + d.origin_y, b->L.Hp);
    b->dev.p_ox = (int)pmod(b->gx - d.border[2] + d.origin_x, b->L.Wp);
}

mdcnn_status border_1d(int k, int stride, int pad, int in_extent, int out_extent, int* before, int* after) {
    if (k == 0) { *before = *after = 0; return MDCNN_OK; }
    if (k < 1 || stride < 1 || pad < 0 || in_extent < 1 || out_extent < 1)
        return fail(MDCNN_ERR_SHAPE, "bad convolution geometry k=%d stride=%d pad=%d", k, stride, pad);
    int b0 = (k - 1 - pad) / stride;       // k-1-pad >= 0 here or the numerator is negative
    if (k - 1 - pad < 0) b0 = 0;
    int b1 = (in_extent - 1 + pad) / stride - (out_extent - 1);
    *before = b0 < 0 ? 0 : b0;
    *after = b1 < 0 ? 0 : b1;
    return MDCNN_OK;
}

// Everything that must hold for the kernels of one edge to stay in bounds.
mdcnn_status validate_edge(const mdcnn_buffer* in, const mdcnn_buffer* out, const mdcnn_conv_desc& c, int idx) {
    if (!out) return fail(MDCNN_ERR_NULL, "edge %d: destination buffer is NULL", idx);
    if (out == in) return fail(MDCNN_ERR_SHAPE, "edge %d: source and destination are the same site", idx);
    if (out->d.kind == MDCNN_SITE_INPUT) return fail(MDCNN_ERR_SHAPE, "edge %d: destination is an INPUT site", idx);
    if (out->d.dtype != in->d.dtype) return fail(MDCNN_ERR_DTYPE, "edge %d: dtype mismatch", idx);
    if (c.Cin != in->d.C || c.Cout != out->d.C)
        return fail(MDCNN_ERR_SHAPE, "edge %d: channels %d->%d do not match sites %d->%d", idx, c.Cin, c.Cout, in->d.C, out->d.C);
    if (c.k == 0 && out->d.truncation_free) return fail(MDCNN_ERR_SHAPE, "edge %d: a residual skip cannot end at a truncation-free site", idx);
    if (c.k == 0) {
        if (c.op != 0 || c.stride != 1 || c.pad != 0 || c.up != 0 || c.Cin != c.Cout || in->d.H != out->d.H || in->d.W != out->d.W)
            return fail(MDCNN_ERR_SHAPE, "edge %d: identity edge needs equal shapes, stride 1, pad 0, up 0", idx);
        return MDCNN_OK;
    }
    if (c.op != 0 && c.op != 1) return fail(MDCNN_ERR_SHAPE, "edge %d: unknown op %d", idx, c.op);
    if (out->d.truncation_free && (c.k != 1 || c.up != 0 || c.pad != 0 || c.op != 0))
        return fail(MDCNN_ERR_SHAPE, "edge %d: the producer of a truncation-free site must be a 1x1 convolution without padding or upsampling", idx);
    if (c.k < 1 || c.k > 5 || c.stride < 1 || c.stride > 4 || c.pad < 0 || c.pad >= c.k || c.up < 0 || c.up > 5)
        return fail(MDCNN_ERR_SHAPE, "edge %d: unsupported geometry k=%d stride=%d pad=%d up=%d", idx, c.k, c.stride, c.pad, c.up);
    if (c.up && (c.k != 1 || c.stride != 1 || c.pad != 0))
        return fail(MDCNN_ERR_SHAPE, "edge %d: upsampling needs a 1x1 stride-1 convolution", idx);
    if (in->d.H + 2 * c.pad < c.k || in->d.W + 2 * c.pad < c.k)
        return fail(MDCNN_ERR_SHAPE, "edge %d: kernel larger than the padded input", idx);
    const int oh = (in->d.H + 2 * c.pad - c.k) / c.stride + 1, ow = (in->d.W + 2 * c.pad - c.k) / c.stride + 1;
    if ((oh << c.up) != out->d.H || (ow << c.up) != out->d.W)
        return fail(MDCNN_ERR_SHAPE, "edge %d: output %dx%d does not match destination %dx%d", idx, oh << c.up, ow << c.up, out->d.H, out->d.W);
    if (c.op == 1) {                                       // max pooling: no weights, no border
        if (c.up || c.Cin != c.Cout) return fail(MDCNN_ERR_SHAPE, "edge %d: max pooling needs up == 0 and Cin == Cout", idx);
        if (out->d.kind != MDCNN_SITE_PREACT || !out->d.pool_prev)
            return fail(MDCNN_ERR_SHAPE, "edge %d: the destination of a max pooling must be a PREACT site with pool_prev = 1", idx);
        return MDCNN_OK;
    }
    int by0, by1, bx0, bx1;
    mdcnn_status st = border_1d(c.k, c.stride, c.pad, in->d.H, oh, &by0, &by1);
    if (st) return st;
    st = border_1d(c.k, c.stride, c.pad, in->d.W, ow, &bx0, &bx1);
    if (st) return st;
    const int* b = out->d.border;
    if (by0 > b[0] || by1 > b[1] || bx0 > b[2] || bx1 > b[3])
        return fail(MDCNN_ERR_SHAPE, "edge %d: destination border {%d,%d,%d,%d} smaller than the convolution reaches {%d,%d,%d,%d}",
                    idx, b[0], b[1], b[2], b[3], by0, by1, bx0, bx1);
    if (!c.w_dev) return fail(MDCNN_ERR_NULL, "edge %d: weights are NULL", idx);
    if ((uintptr_t)c.w_dev & 15) return fail(MDCNN_ERR_ALIGN, "edge %d: weights must be 16-byte aligned", idx);
    if (c.w_packed_dev) {
        if ((uintptr_t)c.w_packed_dev & 15) return fail(MDCNN_ERR_ALIGN, "edge %d: packed weights must be 16-byte aligned", idx);
        if (in->d.dtype != MDCNN_F16 || c.Cin % 16 || c.Cout % 32)
            return fail(MDCNN_ERR_SHAPE, "edge %d: packed weights need fp16, Cin %% 16 == 0, Cout %% 32 == 0", idx);
    }
    return MDCNN_OK;
}

EdgeDev make_edge(const mdcnn_buffer* in, const mdcnn_buffer* out, const mdcnn_conv_desc& c) {
    EdgeDev e{};
    e.delta = in->dev.delta; e.sflags = in->dev.flags; e.pub_list = nullptr; e.pub_lcnt = nullptr; e.scounters = in->dev.counters;
    e.sH = in->d.H; e.sW = in->d.W; e.Cin = c.Cin;
    e.P = out->dev.P; e.dflags = out->d.kind == MDCNN_SITE_OUTPUT ? nullptr : out->dev.flags;
    e.clist = out->dev.clist; e.ccnt = out->dev.ccnt; e.cacc = out->dev.cacc; e.dcounters = out->dev.counters;
    e.dH = out->d.H; e.dW = out->d.W; e.Cout = c.Cout; e.Hp = out->L.Hp; e.Wp = out->L.Wp;
    e.by0 = out->d.border[0]; e.bx0 = out->d.border[2]; e.p_oy = out->dev.p_oy; e.p_ox = out->dev.p_ox;
    e.op = c.k ? c.op : 0;
    if (e.op == 1 && out->d.crops) e.op = 2;               // the reset zeroes the previous pooling output
    e.sA = in->dev.A; e.s_aoy = in->dev.a_oy; e.s_aox = in->dev.a_ox; e.s_relu = in->d.relu;
    e.dY = out->dev.Y; e.d_aoy = out->dev.a_oy; e.d_aox = out->dev.a_ox;
    if (out->d.truncation_free) {                          // no P: the edge adds to A and makes the site's mask and deltas
        e.op = kOpTruncFree;
        e.dY = out->dev.A; e.sA = out->dev.delta; e.s_relu = out->d.relu;
    }
    e.w = c.w_dev; e.wp = out->d.truncation_free ? (const void*)out->dev.bias : c.k && !c.op ? c.w_packed_dev : nullptr; e.k = c.k; e.stride = c.k ? c.stride : 1; e.pad = c.k ? c.pad : 0; e.up = c.k ? c.up : 0;
    return e;
}

mdcnn_status validate_forward(const mdcnn_buffer* in, const void* frame, const uint8_t* forced, const mdcnn_conv_desc* edges,
                              mdcnn_buffer* const* outs, int n_edges) {
    if (!in) return fail(MDCNN_ERR_NULL, "input buffer is NULL");
    if (in->d.kind == MDCNN_SITE_OUTPUT) return fail(MDCNN_ERR_STATE, "OUTPUT sites take no forward call");
    if (in->fresh) return fail(MDCNN_ERR_STATE, "mdcnn_shift_camera must be called before the first forward");
    if (in->d.kind == MDCNN_SITE_INPUT) {
        if (!frame) return fail(MDCNN_ERR_NULL, "frame is NULL for an INPUT site");
        if ((uintptr_t)frame & 15) return fail(MDCNN_ERR_ALIGN, "frame must be 16-byte aligned");
    } else if (frame) {
        return fail(MDCNN_ERR_SHAPE, "frame given for a site that is not INPUT");
    }
    if (n_edges < 0 || (n_edges > 0 && (!edges || !outs))) return fail(MDCNN_ERR_NULL, "edges/outs missing");
    if (in->d.truncation_free && forced) return fail(MDCNN_ERR_STATE, "the mask of a truncation-free site cannot be forced");
    for (int i = 0; i < n_edges; ++i) {
        mdcnn_status st = validate_edge(in, outs[i], edges[i], i);
        if (st) return st;
        if (outs[i]->fresh) return fail(MDCNN_ERR_STATE, "edge %d: destination was never reset (shift first)", i);
    }
    return MDCNN_OK;
}

// One forward call for `n` streams of the same network at once (n <= kMaxBatch;
// the caller has checked that all streams have the same shapes): stream b goes
// from ins[b] along edges[b][0 .. n_edges) to outs[b][0 .. n_edges).
// fuse_skip: index of an identity edge whose add is done by the step-1 kernel (its
// destination is touched there and the edge gets no launch of its own), or -1.
// riders (n == 1 only): jobs[riders[0 .. n_riders)] are run by spare blocks of the step-1 launch.
// Streams and events of one multi-stream frame.  Every wait is on an event that was recorded
// earlier in the same call, so no stream can wait for something that never happens.
constexpr int kMaxStreams = 4;
constexpr int kMaxBatchStreams = 128;     // streams of one mdcnn_frame_batch call (kMaxBatch to a launch)
struct Sched {
    const Plan* plan = nullptr;
    hipStream_t s[kMaxStreams] = {};
    std::vector<hipEvent_t> ev;                            // per node, set where plan->nodes[i].record
    int next = 0;                                          // node of the next launch
    hipError_t err = hipSuccess;
    hipStream_t begin() {                                  // waits of the next node; returns its stream
        const PlanNode& nd = plan->nodes[next];
        for (int w : nd.wait) {
            const hipError_t e = hipStreamWaitEvent(s[nd.stream], ev[w], 0);
            if (e != hipSuccess && err == hipSuccess) err = e;
        }
        return s[nd.stream];
    }
    void end() {
        const PlanNode& nd = plan->nodes[next];
        if (nd.record) {
            const hipError_t e = hipEventRecord(ev[next], s[nd.stream]);
            if (e != hipSuccess && err == hipSuccess) err = e;
        }
        ++next;
    }
};

hipError_t launch_fill_jobs(const FillJob* jobs, const int* which, int count, hipStream_t st);

// Where the by-products of a forward call go instead of the sites' own list regions (n == 1 only).
struct ListScratch {
    int* list; int* lcnt; unsigned long long* lacc;                          // of the source site
    std::vector<int*> clist, ccnt; std::vector<unsigned long long*> cacc;    // per edge
};

mdcnn_status do_forward(int n, mdcnn_buffer* const* ins, const void* const* frames, const uint8_t* const* forced,
                        const mdcnn_conv_desc* const* edges, mdcnn_buffer* const* const* outs, int n_edges,
                        hipStream_t st, int fuse_skip = -1, Sched* sc = nullptr, const FillJob* jobs = nullptr,
                        const int* riders = nullptr, int n_riders = 0, const ListScratch* ls = nullptr) {
    static thread_local Step1Batch sb;                     // 3.4 KiB each: kept off the stack
    static thread_local EdgeBatch eb;
    for (int b = 0; b < n; ++b) {
        sb.s[b] = ins[b]->dev;
        sb.X[b] = frames ? frames[b] : nullptr;
        sb.forced[b] = forced ? forced[b] : nullptr;
        sb.skip[b] = SkipDev{};
        if (fuse_skip >= 0) {
            const mdcnn_buffer* d = outs[b][fuse_skip];
            SkipDev& k = sb.skip[b];
            k.P = d->dev.P;
            k.dflags = d->d.kind == MDCNN_SITE_OUTPUT ? nullptr : d->dev.flags;
            k.Hp = d->L.Hp; k.Wp = d->L.Wp; k.by0 = d->d.border[0]; k.bx0 = d->d.border[2];
            k.p_oy = d->dev.p_oy; k.p_ox = d->dev.p_ox;
        }
    }
    hipError_t err;
    if (ins[0]->d.truncation_free) {
        // step 1 happened in the producer's launch; initialisation jobs that would have ridden along get a launch of their own
        err = n_riders > 0 ? launch_fill_jobs(jobs, riders, n_riders, st) : hipSuccess;
        if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "shift launch: %s", hipGetErrorString(err));
    } else {
    if (sc) st = sc->begin();
    if (n == 1 && n_riders > 0) {
        // initialisation jobs of other sites, which nothing in this launch touches, ride along
        static thread_local Step1Fill sf;
        sf.s = sb.s[0]; sf.skip = sb.skip[0]; sf.X = sb.X[0]; sf.forced = sb.forced[0];
        sf.n = n_riders;
        for (int k = 0; k < n_riders; ++k) sf.j[k] = jobs[riders[k]];
        err = timed(kClsStep1, st, [&] { return launch_step1_fill(sf, st); });
    } else {
        err = timed(kClsStep1, st, [&] { return launch_step1(sb, n, st); });
    }
    if (sc) sc->end();
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "step-1 launch: %s", hipGetErrorString(err));
    }
    auto launch_edge = [&](int idx) -> mdcnn_status {
        if (sc) st = sc->begin();
        struct AtExit { Sched* sc; ~AtExit() { if (sc) sc->end(); } } at_exit{sc};
        int cls = kClsConvPlain;
        TimedLaunch t{0, nullptr, nullptr, g_tag_site, idx >= 0 && g_tag_edge0 >= 0 ? g_tag_edge0 + idx : -1};
        if (g_profile) {              // the class is known only after dispatch: record around, file under it
            t.start = take_event();
            t.stop = take_event();
            if (!t.start || !t.stop) return fail(MDCNN_ERR_HIP, "cannot create profiling events");
            (void)hipEventRecord(t.start, st);
        }
        err = launch_conv(eb, n, ins[0]->d.dtype, g_conv_path, st, &cls);
        if (g_profile) {
            (void)hipEventRecord(t.stop, st);
            t.cls = cls;
            g_timed.push_back(t);
        }
        if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "conv launch (edge %d): %s", idx, hipGetErrorString(err));
        return MDCNN_OK;
    };
    auto with_source_list = [&](EdgeDev& e, const mdcnn_buffer* in) {
        e.pub_list = in->dev.list; e.pub_lcnt = in->dev.lcnt; e.pub_lacc = in->dev.lacc;
        if (ls) { e.pub_list = ls->list; e.pub_lcnt = ls->lcnt; e.pub_lacc = ls->lacc; }
    };
    if (n_edges == 0 || (n_edges == 1 && fuse_skip == 0)) {
        for (int b = 0; b < n; ++b) {
            EdgeDev e{};
            e.sflags = ins[b]->dev.flags; e.sH = ins[b]->d.H; e.sW = ins[b]->d.W;
            e.scounters = ins[b]->dev.counters;
            with_source_list(e, ins[b]);
            e.k = -1;
            eb.d[b] = e;
        }
        return launch_edge(-1);
    }
    bool first = true;
    for (int i = 0; i < n_edges; ++i) {
        if (i == fuse_skip) continue;
        for (int b = 0; b < n; ++b) {
            eb.d[b] = make_edge(ins[b], outs[b][i], edges[b][i]);
            if (ls) { eb.d[b].clist = ls->clist[(size_t)i]; eb.d[b].ccnt = ls->ccnt[(size_t)i]; eb.d[b].cacc = ls->cacc[(size_t)i]; }
            if (first) with_source_list(eb.d[b], ins[b]);
        }
        first = false;
        mdcnn_status rc = launch_edge(i);
        if (rc) return rc;
    }
    return MDCNN_OK;
}

// Two networks can share launches if they have the same topology and the same
// site and edge shapes (weights and buffers may differ).
bool same_shape(const mdcnn_net* a, const mdcnn_net* b) {
    if (a->sites.size() != b->sites.size() || a->esrc != b->esrc || a->edst != b->edst) return false;
    for (size_t i = 0; i < a->sites.size(); ++i) {
        const mdcnn_buffer_desc &x = a->sites[i]->d, &y = b->sites[i]->d;
        if (x.H != y.H || x.W != y.W || x.C != y.C || x.dtype != y.dtype || x.kind != y.kind || x.relu != y.relu || x.crops != y.crops || x.truncation_free != y.truncation_free ||
            x.border[0] != y.border[0] || x.border[1] != y.border[1] || x.border[2] != y.border[2] || x.border[3] != y.border[3])
            return false;
    }
    for (size_t i = 0; i < a->edges.size(); ++i) {
        const mdcnn_conv_desc &x = a->edges[i], &y = b->edges[i];
        if (x.k != y.k || x.stride != y.stride || x.pad != y.pad || x.Cin != y.Cin || x.Cout != y.Cout || x.up != y.up || x.op != y.op ||
            (x.w_packed_dev == nullptr) != (y.w_packed_dev == nullptr))
            return false;
    }
    return true;
}

// Which edge of the forward call of site i (edges [e0, e1)) is added by the step-1 kernel: a
// residual skip keeps its place in the order of the producers of its destination as long as
// no other edge of the call goes to the same destination before it.  -1: none.
int fused_skip(const mdcnn_net* net, int e0, int e1) {
    if (!g_fuse_skip) return -1;
    for (int e = e0; e < e1; ++e) {
        if (net->edges[e].k != 0) continue;
        bool earlier = false;
        for (int q = e0; q < e; ++q) earlier |= net->edst[q] == net->edst[e];
        if (!earlier) return e - e0;
    }
    return -1;
}

// Plan of a frame on up to `ns` streams.  A launch reads its source site and reads and writes
// its destination site (step 1: its own site and the destination of a fused skip), so it has
// to follow the last writer of each; writers of one site keep their program order (the sum in
// P is taken in that order, whatever the streams do).  Every site gets a home stream on which
// everything that writes it runs: that of the source for the first launched edge of a forward
// call - a chain of layers stays on one stream - and the next stream in turn for the others,
// which are the starts of parallel branches.
void make_plan(const mdcnn_net* net, int ns, Plan& plan) {
    const int n_sites = (int)net->sites.size(), n_edges = (int)net->edges.size();
    std::vector<int> home(n_sites, -1), lastw(n_sites, -1);
    plan.nodes.clear();
    home[0] = 0;
    int rr = 0, e0 = 0;
    auto add = [&](int stream, std::initializer_list<int> deps) {
        PlanNode nd{stream, false, {}};
        for (int d : deps) {
            if (d < 0 || plan.nodes[d].stream == stream) continue;      // same stream: already in order
            bool have = false;
            for (int w : nd.wait) have |= w == d;
            if (!have) { nd.wait.push_back(d); plan.nodes[d].record = true; }
        }
        plan.nodes.push_back(nd);
        return (int)plan.nodes.size() - 1;
    };
    for (int i = 0; i < n_sites; ++i) {
        if (net->sites[i]->d.kind == MDCNN_SITE_OUTPUT) continue;
        int e1 = e0;
        while (e1 < n_edges && net->esrc[e1] == i) ++e1;
        if (home[i] < 0) home[i] = 0;
        const int fuse = fused_skip(net, e0, e1);
        const int skip_dst = fuse >= 0 ? net->edst[e0 + fuse] : -1;
        // (a truncation-free site has no delta launch: its edges follow its producer)
        const int s1 = net->sites[i]->d.truncation_free ? lastw[i] : add(home[i], {lastw[i], skip_dst >= 0 ? lastw[skip_dst] : -1});
        lastw[i] = s1;
        if (skip_dst >= 0) {
            lastw[skip_dst] = s1;
            if (home[skip_dst] < 0) home[skip_dst] = home[i];
        }
        bool first = true;
        for (int e = e0; e < e1; ++e) {
            if (e - e0 == fuse) continue;
            const int d = net->edst[e];
            if (home[d] < 0) {
                if (first) home[d] = home[i];
                else {
                    rr = (rr + 1) % ns;
                    if (rr == home[i] && ns > 1) rr = (rr + 1) % ns;
                    home[d] = rr;
                }
            }
            lastw[d] = add(home[d], {s1, lastw[d]});
            first = false;
        }
        if (first) add(home[i], {s1});                     // no launched edge: the compaction-only launch
        e0 = e1;
    }
    plan.streams = 1;
    for (const PlanNode& nd : plan.nodes) plan.streams = nd.stream + 1 > plan.streams ? nd.stream + 1 : plan.streams;
}

// Length of a plan in launches, if every launch took one unit of time and a wait for another
// stream one more (measured: such a wait costs about as much as a small launch).  These
// launches are bound by their latency, not by the size of the GPU, so this is the time a frame
// takes; a plan on one stream is as long as it has nodes.
double plan_length(const Plan& plan) {
    std::vector<double> done(plan.nodes.size(), 0.0);
    double avail[kMaxStreams] = {}, total = 0.0;
    for (size_t i = 0; i < plan.nodes.size(); ++i) {
        const PlanNode& nd = plan.nodes[i];
        double t = avail[nd.stream];
        for (int w : nd.wait) t = done[w] + 1.0 > t ? done[w] + 1.0 : t;
        done[i] = avail[nd.stream] = t + 1.0;
        total = done[i] > total ? done[i] : total;
    }
    return total;
}

// streams = 0: left to itself the library uses four streams, and only where the network has
// branches that are worth it: the plan must be a fifth shorter than the launches in a row.
void choose_plan(const mdcnn_net* net, int streams, Plan& plan) {
    make_plan(net, streams ? streams : kMaxStreams, plan);
    if (!streams && plan_length(plan) > 0.8 * (double)plan.nodes.size()) make_plan(net, 1, plan);
}

// The library's own streams (per host thread, default priority, made on first use) and events.
struct Aux {
    hipStream_t s[kMaxStreams - 1] = {};
    int n = 0, device = -1;
    std::vector<hipEvent_t> events;
};
thread_local Aux g_aux;

hipError_t aux_prepare(int streams, size_t events) {
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (g_aux.device != dev) { g_aux = Aux{}; g_aux.device = dev; }       // streams of another device are left alone
    while (g_aux.n < streams - 1) {
        err = hipStreamCreateWithFlags(&g_aux.s[g_aux.n], hipStreamNonBlocking);
        if (err != hipSuccess) return err;
        ++g_aux.n;
    }
    while (g_aux.events.size() < events) {
        hipEvent_t e = nullptr;
        err = hipEventCreateWithFlags(&e, hipEventDisableTiming);
        if (err != hipSuccess) return err;
        g_aux.events.push_back(e);
    }
    return hipSuccess;
}

// Host part of a camera shift: decides between growth and full reset, moves the buffers and
// makes the initialisation job of every buffer (jobs[i] for bufs[i]; block_begin is left to the
// launch).  Nothing is launched.
mdcnn_status shift_jobs(mdcnn_buffer* const* bufs, int n, int dty, int dtx, std::vector<FillJob>& jobs, bool* full_out) {
    if (!bufs || n < 1) return fail(MDCNN_ERR_NULL, "no buffers");
    for (int i = 0; i < n; ++i) {
        if (!bufs[i]) return fail(MDCNN_ERR_NULL, "buffer %d is NULL", i);
        const mdcnn_buffer *a = bufs[0], *b = bufs[i];
        if (a->fresh != b->fresh || a->r_up != b->r_up || a->r_down != b->r_down || a->r_left != b->r_left ||
            a->r_right != b->r_right)
            return fail(MDCNN_ERR_STATE, "buffer %d has a different shift history than buffer 0", i);
    }
    const mdcnn_buffer* f = bufs[0];
    bool full = f->fresh;
    full |= (dtx > 0 && f->r_right) || (dtx < 0 && f->r_left) || (dty > 0 && f->r_down) || (dty < 0 && f->r_up);
    for (int i = 0; i < n; ++i) {
        const mdcnn_buffer_desc& d = bufs[i]->d;
        const long long sy = (long long)dty * d.tile, sx = (long long)dtx * d.tile;
        full |= (sy >= d.H || -sy >= d.H || sx >= d.W || -sx >= d.W);
    }
    jobs.resize((size_t)n);
    for (int i = 0; i < n; ++i) {
        mdcnn_buffer* b = bufs[i];
        const mdcnn_buffer_desc& d = b->d;
        const long long sy = (long long)dty * d.tile, sx = (long long)dtx * d.tile;
        b->gy += sy;
        b->gx += sx;
        refresh_origins(b);
        FillJob j{};
        j.A = b->dev.A; j.P = b->dev.P; j.flags = b->dev.flags; j.bias = b->dev.bias; j.counters = b->dev.counters;
        j.lacc = b->dev.lacc; j.cacc = b->dev.cacc; j.lcnt = b->dev.lcnt; j.ccnt = b->dev.ccnt;
        j.n_lacc = 2 * b->L.nseg_l; j.n_cacc = b->L.nseg_c;
        j.s_off = b->dev.s_off;
        j.y_off = d.crops && d.pool_prev ? (unsigned)((b->L.Y - b->L.A) / 256) : 0u;
        j.H = d.H; j.W = d.W; j.C = d.C; j.Hp = b->L.Hp; j.Wp = b->L.Wp;
        j.a_oy = b->dev.a_oy; j.a_ox = b->dev.a_ox; j.p_oy = b->dev.p_oy; j.p_ox = b->dev.p_ox;
        j.dtype = d.dtype;
        if (!full) {
            // the old window, expressed in coordinates of the new one, is shifted by (-sy, -sx)
            auto keep = [](int ext, long long s, int& lo, int& hi) {   // |s| < ext here
                lo = -s > 0 ? (int)-s : 0;
                hi = ext - s < ext ? (int)(ext - s) : ext;
                if (hi < lo) hi = lo;
            };
            keep(j.Hp, sy, j.py0, j.py1);
            keep(j.Wp, sx, j.px0, j.px1);
            keep(j.H, sy, j.ay0, j.ay1);
            keep(j.W, sx, j.ax0, j.ax1);
        }
        auto outside = [](int Hn, int Wn, int y0, int y1, int x0, int x1) {
            return (y0 + (Hn - y1)) * Wn + (y1 - y0) * (x0 + (Wn - x1));
        };
        j.nP = j.P ? outside(j.Hp, j.Wp, j.py0, j.py1, j.px0, j.px1) : 0;
        j.nA = j.A ? outside(j.H, j.W, j.ay0, j.ay1, j.ax0, j.ax1) : 0;
        j.reset_counters = b->fresh ? 2 : 1;             // per-frame counters start at zero every frame
        j.per_block = full ? kFillItemsPerBlockFull : kFillItemsPerBlockStrip;
        jobs[(size_t)i] = j;
        if (full) {
            b->r_up = b->r_down = b->r_left = b->r_right = false;
            b->fresh = false;
        } else {
            // growing in one direction overwrites the stash of the opposite side
            if (dtx > 0) b->r_left = true;
            if (dtx < 0) b->r_right = true;
            if (dty > 0) b->r_up = true;
            if (dty < 0) b->r_down = true;
        }
    }
    *full_out = full;
    return MDCNN_OK;
}

// Launches jobs[which[0 .. count)] (which == nullptr: jobs[0 .. count)), kMaxFillJobs to a launch.
hipError_t launch_fill_jobs(const FillJob* jobs, const int* which, int count, hipStream_t st) {
    FillBatch fb{};
    auto flush = [&]() -> hipError_t {
        hipError_t err = timed(kClsShift, st, [&] { return launch_shift_fill(fb, st); });
        fb.n = 0;
        fb.total_blocks = 0;
        return err;
    };
    for (int k = 0; k < count; ++k) {
        FillJob j = jobs[which ? which[k] : k];
        j.block_begin = fb.total_blocks;
        fb.j[fb.n++] = j;
        fb.total_blocks += fill_blocks(j);
        if (fb.n == kMaxFillJobs) {
            hipError_t err = flush();
            if (err != hipSuccess) return err;
        }
    }
    return fb.n ? flush() : hipSuccess;
}

size_t crop_pixels(const mdcnn_buffer* b) {                // sites without crops: the view
    if (!b->d.crops) return (size_t)b->d.H * b->d.W;
    return (size_t)(b->dev.cy1() - b->dev.cy0()) * (size_t)(b->dev.cx1() - b->dev.cx0());
}
bool whole_view(const mdcnn_buffer* b) { return crop_pixels(b) == (size_t)b->d.H * b->d.W; }

// Shift, forward over all non-terminal sites, readout: for n streams at once.
mdcnn_status frame_batch(mdcnn_net* const* nets, int n, const void* const* frames, const uint8_t* const* forced,
                         const int* dty, const int* dtx, void* const* outs_dev, void* stream, int* did_full_reset) {
    hipStream_t st = (hipStream_t)stream;
    // a launch failure between the camera shift and the readout leaves the device state of a frame half
    // done: the sites are then marked as never reset, so that the next camera shift re-initialises them
    struct Unfinished {
        mdcnn_net* const* nets; int n; bool armed = true;
        ~Unfinished() {
            if (!armed) return;
            for (int b = 0; b < n; ++b)
                for (mdcnn_buffer* s : nets[b]->sites) s->fresh = true;
        }
    } unfinished{nets, n};
    for (int b = 0; b < n; ++b) {
        mdcnn_status rc = mdcnn_shift_camera(nets[b]->sites.data(), (int)nets[b]->sites.size(), dty[b], dtx[b], stream,
                                             did_full_reset ? did_full_reset + b : nullptr);
        if (rc) return rc;
    }
    mdcnn_net* net = nets[0];
    const int n_edges = (int)net->edges.size();
    // independent branches of the network on streams of their own; the caller's stream forks into
    // them after the shift and joins them before the readout, so to the caller the call is in
    // stream order as before
    Sched sched, *sc = nullptr;
    if (g_streams != 1) {
        const int key = g_streams * 2 + g_fuse_skip;
        if (net->plan.key != key) {
            choose_plan(net, g_streams, net->plan);
            net->plan.key = key;
        }
        if (net->plan.streams > 1) {
            const size_t n_nodes = net->plan.nodes.size();
            hipError_t err = aux_prepare(net->plan.streams, n_nodes + kMaxStreams);
            if (err == hipSuccess) err = hipEventRecord(g_aux.events[n_nodes], st);          // fork
            for (int k = 1; k < net->plan.streams && err == hipSuccess; ++k) err = hipStreamWaitEvent(g_aux.s[k - 1], g_aux.events[n_nodes], 0);
            if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "stream set-up: %s", hipGetErrorString(err));
            sched.plan = &net->plan;
            sched.s[0] = st;
            for (int k = 1; k < net->plan.streams; ++k) sched.s[k] = g_aux.s[k - 1];
            sched.ev.assign(g_aux.events.begin(), g_aux.events.begin() + n_nodes);
            sc = &sched;
        }
    }
    // whatever happens below, the caller's stream waits for the other streams before the call returns
    struct Join {
        Sched* sc; hipStream_t st; size_t base;
        hipError_t run() {
            hipError_t err = hipSuccess;
            for (int k = 1; sc && k < sc->plan->streams; ++k) {
                hipError_t e = hipEventRecord(g_aux.events[base + k], sc->s[k]);
                if (e == hipSuccess) e = hipStreamWaitEvent(st, g_aux.events[base + k], 0);
                if (e != hipSuccess && err == hipSuccess) err = e;
            }
            sc = nullptr;
            return err;
        }
        ~Join() { (void)run(); }
    } join{sc, st, net->plan.nodes.size()};
    int e0 = 0;
    std::vector<mdcnn_buffer*> outs_flat;
    mdcnn_buffer* ins[kMaxBatch];
    const mdcnn_conv_desc* edges[kMaxBatch];
    mdcnn_buffer* const* outs[kMaxBatch];
    for (int i = 0; i < (int)net->sites.size(); ++i) {
        if (net->sites[i]->d.kind == MDCNN_SITE_OUTPUT) continue;
        int e1 = e0;
        while (e1 < n_edges && net->esrc[e1] == i) ++e1;
        const int ne = e1 - e0;
        outs_flat.resize((size_t)n * (ne > 0 ? ne : 1));
        for (int b = 0; b < n; ++b) {
            ins[b] = nets[b]->sites[i];
            edges[b] = nets[b]->edges.data() + e0;
            for (int e = e0; e < e1; ++e) outs_flat[(size_t)b * ne + (e - e0)] = nets[b]->sites[net->edst[e]];
            outs[b] = outs_flat.data() + (size_t)b * ne;
        }
        // a residual skip is added by the step-1 kernel of its source; its place in the
        // order of the producers of its destination stays the same as long as no other
        // edge of this call goes to the same destination before it
        const int fuse = fused_skip(net, e0, e1);
        g_tag_site = i; g_tag_edge0 = e0;
        mdcnn_status rc = do_forward(n, ins, i == 0 ? frames : nullptr, i == 0 ? forced : nullptr, edges, outs, ne, st, fuse, sc);
        g_tag_site = g_tag_edge0 = -1;
        if (rc) return rc;
        e0 = e1;
    }
    if (sc) {
        hipError_t err = join.run();
        if (err == hipSuccess) err = sched.err;
        if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "stream synchronisation: %s", hipGetErrorString(err));
    }
    for (int b = 0; b < n; ++b) {
        char* o = (char*)outs_dev[b];
        for (mdcnn_buffer* s : nets[b]->sites) {
            if (s->d.kind != MDCNN_SITE_OUTPUT) continue;
            hipError_t err = timed(kClsReadout, st, [&] { return launch_read_view(s->dev, s->d.crops ? MDCNN_VIEW_CROP_OUT : MDCNN_VIEW_OUT, o, st); });
            if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "readout launch: %s", hipGetErrorString(err));
            o += crop_pixels(s) * s->d.C * esize(s->d.dtype);
        }
    }
    unfinished.armed = false;
    return MDCNN_OK;
}

void make_pipe_plan(const mdcnn_net* net, int group_calls, int streams, int mode, PipePlan& pp) {
    const int n_sites = (int)net->sites.size(), n_edges = (int)net->edges.size();
    pp = PipePlan{};
    pp.key = (group_calls * 8 + streams) * 2 + mode;
    pp.streams = streams;
    pp.mode = mode;
    std::vector<int> call_of(n_sites, -1);
    std::vector<double> cost;
    int e0 = 0;
    for (int i = 0; i < n_sites; ++i) {
        if (net->sites[i]->d.kind == MDCNN_SITE_OUTPUT) continue;
        int e1 = e0;
        while (e1 < n_edges && net->esrc[e1] == i) ++e1;
        call_of[i] = (int)pp.call_site.size();
        pp.call_site.push_back(i);
        pp.call_e0.push_back(e0);
        pp.call_e1.push_back(e1);
        // a delta launch counts one, a convolution launch four (measured on the benchmark networks: 5-8 us against 13-27 us)
        const int fuse = fused_skip(net, e0, e1);
        cost.push_back((net->sites[i]->d.truncation_free ? 0.0 : 1.0) + 4.0 * ((e1 - e0) - (fuse >= 0 ? 1 : 0)));
        e0 = e1;
    }
    const int n_calls = (int)pp.call_site.size();
    // runs of calls of about equal cost: the smallest possible largest run (dynamic programme over the cut positions)
    pp.seg_of_call.assign((size_t)n_calls + 1, 0);
    if (mode == 0 && streams > 1) {
        const int S = streams < n_calls ? streams : n_calls;
        std::vector<double> pre((size_t)n_calls + 1, 0.0);
        for (int c = 0; c < n_calls; ++c) pre[(size_t)c + 1] = pre[(size_t)c] + cost[(size_t)c];
        std::vector<std::vector<double>> best((size_t)S + 1, std::vector<double>((size_t)n_calls + 1, 1e300));
        std::vector<std::vector<int>> cut((size_t)S + 1, std::vector<int>((size_t)n_calls + 1, 0));
        best[0][0] = 0.0;
        for (int k = 1; k <= S; ++k)
            for (int c = k; c <= n_calls; ++c)
                for (int b = k - 1; b < c; ++b) {
                    const double run = pre[(size_t)c] - pre[(size_t)b];
                    const double v = best[(size_t)k - 1][(size_t)b] > run ? best[(size_t)k - 1][(size_t)b] : run;
                    if (v < best[(size_t)k][(size_t)c]) { best[(size_t)k][(size_t)c] = v; cut[(size_t)k][(size_t)c] = b; }
                }
        int c = n_calls;
        for (int k = S; k >= 1; --k) {
            const int b = cut[(size_t)k][(size_t)c];
            for (int q = b; q < c; ++q) pp.seg_of_call[(size_t)q] = k - 1;
            c = b;
        }
        pp.seg_of_call[(size_t)n_calls] = S - 1;              // the readout follows the last call
    }
    pp.forward.assign((size_t)n_calls, 0);
    for (int c = 1; c < n_calls; ++c) pp.forward[(size_t)c] = pp.seg_of_call[(size_t)c] != pp.seg_of_call[(size_t)c - 1];
    pp.event_of_call.assign((size_t)n_calls + 1, -1);
    std::vector<char> filled(n_sites, 0);
    for (int c0 = 0; c0 < n_calls; c0 += group_calls) {
        PipeGroup g{c0, c0 + group_calls < n_calls ? c0 + group_calls : n_calls, {}, -1};
        const bool last = g.call1 == n_calls;
        for (int c = g.call0; c < g.call1; ++c) {
            auto touch = [&](int site) {
                if (filled[site]) return;
                filled[site] = 1;
                g.fill.push_back(site);
                const int w = call_of[site] >= 0 ? call_of[site] : n_calls;
                g.wait_call = w > g.wait_call ? w : g.wait_call;
            };
            touch(pp.call_site[c]);
            for (int e = pp.call_e0[c]; e < pp.call_e1[c]; ++e) touch(net->edst[e]);
        }
        if (last)                                              // sites nothing leads to are still initialised
            for (int i = 0; i < n_sites; ++i)
                if (!filled[i]) {
                    filled[i] = 1;
                    g.fill.push_back(i);
                    g.wait_call = n_calls;
                }
        if (g.wait_call >= 0 && pp.event_of_call[g.wait_call] < 0) pp.event_of_call[g.wait_call] = pp.n_events++;
        pp.groups.push_back(g);
    }
    for (int c = 1; c < n_calls; ++c)                         // the end of a run of calls is waited for by the next run
        if (pp.forward[(size_t)c] && pp.event_of_call[(size_t)c - 1] < 0) pp.event_of_call[(size_t)c - 1] = pp.n_events++;
}

constexpr int kMaxFrames = 4096;
constexpr int kDefaultDepth = 4;
constexpr int kMinLaunchesInFlight = 16;   // launches of a frame from which on the default is kDefaultDepth streams

// Masks made by the library itself for the frames of mdcnn_frames_masked.
struct FrontEnd {
    const mdcnn_mask_params* prm;
    const float* const* roi;       // per frame, or nullptr
    uint8_t* const* masks;         // per frame, written by the mask kernel, then forced at the input site
    size_t mask_bytes;
};

mdcnn_status check_mask_params(const mdcnn_mask_params* prm, int Hc, int Wc, size_t mask_bytes) {
    const int q = prm->pool;
    if ((q != 1 && q != 2 && q != 4 && q != 8) || Hc % q || Wc % q)
        return fail(MDCNN_ERR_SHAPE, "input_mask: pool must be 1, 2, 4 or 8 and divide the frame of %dx%d pixels", Hc, Wc);
    if (prm->dilate < 0 || prm->dilate > kMaskMaxDilate || (prm->suppress != 0 && prm->suppress != 1))
        return fail(MDCNN_ERR_SHAPE, "input_mask: 0 <= dilate <= %d, suppress is 0 or 1", kMaskMaxDilate);
    if (mask_bytes != (size_t)Hc * Wc) return fail(MDCNN_ERR_SIZE, "input_mask: mask_bytes is %zu, the frame has %zu pixels", mask_bytes, (size_t)Hc * Wc);
    return MDCNN_OK;
}

// n_frames consecutive frames of one network on `depth` streams (stream 0 is the caller's).  The
// launches of a frame are those of mdcnn_frame on one stream, in the same order, except that the
// initialisation of a camera shift is split up and rides along (see PipeGroup).  Frames are issued
// one after the other; two launches that touch the same site are ordered by being on the same
// stream or by an event: within a frame where the stream changes between two calls, across frames
// by the waits of the plan.  Every site sees the same sequence of launches as with one frame at a
// time, so the results are the same bit for bit.
// Forward calls per group.  Left to itself the library cuts a frame into about twenty groups, four calls at
// most: every group costs an event and a wait per frame, and a long network (config 4: 85 calls) is
// bound by those, while a short one needs the frames to follow each other closely (measured: config 3,
// 18 calls, 3.3 k frames/s with groups of 1 and 2.8 k with groups of 4; config 4 1.45 k and 1.6 k).
int pipe_group(const mdcnn_net* net) {
    if (g_pipe_group) return g_pipe_group;
    int n_calls = 0;
    for (const mdcnn_buffer* b : net->sites) n_calls += b->d.kind != MDCNN_SITE_OUTPUT;
    const int g = (n_calls + 10) / 20;
    return g < 1 ? 1 : g > 4 ? 4 : g;
}

// What the issue of one frame needs, fixed before anything is issued: the sites as they stand after the
// frame's camera shift (ring origins, crop) and their initialisation jobs.  With these, frames can be issued
// by different host threads although the camera state of the network moves on from frame to frame.
struct FrameWork {
    std::vector<mdcnn_buffer> sites;
    std::vector<FillJob> jobs;
};

// Progress of the issue of frame f, for the threads that issue other frames: done[f] = c + 1 once everything
// up to and including forward call c (the readout: n_calls) has been issued, events included.
struct IssueShared {
    std::vector<std::atomic<int>> done;
    std::atomic<bool> abort{false};
    explicit IssueShared(int n) : done((size_t)n) { for (auto& d : done) d.store(0, std::memory_order_relaxed); }
};

// nb > 1: the same for nb videos of networks of equal shape at once (one launch carries a call of all of them; no crops,
// no front end).  Everything per frame is then indexed [frame * nb + video].
mdcnn_status frame_seq(mdcnn_net* const* nets, int nb, int n_frames, const void* const* frames, const uint8_t* const* forced,
                       const int* dty, const int* dtx, const int* crops, const FrontEnd* fe, void* const* outs_dev, int depth,
                       hipStream_t user, int* did_full_reset) {
    mdcnn_net* const net = nets[0];
    const int group = pipe_group(net), key = (group * 8 + depth) * 2 + g_pipe_mode;
    if (net->pipe.key != key) make_pipe_plan(net, group, depth, g_pipe_mode, net->pipe);
    const PipePlan& pp = net->pipe;
    const int n_calls = (int)pp.call_site.size(), n_sites = (int)net->sites.size(), ring = 3;
    // events: ring x n_events for the plan, then one per stream for fork and join
    const size_t ev_sync = (size_t)ring * pp.n_events;
    hipError_t err = aux_prepare(depth, ev_sync + kMaxStreams);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "stream set-up: %s", hipGetErrorString(err));
    hipStream_t s[kMaxStreams];
    s[0] = user;
    for (int k = 1; k < depth; ++k) s[k] = g_aux.s[k - 1];
    // The camera path below moves the host state of the sites (ring origins, restrictions, crop) ahead by
    // the whole run before anything is enqueued.  If the call fails, that state must not stay ahead of the
    // device: while nothing is enqueued it is put back as it was; afterwards every site is marked as never
    // reset, so that the next camera shift re-initialises everything.
    struct HostState {
        mdcnn_net* const* nets; int nb;
        std::vector<mdcnn_buffer> saved;
        bool armed = true, enqueued = false;
        HostState(mdcnn_net* const* n, int count) : nets(n), nb(count) {
            for (int v = 0; v < nb; ++v)
                for (mdcnn_buffer* b : nets[v]->sites) saved.push_back(*b);
        }
        ~HostState() {
            if (!armed) return;
            size_t k = 0;
            for (int v = 0; v < nb; ++v)
                for (mdcnn_buffer* b : nets[v]->sites) {
                    if (!enqueued) *b = saved[k];
                    else b->fresh = true;
                    ++k;
                }
        }
    } host_state(nets, nb);
    // the camera path of the whole run, on the host: every frame gets its own copy of the sites
    std::vector<FrameWork> work((size_t)n_frames);
    {
        std::vector<FillJob> jobs;
        for (int f = 0; f < n_frames; ++f) {
            FrameWork& w = work[(size_t)f];
            w.sites.reserve((size_t)nb * n_sites);
            w.jobs.reserve((size_t)nb * n_sites);
            for (int v = 0; v < nb; ++v) {
                mdcnn_net* nv = nets[v];
                const size_t fv = (size_t)f * nb + v;
                bool full = false;
                mdcnn_status rc = shift_jobs(nv->sites.data(), n_sites, dty[fv], dtx[fv], jobs, &full);
                if (rc) return rc;
                if (did_full_reset) did_full_reset[fv] = full ? 1 : 0;
                if (crops) {                                   // (nb == 1)
                    rc = mdcnn_set_crop(nv->sites.data(), n_sites, crops[4 * f], crops[4 * f + 1], crops[4 * f + 2], crops[4 * f + 3]);
                    if (rc) return rc;
                }
                for (int i = 0; i < n_sites; ++i) w.sites.push_back(*nv->sites[(size_t)i]);
                w.jobs.insert(w.jobs.end(), jobs.begin(), jobs.end());
            }
        }
    }
    host_state.enqueued = true;
    if (depth > 1) err = hipEventRecord(g_aux.events[ev_sync], user);
    for (int k = 1; k < depth && err == hipSuccess; ++k) err = hipStreamWaitEvent(s[k], g_aux.events[ev_sync], 0);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "stream set-up: %s", hipGetErrorString(err));
    // whatever happens below, the caller's stream waits for the other streams before the call returns
    struct Join {
        hipStream_t* s; int depth; size_t base; bool done;
        hipError_t run() {
            hipError_t err = hipSuccess;
            for (int k = 1; !done && k < depth; ++k) {
                hipError_t e = hipEventRecord(g_aux.events[base + k], s[k]);
                if (e == hipSuccess) e = hipStreamWaitEvent(s[0], g_aux.events[base + k], 0);
                if (e != hipSuccess && err == hipSuccess) err = e;
            }
            done = true;
            return err;
        }
        ~Join() { (void)run(); }
    } join{s, depth, ev_sync, false};
    // which events of a frame somebody on another stream waits for (those recorded for nobody cost host time)
    std::vector<char> wanted((size_t)n_calls + 1, 0);
    for (size_t gi = 0; gi < pp.groups.size(); ++gi) {
        const PipeGroup& g = pp.groups[gi];
        const int carrier = gi ? pp.groups[gi - 1].call1 - 1 : 0;
        if (g.wait_call >= 0 && (pp.mode == 1 || pp.seg_of_call[(size_t)g.wait_call] != pp.seg_of_call[(size_t)carrier])) wanted[(size_t)g.wait_call] = 1;
    }
    for (int c = 1; c < n_calls; ++c)
        if (pp.forward[(size_t)c]) wanted[(size_t)c - 1] = 1;
    hipEvent_t* const events = g_aux.events.data();          // (thread-local storage of the calling thread)
    IssueShared shared(n_frames);

    // Issues frame f.  `threaded`: frame f - 1 is being issued by another thread, so an event of it is
    // waited for only after that thread has recorded it.
    auto issue_frame = [&](int f, bool threaded) -> mdcnn_status {
        FrameWork& w = work[(size_t)f];
        const FillJob* jobs = w.jobs.data();
        hipEvent_t* ev_prev = events + (size_t)((f + ring - 1) % ring) * pp.n_events;
        hipEvent_t* ev_mine = events + (size_t)(f % ring) * pp.n_events;
        std::vector<mdcnn_buffer*> outs_flat;
        std::vector<int> fill_all;
        hipError_t err = hipSuccess;
        // the initialisation jobs of the sites `fill` of every video
        auto launch_fills = [&](const std::vector<int>& fill, hipStream_t st) {
            if (nb == 1) return launch_fill_jobs(jobs, fill.data(), (int)fill.size(), st);
            fill_all.clear();
            for (int v = 0; v < nb; ++v)
                for (int site : fill) fill_all.push_back(v * n_sites + site);
            return launch_fill_jobs(jobs, fill_all.data(), (int)fill_all.size(), st);
        };
        auto issued = [&](int call) {                          // everything up to `call` is issued
            if (depth > 1 && wanted[(size_t)call]) err = hipEventRecord(ev_mine[pp.event_of_call[(size_t)call]], s[pp.stream_of(f, call)]);
            shared.done[(size_t)f].store(call + 1, std::memory_order_release);
            return err;
        };
        // the stream that is about to initialise the sites of group g waits for the frame before to be done with them
        auto wait_for = [&](const PipeGroup& g, int carrier) {
            if (f == 0 || depth == 1 || g.wait_call < 0) return hipSuccess;
            const int mine = pp.stream_of(f, carrier);
            if (pp.stream_of(f - 1, g.wait_call) == mine) return hipSuccess;      // same stream: in order anyway
            while (threaded && shared.done[(size_t)f - 1].load(std::memory_order_acquire) <= g.wait_call) {
                if (shared.abort.load(std::memory_order_relaxed)) return hipErrorUnknown;
                std::this_thread::yield();
            }
            return hipStreamWaitEvent(s[mine], ev_prev[pp.event_of_call[(size_t)g.wait_call]], 0);
        };
        for (size_t gi = 0; gi < pp.groups.size(); ++gi) {
            const PipeGroup& g = pp.groups[gi];
            if (gi == 0) {
                err = wait_for(g, 0);
                if (err == hipSuccess) err = launch_fills(g.fill, s[pp.stream_of(f, 0)]);
                if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "frame %d: shift launch: %s", f, hipGetErrorString(err));
                if (fe) {                                      // the input site is initialised: its mask for this frame
                    mdcnn_status rc = mdcnn_input_mask(&w.sites[0], frames[f], fe->roi ? fe->roi[f] : nullptr, fe->prm, fe->masks[f],
                                                       fe->mask_bytes, s[pp.stream_of(f, 0)]);
                    if (rc) return rc;
                }
            }
            for (int c = g.call0; c < g.call1; ++c) {
                hipStream_t st = s[pp.stream_of(f, c)];
                if (c > 0 && pp.forward[(size_t)c] && depth > 1) {            // the calls so far ran on another stream
                    err = hipStreamWaitEvent(st, ev_mine[pp.event_of_call[(size_t)c - 1]], 0);
                    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "frame %d: event: %s", f, hipGetErrorString(err));
                }
                const int* riders = nullptr;
                int n_riders = 0;
                if (c == g.call1 - 1 && gi + 1 < pp.groups.size()) {          // the next group's sites are initialised here
                    const PipeGroup& nx = pp.groups[gi + 1];
                    err = wait_for(nx, c);
                    // (a launch of several videos carries no riders)
                    if (err == hipSuccess && ((int)nx.fill.size() > kMaxRiders || nb > 1)) err = launch_fills(nx.fill, st);
                    else { riders = nx.fill.data(); n_riders = (int)nx.fill.size(); }
                    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "frame %d: shift launch: %s", f, hipGetErrorString(err));
                }
                const int i = pp.call_site[c], e0 = pp.call_e0[c], e1 = pp.call_e1[c], ne = e1 - e0, stride = ne > 0 ? ne : 1;
                outs_flat.resize((size_t)nb * stride);
                mdcnn_buffer* ins[kMaxBatch];
                const mdcnn_conv_desc* edges[kMaxBatch];
                mdcnn_buffer* const* outs[kMaxBatch];
                const void* X[kMaxBatch];
                const uint8_t* fm[kMaxBatch];
                for (int v = 0; v < nb; ++v) {
                    mdcnn_buffer* sites_v = w.sites.data() + (size_t)v * n_sites;
                    for (int e = e0; e < e1; ++e) outs_flat[(size_t)v * stride + (e - e0)] = sites_v + net->edst[e];
                    ins[v] = sites_v + i;
                    edges[v] = nets[v]->edges.data() + e0;
                    outs[v] = outs_flat.data() + (size_t)v * stride;
                    X[v] = frames[(size_t)f * nb + v];
                    fm[v] = fe ? fe->masks[f] : forced ? forced[(size_t)f * nb + v] : nullptr;
                }
                g_tag_site = i; g_tag_edge0 = e0;
                mdcnn_status rc = do_forward(nb, ins, i == 0 ? X : nullptr, i == 0 ? fm : nullptr, edges, outs, ne, st,
                                             fused_skip(net, e0, e1), nullptr, jobs, riders, n_riders);
                g_tag_site = g_tag_edge0 = -1;
                if (rc) return rc;
                if (issued(c) != hipSuccess) return fail(MDCNN_ERR_HIP, "frame %d: event: %s", f, hipGetErrorString(err));
            }
        }
        hipStream_t st = s[pp.stream_of(f, n_calls)];
        for (int v = 0; v < nb; ++v) {
            char* o = (char*)outs_dev[(size_t)f * nb + v];
            for (int i = 0; i < n_sites; ++i) {
                mdcnn_buffer& b = w.sites[(size_t)v * n_sites + i];
                if (b.d.kind != MDCNN_SITE_OUTPUT) continue;
                err = timed(kClsReadout, st, [&] { return launch_read_view(b.dev, crops ? MDCNN_VIEW_CROP_OUT : MDCNN_VIEW_OUT, o, st); });
                if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "frame %d: readout launch: %s", f, hipGetErrorString(err));
                o += crop_pixels(&b) * b.d.C * esize(b.d.dtype);
            }
        }
        if (issued(n_calls) != hipSuccess) return fail(MDCNN_ERR_HIP, "frame %d: event: %s", f, hipGetErrorString(err));
        return MDCNN_OK;
    };

    // One issuing thread per stream where whole frames go to streams and the run is long enough to pay for
    // starting them; the profiling mode keeps its event lists on the calling thread.  Frame 0 is issued first
    // and alone: it takes every kernel of the network through its first launch on this thread.
    const bool threads = g_pipe_threads && pp.mode == 1 && depth > 1 && n_frames >= 4 * depth && !g_profile;
    mdcnn_status rc = MDCNN_OK;
    if (!threads) {
        for (int f = 0; f < n_frames && rc == MDCNN_OK; ++f) rc = issue_frame(f, false);
    } else {
        rc = issue_frame(0, false);
        if (rc == MDCNN_OK) {
            int device = 0;
            (void)hipGetDevice(&device);
            std::vector<mdcnn_status> st_of((size_t)depth, MDCNN_OK);
            std::vector<std::string> msg_of((size_t)depth);
            auto worker = [&](int k) {
                if (k) (void)hipSetDevice(device);
                for (int f = k ? k : depth; f < n_frames; f += depth) {
                    if (shared.abort.load(std::memory_order_relaxed)) break;
                    const mdcnn_status r = issue_frame(f, true);
                    if (r != MDCNN_OK) {
                        st_of[(size_t)k] = r;
                        msg_of[(size_t)k] = g_err;               // the message is in this thread's buffer
                        shared.abort.store(true, std::memory_order_relaxed);
                        break;
                    }
                }
            };
            std::vector<std::thread> pool;
            for (int k = 1; k < depth; ++k) pool.emplace_back(worker, k);
            worker(0);
            for (std::thread& t : pool) t.join();
            for (int k = 0; k < depth && rc == MDCNN_OK; ++k)
                if (st_of[(size_t)k] != MDCNN_OK) rc = fail(st_of[(size_t)k], "%s", msg_of[(size_t)k].c_str());
        }
    }
    if (rc) return rc;
    err = join.run();
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "stream synchronisation: %s", hipGetErrorString(err));
    host_state.armed = false;
    return MDCNN_OK;
}

}  // namespace

extern "C" {

const char* mdcnn_last_error(void) { return g_err; }
const char* mdcnn_version(void) { return "mdcnn 0.1 (gfx950)"; }

mdcnn_status mdcnn_set_option(int option, int value) {
    if (option == MDCNN_OPT_CONV_PATH && value >= 0 && value <= 3) { g_conv_path = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_HALO && value >= 0 && value <= 4) { g_halo = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_STREAMS && value >= 0 && value <= kMaxStreams) { g_streams = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_PIPE_GROUP && value >= 0 && value <= 64) { g_pipe_group = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_PIPE_MODE && (value == 0 || value == 1)) { g_pipe_mode = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_PIPE_THREADS && (value == 0 || value == 1)) { g_pipe_threads = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_FUSE_SKIP && (value == 0 || value == 1)) { g_fuse_skip = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_HALO_SUB && (value == 0 || value == 1 || value == 2 || value == 4)) { g_halo_sub = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_PROFILE && (value == 0 || value == 1)) { g_profile = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_TILE && value >= 0 && value <= 14) { g_tile = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_PIPE && value >= 0 && value <= 2) { g_pipe = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_XCD && (value == 0 || value == 1)) { g_xcd = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_KC && (value == 0 || value == 64)) { g_kc = value; return MDCNN_OK; }
    if (option == MDCNN_OPT_CONV_F32_MFMA && (value == 0 || value == 1)) { g_f32_mfma = value; return MDCNN_OK; }
    return fail(MDCNN_ERR_SIZE, "unknown option %d / value %d", option, value);
}

mdcnn_status mdcnn_profile_read(int n_classes, double* ms, long long* launches) {
    if (!ms || !launches) return fail(MDCNN_ERR_NULL, "ms/launches is NULL");
    if (n_classes != kNumClasses) return fail(MDCNN_ERR_SIZE, "n_classes must be %d", (int)kNumClasses);
    for (int i = 0; i < n_classes; ++i) { ms[i] = 0; launches[i] = 0; }
    mdcnn_status rc = MDCNN_OK;
    for (TimedLaunch& t : g_timed) {
        float dt = 0.f;
        hipError_t err = hipEventSynchronize(t.stop);
        if (err == hipSuccess) err = hipEventElapsedTime(&dt, t.start, t.stop);
        if (err != hipSuccess) rc = fail(MDCNN_ERR_HIP, "profiling event: %s", hipGetErrorString(err));
        else { ms[t.cls] += dt; launches[t.cls] += 1; }
        g_event_pool.push_back(t.start);
        g_event_pool.push_back(t.stop);
    }
    g_timed.clear();
    return rc;
}

mdcnn_status mdcnn_profile_read_launches(int cap, int* cls, int* site, int* edge, float* us, int* n) {
    if (!cls || !site || !edge || !us || !n) return fail(MDCNN_ERR_NULL, "profile_read_launches: NULL argument");
    *n = (int)g_timed.size();
    if ((int)g_timed.size() > cap) return fail(MDCNN_ERR_SIZE, "profile_read_launches: %zu launches, room for %d", g_timed.size(), cap);
    mdcnn_status rc = MDCNN_OK;
    int k = 0;
    for (TimedLaunch& t : g_timed) {
        float dt = 0.f;
        hipError_t err = hipEventSynchronize(t.stop);
        if (err == hipSuccess) err = hipEventElapsedTime(&dt, t.start, t.stop);
        if (err != hipSuccess) rc = fail(MDCNN_ERR_HIP, "profiling event: %s", hipGetErrorString(err));
        cls[k] = t.cls; site[k] = t.site; edge[k] = t.edge; us[k] = 1e3f * dt;
        ++k;
        g_event_pool.push_back(t.start);
        g_event_pool.push_back(t.stop);
    }
    g_timed.clear();
    return rc;
}

mdcnn_status mdcnn_bench_copy(const void* src_dev, void* dst_dev, size_t bytes, void* stream) {
    if (!src_dev || !dst_dev) return fail(MDCNN_ERR_NULL, "bench_copy: NULL argument");
    if (((uintptr_t)src_dev | (uintptr_t)dst_dev | bytes) & 15) return fail(MDCNN_ERR_ALIGN, "bench_copy: pointers and size must be multiples of 16");
    const hipError_t err = launch_bench_copy(src_dev, dst_dev, bytes, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "bench_copy launch: %s", hipGetErrorString(err));
    return MDCNN_OK;
}

mdcnn_status mdcnn_bench_mfma(int iters, int blocks, float* sink_dev, void* stream, double* flops) {
    if (!sink_dev) return fail(MDCNN_ERR_NULL, "bench_mfma: sink is NULL");
    if (iters < 1 || iters > (1 << 24) || blocks < 1 || blocks > 65536) return fail(MDCNN_ERR_SIZE, "bench_mfma: iters or blocks out of range");
    const hipError_t err = launch_bench_mfma(sink_dev, iters, blocks, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "bench_mfma launch: %s", hipGetErrorString(err));
    if (flops) *flops = (double)blocks * 4.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return MDCNN_OK;
}

mdcnn_status mdcnn_pack_weights(const mdcnn_conv_desc* edge, int dtype, void* dst_dev, size_t dst_bytes, void* stream) {
    if (!edge || !edge->w_dev || !dst_dev) return fail(MDCNN_ERR_NULL, "pack_weights: NULL argument");
    if (dtype != MDCNN_F16 || edge->k < 1 || edge->k > 5 || edge->Cin < 16 || edge->Cin % 16 || edge->Cout < 32 || edge->Cout % 32)
        return fail(MDCNN_ERR_SHAPE, "pack_weights: needs fp16, 1 <= k <= 5, Cin %% 16 == 0, Cout %% 32 == 0");
    if (((uintptr_t)edge->w_dev | (uintptr_t)dst_dev) & 15) return fail(MDCNN_ERR_ALIGN, "pack_weights: pointers must be 16-byte aligned");
    const size_t want = (size_t)edge->k * edge->k * edge->Cin * edge->Cout * 2;
    if (dst_bytes != want) return fail(MDCNN_ERR_SIZE, "pack_weights: dst_bytes %zu, expected %zu", dst_bytes, want);
    const hipError_t err = launch_pack_weights(edge->w_dev, dst_dev, edge->k * edge->k, edge->Cout, edge->Cin, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "pack_weights launch: %s", hipGetErrorString(err));
    return MDCNN_OK;
}

mdcnn_status mdcnn_conv_tiles(int Hp, int Wp, int k, int max_pixels, int max_staged, int* th, int* tw, long long* tiles) {
    if (!th || !tw || !tiles) return fail(MDCNN_ERR_NULL, "conv_tiles: NULL argument");
    if (Hp < 1 || Wp < 1 || k < 1 || k > 5 || max_pixels < 1 || max_pixels > kSegPixels || max_staged < 1)
        return fail(MDCNN_ERR_SIZE, "conv_tiles: argument out of range");
    if (!tile_2d(Hp, Wp, k, max_pixels, max_staged, th, tw, tiles)) return fail(MDCNN_ERR_SHAPE, "conv_tiles: no tile of up to %d pixels has a halo of %d pixels or less", max_pixels, max_staged);
    return MDCNN_OK;
}

mdcnn_status mdcnn_conv_border(int k, int stride, int pad, int in_extent, int out_extent, int* before, int* after) {
    if (!before || !after) return fail(MDCNN_ERR_NULL, "before/after is NULL");
    return border_1d(k, stride, pad, in_extent, out_extent, before, after);
}

mdcnn_status mdcnn_buffer_bytes(const mdcnn_buffer_desc* desc, size_t* bytes) {
    mdcnn_status st = check_desc(desc);
    if (st) return st;
    if (!bytes) return fail(MDCNN_ERR_NULL, "bytes is NULL");
    Layout L;
    make_layout(*desc, L);
    *bytes = L.total;
    return MDCNN_OK;
}

mdcnn_status mdcnn_create_buffer(const mdcnn_buffer_desc* desc, void* dev_mem, size_t bytes, mdcnn_buffer** out) {
    mdcnn_status st = check_desc(desc);
    if (st) return st;
    if (!dev_mem || !out) return fail(MDCNN_ERR_NULL, "dev_mem/out is NULL");
    if ((uintptr_t)dev_mem & 255) return fail(MDCNN_ERR_ALIGN, "dev_mem must be 256-byte aligned");
    mdcnn_buffer* b = new (std::nothrow) mdcnn_buffer();
    if (!b) return fail(MDCNN_ERR_SIZE, "out of host memory");
    b->d = *desc;
    make_layout(*desc, b->L);
    if (bytes < b->L.total) {
        size_t need = b->L.total;
        delete b;
        return fail(MDCNN_ERR_SIZE, "dev_mem holds %zu bytes, %zu needed", bytes, need);
    }
    char* base = (char*)dev_mem;
    const bool hasA = desc->kind != MDCNN_SITE_OUTPUT, hasC = desc->kind != MDCNN_SITE_INPUT;
    const bool hasP = hasC && !desc->truncation_free;
    SiteDev& s = b->dev;
    s = SiteDev{};
    s.A = hasA ? base + b->L.A : nullptr;
    s.P = hasP ? base + b->L.P : nullptr;
    s.flags = hasA ? (uint8_t*)(base + b->L.flags) : nullptr;
    s.delta = hasA ? base + b->L.delta : nullptr;
    s.Y = desc->pool_prev ? base + b->L.Y : nullptr;
    s.list = hasA ? (int*)(base + b->L.list) : nullptr;
    s.lcnt = hasA ? (int*)(base + b->L.lcnt) : nullptr;
    s.lacc = hasA ? (unsigned long long*)(base + b->L.lacc) : nullptr;
    s.cacc = hasC ? (unsigned long long*)(base + b->L.cacc) : nullptr;
    s.clist = hasC ? (int*)(base + b->L.clist) : nullptr;
    s.ccnt = hasC ? (int*)(base + b->L.ccnt) : nullptr;
    s.counters = (int*)(base + b->L.counters);
    s.bias = desc->bias_dev;
    s.H = desc->H; s.W = desc->W; s.C = desc->C; s.Hp = b->L.Hp; s.Wp = b->L.Wp;
    s.by0 = desc->border[0]; s.bx0 = desc->border[2];
    s.theta = desc->theta; s.relu = desc->relu; s.kind = desc->kind; s.dtype = desc->dtype;
    s.s_off = desc->crops && hasA ? (unsigned)((b->L.S - b->L.A) / 256) : 0u;
    s.cy = (unsigned)desc->H << 16;                        // the whole view
    s.cx = (unsigned)desc->W << 16;
    b->gy = b->gx = 0;
    b->fresh = true;
    b->r_up = b->r_down = b->r_left = b->r_right = false;
    refresh_origins(b);
    *out = b;
    return MDCNN_OK;
}

mdcnn_status mdcnn_destroy_buffer(mdcnn_buffer* buf) {
    delete buf;
    return MDCNN_OK;
}

mdcnn_status mdcnn_shift_camera(mdcnn_buffer* const* bufs, int n, int dty, int dtx, void* stream, int* did_full_reset) {
    static thread_local std::vector<FillJob> jobs;
    bool full = false;
    mdcnn_status rc = shift_jobs(bufs, n, dty, dtx, jobs, &full);
    if (rc) return rc;
    const hipError_t err = launch_fill_jobs(jobs.data(), nullptr, n, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "shift launch: %s", hipGetErrorString(err));
    if (did_full_reset) *did_full_reset = full ? 1 : 0;
    return MDCNN_OK;
}

mdcnn_status mdcnn_set_crop(mdcnn_buffer* const* bufs, int n, int ty0, int tx0, int th, int tw) {
    if (!bufs || n < 1) return fail(MDCNN_ERR_NULL, "no buffers");
    for (int i = 0; i < n; ++i) {
        if (!bufs[i]) return fail(MDCNN_ERR_NULL, "buffer %d is NULL", i);
        const mdcnn_buffer_desc& d = bufs[i]->d;
        if (!d.crops) return fail(MDCNN_ERR_STATE, "buffer %d was created without crops", i);
        if (ty0 < 0 || tx0 < 0 || th < 1 || tw < 1 || ((long long)ty0 + th) * d.tile > d.H || ((long long)tx0 + tw) * d.tile > d.W)
            return fail(MDCNN_ERR_SHAPE, "buffer %d: crop of %dx%d tiles at (%d, %d) leaves the view of %dx%d pixels (tile %d)",
                        i, th, tw, ty0, tx0, d.H, d.W, d.tile);
    }
    for (int i = 0; i < n; ++i) {
        const int t = bufs[i]->d.tile;
        bufs[i]->dev.cy = (unsigned)(ty0 * t) | (unsigned)((ty0 + th) * t) << 16;
        bufs[i]->dev.cx = (unsigned)(tx0 * t) | (unsigned)((tx0 + tw) * t) << 16;
    }
    return MDCNN_OK;
}

mdcnn_status mdcnn_layer_forward(mdcnn_buffer* in, const void* frame_dev, const uint8_t* forced_mask_dev,
                                 const mdcnn_conv_desc* edges, mdcnn_buffer* const* outs, int n_edges, void* stream) {
    mdcnn_status st = validate_forward(in, frame_dev, forced_mask_dev, edges, outs, n_edges);
    if (st) return st;
    return do_forward(1, &in, &frame_dev, &forced_mask_dev, &edges, &outs, n_edges, (hipStream_t)stream);
}

mdcnn_status mdcnn_layer_forward_noalloc(mdcnn_buffer* in, const void* frame_dev, const uint8_t* forced_mask_dev,
                                         const mdcnn_conv_desc* edges, mdcnn_buffer* const* outs, int n_edges, void* stream) {
    mdcnn_status rc = validate_forward(in, frame_dev, forced_mask_dev, edges, outs, n_edges);
    if (rc) return rc;
    // the address of the array on this device, looked up once per device with that device current
    static std::mutex mu;
    static void* base_of[64] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess || dev < 0 || dev >= 64) return fail(MDCNN_ERR_HIP, "layer_forward_noalloc: cannot tell the current device");
    void* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!base_of[dev]) {
            void* p = nullptr;
            err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (err != hipSuccess || !p) return fail(MDCNN_ERR_HIP, "layer_forward_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(err));
            base_of[dev] = p;
        }
        base = base_of[dev];
    }
    // layout: the source's list, counts and running sums, then the same per edge; 256-byte aligned pieces
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return (char*)base + o; };
    ListScratch ls;
    const size_t nl = (size_t)in->L.nseg_l;
    ls.list = (int*)take(nl * kSegPixels * 4);
    ls.lcnt = (int*)take(nl * 2 * 4);
    ls.lacc = (unsigned long long*)take(nl * 2 * 8);
    for (int i = 0; i < n_edges; ++i) {
        const size_t nc = (size_t)outs[i]->L.nseg_c;
        ls.clist.push_back((int*)take(nc * kSegPixels * 4));
        ls.ccnt.push_back((int*)take(nc * 4));
        ls.cacc.push_back((unsigned long long*)take(nc * 8));
    }
    if (off > kScratchBytes)
        return fail(MDCNN_ERR_SIZE, "layer_forward_noalloc: the lists of this call take %zu bytes, the library keeps %zu", off, kScratchBytes);
    // counts and running sums start from zero (a fill kernel, not a memset: the caller may be capturing a graph)
    err = launch_zero_bytes(base, off, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "layer_forward_noalloc: fill launch: %s", hipGetErrorString(err));
    return do_forward(1, &in, &frame_dev, &forced_mask_dev, &edges, &outs, n_edges, (hipStream_t)stream, -1, nullptr, nullptr, nullptr, 0, &ls);
}

mdcnn_status mdcnn_net_create(mdcnn_buffer* const* sites, int n_sites, const int* edge_src, const int* edge_dst,
                              const mdcnn_conv_desc* edges, int n_edges, mdcnn_net** out) {
    if (!sites || !out || n_sites < 2) return fail(MDCNN_ERR_NULL, "sites/out missing or fewer than 2 sites");
    if (n_edges < 1 || !edge_src || !edge_dst || !edges) return fail(MDCNN_ERR_NULL, "edges missing");
    for (int i = 0; i < n_sites; ++i) {
        if (!sites[i]) return fail(MDCNN_ERR_NULL, "site %d is NULL", i);
        if ((sites[i]->d.kind == MDCNN_SITE_INPUT) != (i == 0))
            return fail(MDCNN_ERR_SHAPE, "site 0, and only site 0, must be the INPUT site");
        if (sites[i]->d.crops != sites[0]->d.crops)
            return fail(MDCNN_ERR_SHAPE, "site %d: crops differs from site 0", i);
    }
    for (int i = 0; i < n_edges; ++i) {
        if (edge_src[i] < 0 || edge_dst[i] >= n_sites || edge_src[i] >= edge_dst[i])
            return fail(MDCNN_ERR_SHAPE, "edge %d: needs 0 <= src < dst < n_sites", i);
        if (i && edge_src[i] < edge_src[i - 1]) return fail(MDCNN_ERR_SHAPE, "edges must be grouped by ascending source site");
        if (sites[edge_src[i]]->d.kind == MDCNN_SITE_OUTPUT) return fail(MDCNN_ERR_SHAPE, "edge %d leaves an OUTPUT site", i);
        mdcnn_status st = validate_edge(sites[edge_src[i]], sites[edge_dst[i]], edges[i], i);
        if (st) return st;
    }
    for (int i = 0; i < n_sites; ++i) {
        if (!sites[i]->d.truncation_free) continue;
        int producers = 0;
        for (int e = 0; e < n_edges; ++e) producers += edge_dst[e] == i;
        if (producers != 1) return fail(MDCNN_ERR_SHAPE, "site %d is truncation-free and has %d producers (it needs exactly one)", i, producers);
    }
    mdcnn_net* net = new (std::nothrow) mdcnn_net();
    if (!net) return fail(MDCNN_ERR_SIZE, "out of host memory");
    net->sites.assign(sites, sites + n_sites);
    net->esrc.assign(edge_src, edge_src + n_edges);
    net->edst.assign(edge_dst, edge_dst + n_edges);
    net->edges.assign(edges, edges + n_edges);
    net->out_bytes = 0;
    for (int i = 0; i < n_sites; ++i)
        if (sites[i]->d.kind == MDCNN_SITE_OUTPUT)
            net->out_bytes += (size_t)sites[i]->d.H * sites[i]->d.W * sites[i]->d.C * esize(sites[i]->d.dtype);
    *out = net;
    return MDCNN_OK;
}

mdcnn_status mdcnn_net_destroy(mdcnn_net* net) {
    delete net;
    return MDCNN_OK;
}

mdcnn_status mdcnn_frame(mdcnn_net* net, const void* frame_dev, const uint8_t* forced_mask_dev, int dty, int dtx,
                         void* out_dev, size_t out_bytes, void* stream, int* did_full_reset) {
    if (!net) return fail(MDCNN_ERR_NULL, "net is NULL");
    if (!frame_dev || !out_dev) return fail(MDCNN_ERR_NULL, "frame/out is NULL");
    if (((uintptr_t)frame_dev | (uintptr_t)out_dev) & 15) return fail(MDCNN_ERR_ALIGN, "frame/out must be 16-byte aligned");
    if (out_bytes != net->out_bytes) return fail(MDCNN_ERR_SIZE, "out_bytes is %zu, the outputs take %zu", out_bytes, net->out_bytes);
    if (!whole_view(net->sites[0])) return fail(MDCNN_ERR_STATE, "the network has a crop smaller than its view: use mdcnn_frame_crop");
    return frame_batch(&net, 1, &frame_dev, &forced_mask_dev, &dty, &dtx, &out_dev, stream, did_full_reset);
}

mdcnn_status mdcnn_frame_crop(mdcnn_net* net, const void* frame_dev, const uint8_t* forced_mask_dev, int dty, int dtx,
                              int ty0, int tx0, int th, int tw, void* out_dev, size_t out_bytes, void* stream,
                              int* did_full_reset) {
    if (!net) return fail(MDCNN_ERR_NULL, "net is NULL");
    if (!frame_dev || !out_dev) return fail(MDCNN_ERR_NULL, "frame/out is NULL");
    if (((uintptr_t)frame_dev | (uintptr_t)out_dev) & 15) return fail(MDCNN_ERR_ALIGN, "frame/out must be 16-byte aligned");
    // all checks first: a refused call changes nothing
    size_t need = 0;
    for (const mdcnn_buffer* b : net->sites) {
        const mdcnn_buffer_desc& d = b->d;
        if (!d.crops) return fail(MDCNN_ERR_STATE, "the network was created without crops");
        if (ty0 < 0 || tx0 < 0 || th < 1 || tw < 1 || ((long long)ty0 + th) * d.tile > d.H || ((long long)tx0 + tw) * d.tile > d.W)
            return fail(MDCNN_ERR_SHAPE, "crop of %dx%d tiles at (%d, %d) leaves a view of %dx%d pixels (tile %d)", th, tw, ty0, tx0, d.H, d.W, d.tile);
        if (d.kind == MDCNN_SITE_OUTPUT) need += (size_t)th * d.tile * tw * d.tile * d.C * esize(d.dtype);
    }
    if (out_bytes != need) return fail(MDCNN_ERR_SIZE, "out_bytes is %zu, the cropped outputs take %zu", out_bytes, need);
    mdcnn_status rc = mdcnn_set_crop(net->sites.data(), (int)net->sites.size(), ty0, tx0, th, tw);
    if (rc) return rc;
    return frame_batch(&net, 1, &frame_dev, &forced_mask_dev, &dty, &dtx, &out_dev, stream, did_full_reset);
}

mdcnn_status mdcnn_frame_plan(mdcnn_net* net, int streams, int* stream_of, int* waits_of, int cap, int* n_launches,
                              int* n_streams) {
    if (!net) return fail(MDCNN_ERR_NULL, "net is NULL");
    if (streams < 0 || streams > kMaxStreams) return fail(MDCNN_ERR_SIZE, "frame_plan: 0 <= streams <= %d", kMaxStreams);
    Plan plan;
    choose_plan(net, streams, plan);
    const int n = (int)plan.nodes.size();
    if ((stream_of || waits_of) && cap < n) return fail(MDCNN_ERR_SIZE, "frame_plan: %d launches, room for %d", n, cap);
    for (int i = 0; i < n; ++i) {
        const PlanNode& nd = plan.nodes[i];
        if (stream_of) stream_of[i] = nd.stream;
        if (waits_of) {
            waits_of[2 * i] = nd.wait.size() > 0 ? nd.wait[0] : -1;
            waits_of[2 * i + 1] = nd.wait.size() > 1 ? nd.wait[1] : -1;
        }
    }
    if (n_launches) *n_launches = n;
    if (n_streams) *n_streams = plan.streams;
    return MDCNN_OK;
}

mdcnn_status mdcnn_frame_batch(mdcnn_net* const* nets, int n_streams, const void* const* frames_dev,
                               const uint8_t* const* forced_masks_dev, const int* dty, const int* dtx,
                               void* const* outs_dev, size_t out_bytes, void* stream, int* did_full_reset) {
    if (!nets || !frames_dev || !dty || !dtx || !outs_dev) return fail(MDCNN_ERR_NULL, "frame_batch: NULL argument");
    if (n_streams < 1 || n_streams > kMaxBatchStreams) return fail(MDCNN_ERR_SIZE, "frame_batch: 1 <= n_streams <= %d", kMaxBatchStreams);
    const uint8_t* no_forced[kMaxBatchStreams] = {};
    for (int b = 0; b < n_streams; ++b) {
        if (!nets[b] || !frames_dev[b] || !outs_dev[b]) return fail(MDCNN_ERR_NULL, "frame_batch: stream %d: net/frame/out is NULL", b);
        if (((uintptr_t)frames_dev[b] | (uintptr_t)outs_dev[b]) & 15) return fail(MDCNN_ERR_ALIGN, "frame_batch: stream %d: frame/out must be 16-byte aligned", b);
        if (out_bytes != nets[b]->out_bytes) return fail(MDCNN_ERR_SIZE, "frame_batch: out_bytes is %zu, the outputs take %zu", out_bytes, nets[b]->out_bytes);
        if (!whole_view(nets[b]->sites[0])) return fail(MDCNN_ERR_STATE, "frame_batch: stream %d has a crop smaller than its view", b);
        if (b && !same_shape(nets[0], nets[b])) return fail(MDCNN_ERR_SHAPE, "frame_batch: stream %d differs from stream 0 in topology or shapes", b);
        for (int c = 0; c < b; ++c)
            if (nets[c] == nets[b] || nets[c]->sites[0] == nets[b]->sites[0])
                return fail(MDCNN_ERR_STATE, "frame_batch: streams %d and %d share a network or buffers", c, b);
    }
    // the descriptors of a launch travel as kernel arguments, kMaxBatch streams to a launch: larger batches go in
    // groups of that many, one group after the other on the caller's stream (the streams are independent)
    if (!forced_masks_dev) forced_masks_dev = no_forced;
    for (int b0 = 0; b0 < n_streams; b0 += kMaxBatch) {
        const int nb = n_streams - b0 < kMaxBatch ? n_streams - b0 : kMaxBatch;
        const mdcnn_status rc = frame_batch(nets + b0, nb, frames_dev + b0, forced_masks_dev + b0, dty + b0, dtx + b0, outs_dev + b0, stream,
                                            did_full_reset ? did_full_reset + b0 : nullptr);
        if (rc) return rc;
    }
    return MDCNN_OK;
}

mdcnn_status mdcnn_frame_batch_crop(mdcnn_net* const* nets, int n_streams, const void* const* frames_dev,
                                    const uint8_t* const* forced_masks_dev, const int* dty, const int* dtx, const int* crops,
                                    void* const* outs_dev, const size_t* out_bytes, void* stream, int* did_full_reset) {
    if (!nets || !frames_dev || !dty || !dtx || !crops || !outs_dev || !out_bytes) return fail(MDCNN_ERR_NULL, "frame_batch_crop: NULL argument");
    if (n_streams < 1 || n_streams > kMaxBatchStreams) return fail(MDCNN_ERR_SIZE, "frame_batch_crop: 1 <= n_streams <= %d", kMaxBatchStreams);
    const uint8_t* no_forced[kMaxBatchStreams] = {};
    // all checks first: a refused call changes nothing
    for (int b = 0; b < n_streams; ++b) {
        if (!nets[b] || !frames_dev[b] || !outs_dev[b]) return fail(MDCNN_ERR_NULL, "frame_batch_crop: stream %d: net/frame/out is NULL", b);
        if (((uintptr_t)frames_dev[b] | (uintptr_t)outs_dev[b]) & 15) return fail(MDCNN_ERR_ALIGN, "frame_batch_crop: stream %d: frame/out must be 16-byte aligned", b);
        if (b && !same_shape(nets[0], nets[b])) return fail(MDCNN_ERR_SHAPE, "frame_batch_crop: stream %d differs from stream 0 in topology or shapes", b);
        for (int c = 0; c < b; ++c)
            if (nets[c] == nets[b] || nets[c]->sites[0] == nets[b]->sites[0])
                return fail(MDCNN_ERR_STATE, "frame_batch_crop: streams %d and %d share a network or buffers", c, b);
        const int ty0 = crops[4 * b], tx0 = crops[4 * b + 1], th = crops[4 * b + 2], tw = crops[4 * b + 3];
        size_t need = 0;
        for (const mdcnn_buffer* s : nets[b]->sites) {
            const mdcnn_buffer_desc& d = s->d;
            if (!d.crops) return fail(MDCNN_ERR_STATE, "frame_batch_crop: stream %d: the network was created without crops", b);
            if (ty0 < 0 || tx0 < 0 || th < 1 || tw < 1 || ((long long)ty0 + th) * d.tile > d.H || ((long long)tx0 + tw) * d.tile > d.W)
                return fail(MDCNN_ERR_SHAPE, "frame_batch_crop: stream %d: crop of %dx%d tiles at (%d, %d) leaves a view of %dx%d pixels (tile %d)", b, th, tw, ty0, tx0, d.H, d.W, d.tile);
            if (d.kind == MDCNN_SITE_OUTPUT) need += (size_t)th * d.tile * tw * d.tile * d.C * esize(d.dtype);
        }
        if (out_bytes[b] != need) return fail(MDCNN_ERR_SIZE, "frame_batch_crop: stream %d: out_bytes is %zu, the cropped outputs take %zu", b, out_bytes[b], need);
    }
    for (int b = 0; b < n_streams; ++b) {
        const mdcnn_status rc = mdcnn_set_crop(nets[b]->sites.data(), (int)nets[b]->sites.size(), crops[4 * b], crops[4 * b + 1], crops[4 * b + 2], crops[4 * b + 3]);
        if (rc) return rc;
    }
    if (!forced_masks_dev) forced_masks_dev = no_forced;
    for (int b0 = 0; b0 < n_streams; b0 += kMaxBatch) {
        const int nb = n_streams - b0 < kMaxBatch ? n_streams - b0 : kMaxBatch;
        const mdcnn_status rc = frame_batch(nets + b0, nb, frames_dev + b0, forced_masks_dev + b0, dty + b0, dtx + b0, outs_dev + b0, stream,
                                            did_full_reset ? did_full_reset + b0 : nullptr);
        if (rc) return rc;
    }
    return MDCNN_OK;
}

// Checks shared by mdcnn_frames and mdcnn_frames_crop; out_bytes[f] (crops) or out_bytes[0] (none) per frame.
static mdcnn_status frames_checked(mdcnn_net* net, int n_frames, const void* const* frames_dev, const uint8_t* const* forced_masks_dev,
                                   const int* dty, const int* dtx, const int* crops, const FrontEnd* fe, void* const* outs_dev,
                                   const size_t* out_bytes, int depth, void* stream, int* did_full_reset) {
    if (!net || !frames_dev || !dty || !dtx || !outs_dev || !out_bytes) return fail(MDCNN_ERR_NULL, "frames: NULL argument");
    if (n_frames < 1 || n_frames > kMaxFrames) return fail(MDCNN_ERR_SIZE, "frames: 1 <= n_frames <= %d", kMaxFrames);
    if (depth < 0 || depth > kMaxStreams) return fail(MDCNN_ERR_SIZE, "frames: 0 <= depth <= %d", kMaxStreams);
    if (!crops && out_bytes[0] != net->out_bytes) return fail(MDCNN_ERR_SIZE, "frames: out_bytes is %zu, the outputs take %zu", out_bytes[0], net->out_bytes);
    if (!crops && !whole_view(net->sites[0])) return fail(MDCNN_ERR_STATE, "frames: the network has a crop smaller than its view: use mdcnn_frames_crop");
    for (int f = 0; f < n_frames; ++f) {
        if (!frames_dev[f] || !outs_dev[f]) return fail(MDCNN_ERR_NULL, "frames: frame %d: frame/out is NULL", f);
        if (((uintptr_t)frames_dev[f] | (uintptr_t)outs_dev[f]) & 15) return fail(MDCNN_ERR_ALIGN, "frames: frame %d: frame/out must be 16-byte aligned", f);
        if (!crops) continue;
        const int ty0 = crops[4 * f], tx0 = crops[4 * f + 1], th = crops[4 * f + 2], tw = crops[4 * f + 3];
        size_t need = 0;
        for (const mdcnn_buffer* b : net->sites) {
            const mdcnn_buffer_desc& d = b->d;
            if (!d.crops) return fail(MDCNN_ERR_STATE, "frames: the network was created without crops");
            if (ty0 < 0 || tx0 < 0 || th < 1 || tw < 1 || ((long long)ty0 + th) * d.tile > d.H || ((long long)tx0 + tw) * d.tile > d.W)
                return fail(MDCNN_ERR_SHAPE, "frames: frame %d: crop of %dx%d tiles at (%d, %d) leaves a view of %dx%d pixels (tile %d)", f, th, tw, ty0, tx0, d.H, d.W, d.tile);
            if (d.kind == MDCNN_SITE_OUTPUT) need += (size_t)th * d.tile * tw * d.tile * d.C * esize(d.dtype);
        }
        if (out_bytes[f] != need) return fail(MDCNN_ERR_SIZE, "frames: frame %d: out_bytes is %zu, the cropped outputs take %zu", f, out_bytes[f], need);
    }
    if (fe) {
        const mdcnn_buffer* in = net->sites[0];
        if (!fe->prm || !fe->masks) return fail(MDCNN_ERR_NULL, "frames: mask parameters / mask buffers missing");
        mdcnn_status rc = check_mask_params(fe->prm, in->d.H, in->d.W, fe->mask_bytes);
        if (rc) return rc;
        std::vector<const uint8_t*> m((size_t)n_frames);
        for (int f = 0; f < n_frames; ++f) {
            if (!fe->masks[f]) return fail(MDCNN_ERR_NULL, "frames: frame %d: mask buffer is NULL", f);
            if (fe->roi && ((uintptr_t)fe->roi[f] & 3)) return fail(MDCNN_ERR_ALIGN, "frames: frame %d: misaligned roi", f);
            m[(size_t)f] = fe->masks[f];
        }
        std::sort(m.begin(), m.end());
        for (int f = 1; f < n_frames; ++f)
            if (m[(size_t)f] < m[(size_t)f - 1] + fe->mask_bytes) return fail(MDCNN_ERR_STATE, "frames: two mask buffers overlap");
    }
    // frames in flight write their outputs in no fixed order: no two may share memory
    std::vector<std::pair<const char*, size_t>> o((size_t)n_frames);
    for (int f = 0; f < n_frames; ++f) o[(size_t)f] = {(const char*)outs_dev[f], out_bytes[crops ? f : 0]};
    std::sort(o.begin(), o.end());
    for (int f = 1; f < n_frames; ++f)
        if (o[(size_t)f].first < o[(size_t)f - 1].first + o[(size_t)f - 1].second) return fail(MDCNN_ERR_STATE, "frames: two output buffers overlap");
    if (depth == 0) {
        // frames of a short network are too small a unit: the events cost more than the overlap gains
        Plan one;
        make_plan(net, 1, one);
        depth = (int)one.nodes.size() >= kMinLaunchesInFlight ? kDefaultDepth : 1;
    }
    if (n_frames == 1) depth = 1;
    return frame_seq(&net, 1, n_frames, frames_dev, forced_masks_dev, dty, dtx, crops, fe, outs_dev, depth, (hipStream_t)stream, did_full_reset);
}

mdcnn_status mdcnn_frames(mdcnn_net* net, int n_frames, const void* const* frames_dev, const uint8_t* const* forced_masks_dev,
                          const int* dty, const int* dtx, void* const* outs_dev, size_t out_bytes, int depth, void* stream,
                          int* did_full_reset) {
    return frames_checked(net, n_frames, frames_dev, forced_masks_dev, dty, dtx, nullptr, nullptr, outs_dev, &out_bytes, depth, stream, did_full_reset);
}

mdcnn_status mdcnn_frames_crop(mdcnn_net* net, int n_frames, const void* const* frames_dev, const uint8_t* const* forced_masks_dev,
                               const int* dty, const int* dtx, const int* crops, void* const* outs_dev, const size_t* out_bytes,
                               int depth, void* stream, int* did_full_reset) {
    if (!crops) return fail(MDCNN_ERR_NULL, "frames_crop: crops is NULL");
    return frames_checked(net, n_frames, frames_dev, forced_masks_dev, dty, dtx, crops, nullptr, outs_dev, out_bytes, depth, stream, did_full_reset);
}

mdcnn_status mdcnn_frames_masked(mdcnn_net* net, int n_frames, const void* const* frames_dev, const float* const* roi_dev,
                                 const mdcnn_mask_params* prm, uint8_t* const* masks_dev, size_t mask_bytes, const int* dty, const int* dtx,
                                 void* const* outs_dev, size_t out_bytes, int depth, void* stream, int* did_full_reset) {
    if (!prm || !masks_dev) return fail(MDCNN_ERR_NULL, "frames_masked: mask parameters / mask buffers missing");
    const FrontEnd fe{prm, roi_dev, masks_dev, mask_bytes};
    return frames_checked(net, n_frames, frames_dev, nullptr, dty, dtx, nullptr, &fe, outs_dev, &out_bytes, depth, stream, did_full_reset);
}

mdcnn_status mdcnn_frames_batch(mdcnn_net* const* nets, int n_streams, int n_frames, const void* const* frames_dev,
                                const uint8_t* const* forced_masks_dev, const int* dty, const int* dtx, void* const* outs_dev,
                                size_t out_bytes, int depth, void* stream, int* did_full_reset) {
    if (!nets || !frames_dev || !dty || !dtx || !outs_dev) return fail(MDCNN_ERR_NULL, "frames_batch: NULL argument");
    if (n_streams < 1 || n_streams > kMaxBatchStreams) return fail(MDCNN_ERR_SIZE, "frames_batch: 1 <= n_streams <= %d", kMaxBatchStreams);
    if (n_frames < 1 || n_frames > kMaxFrames) return fail(MDCNN_ERR_SIZE, "frames_batch: 1 <= n_frames <= %d", kMaxFrames);
    if (depth < 0 || depth > kMaxStreams) return fail(MDCNN_ERR_SIZE, "frames_batch: 0 <= depth <= %d", kMaxStreams);
    for (int b = 0; b < n_streams; ++b) {
        if (!nets[b]) return fail(MDCNN_ERR_NULL, "frames_batch: stream %d: net is NULL", b);
        if (out_bytes != nets[b]->out_bytes) return fail(MDCNN_ERR_SIZE, "frames_batch: out_bytes is %zu, the outputs take %zu", out_bytes, nets[b]->out_bytes);
        if (!whole_view(nets[b]->sites[0])) return fail(MDCNN_ERR_STATE, "frames_batch: stream %d has a crop smaller than its view", b);
        if (b && !same_shape(nets[0], nets[b])) return fail(MDCNN_ERR_SHAPE, "frames_batch: stream %d differs from stream 0 in topology or shapes", b);
        for (int c = 0; c < b; ++c)
            if (nets[c] == nets[b] || nets[c]->sites[0] == nets[b]->sites[0])
                return fail(MDCNN_ERR_STATE, "frames_batch: streams %d and %d share a network or buffers", c, b);
    }
    const size_t total = (size_t)n_frames * n_streams;
    for (size_t k = 0; k < total; ++k) {
        if (!frames_dev[k] || !outs_dev[k]) return fail(MDCNN_ERR_NULL, "frames_batch: frame %zu, stream %zu: frame/out is NULL", k / n_streams, k % n_streams);
        if (((uintptr_t)frames_dev[k] | (uintptr_t)outs_dev[k]) & 15) return fail(MDCNN_ERR_ALIGN, "frames_batch: frame %zu, stream %zu: frame/out must be 16-byte aligned", k / n_streams, k % n_streams);
    }
    {   // frames in flight write their outputs in no fixed order: no two may share memory
        std::vector<const char*> o((size_t)total);
        for (size_t k = 0; k < total; ++k) o[k] = (const char*)outs_dev[k];
        std::sort(o.begin(), o.end());
        for (size_t k = 1; k < total; ++k)
            if (o[k] < o[k - 1] + out_bytes) return fail(MDCNN_ERR_STATE, "frames_batch: two output buffers overlap");
    }
    if (depth == 0) {
        Plan one;
        make_plan(nets[0], 1, one);
        depth = (int)one.nodes.size() >= kMinLaunchesInFlight ? kDefaultDepth : 1;
    }
    if (n_frames == 1) depth = 1;
    if (n_streams <= kMaxBatch)
        return frame_seq(nets, n_streams, n_frames, frames_dev, forced_masks_dev, dty, dtx, nullptr, nullptr, outs_dev, depth, (hipStream_t)stream, did_full_reset);
    // the descriptors of a launch travel as kernel arguments, kMaxBatch videos to a launch: more videos go in groups of
    // that many, the whole run of one group after that of the other on the caller's stream
    std::vector<const void*> fr;
    std::vector<const uint8_t*> fm;
    std::vector<void*> out;
    std::vector<int> sy, sx, reset;
    for (int b0 = 0; b0 < n_streams; b0 += kMaxBatch) {
        const int nb = n_streams - b0 < kMaxBatch ? n_streams - b0 : kMaxBatch;
        fr.clear(); fm.clear(); out.clear(); sy.clear(); sx.clear();
        for (int f = 0; f < n_frames; ++f)
            for (int v = 0; v < nb; ++v) {
                const size_t k = (size_t)f * n_streams + b0 + v;
                fr.push_back(frames_dev[k]);
                fm.push_back(forced_masks_dev ? forced_masks_dev[k] : nullptr);
                out.push_back(outs_dev[k]);
                sy.push_back(dty[k]);
                sx.push_back(dtx[k]);
            }
        reset.assign((size_t)n_frames * nb, 0);
        const mdcnn_status rc = frame_seq(nets + b0, nb, n_frames, fr.data(), forced_masks_dev ? fm.data() : nullptr, sy.data(), sx.data(), nullptr, nullptr,
                                          out.data(), depth, (hipStream_t)stream, reset.data());
        if (rc) return rc;
        for (int f = 0; did_full_reset && f < n_frames; ++f)
            for (int v = 0; v < nb; ++v) did_full_reset[(size_t)f * n_streams + b0 + v] = reset[(size_t)f * nb + v];
    }
    return MDCNN_OK;
}

mdcnn_status mdcnn_frames_plan(mdcnn_net* net, int depth, int* first_call, int* wait_call, int* init_call, int cap_groups,
                               int* group_of_site, int cap_sites, int* stream_of_call, int cap_calls, int* n_groups, int* n_calls) {
    if (!net) return fail(MDCNN_ERR_NULL, "net is NULL");
    if (depth < 0 || depth > kMaxStreams) return fail(MDCNN_ERR_SIZE, "frames_plan: 0 <= depth <= %d", kMaxStreams);
    PipePlan pp;
    make_pipe_plan(net, pipe_group(net), depth ? depth : kDefaultDepth, g_pipe_mode, pp);
    const int n = (int)pp.groups.size(), n_sites = (int)net->sites.size(), nc = (int)pp.call_site.size();
    if ((first_call || wait_call || init_call) && cap_groups < n) return fail(MDCNN_ERR_SIZE, "frames_plan: %d groups, room for %d", n, cap_groups);
    if (group_of_site && cap_sites < n_sites) return fail(MDCNN_ERR_SIZE, "frames_plan: %d sites, room for %d", n_sites, cap_sites);
    if (stream_of_call && cap_calls < nc + 1) return fail(MDCNN_ERR_SIZE, "frames_plan: %d calls and the readout, room for %d", nc, cap_calls);
    for (int g = 0; g < n; ++g) {
        if (first_call) first_call[g] = pp.groups[g].call0;
        if (wait_call) wait_call[g] = pp.groups[g].wait_call;
        if (init_call) init_call[g] = g ? pp.groups[g - 1].call1 - 1 : -1;
        if (group_of_site)
            for (int site : pp.groups[g].fill) group_of_site[site] = g;
    }
    for (int c = 0; stream_of_call && c <= nc; ++c) stream_of_call[c] = pp.mode ? -1 : pp.seg_of_call[(size_t)c];
    if (n_groups) *n_groups = n;
    if (n_calls) *n_calls = nc;
    return MDCNN_OK;
}

mdcnn_status mdcnn_input_mask(const mdcnn_buffer* in, const void* frame_dev, const float* roi_dev,
                              const mdcnn_mask_params* prm, uint8_t* mask_dev, size_t mask_bytes, void* stream) {
    if (!in || !frame_dev || !prm || !mask_dev) return fail(MDCNN_ERR_NULL, "input_mask: NULL argument");
    if (in->d.kind != MDCNN_SITE_INPUT) return fail(MDCNN_ERR_SHAPE, "input_mask: needs an INPUT site");
    if (in->fresh) return fail(MDCNN_ERR_STATE, "input_mask: mdcnn_shift_camera must be called first");
    MaskJob j{};
    j.s = in->dev;
    j.y0 = in->d.crops ? in->dev.cy0() : 0;
    j.x0 = in->d.crops ? in->dev.cx0() : 0;
    j.Hc = in->d.crops ? in->dev.cy1() - j.y0 : in->d.H;
    j.Wc = in->d.crops ? in->dev.cx1() - j.x0 : in->d.W;
    const mdcnn_status rc = check_mask_params(prm, j.Hc, j.Wc, mask_bytes);
    if (rc) return rc;
    const int q = prm->pool;
    if ((uintptr_t)frame_dev & (esize(in->d.dtype) - 1) || (uintptr_t)roi_dev & 3) return fail(MDCNN_ERR_ALIGN, "input_mask: misaligned frame or roi");
    j.X = frame_dev; j.roi = roi_dev; j.mask = mask_dev;
    j.theta = prm->theta; j.base = prm->sens_base; j.gain = prm->sens_gain;
    j.q = q; j.suppress = prm->suppress; j.d = prm->dilate;
    const hipError_t err = launch_input_mask(j, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "input_mask launch: %s", hipGetErrorString(err));
    return MDCNN_OK;
}

static mdcnn_status view_bytes(const mdcnn_buffer* b, int what, size_t* need) {
    const mdcnn_buffer_desc& d = b->d;
    const size_t e = esize(d.dtype);
    const bool hasA = d.kind != MDCNN_SITE_OUTPUT, hasC = d.kind != MDCNN_SITE_INPUT, hasP = hasC && !d.truncation_free;
    switch (what) {
        case MDCNN_VIEW_A:
        case MDCNN_VIEW_DELTA:
            if (!hasA) return fail(MDCNN_ERR_STATE, "OUTPUT sites hold no A / delta");
            *need = (size_t)d.H * d.W * d.C * e; return MDCNN_OK;
        case MDCNN_VIEW_P:
            if (!hasP) return fail(MDCNN_ERR_STATE, "INPUT and truncation-free sites hold no P");
            *need = (size_t)b->L.Hp * b->L.Wp * d.C * e; return MDCNN_OK;
        case MDCNN_VIEW_OUT:
            if (!hasP) return fail(MDCNN_ERR_STATE, "INPUT and truncation-free sites hold no P");
            *need = (size_t)d.H * d.W * d.C * e; return MDCNN_OK;
        case MDCNN_VIEW_FLAGS:
            if (!hasA) return fail(MDCNN_ERR_STATE, "OUTPUT sites hold no flags");
            *need = (size_t)d.H * d.W; return MDCNN_OK;
        case MDCNN_VIEW_LIST:
            if (!hasA) return fail(MDCNN_ERR_STATE, "OUTPUT sites hold no list");
            *need = ((size_t)d.H * d.W + 1) * 4; return MDCNN_OK;
        case MDCNN_VIEW_CLIST:
            if (!hasC) return fail(MDCNN_ERR_STATE, "INPUT sites hold no compute list");
            *need = ((size_t)b->L.Hp * b->L.Wp + 1) * 4; return MDCNN_OK;
        case MDCNN_VIEW_STATS:
            *need = 18 * 4; return MDCNN_OK;
        case MDCNN_VIEW_POOL_PREV:
            if (!d.pool_prev) return fail(MDCNN_ERR_STATE, "the site keeps no previous pooling output");
            *need = (size_t)d.H * d.W * d.C * e; return MDCNN_OK;
        case MDCNN_VIEW_CROP_OUT:
            if (!hasP || !d.crops) return fail(MDCNN_ERR_STATE, "CROP_OUT needs a site with P and crops");
            *need = crop_pixels(b) * d.C * e; return MDCNN_OK;
        case MDCNN_VIEW_PENDING:
            if (!d.crops || !hasA) return fail(MDCNN_ERR_STATE, "the site keeps no crop state");
            *need = (size_t)d.H * d.W; return MDCNN_OK;
        default:
            return fail(MDCNN_ERR_SIZE, "unknown view %d", what);
    }
}

mdcnn_status mdcnn_read_view(const mdcnn_buffer* buf, int what, void* dst_dev, size_t bytes, void* stream) {
    if (!buf || !dst_dev) return fail(MDCNN_ERR_NULL, "buf/dst is NULL");
    if (buf->fresh) return fail(MDCNN_ERR_STATE, "buffer was never reset (shift first)");
    size_t need = 0;
    mdcnn_status st = view_bytes(buf, what, &need);
    if (st) return st;
    if (bytes != need) return fail(MDCNN_ERR_SIZE, "view %d takes %zu bytes, %zu given", what, need, bytes);
    if ((uintptr_t)dst_dev & 15) return fail(MDCNN_ERR_ALIGN, "dst must be 16-byte aligned");
    hipError_t err = launch_read_view(buf->dev, what, dst_dev, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "read launch: %s", hipGetErrorString(err));
    return MDCNN_OK;
}

mdcnn_status mdcnn_write_view(mdcnn_buffer* buf, int what, const void* src_dev, size_t bytes, void* stream) {
    if (!buf || !src_dev) return fail(MDCNN_ERR_NULL, "buf/src is NULL");
    if (buf->fresh) return fail(MDCNN_ERR_STATE, "buffer was never reset (shift first)");
    if (what != MDCNN_VIEW_A && what != MDCNN_VIEW_P && what != MDCNN_VIEW_FLAGS && what != MDCNN_VIEW_POOL_PREV && what != MDCNN_VIEW_PENDING)
        return fail(MDCNN_ERR_SIZE, "only A, P, FLAGS, POOL_PREV and PENDING can be written");
    size_t need = 0;
    mdcnn_status st = view_bytes(buf, what, &need);
    if (st) return st;
    if (bytes != need) return fail(MDCNN_ERR_SIZE, "view %d takes %zu bytes, %zu given", what, need, bytes);
    hipError_t err = launch_write_view(buf->dev, what, src_dev, (hipStream_t)stream);
    if (err != hipSuccess) return fail(MDCNN_ERR_HIP, "write launch: %s", hipGetErrorString(err));
    return MDCNN_OK;
}

}  // extern "C"

// Internal declarations shared by the host API and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "mdcnn.h"

namespace mdcnn {

constexpr int kFlagN = 1;   // newly unveiled this frame
constexpr int kFlagU = 2;   // touched by a producer this frame
constexpr int kFlagM = 4;   // updated (emitted a delta) this frame
constexpr int kFlagC = 8;   // was a candidate of step 1 this frame (statistics)
// ring-ordered state of sites with crops, kept across frames
constexpr int kStateUnseen = 1;   // allocated, no frame has covered the pixel yet
constexpr int kStateDirty = 2;    // touched by a producer while outside the crop

// counters[] of a site (int32 slots, device).  Slots [0, 8) are per-frame values
// zeroed by every camera shift; 64-bit running sums follow (index into
// (unsigned long long*)counters), zeroed when the buffer is first reset.
constexpr int kCntUpdated = 0;      // pixels updated this frame
constexpr int kCntCandidates = 1;   // pixels visited by step 1 this frame
constexpr int kNumPerFrame = 8;
constexpr int kAccUpdated = 4;      // sum of update counts
constexpr int kAccCandidates = 5;   // sum of candidate counts
constexpr int kAccMacs = 6;         // multiply-accumulates of the MFMA kernels into this site (valid taps x Cin x Cout)
constexpr int kAccCompute = 7;      // sum of compute-list lengths of edges into this site
constexpr int kAccMacsPlain = 8;    // multiply-accumulates of the plain-FMA kernels into this site
// The two multiply-accumulate sums are kept as 8 partial sums each (slot + 8 * {1, 2} + block % 8)
// so that the statistics atomics of a launch do not all hit one address.
constexpr int kAccMacsSpread = 16;  // [16, 24): MFMA partials, [24, 32): plain partials
constexpr int kNumCounters = 64;

// Lists are compacted per segment of kSegPixels consecutive linear indices:
// entries of segment g sit at list[g * kSegPixels ...], their number in cnt[g].
// Concatenating the segments in order gives the ascending list.
constexpr int kSegPixels = 256;      // = threads per block: one index per thread

// Device-side view of one site, passed to kernels by value.
struct SiteDev {
    void* A;              // ring H x W x C
    void* P;              // ring Hp x Wp x C
    uint8_t* flags;       // H*W, view order
    void* delta;          // H x W x C, view order
    int* list;            // H*W, segment-local compaction of the update mask
    int* lcnt;            // per segment of list: [2g] entries, [2g+1] candidates of step 1 (this frame)
    unsigned long long* lacc;   // per segment: running sums of the two since the first reset
    int* clist;           // Hp*Wp, segment-local compute list of the last producer
    int* ccnt;            // entries per segment of clist
    unsigned long long* cacc;   // per segment: running sum of compute-list entries
    int* counters;        // kNumCounters
    const float* bias;    // C floats or nullptr
    void* Y;              // ring H x W x C: previous max-pooling output (pool_prev sites), else nullptr
    int H, W, C, Hp, Wp;
    int by0, bx0;         // border before the view (rows, cols)
    int a_oy, a_ox;       // physical ring position of view pixel (0,0) in A
    int p_oy, p_ox;       // physical ring position of window pixel (0,0) in P
    float theta;
    int relu;
    int kind;
    int dtype;
    // Sites with crops (H, W < 65536).  s_off: their state ring S (H x W bytes, kStateUnseen | kStateDirty per
    // pixel, ring order of A) as an offset from A in units of 256 bytes, 0: no crops.  cy, cx: the rows / columns
    // of the view the frame covers, first in the low and end in the high 16 bits (whole view by default).
    unsigned s_off, cy, cx;
    __host__ __device__ uint8_t* S() const { return s_off ? (uint8_t*)A + (size_t)s_off * 256 : nullptr; }
    __host__ __device__ int cy0() const { return (int)(cy & 0xffffu); }
    __host__ __device__ int cy1() const { return (int)(cy >> 16); }
    __host__ __device__ int cx0() const { return (int)(cx & 0xffffu); }
    __host__ __device__ int cx1() const { return (int)(cx >> 16); }
};

// Destination of a residual skip fused into step 1 of its source site: the delta
// a pixel emits is also added to the pending ring of the destination (same view
// shape, same channels) and the pixel is marked touched there.  P == nullptr: none.
struct SkipDev {
    void* P;
    uint8_t* dflags;          // nullptr for OUTPUT sites
    int Hp, Wp, by0, bx0, p_oy, p_ox;
};

// Initialisation job of one site for one camera shift: everything outside the
// kept rectangle of the padded window gets P = bias, everything outside the
// kept rectangle of the view gets A = 0 and flag N.
struct FillJob {
    void* A;
    void* P;
    uint8_t* flags;
    const float* bias;
    int* counters;
    unsigned long long* lacc;   // per-segment running sums, cleared on the first reset
    unsigned long long* cacc;
    int* lcnt;                  // per-segment counts of the frame (n_lacc / n_cacc entries), cleared with them:
    int* ccnt;                  // a site no edge publishes a compute list for must still read as empty
    unsigned s_off, y_off;      // S and Y of the site as offsets from A in units of 256 bytes (0: none): pixels that
                                // enter the view get S = unseen and Y = 0
    int n_lacc, n_cacc;
    int H, W, C, Hp, Wp;
    int a_oy, a_ox, p_oy, p_ox;
    int py0, py1, px0, px1;     // kept rows / cols of the padded window (empty: all new)
    int ay0, ay1, ax0, ax1;     // kept rows / cols of the view
    int nP, nA;                 // pixels to initialise in P / in A
    int dtype;
    int reset_counters;         // 1: per-frame slots, 2: all (first reset)
    int per_block;              // items a block initialises
    unsigned block_begin;       // first block of the launch that works on this job
};
constexpr int kMaxFillJobs = 21;
struct FillBatch {
    FillJob j[kMaxFillJobs];
    int n;
    unsigned total_blocks;
};
// 16-byte chunks (or single elements) a block initialises.  A full reset is a plain fill, bound by the
// number of blocks; after a camera shift a block's time is latency (bias loads, ring arithmetic per item), so
// the strips get more, smaller blocks.
constexpr int kFillItemsPerBlockFull = 2048, kFillItemsPerBlockStrip = 512;
inline unsigned fill_blocks(const FillJob& j) {   // blocks a job takes in a launch (at least one: it clears the counters)
    const int vec = j.dtype == MDCNN_F16 ? 8 : 4;
    const long long items = (long long)(j.nP + j.nA) * (j.C % vec == 0 ? j.C / vec : j.C);
    const long long blocks = (items + j.per_block - 1) / j.per_block;
    return (unsigned)(blocks < 1 ? 1 : blocks);
}
static_assert(sizeof(FillBatch) <= 4000, "kernel arguments stay below 4 KiB");

// One edge as seen by the list and convolution kernels.
struct EdgeDev {
    // source
    const void* delta;
    const uint8_t* sflags;
    int* pub_list;            // non-null on the one edge of a forward call that also compacts
    int* pub_lcnt;            //   the source's update mask into its list L (segment-local)
    unsigned long long* pub_lacc;
    int* scounters;
    int sH, sW, Cin;
    // destination
    void* P;
    uint8_t* dflags;          // nullptr for OUTPUT sites
    int* clist;
    int* ccnt;
    unsigned long long* cacc;
    int* dcounters;
    int dH, dW, Cout, Hp, Wp, by0, bx0, p_oy, p_ox;
    // operator
    const void* w;            // [tap][cout][cin]
    const void* wp;           // the same weights packed [tap][cin/16][cout][16], or nullptr
    int k, stride, pad, up;
    // max pooling (op == 1; op == 2: the previous output of a reset pixel was zeroed with it): the source's
    // accumulated ring and the destination's previous outputs.
    // Truncation-free destination (op == 3, 1x1 convolution): there is no P; dY is the destination's
    // accumulated ring A (addressed with d_aoy, d_aox), sA its delta map (view order, written here),
    // wp its bias (floats, or nullptr) and s_relu its activation.
    const void* sA;
    void* dY;
    int s_aoy, s_aox, s_relu, d_aoy, d_aox, op;
};
constexpr int kOpTruncFree = 3;

// Several independent streams (same network, own buffers and camera paths) share
// one launch: blockIdx.z picks the stream.  The descriptors travel as kernel
// arguments (4 KiB at most), hence the limit.
constexpr int kMaxBatch = 16;
struct EdgeBatch { EdgeDev d[kMaxBatch]; };
struct Step1Batch {
    SiteDev s[kMaxBatch];
    SkipDev skip[kMaxBatch];
    const void* X[kMaxBatch];
    const uint8_t* forced[kMaxBatch];
};
// One site's step 1 and, in the same launch, initialisation jobs of OTHER sites that nothing in this
// launch touches (blocks [0, fill_blocks) of the grid; the site's own blocks follow).
constexpr int kMaxRiders = 6;
struct Step1Fill {
    SiteDev s;
    SkipDev skip;
    const void* X;
    const uint8_t* forced;
    FillJob j[kMaxRiders];
    int n;
    unsigned fill_blocks;
};
static_assert(sizeof(Step1Fill) <= 4000, "kernel arguments stay below 4 KiB");
static_assert(sizeof(EdgeBatch) <= 3800 && sizeof(Step1Batch) <= 3800, "kernel arguments stay below 4 KiB");

enum KernelClass { kClsShift = 0, kClsStep1, kClsLists, kClsConvMfma, kClsConvPlain, kClsIdentity, kClsReadout, kClsPool, kNumClasses };

hipError_t launch_shift_fill(const FillBatch& fb, hipStream_t st);
// n streams; geometry and dtype are those of stream 0 (the host checks that all agree)
hipError_t launch_step1(const Step1Batch& b, int n, hipStream_t st);
// fills in fill_blocks and the jobs' block_begin
hipError_t launch_step1_fill(Step1Fill& a, hipStream_t st);
// e.k < 0: no operator, only the compaction of the source's update mask.
// returns the kernel class that was launched in *cls
hipError_t launch_conv(const EdgeBatch& eb, int n, int dtype, int conv_path, hipStream_t st, int* cls);
extern int g_tile, g_pipe, g_xcd, g_kc, g_halo, g_halo_sub, g_f32_mfma;   // convolution tuning knobs
// host-only: the rectangle th x tw of at most `sub` pixels whose halo fits `cap` staged pixels, with the fewest tiles over an Hp x Wp window
bool tile_2d(int Hp, int Wp, int k, int sub, int cap, int* th_out, int* tw_out, long long* tiles_out);
hipError_t launch_pack_weights(const void* src, void* dst, int taps, int Cout, int Cin, hipStream_t st);
// Post-processed update mask of an INPUT site over the rectangle (y0, x0, Hc, Wc) of its view.
struct MaskJob {
    SiteDev s;
    const void* X;            // Hc x Wc x C, storage dtype
    const float* roi;         // Hc x Wc or nullptr
    uint8_t* mask;            // Hc x Wc
    int y0, x0, Hc, Wc;
    float theta, base, gain;
    int q, suppress, d;
};
constexpr int kMaskMaxDilate = 32;
hipError_t launch_input_mask(const MaskJob& j, hipStream_t st);
hipError_t launch_read_view(const SiteDev& s, int what, void* dst, hipStream_t st);
hipError_t launch_zero_bytes(void* dst, size_t bytes, hipStream_t st);      // bytes a multiple of 16, dst 16-byte aligned
hipError_t launch_bench_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
hipError_t launch_bench_mfma(float* sink, int iters, int blocks, hipStream_t st);
hipError_t launch_write_view(const SiteDev& s, int what, const void* src, hipStream_t st);

}  // namespace mdcnn

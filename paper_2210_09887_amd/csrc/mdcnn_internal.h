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

// counters[] slots (int32, device)
constexpr int kCntUpdated = 0;
constexpr int kCntCandidates = 1;
constexpr int kCntCompute = 2;
constexpr int kNumPerFrame = 8;     // slots [0, 8) are per-frame values, zeroed by every full reset
// 64-bit accumulators since buffer creation (slot = index into (unsigned long long*)counters)
constexpr int kAccUpdated = 4;      // sum of update counts
constexpr int kAccCandidates = 5;   // sum of candidate counts
constexpr int kAccMacs = 6;         // multiply-accumulates of the MFMA kernel into this site (valid taps x Cin x Cout)
constexpr int kAccCompute = 7;      // sum of compute-list lengths of edges into this site
constexpr int kAccMacsPlain = 8;    // multiply-accumulates of the plain-FMA kernel into this site
constexpr int kNumCounters = 64;

constexpr int kSegPixels = 1024;   // pixels per compaction segment

// Device-side view of one site, passed to kernels by value.
struct SiteDev {
    void* A;              // ring H x W x C
    void* P;              // ring Hp x Wp x C
    uint8_t* flags;       // H*W, view order
    void* delta;          // H x W x C, view order
    int* list;            // H*W
    int* clist;           // Hp*Wp
    int* counters;        // kNumCounters
    int* partials;        // per step-1 block update counts
    int* cpartials;       // per segment compute-list counts
    const float* bias;    // C floats or nullptr
    int H, W, C, Hp, Wp;
    int by0, bx0;         // border before the view (rows, cols)
    int a_oy, a_ox;       // physical ring position of view pixel (0,0) in A
    int p_oy, p_ox;       // physical ring position of window pixel (0,0) in P
    float theta;
    int relu;
    int kind;
    int dtype;
};

// A rectangle of "kept" pixels inside an extent; everything outside it is (re)initialised.
struct KeepRect {
    int Hn, Wn;           // extent
    int y0, y1, x0, x1;   // kept rows [y0,y1) and cols [x0,x1); empty => all pixels new
};

inline int keep_count(const KeepRect& r) {
    int rows_out = r.y0 + (r.Hn - r.y1);
    int mid = (r.y1 - r.y0) * (r.x0 + (r.Wn - r.x1));
    return rows_out * r.Wn + mid;
}

// One edge as seen by the list and convolution kernels.
struct EdgeDev {
    // source
    const void* delta;
    const uint8_t* sflags;
    const int* slist;         // L of the source
    const int* scounters;
    int sH, sW, Cin;
    // destination
    void* P;
    uint8_t* dflags;          // nullptr for OUTPUT sites
    int* clist;
    int* cpartials;
    int* dcounters;
    int dH, dW, Cout, Hp, Wp, by0, bx0, p_oy, p_ox;
    // operator
    const void* w;
    int k, stride, pad, up;
};

enum KernelClass { kClsShift = 0, kClsStep1, kClsLists, kClsConvMfma, kClsConvPlain, kClsIdentity, kClsReadout, kNumClasses };

constexpr int kMaxEdgesPerLaunch = 8;
struct EdgeBatch {
    EdgeDev e[kMaxEdgesPerLaunch];
    int n;
};

int step1_pixels_per_block(const SiteDev& s);

// reset_counters: 0 none, 1 per-frame slots, 2 everything (first reset of a buffer)
hipError_t launch_shift_fill(const SiteDev& s, const KeepRect& pr, const KeepRect& ar, int reset_counters,
                             hipStream_t st);
hipError_t launch_step1(const SiteDev& s, const void* frame, const uint8_t* forced, hipStream_t st);
hipError_t launch_lists(const SiteDev& s, const EdgeBatch& eb, bool do_compact, hipStream_t st);
// returns the kernel class that was launched in *cls
hipError_t launch_conv(const EdgeDev& e, int dtype, int conv_path, hipStream_t st, int* cls);
hipError_t launch_read_view(const SiteDev& s, int what, void* dst, hipStream_t st);
hipError_t launch_write_view(const SiteDev& s, int what, const void* src, hipStream_t st);

}  // namespace mdcnn

// Memory-bound kernels of the hot path: dynamic initialisation of unveiled
// pixels, delta + truncation + mask (input and inner sites), view-ordered
// readout.  (Compaction lives with its consumer, the convolution kernels.)
// gfx950 only: 64-wide wavefronts, ballot/popcount compaction, 16-byte accesses.
#include "mdcnn_internal.h"

namespace mdcnn {

typedef _Float16 f16;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int wrap(int v, int n) { return v >= n ? v - n : v; }

template <typename T> struct V16;
template <> struct V16<float> {
    static constexpr int N = 4;
    __device__ static void load(const float* p, float* v) {
        float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    __device__ static void store(float* p, const float* v) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct V16<f16> {
    static constexpr int N = 8;
    __device__ static void load(const f16* p, float* v) {
        f16x8 t = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
    }
    __device__ static void store(f16* p, const float* v) {
        f16x8 t;
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = (f16)v[i];   // round to nearest even
        *reinterpret_cast<f16x8*>(p) = t;
    }
};

__device__ __forceinline__ size_t a_offset(const SiteDev& s, int vy, int vx) {
    int ay = wrap(s.a_oy + vy, s.H), ax = wrap(s.a_ox + vx, s.W);
    return ((size_t)ay * s.W + ax) * s.C;
}
// wy, wx: padded-window coordinates
__device__ __forceinline__ size_t p_offset(const SiteDev& s, int wy, int wx) {
    int py = wrap(s.p_oy + wy, s.Hp), px = wrap(s.p_ox + wx, s.Wp);
    return ((size_t)py * s.Wp + px) * s.C;
}
__device__ __forceinline__ size_t skip_offset(const SkipDev& k, int vy, int vx, int C) {
    int py = wrap(k.p_oy + vy + k.by0, k.Hp), px = wrap(k.p_ox + vx + k.bx0, k.Wp);
    return ((size_t)py * k.Wp + px) * C;
}

// ---------------------------------------------------------------------------
// Dynamic initialisation, all sites of a network in one launch.  Pixels of the
// new padded window outside the kept rectangle get P = bias (the activation
// adds it later on); pixels of the new view outside the kept rectangle get
// A = 0 and flag N (sites with crops: state "unseen" in their ring S and a zero
// previous pooling output).  Per-frame counters are cleared here.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void decode_new(int Wn, int Hn, int y0, int y1, int x0, int x1, int idx, int& y, int& x) {
    const int top = y0 * Wn;
    const int bot = (Hn - y1) * Wn;
    if (idx < top) {
        y = idx / Wn; x = idx - y * Wn;
    } else if (idx < top + bot) {
        const int j = idx - top;
        const int q = j / Wn;
        y = y1 + q; x = j - q * Wn;
    } else {
        const int j = idx - top - bot;
        const int mw = x0 + (Wn - x1);
        const int q = j / mw;
        const int c = j - q * mw;
        y = y0 + q;
        x = c < x0 ? c : x1 + (c - x0);
    }
}

template <typename T, int VEC>
__device__ __forceinline__ void fill_items(const FillJob& j, unsigned lb) {
    const int chunks = j.C / VEC;
    const long long total = (long long)(j.nP + j.nA) * chunks;
    // a full reset (empty kept rectangles) needs no ring arithmetic
    const bool full = j.py0 == j.py1 && j.px0 == j.px1 && j.ay0 == j.ay1 && j.ax0 == j.ax1 && j.py0 == 0 && j.ay0 == 0;
    const long long begin = (long long)lb * j.per_block;
    long long end = begin + j.per_block;
    if (end > total) end = total;
    uint8_t* const Sr = j.s_off ? (uint8_t*)j.A + (size_t)j.s_off * 256 : nullptr;   // rings like A
    T* const Yr = j.y_off ? (T*)((char*)j.A + (size_t)j.y_off * 256) : nullptr;
    if constexpr (VEC > 1) {
        // Full reset with a power-of-two number of 16-byte chunks per pixel (<= 256): the
        // rings are filled front to back, a thread keeps its channel chunk over the whole
        // loop (block starts and the stride of 256 are multiples of `chunks`), so the loop
        // body is one store: no divisions, no bias loads.
        if (full && (chunks & (chunks - 1)) == 0 && chunks <= 256 && total < (1ll << 31)) {
            const unsigned nPc = (unsigned)j.nP * chunks, e32 = (unsigned)end;
            const int c0 = (int)(threadIdx.x & (chunks - 1)) * VEC;
            int sh = 0;
            while ((1 << sh) < chunks) ++sh;
            float bv[VEC], zv[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) { bv[i] = j.bias ? j.bias[c0 + i] : 0.f; zv[i] = 0.f; }
            for (unsigned idx = (unsigned)begin + threadIdx.x; idx < e32; idx += 256) {
                if (idx < nPc) {
                    V16<T>::store((T*)j.P + (size_t)idx * VEC, bv);
                } else {
                    const unsigned ia = idx - nPc;
                    V16<T>::store((T*)j.A + (size_t)ia * VEC, zv);
                    if (Yr) V16<T>::store(Yr + (size_t)ia * VEC, zv);
                    if (c0 == 0) {
                        j.flags[ia >> sh] = (uint8_t)kFlagN;
                        if (Sr) Sr[ia >> sh] = (uint8_t)kStateUnseen;
                    }
                }
            }
            return;
        }
    }
    for (long long idx = begin + threadIdx.x; idx < end; idx += 256) {
        const int pix = (int)(idx / chunks);
        const int c0 = (int)(idx - (long long)pix * chunks) * VEC;
        if (pix < j.nP) {
            size_t poff = (size_t)pix;                     // everything is new: any order covers the ring
            if (!full) {
                int wy, wx;
                decode_new(j.Wp, j.Hp, j.py0, j.py1, j.px0, j.px1, pix, wy, wx);
                const int py = wrap(j.p_oy + wy, j.Hp), px = wrap(j.p_ox + wx, j.Wp);
                poff = (size_t)py * j.Wp + px;
            }
            T* p = (T*)j.P + poff * j.C + c0;
            if constexpr (VEC > 1) {
                float v[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) v[i] = j.bias ? j.bias[c0 + i] : 0.f;
                V16<T>::store(p, v);
            } else {
                p[0] = (T)(j.bias ? j.bias[c0] : 0.f);
            }
        } else {
            const int ap = pix - j.nP;
            size_t aoff = (size_t)ap;
            int vlin = ap;                                 // view-linear index for the flag
            if (!full) {
                int vy, vx;
                decode_new(j.W, j.H, j.ay0, j.ay1, j.ax0, j.ax1, ap, vy, vx);
                const int ay = wrap(j.a_oy + vy, j.H), ax = wrap(j.a_ox + vx, j.W);
                aoff = (size_t)ay * j.W + ax;
                vlin = vy * j.W + vx;
            }
            T* p = (T*)j.A + aoff * j.C + c0;
            if constexpr (VEC > 1) {
                float v[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) v[i] = 0.f;
                V16<T>::store(p, v);
                if (Yr) V16<T>::store(Yr + aoff * j.C + c0, v);
            } else {
                p[0] = (T)0.f;
                if (Yr) Yr[aoff * j.C + c0] = (T)0.f;
            }
            if (c0 == 0) {
                j.flags[vlin] = (uint8_t)kFlagN;
                if (Sr) Sr[aoff] = (uint8_t)kStateUnseen;
            }
        }
    }
}

// Block lb of the initialisation job j.
__device__ __forceinline__ void fill_block(const FillJob& j, unsigned lb) {
    if (lb == 0 && j.reset_counters && (int)threadIdx.x < (j.reset_counters == 2 ? kNumCounters : kNumPerFrame))
        j.counters[threadIdx.x] = 0;
    if (lb == 0 && j.reset_counters == 2) {                // first reset: clear the per-segment running sums
        for (int i = threadIdx.x; i < j.n_lacc; i += 256) { j.lacc[i] = 0ull; j.lcnt[i] = 0; }
        for (int i = threadIdx.x; i < j.n_cacc; i += 256) { j.cacc[i] = 0ull; j.ccnt[i] = 0; }
    }
    if (j.dtype == MDCNN_F16) {
        if (j.C % 8 == 0) fill_items<f16, 8>(j, lb); else fill_items<f16, 1>(j, lb);
    } else {
        if (j.C % 4 == 0) fill_items<float, 4>(j, lb); else fill_items<float, 1>(j, lb);
    }
}

__global__ __launch_bounds__(256) void k_shift_fill(FillBatch fb) {
    int ji = 0;
    while (ji + 1 < fb.n && blockIdx.x >= fb.j[ji + 1].block_begin) ++ji;
    const FillJob& j = fb.j[ji];
    fill_block(j, blockIdx.x - j.block_begin);
}

hipError_t launch_shift_fill(const FillBatch& fb, hipStream_t st) {
    if (fb.n == 0 || fb.total_blocks == 0) return hipSuccess;
    k_shift_fill<<<dim3(fb.total_blocks), dim3(256), 0, st>>>(fb);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Step 1 of a site: delta, truncation, update mask.
//   INPUT : d = X - A
//   PREACT: d = f(A + P) - f(A)     on candidate pixels (U or N, or all if forced)
//   m = N or (forced ? forced[p] : max_c |d_c| > theta)
//   where m: A <- X (A + P), P <- 0, delta <- d
// G lanes share one pixel, each lane owns CH 16-byte chunks of its channels.
// The block writes its update / candidate counts for the compaction pass.
// ---------------------------------------------------------------------------
// Sites with crops.  A pixel inside the crop takes its flags from the state ring: newly
// unveiled if no frame has covered it since it was allocated, touched if a producer touched
// it this frame or while it lay outside earlier crops; its state is cleared.  A pixel outside
// the crop is left alone, and a touch of this frame is remembered in the ring.  All lanes of
// a pixel read the state, `writer` (one of them, same wavefront) updates it afterwards.
// Returns whether the pixel is inside; fl becomes the flags to act on, xpix the pixel's
// index in crop order.
__device__ __forceinline__ bool crop_state(const SiteDev& s, int pix, bool writer, int& fl, int& xpix) {
    const int vy = pix / s.W, vx = pix - vy * s.W;
    uint8_t* sp = s.S() + a_offset(s, vy, vx) / s.C;
    const int y0 = s.cy0(), x0 = s.cx0(), x1 = s.cx1();
    const bool inside = vy >= y0 && vy < s.cy1() && vx >= x0 && vx < x1;
    if (inside) {
        const int st = *sp;
        if (st && writer) *sp = 0;
        fl = (fl & kFlagU) | (st & kStateUnseen ? kFlagN : 0) | (st & kStateDirty ? kFlagU : 0);
        xpix = (vy - y0) * (x1 - x0) + (vx - x0);
    } else {
        if ((fl & kFlagU) && writer) *sp |= (uint8_t)kStateDirty;
        fl = 0;
    }
    return inside;
}

template <typename T, int G, int CH>
__device__ __forceinline__ void step1_block(const SiteDev& s, const SkipDev& skip, const T* __restrict__ X,
                                            const uint8_t* __restrict__ forced, unsigned blk) {
    constexpr int VEC = V16<T>::N;
    constexpr int PPB = 256 / G;
    const int tid = threadIdx.x;
    const int lp = tid % G;
    const int pix = (int)blk * PPB + tid / G;
    const int HW = s.H * s.W;
    bool m = false, cand = false;
    if (pix < HW) {
        int fl = s.flags[pix];
        const bool is_input = s.kind == MDCNN_SITE_INPUT;
        int xpix = pix;                                    // index into the frame and the forced mask
        bool inside = true;
        if (s.s_off) inside = crop_state(s, pix, lp == 0, fl, xpix);
        cand = inside && (is_input || forced != nullptr || (fl & (kFlagN | kFlagU)));
        if (cand) {
            const int vy = pix / s.W, vx = pix - vy * s.W;
            T* Ap = (T*)s.A + a_offset(s, vy, vx);
            T* Pp = is_input ? nullptr : (T*)s.P + p_offset(s, vy + s.by0, vx + s.bx0);
            const T* Xp = is_input ? X + (size_t)xpix * s.C : nullptr;
            float na[CH][VEC], out[CH][VEC];
            float mx = 0.f;
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const int c0 = (lp + j * G) * VEC;
                float a[VEC], t[VEC];
                V16<T>::load(Ap + c0, a);
                if (is_input) {
                    V16<T>::load(Xp + c0, t);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) { na[j][i] = t[i]; out[j][i] = t[i] - a[i]; }
                } else {
                    V16<T>::load(Pp + c0, t);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        float n = a[i] + t[i];
                        na[j][i] = n;
                        out[j][i] = s.relu ? fmaxf(n, 0.f) - fmaxf(a[i], 0.f) : n - a[i];
                    }
                }
#pragma unroll
                for (int i = 0; i < VEC; ++i) mx = fmaxf(mx, fabsf(out[j][i]));
            }
#pragma unroll
            for (int off = G / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
            const bool hit = forced ? forced[xpix] != 0 : mx > s.theta;
            m = (fl & kFlagN) || hit;
            if (m) {
                T* Dp = (T*)s.delta + (size_t)pix * s.C;
                float z[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) z[i] = 0.f;
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int c0 = (lp + j * G) * VEC;
                    V16<T>::store(Ap + c0, na[j]);
                    V16<T>::store(Dp + c0, out[j]);
                    if (!is_input) V16<T>::store(Pp + c0, z);
                }
                if (skip.P) {                              // fused residual skip: P_dst += delta (as stored)
                    T* Sp = (T*)skip.P + skip_offset(skip, vy, vx, s.C);
#pragma unroll
                    for (int j = 0; j < CH; ++j) {
                        const int c0 = (lp + j * G) * VEC;
                        float t[VEC];
                        V16<T>::load(Sp + c0, t);
#pragma unroll
                        for (int i = 0; i < VEC; ++i) t[i] += (float)(T)out[j][i];
                        V16<T>::store(Sp + c0, t);
                    }
                    if (lp == 0 && skip.dflags) skip.dflags[pix] |= (uint8_t)kFlagU;
                }
            }
        }
        if (lp == 0) s.flags[pix] = (uint8_t)((m ? kFlagM : 0) | (cand ? kFlagC : 0));
    }
}

template <typename T, int G, int CH>
__global__ __launch_bounds__(256) void k_step1(Step1Batch bt) {
    step1_block<T, G, CH>(bt.s[blockIdx.z], bt.skip[blockIdx.z], (const T*)bt.X[blockIdx.z], bt.forced[blockIdx.z], blockIdx.x);
}

// One site, and in the same launch the initialisation jobs of other sites: the first fill_blocks
// blocks of the grid, so that they start with the launch and not in its tail.
template <typename T, int G, int CH>
__global__ __launch_bounds__(256) void k_step1_fill(Step1Fill a) {
    if (blockIdx.x >= a.fill_blocks) {
        step1_block<T, G, CH>(a.s, a.skip, (const T*)a.X, a.forced, blockIdx.x - a.fill_blocks);
        return;
    }
    int ji = 0;
    while (ji + 1 < a.n && blockIdx.x >= a.j[ji + 1].block_begin) ++ji;
    fill_block(a.j[ji], blockIdx.x - a.j[ji].block_begin);
}

// Any channel count: one lane per pixel, scalar accesses.
template <typename T>
__device__ __forceinline__ void step1_scalar_block(const SiteDev& s, const SkipDev& skip, const T* __restrict__ X,
                                                   const uint8_t* __restrict__ forced, unsigned blk) {
    const int tid = threadIdx.x;
    const int pix = (int)blk * 256 + tid;
    const int HW = s.H * s.W;
    bool m = false, cand = false;
    if (pix < HW) {
        int fl = s.flags[pix];
        const bool is_input = s.kind == MDCNN_SITE_INPUT;
        int xpix = pix;
        bool inside = true;
        if (s.s_off) inside = crop_state(s, pix, true, fl, xpix);
        cand = inside && (is_input || forced != nullptr || (fl & (kFlagN | kFlagU)));
        if (cand) {
            const int vy = pix / s.W, vx = pix - vy * s.W;
            T* Ap = (T*)s.A + a_offset(s, vy, vx);
            T* Pp = is_input ? nullptr : (T*)s.P + p_offset(s, vy + s.by0, vx + s.bx0);
            const T* Xp = is_input ? X + (size_t)xpix * s.C : nullptr;
            float mx = 0.f;
            for (int c = 0; c < s.C; ++c) {
                float a = (float)Ap[c], o;
                if (is_input) {
                    o = (float)Xp[c] - a;
                } else {
                    float n = a + (float)Pp[c];
                    o = s.relu ? fmaxf(n, 0.f) - fmaxf(a, 0.f) : n - a;
                }
                mx = fmaxf(mx, fabsf(o));
            }
            const bool hit = forced ? forced[xpix] != 0 : mx > s.theta;
            m = (fl & kFlagN) || hit;
            if (m) {
                T* Dp = (T*)s.delta + (size_t)pix * s.C;
                T* Sp = skip.P ? (T*)skip.P + skip_offset(skip, vy, vx, s.C) : nullptr;
                if (Sp && skip.dflags) skip.dflags[pix] |= (uint8_t)kFlagU;
                for (int c = 0; c < s.C; ++c) {
                    float a = (float)Ap[c];
                    if (is_input) {
                        float x = (float)Xp[c];
                        Ap[c] = (T)x;
                        Dp[c] = (T)(x - a);
                        if (Sp) Sp[c] = (T)((float)Sp[c] + (float)Dp[c]);
                    } else {
                        float n = a + (float)Pp[c];
                        Ap[c] = (T)n;
                        Dp[c] = (T)(s.relu ? fmaxf(n, 0.f) - fmaxf(a, 0.f) : n - a);
                        Pp[c] = (T)0.f;
                        if (Sp) Sp[c] = (T)((float)Sp[c] + (float)Dp[c]);
                    }
                }
            }
        }
        s.flags[pix] = (uint8_t)((m ? kFlagM : 0) | (cand ? kFlagC : 0));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_step1_scalar(Step1Batch bt) {
    step1_scalar_block<T>(bt.s[blockIdx.z], bt.skip[blockIdx.z], (const T*)bt.X[blockIdx.z], bt.forced[blockIdx.z], blockIdx.x);
}

template <typename T>
__global__ __launch_bounds__(256) void k_step1_scalar_fill(Step1Fill a) {
    if (blockIdx.x >= a.fill_blocks) {
        step1_scalar_block<T>(a.s, a.skip, (const T*)a.X, a.forced, blockIdx.x - a.fill_blocks);
        return;
    }
    int ji = 0;
    while (ji + 1 < a.n && blockIdx.x >= a.j[ji + 1].block_begin) ++ji;
    fill_block(a.j[ji], blockIdx.x - a.j[ji].block_begin);
}

// Split C/VEC chunks into G lanes x CH chunks per lane (G a power of two <= 64,
// CH <= 4); returns false when the scalar kernel has to be used.
static bool step1_shape(int C, int vec, int& G, int& CH) {
    if (C % vec) return false;
    int n = C / vec;
    for (int ch = 1; ch <= 4; ++ch) {
        if (n % ch) continue;
        int g = n / ch;
        if (g <= 64 && (g & (g - 1)) == 0) { G = g; CH = ch; return true; }
    }
    return false;
}

template <typename T, int G>
static void step1_g(const Step1Batch& bt, int CH, dim3 grid, hipStream_t st) {
    switch (CH) {
        case 1: k_step1<T, G, 1><<<grid, dim3(256), 0, st>>>(bt); break;
        case 2: k_step1<T, G, 2><<<grid, dim3(256), 0, st>>>(bt); break;
        case 3: k_step1<T, G, 3><<<grid, dim3(256), 0, st>>>(bt); break;
        default: k_step1<T, G, 4><<<grid, dim3(256), 0, st>>>(bt); break;
    }
}
template <typename T, int G>
static void step1_g(const Step1Fill& a, int CH, dim3 grid, hipStream_t st) {
    switch (CH) {
        case 1: k_step1_fill<T, G, 1><<<grid, dim3(256), 0, st>>>(a); break;
        case 2: k_step1_fill<T, G, 2><<<grid, dim3(256), 0, st>>>(a); break;
        case 3: k_step1_fill<T, G, 3><<<grid, dim3(256), 0, st>>>(a); break;
        default: k_step1_fill<T, G, 4><<<grid, dim3(256), 0, st>>>(a); break;
    }
}
static void step1_scalar(const Step1Batch& bt, dim3 grid, hipStream_t st, float) { k_step1_scalar<float><<<grid, dim3(256), 0, st>>>(bt); }
static void step1_scalar(const Step1Batch& bt, dim3 grid, hipStream_t st, f16) { k_step1_scalar<f16><<<grid, dim3(256), 0, st>>>(bt); }
static void step1_scalar(const Step1Fill& a, dim3 grid, hipStream_t st, float) { k_step1_scalar_fill<float><<<grid, dim3(256), 0, st>>>(a); }
static void step1_scalar(const Step1Fill& a, dim3 grid, hipStream_t st, f16) { k_step1_scalar_fill<f16><<<grid, dim3(256), 0, st>>>(a); }

// Blocks the step-1 kernel of a site takes per grid layer.
static unsigned step1_blocks_of(const SiteDev& s) {
    int G = 0, CH = 0;
    const int HW = s.H * s.W;
    if (!step1_shape(s.C, s.dtype == MDCNN_F16 ? V16<f16>::N : V16<float>::N, G, CH)) return (unsigned)((HW + 255) / 256);
    const int ppb = 256 / G;
    return (unsigned)((HW + ppb - 1) / ppb);
}

// Args: Step1Batch (n grid layers) or Step1Fill (one site; `extra` blocks of initialisation jobs follow its own)
template <typename T, typename Args>
static hipError_t step1_t(const Args& a, const SiteDev& s, int n, unsigned extra, hipStream_t st) {
    int G = 0, CH = 0;
    const dim3 grid(step1_blocks_of(s) + extra, 1, n);
    if (!step1_shape(s.C, V16<T>::N, G, CH)) {
        step1_scalar(a, grid, st, T{});
        return hipGetLastError();
    }
    switch (G) {
        case 1: step1_g<T, 1>(a, CH, grid, st); break;
        case 2: step1_g<T, 2>(a, CH, grid, st); break;
        case 4: step1_g<T, 4>(a, CH, grid, st); break;
        case 8: step1_g<T, 8>(a, CH, grid, st); break;
        case 16: step1_g<T, 16>(a, CH, grid, st); break;
        case 32: step1_g<T, 32>(a, CH, grid, st); break;
        default: step1_g<T, 64>(a, CH, grid, st); break;
    }
    return hipGetLastError();
}

hipError_t launch_step1(const Step1Batch& bt, int n, hipStream_t st) {
    return bt.s[0].dtype == MDCNN_F16 ? step1_t<f16>(bt, bt.s[0], n, 0u, st) : step1_t<float>(bt, bt.s[0], n, 0u, st);
}

hipError_t launch_step1_fill(Step1Fill& a, hipStream_t st) {
    if (a.n < 0 || a.n > kMaxRiders) return hipErrorInvalidValue;
    unsigned extra = 0;
    for (int k = 0; k < a.n; ++k) {
        a.j[k].block_begin = extra;
        extra += fill_blocks(a.j[k]);
    }
    a.fill_blocks = extra;
    return a.s.dtype == MDCNN_F16 ? step1_t<f16>(a, a.s, 1, extra, st) : step1_t<float>(a, a.s, 1, extra, st);
}

// ---------------------------------------------------------------------------
// Post-processing of the input update mask.  A block owns 32 x 32 output pixels
// and keeps everything in LDS: the cells above the threshold of the region its
// dilation can reach (one more ring of cells for the suppression), the cells
// that survive the suppression, then a separable OR (along rows, then columns).
// Cells outside the frame count as not updated.  fp32 in a fixed order: the
// decisions are those of a sequential evaluation.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int floor_div(int a, int q) { return a >= 0 ? a / q : -((-a + q - 1) / q); }

constexpr int kMaskTile = 32;
constexpr int kMaskCells = kMaskTile + 2 * kMaskMaxDilate;            // cells a tile can need per axis (pool = 1)

template <typename T>
__global__ __launch_bounds__(256) void k_input_mask(MaskJob j) {
    __shared__ uint8_t s_hit[(kMaskCells + 2) * (kMaskCells + 2)];
    __shared__ uint8_t s_keep[kMaskCells * kMaskCells];
    __shared__ uint8_t s_row[kMaskCells * kMaskTile];
    const SiteDev& s = j.s;
    const int tid = threadIdx.x, q = j.q, d = j.d;
    const int ty0 = blockIdx.y * kMaskTile, tx0 = blockIdx.x * kMaskTile;
    const int gh = j.Hc / q, gw = j.Wc / q;                           // cell grid of the frame
    // cells whose pixels the dilated tile can reach
    const int ky0 = floor_div(ty0 - d, q), ky1 = floor_div(ty0 + kMaskTile - 1 + d, q);
    const int kx0 = floor_div(tx0 - d, q), kx1 = floor_div(tx0 + kMaskTile - 1 + d, q);
    const int kh = ky1 - ky0 + 1, kw = kx1 - kx0 + 1;
    const int hy0 = ky0 - 1, hx0 = kx0 - 1, hh = kh + 2, hw = kw + 2;  // one more ring for the 3 x 3 count
    const T* X = (const T*)j.X;
    auto magnitude = [&](int py, int px) {                             // of one pixel of the frame
        const T* xp = X + ((size_t)py * j.Wc + px) * s.C;
        const T* ap = (const T*)s.A + a_offset(s, j.y0 + py, j.x0 + px);
        float e = 0.f;
        if (s.C <= 4) {                                                // images: all loads go out before the first use
            float xv[4], av[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) { xv[c] = (float)xp[c < s.C ? c : 0]; av[c] = (float)ap[c < s.C ? c : 0]; }
#pragma unroll
            for (int c = 0; c < 4; ++c) e = fmaxf(e, fabsf(xv[c] - av[c]));    // a repeated channel does not change the maximum
        } else {
            for (int c = 0; c < s.C; ++c) e = fmaxf(e, fabsf((float)xp[c] - (float)ap[c]));
        }
        if (j.roi) e = e * (j.base + j.gain * j.roi[(size_t)py * j.Wc + px]);
        return e;
    };
    if (q == 1) {
        // a pixel per cell: four cells of a thread at a time, so that their loads overlap
        for (int i0 = tid; i0 < hh * hw; i0 += 4 * 256) {
            float e[4];
            bool in[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * 256;
                const int cy = hy0 + i / hw, cx = hx0 + i % hw;
                in[u] = i < hh * hw && cy >= 0 && cy < gh && cx >= 0 && cx < gw;
                e[u] = magnitude(in[u] ? cy : 0, in[u] ? cx : 0);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + u * 256 < hh * hw) s_hit[i0 + u * 256] = in[u] && e[u] > j.theta;
        }
    } else {
        for (int i = tid; i < hh * hw; i += 256) {
            const int cy = hy0 + i / hw, cx = hx0 + i % hw;
            bool hit = false;
            if (cy >= 0 && cy < gh && cx >= 0 && cx < gw) {
                float acc = 0.f;
                for (int py = cy * q; py < cy * q + q; ++py)
                    for (int px = cx * q; px < cx * q + q; ++px) acc = acc + magnitude(py, px);
                hit = acc / (float)(q * q) > j.theta;
            }
            s_hit[i] = hit;
        }
    }
    __syncthreads();
    for (int i = tid; i < kh * kw; i += 256) {
        const int r = i / kw, c = i % kw;                              // cell (ky0 + r, kx0 + c) = s_hit[(r + 1) * hw + c + 1]
        bool keep = s_hit[(r + 1) * hw + c + 1];
        if (keep && j.suppress) {
            int cnt = 0;
            for (int a = 0; a < 3; ++a)
                for (int b = 0; b < 3; ++b) cnt += s_hit[(r + a) * hw + c + b];
            keep = cnt >= 2;
        }
        s_keep[i] = keep;
    }
    __syncthreads();
    for (int i = tid; i < kh * kMaskTile; i += 256) {
        const int r = i / kMaskTile, x = tx0 + i % kMaskTile;
        const int c0 = floor_div(x - d, q) - kx0, c1 = floor_div(x + d, q) - kx0;
        bool any = false;
        for (int c = c0; c <= c1; ++c) any |= s_keep[r * kw + c] != 0;
        s_row[i] = any;
    }
    __syncthreads();
    for (int i = tid; i < kMaskTile * kMaskTile; i += 256) {
        const int yl = i / kMaskTile, xl = i % kMaskTile;
        const int y = ty0 + yl, x = tx0 + xl;
        if (y >= j.Hc || x >= j.Wc) continue;
        const int r0 = floor_div(y - d, q) - ky0, r1 = floor_div(y + d, q) - ky0;
        bool any = false;
        for (int r = r0; r <= r1; ++r) any |= s_row[r * kMaskTile + xl] != 0;
        j.mask[(size_t)y * j.Wc + x] = any;
    }
}

hipError_t launch_input_mask(const MaskJob& j, hipStream_t st) {
    const dim3 grid((j.Wc + kMaskTile - 1) / kMaskTile, (j.Hc + kMaskTile - 1) / kMaskTile);
    if (j.s.dtype == MDCNN_F16) k_input_mask<f16><<<grid, dim3(256), 0, st>>>(j);
    else k_input_mask<float><<<grid, dim3(256), 0, st>>>(j);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// View-ordered access (readout of OUTPUT sites is on the per-frame path).
// ---------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_read_tensor(SiteDev s, int what, T* __restrict__ dst) {
    const int chunks = s.C / VEC;
    const bool win = what == MDCNN_VIEW_P;
    const bool crop = what == MDCNN_VIEW_CROP_OUT;         // f(P) over the crop, in crop order
    if (crop) what = MDCNN_VIEW_OUT;
    const int Wn = win ? s.Wp : crop ? s.cx1() - s.cx0() : s.W;
    const int Hn = win ? s.Hp : crop ? s.cy1() - s.cy0() : s.H;
    const long long total = (long long)Hn * Wn * chunks;
    const long long step = (long long)gridDim.x * 256;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += step) {
        const int pix = (int)(idx / chunks);
        const int c0 = (int)(idx - (long long)pix * chunks) * VEC;
        int y = pix / Wn, x = pix - y * Wn;
        if (crop) { y += s.cy0(); x += s.cx0(); }
        const T* src;
        bool zero = false;
        if (what == MDCNN_VIEW_A) src = (const T*)s.A + a_offset(s, y, x);
        else if (what == MDCNN_VIEW_P) src = (const T*)s.P + p_offset(s, y, x);
        else if (what == MDCNN_VIEW_OUT) src = (const T*)s.P + p_offset(s, y + s.by0, x + s.bx0);
        else if (what == MDCNN_VIEW_POOL_PREV) src = (const T*)s.Y + a_offset(s, y, x);
        else { src = (const T*)s.delta + (size_t)pix * s.C; zero = !(s.flags[pix] & kFlagM); }
        T* d = dst + (size_t)pix * s.C + c0;
        if constexpr (VEC > 1) {
            float v[VEC];
            V16<T>::load(src + c0, v);
            if (what == MDCNN_VIEW_OUT && s.relu)
#pragma unroll
                for (int i = 0; i < VEC; ++i) v[i] = fmaxf(v[i], 0.f);
            if (zero)
#pragma unroll
                for (int i = 0; i < VEC; ++i) v[i] = 0.f;
            V16<T>::store(d, v);
        } else {
            float v = (float)src[c0];
            if (what == MDCNN_VIEW_OUT && s.relu) v = fmaxf(v, 0.f);
            if (zero) v = 0.f;
            d[0] = (T)v;
        }
    }
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_write_tensor(SiteDev s, int what, const T* __restrict__ src) {
    const int chunks = s.C / VEC;
    const bool win = what == MDCNN_VIEW_P;
    const int Wn = win ? s.Wp : s.W;
    const long long total = (long long)(win ? s.Hp * s.Wp : s.H * s.W) * chunks;
    const long long step = (long long)gridDim.x * 256;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += step) {
        const int pix = (int)(idx / chunks);
        const int c0 = (int)(idx - (long long)pix * chunks) * VEC;
        const int y = pix / Wn, x = pix - y * Wn;
        T* d = what == MDCNN_VIEW_A ? (T*)s.A + a_offset(s, y, x)
             : what == MDCNN_VIEW_POOL_PREV ? (T*)s.Y + a_offset(s, y, x) : (T*)s.P + p_offset(s, y, x);
        const T* sp = src + (size_t)pix * s.C + c0;
#pragma unroll
        for (int i = 0; i < VEC; ++i) d[c0 + i] = sp[i];
    }
}

// Single block: concatenates the segments of a list (ascending order), prefixed by its length.
// cnt[g * stride] = entries of segment g.
__global__ __launch_bounds__(256) void k_read_list(const int* __restrict__ list, const int* __restrict__ cnt, int stride,
                                                   int n, int* __restrict__ dst) {
    const int nseg = (n + kSegPixels - 1) / kSegPixels;
    int running = 0;
    for (int g = 0; g < nseg; ++g) {
        const int c = cnt[g * stride];
        for (int i = threadIdx.x; i < c; i += 256) dst[1 + running + i] = list[g * kSegPixels + i];
        running += c;
    }
    for (int i = running + threadIdx.x; i < n; i += 256) dst[1 + i] = -1;
    if (threadIdx.x == 0) dst[0] = running;
}

// Single block: per-frame counts and running sums of a site, added up over its segments.
__global__ __launch_bounds__(256) void k_read_stats(SiteDev s, int* __restrict__ dst) {
    __shared__ unsigned long long red[256];
    const int tid = threadIdx.x;
    const int nl = s.lcnt ? (s.H * s.W + kSegPixels - 1) / kSegPixels : 0;
    const int nc = s.ccnt ? (s.Hp * s.Wp + kSegPixels - 1) / kSegPixels : 0;
    unsigned long long v[7] = {0, 0, 0, 0, 0, 0, 0};   // upd, cand, clist (frame); upd, cand, clist (sums)
    for (int g = tid; g < nl; g += 256) { v[0] += s.lcnt[2 * g]; v[1] += s.lcnt[2 * g + 1]; v[3] += s.lacc[2 * g]; v[4] += s.lacc[2 * g + 1]; }
    for (int g = tid; g < nc; g += 256) { v[2] += s.ccnt[g]; v[5] += s.cacc[g]; }
    unsigned long long tot[6];
    for (int k = 0; k < 6; ++k) {
        __syncthreads();
        red[tid] = v[k];
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) { if (tid < o) red[tid] += red[tid + o]; __syncthreads(); }
        tot[k] = red[0];
    }
    if (tid != 0) return;
    for (int i = 0; i < 18; ++i) dst[i] = 0;
    dst[kCntUpdated] = (int)tot[0];
    dst[kCntCandidates] = (int)tot[1];
    dst[2] = (int)tot[2];
    const unsigned long long* acc = reinterpret_cast<const unsigned long long*>(s.counters);
    unsigned long long m = 0, p = 0;                        // multiply-accumulate sums: 8 partials each
    for (int j = 0; j < 8; ++j) { m += acc[kAccMacsSpread + j]; p += acc[kAccMacsSpread + 8 + j]; }
    unsigned long long* d64 = reinterpret_cast<unsigned long long*>(dst);
    d64[kAccUpdated] = tot[3];
    d64[kAccCandidates] = tot[4];
    d64[kAccMacs] = m;
    d64[kAccCompute] = tot[5];
    d64[kAccMacsPlain] = p;
}

// The state ring of a site with crops, view order <-> ring order.
__global__ __launch_bounds__(256) void k_copy_state(SiteDev s, uint8_t* __restrict__ view, int to_ring) {
    const int n = s.H * s.W, step = gridDim.x * 256;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += step) {
        const int y = i / s.W, x = i - y * s.W;
        uint8_t* r = s.S() + a_offset(s, y, x) / s.C;
        if (to_ring) *r = view[i]; else view[i] = *r;
    }
}

__global__ __launch_bounds__(256) void k_copy_bytes(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int n) {
    const int step = gridDim.x * 256;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += step) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void k_zero_bytes(uint4* __restrict__ dst, size_t n16) {
    const size_t step = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += step) dst[i] = make_uint4(0u, 0u, 0u, 0u);
}

hipError_t launch_zero_bytes(void* dst, size_t bytes, hipStream_t st) {
    if (bytes == 0) return hipSuccess;
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + 255) / 256;
    k_zero_bytes<<<dim3((unsigned)(blocks > 1024 ? 1024 : blocks)), dim3(256), 0, st>>>((uint4*)dst, n16);
    return hipGetLastError();
}

static unsigned grid_for(long long total) {
    long long b = (total + 255) / 256;
    if (b < 1) b = 1;
    if (b > 16384) b = 16384;
    return (unsigned)b;
}

template <typename T>
static hipError_t read_tensor_t(const SiteDev& s, int what, void* dst, hipStream_t st) {
    constexpr int V = V16<T>::N;
    const bool vec = (s.C % V) == 0;
    const long long pix = what == MDCNN_VIEW_P ? (long long)s.Hp * s.Wp
                        : what == MDCNN_VIEW_CROP_OUT ? (long long)(s.cy1() - s.cy0()) * (s.cx1() - s.cx0())
                                                      : (long long)s.H * s.W;
    if (vec)
        k_read_tensor<T, V><<<dim3(grid_for(pix * (s.C / V))), dim3(256), 0, st>>>(s, what, (T*)dst);
    else
        k_read_tensor<T, 1><<<dim3(grid_for(pix * s.C)), dim3(256), 0, st>>>(s, what, (T*)dst);
    return hipGetLastError();
}

hipError_t launch_read_view(const SiteDev& s, int what, void* dst, hipStream_t st) {
    switch (what) {
        case MDCNN_VIEW_A: case MDCNN_VIEW_P: case MDCNN_VIEW_DELTA: case MDCNN_VIEW_OUT: case MDCNN_VIEW_POOL_PREV:
        case MDCNN_VIEW_CROP_OUT:
            return s.dtype == MDCNN_F16 ? read_tensor_t<f16>(s, what, dst, st) : read_tensor_t<float>(s, what, dst, st);
        case MDCNN_VIEW_FLAGS:
            k_copy_bytes<<<dim3(grid_for(s.H * s.W)), dim3(256), 0, st>>>(s.flags, (uint8_t*)dst, s.H * s.W);
            return hipGetLastError();
        case MDCNN_VIEW_PENDING:
            k_copy_state<<<dim3(grid_for(s.H * s.W)), dim3(256), 0, st>>>(s, (uint8_t*)dst, 0);
            return hipGetLastError();
        case MDCNN_VIEW_LIST:
            k_read_list<<<dim3(1), dim3(256), 0, st>>>(s.list, s.lcnt, 2, s.H * s.W, (int*)dst);
            return hipGetLastError();
        case MDCNN_VIEW_CLIST:
            k_read_list<<<dim3(1), dim3(256), 0, st>>>(s.clist, s.ccnt, 1, s.Hp * s.Wp, (int*)dst);
            return hipGetLastError();
        default:
            k_read_stats<<<dim3(1), dim3(256), 0, st>>>(s, (int*)dst);
            return hipGetLastError();
    }
}

hipError_t launch_write_view(const SiteDev& s, int what, const void* src, hipStream_t st) {
    if (what == MDCNN_VIEW_FLAGS) {
        k_copy_bytes<<<dim3(grid_for(s.H * s.W)), dim3(256), 0, st>>>((const uint8_t*)src, s.flags, s.H * s.W);
        return hipGetLastError();
    }
    if (what == MDCNN_VIEW_PENDING) {
        k_copy_state<<<dim3(grid_for(s.H * s.W)), dim3(256), 0, st>>>(s, (uint8_t*)src, 1);   // read only in this mode
        return hipGetLastError();
    }
    const long long pix = what == MDCNN_VIEW_P ? (long long)s.Hp * s.Wp : (long long)s.H * s.W;
    if (s.dtype == MDCNN_F16)
        k_write_tensor<f16, 1><<<dim3(grid_for(pix * s.C)), dim3(256), 0, st>>>(s, what, (const f16*)src);
    else
        k_write_tensor<float, 1><<<dim3(grid_for(pix * s.C)), dim3(256), 0, st>>>(s, what, (const float*)src);
    return hipGetLastError();
}

}  // namespace mdcnn

// Memory-bound kernels of the hot path: dynamic initialisation of unveiled
// pixels, delta + truncation + mask (input and inner sites), stream compaction
// of the mask, compute lists of the padded convolution, view-ordered readout.
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

// ---------------------------------------------------------------------------
// Dynamic initialisation.  Pixels of the new padded window outside the kept
// rectangle get P = bias (the bias is added by the activation later on);
// pixels of the new view outside the kept rectangle get A = 0 and flag N.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void decode_new(const KeepRect& r, int idx, int& y, int& x) {
    int top = r.y0 * r.Wn;
    int bot = (r.Hn - r.y1) * r.Wn;
    if (idx < top) {
        y = idx / r.Wn; x = idx - y * r.Wn;
    } else if (idx < top + bot) {
        int j = idx - top;
        int q = j / r.Wn;
        y = r.y1 + q; x = j - q * r.Wn;
    } else {
        int j = idx - top - bot;
        int mw = r.x0 + (r.Wn - r.x1);
        int q = j / mw;
        int c = j - q * mw;
        y = r.y0 + q;
        x = c < r.x0 ? c : r.x1 + (c - r.x0);
    }
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_shift_fill(SiteDev s, KeepRect pr, KeepRect ar, int nP, int nA,
                                                    int reset_counters) {
    const int chunks = s.C / VEC;
    const long long total = (long long)(nP + nA) * chunks;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    // per-frame slots on every full reset, the accumulators only on the first one
    if (reset_counters && idx < (reset_counters == 2 ? kNumCounters : kNumPerFrame)) s.counters[idx] = 0;
    const long long step = (long long)gridDim.x * 256;
    for (; idx < total; idx += step) {
        int pix = (int)(idx / chunks);
        int c0 = (int)(idx - (long long)pix * chunks) * VEC;
        if (pix < nP) {
            int wy, wx;
            decode_new(pr, pix, wy, wx);
            T* p = (T*)s.P + p_offset(s, wy, wx) + c0;
#pragma unroll
            for (int i = 0; i < VEC; ++i) p[i] = (T)(s.bias ? s.bias[c0 + i] : 0.f);
        } else {
            int vy, vx;
            decode_new(ar, pix - nP, vy, vx);
            T* p = (T*)s.A + a_offset(s, vy, vx) + c0;
#pragma unroll
            for (int i = 0; i < VEC; ++i) p[i] = (T)0.f;
            if (c0 == 0) s.flags[vy * s.W + vx] = (uint8_t)kFlagN;
        }
    }
}

// OUTPUT sites have no A ring; they still need nothing per view pixel.  INPUT
// sites have no P ring.  The host passes nP / nA = 0 accordingly.

template <typename T>
static hipError_t shift_fill_t(const SiteDev& s, const KeepRect& pr, const KeepRect& ar, int reset_counters,
                               hipStream_t st) {
    int nP = s.P ? keep_count(pr) : 0;
    int nA = s.A ? keep_count(ar) : 0;
    if (nP + nA == 0 && !reset_counters) return hipSuccess;
    constexpr int V = 16 / sizeof(T);
    bool vec = (s.C % V) == 0;
    long long total = (long long)(nP + nA) * (vec ? s.C / V : s.C);
    long long blocks = (total + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 65536) blocks = 65536;
    if (vec)
        k_shift_fill<T, V><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(s, pr, ar, nP, nA, reset_counters);
    else
        k_shift_fill<T, 1><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(s, pr, ar, nP, nA, reset_counters);
    return hipGetLastError();
}

hipError_t launch_shift_fill(const SiteDev& s, const KeepRect& pr, const KeepRect& ar, int reset_counters,
                             hipStream_t st) {
    return s.dtype == MDCNN_F16 ? shift_fill_t<f16>(s, pr, ar, reset_counters, st)
                                : shift_fill_t<float>(s, pr, ar, reset_counters, st);
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
template <typename T, int G, int CH>
__global__ __launch_bounds__(256) void k_step1(SiteDev s, const T* __restrict__ X,
                                               const uint8_t* __restrict__ forced) {
    constexpr int VEC = V16<T>::N;
    constexpr int PPB = 256 / G;
    const int tid = threadIdx.x;
    const int lp = tid % G;
    const int pix = blockIdx.x * PPB + tid / G;
    const int HW = s.H * s.W;
    bool m = false, cand = false;
    if (pix < HW) {
        const int fl = s.flags[pix];
        const bool is_input = s.kind == MDCNN_SITE_INPUT;
        cand = is_input || forced != nullptr || (fl & (kFlagN | kFlagU));
        if (cand) {
            const int vy = pix / s.W, vx = pix - vy * s.W;
            T* Ap = (T*)s.A + a_offset(s, vy, vx);
            T* Pp = is_input ? nullptr : (T*)s.P + p_offset(s, vy + s.by0, vx + s.bx0);
            const T* Xp = is_input ? X + (size_t)pix * s.C : nullptr;
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
            const bool hit = forced ? forced[pix] != 0 : mx > s.theta;
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
            }
        }
        if (lp == 0) s.flags[pix] = (uint8_t)(m ? kFlagM : 0);
    }
    const unsigned long long bm = __ballot(m && lp == 0);
    const unsigned long long bc = __ballot(cand && lp == 0);
    __shared__ int sm[4], sc[4];
    if ((tid & 63) == 0) { sm[tid >> 6] = __popcll(bm); sc[tid >> 6] = __popcll(bc); }
    __syncthreads();
    if (tid == 0) {
        s.partials[blockIdx.x] = sm[0] + sm[1] + sm[2] + sm[3];
        s.partials[gridDim.x + blockIdx.x] = sc[0] + sc[1] + sc[2] + sc[3];
    }
}

// Any channel count: one lane per pixel, scalar accesses.
template <typename T>
__global__ __launch_bounds__(256) void k_step1_scalar(SiteDev s, const T* __restrict__ X,
                                                      const uint8_t* __restrict__ forced) {
    const int tid = threadIdx.x;
    const int pix = blockIdx.x * 256 + tid;
    const int HW = s.H * s.W;
    bool m = false, cand = false;
    if (pix < HW) {
        const int fl = s.flags[pix];
        const bool is_input = s.kind == MDCNN_SITE_INPUT;
        cand = is_input || forced != nullptr || (fl & (kFlagN | kFlagU));
        if (cand) {
            const int vy = pix / s.W, vx = pix - vy * s.W;
            T* Ap = (T*)s.A + a_offset(s, vy, vx);
            T* Pp = is_input ? nullptr : (T*)s.P + p_offset(s, vy + s.by0, vx + s.bx0);
            const T* Xp = is_input ? X + (size_t)pix * s.C : nullptr;
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
            const bool hit = forced ? forced[pix] != 0 : mx > s.theta;
            m = (fl & kFlagN) || hit;
            if (m) {
                T* Dp = (T*)s.delta + (size_t)pix * s.C;
                for (int c = 0; c < s.C; ++c) {
                    float a = (float)Ap[c];
                    if (is_input) {
                        float x = (float)Xp[c];
                        Ap[c] = (T)x;
                        Dp[c] = (T)(x - a);
                    } else {
                        float n = a + (float)Pp[c];
                        Ap[c] = (T)n;
                        Dp[c] = (T)(s.relu ? fmaxf(n, 0.f) - fmaxf(a, 0.f) : n - a);
                        Pp[c] = (T)0.f;
                    }
                }
            }
        }
        s.flags[pix] = (uint8_t)(m ? kFlagM : 0);
    }
    const unsigned long long bm = __ballot(m);
    const unsigned long long bc = __ballot(cand);
    __shared__ int sm[4], sc[4];
    if ((tid & 63) == 0) { sm[tid >> 6] = __popcll(bm); sc[tid >> 6] = __popcll(bc); }
    __syncthreads();
    if (tid == 0) {
        s.partials[blockIdx.x] = sm[0] + sm[1] + sm[2] + sm[3];
        s.partials[gridDim.x + blockIdx.x] = sc[0] + sc[1] + sc[2] + sc[3];
    }
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

int step1_pixels_per_block(const SiteDev& s) {
    int G, CH;
    int vec = s.dtype == MDCNN_F16 ? 8 : 4;
    if (!step1_shape(s.C, vec, G, CH)) return 256;
    return 256 / G;
}

template <typename T, int G>
static void step1_g(const SiteDev& s, const T* X, const uint8_t* forced, int CH, dim3 grid, hipStream_t st) {
    switch (CH) {
        case 1: k_step1<T, G, 1><<<grid, dim3(256), 0, st>>>(s, X, forced); break;
        case 2: k_step1<T, G, 2><<<grid, dim3(256), 0, st>>>(s, X, forced); break;
        case 3: k_step1<T, G, 3><<<grid, dim3(256), 0, st>>>(s, X, forced); break;
        default: k_step1<T, G, 4><<<grid, dim3(256), 0, st>>>(s, X, forced); break;
    }
}

template <typename T>
static hipError_t step1_t(const SiteDev& s, const void* frame, const uint8_t* forced, hipStream_t st) {
    int G = 0, CH = 0;
    const T* X = (const T*)frame;
    const int HW = s.H * s.W;
    if (!step1_shape(s.C, V16<T>::N, G, CH)) {
        k_step1_scalar<T><<<dim3((HW + 255) / 256), dim3(256), 0, st>>>(s, X, forced);
        return hipGetLastError();
    }
    const int ppb = 256 / G;
    dim3 grid((HW + ppb - 1) / ppb);
    switch (G) {
        case 1: step1_g<T, 1>(s, X, forced, CH, grid, st); break;
        case 2: step1_g<T, 2>(s, X, forced, CH, grid, st); break;
        case 4: step1_g<T, 4>(s, X, forced, CH, grid, st); break;
        case 8: step1_g<T, 8>(s, X, forced, CH, grid, st); break;
        case 16: step1_g<T, 16>(s, X, forced, CH, grid, st); break;
        case 32: step1_g<T, 32>(s, X, forced, CH, grid, st); break;
        default: step1_g<T, 64>(s, X, forced, CH, grid, st); break;
    }
    return hipGetLastError();
}

hipError_t launch_step1(const SiteDev& s, const void* frame, const uint8_t* forced, hipStream_t st) {
    return s.dtype == MDCNN_F16 ? step1_t<f16>(s, frame, forced, st) : step1_t<float>(s, frame, forced, st);
}

// ---------------------------------------------------------------------------
// Compaction.  A segment is kSegPixels consecutive linear indices handled by one
// 256-thread block (4 per thread, ascending), so list order = index order.
// Segment bases come from per-block counts written by an earlier kernel: no
// waiting between blocks, no host round trip.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int block_sum(int v, int* sh) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((tid & 63) == 0) sh[tid >> 6] = v;
    __syncthreads();
    return sh[0] + sh[1] + sh[2] + sh[3];
}

// exclusive prefix of v over the 256 threads of the block; total in *tot
__device__ __forceinline__ int block_excl_scan(int v, int* sh, int* tot) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(inc, off);
        if (lane >= off) inc += t;
    }
    __syncthreads();
    if (lane == 63) sh[w] = inc;
    __syncthreads();
    int base = 0;
    for (int i = 0; i < w; ++i) base += sh[i];
    *tot = sh[0] + sh[1] + sh[2] + sh[3];
    return base + inc - v;
}

__device__ __forceinline__ bool covered(const EdgeDev& e, int widx) {
    const int wy = widx / e.Wp, wx = widx - wy * e.Wp;
    const int oy = wy - e.by0, ox = wx - e.bx0;
    if (e.k == 0) {
        if (oy < 0 || oy >= e.sH || ox < 0 || ox >= e.sW) return false;
        return e.sflags[oy * e.sW + ox] & kFlagM;
    }
    const int y0 = oy * e.stride - e.pad, x0 = ox * e.stride - e.pad;
    for (int jy = 0; jy < e.k; ++jy) {
        const int iy = y0 + jy;
        if (iy < 0 || iy >= e.sH) continue;
        for (int jx = 0; jx < e.k; ++jx) {
            const int ix = x0 + jx;
            if (ix < 0 || ix >= e.sW) continue;
            if (e.sflags[iy * e.sW + ix] & kFlagM) return true;
        }
    }
    return false;
}

// blockIdx.y == 0: compact the update mask of site s into its list L.
// blockIdx.y >= 1: count, per segment, the compute-list entries of edge y-1.
__global__ __launch_bounds__(256) void k_lists_a(SiteDev s, int ppb, int nblk1, EdgeBatch eb, int do_compact) {
    __shared__ int sh[4];
    const int tid = threadIdx.x;
    const int seg = blockIdx.x;
    if (blockIdx.y == 0) {
        if (!do_compact) return;
        const int HW = s.H * s.W;
        const int nseg = (HW + kSegPixels - 1) / kSegPixels;
        if (seg >= nseg) return;
        const int nprev = seg * (kSegPixels / ppb);
        int v = 0;
        for (int i = tid; i < nprev; i += 256) v += s.partials[i];
        const int base = block_sum(v, sh);
        const int p0 = seg * kSegPixels + tid * 4;
        int bits = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (p0 + j < HW && (s.flags[p0 + j] & kFlagM)) bits |= 1 << j;
        int tot;
        int off = base + block_excl_scan(__popc(bits), sh, &tot);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (bits & (1 << j)) s.list[off++] = p0 + j;
        if (seg == nseg - 1) {
            int c = 0;
            for (int i = tid; i < nblk1; i += 256) c += s.partials[nblk1 + i];
            c = block_sum(c, sh);
            if (tid == 0) {
                s.counters[kCntUpdated] = base + tot;
                s.counters[kCntCandidates] = c;
                unsigned long long* acc = reinterpret_cast<unsigned long long*>(s.counters);
                acc[kAccUpdated] += (unsigned long long)(base + tot);
                acc[kAccCandidates] += (unsigned long long)c;
            }
        }
    } else {
        const int ei = blockIdx.y - 1;
        if (ei >= eb.n) return;
        const EdgeDev& e = eb.e[ei];
        if (e.up) return;
        const int NW = e.Hp * e.Wp;
        if (seg * kSegPixels >= NW) return;
        const int p0 = seg * kSegPixels + tid * 4;
        int c = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (p0 + j < NW && covered(e, p0 + j)) ++c;
        c = block_sum(c, sh);
        if (tid == 0) e.cpartials[seg] = c;
    }
}

// blockIdx.y = edge: write the compute list (ascending padded-window index).
__global__ __launch_bounds__(256) void k_lists_b(EdgeBatch eb) {
    __shared__ int sh[4];
    const int tid = threadIdx.x;
    const int seg = blockIdx.x;
    const EdgeDev& e = eb.e[blockIdx.y];
    if (e.up) return;
    const int NW = e.Hp * e.Wp;
    const int nseg = (NW + kSegPixels - 1) / kSegPixels;
    if (seg >= nseg) return;
    int v = 0;
    for (int i = tid; i < seg; i += 256) v += e.cpartials[i];
    const int base = block_sum(v, sh);
    const int p0 = seg * kSegPixels + tid * 4;
    int bits = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (p0 + j < NW && covered(e, p0 + j)) bits |= 1 << j;
    int tot;
    int off = base + block_excl_scan(__popc(bits), sh, &tot);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (bits & (1 << j)) e.clist[off++] = p0 + j;
    if (seg == nseg - 1 && tid == 0) {
        e.dcounters[kCntCompute] = base + tot;
        reinterpret_cast<unsigned long long*>(e.dcounters)[kAccCompute] += (unsigned long long)(base + tot);
    }
}

// One batch of edges of site s; the first batch of a site also compacts L.
hipError_t launch_lists(const SiteDev& s, const EdgeBatch& eb, bool do_compact, hipStream_t st) {
    const int HW = s.H * s.W;
    int nseg = do_compact ? (HW + kSegPixels - 1) / kSegPixels : 0;
    int nseg_e = 0;
    bool any = false;
    for (int i = 0; i < eb.n; ++i) {
        if (eb.e[i].up) continue;
        any = true;
        int n = (eb.e[i].Hp * eb.e[i].Wp + kSegPixels - 1) / kSegPixels;
        if (n > nseg_e) nseg_e = n;
    }
    int gx = nseg > nseg_e ? nseg : nseg_e;
    if (gx == 0) return hipSuccess;
    const int ppb = step1_pixels_per_block(s);
    const int nblk1 = (HW + ppb - 1) / ppb;
    k_lists_a<<<dim3(gx, 1 + (any ? eb.n : 0)), dim3(256), 0, st>>>(s, ppb, nblk1, eb, do_compact ? 1 : 0);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (any) {
        k_lists_b<<<dim3(nseg_e, eb.n), dim3(256), 0, st>>>(eb);
        err = hipGetLastError();
    }
    return err;
}

// ---------------------------------------------------------------------------
// View-ordered access (readout of OUTPUT sites is on the per-frame path).
// ---------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_read_tensor(SiteDev s, int what, T* __restrict__ dst) {
    const int chunks = s.C / VEC;
    const bool win = what == MDCNN_VIEW_P;
    const int Wn = win ? s.Wp : s.W;
    const long long total = (long long)(win ? s.Hp * s.Wp : s.H * s.W) * chunks;
    const long long step = (long long)gridDim.x * 256;
    for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += step) {
        const int pix = (int)(idx / chunks);
        const int c0 = (int)(idx - (long long)pix * chunks) * VEC;
        const int y = pix / Wn, x = pix - y * Wn;
        const T* src;
        bool zero = false;
        if (what == MDCNN_VIEW_A) src = (const T*)s.A + a_offset(s, y, x);
        else if (what == MDCNN_VIEW_P) src = (const T*)s.P + p_offset(s, y, x);
        else if (what == MDCNN_VIEW_OUT) src = (const T*)s.P + p_offset(s, y + s.by0, x + s.bx0);
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
        T* d = what == MDCNN_VIEW_A ? (T*)s.A + a_offset(s, y, x) : (T*)s.P + p_offset(s, y, x);
        const T* sp = src + (size_t)pix * s.C + c0;
#pragma unroll
        for (int i = 0; i < VEC; ++i) d[c0 + i] = sp[i];
    }
}

__global__ __launch_bounds__(256) void k_read_ints(SiteDev s, int what, int* __restrict__ dst) {
    const int step = gridDim.x * 256;
    const int i0 = blockIdx.x * 256 + threadIdx.x;
    if (what == MDCNN_VIEW_STATS) {
        if (i0 < 18) dst[i0] = s.counters[i0];
        return;
    }
    const bool cl = what == MDCNN_VIEW_CLIST;
    const int n = cl ? s.Hp * s.Wp : s.H * s.W;
    const int cnt = s.counters[cl ? kCntCompute : kCntUpdated];
    const int* src = cl ? s.clist : s.list;
    for (int i = i0; i < n + 1; i += step) dst[i] = i == 0 ? cnt : (i - 1 < cnt ? src[i - 1] : -1);
}

__global__ __launch_bounds__(256) void k_copy_bytes(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int n) {
    const int step = gridDim.x * 256;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += step) dst[i] = src[i];
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
    const long long pix = what == MDCNN_VIEW_P ? (long long)s.Hp * s.Wp : (long long)s.H * s.W;
    if (vec)
        k_read_tensor<T, V><<<dim3(grid_for(pix * (s.C / V))), dim3(256), 0, st>>>(s, what, (T*)dst);
    else
        k_read_tensor<T, 1><<<dim3(grid_for(pix * s.C)), dim3(256), 0, st>>>(s, what, (T*)dst);
    return hipGetLastError();
}

hipError_t launch_read_view(const SiteDev& s, int what, void* dst, hipStream_t st) {
    switch (what) {
        case MDCNN_VIEW_A: case MDCNN_VIEW_P: case MDCNN_VIEW_DELTA: case MDCNN_VIEW_OUT:
            return s.dtype == MDCNN_F16 ? read_tensor_t<f16>(s, what, dst, st) : read_tensor_t<float>(s, what, dst, st);
        case MDCNN_VIEW_FLAGS:
            k_copy_bytes<<<dim3(grid_for(s.H * s.W)), dim3(256), 0, st>>>(s.flags, (uint8_t*)dst, s.H * s.W);
            return hipGetLastError();
        case MDCNN_VIEW_LIST:
            k_read_ints<<<dim3(grid_for(s.H * s.W + 1)), dim3(256), 0, st>>>(s, what, (int*)dst);
            return hipGetLastError();
        case MDCNN_VIEW_CLIST:
            k_read_ints<<<dim3(grid_for(s.Hp * s.Wp + 1)), dim3(256), 0, st>>>(s, what, (int*)dst);
            return hipGetLastError();
        default:
            k_read_ints<<<dim3(1), dim3(256), 0, st>>>(s, MDCNN_VIEW_STATS, (int*)dst);
            return hipGetLastError();
    }
}

hipError_t launch_write_view(const SiteDev& s, int what, const void* src, hipStream_t st) {
    if (what == MDCNN_VIEW_FLAGS) {
        k_copy_bytes<<<dim3(grid_for(s.H * s.W)), dim3(256), 0, st>>>((const uint8_t*)src, s.flags, s.H * s.W);
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

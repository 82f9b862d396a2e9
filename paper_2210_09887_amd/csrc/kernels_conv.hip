// Padded sparse convolution: for every entry of the compute list (a pixel of
// the destination's padded window whose footprint holds an updated input pixel)
//   y[q, :] = sum over taps with an updated in-view input  W[tap] . delta[p(q, tap), :]
//   P_dst[q] <- P_dst[q] + y[q]        (border pixels included: they are stashed)
// Output-stationary: one owner per output pixel, fixed summation order, so the
// result does not depend on scheduling.  Weights are w[tap][cout][cin].
//
//   k_conv_mfma_f16 : gather-GEMM on the CDNA4 matrix cores (fp16 in, fp32 acc)
//   k_conv_plain    : plain FMA, any dtype / channel count
//   k_identity      : residual skip, P_dst[q] += delta[q]
#include "mdcnn_internal.h"

namespace mdcnn {

typedef _Float16 f16;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int wrapc(int v, int n) { return v >= n ? v - n : v; }

__device__ __forceinline__ size_t pdst_offset(const EdgeDev& e, int wy, int wx) {
    int py = wrapc(e.p_oy + wy, e.Hp), px = wrapc(e.p_ox + wx, e.Wp);
    return ((size_t)py * e.Wp + px) * e.Cout;
}

// Decode list entry -> conv-output coordinates (cy, cx) in the source-aligned
// frame and the top-left destination window pixel (wy, wx).
__device__ __forceinline__ void decode_entry(const EdgeDev& e, int idx, int& cy, int& cx, int& wy, int& wx) {
    if (e.up) {                       // entry = updated source pixel (1x1 conv)
        cy = idx / e.sW; cx = idx - cy * e.sW;
        wy = (cy << e.up) + e.by0; wx = (cx << e.up) + e.bx0;
    } else {                          // entry = destination padded-window pixel
        wy = idx / e.Wp; wx = idx - wy * e.Wp;
        cy = wy - e.by0; cx = wx - e.bx0;
    }
}

__device__ __forceinline__ unsigned tap_mask(const EdgeDev& e, int cy, int cx) {
    unsigned m = 0;
    const int y0 = cy * e.stride - e.pad, x0 = cx * e.stride - e.pad;
    for (int jy = 0; jy < e.k; ++jy) {
        const int iy = y0 + jy;
        if (iy < 0 || iy >= e.sH) continue;
        for (int jx = 0; jx < e.k; ++jx) {
            const int ix = x0 + jx;
            if (ix < 0 || ix >= e.sW) continue;
            if (e.sflags[iy * e.sW + ix] & kFlagM) m |= 1u << (jy * e.k + jx);
        }
    }
    return m;
}

// Statistics: add (valid taps of this wave) x Cin x Cout to the destination's
// multiply-accumulate counter.  Called by whole waves.
__device__ __forceinline__ void count_macs(const EdgeDev& e, int taps, int slot) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) taps += __shfl_xor(taps, off);
    if ((threadIdx.x & 63) == 0 && taps)
        atomicAdd(reinterpret_cast<unsigned long long*>(e.dcounters) + slot,
                  (unsigned long long)taps * (unsigned long long)(e.Cin * e.Cout));
}

__device__ __forceinline__ void mark_touched(const EdgeDev& e, int wy, int wx) {
    if (!e.dflags) return;
    const int f = 1 << e.up;
    for (int a = 0; a < f; ++a)
        for (int b = 0; b < f; ++b) {
            const int oy = wy + a - e.by0, ox = wx + b - e.bx0;
            if (oy >= 0 && oy < e.dH && ox >= 0 && ox < e.dW) e.dflags[oy * e.dW + ox] |= (uint8_t)kFlagU;
        }
}

// ---------------------------------------------------------------------------
// MFMA gather-GEMM, fp16 storage, fp32 accumulate.
// v_mfma_f32_32x32x16_f16: operand A = 32 couts x 16 cin (weights), operand
// B = 16 cin x 32 pixels (gathered deltas); lane l feeds row/col l%32 with the
// 8 consecutive cin starting at 8*(l/32).  The result puts pixel l%32 on lane l
// with couts 8*(r/4) + 4*(l/32) + r%4 in accumulator register r, so every lane
// updates its own pixel of P and needs no exchange.
// Block = 4 waves arranged (4/WN) x WN over (pixels x couts).
// ---------------------------------------------------------------------------
template <int WN>
__global__ __launch_bounds__(256) void k_conv_mfma_f16(EdgeDev e) {
    constexpr int WM = 4 / WN;
    constexpr int TILE_M = 32 * WM;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int col = lane & 31, kh = lane >> 5;
    const int count = e.up ? e.scounters[kCntUpdated] : e.dcounters[kCntCompute];
    const int* __restrict__ lst = e.up ? e.slist : e.clist;
    const int n0 = (blockIdx.y * WN + wn) * 32;
    const f16* __restrict__ delta = (const f16*)e.delta;
    const f16* __restrict__ w = (const f16*)e.w;
    const int taps = e.k * e.k;
    for (int tile = blockIdx.x; tile * TILE_M < count; tile += gridDim.x) {
        const int ent = tile * TILE_M + wm * 32 + col;
        const bool live = ent < count;
        int cy = 0, cx = 0, wy = 0, wx = 0;
        unsigned vmask = 0;
        if (live) {
            decode_entry(e, lst[ent], cy, cx, wy, wx);
            vmask = tap_mask(e, cy, cx);
        }
        if (wn == 0 && blockIdx.y == 0) count_macs(e, kh == 0 ? __popc(vmask) : 0, kAccMacs);
        const int y0 = cy * e.stride - e.pad, x0 = cx * e.stride - e.pad;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        for (int tap = 0; tap < taps; ++tap) {
            const bool v = (vmask >> tap) & 1u;
            if (__ballot(v) == 0ull) continue;                 // no pixel of this wave uses the tap
            const int jy = tap / e.k, jx = tap - jy * e.k;
            const f16* arow = w + ((size_t)(tap * e.Cout + n0 + col)) * e.Cin + kh * 8;
            const f16* brow = delta + (v ? ((size_t)((y0 + jy) * e.sW + (x0 + jx))) * e.Cin + kh * 8 : 0);
            for (int c0 = 0; c0 < e.Cin; c0 += 16) {
                f16x8 a = *reinterpret_cast<const f16x8*>(arow + c0);
                f16x8 b;
                if (v) b = *reinterpret_cast<const f16x8*>(brow + c0);
                else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) b[i] = (f16)0.f;
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
            }
        }
        if (live) {
            const int f = 1 << e.up;
            for (int ua = 0; ua < f; ++ua)
                for (int ub = 0; ub < f; ++ub) {
                    f16* p = (f16*)e.P + pdst_offset(e, wy + ua, wx + ub) + n0 + 4 * kh;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        f16x4 o = *reinterpret_cast<f16x4*>(p + 8 * g);
#pragma unroll
                        for (int i = 0; i < 4; ++i) o[i] = (f16)((float)o[i] + acc[4 * g + i]);
                        *reinterpret_cast<f16x4*>(p + 8 * g) = o;
                    }
                }
            if (kh == 0 && wn == 0 && blockIdx.y == 0) mark_touched(e, wy, wx);
        }
    }
}

// ---------------------------------------------------------------------------
// Plain FMA convolution for any dtype / channel count (small nets, stems).
// Block = 16 list entries x 16 cout lanes; each thread keeps 4 couts at a time.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_conv_plain(EdgeDev e) {
    const int p = threadIdx.x >> 4, cl = threadIdx.x & 15;
    const int count = e.up ? e.scounters[kCntUpdated] : e.dcounters[kCntCompute];
    const int* __restrict__ lst = e.up ? e.slist : e.clist;
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    const int taps = e.k * e.k;
    for (int tile = blockIdx.x; tile * 16 < count; tile += gridDim.x) {
        const int ent = tile * 16 + p;
        const bool live = ent < count;
        int cy = 0, cx = 0, wy = 0, wx = 0;
        unsigned vmask = 0;
        if (live) {
            decode_entry(e, lst[ent], cy, cx, wy, wx);
            vmask = tap_mask(e, cy, cx);
        }
        count_macs(e, cl == 0 ? __popc(vmask) : 0, kAccMacsPlain);
        if (!live) continue;
        const int y0 = cy * e.stride - e.pad, x0 = cx * e.stride - e.pad;
        for (int cg = 0; cg < e.Cout; cg += 64) {
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
            for (int tap = 0; tap < taps; ++tap) {
                if (!((vmask >> tap) & 1u)) continue;
                const int jy = tap / e.k, jx = tap - jy * e.k;
                const T* drow = delta + ((size_t)((y0 + jy) * e.sW + (x0 + jx))) * e.Cin;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int co = cg + cl + 16 * j;
                    if (co >= e.Cout) continue;
                    const T* wrow = w + ((size_t)(tap * e.Cout + co)) * e.Cin;
                    float a = acc[j];
                    for (int ci = 0; ci < e.Cin; ++ci) a = fmaf((float)drow[ci], (float)wrow[ci], a);
                    acc[j] = a;
                }
            }
            const int f = 1 << e.up;
            for (int ua = 0; ua < f; ++ua)
                for (int ub = 0; ub < f; ++ub) {
                    T* pp = (T*)e.P + pdst_offset(e, wy + ua, wx + ub);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int co = cg + cl + 16 * j;
                        if (co < e.Cout) pp[co] = (T)((float)pp[co] + acc[j]);
                    }
                }
        }
        if (cl == 0) mark_touched(e, wy, wx);
    }
}

// Residual skip: P_dst[q] += delta[q] on the compute list (= updated pixels).
template <typename T>
__global__ __launch_bounds__(256) void k_identity(EdgeDev e) {
    const int count = e.dcounters[kCntCompute];
    const long long total = (long long)count * e.Cout;
    const long long step = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += step) {
        const int ent = (int)(i / e.Cout);
        const int c = (int)(i - (long long)ent * e.Cout);
        const int idx = e.clist[ent];
        const int wy = idx / e.Wp, wx = idx - wy * e.Wp;
        const int oy = wy - e.by0, ox = wx - e.bx0;
        T* pp = (T*)e.P + pdst_offset(e, wy, wx);
        const T* d = (const T*)e.delta + ((size_t)(oy * e.sW + ox)) * e.Cin;
        pp[c] = (T)((float)pp[c] + (float)d[c]);
        if (c == 0) mark_touched(e, wy, wx);
    }
}

static unsigned cap_blocks(long long b, long long cap) {
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

hipError_t launch_conv(const EdgeDev& e, int dtype, int conv_path, hipStream_t st, int* cls) {
    const long long max_entries = e.up ? (long long)e.sH * e.sW : (long long)e.Hp * e.Wp;
    if (e.k == 0) {
        *cls = kClsIdentity;
        unsigned g = cap_blocks((max_entries * e.Cout + 255) / 256, 8192);
        if (dtype == MDCNN_F16) k_identity<f16><<<dim3(g), dim3(256), 0, st>>>(e);
        else k_identity<float><<<dim3(g), dim3(256), 0, st>>>(e);
        return hipGetLastError();
    }
    const bool mfma_ok = dtype == MDCNN_F16 && conv_path != 1 && e.Cin % 16 == 0 && e.Cout % 32 == 0;
    if (mfma_ok) {
        *cls = kClsConvMfma;
        if (e.Cout % 64 == 0) {
            unsigned g = cap_blocks((max_entries + 63) / 64, 4096);
            k_conv_mfma_f16<2><<<dim3(g, e.Cout / 64), dim3(256), 0, st>>>(e);
        } else {
            unsigned g = cap_blocks((max_entries + 127) / 128, 4096);
            k_conv_mfma_f16<1><<<dim3(g, e.Cout / 32), dim3(256), 0, st>>>(e);
        }
        return hipGetLastError();
    }
    *cls = kClsConvPlain;
    unsigned g = cap_blocks((max_entries + 15) / 16, 8192);
    if (dtype == MDCNN_F16) k_conv_plain<f16><<<dim3(g), dim3(256), 0, st>>>(e);
    else k_conv_plain<float><<<dim3(g), dim3(256), 0, st>>>(e);
    return hipGetLastError();
}

}  // namespace mdcnn

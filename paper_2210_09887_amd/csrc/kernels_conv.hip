// Padded sparse convolution: for every entry of the compute list (a pixel of
// the destination's padded window whose footprint holds an updated input pixel)
//   y[q, :] = sum over taps with an updated in-view input  W[tap] . delta[p(q, tap), :]
//   P_dst[q] <- P_dst[q] + y[q]        (border pixels included: they are stashed)
// Output-stationary: one owner per output pixel, fixed summation order, so the
// result does not depend on scheduling.  Weights are w[tap][cout][cin].
// Lists are segment-local (kSegPixels indices per segment, count per segment):
// a tile is (segment, offset inside the segment).
//
//   k_conv_mfma_tiled : LDS-tiled gather-GEMM on the CDNA4 matrix cores (fp16 in, fp32 acc)
//   k_conv_mfma_f16   : MFMA without LDS staging (fallback for Cin % 32 != 0)
//   k_conv_ldsw       : plain FMA with the weights resident in LDS (fp32 nets, stems)
//   k_conv_plain      : plain FMA, any dtype / channel count
//   k_identity        : residual skip, P_dst[q] += delta[q]
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

// Which list an edge walks: upsampling edges walk the updated source pixels,
// all others the compute list of the destination.
struct ListRef {
    const int* list;
    const int* cnt;
    int nseg;
};
__device__ __forceinline__ ListRef list_of(const EdgeDev& e) {
    ListRef r;
    if (e.up) { r.list = e.slist; r.cnt = e.slcnt; r.nseg = (e.sH * e.sW + kSegPixels - 1) / kSegPixels; }
    else { r.list = e.clist; r.cnt = e.ccnt; r.nseg = (e.Hp * e.Wp + kSegPixels - 1) / kSegPixels; }
    return r;
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
        const bool yok = iy >= 0 && iy < e.sH;
        for (int jx = 0; jx < e.k; ++jx) {
            const int ix = x0 + jx;
            const bool ok = yok && ix >= 0 && ix < e.sW;
            const unsigned f = ok ? e.sflags[iy * e.sW + ix] : 0u;
            m |= ((f >> 2) & 1u) << (jy * e.k + jx);                  // kFlagM == 4
        }
    }
    return m;
}

// Statistics: add (valid taps of this wave) x Cin x Cout to a multiply-accumulate
// counter of the destination.  Called by whole waves.
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
// Tiled MFMA gather-GEMM (the fast path for fp16 layers with Cin % 32 == 0).
// Block tile = BM list entries (pixels) x BN couts, 4 waves arranged WM x WN,
// each wave owning TM x TN 32x32 accumulators.  K runs over (active tap,
// KC-channel chunk) steps; per step the weight slab [BN][KC] and the gathered
// delta slab [BM][KC] (rows of taps that miss the update mask are zero) go
// global -> registers -> LDS (rows padded by 16 bytes) while the previous step is
// multiplied out of LDS.  Taps no entry of the tile uses are skipped.  The
// accumulators are transposed through LDS so that P is updated with 16-byte
// accesses that are contiguous along the channels.
// v_mfma_f32_32x32x16_f16: operand A = 32 couts x 16 cin (weights), operand
// B = 16 cin x 32 pixels; lane l feeds row/col l%32 with the 8 consecutive cin
// starting at 8*(l/32); the result puts pixel l%32 on lane l with couts
// 8*(r/4) + 4*(l/32) + r%4 in accumulator register r.
// ---------------------------------------------------------------------------
template <int WM, int WN, int TM, int TN, int KC>
struct TiledCfg {
    static constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN;
    static constexpr int LDK = KC + 8;             // slab row, halves
    static constexpr int LDC = BN + 4;             // transposed accumulator row, floats
    static constexpr int CPR = KC / 8;             // 16-byte chunks per slab row
    static constexpr int SLAB_BYTES = (BM + BN) * LDK * 2;
    static constexpr int C_BYTES = BM * LDC * 4;
    static constexpr int SMEM = SLAB_BYTES > C_BYTES ? SLAB_BYTES : C_BYTES;
    static constexpr int TPS = kSegPixels / BM;    // tiles per list segment
};

template <int WM, int WN, int TM, int TN, int KC>
__global__ __launch_bounds__(256) void k_conv_mfma_tiled(EdgeDev e) {
    using Cfg = TiledCfg<WM, WN, TM, TN, KC>;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, LDK = Cfg::LDK, LDC = Cfg::LDC, CPR = Cfg::CPR, TPS = Cfg::TPS;
    constexpr int NB = (BM * CPR + 255) / 256, NA = (BN * CPR + 255) / 256;
    static_assert(WM * WN == 4 && BM % 64 == 0 && kSegPixels % BM == 0, "4 waves, whole waves of entries");
    extern __shared__ __align__(16) unsigned char smem[];
    f16* sB = reinterpret_cast<f16*>(smem);              // [BM][LDK] gathered deltas
    f16* sA = sB + BM * LDK;                             // [BN][LDK] weights
    float* sC = reinterpret_cast<float*>(smem);          // [BM][LDC] after the K loop
    __shared__ int s_base[BM], s_wy[BM], s_wx[BM];
    __shared__ unsigned s_vm[BM];
    __shared__ unsigned s_tilemask;
    __shared__ int s_taps;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int r32 = lane & 31, kh = lane >> 5;
    const ListRef L = list_of(e);
    const int n0 = blockIdx.y * BN;
    const f16* __restrict__ delta = (const f16*)e.delta;
    const f16* __restrict__ w = (const f16*)e.w;

    for (int tile = blockIdx.x; tile < L.nseg * TPS; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * BM;
        const int live = L.cnt[seg] - first;               // entries of this tile (block-uniform)
        if (live <= 0) continue;
        const int* __restrict__ lst = L.list + seg * kSegPixels + first;
        __syncthreads();                                  // previous tile is done with LDS
        if (tid == 0) { s_tilemask = 0; s_taps = 0; }
        unsigned vmask = 0;
        if (tid < BM) {
            int cy = 0, cx = 0, wy = 0, wx = 0;
            if (tid < live) {
                decode_entry(e, lst[tid], cy, cx, wy, wx);
                vmask = tap_mask(e, cy, cx);
                if (blockIdx.y == 0) mark_touched(e, wy, wx);
            }
            s_base[tid] = (cy * e.stride - e.pad) * e.sW + (cx * e.stride - e.pad);
            s_wy[tid] = wy; s_wx[tid] = wx; s_vm[tid] = vmask;
        }
        __syncthreads();
        if (tid < BM) {                                    // whole waves: BM % 64 == 0
            unsigned orm = vmask;
            int taps = __popc(vmask);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) { orm |= __shfl_xor(orm, off); taps += __shfl_xor(taps, off); }
            if (lane == 0) { atomicOr(&s_tilemask, orm); atomicAdd(&s_taps, taps); }
        }
        __syncthreads();
        unsigned rem = s_tilemask;
        if (tid == 0 && blockIdx.y == 0)                   // statistics: one atomic per tile
            atomicAdd(reinterpret_cast<unsigned long long*>(e.dcounters) + kAccMacs,
                      (unsigned long long)s_taps * (unsigned long long)(e.Cin * e.Cout));

        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        f16x8 rb[NB], ra[NA];
        auto load_slab = [&](int tap, int c0) {
            const int jy = tap / e.k, jx = tap - jy * e.k;
            const int toff = jy * e.sW + jx;
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int ch = tid + 256 * i;
                const int row = ch / CPR, cc = ch - row * CPR;
                f16x8 v;
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = (f16)0.f;
                if (ch < BM * CPR && ((s_vm[row] >> tap) & 1u))
                    v = *reinterpret_cast<const f16x8*>(delta + (size_t)(s_base[row] + toff) * e.Cin + c0 + cc * 8);
                rb[i] = v;
            }
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int ch = tid + 256 * i;
                const int row = ch / CPR, cc = ch - row * CPR;
                if (ch < BN * CPR)
                    ra[i] = *reinterpret_cast<const f16x8*>(w + ((size_t)(tap * e.Cout + n0 + row)) * e.Cin + c0 + cc * 8);
            }
        };
        auto store_slab = [&]() {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int ch = tid + 256 * i;
                const int row = ch / CPR, cc = ch - row * CPR;
                if (ch < BM * CPR) *reinterpret_cast<f16x8*>(sB + row * LDK + cc * 8) = rb[i];
            }
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int ch = tid + 256 * i;
                const int row = ch / CPR, cc = ch - row * CPR;
                if (ch < BN * CPR) *reinterpret_cast<f16x8*>(sA + row * LDK + cc * 8) = ra[i];
            }
        };

        int tap = rem ? __ffs(rem) - 1 : -1, c0 = 0;
        if (tap >= 0) { load_slab(tap, c0); store_slab(); }
        __syncthreads();
        while (tap >= 0) {
            int ntap = tap, nc0 = c0 + KC;
            if (nc0 >= e.Cin) { nc0 = 0; rem &= rem - 1; ntap = rem ? __ffs(rem) - 1 : -1; }
            if (ntap >= 0) load_slab(ntap, nc0);            // in flight while this step is multiplied
#pragma unroll
            for (int kk = 0; kk < KC / 16; ++kk) {
                f16x8 fb[TM], fa[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fb[i] = *reinterpret_cast<const f16x8*>(sB + ((wm * TM + i) * 32 + r32) * LDK + kk * 16 + kh * 8);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fa[j] = *reinterpret_cast<const f16x8*>(sA + ((wn * TN + j) * 32 + r32) * LDK + kk * 16 + kh * 8);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[j], fb[i], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
            if (ntap >= 0) store_slab();
            __syncthreads();
            tap = ntap; c0 = nc0;
        }

        // accumulators -> LDS as [pixel][cout]
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                float* dst = sC + ((wm * TM + i) * 32 + r32) * LDC + (wn * TN + j) * 32 + 4 * kh;
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4*>(dst + 8 * g) =
                        make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
            }
        __syncthreads();
        constexpr int TPR = BN / 8;                        // threads per pixel row, 8 couts each
        const int c8 = (tid % TPR) * 8;
        const int f = 1 << e.up;
        for (int row = tid / TPR; row < BM && row < live; row += 256 / TPR) {
            const float4 v0 = *reinterpret_cast<const float4*>(sC + row * LDC + c8);
            const float4 v1 = *reinterpret_cast<const float4*>(sC + row * LDC + c8 + 4);
            const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
            for (int ua = 0; ua < f; ++ua)
                for (int ub = 0; ub < f; ++ub) {
                    f16* p = (f16*)e.P + pdst_offset(e, s_wy[row] + ua, s_wx[row] + ub) + n0 + c8;
                    f16x8 o = *reinterpret_cast<f16x8*>(p);
#pragma unroll
                    for (int q = 0; q < 8; ++q) o[q] = (f16)((float)o[q] + v[q]);
                    *reinterpret_cast<f16x8*>(p) = o;
                }
        }
    }
}

// ---------------------------------------------------------------------------
// MFMA without LDS staging: every wave loads its own fragments from global
// memory.  Block = 4 waves arranged (4/WN) x WN over (pixels x couts); every
// lane updates its own pixel of P.  Fallback for Cin % 32 != 0.
// ---------------------------------------------------------------------------
template <int WN>
__global__ __launch_bounds__(256) void k_conv_mfma_f16(EdgeDev e) {
    constexpr int WM = 4 / WN;
    constexpr int TILE_M = 32 * WM;
    constexpr int TPS = kSegPixels / TILE_M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int col = lane & 31, kh = lane >> 5;
    const ListRef L = list_of(e);
    const int n0 = (blockIdx.y * WN + wn) * 32;
    const f16* __restrict__ delta = (const f16*)e.delta;
    const f16* __restrict__ w = (const f16*)e.w;
    const int taps = e.k * e.k;
    for (int tile = blockIdx.x; tile < L.nseg * TPS; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * TILE_M;
        const int cnt = L.cnt[seg];
        if (first >= cnt) continue;
        const int ent = first + wm * 32 + col;
        const bool live = ent < cnt;
        int cy = 0, cx = 0, wy = 0, wx = 0;
        unsigned vmask = 0;
        if (live) {
            decode_entry(e, L.list[seg * kSegPixels + ent], cy, cx, wy, wx);
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
// Plain FMA convolution with ALL weights resident in LDS as fp32
// [tap][cin][cout]; a thread owns one list entry and 8 consecutive couts.
// Used for fp32 networks and for layers the MFMA path does not take (e.g. a
// 3-channel stem).  Needs Cout % 8 == 0, Cout <= 512 and k*k*Cin*Cout*4 bytes
// of LDS.  Tiles of ppb entries never straddle a list segment.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_conv_ldsw(EdgeDev e, int groups, int ppb) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sW = reinterpret_cast<float*>(smem);             // [tap][Cin][Cout]
    const int tid = threadIdx.x;
    const int cg = tid % groups, pl = tid / groups;         // cout group, local pixel
    const ListRef L = list_of(e);
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    const int taps = e.k * e.k;
    const int cc = e.Cin * e.Cout;
    for (int i = tid; i < taps * cc; i += 256) {
        const int tap = i / cc, r = i - tap * cc;
        const int co = r / e.Cin, ci = r - co * e.Cin;
        sW[tap * cc + ci * e.Cout + co] = (float)w[i];
    }
    __syncthreads();
    const int tps = (kSegPixels + ppb - 1) / ppb;           // tiles per segment
    for (int tile = blockIdx.x; tile < L.nseg * tps; tile += gridDim.x) {
        const int seg = tile / tps, first = (tile - seg * tps) * ppb;
        const int cnt = L.cnt[seg];
        if (first >= cnt) continue;
        const int ent = first + pl;
        const bool live = pl < ppb && ent < cnt;
        int cy = 0, cx = 0, wy = 0, wx = 0;
        unsigned vmask = 0;
        if (live) {
            decode_entry(e, L.list[seg * kSegPixels + ent], cy, cx, wy, wx);
            vmask = tap_mask(e, cy, cx);
            if (cg == 0) mark_touched(e, wy, wx);
        }
        count_macs(e, cg == 0 ? __popc(vmask) : 0, kAccMacsPlain);
        if (!live) continue;
        const int base = (cy * e.stride - e.pad) * e.sW + (cx * e.stride - e.pad);
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int tap = 0; tap < taps; ++tap) {
            if (!((vmask >> tap) & 1u)) continue;
            const int jy = tap / e.k, jx = tap - jy * e.k;
            const T* drow = delta + (size_t)(base + jy * e.sW + jx) * e.Cin;
            const float* wt = sW + tap * cc + cg * 8;
            for (int ci = 0; ci < e.Cin; ++ci) {
                const float a = (float)drow[ci];
                const float4 w0 = *reinterpret_cast<const float4*>(wt + ci * e.Cout);
                const float4 w1 = *reinterpret_cast<const float4*>(wt + ci * e.Cout + 4);
                acc[0] = fmaf(a, w0.x, acc[0]); acc[1] = fmaf(a, w0.y, acc[1]);
                acc[2] = fmaf(a, w0.z, acc[2]); acc[3] = fmaf(a, w0.w, acc[3]);
                acc[4] = fmaf(a, w1.x, acc[4]); acc[5] = fmaf(a, w1.y, acc[5]);
                acc[6] = fmaf(a, w1.z, acc[6]); acc[7] = fmaf(a, w1.w, acc[7]);
            }
        }
        const int f = 1 << e.up;
        for (int ua = 0; ua < f; ++ua)
            for (int ub = 0; ub < f; ++ub) {
                T* pp = (T*)e.P + pdst_offset(e, wy + ua, wx + ub) + cg * 8;
#pragma unroll
                for (int q = 0; q < 8; ++q) pp[q] = (T)((float)pp[q] + acc[q]);
            }
    }
}

// ---------------------------------------------------------------------------
// Plain FMA convolution for any dtype / channel count.
// Block = 16 list entries x 16 cout lanes; each thread keeps 4 couts at a time.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_conv_plain(EdgeDev e) {
    const int p = threadIdx.x >> 4, cl = threadIdx.x & 15;
    const ListRef L = list_of(e);
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    const int taps = e.k * e.k;
    constexpr int TPS = kSegPixels / 16;
    for (int tile = blockIdx.x; tile < L.nseg * TPS; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * 16;
        const int cnt = L.cnt[seg];
        if (first >= cnt) continue;
        const int ent = first + p;
        const bool live = ent < cnt;
        int cy = 0, cx = 0, wy = 0, wx = 0;
        unsigned vmask = 0;
        if (live) {
            decode_entry(e, L.list[seg * kSegPixels + ent], cy, cx, wy, wx);
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

// Residual skip: P_dst[q] += delta[q] for every updated pixel q of the source
// (a scan over the view: one thread per pixel and VEC channels).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_identity(EdgeDev e) {
    const int chunks = e.Cin / VEC;
    const long long total = (long long)e.sH * e.sW * chunks;
    const long long step = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += step) {
        const int pix = (int)(i / chunks);
        if (!(e.sflags[pix] & kFlagM)) continue;
        const int c0 = (int)(i - (long long)pix * chunks) * VEC;
        const int oy = pix / e.sW, ox = pix - oy * e.sW;
        T* pp = (T*)e.P + pdst_offset(e, oy + e.by0, ox + e.bx0) + c0;
        const T* d = (const T*)e.delta + (size_t)pix * e.Cin + c0;
        if constexpr (VEC == 8) {
            f16x8 o = *reinterpret_cast<f16x8*>(pp);
            const f16x8 v = *reinterpret_cast<const f16x8*>(d);
#pragma unroll
            for (int q = 0; q < 8; ++q) o[q] = (f16)((float)o[q] + (float)v[q]);
            *reinterpret_cast<f16x8*>(pp) = o;
        } else {
#pragma unroll
            for (int q = 0; q < VEC; ++q) pp[q] = (T)((float)pp[q] + (float)d[q]);
        }
        if (c0 == 0) mark_touched(e, oy + e.by0, ox + e.bx0);
    }
}

static unsigned cap_blocks(long long b, long long cap) {
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

template <int WM, int WN, int TM, int TN, int KC>
static hipError_t launch_tiled(const EdgeDev& e, long long max_entries, hipStream_t st) {
    using Cfg = TiledCfg<WM, WN, TM, TN, KC>;
    static bool attr_set = false;
    auto kern = k_conv_mfma_tiled<WM, WN, TM, TN, KC>;
    if (!attr_set) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::SMEM);
        if (err != hipSuccess) return err;
        attr_set = true;
    }
    const long long nseg = (max_entries + kSegPixels - 1) / kSegPixels;
    unsigned g = cap_blocks(nseg * Cfg::TPS, 2048);
    kern<<<dim3(g, e.Cout / Cfg::BN), dim3(256), Cfg::SMEM, st>>>(e);
    return hipGetLastError();
}

template <int KC>
static hipError_t launch_tiled_kc(const EdgeDev& e, long long max_entries, hipStream_t st) {
    // the largest tile that still yields about one block per compute unit
    auto blocks = [&](int bm, int bn) { return ((max_entries + bm - 1) / bm) * (e.Cout / bn); };
    const long long want = 224;
    if (e.Cout % 128 == 0) {
        if (blocks(128, 128) >= want) return launch_tiled<2, 2, 2, 2, KC>(e, max_entries, st);
        if (blocks(64, 128) >= want) return launch_tiled<2, 2, 1, 2, KC>(e, max_entries, st);
    }
    if (e.Cout % 64 == 0) {
        if (blocks(256, 64) >= want) return launch_tiled<4, 1, 2, 2, KC>(e, max_entries, st);
        if (blocks(128, 64) >= want) return launch_tiled<2, 2, 2, 1, KC>(e, max_entries, st);
        return launch_tiled<2, 2, 1, 1, KC>(e, max_entries, st);
    }
    return launch_tiled<4, 1, 1, 1, KC>(e, max_entries, st);        // Cout % 32 == 0
}

template <typename T>
static hipError_t launch_ldsw(const EdgeDev& e, long long max_entries, hipStream_t st) {
    static size_t attr_bytes = 0;
    const int groups = e.Cout / 8, ppb = 256 / groups;
    const size_t smem = (size_t)e.k * e.k * e.Cin * e.Cout * 4;
    auto kern = k_conv_ldsw<T>;
    if (smem > 65536 && smem > attr_bytes) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (err != hipSuccess) return err;
        attr_bytes = smem;
    }
    const long long nseg = (max_entries + kSegPixels - 1) / kSegPixels;
    const long long tps = (kSegPixels + ppb - 1) / ppb;
    // weights are staged once per block: keep the blocks few and persistent
    unsigned g = cap_blocks(nseg * tps, smem > 32768 ? 256 : 1024);
    kern<<<dim3(g), dim3(256), smem, st>>>(e, groups, ppb);
    return hipGetLastError();
}

hipError_t launch_conv(const EdgeDev& e, int dtype, int conv_path, hipStream_t st, int* cls) {
    const long long max_entries = e.up ? (long long)e.sH * e.sW : (long long)e.Hp * e.Wp;
    const long long nseg = (max_entries + kSegPixels - 1) / kSegPixels;
    if (e.k == 0) {
        *cls = kClsIdentity;
        const long long px = (long long)e.sH * e.sW;
        if (dtype == MDCNN_F16) {
            if (e.Cin % 8 == 0) k_identity<f16, 8><<<dim3(cap_blocks((px * (e.Cin / 8) + 255) / 256, 8192)), dim3(256), 0, st>>>(e);
            else k_identity<f16, 1><<<dim3(cap_blocks((px * e.Cin + 255) / 256, 8192)), dim3(256), 0, st>>>(e);
        } else {
            if (e.Cin % 4 == 0) k_identity<float, 4><<<dim3(cap_blocks((px * (e.Cin / 4) + 255) / 256, 8192)), dim3(256), 0, st>>>(e);
            else k_identity<float, 1><<<dim3(cap_blocks((px * e.Cin + 255) / 256, 8192)), dim3(256), 0, st>>>(e);
        }
        return hipGetLastError();
    }
    // conv_path: 0 auto, 1 plain FMA (per-thread weights), 2 MFMA without LDS tiling
    const bool mfma_ok = dtype == MDCNN_F16 && conv_path != 1 && e.Cin % 16 == 0 && e.Cout % 32 == 0;
    if (mfma_ok && conv_path == 0 && e.Cin % 32 == 0) {
        *cls = kClsConvMfma;
        return e.Cin % 64 == 0 ? launch_tiled_kc<64>(e, max_entries, st) : launch_tiled_kc<32>(e, max_entries, st);
    }
    if (mfma_ok) {
        *cls = kClsConvMfma;
        if (e.Cout % 64 == 0)
            k_conv_mfma_f16<2><<<dim3(cap_blocks(nseg * (kSegPixels / 64), 4096), e.Cout / 64), dim3(256), 0, st>>>(e);
        else
            k_conv_mfma_f16<1><<<dim3(cap_blocks(nseg * (kSegPixels / 128), 4096), e.Cout / 32), dim3(256), 0, st>>>(e);
        return hipGetLastError();
    }
    *cls = kClsConvPlain;
    const int groups = e.Cout / 8;
    if (conv_path == 0 && e.Cout % 8 == 0 && groups <= 64 && (size_t)e.k * e.k * e.Cin * e.Cout * 4 <= 150 * 1024)
        return dtype == MDCNN_F16 ? launch_ldsw<f16>(e, max_entries, st) : launch_ldsw<float>(e, max_entries, st);
    unsigned g = cap_blocks(nseg * (kSegPixels / 16), 8192);
    if (dtype == MDCNN_F16) k_conv_plain<f16><<<dim3(g), dim3(256), 0, st>>>(e);
    else k_conv_plain<float><<<dim3(g), dim3(256), 0, st>>>(e);
    return hipGetLastError();
}

}  // namespace mdcnn

// Padded sparse convolution: for every entry of the compute list (a pixel of
// the destination's padded window whose footprint holds an updated input pixel)
//   y[q, :] = sum over taps with an updated in-view input  W[tap] . delta[p(q, tap), :]
//   P_dst[q] <- P_dst[q] + y[q]        (border pixels included: they are stashed)
// Output-stationary: one owner per output pixel, fixed summation order, so the
// result does not depend on scheduling.  Weights are w[tap][cout][cin].
// There is no separate list kernel: every block compacts the segment of the
// compute list it works on itself, from the source's update mask (kSegPixels
// indices per segment, one per thread, ballot + popcount ranks); a tile is
// (segment, offset inside the segment).  The first tile of a segment also writes
// the segment to the destination's compute list, the copy the ABI exposes, and
// the first edge of a forward call compacts the source's update mask into L.
//
//   k_conv_halo       : 3x3 stride-1 fp16 layers: source rectangle of a tile staged once per
//                       channel chunk in LDS, packed weights straight into MFMA fragments
//   k_conv_mfma_tiled : LDS-tiled gather-GEMM on the CDNA4 matrix cores (fp16 in, fp32 acc)
//   k_conv_mfma_f16   : MFMA without LDS staging (fallback for Cin % 32 != 0)
//   k_conv_small      : 3-channel 3x3 stems, plain FMA
//   k_conv_ldsw       : plain FMA with the weights resident in LDS (fp32 nets)
//   k_conv_plain      : plain FMA, any dtype / channel count
//   k_identity        : residual skip, P_dst[q] += delta[q] (when it is not fused into step 1)
//   k_pool            : max pooling in delta form against a previous-output ring
//   k_pack_weights    : [tap][cout][cin] -> [tap][cin/16][cout][16]
#include <atomic>
#include <mutex>
#include <type_traits>

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

// Update flags of the K x K footprint of output (cy, cx) as a bit mask.  All loads go out together
// (a pixel outside the source reads flag 0 of the site and is masked afterwards).
template <int K>
__device__ __forceinline__ unsigned tap_mask_k(const EdgeDev& e, int cy, int cx) {
    const int y0 = cy * e.stride - e.pad, x0 = cx * e.stride - e.pad;
    unsigned f[K * K];
#pragma unroll
    for (int t = 0; t < K * K; ++t) {
        const int iy = y0 + t / K, ix = x0 + t % K;
        const bool ok = iy >= 0 && iy < e.sH && ix >= 0 && ix < e.sW;
        const unsigned v = e.sflags[ok ? iy * e.sW + ix : 0];
        f[t] = ok ? v : 0u;
    }
    unsigned m = 0;
#pragma unroll
    for (int t = 0; t < K * K; ++t) m |= ((f[t] >> 2) & 1u) << t;      // kFlagM == 4
    return m;
}

__device__ __forceinline__ unsigned tap_mask(const EdgeDev& e, int cy, int cx) {
    switch (e.k) {
        case 1: return tap_mask_k<1>(e, cy, cx);
        case 3: return tap_mask_k<3>(e, cy, cx);
        case 5: return tap_mask_k<5>(e, cy, cx);
        default: break;
    }
    unsigned m = 0;
    const int y0 = cy * e.stride - e.pad, x0 = cx * e.stride - e.pad;
    for (int jy = 0; jy < e.k; ++jy) {
        const int iy = y0 + jy;
        const bool yok = iy >= 0 && iy < e.sH;
        for (int jx = 0; jx < e.k; ++jx) {
            const int ix = x0 + jx;
            const bool ok = yok && ix >= 0 && ix < e.sW;
            const unsigned f = ok ? e.sflags[iy * e.sW + ix] : 0u;
            m |= ((f >> 2) & 1u) << (jy * e.k + jx);
        }
    }
    return m;
}

// Number of list segments an edge walks: upsampling edges walk the source
// pixels (view order), all others the destination's padded window.
__device__ __forceinline__ int edge_segments(const EdgeDev& e) {
    const int n = e.up ? e.sH * e.sW : e.Hp * e.Wp;
    return (n + kSegPixels - 1) / kSegPixels;
}

// Statistics: add taps x Cin x Cout to one of the partial multiply-accumulate
// sums of the destination (which: 0 MFMA kernels, 1 plain kernels).
__device__ __forceinline__ void add_macs(const EdgeDev& e, long long taps, int which) {
    if (taps)
        atomicAdd(reinterpret_cast<unsigned long long*>(e.dcounters) + kAccMacsSpread + 8 * which + (blockIdx.x & 7),
                  (unsigned long long)taps * (unsigned long long)(e.Cin * e.Cout));
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ void mark_touched(const EdgeDev& e, int wy, int wx) {
    if (!e.dflags) return;
    const int f = 1 << e.up;
    for (int a = 0; a < f; ++a)
        for (int b = 0; b < f; ++b) {
            const int oy = wy + a - e.by0, ox = wx + b - e.bx0;
            if (oy >= 0 && oy < e.dH && ox >= 0 && ox < e.dW) {
                // an atomic OR on the word that holds the flag byte, its result unused: nothing comes back to the wave, so the
                // loads that follow do not queue behind a read-modify-write round trip (the flag region is 256-byte aligned)
                const int idx = oy * e.dW + ox;
                atomicOr(reinterpret_cast<unsigned*>(e.dflags + (idx & ~3)), (unsigned)kFlagU << (8 * (idx & 3)));
            }
        }
}

// Per-tile prologue shared by all convolution kernels.  Thread t looks at index
// seg * kSegPixels + t of the edge's index space, gathers the update flags of its
// footprint (they become the tap mask), and the block ranks the non-empty ones
// with ballot + popcount: the rank is the position in the segment's compute list.
// Entries with rank in [first, first + bm) are decoded into the LDS rows
// s_base / s_wy / s_wx / s_vm (s_vm = 0 beyond the live rows).  With `publish`
// the segment is also written to the destination's compute list.  `touch` marks
// the destination pixels as touched.  Returns the number of entries of the
// segment; sh[4] = valid taps of the tile, sh[5] = OR of its tap masks.
// Block-uniform; two barriers; the caller must have a barrier before the call.
__device__ __forceinline__ int tile_prologue(const EdgeDev& e, int seg, int first, int bm, bool publish, bool touch,
                                             int* s_base, int* s_wy, int* s_wx, unsigned* s_vm, int* sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = e.up ? e.sH * e.sW : e.Hp * e.Wp;
    const int p = seg * kSegPixels + tid;
    if (tid < bm) s_vm[tid] = 0;
    if (tid == 0) { sh[4] = 0; sh[5] = 0; }
    int cy = 0, cx = 0, wy = 0, wx = 0;
    unsigned vm = 0;
    if (p < n) {
        decode_entry(e, p, cy, cx, wy, wx);
        if (e.k == 0) vm = (cy >= 0 && cy < e.sH && cx >= 0 && cx < e.sW && (e.sflags[cy * e.sW + cx] & kFlagM)) ? 1u : 0u;
        else if (e.op && (cy < 0 || cy >= e.dH || cx < 0 || cx >= e.dW)) vm = 0;     // pooling outputs exist inside the view only
        else vm = tap_mask(e, cy, cx);
    }
    const bool has = vm != 0;
    const unsigned long long bal = __ballot(has);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) sh[wave] = __popcll(bal);
    __syncthreads();
    int off = rank;
    for (int i = 0; i < wave; ++i) off += sh[i];
    const int tot = sh[0] + sh[1] + sh[2] + sh[3];
    const int r = off - first;
    const bool mine = has && r >= 0 && r < bm;
    if (mine) {
        s_vm[r] = vm;
        s_base[r] = (cy * e.stride - e.pad) * e.sW + (cx * e.stride - e.pad);
        s_wy[r] = wy;
        s_wx[r] = wx;
        if (touch) mark_touched(e, wy, wx);
    }
    if (publish && has) e.clist[seg * kSegPixels + off] = p;
    if (publish && tid == 0) {                             // single writer per segment: no atomics
        e.ccnt[seg] = tot;
        e.cacc[seg] += (unsigned long long)tot;
    }
    unsigned orm = mine ? vm : 0u;
    int taps = mine ? __popc(vm) : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { orm |= __shfl_xor(orm, o); taps += __shfl_xor(taps, o); }
    if (lane == 0 && orm) { atomicOr(reinterpret_cast<unsigned*>(&sh[5]), orm); atomicAdd(&sh[4], taps); }
    __syncthreads();
    return tot;
}

// The first edge of a forward call also compacts the update mask of the source
// site into its list L (segment-local, ascending) and adds up the per-frame
// statistics.  Called by all threads of every block before their own work.
__device__ __forceinline__ void carry_source_compaction(const EdgeDev& e, int* sh) {
    if (!e.pub_list || blockIdx.y != 0) return;
    const int HW = e.sH * e.sW;
    const int nseg = (HW + kSegPixels - 1) / kSegPixels;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int seg = blockIdx.x; seg < nseg; seg += gridDim.x) {
        const int p = seg * kSegPixels + tid;
        const int f = p < HW && tid < kSegPixels ? e.sflags[p] : 0;       // waves beyond the fourth only keep the barriers
        const unsigned long long bm = __ballot(f & kFlagM), bc = __ballot(f & kFlagC);
        __syncthreads();                                   // sh is free again
        if (lane == 0 && wave < 4) { sh[wave] = __popcll(bm); sh[4 + wave] = __popcll(bc); }
        __syncthreads();
        int off = __popcll(bm & ((1ull << lane) - 1ull));
        for (int i = 0; i < wave; ++i) off += sh[i];
        if (f & kFlagM) e.pub_list[seg * kSegPixels + off] = p;
        if (tid == 0) {                                    // single writer per segment: no atomics
            const int tot = sh[0] + sh[1] + sh[2] + sh[3], c = sh[4] + sh[5] + sh[6] + sh[7];
            e.pub_lcnt[2 * seg] = tot;
            e.pub_lcnt[2 * seg + 1] = c;
            e.pub_lacc[2 * seg] += (unsigned long long)tot;
            e.pub_lacc[2 * seg + 1] += (unsigned long long)c;
        }
    }
    __syncthreads();
}

// Buffer loads: the address is a resource (base, size) in scalar registers + a per-lane byte offset + a
// scalar byte offset, so a wave spends one vector register on all the addresses of a tensor instead of a
// 64-bit pointer per load (reads past `bytes` return zero instead of faulting).
using rsrc_t = __amdgpu_buffer_rsrc_t;
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ f16x8 buf_load16(rsrc_t r, unsigned lane_bytes, unsigned wave_bytes) {
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_bytes, (int)wave_bytes, 0);
    return __builtin_bit_cast(f16x8, v);
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
template <int WM, int WN, int TM, int TN, int KC, int PIPE>
struct TiledCfg {
    static constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN;
    static constexpr int LDK = KC + 8;             // slab row, halves
    static constexpr int LDC = BN + 4;             // transposed accumulator row, floats
    static constexpr int CPR = KC / 8;             // 16-byte chunks per slab row
    static constexpr int STAGE_HALVES = (BM + BN) * LDK;
    static constexpr int SLAB_BYTES = PIPE * STAGE_HALVES * 2;
    static constexpr int C_BYTES = BM * LDC * 4;
    static constexpr int SMEM = SLAB_BYTES > C_BYTES ? SLAB_BYTES : C_BYTES;
    static constexpr int TPS = kSegPixels / BM;    // tiles per list segment
};

// Work item u of a 1-D grid -> (pixel tile m, cout tile n).  Work groups are
// dealt round-robin to the 8 XCDs, each with its own L2: tying u % 8 to the
// cout tile makes all blocks of one XCD share the same weight slice.
__device__ __forceinline__ void map_tile(int u, int NT, int xcd_map, int& m, int& n) {
    if (xcd_map) {
        const int q = 8 / NT, x = u & 7, r = u >> 3;
        n = x % NT;
        m = r * q + x / NT;
    } else {
        n = u % NT;
        m = u / NT;
    }
}

// PIPE = 1: one LDS buffer, loads one step ahead (two barriers per step).
// PIPE = 2: two LDS buffers and two register stages, loads two steps ahead
//           (one barrier per step).
template <int WM, int WN, int TM, int TN, int KC, int PIPE>
__global__ __launch_bounds__(256) void k_conv_mfma_tiled(EdgeBatch eb, int NT, int work_items, int xcd_map) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    using Cfg = TiledCfg<WM, WN, TM, TN, KC, PIPE>;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, LDK = Cfg::LDK, LDC = Cfg::LDC, CPR = Cfg::CPR, TPS = Cfg::TPS;
    constexpr int NB = (BM * CPR + 255) / 256, NA = (BN * CPR + 255) / 256;
    static_assert(WM * WN == 4 && kSegPixels % BM == 0, "4 waves; tiles do not straddle segments");
    extern __shared__ __align__(16) unsigned char smem[];
    f16* slab = reinterpret_cast<f16*>(smem);            // PIPE x { [BM][LDK] deltas, [BN][LDK] weights }
    float* sC = reinterpret_cast<float*>(smem);          // [BM][LDC] after the K loop
    __shared__ int s_base[BM], s_wy[BM], s_wx[BM];
    __shared__ unsigned s_vm[BM];
    __shared__ int sh[8];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int r32 = lane & 31, kh = lane >> 5;
    const int MT = edge_segments(e) * TPS;
    // (the host checks that both tensors are smaller than 2 GiB)
    const rsrc_t drs = make_rsrc(e.delta, (unsigned)e.sH * (unsigned)e.sW * (unsigned)e.Cin * 2u);
    const rsrc_t wrs = make_rsrc(e.w, (unsigned)(e.k * e.k) * (unsigned)e.Cin * (unsigned)e.Cout * 2u);

    carry_source_compaction(e, sh);

    for (int u = blockIdx.x; u < work_items; u += gridDim.x) {
        int mt, nt;
        map_tile(u, NT, xcd_map, mt, nt);
        if (mt >= MT) continue;
        const int seg = mt / TPS, first = (mt - seg * TPS) * BM;
        const int n0 = nt * BN;
        __syncthreads();                                  // previous tile is done with LDS
        const int tot = tile_prologue(e, seg, first, BM, nt == 0 && first == 0 && !e.up, nt == 0,
                                      s_base, s_wy, s_wx, s_vm, sh);
        const int live = tot - first < BM ? tot - first : BM;     // entries of this tile (block-uniform)
        if (live <= 0) continue;
        const unsigned tilemask = (unsigned)sh[5];
        if (tid == 0 && nt == 0) add_macs(e, sh[4], 0);    // statistics: one atomic per tile

        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        // Per-thread chunk descriptors of this tile: which slab rows this thread
        // moves, their source offsets (elements) and tap masks.  Per step only a
        // block-uniform offset is added; a row whose tap misses the update mask is
        // loaded from beyond the end of the tensor, which a buffer load answers with
        // zeros (no divergent branches and no selects on the data in the K loop).
        int offB[NB];
        unsigned offA[NA];
        unsigned vmB[NB];
        int ldsB[NB], ldsA[NA];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int ch = tid + 256 * i;
            const int row = (ch / CPR) % BM, cc = ch % CPR;          // % BM: keep partial last rounds in range
            offB[i] = (s_base[row] * e.Cin + cc * 8) * 2;      // bytes; may be negative: the top left tap of a border pixel
            vmB[i] = (BM * CPR) % 256 == 0 || ch < BM * CPR ? s_vm[row] : 0u;
            ldsB[i] = row * LDK + cc * 8;
        }
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int ch = tid + 256 * i;
            const int row = (ch / CPR) % BN, cc = ch % CPR;
            offA[i] = ((unsigned)(n0 + row) * (unsigned)e.Cin + cc * 8) * 2u;      // bytes
            ldsA[i] = row * LDK + cc * 8;
        }
        const unsigned tap_stride_w = (unsigned)e.Cout * (unsigned)e.Cin * 2u;    // bytes

        // the load iterator runs PIPE steps ahead of the multiplication
        unsigned ld_rem = tilemask;
        int ld_tap = ld_rem ? __ffs(ld_rem) - 1 : -1, ld_c0 = 0;
        f16x8 rb[PIPE][NB], ra[PIPE][NA];
        auto load_next = [&](auto stage) {
            constexpr int S = decltype(stage)::value;
            if (ld_tap < 0) return;
            const int jy = ld_tap / e.k, jx = ld_tap - jy * e.k;
            const int stepB = ((jy * e.sW + jx) * e.Cin + ld_c0) * 2;                 // block-uniform, bytes
            const unsigned stepA = (unsigned)ld_tap * tap_stride_w + (unsigned)ld_c0 * 2u;
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const bool valid = (vmB[i] >> ld_tap) & 1u;                           // then offB + stepB is a pixel of the source
                rb[S][i] = buf_load16(drs, valid ? (unsigned)(offB[i] + stepB) : 0x80000000u, 0u);
            }
#pragma unroll
            for (int i = 0; i < NA; ++i) ra[S][i] = buf_load16(wrs, offA[i], stepA);
            ld_c0 += KC;
            if (ld_c0 >= e.Cin) { ld_c0 = 0; ld_rem &= ld_rem - 1; ld_tap = ld_rem ? __ffs(ld_rem) - 1 : -1; }
        };
        auto store_stage = [&](auto stage) {
            constexpr int S = decltype(stage)::value;
            f16* sB = slab + S * Cfg::STAGE_HALVES;
            f16* sA = sB + BM * LDK;
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                if ((BM * CPR) % 256 == 0 || tid + 256 * i < BM * CPR) *reinterpret_cast<f16x8*>(sB + ldsB[i]) = rb[S][i];
            }
#pragma unroll
            for (int i = 0; i < NA; ++i)
                if ((BN * CPR) % 256 == 0 || tid + 256 * i < BN * CPR) *reinterpret_cast<f16x8*>(sA + ldsA[i]) = ra[S][i];
        };
        auto multiply = [&](auto stage) {
            constexpr int S = decltype(stage)::value;
            constexpr int KK = KC / 16;
            const f16* sB = slab + S * Cfg::STAGE_HALVES + (wm * TM * 32 + r32) * LDK + kh * 8;
            const f16* sA = slab + S * Cfg::STAGE_HALVES + BM * LDK + (wn * TN * 32 + r32) * LDK + kh * 8;
            f16x8 fb[KK][TM], fa[KK][TN];                    // all fragments of the step, then the MFMAs
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
                for (int i = 0; i < TM; ++i) fb[kk][i] = *reinterpret_cast<const f16x8*>(sB + i * 32 * LDK + kk * 16);
#pragma unroll
                for (int j = 0; j < TN; ++j) fa[kk][j] = *reinterpret_cast<const f16x8*>(sA + j * 32 * LDK + kk * 16);
            }
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[kk][j], fb[kk][i], acc[i][j], 0, 0, 0);
        };
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, PIPE - 1>;
        int steps = __popc(tilemask) * (e.Cin / KC);
        if constexpr (PIPE == 1) {
            load_next(S0{});
            store_stage(S0{});
            __syncthreads();
            while (steps > 0) {
                load_next(S0{});                             // in flight while this step is multiplied
                multiply(S0{});
                __syncthreads();
                if (--steps > 0) store_stage(S0{});
                __syncthreads();
            }
        } else {
            load_next(S0{});
            load_next(S1{});
            while (steps > 0) {
                store_stage(S0{});
                load_next(S0{});                             // refill the registers just drained
                __syncthreads();
                multiply(S0{});
                if (--steps == 0) break;
                store_stage(S1{});
                load_next(S1{});
                __syncthreads();
                multiply(S1{});
                --steps;
            }
            __syncthreads();                                 // all multiplications done: LDS becomes the C tile
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
        if (f == 1) {
            // P <- P + sum: all reads of P go out first (their latency is paid once), then the stores
            constexpr int RPP = 256 / TPR, NPASS = (BM + RPP - 1) / RPP;
            f16x8 pold[NPASS];
            f16* pp[NPASS];
#pragma unroll
            for (int t = 0; t < NPASS; ++t) {
                const int row = tid / TPR + t * RPP;
                const int rr = row < live ? row : 0;        // dead rows read entry 0 and store nothing
                pp[t] = (f16*)e.P + pdst_offset(e, s_wy[rr], s_wx[rr]) + n0 + c8;
                pold[t] = *reinterpret_cast<const f16x8*>(pp[t]);
            }
#pragma unroll
            for (int t = 0; t < NPASS; ++t) {
                const int row = tid / TPR + t * RPP;
                if (row < live) {
                    const float4 v0 = *reinterpret_cast<const float4*>(sC + row * LDC + c8);
                    const float4 v1 = *reinterpret_cast<const float4*>(sC + row * LDC + c8 + 4);
                    const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                    f16x8 o = pold[t];
#pragma unroll
                    for (int q = 0; q < 8; ++q) o[q] = (f16)((float)o[q] + v[q]);
                    *reinterpret_cast<f16x8*>(pp[t]) = o;
                }
            }
            continue;
        }
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

// Variant of tile_prologue for tiles that are index sub-ranges of a segment: the
// tile takes the entries among indices [sub_lo, sub_lo + sub_n) of segment `seg`
// (sub_lo a multiple of 64).  Returns their number; rows s_* are filled for them.
__device__ __forceinline__ int tile_prologue_sub(const EdgeDev& e, int seg, int sub_lo, int sub_n, bool publish, bool touch,
                                                 int* s_wy, int* s_wx, int* sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = e.Hp * e.Wp;
    const int p = seg * kSegPixels + tid;
    if (tid == 0) sh[4] = 0;
    int cy = 0, cx = 0, wy = 0, wx = 0;
    unsigned vm = 0;
    if (p < n && tid < kSegPixels) {                       // waves beyond the fourth only keep the barriers
        decode_entry(e, p, cy, cx, wy, wx);
        vm = tap_mask(e, cy, cx);
    }
    const bool has = vm != 0;
    const unsigned long long bal = __ballot(has);
    const int rank = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0 && wave < 4) sh[wave] = __popcll(bal);
    __syncthreads();
    int off = rank, base = 0, cnt = 0;
    for (int i = 0; i < 4; ++i) {
        if (i < wave) off += sh[i];
        if (i * 64 < sub_lo) base += sh[i];
        else if (i * 64 < sub_lo + sub_n) cnt += sh[i];
    }
    const bool mine = has && tid >= sub_lo && tid < sub_lo + sub_n;
    if (mine) {
        s_wy[off - base] = wy;
        s_wx[off - base] = wx;
        if (touch) mark_touched(e, wy, wx);
    }
    if (publish && has) e.clist[seg * kSegPixels + off] = p;
    if (publish && tid == 0) {                             // single writer per segment: no atomics
        const int tot = sh[0] + sh[1] + sh[2] + sh[3];
        e.ccnt[seg] = tot;
        e.cacc[seg] += (unsigned long long)tot;
    }
    int taps = mine ? __popc(vm) : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) taps += __shfl_xor(taps, o);
    if (lane == 0 && taps) atomicAdd(&sh[4], taps);
    __syncthreads();
    return cnt;
}

// Variant of tile_prologue for tiles that are th x tw rectangles of the padded window (th * tw <= 256, top-left
// corner (wy0, wx0)): thread t looks at tile pixel (t / tw, t % tw); the live ones are ranked in that order.
// Returns their number; rows s_wy / s_wx are filled for them, sh[4] = valid taps of the tile.
// The tap mask of a tile pixel is read off the tile's staged rectangle: s_pix[ry * rw + rx] >= 0 where the source pixel
// (ry, rx) of the rectangle (the tile plus its halo) is in view and updated (3x3, stride 1: the footprint of tile pixel
// (ly, lx) is rectangle rows ly .. ly + 2, columns lx .. lx + 2) - no flag loads of its own.
// pub_seg >= 0: the block also ranks list segment pub_seg (256 consecutive window indices), whose tap masks vm_p the
// caller has requested with the rectangle's flags; pub_off = this thread's position in that segment's compute list or
// -1, sh[8 .. 11] the entries of the segment per wave.  Nothing is written to global memory here: the wave's later
// loads would queue behind those stores (tile_effects_2d does it once the tile's own loads are done).
__device__ __forceinline__ int tile_prologue_2d(const EdgeDev& e, int wy0, int wx0, int th, int tw, const int* s_pix, int rw,
                                                int pub_seg, unsigned vm_p, int& pub_off, int* s_wy, int* s_wx, int* sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) sh[4] = 0;
    const int ly = tid / tw, lx = tid - ly * tw;
    const int wy = wy0 + ly, wx = wx0 + lx;
    const bool in_tile = ly < th && wy < e.Hp && wx < e.Wp;
    const bool in_seg = pub_seg >= 0 && pub_seg * kSegPixels + tid < e.Hp * e.Wp;
    unsigned vm = 0;
    if (in_tile) {
        const int* r = s_pix + ly * rw + lx;
#pragma unroll
        for (int t = 0; t < 9; ++t) vm |= (unsigned)(r[(t / 3) * rw + t % 3] >= 0) << t;
    }
    const bool has = vm != 0, hasp = in_seg && vm_p != 0;
    const unsigned long long bal = __ballot(has), balp = __ballot(hasp);
    const unsigned long long below = (1ull << lane) - 1ull;
    if (lane == 0) { sh[wave] = __popcll(bal); sh[8 + wave] = __popcll(balp); }
    __syncthreads();
    int off = __popcll(bal & below), offp = __popcll(balp & below);
    for (int i = 0; i < wave; ++i) { off += sh[i]; offp += sh[8 + i]; }
    const int cnt = sh[0] + sh[1] + sh[2] + sh[3];
    if (has) {
        s_wy[off] = wy;
        s_wx[off] = wx;
    }
    pub_off = hasp ? offp : -1;
    int taps = __popc(vm);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) taps += __shfl_xor(taps, o);
    if (lane == 0 && taps) atomicAdd(&sh[4], taps);
    __syncthreads();
    return cnt;
}

// What a tile leaves behind besides its sums, after tile_prologue_2d: the touched marks of its `tot` entries and the
// multiply-accumulate count (touch), the compute list of segment pub_seg and its counts.  No barrier.
__device__ __forceinline__ void tile_effects_2d(const EdgeDev& e, int tot, bool touch, int pub_seg, int pub_off,
                                                const int* s_wy, const int* s_wx, const int* sh) {
    const int tid = threadIdx.x;
    if (touch) {
        for (int r = tid; r < tot; r += 256) mark_touched(e, s_wy[r], s_wx[r]);
        if (tid == 0) add_macs(e, sh[4], 0);
    }
    if (pub_seg >= 0) {
        if (pub_off >= 0) e.clist[pub_seg * kSegPixels + pub_off] = pub_seg * kSegPixels + tid;
        if (tid == 0) {                                    // single writer per segment: no atomics
            const int n = sh[8] + sh[9] + sh[10] + sh[11];
            e.ccnt[pub_seg] = n;
            e.cacc[pub_seg] += (unsigned long long)n;
        }
    }
}

// ---------------------------------------------------------------------------
// Halo-staged MFMA convolution: KS x KS, stride 1, fp16, weights in the packed
// order [tap][cin/16][cout][16] (k_pack_weights).
// A tile is one NSUB-th of a list segment -- the entries among SUB = kSegPixels
// / NSUB consecutive indices of the padded window -- x BN couts.  Every input
// pixel those entries read lies in a small rectangle of the source (the rows
// the index range spans plus KS-1, full width if it spans more than one row).
// Per KC-channel chunk that rectangle is staged ONCE in LDS -- zero rows for
// pixels out of view or not updated, which is all the masking the taps need --
// and all KS*KS taps multiply out of it: the deltas are fetched once instead
// of once per tap.  The weights never touch LDS: the four waves are WMV
// (row-tile groups) x WK (K split); a wave multiplies its row tiles x TN 32x32
// accumulators over every WK-th 16-channel block of every tap and loads
// exactly the fragments it needs, 1 KiB contiguous each, several steps ahead.
// The body of a chunk is straight-line code (static taps, static register
// rings), so the loads of the next steps and of the next chunk stay in flight
// behind the matrix instructions; two tiles per compute unit cover each
// other's barriers.  The K-split partial sums are added in a fixed order
// through LDS, so the result does not depend on timing; P is then updated with
// 16-byte accesses.
// ---------------------------------------------------------------------------
template <int NSUB, int WMV, int WK, int TM, int TN, int KC, int NLD_, int KS, int RING_ = 3, int MINB_ = (NSUB >= 2 ? 2 : 1)>
struct HaloCfg {
    static constexpr int SUB = kSegPixels / NSUB;    // indices (and at most entries) per tile
    static_assert(WMV * WK == 4 && WMV * TM * 32 == SUB && SUB % 64 == 0, "4 waves cover one tile");
    static constexpr int BN = 32 * TN;
    static constexpr int KB = KC / 16;               // 16-channel blocks per chunk
    static_assert(KB % WK == 0, "every K wave takes the same number of blocks per tap");
    static constexpr int MB = KB / WK;               // blocks per tap and wave
    static constexpr int NS = KS * KS * MB;          // steps per chunk and wave
    static constexpr int RING = RING_;               // weight-fragment sets in flight; divides NS, so the
                                                     // ring carries over from chunk to chunk.  Above 3 the
                                                     // registers go to the ring and the next chunk of the
                                                     // rectangle is fetched at the chunk boundary instead of
                                                     // being prefetched into registers during the chunk
    static_assert(NS % RING == 0, "static ring slots");
    static constexpr int CPR = KC / 8;               // 16-byte pieces per staged pixel
    static constexpr int NLD = NLD_;                 // pieces per thread and chunk
    static constexpr int CAP = NLD * 256 / CPR;      // staged pixels
    static constexpr int LDK = KC + 8;               // staged row, halves (16 bytes of padding)
    static constexpr int LDC = BN + 4;               // accumulator row, floats
    static constexpr int HALO_BYTES = CAP * LDK * 2;
    static constexpr int C_BYTES = SUB * LDC * 4;
    static constexpr int MAIN_BYTES = HALO_BYTES > C_BYTES ? HALO_BYTES : C_BYTES;
    static constexpr int SMEM = MAIN_BYTES + CAP * 4;   // + source pixel index of every staged position
    static constexpr int LPS = (NLD + NS / 2 - 1) / (NS / 2);   // staging loads per step (first steps of a chunk)
    static constexpr int NLS = (NLD + LPS - 1) / LPS;
    static_assert(NLS <= NS, "staging loads fit the steps of a chunk");
    static constexpr int MINB = MINB_;               // tiles per compute unit the registers are budgeted for
};

// T2D: the tiles are th x tw rectangles of the padded window (th * tw <= SUB) instead of index ranges: the staged rectangle
// is the tile plus its KS - 1 halo whatever the width of the window, so wide rows fit and narrow ones stage less.
template <int NSUB, int WMV, int WK, int TM, int TN, int KC, int NLD_, int KS, int RING_ = 3, int MINB_ = (NSUB >= 2 ? 2 : 1), bool T2D = false>
__global__ __launch_bounds__(256, MINB_)
void k_conv_halo(EdgeBatch eb, int NT, int work_items, int th, int tw) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    using Cfg = HaloCfg<NSUB, WMV, WK, TM, TN, KC, NLD_, KS, RING_, MINB_>;
    constexpr int SUB = Cfg::SUB, BN = Cfg::BN, KB = Cfg::KB, MB = Cfg::MB, NS = Cfg::NS, CPR = Cfg::CPR, NLD = Cfg::NLD,
                  LDK = Cfg::LDK, LDC = Cfg::LDC;
    extern __shared__ __align__(16) unsigned char smem[];
    f16* halo = reinterpret_cast<f16*>(smem);            // [CAP][LDK] during the K loop
    float* sC = reinterpret_cast<float*>(smem);          // [SUB][LDC] after it
    int* s_pix = reinterpret_cast<int*>(smem + Cfg::MAIN_BYTES);
    __shared__ int s_wy[SUB], s_wx[SUB];
    __shared__ int sh[12];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: scalar branches below
    const int wm = wave % WMV, wk = wave / WMV;
    const int r32 = lane & 31, kh = lane >> 5;
    const int tiles_x = T2D ? (e.Wp + tw - 1) / tw : 1;
    const int ntiles = T2D ? tiles_x * ((e.Hp + th - 1) / th) : edge_segments(e) * NSUB;
    const int nchunks = e.Cin / KC;
    const int nwin = e.Hp * e.Wp;
    // (the host checks that both tensors are smaller than 2 GiB)
    const rsrc_t drs = make_rsrc(e.delta, (unsigned)e.sH * (unsigned)e.sW * (unsigned)e.Cin * 2u);
    const rsrc_t wrs = make_rsrc(e.wp, (unsigned)(KS * KS) * (unsigned)e.Cin * (unsigned)e.Cout * 2u);
    const unsigned tap_stride = (unsigned)(e.Cin / 16) * (unsigned)e.Cout * 32u;   // packed weights: bytes per tap
    const unsigned blk_stride = (unsigned)e.Cout * 32u;                            //                 per 16-channel block

    unsigned warm = 0;
    if constexpr (T2D) {
        // the blocks of a cout tile touch that tile's weights, a line each, before anything else: the fragments of the
        // K loop then come from the L2 of their XCD instead of following each other to memory
        const unsigned nt0 = blockIdx.x % NT, nblk = gridDim.x / NT > 0 ? gridDim.x / NT : 1, rank = blockIdx.x / NT;
        const unsigned kb = e.Cin / 16, lpf = BN * 32 / 128, nlines = KS * KS * kb * lpf;
        for (unsigned l = rank * 256 + tid; l < nlines; l += nblk * 256) {
            const unsigned f = l / lpf, ln = l - f * lpf;
            const unsigned off = (f / kb) * tap_stride + (f % kb) * blk_stride + nt0 * BN * 32 + ln * 128;
            warm ^= (unsigned)__builtin_amdgcn_raw_buffer_load_b32(wrs, (int)off, 0, 0);
        }
    }
    carry_source_compaction(e, sh);

    for (int u = blockIdx.x; u < work_items; u += gridDim.x) {
        const int nt = u % NT, mt = u / NT;              // u % 8 picks the XCD: few cout tiles per XCD
        if (mt >= ntiles) continue;
        const int n0 = nt * BN;
        __syncthreads();                                  // previous tile is done with LDS
        int tot, wyA, wyB, cxA, cxB;                      // entries; window rows and source columns the tile spans
        constexpr int NRF = (Cfg::CAP + 255) / 256;       // rectangle positions per thread
        int rpix[NRF];                                    // T2D: source pixel of this thread's positions, -1 outside the view
        unsigned rflag[NRF];                              //      and its flags, requested together with those of the prologue
        int pub_seg = -1, pub_off = -1;
        if constexpr (T2D) {
            const int ty = mt / tiles_x, tx = mt - ty * tiles_x;
            wyA = ty * th;
            wyB = (wyA + th < e.Hp ? wyA + th : e.Hp) - 1;
            cxA = tx * tw - e.bx0;
            cxB = (tx * tw + tw < e.Wp ? tx * tw + tw : e.Wp) - 1 - e.bx0;
            const int ry0 = wyA - e.by0 - e.pad, rx0 = cxA - e.pad, rw = cxB - cxA + KS, rn = (wyB - wyA + KS) * rw;
#pragma unroll
            for (int j = 0; j < NRF; ++j) {
                const int pos = tid + 256 * j;
                const int ry = pos / rw, iy = ry0 + ry, ix = rx0 + pos - ry * rw;
                const bool ok = pos < rn && iy >= 0 && iy < e.sH && ix >= 0 && ix < e.sW;
                rpix[j] = ok ? iy * e.sW + ix : -1;
                rflag[j] = e.sflags[ok ? rpix[j] : 0];
            }
            // every list segment is published by one of the first tiles (there are at least as many tiles as segments):
            // the flags of its footprints travel with those of the rectangle
            pub_seg = nt == 0 && mt < edge_segments(e) ? mt : -1;
            unsigned vm_p = 0;
            if (pub_seg >= 0) {
                const int p = pub_seg * kSegPixels + tid, qy = p / e.Wp, qx = p - qy * e.Wp;
                const bool in_seg = p < nwin;              // (threads beyond the window read the flags of pixel (0, 0): unused)
                vm_p = tap_mask(e, in_seg ? qy - e.by0 : 0, in_seg ? qx - e.bx0 : 0);
            }
            // the rectangle: source pixel of every position, -1 where it is out of view or not updated
#pragma unroll
            for (int j = 0; j < NRF; ++j) {
                const int pos = tid + 256 * j;
                if (pos < rn) s_pix[pos] = rpix[j] >= 0 && (rflag[j] & kFlagM) ? rpix[j] : -1;
            }
            __syncthreads();
            tot = tile_prologue_2d(e, ty * th, tx * tw, th, tw, s_pix, rw, pub_seg, vm_p, pub_off, s_wy, s_wx, sh);
            if (tot <= 0) tile_effects_2d(e, 0, false, pub_seg, pub_off, s_wy, s_wx, sh);
        } else {
            const int seg = mt / NSUB, sub_lo = (mt % NSUB) * SUB;
            tot = tile_prologue_sub(e, seg, sub_lo, SUB, nt == 0 && sub_lo == 0, nt == 0, s_wy, s_wx, sh);
            // the source rectangle this index range reads (block-uniform)
            const int a = seg * kSegPixels + sub_lo;
            const int last = (a + SUB < nwin ? a + SUB : nwin) - 1;
            wyA = a / e.Wp; wyB = last / e.Wp;
            cxA = wyA == wyB ? a - wyA * e.Wp - e.bx0 : -e.bx0;
            cxB = wyA == wyB ? last - wyA * e.Wp - e.bx0 : e.Wp - 1 - e.bx0;
        }
        if (tot <= 0) continue;
        if (!T2D && tid == 0 && nt == 0) add_macs(e, sh[4], 0);
        const int iy0 = wyA - e.by0 - e.pad, ix0 = cxA - e.pad;
        const int RW = cxB - cxA + KS, npos = (wyB - wyA + KS) * RW;       // npos <= CAP: checked by the host
        if constexpr (!T2D) {                             // (rectangular tiles: s_pix was filled ahead of the prologue)
            for (int pos = tid; pos < npos; pos += 256) {
                const int ry = pos / RW, rx = pos - ry * RW;
                const int iy = iy0 + ry, ix = ix0 + rx;
                const bool ok = iy >= 0 && iy < e.sH && ix >= 0 && ix < e.sW && (e.sflags[iy * e.sW + ix] & kFlagM);
                s_pix[pos] = ok ? iy * e.sW + ix : -1;
            }
            __syncthreads();
        }
        const int nrt = (tot + 31) >> 5;                  // live 32-entry row tiles of the tile
        const int mylive = nrt > wm ? (nrt - wm + WMV - 1) / WMV : 0;      // of this wave: row tiles wm, wm + WMV, ...

        // staging: piece q = tid + 256 j is 16 bytes of staged pixel q / CPR (q / CPR < CAP: inside the buffer).
        // Dead pieces (outside the rectangle, out of view, not updated) are loaded from beyond the end of the
        // delta map, which a buffer load answers with zeros, and stored like the others: no predicates.
        f16x8 hreg[NLD];
        unsigned hsrc[NLD];                               // byte offsets into the delta map
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int q = tid + 256 * j, pos = q / CPR;
            const int pix = pos < npos ? s_pix[pos] : -1;
            hsrc[j] = pix >= 0 ? ((unsigned)pix * (unsigned)e.Cin + (q % CPR) * 8) * 2u : 0x80000000u;
        }
        auto halo_store = [&]() {
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                const int q = tid + 256 * j;
                *reinterpret_cast<f16x8*>(halo + (q / CPR) * LDK + (q % CPR) * 8) = hreg[j];
            }
        };
#pragma unroll
        for (int j = 0; j < NLD; ++j) hreg[j] = buf_load16(drs, hsrc[j], 0u);
        halo_store();

        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        int rowoff[TM];                                   // this lane's staged row per row tile (halves)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = (i * WMV + wm) * 32 + r32;
            rowoff[i] = kh * 8 + wk * 16 + (r < tot ? ((s_wy[r] - e.by0 - e.pad - iy0) * RW + (s_wx[r] - e.bx0 - e.pad - ix0)) * LDK : 0);
        }
        const unsigned wlane = (unsigned)(r32 * 16 + kh * 8) * 2u;                      // this lane's bytes within a fragment
        const unsigned wwave = ((unsigned)wk * (unsigned)e.Cout + (unsigned)n0) * 32u;   // this wave's K block and cout tile
        __syncthreads();

        // The K loop for L live row tiles of this wave.  Step i of a chunk: tap i / MB,
        // 16-channel block wk + WK * (i % MB) of the chunk.
        auto kloop = [&](auto lc) {
            constexpr int L = decltype(lc)::value;
            constexpr int D = Cfg::RING;
            constexpr int FBR = TM > 4 ? 2 : 3;                      // sets of staged-row fragments in flight
            f16x8 fa[D][TN], fb[FBR][L > 0 ? L : 1];
            auto load_a = [&](int slot, int c, int i) {              // i may run into the next chunk
                const int cc = i < NS ? c : (c + 1 < nchunks ? c + 1 : c), ii = i < NS ? i : i - NS;
                const unsigned src = wwave + (unsigned)(ii / MB) * tap_stride + (unsigned)(cc * KB + WK * (ii % MB)) * blk_stride;
#pragma unroll
                for (int j = 0; j < TN; ++j) fa[slot][j] = buf_load16(wrs, wlane, src + (unsigned)j * 32u * 32u);
            };
            auto load_b = [&](int slot, int i) {
                const int tap = i / MB;
                const f16* hb = halo + ((tap / KS) * RW + tap % KS) * LDK + WK * (i % MB) * 16;
#pragma unroll
                for (int t = 0; t < L; ++t) fb[slot][t] = *reinterpret_cast<const f16x8*>(hb + rowoff[t]);
            };
#pragma unroll
            for (int i = 0; i < D - 1; ++i) load_a(i, 0, i);
            for (int c = 0; c < nchunks; ++c) {
                const int cn = c + 1 < nchunks ? c + 1 : c;          // the last chunk re-reads itself: no branch
                const unsigned hc = (unsigned)cn * KC * 2u;
#pragma unroll
                for (int i = 0; i < FBR - 1; ++i) load_b(i, i);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    if (Cfg::RING <= 3 && i < Cfg::NLS) { // staging loads of the next chunk, a few per step
#pragma unroll
                        for (int j = i * Cfg::LPS; j < (i + 1) * Cfg::LPS && j < NLD; ++j)
                            hreg[j] = buf_load16(drs, hsrc[j], hc);
                    }
                    load_a((i + D - 1) % D, c, i + D - 1);
                    if (i + FBR - 1 < NS) load_b((i + FBR - 1) % FBR, i + FBR - 1);
#pragma unroll
                    for (int t = 0; t < L; ++t)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i % D][j], fb[i % FBR][t], acc[t][j], 0, 0, 0);
                    // the loads just issued (for later steps) stay ahead of these MFMAs and are
                    // spread between them: one LDS read, one global load, a quarter of the MFMAs
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                       // one LDS read
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                       // one global load
                        __builtin_amdgcn_sched_group_barrier(0x008, (L * TN + 3) / 4, 0);        // a quarter of the MFMAs
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();                          // everyone is done reading the staged chunk
                if (c + 1 < nchunks) {
                    if constexpr (Cfg::RING > 3) {        // deep weight ring: the registers go to it, the next chunk is
                                                          // fetched here (the weight loads of its first steps are in flight)
#pragma unroll
                        for (int j = 0; j < NLD; ++j) hreg[j] = buf_load16(drs, hsrc[j], hc);
                    }
                    halo_store();
                    __syncthreads();
                }
            }
        };
        switch (mylive) {
            case 0: kloop(std::integral_constant<int, 0>{}); break;
            case 1: kloop(std::integral_constant<int, 1>{}); break;
            case 2: kloop(std::integral_constant<int, TM >= 2 ? 2 : TM>{}); break;
            case 3: kloop(std::integral_constant<int, (TM > 4 ? 4 : TM >= 3 ? 3 : TM)>{}); break;    // rounded up: dead tiles are not stored
            case 4: kloop(std::integral_constant<int, (TM >= 4 ? 4 : TM)>{}); break;
            default: kloop(std::integral_constant<int, TM>{}); break;
        }

        // K-split partial sums -> LDS [entry][cout].  Every element is added up in a fixed
        // order of the K waves: with four K waves over all rows, wave w takes quarter
        // (w + p) % 4 of the rows in phase p (all waves busy in every phase); otherwise
        // the K waves take turns.
        auto put = [&](int i, bool add) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                float* dst = sC + ((i * WMV + wm) * 32 + r32) * LDC + j * 32 + 4 * kh;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float4 v = make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                    if (add) {
                        const float4 o = *reinterpret_cast<const float4*>(dst + 8 * g);
                        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                    }
                    *reinterpret_cast<float4*>(dst + 8 * g) = v;
                }
            }
        };
        if constexpr (WK == 4 && WMV == 1 && TM % 4 == 0) {
#pragma unroll
            for (int ph = 0; ph < 4; ++ph) {
                const int q = (wk + ph) & 3;
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    if (i / (TM / 4) == q && i < mylive) put(i, ph > 0);
                __syncthreads();
            }
        } else {
#pragma unroll
            for (int kq = 0; kq < WK; ++kq) {
                if (wk == kq) {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (i < mylive) put(i, kq > 0);
                }
                __syncthreads();
            }
        }
        // P <- P + sum: all reads of P go out first (their latency is paid once), then the stores
        constexpr int TPR = BN / 8;                        // threads per entry, 8 couts each
        constexpr int RPP = 256 / TPR, NPASS = (SUB + RPP - 1) / RPP;
        const int c8 = (tid % TPR) * 8;
        f16x8 pold[NPASS];
        f16* pp[NPASS];
#pragma unroll
        for (int t = 0; t < NPASS; ++t) {
            const int row = tid / TPR + t * RPP;
            const int rr = row < tot ? row : 0;             // dead rows read entry 0 and store nothing
            pp[t] = (f16*)e.P + pdst_offset(e, s_wy[rr], s_wx[rr]) + n0 + c8;
            pold[t] = *reinterpret_cast<const f16x8*>(pp[t]);
        }
#pragma unroll
        for (int t = 0; t < NPASS; ++t) {
            const int row = tid / TPR + t * RPP;
            if (row < tot) {
                const float4 v0 = *reinterpret_cast<const float4*>(sC + row * LDC + c8);
                const float4 v1 = *reinterpret_cast<const float4*>(sC + row * LDC + c8 + 4);
                const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                f16x8 o = pold[t];
#pragma unroll
                for (int q = 0; q < 8; ++q) o[q] = (f16)((float)o[q] + v[q]);
                *reinterpret_cast<f16x8*>(pp[t]) = o;
            }
        }
        if constexpr (T2D) tile_effects_2d(e, tot, nt == 0, pub_seg, pub_off, s_wy, s_wx, sh);
    }
    if (warm == 0x9e3779b9u && work_items < 0) e.ccnt[0] = 0;     // (keeps the loads above)
}

// Weights [tap][cout][cin] -> [tap][cin/16][cout][16]: the 32 couts x 16 cin
// operand of one MFMA becomes 1 KiB of consecutive memory.  One thread per 8 halves.
__global__ __launch_bounds__(256) void k_pack_weights(const f16* __restrict__ src, f16* __restrict__ dst, int taps, int Cout, int Cin) {
    const long long n8 = (long long)taps * Cout * Cin / 8;
    const int KBT = Cin / 16;
    for (long long i = blockIdx.x * 256ll + threadIdx.x; i < n8; i += gridDim.x * 256ll) {
        const int h = (int)(i & 1);
        long long r = i >> 1;
        const int co = (int)(r % Cout); r /= Cout;
        const int kb = (int)(r % KBT);
        const int tap = (int)(r / KBT);
        *reinterpret_cast<f16x8*>(dst + i * 8) =
            *reinterpret_cast<const f16x8*>(src + ((long long)tap * Cout + co) * Cin + kb * 16 + h * 8);
    }
}

// ---------------------------------------------------------------------------
// MFMA without LDS staging: every wave loads its own fragments from global
// memory.  Block = 4 waves arranged (4/WN) x WN over (pixels x couts); every
// lane updates its own pixel of P.  Fallback for Cin % 32 != 0.
// ---------------------------------------------------------------------------
template <int WN>
__global__ __launch_bounds__(256) void k_conv_mfma_f16(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    constexpr int WM = 4 / WN;
    constexpr int TILE_M = 32 * WM;
    constexpr int TPS = kSegPixels / TILE_M;
    __shared__ int s_base[TILE_M], s_wy[TILE_M], s_wx[TILE_M];
    __shared__ unsigned s_vm[TILE_M];
    __shared__ int sh[8];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int col = lane & 31, kh = lane >> 5;
    const int MT = edge_segments(e) * TPS;
    const int n0 = (blockIdx.y * WN + wn) * 32;
    const f16* __restrict__ delta = (const f16*)e.delta;
    const f16* __restrict__ w = (const f16*)e.w;
    const int taps = e.k * e.k;
    carry_source_compaction(e, sh);
    for (int tile = blockIdx.x; tile < MT; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * TILE_M;
        __syncthreads();
        const int tot = tile_prologue(e, seg, first, TILE_M, blockIdx.y == 0 && first == 0 && !e.up, blockIdx.y == 0,
                                      s_base, s_wy, s_wx, s_vm, sh);
        if (first >= tot) continue;
        if (threadIdx.x == 0 && blockIdx.y == 0) add_macs(e, sh[4], 0);
        const int row = wm * 32 + col;
        const bool live = first + row < tot;
        const unsigned vmask = s_vm[row];
        const int base = s_base[row], wy = s_wy[row], wx = s_wx[row];
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        for (int tap = 0; tap < taps; ++tap) {
            const bool v = (vmask >> tap) & 1u;
            if (__ballot(v) == 0ull) continue;                 // no pixel of this wave uses the tap
            const int jy = tap / e.k, jx = tap - jy * e.k;
            const f16* arow = w + ((size_t)(tap * e.Cout + n0 + col)) * e.Cin + kh * 8;
            const f16* brow = delta + (v ? ((size_t)(base + jy * e.sW + jx)) * e.Cin + kh * 8 : 0);
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
        }
    }
}

template <typename T> struct Row8;
template <> struct Row8<f16> {
    typedef f16x8 reg;                                      // eight stored values, fetched ahead of their use
    __device__ static reg load(const f16* p) { return *reinterpret_cast<const f16x8*>(p); }
    __device__ static void add_store(f16* p, reg o, const float* v) {
#pragma unroll
        for (int q = 0; q < 8; ++q) o[q] = (f16)((float)o[q] + v[q]);
        *reinterpret_cast<f16x8*>(p) = o;
    }
    __device__ static void add(f16* p, const float* v) { add_store(p, load(p), v); }
};
template <> struct Row8<float> {
    struct reg { float4 a, b; };
    __device__ static reg load(const float* p) { return reg{*reinterpret_cast<const float4*>(p), *reinterpret_cast<const float4*>(p + 4)}; }
    __device__ static void add_store(float* p, reg o, const float* v) {
        o.a.x += v[0]; o.a.y += v[1]; o.a.z += v[2]; o.a.w += v[3];
        o.b.x += v[4]; o.b.y += v[5]; o.b.z += v[6]; o.b.w += v[7];
        *reinterpret_cast<float4*>(p) = o.a;
        *reinterpret_cast<float4*>(p + 4) = o.b;
    }
    __device__ static void add(float* p, const float* v) { add_store(p, load(p), v); }
};

// ---------------------------------------------------------------------------
// Plain FMA convolution with ALL weights resident in LDS as fp32
// [tap][cin][cout]; a thread owns one list entry and 8 consecutive couts.
// Used for fp32 networks and for layers the MFMA path does not take (e.g. a
// 3-channel stem).  Needs Cout % 8 == 0, Cout <= 512 and k*k*Cin*Cout*4 bytes
// of LDS.  Tiles of ppb entries never straddle a list segment.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_conv_ldsw(EdgeBatch eb, int groups, int ppb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    extern __shared__ __align__(16) unsigned char smem[];
    float* sW = reinterpret_cast<float*>(smem);             // [tap][Cin][Cout]
    __shared__ int s_base[256], s_wy[256], s_wx[256];
    __shared__ unsigned s_vm[256];
    __shared__ int sh[8];
    const int tid = threadIdx.x;
    const int cg = tid % groups, pl = tid / groups;         // cout group, local pixel
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    const int taps = e.k * e.k;
    const int cc = e.Cin * e.Cout;
    carry_source_compaction(e, sh);
    // weights [tap][cout][cin] -> LDS [tap][cin][cout] as fp32.  Neighbouring threads take neighbouring couts, so
    // their LDS stores fall into different banks; a thread reads 16 bytes of its weight row at a time.
    constexpr int WV = 16 / (int)sizeof(T);
    if (e.Cin % WV == 0) {
        // Eight reads of a thread are in flight at a time (the copy is a chain of round trips otherwise, and it is
        // the larger part of a launch on sparse frames); a read past the end of the tensor returns zeros and is dropped.
        const int pieces = e.Cin / WV, total = taps * pieces * e.Cout;
        const rsrc_t wrs = make_rsrc(w, (unsigned)(taps * cc) * (unsigned)sizeof(T));
        constexpr int WU = 8;
        for (int i0 = tid; i0 < total; i0 += 256 * WU) {
            u32x4_t raw[WU];
            int dst[WU];
#pragma unroll
            for (int u = 0; u < WU; ++u) {
                const int i = i0 + u * 256;
                const int co = i % e.Cout, q = i / e.Cout;
                const int piece = q % pieces, tap = q / pieces;
                const bool in = i < total;
                dst[u] = in ? tap * cc + piece * WV * e.Cout + co : -1;
                raw[u] = __builtin_amdgcn_raw_buffer_load_b128(
                    wrs, in ? (int)(((unsigned)(tap * e.Cout + co) * (unsigned)e.Cin + (unsigned)(piece * WV)) * (unsigned)sizeof(T)) : (int)0x80000000u, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < WU; ++u) {
                if (dst[u] < 0) continue;
                T a[WV];
                __builtin_memcpy(a, &raw[u], 16);
#pragma unroll
                for (int v = 0; v < WV; ++v) sW[dst[u] + v * e.Cout] = (float)a[v];
            }
        }
    } else {
        for (int i = tid; i < taps * cc; i += 256) {
            const int tap = i / cc, r = i - tap * cc;
            const int co = r / e.Cin, ci = r - co * e.Cin;
            sW[tap * cc + ci * e.Cout + co] = (float)w[i];
        }
    }
    long long block_taps = 0;                               // statistics (thread 0 only)
    const int tps = (kSegPixels + ppb - 1) / ppb;           // tiles per segment
    const int MT = edge_segments(e) * tps;
    for (int tile = blockIdx.x; tile < MT; tile += gridDim.x) {
        const int seg = tile / tps, first = (tile - seg * tps) * ppb;
        __syncthreads();
        const int tot = tile_prologue(e, seg, first, ppb, first == 0 && !e.up, true, s_base, s_wy, s_wx, s_vm, sh);
        if (first >= tot) continue;
        if (tid == 0) block_taps += sh[4];
        if (pl >= ppb || first + pl >= tot) continue;
        const unsigned vmask = s_vm[pl];
        const int base = s_base[pl];
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int tap = 0; tap < taps; ++tap) {
            if (!((vmask >> tap) & 1u)) continue;
            const int jy = tap / e.k, jx = tap - jy * e.k;
            const T* drow = delta + (size_t)(base + jy * e.sW + jx) * e.Cin;
            const float* wt = sW + tap * cc + cg * 8;
            auto mac = [&](float a, int ci) {               // channels in ascending order: the sum does not change
                const float4 w0 = *reinterpret_cast<const float4*>(wt + ci * e.Cout);
                const float4 w1 = *reinterpret_cast<const float4*>(wt + ci * e.Cout + 4);
                acc[0] = fmaf(a, w0.x, acc[0]); acc[1] = fmaf(a, w0.y, acc[1]);
                acc[2] = fmaf(a, w0.z, acc[2]); acc[3] = fmaf(a, w0.w, acc[3]);
                acc[4] = fmaf(a, w1.x, acc[4]); acc[5] = fmaf(a, w1.y, acc[5]);
                acc[6] = fmaf(a, w1.z, acc[6]); acc[7] = fmaf(a, w1.w, acc[7]);
            };
            constexpr int V = 16 / (int)sizeof(T);           // a row is read in 16-byte pieces, several of them in flight
            if (e.Cin % V == 0) {
#pragma unroll 8
                for (int ci = 0; ci < e.Cin; ci += V) {
                    const u32x4_t raw = *reinterpret_cast<const u32x4_t*>(drow + ci);
                    T a[V];
                    __builtin_memcpy(a, &raw, 16);
#pragma unroll
                    for (int v = 0; v < V; ++v) mac((float)a[v], ci + v);
                }
            } else {
                for (int ci = 0; ci < e.Cin; ++ci) mac((float)drow[ci], ci);
            }
        }
        const int f = 1 << e.up;
        for (int ua = 0; ua < f; ++ua)
            for (int ub = 0; ub < f; ++ub)
                Row8<T>::add((T*)e.P + pdst_offset(e, s_wy[pl] + ua, s_wx[pl] + ub) + cg * 8, acc);
    }
    if (tid == 0) add_macs(e, block_taps, 1);               // statistics: one atomic per block
}

// ---------------------------------------------------------------------------
// fp32 layers on the matrix cores (v_mfma_f32_32x32x2_f32), Cin and footprint at
// compile time, Cout 16 or a multiple of 32, no upsampling.  A block owns one tile of
// 32 couts (blockIdx.y) and keeps its weights in LDS as [tap][cin][32]; its four
// waves are 4 / KS groups of 32 list entries x KS shares of the taps (wave k
// of a group takes taps k, k + KS, ...), and the partial sums of a group are
// added through LDS in a fixed order.  The matrix instruction takes the couts
// as rows and the entries as columns: a lane holds entry lane % 32 and half
// lane / 32 of the K pair, which is channel (lane / 32) * CIN / 2 + step - so a
// lane reads CIN / 2 consecutive channels of its entry's source row per tap, in
// 16-byte pieces, one tap ahead of the multiplication, and one weight per
// instruction from LDS (32 consecutive floats per half wave).  Taps outside an
// entry's mask are read from beyond the end of the tensor (zeros); the tap loop
// has no branches.
// ---------------------------------------------------------------------------
template <int KK, int CIN, int KS>
__global__ __launch_bounds__(256) void k_conv_mfma_f32(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    extern __shared__ __align__(16) unsigned char smem[];
    float* sW = reinterpret_cast<float*>(smem);             // [tap][CIN][32]
    constexpr int TAPS = KK * KK, HALF = CIN / 2, NP = HALF / 4, PGS = 4 / KS, BM = PGS * 32, NQ = (TAPS + KS - 1) / KS;
    constexpr int CC = CIN * 32;                            // floats per tap in LDS
    __shared__ int s_base[BM], s_wy[BM], s_wx[BM];
    __shared__ unsigned s_vm[BM];
    __shared__ int sh[8];
    __shared__ float s_red[KS > 1 ? PGS * (KS - 1) * 1024 : 1];    // partial sums of the waves that do not write P
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p32 = lane & 31, h = lane >> 5;
    const int pg = wave % PGS, ks = wave / PGS;             // entry group, share of the taps
    const int nt = blockIdx.y;                              // cout tile
    const int ncout = e.Cout - nt * 32 < 32 ? e.Cout - nt * 32 : 32;      // 16 for a 16-cout layer: the other rows of the tile are not stored
    const float* __restrict__ w = (const float*)e.w;
    carry_source_compaction(e, sh);
    // weights [tap][cout][cin] -> LDS [tap][cin][32], eight 16-byte reads of a thread in flight.  The first eight are
    // requested here and stored after the prologue of the block's first tile, whose flag reads they travel with.
    constexpr int pieces = CIN / 4, WU = 8, wtotal = TAPS * pieces * 32;
    const rsrc_t wrs = make_rsrc(w, (unsigned)(TAPS * CIN) * (unsigned)e.Cout * 4u);
    auto request = [&](int i0, u32x4_t* raw, int* dst) {
#pragma unroll
        for (int u = 0; u < WU; ++u) {
            const int i = i0 + u * 256;
            const int co = i % 32, q = i / 32;
            const int piece = q % pieces, tap = q / pieces;
            const bool in = i < wtotal && co < ncout;
            dst[u] = in ? tap * CC + piece * 4 * 32 + co : -1;
            raw[u] = __builtin_amdgcn_raw_buffer_load_b128(
                wrs, in ? (int)(((unsigned)(tap * e.Cout + nt * 32 + co) * (unsigned)CIN + (unsigned)(piece * 4)) * 4u) : (int)0x80000000u, 0, 0);
        }
    };
    auto store = [&](const u32x4_t* raw, const int* dst) {
#pragma unroll
        for (int u = 0; u < WU; ++u) {
            if (dst[u] < 0) continue;
            float a[4];
            __builtin_memcpy(a, &raw[u], 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) sW[dst[u] + v * 32] = a[v];
        }
    };
    u32x4_t raw0[WU];
    int dst0[WU];
    request(tid, raw0, dst0);
    bool weights_in = false;
    const rsrc_t drs = make_rsrc(e.delta, (unsigned)e.sH * (unsigned)e.sW * (unsigned)CIN * 4u);
    long long block_taps = 0;                               // statistics (thread 0 of the blocks of cout tile 0)
    constexpr int TPS = kSegPixels / BM;                    // tiles per segment
    const int MT = edge_segments(e) * TPS;
    for (int tile = blockIdx.x; tile < MT; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * BM;
        __syncthreads();
        const int tot = tile_prologue(e, seg, first, BM, nt == 0 && first == 0, nt == 0, s_base, s_wy, s_wx, s_vm, sh);
        if (!weights_in) {                                  // first tile of the block (block-uniform)
            store(raw0, dst0);
            for (int i0 = tid + 256 * WU; i0 < wtotal; i0 += 256 * WU) {
                u32x4_t raw[WU];
                int dst[WU];
                request(i0, raw, dst);
                store(raw, dst);
            }
            weights_in = true;
            __syncthreads();
        }
        if (first >= tot) continue;                         // block-uniform
        if (tid == 0 && nt == 0) block_taps += sh[4];
        const bool wave_on = first + pg * 32 < tot;         // wave-uniform: the group has entries
        const int pl = pg * 32 + p32;
        const bool act = first + pl < tot;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        if (wave_on) {
            const unsigned vmask = act ? s_vm[pl] : 0u;
            const int rowb = act ? (s_base[pl] * CIN + h * HALF) * 4 : 0;  // bytes; negative for a border entry's first taps
            auto load_tap = [&](int tap, u32x4_t* r) {      // tap >= TAPS (the last round of some waves): zeros
                const bool v = tap < TAPS && ((vmask >> tap) & 1u);
                const int jy = tap / KK, jx = tap - jy * KK;
                const int tb = rowb + (jy * e.sW + jx) * CIN * 4;
#pragma unroll
                for (int i = 0; i < NP; ++i)
                    r[i] = __builtin_amdgcn_raw_buffer_load_b128(drs, v ? tb + i * 16 : (int)0x80000000u, 0, 0);
            };
            u32x4_t rows[2][NP];
            load_tap(ks, rows[0]);
            const float* wl = sW + h * HALF * 32 + p32;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int tap = ks + KS * q;
                if (q + 1 < NQ) load_tap(tap + KS, rows[(q + 1) & 1]);
                const float* wt = wl + (tap < TAPS ? tap : TAPS - 1) * CC;
#pragma unroll
                for (int i = 0; i < NP; ++i) {
                    float b[4];
                    __builtin_memcpy(b, &rows[q & 1][i], 16);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wt[(i * 4 + j) * 32], b[j], acc, 0, 0, 0);
                }
            }
        }
        if constexpr (KS > 1) {
            if (wave_on && ks > 0) {
                float* red = s_red + (pg * (KS - 1) + ks - 1) * 1024 + lane;
#pragma unroll
                for (int r = 0; r < 16; ++r) red[r * 64] = acc[r];
            }
            __syncthreads();                                // all threads of the block, whatever their wave does
            if (wave_on && ks == 0) {
#pragma unroll
                for (int k = 1; k < KS; ++k) {
                    const float* red = s_red + (pg * (KS - 1) + k - 1) * 1024 + lane;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] += red[r * 64];
                }
            }
        }
        // register r of a lane: cout 8 * (r / 4) + 4 * (lane / 32) + r % 4 of the tile, entry lane % 32
        if (act && ks == 0) {
            float* pp = (float*)e.P + pdst_offset(e, s_wy[pl], s_wx[pl]) + nt * 32 + 4 * h;
            float4 o[4];
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if (8 * g < ncout) o[g] = *reinterpret_cast<const float4*>(pp + 8 * g);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (8 * g >= ncout) continue;
                o[g].x += acc[4 * g]; o[g].y += acc[4 * g + 1]; o[g].z += acc[4 * g + 2]; o[g].w += acc[4 * g + 3];
                *reinterpret_cast<float4*>(pp + 8 * g) = o[g];
            }
        }
    }
    if (tid == 0) add_macs(e, block_taps, 0);               // statistics: one atomic per block
}

// ---------------------------------------------------------------------------
// 3x3 stems with 3 input channels on the matrix cores, fp32 or fp16 storage
// (fp16 values are exact in fp32, so both use v_mfma_f32_32x32x2_f32 with the
// weights as fp32 in LDS).  K = 27 products per output, padded to 28: lane half
// h of a wave holds k = 14 h + step, k = 9 jy + 3 jx + ci, which is element
// (k / 9) * 3 sW + k % 9 after the entry's first tap - the three pixels of a
// footprint row are nine consecutive values.  A block owns 128 list entries and
// one tile of 32 couts (blockIdx.y), a wave 32 entries; a lane fetches its 14
// values with single-element buffer loads that all go out together (a tap
// outside the entry's mask reads beyond the tensor: zero).
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_conv_stem_mfma(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    constexpr int BM = 128, KH = 14;
    __shared__ float sW[2 * KH * 32];                       // [k][32 couts], row 27 zero
    __shared__ int s_base[BM], s_wy[BM], s_wx[BM];
    __shared__ unsigned s_vm[BM];
    __shared__ int sh[8];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p32 = lane & 31, h = lane >> 5;
    const int nt = blockIdx.y;
    const T* __restrict__ w = (const T*)e.w;
    carry_source_compaction(e, sh);
    for (int i = tid; i < 28 * 32; i += 256) {              // weights [tap][cout][3] -> LDS [k = 3 tap + ci][cout of the tile]
        const int k = i >> 5, co = i & 31;
        sW[i] = k < 27 ? (float)w[((k / 3) * e.Cout + nt * 32 + co) * 3 + k % 3] : 0.f;
    }
    const rsrc_t drs = make_rsrc(e.delta, (unsigned)e.sH * (unsigned)e.sW * 3u * (unsigned)sizeof(T));
    long long block_taps = 0;                               // statistics (thread 0 of the blocks of cout tile 0)
    constexpr int TPS = kSegPixels / BM;
    const int MT = edge_segments(e) * TPS;
    for (int tile = blockIdx.x; tile < MT; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * BM;
        __syncthreads();
        const int tot = tile_prologue(e, seg, first, BM, nt == 0 && first == 0, nt == 0, s_base, s_wy, s_wx, s_vm, sh);
        if (first >= tot) continue;                         // block-uniform
        if (tid == 0 && nt == 0) block_taps += sh[4];
        if (first + wave * 32 >= tot) continue;             // no entry for this wave (no barrier until the next tile)
        const int pl = wave * 32 + p32;
        const bool act = first + pl < tot;
        const unsigned vmask = act ? s_vm[pl] : 0u;
        const int base3 = act ? s_base[pl] * 3 : 0;         // elements; negative for a border entry's first taps
        float in[KH];
#pragma unroll
        for (int st = 0; st < KH; ++st) {
            const int k0 = st, k1 = KH + st;                // the two halves of the wave
            const int off = h ? (k1 / 9) * 3 * e.sW + k1 % 9 : (k0 / 9) * 3 * e.sW + k0 % 9;
            const bool v = h ? (k1 < 27 && ((vmask >> (k1 < 27 ? k1 / 3 : 0)) & 1u)) : ((vmask >> (k0 / 3)) & 1u);
            const int byte = v ? (base3 + off) * (int)sizeof(T) : (int)0x80000000u;
            if constexpr (sizeof(T) == 2)
                in[st] = (float)__builtin_bit_cast(f16, __builtin_amdgcn_raw_buffer_load_b16(drs, byte, 0, 0));
            else
                in[st] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(drs, byte, 0, 0));
        }
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        const float* wl = sW + h * KH * 32 + p32;
#pragma unroll
        for (int st = 0; st < KH; ++st) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wl[st * 32], in[st], acc, 0, 0, 0);
        // register r of a lane: cout 8 * (r / 4) + 4 * (lane / 32) + r % 4 of the tile, entry lane % 32
        if (act) {
            T* pp = (T*)e.P + pdst_offset(e, s_wy[pl], s_wx[pl]) + nt * 32 + 4 * h;
            if constexpr (sizeof(T) == 2) {
                f16x4 o[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) o[g] = *reinterpret_cast<const f16x4*>(pp + 8 * g);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) o[g][q] = (f16)((float)o[g][q] + acc[4 * g + q]);
                    *reinterpret_cast<f16x4*>(pp + 8 * g) = o[g];
                }
            } else {
                float4 o[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) o[g] = *reinterpret_cast<const float4*>(pp + 8 * g);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    o[g].x += acc[4 * g]; o[g].y += acc[4 * g + 1]; o[g].z += acc[4 * g + 2]; o[g].w += acc[4 * g + 3];
                    *reinterpret_cast<float4*>(pp + 8 * g) = o[g];
                }
            }
        }
    }
    if (tid == 0) add_macs(e, block_taps, 0);               // statistics: one atomic per block
}

// ---------------------------------------------------------------------------
// Stem-type layers (few input channels, e.g. RGB): compile-time footprint
// KK x KK x CIN.  A thread owns one list entry and CPT couts; all of its
// KK*KK*CIN inputs are fetched up front (independent loads), the weights are
// broadcast from LDS ([tap][cin][cout], fp32).
// ---------------------------------------------------------------------------
template <typename T, int KK, int CIN, int CPT>
__global__ __launch_bounds__(256) void k_conv_small(EdgeBatch eb, int groups, int ppb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    extern __shared__ __align__(16) unsigned char smem[];
    float* sW = reinterpret_cast<float*>(smem);             // [tap][CIN][Cout]
    __shared__ int s_base[256], s_wy[256], s_wx[256];
    __shared__ unsigned s_vm[256];
    __shared__ int sh[8];
    constexpr int TAPS = KK * KK;
    const int tid = threadIdx.x;
    const int cg = tid % groups, pl = tid / groups;
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    const int cc = CIN * e.Cout;
    carry_source_compaction(e, sh);
    for (int i = tid; i < TAPS * cc; i += 256) {
        const int tap = i / cc, r = i - tap * cc;
        const int co = r / CIN, ci = r - co * CIN;
        sW[tap * cc + ci * e.Cout + co] = (float)w[i];
    }
    long long block_taps = 0;
    const int tps = (kSegPixels + ppb - 1) / ppb;
    const int MT = edge_segments(e) * tps;
    for (int tile = blockIdx.x; tile < MT; tile += gridDim.x) {
        const int seg = tile / tps, first = (tile - seg * tps) * ppb;
        __syncthreads();
        const int tot = tile_prologue(e, seg, first, ppb, first == 0 && !e.up, true, s_base, s_wy, s_wx, s_vm, sh);
        if (first >= tot) continue;
        if (tid == 0) block_taps += sh[4];
        if (pl >= ppb || first + pl >= tot) continue;
        const unsigned vmask = s_vm[pl];
        const int base = s_base[pl];
        float in[TAPS * CIN];
#pragma unroll
        for (int tap = 0; tap < TAPS; ++tap) {
            const bool v = (vmask >> tap) & 1u;
            const T* src = delta + (v ? (size_t)(base + (tap / KK) * e.sW + (tap % KK)) * CIN : (size_t)0);
#pragma unroll
            for (int ci = 0; ci < CIN; ++ci) in[tap * CIN + ci] = (float)src[ci];
        }
#pragma unroll
        for (int tap = 0; tap < TAPS; ++tap)
            if (!((vmask >> tap) & 1u))
#pragma unroll
                for (int ci = 0; ci < CIN; ++ci) in[tap * CIN + ci] = 0.f;
        // the pending values this thread adds to travel while it multiplies (no upsampling: one pixel)
        const int f = 1 << e.up;
        T* pp0 = (T*)e.P + pdst_offset(e, s_wy[pl], s_wx[pl]) + cg * CPT;
        typename Row8<T>::reg pold[CPT / 8];
        if (f == 1) {
#pragma unroll
            for (int q = 0; q < CPT; q += 8) pold[q / 8] = Row8<T>::load(pp0 + q);
        }
        float acc[CPT];
#pragma unroll
        for (int q = 0; q < CPT; ++q) acc[q] = 0.f;
#pragma unroll
        for (int t = 0; t < TAPS * CIN; ++t) {
            const float a = in[t];
            const float* wt = sW + t * e.Cout + cg * CPT;
#pragma unroll
            for (int q = 0; q < CPT; q += 4) {
                const float4 w4 = *reinterpret_cast<const float4*>(wt + q);
                acc[q] = fmaf(a, w4.x, acc[q]); acc[q + 1] = fmaf(a, w4.y, acc[q + 1]);
                acc[q + 2] = fmaf(a, w4.z, acc[q + 2]); acc[q + 3] = fmaf(a, w4.w, acc[q + 3]);
            }
        }
        if (f == 1) {
#pragma unroll
            for (int q = 0; q < CPT; q += 8) Row8<T>::add_store(pp0 + q, pold[q / 8], acc + q);
            continue;
        }
        for (int ua = 0; ua < f; ++ua)
            for (int ub = 0; ub < f; ++ub) {
                T* pp = (T*)e.P + pdst_offset(e, s_wy[pl] + ua, s_wx[pl] + ub) + cg * CPT;
#pragma unroll
                for (int q = 0; q < CPT; q += 8) Row8<T>::add(pp + q, acc + q);
            }
    }
    if (tid == 0) add_macs(e, block_taps, 1);
}

// ---------------------------------------------------------------------------
// Plain FMA convolution for any dtype / channel count.
// Block = 16 list entries x 16 cout lanes; each thread keeps 4 couts at a time.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_conv_plain(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    __shared__ int s_base[16], s_wy[16], s_wx[16];
    __shared__ unsigned s_vm[16];
    __shared__ int sh[8];
    const int p = threadIdx.x >> 4, cl = threadIdx.x & 15;
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    const int taps = e.k * e.k;
    constexpr int TPS = kSegPixels / 16;
    const int MT = edge_segments(e) * TPS;
    carry_source_compaction(e, sh);
    for (int tile = blockIdx.x; tile < MT; tile += gridDim.x) {
        const int seg = tile / TPS, first = (tile - seg * TPS) * 16;
        __syncthreads();
        const int tot = tile_prologue(e, seg, first, 16, first == 0 && !e.up, true, s_base, s_wy, s_wx, s_vm, sh);
        if (first >= tot) continue;
        if (threadIdx.x == 0) add_macs(e, sh[4], 1);
        if (first + p >= tot) continue;
        const unsigned vmask = s_vm[p];
        const int base = s_base[p], wy = s_wy[p], wx = s_wx[p];
        for (int cg = 0; cg < e.Cout; cg += 64) {
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
            for (int tap = 0; tap < taps; ++tap) {
                if (!((vmask >> tap) & 1u)) continue;
                const int jy = tap / e.k, jx = tap - jy * e.k;
                const T* drow = delta + ((size_t)(base + jy * e.sW + jx)) * e.Cin;
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
    }
}

// Residual skip: P_dst[q] += delta[q] for every updated pixel q of the source.
// One block per (list segment, group of 8 channel chunks).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_identity(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    __shared__ int s_base[kSegPixels], s_wy[kSegPixels], s_wx[kSegPixels];
    __shared__ unsigned s_vm[kSegPixels];
    __shared__ int sh[8];
    const int nseg = edge_segments(e);
    const int chunks = e.Cin / VEC;
    const int ch0 = blockIdx.y * 8, nch = chunks - ch0 < 8 ? chunks - ch0 : 8;
    carry_source_compaction(e, sh);
    for (int seg = blockIdx.x; seg < nseg; seg += gridDim.x) {
        __syncthreads();
        const int tot = tile_prologue(e, seg, 0, kSegPixels, blockIdx.y == 0, blockIdx.y == 0, s_base, s_wy, s_wx, s_vm, sh);
        for (int i = threadIdx.x; i < tot * nch; i += 256) {
            const int ent = i / nch;
            const int c0 = (ch0 + i - ent * nch) * VEC;
            // stride 1, pad 0: s_base is the source pixel itself
            T* pp = (T*)e.P + pdst_offset(e, s_wy[ent], s_wx[ent]) + c0;
            const T* d = (const T*)e.delta + (size_t)s_base[ent] * e.Cin + c0;
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
        }
    }
}

// Max pooling in delta form: for every destination view pixel whose window holds an
// updated source pixel, y = max of the source's activations f(A) over the in-view
// pixels of the window; P_dst += y - (newly unveiled ? 0 : previous output); the
// previous output is replaced by y.
template <typename T, int VEC> struct PoolVec {
    static __device__ __forceinline__ void load(const T* p, float* v) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) v[q] = (float)p[q];
    }
    static __device__ __forceinline__ void store(T* p, const float* v) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) p[q] = (T)v[q];
    }
};
template <> struct PoolVec<f16, 8> {
    static __device__ __forceinline__ void load(const f16* p, float* v) {
        const f16x8 t = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = (float)t[q];
    }
    static __device__ __forceinline__ void store(f16* p, const float* v) {
        f16x8 t;
#pragma unroll
        for (int q = 0; q < 8; ++q) t[q] = (f16)v[q];
        *reinterpret_cast<f16x8*>(p) = t;
    }
};
template <> struct PoolVec<float, 4> {
    static __device__ __forceinline__ void load(const float* p, float* v) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    static __device__ __forceinline__ void store(float* p, const float* v) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};

// One block per (list segment, channel chunk): thread t owns entry t of the segment and
// VEC channels; the k*k source rows of its window are independent 16-byte loads.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void k_pool(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    __shared__ int s_base[kSegPixels], s_wy[kSegPixels], s_wx[kSegPixels];
    __shared__ unsigned s_vm[kSegPixels];
    __shared__ int sh[8];
    const int nseg = edge_segments(e);
    const int c0 = blockIdx.y * VEC;
    carry_source_compaction(e, sh);
    for (int seg = blockIdx.x; seg < nseg; seg += gridDim.x) {
        __syncthreads();
        // the destination's flags still hold this frame's N (set by the shift); marking the
        // pixels touched only ORs U in, so the channel chunks may read N at any time
        const int tot = tile_prologue(e, seg, 0, kSegPixels, blockIdx.y == 0, blockIdx.y == 0, s_base, s_wy, s_wx, s_vm, sh);
        const int ent = threadIdx.x;
        if (ent >= tot) continue;
        const int oy = s_wy[ent] - e.by0, ox = s_wx[ent] - e.bx0;              // view pixel of the destination
        float y[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) y[q] = -INFINITY;
        for (int jy = 0; jy < e.k; ++jy)
            for (int jx = 0; jx < e.k; ++jx) {
                const int iy = oy * e.stride - e.pad + jy, ix = ox * e.stride - e.pad + jx;
                if (iy < 0 || iy >= e.sH || ix < 0 || ix >= e.sW) continue;
                const int ay = wrapc(e.s_aoy + iy, e.sH), ax = wrapc(e.s_aox + ix, e.sW);
                float v[VEC];
                PoolVec<T, VEC>::load((const T*)e.sA + ((size_t)ay * e.sW + ax) * e.Cin + c0, v);
#pragma unroll
                for (int q = 0; q < VEC; ++q) y[q] = fmaxf(y[q], e.s_relu ? fmaxf(v[q], 0.f) : v[q]);
            }
        // op == 2: the reset of a pixel zeroed its previous output as well (sites with crops, where a
        // reset pixel may be pooled in a later frame than the reset)
        const bool fresh = e.op == 1 && (e.dflags[oy * e.dW + ox] & kFlagN);
        const int yy = wrapc(e.d_aoy + oy, e.dH), yx = wrapc(e.d_aox + ox, e.dW);
        T* prev = (T*)e.dY + ((size_t)yy * e.dW + yx) * e.Cout + c0;
        T* pp = (T*)e.P + pdst_offset(e, s_wy[ent], s_wx[ent]) + c0;
        float pv[VEC], pd[VEC];
        PoolVec<T, VEC>::load(prev, pv);
        PoolVec<T, VEC>::load(pp, pd);
#pragma unroll
        for (int q = 0; q < VEC; ++q) pd[q] = (float)(T)(pd[q] + (y[q] - (fresh ? 0.f : pv[q])));
        PoolVec<T, VEC>::store(pp, pd);
        PoolVec<T, VEC>::store(prev, y);
    }
}

// ---------------------------------------------------------------------------
// 1x1 convolution into a truncation-free site (no pending ring): for every destination pixel q
// whose source pixel was updated
//   t = round(y[q] (+ bias, if q is newly unveiled));  a = newly unveiled ? 0 : A[q]
//   A[q] <- a + t;  delta[q] <- f(a + t) - f(a);  updated if newly unveiled or any channel of the
//   delta is not zero
// which is what the pending ring and the delta kernel do with threshold 0.  A tile is a quarter of a
// list segment (64 destination pixels, the indices of one wave) and ALL output channels, so the block
// owns its pixels: it writes their flag bytes, also those of the pixels nobody touched - the mask of
// the frame is complete after this launch.  The first quarter also publishes the segment's compute list.
// fp16 with Cin % 16 == 0 and Cout % 32 == 0 runs on the matrix cores (operands straight from global
// memory: the layer is bound by the accumulated values it reads and writes); anything else takes one
// thread per (entry, output channel).
// ---------------------------------------------------------------------------
constexpr int kTfTile = 64;
template <typename T, bool MFMA>
__global__ __launch_bounds__(256) void k_conv_tf(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    __shared__ int s_src[kTfTile], s_dst[kTfTile];
    __shared__ unsigned s_any[kTfTile];
    __shared__ uint8_t s_new[kTfTile];
    __shared__ int sh[8];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = e.dH * e.dW;                             // no border: the window is the view
    const int ntiles = ((n + kSegPixels - 1) / kSegPixels) * (kSegPixels / kTfTile);
    T* __restrict__ A = (T*)e.dY;
    T* __restrict__ D = (T*)const_cast<void*>(e.sA);
    const float* __restrict__ bias = (const float*)e.wp;
    const T* __restrict__ delta = (const T*)e.delta;
    const T* __restrict__ w = (const T*)e.w;
    carry_source_compaction(e, sh);
    long long block_taps = 0;                               // statistics (thread 0 only)
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int seg = tile / (kSegPixels / kTfTile), quarter = tile % (kSegPixels / kTfTile);
        __syncthreads();                                    // previous tile is done with LDS
        const int p = seg * kSegPixels + tid;
        const bool own = wave == quarter;                   // this wave's 64 indices are the tile
        bool has = false;
        int fl = 0, src = 0;
        if (p < n) {
            const int oy = p / e.dW, ox = p - oy * e.dW;
            src = oy * e.stride * e.sW + ox * e.stride;       // k == 1, pad == 0: inside the source view
            has = (e.sflags[src] & kFlagM) != 0;
            if (own) fl = e.dflags[p];
        }
        if (tid < kTfTile) s_any[tid] = 0u;
        const unsigned long long bal = __ballot(has);
        const int rank = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) sh[wave] = __popcll(bal);
        __syncthreads();
        const int tot = sh[quarter];
        if (own && has) {
            s_src[rank] = src;
            s_dst[rank] = p;
            s_new[rank] = (uint8_t)(fl & kFlagN);
        }
        if (quarter == 0) {                                // the segment's compute list, by its first tile
            int off = rank;
            for (int i = 0; i < wave; ++i) off += sh[i];
            if (has) e.clist[seg * kSegPixels + off] = p;
            if (tid == 0) {                                // single writer per segment: no atomics
                const int all = sh[0] + sh[1] + sh[2] + sh[3];
                e.ccnt[seg] = all;
                e.cacc[seg] += (unsigned long long)all;
            }
        }
        if (tid == 0) block_taps += tot;
        __syncthreads();
        if constexpr (MFMA) {
            // (32 entries x 32 couts) tiles dealt to the four waves; lane l feeds entry / cout l % 32 with
            // the 8 consecutive cin starting at 8 * (l / 32); register r of a lane holds cout
            // 8 * (r / 4) + 4 * (l / 32) + r % 4 of the tile for entry l % 32
            const int nra = (tot + 31) >> 5, nca = e.Cout >> 5;
            const int col = lane & 31, kh = lane >> 5;
            for (int u = wave; u < nra * nca; u += 4) {
                const int ra = u / nca, ca = u - ra * nca;
                const int ent = ra * 32 + col;
                const bool act = ent < tot;
                const f16* brow = (const f16*)delta + (size_t)s_src[act ? ent : 0] * e.Cin + kh * 8;
                const f16* arow = (const f16*)w + (size_t)(ca * 32 + col) * e.Cin + kh * 8;
                f32x16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
                int c0 = 0;
                for (; c0 + 64 <= e.Cin; c0 += 64) {           // four steps' operands are requested together
                    f16x8 a4[4], b4[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        a4[q] = *reinterpret_cast<const f16x8*>(arow + c0 + 16 * q);
                        b4[q] = *reinterpret_cast<const f16x8*>(brow + c0 + 16 * q);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a4[q], b4[q], acc, 0, 0, 0);
                }
                for (; c0 < e.Cin; c0 += 16) {
                    const f16x8 a = *reinterpret_cast<const f16x8*>(arow + c0);
                    const f16x8 b = *reinterpret_cast<const f16x8*>(brow + c0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
                }
                if (act) {                                   // (a dead column multiplied entry 0's row: dropped here)
                    const int p1 = s_dst[ent];
                    const int vy = p1 / e.dW, vx = p1 - vy * e.dW;
                    f16* Ap = (f16*)A + ((size_t)wrapc(e.d_aoy + vy, e.dH) * e.dW + wrapc(e.d_aox + vx, e.dW)) * e.Cout + ca * 32 + 4 * kh;
                    f16* Dp = (f16*)D + (size_t)p1 * e.Cout + ca * 32 + 4 * kh;
                    const bool fresh = s_new[ent] != 0;
                    f16x4 av[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g) av[g] = *reinterpret_cast<const f16x4*>(Ap + 8 * g);
                    bool any = false;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        f16x4 na, dv;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float a = fresh ? 0.f : (float)av[g][i];
                            const float b = fresh && bias ? (float)(f16)bias[ca * 32 + 8 * g + 4 * kh + i] : 0.f;
                            const float t = (float)(f16)(b + acc[4 * g + i]);      // as the pending ring would hold it
                            const float sum = a + t;
                            const float out = e.s_relu ? fmaxf(sum, 0.f) - fmaxf(a, 0.f) : sum - a;
                            na[i] = (f16)sum;
                            dv[i] = (f16)out;
                            any |= out != 0.f;
                        }
                        *reinterpret_cast<f16x4*>(Ap + 8 * g) = na;
                        *reinterpret_cast<f16x4*>(Dp + 8 * g) = dv;
                    }
                    if (any) atomicOr(&s_any[ent], 1u);        // an OR: the order does not matter
                }
            }
        } else {
            for (int idx = tid; idx < tot * e.Cout; idx += 256) {
                const int ent = idx / e.Cout, co = idx - ent * e.Cout;
                const T* drow = delta + (size_t)s_src[ent] * e.Cin;
                const T* wrow = w + (size_t)co * e.Cin;
                float y = 0.f;
                for (int ci = 0; ci < e.Cin; ++ci) y = fmaf((float)drow[ci], (float)wrow[ci], y);
                const int p1 = s_dst[ent];
                const int vy = p1 / e.dW, vx = p1 - vy * e.dW;
                const size_t aoff = ((size_t)wrapc(e.d_aoy + vy, e.dH) * e.dW + wrapc(e.d_aox + vx, e.dW)) * e.Cout + co;
                const bool fresh = s_new[ent] != 0;
                const float a = fresh ? 0.f : (float)A[aoff];
                const float b = fresh && bias ? (float)(T)bias[co] : 0.f;
                const float t = (float)(T)(b + y);          // as the pending ring would hold it
                const float sum = a + t;
                const float out = e.s_relu ? fmaxf(sum, 0.f) - fmaxf(a, 0.f) : sum - a;
                A[aoff] = (T)sum;
                D[(size_t)p1 * e.Cout + co] = (T)out;
                if (out != 0.f) atomicOr(&s_any[ent], 1u);     // an OR: the order does not matter
            }
        }
        __syncthreads();
        if (own && p < n) e.dflags[p] = (uint8_t)(has ? ((((fl & kFlagN) || s_any[rank]) ? kFlagM : 0) | kFlagC) : 0);
    }
    if (tid == 0) add_macs(e, block_taps, MFMA ? 0 : 1);    // statistics: one atomic per block
}

// Compaction of the update mask alone (a forward call without outgoing edges).
__global__ __launch_bounds__(256) void k_compact_source(EdgeBatch eb) {
    const EdgeDev& e = eb.d[blockIdx.z];                  // blockIdx.z: stream of the batch
    __shared__ int sh[8];
    carry_source_compaction(e, sh);
}

static unsigned cap_blocks(long long b, long long cap) {
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (unsigned)b;
}

// Tuning knobs (mdcnn_set_option): forced tile shape, pipeline depth, XCD mapping.
int g_tile = 0, g_pipe = 0, g_xcd = 1, g_kc = 0;
int g_f32_mfma = 1;     // 1: fp32 layers go to the matrix cores where k_conv_mfma_f32 applies, 0: plain FMA kernels

template <int WM, int WN, int TM, int TN, int KC, int PIPE>
static hipError_t launch_tiled(const EdgeBatch& eb, int nb, long long max_entries, hipStream_t st) {
    const EdgeDev& e = eb.d[0];
    using Cfg = TiledCfg<WM, WN, TM, TN, KC, PIPE>;
    auto kern = k_conv_mfma_tiled<WM, WN, TM, TN, KC, PIPE>;
    // launches come from several host threads (frames in flight): the attribute is set once, by whoever is first
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::SMEM);
        if (err != hipSuccess) { (void)hipGetLastError(); return err; }    // do not leave it for the next call to report
        attr_set.store(true, std::memory_order_release);
    }
    const long long nseg = (max_entries + kSegPixels - 1) / kSegPixels;
    const long long MT = nseg * Cfg::TPS;
    const int NT = e.Cout / Cfg::BN;
    const int xcd = g_xcd && NT <= 8 && (8 % NT) == 0;
    const long long items = xcd ? 8 * ((MT + 8 / NT - 1) / (8 / NT)) : MT * NT;
    unsigned g = cap_blocks(items, 4096);
    g = (g + 7u) & ~7u;                                    // whole rounds over the 8 XCDs
    kern<<<dim3(g, 1, nb), dim3(256), Cfg::SMEM, st>>>(eb, NT, (int)items, xcd);
    return hipGetLastError();
}

template <int WM, int WN, int TM, int TN, int KC>
static hipError_t launch_tiled_p(const EdgeBatch& eb, int nb, long long max_entries, hipStream_t st) {
    const EdgeDev& e = eb.d[0];
    // measured on MI355X: with L2 latencies of ~200 cycles one step of prefetch is
    // enough; the second register stage only costs occupancy
    const bool deep = g_pipe == 2 && TiledCfg<WM, WN, TM, TN, KC, 2>::SMEM <= 150 * 1024;   // two stages must fit the LDS
    return deep ? launch_tiled<WM, WN, TM, TN, KC, 2>(eb, nb, max_entries, st)
                : launch_tiled<WM, WN, TM, TN, KC, 1>(eb, nb, max_entries, st);
}

template <int KC>
static hipError_t launch_tiled_kc(const EdgeBatch& eb, int nb, long long max_entries, hipStream_t st) {
    const EdgeDev& e = eb.d[0];
    auto blocks = [&](int bm, int bn) { return ((max_entries + bm - 1) / bm) * (e.Cout / bn); };
    int tile = g_tile;
    if (tile == 0) {
        // the largest tile that still yields about one block per compute unit
        const long long want = 224;
        if (e.Cout % 128 == 0 && blocks(128, 128) >= want) tile = 4;
        else if (e.Cout % 128 == 0 && blocks(64, 128) >= want) tile = 5;
        else if (e.Cout % 64 == 0) tile = blocks(256, 64) >= want ? 1 : blocks(128, 64) >= want ? 2 : 3;
        else tile = 6;
    }
    switch (tile) {
        case 1: if (e.Cout % 64 == 0) return launch_tiled_p<4, 1, 2, 2, KC>(eb, nb, max_entries, st); break;    // 256 x 64
        case 2: if (e.Cout % 64 == 0) return launch_tiled_p<2, 2, 2, 1, KC>(eb, nb, max_entries, st); break;    // 128 x 64
        case 3: if (e.Cout % 64 == 0) return launch_tiled_p<2, 2, 1, 1, KC>(eb, nb, max_entries, st); break;    //  64 x 64
        case 4: if (e.Cout % 128 == 0) return launch_tiled_p<2, 2, 2, 2, KC>(eb, nb, max_entries, st); break;   // 128 x 128
        case 5: if (e.Cout % 128 == 0) return launch_tiled_p<2, 2, 1, 2, KC>(eb, nb, max_entries, st); break;   //  64 x 128
        case 7: if (e.Cout % 128 == 0) return launch_tiled_p<4, 1, 1, 4, KC>(eb, nb, max_entries, st); break;   // 128 x 128, wave 32 x 128
        case 8: if (e.Cout % 256 == 0) return launch_tiled_p<2, 2, 2, 4, KC>(eb, nb, max_entries, st); break;   // 128 x 256, wave 64 x 128
        case 9: if (e.Cout % 256 == 0) return launch_tiled_p<1, 4, 2, 2, KC>(eb, nb, max_entries, st); break;   //  64 x 256, wave 64 x 64
        case 10: if (e.Cout % 256 == 0) return launch_tiled_p<2, 2, 1, 4, KC>(eb, nb, max_entries, st); break;  //  64 x 256, wave 32 x 128
        case 11: if (e.Cout % 128 == 0) return launch_tiled_p<1, 4, 1, 1, KC>(eb, nb, max_entries, st); break;  //  32 x 128
        case 12: if (e.Cout % 256 == 0) return launch_tiled_p<1, 4, 1, 2, KC>(eb, nb, max_entries, st); break;  //  32 x 256
        case 13: if (e.Cout % 128 == 0) return launch_tiled_p<1, 4, 2, 1, KC>(eb, nb, max_entries, st); break;  //  64 x 128, wave 64 x 32
        case 14: if (e.Cout % 64 == 0) return launch_tiled_p<1, 4, 2, 1, 32>(eb, nb, max_entries, st); break;   //  same, 32-channel steps
        default: break;
    }
    return launch_tiled_p<4, 1, 1, 1, KC>(eb, nb, max_entries, st);                                             // 128 x 32
}

int g_halo = 1;          // 0: never use the halo-staged kernel, 2: force 32-cout tiles, 3: tiles are index ranges only,
                         // 4: rectangular tiles whatever the size of the window
int g_halo_sub = 0;      // 0: auto, 1 / 2 / 4: tiles per list segment of the halo-staged kernel

template <int NSUB, int WMV, int WK, int TM, int TN, int KC, int NLD, int RING = 3, int MINB = (NSUB >= 2 ? 2 : 1), bool T2D = false>
static hipError_t launch_halo_t(const EdgeBatch& eb, int nb, long long nseg, hipStream_t st, int th = 0, int tw = 0) {
    const EdgeDev& e = eb.d[0];
    using Cfg = HaloCfg<NSUB, WMV, WK, TM, TN, KC, NLD, 3, RING, MINB>;
    auto kern = k_conv_halo<NSUB, WMV, WK, TM, TN, KC, NLD, 3, RING, MINB, T2D>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::SMEM);
        if (err != hipSuccess) { (void)hipGetLastError(); return err; }    // do not leave it for the next call to report
        attr_set.store(true, std::memory_order_release);
    }
    const int NT = e.Cout / Cfg::BN;
    const long long tiles = T2D ? (long long)((e.Hp + th - 1) / th) * ((e.Wp + tw - 1) / tw) : nseg * NSUB;
    const long long items = tiles * NT;
    kern<<<dim3(cap_blocks(items, 16384), 1, nb), dim3(256), Cfg::SMEM, st>>>(eb, NT, (int)items, th, tw);
    return hipGetLastError();
}

// Rectangle th x tw of at most `sub` pixels whose halo fits `cap` staged pixels, with the fewest tiles over an Hp x Wp window
// (ties: the smaller halo).  False if none fits.
bool tile_2d(int Hp, int Wp, int k, int sub, int cap, int* th_out, int* tw_out, long long* tiles_out) {
    long long best = -1, best_halo = 0;
    for (int th = 1; th <= sub && th <= Hp; ++th) {
        int tw = sub / th < Wp ? sub / th : Wp;
        while (tw > 1 && (long long)(th + k - 1) * (tw + k - 1) > cap) --tw;
        if ((long long)(th + k - 1) * (tw + k - 1) > cap) continue;
        // the narrowest tile with the same number of columns of tiles
        const int cols = (Wp + tw - 1) / tw;
        tw = (Wp + cols - 1) / cols;
        const long long tiles = (long long)((Hp + th - 1) / th) * cols, halo = (long long)(th + k - 1) * (tw + k - 1);
        if (best < 0 || tiles < best || (tiles == best && halo < best_halo)) { best = tiles; best_halo = halo; *th_out = th; *tw_out = tw; }
    }
    if (best < 0) return false;
    *tiles_out = best;
    return true;
}

// Rectangular tiles.  The tile size follows the number of tiles of ONE stream, whatever the batch - the K split of a
// tile fixes the order of the sums, and a stream in a batch must give the bits it gives alone: whole segments if that
// gives every compute unit a tile, else the smallest split that gives half of them one.  A whole-segment tile keeps its
// four waves on rows (no K split: 64 accumulator registers, two tiles per compute unit); it is what the 64-channel
// layers with rows wider than a segment use.  With many streams to a launch whole segments are the faster choice
// everywhere (ResNet-18-style network, 16 videos: 4.1 k frames/s against 3.9 k; one video: 3.5 k against 3.7 k): a caller
// who serves batches sets MDCNN_OPT_CONV_HALO_SUB to 1.  128-channel chunks (half the chunk boundaries) were measured
// too: no faster alone or in a batch, so chunks stay at 64 channels.
template <int TN>
static hipError_t launch_halo_2d(const EdgeBatch& eb, int nb, hipStream_t st, bool* done) {
    const EdgeDev& e = eb.d[0];
    const int NT = e.Cout / (32 * TN);
    const bool c64 = e.Cin % 64 == 0, c32 = e.Cin % 32 == 0;
    int th = 0, tw = 0;
    long long tiles = 0;
    *done = true;
    const int first = g_halo_sub ? g_halo_sub : 1;
    for (int nsub = first; nsub <= 4; nsub *= 2) {
        const int sub = kSegPixels / nsub;
        // whole segments if every compute unit gets a tile, else the smallest split that gives at least half of them one
        // (a forced split is taken as it is)
        if (!g_halo_sub && nsub < 4 && tile_2d(e.Hp, e.Wp, e.k, sub, 1 << 20, &th, &tw, &tiles) && tiles * NT < (nsub == 1 ? 256 : 128)) continue;
        if (nsub == 1) {
            if (c64 && tile_2d(e.Hp, e.Wp, e.k, sub, HaloCfg<1, 4, 1, 2, TN, 64, 11, 3>::CAP, &th, &tw, &tiles))
                return launch_halo_t<1, 4, 1, 2, TN, 64, 11, 6, 2, true>(eb, nb, 0, st, th, tw);
            if (c32 && tile_2d(e.Hp, e.Wp, e.k, sub, HaloCfg<1, 4, 1, 2, TN, 32, 6, 3>::CAP, &th, &tw, &tiles))
                return launch_halo_t<1, 4, 1, 2, TN, 32, 6, 3, 2, true>(eb, nb, 0, st, th, tw);
        } else if (nsub == 2) {
            if (c64 && tile_2d(e.Hp, e.Wp, e.k, sub, HaloCfg<2, 2, 2, 2, TN, 64, 6, 3>::CAP, &th, &tw, &tiles))
                return launch_halo_t<2, 2, 2, 2, TN, 64, 6, 6, 2, true>(eb, nb, 0, st, th, tw);
            if (c32 && tile_2d(e.Hp, e.Wp, e.k, sub, HaloCfg<2, 2, 2, 2, TN, 32, 3, 3>::CAP, &th, &tw, &tiles))
                return launch_halo_t<2, 2, 2, 2, TN, 32, 3, 3, 2, true>(eb, nb, 0, st, th, tw);
        } else {
            if (c64 && tile_2d(e.Hp, e.Wp, e.k, sub, HaloCfg<4, 1, 4, 2, TN, 64, 4, 3>::CAP, &th, &tw, &tiles))
                return launch_halo_t<4, 1, 4, 2, TN, 64, 4, 9, 2, true>(eb, nb, 0, st, th, tw);
            if (c32 && tile_2d(e.Hp, e.Wp, e.k, sub, HaloCfg<4, 2, 2, 1, TN, 32, 2, 3>::CAP, &th, &tw, &tiles))
                return launch_halo_t<4, 2, 2, 1, TN, 32, 2, 9, 2, true>(eb, nb, 0, st, th, tw);
        }
    }
    *done = false;
    return hipSuccess;
}

// Staged pixels the rectangle of `sub` consecutive window indices can need.
static long long halo_worst(const EdgeDev& e, int sub) {
    const long long span = (sub - 2) / e.Wp + 2;                            // window rows the range can straddle
    const long long width = span > 1 || sub > e.Wp ? e.Wp : sub;
    return (span + e.k - 1) * (width - 1 + e.k);
}

// Halo-staged kernel if the rectangle a tile can read fits the staging buffer
// (the fewer channels per chunk, the more pixels fit; below 32 channels per chunk
// -- rows wider than about 250 pixels -- the tiled kernel is faster).
// *done = false: not applicable.
// Tiles are whole segments, halves or quarters: the smallest split that keeps at
// least half of the compute units busy (measured: finer splits re-read the weights
// more often than the extra parallelism pays back).
template <int TN>
static hipError_t launch_halo_n(const EdgeBatch& eb, int nb, long long nseg, hipStream_t st, bool* done) {
    const EdgeDev& e = eb.d[0];
    const long long per_split = nseg * (e.Cout / (32 * TN));
    int nsub = g_halo_sub ? g_halo_sub : (per_split >= 256 ? 1 : per_split * 2 >= 128 ? 2 : 4);
    *done = true;
    for (; nsub <= 4; nsub *= 2) {
        const long long worst = halo_worst(e, kSegPixels / nsub);
        const bool c64 = e.Cin % 64 == 0, c32 = e.Cin % 32 == 0;
        if (nsub == 1) {
            if (c64 && worst <= HaloCfg<1, 2, 2, 4, TN, 64, 16, 3>::CAP) return launch_halo_t<1, 2, 2, 4, TN, 64, 16>(eb, nb, nseg, st);
            if (c32 && worst <= HaloCfg<1, 2, 2, 4, TN, 32, 12, 3>::CAP) return launch_halo_t<1, 2, 2, 4, TN, 32, 12>(eb, nb, nseg, st);
        } else if (nsub == 2) {
            if (c64 && worst <= HaloCfg<2, 2, 2, 2, TN, 64, 11, 3>::CAP) return launch_halo_t<2, 2, 2, 2, TN, 64, 11, 6>(eb, nb, nseg, st);
            if (c32 && worst <= HaloCfg<2, 2, 2, 2, TN, 32, 9, 3>::CAP) return launch_halo_t<2, 2, 2, 2, TN, 32, 9>(eb, nb, nseg, st);
        } else {
            if (c64 && worst <= HaloCfg<4, 1, 4, 2, TN, 64, 9, 3>::CAP) return launch_halo_t<4, 1, 4, 2, TN, 64, 9, 9>(eb, nb, nseg, st);
            if (c32 && worst <= HaloCfg<4, 2, 2, 1, TN, 32, 6, 3>::CAP) return launch_halo_t<4, 2, 2, 1, TN, 32, 6, 9>(eb, nb, nseg, st);
        }
    }
    *done = false;
    return hipSuccess;
}

static hipError_t launch_halo(const EdgeBatch& eb, int nb, long long nseg, hipStream_t st, bool* done) {
    const EdgeDev& e = eb.d[0];
    *done = false;
    if (!g_halo || !e.wp || e.k != 3 || e.stride != 1 || e.up != 0 || e.Cin % 16 || e.Cout % 32) return hipSuccess;
    if ((long long)e.sH * e.sW * e.Cin >= (1ll << 30) || (long long)e.k * e.k * e.Cin * e.Cout >= (1ll << 30))
        return hipSuccess;                                                     // 32-bit byte offsets into deltas and weights
    // rectangular tiles where they fit; windows of a few list segments stay on index ranges (measured on the HRNet-like
    // network, whose lower branches have 50 x 38 pixels and less: 15.5 against 16.3 us per launch - a tile's by-products are
    // stored at its end there, which a launch of a few blocks has nothing to hide behind)
    if (g_halo != 3 && ((long long)e.Hp * e.Wp >= 4096 || g_halo == 4)) {
        const hipError_t err = e.Cout % 64 == 0 && g_halo != 2 ? launch_halo_2d<2>(eb, nb, st, done) : launch_halo_2d<1>(eb, nb, st, done);
        if (err != hipSuccess || *done) return err;
    }
    return e.Cout % 64 == 0 && g_halo != 2 ? launch_halo_n<2>(eb, nb, nseg, st, done) : launch_halo_n<1>(eb, nb, nseg, st, done);
}

hipError_t launch_pack_weights(const void* src, void* dst, int taps, int Cout, int Cin, hipStream_t st) {
    const long long n8 = (long long)taps * Cout * Cin / 8;
    k_pack_weights<<<dim3(cap_blocks((n8 + 255) / 256, 2048)), dim3(256), 0, st>>>((const f16*)src, (f16*)dst, taps, Cout, Cin);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_ldsw(const EdgeBatch& eb, int nb, long long max_entries, hipStream_t st) {
    const EdgeDev& e = eb.d[0];
    const int groups = e.Cout / 8, ppb = 256 / groups;
    const size_t smem = (size_t)e.k * e.k * e.Cin * e.Cout * 4;
    auto kern = k_conv_ldsw<T>;
    if (smem > 65536) {
        // the limit only grows; the lock keeps two host threads from lowering it under each other
        static std::mutex mu;
        static size_t attr_bytes = 0;
        std::lock_guard<std::mutex> lock(mu);
        if (smem > attr_bytes) {
            hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (err != hipSuccess) return err;
            attr_bytes = smem;
        }
    }
    const long long nseg = (max_entries + kSegPixels - 1) / kSegPixels;
    const long long tps = (kSegPixels + ppb - 1) / ppb;
    // weights are staged once per block: keep the blocks few and persistent
    unsigned g = cap_blocks(nseg * tps, smem > 32768 ? 256 : 768);
    kern<<<dim3(g, 1, nb), dim3(256), smem, st>>>(eb, groups, ppb);
    return hipGetLastError();
}

// fp32 layers the matrix cores take (k_conv_mfma_f32); *done = false: not this layer
template <int KK, int CIN, int KS>
static hipError_t launch_mfma_f32_inst(const EdgeBatch& eb, int nb, long long nseg, hipStream_t st) {
    const EdgeDev& e = eb.d[0];
    static std::atomic<bool> attr_set{false};
    auto kern = k_conv_mfma_f32<KK, CIN, KS>;
    const size_t smem = (size_t)KK * KK * CIN * 32 * 4;
    if (smem > 49152 && !attr_set.load(std::memory_order_acquire)) {
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (err != hipSuccess) return err;
        attr_set.store(true, std::memory_order_release);
    }
    const int nts = (e.Cout + 31) / 32;
    const long long tiles = nseg * (kSegPixels / (32 * (4 / KS)));
    // weights are staged once per block: a bounded number of persistent blocks
    const long long cap = (smem > 49152 ? 512 : 1024) / nts;
    const unsigned g = cap_blocks(tiles, cap > 0 ? cap : 1);
    kern<<<dim3(g, nts, nb), dim3(256), smem, st>>>(eb);
    return hipGetLastError();
}
template <int KK, int CIN>
static hipError_t launch_mfma_f32_ks(const EdgeBatch& eb, int nb, long long nseg, hipStream_t st) {
    const EdgeDev& e = eb.d[0];
    if constexpr (KK == 1) {
        return launch_mfma_f32_inst<KK, CIN, 1>(eb, nb, nseg, st);
    } else {
        // two waves share the taps of a 64-entry tile unless 128-entry tiles already give every compute unit four
        // blocks (config 2, 66 and 17 segments: 10.5 k frames/s with one wave per tile, 11.7 k with two, 10.4 k with four)
        const long long nts = (e.Cout + 31) / 32;
        int ks = nseg * 2 * nts >= 1024 ? 1 : 2;
        if (g_tile == 1 || g_tile == 2 || g_tile == 4) ks = g_tile;
        if (ks == 1) return launch_mfma_f32_inst<KK, CIN, 1>(eb, nb, nseg, st);
        if (ks == 2) return launch_mfma_f32_inst<KK, CIN, 2>(eb, nb, nseg, st);
        return launch_mfma_f32_inst<KK, CIN, 4>(eb, nb, nseg, st);
    }
}
static hipError_t launch_mfma_f32(const EdgeBatch& eb, int nb, long long nseg, hipStream_t st, bool* done) {
    const EdgeDev& e = eb.d[0];
    *done = false;
    if (e.up || (e.k != 1 && e.k != 3) || (e.Cin != 16 && e.Cin != 32 && e.Cin != 64) || (e.Cout % 32 != 0 && e.Cout != 16) || e.Cout > 1024 ||
        (long long)e.sH * e.sW * e.Cin >= (1ll << 29) || (long long)e.k * e.k * e.Cin * e.Cout >= (1ll << 29))
        return hipSuccess;
    *done = true;
    if (e.k == 3)
        return e.Cin == 16 ? launch_mfma_f32_ks<3, 16>(eb, nb, nseg, st)
             : e.Cin == 32 ? launch_mfma_f32_ks<3, 32>(eb, nb, nseg, st) : launch_mfma_f32_ks<3, 64>(eb, nb, nseg, st);
    return e.Cin == 16 ? launch_mfma_f32_ks<1, 16>(eb, nb, nseg, st)
         : e.Cin == 32 ? launch_mfma_f32_ks<1, 32>(eb, nb, nseg, st) : launch_mfma_f32_ks<1, 64>(eb, nb, nseg, st);
}

hipError_t launch_conv(const EdgeBatch& eb, int nb, int dtype, int conv_path, hipStream_t st, int* cls) {
    const EdgeDev& e = eb.d[0];                            // geometry and weights layout are the same for all streams
    const long long max_entries = e.up ? (long long)e.sH * e.sW : (long long)e.Hp * e.Wp;
    const long long nseg = (max_entries + kSegPixels - 1) / kSegPixels;
    if (e.k < 0) {                                         // no operator: source compaction only
        *cls = kClsLists;
        k_compact_source<<<dim3(cap_blocks(((long long)e.sH * e.sW + kSegPixels - 1) / kSegPixels, 4096), 1, nb), dim3(256), 0, st>>>(eb);
        return hipGetLastError();
    }
    if (e.op == kOpTruncFree) {
        const bool mfma = dtype == MDCNN_F16 && conv_path != 1 && e.Cin % 16 == 0 && e.Cout % 32 == 0;
        *cls = mfma ? kClsConvMfma : kClsConvPlain;
        const unsigned g = cap_blocks((((long long)e.dH * e.dW + kSegPixels - 1) / kSegPixels) * (kSegPixels / kTfTile), 8192);
        if (mfma) k_conv_tf<f16, true><<<dim3(g, 1, nb), dim3(256), 0, st>>>(eb);
        else if (dtype == MDCNN_F16) k_conv_tf<f16, false><<<dim3(g, 1, nb), dim3(256), 0, st>>>(eb);
        else k_conv_tf<float, false><<<dim3(g, 1, nb), dim3(256), 0, st>>>(eb);
        return hipGetLastError();
    }
    if (e.op) {
        *cls = kClsPool;
        const unsigned g = cap_blocks(nseg, 4096);
        if (dtype == MDCNN_F16) {
            if (e.Cin % 8 == 0) k_pool<f16, 8><<<dim3(g, e.Cin / 8, nb), dim3(256), 0, st>>>(eb);
            else k_pool<f16, 1><<<dim3(g, e.Cin, nb), dim3(256), 0, st>>>(eb);
        } else {
            if (e.Cin % 4 == 0) k_pool<float, 4><<<dim3(g, e.Cin / 4, nb), dim3(256), 0, st>>>(eb);
            else k_pool<float, 1><<<dim3(g, e.Cin, nb), dim3(256), 0, st>>>(eb);
        }
        return hipGetLastError();
    }
    if (e.k == 0) {
        *cls = kClsIdentity;
        const unsigned g = cap_blocks(nseg, 4096);
        if (dtype == MDCNN_F16) {
            if (e.Cin % 8 == 0) k_identity<f16, 8><<<dim3(g, (e.Cin / 8 + 7) / 8, nb), dim3(256), 0, st>>>(eb);
            else k_identity<f16, 1><<<dim3(g, (e.Cin + 7) / 8, nb), dim3(256), 0, st>>>(eb);
        } else {
            if (e.Cin % 4 == 0) k_identity<float, 4><<<dim3(g, (e.Cin / 4 + 7) / 8, nb), dim3(256), 0, st>>>(eb);
            else k_identity<float, 1><<<dim3(g, (e.Cin + 7) / 8, nb), dim3(256), 0, st>>>(eb);
        }
        return hipGetLastError();
    }
    // conv_path: 0 auto, 1 plain FMA (per-thread weights), 2 MFMA without LDS tiling, 3 auto without halo staging
    const bool mfma_ok = dtype == MDCNN_F16 && conv_path != 1 && e.Cin % 16 == 0 && e.Cout % 32 == 0;
    if (mfma_ok && conv_path == 0) {
        bool done = false;
        const hipError_t err = launch_halo(eb, nb, nseg, st, &done);
        if (done) { *cls = kClsConvMfma; return err; }
    }
    // (the tiled kernel addresses deltas and weights with 32-bit byte offsets)
    const bool small32 = (long long)e.sH * e.sW * e.Cin < (1ll << 30) && (long long)e.k * e.k * e.Cin * e.Cout < (1ll << 30);
    if (mfma_ok && (conv_path == 0 || conv_path == 3) && e.Cin % 32 == 0 && small32) {
        *cls = kClsConvMfma;
        if (e.Cin % 128 == 0 && g_kc != 64) return launch_tiled_kc<128>(eb, nb, max_entries, st);
        return e.Cin % 64 == 0 ? launch_tiled_kc<64>(eb, nb, max_entries, st) : launch_tiled_kc<32>(eb, nb, max_entries, st);
    }
    if (mfma_ok) {
        *cls = kClsConvMfma;
        if (e.Cout % 64 == 0)
            k_conv_mfma_f16<2><<<dim3(cap_blocks(nseg * (kSegPixels / 64), 4096), e.Cout / 64, nb), dim3(256), 0, st>>>(eb);
        else
            k_conv_mfma_f16<1><<<dim3(cap_blocks(nseg * (kSegPixels / 128), 4096), e.Cout / 32, nb), dim3(256), 0, st>>>(eb);
        return hipGetLastError();
    }
    if (dtype == MDCNN_F32 && (conv_path == 0 || conv_path == 3) && g_f32_mfma) {
        bool done = false;
        const hipError_t err = launch_mfma_f32(eb, nb, nseg, st, &done);
        if (done) { *cls = kClsConvMfma; return err; }
    }
    if ((conv_path == 0 || conv_path == 3) && g_f32_mfma && e.k == 3 && e.Cin == 3 && e.Cout % 32 == 0 && e.Cout <= 1024 && !e.up &&
        (long long)e.sH * e.sW * 3 < (1ll << 29)) {
        *cls = kClsConvMfma;
        const unsigned g = cap_blocks(nseg * (kSegPixels / 128), 2048);
        if (dtype == MDCNN_F16) k_conv_stem_mfma<f16><<<dim3(g, e.Cout / 32, nb), dim3(256), 0, st>>>(eb);
        else k_conv_stem_mfma<float><<<dim3(g, e.Cout / 32, nb), dim3(256), 0, st>>>(eb);
        return hipGetLastError();
    }
    *cls = kClsConvPlain;
    if ((conv_path == 0 || conv_path == 3) && e.k == 3 && e.Cin == 3 && e.Cout % 32 == 0 && e.Cout <= 256) {
        const int groups = e.Cout / 32, ppb = 256 / groups;
        const size_t smem = (size_t)27 * e.Cout * 4;
        const long long tps = (kSegPixels + ppb - 1) / ppb;
        const unsigned g = cap_blocks(nseg * tps, 2048);
        if (dtype == MDCNN_F16) k_conv_small<f16, 3, 3, 32><<<dim3(g, 1, nb), dim3(256), smem, st>>>(eb, groups, ppb);
        else k_conv_small<float, 3, 3, 32><<<dim3(g, 1, nb), dim3(256), smem, st>>>(eb, groups, ppb);
        return hipGetLastError();
    }
    const int groups = e.Cout / 8;
    if ((conv_path == 0 || conv_path == 3) && e.Cout % 8 == 0 && groups <= 64 && (size_t)e.k * e.k * e.Cin * e.Cout * 4 <= 150 * 1024)
        return dtype == MDCNN_F16 ? launch_ldsw<f16>(eb, nb, max_entries, st) : launch_ldsw<float>(eb, nb, max_entries, st);
    unsigned g = cap_blocks(nseg * (kSegPixels / 16), 8192);
    if (dtype == MDCNN_F16) k_conv_plain<f16><<<dim3(g, 1, nb), dim3(256), 0, st>>>(eb);
    else k_conv_plain<float><<<dim3(g, 1, nb), dim3(256), 0, st>>>(eb);
    return hipGetLastError();
}

}  // namespace mdcnn

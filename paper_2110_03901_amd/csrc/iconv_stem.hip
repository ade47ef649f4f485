// Low-channel first layers (C = 4 in memory, e.g. RGB padded to four channels): the merged-tap
// kernel.  With so few channels one tap would fill an eighth of an MFMA K slice, so, as in the
// paper's multi-tile computation (section 4.3: compute several taps of a filter row at once
// when C is small; exact by associativity), one K step covers a whole filter ROW: for dilation
// 1 the S taps x 4 channels of output pixel (p, q) and filter row r are one contiguous run of
// the NHWC input, pixels (p*stride + r - pad, q*stride - pad .. + S - 1).  The run is widened to
// eight pixels = 32 K elements (two 32x32x16 MFMAs): a leading pixel when the padding is odd, so
// that the run starts on an even pixel and stays 16-byte aligned in LDS, and trailing pixels up
// to eight.  Those extra positions carry zero weights and are zeroed on the input side as well.
//
// All weights of 64 filters stay in LDS for the whole (persistent) workgroup, which walks through a
// contiguous range of TH x TW output blocks.  One loader wave brings the next block's input patch
// into the other of two patch buffers while four compute waves run the current block's MFMAs and
// store it; the only synchronisation is one barrier per block.  The layer is bound by the write
// of y, which the epilogue issues as 16-byte stores.
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

struct StemGeom {
    int TH, TW_LOG2;     // output block: TH rows, TW = 1 << TW_LOG2 (16 or 32) columns
    int PH, PPAIRS;      // patch rows, 16-byte pixel pairs per patch row
    int tiles_h, tiles_w, tiles_n;
    int total_tiles, tiles_per_wg;
    int shift;           // 1 when pad is odd: the 8-pixel run starts one pixel left of tap 0
    int b_bytes;         // LDS bytes of the weights (R * 4 KiB)
    int patch_bytes;     // LDS bytes of one patch buffer (whole wave-wide loads)
    float inv_ppairs;    // 1 / PPAIRS
};

constexpr int kStemBN = 64;
constexpr int kStemWaves = 4;        // compute waves; one more wave loads the patches

struct StemTile {
    int n, p0, q0, k0;
};

__device__ __forceinline__ StemTile stem_decode(int t, const StemGeom& g) {
    StemTile c;
    const int tile_n = t % g.tiles_n; t /= g.tiles_n;
    const int tile_w = t % g.tiles_w; t /= g.tiles_w;
    const int tile_h = t % g.tiles_h;
    c.n = t / g.tiles_h;
    c.p0 = tile_h * g.TH; c.q0 = tile_w << g.TW_LOG2; c.k0 = tile_n * kStemBN;
    return c;
}

template <typename T, typename TO, int MI>
__global__ void __launch_bounds__((kStemWaves + 1) * 64)
stem_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const StemGeom g) {
    typedef typename Elem<T>::frag frag_t;
    // [weights: (r, k-chunk 0..3, filter 0..63) x 16 B][patch 0][patch 1], a patch = (row, pixel pair) x 16 B
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int TW = 1 << g.TW_LOG2;

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int t_begin = wg * g.tiles_per_wg;
    const int t_end = min(t_begin + g.tiles_per_wg, g.total_tiles);
    // All tiles of a workgroup's range must use the same filters for the resident weights to be
    // valid: the host only makes ranges that do (tiles_n == 1), or ranges of one tile.
    const int k0 = stem_decode(t_begin, g).k0;

    // ---- weights, once: w[k][r][s][0..3] (8 bytes) -> slot (s + shift) of filter row r: 16-byte
    // chunk (s + shift)/2, half (s + shift)%2; the other slots are zero.  Chunk-major so that the
    // 32 lanes of an operand read touch consecutive 16-byte words.
    {
        const uint2* w8 = reinterpret_cast<const uint2*>(w);
        uint2* b8 = reinterpret_cast<uint2*>(lds);
        const int items = kStemBN * s.R * 8;
        for (int it = tid; it < items; it += (kStemWaves + 1) * 64) {
            const int k = it & (kStemBN - 1);     // filter fastest: neighbouring lanes write neighbouring words
            const int rj = it / kStemBN;
            const int j = rj & 7, r = rj >> 3;    // slot within the 8-pixel run, filter row
            const int ss = j - g.shift;
            uint2 v = {0u, 0u};
            if (ss >= 0 && ss < s.S && k0 + k < s.K) v = w8[((size_t)(k0 + k) * s.R + r) * s.S + ss];
            b8[(((r * 4 + (j >> 1)) * kStemBN + k) << 1) + (j & 1)] = v;
        }
    }

    if (wave == kStemWaves) {
        // =========================== loader wave ============================================
        // One 16-byte pixel pair per lane.  A pair never straddles the image edge (W and the patch
        // origin column are even), so a pair is either loaded whole or zero.
        const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * 8u;
        const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
        const uint32_t patch_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds + (uint32_t)g.b_bytes;
        const int npairs = g.PH * g.PPAIRS;
        auto load_patch = [&](int tile, int buf) {
            const StemTile tc = stem_decode(tile, g);
            const int h_org = tc.p0 * s.stride - s.pad;                 // input row of patch row 0
            const int w_org = tc.q0 * s.stride - s.pad - g.shift;       // input column of patch column 0 (even)
            for (int blk = 0; blk * 64 < npairs; ++blk) {
                const int pi = blk * 64 + lane;
                const int ph = (int)(((float)pi + 0.5f) * g.inv_ppairs);
                const int pj = pi - ph * g.PPAIRS;
                const int h = h_org + ph, ww = w_org + 2 * pj;
                const bool ok = (pi < npairs) & ((unsigned)h < (unsigned)s.H) & ((unsigned)ww < (unsigned)s.W);
                const uint32_t off = (uint32_t)((tc.n * s.H + h) * s.W + ww) * 8u;
                dma16(x_rsrc, ok ? off : x_bytes, patch_base + (uint32_t)(buf * g.patch_bytes + blk * 1024));
            }
        };
        load_patch(t_begin, 0);
        wait_vmcnt<0>();
        __syncthreads();                        // weights and patch 0 are in LDS
        for (int tile = t_begin; tile < t_end; ++tile) {
            // the buffer of tile+1 was last read for tile-1, which every compute wave finished
            // before the barrier just passed
            if (tile + 1 < t_end) load_patch(tile + 1, (tile + 1 - t_begin) & 1);
            wait_vmcnt<0>();
            __syncthreads();
        }
        return;
    }

    // =============================== compute waves ==============================================
    const int frow = lane & 31, fk = lane >> 5;
    const int npx = g.TH * TW;
    int a_idx[MI], o_th[MI], o_tw[MI];            // pixel-pair index of the lane's run at filter row 0; block row/column
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int t = (wave * MI + mi) * 32 + frow;
        const int th = t >> g.TW_LOG2, tw = t & (TW - 1);
        a_idx[mi] = t < npx ? th * s.stride * g.PPAIRS + tw * (s.stride >> 1) + fk : fk;
        o_th[mi] = t < npx ? th : (1 << 20);
        o_tw[mi] = tw;
    }
    // which of the lane's two pixels per K slice are padding positions of the run
    bool zero_lo[2], zero_hi[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int j = 4 * kk + 2 * fk;
        zero_lo[kk] = j < g.shift || j >= s.S + g.shift;
        zero_hi[kk] = (j + 1) < g.shift || (j + 1) >= s.S + g.shift;
    }
    const bool vec_ok = (s.K & 3) == 0;

    __syncthreads();                            // weights and patch 0 are in LDS
    for (int tile = t_begin; tile < t_end; ++tile) {
        const u32x4* patch = lds + ((g.b_bytes + ((tile - t_begin) & 1) * g.patch_bytes) >> 4);
        floatx16 acc[MI][2];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

        for (int r = 0; r < s.R; ++r) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                frag_t af[MI], bfr[2];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    u32x4 v = patch[a_idx[mi] + r * g.PPAIRS + 2 * kk];
                    if (zero_lo[kk]) { v.x = 0u; v.y = 0u; }
                    if (zero_hi[kk]) { v.z = 0u; v.w = 0u; }
                    af[mi] = __builtin_bit_cast(frag_t, v);
                }
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    bfr[ni] = __builtin_bit_cast(frag_t, lds[(r * 4 + 2 * kk + fk) * kStemBN + ni * 32 + frow]);
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni) acc[mi][ni] = Elem<T>::mfma32(bfr[ni], af[mi], acc[mi][ni]);
            }
        }

        // ---- epilogue: lane l holds block pixel 32*frag + l%32 and, in accumulator element v, filter
        // 8*(v/4) + 4*(l/32) + v%4 of the 32-wide block (the filters are the MFMA's row operand).
        const StemTile tc = stem_decode(tile, g);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int p = tc.p0 + o_th[mi], q = tc.q0 + o_tw[mi];
            if (p < s.P && q < s.Q) {
                TO* yrow = y + (size_t)((tc.n * s.P + p) * s.Q + q) * s.K;
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int col = k0 + ni * 32 + 8 * gq + 4 * fk;
                        if (vec_ok && col + 3 < s.K) {
                            store4<TO>(yrow + col, acc[mi][ni][4 * gq], acc[mi][ni][4 * gq + 1], acc[mi][ni][4 * gq + 2],
                                       acc[mi][ni][4 * gq + 3]);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < s.K) yrow[col + e] = to_out<TO>(acc[mi][ni][4 * gq + e]);
                        }
                    }
                }
            }
        }
        __syncthreads();                        // next patch has landed; this patch buffer may be refilled
    }
}

constexpr int kStemMI = 2;                       // 4 waves x 2 fragments x 32 = 256 output pixels per block
constexpr int kStemLdsLimit = 64 * 1024;

bool plan_stem(const ConvShape& s, StemGeom* g) {
    if (s.C != 4 || s.dil != 1 || s.stride != 2 || (s.W & 1)) return false;
    const int shift = s.pad & 1;
    if (s.S + shift > 8) return false;
    const int BM = kStemWaves * kStemMI * 32;
    // block width 32 when that tiles Q without waste, else 16
    const int tw_log2 = (s.Q % 32 == 0 || s.Q >= 256) ? 5 : 4;
    const int TW = 1 << tw_log2;
    int TH = BM / TW;
    if (TH > s.P) TH = s.P;
    const int PH = (TH - 1) * s.stride + s.R;
    const int ppairs = ((TW - 1) * s.stride + 8) / 2;
    const long patch_bytes = (((long)PH * ppairs + 63) / 64) * 1024;   // whole wave-wide loads
    const long b_bytes = (long)s.R * 4 * kStemBN * 16;
    if (2 * patch_bytes + b_bytes > kStemLdsLimit) return false;
    g->TH = TH; g->TW_LOG2 = tw_log2; g->PH = PH; g->PPAIRS = ppairs;
    g->tiles_h = (s.P + TH - 1) / TH; g->tiles_w = (s.Q + TW - 1) / TW; g->tiles_n = (s.K + kStemBN - 1) / kStemBN;
    g->shift = shift; g->b_bytes = (int)b_bytes; g->patch_bytes = (int)patch_bytes; g->inv_ppairs = 1.0f / (float)ppairs;
    const long total = (long)s.N * g->tiles_h * g->tiles_w * g->tiles_n;
    if (total > 0x7fffffffL) return false;
    g->total_tiles = (int)total;
    g->tiles_per_wg = 1;
    return true;
}

template <typename T, typename TO>
hipError_t launch_stem_t(const void* x, const void* w, void* y, const ConvShape& s, StemGeom g, hipStream_t st) {
    const int lds_bytes = g.b_bytes + 2 * g.patch_bytes;
    auto kern = stem_kernel<T, TO, kStemMI>;
    const int threads = (kStemWaves + 1) * 64;
    int nwg = g.total_tiles;
    if (g.tiles_n == 1) {
        // one filter tile: workgroups own ranges of blocks and keep the weights resident
        static std::atomic<int> occ_lds{-1}, occ_val{1};
        int occ = occ_val.load(std::memory_order_acquire);
        if (occ_lds.load(std::memory_order_acquire) != lds_bytes) {
            int nb = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)kern, threads, (size_t)lds_bytes) != hipSuccess || nb < 1)
                nb = 1;
            occ = nb;
            occ_val.store(nb, std::memory_order_release);
            occ_lds.store(lds_bytes, std::memory_order_release);
        }
        // The kernel waits on memory most of the time, so every workgroup slot of the device is
        // filled (as many resident workgroups per compute unit as fit), each with an equal range.
        const int cap = g_max_workgroups.load(std::memory_order_relaxed);
        const long slots = cap > 0 ? cap : (long)device_cus() * occ;
        g.tiles_per_wg = (int)((g.total_tiles + slots - 1) / slots);
        nwg = (g.total_tiles + g.tiles_per_wg - 1) / g.tiles_per_wg;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(threads), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

}  // namespace

bool stem_supported(const ConvShape& s) {
    StemGeom g;
    return plan_stem(s, &g);
}

hipError_t launch_stem(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, hipStream_t st) {
    StemGeom g;
    if (!plan_stem(s, &g)) return hipErrorInvalidConfiguration;
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_stem_t<bf16_t, float>(x, w, y, s, g, st);
        return launch_stem_t<bf16_t, bf16_t>(x, w, y, s, g, st);
    }
    if (out_t == OUT_F32) return launch_stem_t<f16_t, float>(x, w, y, s, g, st);
    return launch_stem_t<f16_t, f16_t>(x, w, y, s, g, st);
}

}  // namespace iconv
